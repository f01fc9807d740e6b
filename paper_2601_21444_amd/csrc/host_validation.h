// Host-side argument validation and planning of the C ABI (include/apbv.h).  Plain C++ with no HIP types, so that
// the rejection paths can be compiled alone with the host compiler and its sanitizers (tests/host/).  Everything
// here runs before any launch: a call that fails one of these checks enqueues nothing.
#pragma once
#include <stddef.h>
#include <stdint.h>
#include <cmath>
#include "apbv.h"

namespace apbv {

constexpr int64_t kMaxTokens = (int64_t)1 << 24;
constexpr int kMaxKeySplits = 256;
constexpr int kAttnKeyTile = 64;            // keys per tile of the attention kernel
constexpr int kAttnQueryTile = 256;         // query rows per workgroup
constexpr int kAttnNarrowQueryTile = 64;    // ... of the variant used for query blocks of at most
constexpr int kAttnNarrowMaxRows = 128;     // this many rows

inline bool aligned(const void* p, size_t a) { return (reinterpret_cast<uintptr_t>(p) % a) == 0; }
inline size_t align_up(size_t x, size_t a) { return (x + a - 1) / a * a; }
inline size_t align256(size_t x) { return align_up(x, 256); }

// A view is acceptable if it is empty, or has a 16-byte aligned pointer and strides that keep every
// (token, head) row 16-byte aligned and non-overlapping along the head dimension.
inline apbv_status check_view(const apbv_tensor& t, int heads, int d, int batch, bool may_be_empty) {
  if (t.tokens < 0 || t.tokens > kMaxTokens) return APBV_ERR_SHAPE;
  if (t.tokens == 0) return may_be_empty ? APBV_OK : APBV_ERR_SHAPE;
  if (t.ptr == nullptr) return APBV_ERR_NULL;
  if (!aligned(t.ptr, 16)) return APBV_ERR_SHAPE;
  if (t.stride_token < d || t.stride_token % 8) return APBV_ERR_SHAPE;
  if (t.stride_token >= kMaxTokens) return APBV_ERR_UNSUPPORTED;       // the kernels keep row offsets of a 64-row tile in 32 bits
  if (heads > 1 && (t.stride_head < d || t.stride_head % 8)) return APBV_ERR_SHAPE;
  if (batch > 1 && (t.stride_batch <= 0 || t.stride_batch % 8)) return APBV_ERR_SHAPE;
  return APBV_OK;
}

inline apbv_status check_heads(int batch, int hq, int hkv, int d) {
  if (batch < 1 || hq < 1 || hkv < 1 || batch > 65535 || hq > 65535) return APBV_ERR_SHAPE;
  if (hq % hkv) return APBV_ERR_SHAPE;
  if (d != 64 && d != 128) return APBV_ERR_UNSUPPORTED;
  return APBV_OK;
}

inline bool valid_reducer(int r) { return r == APBV_REDUCE_SUM || r == APBV_REDUCE_MAX || r == APBV_REDUCE_SOFTMAX_SUM; }

// Arguments of the attention entry points (Eq. 4 / Eq. 5).
inline apbv_status validate_attention(int batch, int n_q_heads, int n_kv_heads, int head_dim, const apbv_tensor& q_local,
                                      const apbv_tensor& k_anchor, const apbv_tensor& v_anchor, const apbv_tensor& k_pass,
                                      const apbv_tensor& v_pass, const apbv_tensor& k_local, const apbv_tensor& v_local,
                                      float softmax_scale, const void* out, const float* lse_out) {
  apbv_status st = check_heads(batch, n_q_heads, n_kv_heads, head_dim);
  if (st != APBV_OK) return st;
  if ((st = check_view(q_local, n_q_heads, head_dim, batch, false)) != APBV_OK) return st;
  if ((st = check_view(k_local, n_kv_heads, head_dim, batch, true)) != APBV_OK) return st;
  if ((st = check_view(v_local, n_kv_heads, head_dim, batch, true)) != APBV_OK) return st;
  if ((st = check_view(k_anchor, n_kv_heads, head_dim, batch, true)) != APBV_OK) return st;
  if ((st = check_view(v_anchor, n_kv_heads, head_dim, batch, true)) != APBV_OK) return st;
  if ((st = check_view(k_pass, n_kv_heads, head_dim, batch, true)) != APBV_OK) return st;
  if ((st = check_view(v_pass, n_kv_heads, head_dim, batch, true)) != APBV_OK) return st;
  if ((k_local.tokens != 0 && q_local.tokens != k_local.tokens) || v_local.tokens != k_local.tokens) return APBV_ERR_SHAPE;
  if (v_anchor.tokens != k_anchor.tokens || v_pass.tokens != k_pass.tokens) return APBV_ERR_SHAPE;
  if (k_anchor.tokens + k_pass.tokens + k_local.tokens < 1) return APBV_ERR_SHAPE;       // every query needs a key
  if (!(softmax_scale > 0.0f) || !std::isfinite(softmax_scale)) return APBV_ERR_SHAPE;
  if (out == nullptr) return APBV_ERR_NULL;
  if (!aligned(out, 16) || (lse_out != nullptr && !aligned(lse_out, 4))) return APBV_ERR_SHAPE;
  return APBV_OK;
}

// Arguments of the compression entry points (Sec. 3.3 / Alg. 1) other than the workspace.
inline apbv_status validate_compress(int reducer, float softmax_scale, int batch, int n_q_heads, int n_kv_heads, int head_dim,
                                     const apbv_tensor& q_probe, const apbv_tensor& k_local, const apbv_tensor& v_local,
                                     int64_t l_p, const int32_t* idx_out, const void* k_c_out, const void* v_c_out,
                                     const double* scores_out) {
  apbv_status st = check_heads(batch, n_q_heads, n_kv_heads, head_dim);
  if (st != APBV_OK) return st;
  if ((st = check_view(q_probe, n_q_heads, head_dim, batch, false)) != APBV_OK) return st;
  if ((st = check_view(k_local, n_kv_heads, head_dim, batch, false)) != APBV_OK) return st;
  if ((st = check_view(v_local, n_kv_heads, head_dim, batch, false)) != APBV_OK) return st;
  if (v_local.tokens != k_local.tokens) return APBV_ERR_SHAPE;
  if (l_p < 0 || l_p > k_local.tokens) return APBV_ERR_SHAPE;
  if (l_p > 0) {
    if (idx_out == nullptr || k_c_out == nullptr || v_c_out == nullptr) return APBV_ERR_NULL;
    if (!aligned(k_c_out, 16) || !aligned(v_c_out, 16) || !aligned(idx_out, 4)) return APBV_ERR_SHAPE;
  }
  if (scores_out != nullptr && !aligned(scores_out, 8)) return APBV_ERR_SHAPE;
  if (!valid_reducer(reducer)) return APBV_ERR_SHAPE;
  if (q_probe.tokens * (n_q_heads / n_kv_heads) > (int64_t)1 << 24) return APBV_ERR_UNSUPPORTED;   // rows of the score matrix per KV head
  if (reducer == APBV_REDUCE_SOFTMAX_SUM && (!(softmax_scale > 0.0f) || !std::isfinite(softmax_scale))) return APBV_ERR_SHAPE;
  return APBV_OK;
}

inline apbv_status validate_merge(int n_parts, int64_t rows, int n_q_heads, int head_dim, const void* parts_out,
                                  int64_t part_stride_out, const float* parts_lse, int64_t part_stride_lse,
                                  const void* out, const float* lse_out) {
  if (n_parts < 1 || n_parts > 65536 || rows < 1 || rows > kMaxTokens || n_q_heads < 1 || n_q_heads > 65535)
    return APBV_ERR_SHAPE;
  if (head_dim != 64 && head_dim != 128) return APBV_ERR_UNSUPPORTED;
  if (parts_out == nullptr || parts_lse == nullptr || out == nullptr) return APBV_ERR_NULL;
  if (!aligned(parts_out, 16) || !aligned(out, 16) || !aligned(parts_lse, 4) || (lse_out != nullptr && !aligned(lse_out, 4)))
    return APBV_ERR_SHAPE;
  if (n_parts > 1) {
    if (part_stride_out < rows * n_q_heads * head_dim || part_stride_out % 8) return APBV_ERR_SHAPE;
    if (part_stride_lse < rows * n_q_heads) return APBV_ERR_SHAPE;
  }
  return APBV_OK;
}

// Key split of the query-block attention: how many ranges of how many 64-key tiles.  With `requested` == 0 the
// count is chosen so that (query tiles x heads x batch x splits) reaches about two workgroups per compute unit
// while every range keeps at least four tiles; ranges are equal and none is empty.
struct KeySplit {
  int n_splits, tiles_per_split;
};
inline KeySplit plan_key_split(int batch, int n_q_heads, int64_t n_q, int64_t n_keys, int requested) {
  const int64_t n_tiles = (n_keys + kAttnKeyTile - 1) / kAttnKeyTile;
  int64_t s = requested;
  if (s <= 0) {
    const int64_t tile = n_q <= kAttnNarrowMaxRows ? kAttnNarrowQueryTile : kAttnQueryTile;
    const int64_t wgs = (n_q + tile - 1) / tile * n_q_heads * batch;
    s = (512 + wgs - 1) / wgs;
    const int64_t cap = n_tiles / 4 > 1 ? n_tiles / 4 : 1;
    s = s < cap ? s : cap;
  }
  s = s < n_tiles ? s : n_tiles;
  s = s < kMaxKeySplits ? s : kMaxKeySplits;
  const int64_t per = (n_tiles + s - 1) / s;
  KeySplit ks;
  ks.tiles_per_split = (int)per;
  ks.n_splits = (int)((n_tiles + per - 1) / per);
  return ks;
}

inline size_t query_attention_workspace_bytes(int batch, int n_q_heads, int head_dim, int64_t n_q, int64_t n_keys,
                                              int n_splits) {
  if (batch < 1 || n_q_heads < 1 || (head_dim != 64 && head_dim != 128) || n_q < 1 || n_keys < 1 || n_splits < 0 ||
      n_q > kMaxTokens || n_keys > 3 * kMaxTokens)
    return 0;
  const KeySplit ks = plan_key_split(batch, n_q_heads, n_q, n_keys, n_splits);
  if (ks.n_splits == 1) return 0;
  const size_t rows = (size_t)batch * (size_t)n_q * (size_t)n_q_heads;
  return (size_t)ks.n_splits * (align256(rows * head_dim * 2) + align256(rows * sizeof(float)));
}

// ---- workspace of the compression call: [partial sums of the pooled query | scores | sort arrays of the exact
// fallback when they do not fit the LDS]
constexpr int64_t kLdsSortMax = 8192;          // entries that fit the LDS selection arrays (14 bytes each)
constexpr int kPoolSplitMax = 8;               // workgroups (partial sums) per pooled query

// Ranges the n_rows = n_q * G probe rows of one pooled query are cut into: about 64 rows each, but no more ranges
// than it takes to give every compute unit two (n_pooled = batch * Hkv pooled queries share the 256 of them).
inline int pool_splits(int64_t n_rows, int64_t n_pooled) {
  int64_t s = (n_rows + 63) / 64;
  const int64_t fill = 512 / (n_pooled < 1 ? 1 : n_pooled);
  s = s > fill ? fill : s;
  return (int)(s < 1 ? 1 : (s > kPoolSplitMax ? kPoolSplitMax : s));
}

inline int64_t pow2_ceil(int64_t x) {
  int64_t n = 1;
  while (n < x) n <<= 1;
  return n;
}

struct CompressWorkspace {
  size_t qbar_off, scores_off, sort_keys_off, sort_idx_off, total;
  int64_t n_sort;       // capacity (entries, a power of two) of the selection's sort arrays
  bool sort_in_global;
};

inline CompressWorkspace plan_compress_workspace(int batch, int hkv, int d, int64_t L, int64_t l_p) {
  CompressWorkspace w;
  size_t off = 0;
  w.qbar_off = off;
  off = align256(off + (size_t)batch * hkv * kPoolSplitMax * d * sizeof(double));
  w.scores_off = off;
  off = align256(off + (size_t)batch * hkv * (size_t)L * sizeof(double));
  // capacity of the sort arrays: room for the candidates of the fast path (the winners plus the rest
  // of the threshold bucket) when that fits the LDS, else exactly the padded winners
  w.n_sort = pow2_ceil(l_p > 1 ? l_p : 1);
  w.sort_in_global = w.n_sort > kLdsSortMax;
  if (!w.sort_in_global && 2 * w.n_sort <= kLdsSortMax) w.n_sort *= 2;
  w.sort_keys_off = w.sort_idx_off = off;
  if (w.sort_in_global) {
    w.sort_keys_off = off;
    off = align256(off + (size_t)batch * hkv * (size_t)w.n_sort * sizeof(uint64_t));
    w.sort_idx_off = off;
    off = align256(off + (size_t)batch * hkv * (size_t)w.n_sort * (sizeof(uint32_t) + sizeof(uint16_t)));
  }
  w.total = off;
  return w;
}

inline size_t compress_workspace_bytes_checked(int batch, int n_kv_heads, int head_dim, int64_t L, int64_t l_p) {
  if (batch < 1 || n_kv_heads < 1 || (head_dim != 64 && head_dim != 128) || L < 1 || L > kMaxTokens || l_p < 0 || l_p > L)
    return 0;
  return plan_compress_workspace(batch, n_kv_heads, head_dim, L, l_p).total;
}

}  // namespace apbv
