// C ABI of the library: argument validation on the host, then dispatch to the kernel launchers.
// Nothing is launched when an argument is rejected.
#include <cmath>
#include "apbv_common.h"

using namespace apbv;

namespace {

constexpr int64_t kMaxTokens = (int64_t)1 << 24;

bool aligned(const void* p, size_t a) { return (reinterpret_cast<uintptr_t>(p) % a) == 0; }

// A view is acceptable if it is empty, or has a 16-byte aligned pointer and strides that keep every
// (token, head) row 16-byte aligned and non-overlapping along the head dimension.
apbv_status check_view(const apbv_tensor& t, int heads, int d, int batch, bool may_be_empty) {
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

apbv_status check_heads(int batch, int hq, int hkv, int d) {
  if (batch < 1 || hq < 1 || hkv < 1 || batch > 65535 || hq > 65535) return APBV_ERR_SHAPE;
  if (hq % hkv) return APBV_ERR_SHAPE;
  if (d != 64 && d != 128) return APBV_ERR_UNSUPPORTED;
  return APBV_OK;
}

constexpr int kMaxKeySplits = 256;

// Validation shared by the two attention entry points; fills everything of `p` but the key split.
apbv_status fill_attention(int batch, int n_q_heads, int n_kv_heads, int head_dim, apbv_tensor q_local,
                                  apbv_tensor k_anchor, apbv_tensor v_anchor, apbv_tensor k_pass, apbv_tensor v_pass,
                                  apbv_tensor k_local, apbv_tensor v_local, float softmax_scale, void* out,
                                  float* lse_out, AttnParams& p) {
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

  p.q = to_view(q_local);
  p.k_seg[0] = to_view(k_anchor);
  p.k_seg[1] = to_view(k_pass);
  p.k_seg[2] = to_view(k_local);
  p.v_seg[0] = to_view(v_anchor);
  p.v_seg[1] = to_view(v_pass);
  p.v_seg[2] = to_view(v_local);
  p.out = static_cast<bf16_t*>(out);
  p.lse = lse_out;
  p.L = q_local.tokens;
  p.l_a = k_anchor.tokens;
  p.n_vis = k_anchor.tokens + k_pass.tokens;
  p.s_kv = p.n_vis + k_local.tokens;
  p.batch = batch;
  p.hq = n_q_heads;
  p.hkv = n_kv_heads;
  p.group = n_q_heads / n_kv_heads;
  p.scale_log2 = softmax_scale * 1.4426950408889634f;
  p.n_splits = 1;
  p.tiles_per_split = 1 << 30;
  p.split_stride_out = p.split_stride_lse = 0;
  return APBV_OK;
}

// Key split of the query-block attention: how many ranges of how many 64-key tiles.  With `requested` == 0 the
// count is chosen so that (query tiles x heads x batch x splits) reaches about two workgroups per compute unit
// while every range keeps at least four tiles; ranges are equal and none is empty.
struct KeySplit {
  int n_splits, tiles_per_split;
};
KeySplit plan_key_split(int batch, int n_q_heads, int64_t n_q, int64_t n_keys, int requested) {
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

size_t align256(size_t x) { return (x + 255) / 256 * 256; }

size_t reduced_workspace_bytes(int reducer, int batch, int hq, int hkv, int d, int64_t n_q, int64_t L, int64_t l_p) {
  const size_t base = compress_workspace_bytes(batch, hkv, d, L, l_p);
  if (reducer == APBV_REDUCE_SUM) return base;
  return (base + 255) / 256 * 256 + matrix_scores_workspace_bytes(reducer, batch, hkv, n_q * (hq / hkv), L);
}

apbv_status compress_entry(int reducer, float softmax_scale, int batch, int n_q_heads, int n_kv_heads, int head_dim, apbv_tensor q_probe,
                             apbv_tensor k_local, apbv_tensor v_local, int64_t l_p, int32_t* idx_out, void* k_c_out,
                             void* v_c_out, double* scores_out, void* workspace, size_t workspace_bytes,
                             void* hip_stream) {
  apbv_status st = check_heads(batch, n_q_heads, n_kv_heads, head_dim);
  if (st != APBV_OK) return st;
  if ((st = check_view(q_probe, n_q_heads, head_dim, batch, false)) != APBV_OK) return st;
  if ((st = check_view(k_local, n_kv_heads, head_dim, batch, false)) != APBV_OK) return st;
  if ((st = check_view(v_local, n_kv_heads, head_dim, batch, false)) != APBV_OK) return st;
  if (v_local.tokens != k_local.tokens) return APBV_ERR_SHAPE;
  const int64_t L = k_local.tokens;
  if (l_p < 0 || l_p > L) return APBV_ERR_SHAPE;
  if (l_p > 0) {
    if (idx_out == nullptr || k_c_out == nullptr || v_c_out == nullptr) return APBV_ERR_NULL;
    if (!aligned(k_c_out, 16) || !aligned(v_c_out, 16) || !aligned(idx_out, 4)) return APBV_ERR_SHAPE;
  }
  if (scores_out != nullptr && !aligned(scores_out, 8)) return APBV_ERR_SHAPE;
  if (reducer != APBV_REDUCE_SUM && reducer != APBV_REDUCE_MAX && reducer != APBV_REDUCE_SOFTMAX_SUM) return APBV_ERR_SHAPE;
  if (q_probe.tokens * (n_q_heads / n_kv_heads) > (int64_t)1 << 24) return APBV_ERR_UNSUPPORTED;   // rows of the score matrix per KV head
  if (reducer == APBV_REDUCE_SOFTMAX_SUM && (!(softmax_scale > 0.0f) || !std::isfinite(softmax_scale))) return APBV_ERR_SHAPE;
  const size_t need = reduced_workspace_bytes(reducer, batch, n_q_heads, n_kv_heads, head_dim, q_probe.tokens, L, l_p);
  if (workspace == nullptr || !aligned(workspace, 256) || workspace_bytes < need) return APBV_ERR_WORKSPACE;

  CompressParams p;
  p.q_probe = to_view(q_probe);
  p.k = to_view(k_local);
  p.v = to_view(v_local);
  p.L = L;
  p.l_p = l_p;
  p.batch = batch;
  p.hq = n_q_heads;
  p.hkv = n_kv_heads;
  p.group = n_q_heads / n_kv_heads;
  p.d = head_dim;
  p.idx_out = idx_out;
  p.k_c = static_cast<bf16_t*>(k_c_out);
  p.v_c = static_cast<bf16_t*>(v_c_out);
  p.scores_out = scores_out;
  p.workspace = workspace;
  p.workspace_bytes = workspace_bytes;
  p.reducer = reducer;
  p.scale_log2 = softmax_scale * 1.4426950408889634f;
  return launch_compress(p, static_cast<hipStream_t>(hip_stream));
}


}  // namespace

extern "C" {

const char* apbv_status_string(apbv_status s) {
  switch (s) {
    case APBV_OK: return "APBV_OK";
    case APBV_ERR_NULL: return "APBV_ERR_NULL: a required pointer is NULL";
    case APBV_ERR_SHAPE: return "APBV_ERR_SHAPE: inconsistent or out-of-range sizes or strides";
    case APBV_ERR_UNSUPPORTED: return "APBV_ERR_UNSUPPORTED: head_dim or size not implemented";
    case APBV_ERR_WORKSPACE: return "APBV_ERR_WORKSPACE: workspace NULL, misaligned or too small";
    case APBV_ERR_LAUNCH: return "APBV_ERR_LAUNCH: the HIP runtime refused a kernel launch";
  }
  return "unknown apbv_status";
}

int apbv_version(void) { return 200; }

size_t apbv_compress_workspace_bytes(int batch, int n_kv_heads, int head_dim, int64_t L, int64_t l_p) {
  if (batch < 1 || n_kv_heads < 1 || (head_dim != 64 && head_dim != 128) || L < 1 || L > kMaxTokens || l_p < 0 || l_p > L)
    return 0;
  return compress_workspace_bytes(batch, n_kv_heads, head_dim, L, l_p);
}

apbv_status apbv_compress_kv(int batch, int n_q_heads, int n_kv_heads, int head_dim, apbv_tensor q_probe,
                             apbv_tensor k_local, apbv_tensor v_local, int64_t l_p, int32_t* idx_out, void* k_c_out,
                             void* v_c_out, double* scores_out, void* workspace, size_t workspace_bytes,
                             void* hip_stream) {
  return compress_entry(APBV_REDUCE_SUM, 0.0f, batch, n_q_heads, n_kv_heads, head_dim, q_probe, k_local, v_local, l_p,
                        idx_out, k_c_out, v_c_out, scores_out, workspace, workspace_bytes, hip_stream);
}

size_t apbv_compress_reduced_workspace_bytes(int reducer, int batch, int n_q_heads, int n_kv_heads, int head_dim,
                                             int64_t n_q, int64_t L, int64_t l_p) {
  if (batch < 1 || n_q_heads < 1 || n_kv_heads < 1 || n_q_heads % n_kv_heads || (head_dim != 64 && head_dim != 128) ||
      n_q < 1 || n_q > kMaxTokens || L < 1 || L > kMaxTokens || l_p < 0 || l_p > L)
    return 0;
  if (reducer != APBV_REDUCE_SUM && reducer != APBV_REDUCE_MAX && reducer != APBV_REDUCE_SOFTMAX_SUM) return 0;
  return reduced_workspace_bytes(reducer, batch, n_q_heads, n_kv_heads, head_dim, n_q, L, l_p);
}

apbv_status apbv_compress_kv_reduced(int reducer, float softmax_scale, int batch, int n_q_heads, int n_kv_heads,
                                     int head_dim, apbv_tensor q_probe, apbv_tensor k_local, apbv_tensor v_local,
                                     int64_t l_p, int32_t* idx_out, void* k_c_out, void* v_c_out, double* scores_out,
                                     void* workspace, size_t workspace_bytes, void* hip_stream) {
  return compress_entry(reducer, softmax_scale, batch, n_q_heads, n_kv_heads, head_dim, q_probe, k_local, v_local, l_p,
                        idx_out, k_c_out, v_c_out, scores_out, workspace, workspace_bytes, hip_stream);
}

apbv_status apbv_host_attention(int batch, int n_q_heads, int n_kv_heads, int head_dim, apbv_tensor q_local,
                                apbv_tensor k_anchor, apbv_tensor v_anchor, apbv_tensor k_pass, apbv_tensor v_pass,
                                apbv_tensor k_local, apbv_tensor v_local, float softmax_scale, void* out,
                                float* lse_out, void* hip_stream) {
  AttnParams p;
  const apbv_status st = fill_attention(batch, n_q_heads, n_kv_heads, head_dim, q_local, k_anchor, v_anchor, k_pass,
                                        v_pass, k_local, v_local, softmax_scale, out, lse_out, p);
  if (st != APBV_OK) return st;
  return launch_host_attention(p, head_dim, static_cast<hipStream_t>(hip_stream));
}

apbv_status apbv_host_attention_group(int n_items, const apbv_attention_item* items, int n_q_heads, int n_kv_heads,
                                      int head_dim, float softmax_scale, void* hip_stream) {
  if (n_items < 1 || n_items > kMaxGroupItems) return APBV_ERR_SHAPE;
  if (items == nullptr) return APBV_ERR_NULL;
  AttnGroupParams gp;
  for (int m = 0; m < n_items; ++m) {
    const apbv_attention_item& it = items[m];
    const apbv_status st = fill_attention(1, n_q_heads, n_kv_heads, head_dim, it.q_local, it.k_anchor, it.v_anchor,
                                          it.k_pass, it.v_pass, it.k_local, it.v_local, softmax_scale, it.out,
                                          it.lse_out, gp.item[m]);
    if (st != APBV_OK) return st;
    if (it.k_local.tokens != it.q_local.tokens) return APBV_ERR_UNSUPPORTED;   // the merged schedule assumes a causal segment
  }
  gp.n_items = n_items;
  return launch_host_attention_group(gp, head_dim, static_cast<hipStream_t>(hip_stream));
}

size_t apbv_query_attention_workspace_bytes(int batch, int n_q_heads, int head_dim, int64_t n_q, int64_t n_keys,
                                            int n_splits) {
  if (batch < 1 || n_q_heads < 1 || (head_dim != 64 && head_dim != 128) || n_q < 1 || n_keys < 1 || n_splits < 0 ||
      n_q > kMaxTokens || n_keys > 3 * kMaxTokens)
    return 0;
  const KeySplit ks = plan_key_split(batch, n_q_heads, n_q, n_keys, n_splits);
  if (ks.n_splits == 1) return 0;
  const size_t rows = (size_t)batch * (size_t)n_q * (size_t)n_q_heads;
  return (size_t)ks.n_splits * (align256(rows * head_dim * sizeof(bf16_t)) + align256(rows * sizeof(float)));
}

apbv_status apbv_query_attention(int batch, int n_q_heads, int n_kv_heads, int head_dim, apbv_tensor q_block,
                                 apbv_tensor k_anchor, apbv_tensor v_anchor, apbv_tensor k_pass, apbv_tensor v_pass,
                                 apbv_tensor k_local, apbv_tensor v_local, float softmax_scale, int n_splits,
                                 void* out, float* lse_out, void* workspace, size_t workspace_bytes,
                                 void* hip_stream) {
  AttnParams p;
  const apbv_status st = fill_attention(batch, n_q_heads, n_kv_heads, head_dim, q_block, k_anchor, v_anchor, k_pass,
                                        v_pass, k_local, v_local, softmax_scale, out, lse_out, p);
  if (st != APBV_OK) return st;
  if (n_splits < 0) return APBV_ERR_SHAPE;
  const KeySplit ks = plan_key_split(batch, n_q_heads, p.L, p.s_kv, n_splits);
  hipStream_t stream = static_cast<hipStream_t>(hip_stream);
  if (ks.n_splits == 1) return launch_host_attention(p, head_dim, stream);

  const size_t need = apbv_query_attention_workspace_bytes(batch, n_q_heads, head_dim, p.L, p.s_kv, n_splits);
  if (workspace == nullptr || !aligned(workspace, 256) || workspace_bytes < need) return APBV_ERR_WORKSPACE;
  const size_t rows = (size_t)batch * (size_t)p.L * (size_t)n_q_heads;
  const size_t part_out_bytes = align256(rows * head_dim * sizeof(bf16_t));
  const size_t part_lse_bytes = align256(rows * sizeof(float));
  bf16_t* part_out = static_cast<bf16_t*>(workspace);
  float* part_lse = reinterpret_cast<float*>(static_cast<char*>(workspace) + (size_t)ks.n_splits * part_out_bytes);

  AttnParams ps = p;
  ps.out = part_out;
  ps.lse = part_lse;
  ps.n_splits = ks.n_splits;
  ps.tiles_per_split = ks.tiles_per_split;
  ps.split_stride_out = (int64_t)(part_out_bytes / sizeof(bf16_t));
  ps.split_stride_lse = (int64_t)(part_lse_bytes / sizeof(float));
  const apbv_status sl = launch_host_attention(ps, head_dim, stream);
  if (sl != APBV_OK) return sl;

  MergeParams m;
  m.parts_out = part_out;
  m.parts_lse = part_lse;
  m.stride_out = ps.split_stride_out;
  m.stride_lse = ps.split_stride_lse;
  m.out = p.out;
  m.lse_out = p.lse;
  m.rows = p.L;
  m.n_parts = ks.n_splits;
  m.hq = n_q_heads;
  m.d = head_dim;
  m.batch = batch;
  return launch_merge_lse(m, stream);
}

apbv_status apbv_merge_lse(int n_parts, int64_t rows, int n_q_heads, int head_dim, const void* parts_out,
                           int64_t part_stride_out, const float* parts_lse, int64_t part_stride_lse, void* out,
                           float* lse_out, void* hip_stream) {
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
  MergeParams p;
  p.parts_out = static_cast<const bf16_t*>(parts_out);
  p.parts_lse = parts_lse;
  p.stride_out = part_stride_out;
  p.stride_lse = part_stride_lse;
  p.out = static_cast<bf16_t*>(out);
  p.lse_out = lse_out;
  p.rows = rows;
  p.n_parts = n_parts;
  p.hq = n_q_heads;
  p.d = head_dim;
  p.batch = 1;
  return launch_merge_lse(p, static_cast<hipStream_t>(hip_stream));
}

}  // extern "C"
