// C ABI of the library: argument validation on the host, then dispatch to the kernel launchers.
// Nothing is launched when an argument is rejected.
#include <cmath>
#include "apbv_common.h"

using namespace apbv;

namespace {

// Validation shared by the two attention entry points; fills everything of `p` but the key split.
apbv_status fill_attention(int batch, int n_q_heads, int n_kv_heads, int head_dim, apbv_tensor q_local,
                                  apbv_tensor k_anchor, apbv_tensor v_anchor, apbv_tensor k_pass, apbv_tensor v_pass,
                                  apbv_tensor k_local, apbv_tensor v_local, float softmax_scale, void* out,
                                  float* lse_out, AttnParams& p) {
  const apbv_status st = validate_attention(batch, n_q_heads, n_kv_heads, head_dim, q_local, k_anchor, v_anchor, k_pass,
                                            v_pass, k_local, v_local, softmax_scale, out, lse_out);
  if (st != APBV_OK) return st;

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

size_t reduced_workspace_bytes(int reducer, int batch, int hq, int hkv, int d, int64_t n_q, int64_t L, int64_t l_p) {
  const size_t base = compress_workspace_bytes(batch, hkv, d, L, l_p);
  if (reducer == APBV_REDUCE_SUM) return base;
  return (base + 255) / 256 * 256 + matrix_scores_workspace_bytes(reducer, batch, hkv, n_q * (hq / hkv), L);
}

apbv_status compress_entry(int reducer, float softmax_scale, int batch, int n_q_heads, int n_kv_heads, int head_dim, apbv_tensor q_probe,
                             apbv_tensor k_local, apbv_tensor v_local, int64_t l_p, int32_t* idx_out, void* k_c_out,
                             void* v_c_out, double* scores_out, void* workspace, size_t workspace_bytes,
                             void* hip_stream, bool use_static_scratch = false) {
  const apbv_status st = validate_compress(reducer, softmax_scale, batch, n_q_heads, n_kv_heads, head_dim, q_probe, k_local,
                                           v_local, l_p, idx_out, k_c_out, v_c_out, scores_out);
  if (st != APBV_OK) return st;
  const int64_t L = k_local.tokens;
  const size_t need = reduced_workspace_bytes(reducer, batch, n_q_heads, n_kv_heads, head_dim, q_probe.tokens, L, l_p);
  if (use_static_scratch) {
    if (need > kStaticScratchBytes) return APBV_ERR_WORKSPACE;      // beyond the static array: use apbv_compress_kv
  } else if (workspace == nullptr || !aligned(workspace, 256) || workspace_bytes < need) {
    return APBV_ERR_WORKSPACE;
  }

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
  p.use_static_scratch = use_static_scratch;
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
    case APBV_ERR_WORKSPACE: return "APBV_ERR_WORKSPACE: workspace NULL, misaligned or too small (or, without a workspace argument, the shape needs more than the static scratch array holds)";
    case APBV_ERR_LAUNCH: return "APBV_ERR_LAUNCH: the HIP runtime refused a kernel launch";
  }
  return "unknown apbv_status";
}

int apbv_version(void) { return 212; }

size_t apbv_compress_workspace_bytes(int batch, int n_kv_heads, int head_dim, int64_t L, int64_t l_p) {
  return compress_workspace_bytes_checked(batch, n_kv_heads, head_dim, L, l_p);
}

apbv_status apbv_compress_kv(int batch, int n_q_heads, int n_kv_heads, int head_dim, apbv_tensor q_probe,
                             apbv_tensor k_local, apbv_tensor v_local, int64_t l_p, int32_t* idx_out, void* k_c_out,
                             void* v_c_out, double* scores_out, void* workspace, size_t workspace_bytes,
                             void* hip_stream) {
  return compress_entry(APBV_REDUCE_SUM, 0.0f, batch, n_q_heads, n_kv_heads, head_dim, q_probe, k_local, v_local, l_p,
                        idx_out, k_c_out, v_c_out, scores_out, workspace, workspace_bytes, hip_stream);
}

apbv_status apbv_compress_kv_noalloc(int batch, int n_q_heads, int n_kv_heads, int head_dim, apbv_tensor q_probe,
                                     apbv_tensor k_local, apbv_tensor v_local, int64_t l_p, int32_t* idx_out,
                                     void* k_c_out, void* v_c_out, double* scores_out, void* hip_stream) {
  return compress_entry(APBV_REDUCE_SUM, 0.0f, batch, n_q_heads, n_kv_heads, head_dim, q_probe, k_local, v_local, l_p,
                        idx_out, k_c_out, v_c_out, scores_out, nullptr, 0, hip_stream, true);
}

size_t apbv_compress_reduced_workspace_bytes(int reducer, int batch, int n_q_heads, int n_kv_heads, int head_dim,
                                             int64_t n_q, int64_t L, int64_t l_p) {
  if (batch < 1 || n_q_heads < 1 || n_kv_heads < 1 || n_q_heads % n_kv_heads || (head_dim != 64 && head_dim != 128) ||
      n_q < 1 || n_q > kMaxTokens || L < 1 || L > kMaxTokens || l_p < 0 || l_p > L)
    return 0;
  if (!valid_reducer(reducer)) return 0;
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
  return query_attention_workspace_bytes(batch, n_q_heads, head_dim, n_q, n_keys, n_splits);
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
  const apbv_status st = validate_merge(n_parts, rows, n_q_heads, head_dim, parts_out, part_stride_out, parts_lse,
                                        part_stride_lse, out, lse_out);
  if (st != APBV_OK) return st;
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
