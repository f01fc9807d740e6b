/*
 * apbv.h -- C ABI of the MI355X (gfx950) library for one virtual host's share of APB-V's approximate
 * prefill attention (arXiv 2601.21444).
 *
 * Two operations make up the per-layer hot path of a host (Alg. 1); apbv_query_attention and apbv_merge_lse
 * serve the query block: its partial attention on every host and the merge of those results (Eq. 5):
 *   apbv_compress_kv     Sec. 3.3 / Alg. 1 "Identify Essential KVs" + "Send Block's Essential KVs":
 *                        score every local key against the query block, keep the l_p best per KV head,
 *                        gather them into the compressed block (K_c, V_c).
 *   apbv_host_attention  Eq. 4 (with Eq. 1): attention of the local query block over the concatenation
 *                        [anchor | passing | local], anchor and passing fully visible, local causal.
 * Around them: apbv_host_attention_group (the attention problems of a physical host's two virtual hosts and of the
 * anchor block in one launch, Sec. 4.3) and apbv_compress_kv_reduced (the compression under another reduction of
 * the score matrix to one score per key).
 *
 * General conventions
 *   - Every data pointer is a DEVICE pointer (HIP global memory on the current device) unless a
 *     parameter is explicitly marked host.  bf16 values are passed as their 16-bit patterns.
 *   - The caller owns every buffer (inputs, outputs, workspace).  The library allocates no device
 *     memory.  Its only state is a per-device one-time set-up made by the first compression call on a device
 *     (apbv_compress_kv, apbv_compress_kv_reduced, apbv_compress_kv_noalloc): a function attribute of the selection
 *     kernel and the device address of the static scratch array of apbv_compress_kv_noalloc.  No results depend on it.
 *   - Calls are asynchronous: work is enqueued on `hip_stream` (a hipStream_t passed as void*; NULL is
 *     the default stream) and outputs are valid once the caller has synchronised that stream.  The calls can be
 *     captured into a HIP graph (they enqueue kernels only); make the first compression call on a device before
 *     the capture starts, so that the one-time set-up is not part of it.
 *   - Inputs are never written.  Outputs and workspace must not overlap inputs or each other.
 *   - Every argument error is detected on the host before anything is launched and reported through
 *     the return value; nothing is launched in that case.  No function throws or aborts.
 *   - Inputs must be finite; NaN/Inf give an unspecified ranking / output.
 *   - `batch` = independent problems of identical shape (for instance the two virtual hosts of one
 *     physical host, Sec. 4.3, or concurrent requests).
 */
#ifndef APBV_H_
#define APBV_H_

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum {
  APBV_OK = 0,
  APBV_ERR_NULL = -1,        /* a required pointer is NULL                                   */
  APBV_ERR_SHAPE = -2,       /* inconsistent or out-of-range sizes / strides                 */
  APBV_ERR_UNSUPPORTED = -3, /* head_dim or size outside what the kernels implement          */
  APBV_ERR_WORKSPACE = -4,   /* workspace NULL, misaligned or too small                      */
  APBV_ERR_LAUNCH = -5       /* the HIP runtime refused a launch (hipGetLastError != success)*/
} apbv_status;

/* A [tokens, heads, head_dim] bf16 view.  head_dim is contiguous (stride 1); all strides are in
 * ELEMENTS and must be multiples of 8 (16-byte vector access); stride_token must be below 2^24;
 * ptr must be 16-byte aligned.
 * ptr may be NULL iff tokens == 0.  stride_batch is ignored when batch == 1. */
typedef struct {
  const void* ptr;
  int64_t tokens;
  int64_t stride_token;
  int64_t stride_head;
  int64_t stride_batch;
} apbv_tensor;

/* Host, pure.  Static string naming a status code. */
const char* apbv_status_string(apbv_status s);

/* Host, pure.  Library version, major*10000 + minor*100 + patch. */
int apbv_version(void);

/* Host, pure.  Bytes of workspace apbv_compress_kv needs for this shape (0 on invalid arguments).
 * The workspace must be 256-byte aligned.  Its contents need no initialisation and are garbage
 * afterwards. */
size_t apbv_compress_workspace_bytes(int batch, int n_kv_heads, int head_dim, int64_t L, int64_t l_p);

/*
 * KV compression of one context block (Sec. 3.3; Alg. 1: S_h <- Q_qr K^(h)T, then
 * (K^(h), V^(h)).gather(ArgTop_{l_p}(S_h))).
 *
 * For every batch item b and KV head v (G = n_q_heads / n_kv_heads):
 *   s[j]   = sum_{t < n_q} sum_{g < G} Q_qr[t, v*G+g, :] . K[j, v, :]     (float64 accumulation)
 *   idx    = the l_p indices j with the largest s[j], ordered by descending s; equal scores
 *            (compared as real numbers) by ascending j
 *   K_c[i, v, :] = K[idx[i], v, :],   V_c[i, v, :] = V[idx[i], v, :]      (bit copies)
 *
 *   q_probe   Q_qr  [n_q, Hq,  d], n_q = q_probe.tokens >= 1
 *   k_local   K^(h) [L,   Hkv, d], L = k_local.tokens >= 1
 *   v_local   V^(h) [L,   Hkv, d], same token count
 *   l_p       0 <= l_p <= L   (l_p == 0: nothing is written to idx/k_c/v_c, which may then be NULL)
 *   idx_out   [batch, Hkv, l_p] int32
 *   k_c_out, v_c_out   [batch, l_p, Hkv, d] bf16, dense
 *   scores_out  optional (may be NULL): [batch, Hkv, L] float64, the ranking scores s
 *   workspace / workspace_bytes   at least apbv_compress_workspace_bytes(...) bytes, 256-byte aligned
 *
 * Supported: head_dim in {64, 128}; L <= 2^24; n_q_heads % n_kv_heads == 0; n_q * G <= 2^24.
 */
apbv_status apbv_compress_kv(int batch, int n_q_heads, int n_kv_heads, int head_dim,
                             apbv_tensor q_probe, apbv_tensor k_local, apbv_tensor v_local,
                             int64_t l_p,
                             int32_t* idx_out, void* k_c_out, void* v_c_out, double* scores_out,
                             void* workspace, size_t workspace_bytes, void* hip_stream);

/*
 * apbv_compress_kv for callers that cannot allocate or hand over a workspace: code under HIP graph capture, tight
 * serving loops, harnesses that forbid hipMalloc.  Same operation, arguments, outputs and results as
 * apbv_compress_kv (bit-identical), without the workspace arguments: the intermediate pooled query and scores live in
 * a static device array of APBV_NOALLOC_MAX_WORKSPACE_BYTES bytes inside the library, one copy per GPU, held until
 * the process ends.  The call allocates nothing and frees nothing.
 *
 * Limits: apbv_compress_workspace_bytes(batch, n_kv_heads, head_dim, L, l_p) must not exceed
 * APBV_NOALLOC_MAX_WORKSPACE_BYTES (about batch * n_kv_heads * L <= 500 000 scores), else APBV_ERR_WORKSPACE and
 * nothing is launched.  All calls on one GPU share that GPU's array: calls that overlap in time on one GPU (different
 * streams or host threads without ordering between them) race and give unspecified results; calls ordered on one
 * stream, or by events, are fine.  The array's previous contents are never read before they are rewritten.
 */
#define APBV_NOALLOC_MAX_WORKSPACE_BYTES 4194304
apbv_status apbv_compress_kv_noalloc(int batch, int n_q_heads, int n_kv_heads, int head_dim,
                                     apbv_tensor q_probe, apbv_tensor k_local, apbv_tensor v_local,
                                     int64_t l_p,
                                     int32_t* idx_out, void* k_c_out, void* v_c_out, double* scores_out,
                                     void* hip_stream);

/*
 * How the n_q*G x L score matrix S_h = Q_qr K^(h)T of Alg. 1 becomes one score per key and KV head (the paper does
 * not say; the sum is the reading this library adopts, the others are offered so that a caller can match another):
 *   APBV_REDUCE_SUM          s[j] = sum over rows (t, g) of S[(t, g), j]          (apbv_compress_kv; float64)
 *   APBV_REDUCE_MAX          s[j] = max over rows of S[(t, g), j]
 *   APBV_REDUCE_SOFTMAX_SUM  s[j] = sum over rows of softmax_j(softmax_scale * S[(t, g), :])[j], the attention mass
 *                            the query block puts on key j (softmax over the block's L keys, no mask)
 * MAX and SOFTMAX_SUM form the logits on the matrix cores: bf16 operands, fp32 accumulation and reduction; the
 * scores are then widened to float64 and ranked exactly as in apbv_compress_kv (ties by ascending index).
 */
typedef enum { APBV_REDUCE_SUM = 0, APBV_REDUCE_MAX = 1, APBV_REDUCE_SOFTMAX_SUM = 2 } apbv_reducer;

/* Host, pure.  Bytes of workspace apbv_compress_kv_reduced needs (0 on invalid arguments); 256-byte aligned. */
size_t apbv_compress_reduced_workspace_bytes(int reducer, int batch, int n_q_heads, int n_kv_heads, int head_dim,
                                             int64_t n_q, int64_t L, int64_t l_p);

/*
 * apbv_compress_kv with a chosen reduction (Sec. 3.3 / Alg. 1, same outputs and layouts).  `reducer` is an
 * apbv_reducer; `softmax_scale` is used by APBV_REDUCE_SOFTMAX_SUM only (finite, positive) and ignored otherwise.
 * With APBV_REDUCE_SUM the call is apbv_compress_kv.  APBV_REDUCE_SOFTMAX_SUM supports up to 8192 rows n_q*G.
 */
apbv_status apbv_compress_kv_reduced(int reducer, float softmax_scale,
                                     int batch, int n_q_heads, int n_kv_heads, int head_dim,
                                     apbv_tensor q_probe, apbv_tensor k_local, apbv_tensor v_local,
                                     int64_t l_p,
                                     int32_t* idx_out, void* k_c_out, void* v_c_out, double* scores_out,
                                     void* workspace, size_t workspace_bytes, void* hip_stream);

/*
 * Fused host attention (Eq. 4 by the definition of Eq. 1):
 *   O[i, h, :] = sum_j softmax_j( softmax_scale * Q[i, h, :] . Kcat[j, h/G, :] + mask(i, j) ) Vcat[j, h/G, :]
 * over Kcat = [K_a ; K_p ; K], Vcat = [V_a ; V_p ; V]; mask = 0 for anchor and passing keys; local key
 * j' is visible to local query i iff j' <= i (so every row sees at least one key).
 *
 *   q_local              Q^(h) [L, Hq, d]
 *   k_anchor, v_anchor   [l_a,   Hkv, d]   l_a  >= 0
 *   k_pass,   v_pass     [n_p,   Hkv, d]   n_p = P*l_p >= 0, blocks of the preceding hosts in host order
 *   k_local,  v_local    [L,     Hkv, d]   row i of q_local is the query of local key i; L == q_local.tokens,
 *                                          or 0 tokens: no causal segment, every anchor/passing key is visible to
 *                                          every query (a partial result to be merged by apbv_merge_lse, Eq. 5)
 *   softmax_scale        the paper's 1/sqrt(head_dim); any finite positive value is accepted
 *   out                  [batch, L, Hq, d] bf16, dense
 *   lse_out              optional (may be NULL): [batch, Hq, L] float32, natural-log sum of the
 *                        exponentials of the scaled visible logits (for merging partial results)
 *
 * Arithmetic: bf16 operands, fp32 accumulation and softmax, probabilities rounded to bf16 before the
 * PV product, output rounded to bf16.
 * Supported: head_dim in {64, 128}; n_q_heads % n_kv_heads == 0; each K/V pair must agree in tokens; at least
 * one key in total.
 */
apbv_status apbv_host_attention(int batch, int n_q_heads, int n_kv_heads, int head_dim,
                                apbv_tensor q_local,
                                apbv_tensor k_anchor, apbv_tensor v_anchor,
                                apbv_tensor k_pass, apbv_tensor v_pass,
                                apbv_tensor k_local, apbv_tensor v_local,
                                float softmax_scale, void* out, float* lse_out, void* hip_stream);

/*
 * Merge of partial attention results by their log-sum-exp (Eq. 5: A_qr = Merge({A_qr^(h), lse^(h)}_h), "online
 * softmax" of Sec. 4.2 / App. B.1).  Part h is attention of the SAME queries over its own key set, as produced by
 * apbv_host_attention with lse_out; over the union of disjoint key sets the exact result is
 *   A = sum_h w_h A_h / sum_h w_h,  w_h = exp(lse_h - max_h lse_h),  lse = max_h lse_h + log(sum_h w_h).
 *
 *   parts_out   n_parts partial outputs, part h at parts_out + h*part_stride_out elements, each [rows, Hq, d] bf16 dense
 *   parts_lse   n_parts log-sum-exps,    part h at parts_lse + h*part_stride_lse elements, each [Hq, rows] fp32
 *               (-inf marks a part with no visible key for that row: it contributes nothing)
 *   out         [rows, Hq, d] bf16;  lse_out optional (may be NULL) [Hq, rows] fp32
 * 1 <= n_parts <= 65536; head_dim in {64, 128}; parts_out and out 16-byte aligned, strides multiples of 8 / 1.
 */
apbv_status apbv_merge_lse(int n_parts, int64_t rows, int n_q_heads, int head_dim,
                           const void* parts_out, int64_t part_stride_out,
                           const float* parts_lse, int64_t part_stride_lse,
                           void* out, float* lse_out, void* hip_stream);

/*
 * One attention problem of a group: the arguments of apbv_host_attention for batch 1.
 */
typedef struct {
  apbv_tensor q_local;
  apbv_tensor k_anchor, v_anchor;
  apbv_tensor k_pass, v_pass;
  apbv_tensor k_local, v_local;   /* must hold q_local.tokens tokens (a causal segment) */
  void* out;                      /* [L, Hq, d] bf16 */
  float* lse_out;                 /* optional [Hq, L] fp32 */
} apbv_attention_item;

/*
 * A physical host's attention work of one layer in ONE launch (Alg. 1 "context attention" of both virtual hosts,
 * Sec. 4.3; and the anchor block's own causal attention): n_items independent problems with the same head counts and
 * head_dim but their own lengths -- for host h of H the blocks h and 2H-1-h see h*l_p and (2H-1-h)*l_p passing keys,
 * the anchor block is a problem with no anchor and no passing segment.  Every problem computes exactly what
 * apbv_host_attention computes for it (bit-identical results); the launch orders the query tiles of all problems
 * together, heaviest first, so that the short problems fill the tail of the long one.
 *
 *   items     HOST array of n_items descriptors (read during the call only); 1 <= n_items <= 8
 * Errors as for apbv_host_attention, for any item; a problem without a causal segment is APBV_ERR_UNSUPPORTED here.
 * Outputs of different items must not overlap.
 */
apbv_status apbv_host_attention_group(int n_items, const apbv_attention_item* items,
                                      int n_q_heads, int n_kv_heads, int head_dim,
                                      float softmax_scale, void* hip_stream);

/* Host, pure.  Bytes of workspace apbv_query_attention needs (256-byte aligned; 0 when the call would not split
 * the keys, and 0 on invalid arguments).  n_keys = l_a + n_p + local keys; n_splits as passed to the call. */
size_t apbv_query_attention_workspace_bytes(int batch, int n_q_heads, int head_dim, int64_t n_q, int64_t n_keys,
                                            int n_splits);

/*
 * Attention of a SHORT query block over a host's keys (Eq. 5: A_qr^(h), lse^(h) = Attn(Q_qr, K, V); also the
 * decoding-time attention of Sec. 4.2).  Same operation, arguments, layouts and arithmetic as apbv_host_attention;
 * the difference is the launch: a block of a few hundred queries yields too few (query tile x head) work items to
 * fill the GPU, so the key axis is cut into ranges that run in parallel, each producing a normalised partial result
 * and its log-sum-exp in the workspace, combined by the merge of apbv_merge_lse in a second kernel.  Partial
 * results pass through bf16, so the output can differ from apbv_host_attention's by bf16 rounding of the parts.
 *
 *   n_splits   0: chosen by the library from the shape; >= 1: requested number of key ranges (clipped to the number
 *              of 64-key tiles and to 256; 1 = no split, the call is then apbv_host_attention and needs no workspace)
 *   workspace / workspace_bytes   at least apbv_query_attention_workspace_bytes(...) bytes, 256-byte aligned; may be
 *              NULL / 0 when that is 0.  Contents need no initialisation and are garbage afterwards.
 */
apbv_status apbv_query_attention(int batch, int n_q_heads, int n_kv_heads, int head_dim,
                                 apbv_tensor q_block,
                                 apbv_tensor k_anchor, apbv_tensor v_anchor,
                                 apbv_tensor k_pass, apbv_tensor v_pass,
                                 apbv_tensor k_local, apbv_tensor v_local,
                                 float softmax_scale, int n_splits, void* out, float* lse_out,
                                 void* workspace, size_t workspace_bytes, void* hip_stream);

#ifdef __cplusplus
}
#endif
#endif /* APBV_H_ */
