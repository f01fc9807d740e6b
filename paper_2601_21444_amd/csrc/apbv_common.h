// Shared device/host declarations of the gfx950 library (internal; the public ABI is include/apbv.h).
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>
#include <tuple>
#include <utility>
#include "apbv.h"
#include "attention_schedule.h"
#include "host_validation.h"

namespace apbv {

typedef uint16_t bf16_t;                                                  // bf16 bit pattern
typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8;                // one MFMA A/B operand
typedef __attribute__((ext_vector_type(2))) __bf16 bf16x2;
typedef __attribute__((ext_vector_type(16))) float f32x16;                // one 32x32 MFMA accumulator
typedef __attribute__((ext_vector_type(4))) float f32x4;
typedef __attribute__((ext_vector_type(2))) float f32x2;
typedef __attribute__((ext_vector_type(4))) uint32_t u32x4;               // 16 bytes
typedef __attribute__((ext_vector_type(2))) uint32_t u32x2;               // 8 bytes

// Kernel launches of one entry point.  The status kept is that of THESE launches, as returned by the launch call
// itself: hipGetLastError() would also return -- and clear -- an error left behind by an unrelated earlier runtime
// call of the thread.  After a refused launch nothing further is launched.
class Launcher {
 public:
  explicit Launcher(hipStream_t stream) : stream_(stream) {}
  template <typename... P, typename... A>
  void operator()(void (*kernel)(P...), dim3 grid, dim3 block, size_t lds_bytes, A&&... args) {
    static_assert(sizeof...(P) == sizeof...(A), "one argument per kernel parameter");
    if (err_ != hipSuccess) return;
    std::tuple<P...> vals(static_cast<P>(args)...);          // each argument in its parameter's exact type
    err_ = launch(reinterpret_cast<const void*>(kernel), grid, block, lds_bytes, vals, std::index_sequence_for<P...>{});
  }
  bool ok() const { return err_ == hipSuccess; }
  apbv_status status() const { return err_ == hipSuccess ? APBV_OK : APBV_ERR_LAUNCH; }

 private:
  template <typename Tuple, size_t... I>
  hipError_t launch(const void* fn, dim3 grid, dim3 block, size_t lds_bytes, Tuple& vals, std::index_sequence<I...>) {
    void* ptrs[] = {static_cast<void*>(&std::get<I>(vals))...};
    return hipLaunchKernel(fn, grid, block, ptrs, lds_bytes, stream_);
  }
  hipStream_t stream_;
  hipError_t err_ = hipSuccess;
};

// A [tokens, heads, d] bf16 view already offset to nothing: base pointer plus element strides.
struct View {
  const bf16_t* ptr;
  int64_t tokens;
  int64_t st;   // stride_token
  int64_t sh;   // stride_head
  int64_t sb;   // stride_batch
};

inline View to_view(const apbv_tensor& t) {
  View v;
  v.ptr = static_cast<const bf16_t*>(t.ptr);
  v.tokens = t.tokens;
  v.st = t.stride_token;
  v.sh = t.stride_head;
  v.sb = t.stride_batch;
  return v;
}

// ---- attention --------------------------------------------------------------------------------
struct AttnParams {
  View q;                 // [L, Hq, d]
  View k_seg[3];          // anchor, passing, local  [*, Hkv, d]
  View v_seg[3];
  bf16_t* out;            // [batch, L, Hq, d]
  float* lse;             // [batch, Hq, L] or nullptr
  int64_t L;              // query rows (= local block length when there is a local segment)
  int64_t l_a;            // anchor length
  int64_t n_vis;          // l_a + n_p: keys visible to every query
  int64_t s_kv;           // n_vis + local keys (L of them, or none)
  int batch, hq, hkv, group;
  float scale_log2;       // softmax_scale * log2(e)
  // key split: n_splits ranges of tiles_per_split 64-key tiles; split s writes its partial result at
  // out + s*split_stride_out and lse + s*split_stride_lse (n_splits == 1: the plain call)
  int n_splits, tiles_per_split;
  int64_t split_stride_out, split_stride_lse;
};

apbv_status launch_host_attention(const AttnParams& p, int head_dim, hipStream_t stream);

// Several attention problems (batch 1, one key range each, same head counts) in one launch.  The caller fills
// item[] and n_items; the launcher fills the schedule.
struct AttnGroupParams {
  AttnParams item[kMaxGroupItems];
  GroupSchedule sched;
  int n_items;
};
apbv_status launch_host_attention_group(AttnGroupParams& gp, int head_dim, hipStream_t stream);

// ---- merge of partial attention results -------------------------------------------------------
struct MergeParams {
  const bf16_t* parts_out;   // [n_parts][batch, rows, Hq, d]
  const float* parts_lse;    // [n_parts][batch, Hq, rows]
  int64_t stride_out;        // elements between parts
  int64_t stride_lse;
  bf16_t* out;               // [batch, rows, Hq, d]
  float* lse_out;            // optional [batch, Hq, rows]
  int64_t rows;
  int n_parts, hq, d, batch;
};
apbv_status launch_merge_lse(const MergeParams& p, hipStream_t stream);

// ---- compression ------------------------------------------------------------------------------
struct CompressParams {
  View q_probe;           // [n_q, Hq, d]
  View k;                 // [L, Hkv, d]
  View v;
  int64_t L, l_p;
  int batch, hq, hkv, group, d;
  int32_t* idx_out;       // [batch, Hkv, l_p]
  bf16_t* k_c;            // [batch, l_p, Hkv, d]
  bf16_t* v_c;
  double* scores_out;     // optional [batch, Hkv, L]
  void* workspace;
  size_t workspace_bytes;
  int reducer;            // apbv_reducer: how the score matrix becomes one score per key
  float scale_log2;       // softmax_scale * log2(e), for APBV_REDUCE_SOFTMAX_SUM
  bool use_static_scratch;   // workspace = the library's static device array (workspace / workspace_bytes ignored)
};
constexpr size_t kStaticScratchBytes = APBV_NOALLOC_MAX_WORKSPACE_BYTES;   // size of that array

// workspace = [selection workspace | row statistics of the matrix reductions]
size_t compress_workspace_bytes(int batch, int hkv, int d, int64_t L, int64_t l_p);
size_t matrix_scores_workspace_bytes(int reducer, int batch, int hkv, int64_t n_rows, int64_t L);
apbv_status launch_compress(const CompressParams& p, hipStream_t stream);
apbv_status check_matrix_scores(const CompressParams& p);
apbv_status launch_matrix_scores(const CompressParams& p, double* scores, void* stats_ws, hipStream_t stream);

}  // namespace apbv
