// Merge of partial attention results by their log-sum-exp (Eq. 5: A_qr = Merge({A_qr^(h), lse^(h)})).
//
// Each part h is softmax attention of the same queries over its own set of keys, with
// lse_h = log sum exp of its scaled logits.  Over the union of disjoint key sets the exact result is
//   A = sum_h w_h A_h / sum_h w_h,   w_h = exp(lse_h - max_h lse_h),   lse = max_h lse_h + log sum_h w_h.
// Memory-bound: every partial output is read once (16 bytes per lane per part), fp32 arithmetic.
#include "apbv_common.h"

namespace apbv {
namespace {

// LP lanes share one 16-byte output chunk: lane `sub` takes parts sub, sub + LP, ...; the lanes' maxima and
// weighted sums are combined with shuffles.  LP = 8 turns the chain of dependent loads of a many-part merge
// (a key split into tens of ranges) into a few loads per lane; LP = 1 is the plain loop for a handful of parts.
template <int D, int LP>
__global__ __launch_bounds__(256) void merge_lse_kernel(const MergeParams p) {
  constexpr int KC = D / 8;
  const int64_t thread = (int64_t)blockIdx.x * 256 + threadIdx.x;
  const int sub = (int)(thread % LP);
  int64_t item = thread / LP;                                           // over batch * rows * hq * KC
  const int64_t n_items = (int64_t)p.batch * p.rows * p.hq * KC;
  const bool live = item < n_items;
  if (!live) item = n_items - 1;                                        // keep the lane for the shuffles; it writes nothing
  const int c = (int)(item % KC);
  const int64_t rh = item / KC;                                         // (b * rows + row) * hq + head
  const int h = (int)(rh % p.hq);
  const int64_t brow = rh / p.hq;
  const int64_t row = brow % p.rows, b = brow / p.rows;
  const int64_t lse_idx = (b * p.hq + h) * p.rows + row;

  float m = -INFINITY;
  // (unrolled so that several parts' loads are in flight)
#pragma unroll 4
  for (int s = sub; s < p.n_parts; s += LP) m = fmaxf(m, p.parts_lse[s * p.stride_lse + lse_idx]);
#pragma unroll
  for (int d = 1; d < LP; d <<= 1) m = fmaxf(m, __shfl_xor(m, d));
  float acc[8];
#pragma unroll
  for (int e = 0; e < 8; ++e) acc[e] = 0.f;
  float wsum = 0.f;
  if (m > -INFINITY) {                                                  // uniform over the LP lanes of an item
#pragma unroll 4
    for (int s = sub; s < p.n_parts; s += LP) {
      const float w = __expf(p.parts_lse[s * p.stride_lse + lse_idx] - m);     // exp(-inf) = 0: empty parts drop out
      const u32x4 x = *reinterpret_cast<const u32x4*>(p.parts_out + s * p.stride_out + rh * D + 8 * c);
      wsum += w;
#pragma unroll
      for (int e = 0; e < 4; ++e) {
        acc[2 * e] = __builtin_fmaf(w, __uint_as_float(x[e] << 16), acc[2 * e]);
        acc[2 * e + 1] = __builtin_fmaf(w, __uint_as_float(x[e] & 0xffff0000u), acc[2 * e + 1]);
      }
    }
  }
#pragma unroll
  for (int d = 1; d < LP; d <<= 1) {
    wsum += __shfl_xor(wsum, d);
#pragma unroll
    for (int e = 0; e < 8; ++e) acc[e] += __shfl_xor(acc[e], d);
  }
  if (!live || sub != 0) return;
  const float inv = wsum > 0.f ? 1.0f / wsum : 0.f;
  u32x4 o;
#pragma unroll
  for (int e = 0; e < 4; ++e) {
    f32x2 xy = {acc[2 * e] * inv, acc[2 * e + 1] * inv};
    bf16x2 bb = __builtin_convertvector(xy, bf16x2);
    o[e] = __builtin_bit_cast(uint32_t, bb);
  }
  *reinterpret_cast<u32x4*>(p.out + rh * D + 8 * c) = o;
  if (p.lse_out != nullptr && c == 0) p.lse_out[lse_idx] = wsum > 0.f ? m + __logf(wsum) : -INFINITY;
}

}  // namespace

template <int LP>
static apbv_status launch_merge_variant(const MergeParams& p, hipStream_t stream) {
  const int64_t threads = (int64_t)p.batch * p.rows * p.hq * (p.d / 8) * LP;
  const int64_t blocks = (threads + 255) / 256;
  if (blocks > 0x7fffffff) return APBV_ERR_UNSUPPORTED;
  Launcher launch(stream);
  if (p.d == 128)
    launch(merge_lse_kernel<128, LP>, dim3((unsigned)blocks), dim3(256), 0, p);
  else if (p.d == 64)
    launch(merge_lse_kernel<64, LP>, dim3((unsigned)blocks), dim3(256), 0, p);
  else
    return APBV_ERR_UNSUPPORTED;
  return launch.status();
}

apbv_status launch_merge_lse(const MergeParams& p, hipStream_t stream) {
  return p.n_parts >= 8 ? launch_merge_variant<8>(p, stream) : launch_merge_variant<1>(p, stream);
}

}  // namespace apbv
