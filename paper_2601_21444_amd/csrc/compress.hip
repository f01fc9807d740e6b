// KV compression for gfx950 (Sec. 3.3; Alg. 1 "Identify Essential KVs" and "Send Block's Essential
// KVs"): score every local key, keep the l_p best per KV head, gather them.
//
// The score of key j for KV head v is the sum of the raw logits Q_qr[t, v*G+g] . K[j, v] over all
// query-block rows t and the G query heads of the group.  The sum is linear in the query, so it is
// evaluated as  q_bar[v] . K[j, v]  with the pooled query q_bar[v] = sum_t sum_g Q_qr[t, v*G+g]:
// one streaming pass over K, bound by HBM bandwidth.  Accumulation is in float64 so that the ranking
// agrees with a float64 evaluation (float32 accumulation flips near-equal neighbours).
//
// Four launches on the caller's stream:
//   pool_query_kernel   partial sums of q_bar (float64), up to 8 row ranges per pooled query
//                                                                         [splits x Hkv x batch workgroups]
//   score_kernel        s[v, j], 16-byte coalesced reads of K rows; adds the partial sums of q_bar as it starts;
//                       scores stored through to memory as it runs         [L/64 x Hkv x batch]
//   select_kernel       bucket sort by value of the scores above the l_p-th largest (exact fallback: radix select
//                       + bitonic sort), into (score descending, index ascending) order   [Hkv x batch]
//   gather_kernel       K_c, V_c rows                                     [l_p*Hkv/.. x batch]
#include <mutex>
#include "apbv_common.h"

namespace apbv {
namespace {

constexpr int kSelectThreads = 1024;

__device__ __forceinline__ double bf16_to_f64(uint32_t bits16) {
  return (double)__uint_as_float(bits16 << 16);
}

// A float64 moved across lanes by a DPP control (two 32-bit moves).  Controls: exchanges inside a quad, and
// rotations of a 16-lane row (lane i reads lane i-n of its row).
constexpr int kDppXor1 = 0xB1;    // quad_perm [1,0,3,2]
constexpr int kDppXor2 = 0x4E;    // quad_perm [2,3,0,1]
constexpr int kDppRor4 = 0x124;   // row_ror:4
constexpr int kDppRor8 = 0x128;   // row_ror:8
template <int CTRL>
__device__ __forceinline__ double dpp_f64(double x) {
  int lo = __double2loint(x), hi = __double2hiint(x);
  lo = __builtin_amdgcn_update_dpp(0, lo, CTRL, 0xf, 0xf, false);
  hi = __builtin_amdgcn_update_dpp(0, hi, CTRL, 0xf, 0xf, false);
  return __hiloint2double(hi, lo);
}

// ------------------------------------------------------------------------------------------------
// q_bar[b, v, c] = sum_g sum_t Q_qr[b, t, v*G+g, c]   (float64; the addends are bf16 so the sum is
// exact or within an ulp whatever the order).  The n_q * G probe rows of a (KV head, batch item) are
// cut into n_split equal ranges, one workgroup each (so that even a single item spreads over several
// compute units); a workgroup writes the partial sum of its range and the scoring kernel adds the
// partial sums in index order.  D/8 lanes per probe row (16-byte loads), T/(D/8) rows in flight (T = 1024 threads
// where a range is long enough to feed them four loads each, 256 otherwise).
template <int D, int T>
__global__ __launch_bounds__(T) void pool_query_kernel(View q, int64_t n_q, int group, double* qpart, int hkv, int n_split) {
  constexpr int KC = D / 8;
  constexpr int R = T / KC;                    // row groups
  __shared__ double part[T / 64][D];
  const int sp = blockIdx.x, v = blockIdx.y, b = blockIdx.z;
  const int c8 = threadIdx.x % KC, rg = threadIdx.x / KC;
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const bf16_t* base = q.ptr + (int64_t)b * q.sb + (int64_t)v * group * q.sh + 8 * c8;
  double acc[8];
#pragma unroll
  for (int e = 0; e < 8; ++e) acc[e] = 0.0;
  const int n_rows = (int)(n_q * group);
  const int per = (n_rows + n_split - 1) / n_split;
  const int r_begin = sp * per, r_end = r_begin + per < n_rows ? r_begin + per : n_rows;
  // rows (t, g) in steps of R, four loads in flight; (t, g) advance without divisions in the loop
  const int dt = R / group, dg = R % group;
  int t = (r_begin + rg) / group, g = (r_begin + rg) % group;
  auto advance = [&]() {
    t += dt;
    g += dg;
    if (g >= group) {
      g -= group;
      ++t;
    }
  };
  for (int rr = r_begin + rg; rr < r_end; rr += 4 * R) {
    u32x4 x[4];
#pragma unroll
    for (int u = 0; u < 4; ++u) {
      x[u] = u32x4{0u, 0u, 0u, 0u};                       // +0.0: adds nothing
      if (rr + u * R < r_end) x[u] = *reinterpret_cast<const u32x4*>(base + (int64_t)t * q.st + (int64_t)g * q.sh);
      advance();
    }
#pragma unroll
    for (int u = 0; u < 4; ++u)
#pragma unroll
      for (int e = 0; e < 4; ++e) {
        acc[2 * e] += bf16_to_f64(x[u][e] & 0xffffu);
        acc[2 * e + 1] += bf16_to_f64(x[u][e] >> 16);
      }
  }
#pragma unroll
  for (int e = 0; e < 8; ++e) {
#pragma unroll
    for (int m = KC; m < 64; m <<= 1) acc[e] += __shfl_xor(acc[e], m);
  }
  if (lane < KC) {
#pragma unroll
    for (int e = 0; e < 8; ++e) part[wave][8 * c8 + e] = acc[e];
  }
  __syncthreads();
  if (threadIdx.x < D) {
    double sum = 0.0;
#pragma unroll
    for (int w = 0; w < T / 64; ++w) sum += part[w][threadIdx.x];
    qpart[(((int64_t)b * hkv + v) * n_split + sp) * D + threadIdx.x] = sum;
  }
}

// ------------------------------------------------------------------------------------------------
// s[b, v, j] = q_bar[b, v, :] . K[b, j, v, :].  D/8 lanes per key row, each lane 8 elements (one
// 16-byte load), fixed summation order per row so identical rows get identical scores.
template <int D>
__global__ __launch_bounds__(256) void score_kernel(View k, int64_t L, const double* __restrict__ qpart, int n_split,
                                                    double* __restrict__ s_ws, double* __restrict__ s_out,
                                                    int hkv, int rows_per_block) {
  constexpr int LPR = D / 8;               // lanes per row
  constexpr int RPS = 256 / LPR;           // rows per step of the workgroup
  constexpr int UNROLL = 4;
  static_assert(LPR == 8 || LPR == 16, "the cross-lane reduction below is written for 8 or 16 lanes per row");
  const int v = blockIdx.y, b = blockIdx.z;
  const int c = threadIdx.x % LPR;
  const int rsub = threadIdx.x / LPR;
  __shared__ double qs[D];
  const double* qb = qpart + ((int64_t)b * hkv + v) * n_split * D;      // n_split partial sums of the pooled query
  const bf16_t* base = k.ptr + (int64_t)b * k.sb + (int64_t)v * k.sh + 8 * c;
  const int64_t out_base = ((int64_t)b * hkv + v) * L;
  const int64_t r_begin = (int64_t)blockIdx.x * rows_per_block;
  const int64_t r_end = (r_begin + rows_per_block < L) ? r_begin + rows_per_block : L;

  for (int64_t r0 = r_begin; r0 < r_end; r0 += RPS * UNROLL) {
    u32x4 x[UNROLL];
#pragma unroll
    for (int u = 0; u < UNROLL; ++u) {
      const int64_t j = r0 + u * RPS + rsub;
      u32x4 z = {0u, 0u, 0u, 0u};
      if (j < r_end) z = __builtin_nontemporal_load(reinterpret_cast<const u32x4*>(base + j * k.st));
      x[u] = z;
    }
    // The pooled query reaches the lanes through LDS -- one 16-byte load by D/2 lanes per workgroup, behind the
    // key loads, instead of four loads per lane in front of them.
    if (r0 == r_begin) {
      if (threadIdx.x < D / 2) {
        // all partial sums are fetched before the first addition (independent loads), then added in index order
        double2 part[kPoolSplitMax];
#pragma unroll
        for (int sp = 0; sp < kPoolSplitMax; ++sp) {
          part[sp] = double2{0.0, 0.0};
          if (sp < n_split) part[sp] = *reinterpret_cast<const double2*>(qb + sp * D + 2 * threadIdx.x);
        }
        double2 t = part[0];
#pragma unroll
        for (int sp = 1; sp < kPoolSplitMax; ++sp)
          if (sp < n_split) {
            t.x += part[sp].x;
            t.y += part[sp].y;
          }
        qs[2 * threadIdx.x] = t.x;
        qs[2 * threadIdx.x + 1] = t.y;
      }
      __syncthreads();
    }
    double qv[8];
#pragma unroll
    for (int e = 0; e < 8; ++e) qv[e] = qs[8 * c + e];
    double a[UNROLL];
#pragma unroll
    for (int u = 0; u < UNROLL; ++u) {
      double acc = 0.0;
#pragma unroll
      for (int e = 0; e < 4; ++e) {
        acc = __builtin_fma(qv[2 * e], bf16_to_f64(x[u][e] & 0xffffu), acc);
        acc = __builtin_fma(qv[2 * e + 1], bf16_to_f64(x[u][e] >> 16), acc);
      }
      a[u] = acc;
    }
    // Reduce the four rows over the row's lanes as a reduce-scatter: after the two exchanges inside a quad each
    // lane holds one row's sum over its quad, two rotations by 4 and 8 lanes finish it.  Every row takes the same
    // summation tree (the adds commute), so identical rows get identical scores.
    const bool odd1 = (c & 1) != 0, odd2 = (c & 2) != 0;
    double keep0 = odd1 ? a[2] : a[0], keep1 = odd1 ? a[3] : a[1];
    keep0 += dpp_f64<kDppXor1>(odd1 ? a[0] : a[2]);
    keep1 += dpp_f64<kDppXor1>(odd1 ? a[1] : a[3]);
    double acc = odd2 ? keep1 : keep0;
    acc += dpp_f64<kDppXor2>(odd2 ? keep0 : keep1);
    acc += dpp_f64<kDppRor4>(acc);
    if (LPR == 16) acc += dpp_f64<kDppRor8>(acc);
    const int u = (odd1 ? 2 : 0) + (odd2 ? 1 : 0);     // the row this lane ended up with
    const int64_t j = r0 + u * RPS + rsub;
    if (c >= LPR - 4 && j < r_end) {                   // the last quad of the row's lanes holds complete sums
      // written through to memory as the kernel runs (device-scope store): left to the write-back cache, the
      // scores of a large batch are flushed when the kernel ends, with nothing left to overlap the flush
      __hip_atomic_store(reinterpret_cast<long long*>(s_ws + out_base + j), __double_as_longlong(acc), __ATOMIC_RELAXED,
                         __HIP_MEMORY_SCOPE_AGENT);
      if (s_out) s_out[out_base + j] = acc;
    }
  }
}

// ------------------------------------------------------------------------------------------------
// Order-preserving key: larger score <=> larger unsigned key; -0.0 and +0.0 map to the same key.
__device__ __forceinline__ uint64_t score_key(double s) {
  uint64_t b = (uint64_t)__double_as_longlong(s);
  if ((b << 1) == 0) b = 0;
  return (b >> 63) ? ~b : (b | 0x8000000000000000ull);
}

// (key descending, index ascending)
__device__ __forceinline__ bool precedes(uint64_t ka, uint32_t ia, uint64_t kb, uint32_t ib) {
  return ka > kb || (ka == kb && ia < ib);
}

constexpr int kBins = 2048;                    // value buckets of the fast selection path

constexpr uint32_t kMaxBinRank = 128;          // largest bucket the rank-by-comparison step accepts

struct SelectShared {
  uint32_t hist[kBins];       // entries per bucket
  uint32_t base[kBins];       // entries in higher buckets (output offset of the bucket)
  uint32_t fill[kBins];       // scatter cursor per bucket
  uint64_t prefix;
  uint32_t need, bucket, cnt, n_cand, t_bin, crowded;
  uint32_t wave_tot[kSelectThreads / 64];
  float red_lo[kSelectThreads / 64], red_hi[kSelectThreads / 64];
};

// Wave-wide combinations on the DPP data path (no LDS traffic): shifts inside the 16-lane rows, then lane 15 of
// a row into the next row and lane 31 into the upper half.  A lane whose source lies outside keeps `self`.
constexpr int kDppShr1 = 0x111, kDppShr2 = 0x112, kDppShr4 = 0x114, kDppShr8 = 0x118;   // row_shr:n
constexpr int kDppBcast15 = 0x142, kDppBcast31 = 0x143;
template <int CTRL, int ROW_MASK>
__device__ __forceinline__ uint32_t dpp_or_self(uint32_t self, uint32_t x) {
  return (uint32_t)__builtin_amdgcn_update_dpp((int)self, (int)x, CTRL, ROW_MASK, 0xf, false);
}

// Inclusive prefix sum over the 64 lanes of a wave.
__device__ __forceinline__ uint32_t wave_scan_incl(uint32_t x) {
  x += dpp_or_self<kDppShr1, 0xf>(0u, x);
  x += dpp_or_self<kDppShr2, 0xf>(0u, x);
  x += dpp_or_self<kDppShr4, 0xf>(0u, x);
  x += dpp_or_self<kDppShr8, 0xf>(0u, x);
  x += dpp_or_self<kDppBcast15, 0xa>(0u, x);
  x += dpp_or_self<kDppBcast31, 0xc>(0u, x);
  return x;
}

// op over the 64 lanes of a wave, the result in every lane (lane 63 collects it, one scalar read spreads it).
template <typename Op>
__device__ __forceinline__ uint32_t wave_reduce_bits(uint32_t x, Op op) {
  x = op(x, dpp_or_self<kDppShr1, 0xf>(x, x));
  x = op(x, dpp_or_self<kDppShr2, 0xf>(x, x));
  x = op(x, dpp_or_self<kDppShr4, 0xf>(x, x));
  x = op(x, dpp_or_self<kDppShr8, 0xf>(x, x));
  x = op(x, dpp_or_self<kDppBcast15, 0xa>(x, x));
  x = op(x, dpp_or_self<kDppBcast31, 0xc>(x, x));
  return (uint32_t)__builtin_amdgcn_readlane((int)x, 63);
}
__device__ __forceinline__ float wave_min(float x) {
  return __uint_as_float(wave_reduce_bits(__float_as_uint(x), [](uint32_t a, uint32_t b) {
    return __float_as_uint(fminf(__uint_as_float(a), __uint_as_float(b)));
  }));
}
__device__ __forceinline__ float wave_max(float x) {
  return __uint_as_float(wave_reduce_bits(__float_as_uint(x), [](uint32_t a, uint32_t b) {
    return __float_as_uint(fmaxf(__uint_as_float(a), __uint_as_float(b)));
  }));
}

// Inclusive scan of one value per thread over the whole workgroup (1024 threads); returns the
// inclusive prefix, *total gets the workgroup sum.  kFresh: wave_tot has not been used since the last barrier.
template <bool kFresh = false>
__device__ __forceinline__ uint32_t block_scan_incl(uint32_t x, SelectShared& sh, uint32_t* total) {
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const uint32_t incl = wave_scan_incl(x);
  if (!kFresh) __syncthreads();         // wave_tot may still be read from a previous use
  if (lane == 63) sh.wave_tot[wave] = incl;
  __syncthreads();
  uint32_t base = 0, tot = 0;
#pragma unroll
  for (int w = 0; w < kSelectThreads / 64; ++w) {
    const uint32_t t = sh.wave_tot[w];
    if (w < wave) base += t;
    tot += t;
  }
  *total = tot;
  return incl + base;
}

// Bitonic sort of n_sort (a power of two) entries into (key descending, index ascending) order.
__device__ __forceinline__ void bitonic_sort(uint64_t* skeys, uint32_t* sidx, int64_t n_sort64) {
  const uint32_t tid = threadIdx.x;
  const uint32_t n_sort = (uint32_t)n_sort64, half = n_sort >> 1;
  for (uint32_t k = 2; k <= n_sort; k <<= 1) {
    for (uint32_t j = k >> 1, lj = 31 - __builtin_clz(j); j > 0; j >>= 1, --lj) {
      for (uint32_t pidx = tid; pidx < half; pidx += kSelectThreads) {
        const uint32_t i = ((pidx >> lj) << (lj + 1)) | (pidx & (j - 1));
        const uint32_t q = i + j;
        const bool up = (i & k) == 0;          // this run is sorted "first precedes"
        const uint64_t ka = skeys[i], kb = skeys[q];
        const uint32_t ia = sidx[i], ib = sidx[q];
        const bool in_order = precedes(ka, ia, kb, ib);
        if (in_order != up) {
          skeys[i] = kb;
          skeys[q] = ka;
          sidx[i] = ib;
          sidx[q] = ia;
        }
      }
      __syncthreads();
    }
  }
}

// Fast path: a bucket sort by VALUE.  A monotone map sends every score to one of kBins buckets of equal width
// between the minimum and the maximum (computed in single precision: only the order matters).  A suffix scan of
// the bucket counts gives each bucket its output offset and finds the bucket that holds the l_p-th largest score;
// the entries of that bucket and of all higher ones are scattered into bucket-grouped order, and each entry then
// finds its rank inside its (small) bucket by direct comparison of the full 64-bit keys and indices.  Because the
// map is monotone, bucket order followed by (key descending, index ascending) inside a bucket is the global order,
// ties included.  Returns false (nothing written) if the candidates do not fit `cap` or a bucket is too crowded to
// rank by comparison; the caller then takes the exact radix path.
__device__ __forceinline__ bool bucket_rank_select(const double* __restrict__ s, int64_t L, int64_t l_p, int64_t cap,
                                                   uint64_t* skeys, uint32_t* sidx, uint16_t* sbin,
                                                   int32_t* __restrict__ idx_out, SelectShared& sh) {
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  constexpr int kPer = 16;                                   // scores kept in registers per thread
  const bool resident = L <= (int64_t)kPer * kSelectThreads;
  double sc[kPer];
  uint32_t bins[kPer];                                       // bucket | arrival order in the bucket << 11
  if (resident) {
#pragma unroll
    for (int u = 0; u < kPer; ++u) {
      const int64_t j = tid + (int64_t)u * kSelectThreads;
      sc[u] = j < L ? s[j] : 0.0;
    }
  }
  // minimum and maximum, in single precision (the conversion is monotone, which is all the map needs)
  float lo = INFINITY, hi = -INFINITY;
  if (resident) {
#pragma unroll
    for (int u = 0; u < kPer; ++u)
      if (tid + (int64_t)u * kSelectThreads < L) {
        const float x = (float)sc[u];
        lo = fminf(lo, x);
        hi = fmaxf(hi, x);
      }
  } else {
    for (int64_t j = tid; j < L; j += kSelectThreads) {
      const float x = (float)s[j];
      lo = fminf(lo, x);
      hi = fmaxf(hi, x);
    }
  }
  lo = wave_min(lo);
  hi = wave_max(hi);
  if (lane == 0) {
    sh.red_lo[wave] = lo;
    sh.red_hi[wave] = hi;
  }
  for (int i = tid; i < kBins; i += kSelectThreads) {
    sh.hist[i] = 0;
    sh.fill[i] = 0;
  }
  if (tid == 0) sh.crowded = 0;
  __syncthreads();
#pragma unroll
  for (int w = 0; w < kSelectThreads / 64; ++w) {
    lo = fminf(lo, sh.red_lo[w]);
    hi = fmaxf(hi, sh.red_hi[w]);
  }
  const float inv = (float)kBins / (hi - lo);
  if (!(inv > 0.0f) || !(inv < 1.0e30f)) return false;       // all scores equal in single precision (or range overflow)
  // rounding, subtraction of lo, multiplication by a positive constant and truncation are all monotone
  auto bin_of = [&](double x) {
    const int b = (int)(((float)x - lo) * inv);
    return (uint32_t)(b > kBins - 1 ? kBins - 1 : b);
  };
  // histogram; the count an atomic returns is the entry's arrival order inside its bucket, kept (with the bucket)
  // for the scatter below so that the resident case needs no second pass of atomics
  if (resident) {
#pragma unroll
    for (int u = 0; u < kPer; ++u) {
      bins[u] = 0;
      if (tid + (int64_t)u * kSelectThreads < L) {
        const uint32_t b = bin_of(sc[u]);
        bins[u] = b | (atomicAdd(&sh.hist[b], 1u) << 11);
      }
    }
  } else {
    for (int64_t j = tid; j < L; j += kSelectThreads) atomicAdd(&sh.hist[bin_of(s[j])], 1u);
  }
  __syncthreads();
  // thread t owns buckets kBins-1-2t and kBins-2-2t (descending): suffix counts by an inclusive scan
  const int b0 = kBins - 1 - 2 * tid, b1 = kBins - 2 - 2 * tid;
  const uint32_t c0 = sh.hist[b0], c1 = sh.hist[b1];
  uint32_t total;
  const uint32_t incl = block_scan_incl<true>(c0 + c1, sh, &total);
  const uint32_t excl = incl - (c0 + c1);
  sh.base[b0] = excl;
  sh.base[b1] = excl + c0;
  if (excl < (uint32_t)l_p && (uint32_t)l_p <= incl) {
    const bool first = (uint32_t)l_p <= excl + c0;
    sh.t_bin = first ? b0 : b1;
    sh.n_cand = first ? excl + c0 : incl;
  }
  __syncthreads();
  const uint32_t n_cand = sh.n_cand;
  const int t_bin = (int)sh.t_bin;
  if ((int64_t)n_cand > cap) return false;
  // a candidate bucket too crowded to rank by comparison: seen by every thread after the scatter's barrier
  if ((b0 >= t_bin && c0 > kMaxBinRank) || (b1 >= t_bin && c1 > kMaxBinRank)) sh.crowded = 1;
  // scatter the candidates into bucket-grouped order.  Every wave walks all kPer iterations for the few lanes
  // that hold a candidate, so the body is two stores (index, raw score); key and bucket follow below.
  if (resident) {
    // Every bucket offset is fetched before the first store.  Lanes without a candidate all read one and the
    // same word (a broadcast), so that only the few candidates' reads can collide on an LDS bank.
    uint32_t pos[kPer];
#pragma unroll
    for (int u = 0; u < kPer; ++u) {
      const uint32_t b = bins[u] & (uint32_t)(kBins - 1);
      pos[u] = sh.base[(int)b >= t_bin ? b : (uint32_t)(kBins - 1)] + (bins[u] >> 11);
    }
#pragma unroll
    for (int u = 0; u < kPer; ++u) {
      const uint32_t j = (uint32_t)tid + (uint32_t)u * kSelectThreads;
      if (j < (uint32_t)L && (int)(bins[u] & (uint32_t)(kBins - 1)) >= t_bin) {
        sidx[pos[u]] = j;
        skeys[pos[u]] = (uint64_t)__double_as_longlong(sc[u]);
      }
    }
  } else {
    for (int64_t j = tid; j < L; j += kSelectThreads) {
      const double x = s[j];
      const uint32_t b = bin_of(x);
      if ((int)b >= t_bin) {
        const uint32_t pos = sh.base[b] + atomicAdd(&sh.fill[b], 1u);
        sidx[pos] = (uint32_t)j;
        skeys[pos] = (uint64_t)__double_as_longlong(x);
      }
    }
  }
  __syncthreads();
  // the owner of a candidate position turns the raw score into its key and bucket, in place
  for (uint32_t pos = tid; pos < n_cand; pos += kSelectThreads) {
    const double x = __longlong_as_double((long long)skeys[pos]);
    skeys[pos] = score_key(x);
    sbin[pos] = (uint16_t)bin_of(x);
  }
  __syncthreads();
  if (sh.crowded) return false;
  // rank inside the bucket, write the index at its final position
  const int64_t out_base = ((int64_t)blockIdx.y * gridDim.x + blockIdx.x) * l_p;
  for (uint32_t pos = tid; pos < n_cand; pos += kSelectThreads) {
    const uint32_t b = sbin[pos];
    const uint32_t first = sh.base[b], cnt = sh.hist[b];
    const uint64_t key = skeys[pos];
    const uint32_t idx = sidx[pos];
    uint32_t rank = 0;
    const uint32_t end = first + cnt;                        // cnt >= 1: the entry itself
    for (uint32_t q = first; q < end; q += 4) {              // four entries' reads in flight
      uint64_t kq[4];
      uint32_t iq[4];
#pragma unroll
      for (int e = 0; e < 4; ++e) {
        const uint32_t qq = q + e < end ? q + e : end - 1;
        kq[e] = skeys[qq];
        iq[e] = sidx[qq];
      }
#pragma unroll
      for (int e = 0; e < 4; ++e) rank += (q + e < end && precedes(kq[e], iq[e], key, idx)) ? 1u : 0u;
    }
    if (first + rank < (uint32_t)l_p) idx_out[out_base + first + rank] = (int32_t)idx;
  }
  return true;
}

// Exact path for any input: radix select of the l_p-th largest key, most significant byte first, then
// collection of the l_p winners (ties at the threshold by ascending index).
__device__ __forceinline__ void radix_collect(const double* __restrict__ s, int64_t L, int64_t l_p, uint64_t* skeys,
                                              uint32_t* sidx, SelectShared& sh) {
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  // after 8 passes `prefix` is the l_p-th largest key and `need` says how many keys equal to it belong
  // to the result
  uint64_t prefix = 0;
  uint32_t need = (uint32_t)l_p;
  uint32_t bucket = 0;           // number of keys equal to the final prefix
  for (int pass = 0; pass < 8; ++pass) {
    const int shift = 56 - 8 * pass;
    __syncthreads();
    if (tid < 256) sh.hist[tid] = 0;
    __syncthreads();
    for (int64_t j = tid; j < L; j += kSelectThreads) {
      const uint64_t key = score_key(s[j]);
      if (pass == 0 || (key >> (shift + 8)) == prefix) atomicAdd(&sh.hist[(key >> shift) & 255], 1u);
    }
    __syncthreads();
    if (wave == 0) {
      // lane l owns digits 255-4l .. 252-4l (descending); find the digit holding the need-th largest
      uint32_t c4[4], tot = 0;
#pragma unroll
      for (int q = 0; q < 4; ++q) {
        c4[q] = sh.hist[255 - 4 * lane - q];
        tot += c4[q];
      }
      const uint32_t incl = wave_scan_incl(tot);
      uint32_t excl = incl - tot;
      if (excl < need && need <= incl) {
#pragma unroll
        for (int q = 0; q < 4; ++q) {
          if (excl < need && need <= excl + c4[q]) {
            sh.prefix = (prefix << 8) | (uint64_t)(255 - 4 * lane - q);
            sh.need = need - excl;
            sh.bucket = c4[q];
          }
          excl += c4[q];
        }
      }
    }
    __syncthreads();
    prefix = sh.prefix;
    need = sh.need;
    bucket = sh.bucket;
  }
  const uint64_t kth = prefix;
  const uint32_t n_gt = (uint32_t)l_p - need;     // keys strictly above the threshold

  if (tid == 0) sh.cnt = 0;
  __syncthreads();
  if (bucket == need) {
    // every key equal to the threshold is taken: no ordering constraint while collecting
    for (int64_t j = tid; j < L; j += kSelectThreads) {
      const uint64_t key = score_key(s[j]);
      if (key >= kth) {
        const uint32_t pos = atomicAdd(&sh.cnt, 1u);
        skeys[pos] = key;
        sidx[pos] = (uint32_t)j;
      }
    }
  } else {
    // more equal keys than needed: take the `need` lowest indices.  Each thread scans a contiguous
    // index range; an exclusive scan of the per-thread tie counts gives each tie its rank by index.
    const int64_t chunk = (L + kSelectThreads - 1) / kSelectThreads;
    const int64_t lo = (int64_t)tid * chunk, hi = (lo + chunk < L) ? lo + chunk : L;
    uint32_t n_eq = 0;
    for (int64_t j = lo; j < hi; ++j) n_eq += (score_key(s[j]) == kth);
    uint32_t total;
    uint32_t rank = block_scan_incl(n_eq, sh, &total) - n_eq;
    for (int64_t j = lo; j < hi; ++j) {
      const uint64_t key = score_key(s[j]);
      if (key > kth) {
        const uint32_t pos = atomicAdd(&sh.cnt, 1u);
        skeys[pos] = key;
        sidx[pos] = (uint32_t)j;
      } else if (key == kth) {
        if (rank < need) {
          skeys[n_gt + rank] = key;
          sidx[n_gt + rank] = (uint32_t)j;
        }
        ++rank;
      }
    }
  }
}

// One workgroup per (KV head, batch item).  skeys/sidx hold `cap` entries (LDS or global).
template <bool kGlobalSort>
__global__ __launch_bounds__(kSelectThreads) void select_kernel(const double* __restrict__ s_ws, int64_t L, int64_t l_p,
                                                                int64_t cap, int32_t* __restrict__ idx_out,
                                                                uint64_t* gkeys, uint32_t* gidx, int hkv) {
  extern __shared__ __attribute__((aligned(16))) unsigned char dyn[];
  __shared__ SelectShared sh;

  const int v = blockIdx.x, b = blockIdx.y;
  const int tid = threadIdx.x;
  const int64_t head = (int64_t)b * hkv + v;
  const double* s = s_ws + head * L;
  uint64_t* skeys;
  uint32_t* sidx;
  if (kGlobalSort) {
    skeys = gkeys + head * cap;
    sidx = reinterpret_cast<uint32_t*>(reinterpret_cast<unsigned char*>(gidx) + head * cap * 6);   // [cap] u32 + [cap] u16
  } else {
    skeys = reinterpret_cast<uint64_t*>(dyn);
    sidx = reinterpret_cast<uint32_t*>(dyn + cap * sizeof(uint64_t));
  }

  uint16_t* sbin = reinterpret_cast<uint16_t*>(sidx + cap);
  if (bucket_rank_select(s, L, l_p, cap, skeys, sidx, sbin, idx_out, sh)) return;
  radix_collect(s, L, l_p, skeys, sidx, sh);
  int64_t n_sort = 1;
  while (n_sort < l_p) n_sort <<= 1;
  __syncthreads();
  for (int64_t i = l_p + tid; i < n_sort; i += kSelectThreads) {   // padding sorts last
    skeys[i] = 0;
    sidx[i] = 0xffffffffu;
  }
  __syncthreads();
  bitonic_sort(skeys, sidx, n_sort);
  for (int64_t i = tid; i < l_p; i += kSelectThreads) idx_out[head * l_p + i] = (int32_t)sidx[i];
}

// ------------------------------------------------------------------------------------------------
// K_c[b, i, v, :] = K[b, idx[b, v, i], v, :], same for V.  One thread per 16-byte chunk.
template <int D>
__global__ __launch_bounds__(256) void gather_kernel(View k, View v, const int32_t* __restrict__ idx, int64_t l_p, int hkv,
                                                     int64_t L, bf16_t* __restrict__ k_c, bf16_t* __restrict__ v_c) {
  constexpr int KC = D / 8;
  const int b = blockIdx.y;
  const int64_t item = (int64_t)blockIdx.x * 256 + threadIdx.x;      // over l_p * hkv * KC
  const int64_t n_items = l_p * hkv * KC;
  if (item >= n_items) return;
  const int c = (int)(item % KC);
  const int64_t row = item / KC;            // i * hkv + head
  const int head = (int)(row % hkv);
  const int64_t i = row / hkv;
  const int64_t j = idx[((int64_t)b * hkv + head) * l_p + i];
  if (j < 0 || j >= L) return;              // never read outside the block, whatever idx holds
  const int64_t dst = (((int64_t)b * l_p + i) * hkv + head) * D + 8 * c;
  const u32x4 kk = *reinterpret_cast<const u32x4*>(k.ptr + (int64_t)b * k.sb + j * k.st + (int64_t)head * k.sh + 8 * c);
  const u32x4 vv = *reinterpret_cast<const u32x4*>(v.ptr + (int64_t)b * v.sb + j * v.st + (int64_t)head * v.sh + 8 * c);
  // (the compressed block is written once and read by another kernel or a copy engine: keep it out of the caches)
  __builtin_nontemporal_store(kk, reinterpret_cast<u32x4*>(k_c + dst));
  __builtin_nontemporal_store(vv, reinterpret_cast<u32x4*>(v_c + dst));
}

// Scratch of the entry point that takes no workspace (apbv_compress_kv_noalloc): a fixed array in the code object,
// one copy per GPU at that GPU's own address.  In host code the array's name is only a handle for the symbol lookup
// below; kernels and launch code use the looked-up device address.
__device__ __align__(256) unsigned char scratch[kStaticScratchBytes];

// Per-device one-time set-up (the library's only state): the selection kernel's dynamic-LDS limit, which is a
// per-device property of the loaded code object, and the device address of `scratch`.
constexpr int kMaxDevices = 64;
struct DeviceState {
  bool ready = false;
  void* scratch_ptr = nullptr;
};
std::mutex g_state_mutex;
DeviceState g_state[kMaxDevices];

apbv_status device_state(DeviceState& out) {
  int device = -1;
  if (hipGetDevice(&device) != hipSuccess || device < 0) return APBV_ERR_LAUNCH;
  if (device >= kMaxDevices) return APBV_ERR_UNSUPPORTED;
  std::lock_guard<std::mutex> lock(g_state_mutex);
  DeviceState& st = g_state[device];
  if (!st.ready) {
    if (hipFuncSetAttribute(reinterpret_cast<const void*>(&select_kernel<false>), hipFuncAttributeMaxDynamicSharedMemorySize,
                            (int)(kLdsSortMax * 14)) != hipSuccess)
      return APBV_ERR_LAUNCH;
    void* ptr = nullptr;
    if (hipGetSymbolAddress(&ptr, HIP_SYMBOL(scratch)) != hipSuccess || ptr == nullptr) return APBV_ERR_LAUNCH;
    st.scratch_ptr = ptr;
    st.ready = true;
  }
  out = st;
  return APBV_OK;
}

}  // namespace

size_t compress_workspace_bytes(int batch, int hkv, int d, int64_t L, int64_t l_p) {
  return plan_compress_workspace(batch, hkv, d, L, l_p).total;
}

apbv_status launch_compress(const CompressParams& p_in, hipStream_t stream) {
  CompressParams p = p_in;
  const CompressWorkspace w = plan_compress_workspace(p.batch, p.hkv, p.d, p.L, p.l_p);
  if (p.reducer != APBV_REDUCE_SUM) {
    const apbv_status ok = check_matrix_scores(p);
    if (ok != APBV_OK) return ok;
  }
  DeviceState dev;
  const apbv_status ds = device_state(dev);
  if (ds != APBV_OK) return ds;
  if (p.use_static_scratch) {
    // the workspace is this GPU's copy of the static array: every such call on the GPU shares it
    if (p.reducer != APBV_REDUCE_SUM || w.total > kStaticScratchBytes) return APBV_ERR_WORKSPACE;
    p.workspace = dev.scratch_ptr;
    p.workspace_bytes = kStaticScratchBytes;
  }
  if (p.workspace_bytes < w.total) return APBV_ERR_WORKSPACE;
  unsigned char* ws = static_cast<unsigned char*>(p.workspace);
  double* qbar = reinterpret_cast<double*>(ws + w.qbar_off);
  double* scores = reinterpret_cast<double*>(ws + w.scores_off);
  Launcher launch(stream);

  if (p.reducer != APBV_REDUCE_SUM) {
    // the non-linear reductions form the logit matrix on the matrix cores (score_matrix.hip); their row
    // statistics live behind the selection workspace
    const size_t stats_off = align_up(w.total, 256);
    const size_t stats_bytes = matrix_scores_workspace_bytes(p.reducer, p.batch, p.hkv, p.q_probe.tokens * p.group, p.L);
    if (p.workspace_bytes < stats_off + stats_bytes) return APBV_ERR_WORKSPACE;
    const apbv_status st = launch_matrix_scores(p, scores, ws + stats_off, stream);
    if (st != APBV_OK) return st;
  } else {
    // pooled query, as n_split partial sums
    const int n_split = pool_splits(p.q_probe.tokens * p.group, (int64_t)p.batch * p.hkv);
    const int64_t rows_per_split = (p.q_probe.tokens * p.group + n_split - 1) / n_split;
    const bool wide = rows_per_split >= 4 * 1024 / (p.d / 8);
    const dim3 pool_grid(n_split, p.hkv, p.batch);
    if (p.d == 128 && wide)
      launch(pool_query_kernel<128, 1024>, pool_grid, dim3(1024), 0, p.q_probe, p.q_probe.tokens, p.group, qbar, p.hkv, n_split);
    else if (p.d == 128)
      launch(pool_query_kernel<128, 256>, pool_grid, dim3(256), 0, p.q_probe, p.q_probe.tokens, p.group, qbar, p.hkv, n_split);
    else if (wide)
      launch(pool_query_kernel<64, 1024>, pool_grid, dim3(1024), 0, p.q_probe, p.q_probe.tokens, p.group, qbar, p.hkv, n_split);
    else
      launch(pool_query_kernel<64, 256>, pool_grid, dim3(256), 0, p.q_probe, p.q_probe.tokens, p.group, qbar, p.hkv, n_split);
    // scores: one outer iteration per workgroup: 4 rows in flight per thread, many small workgroups
    const int rows_per_block = 4 * 256 / (p.d / 8);
    dim3 grid((unsigned)((p.L + rows_per_block - 1) / rows_per_block), p.hkv, p.batch);
    if (p.d == 128)
      launch(score_kernel<128>, grid, dim3(256), 0, p.k, p.L, qbar, n_split, scores, p.scores_out, p.hkv, rows_per_block);
    else
      launch(score_kernel<64>, grid, dim3(256), 0, p.k, p.L, qbar, n_split, scores, p.scores_out, p.hkv, rows_per_block);
  }
  if (p.l_p > 0) {
    // select + order
    if (w.sort_in_global) {
      launch(select_kernel<true>, dim3(p.hkv, p.batch), dim3(kSelectThreads), 0, scores, p.L, p.l_p, w.n_sort, p.idx_out, reinterpret_cast<uint64_t*>(ws + w.sort_keys_off), reinterpret_cast<uint32_t*>(ws + w.sort_idx_off), p.hkv);
    } else {
      const size_t dyn = (size_t)w.n_sort * 14;
      launch(select_kernel<false>, dim3(p.hkv, p.batch), dim3(kSelectThreads), dyn, scores, p.L, p.l_p, w.n_sort, p.idx_out, nullptr, nullptr, p.hkv);
    }
    // gather
    const int64_t n_items = p.l_p * p.hkv * (p.d / 8);
    dim3 grid((unsigned)((n_items + 255) / 256), p.batch);
    if (p.d == 128)
      launch(gather_kernel<128>, grid, dim3(256), 0, p.k, p.v, p.idx_out, p.l_p, p.hkv, p.L, p.k_c, p.v_c);
    else
      launch(gather_kernel<64>, grid, dim3(256), 0, p.k, p.v, p.idx_out, p.l_p, p.hkv, p.L, p.k_c, p.v_c);
  }
  return launch.status();
}

}  // namespace apbv
