// Fused host attention for gfx950 (Eq. 4 by the definition of Eq. 1): one pass of online-softmax
// attention of the local query block over the concatenated keys [anchor | passing | local].
//
// The three KV segments are walked as ONE virtual key axis j in [0, n_vis + L): anchor and passing
// keys (j < n_vis) are visible to every query and local key j - n_vis is visible to query i iff
// j - n_vis <= i, so the whole mask is the single test  j <= i + n_vis  (a causal mask shifted by
// n_vis).  Key tiles that lie entirely above that diagonal are never visited.
//
// Tiling: a workgroup of 4 waves owns 128 consecutive query positions of one query head; each wave
// owns 32 of them.  Key tiles of 64 virtual keys are staged in LDS: K row-major [64][D] and V
// transposed [D][64], both with an XOR swizzle of the 16-byte chunks.
//
// MFMA mapping (v_mfma_f32_32x32x16_bf16; A is 32x16 with lane l holding row l%32, k = 8*(l/32)..+7;
// B is 16x32 with lane l holding column l%32, same k; D is 32x32 with lane l holding column l%32 and
// rows 8*(r/4) + 4*(l/32) + r%4 for r = 0..15):
//   S^T = K Q^T  : A = K tile from LDS (rows = keys), B = Q^T kept in registers (columns = queries).
//                  Each lane then holds 16 keys of ONE query per 32-key block, so the row maximum and
//                  row sum of the softmax are in-lane reductions plus one exchange with lane^32.
//   O^T = V^T P^T: B = P^T taken straight from the S^T accumulator registers (rounded to bf16), no
//                  LDS round trip.  The k-slot -> key assignment this induces (for the t-th MFMA of a
//                  32-key block, lane half hh, element e: key 16t + 8*(e/4) + 4*hh + e%4) is baked into
//                  the order in which V^T is stored in LDS, so A = V^T is one 16-byte LDS read.
#include "apbv_common.h"

namespace apbv {
namespace {

constexpr int kWaves = 4;
constexpr int kThreads = kWaves * 64;
constexpr int kBM = 32 * kWaves;   // query rows per workgroup
constexpr int kBN = 64;            // keys per tile

__device__ __forceinline__ u32x4 ld16(const bf16_t* p) { return *reinterpret_cast<const u32x4*>(p); }

// Row pointer of virtual key j in one of the three segments (nullptr past the end).
struct SegRows {
  const bf16_t* base[3];
  int64_t st[3];
  int64_t l_a, n_vis, s_kv;
  __device__ __forceinline__ const bf16_t* row(int64_t j) const {
    if (j < l_a) return base[0] + j * st[0];
    if (j < n_vis) return base[1] + (j - l_a) * st[1];
    if (j < s_kv) return base[2] + (j - n_vis) * st[2];
    return nullptr;
  }
};

template <int D>
struct Tile {
  static constexpr int KC = D / 8;                 // 16-byte chunks per K row
  static constexpr int K_ROWS_PER_PASS = kThreads / KC;
  static constexpr int K_PASSES = kBN / K_ROWS_PER_PASS;
  static constexpr int V_ITEMS = 16 * KC;          // (key quad, dd chunk) items per tile
  static constexpr int KS = D / 16;                // MFMA k-steps over the head dimension
  static constexpr int DB = D / 32;                // 32-row blocks of O^T
  static constexpr int K_BYTES = kBN * D * 2;
  static constexpr int V_BYTES = D * kBN * 2;
};

// LDS offsets (bytes).  K tile: row `key` (D*2 bytes), chunk c of 16 bytes, swizzled by key&7.
template <int D>
__device__ __forceinline__ int k_lds_off(int key, int chunk) {
  return key * (D * 2) + ((chunk ^ (key & 7)) << 4);
}
// V^T tile: row `dd` (128 bytes = 8 chunks), swizzled by (dd ^ dd>>3)&7.
__device__ __forceinline__ int v_lds_off(int dd, int chunk) {
  return dd * (kBN * 2) + ((chunk ^ ((dd ^ (dd >> 3)) & 7)) << 4);
}

template <int D>
__global__ __launch_bounds__(kThreads, 2) void host_attention_kernel(const AttnParams p, const int n_qtiles) {
  using T = Tile<D>;
  __shared__ __attribute__((aligned(16))) unsigned char smem[T::K_BYTES + T::V_BYTES];
  unsigned char* const ks = smem;
  unsigned char* const vt = smem + T::K_BYTES;

  const int tid = threadIdx.x;
  const int lane = tid & 63;
  const int wave = tid >> 6;
  const int lq = lane & 31;       // query column / A-operand row within a 32-block
  const int hh = lane >> 5;       // lane half

  // Heaviest query tiles (most visible keys) first.
  const int qt = n_qtiles - 1 - (int)blockIdx.x;
  const int h = blockIdx.y;
  const int b = blockIdx.z;
  const int kvh = h / p.group;

  const int64_t i0 = (int64_t)qt * kBM;                 // first query position of the workgroup
  const int64_t iw = i0 + wave * 32;                    // first query position of the wave
  const int64_t i_row = iw + lq;                        // this lane's query position

  SegRows kr, vr;
#pragma unroll
  for (int s = 0; s < 3; ++s) {
    kr.base[s] = p.k_seg[s].ptr + (int64_t)b * p.k_seg[s].sb + (int64_t)kvh * p.k_seg[s].sh;
    kr.st[s] = p.k_seg[s].st;
    vr.base[s] = p.v_seg[s].ptr + (int64_t)b * p.v_seg[s].sb + (int64_t)kvh * p.v_seg[s].sh;
    vr.st[s] = p.v_seg[s].st;
  }
  kr.l_a = vr.l_a = p.l_a;
  kr.n_vis = vr.n_vis = p.n_vis;
  kr.s_kv = vr.s_kv = p.s_kv;

  // ---- Q^T fragments (B operand), kept in registers for the whole key loop.
  bf16x8 qf[T::KS];
  {
    const bf16_t* qrow = p.q.ptr + (int64_t)b * p.q.sb + (int64_t)h * p.q.sh + i_row * p.q.st;
    const bool ok = i_row < p.L;
#pragma unroll
    for (int s = 0; s < T::KS; ++s) {
      u32x4 v = {0u, 0u, 0u, 0u};
      if (ok) v = ld16(qrow + 16 * s + 8 * hh);
      qf[s] = __builtin_bit_cast(bf16x8, v);
    }
  }

  // ---- staging assignment
  const int kc = tid % T::KC;                 // K: chunk within the row
  const int kr0 = tid / T::KC;                // K: first row handled
  const int vdg = tid % T::KC;                // V: dd chunk (8 dd)
  const int vkq = tid / T::KC;                // V: key quad (valid if < 16)
  const bool v_active = vkq < 16;
  const int v_chunk = 2 * (vkq >> 2) + (vkq & 1);
  const int v_half = (vkq & 3) >> 1;

  u32x4 kreg[T::K_PASSES];
  u32x4 vreg[4];

  auto load_tile = [&](int64_t j0) {
#pragma unroll
    for (int s = 0; s < T::K_PASSES; ++s) {
      const bf16_t* r = kr.row(j0 + kr0 + s * T::K_ROWS_PER_PASS);
      u32x4 v = {0u, 0u, 0u, 0u};
      if (r) v = ld16(r + 8 * kc);
      kreg[s] = v;
    }
    if (v_active) {
#pragma unroll
      for (int a = 0; a < 4; ++a) {
        const bf16_t* r = vr.row(j0 + 4 * vkq + a);
        u32x4 v = {0u, 0u, 0u, 0u};
        if (r) v = ld16(r + 8 * vdg);
        vreg[a] = v;
      }
    }
  };
  auto store_tile = [&]() {
#pragma unroll
    for (int s = 0; s < T::K_PASSES; ++s) {
      const int row = kr0 + s * T::K_ROWS_PER_PASS;
      *reinterpret_cast<u32x4*>(ks + k_lds_off<D>(row, kc)) = kreg[s];
    }
    if (v_active) {
      // 4 keys x 8 dd in registers -> for each dd the 4 keys as one 8-byte LDS write.
#pragma unroll
      for (int e = 0; e < 8; ++e) {
        const uint32_t sel = (e & 1) ? 0x07060302u : 0x05040100u;
        u32x2 w;
        w.x = __builtin_amdgcn_perm(vreg[1][e >> 1], vreg[0][e >> 1], sel);
        w.y = __builtin_amdgcn_perm(vreg[3][e >> 1], vreg[2][e >> 1], sel);
        const int dd = 8 * vdg + e;
        *reinterpret_cast<u32x2*>(vt + v_lds_off(dd, v_chunk) + 8 * v_half) = w;
      }
    }
  };

  // ---- online softmax state (per lane: one query; the two lane halves hold disjoint key subsets)
  f32x16 o[T::DB];
#pragma unroll
  for (int d = 0; d < T::DB; ++d)
#pragma unroll
    for (int r = 0; r < 16; ++r) o[d][r] = 0.f;
  float m_run = -INFINITY;   // running maximum of the scaled (log2-domain) logits, whole row
  float l_run = 0.f;         // running sum of exp2, this lane half only

  // Keys the workgroup / this wave can see at all.
  const int64_t i_last_wg = (i0 + kBM - 1 < p.L - 1) ? i0 + kBM - 1 : p.L - 1;
  const int64_t n_keys_wg = i_last_wg + 1 + p.n_vis;
  const int n_tiles = (int)((n_keys_wg + kBN - 1) / kBN);
  const int64_t j_lim_wave = iw + 31 + p.n_vis;      // last virtual key any row of the wave may see

  load_tile(0);
  store_tile();
  __syncthreads();

  for (int t = 0; t < n_tiles; ++t) {
    const int64_t j0 = (int64_t)t * kBN;
    if (t + 1 < n_tiles) load_tile(j0 + kBN);

    if (j0 <= j_lim_wave) {
      // ---- S^T = K Q^T for the two 32-key blocks
      f32x16 s[2];
#pragma unroll
      for (int kb = 0; kb < 2; ++kb) {
#pragma unroll
        for (int r = 0; r < 16; ++r) s[kb][r] = 0.f;
#pragma unroll
        for (int c = 0; c < T::KS; ++c) {
          const u32x4 a = *reinterpret_cast<const u32x4*>(ks + k_lds_off<D>(32 * kb + lq, 2 * c + hh));
          s[kb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, a), qf[c], s[kb], 0, 0, 0);
        }
      }
      // ---- mask (only tiles that reach above the wave's first diagonal element)
      if (j0 + kBN - 1 > iw + p.n_vis) {
        const int64_t jmax = i_row + p.n_vis;        // last visible virtual key of this lane's query
#pragma unroll
        for (int kb = 0; kb < 2; ++kb)
#pragma unroll
          for (int r = 0; r < 16; ++r) {
            const int64_t j = j0 + 32 * kb + 8 * (r >> 2) + 4 * hh + (r & 3);
            if (j > jmax) s[kb][r] = -INFINITY;
          }
      }
      // ---- online softmax
      float mx = s[0][0];
#pragma unroll
      for (int kb = 0; kb < 2; ++kb)
#pragma unroll
        for (int r = 0; r < 16; ++r) mx = fmaxf(mx, s[kb][r]);
      mx = fmaxf(mx, __shfl_xor(mx, 32));
      const float m_new = fmaxf(m_run, mx * p.scale_log2);
      const float alpha = __builtin_amdgcn_exp2f(m_run - m_new);
      m_run = m_new;
      float psum = 0.f;
#pragma unroll
      for (int kb = 0; kb < 2; ++kb)
#pragma unroll
        for (int r = 0; r < 16; ++r) {
          const float e = __builtin_amdgcn_exp2f(__builtin_fmaf(s[kb][r], p.scale_log2, -m_new));
          s[kb][r] = e;
          psum += e;
        }
      l_run = l_run * alpha + psum;
#pragma unroll
      for (int d = 0; d < T::DB; ++d)
#pragma unroll
        for (int r = 0; r < 16; ++r) o[d][r] *= alpha;

      // ---- O^T += V^T P^T
#pragma unroll
      for (int kb = 0; kb < 2; ++kb)
#pragma unroll
        for (int tt = 0; tt < 2; ++tt) {
          bf16x8 pf;
#pragma unroll
          for (int e = 0; e < 8; e += 2) {
            f32x2 xy = {s[kb][8 * tt + e], s[kb][8 * tt + e + 1]};
            bf16x2 c = __builtin_convertvector(xy, bf16x2);
            pf[e] = c[0];
            pf[e + 1] = c[1];
          }
#pragma unroll
          for (int d = 0; d < T::DB; ++d) {
            const u32x4 a = *reinterpret_cast<const u32x4*>(vt + v_lds_off(32 * d + lq, 4 * kb + 2 * tt + hh));
            o[d] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, a), pf, o[d], 0, 0, 0);
          }
        }
    }

    __syncthreads();                 // every wave is done reading tile t
    if (t + 1 < n_tiles) {
      store_tile();
      __syncthreads();               // tile t+1 is visible
    }
  }

  // ---- epilogue: normalise, round to bf16, store; optional log-sum-exp
  const float l_tot = l_run + __shfl_xor(l_run, 32);
  const float inv = 1.0f / l_tot;
  if (i_row < p.L) {
    bf16_t* orow = p.out + (((int64_t)b * p.L + i_row) * p.hq + h) * D;
#pragma unroll
    for (int d = 0; d < T::DB; ++d)
#pragma unroll
      for (int g = 0; g < 4; ++g) {
        f32x2 x01 = {o[d][4 * g + 0] * inv, o[d][4 * g + 1] * inv};
        f32x2 x23 = {o[d][4 * g + 2] * inv, o[d][4 * g + 3] * inv};
        bf16x2 c01 = __builtin_convertvector(x01, bf16x2);
        bf16x2 c23 = __builtin_convertvector(x23, bf16x2);
        u32x2 w;
        w.x = __builtin_bit_cast(uint32_t, c01);
        w.y = __builtin_bit_cast(uint32_t, c23);
        *reinterpret_cast<u32x2*>(orow + 32 * d + 8 * g + 4 * hh) = w;
      }
    if (p.lse != nullptr && hh == 0)
      p.lse[((int64_t)b * p.hq + h) * p.L + i_row] = (m_run + __builtin_amdgcn_logf(l_tot)) * 0.6931471805599453f;
  }
}

}  // namespace

apbv_status launch_host_attention(const AttnParams& p, int head_dim, hipStream_t stream) {
  const int n_qtiles = (int)((p.L + kBM - 1) / kBM);
  dim3 grid(n_qtiles, p.hq, p.batch);
  dim3 block(kThreads);
  if (head_dim == 128)
    hipLaunchKernelGGL(host_attention_kernel<128>, grid, block, 0, stream, p, n_qtiles);
  else if (head_dim == 64)
    hipLaunchKernelGGL(host_attention_kernel<64>, grid, block, 0, stream, p, n_qtiles);
  else
    return APBV_ERR_UNSUPPORTED;
  return hipGetLastError() == hipSuccess ? APBV_OK : APBV_ERR_LAUNCH;
}

}  // namespace apbv
