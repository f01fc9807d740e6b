// Fused host attention for gfx950 (Eq. 4 by the definition of Eq. 1): one pass of online-softmax
// attention of the local query block over the concatenated keys [anchor | passing | local].
//
// Mask.  The three KV segments are walked as ONE virtual key axis j in [0, n_vis + L): anchor and
// passing keys (j < n_vis) are visible to every query and local key j - n_vis is visible to query i iff
// j - n_vis <= i, so the whole mask is the single test  j <= i + n_vis  (a causal mask shifted by
// n_vis).  Without a local segment (partial attention of a query block over context keys only, merged
// later by log-sum-exp) the bound is simply the last key.  Key tiles that lie entirely above that diagonal are never visited, and only tiles that
// touch it pay for the comparison.
//
// Tiling.  A workgroup of 8 waves (two per SIMD, one workgroup per CU) owns 256 consecutive query
// positions of one query head; each wave owns 32 of them.  Key tiles of 64 virtual keys are copied global -> LDS by the LDS-direct load
// (global_load_lds_dwordx4: no VGPR staging, no VALU work), double buffered, one barrier per tile.
// Both K and V are stored row-major [64][D] with an XOR swizzle of their 16-byte chunks; the swizzle is
// applied on the global side (which chunk a lane fetches), because an LDS-direct load always writes
// lane l's 16 bytes at base + 16*l.
//
// MFMA mapping (v_mfma_f32_32x32x16_bf16; A is 32x16 with lane l holding row l%32, k = 8*(l/32)..+7;
// B is 16x32 with lane l holding column l%32, same k; D is 32x32 with lane l holding column l%32 and
// rows 8*(r/4) + 4*(l/32) + r%4 for r = 0..15):
//   S^T = K Q^T  : A = K tile rows (one 16-byte LDS read), B = Q^T kept in registers (columns =
//                  queries).  Each lane then holds 16 keys of ONE query per 32-key block, so the row
//                  maximum and row sum of the softmax are in-lane reductions plus one exchange with
//                  lane^32 (v_permlane32_swap).
//   O^T = V^T P^T: B = P^T straight from the S^T accumulator registers (rounded to bf16), no LDS round
//                  trip.  That fixes which key sits in which k-slot (t-th MFMA of a 32-key block, lane
//                  half hh, element e: key 16t + 8*(e/4) + 4*hh + e%4); A = V^T is fetched to match with
//                  two transposing LDS reads (ds_read_b64_tr_b16: within 16 lanes, lane i receives
//                  element i%4 of the 8 bytes addressed by lanes i/4, 4+i/4, 8+i/4, 12+i/4), each
//                  delivering 4 consecutive keys of one head-dim column.
//
// Softmax.  exp2 domain with the scale folded in; the running maximum is only advanced (and O, l
// rescaled) when it would grow by more than 2^8, which keeps exp2 arguments <= 8 and removes the
// per-tile rescale of the 64 accumulator registers from the common path.
//
// Key split.  For a short query block (few query tiles) the key axis can be cut into n_splits ranges of
// tiles_per_split tiles, one workgroup each; every range writes a normalised partial result and
// its log-sum-exp, merged afterwards (Eq. 5's merge).  n_splits = 1 is the plain kernel.
//
// Launch.  One workgroup per (query tile, query head, batch item), heaviest query tiles first.  The
// linear workgroup id is decoded so that the G query heads that share a KV head run on the same XCD
// (workgroup id modulo 8) back to back and stream the same K/V tiles through that XCD's L2.
#include "apbv_common.h"

namespace apbv {
namespace {

constexpr int kWaves = 8;          // waves per workgroup of the main variant: 256 query rows
constexpr int kWavesNarrow = 2;    // of the variant for short query blocks: 64 query rows
constexpr int kBM = 32 * kWaves;   // query rows per workgroup (main variant)
constexpr int kBN = 64;            // keys per tile
constexpr int kXcds = 8;
constexpr float kRescaleThreshold = 8.0f;   // log2 units

#define APBV_LDS(T) __attribute__((address_space(3))) T*
#define APBV_GLB(T) const __attribute__((address_space(1))) T*

typedef __attribute__((ext_vector_type(4))) short s16x4;

template <int D, int W>
struct Tile {
  static constexpr int ROW_BYTES = D * 2;
  static constexpr int KC = D / 8;                        // 16-byte chunks per row
  static constexpr int RPI = 1024 / ROW_BYTES;            // rows covered by one wave-wide LDS-direct load
  static constexpr int IPW = kBN / RPI / W;              // such loads per wave per tile (per tensor)
  static constexpr int KS = D / 16;                       // MFMA k-steps over the head dimension
  static constexpr int DB = D / 32;                       // 32-row blocks of O^T
  static constexpr int TILE_BYTES = kBN * ROW_BYTES;
  // chunk swizzles (functions of the row within the tile)
  __device__ static __forceinline__ int fk(int r) { return D == 128 ? (r & 15) : ((r >> 1) & 7); }
  __device__ static __forceinline__ int fv(int r) { return D == 128 ? ((r & 3) << 2) : (((r >> 1) & 1) << 2); }
};

struct Segs {
  const char *b0, *b1, *b2;   // byte pointers of the three segments, already offset to (batch, kv head)
  int64_t p0, p1, p2;         // bytes between consecutive tokens
  int64_t e0, e1, e2;         // one past the last virtual key of each segment (starts are 0, e0, e1)
};

// Pick the fields of the segment that holds virtual key j (selects, no indexed access).
__device__ __forceinline__ void seg_of(const Segs sg, int64_t j, const char*& base, int64_t& pitch, int64_t& start,
                                       int64_t& end) {
  const bool in0 = j < sg.e0, in1 = j < sg.e1;
  base = in0 ? sg.b0 : (in1 ? sg.b1 : sg.b2);
  pitch = in0 ? sg.p0 : (in1 ? sg.p1 : sg.p2);
  start = in0 ? 0 : (in1 ? sg.e0 : sg.e1);
  end = in0 ? sg.e0 : (in1 ? sg.e1 : sg.e2);
}

// LDS-direct 16-byte load: lane l's bytes land at lds_dst + 16*l (lds_dst uniform, in M0).  Issued through
// inline assembly so that the kernel, not the compiler's wait-count insertion, orders these loads against
// the LDS reads (one s_waitcnt vmcnt + barrier per tile).
__device__ __forceinline__ const char* uniform_ptr(const char* p) {      // a wave-uniform pointer, provably so
  const uint64_t v = (uint64_t)p;
  const uint32_t lo = __builtin_amdgcn_readfirstlane((uint32_t)v), hi = __builtin_amdgcn_readfirstlane((uint32_t)(v >> 32));
  return (const char*)(((uint64_t)hi << 32) | lo);
}
__device__ __forceinline__ void dma16_uniform(const char* base_uniform, uint32_t lane_off, uint32_t lds_dst) {
  asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %1, %2" ::"s"(lds_dst), "v"(lane_off), "s"(base_uniform)
               : "memory", "m0");
}
__device__ __forceinline__ void dma16_lane(const char* addr, uint32_t lds_dst) {
  asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %1, off" ::"s"(lds_dst), "v"(addr) : "memory", "m0");
}
__device__ __forceinline__ uint32_t lds_addr(const unsigned char* p) { return (uint32_t)(size_t)(APBV_LDS(const unsigned char))p; }

// Sequential producer of the K and V tiles of the virtual key axis.  While consecutive tiles stay inside
// one segment ("run") a tile costs two 64-bit scalar adds and its loads are  uniform tile base + a per-lane
// 32-bit offset computed once per run; the tile that straddles a segment boundary (or the end of the keys)
// takes a per-row lookup.
template <int D, int W>
struct TileStream {
  using T = Tile<D, W>;
  Segs ks, vs;             // e0/e1/e2 are shared
  int64_t s_kv;
  int t_next;              // next tile to issue
  int run_end;             // tiles [t_next, run_end) lie inside one segment; kb/vb point at tile t_next
  const char *kb, *vb;
  int64_t kstep, vstep;    // kBN * pitch
  uint32_t koff[T::IPW], voff[T::IPW];
  int wave, lane;

  __device__ __forceinline__ int row(int u) const { return (wave * T::IPW + u) * T::RPI + lane / T::KC; }
  __device__ __forceinline__ uint32_t ldst(int u) const { return (uint32_t)((wave * T::IPW + u) * T::RPI * T::ROW_BYTES); }

  __device__ __forceinline__ void init(const Segs& k, const Segs& v, int64_t skv, int w, int l, int t_first) {
    ks = k;
    vs = v;
    s_kv = skv;
    wave = w;
    lane = l;
    t_next = t_first;
    run_end = t_first;
    kb = vb = nullptr;
    kstep = vstep = 0;
#pragma unroll
    for (int u = 0; u < T::IPW; ++u) koff[u] = voff[u] = 0;
  }

  // Start a run at tile t_next if that tile lies inside one segment.
  __device__ __forceinline__ void start_run() {
    const int64_t j0 = (int64_t)t_next * kBN;
    const char *kbase, *vbase;
    int64_t kp, vp, start, end, dummy0, dummy1;
    seg_of(ks, j0, kbase, kp, start, end);
    seg_of(vs, j0, vbase, vp, dummy0, dummy1);
    if (j0 + kBN > end) return;                      // straddling tile: run stays empty
    run_end = (int)(end / kBN);
    kb = kbase + (j0 - start) * kp;
    vb = vbase + (j0 - start) * vp;
    kstep = kBN * kp;
    vstep = kBN * vp;
#pragma unroll
    for (int u = 0; u < T::IPW; ++u) {
      const int r = row(u);
      koff[u] = (uint32_t)r * (uint32_t)kp + 16u * (uint32_t)((lane % T::KC) ^ T::fk(r));
      voff[u] = (uint32_t)r * (uint32_t)vp + 16u * (uint32_t)((lane % T::KC) ^ T::fv(r));
    }
  }

  // Issue this wave's share of the loads of tile t_next into the LDS tiles at k_dst / v_dst.
  __device__ __forceinline__ void issue(uint32_t k_dst, uint32_t v_dst) {
    if (t_next >= run_end) start_run();
    if (t_next < run_end) {
      const char* kbu = uniform_ptr(kb);
      const char* vbu = uniform_ptr(vb);
#pragma unroll
      for (int u = 0; u < T::IPW; ++u) dma16_uniform(kbu, koff[u], k_dst + ldst(u));
#pragma unroll
      for (int u = 0; u < T::IPW; ++u) dma16_uniform(vbu, voff[u], v_dst + ldst(u));
      kb += kstep;
      vb += vstep;
    } else {
      const int64_t j0 = (int64_t)t_next * kBN;
#pragma unroll
      for (int u = 0; u < T::IPW; ++u) {
        const int r = row(u);
        int64_t j = j0 + r;
        j = j < s_kv ? j : s_kv - 1;                 // rows past the end repeat the last key: always masked
        const char *bk, *bv;
        int64_t pk, pv, sj, ej, d0, d1;
        seg_of(ks, j, bk, pk, sj, ej);
        seg_of(vs, j, bv, pv, d0, d1);
        dma16_lane(bk + (j - sj) * pk + 16 * ((lane % T::KC) ^ T::fk(r)), k_dst + ldst(u));
        dma16_lane(bv + (j - sj) * pv + 16 * ((lane % T::KC) ^ T::fv(r)), v_dst + ldst(u));
      }
    }
    ++t_next;
  }
};

// One workgroup's work: query tile `qt` of query head (kvh, g) of batch item b, key range `split`.
template <int D, int W>
__device__ __forceinline__ void attention_workgroup(const AttnParams& p, const int qt, const int b, const int kvh,
                                                    const int g, const int split) {
  using T = Tile<D, W>;
  constexpr int kRows = 32 * W;      // query rows of the workgroup
  __shared__ __attribute__((aligned(1024))) unsigned char k_lds0[T::TILE_BYTES];
  __shared__ __attribute__((aligned(1024))) unsigned char k_lds1[T::TILE_BYTES];
  __shared__ __attribute__((aligned(1024))) unsigned char v_lds0[T::TILE_BYTES];
  __shared__ __attribute__((aligned(1024))) unsigned char v_lds1[T::TILE_BYTES];
  // the LDS destination of an LDS-direct load travels in M0, which addresses the first 64 KB of the workgroup's LDS
  static_assert(4 * T::TILE_BYTES <= 65536, "the four K/V tiles must lie below 64 KB of LDS");
  const int h = kvh * p.group + g;

  const int tid = threadIdx.x;
  const int lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);   // uniform: keeps LDS tile addresses in SGPRs
  const int lq = lane & 31;       // query column / A-operand row within a 32-block
  const int hh = lane >> 5;       // lane half

  const int64_t i0 = (int64_t)qt * kRows;               // first query position of the workgroup
  const int64_t iw = i0 + wave * 32;                    // first query position of the wave
  const int64_t i_row = iw + lq;                        // this lane's query position

  Segs ks, vs;
  {
    auto kbase = [&](int s) {
      return reinterpret_cast<const char*>(p.k_seg[s].ptr + (int64_t)b * p.k_seg[s].sb + (int64_t)kvh * p.k_seg[s].sh);
    };
    auto vbase = [&](int s) {
      return reinterpret_cast<const char*>(p.v_seg[s].ptr + (int64_t)b * p.v_seg[s].sb + (int64_t)kvh * p.v_seg[s].sh);
    };
    ks.b0 = kbase(0); ks.b1 = kbase(1); ks.b2 = kbase(2);
    vs.b0 = vbase(0); vs.b1 = vbase(1); vs.b2 = vbase(2);
    ks.p0 = p.k_seg[0].st * 2; ks.p1 = p.k_seg[1].st * 2; ks.p2 = p.k_seg[2].st * 2;
    vs.p0 = p.v_seg[0].st * 2; vs.p1 = p.v_seg[1].st * 2; vs.p2 = p.v_seg[2].st * 2;
    ks.e0 = vs.e0 = p.l_a; ks.e1 = vs.e1 = p.n_vis; ks.e2 = vs.e2 = p.s_kv;
  }

  // ---- Q^T fragments (B operand), kept in registers for the whole key loop.
  bf16x8 qf[T::KS];
  {
    const bf16_t* qrow = p.q.ptr + (int64_t)b * p.q.sb + (int64_t)h * p.q.sh + (i_row < p.L ? i_row : p.L - 1) * p.q.st;
#pragma unroll
    for (int s = 0; s < T::KS; ++s) qf[s] = __builtin_bit_cast(bf16x8, *reinterpret_cast<const u32x4*>(qrow + 16 * s + 8 * hh));
  }

  // ---- per-lane LDS read offsets
  // K (A operand of S^T): row 32*kb + lq, chunk (2*ks + hh) ^ fk(row)
  int k_off[T::KS];
#pragma unroll
  for (int c = 0; c < T::KS; ++c) k_off[c] = lq * T::ROW_BYTES + (((2 * c + hh) ^ T::fk(lq)) << 4);
  // V (A operand of O^T, transposing read): within a 16-lane group, source lane s addresses row s/4,
  // head-dim columns 32*db + 16*(group%2) + 4*(s%4) .. +3
  int v_off[T::DB];
  {
    const int grp = lane >> 4, sl = lane & 15;
    const int row = 4 * (grp >> 1) + (sl >> 2);            // + 32*kb + 16*t + 8*eh as an immediate
#pragma unroll
    for (int d = 0; d < T::DB; ++d) {
      const int dd0 = 32 * d + 16 * (grp & 1) + 4 * (sl & 3);
      v_off[d] = row * T::ROW_BYTES + ((((dd0 >> 3) ^ T::fv(row))) << 4) + ((dd0 & 7) >> 2) * 8;
    }
  }

  // ---- online softmax state (per lane: one query; the two lane halves hold disjoint key subsets)
  f32x16 o[T::DB];
#pragma unroll
  for (int d = 0; d < T::DB; ++d)
#pragma unroll
    for (int r = 0; r < 16; ++r) o[d][r] = 0.f;
  float m_ref = -INFINITY;   // reference maximum of the scaled (log2-domain) logits, whole row
  float l_run = 0.f;         // running sum of the bf16-rounded exp2(. - m_ref), this lane half only

  // Keys the workgroup / this wave can see at all.
  // Query i sees the virtual keys 0 .. min(i + n_vis, s_kv - 1); the second bound only matters when there is no
  // causal segment (s_kv == n_vis: every key visible to every query).
  auto last_key = [&](int64_t i) { return (i + p.n_vis < p.s_kv - 1) ? i + p.n_vis : p.s_kv - 1; };
  const int64_t i_last_wg = (i0 + kRows - 1 < p.L - 1) ? i0 + kRows - 1 : p.L - 1;
  const int n_tiles_vis = (int)(last_key(i_last_wg) / kBN) + 1;      // tiles the workgroup can see into
  // key split (partial results merged afterwards): this workgroup walks tiles [t_begin, n_tiles) only
  const int t_begin = split * p.tiles_per_split;
  const int n_tiles = (t_begin + p.tiles_per_split < n_tiles_vis) ? t_begin + p.tiles_per_split : n_tiles_vis;
  const int t_last_wave = (int)(last_key(iw + 31) / kBN);     // last tile any row of the wave can see into
  const int t_mask_wave = (int)((last_key(iw) + 1) / kBN);    // first tile with a key some row of the wave cannot see
  const int jrel0 = (int)last_key(i_row);                     // last visible virtual key of this lane's query

  auto compute = [&](const unsigned char* kt, const unsigned char* vt, int t) {
    if (t > t_last_wave) return;
    // ---- S^T = K Q^T for the two 32-key blocks.  K fragments are read kReadAhead k-steps ahead of the MFMA
    // that consumes them, and the order is pinned (the scheduler would otherwise sink every read next to its
    // use to save registers, exposing the LDS latency once per MFMA).
    f32x16 s[2];
#pragma unroll
    for (int kb = 0; kb < 2; ++kb)
#pragma unroll
      for (int r = 0; r < 16; ++r) s[kb][r] = 0.f;
    {
      constexpr int kReadAhead = 4;
      u32x4 ka[kReadAhead][2];
#pragma unroll
      for (int c = 0; c < kReadAhead; ++c)
#pragma unroll
        for (int kb = 0; kb < 2; ++kb)
          ka[c][kb] = *reinterpret_cast<const u32x4*>(kt + kb * 32 * T::ROW_BYTES + k_off[c]);
#pragma unroll
      for (int c = 0; c < T::KS; ++c) {
#pragma unroll
        for (int kb = 0; kb < 2; ++kb) {
          s[kb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, ka[c % kReadAhead][kb]), qf[c], s[kb], 0, 0, 0);
          if (c + kReadAhead < T::KS)
            ka[c % kReadAhead][kb] = *reinterpret_cast<const u32x4*>(kt + kb * 32 * T::ROW_BYTES + k_off[c + kReadAhead]);
        }
      }
      // scheduling groups: 2*kReadAhead LDS reads, then (MFMA, LDS read) pairs, then the remaining MFMAs
      __builtin_amdgcn_sched_group_barrier(0x100, 2 * kReadAhead, 0);
#pragma unroll
      for (int i = 0; i < 2 * (T::KS - kReadAhead); ++i) {
        __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);
        __builtin_amdgcn_sched_group_barrier(0x100, 1, 0);
      }
      __builtin_amdgcn_sched_group_barrier(0x008, 2 * kReadAhead, 0);
    }
    // ---- mask (only tiles that reach above the wave's first diagonal element)
    if (t >= t_mask_wave) {
      const int jrel_max = jrel0 - t * kBN;          // last visible key of this lane's query, tile-relative
#pragma unroll
      for (int kb = 0; kb < 2; ++kb)
#pragma unroll
        for (int r = 0; r < 16; ++r) {
          const int jr = 32 * kb + 8 * (r >> 2) + 4 * hh + (r & 3);
          if (jr > jrel_max) s[kb][r] = -INFINITY;
        }
    }
    // ---- online softmax with lazy rescaling
    float mx = s[0][0];
#pragma unroll
    for (int kb = 0; kb < 2; ++kb)
#pragma unroll
      for (int r = 0; r < 16; ++r) mx = fmaxf(mx, s[kb][r]);
    {
      auto sw = __builtin_amdgcn_permlane32_swap(__float_as_uint(mx), __float_as_uint(mx), false, false);
      mx = fmaxf(__uint_as_float(sw[0]), __uint_as_float(sw[1]));
    }
    const float m_new = fmaxf(m_ref, mx * p.scale_log2);
    if (__builtin_amdgcn_ballot_w64(m_new > m_ref + kRescaleThreshold) != 0) {
      // m_ref = -inf before the first visible key: alpha = 0; a row still without one (m_new = -inf) keeps its zeros
      const float alpha = m_new > -INFINITY ? __builtin_amdgcn_exp2f(m_ref - m_new) : 1.f;
      m_ref = m_new;
      l_run *= alpha;
#pragma unroll
      for (int d = 0; d < T::DB; ++d)
#pragma unroll
        for (int r = 0; r < 16; ++r) o[d][r] *= alpha;
    }
    // (a row that has not seen a visible key yet -- possible in a key split -- keeps m_ref = -inf: subtract 0,
    // every probability is exp2(-inf) = 0)
    const float m_sub = m_ref > -INFINITY ? m_ref : 0.f;
#pragma unroll
    for (int kb = 0; kb < 2; ++kb)
#pragma unroll
      for (int r = 0; r < 16; ++r) s[kb][r] = __builtin_amdgcn_exp2f(__builtin_fmaf(s[kb][r], p.scale_log2, -m_sub));

    // ---- O^T += V^T P^T
#pragma unroll
    for (int kb = 0; kb < 2; ++kb)
#pragma unroll
      for (int tt = 0; tt < 2; ++tt) {
        // round P to bf16 (the PV operand) and add the rounded values into the row sum, two per dot2
        bf16x8 pf;
#pragma unroll
        for (int e = 0; e < 8; e += 2) {
          f32x2 xy = {s[kb][8 * tt + e], s[kb][8 * tt + e + 1]};
          bf16x2 c = __builtin_convertvector(xy, bf16x2);
          l_run = __builtin_amdgcn_fdot2_f32_bf16(c, bf16x2{(__bf16)1.0f, (__bf16)1.0f}, l_run, false);
          pf[e] = c[0];
          pf[e + 1] = c[1];
        }
        const int row_off = (32 * kb + 16 * tt) * T::ROW_BYTES;
#pragma unroll
        for (int d = 0; d < T::DB; ++d) {
          const s16x4 lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16((APBV_LDS(s16x4))(vt + row_off + v_off[d]));
          const s16x4 hi = __builtin_amdgcn_ds_read_tr16_b64_v4i16((APBV_LDS(s16x4))(vt + row_off + 8 * T::ROW_BYTES + v_off[d]));
          typedef __attribute__((ext_vector_type(8))) short s16x8;
          const s16x8 a = __builtin_shufflevector(lo, hi, 0, 1, 2, 3, 4, 5, 6, 7);
          o[d] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, a), pf, o[d], 0, 0, 0);
        }
      }
  };

  // ---- key loop: LDS double buffer, the loads of tile t+1 in flight while tile t is computed
  TileStream<D, W> ts;
  ts.init(ks, vs, p.s_kv, wave, lane, t_begin);
  const uint32_t k0 = lds_addr(k_lds0), k1 = lds_addr(k_lds1), v0 = lds_addr(v_lds0), v1 = lds_addr(v_lds1);
  // The Q fragments are in (vmcnt 0, other counters untouched): from here on only tile loads are
  // outstanding, and the compiler knows it need not wait for vector memory inside the loop.
  __builtin_amdgcn_s_waitcnt(0x0F70);
  if (t_begin < n_tiles) ts.issue(k0, v0);
  for (int t = t_begin; t < n_tiles; t += 2) {
    asm volatile("s_waitcnt vmcnt(0)" ::: "memory");  // this wave's share of tile t has landed
    __syncthreads();                                  // ... everyone's has, and everyone is done with the other buffer
    if (t + 1 < n_tiles) ts.issue(k1, v1);
    compute(k_lds0, v_lds0, t);
    if (t + 1 >= n_tiles) break;
    asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
    __syncthreads();
    if (t + 2 < n_tiles) ts.issue(k0, v0);
    compute(k_lds1, v_lds1, t + 1);
  }

  // ---- epilogue: normalise, round to bf16, store; optional log-sum-exp
  float l_tot;
  {
    auto sw = __builtin_amdgcn_permlane32_swap(__float_as_uint(l_run), __float_as_uint(l_run), false, false);
    l_tot = __uint_as_float(sw[0]) + __uint_as_float(sw[1]);
  }
  const float inv = l_tot > 0.f ? 1.0f / l_tot : 0.f;     // a key split may leave a row without any visible key
  if (i_row < p.L) {
    bf16_t* orow = p.out + (int64_t)split * p.split_stride_out + (((int64_t)b * p.L + i_row) * p.hq + h) * D;
#pragma unroll
    for (int d = 0; d < T::DB; ++d)
#pragma unroll
      for (int gq = 0; gq < 4; ++gq) {
        f32x2 x01 = {o[d][4 * gq + 0] * inv, o[d][4 * gq + 1] * inv};
        f32x2 x23 = {o[d][4 * gq + 2] * inv, o[d][4 * gq + 3] * inv};
        bf16x2 c01 = __builtin_convertvector(x01, bf16x2);
        bf16x2 c23 = __builtin_convertvector(x23, bf16x2);
        u32x2 w;
        w.x = __builtin_bit_cast(uint32_t, c01);
        w.y = __builtin_bit_cast(uint32_t, c23);
        *reinterpret_cast<u32x2*>(orow + 32 * d + 8 * gq + 4 * hh) = w;
      }
    if (p.lse != nullptr && hh == 0)
      p.lse[(int64_t)split * p.split_stride_lse + ((int64_t)b * p.hq + h) * p.L + i_row] =
          l_tot > 0.f ? (m_ref + __builtin_amdgcn_logf(l_tot)) * 0.6931471805599453f : -INFINITY;
  }
}

// ---- workgroup -> (query tile, head, batch, key range); the heads of one KV group share an XCD
template <int D, int W>
__global__ __launch_bounds__(64 * W, 2) void host_attention_kernel(const AttnParams p, const int n_qtiles,
                                                                   const int n_items) {
  const int xcd = blockIdx.x % kXcds;
  const int slot = blockIdx.x / kXcds;
  const int item_split = (slot / p.group) * kXcds + xcd;
  if (item_split >= n_items) return;
  const int split = item_split % p.n_splits;     // key ranges of one item share nothing: spread them over the XCDs
  const int item = item_split / p.n_splits;
  const int g = slot % p.group;
  const int bh = p.batch * p.hkv;
  const int qt = n_qtiles - 1 - item / bh;       // heaviest query tiles first
  const int b = (item % bh) / p.hkv;
  const int kvh = (item % bh) % p.hkv;
  attention_workgroup<D, W>(p, qt, b, kvh, g, split);
}

// ---- several attention problems of different lengths in one launch (the two virtual hosts and the anchor
// block of a physical host, Alg. 1 / Sec. 4.3): one workgroup per entry of the merged heaviest-first order of
// all (problem, query tile) pairs, per KV head and group member.
template <int D>
__global__ __launch_bounds__(64 * kWaves, 2) void host_attention_group_kernel(const AttnGroupParams gp) {
  const int group = gp.item[0].group, hkv = gp.item[0].hkv;
  const int xcd = blockIdx.x % kXcds;
  const int slot = blockIdx.x / kXcds;
  const int unit = (slot / group) * kXcds + xcd;
  if (unit >= gp.sched.n_entries * hkv) return;
  const int g = slot % group;
  const int entry = unit / hkv, kvh = unit % hkv;
  int m, qt;
  decode_group_entry(gp.sched, entry, m, qt);
  if (m >= gp.n_items || qt < 0 || (int64_t)qt * kBM >= gp.item[m].L) return;      // never taken for a schedule the launcher built
  attention_workgroup<D, kWaves>(gp.item[m], qt, 0, kvh, g, 0);
}

}  // namespace

template <int W>
static apbv_status launch_variant(const AttnParams& p, int head_dim, hipStream_t stream) {
  constexpr int kRows = 32 * W;
  const int n_qtiles = (int)((p.L + kRows - 1) / kRows);
  const int64_t n_items = (int64_t)n_qtiles * p.batch * p.hkv * p.n_splits;
  const int64_t n_blocks = (n_items + kXcds - 1) / kXcds * kXcds * p.group;
  if (n_blocks > 0x7fffffff) return APBV_ERR_UNSUPPORTED;
  dim3 grid((unsigned)n_blocks);
  dim3 block(64 * W);
  Launcher launch(stream);
  if (head_dim == 128)
    launch(host_attention_kernel<128, W>, grid, block, 0, p, n_qtiles, (int)n_items);
  else if (head_dim == 64)
    launch(host_attention_kernel<64, W>, grid, block, 0, p, n_qtiles, (int)n_items);
  else
    return APBV_ERR_UNSUPPORTED;
  return launch.status();
}

// Query blocks of at most kAttnNarrowMaxRows rows take the 64-row workgroups: a 256-row tile would compute mostly
// padding rows for them.
apbv_status launch_host_attention(const AttnParams& p, int head_dim, hipStream_t stream) {
  static_assert(kAttnQueryTile == kBM && kAttnNarrowQueryTile == 32 * kWavesNarrow, "tile sizes the host-side planning assumes");
  if (p.L <= kAttnNarrowMaxRows) return launch_variant<kWavesNarrow>(p, head_dim, stream);
  return launch_variant<kWaves>(p, head_dim, stream);
}

apbv_status launch_host_attention_group(AttnGroupParams& gp, int head_dim, hipStream_t stream) {
  static_assert(kGroupQueryTile == kBM, "the schedule's query tile is the kernel's");
  static_assert(sizeof(AttnGroupParams) <= 4096, "kernel arguments are limited to 4 KB");
  const int n = gp.n_items;
  if (n < 1 || n > kMaxGroupItems) return APBV_ERR_UNSUPPORTED;
  int64_t n_vis[kMaxGroupItems], rows[kMaxGroupItems];
  for (int m = 0; m < n; ++m) {
    n_vis[m] = gp.item[m].n_vis;
    rows[m] = gp.item[m].L;
  }
  if (!build_group_schedule(n, n_vis, rows, gp.sched)) return APBV_ERR_UNSUPPORTED;
  const int64_t first = gp.sched.n_entries;
  const AttnParams& p0 = gp.item[0];
  const int64_t n_units = first * p0.hkv;
  const int64_t n_blocks = (n_units + kXcds - 1) / kXcds * kXcds * p0.group;
  if (n_blocks > 0x7fffffff) return APBV_ERR_UNSUPPORTED;
  dim3 grid((unsigned)n_blocks);
  dim3 block(64 * kWaves);
  Launcher launch(stream);
  if (head_dim == 128)
    launch(host_attention_group_kernel<128>, grid, block, 0, gp);
  else if (head_dim == 64)
    launch(host_attention_group_kernel<64>, grid, block, 0, gp);
  else
    return APBV_ERR_UNSUPPORTED;
  return launch.status();
}

}  // namespace apbv
