// Fused host attention for gfx950 (Eq. 4 by the definition of Eq. 1): one pass of online-softmax
// attention of the local query block over the concatenated keys [anchor | passing | local].
//
// Mask.  The three KV segments are walked as ONE virtual key axis j in [0, n_vis + L): anchor and
// passing keys (j < n_vis) are visible to every query and local key j - n_vis is visible to query i iff
// j - n_vis <= i, so the whole mask is the single test  j <= i + n_vis  (a causal mask shifted by
// n_vis).  Without a local segment (partial attention of a query block over context keys only, merged
// later by log-sum-exp) the bound is simply the last key.  Key tiles that lie entirely above that
// diagonal are never visited, and only tiles that touch it pay for the comparison.
//
// Tiling.  A workgroup of 8 waves (two per SIMD, one workgroup per CU) owns 256 consecutive query
// positions of one query head; each wave owns 32 of them.  Key tiles of 32 virtual keys are copied
// global -> LDS by the LDS-direct load (global_load_lds_dwordx4: no VGPR staging, no VALU work) into rings
// of four K and four V tiles, one barrier per two tiles.  Both are stored row-major [32][D] with an XOR
// swizzle of their 16-byte chunks; the swizzle is applied on the global side (which chunk a lane
// fetches), because an LDS-direct load always writes lane l's 16 bytes at base + 16*l.
//
// MFMA mapping (v_mfma_f32_16x16x32_bf16; with g = lane/16, i = lane%16: A is 16x32 with the lane
// holding row i, k-slots 8g..8g+7; B is 32x16 with the lane holding column i, the same k-slots; D is
// 16x16 with the lane holding column i, rows 4g..4g+3).  The 16x16x32 shape moves half the accumulator
// bytes per flop of the 32x32x16 one; on this power-limited part that is worth a higher clock.
//   S^T = K Q^T  : A = 16 key rows x 32 head-dim columns (one 16-byte LDS read per lane, used for both
//                  16-query blocks of the wave), B = Q^T kept in registers.  A lane then holds, for each of
//                  its two queries (i and 16 + i of the wave), keys 16*mb + 4g + r of the tile (mb = 0, 1).
//   O^T = V^T P^T: B = P^T straight from the S^T accumulator registers (rounded to bf16), no LDS round
//                  trip.  That fixes which key sits in which k-slot (slot 8g + e: key
//                  16 (e/4) + 4g + e%4); A = V^T is fetched to match with two transposing LDS
//                  reads (ds_read_b64_tr_b16: within 16 lanes, lane i receives element i%4 of the 8
//                  bytes addressed by lanes i/4, 4+i/4, 8+i/4, 12+i/4), each delivering 4 consecutive
//                  keys of one head-dim column.
//
// Softmax.  exp2 domain with the scale folded in.  The reference maximum m_ref of a query only moves when
// some logit exceeds it by more than 2^8 (then O and l are rescaled): probabilities stay <= 2^8, and the
// common path needs only each lane's own maximum over its 8 keys per query -- no cross-lane exchange.
//
// Software pipeline.  The steps of a tile form a chain (S^T -> maximum -> exp -> P^T -> O^T); done tile
// after tile a wave alternates between the matrix pipe and the vector ALU, and every LDS fragment read
// is waited for where it is issued.  Here, while the matrix pipe computes S^T of tile t+1, the vector
// ALU exponentiates tile t and the V^T operands of tile t are read; while it accumulates O^T of tile t,
// the vector ALU takes the maxima of tile t+1 and the K fragments of tile t+2 are read.  K therefore
// runs one tile ahead of V in LDS, and no LDS read is consumed in the phase that issues it.  Tiles that
// touch the mask diagonal, and the few rounds around a segment boundary, take the plain sequence.
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
constexpr int kBN = 32;            // keys per tile (one k-step of O^T)
constexpr int kRing = 4;           // K tiles, and V tiles, resident in LDS
constexpr int kXcds = 8;
constexpr float kRescaleThreshold = 8.0f;   // log2 units

#define APBV_LDS(T) __attribute__((address_space(3))) T*

typedef __attribute__((ext_vector_type(4))) short s16x4;
typedef __attribute__((ext_vector_type(8))) short s16x8;

// Compile-time loop: f(std::integral_constant<int, 0>{}) ... f(std::integral_constant<int, N-1>{}).
template <typename F, int... I>
__device__ __forceinline__ void static_for_impl(F&& f, std::integer_sequence<int, I...>) {
  (f(std::integral_constant<int, I>{}), ...);
}
template <int N, typename F>
__device__ __forceinline__ void static_for(F&& f) {
  static_for_impl(f, std::make_integer_sequence<int, N>{});
}

template <int D, int W>
struct Tile {
  static constexpr int ROW_BYTES = D * 2;
  static constexpr int KC = D / 8;                        // 16-byte chunks per row
  static constexpr int RPI = 1024 / ROW_BYTES;            // rows covered by one wave-wide LDS-direct load
  static constexpr int LOADS = kBN / RPI;                 // such loads per tile (per tensor)
  static constexpr int IPW = (LOADS + W - 1) / W;         // ... per wave; wave w issues loads w*IPW + u while < LOADS
  static constexpr int KSD = D / 32;                      // MFMA k-steps over the head dimension (S^T)
  static constexpr int DBN = D / 16;                      // 16-row blocks of O^T
  static constexpr int TILE_BYTES = kBN * ROW_BYTES;
  // chunk swizzles (functions of the row within the tile), chosen so that the 16 rows x 16 bytes of a quarter of
  // a K read and the 8 rows x 32 bytes of half a transposing V read cover the 64 LDS banks exactly once
  __device__ static __forceinline__ int fk(int r) { return D == 128 ? (r & 15) : ((r >> 1) & 7); }
  __device__ static __forceinline__ int fv(int r) { return D == 128 ? ((r & 7) << 1) : (((r >> 1) & 3) << 1); }
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

// Sequential producer of the tiles of ONE tensor (K or V) along the virtual key axis.  While consecutive tiles
// stay inside one segment ("run") a tile costs one 64-bit scalar add and its loads are  uniform tile base + a
// per-lane 32-bit offset computed once per run; the tile that straddles a segment boundary (or the end of the
// keys) takes a per-row lookup.
template <int D, int W, bool kIsV>
struct TileStream {
  using T = Tile<D, W>;
  Segs sg;
  int64_t s_kv;
  int t_next;              // next tile to issue
  int run_end;             // tiles [t_next, run_end) lie inside one segment; base points at tile t_next
  const char* base;
  int64_t step;            // kBN * pitch
  uint32_t off[T::IPW];
  int wave, lane;

  __device__ static __forceinline__ int swz(int r) { return kIsV ? T::fv(r) : T::fk(r); }
  __device__ __forceinline__ int row(int u) const { return (wave * T::IPW + u) * T::RPI + lane / T::KC; }
  __device__ __forceinline__ uint32_t ldst(int u) const { return (uint32_t)((wave * T::IPW + u) * T::RPI * T::ROW_BYTES); }

  __device__ __forceinline__ void init(const Segs& s, int64_t skv, int w, int l, int t_first) {
    sg = s;
    s_kv = skv;
    wave = w;
    lane = l;
    t_next = t_first;
    run_end = t_first;
    base = nullptr;
    step = 0;
#pragma unroll
    for (int u = 0; u < T::IPW; ++u) off[u] = 0;
  }

  // Start a run at tile t_next if that tile lies inside one segment.
  __device__ __forceinline__ void start_run() {
    const int64_t j0 = (int64_t)t_next * kBN;
    const char* b;
    int64_t pitch, start, end;
    seg_of(sg, j0, b, pitch, start, end);
    if (j0 + kBN > end) return;                      // straddling tile: run stays empty
    run_end = (int)(end / kBN);
    base = b + (j0 - start) * pitch;
    step = kBN * pitch;
#pragma unroll
    for (int u = 0; u < T::IPW; ++u) {
      const int r = row(u);
      off[u] = (uint32_t)r * (uint32_t)pitch + 16u * (uint32_t)((lane % T::KC) ^ swz(r));
    }
  }

  // Whether load u of a tile is this wave's to issue (always, when the loads divide evenly among the waves).
  __device__ __forceinline__ bool mine(int u) const { return W * T::IPW == T::LOADS || wave * T::IPW + u < T::LOADS; }

  // Tiles that can still be issued from the current run without a lookup (after trying to start a run if none is open).
  __device__ __forceinline__ int run_left() {
    if (t_next >= run_end) start_run();
    return run_end - t_next;
  }
  // Issue tile t_next, which the caller knows to lie inside the current run: no tests.
  __device__ __forceinline__ void issue_in_run(uint32_t dst) {
    const char* bu = uniform_ptr(base);
#pragma unroll
    for (int u = 0; u < T::IPW; ++u)
      if (mine(u)) dma16_uniform(bu, off[u], dst + ldst(u));
    base += step;
    ++t_next;
  }

  // Issue this wave's share of the loads of tile t_next into the LDS tile at dst.
  __device__ __forceinline__ void issue(uint32_t dst) {
    if (t_next >= run_end) start_run();
    if (t_next < run_end) {
      const char* bu = uniform_ptr(base);
#pragma unroll
      for (int u = 0; u < T::IPW; ++u)
        if (mine(u)) dma16_uniform(bu, off[u], dst + ldst(u));
      base += step;
    } else {
      const int64_t j0 = (int64_t)t_next * kBN;
#pragma unroll
      for (int u = 0; u < T::IPW; ++u) {
        if (!mine(u)) continue;
        const int r = row(u);
        int64_t j = j0 + r;
        j = j < s_kv ? j : s_kv - 1;                 // rows past the end repeat the last key: always masked
        const char* b;
        int64_t pitch, sj, ej;
        seg_of(sg, j, b, pitch, sj, ej);
        dma16_lane(b + (j - sj) * pitch + 16 * ((lane % T::KC) ^ swz(r)), dst + ldst(u));
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
  __shared__ __attribute__((aligned(1024))) unsigned char k_lds[kRing][T::TILE_BYTES];
  __shared__ __attribute__((aligned(1024))) unsigned char v_lds[kRing][T::TILE_BYTES];
  // the LDS destination of an LDS-direct load travels in M0, which addresses the first 64 KB of the workgroup's LDS
  static_assert(2 * kRing * T::TILE_BYTES <= 65536, "the K/V tile rings must lie below 64 KB of LDS");
  const int h = kvh * p.group + g;

  const int tid = threadIdx.x;
  const int lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);   // uniform: keeps LDS tile addresses in SGPRs
  const int li = lane & 15;       // query column / A-operand row within a 16-block
  const int lg = lane >> 4;       // lane group: k-slots 8 lg .. 8 lg + 7, accumulator rows 4 lg .. 4 lg + 3

  const int64_t i0 = (int64_t)qt * kRows;               // first query position of the workgroup
  const int64_t iw = i0 + wave * 32;                    // first query position of the wave
  const int64_t i_row[2] = {iw + li, iw + 16 + li};     // this lane's two query positions

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

  // ---- Q^T fragments (B operand of S^T), kept in registers for the whole key loop.
  bf16x8 qf[T::KSD][2];
#pragma unroll
  for (int nq = 0; nq < 2; ++nq) {
    const bf16_t* qrow = p.q.ptr + (int64_t)b * p.q.sb + (int64_t)h * p.q.sh + (i_row[nq] < p.L ? i_row[nq] : p.L - 1) * p.q.st;
#pragma unroll
    for (int c = 0; c < T::KSD; ++c) qf[c][nq] = __builtin_bit_cast(bf16x8, *reinterpret_cast<const u32x4*>(qrow + 32 * c + 8 * lg));
  }

  // ---- per-lane LDS read offsets
  // K (A operand of S^T): row 16*mb + li, 16-byte chunk (4*c + lg) ^ fk(row); fk does not depend on mb
  int k_off[T::KSD];
#pragma unroll
  for (int c = 0; c < T::KSD; ++c) k_off[c] = li * T::ROW_BYTES + (((4 * c + lg) ^ T::fk(li)) << 4);
  // V (A operand of O^T, transposing read): within a 16-lane group, source lane s addresses key row 4*lg + s/4
  // (+ 16 for the second half of the k-slots, as an immediate; fv does not depend on it), head-dim columns
  // 16*d + 4*(s%4) .. +3
  int v_off[T::DBN];
  {
    const int row = 4 * lg + (li >> 2);
#pragma unroll
    for (int d = 0; d < T::DBN; ++d) {
      const int chunk = 2 * d + ((li & 3) >> 1);
      v_off[d] = row * T::ROW_BYTES + ((chunk ^ T::fv(row)) << 4) + (li & 1) * 8;
    }
  }

  // ---- online softmax state.  Per lane: two queries (nq = 0, 1); the four lane groups hold disjoint key subsets.
  f32x4 o[T::DBN][2];
#pragma unroll
  for (int d = 0; d < T::DBN; ++d)
#pragma unroll
    for (int nq = 0; nq < 2; ++nq) o[d][nq] = f32x4{0.f, 0.f, 0.f, 0.f};
  float m_ref[2] = {-INFINITY, -INFINITY};   // reference maximum of the scaled (log2-domain) logits, whole row
  float m_sub[2] = {0.f, 0.f};               // what the exponent subtracts: m_ref, or 0 while m_ref = -inf
  float s_far[2] = {-INFINITY, -INFINITY};   // raw logits above this move the reference: (m_ref + threshold) / scale
  float l_run[2] = {0.f, 0.f};               // running sum of the bf16-rounded exp2(. - m_ref), this lane's keys only
  const float inv_scale_log2 = 1.0f / p.scale_log2;

  // Keys the workgroup / this wave can see at all.
  // Query i sees the virtual keys 0 .. min(i + n_vis, s_kv - 1); the second bound only matters when there is no
  // causal segment (s_kv == n_vis: every key visible to every query).
  auto last_key = [&](int64_t i) { return (i + p.n_vis < p.s_kv - 1) ? i + p.n_vis : p.s_kv - 1; };
  const int64_t i_last_wg = (i0 + kRows - 1 < p.L - 1) ? i0 + kRows - 1 : p.L - 1;
  const int n_tiles_vis = (int)(last_key(i_last_wg) / kBN) + 1;      // tiles the workgroup can see into
  // key split (partial results merged afterwards): this workgroup walks tiles [t_begin, n_tiles) only; the split is
  // planned in 64-key units
  const int64_t per_split = (int64_t)p.tiles_per_split * (64 / kBN);
  const int64_t t_begin64 = (int64_t)split * per_split;
  const int t_begin = (int)(t_begin64 < n_tiles_vis ? t_begin64 : n_tiles_vis);
  const int n_tiles = (int)(t_begin64 + per_split < n_tiles_vis ? t_begin64 + per_split : n_tiles_vis);
  const int t_last_wave = (int)(last_key(iw + 31) / kBN);     // last tile any row of the wave can see into
  const int n_w = t_last_wave + 1 < n_tiles ? t_last_wave + 1 : n_tiles;     // the wave computes tiles [t_begin, n_w)
  const int t_mask_wave = (int)((last_key(iw) + 1) / kBN);    // first tile with a key some row of the wave cannot see
  const int jrel0[2] = {(int)last_key(i_row[0]), (int)last_key(i_row[1])};   // last visible virtual key of each query

  typedef f32x4 STile[2][2];       // S^T of one tile: [16-key block][16-query block]
  typedef u32x4 PTile[2];          // P^T of one tile as the B operand of O^T: [16-query block], four 32-bit words

  auto read_k = [&](const unsigned char* kt, int mb, int c) {
    return __builtin_bit_cast(bf16x8, *reinterpret_cast<const u32x4*>(kt + mb * 16 * T::ROW_BYTES + k_off[c]));
  };
  auto read_vt = [&](const unsigned char* vt, int d) {
    const s16x4 lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16((APBV_LDS(s16x4))(vt + v_off[d]));
    const s16x4 hi = __builtin_amdgcn_ds_read_tr16_b64_v4i16((APBV_LDS(s16x4))(vt + 16 * T::ROW_BYTES + v_off[d]));
    return __builtin_bit_cast(bf16x8, __builtin_shufflevector(lo, hi, 0, 1, 2, 3, 4, 5, 6, 7));
  };

  // ---- S^T = K Q^T of one tile
  auto qk = [&](const unsigned char* kt, STile& s) {
#pragma unroll
    for (int c = 0; c < T::KSD; ++c)
#pragma unroll
      for (int mb = 0; mb < 2; ++mb) {
        const bf16x8 a = read_k(kt, mb, c);
#pragma unroll
        for (int nq = 0; nq < 2; ++nq)
          s[mb][nq] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(a, qf[c][nq], c == 0 ? f32x4{0.f, 0.f, 0.f, 0.f} : s[mb][nq], 0, 0, 0);
      }
  };

  // ---- mask of a tile that reaches above the wave's first diagonal element
  auto apply_mask = [&](STile& s, int t) {
#pragma unroll
    for (int nq = 0; nq < 2; ++nq) {
      const int jrel_max = jrel0[nq] - t * kBN;          // last visible key of this query, tile-relative
#pragma unroll
      for (int mb = 0; mb < 2; ++mb)
#pragma unroll
        for (int r = 0; r < 4; ++r)
          if (16 * mb + 4 * lg + r > jrel_max) s[mb][nq][r] = -INFINITY;
    }
  };

  // ---- this lane's largest logit per query
  auto lane_max = [&](const STile& s, float (&lm)[2]) {
#pragma unroll
    for (int nq = 0; nq < 2; ++nq) {
      float mx = __builtin_fmaxf(s[0][nq][0], s[0][nq][1]);
#pragma unroll
      for (int mb = 0; mb < 2; ++mb)
#pragma unroll
        for (int r = (mb == 0 ? 2 : 0); r < 4; ++r) mx = __builtin_fmaxf(mx, s[mb][nq][r]);
      lm[nq] = mx;
    }
  };

  // ---- lazy rescaling: the reference maximum moves only when some logit of the tile exceeds it by more than the
  // threshold; then it becomes the exact row maximum so far and O, l are rescaled.  (m_ref = -inf before the first
  // visible key: alpha = 0; a row still without one keeps its zeros.  The test is a NaN-free comparison of raw
  // logits: s_far = -inf while m_ref = -inf, so the first finite logit moves the reference.)
  auto advance_reference = [&](const float (&lm)[2]) {
    if ((__builtin_amdgcn_ballot_w64(lm[0] > s_far[0]) | __builtin_amdgcn_ballot_w64(lm[1] > s_far[1])) != 0) {
#pragma unroll
      for (int nq = 0; nq < 2; ++nq) {
        float mx = lm[nq];
        {
          auto sw = __builtin_amdgcn_permlane16_swap(__float_as_uint(mx), __float_as_uint(mx), false, false);
          mx = fmaxf(__uint_as_float(sw[0]), __uint_as_float(sw[1]));
        }
        {
          auto sw = __builtin_amdgcn_permlane32_swap(__float_as_uint(mx), __float_as_uint(mx), false, false);
          mx = fmaxf(__uint_as_float(sw[0]), __uint_as_float(sw[1]));
        }
        const float m_new = fmaxf(m_ref[nq], mx * p.scale_log2);
        const float alpha = m_new > -INFINITY ? __builtin_amdgcn_exp2f(m_ref[nq] - m_new) : 1.f;
        m_ref[nq] = m_new;
        m_sub[nq] = m_new > -INFINITY ? m_new : 0.f;
        s_far[nq] = (m_new + kRescaleThreshold) * inv_scale_log2;
        l_run[nq] *= alpha;
#pragma unroll
        for (int d = 0; d < T::DBN; ++d) o[d][nq] *= alpha;
      }
    }
  };

  // ---- probabilities of the tile for query block nq: exp2 of the scaled logits minus the reference, rounded to bf16
  // (the PV operand) with the rounded values added into the row sum two at a time.  (A row that has not seen a
  // visible key yet -- possible in a key split -- has m_ref = -inf: subtract 0, every probability is exp2(-inf) = 0.)
  auto exp_block = [&](const STile& s, int nq, PTile& pw) {
#pragma unroll
    for (int mb = 0; mb < 2; ++mb)
#pragma unroll
      for (int e = 0; e < 4; e += 2) {
        f32x2 xy = {__builtin_amdgcn_exp2f(__builtin_fmaf(s[mb][nq][e], p.scale_log2, -m_sub[nq])),
                    __builtin_amdgcn_exp2f(__builtin_fmaf(s[mb][nq][e + 1], p.scale_log2, -m_sub[nq]))};
        const bf16x2 c = __builtin_convertvector(xy, bf16x2);
        l_run[nq] = __builtin_amdgcn_fdot2_f32_bf16(c, bf16x2{(__bf16)1.0f, (__bf16)1.0f}, l_run[nq], false);
        pw[nq][2 * mb + (e >> 1)] = __builtin_bit_cast(uint32_t, c);
      }
  };

  // ---- O^T += V^T P^T for the 32 keys of the tile
  auto pv = [&](const unsigned char* vt, const PTile& pw) {
#pragma unroll
    for (int d = 0; d < T::DBN; ++d) {
      const bf16x8 a = read_vt(vt, d);
#pragma unroll
      for (int nq = 0; nq < 2; ++nq)
        o[d][nq] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(a, __builtin_bit_cast(bf16x8, pw[nq]), o[d][nq], 0, 0, 0);
    }
  };

  // ---- plain sequence, for the first tile and for tiles on the mask diagonal
  auto prepare = [&](const unsigned char* kt, int t, STile& s) {       // S^T, mask, reference
    qk(kt, s);
    if (t >= t_mask_wave) apply_mask(s, t);
    float lm[2];
    lane_max(s, lm);
    advance_reference(lm);
  };
  auto finish = [&](const unsigned char* vt, const STile& s) {          // probabilities, O^T
    PTile pw;
    exp_block(s, 0, pw);
    exp_block(s, 1, pw);
    pv(vt, pw);
  };

  // ---- pipelined body: finishes tile t (S^T in sc, V tile at vt) while it prepares tile t+1 (K fragments already
  // in kf, S^T into sn).  No LDS read is waited for where it is issued: the K fragments of a tile are read one phase
  // ahead, the V^T operands of phase B during phase A.
  //   phase A: S^T(t+1) on the matrix pipe from kf; the exponentials of tile t on the vector ALU; the V^T operands of
  //            tile t read into vf
  //   phase B: O^T(t) from vf; the lane maxima of tile t+1; with kPrefetchK the K fragments of tile t+2 (at
  //            kt_after, landed since the last barrier) read into kf
  typedef bf16x8 KFrags[2 * T::KSD];        // [c][mb]
  auto load_k = [&](const unsigned char* kt, KFrags& kf) {
#pragma unroll
    for (int c = 0; c < T::KSD; ++c)
#pragma unroll
      for (int mb = 0; mb < 2; ++mb) kf[2 * c + mb] = read_k(kt, mb, c);
  };
  auto pipelined = [&](auto prefetch_k, KFrags& kf, const unsigned char* kt_after, const unsigned char* vt,
                       const STile& sc, STile& sn) {
    constexpr bool kPrefetchK = decltype(prefetch_k)::value;
    // The source lists each matrix instruction with its share of the vector and LDS instructions; the compiler's own
    // scheduler keeps that interleaving (pinning it with scheduling fences was measured 3 % slower).
    // exponential pipeline of tile t, one pair of probabilities at a time: pair pi = (nq, mb, first/second two rows);
    // stages F (scale and subtract), E (exp2), C (round to bf16 into the B operand word), D (row sum)
    float xf[8][2];
    uint32_t cw[8];
    PTile pw;
    auto stage_f = [&](int pi) {
      const int nq = pi >> 2, mb = (pi >> 1) & 1, e = 2 * (pi & 1);
      xf[pi][0] = __builtin_fmaf(sc[mb][nq][e], p.scale_log2, -m_sub[nq]);
      xf[pi][1] = __builtin_fmaf(sc[mb][nq][e + 1], p.scale_log2, -m_sub[nq]);
    };
    auto stage_e = [&](int pi) {
      xf[pi][0] = __builtin_amdgcn_exp2f(xf[pi][0]);
      xf[pi][1] = __builtin_amdgcn_exp2f(xf[pi][1]);
    };
    auto stage_c = [&](int pi) {
      const int nq = pi >> 2, mb = (pi >> 1) & 1;
      f32x2 xy = {xf[pi][0], xf[pi][1]};
      cw[pi] = __builtin_bit_cast(uint32_t, __builtin_convertvector(xy, bf16x2));
      pw[nq][2 * mb + (pi & 1)] = cw[pi];
    };
    auto stage_d = [&](int pi) {
      const int nq = pi >> 2;
      l_run[nq] = __builtin_amdgcn_fdot2_f32_bf16(__builtin_bit_cast(bf16x2, cw[pi]), bf16x2{(__bf16)1.0f, (__bf16)1.0f}, l_run[nq], false);
    };
    // ---- phase A: one slice per matrix instruction of S^T(t+1)
    s16x4 vlo[T::DBN], vhi[T::DBN];
    constexpr int nA = 4 * T::KSD;                 // matrix instructions of phase A
    static_for<nA>([&](auto I) {
      constexpr int i = I;
      constexpr int c = i / 4, nq = (i / 2) % 2, mb = i % 2;
      sn[mb][nq] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(kf[2 * c + mb], qf[c][nq],
                                                           c == 0 ? f32x4{0.f, 0.f, 0.f, 0.f} : sn[mb][nq], 0, 0, 0);
      // the 16 slices of the exponential pipeline are spread evenly over the nA matrix instructions
      constexpr int s0 = (16 * i) / nA, s1 = (16 * (i + 1)) / nA;
      static_for<s1 - s0>([&](auto J) {
        constexpr int sl = s0 + J, pi = sl / 2;
        if constexpr (sl % 2 == 0) {
          stage_f(pi);
          if constexpr (pi > 0) stage_c(pi - 1);
        } else {
          stage_e(pi);
          if constexpr (pi > 0) stage_d(pi - 1);
        }
      });
      // ... and the 2 DBN transposing reads of the V^T operands of phase B
      constexpr int r0 = (2 * T::DBN * i) / nA, r1 = (2 * T::DBN * (i + 1)) / nA;
      static_for<r1 - r0>([&](auto J) {
        constexpr int r = r0 + J, d = r / 2;
        if constexpr (r % 2 == 0)
          vlo[d] = __builtin_amdgcn_ds_read_tr16_b64_v4i16((APBV_LDS(s16x4))(vt + v_off[d]));
        else
          vhi[d] = __builtin_amdgcn_ds_read_tr16_b64_v4i16((APBV_LDS(s16x4))(vt + 16 * T::ROW_BYTES + v_off[d]));
      });
    });
    stage_c(7);
    stage_d(7);
    // ---- phase B: one slice per matrix instruction of O^T(t)
    float lm[2];
    constexpr int nB = 2 * T::DBN, nK = kPrefetchK ? 2 * T::KSD : 0;
    static_for<nB>([&](auto I) {
      constexpr int i = I;
      constexpr int d = i / 2, nq = i % 2;
      const bf16x8 a = __builtin_bit_cast(bf16x8, __builtin_shufflevector(vlo[d], vhi[d], 0, 1, 2, 3, 4, 5, 6, 7));
      o[d][nq] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(a, __builtin_bit_cast(bf16x8, pw[nq]), o[d][nq], 0, 0, 0);
      // the K fragments of tile t+2
      constexpr int k0 = (nK * i) / nB, k1 = (nK * (i + 1)) / nB;
      static_for<k1 - k0>([&](auto J) {
        constexpr int k = k0 + J;
        kf[k] = read_k(kt_after, k % 2, k / 2);
      });
      // the lane maxima of tile t+1: 8 instructions
      constexpr int m0 = (8 * i) / nB, m1 = (8 * (i + 1)) / nB;
      static_for<m1 - m0>([&](auto J) {
        constexpr int m = m0 + J, nqm = m / 4, st = m % 4;
        if constexpr (st == 0) lm[nqm] = __builtin_fmaxf(sn[0][nqm][0], sn[0][nqm][1]);
        if constexpr (st == 1) lm[nqm] = __builtin_fmaxf(lm[nqm], __builtin_fmaxf(sn[0][nqm][2], sn[0][nqm][3]));
        if constexpr (st == 2) lm[nqm] = __builtin_fmaxf(lm[nqm], __builtin_fmaxf(sn[1][nqm][0], sn[1][nqm][1]));
        if constexpr (st == 3) lm[nqm] = __builtin_fmaxf(lm[nqm], __builtin_fmaxf(sn[1][nqm][2], sn[1][nqm][3]));
      });
    });
    advance_reference(lm);
  };

  // One tile step of the wave in the plain sequence: K(t+1) is at kt_next, V(t) at vt, S^T(t) in sc; leaves S^T(t+1)
  // in sn.
  auto step = [&](int t, const unsigned char* kt_next, const unsigned char* vt, STile& sc, STile& sn) {
    if (t >= n_w) return;
    finish(vt, sc);
    if (t + 1 < n_w) prepare(kt_next, t + 1, sn);
  };

  // ---- key loop.  With r = t - t_begin, K(t) and V(t) live in slot r % 4 of their rings, and K runs one tile ahead
  // of V in the computation.  One barrier per two tiles: after the barrier in front of tiles t, t+1 the tiles K(t+1),
  // K(t+2), V(t), V(t+1) have landed, everyone is done with K(t-1), K(t), V(t-2), V(t-1), and the loads of K(t+3),
  // K(t+4), V(t+2), V(t+3) go into those slots.
  TileStream<D, W, false> kst;
  TileStream<D, W, true> vst;
  kst.init(ks, p.s_kv, wave, lane, t_begin);
  vst.init(vs, p.s_kv, wave, lane, t_begin);
  uint32_t ka[kRing], va[kRing];
#pragma unroll
  for (int i = 0; i < kRing; ++i) {
    ka[i] = lds_addr(k_lds[i]);
    va[i] = lds_addr(v_lds[i]);
  }
  // The Q fragments are in (vmcnt 0, other counters untouched): from here on only tile loads are
  // outstanding, and the compiler knows it need not wait for vector memory inside the loop.
  __builtin_amdgcn_s_waitcnt(0x0F70);
  STile s_a, s_b;
  if (t_begin < n_tiles) {
    kst.issue(ka[0]);
    asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
    __syncthreads();
    if (t_begin + 1 < n_tiles) kst.issue(ka[1]);
    if (t_begin + 2 < n_tiles) kst.issue(ka[2]);
    vst.issue(va[0]);
    if (t_begin + 1 < n_tiles) vst.issue(va[1]);
    if (t_begin < n_w) prepare(k_lds[0], t_begin, s_a);
  }
  // loads of the two barrier intervals of a four-tile round that starts at tile t
  auto issue_first = [&](int t) {
    if (t + 3 < n_tiles) kst.issue(ka[3]);
    if (t + 4 < n_tiles) kst.issue(ka[0]);
    if (t + 2 < n_tiles) vst.issue(va[2]);
    if (t + 3 < n_tiles) vst.issue(va[3]);
  };
  auto issue_second = [&](int t) {
    if (t + 5 < n_tiles) kst.issue(ka[1]);
    if (t + 6 < n_tiles) kst.issue(ka[2]);
    if (t + 4 < n_tiles) vst.issue(va[0]);
    if (t + 5 < n_tiles) vst.issue(va[1]);
  };
  auto arrive = [&]() {
    asm volatile("s_waitcnt vmcnt(0)" ::: "memory");  // this wave's share of the tiles needed next has landed
    __syncthreads();                                  // ... everyone's has, and everyone is done with the slots reloaded now
  };
  int t = t_begin;
  const int t_pipe_end = n_w < t_mask_wave ? n_w : t_mask_wave;
  while (t < n_tiles) {
    // Rounds in which all four tiles and their successors are fully visible to the wave and every tile to be
    // loaded lies inside the streams' current runs: the pipelined body and unconditional loads, no tests.  (A round
    // loads K(t+3..t+6) and V(t+2..t+5).  Waves leave this loop at different rounds; every round of either kind
    // passes the same two barriers.)
    int n_hot = 0;
    if (t + 4 < t_pipe_end && t + 6 < n_tiles && kst.t_next == t + 3 && vst.t_next == t + 2) {
      const int by_mask = (t_pipe_end - 4 - t + 3) / 4;      // rounds that start at t' with t' + 4 < t_pipe_end
      const int by_end = (n_tiles - 6 - t + 3) / 4;          // ... and load existing tiles only: t' + 6 < n_tiles
      const int by_k = kst.run_left() / 4, by_v = vst.run_left() / 4;
      n_hot = by_mask < by_end ? by_mask : by_end;
      n_hot = n_hot < by_k ? n_hot : by_k;
      n_hot = n_hot < by_v ? n_hot : by_v;
    }
    KFrags kf;
    for (int r = 0; r < n_hot; ++r, t += 4) {
      arrive();
      load_k(k_lds[1], kf);
      kst.issue_in_run(ka[3]);
      kst.issue_in_run(ka[0]);
      vst.issue_in_run(va[2]);
      vst.issue_in_run(va[3]);
      pipelined(std::true_type{}, kf, k_lds[2], v_lds[0], s_a, s_b);
      pipelined(std::false_type{}, kf, nullptr, v_lds[1], s_b, s_a);
      arrive();
      load_k(k_lds[3], kf);
      kst.issue_in_run(ka[1]);
      kst.issue_in_run(ka[2]);
      vst.issue_in_run(va[0]);
      vst.issue_in_run(va[1]);
      pipelined(std::true_type{}, kf, k_lds[0], v_lds[2], s_a, s_b);
      pipelined(std::false_type{}, kf, nullptr, v_lds[3], s_b, s_a);
    }
    if (t >= n_tiles) break;
    // One round of the general kind: tiles on the mask diagonal, the wave's last tiles, rounds the wave only sits
    // through, loads that cross a segment boundary or stop at the last tile.
    arrive();
    issue_first(t);
    step(t, k_lds[1], v_lds[0], s_a, s_b);
    step(t + 1, k_lds[2], v_lds[1], s_b, s_a);
    if (t + 2 >= n_tiles) break;
    arrive();
    issue_second(t);
    step(t + 2, k_lds[3], v_lds[2], s_a, s_b);
    step(t + 3, k_lds[0], v_lds[3], s_b, s_a);
    t += 4;
  }

  // ---- epilogue: normalise, round to bf16, store; optional log-sum-exp
#pragma unroll
  for (int nq = 0; nq < 2; ++nq) {
    float l_tot = l_run[nq];
    {
      auto sw = __builtin_amdgcn_permlane16_swap(__float_as_uint(l_tot), __float_as_uint(l_tot), false, false);
      l_tot = __uint_as_float(sw[0]) + __uint_as_float(sw[1]);
    }
    {
      auto sw = __builtin_amdgcn_permlane32_swap(__float_as_uint(l_tot), __float_as_uint(l_tot), false, false);
      l_tot = __uint_as_float(sw[0]) + __uint_as_float(sw[1]);
    }
    const float inv = l_tot > 0.f ? 1.0f / l_tot : 0.f;     // a key split may leave a row without any visible key
    if (i_row[nq] < p.L) {
      bf16_t* orow = p.out + (int64_t)split * p.split_stride_out + (((int64_t)b * p.L + i_row[nq]) * p.hq + h) * D;
#pragma unroll
      for (int d = 0; d < T::DBN; ++d) {
        f32x2 x01 = {o[d][nq][0] * inv, o[d][nq][1] * inv};
        f32x2 x23 = {o[d][nq][2] * inv, o[d][nq][3] * inv};
        bf16x2 c01 = __builtin_convertvector(x01, bf16x2);
        bf16x2 c23 = __builtin_convertvector(x23, bf16x2);
        u32x2 w;
        w.x = __builtin_bit_cast(uint32_t, c01);
        w.y = __builtin_bit_cast(uint32_t, c23);
        *reinterpret_cast<u32x2*>(orow + 16 * d + 4 * lg) = w;
      }
      if (p.lse != nullptr && lg == 0)
        p.lse[(int64_t)split * p.split_stride_lse + ((int64_t)b * p.hq + h) * p.L + i_row[nq]] =
            l_tot > 0.f ? (m_ref[nq] + __builtin_amdgcn_logf(l_tot)) * 0.6931471805599453f : -INFINITY;
    }
  }
}

// Work items are numbered heaviest first, `period` consecutive ones (the KV heads, batch items and key ranges of one
// query tile) being equally heavy, and are dealt to the XCDs eight at a time.  Dealt always in the same direction,
// XCD 0 would get the heaviest item of every row of eight and XCD 7 the lightest -- 4 to 12 % more work for the one
// than for the other with a causal block.  Odd rows are therefore dealt in the opposite direction, in whole groups of
// `period` XCDs where that divides eight, so that an XCD keeps serving the same KV head (its L2 holds that head's
// K/V), item by item otherwise.
__device__ __forceinline__ int deal(int row, int xcd, int period) {
  if (row & 1) {
    const int s = (period < kXcds && kXcds % period == 0) ? period : (period % kXcds == 0 ? kXcds : 1);
    xcd = (kXcds / s - 1 - xcd / s) * s + xcd % s;
  }
  return row * kXcds + xcd;
}

// ---- workgroup -> (query tile, head, batch, key range); the heads of one KV group share an XCD
template <int D, int W>
__global__ __launch_bounds__(64 * W, 2) void host_attention_kernel(const AttnParams p, const int n_qtiles,
                                                                   const int n_items) {
  const int xcd = blockIdx.x % kXcds;
  const int slot = blockIdx.x / kXcds;
  const int item_split = deal(slot / p.group, xcd, p.batch * p.hkv * p.n_splits);
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
  const int unit = deal(slot / group, xcd, hkv);
  if (unit >= gp.sched.n_entries * hkv) return;
  const int g = slot % group;
  const int entry = unit / hkv, kvh = unit % hkv;
  int m, qt;
  decode_group_entry(gp.sched, entry, m, qt);
  if (m >= gp.n_items || qt < 0 || (int64_t)qt * kBM >= gp.item[m].L) return;      // never taken for a schedule the launcher built
  // (a copy, so that the fields live in scalar registers like the single-problem kernel's by-value argument
  // instead of being fetched from the argument block where they are used)
  const AttnParams item = gp.item[m];
  attention_workgroup<D, kWaves>(item, qt, 0, kvh, g, 0);
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
