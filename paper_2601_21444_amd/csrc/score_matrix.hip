// Alternative reductions of the score matrix S_h = Q_qr K^(h)T of Alg. 1 ("Identify Essential KVs") to one
// score per key and KV head, for gfx950.  The adopted reading (sum of the raw logits) is linear and lives in
// compress.hip as a streaming dot product; the reductions here are not linear, so the n_q*G x L logits are
// formed on the matrix cores (bf16 operands, fp32 accumulation) and reduced on the fly, never stored:
//
//   max           s[v, j] = max over rows (t, g) of S[(t, g), j]
//   softmax-sum   s[v, j] = sum over rows of softmax_j(scale * S[(t, g), :])[j]        (Eq. 1 without a mask)
//
// Rows (t, g) of KV head v are Q_qr[t, v*G+g, :], r = t*G + g, R = n_q*G of them.
//
// One kernel template does all the matrix work.  A workgroup of four waves keeps 256 "resident" vectors in
// registers as MFMA B operands (64 per wave) and streams the other side through LDS in tiles of 32 vectors
// (A operand, a ring of four tiles filled by LDS-direct loads, shared by the four waves).  Each 32x32 accumulator then has the streamed
// vectors along its register axis and one resident vector per lane, so every reduction over the streamed side
// is per lane, plus one exchange between the two lane halves at the end:
//
//   kMax     resident = keys,       streamed = all probe rows:  maximum logit               -> score per key
//   kStats   resident = probe rows, streamed = a chunk of keys: running maximum and sum of exponentials of the
//                                                               scaled logits               -> partial row statistics
//   kMass    resident = keys,       streamed = all probe rows:  sum of exp2(scaled logit - c_r), c_r = the row's
//                                   maximum + log2 of its normaliser (from kStats, merged by
//                                   row_stats_combine_kernel)                                -> score per key
#include "apbv_common.h"

namespace apbv {
namespace {

constexpr int kChunkKeys = 256;        // smallest number of keys per partial row statistic (sizes the workspace)
constexpr int kMaxChunkKeys = 4096;    // largest
constexpr int64_t kStatsMinWorkgroups = 2 * 768;   // keep at least two rounds of workgroups in the statistics launch
constexpr int kMaxStatRows = 8192;     // rows whose statistics fit the LDS of the kMass pass (4 bytes each)
constexpr int kResident = 256;         // resident vectors per workgroup (64 per wave)

enum Mode { kMax = 1, kMass = 2, kStats = 3 };

__device__ __forceinline__ f32x16 mfma(const bf16x8 a, const bf16x8 b, const f32x16 c) {
  return __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, b, c, 0, 0, 0);
}

// LDS-direct 16-byte load: lane l's bytes land at lds_dst + 16*l (lds_dst wave-uniform, in M0, which addresses the
// first 64 KB of the workgroup's LDS).  Issued through inline assembly: the kernel orders these loads against the LDS
// reads itself (s_waitcnt vmcnt(0) + barrier), the compiler's wait-count insertion does not know about them.
__device__ __forceinline__ void dma16_lane(const void* addr, uint32_t lds_dst) {
  asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %1, off" ::"s"(lds_dst), "v"(addr) : "memory", "m0");
}
__device__ __forceinline__ uint32_t lds_addr(const unsigned char* p) {
  return (uint32_t)(size_t)(__attribute__((address_space(3))) const unsigned char*)p;
}

// accumulator register i of lane half hh holds matrix row 8*(i/4) + 4*hh + i%4 (column = lane % 32)
__device__ __forceinline__ int acc_row(int i, int hh) { return 8 * (i / 4) + 4 * hh + i % 4; }

// value of the lane 32 away
__device__ __forceinline__ float other_half(float x) {
  auto sw = __builtin_amdgcn_permlane32_swap(__float_as_uint(x), __float_as_uint(x), false, false);
  // the swap exchanges the upper half of the first operand with the lower half of the second: each lane finds
  // its own value in one result and its partner's in the other
  const float a = __uint_as_float(sw[0]), b = __uint_as_float(sw[1]);
  return (threadIdx.x & 32) ? a : b;
}

struct RowsParams {
  View q, k;
  int64_t L;
  int n_rows;          // R = n_q * G
  int r_pad;           // R rounded up to a multiple of 32
  int group, hkv, n_chunks;
  int chunk_keys;      // keys per partial row statistic: a multiple of kChunkKeys
  float scale_log2;    // softmax_scale * log2(e)
  float2* partial;     // [batch, Hkv, n_chunks, r_pad]  (maximum of the scaled logits in the log2 domain, sum of exp2)
  float* stats;        // [batch, Hkv, r_pad]            c_r = maximum + log2(normaliser); +inf for padding rows
  double* s_ws;        // [batch, Hkv, L]
  double* s_out;       // optional, same layout
};

// First element of probe row r (clamped to the last row) / of key j (clamped to the last key) of head v.
__device__ __forceinline__ const bf16_t* probe_row(const RowsParams& p, int b, int v, int r) {
  const int rc = r < p.n_rows ? r : p.n_rows - 1;
  const int t = rc / p.group, g = rc % p.group;
  return p.q.ptr + (int64_t)b * p.q.sb + (int64_t)t * p.q.st + (int64_t)(v * p.group + g) * p.q.sh;
}
__device__ __forceinline__ const bf16_t* key_row(const RowsParams& p, int b, int v, int64_t j) {
  const int64_t jc = j < p.L ? j : p.L - 1;
  return p.k.ptr + (int64_t)b * p.k.sb + (int64_t)v * p.k.sh + jc * p.k.st;
}

// A cursor keeps one row's address and advances it without divisions
// (the streamed loads would otherwise cost more vector instructions than the reduction itself).  Rows past
// the end read the last row.
struct ProbeCursor {
  const bf16_t *ptr, *last;
  int r, g, dr;
  int64_t step, wrap;      // elements per step of dr rows without / extra on a carry of g
  int dg;
  __device__ __forceinline__ void init(const RowsParams& p, int b, int v, int r0, int chunk_elems, int rows_per_step) {
    r = r0;
    dr = rows_per_step;
    last = probe_row(p, b, v, p.n_rows - 1) + chunk_elems;
    ptr = probe_row(p, b, v, r0) + chunk_elems;
    g = (r0 < p.n_rows ? r0 : p.n_rows - 1) % p.group;
    dg = rows_per_step % p.group;
    step = (int64_t)(rows_per_step / p.group) * p.q.st + (int64_t)dg * p.q.sh;
    wrap = p.q.st - (int64_t)p.group * p.q.sh;
  }
  __device__ __forceinline__ const bf16_t* get(const RowsParams& p) const { return r < p.n_rows ? ptr : last; }
  __device__ __forceinline__ void advance(const RowsParams& p) {
    r += dr;
    g += dg;
    ptr += step;
    if (g >= p.group) {
      g -= p.group;
      ptr += wrap;
    }
  }
};
struct KeyCursor {
  const bf16_t *ptr, *last;
  int64_t j, step;
  int dj;
  __device__ __forceinline__ void init(const RowsParams& p, int b, int v, int64_t j0, int chunk_elems, int rows_per_step) {
    j = j0;
    dj = rows_per_step;
    last = key_row(p, b, v, p.L - 1) + chunk_elems;
    ptr = key_row(p, b, v, j0) + chunk_elems;
    step = (int64_t)rows_per_step * p.k.st;
  }
  __device__ __forceinline__ const bf16_t* get(const RowsParams& p) const { return j < p.L ? ptr : last; }
  __device__ __forceinline__ void advance(const RowsParams&) {
    j += dj;
    ptr += step;
  }
};
template <bool KEYS>
struct CursorOf { using type = ProbeCursor; };
template <>
struct CursorOf<true> { using type = KeyCursor; };

// Grid: kMax / kMass (ceil(L / 256), Hkv, batch); kStats (ceil(r_pad / 256) * n_chunks, Hkv, batch).
template <int D, int MODE>
__global__ __launch_bounds__(256, 3) void matrix_reduce_kernel(const RowsParams p) {
  constexpr int KS = D / 16;                 // MFMA steps along the head dimension
  constexpr int KC = D / 8;                  // 16-byte chunks per vector
  constexpr int ROW_BYTES = D * 2;
  constexpr int TR = 32;                     // streamed vectors per LDS tile (64: no faster, twice the LDS)
  constexpr int PASSES = TR * KC / 256;      // 16-byte loads per thread per streamed tile
  constexpr int RPW = 1024 / ROW_BYTES;      // tile rows one wave-wide LDS-direct load covers
  constexpr int kTiles = 4;                  // streamed tiles resident in LDS
  constexpr bool kKeysResident = MODE != kStats;
  __shared__ __attribute__((aligned(1024))) unsigned char tile[kTiles][TR * ROW_BYTES];
  static_assert(kTiles * TR * ROW_BYTES <= 65536 && PASSES * 4 * RPW == TR, "tile ring below 64 KB; four waves fill a tile");
  extern __shared__ float c_lds[];           // kMass: r_pad entries

  const int v = blockIdx.y, b = blockIdx.z;
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int c = lane & 31, hh = lane >> 5;
  // swizzle of the 16-byte chunks of a tile row, so that the lanes of one A-operand read spread over the banks
  auto swz = [](int row) { return D == 128 ? (row & 15) : ((row >> 1) & 7); };

  int64_t res0;            // first resident vector of the workgroup
  int64_t str0, str_end;   // streamed range
  int ch = 0;
  if (kKeysResident) {
    res0 = (int64_t)blockIdx.x * kResident;
    str0 = 0;
    str_end = p.n_rows;
  } else {
    const int n_rg = (p.r_pad + kResident - 1) / kResident;
    res0 = (int64_t)(blockIdx.x % n_rg) * kResident;
    ch = blockIdx.x / n_rg;
    str0 = (int64_t)ch * p.chunk_keys;
    str_end = str0 + p.chunk_keys < p.L ? str0 + p.chunk_keys : p.L;
  }
  auto resident_row = [&](int64_t i) { return kKeysResident ? key_row(p, b, v, i) : probe_row(p, b, v, (int)i); };

  // ---- resident B operands: lane (c, hh) holds elements 8*hh + 16*kk .. +7 of vectors res + c and res + 32 + c
  const int64_t res = res0 + wave * 64;
  bf16x8 rf[2][KS];
#pragma unroll
  for (int s = 0; s < 2; ++s) {
    const bf16_t* row = resident_row(res + 32 * s + c) + 8 * hh;
#pragma unroll
    for (int kk = 0; kk < KS; ++kk) rf[s][kk] = *reinterpret_cast<const bf16x8*>(row + 16 * kk);
  }
  if (MODE == kMass) {
    const float* st = p.stats + ((int64_t)b * p.hkv + v) * p.r_pad;
    for (int i = tid; i < p.r_pad; i += 256) c_lds[i] = st[i];
  }

  // ---- streamed tiles, global -> LDS without a stop in registers.  Wave-wide load (u, wave) fills the RPW tile rows
  // from (4*u + wave) * RPW; lane l brings the 16-byte chunk that belongs at position l % KC of row l / KC of those,
  // i.e. chunk (l % KC) ^ swz(row) of the vector (the swizzle is applied on the global side).
  typename CursorOf<!kKeysResident>::type cur[PASSES];
#pragma unroll
  for (int u = 0; u < PASSES; ++u) {
    const int row = (4 * u + wave) * RPW + lane / KC;
    cur[u].init(p, b, v, str0 + row, 8 * ((lane % KC) ^ swz(row)), TR);
  }
  const uint32_t tile_lds = lds_addr(tile[0]) + (uint32_t)(__builtin_amdgcn_readfirstlane(wave) * RPW * ROW_BYTES);
  auto issue = [&](int slot) {                       // requests the cursors' tile into a ring slot, moves them on
#pragma unroll
    for (int u = 0; u < PASSES; ++u) {
      dma16_lane(cur[u].get(p), tile_lds + (uint32_t)(slot * TR * ROW_BYTES + 4 * u * RPW * ROW_BYTES));
      cur[u].advance(p);
    }
  };
  auto arrive = [&]() {
    asm volatile("s_waitcnt vmcnt(0)" ::: "memory");  // this wave's share of the requested tiles has landed
    __syncthreads();                                  // ... everyone's has, and everyone is done with the slots reloaded next
  };

  float red[2], z_run[2];
#pragma unroll
  for (int s = 0; s < 2; ++s) {
    red[s] = MODE == kMass ? 0.f : -INFINITY;      // kMax: maximum; kStats: running maximum (scaled); kMass: sum
    z_run[s] = 0.f;
  }

  // per 32 streamed vectors: 16 MFMAs per wave and the mode's reduction of the two accumulators
  auto compute = [&](const int64_t tile0, const int buf) {
#pragma unroll
    for (int sub = 0; sub < TR / 32; ++sub) {
    const int64_t t0 = tile0 + 32 * sub;
    if (t0 >= str_end) break;
    f32x16 acc[2];
#pragma unroll
    for (int s = 0; s < 2; ++s)
#pragma unroll
      for (int i = 0; i < 16; ++i) acc[s][i] = 0.f;
    // A fragments are read RA steps at a time ahead of the MFMAs that use them, which then run back to back (order
    // pinned: left alone, the scheduler sinks every LDS read next to its use and the wave waits out each read's
    // latency in turn).  The exp-bearing modes have fewer registers to spare.
    constexpr int RA = 4;
#pragma unroll
    for (int k0 = 0; k0 < KS; k0 += RA) {
      bf16x8 af[RA];
#pragma unroll
      for (int kk = 0; kk < RA; ++kk)
        af[kk] = *reinterpret_cast<const bf16x8*>(&tile[buf][(32 * sub + c) * ROW_BYTES + 16 * ((2 * (k0 + kk) + hh) ^ swz(c))]);
#pragma unroll
      for (int kk = 0; kk < RA; ++kk) {
        acc[0] = mfma(af[kk], rf[0][k0 + kk], acc[0]);
        acc[1] = mfma(af[kk], rf[1][k0 + kk], acc[1]);
      }
      if (MODE != kStats) {      // (the statistics pass has no registers to spare for a pinned read-ahead)
        __builtin_amdgcn_sched_group_barrier(0x100, RA, 0);        // RA LDS reads
        __builtin_amdgcn_sched_group_barrier(0x008, 2 * RA, 0);    // 2*RA MFMAs
      }
    }
    // the accumulator's register axis runs over the streamed vectors t0 + acc_row(i, hh)
    if (MODE == kMax) {
      // streamed rows past the end repeat the last row: harmless under a maximum
#pragma unroll
      for (int s = 0; s < 2; ++s)
#pragma unroll
        for (int i = 0; i < 16; ++i) red[s] = fmaxf(red[s], acc[s][i]);
    } else if (MODE == kMass) {
      // padding rows carry c_r = +inf: exp2(-inf) = 0
#pragma unroll
      for (int i4 = 0; i4 < 4; ++i4) {
        const f32x4 cr = *reinterpret_cast<const f32x4*>(&c_lds[(t0 - str0) + 8 * i4 + 4 * hh]);
#pragma unroll
        for (int s = 0; s < 2; ++s)
#pragma unroll
          for (int e = 0; e < 4; ++e)
            red[s] += __builtin_amdgcn_exp2f(__builtin_fmaf(acc[s][4 * i4 + e], p.scale_log2, -cr[e]));
      }
    } else {
      const bool ragged = t0 + 32 > str_end;       // keys past the end of the block must not count
#pragma unroll
      for (int s = 0; s < 2; ++s) {
        if (ragged) {
#pragma unroll
          for (int i = 0; i < 16; ++i)
            if (t0 + acc_row(i, hh) >= str_end) acc[s][i] = -INFINITY;
        }
        float bm = acc[s][0];
#pragma unroll
        for (int i = 1; i < 16; ++i) bm = fmaxf(bm, acc[s][i]);
        const float m_new = fmaxf(red[s], bm * p.scale_log2);
        const float m_sub = m_new > -INFINITY ? m_new : 0.f;      // a lane half may hold only keys past the end
        float z = z_run[s] * __builtin_amdgcn_exp2f(red[s] - m_sub);
#pragma unroll
        for (int i = 0; i < 16; ++i) z += __builtin_amdgcn_exp2f(__builtin_fmaf(acc[s][i], p.scale_log2, -m_sub));
        z_run[s] = z;
        red[s] = m_new;
      }
    }
    }
  };

  // Tile t lives in ring slot t % 4.  One barrier per two tiles: after the barrier in front of tiles t, t+1 both have
  // landed and everyone is done with tiles t-2, t-1, whose slots take the loads of tiles t+2, t+3.
  // Everything loaded so far with ordinary loads (the resident operands) has arrived: vmcnt 0, said with the builtin
  // so that the compiler's own wait-count bookkeeping knows it; from here on only tile loads are outstanding.
  __builtin_amdgcn_s_waitcnt(0x0F70);
  issue(0);
  if (str0 + TR < str_end) issue(1);
  arrive();
  int slot = 0;
  for (int64_t tile0 = str0; tile0 < str_end; tile0 += 2 * TR, slot ^= 2) {
    if (tile0 + 2 * TR < str_end) issue(slot ^ 2);
    if (tile0 + 3 * TR < str_end) issue((slot ^ 2) + 1);
    compute(tile0, slot);
    if (tile0 + TR < str_end) compute(tile0 + TR, slot + 1);
    arrive();
  }

  // ---- the two lane halves hold disjoint streamed vectors for the same resident vector
#pragma unroll
  for (int s = 0; s < 2; ++s) {
    const int64_t i = res + 32 * s + c;
    const float o = other_half(red[s]);
    if (MODE == kStats) {
      const float z_o = other_half(z_run[s]);
      const float m_all = fmaxf(red[s], o);
      const float m_sub = m_all > -INFINITY ? m_all : 0.f;
      const float z_all = z_run[s] * __builtin_amdgcn_exp2f(red[s] - m_sub) + z_o * __builtin_amdgcn_exp2f(o - m_sub);
      if (hh == 0 && i < p.r_pad) {
        float2 w;
        w.x = m_all;
        w.y = z_all;
        p.partial[(((int64_t)b * p.hkv + v) * p.n_chunks + ch) * p.r_pad + i] = w;
      }
    } else {
      const float r = MODE == kMax ? fmaxf(red[s], o) : red[s] + o;      // both halves get the same bits
      if (hh == 0 && i < p.L) {
        const int64_t at = ((int64_t)b * p.hkv + v) * p.L + i;
        p.s_ws[at] = (double)r;
        if (p.s_out) p.s_out[at] = (double)r;
      }
    }
  }
}

// One wave per (batch, head, row): merge the chunks' statistics into c_r = maximum + log2(normaliser); padding rows
// get +inf.  Every real row has at least one key, so its normaliser is positive.
__global__ __launch_bounds__(256) void row_stats_combine_kernel(const RowsParams p, int batch) {
  const int64_t w = (int64_t)blockIdx.x * 4 + (threadIdx.x >> 6);
  const int lane = threadIdx.x & 63;
  if (w >= (int64_t)batch * p.hkv * p.r_pad) return;
  const int r = (int)(w % p.r_pad);
  const int64_t bv = w / p.r_pad;
  float cr = INFINITY;
  if (r < p.n_rows) {
    const float2* part = p.partial + bv * p.n_chunks * p.r_pad + r;
    float m = -INFINITY;
    for (int ch = lane; ch < p.n_chunks; ch += 64) m = fmaxf(m, part[(int64_t)ch * p.r_pad].x);
#pragma unroll
    for (int d = 1; d < 64; d <<= 1) m = fmaxf(m, __shfl_xor(m, d));
    float z = 0.f;
    for (int ch = lane; ch < p.n_chunks; ch += 64) {
      const float2 s = part[(int64_t)ch * p.r_pad];
      z += s.y * __builtin_amdgcn_exp2f(s.x - m);
    }
#pragma unroll
    for (int d = 1; d < 64; d <<= 1) z += __shfl_xor(z, d);
    cr = m + __builtin_amdgcn_logf(z);      // v_log_f32 is a base-2 logarithm
  }
  if (lane == 0) p.stats[w] = cr;
}


}  // namespace

size_t matrix_scores_workspace_bytes(int reducer, int batch, int hkv, int64_t n_rows, int64_t L) {
  if (reducer != APBV_REDUCE_SOFTMAX_SUM) return 0;
  const size_t r_pad = (size_t)((n_rows + 31) / 32 * 32);
  const size_t n_chunks = (size_t)((L + kChunkKeys - 1) / kChunkKeys);
  return align256((size_t)batch * hkv * n_chunks * r_pad * sizeof(float2)) + align256((size_t)batch * hkv * r_pad * sizeof(float));
}

// Shapes the matrix reductions do not implement, reported before anything is launched.
apbv_status check_matrix_scores(const CompressParams& cp) {
  const int64_t n_rows = cp.q_probe.tokens * cp.group;
  if (n_rows > (1 << 24)) return APBV_ERR_UNSUPPORTED;
  if (cp.reducer == APBV_REDUCE_SOFTMAX_SUM) {
    if ((n_rows + 31) / 32 * 32 > kMaxStatRows) return APBV_ERR_UNSUPPORTED;
    const int64_t n_chunks = (cp.L + kChunkKeys - 1) / kChunkKeys;
    if (((n_rows + 31) / 32 * 32 + kResident - 1) / kResident * n_chunks > 0x7fffffff) return APBV_ERR_UNSUPPORTED;
  } else if (cp.reducer != APBV_REDUCE_MAX) {
    return APBV_ERR_UNSUPPORTED;
  }
  return APBV_OK;
}

apbv_status launch_matrix_scores(const CompressParams& cp, double* scores, void* stats_ws, hipStream_t stream) {
  const apbv_status ok = check_matrix_scores(cp);
  if (ok != APBV_OK) return ok;
  const int64_t n_rows = cp.q_probe.tokens * cp.group;
  RowsParams p;
  p.q = cp.q_probe;
  p.k = cp.k;
  p.L = cp.L;
  p.n_rows = (int)n_rows;
  p.r_pad = (int)((n_rows + 31) / 32 * 32);
  p.group = cp.group;
  p.hkv = cp.hkv;
  // Keys per workgroup of the statistics pass.  A workgroup loads 256 resident probe rows (64 KB) before it streams
  // its keys, so a chunk of 256 keys spends as long on the prologue as on the matrix work; chunks grow while the
  // launch still has two workgroups for every slot of the chip (three workgroups per compute unit).  (Batch 16 at
  // 512 x 16384 logits per head: 512-key chunks, 102 -> 93 us, and the combine kernel 10 -> 6 us.)
  int chunk = kChunkKeys;
  {
    const int64_t n_rg = ((n_rows + 31) / 32 * 32 + kResident - 1) / kResident;
    auto n_wg_at = [&](int c) { return n_rg * ((cp.L + c - 1) / c) * cp.hkv * cp.batch; };
    while (chunk < kMaxChunkKeys && n_wg_at(2 * chunk) >= kStatsMinWorkgroups) chunk *= 2;
  }
  p.chunk_keys = chunk;
  p.n_chunks = (int)((cp.L + chunk - 1) / chunk);
  p.scale_log2 = cp.scale_log2;
  p.partial = nullptr;
  p.stats = nullptr;
  p.s_ws = scores;
  p.s_out = cp.scores_out;
  const dim3 grid((unsigned)((cp.L + kResident - 1) / kResident), cp.hkv, cp.batch);
  Launcher launch(stream);
  if (cp.reducer == APBV_REDUCE_MAX) {
    if (cp.d == 128)
      launch(matrix_reduce_kernel<128, kMax>, grid, dim3(256), 0, p);
    else
      launch(matrix_reduce_kernel<64, kMax>, grid, dim3(256), 0, p);
  } else if (cp.reducer == APBV_REDUCE_SOFTMAX_SUM) {
    if (p.r_pad > kMaxStatRows) return APBV_ERR_UNSUPPORTED;
    p.partial = static_cast<float2*>(stats_ws);
    p.stats = reinterpret_cast<float*>(static_cast<char*>(stats_ws) +
                                       align256((size_t)cp.batch * cp.hkv * p.n_chunks * p.r_pad * sizeof(float2)));
    const int64_t n_wg = (int64_t)((p.r_pad + kResident - 1) / kResident) * p.n_chunks;
    if (n_wg > 0x7fffffff) return APBV_ERR_UNSUPPORTED;
    const dim3 sgrid((unsigned)n_wg, cp.hkv, cp.batch);
    if (cp.d == 128)
      launch(matrix_reduce_kernel<128, kStats>, sgrid, dim3(256), 0, p);
    else
      launch(matrix_reduce_kernel<64, kStats>, sgrid, dim3(256), 0, p);
    const int64_t n_stat = (int64_t)cp.batch * cp.hkv * p.r_pad;
    launch(row_stats_combine_kernel, dim3((unsigned)((n_stat + 3) / 4)), dim3(256), 0, p, cp.batch);
    const size_t lds = (size_t)p.r_pad * sizeof(float);
    if (cp.d == 128)
      launch(matrix_reduce_kernel<128, kMass>, grid, dim3(256), lds, p);
    else
      launch(matrix_reduce_kernel<64, kMass>, grid, dim3(256), lds, p);
  } else {
    return APBV_ERR_UNSUPPORTED;
  }
  return launch.status();
}

}  // namespace apbv
