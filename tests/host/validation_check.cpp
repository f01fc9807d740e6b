// Host check of the C ABI's argument validation and planning (csrc/host_validation.h), compiled with the plain C++
// compiler under -fsanitize=address,undefined: every rejection case returns its status without touching the forged
// pointers, and the planners stay in range over a sweep of shapes.
#include <initializer_list>
#include <cstdio>
#include <cstdlib>
#include <limits>
#include "attention_schedule.h"
#include "host_validation.h"

using namespace apbv;

static int failures = 0;
#define EXPECT(cond)                                                              \
  do {                                                                            \
    if (!(cond)) {                                                                \
      std::printf("FAILED line %d: %s\n", __LINE__, #cond);                       \
      ++failures;                                                                 \
    }                                                                             \
  } while (0)

static apbv_tensor view(int64_t tokens, int heads, int d, uintptr_t ptr = 0x1000) {
  apbv_tensor t;
  t.ptr = tokens ? reinterpret_cast<const void*>(ptr) : nullptr;      // never dereferenced
  t.tokens = tokens;
  t.stride_token = (int64_t)heads * d;
  t.stride_head = d;
  t.stride_batch = tokens * heads * d;
  return t;
}
static const void* P(uintptr_t x) { return reinterpret_cast<const void*>(x); }

static apbv_status attn(int batch = 1, int hq = 4, int hkv = 2, int d = 128, int64_t L = 64, int64_t l_a = 16, int64_t n_p = 8,
                        float scale = 0.1f, const void* out = P(0x2000), const apbv_tensor* q = nullptr,
                        const apbv_tensor* k = nullptr, const apbv_tensor* v = nullptr) {
  apbv_tensor qq = q ? *q : view(L, hq, d), kk = k ? *k : view(L, hkv, d), vv = v ? *v : view(L, hkv, d);
  return validate_attention(batch, hq, hkv, d, qq, view(l_a, hkv, d), view(l_a, hkv, d), view(n_p, hkv, d), view(n_p, hkv, d),
                            kk, vv, scale, out, nullptr);
}

static apbv_status comp(int reducer = 0, float scale = 0.f, int batch = 1, int hq = 4, int hkv = 2, int d = 128, int64_t n_q = 4,
                        int64_t L = 64, int64_t l_p = 8, const void* idx = P(0x3000), const void* kc = P(0x4000),
                        const void* vc = P(0x5000), const apbv_tensor* v = nullptr) {
  apbv_tensor vv = v ? *v : view(L, hkv, d);
  return validate_compress(reducer, scale, batch, hq, hkv, d, view(n_q, hq, d), view(L, hkv, d), vv, l_p,
                           static_cast<const int32_t*>(idx), kc, vc, nullptr);
}

int main() {
  // ---- attention
  EXPECT(attn() == APBV_OK);
  EXPECT(attn(0) == APBV_ERR_SHAPE && attn(1, 5) == APBV_ERR_SHAPE && attn(1, 4, 2, 96) == APBV_ERR_UNSUPPORTED);
  EXPECT(attn(1, 4, 2, 128, 0) == APBV_ERR_SHAPE);
  EXPECT(attn(1, 4, 2, 128, 64, 16, 8, 0.f) == APBV_ERR_SHAPE && attn(1, 4, 2, 128, 64, 16, 8, -1.f) == APBV_ERR_SHAPE);
  EXPECT(attn(1, 4, 2, 128, 64, 16, 8, std::numeric_limits<float>::infinity()) == APBV_ERR_SHAPE);
  EXPECT(attn(1, 4, 2, 128, 64, 16, 8, std::numeric_limits<float>::quiet_NaN()) == APBV_ERR_SHAPE);
  EXPECT(attn(1, 4, 2, 128, 64, 16, 8, 0.1f, nullptr) == APBV_ERR_NULL && attn(1, 4, 2, 128, 64, 16, 8, 0.1f, P(0x2004)) == APBV_ERR_SHAPE);
  {
    apbv_tensor bad = view(64, 2, 128, 0x1008);                       // misaligned pointer
    EXPECT(attn(1, 4, 2, 128, 64, 16, 8, 0.1f, P(0x2000), nullptr, &bad) == APBV_ERR_SHAPE);
    apbv_tensor nul = view(64, 2, 128);
    nul.ptr = nullptr;
    EXPECT(attn(1, 4, 2, 128, 64, 16, 8, 0.1f, P(0x2000), nullptr, &nul) == APBV_ERR_NULL);
    apbv_tensor overlap = view(64, 2, 128);
    overlap.stride_token = 64;                                         // rows overlap
    EXPECT(attn(1, 4, 2, 128, 64, 16, 8, 0.1f, P(0x2000), nullptr, &overlap) == APBV_ERR_SHAPE);
    apbv_tensor odd = view(64, 2, 128);
    odd.stride_head = 132;                                             // not a multiple of 8
    EXPECT(attn(1, 4, 2, 128, 64, 16, 8, 0.1f, P(0x2000), nullptr, &odd) == APBV_ERR_SHAPE);
    apbv_tensor wide = view(64, 2, 128);
    wide.stride_token = (int64_t)1 << 24;
    EXPECT(attn(1, 4, 2, 128, 64, 16, 8, 0.1f, P(0x2000), nullptr, &wide) == APBV_ERR_UNSUPPORTED);
    apbv_tensor shortv = view(63, 2, 128);
    EXPECT(attn(1, 4, 2, 128, 64, 16, 8, 0.1f, P(0x2000), nullptr, nullptr, &shortv) == APBV_ERR_SHAPE);
    apbv_tensor none = view(0, 2, 128);
    EXPECT(attn(1, 4, 2, 128, 64, 0, 0, 0.1f, P(0x2000), nullptr, &none, &none) == APBV_ERR_SHAPE);      // no key at all
    EXPECT(attn(1, 4, 2, 128, 64, 16, 0, 0.1f, P(0x2000), nullptr, &none, &none) == APBV_OK);            // no causal segment
    apbv_tensor huge = view(((int64_t)1 << 24) + 1, 4, 128);
    EXPECT(attn(1, 4, 2, 128, 64, 16, 8, 0.1f, P(0x2000), &huge) == APBV_ERR_SHAPE);
    apbv_tensor batched = view(64, 4, 128);
    batched.stride_batch = 0;
    EXPECT(attn(2, 4, 2, 128, 64, 16, 8, 0.1f, P(0x2000), &batched) == APBV_ERR_SHAPE);
  }
  // ---- compression
  EXPECT(comp() == APBV_OK);
  EXPECT(comp(0, 0.f, 1, 4, 2, 128, 4, 64, 65) == APBV_ERR_SHAPE && comp(0, 0.f, 1, 4, 2, 128, 4, 64, -1) == APBV_ERR_SHAPE);
  EXPECT(comp(0, 0.f, 1, 5) == APBV_ERR_SHAPE && comp(0, 0.f, 1, 4, 2, 32) == APBV_ERR_UNSUPPORTED);
  EXPECT(comp(0, 0.f, 1, 4, 2, 128, 4, 64, 8, nullptr) == APBV_ERR_NULL);
  EXPECT(comp(0, 0.f, 1, 4, 2, 128, 4, 64, 0, nullptr, nullptr, nullptr) == APBV_OK);                   // l_p = 0 writes nothing
  EXPECT(comp(0, 0.f, 1, 4, 2, 128, 4, 64, 8, P(0x3000), P(0x4002)) == APBV_ERR_SHAPE);
  EXPECT(comp(0, 0.f, 1, 4, 2, 128, 0) == APBV_ERR_SHAPE);
  EXPECT(comp(3) == APBV_ERR_SHAPE && comp(-1) == APBV_ERR_SHAPE);
  EXPECT(comp(2, 0.f) == APBV_ERR_SHAPE && comp(2, 0.1f) == APBV_OK && comp(1, 0.f) == APBV_OK);
  {
    apbv_tensor shortv = view(63, 2, 128);
    EXPECT(comp(0, 0.f, 1, 4, 2, 128, 4, 64, 8, P(0x3000), P(0x4000), P(0x5000), &shortv) == APBV_ERR_SHAPE);
  }
  // ---- merge
  EXPECT(validate_merge(3, 10, 4, 128, P(0x1000), 10 * 4 * 128, static_cast<const float*>(P(0x2000)), 40, P(0x3000), nullptr) == APBV_OK);
  EXPECT(validate_merge(0, 10, 4, 128, P(0x1000), 5120, static_cast<const float*>(P(0x2000)), 40, P(0x3000), nullptr) == APBV_ERR_SHAPE);
  EXPECT(validate_merge(3, 10, 4, 128, P(0x1000), 5112, static_cast<const float*>(P(0x2000)), 40, P(0x3000), nullptr) == APBV_ERR_SHAPE);
  EXPECT(validate_merge(3, 10, 4, 128, P(0x1000), 5120, static_cast<const float*>(P(0x2000)), 39, P(0x3000), nullptr) == APBV_ERR_SHAPE);
  EXPECT(validate_merge(3, 10, 4, 96, P(0x1000), 5120, static_cast<const float*>(P(0x2000)), 40, P(0x3000), nullptr) == APBV_ERR_UNSUPPORTED);
  EXPECT(validate_merge(3, 10, 4, 128, nullptr, 5120, static_cast<const float*>(P(0x2000)), 40, P(0x3000), nullptr) == APBV_ERR_NULL);
  // ---- planners over a sweep: the key split covers every tile exactly once with no empty range; workspaces are
  // aligned, ordered and monotone in the batch
  for (int64_t n_keys = 1; n_keys < 300000; n_keys = n_keys * 3 + 7)
    for (int64_t n_q = 1; n_q <= 4096; n_q *= 4)
      for (int req = 0; req <= 300; req = req * 2 + 1) {
        const KeySplit ks = plan_key_split(1, 16, n_q, n_keys, req);
        const int64_t n_tiles = (n_keys + kAttnKeyTile - 1) / kAttnKeyTile;
        EXPECT(ks.n_splits >= 1 && ks.n_splits <= kMaxKeySplits && ks.tiles_per_split >= 1);
        EXPECT((int64_t)ks.n_splits * ks.tiles_per_split >= n_tiles);
        EXPECT((int64_t)(ks.n_splits - 1) * ks.tiles_per_split < n_tiles);
        const size_t ws = query_attention_workspace_bytes(1, 16, 128, n_q, n_keys, req);
        EXPECT(ws % 256 == 0 && (ks.n_splits == 1) == (ws == 0));
      }
  for (int64_t L = 1; L <= ((int64_t)1 << 24); L = L * 5 + 3)
    for (int64_t l_p = 0; l_p <= L; l_p = l_p * 7 + 1) {
      const CompressWorkspace w1 = plan_compress_workspace(1, 2, 128, L, l_p), w3 = plan_compress_workspace(3, 2, 128, L, l_p);
      EXPECT(w1.total % 256 == 0 && w1.scores_off % 256 == 0 && w1.qbar_off < w1.scores_off && w1.scores_off < w1.total);
      EXPECT(w1.scores_off + (size_t)2 * L * 8 <= w1.sort_keys_off && w1.sort_keys_off <= w1.sort_idx_off && w1.sort_idx_off <= w1.total);
      EXPECT(w1.n_sort >= l_p && (w1.n_sort & (w1.n_sort - 1)) == 0 && w3.total >= w1.total);
      EXPECT(compress_workspace_bytes_checked(1, 2, 128, L, l_p) == w1.total);
    }
  // pooled-query partition: about 64 probe rows per range, at most kPoolSplitMax, no more ranges than fill the chip
  // twice over; and the partial sums of every partition fit the region the workspace plan reserves for them
  EXPECT(pool_splits(512, 2) == 8 && pool_splits(512, 192) == 2 && pool_splits(512, 1000) == 1 && pool_splits(10, 1) == 1);
  EXPECT(pool_splits(100000, 1) == kPoolSplitMax && pool_splits(1, 1) == 1 && pool_splits(130, 4) == 3);
  for (int batch : {1, 2, 7, 96, 300})
    for (int hkv : {1, 2, 4, 8})
      for (int64_t rows : {1, 63, 64, 65, 512, 4096}) {
        const int n = pool_splits(rows, (int64_t)batch * hkv);
        EXPECT(n >= 1 && n <= kPoolSplitMax);
        const CompressWorkspace w = plan_compress_workspace(batch, hkv, 128, 1024, 16);
        EXPECT(w.qbar_off + (size_t)batch * hkv * n * 128 * sizeof(double) <= w.scores_off);
      }
  EXPECT(compress_workspace_bytes_checked(1, 2, 128, 0, 0) == 0 && compress_workspace_bytes_checked(1, 2, 128, 8, 9) == 0);
  EXPECT(compress_workspace_bytes_checked(0, 2, 128, 8, 1) == 0 && compress_workspace_bytes_checked(1, 2, 100, 8, 1) == 0);
  if (failures) return 1;
  std::printf("host validation OK\n");
  return 0;
}
