// Host check of the merged query-tile schedule (csrc/attention_schedule.h), compiled with the plain C++ compiler:
// for random groups, every (problem, query tile) pair must be decoded exactly once, levels never increase along
// the order, and problems inside a level come in index order.
#include <cstdio>
#include <cstdlib>
#include <map>
#include <utility>
#include "attention_schedule.h"

using namespace apbv;

static uint64_t state = 0x9E3779B97F4A7C15ull;
static uint64_t rnd() {                       // splitmix64
  uint64_t z = (state += 0x9E3779B97F4A7C15ull);
  z = (z ^ (z >> 30)) * 0xBF58476D1CE4E5B9ull;
  z = (z ^ (z >> 27)) * 0x94D049BB133111EBull;
  return z ^ (z >> 31);
}

static int check(int n, const int64_t* n_vis, const int64_t* rows) {
  GroupSchedule s;
  if (!build_group_schedule(n, n_vis, rows, s)) { std::printf("build failed\n"); return 1; }
  std::map<std::pair<int, int>, int> seen;
  long expected = 0;
  for (int m = 0; m < n; ++m) expected += (rows[m] + 255) / 256;
  if (s.n_entries != expected) { std::printf("n_entries %d != %ld\n", s.n_entries, expected); return 1; }
  long prev_level = -1;
  int prev_m = -1;
  for (int e = 0; e < s.n_entries; ++e) {
    int m, qt;
    decode_group_entry(s, e, m, qt);
    if (m < 0 || m >= n || qt < 0 || qt >= (rows[m] + 255) / 256) { std::printf("entry %d -> (%d, %d) out of range\n", e, m, qt); return 1; }
    if (seen[{m, qt}]++) { std::printf("entry %d -> (%d, %d) twice\n", e, m, qt); return 1; }
    const long level = n_vis[m] / 256 + qt;
    if (e > 0 && (level > prev_level || (level == prev_level && m <= prev_m))) { std::printf("order broken at entry %d\n", e); return 1; }
    prev_level = level;
    prev_m = m;
  }
  return 0;
}

int main() {
  {  // a physical host of the 128K configuration: anchor block, virtual hosts 0 and 15
    const int64_t n_vis[3] = {0, 2048, 2048 + 15 * 1024}, rows[3] = {2048, 16384, 16384};
    if (check(3, n_vis, rows)) return 1;
  }
  for (int it = 0; it < 20000; ++it) {
    const int n = 1 + (int)(rnd() % kMaxGroupItems);
    int64_t n_vis[kMaxGroupItems], rows[kMaxGroupItems];
    for (int m = 0; m < n; ++m) {
      n_vis[m] = (int64_t)(rnd() % (it % 2 ? 5000 : 600));
      rows[m] = 1 + (int64_t)(rnd() % (it % 3 ? 3000 : 300));
    }
    if (check(n, n_vis, rows)) { std::printf("case %d\n", it); return 1; }
  }
  GroupSchedule s;
  const int64_t z = 0, one = 1, neg = -1;
  if (build_group_schedule(0, &z, &one, s) || build_group_schedule(9, &z, &one, s) || build_group_schedule(1, &neg, &one, s) ||
      build_group_schedule(1, &z, &z, s)) { std::printf("bad sizes accepted\n"); return 1; }
  std::printf("schedule ok\n");
  return 0;
}
