// Merged heaviest-first order of the query tiles of several attention problems (host side builds it, the
// kernel decodes one entry per workgroup).  Plain C++: no HIP types, so host tests can compile it alone.
//
// Query tile qt (256 rows) of a problem with n_vis fully visible keys visits about (n_vis + 256 (qt+1)) / 64 key
// tiles; its level is n_vis / 256 + qt, so one level is one query tile's worth of keys for every problem.
// Levels are walked from the highest down; inside a level the problems come in index order.  The level axis
// is cut where a problem starts or ends, so inside a segment the set of active problems is fixed and an
// entry index decodes with one division.
#pragma once
#include <stdint.h>

#if defined(__HIPCC__)
#define APBV_HOST_DEVICE __host__ __device__
#else
#define APBV_HOST_DEVICE
#endif

namespace apbv {

constexpr int kMaxGroupItems = 8;
constexpr int kGroupQueryTile = 256;     // query rows per workgroup of the attention kernel

struct GroupSchedule {
  struct Segment {
    int first;        // index of the segment's first (problem, query tile) entry
    int level_hi;     // its highest level; entries walk the levels downwards
    int n_active;     // problems with a query tile on each of the segment's levels
    uint32_t items;   // their indices, 4 bits each, in index order
  } seg[2 * kMaxGroupItems];
  int level0[kMaxGroupItems];   // level of query tile 0 of every problem
  int n_segs, n_entries;
};

// rows[m] >= 1 query rows and n_vis[m] >= 0 fully visible keys of problem m.  False if the sizes do not fit.
inline bool build_group_schedule(int n, const int64_t* n_vis, const int64_t* rows, GroupSchedule& s) {
  if (n < 1 || n > kMaxGroupItems) return false;
  int64_t lo[kMaxGroupItems], hi[kMaxGroupItems];      // level range [lo, hi) of every problem
  int64_t cuts[2 * kMaxGroupItems];
  int n_cuts = 0;
  for (int m = 0; m < n; ++m) {
    if (rows[m] < 1 || n_vis[m] < 0) return false;
    lo[m] = n_vis[m] / kGroupQueryTile;
    hi[m] = lo[m] + (rows[m] + kGroupQueryTile - 1) / kGroupQueryTile;
    if (hi[m] > 0x3fffffff) return false;
    s.level0[m] = (int)lo[m];
    cuts[n_cuts++] = lo[m];
    cuts[n_cuts++] = hi[m];
  }
  for (int a = 1; a < n_cuts; ++a)                     // insertion sort, descending
    for (int c = a; c > 0 && cuts[c] > cuts[c - 1]; --c) {
      const int64_t t = cuts[c];
      cuts[c] = cuts[c - 1];
      cuts[c - 1] = t;
    }
  int n_segs = 0;
  int64_t first = 0;
  for (int a = 0; a + 1 < n_cuts; ++a) {
    const int64_t top = cuts[a], bottom = cuts[a + 1];  // levels [bottom, top)
    if (top == bottom) continue;
    uint32_t items = 0;
    int n_active = 0;
    for (int m = 0; m < n; ++m)
      if (lo[m] <= bottom && top <= hi[m]) items |= (uint32_t)m << (4 * n_active++);
    if (n_active == 0) continue;
    GroupSchedule::Segment& sg = s.seg[n_segs++];
    sg.first = (int)first;
    sg.level_hi = (int)(top - 1);
    sg.n_active = n_active;
    sg.items = items;
    first += (top - bottom) * n_active;
    if (first > 0x3fffffff) return false;
  }
  s.n_segs = n_segs;
  s.n_entries = (int)first;
  return true;
}

// Entry index (0 <= entry < n_entries) -> problem m and its query tile qt.
APBV_HOST_DEVICE inline void decode_group_entry(const GroupSchedule& s, int entry, int& m, int& qt) {
  int sg = 0;
  while (sg + 1 < s.n_segs && entry >= s.seg[sg + 1].first) ++sg;
  const int r = entry - s.seg[sg].first;
  const int level = s.seg[sg].level_hi - r / s.seg[sg].n_active;
  m = (int)((s.seg[sg].items >> (4 * (r % s.seg[sg].n_active))) & 15u);
  qt = level - s.level0[m];
}

}  // namespace apbv
