// Exhaustive host-side check of the work distribution in csrc/tofu_balance.h (compiled and run by
// tests/test_host_balance.py): for a grid of tile counts, step counts and workgroup limits, the
// segments of all workgroups must cover every (tile, step) exactly once, every segment must own a
// distinct slot below balance_slots(), the slot walk of a tile must name exactly that tile's slots
// in the order of their steps, and (for long reductions) no workgroup may be more than 5 % busier than
// under an even split of one run of units.
#include <algorithm>
#include <cstdio>
#include <cstdlib>
#include <map>
#include <vector>

#include "tofu_balance.h"

using namespace tofu;

static int check(int n, int steps, int max_groups, int cost, double* worst_over) {
  const Balance b = balance_plan(n, steps, max_groups, cost);
  if (b.groups < 1 || b.groups > max_groups || b.per_tile < 0) { printf("bad plan n=%d steps=%d\n", n, steps); return 1; }
  const int64_t slots = balance_slots(b, steps);
  std::vector<int> cover((size_t)n * steps, 0);
  std::vector<int> slot_used((size_t)slots, 0);
  std::map<int, std::vector<std::pair<int, int>>> by_tile;   // tile -> (begin, slot)
  int64_t busiest = 0;
  for (int wg = 0; wg < b.groups; ++wg) {
    const BalanceWalk w = balance_walk(b, steps, wg);
    int64_t work = 0;
    for (int i = 0; i < w.count; ++i) {
      const BalanceSegment s = balance_segment(w, i);
      if (s.tile < 0 || s.tile >= n || s.begin < 0 || s.end > steps || s.begin >= s.end) { printf("bad segment n=%d steps=%d wg=%d\n", n, steps, wg); return 1; }
      if (s.slot < 0 || s.slot >= slots || slot_used[s.slot]++) { printf("bad slot %d of %lld n=%d steps=%d wg=%d\n", s.slot, (long long)slots, n, steps, wg); return 1; }
      for (int k = s.begin; k < s.end; ++k) cover[(size_t)s.tile * steps + k]++;
      by_tile[s.tile].push_back({s.begin, s.slot});
      work += s.end - s.begin + cost;
    }
    if (work > busiest) busiest = work;
  }
  for (size_t i = 0; i < cover.size(); ++i)
    if (cover[i] != 1) { printf("tile %zu step %zu covered %d times (n=%d steps=%d groups=%d)\n", i / steps, i % steps, cover[i], n, steps, max_groups); return 1; }
  for (int t = 0; t < n; ++t) {
    std::vector<int> got;
    balance_for_each_slot(b, steps, t, [&](int slot) { got.push_back(slot); });
    auto& want = by_tile[t];
    // the segments of one tile come from different workgroups in any order; the walk must list them by step
    std::sort(want.begin(), want.end());
    if (got.size() != want.size()) { printf("tile %d: %zu slots walked, %zu written (n=%d steps=%d)\n", t, got.size(), want.size(), n, steps); return 1; }
    for (size_t i = 0; i < got.size(); ++i)
      if (got[i] != want[i].second) { printf("tile %d: slot order differs (n=%d steps=%d)\n", t, n, steps); return 1; }
  }
  // an even split of one run of units costs every workgroup its share plus about two segments
  const double even = (double)n * steps / (n * (int64_t)steps < max_groups ? n * (int64_t)steps : max_groups);
  const double over = busiest / (even + 2 * cost);
  if (over > *worst_over) *worst_over = over;
  return 0;
}

int main() {
  double worst = 0, worst_long = 0;
  int cases = 0;
  for (int max_groups : {8, 64, 512})
    for (int n = 1; n < 2 * max_groups && n <= 600; n += (n < 70 ? 1 : 7))
      for (int steps : {1, 2, 3, 4, 5, 7, 16, 33, 80, 448, 640}) {
        if (n >= max_groups && n % max_groups == 0) continue;   // whole waves are launched without balancing
        double w = 0;
        if (check(n, steps, max_groups, 2, &w)) return 1;
        if (w > worst) worst = w;
        if (steps >= 80 && w > worst_long) worst_long = w;
        ++cases;
      }
  // the benchmark shapes
  for (auto c : {std::pair<int, int>{490, 640}, {245, 640}, {400, 448}, {400, 112}, {336, 80}}) {
    double w = 0;
    if (check(c.first, c.second, 512, 2, &w)) return 1;
    const Balance b = balance_plan(c.first, c.second, 512, 2);
    printf("n=%d steps=%d: groups=%d per_tile=%d piece=%d tail0=%d rounds=%d slots=%lld busiest/even=%.4f\n", c.first, c.second, b.groups, b.per_tile,
           b.piece, b.tail0, b.rounds, (long long)balance_slots(b, c.second), w);
  }
  {  // a very long reduction: the plan is found by bisection (no loop over the steps), and the segments still add up
    const int64_t n = 400, steps = (int64_t)1 << 28;
    const Balance b = balance_plan(n, steps, 512, 2);
    int64_t total = 0, busiest = 0;
    for (int wg = 0; wg < b.groups; ++wg) {
      const BalanceWalk w = balance_walk(b, (int)steps, wg);
      int64_t work = 0;
      for (int i = 0; i < w.count; ++i) { const BalanceSegment sg = balance_segment(w, i); work += sg.end - sg.begin; }
      total += work;
      if (work > busiest) busiest = work;
    }
    if (total != n * steps || busiest > (n * steps / 512) * 1.001 + 64) { printf("long reduction: total %lld busiest %lld\n", (long long)total, (long long)busiest); return 1; }
  }
  printf("cases=%d worst busiest/(even + 2 cost)=%.3f, with 80 or more steps %.3f\n", cases, worst, worst_long);
  // long reductions (the case the scheme is for) must stay within 5 % of the even share
  return worst_long <= 1.05 ? 0 : 2;
}
