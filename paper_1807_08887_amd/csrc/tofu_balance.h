// How a kernel that cuts its own reduction deals the steps of n tiles to a fixed number of
// workgroups (a partition-n-reduce inside one worker, arXiv 1807.08887 Sec. 3.1 way 2: the pieces of
// a tile are partial results summed afterwards in a fixed order).
//
// Two goals.  (1) Every workgroup gets the same amount of work.  (2) Workgroups that run side by
// side are at the same place of the reduction at the same time, because then the operand rows
// they have in common are read from memory once and found in the shared L2 by the others.  Dealing
// one long run of (tile, step) units evenly reaches (1) but not (2): neighbouring workgroups then
// start at different steps of different tiles.  Instead:
//   * every tile has `per_tile` workgroups of its OWN: workgroup r * n + t takes the steps
//     [r * piece, (r + 1) * piece) of tile t -- all workgroups with the same r walk the same steps;
//   * what these leave of every tile, its steps [tail0, steps), is its TAIL.  The remaining
//     G2 = groups - per_tile * n workgroups take the tails: workgroup j first the whole tails of the
//     tiles j, j + G2, j + 2 G2, ... (`rounds` of them, again the same steps at the same time), and
//     then its even share of the tails of the last n - rounds * G2 tiles, which are cut into units of
//     one step and dealt as one run (a share is shorter than one tail, so it meets at most two tiles).
//     With more tiles than workgroups there are no own workgroups and a tile is all tail.
// Every piece leaves its accumulators in a slot of the workspace:
//   slot r * n + t                               own piece r of tile t
//   slot per_tile * n + t                        whole tail of tile t < rounds * G2
//   slot per_tile * n + rounds * G2 + 2 j + s    segment s (0 or 1) of tail workgroup j's share of the last tails
// and a second kernel sums a tile's slots in the order of the steps.
#ifndef TOFU_BALANCE_H_
#define TOFU_BALANCE_H_

#include <stdint.h>

#if defined(__HIPCC__)
#define TOFU_HD __host__ __device__ __forceinline__
#else
#define TOFU_HD inline
#endif

namespace tofu {

struct Balance {
  int n;          // tiles
  int groups;     // workgroups
  int per_tile;   // own workgroups per tile
  int piece;      // steps of one own piece
  int tail0;      // first step of every tile's tail (== steps: no tails)
  int rounds;     // whole tails per tail workgroup
};

struct BalanceSegment {
  int tile;        // relative tile
  int begin, end;  // steps [begin, end) of the tile's reduction
  int slot;
};

TOFU_HD int balance_tail_groups(const Balance& b) { return b.groups - b.per_tile * b.n; }

// Number of slots the pieces of a launch occupy.
TOFU_HD int64_t balance_slots(const Balance& b, int steps) {
  const int g2 = balance_tail_groups(b);
  return (int64_t)b.per_tile * b.n + (b.tail0 < steps ? (int64_t)b.rounds * g2 + 2 * (int64_t)g2 : 0);
}

// Segments of workgroup `wg` (0 .. groups-1): their number, and the i-th of them.
struct BalanceWalk {
  int count;
  // own piece
  bool own;
  int own_tile, own_begin, own_end, own_slot;
  // tails
  int j, g2, rounds, tail0, steps, slot0;
  int64_t u_begin, u_end;   // run of units in the space of the last tails (tail-major)
  int first_left;           // first of the last tails the run meets
};

TOFU_HD BalanceWalk balance_walk(const Balance& b, int steps, int wg) {
  BalanceWalk w;
  const int n_own = b.per_tile * b.n;
  w.own = wg < n_own;
  w.count = 0;
  w.own_tile = w.own_begin = w.own_end = w.own_slot = 0;
  w.j = wg - n_own; w.g2 = b.groups - n_own; w.rounds = b.rounds; w.tail0 = b.tail0; w.steps = steps;
  w.slot0 = n_own;
  w.u_begin = w.u_end = 0; w.first_left = 0;
  if (w.own) {
    const int r = wg / b.n;
    w.own_tile = wg - r * b.n;
    w.own_begin = r * b.piece;
    w.own_end = w.own_begin + b.piece < b.tail0 ? w.own_begin + b.piece : b.tail0;
    w.own_slot = wg;
    w.count = w.own_begin < w.own_end ? 1 : 0;
  } else if (b.tail0 < steps) {
    const int tail = steps - b.tail0;
    const int64_t left_units = (int64_t)(b.n - b.rounds * w.g2) * tail;
    w.u_begin = w.j * left_units / w.g2;
    w.u_end = (w.j + 1) * left_units / w.g2;
    w.count = b.rounds;
    if (w.u_begin < w.u_end) {
      w.first_left = (int)(w.u_begin / tail);
      w.count += (int)((w.u_end - 1) / tail) - w.first_left + 1;
    }
  }
  return w;
}

TOFU_HD BalanceSegment balance_segment(const BalanceWalk& w, int i) {
  BalanceSegment s;
  if (w.own) {
    s.tile = w.own_tile; s.begin = w.own_begin; s.end = w.own_end; s.slot = w.own_slot;
  } else if (i < w.rounds) {
    s.tile = w.j + i * w.g2; s.begin = w.tail0; s.end = w.steps; s.slot = w.slot0 + s.tile;
  } else {
    const int tail = w.steps - w.tail0, k = i - w.rounds, t_left = w.first_left + k;
    const int64_t t0 = (int64_t)t_left * tail;
    s.tile = w.rounds * w.g2 + t_left;
    s.begin = w.tail0 + (int)((w.u_begin > t0 ? w.u_begin : t0) - t0);
    s.end = w.tail0 + (int)((w.u_end < t0 + tail ? w.u_end : t0 + tail) - t0);
    s.slot = w.slot0 + w.rounds * w.g2 + 2 * w.j + k;
  }
  return s;
}

// Calls f(slot) for every slot that holds a piece of tile `tile`, in the order of the steps.
template <class F>
TOFU_HD void balance_for_each_slot(const Balance& b, int steps, int tile, F f) {
  const int n_own = b.per_tile * b.n;
  for (int r = 0; r < b.per_tile && r * b.piece < b.tail0; ++r) f(r * b.n + tile);
  if (b.tail0 >= steps) return;
  const int g2 = b.groups - n_own, whole = b.rounds * g2;
  if (tile < whole) { f(n_own + tile); return; }
  const int tail = steps - b.tail0, t_left = tile - whole;
  const int64_t left_units = (int64_t)(b.n - whole) * tail;
  // tail workgroups whose runs meet this tail: g(u) = floor(((u + 1) * G2 - 1) / N)
  const int64_t u0 = (int64_t)t_left * tail, u1 = u0 + tail - 1;
  const int g_first = (int)(((u0 + 1) * g2 - 1) / left_units), g_last = (int)(((u1 + 1) * g2 - 1) / left_units);
  for (int g = g_first; g <= g_last; ++g) {
    const int64_t ub = g * left_units / g2, ue = (g + 1) * left_units / g2;
    if (ub >= ue) continue;                          // more workgroups than units: this one has no share
    const int first_left = (int)(ub / tail);         // the tail that holds the run's first unit = its segment 0
    f(n_own + whole + 2 * g + (t_left - first_left));
  }
}

// Host: the plan for n tiles of `steps` steps on at most `max_groups` workgroups.  `segment_cost`
// is what a workgroup loses per segment (setting up, filling its pipeline, writing the slot) in
// steps; it only sizes the tails so that the tail workgroups finish together with the others.
inline Balance balance_plan(int64_t n, int64_t steps, int max_groups, int segment_cost) {
  Balance b;
  const int64_t units = n * steps;
  b.n = (int)n;
  b.groups = (int)(units < max_groups ? units : max_groups);
  b.per_tile = (int)(b.groups / n);
  b.rounds = 0;
  if (b.per_tile == 0) {   // more tiles than workgroups: every tile is all tail
    b.piece = 0;
    b.tail0 = 0;
    b.rounds = (int)(n / b.groups);
    return b;
  }
  const int g2 = (int)(b.groups - b.per_tile * n);
  const int full = (int)((steps + b.per_tile - 1) / b.per_tile);   // piece length that leaves no tail
  b.piece = full;
  if (g2 > 0) {
    const int rounds = (int)(n / g2);
    const int64_t left = n - (int64_t)rounds * g2;
    // the shortest piece whose tails keep the tail workgroups no longer busy than the others; a longer piece
    // means shorter tails, so the condition is monotone and the shortest piece is found by bisection
    auto fits = [&](int64_t piece) {
      const int64_t tail = steps - (int64_t)b.per_tile * piece;
      const int64_t per = rounds * tail + (left * tail + g2 - 1) / g2;
      const int64_t segments = rounds + (left > 0 ? 2 : 0);
      return per + segments * segment_cost <= piece + segment_cost;
    };
    int64_t lo = units / b.groups > 0 ? units / b.groups : 1, hi = full;   // pieces in [lo, full) leave a tail; `full` none
    if (lo < hi && fits(hi - 1)) {
      int64_t bad = lo - 1, good = hi - 1;                                 // fits(good), and bad is below the range or does not fit
      while (good - bad > 1) {
        const int64_t mid = bad + (good - bad) / 2;
        if (fits(mid)) good = mid; else bad = mid;
      }
      b.piece = (int)good;
      b.rounds = rounds;
    }
  }
  const int64_t covered = (int64_t)b.per_tile * b.piece;
  b.tail0 = (int)(covered < steps ? covered : steps);
  if (b.tail0 >= steps) { b.groups = (int)(b.per_tile * n); b.rounds = 0; }   // no tails: spare workgroups would have nothing to do
  return b;
}

}  // namespace tofu

#endif  // TOFU_BALANCE_H_
