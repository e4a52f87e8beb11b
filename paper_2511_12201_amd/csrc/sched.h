// Device-side work list for the query-tile kernels (attention forward, backward dQ).
//
// Work item = one tile (tile_m rows, 128 or 256) of a head's kept queries.  Under the causal mask the
// items differ in length by two orders of magnitude (a head's last tile streams every selected key, its
// first one tile), and a launch has only a few thousand of them for 256 persistent workgroups: handed out
// head by head, the long items of the last heads start late and a few workgroups finish them alone
// (measured: 17 % of the kernel time).  So the items are sorted by cost, longest first, and every
// workgroup pulls the next one from a single atomic counter -- the classic longest-processing-time
// rule, whose tail is bounded by the shortest items.  The cost of an item is the number of key tiles
// it streams: exact when the per-query visible-prefix counts are given, else estimated from the
// position of the tile.
//
// The list can be cut into kSchedQueues queues, one per XCD (workgroups are dealt to the XCDs round-robin, so
// workgroup i sits on XCD i % 8): whole heads are assigned to queues, largest first onto the least loaded
// queue, and inside a queue the heads follow one another, each longest item first (one list after all if some
// head outweighs a queue's fair share, see sched_queues_pay).  The 32 workgroups of an
// XCD then stream the K/V tiles of one head a few tiles apart and find them in the XCD's own L2 instead of
// each fetching its own copy; a workgroup whose queue is drained takes from the queue with the most items left.
// On the 64k forward this cuts the traffic from beyond L2 to a third and leaves the kernel time where it was: the
// kernel is not bound by that traffic, the queues just stop it from wasting memory bandwidth.
//
// Layout of the int array in device memory:
//   [0] unused   [1] number of items   [2..3] unused
//   [4 .. 11] cursor[q]: next position of queue q   [12 .. 19] end[q]   (one queue: cursor[0] = 0, end[0] = items)
//   [20 .. 20 + BH]          head_prefix[BH + 1]  (cumulative tile counts, head-major item ids)
//   [.. + BH]                head_cost[BH]        (sum of the head's item costs)
//   [.. + BH]                head_place[BH]       (queue << 16 | position of the head inside its queue)
//   [.. + 2 * cap]           sort keys of the items by id (64-bit, see sched_key)
//   [.. + cap]               order[k] = (head << 16 | tile) of the k-th item to hand out
// with cap = BH * ceil(N / tile_m) the largest possible number of items.
#pragma once

#include "common.h"

namespace omni {

constexpr int kSchedQueues = 8;
constexpr int kSchedTotal = 1, kSchedCursor = 4, kSchedEnd = kSchedCursor + kSchedQueues, kSchedPrefix = kSchedEnd + kSchedQueues;
constexpr int kSchedMaxQueuedHeads = 1024;       // more heads than this: one queue (the placement is a serial loop)

inline size_t sched_cap(int BH, int N, int tile_m) { return (size_t)BH * ((N + tile_m - 1) / tile_m); }
__host__ __device__ inline size_t sched_head_cost_off(int BH) { return (size_t)kSchedPrefix + BH + 1; }
__host__ __device__ inline size_t sched_head_place_off(int BH) { return sched_head_cost_off(BH) + BH; }
inline size_t sched_keys_off(int BH) { return (sched_head_place_off(BH) + BH + 1) & ~(size_t)1; }      // 8-byte aligned
inline size_t sched_order_off(int BH, int N, int tile_m) { return sched_keys_off(BH) + 2 * sched_cap(BH, N, tile_m); }
inline size_t sched_ints(int BH, int N, int tile_m) { return sched_order_off(BH, N, tile_m) + sched_cap(BH, N, tile_m); }

// qvis (nullable): [B*Hq, N] visible packed keys per kept-query position, for exact costs
// queues: 1 (one longest-first list) or kSchedQueues (one list per XCD, whole heads per queue)
int run_schedule(const Layer& L, const int* q_cnt, const int* budget, int b_cap, int tile_m, const int* qvis, int* sched,
                 hipStream_t st, int queues = 1);
int persistent_grid();      // workgroups that fill the device at two per CU

// Called by one thread.  Position in the hand-out order of the next item, or -1 when every queue is drained:
// the workgroup's own queue (its XCD's) while it lasts, then whichever queue has the most items left.
__device__ __forceinline__ int sched_next(int* __restrict__ sched) {
  const int home = blockIdx.x % kSchedQueues;
  {
    const int end = sched[kSchedEnd + home];
    if (__atomic_load_n(sched + kSchedCursor + home, __ATOMIC_RELAXED) < end) {
      const int k = atomicAdd(sched + kSchedCursor + home, 1);
      if (k < end) return k;
    }
  }
  for (;;) {                                   // every pass either returns or finds one more queue drained
    int best = -1, left = 0;
    for (int q = 0; q < kSchedQueues; ++q) {
      const int rem = sched[kSchedEnd + q] - __atomic_load_n(sched + kSchedCursor + q, __ATOMIC_RELAXED);
      if (rem > left) left = rem, best = q;
    }
    if (best < 0) return -1;
    const int k = atomicAdd(sched + kSchedCursor + best, 1);
    if (k < sched[kSchedEnd + best]) return k;
  }
}

// hand-out position -> (head index bh, query tile tq)
__host__ __device__ inline void sched_decode(const int* __restrict__ sched, size_t order_off, int k, int& bh, int& tq) {
  const unsigned v = (unsigned)sched[order_off + k];
  bh = (int)(v >> 16);
  tq = (int)(v & 0xffffu);
}

// key tiles streamed by tile tq of a head with nt tiles and nk selected keys, estimated from its position
__host__ __device__ inline int sched_estimate(int tq, int nt, int nk, int causal) {
  if (!causal) return (nk + kTileN - 1) / kTileN;
  const long long keys = ((long long)nk * (tq + 1) + nt - 1) / nt;
  return (int)((keys + kTileN - 1) / kTileN);
}

// head-major item id -> 64-bit sort key, handed out in descending order: queue 0 first, inside a queue the heads in
// the order they were placed, inside a head larger cost first, lower id first among equals.  place = queue << 16 |
// position of the head in its queue (0 for the single list); cost < 2^16 key tiles.
__host__ __device__ inline unsigned long long sched_key(int cost, int id, unsigned place = 0u) {
  const unsigned long long q = 7u - (place >> 16), pos = 0x1fffu - (place & 0x1fffu);
  const unsigned c = cost < 0xffff ? (unsigned)cost : 0xffffu;
  return (q << 61) | (pos << 48) | ((unsigned long long)c << 32) | (unsigned)(0xffffffffu - (unsigned)id);
}

// Placement of the heads on the queues: in order of cost (descending, lower index first among equals) every head
// goes to the least loaded queue (lowest index among equals).  Loads are kept as (load << 3 | queue) in 32 bits so
// that the least loaded queue is one unsigned minimum; head costs are scaled down by `shift` bits to fit.
__host__ __device__ inline int sched_cost_shift(long long total_cost) {
  int shift = 0;
  while ((total_cost >> shift) >= (1ll << 27)) ++shift;
  return shift;
}

// Queues only pay while no head outweighs a queue's fair share by much: the workgroups of the other XCDs come to
// help such a head only when their own queues are drained, and what they then take are its middle-sized items, one
// of which is the tail (per-head budgets on the 64k layer, where one head holds 30 % of the work: 1.68 -> 1.92 ms
// with queues; at 13 % of the work, the shared budget, nothing is lost).  The line is drawn at 1.5 fair shares.
__host__ __device__ inline bool sched_queues_pay(long long total_cost, long long largest_head, int queues) {
  return 2 * largest_head * queues <= 3 * total_cost;
}

// Heads onto queues (host mirror of sched_assign_kernel).  Writes head_place, cursor and end.
inline void sched_assign_host(int* sched, int BH, int queues) {
  const int* prefix = sched + kSchedPrefix;
  const int* hcost = sched + sched_head_cost_off(BH);
  int* place = sched + sched_head_place_off(BH);
  int items[kSchedQueues], heads[kSchedQueues];
  unsigned load[kSchedQueues];
  for (int q = 0; q < kSchedQueues; ++q) items[q] = 0, heads[q] = 0, load[q] = (unsigned)q;
  long long total = 0;
  for (int bh = 0; bh < BH; ++bh) total += hcost[bh];
  const int shift = sched_cost_shift(total);
  long long largest = 0;
  for (int bh = 0; bh < BH; ++bh) largest = hcost[bh] > largest ? hcost[bh] : largest;
  if (queues <= 1 || BH > kSchedMaxQueuedHeads || !sched_queues_pay(total, largest, queues)) {
    for (int bh = 0; bh < BH; ++bh) place[bh] = 0;
    items[0] = prefix[BH];
  } else {
    for (int bh = 0; bh < BH; ++bh) place[bh] = -1;
    for (int n = 0; n < BH; ++n) {
      int best = -1;                                   // largest head not placed yet (lowest index among equals)
      for (int bh = 0; bh < BH; ++bh)
        if (place[bh] < 0 && (best < 0 || hcost[bh] > hcost[best])) best = bh;
      unsigned m = load[0];
      for (int r = 1; r < queues; ++r) m = load[r] < m ? load[r] : m;
      const int q = (int)(m & 7u);
      place[best] = (q << 16) | heads[q];
      heads[q] += 1;
      load[q] += (unsigned)(hcost[best] >> shift) << 3;
      items[q] += prefix[best + 1] - prefix[best];
    }
  }
  int start = 0;
  for (int q = 0; q < kSchedQueues; ++q) {
    sched[kSchedCursor + q] = start;
    start += items[q];
    sched[kSchedEnd + q] = start;
  }
}

// Host mirror of the device kernels (diagnostic entry point and CPU tests): fills prefix, total and order.
void sched_build_host(const int* q_cnt, const int* budget, int B, int Hq, int N, int b_cap, int causal, int tile_m,
                      int* sched, int queues = 1);

}  // namespace omni
