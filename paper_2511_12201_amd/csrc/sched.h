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
// position of the tile.  (Keeping neighbouring tiles of a head on one XCD, so that they share K/V tiles
// in its L2, was tried first: with all K/V made cache-resident the kernel time does not change, so
// locality is not what limits it.)
//
// Layout of the int array in device memory:
//   [0] counter (zeroed before every launch)   [1] number of items   [2..3] unused
//   [4 .. 4 + BH]            head_prefix[BH + 1]  (cumulative tile counts, head-major item ids)
//   [.. + 2 * cap]           cost keys of the items by id (64-bit: cost << 32 | ~id)
//   [.. + cap]               order[k] = (head << 16 | tile) of the k-th item to hand out
// with cap = BH * ceil(N / tile_m) the largest possible number of items.
#pragma once

#include "common.h"

namespace omni {

constexpr int kSchedCounter = 0, kSchedTotal = 1, kSchedPrefix = 4;

inline size_t sched_cap(int BH, int N, int tile_m) { return (size_t)BH * ((N + tile_m - 1) / tile_m); }
inline size_t sched_keys_off(int BH) { return (size_t)((kSchedPrefix + BH + 1 + 1) & ~1); }            // 8-byte aligned
inline size_t sched_order_off(int BH, int N, int tile_m) { return sched_keys_off(BH) + 2 * sched_cap(BH, N, tile_m); }
inline size_t sched_ints(int BH, int N, int tile_m) { return sched_order_off(BH, N, tile_m) + sched_cap(BH, N, tile_m); }

// qvis (nullable): [B*Hq, N] visible packed keys per kept-query position, for exact costs
int run_schedule(const Layer& L, const int* q_cnt, const int* budget, int b_cap, int tile_m, const int* qvis, int* sched,
                 hipStream_t st);
int persistent_grid();      // workgroups that fill the device at two per CU

// Called by one thread.  Position in the hand-out order of the next item, or -1 when the list is drained.
__device__ __forceinline__ int sched_next(int* __restrict__ sched) {
  if (__atomic_load_n(sched + kSchedCounter, __ATOMIC_RELAXED) >= sched[kSchedTotal]) return -1;
  const int k = atomicAdd(sched + kSchedCounter, 1);
  return k < sched[kSchedTotal] ? k : -1;
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

// head-major item id -> 64-bit sort key: larger cost first, lower id first among equals
__host__ __device__ inline unsigned long long sched_key(int cost, int id) {
  return ((unsigned long long)(unsigned)cost << 32) | (unsigned)(0xffffffffu - (unsigned)id);
}

// Host mirror of the device kernels (diagnostic entry point and CPU tests): fills prefix, total and order.
void sched_build_host(const int* q_cnt, const int* budget, int B, int Hq, int N, int b_cap, int causal, int tile_m,
                      int* sched);

}  // namespace omni
