// Device-side work list for the query-tile kernels (attention forward, backward dQ).
//
// Work item = one tile (tile_m rows, 128 or 256) of a head's kept queries.  Items are ordered head
// by head, longest tile first (under the causal mask the last tile of a head
// sees the most keys), and cut into 8 contiguous segments of about equal cost,
// one per XCD.  The kernels are persistent: every workgroup reads the id of the
// XCD it runs on, pulls items from that XCD's segment through an atomic
// counter, and moves on to the other segments when its own is empty.  The
// workgroups resident on an XCD therefore work on neighbouring tiles of the same
// head and stream the same packed K/V tiles through that XCD's L2 at about the
// same time, instead of every workgroup pulling its own copy from HBM.
//
// Layout of the int array in device memory:
//   [0..8]   seg_begin  (item index ranges per XCD)
//   [9..16]  counters   (zeroed by the scheduler kernel before every launch)
//   [17]     total number of items
//   [18..]   head_prefix[BH + 1] (cumulative tile counts)
#pragma once

#include "common.h"

namespace omni {

constexpr int kSchedSeg = 0, kSchedCounter = 9, kSchedTotal = 17, kSchedPrefix = 18;
constexpr int kNumXcd = 8;

inline size_t sched_ints(int BH) { return (size_t)kSchedPrefix + BH + 1; }

int run_schedule(const Layer& L, const int* q_cnt, const int* budget, int b_cap, int tile_m, int* sched,
                 hipStream_t st);
int persistent_grid();      // workgroups that fill the device at two per CU

// XCC_ID hardware register (id 20), bits [3:0]
__device__ __forceinline__ int xcc_id() { return (int)(__builtin_amdgcn_s_getreg((3 << 11) | 20) & 7u); }

// Called by one thread.  Next item for a workgroup on `xcd`, or -1 when every segment is drained.
__device__ __forceinline__ int sched_next(int* __restrict__ sched, int xcd) {
  for (int t = 0; t < kNumXcd; ++t) {
    const int x = (xcd + t) & (kNumXcd - 1);
    const int len = sched[kSchedSeg + x + 1] - sched[kSchedSeg + x];
    if (len <= 0) continue;
    int* ctr = sched + kSchedCounter + x;
    if (__atomic_load_n(ctr, __ATOMIC_RELAXED) >= len) continue;
    const int k = atomicAdd(ctr, 1);
    if (k < len) return sched[kSchedSeg + x] + k;
  }
  return -1;
}

// item -> (head index bh, query tile tq); tiles of a head are handed out last first
__host__ __device__ inline void sched_decode(const int* __restrict__ sched, int BH, int item, int& bh, int& tq) {
  const int* prefix = sched + kSchedPrefix;
  int lo = 0, hi = BH;                     // largest bh with prefix[bh] <= item
  while (hi - lo > 1) {
    const int mid = (lo + hi) >> 1;
    if (prefix[mid] <= item) lo = mid; else hi = mid;
  }
  bh = lo;
  tq = prefix[lo + 1] - 1 - item;          // = (tiles of the head) - 1 - (item - prefix[lo])
}

// cost model: keys visited by the m longest tiles of a head (+ a fixed per-tile overhead)
__host__ __device__ inline double sched_head_cost(int m, int nt, int nk, int causal) {
  const double overhead = 64.0 * m;
  if (!causal) return overhead + (double)nk * m;
  return overhead + (double)nk / nt * ((double)m * nt - 0.5 * (double)m * (m - 1));
}

// Fills the whole array (run by one device thread, or on the host by the diagnostic entry point).
__host__ __device__ inline void sched_build(const int* q_cnt, const int* budget, int B, int Hq, int N, int b_cap,
                                            int causal, int tile_m, int* sched) {
  const int BH = B * Hq;
  int* prefix = sched + kSchedPrefix;
  int items = 0;
  double total = 0.0;
  for (int bh = 0; bh < BH; ++bh) {
    const int nq = q_cnt ? q_cnt[bh] : N;
    const int nt = nq > 0 ? (nq + tile_m - 1) / tile_m : 0;
    int nk = budget ? budget[bh / Hq] : N;
    nk = nk < 0 ? 0 : (nk > b_cap ? b_cap : nk);
    prefix[bh] = items;
    items += nt;
    if (nt) total += sched_head_cost(nt, nt, nk, causal);
  }
  prefix[BH] = items;
  sched[kSchedTotal] = items;
  for (int x = 0; x < kNumXcd; ++x) sched[kSchedCounter + x] = 0;
  sched[kSchedSeg] = 0;
  sched[kSchedSeg + kNumXcd] = items;
  int bh = 0;
  double cum = 0.0;                        // cost of the heads before bh
  for (int x = 1; x < kNumXcd; ++x) {
    const double target = total * x / kNumXcd;
    int cut = items;
    while (bh < BH) {
      const int nq = q_cnt ? q_cnt[bh] : N;
      const int nt = nq > 0 ? (nq + tile_m - 1) / tile_m : 0;
      int nk = budget ? budget[bh / Hq] : N;
      nk = nk < 0 ? 0 : (nk > b_cap ? b_cap : nk);
      const double hc = nt ? sched_head_cost(nt, nt, nk, causal) : 0.0;
      if (nt && cum + hc >= target) {
        int lo = 0, hi = nt;               // smallest m with cum + cost(m) >= target
        while (lo < hi) {
          const int mid = (lo + hi) >> 1;
          if (cum + sched_head_cost(mid, nt, nk, causal) >= target) hi = mid; else lo = mid + 1;
        }
        cut = prefix[bh] + lo;
        break;
      }
      cum += hc;
      ++bh;
    }
    sched[kSchedSeg + x] = cut;
  }
}

}  // namespace omni
