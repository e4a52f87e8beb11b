// Builds the cost-sorted work list described in sched.h (three tiny kernels, no host sync).
#include "sched.h"

#include <algorithm>
#include <vector>

namespace omni {

namespace {

// one thread: cumulative tile counts of the heads, total, counter
__global__ void sched_prefix_kernel(const int* __restrict__ q_cnt, int BH, int N, int tile_m, int* __restrict__ sched) {
  if (threadIdx.x != 0 || blockIdx.x != 0) return;
  int items = 0;
  for (int bh = 0; bh < BH; ++bh) {
    const int nq = q_cnt ? q_cnt[bh] : N;
    sched[kSchedPrefix + bh] = items;
    items += nq > 0 ? (nq + tile_m - 1) / tile_m : 0;
  }
  sched[kSchedPrefix + BH] = items;
  sched[kSchedTotal] = items;
  for (int q = 0; q < kSchedQueues; ++q) {                 // one list; sched_assign_kernel cuts it into queues if asked to
    sched[kSchedCursor + q] = q == 0 ? 0 : items;
    sched[kSchedEnd + q] = items;
  }
}

struct ItemRef {
  int bh, tq, nt;
};

__device__ __forceinline__ ItemRef item_of(const int* __restrict__ prefix, int BH, int id) {
  int lo = 0, hi = BH;                     // largest bh with prefix[bh] <= id
  while (hi - lo > 1) {
    const int mid = (lo + hi) >> 1;
    if (prefix[mid] <= id) lo = mid; else hi = mid;
  }
  ItemRef r;
  r.bh = lo;
  r.tq = id - prefix[lo];
  r.nt = prefix[lo + 1] - prefix[lo];
  return r;
}

// thread per item id: its cost key
__global__ __launch_bounds__(256) void sched_cost_kernel(const int* __restrict__ q_cnt, const int* __restrict__ budget,
                                                         const int* __restrict__ qvis, int bph, int BH, int Hq, int N, int b_cap,
                                                         int causal, int tile_m, size_t keys_off, int* __restrict__ sched) {
  const int id = blockIdx.x * blockDim.x + threadIdx.x;
  if (id >= sched[kSchedTotal]) return;
  const ItemRef it = item_of(sched + kSchedPrefix, BH, id);
  int nk = budget ? budget[budget_slot(bph, it.bh / Hq, it.bh)] : N;
  nk = nk < 0 ? 0 : (nk > b_cap ? b_cap : nk);
  int cost;
  if (qvis) {
    const int nq = q_cnt ? q_cnt[it.bh] : N;
    const int last = min((it.tq + 1) * tile_m, nq) - 1;
    cost = (qvis[(long long)it.bh * N + last] + kTileN - 1) / kTileN;
  } else {
    cost = sched_estimate(it.tq, it.nt, nk, causal);
  }
  reinterpret_cast<unsigned long long*>(sched + keys_off)[id] = sched_key(cost, id);
}

// One workgroup: cost of every head, heads onto queues (largest first onto the least loaded queue), queue bounds,
// and the queue and position of its head folded into every item's sort key.  queues <= 1 or too many heads: one
// queue.  Everything the serial placement loop and the binary searches touch sits in LDS.
constexpr int kAssignThreads = 1024;
__global__ __launch_bounds__(kAssignThreads) void sched_assign_kernel(int BH, int queues, size_t keys_off, int* __restrict__ sched) {
  __shared__ int sPrefix[kSchedMaxQueuedHeads + 1], sCost[kSchedMaxQueuedHeads], sOrder[kSchedMaxQueuedHeads],
      sPlace[kSchedMaxQueuedHeads], sRankItems[kSchedMaxQueuedHeads], sRankPlace[kSchedMaxQueuedHeads], sShift;
  __shared__ unsigned sRankCost[kSchedMaxQueuedHeads];
  const int items_all = sched[kSchedTotal];
  auto one_queue = [&]() {                                // the keys already carry place 0
    if (threadIdx.x < kSchedQueues) {
      sched[kSchedCursor + threadIdx.x] = threadIdx.x == 0 ? 0 : items_all;
      sched[kSchedEnd + threadIdx.x] = items_all;
    }
    for (int bh = threadIdx.x; bh < BH; bh += kAssignThreads) sched[sched_head_place_off(BH) + bh] = 0;
  };
  if (queues <= 1 || BH > kSchedMaxQueuedHeads) {
    one_queue();
    return;
  }
  unsigned long long* keys = reinterpret_cast<unsigned long long*>(sched + keys_off);
  for (int bh = threadIdx.x; bh <= BH; bh += kAssignThreads) sPrefix[bh] = sched[kSchedPrefix + bh];
  for (int bh = threadIdx.x; bh < BH; bh += kAssignThreads) sCost[bh] = 0;
  __syncthreads();
  // head costs: a wavefront's 64 consecutive items belong to one head most of the time.  kBatch key loads are in
  // flight together (one workgroup walks the whole list: a load per trip would cost a memory latency per trip).
  constexpr int kBatch = 8;
  for (int base = (threadIdx.x & ~63); base < items_all; base += kBatch * kAssignThreads) {
    unsigned long long kv[kBatch];
#pragma unroll
    for (int e = 0; e < kBatch; ++e) {
      const int id = base + e * kAssignThreads + (threadIdx.x & 63);
      kv[e] = id < items_all ? keys[id] : 0ull;
    }
#pragma unroll
    for (int e = 0; e < kBatch; ++e) {
      const int id = base + e * kAssignThreads + (threadIdx.x & 63);
      int bh = -1, c = 0;
      if (id < items_all) {
        bh = item_of(sPrefix, BH, id).bh;
        c = (int)((kv[e] >> 32) & 0xffffu);
      }
      const int first = __shfl(bh, 0, 64);
      if (__all(bh == first || bh < 0)) {
        c = wave_sum(c);
        if ((threadIdx.x & 63) == 0 && first >= 0) atomicAdd(&sCost[first], c);
      } else if (bh >= 0) {
        atomicAdd(&sCost[bh], c);
      }
    }
  }
  __syncthreads();
  for (int bh = threadIdx.x; bh < BH; bh += kAssignThreads) {       // rank of a head: cost descending, index ascending
    const int mine = sCost[bh];
    int r = 0;
    for (int j = 0; j < BH; ++j) r += (sCost[j] > mine || (sCost[j] == mine && j < bh)) ? 1 : 0;
    sOrder[r] = bh;
  }
  __syncthreads();
  // cost and item count in rank order, so that the serial placement loop reads LDS sequentially
  if (threadIdx.x == 0) {
    long long total = 0;
    for (int bh = 0; bh < BH; ++bh) total += sCost[bh];
    sShift = sched_queues_pay(total, sCost[sOrder[0]], queues) ? sched_cost_shift(total) : -1;
  }
  __syncthreads();
  if (sShift < 0) {                                       // a head too large for a queue of its own: one list
    one_queue();
    return;
  }
  for (int r = threadIdx.x; r < BH; r += kAssignThreads) {
    const int bh = sOrder[r];
    sRankCost[r] = (unsigned)(sCost[bh] >> sShift) << 3;
    sRankItems[r] = sPrefix[bh + 1] - sPrefix[bh];
  }
  __syncthreads();
  if (threadIdx.x == 0) {
    unsigned load[kSchedQueues];               // load << 3 | queue: the least loaded queue is one unsigned minimum
    int heads[kSchedQueues], items[kSchedQueues];
#pragma unroll
    for (int q = 0; q < kSchedQueues; ++q) load[q] = q < queues ? (unsigned)q : 0xffffffffu, heads[q] = 0, items[q] = 0;
    for (int n = 0; n < BH; ++n) {
      unsigned m = load[0];
#pragma unroll
      for (int r = 1; r < kSchedQueues; ++r) m = min(m, load[r]);
      const int q = (int)(m & 7u);
      const unsigned c = sRankCost[n];
      const int ni = sRankItems[n];
#pragma unroll
      for (int r = 0; r < kSchedQueues; ++r)               // compile-time indices keep the arrays in registers
        if (r == q) {
          sRankPlace[n] = (r << 16) | heads[r];
          heads[r] += 1;
          load[r] += c;
          items[r] += ni;
        }
    }
    int start = 0;
#pragma unroll
    for (int q = 0; q < kSchedQueues; ++q) {
      sched[kSchedCursor + q] = start;
      start += items[q];
      sched[kSchedEnd + q] = start;
    }
  }
  __syncthreads();
  for (int r = threadIdx.x; r < BH; r += kAssignThreads) sPlace[sOrder[r]] = sRankPlace[r];
  __syncthreads();
  for (int bh = threadIdx.x; bh < BH; bh += kAssignThreads) {
    sched[sched_head_place_off(BH) + bh] = sPlace[bh];
    sched[sched_head_cost_off(BH) + bh] = sCost[bh];
  }
  for (int base = threadIdx.x; base < items_all; base += kBatch * kAssignThreads) {
    unsigned long long kv[kBatch];
#pragma unroll
    for (int e = 0; e < kBatch; ++e) {
      const int id = base + e * kAssignThreads;
      kv[e] = id < items_all ? keys[id] : 0ull;
    }
#pragma unroll
    for (int e = 0; e < kBatch; ++e) {
      const int id = base + e * kAssignThreads;
      if (id < items_all)
        keys[id] = sched_key((int)((kv[e] >> 32) & 0xffffu), id, (unsigned)sPlace[item_of(sPrefix, BH, id).bh]);
    }
  }
}

// kRankLanes threads per item id: its rank among the keys (all distinct) is its place in the hand-out order
constexpr int kRankLanes = 4;
constexpr int kRankItems = 256 / kRankLanes;                // items per workgroup
__global__ __launch_bounds__(256) void sched_rank_kernel(int BH, size_t keys_off, size_t order_off, int* __restrict__ sched) {
  constexpr int kTile = 2048;                               // keys staged per pass: a 64k layer's list in one
  __shared__ unsigned long long tile[kTile];
  const int n = sched[kSchedTotal];
  const int id = blockIdx.x * kRankItems + threadIdx.x / kRankLanes, sub = threadIdx.x % kRankLanes;
  const unsigned long long* keys = reinterpret_cast<const unsigned long long*>(sched + keys_off);
  const unsigned long long mine = id < n ? keys[id] : 0ull;
  int rank = 0;
  for (int j0 = 0; j0 < n; j0 += kTile) {                   // uniform trip count: every thread helps to stage
    __syncthreads();
#pragma unroll
    for (int u = 0; u < kTile / 256; ++u) {                 // independent loads: one memory latency per pass
      const int j = j0 + u * 256 + (int)threadIdx.x;
      tile[u * 256 + threadIdx.x] = j < n ? keys[j] : 0ull;
    }
    __syncthreads();
    const int m = min(kTile, n - j0);
#pragma unroll 16
    for (int j = sub; j < m; j += kRankLanes) rank += tile[j] > mine ? 1 : 0;     // unrolled: LDS reads in flight together
  }
#pragma unroll
  for (int o = 1; o < kRankLanes; o <<= 1) rank += __shfl_xor(rank, o, 64);
  if (id < n && sub == 0) {
    const ItemRef it = item_of(sched + kSchedPrefix, BH, id);
    sched[order_off + rank] = (int)(((unsigned)it.bh << 16) | (unsigned)it.tq);
  }
}

}  // namespace

int run_schedule(const Layer& L, const int* q_cnt, const int* budget, int b_cap, int tile_m, const int* qvis, int* sched,
                 hipStream_t st, int queues) {
  const int BH = L.B * L.Hq;
  if (BH >= 65536 || cdiv(L.N, tile_m) >= 65536) OMNI_FAIL(OMNI_ERR_UNSUPPORTED, "work list: too many heads or tiles");
  const size_t cap = sched_cap(BH, L.N, tile_m);
  const size_t keys_off = sched_keys_off(BH), order_off = sched_order_off(BH, L.N, tile_m);
  hipLaunchKernelGGL(sched_prefix_kernel, dim3(1), dim3(64), 0, st, q_cnt, BH, L.N, tile_m, sched);
  OMNI_LAUNCH_CHECK();
  const int blocks = (int)cdiv(cap, (size_t)256);
  hipLaunchKernelGGL(sched_cost_kernel, dim3(blocks), dim3(256), 0, st, q_cnt, budget, qvis, L.bph, BH, L.Hq, L.N, b_cap, L.causal,
                     tile_m, keys_off, sched);
  OMNI_LAUNCH_CHECK();
  if (queues > 1 && BH <= kSchedMaxQueuedHeads) {
    hipLaunchKernelGGL(sched_assign_kernel, dim3(1), dim3(kAssignThreads), 0, st, BH, queues, keys_off, sched);
    OMNI_LAUNCH_CHECK();
  }
  hipLaunchKernelGGL(sched_rank_kernel, dim3((unsigned)cdiv(cap, (size_t)kRankItems)), dim3(256), 0, st, BH, keys_off, order_off,
                     sched);
  OMNI_LAUNCH_CHECK();
  return OMNI_OK;
}

void sched_build_host(const int* q_cnt, const int* budget, int B, int Hq, int N, int b_cap, int causal, int tile_m,
                      int* sched, int queues) {
  const int BH = B * Hq;
  int items = 0;
  std::vector<int> costs, packed;
  for (int bh = 0; bh < BH; ++bh) {
    const int nq = q_cnt ? q_cnt[bh] : N;
    const int nt = nq > 0 ? (nq + tile_m - 1) / tile_m : 0;
    int nk = budget ? budget[bh / Hq] : N;
    nk = nk < 0 ? 0 : (nk > b_cap ? b_cap : nk);
    sched[kSchedPrefix + bh] = items;
    sched[sched_head_cost_off(BH) + bh] = 0;
    for (int tq = 0; tq < nt; ++tq) {
      costs.push_back(sched_estimate(tq, nt, nk, causal));
      sched[sched_head_cost_off(BH) + bh] += costs.back();
      packed.push_back((int)(((unsigned)bh << 16) | (unsigned)tq));
    }
    items += nt;
  }
  sched[kSchedPrefix + BH] = items;
  sched[kSchedTotal] = items;
  sched_assign_host(sched, BH, queues);
  std::vector<unsigned long long> keys(items);
  for (int id = 0; id < items; ++id)
    keys[id] = sched_key(costs[id], id, (unsigned)sched[sched_head_place_off(BH) + (int)((unsigned)packed[id] >> 16)]);
  std::vector<int> idx(items);
  for (int i = 0; i < items; ++i) idx[i] = i;
  std::sort(idx.begin(), idx.end(), [&](int a, int b) { return keys[a] > keys[b]; });
  const size_t order_off = sched_order_off(BH, N, tile_m);
  for (int k = 0; k < items; ++k) sched[order_off + k] = packed[idx[k]];
}

int persistent_grid() {
  static int grid = 0;
  if (grid == 0) {
    int dev = 0, cus = 0;
    if (hipGetDevice(&dev) != hipSuccess ||
        hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess || cus <= 0)
      cus = 256;
    grid = 2 * cus;
  }
  return grid;
}

}  // namespace omni
