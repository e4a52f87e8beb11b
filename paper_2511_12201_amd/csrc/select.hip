// Selection machinery: k-th largest by radix select over LDS histograms, the
// recall budget search, distribution moments, and ordered stream compaction.
// Serves omni_select_queries (query-mask equation), omni_kv_budget (kurtosis,
// budget equation) and omni_select_kv (key-mask equation).
//
// All decisions are taken on the float32 score arrays through an
// order-preserving map to unsigned keys, so the kept sets are exact functions
// of the input bits.  Sums that decide the budget are accumulated as 64-bit
// fixed point (2^-40 units) with integer atomics: exact, hence independent of
// the order in which lanes arrive.
#include <cmath>
#include <cstring>

#include <algorithm>

#include "common.h"
#include "kernels.h"

namespace omni {

namespace {

constexpr int kSelThreads = 1024;
constexpr int kChunk = kSelectChunk;    // elements per compaction workgroup
constexpr int kChunkThreads = 256;
constexpr int kPerThread = kChunk / kChunkThreads;
constexpr double kFixScale = 1099511627776.0;   // 2^40

__device__ __forceinline__ unsigned long long to_fixed(float a) {
  return a > 0.f ? (unsigned long long)((double)a * kFixScale) : 0ull;
}

constexpr int kRep = 32;     // replicas per histogram bin

struct RadixShared {
  // Every bin is replicated kRep times and a lane updates replica lane % kRep, so the lanes of one
  // LDS atomic never collide on an address (scores cluster in a few exponent bins, which would
  // otherwise serialise 64 ways) and each replica row maps to distinct banks.
  unsigned rcnt[256 * kRep];
  unsigned long long rsum[256 * kRep];
  unsigned cnt[256];
  unsigned long long sum[256];
  unsigned prefix, mask;
  long long remaining;                 // count (select) or fixed-point mass (budget) still to cover
  unsigned long long cnt_above;
  unsigned long long sum_above;
  int done;
};

// One radix pass: histogram (count and fixed-point mass) of the digit at `shift`
// among elements of x[lo,hi) whose key matches (prefix, mask).
__device__ __forceinline__ void radix_histogram(const float* __restrict__ x, int lo, int hi, int shift,
                                                RadixShared& sh, bool with_sum) {
  for (int t = threadIdx.x; t < 256 * kRep; t += blockDim.x) {
    sh.rcnt[t] = 0;
    if (with_sum) sh.rsum[t] = 0;
  }
  __syncthreads();
  const unsigned prefix = sh.prefix, mask = sh.mask;
  const int rep = threadIdx.x & (kRep - 1);
  // kBatch loads are in flight together: one workgroup walks a whole vector, and with one load per
  // trip the pass would cost a memory latency per element
  constexpr int kBatch = 16;
  for (int n0 = lo + threadIdx.x; n0 < hi; n0 += kBatch * blockDim.x) {
    float v[kBatch];
#pragma unroll
    for (int e = 0; e < kBatch; ++e) {
      const int n = n0 + e * blockDim.x;
      v[e] = n < hi ? x[n] : 0.f;
    }
#pragma unroll
    for (int e = 0; e < kBatch; ++e) {
      const unsigned key = float_key(v[e]);
      if (n0 + e * (int)blockDim.x < hi && (key & mask) == prefix) {
        const unsigned d = (key >> shift) & 255u;
        atomicAdd(&sh.rcnt[d * kRep + rep], 1u);
        if (with_sum) atomicAdd(&sh.rsum[d * kRep + rep], to_fixed(v[e]));
      }
    }
  }
  __syncthreads();
  if (threadIdx.x < 256) {
    unsigned c = 0;
    unsigned long long m = 0;
    for (int r = 0; r < kRep; ++r) {
      const int o = threadIdx.x * kRep + ((r + threadIdx.x) & (kRep - 1));   // rotate: spread banks across lanes
      c += sh.rcnt[o];
      if (with_sum) m += sh.rsum[o];
    }
    sh.cnt[threadIdx.x] = c;
    sh.sum[threadIdx.x] = m;
  }
  __syncthreads();
}

// Run by the first wavefront after a histogram pass.  Walks the 256 bins from the top and finds the
// first bin at which the running total (of counts, or of fixed-point mass when by_sum) reaches
// sh.remaining; updates prefix / mask / remaining / cnt_above / sum_above.  Returns false (all lanes)
// when even the whole histogram falls short.  Each lane owns 4 consecutive bins; totals are combined
// with a wavefront prefix scan.
__device__ __forceinline__ bool radix_pick_bin(RadixShared& sh, int shift, bool by_sum) {
  const int lane = threadIdx.x;
  const int base = 255 - 4 * lane;
  unsigned long long c[4], m[4];
#pragma unroll
  for (int j = 0; j < 4; ++j) {
    c[j] = sh.cnt[base - j];
    m[j] = sh.sum[base - j];
  }
  const unsigned long long ctot = c[0] + c[1] + c[2] + c[3], mtot = m[0] + m[1] + m[2] + m[3];
  unsigned long long cs = ctot, ms = mtot;
#pragma unroll
  for (int o = 1; o < 64; o <<= 1) {
    const unsigned long long tc = __shfl_up(cs, o, 64), tm = __shfl_up(ms, o, 64);
    if (lane >= o) {
      cs += tc;
      ms += tm;
    }
  }
  const long long rem = sh.remaining;
  const bool cross = (long long)(by_sum ? ms : cs) >= rem;
  const unsigned long long hit = __ballot(cross);
  if (hit == 0) return false;
  const int leader = __ffsll((long long)hit) - 1;
  if (lane == leader) {
    unsigned long long cb = cs - ctot, mb = ms - mtot;      // totals of the bins above this lane's
    int j = 0;
    for (; j < 3; ++j) {
      if ((long long)((by_sum ? mb + m[j] : cb + c[j])) >= rem) break;
      cb += c[j];
      mb += m[j];
    }
    sh.remaining = rem - (long long)(by_sum ? mb : cb);
    sh.cnt_above += cb;
    sh.sum_above += mb;
    sh.prefix |= (unsigned)(base - j) << shift;
    sh.mask |= 255u << shift;
  }
  return true;
}

// k-th largest element of x[lo,hi): writes its key, the number of elements that
// must be taken among those equal to it, and the fixed-point mass of the k
// largest.  k <= 0 selects nothing, k >= hi-lo selects everything.
__device__ void radix_select_block(const float* __restrict__ x, int lo, int hi, long long k, RadixShared& sh,
                                   unsigned* thr_key, int* need_eq, unsigned long long* mass, bool with_sum) {
  const int n = hi - lo;
  if (k <= 0 || k >= n) {
    unsigned long long total = 0;
    if (with_sum && k >= n) {
      if (threadIdx.x == 0) sh.sum_above = 0;
      __syncthreads();
      unsigned long long local = 0;
      for (int j = lo + threadIdx.x; j < hi; j += blockDim.x) local += to_fixed(x[j]);
      local = wave_sum(local);
      if (lane_id() == 0) atomicAdd(&sh.sum_above, local);
      __syncthreads();
      total = sh.sum_above;
    }
    if (threadIdx.x == 0) {
      *thr_key = k <= 0 ? 0xffffffffu : 0u;
      *need_eq = 0;
      if (mass) *mass = total;
    }
    __syncthreads();
    return;
  }
  if (threadIdx.x == 0) {
    sh.prefix = 0;
    sh.mask = 0;
    sh.remaining = k;
    sh.cnt_above = 0;
    sh.sum_above = 0;
  }
  __syncthreads();
  // The four passes count only: the 64-bit mass atomics are the slow half of a histogram pass, and the mass of the
  // k largest is one plain sweep once the cut is known (fixed point: the order of the additions does not matter).
  for (int pass = 0; pass < 4; ++pass) {
    const int shift = 24 - 8 * pass;
    radix_histogram(x, lo, hi, shift, sh, false);
    if (threadIdx.x < 64) radix_pick_bin(sh, shift, false);     // k <= matching count: always found
    __syncthreads();
  }
  if (with_sum) {
    const unsigned cut = sh.prefix;
    unsigned long long local = 0;
    for (int j = lo + threadIdx.x; j < hi; j += blockDim.x) {
      const float v = x[j];
      if (float_key(v) > cut) local += to_fixed(v);
    }
    local = wave_sum(local);
    if (lane_id() == 0 && local) atomicAdd(&sh.sum_above, local);
    __syncthreads();
  }
  if (threadIdx.x == 0) {
    *thr_key = sh.prefix;
    *need_eq = (int)sh.remaining;
    if (mass) {
      // every element left in the last bin has the same bits: recover its value from the key
      const unsigned key = sh.prefix;
      const unsigned bits = (key & 0x80000000u) ? (key & 0x7fffffffu) : ~key;
      *mass = sh.sum_above + (unsigned long long)sh.remaining * to_fixed(__uint_as_float(bits));
    }
  }
  __syncthreads();
}

// Smallest count b such that the b largest elements of x[0,n) sum to >= target
// (fixed point).  n if the whole vector falls short.
__device__ int radix_budget_block(const float* __restrict__ x, int n, unsigned long long target, RadixShared& sh) {
  if (threadIdx.x == 0) {
    sh.prefix = 0;
    sh.mask = 0;
    sh.remaining = (long long)target;
    sh.cnt_above = 0;
    sh.sum_above = 0;
    sh.done = 0;
  }
  __syncthreads();
  for (int pass = 0; pass < 4; ++pass) {
    const int shift = 24 - 8 * pass;
    if (sh.done) break;                   // uniform: written before the barrier below
    radix_histogram(x, 0, n, shift, sh, true);
    if (threadIdx.x < 64) {
      const bool found = radix_pick_bin(sh, shift, true);
      if (!found && threadIdx.x == 0) sh.done = 1;   // even all matching elements fall short: take everything
    }
    __syncthreads();
  }
  int b;
  if (sh.done) {
    b = n;
  } else {
    const unsigned key = sh.prefix;
    const unsigned bits = (key & 0x80000000u) ? (key & 0x7fffffffu) : ~key;
    const unsigned long long v = to_fixed(__uint_as_float(bits));
    const long long rem = sh.remaining;
    long long j = rem <= 0 ? 0 : (v ? (rem + (long long)v - 1) / (long long)v : 0);
    if (j < 1) j = 1;           // the crossing element itself is always needed
    b = (int)min((long long)n, (long long)sh.cnt_above + j);
  }
  __syncthreads();
  return b;
}

// ------------------------------------------------------------------ kernels

// grid: B*H.  Threshold for "keep the k best of x[lo,hi)".  k from a scalar, or
// min(k_dev[batch], k_cap) when k_dev is given.  skip_head0: head 0 gets the
// keep-everything threshold (the first head's queries are all preserved).
__global__ __launch_bounds__(kSelThreads) void radix_select_kernel(const float* __restrict__ x, int n_stride, int H,
                                                                  int lo, int hi, int k_scalar,
                                                                  const int* __restrict__ k_dev, int k_per_head,
                                                                  int k_cap, int skip_head0, unsigned* __restrict__ thr,
                                                                  int* __restrict__ need, float* __restrict__ recall,
                                                                  float recall_div) {
  __shared__ RadixShared sh;
  const int bh = blockIdx.x;
  const int b = bh / H, h = bh % H;
  if (skip_head0 && h == 0) {
    if (threadIdx.x == 0) {
      thr[bh] = 0u;
      need[bh] = 0;
    }
    return;
  }
  long long k = k_dev ? (long long)min(k_dev[budget_slot(k_per_head, b, bh)], k_cap) : (long long)k_scalar;
  __shared__ unsigned long long mass;
  radix_select_block(x + (long long)bh * n_stride, lo, hi, k, sh, &thr[bh], &need[bh], recall ? &mass : nullptr,
                     recall != nullptr);
  if (recall && threadIdx.x == 0) recall[bh] = (float)((double)mass / kFixScale / (double)recall_div);
}

// grid: (H or 1, B).  Budget of head h (or of the flattest head when per_head == 0).
__global__ __launch_bounds__(kSelThreads) void radix_budget_kernel(const float* __restrict__ a, int N, int ld, int H,
                                                                  const int* __restrict__ flattest, int per_head,
                                                                  double target_mass, int* __restrict__ out) {
  __shared__ RadixShared sh;
  const int b = blockIdx.y;
  const int h = per_head ? (int)blockIdx.x : flattest[b];
  // rounded up: the truncated element masses must never reach a target below the real one
  const unsigned long long target = (unsigned long long)ceil(target_mass * kFixScale);
  const int r = radix_budget_block(a + ((long long)b * H + h) * ld, N, target, sh);
  if (threadIdx.x == 0) out[per_head ? b * H + h : b] = r;
}

__global__ void max_over_heads_kernel(const int* __restrict__ per_head, int H, int* __restrict__ out) {
  const int b = blockIdx.x;
  if (threadIdx.x == 0) {
    int m = 0;
    for (int h = 0; h < H; ++h) m = max(m, per_head[b * H + h]);
    out[b] = m;
  }
}

// grid: B*H.  Excess kurtosis m4/m2^2 - 3 in fp64 with a fixed reduction tree.
__global__ __launch_bounds__(kSelThreads) void kurtosis_kernel(const float* __restrict__ a, int N, int ld,
                                                              double* __restrict__ kurt) {
  __shared__ double red[2][kSelThreads / 64];
  __shared__ double mean_sh;
  const float* x = a + (long long)blockIdx.x * ld;
  const int w = threadIdx.x >> 6;
  double s = 0.0;
#pragma unroll 8
  for (int n = threadIdx.x; n < N; n += kSelThreads) s += (double)x[n];
  s = wave_sum(s);
  if (lane_id() == 0) red[0][w] = s;
  __syncthreads();
  if (threadIdx.x == 0) {
    double t = 0.0;
    for (int i = 0; i < kSelThreads / 64; ++i) t += red[0][i];
    mean_sh = t / (double)N;
  }
  __syncthreads();
  const double mu = mean_sh;
  double s2 = 0.0, s4 = 0.0;
#pragma unroll 8
  for (int n = threadIdx.x; n < N; n += kSelThreads) {
    const double c = (double)x[n] - mu;
    const double c2 = c * c;
    s2 += c2;
    s4 += c2 * c2;
  }
  s2 = wave_sum(s2);
  s4 = wave_sum(s4);
  __syncthreads();
  if (lane_id() == 0) {
    red[0][w] = s2;
    red[1][w] = s4;
  }
  __syncthreads();
  if (threadIdx.x == 0) {
    double t2 = 0.0, t4 = 0.0;
    for (int i = 0; i < kSelThreads / 64; ++i) {
      t2 += red[0][i];
      t4 += red[1][i];
    }
    const double m2 = t2 / (double)N, m4 = t4 / (double)N;
    kurt[blockIdx.x] = m2 > 0.0 ? m4 / (m2 * m2) - 3.0 : -2.0;
  }
}

__global__ void argmin_kernel(const double* __restrict__ kurt, int H, int* __restrict__ flattest) {
  const int b = blockIdx.x;
  if (threadIdx.x == 0) {
    // heads within 1e-9 (relative) of the smallest kurtosis tie and the lowest index wins: for two or
    // three scores the statistic is one constant for every head and rounding would pick the head
    double v = kurt[b * H];
    for (int h = 1; h < H; ++h) v = fmin(v, kurt[b * H + h]);
    const double bar = v + 1e-9 * fabs(v);
    int best = 0;
    while (best < H - 1 && !(kurt[b * H + best] <= bar)) ++best;
    flattest[b] = best;
  }
}

// Membership rule shared by the counting and the writing pass.
struct KeepRule {
  int lo, hi;            // classified region; elements outside are always kept (queries) -- for keys lo=0, hi=N
  int keep_all_head0;    // head 0 keeps everything
  int use_table;         // thresholds from thr/need arrays, else from thr_scalar with need 0
  unsigned thr_scalar;
};

__device__ __forceinline__ void classify(const KeepRule& r, int h, int n, float v, unsigned thr, bool& always,
                                         bool& eq) {
  if ((r.keep_all_head0 && h == 0) || n < r.lo || n >= r.hi) {
    always = true;
    eq = false;
    return;
  }
  const unsigned key = float_key(v);
  always = key > thr;
  eq = key == thr;
}

// grid: (nchunk, B*H).  Per chunk: number of always-kept and of cut-valued elements.
__global__ __launch_bounds__(kChunkThreads) void chunk_count_kernel(const float* __restrict__ x, int N, int ld, int H,
                                                                   KeepRule rule, const unsigned* __restrict__ thr_tab,
                                                                   int nchunk, int* __restrict__ cnt_keep,
                                                                   int* __restrict__ cnt_eq) {
  __shared__ int red[2][kChunkThreads / 64];
  const int bh = blockIdx.y, h = bh % H;
  const unsigned thr = rule.use_table ? thr_tab[bh] : rule.thr_scalar;
  const float* row = x + (long long)bh * ld;
  const int base = blockIdx.x * kChunk + threadIdx.x * kPerThread;
  int ck = 0, ce = 0;
#pragma unroll
  for (int e = 0; e < kPerThread; ++e) {
    const int n = base + e;
    if (n < N) {
      bool al, eq;
      classify(rule, h, n, row[n], thr, al, eq);
      ck += al;
      ce += eq;
    }
  }
  ck = wave_sum(ck);
  ce = wave_sum(ce);
  if (lane_id() == 0) {
    red[0][threadIdx.x >> 6] = ck;
    red[1][threadIdx.x >> 6] = ce;
  }
  __syncthreads();
  if (threadIdx.x == 0) {
    int a = 0, b = 0;
    for (int i = 0; i < kChunkThreads / 64; ++i) {
      a += red[0][i];
      b += red[1][i];
    }
    cnt_keep[(long long)bh * nchunk + blockIdx.x] = a;
    cnt_eq[(long long)bh * nchunk + blockIdx.x] = b;
  }
}

// grid: B*H, one wavefront.  In-place exclusive scan over the chunks; total count out.
__global__ void chunk_scan_kernel(int nchunk, KeepRule rule, const int* __restrict__ need_tab, int* __restrict__ cnt_keep,
                                  int* __restrict__ cnt_eq, int* __restrict__ total_out, int out_cap) {
  const int bh = blockIdx.x;
  int* ck = cnt_keep + (long long)bh * nchunk;
  int* ce = cnt_eq + (long long)bh * nchunk;
  const int lane = threadIdx.x;
  int run_k = 0, run_e = 0;
  for (int c0 = 0; c0 < nchunk; c0 += 64) {
    const int c = c0 + lane;
    const int vk = c < nchunk ? ck[c] : 0;
    const int ve = c < nchunk ? ce[c] : 0;
    int sk = vk, se = ve;
#pragma unroll
    for (int o = 1; o < 64; o <<= 1) {
      const int tk = __shfl_up(sk, o, 64);
      const int te = __shfl_up(se, o, 64);
      if (lane >= o) {
        sk += tk;
        se += te;
      }
    }
    if (c < nchunk) {
      ck[c] = run_k + sk - vk;
      ce[c] = run_e + se - ve;
    }
    run_k += __shfl(sk, 63, 64);
    run_e += __shfl(se, 63, 64);
  }
  if (lane == 0 && total_out) {
    const int need = rule.use_table ? need_tab[bh] : 0;
    total_out[bh] = min(out_cap, run_k + min(run_e, need));
  }
}

// grid: (nchunk, B*H).  Writes the kept indices of the chunk, ascending, at their global rank.
__global__ __launch_bounds__(kChunkThreads) void chunk_write_kernel(const float* __restrict__ x, int N, int ld, int H,
                                                                   KeepRule rule, const unsigned* __restrict__ thr_tab,
                                                                   const int* __restrict__ need_tab, int nchunk,
                                                                   const int* __restrict__ off_keep,
                                                                   const int* __restrict__ off_eq,
                                                                   int* __restrict__ out, int out_stride) {
  __shared__ int wsum[2][kChunkThreads / 64];
  const int bh = blockIdx.y, h = bh % H;
  const unsigned thr = rule.use_table ? thr_tab[bh] : rule.thr_scalar;
  const int need = rule.use_table ? need_tab[bh] : 0;
  const float* row = x + (long long)bh * ld;
  const int base = blockIdx.x * kChunk + threadIdx.x * kPerThread;
  bool al[kPerThread], eq[kPerThread];
  int ck = 0, ce = 0;
#pragma unroll
  for (int e = 0; e < kPerThread; ++e) {
    const int n = base + e;
    al[e] = false;
    eq[e] = false;
    if (n < N) classify(rule, h, n, row[n], thr, al[e], eq[e]);
    ck += al[e];
    ce += eq[e];
  }
  // exclusive scan of (ck, ce) over the workgroup
  const int lane = lane_id(), w = threadIdx.x >> 6;
  int sk = ck, se = ce;
#pragma unroll
  for (int o = 1; o < 64; o <<= 1) {
    const int tk = __shfl_up(sk, o, 64);
    const int te = __shfl_up(se, o, 64);
    if (lane >= o) {
      sk += tk;
      se += te;
    }
  }
  if (lane == 63) {
    wsum[0][w] = sk;
    wsum[1][w] = se;
  }
  __syncthreads();
  int pk = off_keep[(long long)bh * nchunk + blockIdx.x] + sk - ck;
  int pe = off_eq[(long long)bh * nchunk + blockIdx.x] + se - ce;
  for (int i = 0; i < w; ++i) {
    pk += wsum[0][i];
    pe += wsum[1][i];
  }
  int* dst = out + (long long)bh * out_stride;
#pragma unroll
  for (int e = 0; e < kPerThread; ++e) {
    const bool take = al[e] || (eq[e] && pe < need);
    if (take) {
      const int pos = pk + min(pe, need);
      if (pos < out_stride) dst[pos] = base + e;
    }
    pk += al[e];
    pe += eq[e];
  }
}

// grid: B*H.  The sub-range of an ascending index list that lies in [v0, v1).
__global__ void visual_subset_kernel(const int* __restrict__ kv_idx, const int* __restrict__ budget, int bph, int H, int b_cap,
                                     int v0, int v1, int* __restrict__ vis_idx, int* __restrict__ vis_cnt) {
  __shared__ int range[2];
  const int bh = blockIdx.x, b = bh / H;
  const int* src = kv_idx + (long long)bh * b_cap;
  const int n = min(budget[budget_slot(bph, b, bh)], b_cap);
  if (threadIdx.x < 2) {
    const int target = threadIdx.x == 0 ? v0 : v1;      // first position with index >= target
    int lo = 0, hi = n;
    while (lo < hi) {
      const int mid = (lo + hi) >> 1;
      if (src[mid] < target) lo = mid + 1; else hi = mid;
    }
    range[threadIdx.x] = lo;
  }
  __syncthreads();
  const int first = range[0], cnt = range[1] - range[0];
  for (int t = threadIdx.x; t < cnt; t += blockDim.x) vis_idx[(long long)bh * b_cap + t] = src[first + t];
  if (threadIdx.x == 0) vis_cnt[bh] = cnt;
}

int compact(const float* x, int BH, int N, int ld, int H, const KeepRule& rule, const unsigned* thr, const int* need,
            int* cnt_keep, int* cnt_eq, int* out, int out_stride, int* total_out, hipStream_t st) {
  const int nchunk = cdiv(N, kChunk);
  hipLaunchKernelGGL(chunk_count_kernel, dim3(nchunk, BH), dim3(kChunkThreads), 0, st, x, N, ld, H, rule, thr, nchunk,
                     cnt_keep, cnt_eq);
  OMNI_LAUNCH_CHECK();
  hipLaunchKernelGGL(chunk_scan_kernel, dim3(BH), dim3(64), 0, st, nchunk, rule, need, cnt_keep, cnt_eq, total_out,
                     out_stride);
  OMNI_LAUNCH_CHECK();
  hipLaunchKernelGGL(chunk_write_kernel, dim3(nchunk, BH), dim3(kChunkThreads), 0, st, x, N, ld, H, rule, thr, need, nchunk,
                     cnt_keep, cnt_eq, out, out_stride);
  OMNI_LAUNCH_CHECK();
  return OMNI_OK;
}

struct SelWs {
  unsigned* thr;
  int* need;
  int* cnt_keep;
  int* cnt_eq;
};

SelWs carve_select(Arena& a, const Layer& L) {
  SelWs w;
  const size_t BH = (size_t)L.B * L.Hq;
  w.thr = a.take<unsigned>(BH);
  w.need = a.take<int>(BH);
  w.cnt_keep = a.take<int>(BH * cdiv(L.N, kChunk));
  w.cnt_eq = a.take<int>(BH * cdiv(L.N, kChunk));
  return w;
}

}  // namespace

size_t select_ws(const Layer& L) {
  Arena a(nullptr);
  carve_select(a, L);
  return a.used();
}

int run_select_queries(const Layer& L, const float* scores, int mode, float param, int* q_idx, int* q_cnt, void* ws,
                       hipStream_t st) {
  Arena a(ws);
  SelWs w = carve_select(a, L);
  const int BH = L.B * L.Hq;
  KeepRule rule;
  rule.lo = L.v0;
  rule.hi = L.v1;
  rule.keep_all_head0 = 1;
  if (mode == 0) {
    rule.use_table = 0;
    unsigned u;
    std::memcpy(&u, &param, 4);
    rule.thr_scalar = (u & 0x80000000u) ? ~u : (u | 0x80000000u);
  } else {
    rule.use_table = 1;
    rule.thr_scalar = 0;
    const int n_vis = L.v1 - L.v0;
    long long want = (long long)std::ceil((double)param * (double)n_vis);
    if (want < 0) want = 0;
    if (want > n_vis) want = n_vis;
    hipLaunchKernelGGL(radix_select_kernel, dim3(BH), dim3(kSelThreads), 0, st, scores, L.ld, L.Hq, L.v0, L.v1,
                       (int)want, (const int*)nullptr, 0, 0, 1, w.thr, w.need, (float*)nullptr, 1.f);
    OMNI_LAUNCH_CHECK();
  }
  return compact(scores, BH, L.N, L.ld, L.Hq, rule, w.thr, w.need, w.cnt_keep, w.cnt_eq, q_idx, L.ld, q_cnt, st);
}

int run_select_kv(const Layer& L, const float* key_scores, const int* budget, int b_cap, int* kv_idx, void* ws,
                  hipStream_t st) {
  Arena a(ws);
  SelWs w = carve_select(a, L);
  const int BH = L.B * L.Hq;
  hipLaunchKernelGGL(radix_select_kernel, dim3(BH), dim3(kSelThreads), 0, st, key_scores, L.ld, L.Hq, 0, L.N, 0, budget,
                     L.bph, b_cap, 0, w.thr, w.need, (float*)nullptr, 1.f);
  OMNI_LAUNCH_CHECK();
  KeepRule rule;
  rule.lo = 0;
  rule.hi = L.N;
  rule.keep_all_head0 = 0;
  rule.use_table = 1;
  rule.thr_scalar = 0;
  return compact(key_scores, BH, L.N, L.ld, L.Hq, rule, w.thr, w.need, w.cnt_keep, w.cnt_eq, kv_idx, b_cap, nullptr, st);
}

size_t budget_stats_ws(const Layer& L) {
  Arena a(nullptr);
  const size_t BH = (size_t)L.B * L.Hq;
  a.take<unsigned>(BH);
  a.take<int>(BH);
  a.take<int>(BH);
  return a.used();
}

int run_budget_stats(const Layer& L, const float* key_scores, float recall_p, int budget_mode, double* kurt,
                     int* flattest, int* budget, float* recall, void* ws, hipStream_t st, int k_cap) {
  Arena a(ws);
  const int BH = L.B * L.Hq;
  unsigned* thr = a.take<unsigned>(BH);
  int* need = a.take<int>(BH);
  int* per_head = a.take<int>(BH);
  hipLaunchKernelGGL(kurtosis_kernel, dim3(BH), dim3(kSelThreads), 0, st, key_scores, L.N, L.ld, kurt);
  OMNI_LAUNCH_CHECK();
  hipLaunchKernelGGL(argmin_kernel, dim3(L.B), dim3(64), 0, st, kurt, L.Hq, flattest);
  OMNI_LAUNCH_CHECK();
  const double target = (double)recall_p * (double)L.N;
  if (budget_mode == 2) {                      // every head its own budget, written straight to budget[B,Hq]
    hipLaunchKernelGGL(radix_budget_kernel, dim3(L.Hq, L.B), dim3(kSelThreads), 0, st, key_scores, L.N, L.ld, L.Hq, flattest,
                       1, target, budget);
    OMNI_LAUNCH_CHECK();
  } else if (budget_mode == 0) {
    hipLaunchKernelGGL(radix_budget_kernel, dim3(1, L.B), dim3(kSelThreads), 0, st, key_scores, L.N, L.ld, L.Hq, flattest, 0,
                       target, budget);
    OMNI_LAUNCH_CHECK();
  } else {
    hipLaunchKernelGGL(radix_budget_kernel, dim3(L.Hq, L.B), dim3(kSelThreads), 0, st, key_scores, L.N, L.ld, L.Hq, flattest,
                       1, target, per_head);
    OMNI_LAUNCH_CHECK();
    hipLaunchKernelGGL(max_over_heads_kernel, dim3(L.B), dim3(64), 0, st, per_head, L.Hq, budget);
    OMNI_LAUNCH_CHECK();
  }
  hipLaunchKernelGGL(radix_select_kernel, dim3(BH), dim3(kSelThreads), 0, st, key_scores, L.ld, L.Hq, 0, L.N, 0, budget,
                     budget_mode == 2 ? 1 : 0, std::min(k_cap, L.N), 0, thr, need, recall, (float)L.N);
  OMNI_LAUNCH_CHECK();
  return OMNI_OK;
}

// Key selection from the thresholds that run_budget_stats left in its workspace (the recall pass finds, per
// head, the k-th largest score for k = min(budget, k_cap): the cut of the key-mask equation for that budget).
int run_select_kv_from_stats(const Layer& L, const float* key_scores, void* stats_ws, int b_cap, int* kv_idx,
                             void* ws, hipStream_t st) {
  Arena sa(stats_ws);
  const int BH = L.B * L.Hq;
  const unsigned* thr = sa.take<unsigned>(BH);
  const int* need = sa.take<int>(BH);
  Arena a(ws);
  SelWs w = carve_select(a, L);
  KeepRule rule;
  rule.lo = 0;
  rule.hi = L.N;
  rule.keep_all_head0 = 0;
  rule.use_table = 1;
  rule.thr_scalar = 0;
  return compact(key_scores, BH, L.N, L.ld, L.Hq, rule, thr, need, w.cnt_keep, w.cnt_eq, kv_idx, b_cap, nullptr, st);
}

int run_select_kv_counts(const Layer& L, const float* key_scores, void* stats_ws, int b_cap, int* kv_idx, void* ws,
                         SelectSource* src, hipStream_t st) {
  Arena sa(stats_ws);
  const int BH = L.B * L.Hq;
  const unsigned* thr = sa.take<unsigned>(BH);
  const int* need = sa.take<int>(BH);
  Arena a(ws);
  SelWs w = carve_select(a, L);
  KeepRule rule;
  rule.lo = 0;
  rule.hi = L.N;
  rule.keep_all_head0 = 0;
  rule.use_table = 1;
  rule.thr_scalar = 0;
  const int nchunk = cdiv(L.N, kChunk);
  hipLaunchKernelGGL(chunk_count_kernel, dim3(nchunk, BH), dim3(kChunkThreads), 0, st, key_scores, L.N, L.ld, L.Hq, rule,
                     thr, nchunk, w.cnt_keep, w.cnt_eq);
  OMNI_LAUNCH_CHECK();
  hipLaunchKernelGGL(chunk_scan_kernel, dim3(BH), dim3(64), 0, st, nchunk, rule, need, w.cnt_keep, w.cnt_eq,
                     (int*)nullptr, b_cap);
  OMNI_LAUNCH_CHECK();
  src->x = key_scores;
  src->ld = L.ld;
  src->nchunk = nchunk;
  src->thr = thr;
  src->need = need;
  src->off_keep = w.cnt_keep;
  src->off_eq = w.cnt_eq;
  src->out = kv_idx;
  src->out_stride = b_cap;
  return OMNI_OK;
}

// ---- union of the stored visual rows over the heads of a KV group, with a membership bit per head
// (paper Sec. "KV Cache Slimming": per-head token-level storage; under grouped-query attention the heads
// of a group index one shared cache, so the group's union is what a decode step can touch at all)

__global__ void fill_u32_kernel(unsigned* p, long long n, unsigned v) {
  const long long stride = (long long)gridDim.x * blockDim.x;
  for (long long i = (long long)blockIdx.x * blockDim.x + threadIdx.x; i < n; i += stride) p[i] = v;
}

// grid: (cdiv(b_cap, 256), B*Hq)
__global__ void group_mark_kernel(const int* __restrict__ kv_idx, const int* __restrict__ budget, int bph, int Hq, int Hkv, int b_cap,
                                  int v0, int v1, unsigned* __restrict__ umask) {
  const int bh = blockIdx.y, b = bh / Hq, i = bh % Hq, G = Hq / Hkv, g = i / G;
  const int n = min(budget[budget_slot(bph, b, bh)], b_cap);
  const int t = blockIdx.x * blockDim.x + threadIdx.x;
  if (t >= n) return;
  const int tok = kv_idx[(long long)bh * b_cap + t];
  if (tok < v0 || tok >= v1) return;
  atomicOr(&umask[(long long)(b * Hkv + g) * (v1 - v0) + (tok - v0)], 1u << (i % G));
}

// grid: B*Hkv, 1024 threads.  Ordered compaction of the marked tokens.
__global__ __launch_bounds__(1024) void group_compact_kernel(const unsigned* __restrict__ umask, int nv, int v0, int u_cap,
                                                             int* __restrict__ grp_idx, unsigned* __restrict__ grp_mask,
                                                             int* __restrict__ grp_cnt) {
  __shared__ int wave_cnt[16];
  __shared__ int base;
  const int bg = blockIdx.x;
  const unsigned* src = umask + (long long)bg * nv;
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  if (threadIdx.x == 0) base = 0;
  __syncthreads();
  for (int c0 = 0; c0 < nv; c0 += 1024) {
    const int t = c0 + threadIdx.x;
    const unsigned m = t < nv ? src[t] : 0u;
    const unsigned long long bal = __ballot(m != 0u);
    if (lane == 0) wave_cnt[wave] = __popcll(bal);
    __syncthreads();
    int off = base;
    for (int w = 0; w < wave; ++w) off += wave_cnt[w];
    off += __popcll(bal & ((1ull << lane) - 1ull));
    if (m != 0u && off < u_cap) {
      grp_idx[(long long)bg * u_cap + off] = v0 + t;
      grp_mask[(long long)bg * u_cap + off] = m;
    }
    __syncthreads();
    if (threadIdx.x == 0) {
      int tot = 0;
      for (int w = 0; w < 16; ++w) tot += wave_cnt[w];
      base += tot;
    }
    __syncthreads();
  }
  if (threadIdx.x == 0) grp_cnt[bg] = base;
}

size_t group_subset_ws(const Layer& L) {
  Arena a(nullptr);
  a.take<unsigned>((size_t)L.B * L.Hkv * (L.v1 - L.v0));
  return a.used();
}

int run_group_subset(const Layer& L, const int* kv_idx, const int* budget, int b_cap, int* grp_idx, unsigned* grp_mask,
                     int* grp_cnt, int u_cap, void* ws, hipStream_t st) {
  Arena a(ws);
  const int nv = L.v1 - L.v0;
  const long long n = (long long)L.B * L.Hkv * nv;
  unsigned* umask = a.take<unsigned>((size_t)n);
  hipLaunchKernelGGL(fill_u32_kernel, dim3((unsigned)std::min<long long>(cdiv(n, 256LL), 4096)), dim3(256), 0, st, umask, n,
                     0u);
  OMNI_LAUNCH_CHECK();
  hipLaunchKernelGGL(group_mark_kernel, dim3(cdiv(b_cap, 256), L.B * L.Hq), dim3(256), 0, st, kv_idx, budget, L.bph, L.Hq, L.Hkv,
                     b_cap, L.v0, L.v1, umask);
  OMNI_LAUNCH_CHECK();
  hipLaunchKernelGGL(group_compact_kernel, dim3(L.B * L.Hkv), dim3(1024), 0, st, umask, nv, L.v0, u_cap, grp_idx, grp_mask,
                     grp_cnt);
  OMNI_LAUNCH_CHECK();
  return OMNI_OK;
}

int run_visual_subset(const Layer& L, const int* kv_idx, const int* budget, int b_cap, int* vis_idx, int* vis_cnt,
                      hipStream_t st) {
  hipLaunchKernelGGL(visual_subset_kernel, dim3(L.B * L.Hq), dim3(256), 0, st, kv_idx, budget, L.bph, L.Hq, b_cap, L.v0, L.v1,
                     vis_idx, vis_cnt);
  OMNI_LAUNCH_CHECK();
  return OMNI_OK;
}

}  // namespace omni
