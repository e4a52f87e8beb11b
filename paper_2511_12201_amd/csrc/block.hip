// Block-granular variant of the KV selection (paper Sec. "Block-wise probing and sparse flash attention
// kernel", the way the paper runs it): queries AND keys are mean-pooled along the sequence in blocks, the
// pooled attention map gives one accumulated score per key block, the recall budget is a number of
// blocks, and the selected blocks are handed to the attention kernels as token lists.
//
//  * pool_rows_kernel: block means of the rows of one head, fp32 (HBM-bound, one pass over Q and K).
//  * block_scores_kernel: one workgroup per query head.  Thread m owns key block m: for every query block
//    j it computes the pooled logit, the row's softmax over the visible key blocks (a key block of c
//    tokens weighs c), and adds w_j P_j[m] to its own register -- column sums without atomics, in a fixed
//    order.  n_blocks^2 * d MACs per head: a few tens of microseconds at 256 blocks.
//  * expand_blocks_kernel: ascending block ids -> ascending token ids (tokens past the end of the sequence
//    in a partial last block become pad entries, which the packers turn into zero rows nobody sees).
#include "common.h"
#include "kernels.h"

namespace omni {

namespace {

constexpr int kThreads = 256;
constexpr float kLog2e = 1.4426950408889634f;

// grid: (n_blocks, B * H).  X is [B, H, N, D] with element strides sb, sh, sn.
template <typename T, int D>
__global__ __launch_bounds__(kThreads) void pool_rows_kernel(const T* __restrict__ X, long long sb, long long sh,
                                                            long long sn, int H, int N, int block, int nblk,
                                                            float* __restrict__ out) {
  constexpr int E = Elem<T>::kPer16B;
  constexpr int LPR = D / E;
  constexpr int RPP = kThreads / LPR;
  __shared__ float red[RPP][D];
  const int j = blockIdx.x, bh = blockIdx.y;
  const int b = bh / H, i = bh % H;
  const T* base = X + b * sb + i * sh;
  const int c = threadIdx.x % LPR, r0 = threadIdx.x / LPR;
  const int row_begin = j * block, row_end = min(N, row_begin + block);
  float acc[E];
#pragma unroll
  for (int e = 0; e < E; ++e) acc[e] = 0.f;
  for (int r = row_begin + r0; r < row_end; r += RPP) {
    const u32x4 raw = *reinterpret_cast<const u32x4*>(base + (long long)r * sn + c * E);
    float v[E];
    unpack16(raw, v, (const T*)nullptr);
#pragma unroll
    for (int e = 0; e < E; ++e) acc[e] += v[e];
  }
#pragma unroll
  for (int e = 0; e < E; ++e) red[r0][c * E + e] = acc[e];
  __syncthreads();
  if (threadIdx.x < D) {
    float s = 0.f;
    for (int r = 0; r < RPP; ++r) s += red[r][threadIdx.x];
    out[((long long)bh * nblk + j) * D + threadIdx.x] = s / (float)(row_end - row_begin);
  }
}

// grid: B * Hq, kThreads threads; thread t owns the key blocks t, t + kThreads, ... (kMaxOwn of them at most)
constexpr int kMaxOwn = 8;

template <int D>
__global__ __launch_bounds__(kThreads) void block_scores_kernel(const float* __restrict__ qbar, const float* __restrict__ kbar,
                                                               int Hq, int Hkv, int N, int block, int nblk, int causal,
                                                               float scale, float* __restrict__ out) {
  __shared__ float sq[D];
  __shared__ float sred[kThreads / 64];
  __shared__ float sbc;
  const int bh = blockIdx.x, b = bh / Hq, i = bh % Hq, g = i / (Hq / Hkv);
  const float* qh = qbar + (long long)bh * nblk * D;
  const float* kh = kbar + (long long)(b * Hkv + g) * nblk * D;
  const float c2 = scale * kLog2e;
  float acc[kMaxOwn];
#pragma unroll
  for (int o = 0; o < kMaxOwn; ++o) acc[o] = 0.f;
  auto block_reduce = [&](float v, bool is_max) {
    v = is_max ? wave_max(v) : wave_sum(v);
    __syncthreads();
    if ((threadIdx.x & 63) == 0) sred[threadIdx.x >> 6] = v;
    __syncthreads();
    if (threadIdx.x == 0) {
      float r = sred[0];
      for (int w = 1; w < kThreads / 64; ++w) r = is_max ? fmaxf(r, sred[w]) : r + sred[w];
      sbc = r;
    }
    __syncthreads();
    return sbc;
  };
  for (int j = 0; j < nblk; ++j) {
    __syncthreads();
    for (int d = threadIdx.x; d < D; d += kThreads) sq[d] = qh[(long long)j * D + d];
    __syncthreads();
    const int last = causal ? j : nblk - 1;                  // visible key blocks: 0 .. last
    float l[kMaxOwn], mx = -INFINITY;
#pragma unroll
    for (int o = 0; o < kMaxOwn; ++o) {
      const int m = threadIdx.x + o * kThreads;
      l[o] = -INFINITY;
      if (m <= last) {
        const float* kr = kh + (long long)m * D;
        float dot = 0.f;
#pragma unroll 8
        for (int d = 0; d < D; d += 4) {
          const f32x4 kv = *reinterpret_cast<const f32x4*>(kr + d);
          dot = fmaf(sq[d], kv[0], dot);
          dot = fmaf(sq[d + 1], kv[1], dot);
          dot = fmaf(sq[d + 2], kv[2], dot);
          dot = fmaf(sq[d + 3], kv[3], dot);
        }
        l[o] = dot * c2;
        mx = fmaxf(mx, l[o]);
      }
    }
    mx = block_reduce(mx, true);
    float pw[kMaxOwn], sum = 0.f;
#pragma unroll
    for (int o = 0; o < kMaxOwn; ++o) {
      const int m = threadIdx.x + o * kThreads;
      const float cm = (float)(min(N, (m + 1) * block) - m * block);      // tokens in key block m
      pw[o] = m <= last ? cm * exp2f(l[o] - mx) : 0.f;
      sum += pw[o];
    }
    sum = block_reduce(sum, false);
    const float wj = (float)(min(N, (j + 1) * block) - j * block) / sum;   // queries in block j over the row's normaliser
#pragma unroll
    for (int o = 0; o < kMaxOwn; ++o) acc[o] = fmaf(wj, pw[o], acc[o]);
  }
  const float norm = (float)nblk / (float)N;                              // scores sum to the number of blocks
#pragma unroll
  for (int o = 0; o < kMaxOwn; ++o) {
    const int m = threadIdx.x + o * kThreads;
    if (m < nblk) out[(long long)bh * nblk + m] = acc[o] * norm;
  }
}

// grid: (cdiv(blk_cap * block, 256), B * Hq)
__global__ __launch_bounds__(256) void expand_blocks_kernel(const int* __restrict__ blk_idx, const int* __restrict__ blk_budget,
                                                            int Hq, int blk_cap, int block, int N, int b_cap,
                                                            int* __restrict__ kv_idx, int* __restrict__ budget) {
  const int bh = blockIdx.y, b = bh / Hq;
  const int nb = min(blk_budget[b], blk_cap);
  const int t = blockIdx.x * blockDim.x + threadIdx.x;
  if (bh % Hq == 0 && t == 0) budget[b] = min(nb * block, b_cap);
  if (t >= nb * block || t >= b_cap) return;
  const int tok = blk_idx[(long long)bh * blk_cap + t / block] * block + t % block;
  kv_idx[(long long)bh * b_cap + t] = tok < N ? tok : kPadKeyIndex;
}

struct BlockWs {
  float* qbar;
  float* kbar;
};

BlockWs carve_block(Arena& a, const Layer& L, int nblk) {
  BlockWs w;
  w.qbar = a.take<float>((size_t)L.B * L.Hq * nblk * L.D);
  w.kbar = a.take<float>((size_t)L.B * L.Hkv * nblk * L.D);
  return w;
}

template <typename T, int D>
int launch_block_scores(const Layer& L, const void* Q, const void* K, int block, float* out, void* ws, hipStream_t st) {
  const int nblk = cdiv(L.N, block);
  Arena a(ws);
  BlockWs w = carve_block(a, L, nblk);
  hipLaunchKernelGGL((pool_rows_kernel<T, D>), dim3(nblk, L.B * L.Hq), dim3(kThreads), 0, st, static_cast<const T*>(Q),
                     L.qs[0], L.qs[1], L.qs[2], L.Hq, L.N, block, nblk, w.qbar);
  OMNI_LAUNCH_CHECK();
  hipLaunchKernelGGL((pool_rows_kernel<T, D>), dim3(nblk, L.B * L.Hkv), dim3(kThreads), 0, st, static_cast<const T*>(K),
                     L.ks[0], L.ks[1], L.ks[2], L.Hkv, L.N, block, nblk, w.kbar);
  OMNI_LAUNCH_CHECK();
  hipLaunchKernelGGL((block_scores_kernel<D>), dim3(L.B * L.Hq), dim3(kThreads), 0, st, w.qbar, w.kbar, L.Hq, L.Hkv, L.N,
                     block, nblk, L.causal, L.scale, out);
  OMNI_LAUNCH_CHECK();
  return OMNI_OK;
}

}  // namespace

int block_scores_max_blocks() { return kThreads * kMaxOwn; }

size_t block_scores_ws(const Layer& L, int block) {
  Arena a(nullptr);
  carve_block(a, L, cdiv(L.N, block));
  return a.used();
}

int run_block_scores(const Layer& L, int dtype, const void* Q, const void* K, int block, float* out, void* ws,
                     hipStream_t st) {
  if (dtype == OMNI_BF16) {
    if (L.D == 128) return launch_block_scores<u16, 128>(L, Q, K, block, out, ws, st);
    return launch_block_scores<u16, 64>(L, Q, K, block, out, ws, st);
  }
  if (L.D == 128) return launch_block_scores<float, 128>(L, Q, K, block, out, ws, st);
  return launch_block_scores<float, 64>(L, Q, K, block, out, ws, st);
}

int run_expand_blocks(const Layer& L, const int* blk_idx, const int* blk_budget, int blk_cap, int block, int* kv_idx,
                      int* budget, int b_cap, hipStream_t st) {
  hipLaunchKernelGGL(expand_blocks_kernel, dim3(cdiv((long long)blk_cap * block, 256LL), L.B * L.Hq), dim3(256), 0, st,
                     blk_idx, blk_budget, L.Hq, blk_cap, block, L.N, b_cap, kv_idx, budget);
  OMNI_LAUNCH_CHECK();
  return OMNI_OK;
}

}  // namespace omni
