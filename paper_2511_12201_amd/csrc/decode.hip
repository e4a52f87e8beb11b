// Decode step with KV cache slimming (paper Sec. "KV Cache Slimming",
// decoding-attention equation) and the plain decode baseline.
//
// HBM-bound: one query row per head, so no matrix cores.  The row list of a head
// (its stored visual rows if the decoding query is active, then every
// non-visual row below ctx_len) is split over `nsplit` workgroups; a cache row
// is read by D*sizeof(T)/16 lanes with one 16-byte load each for K and for V.
// Every lane group keeps an online-softmax state; groups, then splits, are
// merged with the usual (max, sum, weighted output) rule in a fixed order.
#include "common.h"
#include "kernels.h"

namespace omni {

namespace {

constexpr int kThreads = 256;
constexpr float kLog2e = 1.4426950408889634f;

struct DecodeParams {
  const void* q;
  const void* K;
  const void* V;
  const int* ctx_len;
  const float* probe;      // nullptr: plain decode (every head attends every row)
  const int* vis_idx;
  const int* vis_cnt;
  int b_cap;
  void* O;
  unsigned char* active;
  float* part;             // [B*Hq, nsplit, D + 2]
  int B, Hq, Hkv, G, D, cap, v0, v1, nsplit;
  float scale, tau;
  long long ks[3];
};

template <typename T, int D>
__global__ __launch_bounds__(kThreads) void decode_partial_kernel(DecodeParams p) {
  constexpr int E = Elem<T>::kPer16B;
  constexpr int LPR = D / E;
  constexpr int RPP = kThreads / LPR;
  __shared__ float sM[RPP], sL[RPP];
  __shared__ float sO[RPP][D];
  __shared__ int sActive;
  const int split = blockIdx.x, bh = blockIdx.y;
  const int b = bh / p.Hq, i = bh % p.Hq, g = i / p.G;
  const int c = threadIdx.x % LPR, grp = threadIdx.x / LPR;
  const T* qptr = static_cast<const T*>(p.q) + (long long)bh * D;
  float qv[E];
  {
    u32x4 raw = *reinterpret_cast<const u32x4*>(qptr + c * E);
    unpack16(raw, qv, (const T*)nullptr);
  }
  // lazy/active classification of the decoding query (every workgroup of the head repeats it)
  int act = 1;
  if (p.probe) {
    if (threadIdx.x < 64) {
      const float* pk = p.probe + ((long long)(b * p.Hkv + g) * 2) * D;
      float dot = 0.f;
      for (int d = threadIdx.x; d < D; d += 64) dot = fmaf(Elem<T>::load(qptr + d), pk[D + d] - pk[d], dot);
      dot = wave_sum(dot);
      if (threadIdx.x == 0) {
        const float score = 1.0f / (1.0f + expf(-dot * p.scale));
        sActive = (i == 0 || score > p.tau) ? 1 : 0;
      }
    }
    __syncthreads();
    act = sActive;
    if (split == 0 && threadIdx.x == 0 && p.active) p.active[bh] = (unsigned char)act;
  }
  const int ctx = min(p.ctx_len[b], p.cap);
  const int n_vis = (p.probe && act) ? min(p.vis_cnt[bh], p.b_cap) : 0;
  const int n_lo = p.probe ? min(p.v0, ctx) : ctx;
  const int hi0 = min(p.v1, ctx);
  const int n_hi = p.probe ? ctx - hi0 : 0;
  const int total = n_vis + n_lo + n_hi;
  int per = cdiv(total, p.nsplit);
  per = cdiv(per, RPP) * RPP;
  const int begin = split * per, end = min(total, begin + per);
  const int* vlist = p.vis_idx ? p.vis_idx + (long long)bh * p.b_cap : nullptr;
  const T* kbase = static_cast<const T*>(p.K) + b * p.ks[0] + g * p.ks[1];
  const T* vbase = static_cast<const T*>(p.V) + b * p.ks[0] + g * p.ks[1];
  const float c2 = p.scale * kLog2e;

  float m = -INFINITY, l = 0.f, acc[E];
#pragma unroll
  for (int e = 0; e < E; ++e) acc[e] = 0.f;
  for (int it0 = begin; it0 < end; it0 += RPP) {     // uniform trip count over the workgroup
    const int it = it0 + grp;
    int row = -1;
    if (it < end) {
      if (it < n_vis) {
        row = vlist[it];
        if (row >= ctx) row = -1;                       // stored rows beyond the context are ignored
      } else if (it < n_vis + n_lo) {
        row = it - n_vis;
      } else {
        row = hi0 + (it - n_vis - n_lo);
      }
    }
    float dot = 0.f;
    u32x4 vraw = {0u, 0u, 0u, 0u};
    if (row >= 0) {
      const u32x4 kraw = *reinterpret_cast<const u32x4*>(kbase + (long long)row * p.ks[2] + c * E);
      vraw = *reinterpret_cast<const u32x4*>(vbase + (long long)row * p.ks[2] + c * E);
      float kv[E];
      unpack16(kraw, kv, (const T*)nullptr);
#pragma unroll
      for (int e = 0; e < E; ++e) dot = fmaf(qv[e], kv[e], dot);
    }
#pragma unroll
    for (int o = LPR / 2; o > 0; o >>= 1) dot += __shfl_xor(dot, o, 64);
    if (row >= 0) {
      const float s2 = dot * c2;
      const float m_new = fmaxf(m, s2);
      const float alpha = exp2f(m - m_new);          // m = -inf -> 0
      const float pw = exp2f(s2 - m_new);
      float vv[E];
      unpack16(vraw, vv, (const T*)nullptr);
      l = l * alpha + pw;
#pragma unroll
      for (int e = 0; e < E; ++e) acc[e] = fmaf(acc[e], alpha, pw * vv[e]);
      m = m_new;
    }
  }
  // merge the lane groups of the workgroup in group order
  if (c == 0) {
    sM[grp] = m;
    sL[grp] = l;
  }
#pragma unroll
  for (int e = 0; e < E; ++e) sO[grp][c * E + e] = acc[e];
  __syncthreads();
  if (threadIdx.x < D) {
    float M = -INFINITY;
    for (int r = 0; r < RPP; ++r) M = fmaxf(M, sM[r]);
    const float Mr = M == -INFINITY ? 0.f : M;
    float Ls = 0.f, Os = 0.f;
    for (int r = 0; r < RPP; ++r) {
      const float w = sM[r] == -INFINITY ? 0.f : exp2f(sM[r] - Mr);
      Ls = fmaf(sL[r], w, Ls);
      Os = fmaf(sO[r][threadIdx.x], w, Os);
    }
    float* dst = p.part + ((long long)bh * p.nsplit + split) * (D + 2);
    dst[threadIdx.x] = Os;
    if (threadIdx.x == 0) {
      dst[D] = M;
      dst[D + 1] = Ls;
    }
  }
}

template <typename T, int D>
__global__ void decode_combine_kernel(DecodeParams p) {
  const int bh = blockIdx.x, d = threadIdx.x;
  if (d >= D) return;
  const float* src = p.part + (long long)bh * p.nsplit * (D + 2);
  float M = -INFINITY;
  for (int s = 0; s < p.nsplit; ++s) M = fmaxf(M, src[s * (D + 2) + D]);
  const float Mr = M == -INFINITY ? 0.f : M;
  float Ls = 0.f, Os = 0.f;
  for (int s = 0; s < p.nsplit; ++s) {
    const float ms = src[s * (D + 2) + D];
    const float w = ms == -INFINITY ? 0.f : exp2f(ms - Mr);
    Ls = fmaf(src[s * (D + 2) + D + 1], w, Ls);
    Os = fmaf(src[s * (D + 2) + d], w, Os);
  }
  Elem<T>::store(static_cast<T*>(p.O) + (long long)bh * D + d, Ls > 0.f ? Os / Ls : 0.f);
}

template <typename T, int D>
int launch_decode(const DecodeParams& p, hipStream_t st) {
  {
    ProfScope prof__(kProfDecode, st);
    hipLaunchKernelGGL((decode_partial_kernel<T, D>), dim3(p.nsplit, p.B * p.Hq), dim3(kThreads), 0, st, p);
    OMNI_LAUNCH_CHECK();
  }
  hipLaunchKernelGGL((decode_combine_kernel<T, D>), dim3(p.B * p.Hq), dim3(128), 0, st, p);
  OMNI_LAUNCH_CHECK();
  return OMNI_OK;
}

}  // namespace

int decode_splits(int batch, int n_q_heads) {
  int s = cdiv(2048, batch * n_q_heads);
  if (s < 1) s = 1;
  if (s > 64) s = 64;
  return s;
}

size_t decode_ws(const omni_decode_desc* d) {
  Arena a(nullptr);
  a.take<float>((size_t)d->batch * d->n_q_heads * decode_splits(d->batch, d->n_q_heads) * (d->head_dim + 2));
  return a.used();
}

int run_decode(const omni_decode_desc* d, const void* q, const void* K, const void* V, const int* ctx_len,
               const float* probe, const int* vis_idx, const int* vis_cnt, int b_cap, void* O,
               unsigned char* active, void* ws, hipStream_t st) {
  Arena a(ws);
  DecodeParams p;
  p.q = q;
  p.K = K;
  p.V = V;
  p.ctx_len = ctx_len;
  p.probe = probe;
  p.vis_idx = vis_idx;
  p.vis_cnt = vis_cnt;
  p.b_cap = b_cap;
  p.O = O;
  p.active = active;
  p.B = d->batch;
  p.Hq = d->n_q_heads;
  p.Hkv = d->n_kv_heads;
  p.G = p.Hq / p.Hkv;
  p.D = d->head_dim;
  p.cap = d->cache_capacity;
  p.v0 = d->vis_begin;
  p.v1 = d->vis_end;
  p.nsplit = decode_splits(p.B, p.Hq);
  p.scale = d->softmax_scale;
  p.tau = d->tau;
  for (int k = 0; k < 3; ++k) p.ks[k] = d->kv_stride[k];
  p.part = a.take<float>((size_t)p.B * p.Hq * p.nsplit * (p.D + 2));
  if (d->dtype == OMNI_BF16) {
    if (p.D == 128) return launch_decode<u16, 128>(p, st);
    return launch_decode<u16, 64>(p, st);
  }
  if (p.D == 128) return launch_decode<float, 128>(p, st);
  return launch_decode<float, 64>(p, st);
}

}  // namespace omni
