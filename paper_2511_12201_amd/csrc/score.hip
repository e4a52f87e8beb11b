// Probe keys and lazy/active query scores (paper Sec. "Query Selection as Binary
// Lazy-Active Classification", probe-softmax equation).
//
// HBM-bound streaming kernels: every K row of the visual range is read once for
// the mean key, every Q row once for the score.  A row is split over
// D*sizeof(T)/16 lanes with one 16-byte load per lane, so a wavefront reads
// whole contiguous rows.
#include "common.h"
#include "kernels.h"

namespace omni {

namespace {

constexpr int kThreads = 256;
constexpr int kMeanRowsPerChunk = 256;     // ~1000 workgroups at 64k: enough to fill the memory system

template <typename T, int D>
__global__ __launch_bounds__(kThreads) void mean_key_partial_kernel(const T* __restrict__ K, Layer L, int nchunk,
                                                                   float* __restrict__ partial) {
  constexpr int E = Elem<T>::kPer16B;
  constexpr int LPR = D / E;              // lanes per row
  constexpr int RPP = kThreads / LPR;     // rows per pass
  __shared__ float red[RPP][D];
  const int chunk = blockIdx.x;
  const int bg = blockIdx.y;
  const int b = bg / L.Hkv, g = bg % L.Hkv;
  const T* base = K + b * L.ks[0] + g * L.ks[1];
  const int c = threadIdx.x % LPR, r0 = threadIdx.x / LPR;
  const int row_begin = L.v0 + chunk * kMeanRowsPerChunk;
  const int row_end = min(L.v1, row_begin + kMeanRowsPerChunk);
  float acc[E];
#pragma unroll
  for (int e = 0; e < E; ++e) acc[e] = 0.f;
  for (int r = row_begin + r0; r < row_end; r += RPP) {
    u32x4 raw = *reinterpret_cast<const u32x4*>(base + (long long)r * L.ks[2] + c * E);
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
#pragma unroll 4
    for (int r = 0; r < RPP; ++r) s += red[r][threadIdx.x];
    partial[((long long)bg * nchunk + chunk) * D + threadIdx.x] = s;
  }
}

constexpr int kFinalSplit = 8;

template <typename T, int D>
__global__ void probe_keys_finalize_kernel(const T* __restrict__ K, Layer L, int nchunk,
                                           const float* __restrict__ partial, float* __restrict__ probe) {
  const int bg = blockIdx.x;
  const int b = bg / L.Hkv, g = bg % L.Hkv;
  // blockDim.x = kFinalSplit * D: kFinalSplit interleaved partial sums per element, added in a fixed order
  __shared__ float part[kFinalSplit][128];
  const int t = threadIdx.x % D, k = threadIdx.x / D;
  float s = 0.f;
#pragma unroll 4
  for (int c = k; c < nchunk; c += kFinalSplit) s += partial[((long long)bg * nchunk + c) * D + t];
  part[k][t] = s;
  __syncthreads();
  if (k != 0) return;
  s = 0.f;
#pragma unroll
  for (int j = 0; j < kFinalSplit; ++j) s += part[j][t];
  const T* sink = K + b * L.ks[0] + g * L.ks[1] + (long long)L.sink * L.ks[2];
  probe[((long long)bg * 2 + 0) * D + t] = Elem<T>::load(sink + t);
  probe[((long long)bg * 2 + 1) * D + t] = s / (float)(L.v1 - L.v0);
}

// score = softmax([q.k_lazy, q.k_act] * scale)[1] = 1 / (1 + exp(-(q.(k_act - k_lazy)) * scale))
template <typename T, int D>
__global__ __launch_bounds__(kThreads) void score_queries_kernel(const T* __restrict__ Q, Layer L,
                                                                const float* __restrict__ probe,
                                                                float* __restrict__ scores, int rows_per_block) {
  constexpr int E = Elem<T>::kPer16B;
  constexpr int LPR = D / E;
  constexpr int RPP = kThreads / LPR;
  const int bh = blockIdx.y;
  const int b = bh / L.Hq, i = bh % L.Hq;
  const int g = i / L.G;
  const int c = threadIdx.x % LPR, r0 = threadIdx.x / LPR;
  const float* pk = probe + ((long long)(b * L.Hkv + g) * 2) * D;
  float diff[E];
#pragma unroll
  for (int e = 0; e < E; ++e) diff[e] = pk[D + c * E + e] - pk[c * E + e];
  const T* base = Q + b * L.qs[0] + i * L.qs[1];
  float* out = scores + (long long)bh * L.ld;
  const int row_begin = blockIdx.x * rows_per_block;
  const int row_end = min(L.N, row_begin + rows_per_block);
  for (int rb = row_begin; rb < row_end; rb += RPP) {      // uniform trip count: shuffles need every lane
    const int r = rb + r0;
    const bool live = r < row_end;
    float dot = 0.f;
    if (live) {
      u32x4 raw = *reinterpret_cast<const u32x4*>(base + (long long)r * L.qs[2] + c * E);
      float v[E];
      unpack16(raw, v, (const T*)nullptr);
#pragma unroll
      for (int e = 0; e < E; ++e) dot = fmaf(v[e], diff[e], dot);
    }
#pragma unroll
    for (int o = LPR / 2; o > 0; o >>= 1) dot += __shfl_xor(dot, o, 64);
    if (live && c == 0) out[r] = 1.0f / (1.0f + expf(-dot * L.scale));
  }
}

template <typename T, int D>
int launch_probe_keys(const Layer& L, const void* K, float* probe, float* partial, int nchunk, hipStream_t st) {
  const T* k = static_cast<const T*>(K);
  hipLaunchKernelGGL((mean_key_partial_kernel<T, D>), dim3(nchunk, L.B * L.Hkv), dim3(kThreads), 0, st, k, L, nchunk,
                     partial);
  OMNI_LAUNCH_CHECK();
  hipLaunchKernelGGL((probe_keys_finalize_kernel<T, D>), dim3(L.B * L.Hkv), dim3(kFinalSplit * D), 0, st, k, L, nchunk, partial,
                     probe);
  OMNI_LAUNCH_CHECK();
  return OMNI_OK;
}

template <typename T, int D>
int launch_score(const Layer& L, const void* Q, const void* K, float* probe, float* scores, float* partial,
                 int nchunk, hipStream_t st) {
  const T* q = static_cast<const T*>(Q);
  const int rc = launch_probe_keys<T, D>(L, K, probe, partial, nchunk, st);
  if (rc != OMNI_OK) return rc;
  const int rows_per_block = 256;
  {
    ProfScope prof__(kProfScore, st);
    hipLaunchKernelGGL((score_queries_kernel<T, D>), dim3(cdiv(L.N, rows_per_block), L.B * L.Hq), dim3(kThreads), 0, st,
                       q, L, probe, scores, rows_per_block);
    OMNI_LAUNCH_CHECK();
  }
  return OMNI_OK;
}

}  // namespace

int score_mean_chunks(const Layer& L) { return cdiv(L.v1 - L.v0, kMeanRowsPerChunk); }

size_t score_queries_ws(const Layer& L) {
  Arena a(nullptr);
  a.take<float>((size_t)L.B * L.Hkv * score_mean_chunks(L) * L.D);
  return a.used();
}

int run_probe_keys(const Layer& L, int dtype, const void* K, float* probe, void* ws, hipStream_t st) {
  Arena a(ws);
  const int nchunk = score_mean_chunks(L);
  float* partial = a.take<float>((size_t)L.B * L.Hkv * nchunk * L.D);
  if (dtype == OMNI_BF16) {
    if (L.D == 128) return launch_probe_keys<u16, 128>(L, K, probe, partial, nchunk, st);
    return launch_probe_keys<u16, 64>(L, K, probe, partial, nchunk, st);
  }
  if (L.D == 128) return launch_probe_keys<float, 128>(L, K, probe, partial, nchunk, st);
  return launch_probe_keys<float, 64>(L, K, probe, partial, nchunk, st);
}

int run_score_queries(const Layer& L, int dtype, const void* Q, const void* K, float* probe, float* scores, void* ws,
                      hipStream_t st) {
  Arena a(ws);
  const int nchunk = score_mean_chunks(L);
  float* partial = a.take<float>((size_t)L.B * L.Hkv * nchunk * L.D);
  if (dtype == OMNI_BF16) {
    if (L.D == 128) return launch_score<u16, 128>(L, Q, K, probe, scores, partial, nchunk, st);
    return launch_score<u16, 64>(L, Q, K, probe, scores, partial, nchunk, st);
  }
  if (L.D == 128) return launch_score<float, 128>(L, Q, K, probe, scores, partial, nchunk, st);
  return launch_score<float, 64>(L, Q, K, probe, scores, partial, nchunk, st);
}

}  // namespace omni
