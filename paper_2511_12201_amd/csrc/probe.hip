// Block-wise probe of the attention map (paper paragraph "Block-wise probing and
// sparse flash attention kernel"; accumulated key score of Sec. "KV Selection
// with Head-level Dynamic Budget Allocation").
//
// Queries are mean-pooled over blocks of `pb` tokens; keys stay at token level.
// Two passes over S^T = K . Qbar^T on the matrix cores: pass 1 reduces each
// pooled row's log-sum-exp, pass 2 accumulates a[k] = sum_j w_j exp(s_jk - lse_j).
// A wavefront keeps its 32/64 keys' K fragment in registers (MFMA A operand) and
// streams 32-row blocks of Qbar through LDS (B operand), so each lane owns one
// pooled row: the row statistics are per-lane scalars and the column sums are
// accumulated per lane and reduced across lanes once at the end.
//
// bf16 inputs: Qbar is an fp32 mean; it is split into three bf16 terms
// (hi + mid + lo carry all 24 mantissa bits) and multiplied with the exact bf16
// keys in three MFMAs, so the logits have fp32 accuracy and the key scores that
// decide the selection do not inherit bf16 rounding of the pooled query.
// fp32 inputs use the fp32 MFMA.
#include "common.h"
#include "kernels.h"

namespace omni {

namespace {

constexpr int kThreads = 256;
constexpr float kLog2e = 1.4426950408889634f;

// ---------------------------------------------------------------- pooling

template <typename T, int D>
__global__ __launch_bounds__(kThreads) void pool_queries_kernel(const T* __restrict__ Q, Layer L, int pb, int nblk,
                                                               float* __restrict__ qbar) {
  constexpr int E = Elem<T>::kPer16B;
  constexpr int LPR = D / E;
  constexpr int RPP = kThreads / LPR;
  __shared__ float red[RPP][D];
  const int j = blockIdx.x, bh = blockIdx.y;
  const int b = bh / L.Hq, i = bh % L.Hq;
  const T* base = Q + b * L.qs[0] + i * L.qs[1];
  const int c = threadIdx.x % LPR, r0 = threadIdx.x / LPR;
  const int row_begin = j * pb, row_end = min(L.N, row_begin + pb);
  float acc[E];
#pragma unroll
  for (int e = 0; e < E; ++e) acc[e] = 0.f;
  for (int r = row_begin + r0; r < row_end; r += RPP) {
    u32x4 raw = *reinterpret_cast<const u32x4*>(base + (long long)r * L.qs[2] + c * E);
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
    qbar[((long long)bh * nblk + j) * D + threadIdx.x] = s / (float)(row_end - row_begin);
  }
}

// ---------------------------------------------------------------- probe passes

template <typename T>
struct ProbeTraits;
template <>
struct ProbeTraits<u16> {
  static constexpr int kKeyBlocks = 2;   // 32-key blocks per wavefront
};
template <>
struct ProbeTraits<float> {
  static constexpr int kKeyBlocks = 1;
};

template <typename T>
__host__ __device__ constexpr int probe_keys_per_wg() {
  return 4 * ProbeTraits<T>::kKeyBlocks * 32;
}

// PASS 1: partial (max, sum) per pooled row for this workgroup's key range.
// PASS 2: column sums.
template <typename T, int D, int PASS>
__global__ __launch_bounds__(kThreads) void probe_kernel(const T* __restrict__ K, Layer L, int pb, int nblk, int nchunk,
                                                        const float* __restrict__ qbar,
                                                        float* __restrict__ part_m, float* __restrict__ part_l,
                                                        const float* __restrict__ lse2w, float* __restrict__ a_out) {
  constexpr bool kBf16 = sizeof(T) == 2;
  constexpr int KB = ProbeTraits<T>::kKeyBlocks;
  constexpr int KPW = KB * 32;            // keys per wavefront
  constexpr int KPG = 4 * KPW;            // keys per workgroup
  constexpr int QLD = kBf16 ? D + 8 : D + 4;
  // Qbar block as MFMA B operand: bf16 -> three split terms, fp32 -> as is
  __shared__ __attribute__((aligned(16))) unsigned char sQ_raw[(kBf16 ? 3 * 32 * QLD * 2 : 32 * QLD * 4)];
  __shared__ float sLse[32];
  __shared__ float sRedM[4][32], sRedL[4][32];

  const int chunk = blockIdx.x, bh = blockIdx.y;
  const int b = bh / L.Hq, i = bh % L.Hq, g = i / L.G;
  const int lane = lane_id(), wave = threadIdx.x >> 6;
  const int ln = lane & 31, h = lane >> 5;
  const int k0 = chunk * KPG + wave * KPW;       // first key of this wavefront
  const float c2 = L.scale * kLog2e;
  const T* kbase = K + b * L.ks[0] + g * L.ks[1];

  // K fragment (A operand), rows clamped into range; out-of-range keys are masked below
  bf16x8 kf16[kBf16 ? KB : 1][kBf16 ? D / 16 : 1];
  f32x4 kf32[kBf16 ? 1 : KB][kBf16 ? 1 : D / 8];
#pragma unroll
  for (int kb = 0; kb < KB; ++kb) {
    const int key = min(k0 + kb * 32 + ln, L.N - 1);
    const T* row = kbase + (long long)key * L.ks[2];
    if constexpr (kBf16) {
#pragma unroll
      for (int ks = 0; ks < D / 16; ++ks) kf16[kb][ks] = *reinterpret_cast<const bf16x8*>(row + ks * 16 + h * 8);
    } else {
#pragma unroll
      for (int ks = 0; ks < D / 8; ++ks) kf32[kb][ks] = *reinterpret_cast<const f32x4*>(row + ks * 8 + h * 4);
    }
  }

  float colacc[KB][16];
#pragma unroll
  for (int kb = 0; kb < KB; ++kb)
#pragma unroll
    for (int r = 0; r < 16; ++r) colacc[kb][r] = 0.f;

  const int nrb = cdiv(nblk, 32);
  const int jb0 = L.causal ? ((chunk * KPG) / pb) / 32 : 0;
  const float* qsrc = qbar + (long long)bh * nblk * D;

  for (int jb = jb0; jb < nrb; ++jb) {
    __syncthreads();          // previous iteration's LDS reads are done
    // stage 32 pooled rows
    for (int t = threadIdx.x; t < 32 * D / 4; t += kThreads) {
      const int row = t / (D / 4), col = (t % (D / 4)) * 4;
      const int j = jb * 32 + row;
      f32x4 v = {0.f, 0.f, 0.f, 0.f};
      if (j < nblk) v = *reinterpret_cast<const f32x4*>(qsrc + (long long)j * D + col);
      if constexpr (kBf16) {
        u16* s0 = reinterpret_cast<u16*>(sQ_raw);
#pragma unroll
        for (int e = 0; e < 4; ++e) {
          const float x = v[e];
          const u16 hi = f32_to_bf16_bits(x);
          const float r1 = x - bf16_bits_to_f32(hi);
          const u16 mid = f32_to_bf16_bits(r1);
          const float r2 = r1 - bf16_bits_to_f32(mid);
          const u16 lo = f32_to_bf16_bits(r2);
          s0[(0 * 32 + row) * QLD + col + e] = hi;
          s0[(1 * 32 + row) * QLD + col + e] = mid;
          s0[(2 * 32 + row) * QLD + col + e] = lo;
        }
      } else {
        float* s0 = reinterpret_cast<float*>(sQ_raw);
        *reinterpret_cast<f32x4*>(s0 + row * QLD + col) = v;
      }
    }
    if (PASS == 2 && threadIdx.x < 32) {
      const int j = jb * 32 + threadIdx.x;
      sLse[threadIdx.x] = j < nblk ? lse2w[(long long)bh * nblk + j] : 0.f;
    }
    __syncthreads();

    const int j = jb * 32 + ln;                     // this lane's pooled row
    const int vis_end = j < nblk ? (L.causal ? min((j + 1) * pb, L.N) : L.N) : 0;
    float m_lane = -INFINITY, l_lane = 0.f;
    f32x16 acc[KB];
#pragma unroll
    for (int kb = 0; kb < KB; ++kb) {
#pragma unroll
      for (int r = 0; r < 16; ++r) acc[kb][r] = 0.f;
      if constexpr (kBf16) {
        const u16* s0 = reinterpret_cast<const u16*>(sQ_raw);
#pragma unroll
        for (int ks = 0; ks < D / 16; ++ks) {
#pragma unroll
          for (int s = 2; s >= 0; --s) {            // small terms first
            const bf16x8 qf = *reinterpret_cast<const bf16x8*>(s0 + (s * 32 + ln) * QLD + ks * 16 + h * 8);
            acc[kb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(kf16[kb][ks], qf, acc[kb], 0, 0, 0);
          }
        }
      } else {
        const float* s0 = reinterpret_cast<const float*>(sQ_raw);
#pragma unroll
        for (int ks = 0; ks < D / 8; ++ks) {
          const f32x4 qf = *reinterpret_cast<const f32x4*>(s0 + ln * QLD + ks * 8 + h * 4);
#pragma unroll
          for (int e = 0; e < 4; ++e)
            acc[kb] = __builtin_amdgcn_mfma_f32_32x32x2f32(kf32[kb][ks][e], qf[e], acc[kb], 0, 0, 0);
        }
      }
    }
    if (PASS == 1) {
#pragma unroll
      for (int kb = 0; kb < KB; ++kb)
#pragma unroll
        for (int r = 0; r < 16; ++r) {
          const int key = k0 + kb * 32 + 8 * (r >> 2) + 4 * h + (r & 3);
          const float s2 = key < vis_end ? acc[kb][r] * c2 : -INFINITY;
          acc[kb][r] = s2;
          m_lane = fmaxf(m_lane, s2);
        }
      const float m_safe = m_lane == -INFINITY ? 0.f : m_lane;
#pragma unroll
      for (int kb = 0; kb < KB; ++kb)
#pragma unroll
        for (int r = 0; r < 16; ++r) l_lane += exp2f(acc[kb][r] - m_safe);
      // the partner lane (other half) holds the other keys of the same pooled row
      const float m_o = __shfl_xor(m_lane, 32, 64), l_o = __shfl_xor(l_lane, 32, 64);
      const float m_new = fmaxf(m_lane, m_o);
      const float m_ref = m_new == -INFINITY ? 0.f : m_new;
      const float l_new = l_lane * exp2f((m_lane == -INFINITY ? m_ref : m_lane) - m_ref) +
                          l_o * exp2f((m_o == -INFINITY ? m_ref : m_o) - m_ref);
      if (h == 0) {
        sRedM[wave][ln] = m_new;
        sRedL[wave][ln] = l_new;
      }
      __syncthreads();
      if (threadIdx.x < 32 && jb * 32 + (int)threadIdx.x < nblk) {
        float M = -INFINITY;
#pragma unroll
        for (int w = 0; w < 4; ++w) M = fmaxf(M, sRedM[w][threadIdx.x]);
        const float Mr = M == -INFINITY ? 0.f : M;
        float Ls = 0.f;
#pragma unroll
        for (int w = 0; w < 4; ++w) {
          const float mw = sRedM[w][threadIdx.x];
          Ls += mw == -INFINITY ? 0.f : sRedL[w][threadIdx.x] * exp2f(mw - Mr);
        }
        const long long o = ((long long)bh * nblk + jb * 32 + threadIdx.x) * nchunk + chunk;
        part_m[o] = M;
        part_l[o] = Ls;
      }
    } else {
      const float lse = sLse[ln];
#pragma unroll
      for (int kb = 0; kb < KB; ++kb)
#pragma unroll
        for (int r = 0; r < 16; ++r) {
          const int key = k0 + kb * 32 + 8 * (r >> 2) + 4 * h + (r & 3);
          const float p = key < vis_end ? exp2f(acc[kb][r] * c2 - lse) : 0.f;
          colacc[kb][r] += p;
        }
    }
  }

  if (PASS == 2) {
#pragma unroll
    for (int kb = 0; kb < KB; ++kb)
#pragma unroll
      for (int r = 0; r < 16; ++r) {
        float v = colacc[kb][r];
#pragma unroll
        for (int o = 16; o > 0; o >>= 1) v += __shfl_xor(v, o, 64);     // over the 32 pooled rows of a half
        colacc[kb][r] = v;
      }
    if (ln == 0) {
      float* dst = a_out + (long long)bh * L.N;
#pragma unroll
      for (int kb = 0; kb < KB; ++kb)
#pragma unroll
        for (int r = 0; r < 16; ++r) {
          const int key = k0 + kb * 32 + 8 * (r >> 2) + 4 * h + (r & 3);
          if (key < L.N) dst[key] = colacc[kb][r];
        }
    }
  }
}

// One wavefront per pooled row: combine the per-chunk (max, sum) into
// lse2w[j] = log2(sum_k 2^{s2_jk}) - log2(w_j).
__global__ __launch_bounds__(kThreads) void probe_lse_kernel(Layer L, int pb, int nblk, int nchunk, int keys_per_chunk,
                                                            const float* __restrict__ part_m,
                                                            const float* __restrict__ part_l,
                                                            float* __restrict__ lse2w) {
  const int bh = blockIdx.y;
  const int j = blockIdx.x * 4 + (threadIdx.x >> 6);
  if (j >= nblk) return;
  const int lane = lane_id();
  const int row_end = min((j + 1) * pb, L.N);
  const int vis_end = L.causal ? row_end : L.N;
  const int nvis = cdiv(vis_end, keys_per_chunk);            // chunks that hold a visible key
  const float* pm = part_m + ((long long)bh * nblk + j) * nchunk;
  const float* pl = part_l + ((long long)bh * nblk + j) * nchunk;
  float M = -INFINITY;
  for (int c = lane; c < nvis; c += 64) M = fmaxf(M, pm[c]);
  M = wave_max(M);
  const float Mr = M == -INFINITY ? 0.f : M;
  float s = 0.f;
  for (int c = lane; c < nvis; c += 64) {
    const float m = pm[c];
    s += m == -INFINITY ? 0.f : pl[c] * exp2f(m - Mr);
  }
  s = wave_sum(s);
  if (lane == 0) lse2w[(long long)bh * nblk + j] = Mr + log2f(s) - log2f((float)(row_end - j * pb));
}

struct ProbeWs {
  float* qbar;
  float* part_m;
  float* part_l;
  float* lse2w;
};

template <typename T>
ProbeWs carve_probe(Arena& a, const Layer& L, int pb) {
  ProbeWs w;
  const size_t BH = (size_t)L.B * L.Hq;
  const int nblk = cdiv(L.N, pb);
  const int nchunk = cdiv(L.N, probe_keys_per_wg<T>());
  w.qbar = a.take<float>(BH * nblk * L.D);
  w.part_m = a.take<float>(BH * nblk * nchunk);
  w.part_l = a.take<float>(BH * nblk * nchunk);
  w.lse2w = a.take<float>(BH * nblk);
  return w;
}

template <typename T, int D>
int launch_probe(const Layer& L, const void* Q, const void* K, int pb, float* key_scores, void* ws, hipStream_t st) {
  Arena a(ws);
  ProbeWs w = carve_probe<T>(a, L, pb);
  const int nblk = cdiv(L.N, pb);
  constexpr int KPG = probe_keys_per_wg<T>();
  const int nchunk = cdiv(L.N, KPG);
  const int BH = L.B * L.Hq;
  {
    ProfScope prof__(kProfPool, st);
    hipLaunchKernelGGL((pool_queries_kernel<T, D>), dim3(nblk, BH), dim3(kThreads), 0, st, static_cast<const T*>(Q), L,
                       pb, nblk, w.qbar);
    OMNI_LAUNCH_CHECK();
  }
  {
    ProfScope prof__(kProfProbeLse, st);
    hipLaunchKernelGGL((probe_kernel<T, D, 1>), dim3(nchunk, BH), dim3(kThreads), 0, st, static_cast<const T*>(K), L, pb,
                       nblk, nchunk, w.qbar, w.part_m, w.part_l, (const float*)nullptr, (float*)nullptr);
    OMNI_LAUNCH_CHECK();
  }
  hipLaunchKernelGGL(probe_lse_kernel, dim3(cdiv(nblk, 4), BH), dim3(kThreads), 0, st, L, pb, nblk, nchunk, KPG,
                     w.part_m, w.part_l, w.lse2w);
  OMNI_LAUNCH_CHECK();
  {
    ProfScope prof__(kProfProbeSum, st);
    hipLaunchKernelGGL((probe_kernel<T, D, 2>), dim3(nchunk, BH), dim3(kThreads), 0, st, static_cast<const T*>(K), L, pb,
                       nblk, nchunk, w.qbar, (float*)nullptr, (float*)nullptr, w.lse2w, key_scores);
    OMNI_LAUNCH_CHECK();
  }
  return OMNI_OK;
}

}  // namespace

size_t probe_ws(const Layer& L, int dtype, int pb) {
  Arena a(nullptr);
  if (dtype == OMNI_BF16) carve_probe<u16>(a, L, pb); else carve_probe<float>(a, L, pb);
  return a.used();
}

int run_probe(const Layer& L, int dtype, const void* Q, const void* K, int pb, float* key_scores, void* ws,
              hipStream_t st) {
  if (dtype == OMNI_BF16) {
    if (L.D == 128) return launch_probe<u16, 128>(L, Q, K, pb, key_scores, ws, st);
    return launch_probe<u16, 64>(L, Q, K, pb, key_scores, ws, st);
  }
  if (L.D == 128) return launch_probe<float, 128>(L, Q, K, pb, key_scores, ws, st);
  return launch_probe<float, 64>(L, Q, K, pb, key_scores, ws, st);
}

}  // namespace omni
