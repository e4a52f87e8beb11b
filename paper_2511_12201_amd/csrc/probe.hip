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
// bf16 inputs: Qbar is an fp32 mean; the pooling kernel splits it into two bf16
// terms (hi + mid carry 16 mantissa bits) that are multiplied with the exact bf16
// keys in two MFMAs, so the logits are good to ~1e-5 relative and the key scores
// that decide the selection do not inherit bf16 rounding of the pooled query.
// One workgroup serves all query heads of a KV group with one K fragment; the
// Qbar blocks of its heads arrive by global->LDS DMA, double buffered, one
// barrier per block.  fp32 inputs use the fp32 MFMA and stage Qbar by hand.
#include "common.h"
#include "kernels.h"

namespace omni {

namespace {

constexpr int kThreads = 256;
constexpr float kLog2e = 1.4426950408889634f;

// bf16 terms that carry the fp32 pooled query into the bf16 matrix cores (hi + mid [+ lo])
constexpr int kQbarTerms = 2;

// ---------------------------------------------------------------- pooling

// SCORE: the same pass over Q also writes the lazy/active score of every row (paper Sec. "Query Selection",
// probe-softmax equation), with the arithmetic of the stand-alone scoring kernel, so that Q is read once.
template <typename T, int D, bool SCORE>
__global__ __launch_bounds__(kThreads) void pool_queries_kernel(const T* __restrict__ Q, Layer L, int pb, int nblk,
                                                               float* __restrict__ qbar, u16* __restrict__ qsplit,
                                                               const float* __restrict__ probe_keys,
                                                               float* __restrict__ scores) {
  constexpr int E = Elem<T>::kPer16B;
  constexpr int LPR = D / E;
  constexpr int RPP = kThreads / LPR;
  __shared__ float red[RPP][D];
  const int j = blockIdx.x, bh = blockIdx.y;          // j >= nblk (bf16 only): a zero row that pads the last 32-row block
  const int b = bh / L.Hq, i = bh % L.Hq;
  const T* base = Q + b * L.qs[0] + i * L.qs[1];
  const int c = threadIdx.x % LPR, r0 = threadIdx.x / LPR;
  const int row_begin = min(j * pb, L.N), row_end = min(L.N, row_begin + pb);
  float acc[E];
#pragma unroll
  for (int e = 0; e < E; ++e) acc[e] = 0.f;
  if constexpr (SCORE) {
    const float* pk = probe_keys + ((long long)(b * L.Hkv + i / L.G) * 2) * D;
    float diff[E];
#pragma unroll
    for (int e = 0; e < E; ++e) diff[e] = pk[D + c * E + e] - pk[c * E + e];
    float* out = scores + (long long)bh * L.ld;
    constexpr int kRowsInFlight = 4;                       // loads of this many rows per lane group are issued together
    for (int rb = row_begin; rb < row_end; rb += RPP * kRowsInFlight) {   // uniform trip count: shuffles need every lane
      u32x4 raw[kRowsInFlight];
#pragma unroll
      for (int u = 0; u < kRowsInFlight; ++u) {
        const int r = rb + u * RPP + r0;
        raw[u] = u32x4{0u, 0u, 0u, 0u};
        if (r < row_end) raw[u] = *reinterpret_cast<const u32x4*>(base + (long long)r * L.qs[2] + c * E);
      }
#pragma unroll
      for (int u = 0; u < kRowsInFlight; ++u) {            // rows in ascending order: the sums match the plain pooling pass
        const int r = rb + u * RPP + r0;
        const bool live = r < row_end;
        float dot = 0.f;
        if (live) {
          float v[E];
          unpack16(raw[u], v, (const T*)nullptr);
#pragma unroll
          for (int e = 0; e < E; ++e) {
            acc[e] += v[e];
            dot = fmaf(v[e], diff[e], dot);
          }
        }
#pragma unroll
        for (int o = LPR / 2; o > 0; o >>= 1) dot += __shfl_xor(dot, o, 64);
        if (live && c == 0) out[r] = 1.0f / (1.0f + expf(-dot * L.scale));
      }
    }
  } else {
    for (int r = row_begin + r0; r < row_end; r += RPP) {
      u32x4 raw = *reinterpret_cast<const u32x4*>(base + (long long)r * L.qs[2] + c * E);
      float v[E];
      unpack16(raw, v, (const T*)nullptr);
#pragma unroll
      for (int e = 0; e < E; ++e) acc[e] += v[e];
    }
  }
#pragma unroll
  for (int e = 0; e < E; ++e) red[r0][c * E + e] = acc[e];
  __syncthreads();
  if (threadIdx.x < D) {
    float s = 0.f;
#pragma unroll 4
    for (int r = 0; r < RPP; ++r) s += red[r][threadIdx.x];
    const float mean = row_end > row_begin ? s / (float)(row_end - row_begin) : 0.f;
    if constexpr (sizeof(T) == 2) {
      // split terms, laid out as the probe's LDS stage: [head][row block][term][32 rows][16-byte chunks, XOR-swizzled by row]
      constexpr int CH = D / 8;
      const int nrb = cdiv(nblk, 32);
      const int jb = j >> 5, r = j & 31, d = threadIdx.x;
      const u16 hi = f32_to_bf16_bits(mean);
      const float r1 = mean - bf16_bits_to_f32(hi);
      u16 term[3];
      term[0] = hi;
      term[1] = f32_to_bf16_bits(r1);
      term[2] = f32_to_bf16_bits(r1 - bf16_bits_to_f32(term[1]));
      const int col = (((d >> 3) ^ (r % CH)) << 3) + (d & 7);
#pragma unroll
      for (int t = 0; t < kQbarTerms; ++t)
        qsplit[((((long long)bh * nrb + jb) * kQbarTerms + t) * 32 + r) * D + col] = term[t];
    } else {
      qbar[((long long)bh * nblk + j) * D + threadIdx.x] = mean;
    }
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

// fp32 inputs: one workgroup per (key chunk, query head), fp32 MFMA, Qbar blocks staged through LDS by hand.
// PASS 1: partial (max, sum) per pooled row for this workgroup's key range.
// PASS 2: column sums.
template <int D, int PASS>
__global__ __launch_bounds__(kThreads) void probe_f32_kernel(const float* __restrict__ K, Layer L, int pb, int nblk,
                                                            int nchunk, const float* __restrict__ qbar,
                                                            float* __restrict__ part_m, float* __restrict__ part_l,
                                                            const float* __restrict__ lse2w,
                                                            float* __restrict__ a_out) {
  using T = float;
  constexpr int KB = ProbeTraits<T>::kKeyBlocks;
  constexpr int KPW = KB * 32;            // keys per wavefront
  constexpr int KPG = 4 * KPW;            // keys per workgroup
  constexpr int QLD = D + 4;
  __shared__ __attribute__((aligned(16))) float sQ[32 * QLD];   // Qbar block, MFMA B operand
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
  f32x4 kf32[KB][D / 8];
#pragma unroll
  for (int kb = 0; kb < KB; ++kb) {
    const int key = min(k0 + kb * 32 + ln, L.N - 1);
    const T* row = kbase + (long long)key * L.ks[2];
#pragma unroll
    for (int ks = 0; ks < D / 8; ++ks) kf32[kb][ks] = *reinterpret_cast<const f32x4*>(row + ks * 8 + h * 4);
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
      *reinterpret_cast<f32x4*>(sQ + row * QLD + col) = v;
    }
    if (PASS == 2 && threadIdx.x < 32) {
      const int j = jb * 32 + threadIdx.x;
      sLse[threadIdx.x] = j < nblk ? lse2w[(long long)bh * nrb * 32 + j] : 0.f;
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
#pragma unroll
      for (int ks = 0; ks < D / 8; ++ks) {
        const f32x4 qf = *reinterpret_cast<const f32x4*>(sQ + ln * QLD + ks * 8 + h * 4);
#pragma unroll
        for (int e = 0; e < 4; ++e)
          acc[kb] = __builtin_amdgcn_mfma_f32_32x32x2f32(kf32[kb][ks][e], qf[e], acc[kb], 0, 0, 0);
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
      float* dst = a_out + (long long)bh * L.ld;
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

// ---------------------------------------------------------------- bf16 probe: one workgroup per (key chunk, KV group)

// Sum of v[i] over the 32 lanes of a half-wave, for 32 values at once: a reduce-scatter butterfly (31 exchanges)
// that leaves the total of value index (lane & 31) in v[0].
template <int W>
__device__ __forceinline__ void reduce_scatter_step(float (&v)[32], int ln) {
  const bool up = (ln & W) != 0;
#pragma unroll
  for (int i = 0; i < W; ++i) {
    const float send = up ? v[i] : v[i + W];
    const float keep = up ? v[i + W] : v[i];
    v[i] = keep + __shfl_xor(send, W, 64);
  }
}
__device__ __forceinline__ float half_wave_reduce_scatter(float (&v)[32], int ln) {
  reduce_scatter_step<16>(v, ln);
  reduce_scatter_step<8>(v, ln);
  reduce_scatter_step<4>(v, ln);
  reduce_scatter_step<2>(v, ln);
  reduce_scatter_step<1>(v, ln);
  return v[0];
}

// grid: nchunk * B*Hkv workgroups, chunk-major (the chunks of low key index see the most pooled rows: longest first).
// PASS 1: (max, sum) of every pooled row over this workgroup's 256 keys -> part_m / part_l.
// PASS 2: a[head, key] = sum over pooled rows of exp2(s2 - lse2w[row]).
template <int D, int PASS>
__global__ __launch_bounds__(kThreads, 2) void probe_bf16_kernel(const u16* __restrict__ K, Layer L, int pb, int nblk,
                                                             int nchunk, const u16* __restrict__ qsplit,
                                                             float* __restrict__ part_m, float* __restrict__ part_l,
                                                             const float* __restrict__ lse2w,
                                                             float* __restrict__ a_out) {
  constexpr int KB = 2;                        // 32-key blocks per wavefront
  constexpr int KPW = KB * 32, KPG = 4 * KPW;
  constexpr int CH = D / 8;                    // 16-byte chunks per row
  constexpr int kStage = kQbarTerms * 32 * D * 2;
  constexpr int IPW = kStage / 1024 / 4;       // DMA instructions (1 KiB each) per wavefront per stage
  constexpr int IPB = IPW + (PASS == 2 ? 1 : 0);   // ... per block, with the lse row
  constexpr int NS = 3;                        // ring of stages: blocks it+1 and it+2 are in flight while block it is used
  static_assert(kStage % 4096 == 0, "stage must split evenly over the four wavefronts");
  __shared__ __attribute__((aligned(1024))) unsigned char sQ[NS][kStage];
  __shared__ float sRedM[2][4][32], sRedL[2][4][32];
  __shared__ __attribute__((aligned(256))) float sLse[NS][64];

  const int ngrp = L.B * L.Hkv;
  const int chunk = blockIdx.x / ngrp, bg = blockIdx.x % ngrp;
  const int b = bg / L.Hkv, g = bg % L.Hkv;
  const int lane = lane_id();
  const int wave = __builtin_amdgcn_readfirstlane((int)(threadIdx.x >> 6));
  const int ln = lane & 31, h = lane >> 5;
  const int k0 = chunk * KPG + wave * KPW;     // first key of this wavefront
  const int wg_end = chunk * KPG + KPG;
  const float c2 = L.scale * kLog2e;
  const int nrb = cdiv(nblk, 32);
  const int jb0 = L.causal ? ((chunk * KPG) / pb) / 32 : 0;
  const int n_it = L.G * (nrb - jb0);
  const int bh0 = b * L.Hq + g * L.G;
  const unsigned lds_base = (unsigned)(size_t)(__attribute__((address_space(3))) unsigned char*)&sQ[0][0];
  const unsigned lane_off = (unsigned)(wave * 1024 + lane * 16);
  const unsigned lse_base = (unsigned)(size_t)(__attribute__((address_space(3))) unsigned char*)&sLse[0][0];

  auto issue = [&](int jh, int jb, int stage) {
    const unsigned char* src =
        reinterpret_cast<const unsigned char*>(qsplit) + ((long long)(bh0 + jh) * nrb + jb) * kStage;
#pragma unroll
    for (int q = 0; q < IPW; ++q)
      gload_lds16(src + q * 4096, lane_off, lds_base + stage * kStage + q * 4096 + wave * 1024);
    // the rows' lse ride along (64 floats: this block's 32 and 32 that nobody reads), so that no ordinary load --
    // whose wait would also drain the DMA queue -- sits in the loop; every wavefront fetches them (same bytes, same
    // place) so that all wavefronts have the same number of loads in flight
    if (PASS == 2)
      gload_lds4(lse2w + ((long long)(bh0 + jh) * nrb + jb) * 32 + lane, lse_base + stage * 256);
  };

  // block `it` of this workgroup is (head jh, row block jb); the issue cursor runs NS-1 blocks ahead
  int jh_i = 0, jb_i = jb0, it_i = 0;
  auto issue_next = [&]() {
    if (it_i < n_it) {
      issue(jh_i, jb_i, it_i % NS);
      ++it_i;
      if (++jb_i == nrb) {
        jb_i = jb0;
        ++jh_i;
      }
    }
  };
#pragma unroll
  for (int pre = 0; pre < NS - 1; ++pre) issue_next();

  // K fragment (A operand), rows clamped into range; out-of-range keys are masked below
  const u16* kbase = K + b * L.ks[0] + g * L.ks[1];
  bf16x8 kf[KB][D / 16];
#pragma unroll
  for (int kb = 0; kb < KB; ++kb) {
    const int key = min(k0 + kb * 32 + ln, L.N - 1);
    const u16* row = kbase + (long long)key * L.ks[2];
#pragma unroll
    for (int ks = 0; ks < D / 16; ++ks) kf[kb][ks] = *reinterpret_cast<const bf16x8*>(row + ks * 16 + h * 8);
  }
#pragma unroll
  for (int kb = 0; kb < KB; ++kb)
#pragma unroll
    for (int ks = 0; ks < D / 16; ++ks) asm volatile("" : "+v"(kf[kb][ks]));      // landed before the loop starts

  float colacc[32];
#pragma unroll
  for (int r = 0; r < 32; ++r) colacc[r] = 0.f;

  // combine the four wavefronts' (max, sum) of one row block and write the workgroup's partial
  auto combine = [&](int jh, int jb, int buf) {
    const int j = jb * 32 + lane;
    if (lane < 32 && j < nblk) {
      float M = -INFINITY;
#pragma unroll
      for (int w = 0; w < 4; ++w) M = fmaxf(M, sRedM[buf][w][lane]);
      const float Mr = M == -INFINITY ? 0.f : M;
      float Ls = 0.f;
#pragma unroll
      for (int w = 0; w < 4; ++w) {
        const float mw = sRedM[buf][w][lane];
        Ls += mw == -INFINITY ? 0.f : sRedL[buf][w][lane] * fast_exp2(mw - Mr);
      }
      const long long o = ((long long)(bh0 + jh) * nblk + j) * nchunk + chunk;
      part_m[o] = M;
      part_l[o] = Ls;
    }
  };

  int jh = 0, jb = jb0, jh_prev = 0, jb_prev = jb0;
  for (int it = 0; it < n_it; ++it) {
    // this wavefront's share of block `it` has landed (the blocks after it may still be in flight)
    if (it + NS - 2 < n_it) {
      wait_vmcnt<(NS - 2) * IPB>();
    } else {
      wait_vmcnt<0>();
    }
    __syncthreads();                               // everyone's has; everyone is done reading block it-1
    int jh_n = jh, jb_n = jb + 1;
    if (jb_n == nrb) {
      jb_n = jb0;
      ++jh_n;
    }
    issue_next();                                  // block it+NS-1 into the stage that block it-1 used
    if (PASS == 1 && it > 0 && wave == (it & 3)) combine(jh_prev, jb_prev, (it - 1) & 1);

    const unsigned char* st = sQ[it % NS];
    f32x16 acc[KB];
#pragma unroll
    for (int kb = 0; kb < KB; ++kb)
#pragma unroll
      for (int r = 0; r < 16; ++r) acc[kb][r] = 0.f;
#pragma unroll
    for (int ks = 0; ks < D / 16; ++ks) {
#pragma unroll
      for (int s = kQbarTerms - 1; s >= 0; --s) {  // small terms first
        const bf16x8 qf =
            *reinterpret_cast<const bf16x8*>(st + ((s * 32 + ln) * CH + ((ks * 2 + h) ^ (ln % CH))) * 16);
#pragma unroll
        for (int kb = 0; kb < KB; ++kb) acc[kb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(kf[kb][ks], qf, acc[kb], 0, 0, 0);
      }
    }

    // every key of the workgroup is real and visible to every row of the block?
    const bool full = jb * 32 + 32 <= nblk && wg_end <= L.N && (!L.causal || (long long)(jb * 32 + 1) * pb >= wg_end);
    const int j = jb * 32 + ln;                    // this lane's pooled row
    const int vis_end = j < nblk ? (L.causal ? min((j + 1) * pb, L.N) : L.N) : 0;
    const int rel = vis_end - k0 - 4 * h;          // element (kb, r) is visible iff kb*32 + 8*(r>>2) + (r&3) < rel

    if (PASS == 1) {
      float m = -INFINITY;
      if (full) {
#pragma unroll
        for (int kb = 0; kb < KB; ++kb)
#pragma unroll
          for (int r = 0; r < 16; ++r) m = fmaxf(m, acc[kb][r]);
      } else {
#pragma unroll
        for (int kb = 0; kb < KB; ++kb)
#pragma unroll
          for (int r = 0; r < 16; ++r) {
            if (kb * 32 + 8 * (r >> 2) + (r & 3) >= rel) acc[kb][r] = -INFINITY;
            m = fmaxf(m, acc[kb][r]);
          }
      }
      m = pair_max(m);                             // the other half-wave holds the other keys of the same row
      const float ms = m == -INFINITY ? 0.f : m * c2;
      float l = 0.f;
#pragma unroll
      for (int kb = 0; kb < KB; ++kb)
#pragma unroll
        for (int r = 0; r < 16; ++r) l += fast_exp2(fmaf(acc[kb][r], c2, -ms));
      l = pair_sum(l);
      if (h == 0) {
        sRedM[it & 1][wave][ln] = m == -INFINITY ? m : m * c2;
        sRedL[it & 1][wave][ln] = l;
      }
    } else {
      const float lse = sLse[it % NS][ln];
      if (full) {
#pragma unroll
        for (int kb = 0; kb < KB; ++kb)
#pragma unroll
          for (int r = 0; r < 16; ++r) colacc[kb * 16 + r] += fast_exp2(fmaf(acc[kb][r], c2, -lse));
      } else {
#pragma unroll
        for (int kb = 0; kb < KB; ++kb)
#pragma unroll
          for (int r = 0; r < 16; ++r) {
            const float pv = fast_exp2(fmaf(acc[kb][r], c2, -lse));
            colacc[kb * 16 + r] += kb * 32 + 8 * (r >> 2) + (r & 3) < rel ? pv : 0.f;
          }
      }
      if (jb == nrb - 1) {                         // last row block of this head: reduce over its rows and store
        const float total = half_wave_reduce_scatter(colacc, ln);
        const int key = k0 + (ln >> 4) * 32 + 8 * ((ln & 15) >> 2) + 4 * h + (ln & 3);
        if (key < L.N) a_out[(long long)(bh0 + jh) * L.ld + key] = total;
#pragma unroll
        for (int r = 0; r < 32; ++r) colacc[r] = 0.f;
      }
    }
    jh_prev = jh;
    jb_prev = jb;
    jh = jh_n;
    jb = jb_n;
  }
  if (PASS == 1) {
    __syncthreads();
    if (wave == 0) combine(jh_prev, jb_prev, (n_it - 1) & 1);
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
  if (lane == 0) lse2w[(long long)bh * cdiv(nblk, 32) * 32 + j] = Mr + log2f(s) - log2f((float)(row_end - j * pb));
}

struct ProbeWs {
  float* qbar;                 // fp32 path: pooled queries [BH, nblk, D]
  u16* qsplit;                 // bf16 path: split terms in the probe's stage layout
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
  w.qbar = nullptr;
  w.qsplit = nullptr;
  if (sizeof(T) == 2)
    w.qsplit = a.take<u16>(BH * cdiv(nblk, 32) * kQbarTerms * 32 * L.D);
  else
    w.qbar = a.take<float>(BH * nblk * L.D);
  w.part_m = a.take<float>(BH * nblk * nchunk);
  w.part_l = a.take<float>(BH * nblk * nchunk);
  w.lse2w = a.take<float>(BH * cdiv(nblk, 32) * 32 + 32);   // [BH, 32-row blocks, 32] and one block of slack for 64-wide reads
  return w;
}

template <typename T, int D>
int launch_probe(const Layer& L, const void* Q, const void* K, int pb, float* key_scores, void* ws, hipStream_t st,
                 const float* probe_keys, float* scores) {
  Arena a(ws);
  ProbeWs w = carve_probe<T>(a, L, pb);
  const int nblk = cdiv(L.N, pb);
  constexpr int KPG = probe_keys_per_wg<T>();
  const int nchunk = cdiv(L.N, KPG);
  const int BH = L.B * L.Hq;
  {
    ProfScope prof__(kProfPool, st);
    const int pooled_rows = sizeof(T) == 2 ? cdiv(nblk, 32) * 32 : nblk;
    if (scores) {
      hipLaunchKernelGGL((pool_queries_kernel<T, D, true>), dim3(pooled_rows, BH), dim3(kThreads), 0, st,
                         static_cast<const T*>(Q), L, pb, nblk, w.qbar, w.qsplit, probe_keys, scores);
    } else {
      hipLaunchKernelGGL((pool_queries_kernel<T, D, false>), dim3(pooled_rows, BH), dim3(kThreads), 0, st,
                         static_cast<const T*>(Q), L, pb, nblk, w.qbar, w.qsplit, (const float*)nullptr,
                         (float*)nullptr);
    }
    OMNI_LAUNCH_CHECK();
  }
  if constexpr (sizeof(T) == 2) {
    const u16* Kp = static_cast<const u16*>(K);
    const int nwg = nchunk * L.B * L.Hkv;
    {
      ProfScope prof__(kProfProbeLse, st);
      hipLaunchKernelGGL((probe_bf16_kernel<D, 1>), dim3(nwg), dim3(kThreads), 0, st, Kp, L, pb, nblk, nchunk, w.qsplit,
                         w.part_m, w.part_l, (const float*)nullptr, (float*)nullptr);
      OMNI_LAUNCH_CHECK();
    }
    hipLaunchKernelGGL(probe_lse_kernel, dim3(cdiv(nblk, 4), BH), dim3(kThreads), 0, st, L, pb, nblk, nchunk, KPG,
                       w.part_m, w.part_l, w.lse2w);
    OMNI_LAUNCH_CHECK();
    {
      ProfScope prof__(kProfProbeSum, st);
      hipLaunchKernelGGL((probe_bf16_kernel<D, 2>), dim3(nwg), dim3(kThreads), 0, st, Kp, L, pb, nblk, nchunk, w.qsplit,
                         (float*)nullptr, (float*)nullptr, w.lse2w, key_scores);
      OMNI_LAUNCH_CHECK();
    }
    return OMNI_OK;
  } else {
  {
    ProfScope prof__(kProfProbeLse, st);
    hipLaunchKernelGGL((probe_f32_kernel<D, 1>), dim3(nchunk, BH), dim3(kThreads), 0, st, static_cast<const T*>(K), L, pb,
                       nblk, nchunk, w.qbar, w.part_m, w.part_l, (const float*)nullptr, (float*)nullptr);
    OMNI_LAUNCH_CHECK();
  }
  hipLaunchKernelGGL(probe_lse_kernel, dim3(cdiv(nblk, 4), BH), dim3(kThreads), 0, st, L, pb, nblk, nchunk, KPG,
                     w.part_m, w.part_l, w.lse2w);
  OMNI_LAUNCH_CHECK();
  {
    ProfScope prof__(kProfProbeSum, st);
    hipLaunchKernelGGL((probe_f32_kernel<D, 2>), dim3(nchunk, BH), dim3(kThreads), 0, st, static_cast<const T*>(K), L, pb,
                       nblk, nchunk, w.qbar, (float*)nullptr, (float*)nullptr, w.lse2w, key_scores);
    OMNI_LAUNCH_CHECK();
  }
  return OMNI_OK;
  }
}

}  // namespace

size_t probe_ws(const Layer& L, int dtype, int pb) {
  Arena a(nullptr);
  if (dtype == OMNI_BF16) carve_probe<u16>(a, L, pb); else carve_probe<float>(a, L, pb);
  return a.used();
}

int run_probe(const Layer& L, int dtype, const void* Q, const void* K, int pb, float* key_scores, void* ws,
              hipStream_t st, const float* probe_keys, float* scores) {
  if (dtype == OMNI_BF16) {
    if (L.D == 128) return launch_probe<u16, 128>(L, Q, K, pb, key_scores, ws, st, probe_keys, scores);
    return launch_probe<u16, 64>(L, Q, K, pb, key_scores, ws, st, probe_keys, scores);
  }
  if (L.D == 128) return launch_probe<float, 128>(L, Q, K, pb, key_scores, ws, st, probe_keys, scores);
  return launch_probe<float, 64>(L, Q, K, pb, key_scores, ws, st, probe_keys, scores);
}

}  // namespace omni
