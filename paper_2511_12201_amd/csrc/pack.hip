// Gather / re-layout passes that feed the attention kernels (HBM-bound copies).
//
// pack_kv: per head, the selected K/V rows are gathered into dense buffers,
// padded with zero rows to whole 64-key tiles, and the original token index of
// every slot is recorded (pad slots: kPadKeyIndex).  Two layouts are produced on
// request: "natural" [slot][d], and "k-packed" [16-slot group][half h][d][8 slots]
// with slot(group,h,j) = 16 group + 8 (j/4) + 4 h + j%4 -- the order in which a
// 32x32 MFMA accumulator holds its rows -- so that the operand of a GEMM that
// contracts over the slots is one 16-byte LDS read per lane.  fp32 inputs only
// use the natural layout (the fp32 MFMA takes one element per lane).  The k-packed
// V (the forward's operand; the backward does not use it) is written in f16: the
// forward multiplies its f16-rounded weights with it.
//
// pack_q: for the backward pass, the kept rows of Q and dO in the k-packed
// layout (contraction over queries) and, for bf16, also as contiguous natural
// rows in kept order (so that a tile of them is one linear stream), plus per
// kept row lse * log2(e) and delta = rowsum(dO * O).
#include "common.h"
#include "kernels.h"

namespace omni {

namespace {

constexpr int kThreads = 256;
constexpr float kLog2e = 1.4426950408889634f;

// Eight bf16 values as f16.  Every bf16 value of magnitude in [2^-14, 65504] is an f16 value (8 significant bits
// into 11); smaller ones land on the f16 subnormal grid (absolute error below 3e-8), larger ones saturate at 65504
// (the conversion rounds towards zero, which never produces an infinity from a finite value).
__device__ __forceinline__ u32x4 bf16x8_to_f16x8(const u32x4& x) {
  u32x4 r;
#pragma unroll
  for (int j = 0; j < 4; ++j) {
    const float lo = __uint_as_float(x[j] << 16), hi = __uint_as_float(x[j] & 0xffff0000u);
    const auto pk = __builtin_amdgcn_cvt_pkrtz(lo, hi);
    r[j] = __builtin_bit_cast(unsigned, pk);
  }
  return r;
}

// 8 rows x 8 bf16 (one 16-byte chunk per row) -> 8 columns x 8 rows, written as 8 x 16 bytes
__device__ __forceinline__ void transpose8x8_store(const u32x4 (&in)[8], u16* dst) {
#pragma unroll
  for (int e = 0; e < 8; ++e) {
    unsigned w[4];
#pragma unroll
    for (int jj = 0; jj < 4; ++jj) {
      const unsigned a = in[2 * jj][e >> 1], b = in[2 * jj + 1][e >> 1];
      const unsigned lo = (e & 1) ? (a >> 16) : (a & 0xffffu);
      const unsigned hi = (e & 1) ? (b >> 16) : (b & 0xffffu);
      w[jj] = lo | (hi << 16);
    }
    u32x4 o = {w[0], w[1], w[2], w[3]};
    *reinterpret_cast<u32x4*>(dst + e * 8) = o;
  }
}

// The list entries [p0, p1) of head bh, formed from the key scores and the head's cut instead of read from a list
// (Eq. 5: the keys above the cut, and the first `need` of those at the cut, in index order).  The chunk offsets say
// which chunks of kSelectChunk scores hold those ranks; they are classified and ranked again here, as the list
// writer of the selection does.  Workgroup-uniform control flow; sIdx must hold the pad index beforehand.
__device__ __forceinline__ void select_tile_entries(const SelectSource& sel, int bh, int N, int p0, int p1, int* sIdx) {
  static_assert(kSelectChunk == 4 * kThreads, "four scores per thread");
  __shared__ int wsum[2][kThreads / 64];
  const unsigned thr = sel.thr[bh];
  const int need = sel.need[bh];
  const int* ok = sel.off_keep + (long long)bh * sel.nchunk;
  const int* oe = sel.off_eq + (long long)bh * sel.nchunk;
  const float* row = sel.x + (long long)bh * sel.ld;
  // last chunk whose first rank is <= p0 (the first ranks are non-decreasing and chunk 0 starts at rank 0)
  int c0 = -1;
  for (int cb = 0; cb < sel.nchunk; cb += kThreads) {
    const int c = cb + threadIdx.x;
    c0 += __syncthreads_count(c < sel.nchunk && ok[c] + min(oe[c], need) <= p0);
  }
  const int lane = lane_id(), w = threadIdx.x >> 6;
  for (int c = c0; c < sel.nchunk; ++c) {
    if (ok[c] + min(oe[c], need) >= p1) break;
    const int base = c * kSelectChunk + threadIdx.x * 4;
    bool al[4], eq[4];
    int ck = 0, ce = 0;
#pragma unroll
    for (int e = 0; e < 4; ++e) {
      al[e] = false;
      eq[e] = false;
      if (base + e < N) {
        const unsigned key = float_key(row[base + e]);
        al[e] = key > thr;
        eq[e] = key == thr;
      }
      ck += al[e];
      ce += eq[e];
    }
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
    int pk = ok[c] + sk - ck, pe = oe[c] + se - ce;
    for (int i = 0; i < w; ++i) {
      pk += wsum[0][i];
      pe += wsum[1][i];
    }
#pragma unroll
    for (int e = 0; e < 4; ++e) {
      if (al[e] || (eq[e] && pe < need)) {
        const int pos = pk + min(pe, need);
        if (pos >= p0 && pos < p1) sIdx[pos - p0] = base + e;
      }
      pk += al[e];
      pe += eq[e];
    }
    __syncthreads();
  }
}

// grid: (npad/64, BHx)
template <typename T, int D, bool SELECT>
__global__ __launch_bounds__(kThreads) void pack_kv_kernel(const T* __restrict__ K, const T* __restrict__ V, Layer L,
                                                          int per_q_head, const int* __restrict__ src_idx,
                                                          int idx_stride, const int* __restrict__ budget, int b_cap,
                                                          int npad, int pad_to, T* __restrict__ Kn, T* __restrict__ Vn,
                                                          T* __restrict__ Kt, T* __restrict__ Vt,
                                                          int* __restrict__ kidx, SelectSource sel) {
  constexpr bool kBf16 = sizeof(T) == 2;
  constexpr int E = Elem<T>::kPer16B;
  constexpr int CPR = D / E;
  __shared__ int sIdx[kTileN];
  const int tile = blockIdx.x, bhx = blockIdx.y;
  const int H = per_q_head ? L.Hq : L.Hkv;
  const int b = bhx / H, hx = bhx % H;
  const int g = per_q_head ? hx / L.G : hx;
  const int nkeys = budget ? min(budget[per_q_head ? budget_slot(L.bph, b, bhx) : b], b_cap) : L.N;
  if (tile * kTileN >= (int)align_up((size_t)max(nkeys, 0), (size_t)pad_to)) return;   // consumers read whole pad_to-slot groups
  if constexpr (SELECT) {
    const int p0 = tile * kTileN;
    if (threadIdx.x < kTileN) sIdx[threadIdx.x] = kPadKeyIndex;
    __syncthreads();
    if (p0 < nkeys) select_tile_entries(sel, bhx, L.N, p0, min(p0 + kTileN, nkeys), sIdx);
    __syncthreads();
    if (threadIdx.x < kTileN) {
      const int p = p0 + threadIdx.x, id = sIdx[threadIdx.x];
      kidx[(long long)bhx * npad + p] = id;
      if (p < nkeys) sel.out[(long long)bhx * sel.out_stride + p] = id;
    }
  } else {
    if (threadIdx.x < kTileN) {
      const int p = tile * kTileN + threadIdx.x;
      int id = kPadKeyIndex;
      if (p < nkeys) id = src_idx ? src_idx[(long long)bhx * idx_stride + p] : p;
      sIdx[threadIdx.x] = id;
      kidx[(long long)bhx * npad + p] = id;
    }
  }
  __syncthreads();
  const T* kbase = K + b * L.ks[0] + g * L.ks[1];
  const T* vbase = V + b * L.ks[0] + g * L.ks[1];
  const long long tile_off = ((long long)bhx * npad + tile * kTileN) * D;
  const u32x4 zero = {0u, 0u, 0u, 0u};
  if (Kn || Vn) {
    for (int c = threadIdx.x; c < kTileN * CPR; c += kThreads) {
      const int row = c / CPR, col = (c % CPR) * E;
      const int id = sIdx[row];
      if (Kn) {
        u32x4 v = zero;
        if (id != kPadKeyIndex) v = *reinterpret_cast<const u32x4*>(kbase + (long long)id * L.ks[2] + col);
        *reinterpret_cast<u32x4*>(Kn + tile_off + row * D + col) = v;
      }
      if (Vn) {
        u32x4 v = zero;
        if (id != kPadKeyIndex) v = *reinterpret_cast<const u32x4*>(vbase + (long long)id * L.ks[2] + col);
        *reinterpret_cast<u32x4*>(Vn + tile_off + row * D + col) = v;
      }
    }
  }
  if constexpr (kBf16) {
    // work item = (tensor, 16-slot group, half, 8-wide d chunk): 8x8 transpose in registers
    constexpr int kItems = (kTileN / 16) * 2 * (D / 8);
    for (int it0 = threadIdx.x; it0 < 2 * kItems; it0 += kThreads) {
      const int which = it0 / kItems, it = it0 % kItems;
      T* dst_t = which ? Vt : Kt;
      if (!dst_t) continue;
      const T* src = which ? vbase : kbase;
      const int dc = it % (D / 8);
      const int h = (it / (D / 8)) & 1;
      const int grp = it / (D / 8) / 2;
      u32x4 in[8];
#pragma unroll
      for (int j = 0; j < 8; ++j) {
        const int id = sIdx[16 * grp + 8 * (j >> 2) + 4 * h + (j & 3)];
        in[j] = zero;
        if (id != kPadKeyIndex) in[j] = *reinterpret_cast<const u32x4*>(src + (long long)id * L.ks[2] + dc * 8);
        if (which) in[j] = bf16x8_to_f16x8(in[j]);     // the forward multiplies its weights and V in f16
      }
      transpose8x8_store(in, reinterpret_cast<u16*>(dst_t) + tile_off + ((grp * 2 + h) * D + dc * 8) * 8);
    }
  }
}

// grid: (ceil(N/64), B*Hq).  Tile t covers kept positions [64 t, 64 t + 64).
template <typename T, int D>
__global__ __launch_bounds__(kThreads) void pack_q_kernel(const T* __restrict__ Q, const T* __restrict__ O,
                                                         const T* __restrict__ dO, const float* __restrict__ lse,
                                                         Layer L, const int* __restrict__ q_idx,
                                                         const int* __restrict__ q_cnt, int nqpad,
                                                         T* __restrict__ Qt, T* __restrict__ dOt,
                                                         T* __restrict__ Qn, T* __restrict__ dOn,
                                                         float* __restrict__ lse2c, float* __restrict__ deltac) {
  constexpr bool kBf16 = sizeof(T) == 2;
  constexpr int E = Elem<T>::kPer16B;
  constexpr int LPR = D / E;
  constexpr int RPP = kThreads / LPR;
  __shared__ int sIdx[64];
  const int tile = blockIdx.x, bh = blockIdx.y;
  const int b = bh / L.Hq, i = bh % L.Hq;
  const int nq = q_cnt[bh];
  if (tile * 64 >= nq) return;
  if (threadIdx.x < 64) {
    const int p = tile * 64 + threadIdx.x;
    sIdx[threadIdx.x] = p < nq ? q_idx[(long long)bh * L.N + p] : -1;
  }
  __syncthreads();
  const long long head_off = b * L.qs[0] + i * L.qs[1];
  // delta = rowsum(dO * O), lse in log2 units; rows that contribute nothing get lse = +inf (P = 0)
  const int c = threadIdx.x % LPR, r0 = threadIdx.x / LPR;
  for (int rb = 0; rb < 64; rb += RPP) {
    const int r = rb + r0;
    const int row = sIdx[r];
    float dot = 0.f;
    u32x4 g = {0u, 0u, 0u, 0u}, qc = {0u, 0u, 0u, 0u};
    if (row >= 0) {
      const u32x4 a = *reinterpret_cast<const u32x4*>(O + head_off + (long long)row * L.qs[2] + c * E);
      g = *reinterpret_cast<const u32x4*>(dO + head_off + (long long)row * L.qs[2] + c * E);
      if (Qn) qc = *reinterpret_cast<const u32x4*>(Q + head_off + (long long)row * L.qs[2] + c * E);
      float av[E], gv[E];
      unpack16(a, av, (const T*)nullptr);
      unpack16(g, gv, (const T*)nullptr);
#pragma unroll
      for (int e = 0; e < E; ++e) dot = fmaf(av[e], gv[e], dot);
    }
    if (Qn) {                                   // natural packed copies (pad rows zero)
      const long long o = ((long long)bh * nqpad + tile * 64 + r) * D + c * E;
      *reinterpret_cast<u32x4*>(Qn + o) = qc;
      *reinterpret_cast<u32x4*>(dOn + o) = g;
    }
#pragma unroll
    for (int o = LPR / 2; o > 0; o >>= 1) dot += __shfl_xor(dot, o, 64);
    if (c == 0) {
      const long long o = (long long)bh * nqpad + tile * 64 + r;
      float l2 = INFINITY;
      if (row >= 0) {
        const float lv = lse[(long long)bh * L.N + row];
        l2 = lv == -INFINITY ? INFINITY : lv * kLog2e;
      }
      lse2c[o] = l2;
      deltac[o] = row >= 0 ? dot : 0.f;
    }
  }
  if constexpr (kBf16) {
    constexpr int kItems = (64 / 16) * 2 * (D / 8);
    const u32x4 zero = {0u, 0u, 0u, 0u};
    const long long tile_off = ((long long)bh * nqpad + tile * 64) * D;
    for (int it0 = threadIdx.x; it0 < 2 * kItems; it0 += kThreads) {
      const int which = it0 / kItems, it = it0 % kItems;
      const T* src = (which ? dO : Q) + head_off;
      T* dst_t = which ? dOt : Qt;
      const int dc = it % (D / 8);
      const int h = (it / (D / 8)) & 1;
      const int grp = it / (D / 8) / 2;
      u32x4 in[8];
#pragma unroll
      for (int j = 0; j < 8; ++j) {
        const int row = sIdx[16 * grp + 8 * (j >> 2) + 4 * h + (j & 3)];
        in[j] = zero;
        if (row >= 0) in[j] = *reinterpret_cast<const u32x4*>(src + (long long)row * L.qs[2] + dc * 8);
      }
      transpose8x8_store(in, reinterpret_cast<u16*>(dst_t) + tile_off + ((grp * 2 + h) * D + dc * 8) * 8);
    }
  }
}

template <typename T, int D>
int launch_pack_kv(const Layer& L, const void* K, const void* V, int per_q_head, const int* src_idx, int idx_stride,
                   const int* budget, int b_cap, int npad, int pad_to, void* Kn, void* Vn, void* Kt, void* Vt,
                   int* kidx, hipStream_t st, const SelectSource* sel) {
  const int heads = per_q_head ? L.Hq : L.Hkv;
  ProfScope prof__(kProfPack, st);
  if (sel) {
    if (!per_q_head || !budget) return OMNI_ERR_INVALID;
    hipLaunchKernelGGL((pack_kv_kernel<T, D, true>), dim3(npad / kTileN, L.B * heads), dim3(kThreads), 0, st,
                       static_cast<const T*>(K), static_cast<const T*>(V), L, per_q_head, src_idx, idx_stride, budget,
                       b_cap, npad, pad_to, static_cast<T*>(Kn), static_cast<T*>(Vn), static_cast<T*>(Kt),
                       static_cast<T*>(Vt), kidx, *sel);
  } else {
    hipLaunchKernelGGL((pack_kv_kernel<T, D, false>), dim3(npad / kTileN, L.B * heads), dim3(kThreads), 0, st,
                       static_cast<const T*>(K), static_cast<const T*>(V), L, per_q_head, src_idx, idx_stride, budget,
                       b_cap, npad, pad_to, static_cast<T*>(Kn), static_cast<T*>(Vn), static_cast<T*>(Kt),
                       static_cast<T*>(Vt), kidx, SelectSource{});
  }
  OMNI_LAUNCH_CHECK();
  return OMNI_OK;
}

template <typename T, int D>
int launch_pack_q(const Layer& L, const void* Q, const void* O, const void* dO, const float* lse, const int* q_idx,
                  const int* q_cnt, int nqpad, void* Qt, void* dOt, void* Qn, void* dOn, float* lse2c, float* deltac,
                  hipStream_t st) {
  hipLaunchKernelGGL((pack_q_kernel<T, D>), dim3(nqpad / 64, L.B * L.Hq), dim3(kThreads), 0, st,
                     static_cast<const T*>(Q), static_cast<const T*>(O), static_cast<const T*>(dO), lse, L, q_idx,
                     q_cnt, nqpad, static_cast<T*>(Qt), static_cast<T*>(dOt), static_cast<T*>(Qn), static_cast<T*>(dOn),
                     lse2c, deltac);
  OMNI_LAUNCH_CHECK();
  return OMNI_OK;
}

// Visibility bounds of the causal mask on the packed lists.  The packed key list and the kept-query list
// are both ascending in token index, so the keys a query may see are a prefix of the key list and the
// queries that may see a key are a suffix of the query list; the masks of the tile loops are then
// comparisons of positions with these counts -- no index loads inside the loops.
//   qvis[bh, pos]    = number of packed keys with token index <= that of kept query `pos`
//   kfirst[bh, slot] = first kept-query position whose token index is >= that of packed key `slot`
// grid: (cdiv(max(N, npad), 256), B*Hq)
__global__ __launch_bounds__(256) void visibility_kernel(const int* __restrict__ q_idx, const int* __restrict__ q_cnt,
                                                         const int* __restrict__ kidx, const int* __restrict__ budget,
                                                         int bph, int b_cap, int npad, int N, int Hq, int causal,
                                                         int* __restrict__ qvis, int* __restrict__ kfirst) {
  const int bh = blockIdx.y, b = bh / Hq;
  const int nq = q_cnt[bh], nkeys = min(budget[budget_slot(bph, b, bh)], b_cap);
  const int t = blockIdx.x * blockDim.x + threadIdx.x;
  const int* qlist = q_idx + (long long)bh * N;
  const int* klist = kidx + (long long)bh * npad;
  if (qvis && t < nq) qvis[(long long)bh * N + t] = causal ? upper_count(klist, nkeys, qlist[t]) : nkeys;
  if (kfirst && t < npad) {
    int v = 0;
    if (t >= nkeys) {
      v = nq;                                  // pad slot: nobody sees it
    } else if (causal) {
      const int key = klist[t];
      int lo = 0, hi = nq;
      while (lo < hi) {
        const int mid = (lo + hi) >> 1;
        if (qlist[mid] < key) lo = mid + 1; else hi = mid;
      }
      v = lo;
    }
    kfirst[(long long)bh * npad + t] = v;
  }
}

}  // namespace

int run_visible_counts(const Layer& L, const int* q_idx, const int* q_cnt, const int* kidx, const int* budget,
                       int b_cap, int npad, int* qvis, int* kfirst, hipStream_t st) {
  const int n = kfirst ? max(L.N, npad) : L.N;
  hipLaunchKernelGGL(visibility_kernel, dim3(cdiv(n, 256), L.B * L.Hq), dim3(256), 0, st, q_idx, q_cnt, kidx, budget,
                     L.bph, b_cap, npad, L.N, L.Hq, L.causal, qvis, kfirst);
  OMNI_LAUNCH_CHECK();
  return OMNI_OK;
}

int run_pack_kv(const Layer& L, int dtype, const void* K, const void* V, int per_q_head, const int* src_idx,
                int idx_stride, const int* budget, int b_cap, int npad, int pad_to, void* Kn, void* Vn, void* Kt,
                void* Vt, int* kidx, hipStream_t st, const SelectSource* sel) {
  if (dtype == OMNI_BF16) {
    if (L.D == 128)
      return launch_pack_kv<u16, 128>(L, K, V, per_q_head, src_idx, idx_stride, budget, b_cap, npad, pad_to, Kn, Vn, Kt,
                                      Vt, kidx, st, sel);
    return launch_pack_kv<u16, 64>(L, K, V, per_q_head, src_idx, idx_stride, budget, b_cap, npad, pad_to, Kn, Vn, Kt, Vt,
                                   kidx, st, sel);
  }
  if (L.D == 128)
    return launch_pack_kv<float, 128>(L, K, V, per_q_head, src_idx, idx_stride, budget, b_cap, npad, pad_to, Kn, Vn,
                                      nullptr, nullptr, kidx, st, sel);
  return launch_pack_kv<float, 64>(L, K, V, per_q_head, src_idx, idx_stride, budget, b_cap, npad, pad_to, Kn, Vn,
                                   nullptr, nullptr, kidx, st, sel);
}

int run_pack_q(const Layer& L, int dtype, const void* Q, const void* O, const void* dO, const float* lse,
               const int* q_idx, const int* q_cnt, int nqpad, void* Qt, void* dOt, void* Qn, void* dOn, float* lse2c,
               float* deltac, hipStream_t st) {
  if (dtype == OMNI_BF16) {
    if (L.D == 128)
      return launch_pack_q<u16, 128>(L, Q, O, dO, lse, q_idx, q_cnt, nqpad, Qt, dOt, Qn, dOn, lse2c, deltac, st);
    return launch_pack_q<u16, 64>(L, Q, O, dO, lse, q_idx, q_cnt, nqpad, Qt, dOt, Qn, dOn, lse2c, deltac, st);
  }
  if (L.D == 128)
    return launch_pack_q<float, 128>(L, Q, O, dO, lse, q_idx, q_cnt, nqpad, Qt, dOt, nullptr, nullptr, lse2c, deltac, st);
  return launch_pack_q<float, 64>(L, Q, O, dO, lse, q_idx, q_cnt, nqpad, Qt, dOt, nullptr, nullptr, lse2c, deltac, st);
}

}  // namespace omni
