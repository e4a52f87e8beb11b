// Backward of the sparse attention (omni_sparse_attn_bwd): gradients of
// O = softmax(Q K^T scale) V over kept queries x selected keys with the index
// sets held constant (the paper trains with the same sparse attention and gives
// no gradient through the selection):
//   P = exp(S - lse), dV = P^T dO, dP = dO V^T, dS = P (dP - delta),
//   delta = rowsum(dO O), dQ = scale dS K, dK = scale dS^T Q.
//
// Deterministic, no floating-point atomics.  bf16 (the measured path), three kernels in the forward's style
// (8 wavefronts, LDS-DMA ring, position masks from the visible-prefix counts):
//  * attn_bwd_dq_bf16_kernel: a work item is 256 kept queries of a head (32 per wavefront) from the forward's
//    longest-first list; it streams 64-key tiles of K, V (natural) and K^T (k-packed): S^T = K Q^T,
//    dP^T = V dO^T, dQ^T += K^T dS^T.
//  * attn_bwd_key_bf16_kernel<D, MODE>: a workgroup owns 256 packed keys of a query head (32 per wavefront, K or V
//    fragments resident) and streams 64-query tiles of the packed kept rows (Q, dO natural and k-packed, lse and
//    delta by 4-byte LDS-DMA).  MODE 0 forms dK' = dS^T Q, MODE 1 dV' = P^T dO: two launches, because the resident
//    fragments and accumulators of both do not fit two wavefronts per SIMD; S = Q K^T is computed in both.  Items
//    (head, key tile, split) come from a list a small kernel compacts; a key tile seen by many query tiles is
//    shared by up to four workgroups, each with a partial plane of its own.
//  * attn_bwd_reduce_kernel adds the per-query-head dK', dV' rows (and split planes) of a KV group in a fixed order
//    into dK, dV -- a head's row is found through an inverse slot map -- and writes zeros for unselected tokens.
// fp32 inputs (the 1e-4 parity cases) keep the older register-staged pair attn_bwd_dkdv_kernel (128 keys per
// workgroup, dK' and dV' together) / attn_bwd_dq_kernel on the fp32 32x32x2 MFMA with natural layouts.
#include <algorithm>

#include <type_traits>

#include "common.h"
#include "kernels.h"
#include "sched.h"

namespace omni {

namespace {

constexpr int kThreads = 256;
constexpr float kLog2e = 1.4426950408889634f;
constexpr int kBwdKeys = 128;     // keys per dkdv workgroup
constexpr int kBwdQ = 64;         // queries per dkdv iteration

struct BwdParams {
  const void* Q;
  const void* dO;
  Layer L;
  const int* q_idx;
  const int* q_cnt;
  const int* budget;
  int b_cap, npad, nqpad;
  const void* Kn;       // packed natural K, V
  const void* Vn;
  const void* Kt;       // k-packed K (bf16 only)
  const int* kidx;
  const void* Qt;       // k-packed kept Q, dO (bf16 only)
  const void* dOt;
  const void* Qn;       // kept Q, dO rows in kept order, contiguous (bf16 only)
  const void* dOn;
  const float* lse2c;   // per kept position: lse * log2e (+inf: contributes nothing)
  const float* deltac;
  float* dKp;           // [B*Hq, npad, D] fp32 per-query-head partial gradients
  float* dVp;
  void* dQ;
  int* sched;           // work list of the dQ kernel (sched.h)
  size_t order_off;     // where its hand-out order starts
  const int* qvis;      // [B*Hq, N] visible packed keys per kept-query position (bf16 fast path)
  const int* kfirst;    // [B*Hq, npad] first kept-query position that sees a packed key
  int head_group;       // heads per dispatch group of the key kernels
  int nsplit;           // most workgroups that share the query tiles of one key tile (bf16 key kernels)
  int split_len;        // query tiles per split, at least
  long long plane;      // floats between the partial-gradient planes of two splits
  int* klist;           // work list of the key kernels: [0], [1] counters (dV, dK kernel), [2] items, [4..] items
  // In-place block lists (TILEMAP kernels): Kn, Vn, Kt hold every KV head once, in token order ([B*Hkv, npad_kv, D]),
  // and tile t of a head's key list is tile tile_map[bh * tile_stride + t] of its KV head's copy.
  const int* tile_map;
  int tile_stride;
  int npad_kv;          // rows per (head) buffer of Kn / Vn / Kt: npad for the gathered copies
};

// first position in ascending a[0,n) with a[pos] >= v
__device__ __forceinline__ int lower_pos(const int* __restrict__ a, int n, int v) {
  int lo = 0, hi = n;
  while (lo < hi) {
    const int mid = (lo + hi) >> 1;
    if (a[mid] < v) lo = mid + 1; else hi = mid;
  }
  return lo;
}
// number of entries <= v
__device__ __forceinline__ int upper_cnt(const int* __restrict__ a, int n, int v) {
  int lo = 0, hi = n;
  while (lo < hi) {
    const int mid = (lo + hi) >> 1;
    if (a[mid] <= v) lo = mid + 1; else hi = mid;
  }
  return lo;
}

__device__ __forceinline__ bf16x8 pack8(const f32x16& v, int r0) {
  union { bf16x8 v; unsigned u[4]; } o;
#pragma unroll
  for (int jj = 0; jj < 4; ++jj) o.u[jj] = pack_bf16x2(v[r0 + 2 * jj], v[r0 + 2 * jj + 1]);
  return o.v;
}

// ------------------------------------------------------------------ dK', dV'

template <typename T, int D>
__global__ __launch_bounds__(kThreads, 1) void attn_bwd_dkdv_kernel(BwdParams p) {
  constexpr bool kBf16 = sizeof(T) == 2;
  constexpr int LD = D + 8;                               // row pitch of natural tiles (elements)
  constexpr int NBUF = kBf16 ? 2 : 1;
  constexpr int kNatBytes = kBwdQ * LD * (int)sizeof(T);
  constexpr int kPackBytes = kBf16 ? kBwdQ * D * 2 : 16;
  __shared__ __attribute__((aligned(16))) unsigned char sQn_raw[NBUF * kNatBytes];
  __shared__ __attribute__((aligned(16))) unsigned char sGn_raw[NBUF * kNatBytes];
  __shared__ __attribute__((aligned(16))) unsigned char sQt_raw[NBUF * kPackBytes];
  __shared__ __attribute__((aligned(16))) unsigned char sGt_raw[NBUF * kPackBytes];
  __shared__ __attribute__((aligned(16))) float sLse[NBUF][kBwdQ];
  __shared__ __attribute__((aligned(16))) float sDel[NBUF][kBwdQ];
  __shared__ __attribute__((aligned(16))) int sQi[NBUF][kBwdQ];
  __shared__ int sBound[2];

  const Layer& L = p.L;
  const int ktile = blockIdx.x, bh = blockIdx.y;
  const int b = bh / L.Hq, i = bh % L.Hq;
  const int nkeys = min(p.budget[budget_slot(L.bph, b, bh)], p.b_cap);
  if (ktile * kBwdKeys >= nkeys) return;
  const int nq = p.q_cnt[bh];
  const int lane = lane_id(), wave = threadIdx.x >> 6;
  const int ln = lane & 31, h = lane >> 5;
  const int* kidx = p.kidx + (long long)bh * p.npad;
  const int* qlist = p.q_idx + (long long)bh * L.N;
  const int slot0 = ktile * kBwdKeys;
  const int slot = slot0 + wave * 32 + ln;                  // this lane's key slot (< npad by construction)
  const int my_kidx = kidx[slot];
  const float c2 = L.scale * kLog2e;

  // query range that can see this key tile, and the part of it that sees every key of the tile
  if (threadIdx.x == 0 || threadIdx.x == 64) {
    const int which = threadIdx.x ? 1 : 0;
    const int last_slot = min(slot0 + kBwdKeys, nkeys) - 1;
    int v;
    if (!L.causal) v = 0;
    else v = lower_pos(qlist, nq, which ? kidx[last_slot] : kidx[slot0]);
    sBound[which] = v;
  }
  __syncthreads();
  const bool has_pad = slot0 + kBwdKeys > nkeys;
  const int q_begin = sBound[0] / kBwdQ;                    // first query tile with an admissible pair
  const int q_full_pos = has_pad ? 0x7fffffff : sBound[1];  // tiles starting at or after this position need no mask
  const int n_qtiles = cdiv(nq, kBwdQ);

  // resident K, V fragments (B operands: lane = key column)
  const T* krow = static_cast<const T*>(p.Kn) + ((long long)bh * p.npad + slot) * D;
  const T* vrow = static_cast<const T*>(p.Vn) + ((long long)bh * p.npad + slot) * D;
  bf16x8 kf16[kBf16 ? D / 16 : 1], vf16[kBf16 ? D / 16 : 1];
  f32x4 kf32[kBf16 ? 1 : D / 8], vf32[kBf16 ? 1 : D / 8];
  if constexpr (kBf16) {
#pragma unroll
    for (int ks = 0; ks < D / 16; ++ks) {
      kf16[ks] = *reinterpret_cast<const bf16x8*>(krow + ks * 16 + h * 8);
      vf16[ks] = *reinterpret_cast<const bf16x8*>(vrow + ks * 16 + h * 8);
    }
  } else {
#pragma unroll
    for (int ks = 0; ks < D / 8; ++ks) {
      kf32[ks] = *reinterpret_cast<const f32x4*>(krow + ks * 8 + h * 4);
      vf32[ks] = *reinterpret_cast<const f32x4*>(vrow + ks * 8 + h * 4);
    }
  }

  f32x16 dk[D / 32], dv[D / 32];
#pragma unroll
  for (int db = 0; db < D / 32; ++db)
#pragma unroll
    for (int r = 0; r < 16; ++r) {
      dk[db][r] = 0.f;
      dv[db][r] = 0.f;
    }

  // ---- staging of a 64-query tile
  constexpr int E = Elem<T>::kPer16B;
  constexpr int CPR = D / E;
  constexpr int kChunks = kBwdQ * CPR / kThreads;
  const T* qbase = static_cast<const T*>(p.Q) + b * L.qs[0] + i * L.qs[1];
  const T* gbase = static_cast<const T*>(p.dO) + b * L.qs[0] + i * L.qs[1];
  const T* qt = static_cast<const T*>(p.Qt) + (long long)bh * p.nqpad * D;
  const T* gt = static_cast<const T*>(p.dOt) + (long long)bh * p.nqpad * D;
  const float* lsec = p.lse2c + (long long)bh * p.nqpad;
  const float* delc = p.deltac + (long long)bh * p.nqpad;
  u32x4 stQ[kChunks], stG[kChunks], stQt[kBf16 ? kChunks : 1], stGt[kBf16 ? kChunks : 1];
  float stL = 0.f, stD = 0.f;
  int stI = -1;
  const u32x4 zero4 = {0u, 0u, 0u, 0u};

  auto load_tile = [&](int t) {
    const int pos0 = t * kBwdQ;
#pragma unroll
    for (int c = 0; c < kChunks; ++c) {
      const int ch = threadIdx.x + c * kThreads;
      const int row = ch / CPR, col = (ch % CPR) * E;
      const int pos = pos0 + row;
      stQ[c] = zero4;
      stG[c] = zero4;
      if (pos < nq) {
        const long long qrow = qlist[pos];
        stQ[c] = *reinterpret_cast<const u32x4*>(qbase + qrow * L.qs[2] + col);
        stG[c] = *reinterpret_cast<const u32x4*>(gbase + qrow * L.qs[2] + col);
      }
      if constexpr (kBf16) {
        stQt[c] = *reinterpret_cast<const u32x4*>(qt + (long long)pos0 * D + ch * E);
        stGt[c] = *reinterpret_cast<const u32x4*>(gt + (long long)pos0 * D + ch * E);
      }
    }
    if (threadIdx.x < kBwdQ) {
      const int pos = pos0 + threadIdx.x;
      stL = lsec[pos];
      stD = delc[pos];
      stI = pos < nq ? qlist[pos] : -1;
    }
  };
  auto store_tile = [&](int buf) {
    T* sq = reinterpret_cast<T*>(sQn_raw + buf * kNatBytes);
    T* sg = reinterpret_cast<T*>(sGn_raw + buf * kNatBytes);
#pragma unroll
    for (int c = 0; c < kChunks; ++c) {
      const int ch = threadIdx.x + c * kThreads;
      const int row = ch / CPR, col = (ch % CPR) * E;
      *reinterpret_cast<u32x4*>(sq + row * LD + col) = stQ[c];
      *reinterpret_cast<u32x4*>(sg + row * LD + col) = stG[c];
      if constexpr (kBf16) {
        *reinterpret_cast<u32x4*>(reinterpret_cast<T*>(sQt_raw + buf * kPackBytes) + ch * E) = stQt[c];
        *reinterpret_cast<u32x4*>(reinterpret_cast<T*>(sGt_raw + buf * kPackBytes) + ch * E) = stGt[c];
      }
    }
    if (threadIdx.x < kBwdQ) {
      sLse[buf][threadIdx.x] = stL;
      sDel[buf][threadIdx.x] = stD;
      sQi[buf][threadIdx.x] = stI;
    }
  };

  auto compute_tile = [&](int buf, bool masked) {
    const T* sq = reinterpret_cast<const T*>(sQn_raw + buf * kNatBytes);
    const T* sg = reinterpret_cast<const T*>(sGn_raw + buf * kNatBytes);
#pragma unroll
    for (int qb = 0; qb < kBwdQ / 32; ++qb) {
      f32x16 s, dp;
#pragma unroll
      for (int r = 0; r < 16; ++r) {
        s[r] = 0.f;
        dp[r] = 0.f;
      }
      if constexpr (kBf16) {
#pragma unroll
        for (int ks = 0; ks < D / 16; ++ks) {
          const bf16x8 qa = *reinterpret_cast<const bf16x8*>(sq + (qb * 32 + ln) * LD + ks * 16 + h * 8);
          s = __builtin_amdgcn_mfma_f32_32x32x16_bf16(qa, kf16[ks], s, 0, 0, 0);
          const bf16x8 ga = *reinterpret_cast<const bf16x8*>(sg + (qb * 32 + ln) * LD + ks * 16 + h * 8);
          dp = __builtin_amdgcn_mfma_f32_32x32x16_bf16(ga, vf16[ks], dp, 0, 0, 0);
        }
      } else {
#pragma unroll
        for (int ks = 0; ks < D / 8; ++ks) {
          const f32x4 qa = *reinterpret_cast<const f32x4*>(sq + (qb * 32 + ln) * LD + ks * 8 + h * 4);
          const f32x4 ga = *reinterpret_cast<const f32x4*>(sg + (qb * 32 + ln) * LD + ks * 8 + h * 4);
#pragma unroll
          for (int e = 0; e < 4; ++e) {
            s = __builtin_amdgcn_mfma_f32_32x32x2f32(qa[e], kf32[ks][e], s, 0, 0, 0);
            dp = __builtin_amdgcn_mfma_f32_32x32x2f32(ga[e], vf32[ks][e], dp, 0, 0, 0);
          }
        }
      }
      // accumulator rows are queries 8 (r/4) + 4 h + r%4 of this block, the column is this lane's key
#pragma unroll
      for (int q4 = 0; q4 < 4; ++q4) {
        const int qo = qb * 32 + 8 * q4 + 4 * h;
        const f32x4 l4 = *reinterpret_cast<const f32x4*>(&sLse[buf][qo]);
        const f32x4 d4 = *reinterpret_cast<const f32x4*>(&sDel[buf][qo]);
        i32x4 qi4 = {0, 0, 0, 0};
        if (masked) qi4 = *reinterpret_cast<const i32x4*>(&sQi[buf][qo]);
#pragma unroll
        for (int e = 0; e < 4; ++e) {
          const int r = q4 * 4 + e;
          float pv = fast_exp2(fmaf(s[r], c2, -l4[e]));
          if (masked) {
            const int qcmp = L.causal ? qi4[e] : kPadKeyIndex - 1;
            if (my_kidx > qcmp) pv = 0.f;
          }
          s[r] = pv;
          dp[r] = pv * (dp[r] - d4[e]);
        }
      }
      if constexpr (kBf16) {
        const T* sqt = reinterpret_cast<const T*>(sQt_raw + buf * kPackBytes);
        const T* sgt = reinterpret_cast<const T*>(sGt_raw + buf * kPackBytes);
#pragma unroll
        for (int u = 0; u < 2; ++u) {
          const int t16 = qb * 2 + u;
          const bf16x8 pf = pack8(s, u * 8);
          const bf16x8 dsf = pack8(dp, u * 8);
#pragma unroll
          for (int db = 0; db < D / 32; ++db) {
            const bf16x8 ga = *reinterpret_cast<const bf16x8*>(sgt + ((t16 * 2 + h) * D + db * 32 + ln) * 8);
            dv[db] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(ga, pf, dv[db], 0, 0, 0);
            const bf16x8 qa = *reinterpret_cast<const bf16x8*>(sqt + ((t16 * 2 + h) * D + db * 32 + ln) * 8);
            dk[db] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(qa, dsf, dk[db], 0, 0, 0);
          }
        }
      } else {
#pragma unroll
        for (int r = 0; r < 16; ++r) {
          const int qrow = qb * 32 + 8 * (r >> 2) + 4 * h + (r & 3);
#pragma unroll
          for (int db = 0; db < D / 32; ++db) {
            dv[db] = __builtin_amdgcn_mfma_f32_32x32x2f32(sg[qrow * LD + db * 32 + ln], s[r], dv[db], 0, 0, 0);
            dk[db] = __builtin_amdgcn_mfma_f32_32x32x2f32(sq[qrow * LD + db * 32 + ln], dp[r], dk[db], 0, 0, 0);
          }
        }
      }
    }
  };

  if (q_begin < n_qtiles) {
    if constexpr (kBf16) {
      load_tile(q_begin);
      store_tile(0);
      __syncthreads();
      for (int t = q_begin; t < n_qtiles; ++t) {
        const int buf = (t - q_begin) & 1;
        if (t + 1 < n_qtiles) load_tile(t + 1);
        compute_tile(buf, t * kBwdQ < q_full_pos || (t + 1) * kBwdQ > nq);
        if (t + 1 < n_qtiles) store_tile(buf ^ 1);
        __syncthreads();
      }
    } else {
      for (int t = q_begin; t < n_qtiles; ++t) {
        __syncthreads();
        load_tile(t);
        store_tile(0);
        __syncthreads();
        compute_tile(0, t * kBwdQ < q_full_pos || (t + 1) * kBwdQ > nq);
      }
    }
  }

  // ---- write dK' (scaled) and dV' for this lane's key slot; accumulator rows are d
  float* dkrow = p.dKp + ((long long)bh * p.npad + slot) * D;
  float* dvrow = p.dVp + ((long long)bh * p.npad + slot) * D;
#pragma unroll
  for (int db = 0; db < D / 32; ++db)
#pragma unroll
    for (int q4 = 0; q4 < 4; ++q4) {
      const int d = db * 32 + 8 * q4 + 4 * h;
      f32x4 a = {dk[db][q4 * 4] * L.scale, dk[db][q4 * 4 + 1] * L.scale, dk[db][q4 * 4 + 2] * L.scale,
                 dk[db][q4 * 4 + 3] * L.scale};
      f32x4 c = {dv[db][q4 * 4], dv[db][q4 * 4 + 1], dv[db][q4 * 4 + 2], dv[db][q4 * 4 + 3]};
      *reinterpret_cast<f32x4*>(dkrow + d) = a;
      *reinterpret_cast<f32x4*>(dvrow + d) = c;
    }
}

// ------------------------------------------------------------------ dQ

template <typename T, int D>
__global__ __launch_bounds__(kThreads, 1) void attn_bwd_dq_kernel(BwdParams p) {
  constexpr bool kBf16 = sizeof(T) == 2;
  constexpr int LD = D + 8;
  constexpr int NBUF = kBf16 ? 2 : 1;
  constexpr int kNatBytes = kTileN * LD * (int)sizeof(T);
  constexpr int kPackBytes = kBf16 ? kTileN * D * 2 : 16;
  __shared__ __attribute__((aligned(16))) unsigned char sK_raw[NBUF * kNatBytes];
  __shared__ __attribute__((aligned(16))) unsigned char sV_raw[NBUF * kNatBytes];
  __shared__ __attribute__((aligned(16))) unsigned char sKt_raw[NBUF * kPackBytes];
  __shared__ __attribute__((aligned(16))) int sIdx[NBUF][kTileN];
  __shared__ int sBound[2];

  __shared__ int sItem;
  const Layer& L = p.L;
  const int lane = lane_id(), wave = threadIdx.x >> 6;
  const int ln = lane & 31, h = lane >> 5;

  for (;;) {                                 // persistent: one (head, query tile) per iteration
  __syncthreads();
  if (threadIdx.x == 0) sItem = sched_next(p.sched);
  __syncthreads();
  const int item = sItem;
  if (item < 0) break;
  int bh, tq;
  sched_decode(p.sched, p.order_off, item, bh, tq);
  const int b = bh / L.Hq, i = bh % L.Hq;
  const int nq = p.q_cnt[bh];
  const int nkeys = min(p.budget[budget_slot(L.bph, b, bh)], p.b_cap);
  const int* kidx = p.kidx + (long long)bh * p.npad;
  const int* qlist = p.q_idx + (long long)bh * L.N;

  const int pos_first = tq * kTileM, pos_last = min(pos_first + kTileM, nq) - 1;
  if (threadIdx.x == 0 || threadIdx.x == 64) {
    const int which = threadIdx.x ? 1 : 0;
    const int row = qlist[which ? pos_last : pos_first];
    sBound[which] = L.causal ? upper_cnt(kidx, nkeys, row) : nkeys;
  }
  __syncthreads();
  const int n_full_tiles = sBound[0] / kTileN;
  const int ntiles = cdiv(sBound[1], kTileN);

  const int qpos = pos_first + wave * 32 + ln;
  const bool qvalid = qpos < nq;
  const int qpos_c = min(qpos, nq - 1);
  const int qrow = qlist[qpos_c];
  const int qcmp = L.causal ? qrow : kPadKeyIndex - 1;
  const float lse2 = p.lse2c[(long long)bh * p.nqpad + qpos_c];
  const float delta = p.deltac[(long long)bh * p.nqpad + qpos_c];
  const float c2 = L.scale * kLog2e;
  const T* qptr = static_cast<const T*>(p.Q) + b * L.qs[0] + i * L.qs[1] + (long long)qrow * L.qs[2];
  const T* gptr = static_cast<const T*>(p.dO) + b * L.qs[0] + i * L.qs[1] + (long long)qrow * L.qs[2];
  bf16x8 qf16[kBf16 ? D / 16 : 1], gf16[kBf16 ? D / 16 : 1];
  f32x4 qf32[kBf16 ? 1 : D / 8], gf32[kBf16 ? 1 : D / 8];
  if constexpr (kBf16) {
#pragma unroll
    for (int ks = 0; ks < D / 16; ++ks) {
      qf16[ks] = *reinterpret_cast<const bf16x8*>(qptr + ks * 16 + h * 8);
      gf16[ks] = *reinterpret_cast<const bf16x8*>(gptr + ks * 16 + h * 8);
    }
  } else {
#pragma unroll
    for (int ks = 0; ks < D / 8; ++ks) {
      qf32[ks] = *reinterpret_cast<const f32x4*>(qptr + ks * 8 + h * 4);
      gf32[ks] = *reinterpret_cast<const f32x4*>(gptr + ks * 8 + h * 4);
    }
  }
  f32x16 dq[D / 32];
#pragma unroll
  for (int db = 0; db < D / 32; ++db)
#pragma unroll
    for (int r = 0; r < 16; ++r) dq[db][r] = 0.f;

  constexpr int E = Elem<T>::kPer16B;
  constexpr int CPR = D / E;
  constexpr int kChunks = kTileN * CPR / kThreads;
  const T* kn = static_cast<const T*>(p.Kn) + (long long)bh * p.npad * D;
  const T* vn = static_cast<const T*>(p.Vn) + (long long)bh * p.npad * D;
  const T* kt = static_cast<const T*>(p.Kt) + (long long)bh * p.npad * D;
  u32x4 stK[kChunks], stV[kChunks], stKt[kBf16 ? kChunks : 1];
  i32x4 stI;

  auto load_tile = [&](int t) {
#pragma unroll
    for (int c = 0; c < kChunks; ++c) {
      const int ch = threadIdx.x + c * kThreads;
      stK[c] = *reinterpret_cast<const u32x4*>(kn + (long long)t * kTileN * D + ch * E);
      stV[c] = *reinterpret_cast<const u32x4*>(vn + (long long)t * kTileN * D + ch * E);
      if constexpr (kBf16) stKt[c] = *reinterpret_cast<const u32x4*>(kt + (long long)t * kTileN * D + ch * E);
    }
    if (threadIdx.x < kTileN / 4) stI = *reinterpret_cast<const i32x4*>(kidx + t * kTileN + threadIdx.x * 4);
  };
  auto store_tile = [&](int buf) {
    T* sk = reinterpret_cast<T*>(sK_raw + buf * kNatBytes);
    T* sv = reinterpret_cast<T*>(sV_raw + buf * kNatBytes);
#pragma unroll
    for (int c = 0; c < kChunks; ++c) {
      const int ch = threadIdx.x + c * kThreads;
      const int row = ch / CPR, col = (ch % CPR) * E;
      *reinterpret_cast<u32x4*>(sk + row * LD + col) = stK[c];
      *reinterpret_cast<u32x4*>(sv + row * LD + col) = stV[c];
      if constexpr (kBf16) *reinterpret_cast<u32x4*>(reinterpret_cast<T*>(sKt_raw + buf * kPackBytes) + ch * E) = stKt[c];
    }
    if (threadIdx.x < kTileN / 4) *reinterpret_cast<i32x4*>(&sIdx[buf][threadIdx.x * 4]) = stI;
  };
  auto compute_tile = [&](int buf, bool masked) {
    const T* sk = reinterpret_cast<const T*>(sK_raw + buf * kNatBytes);
    const T* sv = reinterpret_cast<const T*>(sV_raw + buf * kNatBytes);
    f32x16 s[2], dp[2];
#pragma unroll
    for (int kb = 0; kb < 2; ++kb) {
#pragma unroll
      for (int r = 0; r < 16; ++r) {
        s[kb][r] = 0.f;
        dp[kb][r] = 0.f;
      }
      if constexpr (kBf16) {
#pragma unroll
        for (int ks = 0; ks < D / 16; ++ks) {
          const bf16x8 ka = *reinterpret_cast<const bf16x8*>(sk + (kb * 32 + ln) * LD + ks * 16 + h * 8);
          s[kb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(ka, qf16[ks], s[kb], 0, 0, 0);
          const bf16x8 va = *reinterpret_cast<const bf16x8*>(sv + (kb * 32 + ln) * LD + ks * 16 + h * 8);
          dp[kb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(va, gf16[ks], dp[kb], 0, 0, 0);
        }
      } else {
#pragma unroll
        for (int ks = 0; ks < D / 8; ++ks) {
          const f32x4 ka = *reinterpret_cast<const f32x4*>(sk + (kb * 32 + ln) * LD + ks * 8 + h * 4);
          const f32x4 va = *reinterpret_cast<const f32x4*>(sv + (kb * 32 + ln) * LD + ks * 8 + h * 4);
#pragma unroll
          for (int e = 0; e < 4; ++e) {
            s[kb] = __builtin_amdgcn_mfma_f32_32x32x2f32(ka[e], qf32[ks][e], s[kb], 0, 0, 0);
            dp[kb] = __builtin_amdgcn_mfma_f32_32x32x2f32(va[e], gf32[ks][e], dp[kb], 0, 0, 0);
          }
        }
      }
    }
#pragma unroll
    for (int kb = 0; kb < 2; ++kb)
#pragma unroll
      for (int q4 = 0; q4 < 4; ++q4) {
        i32x4 id = {0, 0, 0, 0};
        if (masked) id = *reinterpret_cast<const i32x4*>(&sIdx[buf][kb * 32 + 8 * q4 + 4 * h]);
#pragma unroll
        for (int e = 0; e < 4; ++e) {
          const int r = q4 * 4 + e;
          float pv = fast_exp2(fmaf(s[kb][r], c2, -lse2));
          if (masked && id[e] > qcmp) pv = 0.f;
          dp[kb][r] = pv * (dp[kb][r] - delta);
        }
      }
    if constexpr (kBf16) {
      const T* skt = reinterpret_cast<const T*>(sKt_raw + buf * kPackBytes);
#pragma unroll
      for (int t16 = 0; t16 < 4; ++t16) {
        const bf16x8 dsf = pack8(dp[t16 >> 1], (t16 & 1) * 8);
#pragma unroll
        for (int db = 0; db < D / 32; ++db) {
          const bf16x8 ka = *reinterpret_cast<const bf16x8*>(skt + ((t16 * 2 + h) * D + db * 32 + ln) * 8);
          dq[db] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(ka, dsf, dq[db], 0, 0, 0);
        }
      }
    } else {
#pragma unroll
      for (int kb = 0; kb < 2; ++kb)
#pragma unroll
        for (int r = 0; r < 16; ++r) {
          const int ks_slot = kb * 32 + 8 * (r >> 2) + 4 * h + (r & 3);
#pragma unroll
          for (int db = 0; db < D / 32; ++db)
            dq[db] = __builtin_amdgcn_mfma_f32_32x32x2f32(sk[ks_slot * LD + db * 32 + ln], dp[kb][r], dq[db], 0, 0, 0);
        }
    }
  };

  if (ntiles > 0) {
    if constexpr (kBf16) {
      load_tile(0);
      store_tile(0);
      __syncthreads();
      for (int t = 0; t < ntiles; ++t) {
        if (t + 1 < ntiles) load_tile(t + 1);
        compute_tile(t & 1, t >= n_full_tiles);
        if (t + 1 < ntiles) store_tile((t + 1) & 1);
        __syncthreads();
      }
    } else {
      for (int t = 0; t < ntiles; ++t) {
        __syncthreads();
        load_tile(t);
        store_tile(0);
        __syncthreads();
        compute_tile(0, t >= n_full_tiles);
      }
    }
  }
  if (qvalid) {
    T* optr = static_cast<T*>(p.dQ) + b * L.qs[0] + i * L.qs[1] + (long long)qrow * L.qs[2];
#pragma unroll
    for (int db = 0; db < D / 32; ++db)
#pragma unroll
      for (int q4 = 0; q4 < 4; ++q4) {
        const int d = db * 32 + 8 * q4 + 4 * h;
        const float v0 = dq[db][q4 * 4 + 0] * L.scale, v1 = dq[db][q4 * 4 + 1] * L.scale;
        const float v2 = dq[db][q4 * 4 + 2] * L.scale, v3 = dq[db][q4 * 4 + 3] * L.scale;
        if constexpr (kBf16) {
          uint2 w;
          w.x = pack_bf16x2(v0, v1);
          w.y = pack_bf16x2(v2, v3);
          *reinterpret_cast<uint2*>(optr + d) = w;
        } else {
          f32x4 w = {v0, v1, v2, v3};
          *reinterpret_cast<f32x4*>(optr + d) = w;
        }
      }
  }
  }  // work-item loop
}

// ------------------------------------------------------------------ dQ, bf16 fast path
//
// Same organisation as the bf16 forward kernel: 512 threads = 8 wavefronts x 32 kept queries (256-row work
// items from the longest-first persistent list), K / V / K^T tiles of 64 keys streamed memory -> LDS with
// LDS-DMA loads into a ring of kDqStages buffers (natural tiles unpadded with the XOR chunk swizzle), one
// barrier per tile, the loads of tile t+2 spread over the MFMAs of tile t, causal mask from the per-query
// visible-prefix count.  Per tile and wavefront: S^T = K Q^T and dP^T = V dO^T (32 MFMAs), dS^T on the
// vector ALU, dQ^T += K^T dS^T (16 MFMAs).

constexpr int kDqWaves = 8;
constexpr int kDqThreads = kDqWaves * 64;
constexpr int kDqTileM = kDqWaves * 32;
constexpr int kDqStages = 3;

constexpr int kBwdMaxMapTiles = 2048;               // key tiles of one head in the in-place variant (128k tokens)

template <int D, bool TILEMAP>
__global__ __launch_bounds__(kDqThreads, 2) void attn_bwd_dq_bf16_kernel(BwdParams p) {
  typedef u16 T;
  constexpr int CH = D / 8;                          // 16-byte chunks per natural row
  constexpr int kOpBytes = kTileN * D * 2;           // one operand tile
  constexpr int kStageBytes = 3 * kOpBytes;          // K natural, V natural, K k-packed
  constexpr int LPH = kOpBytes / 1024 / kDqWaves;    // load instructions per operand per wavefront per tile
  constexpr int LPT = 3 * LPH;
  constexpr int NB = D / 32;
  static_assert(LPH >= 1, "tile too small for the copy scheme");
  __shared__ __attribute__((aligned(1024))) unsigned char smem[kDqStages * kStageBytes];
  __shared__ int sBound[2];
  __shared__ int sItem;
  __shared__ int sTileMap[TILEMAP ? kBwdMaxMapTiles : 1];

  const Layer& L = p.L;
  const int lane = lane_id();
  const int wave = __builtin_amdgcn_readfirstlane((int)(threadIdx.x >> 6));
  const int ln = lane & 31, h = lane >> 5;
  const float c2 = L.scale * kLog2e;
  const unsigned lds_base = (unsigned)(size_t)(__attribute__((address_space(3))) unsigned char*)smem;

  unsigned ngoff[LPH], pgoff[LPH];                   // byte offsets of this lane's 16-byte chunk: natural (swizzled), packed
#pragma unroll
  for (int j = 0; j < LPH; ++j) {
    const int pchunk = (j * kDqWaves + wave) * 64 + lane;
    const int row = pchunk / CH, pc = pchunk % CH;
    ngoff[j] = (row * D + ((pc ^ (row % CH)) << 3)) * 2;
    pgoff[j] = pchunk << 4;
  }
  const int krow_b = ln * (CH * 16);
  const int khx = (h << 4) ^ ((ln % CH) << 4);
  const int plane_b = (h * D + ln) * 16;

  for (;;) {
  __syncthreads();
  if (threadIdx.x == 0) sItem = sched_next(p.sched);
  __syncthreads();
  const int item = __builtin_amdgcn_readfirstlane(sItem);   // wave-uniform, and known to be: tile bases stay in SGPRs
  if (item < 0) break;
  int bh, tq;
  sched_decode(p.sched, p.order_off, item, bh, tq);
  bh = __builtin_amdgcn_readfirstlane(bh);
  tq = __builtin_amdgcn_readfirstlane(tq);
  const int b = bh / L.Hq, i = bh % L.Hq;
  const int nq = p.q_cnt[bh];
  const int* qlist = p.q_idx + (long long)bh * L.N;
  const int* qvis = p.qvis + (long long)bh * L.N;

  const int pos_first = tq * kDqTileM, pos_last = min(pos_first + kDqTileM, nq) - 1;
  if (threadIdx.x == 0 || threadIdx.x == 64) sBound[threadIdx.x ? 1 : 0] = qvis[threadIdx.x ? pos_last : pos_first];
  __syncthreads();
  const int n_full_tiles = sBound[0] / kTileN;
  const int ntiles = cdiv(sBound[1], kTileN);
  if constexpr (TILEMAP) {                                   // this item's share of the head's tile map
    const int* tm = p.tile_map + (long long)bh * p.tile_stride;
    for (int t = threadIdx.x; t < ntiles; t += kDqThreads) sTileMap[t] = tm[t];
    __syncthreads();
  }

  const int qpos = pos_first + wave * 32 + ln;
  const bool qvalid = qpos < nq;
  const int qpos_c = min(qpos, nq - 1);
  const int qrow = qlist[qpos_c];
  const int qvisible = qvis[qpos_c] - 4 * h;
  const float lse2 = p.lse2c[(long long)bh * p.nqpad + qpos_c];
  const float delta = p.deltac[(long long)bh * p.nqpad + qpos_c];
  const T* qptr = static_cast<const T*>(p.Q) + b * L.qs[0] + i * L.qs[1] + (long long)qrow * L.qs[2];
  const T* gptr = static_cast<const T*>(p.dO) + b * L.qs[0] + i * L.qs[1] + (long long)qrow * L.qs[2];
  bf16x8 qf[D / 16], gf[D / 16];
#pragma unroll
  for (int ks = 0; ks < D / 16; ++ks) {
    qf[ks] = *reinterpret_cast<const bf16x8*>(qptr + ks * 16 + h * 8);
    gf[ks] = *reinterpret_cast<const bf16x8*>(gptr + ks * 16 + h * 8);
  }
  float lse2r = lse2, deltar = delta;
  // finish every ordinary load here: a compiler-placed wait inside the tile loop would drain the ring
#pragma unroll
  for (int ks = 0; ks < D / 16; ++ks) {
    asm volatile("" : "+v"(qf[ks]));
    asm volatile("" : "+v"(gf[ks]));
  }
  asm volatile("" : "+v"(lse2r), "+v"(deltar));

  f32x16 dq[NB];
#pragma unroll
  for (int db = 0; db < NB; ++db)
#pragma unroll
    for (int r = 0; r < 16; ++r) dq[db][r] = 0.f;

  const int bhx = TILEMAP ? b * L.Hkv + i / L.G : bh;
  const T* kn = static_cast<const T*>(p.Kn) + (long long)bhx * p.npad_kv * D;
  const T* vn = static_cast<const T*>(p.Vn) + (long long)bhx * p.npad_kv * D;
  const T* kt = static_cast<const T*>(p.Kt) + (long long)bhx * p.npad_kv * D;
  auto issue_part = [&](int t, int part) {
    const int op = part / LPH, j = part % LPH;
    const unsigned dst = lds_base + (unsigned)(t % kDqStages) * kStageBytes + op * kOpBytes + (j * kDqWaves + wave) * 1024;
    // where tile t of the key list lives (wave-uniform: the tile base stays in scalar registers)
    const int src = TILEMAP ? __builtin_amdgcn_readfirstlane(sTileMap[t]) : t;
    const long long tile_off = (long long)src * kTileN * D;
    if (op == 0) gload_lds16(kn + tile_off, ngoff[j], dst);
    else if (op == 1) gload_lds16(vn + tile_off, ngoff[j], dst);
    else gload_lds16(kt + tile_off, pgoff[j], dst);
  };
  auto issue_tile = [&](int t) {
#pragma unroll
    for (int j = 0; j < LPT; ++j) issue_part(t, j);
  };

  constexpr int NA = 4 * (D / 16);           // MFMAs of the S^T and dP^T tiles: 2 key blocks x D/16 k-steps x 2
  constexpr int NC = 4 * NB;                 // MFMAs of the dQ^T update: 4 key steps x D/32 row blocks
  constexpr int kAhead = 2;
  static_assert(NA % (2 * LPH) == 0 && NC % LPH == 0, "loads are spread evenly over the MFMAs");
  const f32x16 zero16 = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};

  auto compute_tile = [&](int t, int pre, bool masked) {
    const unsigned char* st = smem + (t % kDqStages) * kStageBytes;
    // chunk c of phase A: key block kb, k-step ks, operand (0: K for S, 1: V for dP)
    auto afrag = [&](int c) {
      const int which = c % 2, ks = (c / 2) % (D / 16), kb = c / (D / 8);
      return *reinterpret_cast<const bf16x8*>(st + which * kOpBytes + kb * (32 * CH * 16) + krow_b + ((ks << 5) ^ khx));
    };
    auto cfrag = [&](int c) {
      const int t16 = c / NB, db = c % NB;
      return *reinterpret_cast<const bf16x8*>(st + 2 * kOpBytes + plane_b + (t16 * 2 * D + db * 32) * 16);
    };
    f32x16 s[2], dp[2];
    bf16x8 fa[kAhead];
#pragma unroll
    for (int c = 0; c < kAhead; ++c) fa[c] = afrag(c);
#pragma unroll
    for (int c = 0; c < NA; ++c) {
      const int which = c % 2, ks = (c / 2) % (D / 16), kb = c / (D / 8);
      __builtin_amdgcn_sched_barrier(0);
      if (which == 0) s[kb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fa[c % kAhead], qf[ks], ks == 0 ? zero16 : s[kb], 0, 0, 0);
      else dp[kb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fa[c % kAhead], gf[ks], ks == 0 ? zero16 : dp[kb], 0, 0, 0);
      if (c + kAhead < NA) fa[c % kAhead] = afrag(c + kAhead);
      if (c % (NA / (2 * LPH)) == 0 && pre >= 0) issue_part(pre, c / (NA / (2 * LPH)));      // K and V parts of tile t+2
    }
    __builtin_amdgcn_sched_barrier(0);
    // dS^T = P^T (dP^T - delta); the lane's query fixes lse and delta, the register fixes the key.  Only the tiles
    // at the causal diagonal of the item pay for the position compares (a wavefront-uniform branch).
    bf16x8 fc[kAhead];
#pragma unroll
    for (int c = 0; c < kAhead; ++c) fc[c] = cfrag(c);
    bf16x8 dsf[4];
    auto weights = [&](auto with_mask) {
      const int rel = qvisible - t * kTileN;
#pragma unroll
      for (int kb = 0; kb < 2; ++kb) {
#pragma unroll
        for (int r = 0; r < 16; ++r) {
          float pv = fast_exp2(fmaf(s[kb][r], c2, -lse2r));
          if (decltype(with_mask)::value && kb * 32 + 8 * (r >> 2) + (r & 3) >= rel) pv = 0.f;
          dp[kb][r] = pv * (dp[kb][r] - deltar);
        }
        dsf[kb * 2] = pack8(dp[kb], 0);
        dsf[kb * 2 + 1] = pack8(dp[kb], 8);
      }
    };
    if (masked) weights(std::true_type{});
    else weights(std::false_type{});
#pragma unroll
    for (int c = 0; c < NC; ++c) {
      const int t16 = c / NB, db = c % NB;
      __builtin_amdgcn_sched_barrier(0);
      dq[db] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fc[c % kAhead], dsf[t16], dq[db], 0, 0, 0);
      if (c + kAhead < NC) fc[c % kAhead] = cfrag(c + kAhead);
      if (c % (NC / LPH) == 0 && pre >= 0) issue_part(pre, 2 * LPH + c / (NC / LPH));            // K^T parts
    }
    __builtin_amdgcn_sched_barrier(0);
  };

  // Ring of kDqStages buffers, one barrier per tile: at the top of step t the tiles up to t+1 have been
  // issued; after its barrier everyone is done with tile t-1, whose buffer takes tile t+2.
  static_assert(kDqStages == 3, "the wait counts assume this ring depth");
  if (ntiles > 0) {
    wait_vmcnt<0>();
    issue_tile(0);
    if (ntiles > 1) issue_tile(1);
    for (int t = 0; t < ntiles; ++t) {
      if (t + 1 < ntiles) wait_vmcnt<LPT>();
      else wait_vmcnt<0>();
      __syncthreads();
      compute_tile(t, t + 2 < ntiles ? t + 2 : -1, t >= n_full_tiles);
    }
  }

  if (qvalid) {
    T* optr = static_cast<T*>(p.dQ) + b * L.qs[0] + i * L.qs[1] + (long long)qrow * L.qs[2];
#pragma unroll
    for (int db = 0; db < NB; ++db)
#pragma unroll
      for (int q4 = 0; q4 < 4; ++q4) {
        const int d = db * 32 + 8 * q4 + 4 * h;
        uint2 w;
        w.x = pack_bf16x2(dq[db][q4 * 4 + 0] * L.scale, dq[db][q4 * 4 + 1] * L.scale);
        w.y = pack_bf16x2(dq[db][q4 * 4 + 2] * L.scale, dq[db][q4 * 4 + 3] * L.scale);
        *reinterpret_cast<uint2*>(optr + d) = w;
      }
  }
  }  // work-item loop
}

// ------------------------------------------------------------------ dK' and dV', bf16 fast path
//
// Two kernels of the same shape as the dQ kernel with the roles of keys and queries swapped: a workgroup
// of 8 wavefronts owns 256 packed keys of one query head (32 per wavefront, K and V fragments resident in
// registers) and streams 64-query tiles of the packed kept rows memory -> LDS with LDS-DMA loads into a
// ring.  Keeping dK and dV in one kernel needs 192 registers for the resident fragments and the two
// accumulators alone, which does not fit two wavefronts per SIMD; split, each kernel does, and the price
// is that S = Q K^T is computed twice (8 GEMMs per pair in the whole backward instead of 7).
//   MODE 0 (dK): streams Q, dO (natural) and Q (k-packed):  S, dP -> dS;  dK'^T += Q^T dS
//   MODE 1 (dV): streams Q (natural) and dO (k-packed):     S -> P;       dV'^T += dO^T P
// lse * log2e and delta of the tile's queries come with the tile (LDS-DMA of 4 bytes per lane); the causal
// mask is a comparison of the query position with the first position that sees the lane's key.

constexpr int kKeyWaves = 8;
constexpr int kKeyThreads = kKeyWaves * 64;
constexpr int kKeyTile = kKeyWaves * 32;     // packed keys per workgroup
constexpr int kKeyQ = 64;                    // queries per streamed tile
// A key tile seen by many query tiles (the first tiles of a head that keeps every query: 512 query tiles at 32k,
// against a few dozen for most workgroups) is shared by several workgroups, each with a contiguous range of the
// query tiles and a partial-gradient plane of its own; the group reduction adds the planes in split order.
constexpr int kKeySplitLen = 128;            // query tiles per split, at least (64..128 measure alike, 32 and 256 worse)
constexpr int kKeyMaxSplits = 4;             // at most 8: a work item carries the split in 3 bits
__host__ __device__ inline int key_tile_splits(int n_qtiles, int max_splits, int split_len) {
  const int s = n_qtiles / split_len;
  return s < 1 ? 1 : (s > max_splits ? max_splits : s);
}

// Work items of the key kernels: (head, key tile, split), in dispatch order -- heads in groups of p.head_group,
// inside a group key tile by key tile (the first key tiles, seen by the most queries, first), the splits of a
// tile side by side.  Slot i of that order decodes to an item; most slots are empty (key tiles beyond a head's
// budget, splits a tile does not need), so one workgroup compacts the live ones into a list that the
// persistent key kernels pull from: an empty workgroup would still wait for a whole CU's LDS.
constexpr int kKeyListHeader = 4;
__device__ __forceinline__ int key_slot_item(const BwdParams& p, long long i) {
  const Layer& L = p.L;
  const int BH = L.B * L.Hq, nkt = p.npad / kKeyTile;
  const long long per_group = (long long)p.head_group * nkt * p.nsplit;
  const int grp = (int)(i / per_group);
  const int within = (int)(i % per_group);
  const int heads_here = min(p.head_group, BH - grp * p.head_group);
  if (heads_here <= 0) return -1;
  const int kts = within / heads_here, bh = grp * p.head_group + within % heads_here;
  const int ktile = kts / p.nsplit, sp = kts % p.nsplit;
  if (ktile >= nkt) return -1;
  const int nkeys = min(p.budget[budget_slot(L.bph, bh / L.Hq, bh)], p.b_cap);
  if (ktile * kKeyTile >= nkeys) return -1;
  if (sp > 0) {
    const int first = p.kfirst[(long long)bh * p.npad + ktile * kKeyTile];
    if (sp >= key_tile_splits(cdiv(p.q_cnt[bh], kKeyQ) - first / kKeyQ, p.nsplit, p.split_len)) return -1;
  }
  return (bh << 16) | (ktile << 3) | sp;
}

// one workgroup of 1024 threads; stable compaction of the live slots
__global__ __launch_bounds__(1024) void key_list_kernel(BwdParams p, long long n_slots) {
  __shared__ int wave_cnt[16];
  __shared__ int base;
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  if (threadIdx.x == 0) base = 0;
  __syncthreads();
  for (long long i0 = 0; i0 < n_slots; i0 += 1024) {
    const long long i = i0 + threadIdx.x;
    const int item = i < n_slots ? key_slot_item(p, i) : -1;
    const unsigned long long live = __ballot(item >= 0);
    if (lane == 0) wave_cnt[wave] = __popcll(live);
    __syncthreads();
    int before = base;
    for (int w = 0; w < wave; ++w) before += wave_cnt[w];
    if (item >= 0) p.klist[kKeyListHeader + before + __popcll(live & ((1ull << lane) - 1ull))] = item;
    __syncthreads();
    if (threadIdx.x == 0) {
      int t = base;
      for (int w = 0; w < 16; ++w) t += wave_cnt[w];
      base = t;
    }
    __syncthreads();
  }
  if (threadIdx.x == 0) {
    p.klist[0] = 0;
    p.klist[1] = 0;
    p.klist[2] = base;
  }
}

template <int D, int MODE, bool TILEMAP>
__global__ __launch_bounds__(kKeyThreads, 2) void attn_bwd_key_bf16_kernel(BwdParams p) {
  typedef u16 T;
  constexpr int CH = D / 8;
  constexpr int NB = D / 32;
  constexpr int NOPS = MODE == 0 ? 3 : 2;            // streamed operand tiles
  constexpr int kStages = MODE == 0 ? 3 : 4;
  constexpr int kAheadTiles = kStages - 1;
  constexpr int NSMALL = MODE == 0 ? 2 : 1;          // wavefronts that also bring a 256-byte per-query array
  constexpr int kOpBytes = kKeyQ * D * 2;
  constexpr int kSmallOff = NOPS * kOpBytes;
  constexpr int kStageBytes = kSmallOff + 1024;
  constexpr int LPH = kOpBytes / 1024 / kKeyWaves;
  constexpr int LPT = NOPS * LPH;
  static_assert(LPH >= 1, "tile too small for the copy scheme");
  __shared__ __attribute__((aligned(1024))) unsigned char smem[kStages * kStageBytes];
  __shared__ int sBound[2];
  __shared__ int sItem;

  const Layer& L = p.L;
  const int lane = lane_id();
  const int wave = __builtin_amdgcn_readfirstlane((int)(threadIdx.x >> 6));
  const int ln = lane & 31, h = lane >> 5;
  const float c2 = L.scale * kLog2e;
  const unsigned lds_base = (unsigned)(size_t)(__attribute__((address_space(3))) unsigned char*)smem;

  for (;;) {                                   // persistent: one item of the work list per iteration
  __syncthreads();                             // LDS of the previous item is no longer read
  if (threadIdx.x == 0) {
    const int k = atomicAdd(&p.klist[MODE], 1);
    sItem = k < p.klist[2] ? p.klist[kKeyListHeader + k] : -1;
  }
  __syncthreads();
  const int item = __builtin_amdgcn_readfirstlane(sItem);
  if (item < 0) break;
  const int bh = item >> 16, ktile = (item >> 3) & 0x1fff, sp = item & 7;
  const int b = bh / L.Hq;
  const int nkeys = min(p.budget[budget_slot(L.bph, b, bh)], p.b_cap);
  const int nq = p.q_cnt[bh];
  const int slot0 = ktile * kKeyTile;
  const int slot = slot0 + wave * 32 + ln;                  // this lane's key slot (< npad by construction)
  const int* kfirst = p.kfirst + (long long)bh * p.npad;
  if (threadIdx.x == 0 || threadIdx.x == 64) {
    const int last_slot = min(slot0 + kKeyTile, nkeys) - 1;
    sBound[threadIdx.x ? 1 : 0] = kfirst[threadIdx.x ? last_slot : slot0];
  }
  int my_first = kfirst[slot];
  __syncthreads();
  const bool has_pad = slot0 + kKeyTile > nkeys;
  const int q_full_pos = has_pad ? 0x7fffffff : sBound[1];  // tiles starting at or after this position need no mask
  const int n_qtiles = cdiv(nq, kKeyQ);
  const int q_first = sBound[0] / kKeyQ;                    // first query tile with an admissible pair
  const int n_all = n_qtiles - q_first;
  const int n_sp = key_tile_splits(n_all, p.nsplit, p.split_len);
  const int per_split = cdiv(n_all, n_sp);
  const int q_begin = q_first + sp * per_split;             // this workgroup's query tiles: [q_begin, q_begin + n)

  // resident K (and V) fragments: B operands, lane = key column
  long long kv_row = (long long)bh * p.npad + slot;
  if constexpr (TILEMAP) {           // the slot's row inside its KV head's token-ordered copy (slots past the map: masked)
    const int t = slot / kTileN;
    const int src = t < p.tile_stride ? p.tile_map[(long long)bh * p.tile_stride + t] : 0;
    kv_row = (long long)(b * L.Hkv + (bh % L.Hq) / L.G) * p.npad_kv + (long long)src * kTileN + slot % kTileN;
  }
  const T* krow = static_cast<const T*>(p.Kn) + kv_row * D;
  const T* vrow = static_cast<const T*>(p.Vn) + kv_row * D;
  bf16x8 kf[D / 16], vf[MODE == 0 ? D / 16 : 1];
#pragma unroll
  for (int ks = 0; ks < D / 16; ++ks) {
    kf[ks] = *reinterpret_cast<const bf16x8*>(krow + ks * 16 + h * 8);
    if (MODE == 0) vf[ks] = *reinterpret_cast<const bf16x8*>(vrow + ks * 16 + h * 8);
  }
  // finish every ordinary load here: a compiler-placed wait inside the tile loop would drain the ring
#pragma unroll
  for (int ks = 0; ks < D / 16; ++ks) {
    asm volatile("" : "+v"(kf[ks]));
    if (MODE == 0) asm volatile("" : "+v"(vf[ks]));
  }
  asm volatile("" : "+v"(my_first));
  const int first_h = my_first - 4 * h;

  f32x16 acc[NB];
#pragma unroll
  for (int db = 0; db < NB; ++db)
#pragma unroll
    for (int r = 0; r < 16; ++r) acc[db][r] = 0.f;

  unsigned ngoff[LPH], pgoff[LPH];                          // byte offsets of this lane's chunk: natural (swizzled), packed
#pragma unroll
  for (int j = 0; j < LPH; ++j) {
    const int pchunk = (j * kKeyWaves + wave) * 64 + lane;
    const int row = pchunk / CH, pc = pchunk % CH;
    ngoff[j] = (row * D + ((pc ^ (row % CH)) << 3)) * 2;      // bytes
    pgoff[j] = pchunk << 4;
  }
  const int krow_b = ln * (CH * 16);
  const int khx = (h << 4) ^ ((ln % CH) << 4);
  const int plane_b = (h * D + ln) * 16;

  const T* qn = static_cast<const T*>(p.Qn) + (long long)bh * p.nqpad * D;
  const T* gn = static_cast<const T*>(p.dOn) + (long long)bh * p.nqpad * D;
  const T* qt = static_cast<const T*>(p.Qt) + (long long)bh * p.nqpad * D;
  const T* gt = static_cast<const T*>(p.dOt) + (long long)bh * p.nqpad * D;
  const float* lsec = p.lse2c + (long long)bh * p.nqpad;
  const float* delc = p.deltac + (long long)bh * p.nqpad;
  const bool has_small = wave < NSMALL;

  // u = tile index relative to q_begin (ring position); operand order: MODE 0: Q nat, dO nat, Q packed; MODE 1: Q nat, dO packed
  auto issue_part = [&](int u, int part) {
    const int op = part / LPH, j = part % LPH;
    const unsigned dst = lds_base + (unsigned)(u % kStages) * kStageBytes + op * kOpBytes + (j * kKeyWaves + wave) * 1024;
    const long long tile_off = (long long)(q_begin + u) * kKeyQ * D;
    if (op == 0) gload_lds16(qn + tile_off, ngoff[j], dst);
    else if (MODE == 0 && op == 1) gload_lds16(gn + tile_off, ngoff[j], dst);
    else if (MODE == 0) gload_lds16(qt + tile_off, pgoff[j], dst);
    else gload_lds16(gt + tile_off, pgoff[j], dst);
  };
  auto issue_small = [&](int u) {
    if (!has_small) return;
    const unsigned dst = lds_base + (unsigned)(u % kStages) * kStageBytes + kSmallOff + wave * 256;
    const float* src = (wave == 0 ? lsec : delc) + (long long)(q_begin + u) * kKeyQ + lane;
    gload_lds4(src, dst);
  };
  auto issue_tile = [&](int u) {
#pragma unroll
    for (int j = 0; j < LPT; ++j) issue_part(u, j);
    issue_small(u);
  };

  constexpr int NA = (MODE == 0 ? 2 : 1) * (D / 16);   // MFMAs of phase A per 32-query block
  constexpr int NC = 4 * NB;
  constexpr int kAhead = 2;                    // fragment reads run this many MFMAs ahead
  const f32x16 zero16 = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};

  auto compute_tile = [&](int u, int pre, bool masked) {
    const unsigned char* st = smem + (u % kStages) * kStageBytes;
    const int rel = first_h - (q_begin + u) * kKeyQ;                 // query positions below rel do not see this key
    auto cfrag = [&](int c) {
      const int t16 = c / NB, db = c % NB;
      return *reinterpret_cast<const bf16x8*>(st + (NOPS - 1) * kOpBytes + plane_b + (t16 * 2 * D + db * 32) * 16);
    };
    // phase A of query block qb: S^T (and dP^T) of its 32 queries; under(c) is vector work placed behind MFMA c
    auto phase_a = [&](int qb, f32x16& s, f32x16& dp, auto under) {
      // chunk c: k-step ks, operand (0: Q for S, 1: dO for dP)
      auto afrag = [&](int c) {
        const int which = MODE == 0 ? c % 2 : 0, ks = MODE == 0 ? c / 2 : c;
        return *reinterpret_cast<const bf16x8*>(st + which * kOpBytes + qb * (32 * CH * 16) + krow_b + ((ks << 5) ^ khx));
      };
      bf16x8 fa[kAhead];
#pragma unroll
      for (int c = 0; c < kAhead; ++c) fa[c] = afrag(c);
#pragma unroll
      for (int c = 0; c < NA; ++c) {
        const int which = MODE == 0 ? c % 2 : 0, ks = MODE == 0 ? c / 2 : c;
        __builtin_amdgcn_sched_barrier(0);
        if (which == 0) s = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fa[c % kAhead], kf[ks], ks == 0 ? zero16 : s, 0, 0, 0);
        else dp = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fa[c % kAhead], vf[MODE == 0 ? ks : 0], ks == 0 ? zero16 : dp, 0, 0, 0);
        if (c + kAhead < NA) fa[c % kAhead] = afrag(c + kAhead);
        under(c);
        // natural operand parts of the tile to prefetch: NOPS - 1 operands x LPH parts over 2 * NA MFMAs
        constexpr int kParts = (NOPS - 1) * LPH, kEvery = 2 * NA / kParts;
        if ((qb * NA + c) % kEvery == 0 && pre >= 0) issue_part(pre, (qb * NA + c) / kEvery);
      }
      __builtin_amdgcn_sched_barrier(0);
    };
    // weights (MODE 1) or dS (MODE 0) of four queries of block qb, in place: accumulator rows are queries
    // 8 (r/4) + 4 h + r%4 of the block, the column is this lane's key.  Only the query tiles at the causal diagonal
    // of the key tile pay for the position compares (with_mask; a wavefront-uniform choice).
    auto quad = [&](auto with_mask, int qb, f32x16& s, const f32x16& dp, int q4) {
      const int qo = qb * 32 + 8 * q4 + 4 * h;
      const f32x4 l4 = *reinterpret_cast<const f32x4*>(st + kSmallOff + qo * 4);
      f32x4 d4 = {0.f, 0.f, 0.f, 0.f};
      if (MODE == 0) d4 = *reinterpret_cast<const f32x4*>(st + kSmallOff + 256 + qo * 4);
#pragma unroll
      for (int e = 0; e < 4; ++e) {
        const int r = q4 * 4 + e;
        float pv = fast_exp2(fmaf(s[r], c2, -l4[e]));
        if (decltype(with_mask)::value && qb * 32 + 8 * q4 + e < rel) pv = 0.f;
        s[r] = MODE == 0 ? pv * (dp[r] - d4[e]) : pv;
      }
    };
    // phase C of block qb: its P (or dS), as two B operands of 16 queries each, into the update
    auto phase_c = [&](int qb, const f32x16& s, auto under) {
      bf16x8 bfrag[2];
      bfrag[0] = pack8(s, 0);
      bfrag[1] = pack8(s, 8);
      bf16x8 fc[kAhead];
#pragma unroll
      for (int c = 0; c < kAhead; ++c) fc[c] = cfrag(qb * (NC / 2) + c);
#pragma unroll
      for (int c = 0; c < NC / 2; ++c) {
        const int cc = qb * (NC / 2) + c, db = cc % NB;
        __builtin_amdgcn_sched_barrier(0);
        acc[db] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fc[c % kAhead], bfrag[c / NB], acc[db], 0, 0, 0);
        if (c + kAhead < NC / 2) fc[c % kAhead] = cfrag(cc + kAhead);
        under(c);
        if (cc % (NC / LPH) == 0 && pre >= 0) issue_part(pre, (NOPS - 1) * LPH + cc / (NC / LPH));   // k-packed operand parts
      }
      __builtin_amdgcn_sched_barrier(0);
    };
    auto nothing = [](int) {};
    auto run = [&](auto with_mask) {
      if constexpr (MODE == 1) {
        // dV': the weights of a block run on the vector ALU under the matrix-core work of the other block -- S of
        // block 1 over the weights of block 0, the update of block 0 over the weights of block 1 (a quad of queries
        // behind every second MFMA).  Two S accumulators are live at once; this kernel has the registers for it.
        static_assert(MODE != 1 || (NA == 2 * 4 || NA == 4) && NC / 2 >= 4, "a quad per MFMA or per two");
        constexpr int kPerA = NA / 4, kPerC = (NC / 2) / 4;
        f32x16 s0, s1, none;
        phase_a(0, s0, none, nothing);
        if (pre >= 0) issue_small(pre);
        phase_a(1, s1, none, [&](int c) { if (c % kPerA == 0) quad(with_mask, 0, s0, none, c / kPerA); });
        phase_c(0, s0, [&](int c) { if (c % kPerC == 0 && c / kPerC < 4) quad(with_mask, 1, s1, none, c / kPerC); });
        phase_c(1, s1, nothing);
      } else {
#pragma unroll
        for (int qb = 0; qb < 2; ++qb) {
          f32x16 s, dp;
          phase_a(qb, s, dp, nothing);
          if (qb == 0 && pre >= 0) issue_small(pre);
#pragma unroll
          for (int q4 = 0; q4 < 4; ++q4) {
            quad(with_mask, qb, s, dp, q4);
            __builtin_amdgcn_sched_barrier(0);    // one quad of lse / delta values in registers at a time
          }
          phase_c(qb, s, nothing);                // the two blocks stay apart: their accumulators would double up
        }
      }
    };
    if (masked) run(std::true_type{});
    else run(std::false_type{});
  };

  // Ring of kStages buffers, one barrier per tile: at the top of step u the tiles up to u + kStages - 2 have
  // been issued; after its barrier everyone is done with tile u-1, whose buffer takes tile u + kStages - 1.
  const int n = min(per_split, n_qtiles - q_begin);
  if (n > 0) {
    wait_vmcnt<0>();
#pragma unroll
    for (int a = 0; a < kAheadTiles; ++a)
      if (a < n) issue_tile(a);
    for (int u = 0; u < n; ++u) {
      const int ahead = min(n - 1 - u, kAheadTiles - 1);      // tiles issued after tile u
      if (has_small) {
        if (ahead >= 2) wait_vmcnt<2 * (LPT + 1)>();
        else if (ahead == 1) wait_vmcnt<LPT + 1>();
        else wait_vmcnt<0>();
      } else {
        if (ahead >= 2) wait_vmcnt<2 * LPT>();
        else if (ahead == 1) wait_vmcnt<LPT>();
        else wait_vmcnt<0>();
      }
      __syncthreads();
      const int pos0 = (q_begin + u) * kKeyQ;
      compute_tile(u, u + kAheadTiles < n ? u + kAheadTiles : -1, pos0 < q_full_pos);
    }
  }

  // ---- write dK' (scaled) or dV' for this lane's key slot; accumulator rows are d
  float* orow = (MODE == 0 ? p.dKp : p.dVp) + sp * p.plane + ((long long)bh * p.npad + slot) * D;
  const float osc = MODE == 0 ? L.scale : 1.0f;
#pragma unroll
  for (int db = 0; db < NB; ++db)
#pragma unroll
    for (int q4 = 0; q4 < 4; ++q4) {
      const int d = db * 32 + 8 * q4 + 4 * h;
      f32x4 a = {acc[db][q4 * 4] * osc, acc[db][q4 * 4 + 1] * osc, acc[db][q4 * 4 + 2] * osc, acc[db][q4 * 4 + 3] * osc};
      *reinterpret_cast<f32x4*>(orow + d) = a;
    }
  }   // items
}

// ------------------------------------------------------------------ dK, dV = sum over the heads of a KV group

// inv[bh, token] = slot of the token in the head's selected list, -1 if it is not selected: the reduction then
// finds a head's partial row with one load instead of a binary search of dependent loads.
__global__ __launch_bounds__(256) void fill_int_kernel(int* __restrict__ p, long long n, int v) {
  const long long stride = (long long)gridDim.x * blockDim.x;
  for (long long i = (long long)blockIdx.x * blockDim.x + threadIdx.x; i < n; i += stride) p[i] = v;
}
// grid: (cdiv(b_cap, 256), B*Hq)
__global__ __launch_bounds__(256) void inverse_list_kernel(const int* __restrict__ kv_idx, const int* __restrict__ budget,
                                                           int bph, int Hq, int b_cap, int N, int* __restrict__ inv) {
  const int bh = blockIdx.y, b = bh / Hq;
  const int nkeys = min(budget[budget_slot(bph, b, bh)], b_cap);
  const int t = blockIdx.x * blockDim.x + threadIdx.x;
  if (t >= nkeys) return;
  const int tok = kv_idx[(long long)bh * b_cap + t];
  if (tok >= 0 && tok < N) inv[(long long)bh * N + tok] = t;
}


// grid: (ceil(N / rows_per_block), B*Hkv); one token row per D/4 lanes.
template <typename T, int D>
__global__ __launch_bounds__(kThreads) void attn_bwd_reduce_kernel(BwdParams p, const int* __restrict__ kv_idx,
                                                                  const int* __restrict__ inv, T* __restrict__ dK,
                                                                  T* __restrict__ dV) {
  constexpr int LPR = D / 4;
  constexpr int RPB = kThreads / LPR;
  const Layer& L = p.L;
  const int bg = blockIdx.y, b = bg / L.Hkv, g = bg % L.Hkv;
  const int c = threadIdx.x % LPR, r0 = threadIdx.x / LPR;
  const int n = blockIdx.x * RPB + r0;
  if (n >= L.N) return;
  f32x4 ak = {0.f, 0.f, 0.f, 0.f}, av = {0.f, 0.f, 0.f, 0.f};
  for (int j = 0; j < L.G; ++j) {
    const int bh = b * L.Hq + g * L.G + j;
    int pos;
    if (inv) {
      pos = inv[(long long)bh * L.N + n];                       // slot of token n in the head's list, or -1
    } else {
      const int* list = kv_idx + (long long)bh * p.b_cap;
      const int nkeys = min(p.budget[budget_slot(L.bph, b, bh)], p.b_cap);
      pos = lower_pos(list, nkeys, n);
      if (!(pos < nkeys && list[pos] == n)) pos = -1;
    }
    if (pos >= 0) {
      int n_sp = 1;
      if (p.nsplit > 1) {                  // as the key kernels counted: the query tiles from the tile's first visible pair on
        const int first = p.kfirst[(long long)bh * p.npad + pos / kKeyTile * kKeyTile];
        n_sp = key_tile_splits(cdiv(p.q_cnt[bh], kKeyQ) - first / kKeyQ, p.nsplit, p.split_len);
      }
      const long long o = ((long long)bh * p.npad + pos) * D + c * 4;
      for (int sp = 0; sp < n_sp; ++sp) {
        ak += *reinterpret_cast<const f32x4*>(p.dKp + sp * p.plane + o);
        av += *reinterpret_cast<const f32x4*>(p.dVp + sp * p.plane + o);
      }
    }
  }
  const long long o = b * L.ks[0] + g * L.ks[1] + (long long)n * L.ks[2] + c * 4;
  if constexpr (sizeof(T) == 2) {
    uint2 wk, wv;
    wk.x = pack_bf16x2(ak[0], ak[1]);
    wk.y = pack_bf16x2(ak[2], ak[3]);
    wv.x = pack_bf16x2(av[0], av[1]);
    wv.y = pack_bf16x2(av[2], av[3]);
    *reinterpret_cast<uint2*>(dK + o) = wk;
    *reinterpret_cast<uint2*>(dV + o) = wv;
  } else {
    *reinterpret_cast<f32x4*>(dK + o) = ak;
    *reinterpret_cast<f32x4*>(dV + o) = av;
  }
}

template <typename T>
__global__ __launch_bounds__(kThreads) void clear_rows_kernel(T* __restrict__ X, Layer L) {
  constexpr int E = Elem<T>::kPer16B;
  const int CPR = L.D / E;
  const int bh = blockIdx.y, b = bh / L.Hq, i = bh % L.Hq;
  T* base = X + b * L.qs[0] + i * L.qs[1];
  const int row0 = blockIdx.x * 64;
  const u32x4 zero = {0u, 0u, 0u, 0u};
  for (int c = threadIdx.x; c < 64 * CPR; c += kThreads) {
    const int r = row0 + c / CPR;
    if (r < L.N) *reinterpret_cast<u32x4*>(base + (long long)r * L.qs[2] + (c % CPR) * E) = zero;
  }
}

struct BwdWs {
  void *Kn, *Vn, *Kt, *Qt, *dOt, *Qn, *dOn;
  int* kidx;
  float *lse2c, *deltac, *dKp, *dVp;
  int* sched;
  int *qvis, *kfirst, *inv, *klist;
  int *kidx_kv, *vbudget, *tile_map;      // in-place block lists only
};

// Block lists walked in place (omni_block_attn_bwd): ascending block ids per head, one budget per batch item.
struct BlockLists {
  const int* blk_idx;
  const int* blk_budget;
  int blk_cap, block;
};

constexpr int kKeyHeadGroup = 7;
int g_key_split_len = kKeySplitLen;          // omni_debug_key_split_len: tests split short key tiles too
// slots of the key kernels' dispatch order (an upper bound of the live items)
size_t key_list_slots(const Layer& L, int npad) {
  return (size_t)cdiv(L.B * L.Hq, kKeyHeadGroup) * kKeyHeadGroup * (npad / kKeyTile) * kKeyMaxSplits;
}

// npad_kv > 0: Kn, Vn, Kt hold every KV head once ([B*Hkv, npad_kv, D], the in-place block lists) instead of one
// gathered copy per query head; cap_tiles = key tiles of a head's list then.
BwdWs carve_bwd(Arena& a, const Layer& L, int dtype, int npad, int nqpad, int npad_kv = 0, int cap_tiles = 0) {
  BwdWs w;
  const size_t es = dtype == OMNI_BF16 ? 2 : 4;
  const size_t BH = (size_t)L.B * L.Hq;
  const size_t krows = BH * npad, qrows = BH * nqpad;
  const size_t kvrows = npad_kv > 0 ? (size_t)L.B * L.Hkv * npad_kv : krows;
  w.Kn = a.take<unsigned char>(kvrows * L.D * es);
  w.Vn = a.take<unsigned char>(kvrows * L.D * es);
  w.Kt = a.take<unsigned char>(dtype == OMNI_BF16 ? kvrows * L.D * es : 16);
  w.Qt = a.take<unsigned char>(dtype == OMNI_BF16 ? qrows * L.D * es : 16);
  w.dOt = a.take<unsigned char>(dtype == OMNI_BF16 ? qrows * L.D * es : 16);
  w.Qn = a.take<unsigned char>(dtype == OMNI_BF16 ? qrows * L.D * es : 16);
  w.dOn = a.take<unsigned char>(dtype == OMNI_BF16 ? qrows * L.D * es : 16);
  w.kidx = a.take<int>(krows);
  w.lse2c = a.take<float>(qrows);
  w.deltac = a.take<float>(qrows);
  const size_t planes = dtype == OMNI_BF16 ? kKeyMaxSplits : 1;
  w.dKp = a.take<float>(planes * krows * L.D);
  w.dVp = a.take<float>(planes * krows * L.D);
  w.sched = a.take<int>(sched_ints(L.B * L.Hq, L.N, kTileM));   // sized for the smaller tile: the longer list
  w.qvis = a.take<int>(dtype == OMNI_BF16 ? BH * L.N : 4);
  w.kfirst = a.take<int>(dtype == OMNI_BF16 ? krows : 4);
  w.inv = a.take<int>(BH * L.N);
  w.klist = a.take<int>(kKeyListHeader + key_list_slots(L, npad));
  w.kidx_kv = a.take<int>(npad_kv > 0 ? kvrows : 4);
  w.vbudget = a.take<int>(L.B);
  w.tile_map = a.take<int>(npad_kv > 0 ? BH * cap_tiles : 4);
  return w;
}

// Rows of a head's packed buffers: whole workgroup tiles, and never a multiple of 4096 rows -- with a
// power-of-two stride between the heads, workgroups that stream different heads at the same tile index hit the
// same cache sets and memory channels.
int bwd_npad(int b_cap) {                     // a multiple of kKeyTile, hence of kBwdKeys
  int n = (int)align_up(b_cap, kKeyTile);
  if (n % 4096 == 0) n += kKeyTile;
  return n;
}
int bwd_nqpad(const Layer& L) {
  int n = (int)align_up(L.N, kTileM);
  if (n % 4096 == 0) n += kTileM;
  return n;
}

int bwd_npad_kv(const Layer& L) { return (int)align_up(L.N, kTileN); }

// BLOCKS (bf16 only): kv_idx / budget / b_cap are ignored and the key lists are the block lists `blk`, walked in place.
template <typename T, int D, bool BLOCKS>
int launch_bwd(const Layer& L, const void* Q, const void* K, const void* V, const void* O, const void* dO,
               const float* lse, const int* q_idx, const int* q_cnt, const int* kv_idx, const int* budget, int b_cap,
               void* dQ, void* dK, void* dV, void* ws, hipStream_t st, const BlockLists* blk = nullptr) {
  constexpr int dt = sizeof(T) == 2 ? OMNI_BF16 : OMNI_F32;
  static_assert(!BLOCKS || sizeof(T) == 2, "block lists run in bf16");
  Arena a(ws);
  const int cap_keys = BLOCKS ? blk->blk_cap * blk->block : b_cap;
  const int npad = bwd_npad(cap_keys), nqpad = bwd_nqpad(L);
  const int npad_kv = BLOCKS ? bwd_npad_kv(L) : 0;
  BwdWs w = carve_bwd(a, L, dt, npad, nqpad, npad_kv, cap_keys / kTileN);
  int rc;
  if constexpr (BLOCKS) {
    // K, V (natural) and K (k-packed) of every KV head once, in token order: shared by the heads of a group
    rc = run_pack_kv(L, dt, K, V, 0, nullptr, L.N, nullptr, L.N, npad_kv, kTileN, w.Kn, w.Vn, w.Kt, nullptr, w.kidx_kv, st);
    if (rc != OMNI_OK) return rc;
    // token lists of the selected blocks (causal bounds, the reduction's slot map), rows npad apart, and the tile map
    rc = run_expand_blocks(L, blk->blk_idx, blk->blk_budget, blk->blk_cap, blk->block, w.kidx, w.vbudget, npad, st);
    if (rc != OMNI_OK) return rc;
    rc = run_tile_map(L, blk->blk_idx, blk->blk_budget, blk->blk_cap, blk->block, npad_kv / kTileN - 1, w.tile_map, st);
    if (rc != OMNI_OK) return rc;
    kv_idx = w.kidx;
    budget = w.vbudget;
    b_cap = npad;                             // the lists' row pitch; their lengths are in vbudget
  } else {
    rc = run_pack_kv(L, dt, K, V, 1, kv_idx, b_cap, budget, b_cap, npad, kKeyTile, w.Kn, w.Vn,
                     dt == OMNI_BF16 ? w.Kt : nullptr, nullptr, w.kidx, st);
    if (rc != OMNI_OK) return rc;
  }
  rc = run_pack_q(L, dt, Q, O, dO, lse, q_idx, q_cnt, nqpad, w.Qt, w.dOt, dt == OMNI_BF16 ? w.Qn : nullptr,
                  dt == OMNI_BF16 ? w.dOn : nullptr, w.lse2c, w.deltac, st);
  if (rc != OMNI_OK) return rc;
  hipLaunchKernelGGL((clear_rows_kernel<T>), dim3(cdiv(L.N, 64), L.B * L.Hq), dim3(kThreads), 0, st,
                     static_cast<T*>(dQ), L);
  OMNI_LAUNCH_CHECK();
  BwdParams p;
  p.Q = Q;
  p.dO = dO;
  p.L = L;
  p.q_idx = q_idx;
  p.q_cnt = q_cnt;
  p.budget = budget;
  p.b_cap = b_cap;
  p.npad = npad;
  p.nqpad = nqpad;
  p.Kn = w.Kn;
  p.Vn = w.Vn;
  p.Kt = w.Kt;
  p.kidx = w.kidx;
  p.Qt = w.Qt;
  p.dOt = w.dOt;
  p.Qn = w.Qn;
  p.dOn = w.dOn;
  p.lse2c = w.lse2c;
  p.deltac = w.deltac;
  p.dKp = w.dKp;
  p.dVp = w.dVp;
  p.nsplit = sizeof(T) == 2 ? kKeyMaxSplits : 1;
  p.split_len = g_key_split_len;
  p.plane = (long long)L.B * L.Hq * npad * D;
  p.dQ = dQ;
  p.sched = w.sched;
  p.qvis = w.qvis;
  p.kfirst = w.kfirst;
  p.tile_map = w.tile_map;
  p.tile_stride = cap_keys / kTileN;
  p.npad_kv = BLOCKS ? npad_kv : npad;
  constexpr bool kFast = sizeof(T) == 2;
  if constexpr (kFast) {
    rc = run_visible_counts(L, q_idx, q_cnt, w.kidx, budget, b_cap, npad, w.qvis, w.kfirst, st);
    if (rc != OMNI_OK) return rc;
  }
  p.order_off = sched_order_off(L.B * L.Hq, L.N, kFast ? kDqTileM : kTileM);
  rc = run_schedule(L, q_cnt, budget, b_cap, kFast ? kDqTileM : kTileM, kFast ? w.qvis : nullptr, w.sched, st);
  if (rc != OMNI_OK) return rc;
  {
    ProfScope prof__(kProfBwdDkDv, st);
    if constexpr (sizeof(T) == 2) {
      // Dispatch order: heads in groups of 7, key tile by key tile inside a group.  Head after head leaves the long
      // first key tiles of the last heads for the end (measured 3.9 ms at 32k), all heads at once spreads 28
      // query streams over the caches (4.4 ms); groups of 7 take 3.4 ms.  Group sizes that share a factor with
      // the 8 XCDs (workgroup i runs on XCD i mod 8) pin heads to XCDs and unbalance them: 8 takes 5.6 ms.
      p.head_group = kKeyHeadGroup;
      if (L.B * L.Hq >= 32768 || npad / kKeyTile >= 8192)
        OMNI_FAIL(OMNI_ERR_UNSUPPORTED, "key work list: too many heads or key tiles");
      p.klist = w.klist;
      hipLaunchKernelGGL(key_list_kernel, dim3(1), dim3(1024), 0, st, p, (long long)key_list_slots(L, npad));
      OMNI_LAUNCH_CHECK();
      const unsigned key_wgs = (unsigned)persistent_grid() / 2;       // one workgroup per CU (its LDS ring fills it)
      hipLaunchKernelGGL((attn_bwd_key_bf16_kernel<D, 1, BLOCKS>), dim3(key_wgs), dim3(kKeyThreads), 0, st, p);
      OMNI_LAUNCH_CHECK();
      hipLaunchKernelGGL((attn_bwd_key_bf16_kernel<D, 0, BLOCKS>), dim3(key_wgs), dim3(kKeyThreads), 0, st, p);
    } else {
      hipLaunchKernelGGL((attn_bwd_dkdv_kernel<T, D>), dim3(npad / kBwdKeys, L.B * L.Hq), dim3(kThreads), 0, st, p);
    }
    OMNI_LAUNCH_CHECK();
  }
  {
    ProfScope prof__(kProfBwdDq, st);
    if constexpr (kFast)
      hipLaunchKernelGGL((attn_bwd_dq_bf16_kernel<D, BLOCKS>), dim3(persistent_grid() / 2), dim3(kDqThreads), 0, st, p);
    else
      hipLaunchKernelGGL((attn_bwd_dq_kernel<T, D>), dim3(persistent_grid() / 2), dim3(kThreads), 0, st, p);
    OMNI_LAUNCH_CHECK();
  }
  {
    ProfScope prof__(kProfBwdReduce, st);
    constexpr int RPB = kThreads / (D / 4);
    const long long n_inv = (long long)L.B * L.Hq * L.N;
    hipLaunchKernelGGL(fill_int_kernel, dim3((unsigned)std::min<long long>(cdiv(n_inv, 256LL), 8192)), dim3(256), 0, st,
                       w.inv, n_inv, -1);
    OMNI_LAUNCH_CHECK();
    hipLaunchKernelGGL(inverse_list_kernel, dim3(cdiv(b_cap, 256), L.B * L.Hq), dim3(256), 0, st, kv_idx, budget, L.bph, L.Hq,
                       b_cap, L.N, w.inv);
    OMNI_LAUNCH_CHECK();
    hipLaunchKernelGGL((attn_bwd_reduce_kernel<T, D>), dim3(cdiv(L.N, RPB), L.B * L.Hkv), dim3(kThreads), 0, st, p,
                       kv_idx, w.inv, static_cast<T*>(dK), static_cast<T*>(dV));
    OMNI_LAUNCH_CHECK();
  }
  return OMNI_OK;
}

}  // namespace

void set_key_split_len(int tiles) { g_key_split_len = tiles > 0 ? tiles : kKeySplitLen; }

size_t attn_bwd_ws(const Layer& L, int dtype, int b_cap) {
  Arena a(nullptr);
  carve_bwd(a, L, dtype, bwd_npad(b_cap), bwd_nqpad(L));
  return a.used();
}

int run_attn_bwd(const Layer& L, int dtype, const void* Q, const void* K, const void* V, const void* O,
                 const void* dO, const float* lse, const int* q_idx, const int* q_cnt, const int* kv_idx,
                 const int* budget, int b_cap, void* dQ, void* dK, void* dV, void* ws, hipStream_t st) {
  if (dtype == OMNI_BF16) {
    if (L.D == 128)
      return launch_bwd<u16, 128, false>(L, Q, K, V, O, dO, lse, q_idx, q_cnt, kv_idx, budget, b_cap, dQ, dK, dV, ws, st);
    return launch_bwd<u16, 64, false>(L, Q, K, V, O, dO, lse, q_idx, q_cnt, kv_idx, budget, b_cap, dQ, dK, dV, ws, st);
  }
  if (L.D == 128)
    return launch_bwd<float, 128, false>(L, Q, K, V, O, dO, lse, q_idx, q_cnt, kv_idx, budget, b_cap, dQ, dK, dV, ws, st);
  return launch_bwd<float, 64, false>(L, Q, K, V, O, dO, lse, q_idx, q_cnt, kv_idx, budget, b_cap, dQ, dK, dV, ws, st);
}

int attn_bwd_blocks_max_keys() { return kBwdMaxMapTiles * kTileN; }

size_t attn_bwd_blocks_ws(const Layer& L, int cap_keys) {
  Arena a(nullptr);
  carve_bwd(a, L, OMNI_BF16, bwd_npad(cap_keys), bwd_nqpad(L), bwd_npad_kv(L), cap_keys / kTileN);
  return a.used();
}

int run_attn_bwd_blocks(const Layer& L, const void* Q, const void* K, const void* V, const void* O, const void* dO,
                        const float* lse, const int* q_idx, const int* q_cnt, const int* blk_idx, const int* blk_budget,
                        int blk_cap, int block, void* dQ, void* dK, void* dV, void* ws, hipStream_t st) {
  const BlockLists blk{blk_idx, blk_budget, blk_cap, block};
  if (L.D == 128)
    return launch_bwd<u16, 128, true>(L, Q, K, V, O, dO, lse, q_idx, q_cnt, nullptr, nullptr, 0, dQ, dK, dV, ws, st, &blk);
  return launch_bwd<u16, 64, true>(L, Q, K, V, O, dO, lse, q_idx, q_cnt, nullptr, nullptr, 0, dQ, dK, dV, ws, st, &blk);
}

}  // namespace omni
