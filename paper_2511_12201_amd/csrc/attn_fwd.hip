// FlashAttention-style forward over kept queries and packed (gathered) keys:
// omni_sparse_attn_fwd and the dense baseline omni_dense_attn_fwd (paper Sec.
// "Preliminary", attention equation, restricted by the masks M^Q, M^K, M^V).
//
// Design for gfx950:
//  * A pack pass (pack.hip) gathers each head's selected K rows into a dense
//    row-major buffer and its V rows into the exact operand order the matrix
//    cores need (below), zero-padding to whole 64-key tiles and recording the
//    original token index of every slot.  The dense baseline runs the same pack
//    with identity indices per KV head.  The main loop is then free of gathers.
//  * Both GEMMs are computed transposed, S^T = K Q^T and O^T = V^T P^T, with
//    32x32 MFMA tiles.  Each lane then owns one query column: the softmax row
//    statistics are per-lane scalars (one exchange with the partner lane that
//    holds the other half of the keys), and the S^T accumulator registers are
//    already in the B-operand order of the second GEMM, so P never moves.
//  * V is packed so that the A operand of O^T = V^T P^T is one 16-byte LDS read:
//    [16-key group][half h][d][8 keys], key(group,h,j) = 16 group + 8 (j/4) + 4 h + j%4,
//    which is the order in which the S^T accumulators hold the keys.
//  * bf16 inputs, second product in f16: S^T = K Q^T runs on the bf16 matrix cores; the weights are rounded to
//    f16 (11 significant bits against bf16's 8, same matrix-core rate) and multiplied with V converted to f16 by
//    the pack pass (exact for magnitudes in [2^-14, 65504]; beyond that V saturates, below it keeps 3e-8 absolute).
//    The normaliser is the sum of the weights as rounded, so a row that one key dominates returns that key's V row
//    whatever value the weights are taken against, and the log-sum-exp is off by at most 2^-11 relative in the sum.
//  * bf16 (attn_fwd_bf16_kernel, the measured path): 512 threads = 8 wavefronts x
//    32 query rows per work item of 256 kept queries; 64-key K/V tiles go from
//    memory straight into a ring of four LDS stages (global_load_lds, hand-placed
//    s_waitcnt), one barrier per tile; inside a wavefront the softmax of tile t
//    runs under the MFMAs of tile t+1.  Work items come from a persistent,
//    longest-first work list with one queue per XCD (sched.hip); causal masks are
//    position compares against per-query visible-prefix counts (pack.hip).
//  * fp32 inputs (attn_fwd_kernel, the accuracy path of the 1e-4 parity cases):
//    256 threads = 4 wavefronts x 32 rows, fp32 32x32x2 MFMA, register-staged
//    double buffer; not tuned.

#include <type_traits>

#include "common.h"
#include "kernels.h"
#include "sched.h"

namespace omni {

namespace {

constexpr int kThreads = 256;
constexpr float kLog2e = 1.4426950408889634f;
constexpr float kLn2 = 0.6931471805599453f;

// O = 0, lse = -inf for every row (kept rows are overwritten by the attention kernel).
template <typename T>
__global__ __launch_bounds__(kThreads) void clear_output_kernel(T* __restrict__ O, float* __restrict__ lse, Layer L) {
  constexpr int E = Elem<T>::kPer16B;
  const int CPR = L.D / E;
  const int bh = blockIdx.y, b = bh / L.Hq, i = bh % L.Hq;
  T* base = O + b * L.qs[0] + i * L.qs[1];
  const int row0 = blockIdx.x * 64;
  const u32x4 zero = {0u, 0u, 0u, 0u};
  for (int c = threadIdx.x; c < 64 * CPR; c += kThreads) {
    const int r = row0 + c / CPR;
    if (r < L.N) *reinterpret_cast<u32x4*>(base + (long long)r * L.qs[2] + (c % CPR) * E) = zero;
  }
  if (threadIdx.x < 64 && row0 + (int)threadIdx.x < L.N) lse[(long long)bh * L.N + row0 + threadIdx.x] = -INFINITY;
}

// ------------------------------------------------------------------ attention

struct FwdParams {
  const void* Q;
  void* O;
  float* lse;
  Layer L;
  const int* q_idx;     // [B*Hq, N] kept query rows, ascending; nullptr: all rows
  const int* q_cnt;     // [B*Hq]; nullptr: N
  const void* Kp;       // packed keys  [BHx, npad, D]
  const void* Vp;       // packed values, tile layout (bf16) or row-major (fp32)
  const int* kidx;      // [BHx, npad] original token index of every slot
  const int* budget;    // [B] (or [B,Hq] when L.bph) number of packed keys (device); nullptr: N
  int b_cap;
  int npad;
  int per_q_head;       // packed buffers per query head (sparse) or per KV head (dense)
  int identity_keys;
  const int* qvis;       // [B*Hq, N] visible packed keys per kept-query position (sparse bf16 path), else nullptr    // kidx[p] == p: causal bounds by arithmetic
  int* sched;           // work list (sched.h)
  size_t order_off;     // where its hand-out order starts
  const int* tile_map;  // in-place variant: [B*Hq, tile_stride] tile of the packed K/V that tile t of a head's key list is
  int tile_stride;
};

// number of entries <= v in ascending a[0,n)
template <typename T, int D>
__global__ __launch_bounds__(kThreads, 2) void attn_fwd_kernel(FwdParams p) {
  constexpr bool kBf16 = sizeof(T) == 2;
  constexpr int KLD = kBf16 ? D + 8 : D + 4;        // K tile row pitch in elements
  constexpr int VLD = D + 8;                        // fp32 V tile row pitch
  constexpr int NBUF = kBf16 ? 2 : 1;
  constexpr int kKBytes = kTileN * KLD * (int)sizeof(T);
  constexpr int kVBytes = kBf16 ? kTileN * D * 2 : kTileN * VLD * 4;
  __shared__ __attribute__((aligned(16))) unsigned char sK_raw[NBUF * kKBytes];
  __shared__ __attribute__((aligned(16))) unsigned char sV_raw[NBUF * kVBytes];
  __shared__ __attribute__((aligned(16))) int sIdx[NBUF][kTileN];
  __shared__ int sBound[2];

  __shared__ int sItem;
  const Layer& L = p.L;
  const int lane = lane_id(), wave = threadIdx.x >> 6;
  const int ln = lane & 31, h = lane >> 5;
  const float c2 = L.scale * kLog2e;

  for (;;) {                                 // persistent: one work item (head, query tile) per iteration
  __syncthreads();                           // LDS of the previous item is no longer read
  if (threadIdx.x == 0) sItem = sched_next(p.sched);
  __syncthreads();
  const int item = sItem;
  if (item < 0) break;
  int bh, tq;
  sched_decode(p.sched, p.order_off, item, bh, tq);
  const int b = bh / L.Hq, i = bh % L.Hq, g = i / L.G;
  const int nq = p.q_cnt ? p.q_cnt[bh] : L.N;
  const int nkeys = p.budget ? min(p.budget[budget_slot(L.bph, b, bh)], p.b_cap) : L.N;
  const int bhx = p.per_q_head ? bh : b * L.Hkv + g;
  const int* kidx = p.kidx + (long long)bhx * p.npad;
  const int* qlist = p.q_idx ? p.q_idx + (long long)bh * L.N : nullptr;

  // ---- key range of this query tile
  const int pos_first = tq * kTileM, pos_last = min(pos_first + kTileM, nq) - 1;
  if (threadIdx.x == 0 || threadIdx.x == 64) {
    const int which = threadIdx.x ? 1 : 0;
    const int pos = which ? pos_last : pos_first;
    const int row = qlist ? qlist[pos] : pos;
    int cnt;
    if (!L.causal) cnt = nkeys;
    else if (p.identity_keys) cnt = min(row + 1, nkeys);
    else cnt = upper_count(kidx, nkeys, row);
    sBound[which] = cnt;
  }
  __syncthreads();
  const int n_full_tiles = sBound[0] / kTileN;         // tiles with every key admissible for every row
  const int ntiles = cdiv(sBound[1], kTileN);

  // ---- this lane's query row
  const int qpos = pos_first + wave * 32 + ln;
  const bool qvalid = qpos < nq;
  const int qpos_c = min(qpos, nq - 1);
  const int qrow = qlist ? qlist[qpos_c] : qpos_c;
  const int qcmp = L.causal ? qrow : kPadKeyIndex - 1;  // key admissible iff its index <= qcmp
  const T* qptr = static_cast<const T*>(p.Q) + b * L.qs[0] + i * L.qs[1] + (long long)qrow * L.qs[2];

  bf16x8 qf16[kBf16 ? D / 16 : 1];
  f32x4 qf32[kBf16 ? 1 : D / 8];
  if constexpr (kBf16) {
#pragma unroll
    for (int ks = 0; ks < D / 16; ++ks) qf16[ks] = *reinterpret_cast<const bf16x8*>(qptr + ks * 16 + h * 8);
  } else {
#pragma unroll
    for (int ks = 0; ks < D / 8; ++ks) qf32[ks] = *reinterpret_cast<const f32x4*>(qptr + ks * 8 + h * 4);
  }

  f32x16 o[D / 32];
#pragma unroll
  for (int db = 0; db < D / 32; ++db)
#pragma unroll
    for (int r = 0; r < 16; ++r) o[db][r] = 0.f;
  float m_run = -INFINITY, l_run = 0.f;

  // ---- tile staging
  constexpr int E = Elem<T>::kPer16B;
  constexpr int CPR = D / E;
  constexpr int kChunks = kTileN * CPR / kThreads;   // 16-byte chunks per thread per operand
  const T* kp = static_cast<const T*>(p.Kp) + (long long)bhx * p.npad * D;
  const T* vp = static_cast<const T*>(p.Vp) + (long long)bhx * p.npad * D;
  u32x4 stK[kChunks], stV[kChunks];
  i32x4 stI;

  auto load_k = [&](int t) {
    const T* ks = kp + (long long)t * kTileN * D;
#pragma unroll
    for (int c = 0; c < kChunks; ++c) stK[c] = *reinterpret_cast<const u32x4*>(ks + (threadIdx.x + c * kThreads) * E);
  };
  auto load_v = [&](int t) {
    const T* vs = vp + (long long)t * kTileN * D;
#pragma unroll
    for (int c = 0; c < kChunks; ++c) stV[c] = *reinterpret_cast<const u32x4*>(vs + (threadIdx.x + c * kThreads) * E);
    if (threadIdx.x < kTileN / 4) stI = *reinterpret_cast<const i32x4*>(kidx + t * kTileN + threadIdx.x * 4);
  };
  auto store_k = [&](int buf) {
    T* sk = reinterpret_cast<T*>(sK_raw + buf * kKBytes);
#pragma unroll
    for (int c = 0; c < kChunks; ++c) {
      const int ch = threadIdx.x + c * kThreads;
      *reinterpret_cast<u32x4*>(sk + (ch / CPR) * KLD + (ch % CPR) * E) = stK[c];
    }
  };
  auto store_v = [&](int buf) {          // the slot indices travel with the V tile
    T* sv = reinterpret_cast<T*>(sV_raw + buf * kVBytes);
#pragma unroll
    for (int c = 0; c < kChunks; ++c) {
      const int ch = threadIdx.x + c * kThreads;
      if constexpr (kBf16) *reinterpret_cast<u32x4*>(sv + ch * E) = stV[c];
      else *reinterpret_cast<u32x4*>(sv + (ch / CPR) * VLD + (ch % CPR) * E) = stV[c];
    }
    if (threadIdx.x < kTileN / 4) *reinterpret_cast<i32x4*>(&sIdx[buf][threadIdx.x * 4]) = stI;
  };

  // S^T tile = K tile . Q^T (64 keys x 32 queries per wavefront)
  auto qk_tile = [&](int buf, f32x16 (&s)[2]) {
    const T* sk = reinterpret_cast<const T*>(sK_raw + buf * kKBytes);
#pragma unroll
    for (int kb = 0; kb < 2; ++kb) {
#pragma unroll
      for (int r = 0; r < 16; ++r) s[kb][r] = 0.f;
      if constexpr (kBf16) {
        // LDS fragment reads are issued one group of 4 ahead of the MFMAs that consume them; the
        // scheduling fences keep the compiler from pulling each read back next to its MFMA
        // (which would expose the full LDS latency 16 times per tile).
        constexpr int NG = D / 64;          // groups of 4 k-steps
        bf16x8 ka[4], kb4[4];
#pragma unroll
        for (int j = 0; j < 4; ++j)
          ka[j] = *reinterpret_cast<const bf16x8*>(sk + (kb * 32 + ln) * KLD + j * 16 + h * 8);
#pragma unroll
        for (int gi = 0; gi < NG; ++gi) {
          __builtin_amdgcn_sched_barrier(0);
          if (gi + 1 < NG) {
#pragma unroll
            for (int j = 0; j < 4; ++j)
              kb4[j] = *reinterpret_cast<const bf16x8*>(sk + (kb * 32 + ln) * KLD + ((gi + 1) * 4 + j) * 16 + h * 8);
          }
          __builtin_amdgcn_sched_barrier(0);
#pragma unroll
          for (int j = 0; j < 4; ++j)
            s[kb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(ka[j], qf16[gi * 4 + j], s[kb], 0, 0, 0);
#pragma unroll
          for (int j = 0; j < 4; ++j) ka[j] = kb4[j];
        }
        __builtin_amdgcn_sched_barrier(0);
      } else {
#pragma unroll
        for (int ks = 0; ks < D / 8; ++ks) {
          const f32x4 kf = *reinterpret_cast<const f32x4*>(sk + (kb * 32 + ln) * KLD + ks * 8 + h * 4);
#pragma unroll
          for (int e = 0; e < 4; ++e)
            s[kb] = __builtin_amdgcn_mfma_f32_32x32x2f32(kf[e], qf32[ks][e], s[kb], 0, 0, 0);
        }
      }
    }
  };

  // mask + online softmax on a finished S^T tile; leaves P in s
  auto softmax_tile = [&](int buf, bool masked, f32x16 (&s)[2]) {
    if (masked) {
#pragma unroll
      for (int kb = 0; kb < 2; ++kb)
#pragma unroll
        for (int q4 = 0; q4 < 4; ++q4) {
          const i32x4 id = *reinterpret_cast<const i32x4*>(&sIdx[buf][kb * 32 + 8 * q4 + 4 * h]);
#pragma unroll
          for (int e = 0; e < 4; ++e)
            if (id[e] > qcmp) s[kb][q4 * 4 + e] = -INFINITY;
        }
    }
    // this lane and lane^32 share the query row
    float mloc = s[0][0];
#pragma unroll
    for (int kb = 0; kb < 2; ++kb)
#pragma unroll
      for (int r = 0; r < 16; ++r) mloc = fmaxf(mloc, s[kb][r]);
    mloc = pair_max(mloc);
    const float m_new = fmaxf(m_run, mloc);
    const float m_ref = m_new == -INFINITY ? 0.f : m_new;
    if (__any(m_new > m_run)) {
      const float alpha = fast_exp2((m_run - m_ref) * c2);
      l_run *= alpha;
#pragma unroll
      for (int db = 0; db < D / 32; ++db)
#pragma unroll
        for (int r = 0; r < 16; ++r) o[db][r] *= alpha;
      m_run = m_new;
    }
    const float mc = m_ref * c2;
    float lsum = 0.f;
#pragma unroll
    for (int kb = 0; kb < 2; ++kb)
#pragma unroll
      for (int r = 0; r < 16; ++r) {
        const float pv = fast_exp2(fmaf(s[kb][r], c2, -mc));
        s[kb][r] = pv;
        lsum += pv;
      }
    l_run += lsum;
  };

  // O^T += V^T . P^T
  auto pv_tile = [&](int buf, const f32x16 (&s)[2]) {
    const T* sv = reinterpret_cast<const T*>(sV_raw + buf * kVBytes);
    if constexpr (kBf16) {
      constexpr int NB = D / 32;
      bf16x8 va[NB], vb[NB];
#pragma unroll
      for (int db = 0; db < NB; ++db)
        va[db] = *reinterpret_cast<const bf16x8*>(sv + ((0 * 2 + h) * D + db * 32 + ln) * 8);
#pragma unroll
      for (int t16 = 0; t16 < 4; ++t16) {
        const int kb = t16 >> 1, r0 = (t16 & 1) * 8;
        __builtin_amdgcn_sched_barrier(0);
        if (t16 + 1 < 4) {
#pragma unroll
          for (int db = 0; db < NB; ++db)
            vb[db] = *reinterpret_cast<const bf16x8*>(sv + (((t16 + 1) * 2 + h) * D + db * 32 + ln) * 8);
        }
        union { bf16x8 v; unsigned u[4]; } pf;
#pragma unroll
        for (int jj = 0; jj < 4; ++jj) pf.u[jj] = pack_bf16x2(s[kb][r0 + 2 * jj], s[kb][r0 + 2 * jj + 1]);
        __builtin_amdgcn_sched_barrier(0);
#pragma unroll
        for (int db = 0; db < NB; ++db)
          o[db] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(va[db], pf.v, o[db], 0, 0, 0);
#pragma unroll
        for (int db = 0; db < NB; ++db) va[db] = vb[db];
      }
      __builtin_amdgcn_sched_barrier(0);
    } else {
#pragma unroll
      for (int kb = 0; kb < 2; ++kb)
#pragma unroll
        for (int r = 0; r < 16; ++r) {
          const int slot = kb * 32 + 8 * (r >> 2) + 4 * h + (r & 3);
#pragma unroll
          for (int db = 0; db < D / 32; ++db) {
            const float vf = sv[slot * VLD + db * 32 + ln];
            o[db] = __builtin_amdgcn_mfma_f32_32x32x2f32(vf, s[kb][r], o[db], 0, 0, 0);
          }
        }
    }
  };

  if (ntiles > 0) {
    if constexpr (kBf16) {
      f32x16 s[2];
      load_k(0);
      load_v(0);
      store_k(0);
      store_v(0);
      __syncthreads();
      for (int t = 0; t < ntiles; ++t) {
        if (t + 1 < ntiles) {
          load_k(t + 1);
          load_v(t + 1);
        }
        qk_tile(t & 1, s);
        softmax_tile(t & 1, t >= n_full_tiles, s);
        pv_tile(t & 1, s);
        if (t + 1 < ntiles) {
          store_k((t + 1) & 1);
          store_v((t + 1) & 1);
        }
        __syncthreads();
      }
    } else {
      f32x16 s[2];
      for (int t = 0; t < ntiles; ++t) {
        __syncthreads();
        load_k(t);
        load_v(t);
        store_k(0);
        store_v(0);
        __syncthreads();
        qk_tile(0, s);
        softmax_tile(0, t >= n_full_tiles, s);
        pv_tile(0, s);
      }
    }
  }

  // ---- epilogue
  const float l_tot = pair_sum(l_run);
  const float inv = l_tot > 0.f ? 1.0f / l_tot : 0.f;
  if (qvalid) {
    T* optr = static_cast<T*>(p.O) + b * L.qs[0] + i * L.qs[1] + (long long)qrow * L.qs[2];
#pragma unroll
    for (int db = 0; db < D / 32; ++db)
#pragma unroll
      for (int q4 = 0; q4 < 4; ++q4) {
        const int d = db * 32 + 8 * q4 + 4 * h;
        const float v0 = o[db][q4 * 4 + 0] * inv, v1 = o[db][q4 * 4 + 1] * inv;
        const float v2 = o[db][q4 * 4 + 2] * inv, v3 = o[db][q4 * 4 + 3] * inv;
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
    if (h == 0)
      p.lse[(long long)bh * L.N + qrow] = l_tot > 0.f ? (m_run * c2 + log2f(l_tot)) * kLn2 : -INFINITY;
  }
  }  // work-item loop
}

// ------------------------------------------------------------------ bf16 fast path
//
// 512 threads = 8 wavefronts x 32 query rows (256-row work items, one workgroup per CU).
// K/V tiles go from global memory straight into LDS (global_load_lds, no VGPR staging) into a
// ring of kStages buffers, so up to kStages - 1 tiles are in flight while one is computed and a
// single barrier per tile is enough.  The loads are inline assembly with hand-placed
// s_waitcnt vmcnt(n): the compiler would wait for *every* outstanding LDS-DMA load before the
// first LDS read, which collapses the ring to one tile of prefetch.
// A wavefront's LDS-DMA instruction writes 64 x 16 contiguous bytes, so the K tile cannot be
// row-padded; it is stored unpadded with an XOR swizzle of the 16-byte chunk index
// (chunk ^ row % chunks_per_row), applied on the global-address side of the copy, which keeps
// the 16 rows a ds_read_b128 touches on distinct banks.  V is already in operand order.

constexpr int kFastWaves = 8;
constexpr int kFastThreads = kFastWaves * 64;
constexpr int kFastTileM = kFastWaves * 32;
constexpr int kStages = 4;
constexpr int kMaxMapTiles = 2048;                   // key tiles of one head in the in-place variant (128k tokens)

// TILEMAP: the key list of a head is a sequence of whole 64-key tiles of the KV head's (ungathered) K/V -- the
// block-granular selection -- and tile t of the list is read in place, at tile p.tile_map[head][t].
template <int D, bool TILEMAP>
__global__ __launch_bounds__(kFastThreads, 2) void attn_fwd_bf16_kernel(FwdParams p) {
  typedef u16 T;
  constexpr int CH = D / 8;                          // 16-byte chunks per K row
  constexpr int kKBytes = kTileN * D * 2;
  constexpr int kStageBytes = 2 * kKBytes;           // K tile then V tile
  constexpr int LPH = kKBytes / 1024 / kFastWaves;   // load instructions per operand per wavefront per tile
  constexpr int LPT = 2 * LPH;
  static_assert(LPH >= 1, "tile too small for the copy scheme");
  __shared__ __attribute__((aligned(1024))) unsigned char smem[kStages * kStageBytes];
  __shared__ int sBound[2];
  __shared__ int sItem;
  __shared__ int sTileMap[TILEMAP ? kMaxMapTiles : 1];

  const Layer& L = p.L;
  const int lane = lane_id();
  const int wave = __builtin_amdgcn_readfirstlane((int)(threadIdx.x >> 6));
  const int ln = lane & 31, h = lane >> 5;
  const float c2 = L.scale * kLog2e;
  const unsigned lds_base = (unsigned)(size_t)(__attribute__((address_space(3))) unsigned char*)smem;

  // per-lane pieces of the copy: which global chunk lands in this lane's LDS slot
  unsigned kgoff[LPH], vgoff[LPH];                             // byte offsets inside a tile
#pragma unroll
  for (int j = 0; j < LPH; ++j) {
    const int pchunk = (j * kFastWaves + wave) * 64 + lane;   // physical 16-byte slot in the K tile
    const int row = pchunk / CH, pc = pchunk % CH;
    kgoff[j] = (row * D + ((pc ^ (row % CH)) << 3)) * 2;
    vgoff[j] = pchunk << 4;
  }
  // per-lane pieces of the fragment reads
  const int krow_b = ln * (CH * 16);                           // byte offset of row ln in a 32-row block
  const int khx = (h << 4) ^ ((ln % CH) << 4);                 // (chunk ^ swizzle) << 4 = (ks << 5) ^ khx
  const int vlane_b = (h * D + ln) * 16;

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
  const int b = bh / L.Hq, i = bh % L.Hq, g = i / L.G;
  const int nq = p.q_cnt ? p.q_cnt[bh] : L.N;
  const int nkeys = p.budget ? min(p.budget[budget_slot(L.bph, b, bh)], p.b_cap) : L.N;
  const int bhx = p.per_q_head ? bh : b * L.Hkv + g;
  const int* kidx = p.kidx + (long long)bhx * p.npad;
  const int* qlist = p.q_idx ? p.q_idx + (long long)bh * L.N : nullptr;

  const int pos_first = tq * kFastTileM, pos_last = min(pos_first + kFastTileM, nq) - 1;
  const int* qvis = p.qvis ? p.qvis + (long long)bh * L.N : nullptr;
  // visible prefix length of the packed key list for a kept-query position
  auto visible = [&](int pos, int row) {
    if (!L.causal) return nkeys;
    if (p.identity_keys) return min(row + 1, nkeys);
    return qvis ? qvis[pos] : upper_count(kidx, nkeys, row);
  };
  if (threadIdx.x == 0 || threadIdx.x == 64) {
    const int which = threadIdx.x ? 1 : 0;
    const int pos = which ? pos_last : pos_first;
    sBound[which] = visible(pos, qlist ? qlist[pos] : pos);
  }
  __syncthreads();
  const int n_full_tiles = sBound[0] / kTileN;
  const int ntiles = cdiv(sBound[1], kTileN);
  if constexpr (TILEMAP) {                                     // this item's share of the head's tile map
    const int* tm = p.tile_map + (long long)bh * p.tile_stride;
    for (int t = threadIdx.x; t < ntiles; t += kFastThreads) sTileMap[t] = tm[t];
    __syncthreads();
  }

  const int qpos = pos_first + wave * 32 + ln;
  const bool qvalid = qpos < nq;
  const int qpos_c = min(qpos, nq - 1);
  const int qrow = qlist ? qlist[qpos_c] : qpos_c;
  const int qvisible = visible(qpos_c, qrow) - 4 * h;          // compared with key positions that leave out 4 * h
  const T* qptr = static_cast<const T*>(p.Q) + b * L.qs[0] + i * L.qs[1] + (long long)qrow * L.qs[2];
  bf16x8 qf[D / 16];
#pragma unroll
  for (int ks = 0; ks < D / 16; ++ks) qf[ks] = *reinterpret_cast<const bf16x8*>(qptr + ks * 16 + h * 8);
  // Make the compiler finish these loads here.  Otherwise it places their s_waitcnt vmcnt at the first
  // use inside the tile loop, where it would also drain the K/V prefetch ring on every iteration.
#pragma unroll
  for (int ks = 0; ks < D / 16; ++ks) asm volatile("" : "+v"(qf[ks]));

  f32x16 o[D / 32];
#pragma unroll
  for (int db = 0; db < D / 32; ++db)
#pragma unroll
    for (int r = 0; r < 16; ++r) o[db][r] = 0.f;
  float m_run = -INFINITY, l_run = 0.f;

  const T* kp = static_cast<const T*>(p.Kp) + (long long)bhx * p.npad * D;
  const T* vp = static_cast<const T*>(p.Vp) + (long long)bhx * p.npad * D;

  // one load instruction of tile t: part < LPH is a K part, the rest are V parts
  auto issue_part = [&](int t, int part) {
    const unsigned dst = lds_base + (unsigned)(t % kStages) * kStageBytes;
    // where tile t of the key list lives (wave-uniform: the tile base stays in scalar registers)
    const int src = TILEMAP ? __builtin_amdgcn_readfirstlane(sTileMap[t]) : t;
    if (part < LPH) {
      gload_lds16(kp + (long long)src * kTileN * D, kgoff[part], dst + (part * kFastWaves + wave) * 1024);
    } else {
      const int j = part - LPH;
      gload_lds16(vp + (long long)src * kTileN * D, vgoff[j], dst + kKBytes + (j * kFastWaves + wave) * 1024);
    }
  };
  auto issue_tile = [&](int t) {
#pragma unroll
    for (int j = 0; j < LPT; ++j) issue_part(t, j);
  };

  // Software pipeline over key tiles.  While the matrix cores compute S(t+1)^T = K(t+1) . Q^T the
  // same wavefront turns S(t) into P(t) on the vector ALU (exp2, f16 pack, row sum); while they
  // accumulate O^T += V(t)^T . P(t)^T it scans S(t+1) for the running maximum (in the steps that follow
  // it; see `step`).  Each MFMA is followed
  // in program order by its share of the vector work and a scheduling fence, so the hardware always
  // has independent vector instructions to issue under a running MFMA.  Without this the two
  // wavefronts of a SIMD, which the per-tile barrier keeps in step, are in their softmax phases at
  // the same time and the matrix cores idle for that long.
  constexpr int NQK = 2 * (D / 16);          // MFMAs of one S tile: 2 key blocks x D/16 k-steps
  constexpr int NPV = 4 * (D / 32);          // MFMAs of one P.V tile: 4 key steps x D/32 row blocks
  constexpr int NB = D / 32;
  constexpr int kAhead = 2;                  // fragment reads run this many MFMAs ahead
  static_assert(32 % NQK == 0 && 32 % NPV == 0 && 16 % NPV == 0, "chunking of the vector work");
  const f32x16 zero16 = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};

  auto kfrag = [&](const unsigned char* sk, int c) {
    const int kb = c % 2, ks = c / 2;
    return *reinterpret_cast<const bf16x8*>(sk + kb * (32 * CH * 16) + krow_b + ((ks << 5) ^ khx));
  };
  auto vfrag = [&](const unsigned char* sv, int c) {
    const int t16 = c / NB, db = c % NB;
    return *reinterpret_cast<const f16x8*>(sv + vlane_b + (t16 * 2 * D + db * 32) * 16);
  };

  // S^T of tile t alone (first tile of an item)
  auto qk_only = [&](f32x16 (&sn)[2], int t) {
    const unsigned char* sk = smem + (t % kStages) * kStageBytes;
    bf16x8 kf[kAhead];
#pragma unroll
    for (int c = 0; c < kAhead; ++c) kf[c] = kfrag(sk, c);
#pragma unroll
    for (int c = 0; c < NQK; ++c) {
      const int kb = c % 2, ks = c / 2;
      __builtin_amdgcn_sched_barrier(0);
      sn[kb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(kf[c % kAhead], qf[ks], ks == 0 ? zero16 : sn[kb], 0, 0, 0);
      if (c + kAhead < NQK) kf[c % kAhead] = kfrag(sk, c + kAhead);
    }
    __builtin_amdgcn_sched_barrier(0);
  };

  // Reference value of the softmax from a finished S tile.  m_run is the value the weights are taken against, not
  // the exact running maximum: it moves (and the accumulators are rescaled) only when some row of the wavefront
  // exceeds it by more than kRescaleSlack in the exponent, so a weight is at most 2^kRescaleSlack and the rescale
  // is rare.  Output and log-sum-exp do not depend on the reference value beyond rounding.
  float mc = 0.f;                              // (reference value, 0 if none yet) * c2
  constexpr float kRescaleSlack = 6.0f;
  auto update_max = [&](float mloc) {
    mloc = pair_max(mloc);
    if (__any(mloc > m_run + kRescaleSlack / c2)) {
      const float m_new = fmaxf(m_run, mloc);
      const float m_ref = m_new == -INFINITY ? 0.f : m_new;
      const float alpha = fast_exp2((m_run - m_ref) * c2);
      l_run *= alpha;
#pragma unroll
      for (int db = 0; db < NB; ++db)
#pragma unroll
        for (int r = 0; r < 16; ++r) o[db][r] *= alpha;
      m_run = m_new;
      mc = m_ref * c2;
    }
  };
  auto mask_tile = [&](f32x16 (&sn)[2], int t) {
    const int rel = qvisible - t * kTileN;     // keys of this tile at positions >= rel are hidden (pad rows too)
#pragma unroll
    for (int kb = 0; kb < 2; ++kb)
#pragma unroll
      for (int q4 = 0; q4 < 4; ++q4)
#pragma unroll
        for (int e = 0; e < 4; ++e)
          if (kb * 32 + 8 * q4 + e >= rel) sn[kb][q4 * 4 + e] = -INFINITY;   // register r holds key 8 (r/4) + 4 h + r%4
    float mloc = sn[0][0];
#pragma unroll
    for (int kb = 0; kb < 2; ++kb)
#pragma unroll
      for (int r = 0; r < 16; r += 2) mloc = fmaxf(fmaxf(sn[kb][r], sn[kb][r + 1]), mloc);
    return mloc;
  };

  // Steps that do not follow the maximum (below) call this when a weight left the safe range: the reference value
  // moves to the maximum of the tile at hand, the accumulators are rescaled, and the tile's weights are formed again.
  union PFrag { f16x8 v[4]; f16x2 h[16]; };
  // acc + both halves of pk, one instruction each: the sum of the weights exactly as the matrix cores get them
  auto add_halves = [](float acc, f16x2 pk) {
    asm("v_fma_mix_f32 %0, %1, 1.0, %0 op_sel:[0,0,0] op_sel_hi:[1,0,0]" : "+v"(acc) : "v"(pk));
    asm("v_fma_mix_f32 %0, %1, 1.0, %0 op_sel:[1,0,0] op_sel_hi:[1,0,0]" : "+v"(acc) : "v"(pk));
    return acc;
  };
  auto refit = [&](const f32x16 (&sc)[2], PFrag& pf, float& lsum) {
    float mloc = sc[0][0];
#pragma unroll
    for (int kb = 0; kb < 2; ++kb)
#pragma unroll
      for (int r = 0; r < 16; r += 2) mloc = fmaxf(fmaxf(sc[kb][r], sc[kb][r + 1]), mloc);
    mloc = pair_max(mloc);
    const float m_new = fmaxf(m_run, mloc);
    const float m_ref = m_new == -INFINITY ? 0.f : m_new;
    const float alpha = fast_exp2((m_run - m_ref) * c2);
    l_run *= alpha;
#pragma unroll
    for (int db = 0; db < NB; ++db)
#pragma unroll
      for (int r = 0; r < 16; ++r) o[db][r] *= alpha;
    m_run = m_new;
    mc = m_ref * c2;
    lsum = 0.f;
#pragma unroll
    for (int r = 0; r < 32; r += 2) {
      f32x2 pv;
      pv[0] = fast_exp2(fmaf(sc[r / 16][r % 16], c2, -mc));
      pv[1] = fast_exp2(fmaf(sc[r / 16][r % 16 + 1], c2, -mc));
      const f16x2 pk = __builtin_convertvector(pv, f16x2);
      pf.h[r / 2] = pk;
      lsum = add_halves(lsum, pk);
    }
  };

  // One pipeline step: P(t) from sc, O += V(t) P(t); if there is a tile t+1: S(t+1) into sn and its maximum.
  // `steady` steps are the ones with t + 3 < ntiles: they always have a next tile and always prefetch,
  // so the step is straight-line code and the fences keep the interleaving as written.
  // `follow` steps scan S(t+1) for its maximum and move the reference value by the slack rule.  Once every row of
  // the wavefront has a reference value (a finite one: it has seen a key), the steady steps stop following: a
  // reference value that is the maximum of some of the row's logits can only be too low, never too high, so a weight
  // that underflows is below 2^-126 of the row's largest and does not matter, and one that grows past kHuge shows in
  // the tile's sum of weights, which is there anyway -- then refit() moves the reference.  That takes the maximum
  // scan and its bookkeeping (a sixth of the step's vector instructions) out of the loop.
  constexpr float kHuge = 16384.f;                 // 2^14: a weight stays inside the f16 range
  auto step = [&](auto steady, auto follows, f32x16 (&sc)[2], f32x16 (&sn)[2], int t) {
    constexpr bool kSteady = decltype(steady)::value;
    constexpr bool kFollow = decltype(follows)::value;
    const bool has_next = kSteady || t + 1 < ntiles;
    const int pre = (kSteady || t + 3 < ntiles) ? t + 3 : -1;
    const unsigned char* sk = smem + ((t + 1) % kStages) * kStageBytes;
    const unsigned char* sv = smem + (t % kStages) * kStageBytes + kKBytes;
    PFrag pf;
    float lsum = 0.f;
    f16x8 vf[kAhead];
    constexpr int EQ = 32 / NQK;             // S elements turned into P per QK MFMA
    auto softmax_chunk = [&](int c) {
#pragma unroll
      for (int e = 0; e < EQ; e += 2) {
        const int r = c * EQ + e;
        f32x2 pv;
        pv[0] = fast_exp2(fmaf(sc[r / 16][r % 16], c2, -mc));
        pv[1] = fast_exp2(fmaf(sc[r / 16][r % 16 + 1], c2, -mc));
        const f16x2 pk = __builtin_convertvector(pv, f16x2);
        pf.h[r / 2] = pk;
        lsum = add_halves(lsum, pk);           // the weights as rounded: numerator and normaliser agree
      }
    };
    if (has_next) {
      if (kSteady || t + 2 < ntiles) wait_vmcnt<LPT>();   // this wavefront's share of tile t+1 has landed
      else wait_vmcnt<0>();
      __syncthreads();                        // ... and everyone else's; tile t-1 is retired
      __builtin_amdgcn_sched_barrier(0);
      bf16x8 kf[kAhead];
#pragma unroll
      for (int c = 0; c < kAhead; ++c) kf[c] = kfrag(sk, c);
#pragma unroll
      for (int c = 0; c < NQK; ++c) {
        const int kb = c % 2, ks = c / 2;
        __builtin_amdgcn_sched_barrier(0);
        sn[kb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(kf[c % kAhead], qf[ks], ks == 0 ? zero16 : sn[kb], 0, 0, 0);
        if (c + kAhead < NQK) kf[c % kAhead] = kfrag(sk, c + kAhead);
        else vf[c + kAhead - NQK] = vfrag(sv, c + kAhead - NQK);
        softmax_chunk(c);
        if (c * LPH % NQK == 0 && (kSteady || pre >= 0)) issue_part(pre, c * LPH / NQK);
      }
    } else {
#pragma unroll
      for (int c = 0; c < kAhead; ++c) vf[c] = vfrag(sv, c);
#pragma unroll
      for (int c = 0; c < NQK; ++c) softmax_chunk(c);
    }
    // (also in the following steps: the first one after a stretch that did not follow forms its weights against
    // the reference value that stretch left behind)
    if (__any(lsum > kHuge)) refit(sc, pf, lsum);
    l_run += lsum;
    __builtin_amdgcn_s_setprio(0);
    float mloc = -INFINITY;
    constexpr int EV = 32 / NPV;             // S(t+1) elements scanned per P.V MFMA
#pragma unroll
    for (int c = 0; c < NPV; ++c) {
      const int t16 = c / NB, db = c % NB;
      __builtin_amdgcn_sched_barrier(0);
      o[db] = __builtin_amdgcn_mfma_f32_32x32x16_f16(vf[c % kAhead], pf.v[t16], o[db], 0, 0, 0);
      if (c + kAhead < NPV) vf[c % kAhead] = vfrag(sv, c + kAhead);
      if constexpr (kFollow) {
#pragma unroll
        for (int e = 0; e < EV; e += 2) {
          const int r = c * EV + e;
          mloc = fmaxf(fmaxf(sn[r / 16][r % 16], sn[r / 16][r % 16 + 1]), mloc);
        }
      }
      if (c * LPH % NPV == 0 && (kSteady || pre >= 0)) issue_part(pre, LPH + c * LPH / NPV);
    }
    __builtin_amdgcn_sched_barrier(0);
    // The mixed MFMA + vector block and the bookkeeping run at raised priority, the pure MFMA block at the
    // base one: the wavefront with vector work to issue wins the arbiter, the other one's MFMAs fill in.
    __builtin_amdgcn_s_setprio(1);
    if (has_next) {
      if (t + 1 >= n_full_tiles) mloc = mask_tile(sn, t + 1);
      if constexpr (kFollow) update_max(mloc);
    }
  };

  // Ring of kStages buffers, one barrier per tile.  At the top of step t the tiles up to t+2 have been
  // issued; after its barrier everyone is done with tile t-1, whose buffer takes tile t+3.  The loads of
  // tile t+3 are spread over the MFMAs of the step instead of being issued in one burst: the CU moves
  // about 64 bytes per clock from memory into LDS, so a burst of all eight wavefronts backs the queue
  // up and stalls the issuing wavefronts for hundreds of cycles.
  static_assert(kStages == 4, "the wait counts assume this ring depth");
  if (ntiles > 0) {
    f32x16 sa[2], sb[2];
    sb[0] = zero16;
    sb[1] = zero16;
    wait_vmcnt<0>();                        // nothing of the previous item (its output stores) is counted below
    issue_tile(0);
    if (ntiles > 1) issue_tile(1);
    if (ntiles > 2) issue_tile(2);
    if (ntiles > 2) wait_vmcnt<2 * LPT>();
    else if (ntiles > 1) wait_vmcnt<LPT>();
    else wait_vmcnt<0>();
    __syncthreads();
    qk_only(sa, 0);
    {
      float mloc;
      if (0 >= n_full_tiles) {
        mloc = mask_tile(sa, 0);
      } else {
        mloc = sa[0][0];
#pragma unroll
        for (int kb = 0; kb < 2; ++kb)
#pragma unroll
          for (int r = 0; r < 16; r += 2) mloc = fmaxf(fmaxf(sa[kb][r], sa[kb][r + 1]), mloc);
      }
      update_max(mloc);
    }
    int t = 0;
    for (; t + 4 < ntiles && __any(m_run == -INFINITY); t += 2) {   // some row has not seen a key yet
      step(std::true_type{}, std::true_type{}, sa, sb, t);
      step(std::true_type{}, std::true_type{}, sb, sa, t + 1);
    }
    for (; t + 4 < ntiles; t += 2) {
      step(std::true_type{}, std::false_type{}, sa, sb, t);
      step(std::true_type{}, std::false_type{}, sb, sa, t + 1);
    }
    for (; t < ntiles; t += 2) {
      step(std::false_type{}, std::true_type{}, sa, sb, t);
      if (t + 1 < ntiles) step(std::false_type{}, std::true_type{}, sb, sa, t + 1);
    }
  }

  const float l_tot = pair_sum(l_run);
  const float inv = l_tot > 0.f ? 1.0f / l_tot : 0.f;
  if (qvalid) {
    T* optr = static_cast<T*>(p.O) + b * L.qs[0] + i * L.qs[1] + (long long)qrow * L.qs[2];
#pragma unroll
    for (int db = 0; db < D / 32; ++db)
#pragma unroll
      for (int q4 = 0; q4 < 4; ++q4) {
        const int d = db * 32 + 8 * q4 + 4 * h;
        uint2 w;
        w.x = pack_bf16x2(o[db][q4 * 4 + 0] * inv, o[db][q4 * 4 + 1] * inv);
        w.y = pack_bf16x2(o[db][q4 * 4 + 2] * inv, o[db][q4 * 4 + 3] * inv);
        *reinterpret_cast<uint2*>(optr + d) = w;
      }
    if (h == 0)
      p.lse[(long long)bh * L.N + qrow] = l_tot > 0.f ? (m_run * c2 + log2f(l_tot)) * kLn2 : -INFINITY;
  }
  }  // work-item loop
}

// Rows of a head's packed K/V buffer: whole tiles, and never a multiple of 4096 rows -- with a power-of-two
// stride between the heads, workgroups that stream different heads at the same tile index (all of them start
// at tile 0 together) hit the same cache sets and memory channels.
int fwd_npad(int rows) {
  int npad = (int)align_up(rows, kTileN);
  if (npad % 4096 == 0) npad += kTileN;
  return npad;
}

struct FwdWs {
  void* Kp;
  void* Vp;
  int* kidx;
  int* sched;
  int* qvis;
};

FwdWs carve_fwd(Arena& a, const Layer& L, int dtype, int heads, int npad, bool sparse) {
  FwdWs w;
  const size_t es = dtype == OMNI_BF16 ? 2 : 4;
  const size_t rows = (size_t)L.B * heads * npad;
  w.Kp = a.take<unsigned char>(rows * L.D * es);
  w.Vp = a.take<unsigned char>(rows * L.D * es);
  w.kidx = a.take<int>(rows);
  w.sched = a.take<int>(sched_ints(L.B * L.Hq, L.N, kTileM));   // sized for the smaller tile: the longer list
  w.qvis = (sparse && dtype == OMNI_BF16) ? a.take<int>((size_t)L.B * L.Hq * L.N) : nullptr;
  return w;
}

template <typename T, int D>
int launch_fwd(const Layer& L, const void* Q, const void* K, const void* V, const int* q_idx, const int* q_cnt,
               const int* kv_idx, const int* budget, int b_cap, void* O, float* lse, void* ws, bool sparse,
               hipStream_t st, const SelectSource* sel) {
  Arena a(ws);
  const int heads = sparse ? L.Hq : L.Hkv;
  const int npad = fwd_npad(sparse ? b_cap : L.N);
  FwdWs w = carve_fwd(a, L, sizeof(T) == 2 ? OMNI_BF16 : OMNI_F32, heads, npad, sparse);
  {
    const int dt = sizeof(T) == 2 ? OMNI_BF16 : OMNI_F32;
    // bf16: K natural + V k-packed and converted to f16; fp32: both natural
    int rc = run_pack_kv(L, dt, K, V, sparse ? 1 : 0, kv_idx, b_cap, budget, b_cap, npad, kTileN, w.Kp,
                         dt == OMNI_BF16 ? nullptr : w.Vp, nullptr, dt == OMNI_BF16 ? w.Vp : nullptr, w.kidx, st,
                         sparse ? sel : nullptr);
    if (rc != OMNI_OK) return rc;
  }
  if (sparse) {
    {
      ProfScope prof__(kProfClear, st);
      hipLaunchKernelGGL((clear_output_kernel<T>), dim3(cdiv(L.N, 64), L.B * L.Hq), dim3(kThreads), 0, st,
                         static_cast<T*>(O), lse, L);
      OMNI_LAUNCH_CHECK();
    }
  }
  FwdParams p;
  p.Q = Q;
  p.O = O;
  p.lse = lse;
  p.L = L;
  p.q_idx = q_idx;
  p.q_cnt = q_cnt;
  p.Kp = w.Kp;
  p.Vp = w.Vp;
  p.kidx = w.kidx;
  p.budget = budget;
  p.b_cap = b_cap;
  p.npad = npad;
  p.per_q_head = sparse ? 1 : 0;
  p.identity_keys = sparse ? 0 : 1;
  p.sched = w.sched;
  p.qvis = w.qvis;
  p.tile_map = nullptr;
  p.tile_stride = 0;
  if (w.qvis) {
    int rc = run_visible_counts(L, q_idx, q_cnt, w.kidx, budget, b_cap, npad, w.qvis, nullptr, st);
    if (rc != OMNI_OK) return rc;
  }
  constexpr bool kFast = sizeof(T) == 2;
  {
    p.order_off = sched_order_off(L.B * L.Hq, L.N, kFast ? kFastTileM : kTileM);
    // Per-head gathered K/V: one queue per XCD, so that the workgroups on a head share its tiles in that XCD's L2
    // (16.2 -> 5.3 GB from beyond L2 per launch at 64k, at the same kernel time).  The dense baseline and the
    // in-place block lists read one copy per KV group, which the heads of a group already share: splitting them
    // over queues only costs (25.7 -> 25.9 ms dense).
    int rc = run_schedule(L, q_cnt, budget, b_cap, kFast ? kFastTileM : kTileM, w.qvis, w.sched, st,
                          kFast && sparse ? kSchedQueues : 1);
    if (rc != OMNI_OK) return rc;
  }
  {
    ProfScope prof__(kProfAttnFwd, st);
    if constexpr (kFast) {
      hipLaunchKernelGGL((attn_fwd_bf16_kernel<D, false>), dim3(persistent_grid() / 2), dim3(kFastThreads), 0, st, p);
    } else {
      hipLaunchKernelGGL((attn_fwd_kernel<T, D>), dim3(persistent_grid()), dim3(kThreads), 0, st, p);
    }
    OMNI_LAUNCH_CHECK();
  }
  return OMNI_OK;
}

// ---- in-place variant for block lists (the paper's block-sparse kernel: no gather)

// tile_map[bh, t] = tile of the KV head's packed K/V that holds tile t of the head's key list
// grid: (cdiv(blk_cap * tiles_per_block, 256), B*Hq)
__global__ __launch_bounds__(256) void tile_map_kernel(const int* __restrict__ blk_idx, const int* __restrict__ blk_budget,
                                                       int Hq, int blk_cap, int tiles_per_block, int last_tile,
                                                       int* __restrict__ tile_map) {
  const int bh = blockIdx.y, b = bh / Hq;
  const int t = blockIdx.x * blockDim.x + threadIdx.x;
  const int nb = min(blk_budget[b], blk_cap);
  if (t >= blk_cap * tiles_per_block) return;
  int tile = 0;
  if (t < nb * tiles_per_block)
    tile = min(blk_idx[(long long)bh * blk_cap + t / tiles_per_block] * tiles_per_block + t % tiles_per_block, last_tile);
  tile_map[(long long)bh * blk_cap * tiles_per_block + t] = tile;
}

struct BlockFwdWs {
  FwdWs f;
  int* klist;       // [B*Hq, blk_cap * block] token index of every entry of the heads' key lists
  int* vbudget;     // [B] their length
  int* tile_map;    // [B*Hq, blk_cap * block / 64]
};

BlockFwdWs carve_block_fwd(Arena& a, const Layer& L, int cap_keys) {
  BlockFwdWs w;
  w.f = carve_fwd(a, L, OMNI_BF16, L.Hkv, fwd_npad(L.N), false);
  const size_t BH = (size_t)L.B * L.Hq;
  w.f.qvis = a.take<int>(BH * L.N);
  w.klist = a.take<int>(BH * cap_keys);
  w.vbudget = a.take<int>(L.B);
  w.tile_map = a.take<int>(BH * (cap_keys / kTileN));
  return w;
}

template <int D>
int launch_fwd_blocks(const Layer& L, const void* Q, const void* K, const void* V, const int* q_idx, const int* q_cnt,
                      const int* blk_idx, const int* blk_budget, int blk_cap, int block, void* O, float* lse, void* ws,
                      hipStream_t st) {
  typedef u16 T;
  Arena a(ws);
  const int tpb = block / kTileN, cap_keys = blk_cap * block;
  BlockFwdWs w = carve_block_fwd(a, L, cap_keys);
  const int npad = fwd_npad(L.N);
  // K and V of every KV head once, in the kernel's tile layouts, in token order: shared by the heads of a group
  int rc = run_pack_kv(L, OMNI_BF16, K, V, 0, nullptr, L.N, nullptr, L.N, npad, kTileN, w.f.Kp, nullptr, nullptr, w.f.Vp,
                       w.f.kidx, st);
  if (rc != OMNI_OK) return rc;
  {
    ProfScope prof__(kProfClear, st);
    hipLaunchKernelGGL((clear_output_kernel<T>), dim3(cdiv(L.N, 64), L.B * L.Hq), dim3(kThreads), 0, st,
                       static_cast<T*>(O), lse, L);
    OMNI_LAUNCH_CHECK();
  }
  // token lists of the selected blocks (for the causal bounds) and the tile map
  rc = run_expand_blocks(L, blk_idx, blk_budget, blk_cap, block, w.klist, w.vbudget, cap_keys, st);
  if (rc != OMNI_OK) return rc;
  hipLaunchKernelGGL(tile_map_kernel, dim3(cdiv(blk_cap * tpb, 256), L.B * L.Hq), dim3(256), 0, st, blk_idx, blk_budget,
                     L.Hq, blk_cap, tpb, npad / kTileN - 1, w.tile_map);
  OMNI_LAUNCH_CHECK();
  rc = run_visible_counts(L, q_idx, q_cnt, w.klist, w.vbudget, cap_keys, cap_keys, w.f.qvis, nullptr, st);
  if (rc != OMNI_OK) return rc;
  FwdParams p;
  p.Q = Q;
  p.O = O;
  p.lse = lse;
  p.L = L;
  p.q_idx = q_idx;
  p.q_cnt = q_cnt;
  p.Kp = w.f.Kp;
  p.Vp = w.f.Vp;
  p.kidx = w.f.kidx;
  p.budget = w.vbudget;
  p.b_cap = cap_keys;
  p.npad = npad;
  p.per_q_head = 0;
  p.identity_keys = 0;
  p.sched = w.f.sched;
  p.qvis = w.f.qvis;
  p.tile_map = w.tile_map;
  p.tile_stride = blk_cap * tpb;
  p.order_off = sched_order_off(L.B * L.Hq, L.N, kFastTileM);
  rc = run_schedule(L, q_cnt, w.vbudget, cap_keys, kFastTileM, w.f.qvis, w.f.sched, st);
  if (rc != OMNI_OK) return rc;
  {
    ProfScope prof__(kProfAttnFwd, st);
    hipLaunchKernelGGL((attn_fwd_bf16_kernel<D, true>), dim3(persistent_grid() / 2), dim3(kFastThreads), 0, st, p);
    OMNI_LAUNCH_CHECK();
  }
  return OMNI_OK;
}

}  // namespace

size_t attn_fwd_blocks_ws(const Layer& L, int cap_keys) {
  Arena a(nullptr);
  carve_block_fwd(a, L, cap_keys);
  return a.used();
}

int attn_fwd_blocks_max_keys() { return kMaxMapTiles * kTileN; }

int run_tile_map(const Layer& L, const int* blk_idx, const int* blk_budget, int blk_cap, int block, int last_tile,
                 int* tile_map, hipStream_t st) {
  const int tpb = block / kTileN;
  hipLaunchKernelGGL(tile_map_kernel, dim3(cdiv(blk_cap * tpb, 256), L.B * L.Hq), dim3(256), 0, st, blk_idx, blk_budget,
                     L.Hq, blk_cap, tpb, last_tile, tile_map);
  OMNI_LAUNCH_CHECK();
  return OMNI_OK;
}

int run_attn_fwd_blocks(const Layer& L, const void* Q, const void* K, const void* V, const int* q_idx, const int* q_cnt,
                        const int* blk_idx, const int* blk_budget, int blk_cap, int block, void* O, float* lse,
                        void* ws, hipStream_t st) {
  if (L.D == 128)
    return launch_fwd_blocks<128>(L, Q, K, V, q_idx, q_cnt, blk_idx, blk_budget, blk_cap, block, O, lse, ws, st);
  return launch_fwd_blocks<64>(L, Q, K, V, q_idx, q_cnt, blk_idx, blk_budget, blk_cap, block, O, lse, ws, st);
}

size_t attn_fwd_ws(const Layer& L, int dtype, int b_cap, bool sparse) {
  Arena a(nullptr);
  carve_fwd(a, L, dtype, sparse ? L.Hq : L.Hkv, fwd_npad(sparse ? b_cap : L.N), sparse);
  return a.used();
}

int run_attn_fwd(const Layer& L, int dtype, const void* Q, const void* K, const void* V, const int* q_idx,
                 const int* q_cnt, const int* kv_idx, const int* budget, int b_cap, void* O, float* lse, void* ws,
                 bool sparse, hipStream_t st, const SelectSource* sel) {
  if (dtype == OMNI_BF16) {
    if (L.D == 128)
      return launch_fwd<u16, 128>(L, Q, K, V, q_idx, q_cnt, kv_idx, budget, b_cap, O, lse, ws, sparse, st, sel);
    return launch_fwd<u16, 64>(L, Q, K, V, q_idx, q_cnt, kv_idx, budget, b_cap, O, lse, ws, sparse, st, sel);
  }
  if (L.D == 128)
    return launch_fwd<float, 128>(L, Q, K, V, q_idx, q_cnt, kv_idx, budget, b_cap, O, lse, ws, sparse, st, sel);
  return launch_fwd<float, 64>(L, Q, K, V, q_idx, q_cnt, kv_idx, budget, b_cap, O, lse, ws, sparse, st, sel);
}

}  // namespace omni
