// Decode step with KV cache slimming (paper Sec. "KV Cache Slimming",
// decoding-attention equation) and the plain decode baseline.
//
// HBM-bound: one query row per head, so the job is to stream cache rows at memory speed and read
// each of them as few times as possible.  Two kinds of workgroups write partial softmax states:
//
//  * shared rows -- rows that every head of a KV group attends (the whole context for the plain
//    decode, the non-visual rows for the slimmed one).  One workgroup handles a slice of these
//    rows for ALL heads of the group: a row's K and V are loaded once and used for every head.
//  * per-head rows -- the stored visual rows of one query head, read through its index list, only
//    if the head's decoding query is active (omni_slim_decode).
//  * group rows -- the union of the stored visual rows of the heads of a KV group with a membership
//    bit per head (omni_slim_decode_grouped): a row is loaded once if any ACTIVE head of the group
//    stores it, and only the heads that store it see it.  Under grouped-query attention this is
//    what turns fewer rows per head into fewer bytes from HBM, since the plain decode already
//    shares every row between the heads of a group.
//
// bf16 with 2..8 heads per workgroup (stream_rows_mma): a wavefront takes 32 rows per trip and forms both
// products on the matrix cores -- K rows loaded in fragment layout, V rows transposed through a
// wavefront-private LDS tile, the online softmax in the accumulator layout.  Otherwise (fp32 inputs, one
// head per workgroup) a cache row is read by D*sizeof(T)/16 lanes (a lane group) with one 16-byte load
// each for K and V, and the lane group forms the row's dot products and weighted sums on the vector ALU.
// Wavefronts (or lane groups), then slices, are merged with the usual (max, sum, weighted output) rule
// in a fixed order, so results are bitwise reproducible.
#include "common.h"
#include "kernels.h"

#include <algorithm>

namespace omni {

namespace {

constexpr int kThreads = 256;
constexpr int kUnroll = 4;
constexpr float kLog2e = 1.4426950408889634f;
constexpr int kMinRowsPerSlice = 64;  // rows of one pass of a workgroup (bf16, d = 128)
constexpr int kMaxSlices = 256;
constexpr int kRowBlocks = 768;        // workgroups a row-streaming launch aims for: three per CU

struct DecodeParams {
  const void* q;
  const void* K;
  const void* V;
  const int* ctx_len;
  const float* probe;      // nullptr: plain decode (every head attends every row)
  const int* vis_idx;      // per-head lists [B*Hq, b_cap], or group lists [B*Hkv, b_cap] (grouped call)
  const int* vis_cnt;
  const unsigned* grp_mask; // membership bits of the group lists, nullptr for the per-head call
  const void* Kcomp;       // compacted copies of the group lists' rows [B*Hkv, b_cap, D] (row u = cache row
  const void* Vcomp;       // vis_idx[u]), or nullptr: the listed rows are read from the cache itself
  const int* page_table;   // not nullptr: Kcomp / Vcomp are a pool [pool_pages, 1 << page_shift, D] and list position u
  int page_shift, pages_cap, pool_pages;   // of group bg sits in page page_table[bg, u >> page_shift] of it
  int b_cap;
  void* O;
  unsigned char* active;
  float* part;             // [B*Hq, n_shared + n_head, D + 2]
  int B, Hq, Hkv, G, D, cap, v0, v1;
  int n_shared, n_head;    // slices of the shared rows / of a head's own rows
  float scale, tau;
  long long ks[3];
};

// dot of a lane's chunk of q with its chunk of a key row
__device__ __forceinline__ float chunk_dot(const u32x4& qraw, const u32x4& kraw, const u16*) {
  float qv[8], kv[8];
  unpack16(qraw, qv, (const u16*)nullptr);
  unpack16(kraw, kv, (const u16*)nullptr);
  float acc = qv[0] * kv[0];
#pragma unroll
  for (int e = 1; e < 8; ++e) acc = fmaf(qv[e], kv[e], acc);
  return acc;
}
__device__ __forceinline__ float chunk_dot(const u32x4& qraw, const u32x4& kraw, const float*) {
  float acc = __uint_as_float(qraw.x) * __uint_as_float(kraw.x);
  acc = fmaf(__uint_as_float(qraw.y), __uint_as_float(kraw.y), acc);
  acc = fmaf(__uint_as_float(qraw.z), __uint_as_float(kraw.z), acc);
  acc = fmaf(__uint_as_float(qraw.w), __uint_as_float(kraw.w), acc);
  return acc;
}

// Sum over the LPR (a power of two) lanes that share a cache row; every lane gets the total.  Within
// a row of 16 lanes the exchanges are DPP modifiers of the add itself (no LDS traffic).
template <int LPR>
__device__ __forceinline__ float row_group_sum(float v) {
  v += __builtin_bit_cast(float, __builtin_amdgcn_update_dpp(0, __builtin_bit_cast(int, v), 0xB1, 0xF, 0xF, true));   // lane ^ 1
  v += __builtin_bit_cast(float, __builtin_amdgcn_update_dpp(0, __builtin_bit_cast(int, v), 0x4E, 0xF, 0xF, true));   // lane ^ 2
  if (LPR >= 8) v += __builtin_bit_cast(float, __builtin_amdgcn_update_dpp(0, __builtin_bit_cast(int, v), 0x141, 0xF, 0xF, true));  // 7 - lane in a half row
  if (LPR >= 16) v += __builtin_bit_cast(float, __builtin_amdgcn_update_dpp(0, __builtin_bit_cast(int, v), 0x140, 0xF, 0xF, true)); // 15 - lane in a row
#pragma unroll
  for (int o = 16; o < LPR; o <<= 1) v += __shfl_xor(v, o, 64);
  return v;
}

template <int BYTES>
__device__ __forceinline__ unsigned char* lds_block() {
  __shared__ __attribute__((aligned(16))) unsigned char buf[BYTES];
  return buf;
}

// bf16, 2..8 heads per workgroup: both products of a row block on the matrix cores.  A wavefront owns 32
// consecutive list positions per trip and nothing in the loop is shared between wavefronts (no barriers):
//  * S^T = K . q^T: the K rows are the A operand straight from memory (lane = row), the heads' queries the B
//    operand (columns beyond GT are padding that the member words mask: the matrix cores are idle anyway).  Lane (n, h) of the accumulator
//    then holds head n's scores of 16 of the 32 rows, so the online softmax is per-lane arithmetic plus one
//    exchange with lane n + 32, and the weights are a B operand as they stand.
//  * O^T += V^T . P^T: V rows go to a wavefront-private LDS tile as they come from memory (whole rows, coalesced)
//    and are read back transposed, 2 bytes at a time, in the row order the accumulator layout dictates
//    (k index 8 h + e of step s <-> row 16 s + 8 (e / 4) + 4 h + e % 4 on both operands).
// Same contract as stream_rows below.
// The rows come as nsub successive stretches: prep(sub, begin, end) sets the list positions of stretch `sub`
// (it may stage them in LDS and may contain barriers; every thread calls it).
template <int D, int GT, typename RowOf, typename MaskOf, typename Prep>
__device__ __forceinline__ void stream_rows_mma(const DecodeParams& p, int b, int head0, int nsub, Prep prep,
                                                RowOf row_of, MaskOf mask_of, unsigned head_bits, int slot,
                                                const u16* krows, const u16* vrows, long long row_stride) {
  constexpr int kWaves = kThreads / 64;
  constexpr int CPR = D / 8;                 // 16-byte chunks of a row
  constexpr int RPI = 64 / CPR;              // rows one load instruction of a wavefront covers
  constexpr int NVL = 32 / RPI;              // V load instructions of a trip
  constexpr int PITCH = D * 2 + 16;          // bytes between rows of the V tile: lanes n and n + 32 read rows 4 apart
  constexpr int NB = D / 32;
  constexpr int OP = D + 8;                  // floats between (wavefront, head) rows of the merge buffer
  static_assert(kWaves * 8 * OP * 4 <= kWaves * 32 * PITCH, "the merge buffer reuses the V tiles");
  // One LDS block per kernel whatever the list type: the instantiations for the different row_of / mask_of of a
  // kernel are alternatives of which a workgroup runs one.
  constexpr int kTileBytes = kWaves * 32 * PITCH;
  constexpr int QP = D * 2 + 16;             // bytes between the heads' queries in LDS
  unsigned char* sV = lds_block<kTileBytes + kWaves * (32 + 8 + 8) * 4 + 8 * QP>();
  unsigned char* sQ = sV + kTileBytes + kWaves * 48 * 4;
  unsigned (*sMem)[32] = reinterpret_cast<unsigned (*)[32]>(sV + kTileBytes);
  float (*sM)[8] = reinterpret_cast<float (*)[8]>(sV + kTileBytes + kWaves * 32 * 4);
  float (*sL)[8] = reinterpret_cast<float (*)[8]>(sV + kTileBytes + kWaves * 40 * 4);
  const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
  const int n = lane & 31, h = lane >> 5;
  const float c2 = p.scale * kLog2e;
  unsigned char* tile = sV + wave * 32 * PITCH;

  // The queries, B operand of the scores (column n = head, 8 elements of k chunk h), are re-read from LDS every
  // trip: resident they cost 32 registers, a third wavefront per SIMD is worth more.  Columns beyond GT read
  // zero rows or another head's row; the member words mask them either way.
  for (int idx = threadIdx.x; idx < 8 * CPR; idx += kThreads) {
    const int hh = idx / CPR, c = idx % CPR;
    u32x4 raw = {0u, 0u, 0u, 0u};
    if (hh < GT) raw = *reinterpret_cast<const u32x4*>(static_cast<const u16*>(p.q) + (long long)(b * p.Hq + head0 + hh) * D + c * 8);
    *reinterpret_cast<u32x4*>(sQ + hh * QP + c * 16) = raw;
  }
  __syncthreads();
  const unsigned char* qlane = sQ + (n & 7) * QP + h * 16;
  f32x16 o[NB];
#pragma unroll
  for (int db = 0; db < NB; ++db)
#pragma unroll
    for (int i = 0; i < 16; ++i) o[db][i] = 0.f;
  float m = -INFINITY, l = 0.f;              // head n: running maximum (scaled), sum over this lane's rows

  bool any_rows = false;
  for (int sub = 0; sub < nsub; ++sub) {
  int begin = 0, end = 0;
  prep(sub, begin, end);
  any_rows |= begin < end;
  // cache row and member word of list position it0 + 32 wave + n (both lane halves hold it); -1 / 0: nothing to read
  auto fetch_meta = [&](int it0, int& krow, unsigned& mem) {
    const int it = it0 + wave * 32 + n;
    krow = it < end ? row_of(it) : -1;
    mem = krow >= 0 ? (mask_of(it) & head_bits) : 0u;
    if (mem == 0u) krow = -1;
  };
  int krow = -1;
  unsigned mem = 0u;
  if (begin < end) fetch_meta(begin, krow, mem);

  for (int it0 = begin; it0 < end; it0 += kWaves * 32) {
    bf16x8 kf[D / 16];
#pragma unroll
    for (int ks = 0; ks < D / 16; ++ks) {
      u32x4 raw = {0u, 0u, 0u, 0u};
      if (krow >= 0) raw = *reinterpret_cast<const u32x4*>(krows + (long long)krow * row_stride + ks * 16 + h * 8);
      kf[ks] = __builtin_bit_cast(bf16x8, raw);
    }
    u32x4 vraw[NVL];
#pragma unroll
    for (int j = 0; j < NVL; ++j) {
      const int vr = __shfl(krow, j * RPI + lane / CPR, 64);
      vraw[j] = u32x4{0u, 0u, 0u, 0u};
      if (vr >= 0) vraw[j] = *reinterpret_cast<const u32x4*>(vrows + (long long)vr * row_stride + (lane % CPR) * 8);
    }
    if (h == 0) sMem[wave][n] = mem;
    // list lookups of the next trip: a row's address depends on its entry, two dependent latencies would add up
    int krow_n = -1;
    unsigned mem_n = 0u;
    if (it0 + kWaves * 32 < end) fetch_meta(it0 + kWaves * 32, krow_n, mem_n);

    f32x16 sacc;
#pragma unroll
    for (int i = 0; i < 16; ++i) sacc[i] = 0.f;
#pragma unroll
    for (int ks = 0; ks < D / 16; ++ks) sacc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(kf[ks], *reinterpret_cast<const bf16x8*>(qlane + ks * 32), sacc, 0, 0, 0);
#pragma unroll
    for (int j = 0; j < NVL; ++j)
      *reinterpret_cast<u32x4*>(tile + (j * RPI + lane / CPR) * PITCH + (lane % CPR) * 16) = vraw[j];
    asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");        // same wavefront: LDS operations complete in order

    // accumulator register i: row 8 (i / 4) + 4 h + i % 4 of the block, head n
    float sc[16], mx = m;
#pragma unroll
    for (int q4 = 0; q4 < 4; ++q4) {
      const u32x4 mw = *reinterpret_cast<const u32x4*>(&sMem[wave][8 * q4 + 4 * h]);
#pragma unroll
      for (int e = 0; e < 4; ++e) {
        const int i = q4 * 4 + e;
        sc[i] = ((mw[e] >> n) & 1u) ? sacc[i] * c2 : -INFINITY;
        mx = fmaxf(mx, sc[i]);
      }
    }
    mx = pair_max(mx);
    const float mref = mx == -INFINITY ? 0.f : mx;
    const float alpha = mx == m ? 1.f : fast_exp2(m - mref);   // m = -inf -> 0
    float pw[16], ps = 0.f;
#pragma unroll
    for (int i = 0; i < 16; ++i) {
      pw[i] = fast_exp2(sc[i] - mref);
      ps += pw[i];
    }
    l = fmaf(l, alpha, ps);
    m = mx;
    if (__any(alpha != 1.f)) {
#pragma unroll
      for (int db = 0; db < NB; ++db)
#pragma unroll
        for (int i = 0; i < 16; ++i) o[db][i] *= alpha;
    }
    union { bf16x8 v[2]; unsigned w[8]; } pf;
#pragma unroll
    for (int i = 0; i < 16; i += 2) pf.w[i / 2] = pack_bf16x2(pw[i], pw[i + 1]);
#pragma unroll
    for (int s2 = 0; s2 < 2; ++s2)
#pragma unroll
      for (int db = 0; db < NB; ++db) {
        bf16x8 vf;
#pragma unroll
        for (int e = 0; e < 8; ++e)
          vf[e] = *reinterpret_cast<const __bf16*>(tile + (16 * s2 + 8 * (e / 4) + 4 * h + e % 4) * PITCH + (32 * db + n) * 2);
        o[db] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(vf, pf.v[s2], o[db], 0, 0, 0);
      }
    krow = krow_n;
    mem = mem_n;
  }
  }  // stretches

  if (!any_rows) {                          // empty slice: mark it, the combine pass skips its output row
    if (threadIdx.x < GT) {
      float* dst = p.part + ((long long)(b * p.Hq + head0 + threadIdx.x) * (p.n_shared + p.n_head) + slot) * (D + 2);
      dst[D] = -INFINITY;
      dst[D + 1] = 0.f;
    }
    return;
  }
  // merge the wavefronts in wavefront order, one (head, d) per thread
  const float l_tot = pair_sum(l);
  __syncthreads();                          // everyone is done with its V tile: the merge buffer takes its place
  float* sO = reinterpret_cast<float*>(sV);
  if (n < GT) {
#pragma unroll
    for (int db = 0; db < NB; ++db)
#pragma unroll
      for (int q4 = 0; q4 < 4; ++q4) {
        f32x4 v = {o[db][q4 * 4], o[db][q4 * 4 + 1], o[db][q4 * 4 + 2], o[db][q4 * 4 + 3]};
        *reinterpret_cast<f32x4*>(sO + (wave * GT + n) * OP + 32 * db + 8 * q4 + 4 * h) = v;
      }
    if (h == 0) {
      sM[wave][n] = m;
      sL[wave][n] = l_tot;
    }
  }
  __syncthreads();
  for (int idx = threadIdx.x; idx < GT * D; idx += kThreads) {
    const int hh = idx / D, d = idx % D;
    float M = -INFINITY;
#pragma unroll
    for (int w = 0; w < kWaves; ++w) M = fmaxf(M, sM[w][hh]);
    const float Mr = M == -INFINITY ? 0.f : M;
    float Ls = 0.f, Os = 0.f;
#pragma unroll
    for (int w = 0; w < kWaves; ++w) {
      const float wgt = sM[w][hh] == -INFINITY ? 0.f : exp2f(sM[w][hh] - Mr);
      Ls = fmaf(sL[w][hh], wgt, Ls);
      Os = fmaf(sO[(w * GT + hh) * OP + d], wgt, Os);
    }
    float* dst = p.part + ((long long)(b * p.Hq + head0 + hh) * (p.n_shared + p.n_head) + slot) * (D + 2);
    dst[d] = Os;
    if (d == 0) {
      dst[D] = M;
      dst[D + 1] = Ls;
    }
  }
}

// Streams the rows [begin, end) of a virtual row list for GT heads at once and leaves the merged
// partial state of the workgroup in part[head][slot].  row_of maps a list position to a cache row
// or -1.  Every thread of the workgroup must call it (it contains barriers).
// mask_of gives the heads (bit h = head0 + h) that attend the row; heads outside head_bits are skipped
// altogether (a wave-uniform decision) and get an empty partial state.
// krows / vrows point at row 0 of the (batch, KV head) the rows belong to; rows are row_stride elements apart.
template <typename T, int D, int GT, typename RowOf, typename MaskOf, typename Prep>
__device__ __forceinline__ void stream_rows(const DecodeParams& p, int b, int g, int head0, int nsub, Prep prep,
                                            RowOf row_of, MaskOf mask_of, unsigned head_bits, int slot,
                                            const T* krows, const T* vrows, long long row_stride) {
  constexpr int E = Elem<T>::kPer16B;
  constexpr int LPR = D / E;              // lanes per row
  constexpr int RPP = kThreads / LPR;     // lane groups = rows per pass
  // bf16 with 2..8 heads per workgroup: both products on the matrix cores.  Otherwise (fp32, one head, more than
  // 8 heads) every lane group forms its rows' dot products and weighted sums on the vector ALU.
  if constexpr (sizeof(T) == 2 && GT >= 2 && GT <= 8) {
    stream_rows_mma<D, GT>(p, b, head0, nsub, prep, row_of, mask_of, head_bits, slot, krows, vrows, row_stride);
    return;
  }
  constexpr int U = kUnroll;              // rows per lane group and trip
  __shared__ float sM[GT][RPP], sL[GT][RPP];
  __shared__ float sO[RPP][D];
  const int c = threadIdx.x % LPR, grp = threadIdx.x / LPR;
  const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
  const T* kbase = krows + c * E;
  const T* vbase = vrows + c * E;
  const float c2 = p.scale * kLog2e;

  u32x4 qraw[GT];
#pragma unroll
  for (int h = 0; h < GT; ++h)
    qraw[h] = *reinterpret_cast<const u32x4*>(static_cast<const T*>(p.q) + (long long)(b * p.Hq + head0 + h) * D + c * E);
  float m[GT], l[GT], acc[GT][E];
#pragma unroll
  for (int h = 0; h < GT; ++h) {
    m[h] = -INFINITY;
    l[h] = 0.f;
#pragma unroll
    for (int e = 0; e < E; ++e) acc[h][e] = 0.f;
  }

  // online-softmax update of this lane group's state with kUnroll rows: scores s (unscaled), V chunks, members
  auto consume = [&](float (&s)[GT][kUnroll], const u32x4 (&vraw)[kUnroll], const unsigned (&member)[kUnroll]) {
    float vv[kUnroll][E];
#pragma unroll
    for (int u = 0; u < kUnroll; ++u) unpack16(vraw[u], vv[u], (const T*)nullptr);
#pragma unroll
    for (int h = 0; h < GT; ++h) {
      if (!((head_bits >> h) & 1u)) continue;
      float mx = m[h];
#pragma unroll
      for (int u = 0; u < kUnroll; ++u) {
        s[h][u] = ((member[u] >> h) & 1u) ? s[h][u] * c2 : -INFINITY;
        mx = fmaxf(mx, s[h][u]);
      }
      const float mref = mx == -INFINITY ? 0.f : mx;
      const float alpha = fast_exp2(m[h] - mref);               // m = -inf -> 0
      float pw[kUnroll], ps = 0.f;
#pragma unroll
      for (int u = 0; u < kUnroll; ++u) {
        pw[u] = fast_exp2(s[h][u] - mref);
        ps += pw[u];
      }
      l[h] = fmaf(l[h], alpha, ps);
#pragma unroll
      for (int e = 0; e < E; ++e) {
        float a = acc[h][e] * alpha;
#pragma unroll
        for (int u = 0; u < kUnroll; ++u) a = fmaf(pw[u], vv[u][e], a);
        acc[h][e] = a;
      }
      m[h] = mx;
    }
  };

  bool any_rows = false;
  for (int sub = 0; sub < nsub; ++sub) {
  int begin = 0, end = 0;
  prep(sub, begin, end);
  any_rows |= begin < end;
  // rows (and member bits) of a trip: list lookups, so they are fetched one trip ahead of the rows themselves --
  // a row's address depends on its list entry, and two dependent memory latencies per trip would otherwise add up
  auto fetch_meta = [&](int it0, int (&row)[U], unsigned (&member)[U]) {
#pragma unroll
    for (int u = 0; u < U; ++u) {
      const int it = it0 + u * RPP + grp;
      row[u] = it < end ? row_of(it) : -1;
      member[u] = (it < end && row[u] >= 0) ? (mask_of(it) & head_bits) : 0u;
      if (member[u] == 0u) row[u] = -1;                     // nobody wants it: not loaded
    }
  };
  int row[U];
  unsigned member[U];
  if (begin < end) fetch_meta(begin, row, member);

  for (int it0 = begin; it0 < end; it0 += RPP * U) {      // uniform trip count over the workgroup
    u32x4 kraw[U], vraw[U];
    int row_n[U];
    unsigned member_n[U];
#pragma unroll
    for (int u = 0; u < U; ++u) {
      kraw[u] = u32x4{0u, 0u, 0u, 0u};
      vraw[u] = u32x4{0u, 0u, 0u, 0u};
      if (row[u] >= 0) {
        const long long off = (long long)row[u] * row_stride;
        kraw[u] = *reinterpret_cast<const u32x4*>(kbase + off);
        vraw[u] = *reinterpret_cast<const u32x4*>(vbase + off);
      }
    }
    if (it0 + RPP * U < end) fetch_meta(it0 + RPP * U, row_n, member_n);
    float s[GT][kUnroll];
#pragma unroll
    for (int h = 0; h < GT; ++h) {
      if (!((head_bits >> h) & 1u)) continue;
#pragma unroll
      for (int u = 0; u < kUnroll; ++u) s[h][u] = row_group_sum<LPR>(chunk_dot(qraw[h], kraw[u], (const T*)nullptr));
    }
    consume(s, vraw, member);
#pragma unroll
    for (int u = 0; u < U; ++u) {
      row[u] = row_n[u];
      member[u] = member_n[u];
    }
  }
  }  // stretches

  if (!any_rows) {                          // empty slice: mark it, the combine pass skips its output row
    if (threadIdx.x < GT) {
      float* dst = p.part + ((long long)(b * p.Hq + head0 + threadIdx.x) * (p.n_shared + p.n_head) + slot) * (D + 2);
      dst[D] = -INFINITY;
      dst[D + 1] = 0.f;
    }
    return;
  }
  // merge the lane groups of the workgroup in group order, one head at a time
#pragma unroll
  for (int h = 0; h < GT; ++h) {
    __syncthreads();
    if (c == 0) {
      sM[h][grp] = m[h];
      sL[h][grp] = l[h];
    }
#pragma unroll
    for (int e = 0; e < E; ++e) sO[grp][c * E + e] = acc[h][e];
    __syncthreads();
    if (threadIdx.x < D) {
      float M = -INFINITY;
      for (int r = 0; r < RPP; ++r) M = fmaxf(M, sM[h][r]);
      const float Mr = M == -INFINITY ? 0.f : M;
      float Ls = 0.f, Os = 0.f;
      for (int r = 0; r < RPP; ++r) {
        const float w = sM[h][r] == -INFINITY ? 0.f : exp2f(sM[h][r] - Mr);
        Ls = fmaf(sL[h][r], w, Ls);
        Os = fmaf(sO[r][threadIdx.x], w, Os);
      }
      float* dst = p.part + ((long long)(b * p.Hq + head0 + h) * (p.n_shared + p.n_head) + slot) * (D + 2);
      dst[threadIdx.x] = Os;
      if (threadIdx.x == 0) {
        dst[D] = M;
        dst[D + 1] = Ls;
      }
    }
  }
}

// Shared rows of one KV group, GT heads per workgroup: slice `slice` of unit `unit` in [0, B * Hkv * (G / GT)).
template <typename T, int D, int GT>
__device__ __forceinline__ void decode_shared_rows(const DecodeParams& p, int slice, int unit) {
  constexpr int RPP = kThreads / (D / Elem<T>::kPer16B);
  const int chunks = p.G / GT;
  const int chunk = unit % chunks, bg = unit / chunks;
  const int b = bg / p.Hkv, g = bg % p.Hkv;
  const int ctx = min(p.ctx_len[b], p.cap);
  const int n_lo = p.probe ? min(p.v0, ctx) : ctx;       // rows below the visual segment (all rows if plain)
  const int hi0 = min(p.v1, ctx);
  const int n_hi = p.probe ? ctx - hi0 : 0;              // rows above it
  const int total = n_lo + n_hi;
  int per = cdiv(total, p.n_shared);
  per = cdiv(per, RPP * kUnroll) * (RPP * kUnroll);
  const int begin = min(total, slice * per), end = min(total, begin + per);
  stream_rows<T, D, GT>(p, b, g, g * p.G + chunk * GT, 1, [&](int, int& b0_, int& e0_) { b0_ = begin; e0_ = end; },
                        [&](int it) { return it < n_lo ? it : hi0 + (it - n_lo); }, [](int) { return ~0u; },
                        (1u << GT) - 1u, slice, static_cast<const T*>(p.K) + b * p.ks[0] + g * p.ks[1],
                        static_cast<const T*>(p.V) + b * p.ks[0] + g * p.ks[1], p.ks[2]);
}

// A head's own (stored visual) rows: slice `slice` of head bh.  Also classifies the decoding query.
template <typename T, int D>
__device__ __forceinline__ void decode_head_rows(const DecodeParams& p, int slice, int bh) {
  constexpr int RPP = kThreads / (D / Elem<T>::kPer16B);
  __shared__ int sActive;
  const int b = bh / p.Hq, i = bh % p.Hq, g = i / p.G;
  if (threadIdx.x < 64) {
    const T* qptr = static_cast<const T*>(p.q) + (long long)bh * D;
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
  const int act = sActive;
  if (slice == 0 && threadIdx.x == 0 && p.active) p.active[bh] = (unsigned char)act;
  const int ctx = min(p.ctx_len[b], p.cap);
  const int total = act ? min(p.vis_cnt[bh], p.b_cap) : 0;
  int per = cdiv(total, p.n_head);
  per = cdiv(per, RPP * kUnroll) * (RPP * kUnroll);
  const int begin = min(total, slice * per), end = min(total, begin + per);
  const int* vlist = p.vis_idx + (long long)bh * p.b_cap;
  stream_rows<T, D, 1>(p, b, g, i, 1, [&](int, int& b0_, int& e0_) { b0_ = begin; e0_ = end; },
                       [&](int it) {
                         const int r = vlist[it];
                         return (unsigned)r < (unsigned)ctx ? r : -1;          // stored rows beyond the context are ignored
                       },
                       [](int) { return 1u; }, 1u, p.n_shared + slice,
                       static_cast<const T*>(p.K) + b * p.ks[0] + g * p.ks[1],
                       static_cast<const T*>(p.V) + b * p.ks[0] + g * p.ks[1], p.ks[2]);
}

// The union list of a KV group, GT heads per workgroup: slice `slice` of unit `unit`.  Classifies the
// decoding queries of its heads first: only active heads take part.
template <typename T, int D, int GT>
__device__ __forceinline__ void decode_group_rows(const DecodeParams& p, int slice, int unit) {
  constexpr int RPP = kThreads / (D / Elem<T>::kPer16B);
  __shared__ unsigned sBits;
  const int chunks = p.G / GT;
  const int chunk = unit % chunks, bg = unit / chunks;
  const int b = bg / p.Hkv, g = bg % p.Hkv;
  const int head0 = g * p.G + chunk * GT;
  if (threadIdx.x == 0) sBits = 0u;
  __syncthreads();
  {
    const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
    const float* pk = p.probe + ((long long)(b * p.Hkv + g) * 2) * D;
    for (int h = wave; h < GT; h += kThreads / 64) {
      const int i = head0 + h;
      const T* qptr = static_cast<const T*>(p.q) + (long long)(b * p.Hq + i) * D;
      float dot = 0.f;
      for (int d = lane; d < D; d += 64) dot = fmaf(Elem<T>::load(qptr + d), pk[D + d] - pk[d], dot);
      dot = wave_sum(dot);
      if (lane == 0) {
        const float score = 1.0f / (1.0f + expf(-dot * p.scale));
        const int act = (i == 0 || score > p.tau) ? 1 : 0;
        if (act) atomicOr(&sBits, 1u << h);
        if (slice == 0 && p.active) p.active[b * p.Hq + i] = (unsigned char)act;
      }
    }
  }
  __syncthreads();
  const unsigned bits = sBits;
  const int ctx = min(p.ctx_len[b], p.cap);
  const int total = bits ? min(p.vis_cnt[bg], p.b_cap) : 0;
  int per = cdiv(total, p.n_head);
  per = cdiv(per, RPP * kUnroll) * (RPP * kUnroll);
  const int begin = min(total, slice * per), end = min(total, begin + per);
  const int* vlist = p.vis_idx + (long long)bg * p.b_cap;
  const unsigned* mlist = p.grp_mask + (long long)bg * p.b_cap;
  const int shift = chunk * GT;
  if (p.page_table) {            // the listed rows sit in pages of a pool: position -> (page, offset) -> pool row
    // The slice's stretch of the page table goes to LDS first: a table entry fetched from memory next to every
    // list entry costs 4 % of the call at batch 8.
    constexpr int kStaged = 128;
    __shared__ int sPages[kStaged];
    const int* table = p.page_table + (long long)bg * p.pages_cap;
    const int pshift = p.page_shift, pmask = (1 << p.page_shift) - 1;
    const int slot0 = begin >> pshift, nslots = begin < end ? ((end - 1) >> pshift) - slot0 + 1 : 0;
    const bool staged = nslots <= kStaged;
    if (staged) {
      for (int i = threadIdx.x; i < nslots; i += kThreads) sPages[i] = slot0 + i < p.pages_cap ? table[slot0 + i] : -1;
      __syncthreads();
    }
    stream_rows<T, D, GT>(p, b, g, head0, 1, [&](int, int& b0_, int& e0_) { b0_ = begin; e0_ = end; },
                          [&](int it) {
                            const int slot = it >> pshift;
                            if ((unsigned)vlist[it] >= (unsigned)ctx || slot >= p.pages_cap) return -1;
                            const int page = staged ? sPages[slot - slot0] : table[slot];
                            return (unsigned)page < (unsigned)p.pool_pages ? (page << pshift) + (it & pmask) : -1;
                          },
                          [&](int it) { return mlist[it] >> shift; }, bits, p.n_shared + slice,
                          static_cast<const T*>(p.Kcomp), static_cast<const T*>(p.Vcomp), (long long)D);
    return;
  }
  if (p.Kcomp) {                 // the listed rows sit side by side in the compacted store: position = row
    const long long base = (long long)bg * p.b_cap * D;
    stream_rows<T, D, GT>(p, b, g, head0, 1, [&](int, int& b0_, int& e0_) { b0_ = begin; e0_ = end; },
                          [&](int it) { return (unsigned)vlist[it] < (unsigned)ctx ? it : -1; },
                          [&](int it) { return mlist[it] >> shift; }, bits, p.n_shared + slice,
                          static_cast<const T*>(p.Kcomp) + base, static_cast<const T*>(p.Vcomp) + base, (long long)D);
    return;
  }
  stream_rows<T, D, GT>(p, b, g, head0, 1, [&](int, int& b0_, int& e0_) { b0_ = begin; e0_ = end; },
                        [&](int it) {
                          const int r = vlist[it];
                          return (unsigned)r < (unsigned)ctx ? r : -1;
                        },
                        [&](int it) { return mlist[it] >> shift; }, bits, p.n_shared + slice,
                        static_cast<const T*>(p.K) + b * p.ks[0] + g * p.ks[1],
                        static_cast<const T*>(p.V) + b * p.ks[0] + g * p.ks[1], p.ks[2]);
}

// The per-head lists of a KV group merged on the fly (omni_slim_decode under grouped-query attention): slice `slice`
// of unit `unit` owns a stretch of the visual token range and walks it kMergeSpan tokens at a time.  For every span
// the active heads' list entries that fall into it are marked in an LDS bitmap (bit h of word t: head h stores
// token t), the marked tokens are compacted, in ascending order, into an LDS list with their member words, and the
// rows are streamed exactly as from a stored group list -- a row is loaded once, whichever of the heads store it.
// Reading the lists costs 4 bytes per stored entry and active head, against 4 D bytes per row.
constexpr int kMergeSpan = 1024;            // tokens of a span
constexpr int kMergeWindow = kMergeSpan;    // list entries read per head and span: no more can fall into it

// First positions of two ascending lists a0[0, n0), a1[0, n1) whose values are >= v, found together by one
// wavefront (all lanes take part and get both results): 64 probes per list and round, the loads of both lists in
// flight at once.  Three rounds for lists of up to 2^18 entries.  (More probes per round would save a round but
// every probe is a cache line of its own: with a thousand workgroups searching seven lists each, 256 probes per
// round move more bytes than the rows of the step.)
__device__ __forceinline__ void wave_lower_bound2(const int* __restrict__ a0, int n0, const int* __restrict__ a1, int n1,
                                                  int v, int& r0, int& r1) {
  const int lane = threadIdx.x & 63;
  const int* a[2] = {a0, a1};
  int lo[2] = {0, 0}, hi[2] = {n0, n1};                 // the answers lie in [lo, hi]
  for (;;) {
    const bool last = hi[0] - lo[0] <= 64 && hi[1] - lo[1] <= 64;        // wave-uniform
    int val[2], step[2];
#pragma unroll
    for (int w = 0; w < 2; ++w) {
      step[w] = max(1, cdiv(hi[w] - lo[w], 64));
      const int idx = lo[w] + lane * step[w];
      val[w] = idx < hi[w] ? a[w][idx] : 0x7fffffff;
    }
#pragma unroll
    for (int w = 0; w < 2; ++w) {
      const int below = __popcll(__ballot(val[w] < v));  // probes ascend with the lane: those below v are a prefix
      if (below == 0) {
        hi[w] = lo[w];
      } else {
        const int nlo = lo[w] + (below - 1) * step[w] + 1;
        hi[w] = min(hi[w], lo[w] + below * step[w]);
        lo[w] = nlo;
      }
    }
    if (last) break;                                    // the steps were 1: lo = hi = the answer
  }
  r0 = lo[0];
  r1 = lo[1];
}

template <typename T, int D, int GT>
__device__ __forceinline__ void decode_merged_rows(const DecodeParams& p, int slice, int unit) {
  __shared__ unsigned sBits;
  __shared__ int sCur[GT];                              // per head: first list entry not yet consumed
  __shared__ int sCount;
  __shared__ int sWaveSum[kThreads / 64];
  __shared__ unsigned sWord[kMergeSpan];                // bitmap of a span, then the member words of its list
  __shared__ int sTok[kMergeSpan];
  const int chunks = p.G / GT;
  const int chunk = unit % chunks, bg = unit / chunks;
  const int b = bg / p.Hkv, g = bg % p.Hkv;
  const int head0 = g * p.G + chunk * GT;
  const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
  const int ctx = min(p.ctx_len[b], p.cap);
  const int vis_hi = min(p.v1, ctx);                    // stored rows beyond the context are ignored
  const int span_tokens = max(0, vis_hi - p.v0);
  const int per = cdiv(max(1, p.v1 - p.v0), p.n_head);   // tokens per slice
  const int t_begin = p.v0 + min(span_tokens, slice * per), t_end = p.v0 + min(span_tokens, (slice + 1) * per);
  const int nsub_all = cdiv(t_end - t_begin, kMergeSpan);
  if (threadIdx.x == 0) sBits = 0u;
  __syncthreads();
  {
    const float* pk = p.probe + ((long long)(b * p.Hkv + g) * 2) * D;
    for (int h = wave; h < GT; h += kThreads / 64) {
      const int i = head0 + h;
      const T* qptr = static_cast<const T*>(p.q) + (long long)(b * p.Hq + i) * D;
      float dot = 0.f;
      for (int d = lane; d < D; d += 64) dot = fmaf(Elem<T>::load(qptr + d), pk[D + d] - pk[d], dot);
      dot = wave_sum(dot);
      if (lane == 0) {
        const float score = 1.0f / (1.0f + expf(-dot * p.scale));
        const int act = (i == 0 || score > p.tau) ? 1 : 0;
        if (act) atomicOr(&sBits, 1u << h);
        if (slice == 0 && p.active) p.active[b * p.Hq + i] = (unsigned char)act;
      }
    }
  }
  __syncthreads();
  const unsigned bits = sBits;
  const int nsub = bits ? nsub_all : 0;
  // A wavefront looks after heads `wave` and `wave + 4` of the tile (GT <= 8), both at once; a head that is lazy,
  // or beyond GT, is an empty list.
  static_assert(GT <= 2 * (kThreads / 64), "two heads per wavefront");
  const int* hlist[2];
  int hcnt[2];
#pragma unroll
  for (int w = 0; w < 2; ++w) {
    const int h = wave + w * (kThreads / 64);
    const bool on = h < GT && ((bits >> h) & 1u) && nsub > 0;
    const int bh = b * p.Hq + head0 + (h < GT ? h : 0);
    hlist[w] = p.vis_idx + (long long)bh * p.b_cap;
    hcnt[w] = on ? max(0, min(p.vis_cnt[bh], p.b_cap)) : 0;
  }
  if (nsub > 0) {                                       // where the lists enter the slice
    int c0, c1;
    wave_lower_bound2(hlist[0], hcnt[0], hlist[1], hcnt[1], t_begin, c0, c1);
    if (lane == 0) {
      if (wave < GT) sCur[wave] = c0;
      if (wave + kThreads / 64 < GT) sCur[wave + kThreads / 64] = c1;
    }
  }
  __syncthreads();
  auto prep = [&](int sub, int& begin, int& end) {
    const int t_lo = t_begin + sub * kMergeSpan, t_hi = min(t_end, t_lo + kMergeSpan);
    __syncthreads();                                    // the previous span's list is no longer read
    for (int t = threadIdx.x; t < kMergeSpan; t += kThreads) sWord[t] = 0u;
    __syncthreads();
    {
      // ascending entries: those of this span are among the next kMergeWindow entries of a list.  The loads of both
      // lists of the wavefront are issued before any is used.
      constexpr int NK = kMergeWindow / 64;
      int tok[2][NK], cur[2];
#pragma unroll
      for (int w = 0; w < 2; ++w) {
        const int h = wave + w * (kThreads / 64);
        cur[w] = h < GT ? sCur[h] : 0;
#pragma unroll
        for (int k = 0; k < NK; ++k) {
          const int e = cur[w] + k * 64 + lane;
          tok[w][k] = e < hcnt[w] ? hlist[w][e] : 0x7fffffff;
        }
      }
#pragma unroll
      for (int w = 0; w < 2; ++w) {
        const int h = wave + w * (kThreads / 64);
        if (hcnt[w] == 0) continue;                     // wave-uniform
        int taken = 0;
#pragma unroll
        for (int k = 0; k < NK; ++k) {
          const bool in = tok[w][k] < t_hi;
          if (in && tok[w][k] >= t_lo) atomicOr(&sWord[tok[w][k] - t_lo], 1u << h);
          taken += __popcll(__ballot(in));
        }
        if (lane == 0) sCur[h] = cur[w] + taken;
      }
    }
    __syncthreads();
    // compaction in token order: every thread owns kMergeSpan / kThreads consecutive words
    constexpr int PER = kMergeSpan / kThreads;
    unsigned w[PER];
    int mine = 0;
#pragma unroll
    for (int j = 0; j < PER; ++j) {
      w[j] = sWord[threadIdx.x * PER + j];
      mine += w[j] != 0u;
    }
    int incl = mine;
#pragma unroll
    for (int o = 1; o < 64; o <<= 1) {
      const int up = __shfl_up(incl, o, 64);
      if (lane >= o) incl += up;
    }
    if (lane == 63) sWaveSum[wave] = incl;
    __syncthreads();                                    // every word is in registers: the list may take their place
    int base = 0;
    for (int k = 0; k < wave; ++k) base += sWaveSum[k];
    if (threadIdx.x == kThreads - 1) sCount = base + incl;
    int at = base + incl - mine;
#pragma unroll
    for (int j = 0; j < PER; ++j)
      if (w[j] != 0u) {
        sTok[at] = t_lo + threadIdx.x * PER + j;
        sWord[at] = w[j];
        ++at;
      }
    __syncthreads();
    begin = 0;
    end = sCount;
  };
  stream_rows<T, D, GT>(p, b, g, head0, nsub, prep, [&](int it) { return sTok[it]; }, [&](int it) { return sWord[it]; },
                        bits, p.n_shared + slice, static_cast<const T*>(p.K) + b * p.ks[0] + g * p.ks[1],
                        static_cast<const T*>(p.V) + b * p.ks[0] + g * p.ks[1], p.ks[2]);
}

// Merges the slices of one head.  grid = B * Hq, kCombineThreads threads: lane groups of D/2 threads (two
// output elements each) take the slices round-robin with many independent loads in flight, then the
// groups are summed in group order.
constexpr int kCombineThreads = 1024;

template <typename T, int D>
__global__ __launch_bounds__(kCombineThreads) void decode_combine_kernel(DecodeParams p) {
  constexpr int LG = D / 2;                        // threads per slice
  constexpr int NG = kCombineThreads / LG;         // slices in flight per pass
  __shared__ float sRed[kCombineThreads / 64];
  __shared__ float sMax;
  __shared__ float sL[NG];
  __shared__ float sO[NG][D];
  const int bh = blockIdx.x;
  const int n = p.n_shared + p.n_head;
  const float* src = p.part + (long long)bh * n * (D + 2);
  // global maximum over the slices
  float M = -INFINITY;
  for (int s = threadIdx.x; s < n; s += kCombineThreads) M = fmaxf(M, src[s * (D + 2) + D]);
  M = wave_max(M);
  if ((threadIdx.x & 63) == 0) sRed[threadIdx.x >> 6] = M;
  __syncthreads();
  if (threadIdx.x == 0) {
    float m = -INFINITY;
    for (int w = 0; w < kCombineThreads / 64; ++w) m = fmaxf(m, sRed[w]);
    sMax = m;
  }
  __syncthreads();
  const float Mr = sMax == -INFINITY ? 0.f : sMax;
  const int grp = threadIdx.x / LG, c = threadIdx.x % LG;
  float Ls = 0.f, O0 = 0.f, O1 = 0.f;
  // every load of a trip is issued before any is used (a branch on the slice's maximum would put two memory
  // latencies in sequence per slice); an empty slice, or one with nothing visible in it, may hold an unwritten
  // output row, so it is dropped by selection, not by a zero weight
#pragma unroll 4
  for (int s = grp; s < n; s += NG) {
    const float* row = src + s * (D + 2);
    const float ms = row[D], ls = row[D + 1];
    const float2 o = *reinterpret_cast<const float2*>(row + 2 * c);
    const bool live = ms != -INFINITY;
    const float w = fast_exp2(ms - Mr);
    Ls = live ? fmaf(ls, w, Ls) : Ls;
    O0 = live ? fmaf(o.x, w, O0) : O0;
    O1 = live ? fmaf(o.y, w, O1) : O1;
  }
  if (c == 0) sL[grp] = Ls;
  sO[grp][2 * c] = O0;
  sO[grp][2 * c + 1] = O1;
  __syncthreads();
  if (threadIdx.x < D) {
    float Lt = 0.f, Ot = 0.f;
    for (int g2 = 0; g2 < NG; ++g2) {
      Lt += sL[g2];
      Ot += sO[g2][threadIdx.x];
    }
    Elem<T>::store(static_cast<T*>(p.O) + (long long)bh * D + threadIdx.x, Lt > 0.f ? Ot / Lt : 0.f);
  }
}

// heads of a KV group handled by one workgroup of the shared-row kernel: the largest supported divisor of G
int group_tile(int G) {
  if (G % 8 == 0) return 8;
  if (G % 7 == 0) return 7;
  if (G % 4 == 0) return 4;
  if (G % 2 == 0) return 2;
  return 1;
}

constexpr int kNoLists = 0, kStoredGroupLists = 1, kMergedHeadLists = 2;

// One launch for the row streams of a step that share a register footprint.  With lists (the stored group lists, or
// the per-head lists of a group merged on the fly -- a kernel of its own, so that its bookkeeping does not cost the
// stored-list kernel registers): the lists, then the
// shared rows -- the list workgroups come first in the grid (they are the long ones) and the few shared
// (non-visual) rows of a slimmed step fill in behind them instead of costing a launch of their own (11 us at
// batch 1).  Otherwise the shared rows only (plain decode; per-head lists, whose one-head workgroups need half
// the registers and lose their occupancy inside a common kernel: 70 -> 84 us when fused).
template <typename T, int D, int GT, int LISTS>
__global__ __launch_bounds__(kThreads, 3) void decode_rows_kernel(DecodeParams p) {
  const int units_s = p.B * p.Hkv * (p.G / GT);
  const int n_list = LISTS ? p.n_head * units_s : 0;
  const int i = blockIdx.x;
  if constexpr (LISTS == kStoredGroupLists) {
    if (i < n_list) {
      decode_group_rows<T, D, GT>(p, i % p.n_head, i / p.n_head);
      return;
    }
  }
  if constexpr (LISTS == kMergedHeadLists) {
    if (i < n_list) {
      decode_merged_rows<T, D, GT>(p, i % p.n_head, i / p.n_head);
      return;
    }
  }
  const int j = i - n_list;
  decode_shared_rows<T, D, GT>(p, j % p.n_shared, j / p.n_shared);
}

// grid = (n_head, B * Hq)
template <typename T, int D>
__global__ __launch_bounds__(kThreads) void decode_head_kernel(DecodeParams p) {
  decode_head_rows<T, D>(p, blockIdx.x, blockIdx.y);
}

template <typename T, int D, int GT>
void launch_rows(const DecodeParams& p, hipStream_t st) {
  const int units_s = p.B * p.Hkv * (p.G / GT);
  const int n_shared = p.n_shared * units_s;
  // group lists, or per-head lists of a group of two or more heads (merged on the fly into the rows of the group)
  if (p.n_head > 0 && p.grp_mask) {
    hipLaunchKernelGGL((decode_rows_kernel<T, D, GT, kStoredGroupLists>), dim3(n_shared + p.n_head * units_s),
                       dim3(kThreads), 0, st, p);
    return;
  }
  if (p.n_head > 0 && GT >= 2) {
    hipLaunchKernelGGL((decode_rows_kernel<T, D, GT, kMergedHeadLists>), dim3(n_shared + p.n_head * units_s),
                       dim3(kThreads), 0, st, p);
    return;
  }
  if (p.n_head > 0)      // per-head lists: the long kernel first
    hipLaunchKernelGGL((decode_head_kernel<T, D>), dim3(p.n_head, p.B * p.Hq), dim3(kThreads), 0, st, p);
  hipLaunchKernelGGL((decode_rows_kernel<T, D, GT, kNoLists>), dim3(n_shared), dim3(kThreads), 0, st, p);
}

template <typename T, int D>
int launch_decode(const DecodeParams& p, hipStream_t st) {
  {
    ProfScope prof__(kProfDecode, st);
    switch (group_tile(p.G)) {
      case 8: launch_rows<T, D, 8>(p, st); break;
      case 7: launch_rows<T, D, 7>(p, st); break;
      case 4: launch_rows<T, D, 4>(p, st); break;
      case 2: launch_rows<T, D, 2>(p, st); break;
      default: launch_rows<T, D, 1>(p, st); break;
    }
    OMNI_LAUNCH_CHECK();
    hipLaunchKernelGGL((decode_combine_kernel<T, D>), dim3(p.B * p.Hq), dim3(kCombineThreads), 0, st, p);
    OMNI_LAUNCH_CHECK();
  }
  return OMNI_OK;
}

int slices_for(long long rows, int units, int target_blocks) {
  // as many slices as it takes to reach the wanted number of workgroups, but no slice below one pass of a
  // workgroup (64 rows): a short row list (the few thousand non-visual rows of the slimmed decode) would
  // otherwise run as a handful of long, latency-bound workgroups
  long long s = cdiv(rows, (long long)kMinRowsPerSlice);
  const long long want = cdiv(target_blocks, units);
  if (s > want) s = want;
  if (s < 1) s = 1;
  if (s > kMaxSlices) s = kMaxSlices;
  return (int)s;
}

struct Slices {
  int n_shared, n_head;
};

// Slice counts depend on the descriptor only (not on device-side counts), so the workspace size is static.
Slices decode_slices(const omni_decode_desc* d, bool slim) {
  Slices s;
  const int G = d->n_q_heads / d->n_kv_heads;
  const int units = d->batch * d->n_kv_heads * (G / group_tile(G));
  const long long shared_rows = slim ? (long long)d->cache_capacity - (d->vis_end - d->vis_begin) : d->cache_capacity;
  // two workgroups per CU: with more, the merge of a workgroup's lane groups and the slice combine weigh more
  // than the parallelism gains (plain decode at batch 1: 89 us with 1024 workgroups, 75 us with 512)
  s.n_shared = slices_for(shared_rows, units, kRowBlocks);
  // only the active heads (typically a quarter) have rows to read, so aim higher
  s.n_head = slim ? slices_for(d->vis_end - d->vis_begin, d->batch * d->n_q_heads, 8192) : 0;
  return s;
}

}  // namespace

// ---- compaction of the group lists' rows (paper Sec. "KV Cache Slimming": the selected KV pairs are what is stored)

namespace {
// grid: (cdiv(u_cap, rows per block), B*Hkv); a row is copied by D*sizeof(T)/16 lanes
template <typename T, int D>
__global__ __launch_bounds__(kThreads) void compact_rows_kernel(const T* __restrict__ K, const T* __restrict__ V,
                                                               const int* __restrict__ idx,
                                                               const int* __restrict__ cnt, int u_cap, int Hkv, int cap,
                                                               long long s0, long long s1, long long s2,
                                                               T* __restrict__ Kc, T* __restrict__ Vc,
                                                               const int* __restrict__ page_table, int page_shift,
                                                               int pages_cap, int pool_pages) {
  constexpr int E = Elem<T>::kPer16B;
  constexpr int LPR = D / E;
  constexpr int RPB = kThreads / LPR;
  const int bg = blockIdx.y, b = bg / Hkv, g = bg % Hkv;
  const int c = threadIdx.x % LPR, u = blockIdx.x * RPB + threadIdx.x / LPR;
  if (u >= min(cnt[bg], u_cap)) return;
  const int row = idx[(long long)bg * u_cap + u];
  if (row < 0 || row >= cap) return;
  const long long src = b * s0 + g * s1 + (long long)row * s2 + c * E;
  long long dst = ((long long)bg * u_cap + u) * D + c * E;
  if (page_table) {
    const int slot = u >> page_shift;
    if (slot >= pages_cap) return;
    const int page = page_table[(long long)bg * pages_cap + slot];
    if ((unsigned)page >= (unsigned)pool_pages) return;          // page not allocated: the row is not stored
    dst = ((long long)((page << page_shift) + (u & ((1 << page_shift) - 1)))) * D + c * E;
  }
  *reinterpret_cast<u32x4*>(Kc + dst) = *reinterpret_cast<const u32x4*>(K + src);
  *reinterpret_cast<u32x4*>(Vc + dst) = *reinterpret_cast<const u32x4*>(V + src);
}

template <typename T, int D>
int launch_compact(const omni_decode_desc* d, const void* K, const void* V, const int* idx, const int* cnt, int u_cap,
                   void* Kc, void* Vc, const PagePool* pool, hipStream_t st) {
  constexpr int RPB = kThreads / (D / Elem<T>::kPer16B);
  hipLaunchKernelGGL((compact_rows_kernel<T, D>), dim3(cdiv(u_cap, RPB), d->batch * d->n_kv_heads), dim3(kThreads), 0,
                     st, static_cast<const T*>(K), static_cast<const T*>(V), idx, cnt, u_cap, d->n_kv_heads,
                     d->cache_capacity, d->kv_stride[0], d->kv_stride[1], d->kv_stride[2], static_cast<T*>(Kc),
                     static_cast<T*>(Vc), pool ? pool->page_table : nullptr, pool ? pool->page_shift : 0,
                     pool ? pool->pages_cap : 0, pool ? pool->pool_pages : 0);
  OMNI_LAUNCH_CHECK();
  return OMNI_OK;
}
}  // namespace

int run_compact_cache(const omni_decode_desc* d, const void* K, const void* V, const int* grp_idx, const int* grp_cnt,
                      int u_cap, void* Kc, void* Vc, hipStream_t st, const PagePool* pool) {
  if (d->dtype == OMNI_BF16) {
    if (d->head_dim == 128) return launch_compact<u16, 128>(d, K, V, grp_idx, grp_cnt, u_cap, Kc, Vc, pool, st);
    return launch_compact<u16, 64>(d, K, V, grp_idx, grp_cnt, u_cap, Kc, Vc, pool, st);
  }
  if (d->head_dim == 128) return launch_compact<float, 128>(d, K, V, grp_idx, grp_cnt, u_cap, Kc, Vc, pool, st);
  return launch_compact<float, 64>(d, K, V, grp_idx, grp_cnt, u_cap, Kc, Vc, pool, st);
}

size_t decode_ws(const omni_decode_desc* d) {
  Arena a(nullptr);
  // one size for both calls: the larger of the slimmed and the plain slice counts
  const Slices s1 = decode_slices(d, true);
  const Slices s0 = decode_slices(d, false);
  const int n = s1.n_shared + s1.n_head > s0.n_shared ? s1.n_shared + s1.n_head : s0.n_shared;
  a.take<float>((size_t)d->batch * d->n_q_heads * n * (d->head_dim + 2));
  return a.used();
}

int run_decode(const omni_decode_desc* d, const void* q, const void* K, const void* V, const int* ctx_len,
               const float* probe, const int* vis_idx, const int* vis_cnt, const unsigned* grp_mask, int b_cap,
               void* O, unsigned char* active, void* ws, hipStream_t st, const void* Kcomp, const void* Vcomp,
               const PagePool* pool) {
  Arena a(ws);
  DecodeParams p;
  p.q = q;
  p.K = K;
  p.V = V;
  p.ctx_len = ctx_len;
  p.probe = probe;
  p.vis_idx = vis_idx;
  p.vis_cnt = vis_cnt;
  p.grp_mask = grp_mask;
  p.Kcomp = Kcomp;
  p.Vcomp = Vcomp;
  p.page_table = pool ? pool->page_table : nullptr;
  p.page_shift = pool ? pool->page_shift : 0;
  p.pages_cap = pool ? pool->pages_cap : 0;
  p.pool_pages = pool ? pool->pool_pages : 0;
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
  const Slices s = decode_slices(d, probe != nullptr);
  p.n_shared = s.n_shared;
  p.n_head = s.n_head;
  if (grp_mask || (probe && group_tile(p.G) >= 2)) {
    // group lists (stored, or merged on the fly from the per-head lists): one workgroup serves all heads of a
    // group, so fewer, longer slices do
    const int units = p.B * p.Hkv * (p.G / group_tile(p.G));
    p.n_head = std::min(s.n_head, slices_for(d->vis_end - d->vis_begin, units, kRowBlocks));
  }
  p.scale = d->softmax_scale;
  p.tau = d->tau;
  for (int k = 0; k < 3; ++k) p.ks[k] = d->kv_stride[k];
  p.part = a.take<float>((size_t)p.B * p.Hq * (p.n_shared + p.n_head) * (p.D + 2));
  if (d->dtype == OMNI_BF16) {
    if (p.D == 128) return launch_decode<u16, 128>(p, st);
    return launch_decode<u16, 64>(p, st);
  }
  if (p.D == 128) return launch_decode<float, 128>(p, st);
  return launch_decode<float, 64>(p, st);
}

}  // namespace omni
