// Shared host/device helpers of the gfx950 OmniSparse library (internal).
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>
#include <stddef.h>

#include "../../include/omnisparse.h"

namespace omni {

// ---------------------------------------------------------------- host side

void set_error(const char* fmt, ...);
void clear_error();

#define OMNI_FAIL(code, ...)        \
  do {                              \
    ::omni::set_error(__VA_ARGS__); \
    return (code);                  \
  } while (0)

#define OMNI_HIP_CHECK(expr)                                                          \
  do {                                                                                \
    hipError_t e__ = (expr);                                                          \
    if (e__ != hipSuccess) OMNI_FAIL(OMNI_ERR_HIP, "%s: %s", #expr, hipGetErrorString(e__)); \
  } while (0)

#define OMNI_LAUNCH_CHECK() OMNI_HIP_CHECK(hipGetLastError())

__host__ __device__ static inline size_t align_up(size_t x, size_t a) { return (x + a - 1) / a * a; }
__host__ __device__ static inline int cdiv(int a, int b) { return (a + b - 1) / b; }

// Bump allocator over the caller's workspace.
struct Arena {
  char* base;
  size_t off;
  explicit Arena(void* p) : base(static_cast<char*>(p)), off(0) {}
  template <typename T>
  T* take(size_t n) {
    off = align_up(off, 256);
    T* r = base ? reinterpret_cast<T*>(base + off) : nullptr;
    off += n * sizeof(T);
    return r;
  }
  size_t used() const { return align_up(off, 256); }
};

int validate_layer(const omni_layer_desc* d);
int validate_decode(const omni_decode_desc* d);
int check_ws(const void* ws, size_t have, size_t need);

// Plain-data copy of the descriptor with derived fields, passed to kernels by value.
struct Layer {
  int B, Hq, Hkv, G, D, N;
  int ld;                        // elements between the heads' rows of the caller's [B,Hq,.] score and query-index arrays:
                                 // N, or the padded length when the layer is one sequence of a padded batch
  int v0, v1, sink;
  int causal;
  int bph;                       // 1: the budget array holds one key count per head [B,Hq], 0: one per batch item [B]
  float scale;
  long long qs[3];
  long long ks[3];
};
Layer make_layer(const omni_layer_desc* d);
// Entry of a budget array that holds the key count of head bh (b = bh / Hq).
__host__ __device__ inline int budget_slot(int bph, int b, int bh) { return bph ? bh : b; }

// Optional HIP-event timing of individual kernels (omni_profile_* in the C ABI).
enum ProfId {
  kProfAttnFwd = 0, kProfPack = 1, kProfClear = 2, kProfPool = 3, kProfProbeLse = 4, kProfProbeSum = 5,
  kProfScore = 6, kProfBwdDkDv = 7, kProfBwdDq = 8, kProfBwdReduce = 9, kProfDecode = 10, kProfSelect = 11,
  kProfCount = 12
};
void prof_begin(int id, hipStream_t st);
void prof_end(int id, hipStream_t st);
struct ProfScope {
  int id;
  hipStream_t st;
  ProfScope(int i, hipStream_t s) : id(i), st(s) { prof_begin(id, st); }
  ~ProfScope() { prof_end(id, st); }
};

constexpr int kTileM = 128;   // query rows per attention workgroup
constexpr int kTileN = 64;    // keys per attention tile
constexpr int kPadKeyIndex = 0x7fffffff;

// ---------------------------------------------------------------- device side

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef __bf16 bf16x4 __attribute__((ext_vector_type(4)));
typedef __bf16 bf16x2 __attribute__((ext_vector_type(2)));
typedef _Float16 f16x8 __attribute__((ext_vector_type(8)));
typedef _Float16 f16x2 __attribute__((ext_vector_type(2)));
typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef float f32x4 __attribute__((ext_vector_type(4)));
typedef float f32x2 __attribute__((ext_vector_type(2)));
typedef int i32x4 __attribute__((ext_vector_type(4)));
typedef unsigned int u32x4 __attribute__((ext_vector_type(4)));
typedef unsigned int u32x2 __attribute__((ext_vector_type(2)));
typedef unsigned short u16;

__device__ __forceinline__ float bf16_bits_to_f32(u16 h) {
  return __uint_as_float(((unsigned)h) << 16);
}
// float -> bf16, round to nearest even (v_cvt_pk_bf16_f32 on gfx950)
__device__ __forceinline__ u16 f32_to_bf16_bits(float f) { return __builtin_bit_cast(u16, (__bf16)f); }
__device__ __forceinline__ unsigned pack_bf16x2(float lo, float hi) {
  const f32x2 v = {lo, hi};
  return __builtin_bit_cast(unsigned, __builtin_convertvector(v, bf16x2));
}
// 2^x as one v_exp_f32 (no denormal range fix-up: tiny results flush towards 0, which is what softmax wants)
__device__ __forceinline__ float fast_exp2(float x) { return __builtin_amdgcn_exp2f(x); }

// A 32x32 MFMA accumulator column is shared by lane l and lane l ^ 32: combine the two halves
// with one v_permlane32_swap instead of a trip through the LDS crossbar.
__device__ __forceinline__ float pair_max(float x) {
  const u32x2 r = __builtin_amdgcn_permlane32_swap(__float_as_uint(x), __float_as_uint(x), false, false);
  return fmaxf(__uint_as_float(r.x), __uint_as_float(r.y));
}
__device__ __forceinline__ float pair_sum(float x) {
  const u32x2 r = __builtin_amdgcn_permlane32_swap(__float_as_uint(x), __float_as_uint(x), false, false);
  return __uint_as_float(r.x) + __uint_as_float(r.y);
}

template <typename T>
struct Elem;
template <>
struct Elem<float> {
  static constexpr int kPer16B = 4;
  __device__ static __forceinline__ float load(const float* p) { return *p; }
  __device__ static __forceinline__ void store(float* p, float v) { *p = v; }
};
template <>
struct Elem<u16> {
  static constexpr int kPer16B = 8;
  __device__ static __forceinline__ float load(const u16* p) { return bf16_bits_to_f32(*p); }
  __device__ static __forceinline__ void store(u16* p, float v) { *p = f32_to_bf16_bits(v); }
};

// 16-byte chunk -> floats
__device__ __forceinline__ void unpack16(const u32x4& raw, float (&out)[4], const float*) {
  out[0] = __uint_as_float(raw.x);
  out[1] = __uint_as_float(raw.y);
  out[2] = __uint_as_float(raw.z);
  out[3] = __uint_as_float(raw.w);
}
__device__ __forceinline__ void unpack16(const u32x4& raw, float (&out)[8], const u16*) {
  out[0] = __uint_as_float(raw.x << 16);
  out[1] = __uint_as_float(raw.x & 0xffff0000u);
  out[2] = __uint_as_float(raw.y << 16);
  out[3] = __uint_as_float(raw.y & 0xffff0000u);
  out[4] = __uint_as_float(raw.z << 16);
  out[5] = __uint_as_float(raw.z & 0xffff0000u);
  out[6] = __uint_as_float(raw.w << 16);
  out[7] = __uint_as_float(raw.w & 0xffff0000u);
}

// 16 bytes per lane, global -> LDS at lds_addr + lane * 16 (lds_addr wave-uniform).  M0 is saved and restored.
__device__ __forceinline__ void gload_lds16(const void* gptr, unsigned lds_addr) {
  unsigned saved;
  asm volatile(
      "s_mov_b32 %0, m0\n\t"
      "s_mov_b32 m0, %2\n\t"
      "s_nop 0\n\t"
      "global_load_lds_dwordx4 %1, off\n\t"
      "s_mov_b32 m0, %0"
      : "=&s"(saved)
      : "v"(gptr), "s"(lds_addr)
      : "memory");
}
// The same with the global address split into a wave-uniform base (SGPR pair) and a 32-bit per-lane byte
// offset: no 64-bit vector address arithmetic, and one VGPR per distinct lane pattern instead of two per load.
__device__ __forceinline__ void gload_lds16(const void* sbase, unsigned lane_off, unsigned lds_addr) {
  unsigned saved;
  asm volatile(
      "s_mov_b32 %0, m0\n\t"
      "s_mov_b32 m0, %3\n\t"
      "s_nop 0\n\t"
      "global_load_lds_dwordx4 %1, %2\n\t"
      "s_mov_b32 m0, %0"
      : "=&s"(saved)
      : "v"(lane_off), "s"(sbase), "s"(lds_addr)
      : "memory");
}
// 4 bytes per lane, global -> LDS at lds_addr + lane * 4
__device__ __forceinline__ void gload_lds4(const void* gptr, unsigned lds_addr) {
  unsigned saved;
  asm volatile(
      "s_mov_b32 %0, m0\n\t"
      "s_mov_b32 m0, %2\n\t"
      "s_nop 0\n\t"
      "global_load_lds_dword %1, off\n\t"
      "s_mov_b32 m0, %0"
      : "=&s"(saved)
      : "v"(gptr), "s"(lds_addr)
      : "memory");
}
template <int N>
__device__ __forceinline__ void wait_vmcnt() {
  asm volatile("s_waitcnt vmcnt(%0)" ::"n"(N) : "memory");
}

__device__ __forceinline__ int upper_count(const int* __restrict__ a, int n, int v) {
  int lo = 0, hi = n;
  while (lo < hi) {
    const int mid = (lo + hi) >> 1;
    if (a[mid] <= v) lo = mid + 1; else hi = mid;
  }
  return lo;
}

__device__ __forceinline__ int lane_id() { return threadIdx.x & 63; }

template <typename T>
__device__ __forceinline__ T wave_sum(T v) {
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) v += __shfl_xor(v, o, 64);
  return v;
}
__device__ __forceinline__ float wave_max(float v) {
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) v = fmaxf(v, __shfl_xor(v, o, 64));
  return v;
}

// order-preserving map float bits -> unsigned (larger float <=> larger key)
__device__ __forceinline__ unsigned float_key(float f) {
  unsigned u = __float_as_uint(f);
  return (u & 0x80000000u) ? ~u : (u | 0x80000000u);
}

}  // namespace omni
