// Builds the per-XCD work list described in sched.h (one tiny kernel, no host sync).
#include "sched.h"

namespace omni {

namespace {

__global__ void schedule_kernel(const int* __restrict__ q_cnt, const int* __restrict__ budget, int B, int Hq, int N,
                                int b_cap, int causal, int tile_m, int* __restrict__ sched) {
  if (threadIdx.x == 0 && blockIdx.x == 0) sched_build(q_cnt, budget, B, Hq, N, b_cap, causal, tile_m, sched);
}

}  // namespace

int run_schedule(const Layer& L, const int* q_cnt, const int* budget, int b_cap, int tile_m, int* sched,
                 hipStream_t st) {
  hipLaunchKernelGGL(schedule_kernel, dim3(1), dim3(64), 0, st, q_cnt, budget, L.B, L.Hq, L.N, b_cap, L.causal, tile_m,
                     sched);
  OMNI_LAUNCH_CHECK();
  return OMNI_OK;
}

int persistent_grid() {
  static int grid = 0;
  if (grid == 0) {
    int dev = 0, cus = 0;
    if (hipGetDevice(&dev) != hipSuccess ||
        hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess || cus <= 0)
      cus = 256;
    grid = 2 * cus;
  }
  return grid;
}

}  // namespace omni
