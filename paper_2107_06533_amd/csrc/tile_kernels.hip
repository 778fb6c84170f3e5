// Grouped tile kernels: one launch runs a whole list of 128x128 tile jobs that may belong to
// different layers / matrices / operand layouts.
#include "tile_core.h"
#include "launch.h"

namespace kfac {

// XCD-aware job order: consecutive workgroup ids are dealt round-robin to the 8 XCDs, so
// workgroup g runs job  (g % 8) * ceil(n/8) + g / 8 : every XCD walks one contiguous
// eighth of the (locality-ordered) job list and its L2 sees neighbouring tiles.
__device__ __forceinline__ int xcd_job_index(int g, int n) {
  const int per = (n + 7) >> 3;
  return (g & 7) * per + (g >> 3);
}

__global__ __launch_bounds__(NT, 2) void tile_any_kernel(const TileDesc* __restrict__ descs,
                                                         const TileJob* __restrict__ jobs, int njobs,
                                                         int xcd_order) {
  __shared__ float smem[TILE_LDS_FLOATS];
  int g = blockIdx.x;
  if (xcd_order) g = xcd_job_index(g, njobs);
  if (g >= njobs) return;
  const TileJob J = jobs[g];
  const TileDesc& D = descs[J.desc];
  run_tile_any(D, J, smem);
}

// Only row-major operands (preconditioning products, sweep updates): smaller code, same engine.
__global__ __launch_bounds__(NT, 2) void tile_gemm_kernel(const TileDesc* __restrict__ descs,
                                                          const TileJob* __restrict__ jobs, int njobs,
                                                          int xcd_order) {
  __shared__ float smem[TILE_LDS_FLOATS];
  int g = blockIdx.x;
  if (xcd_order) g = xcd_job_index(g, njobs);
  if (g >= njobs) return;
  const TileJob J = jobs[g];
  const TileDesc& D = descs[J.desc];
  if (D.a.type == OP_KMAJOR)
    run_tile<KMajorLoader, KMajorLoader>(D, J, smem);
  else
    run_tile<ConvLoader<1, 1>, KMajorLoader>(D, J, smem);
}

// out = beta*out + alpha * (partial[part0] + partial[part0+1] + ...) in slot order (deterministic).
__global__ __launch_bounds__(NT) void tile_reduce_kernel(const TileDesc* __restrict__ descs,
                                                         const ReduceJob* __restrict__ jobs, int njobs) {
  const int g = blockIdx.x;
  if (g >= njobs) return;
  const ReduceJob J = jobs[g];
  const TileDesc& D = descs[J.desc];
  const bool diag = D.sym && J.bi == J.bj;
  const bool mirror = D.mirror == MIRROR_ALL || (D.mirror == MIRROR_DIAG_TILE && diag);
  const float* P = D.partial + (size_t)J.part0 * (BM * BN);
  for (int e = threadIdx.x; e < BM * BN; e += NT) {
    const int li = e >> 7, lj = e & (BN - 1);
    const int gi = J.bi * BM + li, gj = J.bj * BN + lj;
    if (gi >= D.M || gj >= D.N || (D.sym && gi < gj)) continue;
    float s = 0.f;
    for (int k = 0; k < J.nsplit; ++k) s += P[(size_t)k * (BM * BN) + e];
    float* o = D.out + (size_t)gi * D.ldo + gj;
    float val = D.alpha * s;
    if (D.beta != 0.f) val += D.beta * *o;
    *o = val;
    if (mirror && gi != gj) D.out[(size_t)gj * D.ldo + gi] = val;
  }
}

void launch_tile_any(const TileDesc* descs, const TileJob* jobs, int njobs, int xcd_order, hipStream_t s) {
  if (njobs <= 0) return;
  const int grid = xcd_order ? ((njobs + 7) / 8) * 8 : njobs;
  hipLaunchKernelGGL(tile_any_kernel, dim3(grid), dim3(NT), 0, s, descs, jobs, njobs, xcd_order);
}

void launch_tile_gemm(const TileDesc* descs, const TileJob* jobs, int njobs, int xcd_order, hipStream_t s) {
  if (njobs <= 0) return;
  const int grid = xcd_order ? ((njobs + 7) / 8) * 8 : njobs;
  hipLaunchKernelGGL(tile_gemm_kernel, dim3(grid), dim3(NT), 0, s, descs, jobs, njobs, xcd_order);
}

void launch_tile_reduce(const TileDesc* descs, const ReduceJob* jobs, int njobs, hipStream_t s) {
  if (njobs <= 0) return;
  hipLaunchKernelGGL(tile_reduce_kernel, dim3(njobs), dim3(NT), 0, s, descs, jobs, njobs);
}

}  // namespace kfac
