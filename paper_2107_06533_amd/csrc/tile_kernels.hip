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

#ifndef KFAC_WAVES
#define KFAC_WAVES 2
#endif
__global__ __launch_bounds__(NT, KFAC_WAVES) void tile_any_kernel(const TileDesc* __restrict__ descs,
                                                         const TileJob* __restrict__ jobs, int njobs,
                                                         int xcd_order) {
  __shared__ float smem[TILE_LDS_FLOATS];
  int g = blockIdx.x;
  if (xcd_order) g = xcd_job_index(g, njobs);
  if (g >= njobs) return;
  const TileJob J = jobs[g];
  if (J.desc < 0) return;   // padding of an XCD segment
  const TileDesc& D = descs[J.desc];
  if (D.sym) run_tile_sym(D, J, smem);
  else run_tile_lag(D, J, smem);
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
  if (J.desc < 0) return;   // padding of an XCD segment
  const TileDesc& D = descs[J.desc];
  if (D.a.type == OP_KMAJOR)
    run_tile<KMajorLoader, KMajorLoader, true>(D, J, smem);
  else
    run_tile<ConvLoader<1, 1>, KMajorLoader, true>(D, J, smem);
}

// out = beta*out + alpha * (partial[part0] + partial[part0+1] + ...) in slot order (deterministic).
// Four workgroups per tile; a thread owns four float4 pieces and keeps all their loads in flight.
__global__ __launch_bounds__(NT) void tile_reduce_kernel(const TileDesc* __restrict__ descs,
                                                         const ReduceJob* __restrict__ jobs, int njobs) {
  const int g = blockIdx.x >> 2, quarter = blockIdx.x & 3;
  if (g >= njobs) return;
  const ReduceJob J = jobs[g];
  const TileDesc& D = descs[J.desc];
  const bool diag = D.sym && J.bi == J.bj;
  const bool mirror = D.mirror == MIRROR_ALL || (D.mirror == MIRROR_DIAG_TILE && diag);
  typedef float f32x4 __attribute__((ext_vector_type(4)));
  typedef const f32x4 __attribute__((address_space(1)))* gc4_ptr;
  gc4_ptr P = (gc4_ptr)(D.partial + (size_t)J.part0 * (BM * BN));
  const uint32_t ldo4 = (uint32_t)D.ldo * 4u;
  const rsrc_t ro = make_rsrc(D.out, (uint32_t)D.M * ldo4);
  f32x4 acc[4];
  float old[4][4];
  uint32_t off[4][4];
#pragma unroll
  for (int u = 0; u < 4; ++u) {
    acc[u] = f32x4{0.f, 0.f, 0.f, 0.f};
    const int e = (quarter * 1024 + u * NT + (int)threadIdx.x) * 4;
    const int gi = J.bi * BM + (e >> 7);
#pragma unroll
    for (int c = 0; c < 4; ++c) {
      const int gj = J.bj * BN + (e & (BN - 1)) + c;
      const bool ok = gi < D.M && gj < D.N && (!D.sym || gi >= gj);
      off[u][c] = ok ? (uint32_t)gi * ldo4 + (uint32_t)gj * 4u : OOB_OFFSET;
      old[u][c] = D.beta != 0.f ? buf_load(ro, off[u][c]) : 0.f;
    }
  }
  for (int k = 0; k < J.nsplit; ++k) {
#pragma unroll
    for (int u = 0; u < 4; ++u) {
      acc[u] += P[(size_t)k * (BM * BN / 4) + quarter * 1024 + u * NT + threadIdx.x];
    }
  }
#pragma unroll
  for (int u = 0; u < 4; ++u) {
    const float a4[4] = {acc[u][0], acc[u][1], acc[u][2], acc[u][3]};
    const int e = (quarter * 1024 + u * NT + (int)threadIdx.x) * 4;
    const int gi = J.bi * BM + (e >> 7);
#pragma unroll
    for (int c = 0; c < 4; ++c) {
      const int gj = J.bj * BN + (e & (BN - 1)) + c;
      const float val = D.alpha * a4[c] + D.beta * old[u][c];
      buf_store(ro, off[u][c], val);
      if (mirror)
        buf_store(ro, (off[u][c] != OOB_OFFSET && gi != gj) ? (uint32_t)gj * ldo4 + (uint32_t)gi * 4u : OOB_OFFSET, val);
    }
  }
}

// Assembly of a lag-product activation factor (see LagAsm): one 64 x 64 tile of the lower triangle
// of A per workgroup; every element is a sum of at most four entries of the small lag matrices,
// blended with the old value and written to both (q, q') and (q', q).
constexpr int LAG_TILE = 64;
__device__ __forceinline__ float lag_value(const LagAsm& L, int q, int q2) {
  // value of the raw sum for row q (a real tap column) and column q2 (tap column or the bias column)
  const int C = L.C, ld1 = 10 * C, ld2 = 3 * C + L.bias, lds = 25 * C + L.bias;
  const int c = q / 9, t = q - 9 * c, i = t / 3, j = t - 3 * i;
  float v;
  int col;
  if (q2 == 9 * C) {            // bias column: sums of a over the pixels the tap keeps
    v = L.G[LAG_G2][(size_t)c * ld2 + 3 * C];
    col = 25 * C;
  } else {
    const int c2 = q2 / 9, t2 = q2 - 9 * c2, i2 = t2 / 3, j2 = t2 - 3 * i2;
    const int dy = i2 - i, dx = j2 - j;
    if (dy > 0) v = L.G[LAG_G1][(size_t)c * ld1 + c2 * 10 + (dy - 1) * 5 + dx + 2];
    else if (dy == 0 && dx >= 0) v = L.G[LAG_G2][(size_t)c * ld2 + c2 * 3 + dx];
    else if (dy < 0) v = L.G[LAG_G1][(size_t)c2 * ld1 + c * 10 + (-dy - 1) * 5 - dx + 2];
    else v = L.G[LAG_G2][(size_t)c2 * ld2 + c * 3 - dx];
    col = c2 * 25 + (dy + 2) * 5 + dx + 2;
  }
  // pixels q whose output pixel q - (t - 1) lies outside the grid: bottom row for i = 0, top row
  // for i = 2, right column for j = 0, left column for j = 2
  const int rs = i == 0 ? LAG_BOT : (i == 2 ? LAG_TOP : -1);
  const int cs = j == 0 ? LAG_RIGHT : (j == 2 ? LAG_LEFT : -1);
  const size_t e = (size_t)c * lds + col;
  if (rs >= 0) v -= L.G[rs][e];
  if (cs >= 0) v -= L.G[cs][e];
  if (rs >= 0 && cs >= 0) v += L.G[LAG_TL + (rs == LAG_BOT ? 2 : 0) + (cs == LAG_RIGHT ? 1 : 0)][e];
  return v;
}

__global__ __launch_bounds__(NT) void lag_assemble_kernel(const LagAsm* __restrict__ lags,
                                                          const LagJob* __restrict__ jobs, int njobs) {
  const int g = blockIdx.x;
  if (g >= njobs) return;
  const LagJob J = jobs[g];
  const LagAsm L = lags[J.lag];
  const int dA = L.dA, nb = 9 * L.C;
  for (int e = threadIdx.x; e < LAG_TILE * LAG_TILE; e += NT) {
    const int q = J.bi * LAG_TILE + (e >> 6), q2 = J.bj * LAG_TILE + (e & (LAG_TILE - 1));
    if (q >= dA || q2 > q) continue;
    float v;
    if (q < nb) v = lag_value(L, q, q2);               // q2 <= q < nb: both are tap columns
    else if (q2 < nb) v = lag_value(L, q2, q);         // bias row: the mirrored bias-column entry
    else v = L.rows;                                   // bias-bias
    const float old = L.beta != 0.f ? L.A[(size_t)q * dA + q2] : 0.f;
    const float val = L.alpha * v + L.beta * old;
    L.A[(size_t)q * dA + q2] = val;
    if (q2 != q) L.A[(size_t)q2 * dA + q] = val;
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

void launch_lag_assemble(const LagAsm* lags, const LagJob* jobs, int njobs, hipStream_t s) {
  if (njobs <= 0) return;
  hipLaunchKernelGGL(lag_assemble_kernel, dim3(njobs), dim3(NT), 0, s, lags, jobs, njobs);
}

void launch_tile_reduce(const TileDesc* descs, const ReduceJob* jobs, int njobs, hipStream_t s) {
  if (njobs <= 0) return;
  hipLaunchKernelGGL(tile_reduce_kernel, dim3(njobs * 4), dim3(NT), 0, s, descs, jobs, njobs);
}

}  // namespace kfac
