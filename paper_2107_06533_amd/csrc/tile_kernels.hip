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
#ifdef KFAC_TRACE
__device__ long long* g_factor_trace = nullptr;   // debugging aid: [0] = record count, then 4 words per tile job
#endif
__global__ __launch_bounds__(NT, KFAC_WAVES) void tile_any_kernel(const TileDesc* __restrict__ descs,
                                                         const TileJob* __restrict__ jobs, int njobs,
                                                         int xcd_order) {
  __shared__ __attribute__((aligned(16))) float smem[TILE_LDS_FLOATS];
  int g = blockIdx.x;
  if (xcd_order) g = xcd_job_index(g, njobs);
  if (g >= njobs) return;
  const TileJob J = jobs[g];
  if (J.desc < 0) return;   // padding of an XCD segment
  const TileDesc& D = descs[J.desc];
#ifdef KFAC_TRACE
  const long long t0 = wall_clock64();
#endif
  if (D.sym) run_tile_sym(D, J, smem);
  else run_tile_lag(D, J, smem);
#ifdef KFAC_TRACE
  if (g_factor_trace && threadIdx.x == 0) {
    const unsigned long long r = atomicAdd((unsigned long long*)g_factor_trace, 1ull);
    if (r < 100000) {
      long long* rec = g_factor_trace + 1 + r * 4;
      rec[0] = ((long long)D.a.type << 8) | ((long long)D.b.type << 16) | (D.sym ? 1 : 0) | ((long long)(J.part >= 0) << 1);
      rec[1] = J.kend - J.kbeg; rec[2] = t0; rec[3] = wall_clock64();
    }
  }
#endif
}
#ifdef KFAC_TRACE
extern "C" int kfac_debug_factor_trace(long long* out, int max_recs) {   // first call arms the trace
  static long long* buf = nullptr;
  if (!buf) {
    (void)hipMalloc(reinterpret_cast<void**>(&buf), (1 + 4 * 100000) * sizeof(long long));
    (void)hipMemset(buf, 0, (1 + 4 * 100000) * sizeof(long long));
    (void)hipMemcpyToSymbol(HIP_SYMBOL(g_factor_trace), &buf, sizeof(buf));
    return 0;
  }
  (void)hipDeviceSynchronize();
  long long n = 0;
  (void)hipMemcpy(&n, buf, sizeof(n), hipMemcpyDeviceToHost);
  if (n > 100000) n = 100000;
  if (n > max_recs) n = max_recs;
  if (out && n > 0) (void)hipMemcpy(out, buf + 1, size_t(n) * 32, hipMemcpyDeviceToHost);
  (void)hipMemset(buf, 0, sizeof(long long));
  return int(n);
}
#endif

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
  if (D.b.type == OP_KMAJOR)
    run_tile<KMajorLoader, KMajorLoader, true>(D, J, smem);
  else
    run_tile<KMajorLoader, ConvLoader<1, 1>, true>(D, J, smem);   // second operand stored [N, K] (read transposed)
}

// Plain products of two row-major operands through the direct-to-LDS loop (32 KB of LDS, four
// workgroups per compute unit): the second product of the preconditioning.
__global__ __launch_bounds__(NT, 4) void tile_gemm_dl_kernel(const TileDesc* __restrict__ descs,
                                                             const TileJob* __restrict__ jobs, int njobs) {
  __shared__ __attribute__((aligned(16))) float smem[DL_LDS_FLOATS];
  const int g = blockIdx.x;
  if (g >= njobs) return;
  const TileJob J = jobs[g];
  run_tile_dl<false, false>(descs[J.desc], J, smem);
}

// The same for the bulk products of the inverse, which give way to the latency-critical kernels of the
// sweep chain that share their compute unit (see cu_enter in tile_core.h).  The off-chain launches add
// unused LDS so that one such workgroup fills a compute unit but for the room a chain kernel needs;
// nothing then hides the epilogue, so the old output values are fetched before the k loop.
__global__ __launch_bounds__(NT, 2) void tile_gemm_yield_kernel(const TileDesc* __restrict__ descs, const TileJob* __restrict__ jobs,
                                                                int njobs, const int* __restrict__ cu_flags) {
  __shared__ __attribute__((aligned(16))) float smem[DL_LDS_FLOATS];
  const int g = blockIdx.x;
  if (g >= njobs) return;
  const TileJob J = jobs[g];
  run_tile_dl<true, true>(descs[J.desc], J, smem, cu_flags);
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
      if (D.packed && D.sym && off[u][c] != OOB_OFFSET)   // element (gj, gi) of the upper triangle
        as_global(D.packed)[(size_t)gj * D.M - (size_t)gj * (gj - 1) / 2 + (size_t)(gi - gj)] = val;
    }
  }
}

// Assembly of a lag-product activation factor (see LagAsm): one 64 x 64 tile of the lower triangle
// of A per workgroup; every element is a sum of at most four entries of the small lag matrices,
// blended with the old value and written to both (q, q') and (q', q).
constexpr int LAG_TILE = 64;
// Raw sum for the tap column (c, i, j) against the tap column (c2, i2, j2), or against the bias
// column when isbias (then c2 = C, i2 = j2 = 0 are ignored).  All offsets fit 32 bits.
__device__ __forceinline__ float lag_value(const LagAsm& L, int c, int i, int j, int c2, int i2, int j2, bool isbias) {
  const uint32_t C = (uint32_t)L.C, ld1 = 10u * C, ld2 = 3u * C + L.bias, ld5 = 5u * C + L.bias, ldc = C + L.bias;
  const int dy = isbias ? 0 : i2 - i, dx = isbias ? 0 : j2 - j;
  gcf_ptr G1 = as_global(L.G[LAG_G1]);
  gcf_ptr G2 = as_global(L.G[LAG_G2]);
  float v;   // forward lags are stored; a backward lag is the transposed entry of its opposite
  if (isbias) v = G2[c * ld2 + 3u * C];   // sums of a over the whole image
  else if (dy > 0) v = G1[c * ld1 + c2 * 10 + (dy - 1) * 5 + dx + 2];
  else if (dy == 0 && dx >= 0) v = G2[c * ld2 + c2 * 3 + dx];
  else if (dy < 0) v = G1[c2 * ld1 + c * 10 + (-dy - 1) * 5 - dx + 2];
  else v = G2[c2 * ld2 + c * 3 - dx];
  // Pixels q whose output pixel q - (t - 1) lies outside the grid are taken out again: bottom row for
  // i = 0, top row for i = 2, right column for j = 0, left column for j = 2.  The partner pixel q + lag
  // of a pixel in the bottom row lies below the image unless dy <= 0, and the tap i = 0 only asks for
  // dy >= 0 (the top row: the other way round), so a row strip contributes for dy = 0 only; a column
  // strip for dx = 0 only; their common corner pixel for lag 0 only.  In the bias column (c2 = C,
  // dy = dx = 0) the indices below land on the ones column of every strip.
  if (i != 1 && dy == 0) {
    gcf_ptr S = as_global(i == 0 ? L.G[LAG_BOT] : L.G[LAG_TOP]);                           // [C][5C + bias], lags dx = -2..2
    v -= S[c * ld5 + c2 * 5 + (isbias ? 0 : dx + 2)];
  }
  if (j != 1 && dx == 0) {
    gcf_ptr S = as_global(j == 0 ? L.G[LAG_RIGHT] : L.G[LAG_LEFT]);                        // [C][5C + bias], lags dy = -2..2
    v -= S[c * ld5 + c2 * 5 + (isbias ? 0 : dy + 2)];
  }
  if (i != 1 && j != 1 && dy == 0 && dx == 0) {
    gcf_ptr S = as_global(i == 0 ? (j == 0 ? L.G[LAG_BR] : L.G[LAG_BL]) : (j == 0 ? L.G[LAG_TR] : L.G[LAG_TL]));   // [C][C + bias]
    v += S[c * ldc + c2];
  }
  return v;
}

// One 64 x 64 tile of the lower triangle of A per workgroup (thread = one column, 16 rows).  Only
// elements on or below the diagonal are computed; the mirror image goes through LDS so that both
// copies are stored row by row, and both hold the same bits.
__global__ __launch_bounds__(NT) void lag_assemble_kernel(const LagAsm* __restrict__ lags,
                                                          const LagJob* __restrict__ jobs, int njobs) {
  __shared__ float tile[LAG_TILE][LAG_TILE + 1];
  const int g = blockIdx.x;
  if (g >= njobs) return;
  const LagJob J = jobs[g];
  const LagAsm L = lags[J.lag];
  const int dA = L.dA, nb = 9 * L.C;
  constexpr int PER = LAG_TILE * LAG_TILE / NT;
  gf_ptr A = as_global(L.A);
  // a wave shares its row: row-derived index arithmetic runs on the scalar unit
  const int lc = threadIdx.x & (LAG_TILE - 1), lr0 = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
  const int cc = J.bj * LAG_TILE + lc;                  // this thread's column
  const bool cbias = cc >= nb;
  const int c2 = cbias ? L.C : cc / 9, t2 = cbias ? 0 : cc - 9 * c2, i2 = t2 / 3, j2 = t2 - 3 * i2;
  float v[PER], old[PER];
#pragma unroll
  for (int u = 0; u < PER; ++u) {
    const int r = J.bi * LAG_TILE + lr0 + 4 * u;
    v[u] = 0.f; old[u] = 0.f;
    if (r >= dA || cc > r) continue;
    if (r < nb) {
      const int c = r / 9, t = r - 9 * c, i = t / 3, j = t - 3 * i;
      v[u] = lag_value(L, c, i, j, c2, i2, j2, false);
    } else if (!cbias) {
      v[u] = lag_value(L, c2, i2, j2, L.C, 0, 0, true);   // bias row: the mirrored bias-column entry
    } else {
      v[u] = L.rows;                                      // bias-bias
    }
    if (L.beta != 0.f) old[u] = A[(uint32_t)r * (uint32_t)dA + (uint32_t)cc];
  }
#pragma unroll
  for (int u = 0; u < PER; ++u) {
    const int lr = lr0 + 4 * u, r = J.bi * LAG_TILE + lr;
    const float val = L.alpha * v[u] + L.beta * old[u];
    tile[lr][lc] = val;
    if (r < dA && cc <= r) A[(uint32_t)r * (uint32_t)dA + (uint32_t)cc] = val;
    if (L.P && r < dA && cc == r) as_global(L.P)[(size_t)r * dA - (size_t)r * (r - 1) / 2] = val;
  }
  __syncthreads();
#pragma unroll
  for (int u = 0; u < PER; ++u) {
    const int lr = lr0 + 4 * u;
    const int r = J.bj * LAG_TILE + lr, c = J.bi * LAG_TILE + lc;   // element (r, c) of the mirrored tile = tile[lc][lr]
    if (c < dA && r < c) {
      A[(uint32_t)r * (uint32_t)dA + (uint32_t)c] = tile[lc][lr];
      if (L.P) as_global(L.P)[(size_t)r * dA - (size_t)r * (r - 1) / 2 + (size_t)(c - r)] = tile[lc][lr];   // row r of the upper triangle
    }
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

void launch_tile_gemm_dl(const TileDesc* descs, const TileJob* jobs, int njobs, hipStream_t s) {
  if (njobs <= 0) return;
  hipLaunchKernelGGL(tile_gemm_dl_kernel, dim3(njobs), dim3(NT), 0, s, descs, jobs, njobs);
}

void launch_tile_gemm_yield(const TileDesc* descs, const TileJob* jobs, int njobs, int pad_bytes, const int* cu_flags, hipStream_t s) {
  if (njobs <= 0) return;
  hipLaunchKernelGGL(tile_gemm_yield_kernel, dim3(njobs), dim3(NT), pad_bytes, s, descs, jobs, njobs, cu_flags);
}

void launch_tile_gemm_pad(const TileDesc* descs, const TileJob* jobs, int njobs, int pad_bytes, hipStream_t s) {
  if (njobs <= 0) return;
  hipLaunchKernelGGL(tile_gemm_kernel, dim3(njobs), dim3(NT), pad_bytes, s, descs, jobs, njobs, 0);
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
