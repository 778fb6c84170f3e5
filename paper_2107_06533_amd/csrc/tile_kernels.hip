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
template <int KCD>
__global__ __launch_bounds__(NT, 2) void tile_gemm_yield_kernel(const TileDesc* __restrict__ descs, const TileJob* __restrict__ jobs,
                                                                int njobs, const int* __restrict__ cu_flags) {
  __shared__ __attribute__((aligned(16))) float smem[4 * KCD * BM];
  const int g = blockIdx.x;
  if (g >= njobs) return;
  const TileJob J = jobs[g];
  run_tile_dl<true, true, KCD>(descs[J.desc], J, smem, cu_flags);
}

// The same products cut into 32 x 32 blocks, one a wave, fed from memory without LDS (TileJob::quarter), for
// the launches on the sweep chain of the inverse: see run_tile_quarter.
__global__ __launch_bounds__(NT, 2) void tile_gemm_quarter_kernel(const TileDesc* __restrict__ descs, const TileJob* __restrict__ jobs,
                                                                   int njobs, int* cu_flags) {
  const int g = blockIdx.x;
  if (g >= njobs) return;
  const TileJob J = jobs[g];
  cu_enter(cu_flags);   // the products that share its compute unit give way (cu_flags may be null)
  run_tile_quarter(descs[J.desc], J);
  __syncthreads();      // every wave is done before the workgroup counts itself out
  cu_leave(cu_flags);
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

// Assembly of a lag-product activation factor (see LagAsm), lower triangle: a thread owns one pair of
// channels (c, c2), c2 <= c, i.e. the 9 x 9 block of A at rows 9c.., columns 9c2..  Its 81 entries
// are sums of at most four of 49 entries of the small lag matrices, picked by compile-time tap indices:
//   the lag product   dy > 0: G1[c][(c2, dy, dx)]      dy = 0, dx >= 0: G2[c][(c2, dx)]
//                     dy < 0: G1[c2][(c, -dy, -dx)]    dy = 0, dx < 0:  G2[c2][(c, -dx)]     (backward lags: transposes)
//   minus the border row that tap row i drops (bottom row for i = 0, top row for i = 2), which pairs
//   with itself only (dy = 0), minus the border column that tap column j drops (dx = 0 only), plus
//   their common corner pixel (dy = dx = 0).
// The pseudo-channel c = C is the bias row: its entries against (c2, t2) are the sums of a over the
// pixels tap t2 keeps, its last entry the number of rows.  Consecutive lanes hold consecutive c2, so a
// wave reads and writes runs of 9 x 32 consecutive floats of a row of A.  The upper triangle is
// filled in by lag_mirror_kernel.  All offsets fit 32 bits.
constexpr int LAG_PC = 32, LAG_PR = NT / LAG_PC;   // pair tile: 8 row channels x 32 column channels
__global__ __launch_bounds__(NT) void lag_pairs_kernel(const LagAsm* __restrict__ lags,
                                                       const LagJob* __restrict__ jobs, int njobs) {
  const int g = blockIdx.x;
  if (g >= njobs) return;
  const LagJob J = jobs[g];
  const LagAsm L = lags[J.lag];
  const int C = L.C;
  const uint32_t uC = (uint32_t)C, dA = (uint32_t)L.dA;
  const uint32_t ld1 = 10u * uC, ld2 = 3u * uC + L.bias, ld3 = ld2, ldc = uC + L.bias;   // strips: [C][3C + bias] as G2
  const int c2 = J.bj * LAG_PC + (int)(threadIdx.x & (LAG_PC - 1));
  const int c = J.bi * LAG_PR + (int)(threadIdx.x / LAG_PC);
  const int cmax = L.bias ? C : C - 1;
  if (c > cmax || c2 > c) return;
  gf_ptr A = as_global(L.A);
  gcf_ptr G1 = as_global(L.G[LAG_G1]);
  gcf_ptr G2 = as_global(L.G[LAG_G2]);
  gcf_ptr TOP = as_global(L.G[LAG_TOP]), BOT = as_global(L.G[LAG_BOT]);
  gcf_ptr LEFT = as_global(L.G[LAG_LEFT]), RIGHT = as_global(L.G[LAG_RIGHT]);
  gcf_ptr TL = as_global(L.G[LAG_TL]), TR = as_global(L.G[LAG_TR]), BL = as_global(L.G[LAG_BL]), BR = as_global(L.G[LAG_BR]);
  const float alpha = L.alpha, beta = L.beta;
  const uint32_t uc = (uint32_t)c, uc2 = (uint32_t)c2;

  if (c == C) {   // bias row
    const uint32_t row = 9u * uC * dA;
    if (c2 == C) {
      const float old = beta != 0.f ? A[row + 9u * uC] : 0.f;
      A[row + 9u * uC] = alpha * L.rows + beta * old;
      return;
    }
    const float whole = G2[uc2 * ld2 + 3u * uC];
    const float bot = BOT[uc2 * ld3 + 3u * uC], top = TOP[uc2 * ld3 + 3u * uC];
    const float rgt = RIGHT[uc2 * ld3 + 3u * uC], lft = LEFT[uc2 * ld3 + 3u * uC];
    const float br = BR[uc2 * ldc + uC], bl = BL[uc2 * ldc + uC], tr = TR[uc2 * ldc + uC], tl = TL[uc2 * ldc + uC];
    float old[9];
#pragma unroll
    for (int t2 = 0; t2 < 9; ++t2) old[t2] = beta != 0.f ? A[row + 9u * uc2 + t2] : 0.f;
#pragma unroll
    for (int t2 = 0; t2 < 9; ++t2) {
      const int i2 = t2 / 3, j2 = t2 % 3;
      float v = whole;
      if (i2 != 1) v -= i2 == 0 ? bot : top;
      if (j2 != 1) v -= j2 == 0 ? rgt : lft;
      if (i2 != 1 && j2 != 1) v += i2 == 0 ? (j2 == 0 ? br : bl) : (j2 == 0 ? tr : tl);
      A[row + 9u * uc2 + t2] = alpha * v + beta * old[t2];
    }
    return;
  }

  float g1a[10], g1b[10], g2a[3], g2b[3], srow[2][5], scol[2][5], cor[4];
#pragma unroll
  for (int q = 0; q < 10; ++q) {
    g1a[q] = G1[uc * ld1 + uc2 * 10u + q];
    g1b[q] = G1[uc2 * ld1 + uc * 10u + q];
  }
#pragma unroll
  for (int q = 0; q < 3; ++q) {
    g2a[q] = G2[uc * ld2 + uc2 * 3u + q];
    g2b[q] = G2[uc2 * ld2 + uc * 3u + q];
  }
  // strips hold the forward lags 0, 1, 2 along themselves; a backward lag is the transposed entry
  // of its opposite: index 2 + lag in the arrays below
#pragma unroll
  for (int q = 0; q < 3; ++q) {
    srow[0][2 + q] = BOT[uc * ld3 + uc2 * 3u + q];     // tap row i = 0 drops the bottom row
    srow[1][2 + q] = TOP[uc * ld3 + uc2 * 3u + q];     // i = 2: the top row
    scol[0][2 + q] = RIGHT[uc * ld3 + uc2 * 3u + q];   // tap column j = 0 drops the right column
    scol[1][2 + q] = LEFT[uc * ld3 + uc2 * 3u + q];    // j = 2: the left column
  }
#pragma unroll
  for (int q = 1; q < 3; ++q) {
    srow[0][2 - q] = BOT[uc2 * ld3 + uc * 3u + q];
    srow[1][2 - q] = TOP[uc2 * ld3 + uc * 3u + q];
    scol[0][2 - q] = RIGHT[uc2 * ld3 + uc * 3u + q];
    scol[1][2 - q] = LEFT[uc2 * ld3 + uc * 3u + q];
  }
  cor[0] = BR[uc * ldc + uc2]; cor[1] = BL[uc * ldc + uc2];   // i = 0: j = 0, j = 2
  cor[2] = TR[uc * ldc + uc2]; cor[3] = TL[uc * ldc + uc2];   // i = 2: j = 0, j = 2
  const bool dpair = c == c2;   // diagonal block: entries with t2 <= t only
#pragma unroll
  for (int t = 0; t < 9; ++t) {
    const int i = t / 3, j = t % 3;
    const uint32_t row = (9u * uc + t) * dA + 9u * uc2;
    float old[9];
#pragma unroll
    for (int t2 = 0; t2 < 9; ++t2) old[t2] = (beta != 0.f && (!dpair || t2 <= t)) ? A[row + t2] : 0.f;
#pragma unroll
    for (int t2 = 0; t2 < 9; ++t2) {
      const int i2 = t2 / 3, j2 = t2 % 3, dy = i2 - i, dx = j2 - j;
      float v;
      if (dy > 0) v = g1a[(dy - 1) * 5 + dx + 2];
      else if (dy == 0 && dx >= 0) v = g2a[dx];
      else if (dy < 0) v = g1b[(-dy - 1) * 5 - dx + 2];
      else v = g2b[-dx];
      if (i != 1 && dy == 0) v -= srow[i == 0 ? 0 : 1][dx + 2];
      if (j != 1 && dx == 0) v -= scol[j == 0 ? 0 : 1][dy + 2];
      if (i != 1 && j != 1 && dy == 0 && dx == 0) v += cor[(i == 0 ? 0 : 2) + (j == 0 ? 0 : 1)];
      if (!dpair || t2 <= t) A[row + t2] = alpha * v + beta * old[t2];
    }
  }
}

// Upper triangle (and packed copy) of a lag-product activation factor from its finished lower
// triangle: one 64 x 64 tile per workgroup, transposed through LDS so that both sides are moved row
// by row; both triangles hold the same bits.
constexpr int LAG_TILE = 64;
__global__ __launch_bounds__(NT) void lag_mirror_kernel(const LagAsm* __restrict__ lags,
                                                        const LagJob* __restrict__ jobs, int njobs) {
  __shared__ float tile[LAG_TILE][LAG_TILE + 1];
  const int g = blockIdx.x;
  if (g >= njobs) return;
  const LagJob J = jobs[g];
  const LagAsm L = lags[J.lag];
  const int dA = L.dA;
  constexpr int PER = LAG_TILE * LAG_TILE / NT;
  gf_ptr A = as_global(L.A);
  const int lc = threadIdx.x & (LAG_TILE - 1), lr0 = threadIdx.x >> 6;
  const int cc = J.bj * LAG_TILE + lc;
#pragma unroll
  for (int u = 0; u < PER; ++u) {
    const int lr = lr0 + 4 * u, r = J.bi * LAG_TILE + lr;
    float val = 0.f;
    if (r < dA && cc <= r) val = A[(uint32_t)r * (uint32_t)dA + (uint32_t)cc];
    tile[lr][lc] = val;
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

int deep_lds_extra() { return 4 * (DL_DEEP_LDS_FLOATS - DL_LDS_FLOATS); }
void launch_tile_gemm_yield(const TileDesc* descs, const TileJob* jobs, int njobs, int pad_bytes, const int* cu_flags, bool deep, hipStream_t s) {
  if (njobs <= 0) return;
  if (deep) hipLaunchKernelGGL(tile_gemm_yield_kernel<DL_KC_DEEP>, dim3(njobs), dim3(NT), pad_bytes, s, descs, jobs, njobs, cu_flags);
  else hipLaunchKernelGGL(tile_gemm_yield_kernel<DL_KC>, dim3(njobs), dim3(NT), pad_bytes, s, descs, jobs, njobs, cu_flags);
}

void launch_tile_gemm_quarter(const TileDesc* descs, const TileJob* jobs, int njobs, int* cu_flags, hipStream_t s) {
  if (njobs <= 0) return;
  hipLaunchKernelGGL(tile_gemm_quarter_kernel, dim3(njobs), dim3(NT), 0, s, descs, jobs, njobs, cu_flags);
}

void launch_tile_gemm_pad(const TileDesc* descs, const TileJob* jobs, int njobs, int pad_bytes, hipStream_t s) {
  if (njobs <= 0) return;
  hipLaunchKernelGGL(tile_gemm_kernel, dim3(njobs), dim3(NT), pad_bytes, s, descs, jobs, njobs, 0);
}

void launch_lag_assemble(const LagAsm* lags, const LagJob* pair_jobs, int npair, const LagJob* mirror_jobs, int nmirror, hipStream_t s) {
  if (npair > 0) hipLaunchKernelGGL(lag_pairs_kernel, dim3(npair), dim3(NT), 0, s, lags, pair_jobs, npair);
  if (nmirror > 0) hipLaunchKernelGGL(lag_mirror_kernel, dim3(nmirror), dim3(NT), 0, s, lags, mirror_jobs, nmirror);
}
int lag_pair_rows() { return LAG_PR; }
int lag_pair_cols() { return LAG_PC; }

void launch_tile_reduce(const TileDesc* descs, const ReduceJob* jobs, int njobs, hipStream_t s) {
  if (njobs <= 0) return;
  hipLaunchKernelGGL(tile_reduce_kernel, dim3(njobs * 4), dim3(NT), 0, s, descs, jobs, njobs);
}

}  // namespace kfac
