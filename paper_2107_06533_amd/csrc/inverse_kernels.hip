// Batched damped SPD inverse by a blocked symmetric sweep (block Gauss-Jordan on the lower
// triangle).  For a symmetric matrix M partitioned in NB-wide blocks, sweeping pivot block k
//     M_kk <- -P^-1,   M_ik <- M_ik P^-1,   M_ij <- M_ij - M_ik P^-1 M_kj   (i, j != k),  P = M_kk
// for every k leaves -M^-1.  Every step is one pivot-block inverse (in registers, one workgroup),
// one panel product and one rank-NB update of the whole lower triangle, so all steps expose
// the same parallelism; total work is d^3 flops, the same as Cholesky + triangular inverse +
// triangular product.  Pivot blocks are Schur complements of an SPD matrix, hence SPD: a
// non-positive scalar pivot is exactly a non-positive leading minor.
#include "tile_core.h"
#include "launch.h"

namespace kfac {

struct MatJob {
  int32_t mat, bi, bj, aux;
};

// ---- X(lower tiles) = F + gamma I; info = 0 ---------------------------------------------------
__global__ __launch_bounds__(NT) void gj_init_kernel(const InvMat* __restrict__ mats,
                                                     const MatJob* __restrict__ jobs, int njobs, float gamma) {
  const int g = blockIdx.x;
  if (g >= njobs) return;
  const MatJob J = jobs[g];
  const InvMat Mx = mats[J.mat];
  const int d = Mx.d;
  if (J.bi == 0 && J.bj == 0 && threadIdx.x == 0 && Mx.info) *Mx.info = 0;
  for (int e = threadIdx.x; e < BM * BN; e += NT) {
    const int i = J.bi * BM + (e >> 7), j = J.bj * BN + (e & 127);
    if (i >= d || j >= d) continue;
    const int hi = i > j ? i : j, lo = i > j ? j : i;   // diagonal tiles are kept full
    float v = Mx.F[(size_t)hi * d + lo];
    if (i == j) v += gamma;
    Mx.X[(size_t)i * d + j] = v;
  }
}

// ---- pivot block: in-register symmetric sweep of an n x n (n <= 128) SPD block ------------------
// 256 threads as 16 x 16; thread (ty, tx) holds elements (ty + 16a, tx + 16b) for a >= b only: the
// sweep keeps the lower triangle and mirrors it at the end, so the result is exactly symmetric.
// Step k broadcasts column k of the symmetric matrix through LDS (rows >= k from column k, rows < k
// from row k), then every element does one fused multiply-add  m_ij -= (c_i / p) * c_j.
// small = 1: block = F + gamma I (whole matrix, d <= NB), result written to X as +inverse.
// small = 0: block = diagonal block `step` of X; writes Q = +inverse (zero padded to NB x NB)
//            and the swept block (-inverse) back into X.
__global__ __launch_bounds__(NT) void gj_pivot_kernel(const InvMat* __restrict__ mats, int mat0, int step,
                                                      float gamma, int small) {
  __shared__ float col[2][NB];
  __shared__ float tileT[NB][NB + 1];   // mirror staging
  __shared__ int bad;
  const InvMat Mx = mats[mat0 + blockIdx.x];
  const int t = threadIdx.x, ty = t >> 4, tx = t & 15;
  const int d = Mx.d;
  const int k0 = small ? 0 : step * NB;
  const int n = small ? d : (d - k0 < NB ? d - k0 : NB);
  gcf_ptr src = as_global(small ? Mx.F : Mx.X);
  const float damp = small ? gamma : 0.f;

  float m[8][8];
#pragma unroll
  for (int a = 0; a < 8; ++a)
#pragma unroll
    for (int b = 0; b < 8; ++b) {
      if (b > a) continue;
      const int i = ty + 16 * a, j = tx + 16 * b;
      float v = (i == j) ? 1.f : 0.f;
      if (i < n && j < n && i >= j) {
        v = src[(size_t)(k0 + i) * d + k0 + j];
        if (i == j) v += damp;
      }
      m[a][b] = v;
    }
  if (t == 0) bad = 0;
  __syncthreads();

#pragma unroll
  for (int kb = 0; kb < 8; ++kb) {
    if (kb * 16 < n) {
      const int kk_end = (n - kb * 16 < 16) ? n - kb * 16 : 16;
      for (int kk = 0; kk < kk_end; ++kk) {
        const int k = kb * 16 + kk;
        float* cb = col[k & 1];
        if (tx == kk) {            // rows i >= k of column k
#pragma unroll
          for (int a = kb; a < 8; ++a)
            if (a > kb || ty >= kk) cb[ty + 16 * a] = m[a][kb];
        }
        if (ty == kk) {            // rows i < k come from row k
#pragma unroll
          for (int b = 0; b <= kb; ++b)
            if (b < kb || tx < kk) cb[tx + 16 * b] = m[kb][b];
        }
        __syncthreads();
        const float p = cb[k];
        if (!(p > 0.f) && t == 0 && bad == 0) bad = k + 1;
        const float ip = 1.f / p;
        float wi[8], cj[8];
#pragma unroll
        for (int a = 0; a < 8; ++a) wi[a] = cb[ty + 16 * a] * ip;
#pragma unroll
        for (int b = 0; b < 8; ++b) cj[b] = cb[tx + 16 * b];
#pragma unroll
        for (int a = 0; a < 8; ++a)
#pragma unroll
          for (int b = 0; b <= a; ++b) m[a][b] = fmaf(-wi[a], cj[b], m[a][b]);
        if (tx == kk) {            // column k: m_ik = c_i / p
#pragma unroll
          for (int a = kb; a < 8; ++a) m[a][kb] = wi[a];
        }
        if (ty == kk) {            // row k: m_kj = c_j / p
#pragma unroll
          for (int b = 0; b <= kb; ++b) m[kb][b] = cj[b] * ip;
        }
        if (tx == kk && ty == kk) m[kb][kb] = -ip;
      }
    }
  }
  if (t == 0 && Mx.info) {
    if (small) *Mx.info = bad;                                // whole matrix: sole writer
    else if (bad && *Mx.info == 0) *Mx.info = k0 + bad;       // first failing sweep wins (zeroed by the init kernel)
  }

  // mirror the lower triangle through LDS, then write rows contiguously
#pragma unroll
  for (int a = 0; a < 8; ++a)
#pragma unroll
    for (int b = 0; b <= a; ++b) {
      const int i = ty + 16 * a, j = tx + 16 * b;
      if (i >= j) {
        tileT[i][j] = m[a][b];
        tileT[j][i] = m[a][b];
      }
    }
  __syncthreads();
  gf_ptr X = as_global(Mx.X);
  gf_ptr Q = as_global(Mx.Q);
  for (int e = t; e < NB * NB; e += NT) {
    const int i = e >> 7, j = e & (NB - 1);
    const bool in = i < n && j < n;
    const float v = tileT[i][j];
    if (small) {
      if (in) X[(size_t)i * d + j] = -v;
    } else {
      Q[i * NB + j] = in ? -v : 0.f;
      if (in) X[(size_t)(k0 + i) * d + k0 + j] = v;
    }
  }
}

// ---- panel: Zt = old block column `step` (as [NB][ldp], k-major), Wt = Q * Zt, X panel <- W -----
// One job per 128-row tile `it` of the block column (it != step).  Tiles above the pivot live in
// block row `step` of the lower triangle (read along rows), tiles below in block column `step`.
__global__ __launch_bounds__(NT, 2) void gj_panel_kernel(const InvMat* __restrict__ mats,
                                                         const MatJob* __restrict__ jobs, int njobs, int step) {
  __shared__ float Qs[PANEL];
  __shared__ float Zs[PANEL];
  const int g = blockIdx.x;
  if (g >= njobs) return;
  const MatJob J = jobs[g];
  const InvMat Mx = mats[J.mat];
  const int it = J.bi, slot = J.aux;   // slot: which 128 rows of the aggregated panel buffers this sweep fills
  const int t = threadIdx.x, lane = t & 63, w = t >> 6, wm = w >> 1, wn = w & 1;
  const int d = Mx.d, ldp = Mx.ldp;
  const int k0 = step * NB, i0 = it * BM;
  const int kb = d - k0 < NB ? d - k0 : NB;
  const bool above = it < step;
  const int ml = t & 127, kp = t >> 7;   // row-contiguous mapping
  const int kl = t & (KC - 1), mg = t / KC;    // column-contiguous mapping

  unsigned mask = 0;
#pragma unroll
  for (int a = 0; a < 2; ++a)
#pragma unroll
    for (int b = 0; b < 2; ++b)
      if (wm * 64 + a * 32 < kb && i0 + wn * 64 + b * 32 < d) mask |= 1u << (a * 2 + b);

  const unsigned pat = cover_pattern(mask);
  mask = pat;   // blocks the pattern adds hold exact zeros (zero-padded operands)
  // Buffer resources: Q is a dense 128 x 128 block; X is cut at the pivot block's last row when the
  // panel tile is read along rows, so rows of a ragged last pivot block read 0.
  const rsrc_t rs_q = make_rsrc(Mx.Q, NB * NB * 4u);
  const rsrc_t rs_x = make_rsrc(Mx.X, (uint32_t)(above ? k0 + kb : d) * (uint32_t)d * 4u);
  const uint32_t d4 = (uint32_t)d * 4u;
  float rq[NU], rz[NU];
  auto issue = [&](int kk0) {
#pragma unroll
    for (int u = 0; u < NU; ++u) rq[u] = buf_load(rs_q, (uint32_t)((kk0 + kp + 2 * u) * NB + ml) * 4u);
    if (above) {
      const uint32_t base = (uint32_t)(k0 + kk0 + kp) * d4 + (uint32_t)(i0 + ml) * 4u;
#pragma unroll
      for (int u = 0; u < NU; ++u) rz[u] = buf_load(rs_x, base + (uint32_t)(2 * u) * d4);
    } else {
      const int kk = kk0 + kl;
      const uint32_t base = kk < kb ? (uint32_t)(k0 + kk) * 4u : OOB_OFFSET;   // rows i >= d fall off the end
#pragma unroll
      for (int u = 0; u < NU; ++u) rz[u] = buf_load(rs_x, base + (uint32_t)(i0 + mg + MG * u) * d4);
    }
  };

  Acc4 acc;
  acc_zero(acc);
  gf_ptr Zt = as_global(Mx.Zt);
  issue(0);
  for (int kk0 = 0; kk0 < NB; kk0 += KC) {
    __syncthreads();   // previous chunk fully consumed
#pragma unroll
    for (int u = 0; u < NU; ++u) Qs[lds_idx(ml, kp + 2 * u)] = rq[u];
    if (above) {
#pragma unroll
      for (int u = 0; u < NU; ++u) Zs[lds_idx(ml, kp + 2 * u)] = rz[u];
    } else {
#pragma unroll
      for (int u = 0; u < NU; ++u) Zs[lds_idx(mg + MG * u, kl)] = rz[u];
    }
    if (kk0 + KC < NB) issue(kk0 + KC);   // next chunk's loads fly during this chunk's MFMAs
    __syncthreads();
#pragma unroll
    for (int u = 0; u < NU; ++u) Zt[(size_t)(slot * NB + kk0 + kp + 2 * u) * ldp + i0 + ml] = Zs[lds_idx(ml, kp + 2 * u)];
    switch (pat) {
      case PAT_FULL: mma_ktile<PAT_FULL>(Qs, Zs, acc, wm, wn, lane); break;
      case PAT_ROW1: mma_ktile<PAT_ROW1>(Qs, Zs, acc, wm, wn, lane); break;
      case PAT_COL1: mma_ktile<PAT_COL1>(Qs, Zs, acc, wm, wn, lane); break;
      case PAT_ONE: mma_ktile<PAT_ONE>(Qs, Zs, acc, wm, wn, lane); break;
      default: break;
    }
  }

  // acc(m, i) = W[i][m]: new panel entry for matrix row/col i0+i and pivot column k0+m
  gf_ptr Wt = as_global(Mx.Wt);
  const rsrc_t rs_o = make_rsrc(Mx.X, (uint32_t)d * d4);
#pragma unroll
  for (int qd = 0; qd < 4; ++qd) {
    const int mb0 = wm * 64 + (qd >> 1) * 32, ib0 = wn * 64 + (qd & 1) * 32;
    const int i = ib0 + mfma_col(lane);
#pragma unroll
    for (int v = 0; v < 16; ++v) {
      const int mm = mb0 + mfma_row(v, lane);
      const float val = (mask & (1u << qd)) ? acc.c[qd][v] : 0.f;
      Wt[(size_t)(slot * NB + mm) * ldp + i0 + i] = val;
      const bool in = mm < kb && i0 + i < d;
      const uint32_t off = above ? (uint32_t)(k0 + mm) * d4 + (uint32_t)(i0 + i) * 4u
                                 : (uint32_t)(i0 + i) * d4 + (uint32_t)(k0 + mm) * 4u;
      buf_store(rs_o, in ? off : OOB_OFFSET, val);
    }
  }
}

// ---- finish: X = -(swept lower triangle), mirrored to a full symmetric matrix -------------------
__global__ __launch_bounds__(NT) void gj_finish_kernel(const InvMat* __restrict__ mats,
                                                       const MatJob* __restrict__ jobs, int njobs) {
  __shared__ float tile[32][33];
  const int g = blockIdx.x;
  if (g >= njobs) return;
  const MatJob J = jobs[g];
  const InvMat Mx = mats[J.mat];
  const int d = Mx.d;
  const int tx = threadIdx.x & 31, ty = threadIdx.x >> 5;   // 32 x 8
  const int i0 = J.bi * 32, j0 = J.bj * 32;
#pragma unroll
  for (int r = 0; r < 4; ++r) {
    const int li = ty + 8 * r;
    const int i = i0 + li, j = j0 + tx;
    float v = 0.f;
    if (i < d && j < d && i >= j) {
      v = -Mx.X[(size_t)i * d + j];
      Mx.X[(size_t)i * d + j] = v;
    }
    tile[li][tx] = v;
  }
  __syncthreads();
#pragma unroll
  for (int r = 0; r < 4; ++r) {
    const int lj = ty + 8 * r;             // row of the mirrored tile = column index of the source
    const int j = j0 + lj, i = i0 + tx;    // writes X[j][i] = X[i][j], i > j
    if (i < d && j < d && i > j) Mx.X[(size_t)j * d + i] = tile[tx][lj];
  }
}

void launch_gj_init(const InvMat* mats, const void* jobs, int njobs, float gamma, hipStream_t s) {
  if (njobs <= 0) return;
  hipLaunchKernelGGL(gj_init_kernel, dim3(njobs), dim3(NT), 0, s, mats, (const MatJob*)jobs, njobs, gamma);
}
void launch_gj_pivot(const InvMat* mats, int mat0, int nmats, int step, float gamma, int small, hipStream_t s) {
  if (nmats <= 0) return;
  hipLaunchKernelGGL(gj_pivot_kernel, dim3(nmats), dim3(NT), 0, s, mats, mat0, step, gamma, small);
}
void launch_gj_panel(const InvMat* mats, const void* jobs, int njobs, int step, hipStream_t s) {
  if (njobs <= 0) return;
  hipLaunchKernelGGL(gj_panel_kernel, dim3(njobs), dim3(NT), 0, s, mats, (const MatJob*)jobs, njobs, step);
}
void launch_gj_finish(const InvMat* mats, const void* jobs, int njobs, hipStream_t s) {
  if (njobs <= 0) return;
  hipLaunchKernelGGL(gj_finish_kernel, dim3(njobs), dim3(NT), 0, s, mats, (const MatJob*)jobs, njobs);
}

}  // namespace kfac
