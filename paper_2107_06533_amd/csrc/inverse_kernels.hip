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

// ---- pivot block: symmetric sweep of an n x n (n <= 128) SPD block in one workgroup ---------------
// The block lives in LDS as 4 x 4 sub-blocks of 32 x 32 and is swept sub-block by sub-block:
//   (A) every wave inverts the 32 x 32 diagonal sub-block D in registers (redundantly, so no
//       exchange between waves is needed) by the scalar sweep, 16 fused multiply-adds per lane and
//       step (see sweep32_step);
//   (B) wave w != kb owns sub-block row w:  W_w = Z_w D^-1  (Z_w = old sub-block (w, kb)), then
//       S_wj -= W_w Z_j^T for j != kb, all on the matrix cores (v_mfma_f32_32x32x2_f32: lane
//       (i, h) = i + 32 h supplies element [i][2q + h] of an operand in step q).  Sub-block (kb, w),
//       which no wave reads during the step, serves the wave as scratch for the two layout changes
//       (D^-1 and W_w into operand layout) and ends as W_w^T; after a barrier the wave stores W_w
//       into sub-block (w, kb), and wave kb stores -D^-1.
// Sub-blocks past n are identity and are skipped.  The lower triangle is mirrored on the way out,
// so the result is exactly symmetric.
// small = 1: block = F + gamma I (whole matrix, d <= NB), result written to X as +inverse.
// small = 0: block = diagonal block `step` of X (lower triangle valid); writes Q = +inverse (zero
//            padded to NB x NB) and the swept block (-inverse) back into X.
constexpr int SB = 32;          // sub-block order
constexpr int SP = NB + 1;      // LDS row pitch of the block (odd: conflict-free rows and columns)

// In-register sweep of a 32 x 32 SPD sub-block.  Lane 16 g + m holds rows m and m + 16 of the
// column group 8g .. 8g+7:  r[8a + b] = D[m + 16a][8g + b].  Step k needs row k (for the lane's
// eight columns: a DPP broadcast inside the lane's 16-lane row) and column k (for the lane's two rows: two cross-lane reads from column group k / 8).
// Returns +D^-1 in the same layout; `bad` receives the 1-based index of the first non-positive
// pivot (0 if none).
template <int KM>
__device__ __forceinline__ float row_bcast(float x) {   // lane KM of every 16-lane row, to the whole row
  return __builtin_bit_cast(float, __builtin_amdgcn_mov_dpp(__builtin_bit_cast(int, x), 0x150 + KM, 0xF, 0xF, true));
}

// Step K gets column K (ci0, ci1: the lane's two rows) and the pivot p as arguments; it fetches
// those of step K + 1 itself as soon as the column of step K + 1 has been updated, ahead of the
// other seven columns, so that the cross-lane reads are in flight during the rest of the update.
template <int K>
__device__ __forceinline__ void sweep32_step(float (&r)[16], int m, int g, int& bad, float ci0, float ci1, float p) {
  constexpr int ka = K >> 4, km = K & 15, kg = K >> 3, kb = K & 7;
  constexpr int K1 = (K + 1) & 31, ka1 = K1 >> 4, km1 = K1 & 15, kg1 = K1 >> 3, kb1 = K1 & 7;
  if (!(p > 0.f) && bad == 0) bad = K + 1;
  float ip = __builtin_amdgcn_rcpf(p);
  ip = fmaf(fmaf(-p, ip, 1.f), ip, ip);   // one Newton step on the hardware reciprocal
  const float w0 = ci0 * ip, w1 = ci1 * ip;
  // the lane that holds row k: r - (1 - 1/p) r = r / p, the swept pivot row
  const bool prow = m == km;
  const float nwu0 = (prow && ka == 0) ? ip - 1.f : -w0;
  const float nwu1 = (prow && ka == 1) ? ip - 1.f : -w1;
  auto upd = [&](int b) {
    const float c = row_bcast<km>(r[8 * ka + b]);   // row k, this lane's column b (read before it is updated)
    r[b] = fmaf(c, nwu0, r[b]);
    r[8 + b] = fmaf(c, nwu1, r[8 + b]);
  };
  float nci0 = 0.f, nci1 = 0.f, np = 1.f;
  if constexpr (K + 1 < 32) {
    upd(kb1);
    const int src = (16 * kg1 + m) << 2;
    nci0 = __builtin_bit_cast(float, __builtin_amdgcn_ds_bpermute(src, __builtin_bit_cast(int, r[kb1])));
    nci1 = __builtin_bit_cast(float, __builtin_amdgcn_ds_bpermute(src, __builtin_bit_cast(int, r[8 + kb1])));
    np = __builtin_bit_cast(float, __builtin_amdgcn_readlane(__builtin_bit_cast(int, r[8 * ka1 + kb1]), 16 * kg1 + km1));
    __builtin_amdgcn_sched_barrier(0);
  }
#pragma unroll
  for (int b = 0; b < 8; ++b)
    if (K + 1 >= 32 || b != kb1) upd(b);
  if (g == kg) {   // pivot column
    r[kb] = (prow && ka == 0) ? -ip : w0;
    r[8 + kb] = (prow && ka == 1) ? -ip : w1;
  }
  if constexpr (K + 1 < 32) sweep32_step<K + 1>(r, m, g, bad, nci0, nci1, np);
}

__device__ __forceinline__ void sweep32(float (&r)[16], int lane, int& bad) {
  const int m = lane & 15;
  const float ci0 = __builtin_bit_cast(float, __builtin_amdgcn_ds_bpermute(m << 2, __builtin_bit_cast(int, r[0])));
  const float ci1 = __builtin_bit_cast(float, __builtin_amdgcn_ds_bpermute(m << 2, __builtin_bit_cast(int, r[8])));
  const float p = __builtin_bit_cast(float, __builtin_amdgcn_readlane(__builtin_bit_cast(int, r[0]), 0));
  sweep32_step<0>(r, m, lane >> 4, bad, ci0, ci1, p);
#pragma unroll
  for (int t = 0; t < 16; ++t) r[t] = -r[t];
}

constexpr int PIVOT_LDS_FLOATS = NB * SP;

#ifdef KFAC_TRACE
// debugging aid: per-workgroup phase time stamps (100 MHz) appended behind the compute-unit words
__device__ __forceinline__ void trace_rec(int* flags, int kind, int step, const long long (&t)[5]) {
  if (!flags || threadIdx.x != 0) return;
  int* cnt = flags + CU_SLOTS;
  const int r = __hip_atomic_fetch_add(cnt, 1, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
  if (r >= 60000) return;
  long long* rec = reinterpret_cast<long long*>(flags + CU_SLOTS + 2) + (size_t)r * 8;
  rec[0] = kind; rec[1] = step; rec[2] = cu_slot();
  for (int k = 0; k < 5; ++k) rec[3 + k] = t[k];
}
#define TRACE_T(k) tr[k] = wall_clock64()
#else
#define TRACE_T(k)
#endif

// block -= Wt^T Zt on the ten 32 x 32 sub-blocks of the block's lower triangle (mirrored into the
// upper one), Wt/Zt k-major with NB rows.  Wave WV takes the sub-blocks
//   0: (0,0) (1,0) (2,0)    1: (3,0) (3,1) (3,2)    2: (1,1) (2,1)    3: (2,2) (3,3)
// so that it needs at most four 32-column operand panels; all of them are requested before the
// first product (operands come straight from memory: lane (i, h) reads row 2q + h, column i), so
// the wave pays the memory latency once.
template <int WV>
__device__ __forceinline__ void own_update(float* __restrict__ S, gcf_ptr Wp, gcf_ptr Zp, uint32_t ldp, int lane) {
  constexpr int NA = WV == 0 ? 3 : WV == 1 ? 1 : 2;    // row panels (from Wt)
  constexpr int NZ = WV == 1 ? 3 : WV == 3 ? 2 : 1;    // column panels (from Zt)
  constexpr int A0 = WV == 0 ? 0 : WV == 1 ? 3 : WV == 2 ? 1 : 2;
  constexpr int Z0 = WV == 0 ? 0 : WV == 1 ? 0 : WV == 2 ? 1 : 2;
  constexpr int NJ = WV < 2 ? 3 : 2;
  const int li = lane & 31, lh = lane >> 5;
  float a[NA][64], b[NZ][64];
  const uint32_t base = (uint32_t)lh * ldp + (uint32_t)li;
#pragma unroll
  for (int x = 0; x < (NA > NZ ? NA : NZ); ++x)
#pragma unroll
    for (int q = 0; q < 64; ++q) {
      if (x < NA) a[x][q] = Wp[base + (uint32_t)(2 * q) * ldp + (uint32_t)((A0 + x) * SB)];
      if (x < NZ) b[x][q] = Zp[base + (uint32_t)(2 * q) * ldp + (uint32_t)((Z0 + x) * SB)];
    }
#pragma unroll
  for (int k = 0; k < NJ; ++k) {
    constexpr bool zfix = WV == 0 || WV == 2;          // one column panel, rows vary
    const int ia = WV == 1 ? 0 : k, iz = zfix ? 0 : k;
    const int bi = A0 + ia, bj = Z0 + iz;
    f32x16 acc;
#pragma unroll
    for (int v = 0; v < 16; ++v) acc[v] = 0.f;
#pragma unroll
    for (int q = 0; q < 64; ++q) acc = __builtin_amdgcn_mfma_f32_32x32x2f32(a[ia][q], b[iz][q], acc, 0, 0, 0);
#pragma unroll
    for (int v = 0; v < 16; ++v) {
      const int i = bi * SB + mfma_row(v, lane), j = bj * SB + mfma_col(lane);
      if (j > i) continue;               // diagonal sub-blocks: lower half, mirrored like the load
      const float x = S[i * SP + j] - acc[v];
      S[i * SP + j] = x;
      S[j * SP + i] = x;
    }
  }
}

// fuse = 1 (small = 0, step > 0): the block has not yet received the rank-NB update of the previous
// pivot block of the same matrix; its panels (Wt, Zt: k-major, NB rows) are applied here first,
// block -= Wt^T Zt restricted to the block's columns, so that the update launch can leave this
// block out and run beside this kernel instead of before it.
__device__ __forceinline__ void pivot_body(const InvMat& Mx, int step, float gamma, int small, int fuse, float* __restrict__ smem,
                                           int* trace = nullptr) {
#ifdef KFAC_TRACE
  long long tr[5] = {0, 0, 0, 0, 0};
#endif
  TRACE_T(0);
  float* S = smem;
  const int t = threadIdx.x, lane = t & 63, w = t >> 6;
  const int li = lane & 31, lh = lane >> 5;
  const int d = Mx.d, ld = small ? Mx.d : Mx.ld;
  const int k0 = small ? 0 : step * NB;
  const int n = small ? d : (d - k0 < NB ? d - k0 : NB);
  const int nsb = (n + SB - 1) / SB;
  const float damp = small ? gamma : 0.f;

  // lower triangle -> full symmetric block in LDS, identity past n (range-checked buffer loads;
  // skipped elements cost no memory traffic).  Thread t owns column j = t % 128 and every second row.
  const rsrc_t rs_src = make_rsrc(small ? Mx.F : Mx.X, small ? (uint32_t)d * (uint32_t)d * 4u : Mx.xelems * 4u);
  {
    const int j = t & (NB - 1), i0 = t >> 7;
    const uint32_t row2 = 2u * (uint32_t)ld * 4u;
    if (n == NB) {   // a whole block: all 64 loads of the thread in flight at once
      float v[64];
      uint32_t off = ((uint32_t)(k0 + i0) * (uint32_t)ld + (uint32_t)(k0 + j)) * 4u;
#pragma unroll
      for (int u = 0; u < 64; ++u) {
        v[u] = buf_load(rs_src, j <= i0 + 2 * u ? off : OOB_OFFSET);
        off += row2;
      }
      int la = i0 * SP + j, lb = j * SP + i0;
#pragma unroll
      for (int u = 0; u < 64; ++u) {
        const int i = i0 + 2 * u;
        if (j <= i) {
          const float x = i == j ? v[u] + damp : v[u];
          S[la] = x;
          S[lb] = x;
        }
        la += 2 * SP;
        lb += 2;
      }
    } else {
#pragma unroll
      for (int b = 0; b < 2; ++b) {
        float v[32];
#pragma unroll
        for (int u = 0; u < 32; ++u) {
          const int i = i0 + 2 * (b * 32 + u);
          v[u] = buf_load(rs_src, (i < n && j <= i) ? ((uint32_t)(k0 + i) * (uint32_t)ld + (uint32_t)(k0 + j)) * 4u : OOB_OFFSET);
        }
#pragma unroll
        for (int u = 0; u < 32; ++u) {
          const int i = i0 + 2 * (b * 32 + u);
          if (j > i) continue;
          float x = v[u];
          if (i == j) x = i < n ? x + damp : 1.f;
          S[i * SP + j] = x;
          S[j * SP + i] = x;
        }
      }
    }
  }
  __syncthreads();
  TRACE_T(1);

  if (fuse) {
    gcf_ptr Wp = as_global((const float*)Mx.Wt) + k0;
    gcf_ptr Zp = as_global((const float*)Mx.Zt) + k0;
    switch (w) {
      case 0: own_update<0>(S, Wp, Zp, (uint32_t)Mx.ldp, lane); break;
      case 1: own_update<1>(S, Wp, Zp, (uint32_t)Mx.ldp, lane); break;
      case 2: own_update<2>(S, Wp, Zp, (uint32_t)Mx.ldp, lane); break;
      default: own_update<3>(S, Wp, Zp, (uint32_t)Mx.ldp, lane); break;
    }
    __syncthreads();
  }

  TRACE_T(2);
  int bad = 0;
  for (int kb = 0; kb < nsb; ++kb) {
    // (A) inverse of the diagonal sub-block, in every wave (r: +D^-1 in the sweep's layout)
    const int m = lane & 15, g = lane >> 4;
    float r[16];
#pragma unroll
    for (int a = 0; a < 2; ++a)
#pragma unroll
      for (int b = 0; b < 8; ++b) r[8 * a + b] = S[(kb * SB + m + 16 * a) * SP + kb * SB + 8 * g + b];
    int bad_k = 0;
    sweep32(r, lane, bad_k);
    if (bad_k && bad == 0) bad = kb * SB + bad_k;

    // (B) panel and update of sub-block row w.  Sub-block (kb, w) is read by nobody during this
    // step and ends as W_w^T: the wave first uses it to turn D^-1 into the operand layout
    // dinv[q] = D^-1[li][2q + lh], then stores W_w^T there and reads -W_w back as an operand.
    f32x16 wacc;
#pragma unroll
    for (int v = 0; v < 16; ++v) wacc[v] = 0.f;
    const bool work = (w != kb) && (w < nsb);
    if (work) {
      float* st = S + (kb * SB) * SP + w * SB;
#pragma unroll
      for (int a = 0; a < 2; ++a)
#pragma unroll
        for (int b = 0; b < 8; ++b) st[(m + 16 * a) * SP + 8 * g + b] = r[8 * a + b];
      __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
      __builtin_amdgcn_wave_barrier();
      __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
      float dinv[16], z[16];
#pragma unroll
      for (int q = 0; q < 16; ++q) dinv[q] = st[li * SP + 2 * q + lh];
#pragma unroll
      for (int q = 0; q < 16; ++q) z[q] = S[(w * SB + li) * SP + kb * SB + 2 * q + lh];
#pragma unroll
      for (int q = 0; q < 16; ++q) wacc = __builtin_amdgcn_mfma_f32_32x32x2f32(z[q], dinv[q], wacc, 0, 0, 0);
      __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
      __builtin_amdgcn_wave_barrier();   // every lane has read dinv before the sub-block is rewritten
      __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
#pragma unroll
      for (int v = 0; v < 16; ++v) st[mfma_col(lane) * SP + mfma_row(v, lane)] = wacc[v];
      __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
      __builtin_amdgcn_wave_barrier();
      __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
      float wn[16];
#pragma unroll
      for (int q = 0; q < 16; ++q) wn[q] = -st[(2 * q + lh) * SP + li];
      for (int j = 0; j < nsb; ++j) {
        if (j == kb) continue;
        float zj[16];
#pragma unroll
        for (int q = 0; q < 16; ++q) zj[q] = S[(j * SB + li) * SP + kb * SB + 2 * q + lh];
        f32x16 acc;
#pragma unroll
        for (int v = 0; v < 16; ++v) acc[v] = S[(w * SB + mfma_row(v, lane)) * SP + j * SB + mfma_col(lane)];
#pragma unroll
        for (int q = 0; q < 16; ++q) acc = __builtin_amdgcn_mfma_f32_32x32x2f32(wn[q], zj[q], acc, 0, 0, 0);
#pragma unroll
        for (int v = 0; v < 16; ++v) S[(w * SB + mfma_row(v, lane)) * SP + j * SB + mfma_col(lane)] = acc[v];
      }
    }
    __syncthreads();   // every read of the old sub-block column kb (and of the diagonal sub-block) is done
    if (work) {
#pragma unroll
      for (int v = 0; v < 16; ++v) S[(w * SB + mfma_row(v, lane)) * SP + kb * SB + mfma_col(lane)] = wacc[v];
    } else if (w == kb) {
#pragma unroll
      for (int a = 0; a < 2; ++a)
#pragma unroll
        for (int b = 0; b < 8; ++b) S[(kb * SB + m + 16 * a) * SP + kb * SB + 8 * g + b] = -r[8 * a + b];
    }
    __syncthreads();
  }
  TRACE_T(3);
  if (t == 0 && Mx.info) {
    if (small) *Mx.info = bad;                                // whole matrix: sole writer
    else if (bad && *Mx.info == 0) *Mx.info = Mx.info_base + k0 + bad;   // first failing sweep wins (zeroed by the init kernel)
  }

  // Result: the lower triangle mirrored (exactly symmetric).  small: X = +inverse.  Otherwise
  // Q = +inverse, zero padded, and the swept block (-inverse) back into X.
  const int j = t & (NB - 1), i0 = t >> 7;
  if (n == NB) {
    const rsrc_t rs_q = make_rsrc(Mx.Q, small ? 0u : NB * NB * 4u);
    const rsrc_t rs_out = make_rsrc(Mx.X, small ? (uint32_t)d * (uint32_t)d * 4u : Mx.xelems * 4u);
    uint32_t offq = (uint32_t)(i0 * NB + j) * 4u;
    uint32_t offx = ((uint32_t)(k0 + i0) * (uint32_t)ld + (uint32_t)(k0 + j)) * 4u;
    const uint32_t row2 = 2u * (uint32_t)ld * 4u;
    int la = i0 * SP + j, lb = j * SP + i0;
#pragma unroll 16
    for (int u = 0; u < 64; ++u) {
      const float v = S[i0 + 2 * u >= j ? la : lb];
      if (small) {
        buf_store(rs_out, offx, -v);
        const int i = i0 + 2 * u;
        if (Mx.P && j >= i) Mx.P[(size_t)i * d - (size_t)i * (i - 1) / 2 + (j - i)] = -v;
      } else {
        buf_store(rs_q, offq, -v);
        buf_store(rs_out, offx, v);
      }
      la += 2 * SP; lb += 2;
      offq += 2u * NB * 4u; offx += row2;
    }
  } else {
    gf_ptr X = as_global(Mx.X);
    gf_ptr Q = as_global(Mx.Q);
#pragma unroll 8
    for (int e = t; e < NB * NB; e += NT) {
      const int i = e >> 7, jj = e & (NB - 1);
      const bool in = i < n && jj < n;
      const float v = i >= jj ? S[i * SP + jj] : S[jj * SP + i];
      if (small) {
        if (in) X[(size_t)i * ld + jj] = -v;
        if (in && Mx.P && jj >= i) Mx.P[(size_t)i * d - (size_t)i * (i - 1) / 2 + (jj - i)] = -v;
      } else {
        Q[i * NB + jj] = in ? -v : 0.f;
        if (in) X[(size_t)(k0 + i) * ld + k0 + jj] = v;
      }
    }
  }
#ifdef KFAC_TRACE
  __builtin_amdgcn_s_waitcnt(0);
  TRACE_T(4);
  trace_rec(trace, 1 + fuse + 8 * Mx.ld, step, tr);
#endif
}

__global__ __launch_bounds__(NT) void gj_pivot_kernel(const InvMat* __restrict__ mats, const MatJob* __restrict__ jobs,
                                                      int mat0, int step, float gamma, int small, int* cu_flags) {
  __shared__ float smem[PIVOT_LDS_FLOATS];
  const InvMat Mx = mats[jobs ? jobs[blockIdx.x].mat : mat0 + (int)blockIdx.x];   // a job list, or consecutive matrices
  cu_enter(cu_flags);
  pivot_body(Mx, step, gamma, small, 0, smem, cu_flags);
  cu_leave(cu_flags);
}

// One launch for two things that do not depend on each other: workgroups [0, npiv) sweep pivot
// block `step` of their matrices (applying the previous block's update to it themselves, fuse = 1),
// the others run the previous block's rank-NB update on every other tile.
__global__ __launch_bounds__(NT) void gj_pivot_update_kernel(const InvMat* __restrict__ mats, const MatJob* __restrict__ pjobs,
                                                             int npiv, int step, float gamma,
                                                             const TileDesc* __restrict__ descs,
                                                             const TileJob* __restrict__ ujobs, int nupd, int* cu_flags, int critical) {
  __shared__ __attribute__((aligned(16))) float smem[PIVOT_LDS_FLOATS > DL_DEEP_LDS_FLOATS ? PIVOT_LDS_FLOATS : DL_DEEP_LDS_FLOATS];
  const int g = blockIdx.x;
  if (g < npiv) {
    const InvMat Mx = mats[pjobs[g].mat];
    int* const mine = critical ? cu_flags : nullptr;
    cu_enter(mine);
    pivot_body(Mx, step, gamma, 0, 1, smem, cu_flags);
    cu_leave(mine);
  } else if (g - npiv < nupd) {
    const TileJob J = ujobs[g - npiv];
    run_tile_dl<true, true, DL_KC_DEEP>(descs[J.desc], J, smem, cu_flags);
  }
}

// ---- panel: Zt = old block column `step` (as [NB][ldp], k-major), Wt = Q * Zt, X panel <- W -----
// One job per 128-row tile `it` of the block column (it != step).  Tiles above the pivot live in
// block row `step` of the lower triangle (read along rows), tiles below in block column `step`.
__global__ __launch_bounds__(NT) void gj_panel_kernel(const InvMat* __restrict__ mats,
                                                      const MatJob* __restrict__ jobs, int njobs, int step, int* cu_flags) {
  // All loads of the 128-deep contraction (4 k chunks of Q and of the tile) are requested up front:
  // the kernel sits on the critical path with few workgroups, so it pays the memory latency once
  // instead of once per chunk.  The chunks then pass through two LDS buffers (the footprint of a
  // product workgroup, so the kernel fits beside one on a compute unit).
  constexpr int NCH = NB / KC;
  __shared__ float Qs[2 * PANEL];
  __shared__ float Zs[2 * PANEL];
  const int g = blockIdx.x;
  if (g >= njobs) return;
#ifdef KFAC_TRACE
  long long tr[5] = {0, 0, 0, 0, 0};
#endif
  TRACE_T(0);
  cu_enter(cu_flags);
  const MatJob J = jobs[g];
  const InvMat Mx = mats[J.mat];
  const int it = J.bi, slot = J.aux;   // slot: which 128 rows of the aggregated panel buffers this sweep fills
  const int t = threadIdx.x, lane = t & 63, w = t >> 6, wm = w >> 1, wn = w & 1;
  const int d = Mx.d, ldp = Mx.ldp;
  const uint32_t ld = (uint32_t)Mx.ld;
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
  const uint32_t cut = (uint32_t)(k0 + kb) * ld;
  const rsrc_t rs_x = make_rsrc(Mx.X, (above && cut < Mx.xelems ? cut : Mx.xelems) * 4u);
  const uint32_t d4 = ld * 4u;
  float rq[NCH][NU], rz[NCH][NU];
#pragma unroll
  for (int c = 0; c < NCH; ++c) {
    const int kk0 = c * KC;
#pragma unroll
    for (int u = 0; u < NU; ++u) rq[c][u] = buf_load(rs_q, (uint32_t)((kk0 + kp + 2 * u) * NB + ml) * 4u);
    if (above) {
      const uint32_t base = (uint32_t)(k0 + kk0 + kp) * d4 + (uint32_t)(i0 + ml) * 4u;
#pragma unroll
      for (int u = 0; u < NU; ++u) rz[c][u] = buf_load(rs_x, base + (uint32_t)(2 * u) * d4);
    } else {
      const int kk = kk0 + kl;
      const uint32_t base = kk < kb ? (uint32_t)(k0 + kk) * 4u : OOB_OFFSET;
#pragma unroll
      for (int u = 0; u < NU; ++u)     // rows past the (sub-)matrix read 0
        rz[c][u] = buf_load(rs_x, i0 + mg + MG * u < d ? base + (uint32_t)(i0 + mg + MG * u) * d4 : OOB_OFFSET);
    }
  }
  Acc4 acc;
  acc_zero(acc);
  gf_ptr Zt = as_global(Mx.Zt);
#pragma unroll
  for (int c = 0; c < NCH; ++c) {
    float* Qc = Qs + (c & 1) * PANEL;
    float* Zc = Zs + (c & 1) * PANEL;
    // rows kp + 2u, u = 4g .. 4g+3, are the contiguous positions 8g + 4kp .. +3 of row ml (16-byte stores)
#pragma unroll
    for (int gq = 0; gq < NU / 4; ++gq)
      *reinterpret_cast<f32x4*>(Qc + ml * PK + 8 * gq + 4 * kp) = f32x4{rq[c][4 * gq], rq[c][4 * gq + 1], rq[c][4 * gq + 2], rq[c][4 * gq + 3]};
    if (above) {
#pragma unroll
      for (int gq = 0; gq < NU / 4; ++gq)
        *reinterpret_cast<f32x4*>(Zc + ml * PK + 8 * gq + 4 * kp) = f32x4{rz[c][4 * gq], rz[c][4 * gq + 1], rz[c][4 * gq + 2], rz[c][4 * gq + 3]};
    } else {
#pragma unroll
      for (int u = 0; u < NU; ++u) Zc[lds_idx(mg + MG * u, kl)] = rz[c][u];
    }
    __syncthreads();   // chunk c staged; the other buffer (chunk c - 1) may still be read by slower waves
#ifdef KFAC_TRACE
    if (c == 0) TRACE_T(1);
    if (c == NCH - 1) TRACE_T(2);
#endif
#pragma unroll
    for (int gq = 0; gq < NU / 4; ++gq) {
      const f32x4 zv = *reinterpret_cast<const f32x4*>(Zc + ml * PK + 8 * gq + 4 * kp);
#pragma unroll
      for (int e = 0; e < 4; ++e) Zt[(size_t)(slot * NB + c * KC + kp + 2 * (4 * gq + e)) * ldp + i0 + ml] = zv[e];
    }
    switch (pat) {
      case PAT_FULL: mma_ktile<PAT_FULL>(Qc, Zc, acc, wm * 64, wn * 64, lane); break;
      case PAT_ROW1: mma_ktile<PAT_ROW1>(Qc, Zc, acc, wm * 64, wn * 64, lane); break;
      case PAT_COL1: mma_ktile<PAT_COL1>(Qc, Zc, acc, wm * 64, wn * 64, lane); break;
      case PAT_ONE: mma_ktile<PAT_ONE>(Qc, Zc, acc, wm * 64, wn * 64, lane); break;
      default: break;
    }
  }

  // acc(m, i) = W[i][m]: new panel entry for matrix row/col i0+i and pivot column k0+m
  gf_ptr Wt = as_global(Mx.Wt);
  const rsrc_t rs_o = make_rsrc(Mx.X, Mx.xelems * 4u);
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
#ifdef KFAC_TRACE
  TRACE_T(3);
  __builtin_amdgcn_s_waitcnt(0);
  TRACE_T(4);
  trace_rec(cu_flags, 8 * Mx.ld, step, tr);
#endif
  cu_leave(cu_flags);
}

// ---- finish: X = -(swept lower triangle), mirrored to a full symmetric matrix -------------------
__global__ __launch_bounds__(NT) void gj_finish_kernel(const InvMat* __restrict__ mats,
                                                       const MatJob* __restrict__ jobs, int njobs) {
  constexpr int FT = FINISH_TILE, PER = FT * FT / NT;
  __shared__ float tile[FT][FT + 1];
  const int g = blockIdx.x;
  if (g >= njobs) return;
  const MatJob J = jobs[g];
  const InvMat Mx = mats[J.mat];
  const int d = Mx.d;
  const int tx = threadIdx.x & (FT - 1), ty = threadIdx.x >> 6;   // 64 x 4: a wave moves 256 bytes of a row
  const int i0 = J.bi * FT, j0 = J.bj * FT;
  gf_ptr X = as_global(Mx.X);
  float v[PER];
#pragma unroll
  for (int r = 0; r < PER; ++r) {
    const int i = i0 + ty + 4 * r, j = j0 + tx;
    v[r] = (i < d && j < d && i >= j) ? X[(size_t)i * d + j] : 0.f;
  }
#pragma unroll
  for (int r = 0; r < PER; ++r) {
    const int li = ty + 4 * r, i = i0 + li, j = j0 + tx;
    const float x = -v[r];
    if (i < d && j < d && i >= j) X[(size_t)i * d + j] = x;
    tile[li][tx] = x;
  }
  __syncthreads();
#pragma unroll
  for (int r = 0; r < PER; ++r) {
    const int lj = ty + 4 * r;             // row of the mirrored tile = column index of the source
    const int j = j0 + lj, i = i0 + tx;    // writes X[j][i] = X[i][j], i > j
    if (i < d && j < d && i > j) X[(size_t)j * d + i] = tile[tx][lj];
    // packed upper triangle, row j: element (j, i), i >= j, at j*d - j(j-1)/2 + (i - j)
    if (Mx.P && i < d && j < d && i >= j) as_global(Mx.P)[(size_t)j * d - (size_t)j * (j - 1) / 2 + (i - j)] = tile[tx][lj];
  }
}

// ---- QB = +inverse of a swept sub-matrix view, full symmetric ------------------------------------
// The view holds -inverse in its lower triangle (diagonal tiles full).  One job per 32 x 32 tile
// (bi, bj) of the output; tiles above the diagonal are read transposed through LDS.
__global__ __launch_bounds__(NT) void gj_qmirror_kernel(const InvMat* __restrict__ mats,
                                                        const MatJob* __restrict__ jobs, int njobs) {
  __shared__ float tile[32][33];
  const int g = blockIdx.x;
  if (g >= njobs) return;
  const MatJob J = jobs[g];
  const InvMat Mx = mats[J.mat];
  const int d = Mx.d, ld = Mx.ld, ldq = Mx.ldp;
  const int tx = threadIdx.x & 31, ty = threadIdx.x >> 5;   // 32 x 8
  const bool upper = J.bi < J.bj;
  const int si = (upper ? J.bj : J.bi) * 32, sj = (upper ? J.bi : J.bj) * 32;   // source tile in the lower triangle
#pragma unroll
  for (int r = 0; r < 4; ++r) {
    const int li = ty + 8 * r;
    const int i = si + li, j = sj + tx;
    float v = 0.f;
    if (i < d && j < d) {
      // inside a diagonal 32 x 32 tile only the lower triangle is taken, which makes QB exactly symmetric
      const int hi = i > j ? i : j, lo = i > j ? j : i;
      v = -Mx.X[(size_t)hi * ld + lo];
    }
    tile[li][tx] = v;
  }
  __syncthreads();
#pragma unroll
  for (int r = 0; r < 4; ++r) {
    const int li = ty + 8 * r;
    const int i = J.bi * 32 + li, j = J.bj * 32 + tx;
    if (i < d && j < d) Mx.QB[(size_t)i * ldq + j] = upper ? tile[tx][li] : tile[li][tx];
  }
}

// ---- block column <-> k-major panel buffer ---------------------------------------------------------
// Grid (jobs, 32-wide k chunks): one workgroup moves a 128 (i) x 32 (k) piece of the 128-row tile
// `it` of the whole matrix outside the block column [c0, c0 + w).  Tiles above the block column
// live in block rows c0.. of the lower triangle (plain 2-D copy); tiles below are transposed
// through LDS.  to_matrix = 0: buf <- matrix (columns past d are zero-filled); 1: matrix <- buf.
__global__ __launch_bounds__(NT) void gj_move_kernel(const PanelMove* __restrict__ moves,
                                                     const MatJob* __restrict__ jobs, int njobs, int to_matrix) {
  __shared__ float tile[4][32][33];
  const int g = blockIdx.x;
  if (g >= njobs) return;
  const MatJob J = jobs[g];
  const PanelMove Mv = moves[J.mat];
  const int d = Mv.d, ldp = Mv.ldp, c0 = Mv.c0, w = Mv.w;
  const int kt = blockIdx.y * 32;
  if (kt >= w) return;
  const int i0 = J.bi * BM;
  const int tx = threadIdx.x & 31, ty = threadIdx.x >> 5;   // 32 x 8
  gf_ptr X = as_global(Mv.X);
  gf_ptr B = as_global(Mv.buf);
  float v[4][4];
  if (i0 < c0) {
    // above: buf[k][i] <-> X[(c0 + k) * d + i], both contiguous in i
#pragma unroll
    for (int r = 0; r < 4; ++r)
#pragma unroll
      for (int q = 0; q < 4; ++q) {
        const int k = kt + ty + 8 * r, i = i0 + tx + 32 * q;
        v[r][q] = 0.f;
        if (k < w && i < d) v[r][q] = to_matrix ? B[(size_t)k * ldp + i] : X[(size_t)(c0 + k) * d + i];
      }
#pragma unroll
    for (int r = 0; r < 4; ++r)
#pragma unroll
      for (int q = 0; q < 4; ++q) {
        const int k = kt + ty + 8 * r, i = i0 + tx + 32 * q;
        if (k >= w) continue;
        if (to_matrix) {
          if (i < d) X[(size_t)(c0 + k) * d + i] = v[r][q];
        } else {
          B[(size_t)k * ldp + i] = v[r][q];
        }
      }
    return;
  }
  // below: buf[k][i] <-> X[i * d + c0 + k]; q = 32-row group of i, a = slow index inside a 32 x 32 tile
#pragma unroll
  for (int q = 0; q < 4; ++q)
#pragma unroll
    for (int r = 0; r < 4; ++r) {
      const int a = ty + 8 * r;
      v[q][r] = 0.f;
      if (to_matrix) {            // source rows k, columns i
        const int k = kt + a, i = i0 + 32 * q + tx;
        if (k < w) v[q][r] = B[(size_t)k * ldp + i];
      } else {                    // source rows i, columns k
        const int i = i0 + 32 * q + a, k = kt + tx;
        if (i < d && k < w) v[q][r] = X[(size_t)i * d + c0 + k];
      }
    }
#pragma unroll
  for (int q = 0; q < 4; ++q)
#pragma unroll
    for (int r = 0; r < 4; ++r) tile[q][ty + 8 * r][tx] = v[q][r];
  __syncthreads();
#pragma unroll
  for (int q = 0; q < 4; ++q)
#pragma unroll
    for (int r = 0; r < 4; ++r) {
      const int a = ty + 8 * r;
      const float x = tile[q][tx][a];
      if (to_matrix) {            // destination rows i, columns k
        const int i = i0 + 32 * q + a, k = kt + tx;
        if (i < d && k < w) X[(size_t)i * d + c0 + k] = x;
      } else {                    // destination rows k, columns i
        const int k = kt + a, i = i0 + 32 * q + tx;
        if (k < w) B[(size_t)k * ldp + i] = x;
      }
    }
}

// ---- packed upper triangles <-> full symmetric matrices -------------------------------------------
// One job per 64 x 64 tile (bi <= bj) of the upper triangle.  to_full = 0: packed <- upper triangle
// of M (rows are contiguous on both sides).  to_full = 1: M <- packed, both triangles; the mirror
// image goes through LDS so that it is stored row by row as well.
constexpr int PT = 64;
__global__ __launch_bounds__(NT) void tri_pack_kernel(const PackMat* __restrict__ mats, const MatJob* __restrict__ jobs,
                                                      int njobs, float* __restrict__ packed, int to_full) {
  __shared__ float tile[PT][PT + 1];
  const int g = blockIdx.x;
  if (g >= njobs) return;
  const MatJob J = jobs[g];
  const PackMat P = mats[J.mat];
  const int d = P.d;
  const int tx = threadIdx.x & (PT - 1), ty = threadIdx.x >> 6;   // 64 x 4
  gf_ptr M = as_global(P.M);
  gf_ptr T = as_global(packed) + P.off;
  constexpr int PER = PT * PT / NT;
  float v[PER];
#pragma unroll
  for (int r = 0; r < PER; ++r) {
    const int i = J.bi * PT + ty + 4 * r, j = J.bj * PT + tx;
    const size_t p = (size_t)i * d - (size_t)i * (i - 1) / 2 + (size_t)(j - i);
    v[r] = 0.f;
    if (i < d && j < d && i <= j) v[r] = to_full ? T[p] : M[(size_t)i * d + j];
  }
#pragma unroll
  for (int r = 0; r < PER; ++r) {
    const int i = J.bi * PT + ty + 4 * r, j = J.bj * PT + tx;
    const size_t p = (size_t)i * d - (size_t)i * (i - 1) / 2 + (size_t)(j - i);
    if (i < d && j < d && i <= j) {
      if (to_full) M[(size_t)i * d + j] = v[r];
      else T[p] = v[r];
    }
    tile[ty + 4 * r][tx] = v[r];
  }
  if (!to_full) return;
  __syncthreads();
#pragma unroll
  for (int r = 0; r < PER; ++r) {   // element (jj, ii) of the mirrored tile = tile[ii - i0][jj - j0]
    const int jj = J.bj * PT + ty + 4 * r, ii = J.bi * PT + tx;
    if (jj < d && ii < jj) M[(size_t)jj * d + ii] = tile[tx][ty + 4 * r];
  }
}

void launch_gj_init(const InvMat* mats, const void* jobs, int njobs, float gamma, hipStream_t s) {
  if (njobs <= 0) return;
  hipLaunchKernelGGL(gj_init_kernel, dim3(njobs), dim3(NT), 0, s, mats, (const MatJob*)jobs, njobs, gamma);
}
int cu_flag_slots() { return CU_SLOTS; }
void launch_gj_pivot(const InvMat* mats, const void* jobs, int mat0, int nmats, int step, float gamma, int small, hipStream_t s, int lds_pad,
                     int* cu_flags) {
  if (nmats <= 0) return;
  hipLaunchKernelGGL(gj_pivot_kernel, dim3(nmats), dim3(NT), lds_pad, s, mats, (const MatJob*)jobs, mat0, step, gamma, small, cu_flags);
}
void launch_gj_pivot_update(const InvMat* mats, const void* pjobs, int npiv, int step, float gamma,
                            const TileDesc* descs, const TileJob* ujobs, int nupd, hipStream_t s, int lds_pad, int* cu_flags, int critical) {
  if (npiv <= 0 && nupd <= 0) return;
  hipLaunchKernelGGL(gj_pivot_update_kernel, dim3(npiv + nupd), dim3(NT), lds_pad, s, mats, (const MatJob*)pjobs, npiv, step, gamma,
                     descs, ujobs, nupd, cu_flags, critical);
}
void launch_gj_panel(const InvMat* mats, const void* jobs, int njobs, int step, hipStream_t s, int lds_pad, int* cu_flags) {
  if (njobs <= 0) return;
  hipLaunchKernelGGL(gj_panel_kernel, dim3(njobs), dim3(NT), lds_pad, s, mats, (const MatJob*)jobs, njobs, step, cu_flags);
}
void launch_gj_qmirror(const InvMat* mats, const void* jobs, int njobs, hipStream_t s) {
  if (njobs <= 0) return;
  hipLaunchKernelGGL(gj_qmirror_kernel, dim3(njobs), dim3(NT), 0, s, mats, (const MatJob*)jobs, njobs);
}
void launch_gj_move(const PanelMove* moves, const void* jobs, int njobs, int kchunks, int to_matrix, hipStream_t s) {
  if (njobs <= 0 || kchunks <= 0) return;
  hipLaunchKernelGGL(gj_move_kernel, dim3(njobs, kchunks), dim3(NT), 0, s, moves, (const MatJob*)jobs, njobs, to_matrix);
}
void launch_tri_pack(const PackMat* mats, const void* jobs, int njobs, float* packed, int to_full, hipStream_t s) {
  if (njobs <= 0) return;
  hipLaunchKernelGGL(tri_pack_kernel, dim3(njobs), dim3(NT), 0, s, mats, (const MatJob*)jobs, njobs, packed, to_full);
}
void launch_gj_finish(const InvMat* mats, const void* jobs, int njobs, hipStream_t s) {
  if (njobs <= 0) return;
  hipLaunchKernelGGL(gj_finish_kernel, dim3(njobs), dim3(NT), 0, s, mats, (const MatJob*)jobs, njobs);
}

}  // namespace kfac
