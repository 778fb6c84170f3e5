// 128x128 output-tile engine for gfx950: operand loaders (plain row-major and fused
// patch-expansion of NCHW tensors), LDS staging, fp32 MFMA contraction, epilogues.
//
// One workgroup of 256 threads (4 wavefronts as 2x2, 64x64 outputs each, built from
// v_mfma_f32_32x32x2_f32 blocks) computes  acc[i][j] = sum_k a(k, i0+i) * b(k, j0+j)
// over a k-range.  Operands are staged as [k][m] panels in LDS (double-buffered, one
// barrier per 32-deep k step); the next panel's global loads are in flight while the
// current one is multiplied.  Every 2048 contraction rows the MFMA accumulator is
// flushed into a second register set, so long sums of non-negative products (ReLU
// activations over 10^5 rows) keep fp32-level relative error.
#pragma once
#include "common.h"

namespace kfac {

typedef float f32x16 __attribute__((ext_vector_type(16)));

struct Acc4 {
  f32x16 c[4];   // block (a, b) of the wave's 2x2 grid of 32x32 blocks at index a*2+b
};

__device__ __forceinline__ void acc_zero(Acc4& x) {
#pragma unroll
  for (int q = 0; q < 4; ++q)
#pragma unroll
    for (int v = 0; v < 16; ++v) x.c[q][v] = 0.f;
}

__device__ __forceinline__ void acc_add(Acc4& t, const Acc4& x) {
#pragma unroll
  for (int q = 0; q < 4; ++q) t.c[q] += x.c[q];
}

// ------------------------------------------------------------------------------ loaders
// Each loader owns the per-thread part of moving one [KC x 128] operand panel:
//   load(k0, r)  : global -> 16 registers (predicated; out-of-range elements are 0)
//   store(lds, r): registers -> LDS panel laid out [k][m] with row pitch PITCH

// (k, m) at ptr[k*ld + m]: consecutive threads read consecutive m.
struct KMajorLoader {
  const float* colp;
  size_t ld;
  int kend, ml, kp;
  bool mvalid, isbias;

  __device__ __forceinline__ void init(const Operand& op, int m0, int kend_, int2* /*qtab*/, int t) {
    ml = t & (BM - 1);
    kp = t >> 7;
    const int m = m0 + ml;
    const int mreal = op.M - op.bias;
    mvalid = m < mreal;
    isbias = op.bias && m == mreal;
    colp = op.ptr + (mvalid ? m : 0);
    ld = (size_t)op.ld;
    kend = kend_;
  }
  __device__ __forceinline__ void load(int k0, float (&r)[16]) const {
#pragma unroll
    for (int u = 0; u < 16; ++u) {
      const int k = k0 + kp + 2 * u;
      const bool ok = k < kend;
      float v = (isbias && ok) ? 1.f : 0.f;
      if (ok && mvalid) v = colp[(size_t)k * ld];
      r[u] = v;
    }
  }
  __device__ __forceinline__ void store(float* lds, const float (&r)[16]) const {
#pragma unroll
    for (int u = 0; u < 16; ++u) lds[(kp + 2 * u) * PITCH + ml] = r[u];
  }
};

// NCHW tensor viewed through a KH x KW window: k = output pixel (n, oy, ox), m = (c, i, j).
// Consecutive threads read consecutive k (contiguous along ox for stride 1).
// KH_ = KW_ = 0 selects run-time window sizes.  KH_ = KW_ = 1 assumes pad = 0.
template <int KH_, int KW_>
struct ConvLoader {
  const float* base;
  const int2* q;
  size_t CHW;
  int kend, H, W, OHW, OW, stride, kl, mg;
  FastDiv dOW, dOHW;

  __device__ __forceinline__ void init(const Operand& op, int m0, int kend_, int2* qtab, int t) {
    const int KH = KH_ ? KH_ : op.KH, KW = KW_ ? KW_ : op.KW;
    if (t < BM) {
      const int m = m0 + t;
      const int mreal = op.M - op.bias;
      int2 e;
      if (m < mreal) {
        const int c = m / (KH * KW);
        const int rem = m - c * (KH * KW);
        const int i = rem / KW, j = rem - i * KW;
        const int dy = i - op.pad, dx = j - op.pad;
        e.x = c * op.H * op.W + dy * op.W + dx;
        e.y = ((dy + 128) & 0xff) | (((dx + 128) & 0xff) << 8);
      } else if (op.bias && m == mreal) {
        e.x = 0;
        e.y = 1 << 16;   // ones column
      } else {
        e.x = 0;
        e.y = 2 << 16;   // beyond the matrix: zero
      }
      qtab[t] = e;
    }
    base = op.ptr;
    q = qtab;
    CHW = (size_t)op.C * op.H * op.W;
    kend = kend_;
    H = op.H; W = op.W; OW = op.OW; OHW = op.OH * op.OW; stride = op.stride;
    dOW = op.dOW; dOHW = op.dOHW;
    kl = t & 31;
    mg = t >> 5;
  }
  __device__ __forceinline__ void load(int k0, float (&r)[16]) const {
    const int k = k0 + kl;
    const bool ok = k < kend;
    const uint32_t kk = ok ? (uint32_t)k : 0u;
    const uint32_t n = fast_div(kk, dOHW);
    const uint32_t rem = kk - n * (uint32_t)OHW;
    const uint32_t oy = fast_div(rem, dOW);
    const uint32_t ox = rem - oy * (uint32_t)OW;
    const int y0 = (int)oy * stride, x0 = (int)ox * stride;
    const float* pn = base + (size_t)n * CHW + (y0 * W + x0);
#pragma unroll
    for (int u = 0; u < 16; ++u) {
      const int2 e = q[mg + 8 * u];
      const int kind = e.y >> 16;
      float v = (kind == 1 && ok) ? 1.f : 0.f;
      bool in = ok && kind == 0;
      if (!(KH_ == 1 && KW_ == 1)) {
        const int dy = (e.y & 0xff) - 128, dx = ((e.y >> 8) & 0xff) - 128;
        in = in && (unsigned)(y0 + dy) < (unsigned)H && (unsigned)(x0 + dx) < (unsigned)W;
      }
      if (in) v = pn[e.x];
      r[u] = v;
    }
  }
  __device__ __forceinline__ void store(float* lds, const float (&r)[16]) const {
#pragma unroll
    for (int u = 0; u < 16; ++u) lds[kl * PITCH + mg + 8 * u] = r[u];
  }
};

// ------------------------------------------------------------------------------ MFMA step
// One staged k step (KC deep).  Lane l supplies a(k = l/32, i = l%32) and b(k = l/32, j = l%32).
template <bool MASKED>
__device__ __forceinline__ void mma_ktile(const float* __restrict__ As, const float* __restrict__ Bs,
                                          Acc4& acc, int wm, int wn, int lane, unsigned mask) {
  const float* ap = As + (lane >> 5) * PITCH + wm * 64 + (lane & 31);
  const float* bp = Bs + (lane >> 5) * PITCH + wn * 64 + (lane & 31);
#pragma unroll
  for (int ks = 0; ks < KC / 2; ++ks) {
    const float a0 = ap[ks * 2 * PITCH], a1 = ap[ks * 2 * PITCH + 32];
    const float b0 = bp[ks * 2 * PITCH], b1 = bp[ks * 2 * PITCH + 32];
    if (!MASKED || (mask & 1u)) acc.c[0] = __builtin_amdgcn_mfma_f32_32x32x2f32(a0, b0, acc.c[0], 0, 0, 0);
    if (!MASKED || (mask & 2u)) acc.c[1] = __builtin_amdgcn_mfma_f32_32x32x2f32(a0, b1, acc.c[1], 0, 0, 0);
    if (!MASKED || (mask & 4u)) acc.c[2] = __builtin_amdgcn_mfma_f32_32x32x2f32(a1, b0, acc.c[2], 0, 0, 0);
    if (!MASKED || (mask & 8u)) acc.c[3] = __builtin_amdgcn_mfma_f32_32x32x2f32(a1, b1, acc.c[3], 0, 0, 0);
  }
}

// Row / column of register v of a 32x32 MFMA result held by `lane`.
__device__ __forceinline__ int mfma_row(int v, int lane) { return 8 * (v >> 2) + 4 * (lane >> 5) + (v & 3); }
__device__ __forceinline__ int mfma_col(int lane) { return lane & 31; }

// Which of the wave's four 32x32 blocks hold any wanted output.
__device__ __forceinline__ unsigned block_mask(const TileDesc& D, int bi, int bj, int wm, int wn) {
  unsigned mask = 0;
  const bool diag = D.sym && bi == bj;
#pragma unroll
  for (int a = 0; a < 2; ++a)
#pragma unroll
    for (int b = 0; b < 2; ++b) {
      const int rlo = bi * BM + wm * 64 + a * 32, clo = bj * BN + wn * 64 + b * 32;
      bool v = rlo < D.M && clo < D.N;
      if (diag) v = v && (wm * 2 + a >= wn * 2 + b);
      if (v) mask |= 1u << (a * 2 + b);
    }
  return mask;
}

// LDS floats needed by run_tile: 2 operands x 2 buffers + two 128-entry int2 tables
constexpr int TILE_LDS_FLOATS = 4 * PANEL + 4 * BM;

template <class LA, class LB>
__device__ __forceinline__ void run_tile(const TileDesc& D, const TileJob& J, float* smem) {
  const int t = threadIdx.x, lane = t & 63, w = t >> 6, wm = w >> 1, wn = w & 1;
  const int i0 = J.bi * BM, j0 = J.bj * BN;
  const bool diag = D.sym && (J.bi == J.bj);
  const bool share = diag && D.a.ptr == D.b.ptr;   // a == b on a diagonal tile: stage one panel only
  float* As = smem;
  float* Bs = share ? As : smem + 2 * PANEL;
  int2* qA = reinterpret_cast<int2*>(smem + 4 * PANEL);
  int2* qB = qA + BM;

  LA la;
  LB lb;
  la.init(D.a, i0, J.kend, qA, t);
  if (!share) lb.init(D.b, j0, J.kend, qB, t);
  __syncthreads();

  const unsigned mask = block_mask(D, J.bi, J.bj, wm, wn);

  Acc4 acc, tot;
  acc_zero(acc);
  acc_zero(tot);
  float ra[16], rb[16];
  const int nkt = (J.kend - J.kbeg + KC - 1) / KC;
  if (nkt > 0) {
    la.load(J.kbeg, ra);
    if (!share) lb.load(J.kbeg, rb);
    la.store(As, ra);
    if (!share) lb.store(Bs, rb);
  }
  __syncthreads();
  int cur = 0;
  for (int kt = 0; kt < nkt; ++kt) {
    const bool more = kt + 1 < nkt;
    if (more) {
      la.load(J.kbeg + (kt + 1) * KC, ra);
      if (!share) lb.load(J.kbeg + (kt + 1) * KC, rb);
    }
    if (mask == 0xFu)
      mma_ktile<false>(As + cur * PANEL, Bs + cur * PANEL, acc, wm, wn, lane, mask);
    else if (mask)
      mma_ktile<true>(As + cur * PANEL, Bs + cur * PANEL, acc, wm, wn, lane, mask);
    if (more) {
      la.store(As + (cur ^ 1) * PANEL, ra);
      if (!share) lb.store(Bs + (cur ^ 1) * PANEL, rb);
    }
    __syncthreads();
    cur ^= 1;
    if ((kt % ACC_FLUSH) == ACC_FLUSH - 1) {
      acc_add(tot, acc);
      acc_zero(acc);
    }
  }
  acc_add(tot, acc);

  // ---- epilogue
  if (J.part >= 0) {
    float* P = D.partial + (size_t)J.part * (BM * BN);
#pragma unroll
    for (int qd = 0; qd < 4; ++qd) {
      if (!(mask & (1u << qd))) continue;
      const int rb0 = wm * 64 + (qd >> 1) * 32, cb0 = wn * 64 + (qd & 1) * 32;
#pragma unroll
      for (int v = 0; v < 16; ++v) P[(rb0 + mfma_row(v, lane)) * BN + cb0 + mfma_col(lane)] = tot.c[qd][v];
    }
    return;
  }
  const float alpha = D.alpha, beta = D.beta;
  const bool mirror = D.mirror == MIRROR_ALL || (D.mirror == MIRROR_DIAG_TILE && diag);
#pragma unroll
  for (int qd = 0; qd < 4; ++qd) {
    if (!(mask & (1u << qd))) continue;
    const int rb0 = i0 + wm * 64 + (qd >> 1) * 32, cb0 = j0 + wn * 64 + (qd & 1) * 32;
    const int gj = cb0 + mfma_col(lane);
#pragma unroll
    for (int v = 0; v < 16; ++v) {
      const int gi = rb0 + mfma_row(v, lane);
      if (gi < D.M && gj < D.N && (!D.sym || gi >= gj)) {
        float* o = D.out + (size_t)gi * D.ldo + gj;
        float val = alpha * tot.c[qd][v];
        if (beta != 0.f) val += beta * *o;
        *o = val;
        if (mirror && gi != gj) D.out[(size_t)gj * D.ldo + gi] = val;
      }
    }
  }
}

// Dispatch on the operand pair of a descriptor (wave-uniform).
__device__ __forceinline__ void run_tile_any(const TileDesc& D, const TileJob& J, float* smem) {
  const int ta = D.a.type, tb = D.b.type;
  if (ta == OP_KMAJOR && tb == OP_KMAJOR) run_tile<KMajorLoader, KMajorLoader>(D, J, smem);
  else if (ta == OP_CONV11 && tb == OP_CONV11) run_tile<ConvLoader<1, 1>, ConvLoader<1, 1>>(D, J, smem);
  else if (ta == OP_CONV33 && tb == OP_CONV33) run_tile<ConvLoader<3, 3>, ConvLoader<3, 3>>(D, J, smem);
  else if (ta == OP_CONV77 && tb == OP_CONV77) run_tile<ConvLoader<7, 7>, ConvLoader<7, 7>>(D, J, smem);
  else if (ta == OP_CONV11 && tb == OP_KMAJOR) run_tile<ConvLoader<1, 1>, KMajorLoader>(D, J, smem);
  else run_tile<ConvLoader<0, 0>, ConvLoader<0, 0>>(D, J, smem);
}

}  // namespace kfac
