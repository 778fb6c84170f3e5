// Shared host/device descriptors of the K-FAC kernels (gfx950).
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace kfac {

// ---- exact unsigned division by a run-time invariant (multiply-high + shifts) -------------
struct FastDiv {
  uint32_t m, sh1, sh2;
};

__host__ __device__ inline FastDiv make_fastdiv(uint32_t d) {
  // round-up method for invariant divisors: l = ceil(log2 d), m = floor(2^32 (2^l - d) / d) + 1
  uint32_t l = 0;
  while ((uint64_t(1) << l) < d) ++l;
  FastDiv f;
  f.m = uint32_t(((uint64_t(1) << 32) * ((uint64_t(1) << l) - d)) / d + 1);
  f.sh1 = l < 1 ? l : 1;
  f.sh2 = l > 0 ? l - 1 : 0;
  return f;
}

__host__ __device__ inline uint32_t fast_div(uint32_t n, FastDiv f) {
#if defined(__HIP_DEVICE_COMPILE__)
  uint32_t t = __umulhi(f.m, n);
#else
  uint32_t t = uint32_t((uint64_t(f.m) * n) >> 32);
#endif
  return (t + ((n - t) >> f.sh1)) >> f.sh2;
}

// ---- tile geometry -------------------------------------------------------------------------
constexpr int BM = 128;   // output tile rows
constexpr int BN = 128;   // output tile columns
#ifndef KFAC_KC
#define KFAC_KC 32
#endif
constexpr int KC = KFAC_KC;    // contraction depth staged in LDS per step
constexpr int NT = 256;   // threads per workgroup (4 wavefronts, 2x2, 64x64 outputs each)
constexpr int PK = KC + 4;                // LDS row pitch in floats: one row per operand column, 16-byte aligned
constexpr int PANEL = BM * PK;            // floats of one staged operand panel
constexpr int MAX_JOB_ROWS = 8192;       // longest run one job accumulates in its fp32 accumulator

// ---- a GEMM operand seen as a [K x M] matrix, k = contraction index ------------------------
enum : int32_t {
  OP_KMAJOR = 0,   // element (k, m) at ptr[k*ld + m]; optional virtual ones column at m = M-1
  OP_CONV11 = 1,   // NCHW tensor through a 1x1 window (also: plain [M, K] row-major matrices)
  OP_CONV33 = 2,   // 3x3 window
  OP_CONV77 = 3,   // 7x7 window
  OP_CONVGEN = 4,  // any window (run-time kh, kw)
  OP_CONV25 = 5,   // 2x5 window (lag products)
  OP_CONV13 = 6,   // 1x3 window (lag products)
  OP_CONV11V = 7   // 1x1 window, stride 1, whole images of 4p pixels: read four pixels at a time
};

struct Operand {
  const float* ptr;
  int32_t type;
  int32_t K;        // contraction extent (rows R of the activation / gradient matrix)
  int32_t M;        // free extent, including the ones column when bias = 1
  int32_t bias;     // 1: column M-1 is an implicit column of ones
  int32_t ld;       // OP_KMAJOR: row pitch in elements
  uint32_t bytes;   // size of the tensor behind ptr (buffer-load range check); < 2 GiB
  // convolution view: k = (n*OH + oy)*OW + ox,  m = (c*KH + i)*KW + j; element = input pixel
  // ((oy + oy0)*stride - pad_h + i, (ox + ox0)*stride - pad_w + j), 0 outside the image.
  // OH x OW is the extent of the window of output pixels that is contracted, (oy0, ox0) its origin;
  // pads may be negative (windows that look only forward).
  int32_t C, H, W, OH, OW, stride, pad_h, pad_w, oy0, ox0, KH, KW;
  FastDiv dOW, dOHW;
};

// out = beta * out + alpha * (a^T b), optionally on the lower triangle with mirroring
enum : int32_t { MIRROR_NONE = 0, MIRROR_ALL = 1, MIRROR_DIAG_TILE = 2 };

struct TileDesc {
  Operand a, b;
  float* out;
  float* partial;   // split-reduction slots, [slot][BM*BN]
  float* packed;    // symmetric outputs, may be null: packed upper triangle of out (element (i, j), i <= j, at
                    // i*M - i*(i-1)/2 + (j - i)), written by the kernel that writes out
  int32_t ldo;
  int32_t M, N;     // output extents
  int32_t sym;      // 1: only tiles bi >= bj exist; a diagonal tile stages one panel, skips blocks above the diagonal
  int32_t mirror;
  float alpha, beta;
};

struct TileJob {
  int32_t desc;
  int32_t bi, bj;
  int32_t kbeg, kend;
  int32_t part;     // >= 0: write the raw tile to partial slot `part`; -1: apply the epilogue directly
  int32_t quarter;  // jobs of the quarter-tile kernel: 1 + the 32-column block of the tile this job computes
  int32_t pad1;
};

// reduction of split tiles: out = beta*out + alpha * sum_s partial[part0 + s]
struct ReduceJob {
  int32_t desc;
  int32_t bi, bj;
  int32_t part0, nsplit;
  int32_t pad0, pad1, pad2;
};

// ---- activation factor of a 3x3 / stride 1 / pad 1 convolution from lag products --------------
// With a the [n, C, H, W] activations (zero outside the image) and t = (i, j), t' = (i', j') two taps,
//   A[(c,t),(c',t')] = sum over pixels q with q - (t - 1) inside the image of a[c, q] * a[c', q + (t' - t)],
// which depends on the taps only through the lag t' - t and through which border row / column of q
// the first tap excludes.  So the 81 C x C blocks follow from lag products over the whole image,
//   G1[c, (c', dy, dx)], dy in {1, 2}, dx in {-2..2};   G2[c, (c', 0, dx)], dx in {0, 1, 2}
// (negative lags are transposes), minus the same products restricted to one border row and one
// border column of q, plus the corner pixel.  Of the lags the excluding tap can ask for, only those
// along the strip pair two pixels inside the image (the tap that drops the bottom row asks for
// dy >= 0, and nothing lies below that row), and a strip is closed under shifts along itself, so a row
// strip needs the forward lags dx = 0, 1, 2 (backward: transposes), a column strip dy = 0, 1, 2 and a
// corner lag 0; a ones column gives the bias sums.
enum : int32_t { LAG_G1 = 0, LAG_G2, LAG_TOP, LAG_BOT, LAG_LEFT, LAG_RIGHT, LAG_TL, LAG_TR, LAG_BL, LAG_BR, LAG_NMAT };

struct LagAsm {
  const float* G[LAG_NMAT];   // G1 [C][10C], G2 [C][3C + bias], rows/columns [C][3C + bias], corners [C][C + bias]
  float* A;                   // [dA][dA], dA = 9C + bias
  float* P;                   // may be null: packed upper triangle of A, dA (dA + 1) / 2 floats
  int32_t C, bias, dA, pad0;
  float alpha, beta;          // A <- beta * A + alpha * (assembled sums)
  float rows;                 // number of rows R (the bias-bias entry sums R ones)
  float pad1;
};

struct LagJob {
  int32_t lag, bi, bj, pad;
};

// ---- batched inversion ---------------------------------------------------------------------
constexpr int NB = 128;   // pivot block order of the blocked symmetric sweep
constexpr int FINISH_TILE = 64;   // tile of the final negate-and-mirror pass

struct InvMat {
  const float* F;   // input [d, d] (whole matrices only)
  float* X;         // work matrix, or a diagonal sub-matrix of it: element (i, j) at X[i*ld + j]
  float* Wt;        // panel workspace [NB][ldp]: new column panel (scaled by the inverse pivot)
  float* Zt;        // panel workspace [NB][ldp]: old column panel
  float* Q;         // inverse pivot block [NB][NB]
  float* QB;        // sub-matrix views: full symmetric inverse of the swept view, [d][ldp]
  int32_t* info;    // may be null
  float* P;         // whole matrices only, may be null: packed upper triangle of the result, d(d+1)/2 floats
  int32_t d, ld, ldp;
  int32_t info_base;   // row of the whole matrix at which this view starts
  uint32_t xelems;     // floats from X to the end of the allocation behind it (buffer range checks)
  int32_t pad;
};

// One block column of a whole matrix being moved between the matrix and a k-major panel buffer:
// buf[k][i] <-> column c0 + k, row i of the symmetric matrix (lower triangle storage), k < w.
struct PanelMove {
  float* X;
  float* buf;
  int32_t d, ldp, c0, w;
};

// ---- packed upper triangles ---------------------------------------------------------------------
// Element (i, j), i <= j, of matrix m lives at packed[off + i*d - i*(i-1)/2 + (j - i)].
struct PackMat {
  float* M;        // full matrix [d][d]
  uint64_t off;    // float offset of the matrix's triangle in the concatenated buffer
  int32_t d, pad;
};

}  // namespace kfac
