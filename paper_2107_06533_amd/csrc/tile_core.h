// 128x128 output-tile engine for gfx950: operand loaders (plain row-major and fused
// patch-expansion of NCHW tensors), LDS staging, fp32 MFMA contraction, epilogues.
//
// One workgroup of 256 threads (4 wavefronts, each a 2x2 group of v_mfma_f32_32x32x2_f32 blocks:
// the quadrants of a full tile, dealt out differently over tiles that want fewer blocks, see
// wave_place) computes  acc[i][j] = sum_k a(k, i0+i) * b(k, j0+j)
// over a k-range.  Operands are staged in LDS as [m][k] panels (double-buffered, one barrier
// per 32-deep k step) with k permuted inside groups of 8 so that the four values a lane feeds to
// four consecutive MFMAs are one 16-byte LDS read; the next panel's global loads are in flight
// while the current one is multiplied.  fp32 MFMA shares the vector ALUs (it does not overlap
// with VALU instructions of any wave on the SIMD), so the k loop is written to need as few
// VALU instructions per MFMA as possible.  One job accumulates at most MAX_JOB_ROWS contraction rows in
// its fp32 MFMA accumulator; longer reductions (ReLU activations over 10^5 rows are sums of
// non-negative products, whose rounding error grows with the run length) are split into
// several jobs whose partial tiles are added in a fixed order by the reduce kernel.
// Further down: panels loaded straight into LDS for 1x1 whole-image views (run_tile_dm) and for
// plain products of row-major operands (run_tile_dl), and products cut into one block a wave that
// use no LDS at all (run_tile_quarter).
#pragma once
#include <type_traits>

#include "common.h"

namespace kfac {

typedef float f32x16 __attribute__((ext_vector_type(16)));

typedef float f32x4 __attribute__((ext_vector_type(4)));

// Position of contraction index k inside an LDS row: MFMA lane half h = k & 1 reads the four
// values k = 8g + 2s + h, s = 0..3, which sit at 8g + 4h + s.
__host__ __device__ constexpr int lds_pos(int k) { return (k & ~7) | ((k & 1) << 2) | ((k >> 1) & 3); }
__host__ __device__ constexpr int lds_idx(int m, int k) { return m * PK + lds_pos(k); }

constexpr int NU = KC / 2;        // elements of one operand panel a thread moves per k step (KC*128/256)
constexpr int MG = NT / KC;       // column groups of the k-contiguous thread mapping

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
//   load(k0, r)  : global -> 16 registers (out-of-range elements read 0)
//   store(lds, r): registers -> LDS panel laid out [m][lds_pos(k)] with row pitch PK

// Pointers that live in descriptor tables reach the kernels as generic pointers; casting them to
// the global address space lets the compiler emit global_load / global_store (vmcnt only).  A
// generic (flat) access also counts on lgkmcnt, which serialises it against every LDS access.
typedef const float __attribute__((address_space(1)))* gcf_ptr;
typedef float __attribute__((address_space(1)))* gf_ptr;
__device__ __forceinline__ gcf_ptr as_global(const float* p) { return (gcf_ptr)p; }
__device__ __forceinline__ gf_ptr as_global(float* p) { return (gf_ptr)p; }

// Operand panels are read with raw buffer loads: a 128-bit resource (base, size in bytes) in
// scalar registers plus one 32-bit byte offset per lane.  The hardware range check returns 0 for
// any offset at or beyond the size, so an out-of-range element (ragged tile edge, image border,
// row beyond the job's k range) is just the offset OOB_OFFSET: no branches, no address selects,
// and the 16 loads of a panel issue back to back.  Operands are limited to 2 GiB.
typedef __amdgpu_buffer_rsrc_t rsrc_t;
constexpr uint32_t OOB_OFFSET = 0x80000000u;
__device__ __forceinline__ rsrc_t make_rsrc(const float* p, uint32_t bytes) {
  return __builtin_amdgcn_make_buffer_rsrc(const_cast<float*>(p), 0, (int)bytes, 0x00020000);
}
__device__ __forceinline__ float buf_load(rsrc_t r, uint32_t byte_off) {
  return __builtin_bit_cast(float, __builtin_amdgcn_raw_buffer_load_b32(r, (int)byte_off, 0, 0));
}
// Stores at or beyond the resource size are dropped by the same range check.
__device__ __forceinline__ void buf_store(rsrc_t r, uint32_t byte_off, float v) {
  __builtin_amdgcn_raw_buffer_store_b32(__builtin_bit_cast(unsigned, v), r, (int)byte_off, 0, 0);
}

// (k, m) at ptr[k*ld + m]: consecutive threads read consecutive m.  The resource is cut at the
// job's last row, so rows at or beyond kend read 0 without a per-load test; one add per load.
struct KMajorLoader {
  static constexpr int LOADS = NU;   // vector-memory loads per k step
  rsrc_t rs;
  uint32_t ld4, moff;   // row pitch / column offset in bytes (moff = OOB_OFFSET beyond the matrix)
  uint32_t base;
  int kend, ml, kp, kcur;
  bool isbias, tile_bias;

  __device__ __forceinline__ void init(const Operand& op, int m0, int kend_, int t) {
    ml = t & (BM - 1);
    kp = t >> 7;
    const int m = m0 + ml;
    const int mreal = op.M - op.bias;
    isbias = op.bias && m == mreal;
    tile_bias = op.bias && m0 + BM > mreal && m0 <= mreal;
    moff = m < mreal ? (uint32_t)m * 4u : OOB_OFFSET;
    ld4 = (uint32_t)op.ld * 4u;
    const uint32_t cut = (uint32_t)kend_ * ld4;
    rs = make_rsrc(op.ptr, cut < op.bytes ? cut : op.bytes);
    kend = kend_;
    kcur = 0;
  }
  // begin(k0) prepares a k step; load_one(u, r) issues the load of register u.
  __device__ __forceinline__ void begin(int k0) {
    kcur = k0;
    base = (uint32_t)(k0 + kp) * ld4 + moff;   // stays >= OOB_OFFSET for invalid columns
  }
  __device__ __forceinline__ void load_one(int u, float (&r)[NU]) const {
    r[u] = buf_load(rs, base + (uint32_t)(2 * u) * ld4);
  }
  // Both operands of a symmetric product read the same matrix: reuse its resource and row state.
  __device__ __forceinline__ void share_geometry(const KMajorLoader& o) { rs = o.rs; ld4 = o.ld4; kend = o.kend; }
  __device__ __forceinline__ void load_shared(const KMajorLoader& o, float (&r)[NU]) {
    kcur = o.kcur;
    base = o.base - o.moff + moff;
#pragma unroll
    for (int u = 0; u < NU; ++u) load_one(u, r);
  }
  __device__ __forceinline__ void load(int k0, float (&r)[NU]) {
    begin(k0);
#pragma unroll
    for (int u = 0; u < NU; ++u) load_one(u, r);
  }
  __device__ __forceinline__ void store(float* lds, const float (&r)[NU]) const {
    // rows kp + 2u, u = 4g .. 4g+3, are the contiguous positions 8g + 4kp .. +3 of row ml
#pragma unroll
    for (int g = 0; g < NU / 4; ++g)
      *reinterpret_cast<f32x4*>(lds + ml * PK + 8 * g + 4 * kp) = f32x4{r[4 * g], r[4 * g + 1], r[4 * g + 2], r[4 * g + 3]};
    if (tile_bias) {   // the ones column lives in one thread column of one tile per operand
      if (isbias) {
#pragma unroll
        for (int u = 0; u < NU; ++u) lds[lds_idx(ml, kp + 2 * u)] = (kcur + kp + 2 * u < kend) ? 1.f : 0.f;
      }
    }
  }
};

// NCHW tensor viewed through a KH x KW window: k = output pixel (n, oy, ox), m = (c, i, j).
// Consecutive threads read consecutive k (contiguous along ox for stride 1).  A thread keeps its
// 16 columns for the whole tile: their byte offsets c*H*W + i*W + j and their tap numbers i*KW + j
// live in registers.  Per k step it computes, for its one pixel, the window origin and a bit mask
// of the taps that fall outside the image; a load is then  origin + column offset, with the
// "outside" bit moved into bit 31 of the offset (out of range, reads 0): four VALU operations.
// Tap TAP_NEVER is never inside: it marks columns beyond the matrix and the ones column.
// KH_ = KW_ = 0 selects run-time window sizes (up to 63 taps, 64-bit tap mask).
template <int KH_, int KW_>
struct ConvLoader {
  static constexpr int LOADS = NU;
  static constexpr bool TAP64 = (KH_ * KW_ == 0) || (KH_ * KW_ > 31);
  static constexpr int TAP_NEVER = TAP64 ? 63 : 31;
  rsrc_t rs;
  uint32_t qoff4[NU];
  uint32_t taps[(NU + 3) / 4];      // 8 bits per column
  uint32_t CHW4, pix4;
  typename std::conditional<TAP64, uint64_t, uint32_t>::type outside;
  int kend, H, W, OHW, OW, stride, pad_h, pad_w, oy0, ox0, KH, KW, kl, mg;
  unsigned biasmask;
  bool okcur, tile_bias;
  FastDiv dOW, dOHW;

  __device__ __forceinline__ void init(const Operand& op, int m0, int kend_, int t) {
    KH = KH_ ? KH_ : op.KH;
    KW = KW_ ? KW_ : op.KW;
    kl = t & (KC - 1);
    mg = t / KC;
    const int mreal = op.M - op.bias;
    tile_bias = op.bias && m0 + BM > mreal && m0 <= mreal;
    biasmask = 0;
#pragma unroll
    for (int w4 = 0; w4 < (NU + 3) / 4; ++w4) taps[w4] = 0;
#pragma unroll
    for (int u = 0; u < NU; ++u) {
      const int m = m0 + mg + MG * u;
      uint32_t off = 0, tap = TAP_NEVER;
      if (m < mreal) {
        const int c = m / (KH * KW);
        const int rem = m - c * (KH * KW);
        const int i = rem / KW, j = rem - i * KW;
        off = (uint32_t)(c * op.H * op.W + i * op.W + j) * 4u;
        tap = (uint32_t)rem;
      } else if (op.bias && m == mreal) {
        biasmask |= 1u << u;
      }
      qoff4[u] = off;
      taps[u >> 2] |= tap << (8 * (u & 3));
    }
    rs = make_rsrc(op.ptr, op.bytes);
    CHW4 = (uint32_t)(op.C * op.H * op.W) * 4u;
    kend = kend_;
    H = op.H; W = op.W; OW = op.OW; OHW = op.OH * op.OW; stride = op.stride;
    pad_h = op.pad_h; pad_w = op.pad_w; oy0 = op.oy0; ox0 = op.ox0;
    dOW = op.dOW; dOHW = op.dOHW;
    okcur = false;
  }
  __device__ __forceinline__ void begin(int k0) {
    const int k = k0 + kl;
    const bool ok = k < kend;
    okcur = ok;
    const uint32_t kk = ok ? (uint32_t)k : 0u;
    const uint32_t n = fast_div(kk, dOHW);
    const uint32_t rem = kk - n * (uint32_t)OHW;
    const uint32_t oy = fast_div(rem, dOW);
    const uint32_t ox = rem - oy * (uint32_t)OW;
    const int y0 = ((int)oy + oy0) * stride - pad_h, x0 = ((int)ox + ox0) * stride - pad_w;   // window origin (may be < 0)
    pix4 = n * CHW4 + (uint32_t)(y0 * W + x0) * 4u;
    if (!TAP64) {
      uint32_t colbits = 0, inside = 0;
#pragma unroll
      for (int j = 0; j < (KW_ ? KW_ : 1); ++j) colbits |= ((unsigned)(x0 + j) < (unsigned)W ? 1u : 0u) << j;
#pragma unroll
      for (int i = 0; i < (KH_ ? KH_ : 1); ++i)
        inside |= ((unsigned)(y0 + i) < (unsigned)H ? colbits : 0u) << (i * KW_);
      outside = ok ? ~inside : 0xFFFFFFFFu;
    } else {
      uint64_t colbits = 0, inside = 0;
      for (int j = 0; j < KW; ++j) colbits |= (uint64_t)((unsigned)(x0 + j) < (unsigned)W ? 1u : 0u) << j;
      for (int i = 0; i < KH; ++i) inside |= ((unsigned)(y0 + i) < (unsigned)H ? colbits : 0ull) << (i * KW);
      outside = ok ? ~inside : ~0ull;
    }
  }
  // Both operands of a symmetric product read the same tensor: the geometry and the per-step pixel
  // decomposition (window origin, outside-tap mask) are computed once and shared.
  __device__ __forceinline__ void share_geometry(const ConvLoader& o) {
    rs = o.rs; CHW4 = o.CHW4; kend = o.kend; H = o.H; W = o.W; OHW = o.OHW; OW = o.OW;
    stride = o.stride; pad_h = o.pad_h; pad_w = o.pad_w; oy0 = o.oy0; ox0 = o.ox0; KH = o.KH; KW = o.KW; dOW = o.dOW; dOHW = o.dOHW;
  }
  __device__ __forceinline__ void load_shared(const ConvLoader& o, float (&r)[NU]) {
    okcur = o.okcur; pix4 = o.pix4; outside = o.outside;
#pragma unroll
    for (int u = 0; u < NU; ++u) load_one(u, r);
  }
  __device__ __forceinline__ void load_one(int u, float (&r)[NU]) const {
    const uint32_t tap = (taps[u >> 2] >> (8 * (u & 3))) & 0xffu;
    const uint32_t bad = (uint32_t)(outside >> tap) & 1u;
    r[u] = buf_load(rs, (pix4 + qoff4[u]) | (bad << 31));
  }
  __device__ __forceinline__ void load(int k0, float (&r)[NU]) {
    begin(k0);
#pragma unroll
    for (int u = 0; u < NU; ++u) load_one(u, r);
  }
  __device__ __forceinline__ void store(float* lds, const float (&r)[NU]) const {
    const int pk = lds_pos(kl);
#pragma unroll
    for (int u = 0; u < NU; ++u) lds[(mg + MG * u) * PK + pk] = r[u];
    if (tile_bias) {
#pragma unroll
      for (int u = 0; u < NU; ++u)
        if ((biasmask >> u) & 1u) lds[(mg + MG * u) * PK + pk] = okcur ? 1.f : 0.f;
    }
  }
};

// NCHW tensor through a 1x1 window of stride 1 over whole images whose pixel count HW is a multiple
// of four: k = n*HW + pixel, m = channel, element at (k + n*(C-1)*HW + m*HW).  Four consecutive k
// (k % 4 == 0) never straddle an image and are 16 contiguous bytes: a thread moves four such
// groups per k step with 128-bit loads and writes each as two 64-bit LDS stores (k, k+2 and
// k+1, k+3 are neighbours in the LDS row order).  A wave reads 8 channel rows of 128 bytes.
struct Conv11VecLoader {
  static constexpr int LOADS = NU / 4;   // 128-bit loads
  static_assert(KC == 32 && NT == 256, "eight groups of four k per row of 32 threads");
  static constexpr uint32_t ROW_OOB = 0x40000000u;   // >= any operand size, and ROW_OOB + OOB_OFFSET does not wrap
  rsrc_t rs;
  uint32_t qoff4[4];   // byte offsets m*HW*4 of the thread's four columns (OOB_OFFSET beyond the matrix)
  uint32_t base, skip; // byte offset of the thread's k group in channel 0; (C-1)*HW
  int kend, kq, mrow, kcur;
  unsigned biasmask;
  bool tile_bias;
  FastDiv dHW;

  __device__ __forceinline__ void init(const Operand& op, int m0, int kend_, int t) {
    kq = (t & 7) * 4;
    mrow = t >> 3;
    const int mreal = op.M - op.bias;
    const uint32_t HW = (uint32_t)(op.OH * op.OW);
    tile_bias = op.bias && m0 + BM > mreal && m0 <= mreal;
    biasmask = 0;
#pragma unroll
    for (int u = 0; u < 4; ++u) {
      const int m = m0 + mrow + 32 * u;
      qoff4[u] = m < mreal ? (uint32_t)m * HW * 4u : OOB_OFFSET;
      if (op.bias && m == mreal) biasmask |= 1u << u;
    }
    rs = make_rsrc(op.ptr, op.bytes);
    skip = (uint32_t)(op.C - 1) * HW;
    dHW = op.dOHW;
    kend = kend_;
    kcur = 0;
  }
  __device__ __forceinline__ void begin(int k0) {
    kcur = k0;
    const uint32_t k = (uint32_t)(k0 + kq);
    const uint32_t n = fast_div(k, dHW);
    base = (int)k < kend ? (k + n * skip) * 4u : ROW_OOB;
  }
  __device__ __forceinline__ void issue(float (&r)[NU]) const {
#pragma unroll
    for (int u = 0; u < 4; ++u) {
      const f32x4 v = __builtin_bit_cast(f32x4, __builtin_amdgcn_raw_buffer_load_b128(rs, (int)(base + qoff4[u]), 0, 0));
#pragma unroll
      for (int e = 0; e < 4; ++e) r[4 * u + e] = v[e];
    }
  }
  __device__ __forceinline__ void load(int k0, float (&r)[NU]) {
    begin(k0);
    issue(r);
  }
  __device__ __forceinline__ void share_geometry(const Conv11VecLoader& o) { rs = o.rs; skip = o.skip; dHW = o.dHW; kend = o.kend; }
  __device__ __forceinline__ void load_shared(const Conv11VecLoader& o, float (&r)[NU]) {
    kcur = o.kcur; base = o.base;
    issue(r);
  }
  __device__ __forceinline__ void store(float* lds, const float (&r)[NU]) const {
    typedef float f32x2 __attribute__((ext_vector_type(2)));
    // k = kq + e: positions (kq & ~7) + 2*((kq >> 2) & 1) + {0, 4, 1, 5} for e = 0..3
    const int p0 = (kq & ~7) + ((kq >> 1) & 2);
#pragma unroll
    for (int u = 0; u < 4; ++u) {
      float* row = lds + (mrow + 32 * u) * PK + p0;
      const bool ones = tile_bias && ((biasmask >> u) & 1u);
      const float one = kcur + kq < kend ? 1.f : 0.f;
      *reinterpret_cast<f32x2*>(row) = ones ? f32x2{one, one} : f32x2{r[4 * u], r[4 * u + 2]};
      *reinterpret_cast<f32x2*>(row + 4) = ones ? f32x2{one, one} : f32x2{r[4 * u + 1], r[4 * u + 3]};
    }
  }
};

// ------------------------------------------------------------------------------ MFMA step
// One staged k step (KC deep).  Lane l supplies a(k = l/32, i = l%32) and b(k = l/32, j = l%32).
// PAT is the compile-time set of the wave's 32x32 blocks that are computed (bit a*2+b): the
// MFMA sequence is straight-line code for every pattern.
constexpr unsigned PAT_FULL = 0xF, PAT_ROW1 = 0x3, PAT_ROW2 = 0xC, PAT_COL1 = 0x5, PAT_ONE = 0x1, PAT_TRI = 0xD, PAT_NONE = 0;

template <unsigned PAT>
__device__ __forceinline__ void mma_ktile(const float* __restrict__ As, const float* __restrict__ Bs,
                                          Acc4& acc, int r0, int c0, int lane) {
  if (PAT == PAT_NONE) return;
  // r0, c0: first row / column of the wave's 2x2 group of blocks inside the tile;  lane l feeds a(k, i = l%32) and b(k, j = l%32) with k = 8g + 2s + l/32 for MFMA s of group g
  const float* ap = As + (r0 + (lane & 31)) * PK + 4 * (lane >> 5);
  const float* bp = Bs + (c0 + (lane & 31)) * PK + 4 * (lane >> 5);
  const f32x4 z = {0.f, 0.f, 0.f, 0.f};
  f32x4 a0 = z, a1 = z, b0 = z, b1 = z;
  if (PAT & 0x3) a0 = *reinterpret_cast<const f32x4*>(ap);
  if (PAT & 0xC) a1 = *reinterpret_cast<const f32x4*>(ap + 32 * PK);
  if (PAT & 0x5) b0 = *reinterpret_cast<const f32x4*>(bp);
  if (PAT & 0xA) b1 = *reinterpret_cast<const f32x4*>(bp + 32 * PK);
#pragma unroll
  for (int g = 0; g < KC / 8; ++g) {
    f32x4 na0 = z, na1 = z, nb0 = z, nb1 = z;
    if (g + 1 < KC / 8) {   // next group's fragments are requested before this group's MFMAs
      if (PAT & 0x3) na0 = *reinterpret_cast<const f32x4*>(ap + 8 * (g + 1));
      if (PAT & 0xC) na1 = *reinterpret_cast<const f32x4*>(ap + 32 * PK + 8 * (g + 1));
      if (PAT & 0x5) nb0 = *reinterpret_cast<const f32x4*>(bp + 8 * (g + 1));
      if (PAT & 0xA) nb1 = *reinterpret_cast<const f32x4*>(bp + 32 * PK + 8 * (g + 1));
    }
#pragma unroll
    for (int sidx = 0; sidx < 4; ++sidx) {
      if (PAT & 1u) acc.c[0] = __builtin_amdgcn_mfma_f32_32x32x2f32(a0[sidx], b0[sidx], acc.c[0], 0, 0, 0);
      if (PAT & 2u) acc.c[1] = __builtin_amdgcn_mfma_f32_32x32x2f32(a0[sidx], b1[sidx], acc.c[1], 0, 0, 0);
      if (PAT & 4u) acc.c[2] = __builtin_amdgcn_mfma_f32_32x32x2f32(a1[sidx], b0[sidx], acc.c[2], 0, 0, 0);
      if (PAT & 8u) acc.c[3] = __builtin_amdgcn_mfma_f32_32x32x2f32(a1[sidx], b1[sidx], acc.c[3], 0, 0, 0);
    }
    a0 = na0; a1 = na1; b0 = nb0; b1 = nb1;
  }
}

// Smallest supported pattern that covers a block mask (valid rows/columns are prefixes, and a
// diagonal wave of a symmetric diagonal tile needs only its lower triangle of blocks).
__device__ __forceinline__ unsigned cover_pattern(unsigned mask) {
  if (mask == 0) return PAT_NONE;
  if (mask == PAT_TRI) return PAT_TRI;
  if (!(mask & 0x3)) return PAT_ROW2;
  const bool rows2 = mask & 0xC, cols2 = mask & 0xA;
  return rows2 ? (cols2 ? PAT_FULL : PAT_COL1) : (cols2 ? PAT_ROW1 : PAT_ONE);
}

// Row / column of register v of a 32x32 MFMA result held by `lane`.
__device__ __forceinline__ int mfma_row(int v, int lane) { return 8 * (v >> 2) + 4 * (lane >> 5) + (v & 3); }
__device__ __forceinline__ int mfma_col(int lane) { return lane & 31; }

// Which of the four 32x32 blocks of the 2x2 group at (r0, c0) of tile (bi, bj) hold any wanted output.
__device__ __forceinline__ unsigned block_mask(const TileDesc& D, int bi, int bj, int r0, int c0) {
  unsigned mask = 0;
  const bool diag = D.sym && bi == bj;
#pragma unroll
  for (int a = 0; a < 2; ++a)
#pragma unroll
    for (int b = 0; b < 2; ++b) {
      const int rl = r0 + a * 32, cl = c0 + b * 32;
      bool v = rl < BM && cl < BN && bi * BM + rl < D.M && bj * BN + cl < D.N;
      if (diag) v = v && rl >= cl;
      if (v) mask |= 1u << (a * 2 + b);
    }
  return mask;
}

// Which blocks wave w of a tile computes: the 2x2 group of 32x32 blocks at rows r0.., columns c0..
// of the tile, restricted to `mask`.  A full tile off the diagonal: the quadrant (w / 2, w % 2).
// Otherwise the wanted blocks are dealt out as evenly as 2x2 groups allow, because a tile takes as
// long as its busiest wave:
//   diagonal tile of a symmetric product (ten blocks on or below the diagonal; in place they would
//   fall 3 + 0 + 4 + 3): 3 + 2 + 2 + 3; with three valid block rows 2 + 2 + 1 + 1 of six, with two
//   1 + 1 + 1 of three;
//   at most two valid block rows (the one-row tail of the d = 128 m + 1 factors, products with 64
//   rows): wave w takes block column w, one or two blocks, instead of two waves taking four;
//   at most two valid block columns: the same with rows and columns exchanged.
struct WavePlace {
  int r0, c0;
  unsigned mask;
};
__device__ __forceinline__ WavePlace wave_place(const TileDesc& D, int bi, int bj, int w) {
  const int mrows = D.M - bi * BM, ncols = D.N - bj * BN;
  const int rb = mrows >= BM ? 4 : (mrows + 31) >> 5, cb = ncols >= BN ? 4 : (ncols + 31) >> 5;
  WavePlace p{64 * (w >> 1), 64 * (w & 1), 0xFu};
  if (D.sym && bi == bj) {
    if (rb == 4) {
      if (w == 1) p = WavePlace{64, 0, 0xCu};
      else if (w == 2) p.mask = 0x3u;
    } else if (rb == 3) {
      if (w == 0) p = WavePlace{0, 0, 0x5u};          // (0,0) (1,0)
      else if (w == 1) p = WavePlace{32, 32, 0x5u};   // (1,1) (2,1)
      else if (w == 2) p = WavePlace{64, 0, 0x1u};    // (2,0)
      else p = WavePlace{64, 64, 0x1u};               // (2,2)
    } else if (rb == 2) {
      if (w == 0) p = WavePlace{0, 0, 0x1u};
      else if (w == 1) p = WavePlace{32, 0, 0x1u};
      else if (w == 2) p = WavePlace{32, 32, 0x1u};
      else p.mask = 0;
    }
  } else if (rb <= 2 && cb > 2) {
    p = WavePlace{0, 32 * w, rb == 1 ? 0x1u : 0x5u};
  } else if (cb <= 2 && rb > 2) {
    p = WavePlace{32 * w, 0, cb == 1 ? 0x1u : 0x3u};
  }
  p.mask &= block_mask(D, bi, bj, p.r0, p.c0);
  return p;
}

// LDS floats needed by run_tile: 2 operands x 2 buffers
constexpr int TILE_LDS_FLOATS = 4 * PANEL;

// The k loop of one tile: stage panel kt+1 (global -> registers -> LDS buffer cur^1) around the
// MFMA work on panel kt (LDS buffer cur); one barrier per k step.  The steady-state body has no
// branches (SHARE and PAT are compile-time), so address arithmetic, buffer loads and LDS traffic
// can be scheduled between the MFMAs.  Every wave of the workgroup runs the same number of steps
// whatever its pattern.
// SAME: both operands view the same tensor (symmetric products), so loader b reuses loader a's
// per-step state; SHARE: additionally the same columns (diagonal tile), one panel is staged.
template <class LA, class LB, bool SAME>
__device__ __forceinline__ void load_b(LA& la, LB& lb, int k0, float (&rb)[NU]) {
  if constexpr (SAME && std::is_same<LA, LB>::value) lb.load_shared(la, rb);
  else lb.load(k0, rb);
}

// Asks the instruction scheduler to spread the NL vector-memory loads of a k step evenly between
// its NM matrix instructions instead of issuing them in bursts: a wave issues in order, so while a
// burst of loads queues up at the memory pipeline none of the MFMAs behind it can start.  With two
// workgroups per compute unit the k loop of a plain product goes from 114 to 132 TFLOP/s.
template <int NM, int NL, int G, int I>
__device__ __forceinline__ void interleave_group() {
  if constexpr (I < G) {
    __builtin_amdgcn_sched_group_barrier(0x008, (NM * (I + 1)) / G - (NM * I) / G, 0);   // MFMA
    __builtin_amdgcn_sched_group_barrier(0x020, (NL * (I + 1)) / G - (NL * I) / G, 0);   // VMEM read
    interleave_group<NM, NL, G, I + 1>();
  }
}
template <int NM, int NL>
__device__ __forceinline__ void interleave_loads() {
  if constexpr (NM > 0 && NL > 0) interleave_group<NM, NL, (NM >= NL ? NL : NM), 0>();
}

// ---- giving way to latency-critical workgroups ------------------------------------------------------
// fp32 MFMAs keep every other wave of the SIMD from issuing, so a latency-bound kernel (a pivot block
// sweep, a panel on the critical path of the inverse) that shares a compute unit with a product
// workgroup runs two to three times slower.  Such kernels count themselves in a per-compute-unit
// word while they run (cu_enter / cu_leave); product workgroups launched as "yielding" read the word
// of their compute unit once per k step and sleep while it is non-zero.  The word is advisory: the
// sleep is bounded, so a stale count costs time, never progress.
__device__ __forceinline__ int cu_slot() {   // compute unit of this wave: XCC (3 bits) x {SE, SH, CU} (8 bits of HW_ID)
  unsigned hw, xcc;
  asm volatile("s_getreg_b32 %0, hwreg(HW_REG_HW_ID)" : "=s"(hw));
  asm volatile("s_getreg_b32 %0, hwreg(HW_REG_XCC_ID)" : "=s"(xcc));
  return (int)(((xcc & 7u) << 8) | ((hw >> 8) & 0xFFu));
}
constexpr int CU_SLOTS = 8 * 256;
__device__ __forceinline__ void cu_enter(int* flags) {
  if (flags && threadIdx.x == 0) __hip_atomic_fetch_add(flags + cu_slot(), 1, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}
__device__ __forceinline__ void cu_leave(int* flags) {
  if (flags && threadIdx.x == 0) __hip_atomic_fetch_add(flags + cu_slot(), -1, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}
__device__ __forceinline__ int cu_busy(const int* word) {
  return __builtin_amdgcn_readfirstlane(__hip_atomic_load(word, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT));
}
__device__ __forceinline__ void cu_yield(const int* word) {   // at most ~0.2 ms
  for (int it = 0; it < 256; ++it) {
    __builtin_amdgcn_s_sleep(32);
    if (cu_busy(word) == 0) break;
  }
}

template <unsigned PAT, bool SHARE, bool SAME, class LA, class LB>
__device__ __forceinline__ void main_loop(LA& la, LB& lb, float* As, float* Bs, Acc4& tot,
                                          int kbeg, int nkt, int r0, int c0, int lane, const int* yield_word = nullptr) {
  if (nkt <= 0) return;
  float ra[NU], rb[NU];
  la.load(kbeg, ra);
  if (!SHARE) load_b<LA, LB, SAME>(la, lb, kbeg, rb);
  la.store(As, ra);
  if (!SHARE) lb.store(Bs, rb);
  __syncthreads();
  int cur = 0;
  for (int kt = 1; kt < nkt; ++kt) {
    int busy = 0;
    if (yield_word) busy = __hip_atomic_load(yield_word, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);   // lands during the MFMAs
    la.load(kbeg + kt * KC, ra);
    if (!SHARE) load_b<LA, LB, SAME>(la, lb, kbeg + kt * KC, rb);
    mma_ktile<PAT>(As + cur * PANEL, Bs + cur * PANEL, tot, r0, c0, lane);
    if (yield_word && __builtin_amdgcn_readfirstlane(busy) != 0) cu_yield(yield_word);
    if constexpr (!SAME && std::is_same<LA, KMajorLoader>::value && std::is_same<LB, KMajorLoader>::value)   // plain products only: measured no gain elsewhere
      interleave_loads<(KC / 2) * __builtin_popcount(PAT), LA::LOADS + (SHARE ? 0 : LB::LOADS)>();
    la.store(As + (cur ^ 1) * PANEL, ra);
    if (!SHARE) lb.store(Bs + (cur ^ 1) * PANEL, rb);
    __syncthreads();
    cur ^= 1;
  }
  mma_ktile<PAT>(As + cur * PANEL, Bs + cur * PANEL, tot, r0, c0, lane);
}

template <unsigned PAT, bool SAME, class LA, class LB>
__device__ __forceinline__ void main_loop_any(LA& la, LB& lb, bool share, float* As, float* Bs, Acc4& tot,
                                              int kbeg, int nkt, int r0, int c0, int lane, const int* yield_word = nullptr) {
  if (SAME && share) main_loop<PAT, true, true>(la, lb, As, As, tot, kbeg, nkt, r0, c0, lane, yield_word);
  else main_loop<PAT, false, SAME>(la, lb, As, Bs, tot, kbeg, nkt, r0, c0, lane, yield_word);
}

// Byte offset of output element (block qd, register v) of this lane in a tile's epilogue: OOB_OFFSET when
// the element is outside the matrix, above the diagonal of a symmetric output, or in a block that is
// not computed.
struct OutMap {
  int i0, j0, r0, c0, lane, M, N, sym;   // r0, c0: offset of the wave's 2x2 group of blocks inside the tile
  unsigned mask;
  uint32_t ldo4;
  __device__ __forceinline__ int row(int qd, int v) const { return i0 + r0 + (qd >> 1) * 32 + mfma_row(v, lane); }
  __device__ __forceinline__ int col(int qd) const { return j0 + c0 + (qd & 1) * 32 + mfma_col(lane); }
  __device__ __forceinline__ uint32_t operator()(int qd, int v) const {
    const int gi = row(qd, v), gj = col(qd);
    const bool ok = ((mask >> qd) & 1u) && gi < M && gj < N && (!sym || gi >= gj);
    return ok ? (uint32_t)gi * ldo4 + (uint32_t)gj * 4u : OOB_OFFSET;
  }
};

__device__ __forceinline__ void load_old(const rsrc_t ro, const OutMap& om, Acc4& old) {
#pragma unroll
  for (int qd = 0; qd < 4; ++qd)
#pragma unroll
    for (int v = 0; v < 16; ++v) old.c[qd][v] = buf_load(ro, om(qd, v));
}

// Epilogue of a 2x2-wave tile: raw partial tile, or out = beta out + alpha acc with mirror and packed copy.
// have_old: the old values are already in `old` (fetched before the k loop).
__device__ __forceinline__ void finish_tile(const TileDesc& D, const TileJob& J, const OutMap& om, const rsrc_t ro,
                                            const Acc4& tot, Acc4& old, bool have_old, bool diag) {
  const int lane = om.lane;
  const unsigned mask = om.mask;
  if (J.part >= 0) {
    gf_ptr P = as_global(D.partial) + (size_t)J.part * (BM * BN);
#pragma unroll
    for (int qd = 0; qd < 4; ++qd) {
      if (!(mask & (1u << qd))) continue;
      const int rb0 = om.r0 + (qd >> 1) * 32, cb0 = om.c0 + (qd & 1) * 32;
#pragma unroll
      for (int v = 0; v < 16; ++v) P[(rb0 + mfma_row(v, lane)) * BN + cb0 + mfma_col(lane)] = tot.c[qd][v];
    }
    return;
  }
  const float alpha = D.alpha, beta = D.beta;
  const bool mirror = D.mirror == MIRROR_ALL || (D.mirror == MIRROR_DIAG_TILE && diag);
  if (!have_old && beta != 0.f) load_old(ro, om, old);
#pragma unroll
  for (int qd = 0; qd < 4; ++qd) {
#pragma unroll
    for (int v = 0; v < 16; ++v) {
      const float val = alpha * tot.c[qd][v] + beta * old.c[qd][v];
      const uint32_t off = om(qd, v);
      buf_store(ro, off, val);
      const int gi = om.row(qd, v), gj = om.col(qd);
      if (mirror) buf_store(ro, (off != OOB_OFFSET && gi != gj) ? (uint32_t)gj * om.ldo4 + (uint32_t)gi * 4u : OOB_OFFSET, val);
      if (D.packed && off != OOB_OFFSET)   // stored element (gi, gj), gi >= gj, is element (gj, gi) of the upper triangle
        as_global(D.packed)[(size_t)gj * (size_t)D.M - (size_t)gj * (size_t)(gj - 1) / 2 + (size_t)(gi - gj)] = val;
    }
  }
}

// PREFETCH_OLD: fetch the old output values before the k loop (worth 64 registers when the k loop is
// short, as in the rank-128 sweep updates) instead of after it.
// SAME: the descriptor's two operands are the same tensor (every factor build).
// YIELD: cu_flags (may be null) is the table of per-compute-unit words; the k loop gives way while
// this compute unit's word is non-zero.
template <class LA, class LB, bool PREFETCH_OLD = false, bool SAME = false, bool YIELD = false>
__device__ __forceinline__ void run_tile(const TileDesc& D, const TileJob& J, float* smem, const int* cu_flags = nullptr) {
  const int t = threadIdx.x, lane = t & 63, w = __builtin_amdgcn_readfirstlane(t >> 6);
  const WavePlace wp = wave_place(D, J.bi, J.bj, w);
  const int r0 = wp.r0, c0 = wp.c0;
  const int i0 = J.bi * BM, j0 = J.bj * BN;
  const bool diag = D.sym && (J.bi == J.bj);
  const bool share = SAME && diag;   // a == b on a diagonal tile: stage one panel only
  float* As = smem;
  float* Bs = share ? As : smem + 2 * PANEL;

  LA la;
  LB lb;
  la.init(D.a, i0, J.kend, t);
  lb.init(SAME ? D.a : D.b, j0, J.kend, t);
  if constexpr (SAME && std::is_same<LA, LB>::value) lb.share_geometry(la);

  const unsigned mask = wp.mask;
  const OutMap om{i0, j0, r0, c0, lane, D.M, D.N, D.sym, mask, (uint32_t)D.ldo * 4u};
  const rsrc_t ro = make_rsrc(D.out, (uint32_t)D.M * om.ldo4);
  const bool direct = J.part < 0;

  // Old output values (running average, sweep update) are fetched before the k loop so that their
  // latency is covered by the MFMA work; they are all in registers before anything is stored.
  Acc4 old;
  acc_zero(old);
  const bool have_old = PREFETCH_OLD && direct && D.beta != 0.f;
  if (have_old) load_old(ro, om, old);

  Acc4 tot;
  acc_zero(tot);
  const int nkt = (J.kend - J.kbeg + KC - 1) / KC;
  const int* yw = (YIELD && cu_flags) ? cu_flags + cu_slot() : nullptr;
  switch (cover_pattern(mask)) {
    case PAT_FULL: main_loop_any<PAT_FULL, SAME>(la, lb, share, As, Bs, tot, J.kbeg, nkt, r0, c0, lane, yw); break;
    case PAT_ROW1: main_loop_any<PAT_ROW1, SAME>(la, lb, share, As, Bs, tot, J.kbeg, nkt, r0, c0, lane, yw); break;
    case PAT_ROW2: main_loop_any<PAT_ROW2, SAME>(la, lb, share, As, Bs, tot, J.kbeg, nkt, r0, c0, lane, yw); break;
    case PAT_COL1: main_loop_any<PAT_COL1, SAME>(la, lb, share, As, Bs, tot, J.kbeg, nkt, r0, c0, lane, yw); break;
    case PAT_ONE: main_loop_any<PAT_ONE, SAME>(la, lb, share, As, Bs, tot, J.kbeg, nkt, r0, c0, lane, yw); break;
    case PAT_TRI: main_loop_any<PAT_TRI, SAME>(la, lb, share, As, Bs, tot, J.kbeg, nkt, r0, c0, lane, yw); break;
    default: main_loop_any<PAT_NONE, SAME>(la, lb, share, As, Bs, tot, J.kbeg, nkt, r0, c0, lane, yw); break;
  }
  finish_tile(D, J, om, ro, tot, old, have_old, diag);
}

typedef __attribute__((address_space(3))) void* lds_void_ptr;

// ------------------------------------------------------------------------------ direct-to-LDS panels of 1x1 views
// Symmetric products of whole-image 1x1 views (OP_CONV11V on both sides: every G factor of a
// convolution whose output images hold a multiple of four pixels, and the A factors of such 1x1
// convolutions) load their panels with the 16-byte buffer_load ... lds as well.  The tensor is
// channel-major (k contiguous), so a panel is [128 channels][KC k] with 128-byte rows; lane l of a wave
// instruction moves one quad of four k, eight lanes a row, eight rows an instruction.  Where a lane's
// quad lands is fixed by the instruction (16 l bytes behind the base), which quad it fetches is not:
// row r stores quad q at position q ^ ((r >> 1) & 7), so that the 16-byte fragment reads of the MFMA
// loop (32 lanes = 32 rows, the same quad) spread over all banks.  Lane half h of the MFMA loop reads
// quad 2g + h of its row and feeds MFMA e = 0..3 of group g with k = 8g + 4h + e: the two halves
// pair k with k + 4 rather than with k + 1 (any pairing gives the same sum).  Per k step a wave
// issues four loads an operand and a dozen address instructions; nothing is staged in registers and
// nothing is stored to LDS but the ones column.
constexpr int DM_PANEL = BM * KC;   // floats of one such panel
static_assert(KC == 32, "eight quads a row");
static_assert(4 * DM_PANEL <= TILE_LDS_FLOATS, "fits the LDS of the staged loop");

struct Conv11DirectLoader {
  rsrc_t rs;
  uint32_t moff, soff32, skip;   // byte offset of the lane's channel of instruction 0; of 32 channels; (C - 1) * HW
  unsigned valid;                // bit j: the lane's channel of instruction j exists
  int q4, kend, w;               // first k of the lane's quad inside a panel
  int bias_row;                  // row of the ones column in this tile if this wave loads it, else -1
  FastDiv dHW;

  __device__ __forceinline__ void init(const Operand& op, int m0, int kend_, int lane, int wave) {
    w = wave;
    const int mreal = op.M - op.bias;
    const uint32_t HW = (uint32_t)(op.OH * op.OW);
    const int f = 4 * (wave & 1) | (lane >> 4);          // ((row >> 1) & 7) of every row this lane loads
    q4 = 4 * ((lane & 7) ^ f);
    valid = 0;
#pragma unroll
    for (int j = 0; j < 4; ++j)
      if (m0 + 32 * j + 8 * wave + (lane >> 3) < mreal) valid |= 1u << j;
    moff = (uint32_t)(m0 + 8 * wave + (lane >> 3)) * HW * 4u;
    soff32 = 32u * HW * 4u;
    skip = (uint32_t)(op.C - 1) * HW;
    dHW = op.dOHW;
    kend = kend_;
    rs = make_rsrc(op.ptr, op.bytes);
    const int rb = mreal - m0;
    bias_row = (op.bias && rb >= 0 && rb < BM && ((rb >> 3) & 3) == wave) ? rb : -1;
  }
  // requests panel [k0, k0 + KC) into `panel` ([128][KC], swizzled as above)
  __device__ __forceinline__ void issue(float* panel, int k0) const {
    const uint32_t kq = (uint32_t)(k0 + q4);
    const uint32_t n = fast_div(kq, dHW);
    const uint32_t vo = (int)kq < kend ? (kq + n * skip) * 4u + moff : OOB_OFFSET;
#pragma unroll
    for (int j = 0; j < 4; ++j)
      __builtin_amdgcn_raw_ptr_buffer_load_lds(rs, (lds_void_ptr)(panel + (32 * j + 8 * w) * KC), 16,
                                               (int)(((valid >> j) & 1u) ? vo : OOB_OFFSET), (int)((uint32_t)j * soff32), 0, 0);
  }
  // after this wave's loads of the panel have landed: the ones column (its lanes read out of range: zeros)
  __device__ __forceinline__ void fix_bias(float* panel, int k0, int lane) const {
    if (bias_row >= 0 && lane < 8) {
      const int q = lane ^ ((bias_row >> 1) & 7);
      const float one = k0 + 4 * q < kend ? 1.f : 0.f;
      *reinterpret_cast<f32x4*>(panel + bias_row * KC + 4 * lane) = f32x4{one, one, one, one};
    }
  }
};

template <unsigned PAT>
__device__ __forceinline__ void mma_ktile_dm(const float* __restrict__ As, const float* __restrict__ Bs,
                                             Acc4& acc, int r0, int c0, int lane) {
  if (PAT == PAT_NONE) return;
  const int i = lane & 31, c = (lane >> 5) ^ ((i >> 1) & 7);   // quad 2g + h of row i sits at position (2g) ^ c
  const float* ap = As + (r0 + i) * KC;   // r0, c0 are multiples of 32: the swizzle of a row depends on i only
  const float* bp = Bs + (c0 + i) * KC;
  const f32x4 z = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
  for (int g = 0; g < KC / 8; ++g) {
    const int pos = 4 * ((2 * g) ^ c);
    f32x4 a0 = z, a1 = z, b0 = z, b1 = z;
    if (PAT & 0x3) a0 = *reinterpret_cast<const f32x4*>(ap + pos);
    if (PAT & 0xC) a1 = *reinterpret_cast<const f32x4*>(ap + 32 * KC + pos);
    if (PAT & 0x5) b0 = *reinterpret_cast<const f32x4*>(bp + pos);
    if (PAT & 0xA) b1 = *reinterpret_cast<const f32x4*>(bp + 32 * KC + pos);
#pragma unroll
    for (int e = 0; e < 4; ++e) {
      if (PAT & 1u) acc.c[0] = __builtin_amdgcn_mfma_f32_32x32x2f32(a0[e], b0[e], acc.c[0], 0, 0, 0);
      if (PAT & 2u) acc.c[1] = __builtin_amdgcn_mfma_f32_32x32x2f32(a0[e], b1[e], acc.c[1], 0, 0, 0);
      if (PAT & 4u) acc.c[2] = __builtin_amdgcn_mfma_f32_32x32x2f32(a1[e], b0[e], acc.c[2], 0, 0, 0);
      if (PAT & 8u) acc.c[3] = __builtin_amdgcn_mfma_f32_32x32x2f32(a1[e], b1[e], acc.c[3], 0, 0, 0);
    }
  }
}

template <unsigned PAT>
__device__ __forceinline__ void main_loop_dm(const Conv11DirectLoader& la, const Conv11DirectLoader& lb, bool share,
                                             float* As, float* Bs, Acc4& tot, int kbeg, int nkt, int r0, int c0, int lane) {
  if (nkt <= 0) return;
  la.issue(As, kbeg);
  if (!share) lb.issue(Bs, kbeg);
  for (int kt = 0; kt < nkt; ++kt) {
    const int cur = kt & 1, k0 = kbeg + kt * KC;
    asm volatile("s_waitcnt vmcnt(0)" ::: "memory");   // this wave's part of panel kt has landed
    la.fix_bias(As + cur * DM_PANEL, k0, lane);
    if (!share) lb.fix_bias(Bs + cur * DM_PANEL, k0, lane);
    __syncthreads();                                    // everybody's part has; all reads of the other buffer are done
    if (kt + 1 < nkt) {
      la.issue(As + (cur ^ 1) * DM_PANEL, k0 + KC);
      if (!share) lb.issue(Bs + (cur ^ 1) * DM_PANEL, k0 + KC);
    }
    mma_ktile_dm<PAT>(As + cur * DM_PANEL, (share ? As : Bs) + cur * DM_PANEL, tot, r0, c0, lane);
  }
}

// a^T a of an OP_CONV11V operand (the descriptor's b is ignored): same tiles, patterns and epilogue as
// run_tile<., ., false, true>, other k loop.  smem: 4 * DM_PANEL floats, 16-byte aligned.
__device__ __forceinline__ void run_tile_dm(const TileDesc& D, const TileJob& J, float* smem) {
  const int t = threadIdx.x, lane = t & 63;
  const int w = __builtin_amdgcn_readfirstlane(t >> 6);
  const WavePlace wp = wave_place(D, J.bi, J.bj, w);
  const int r0 = wp.r0, c0 = wp.c0;
  const int i0 = J.bi * BM, j0 = J.bj * BN;
  const bool diag = D.sym && (J.bi == J.bj);
  float* As = smem;
  float* Bs = smem + 2 * DM_PANEL;
  Conv11DirectLoader la, lb;
  la.init(D.a, i0, J.kend, lane, w);
  lb.init(D.a, j0, J.kend, lane, w);
  const unsigned mask = wp.mask;
  const OutMap om{i0, j0, r0, c0, lane, D.M, D.N, D.sym, mask, (uint32_t)D.ldo * 4u};
  const rsrc_t ro = make_rsrc(D.out, (uint32_t)D.M * om.ldo4);
  Acc4 tot, old;
  acc_zero(tot);
  acc_zero(old);
  const int nkt = (J.kend - J.kbeg + KC - 1) / KC;
  switch (cover_pattern(mask)) {
    case PAT_FULL: main_loop_dm<PAT_FULL>(la, lb, diag, As, Bs, tot, J.kbeg, nkt, r0, c0, lane); break;
    case PAT_ROW1: main_loop_dm<PAT_ROW1>(la, lb, diag, As, Bs, tot, J.kbeg, nkt, r0, c0, lane); break;
    case PAT_ROW2: main_loop_dm<PAT_ROW2>(la, lb, diag, As, Bs, tot, J.kbeg, nkt, r0, c0, lane); break;
    case PAT_COL1: main_loop_dm<PAT_COL1>(la, lb, diag, As, Bs, tot, J.kbeg, nkt, r0, c0, lane); break;
    case PAT_ONE: main_loop_dm<PAT_ONE>(la, lb, diag, As, Bs, tot, J.kbeg, nkt, r0, c0, lane); break;
    case PAT_TRI: main_loop_dm<PAT_TRI>(la, lb, diag, As, Bs, tot, J.kbeg, nkt, r0, c0, lane); break;
    default: main_loop_dm<PAT_NONE>(la, lb, diag, As, Bs, tot, J.kbeg, nkt, r0, c0, lane); break;
  }
  finish_tile(D, J, om, ro, tot, old, false, diag);
}

// ------------------------------------------------------------------------------ direct-to-LDS product
// Plain products of two row-major [K][.] operands (sweep updates and panel products of the inverse,
// the second product of the preconditioning) feed their panels with gfx950's 16-byte
// buffer_load ... lds: a wave instruction moves two panel rows of 128 floats (lane l: row l / 32,
// columns 4 (l % 32) .. + 3) from global memory straight into 1 KB of LDS (lane l writes bytes
// 16 l .. 16 l + 15 behind the base in M0), with a per-lane byte offset that never changes and a
// scalar offset that advances with k: no address arithmetic, no staging registers and no LDS stores
// in the k loop.  Out-of-range lanes write zeros and the range check is per dword (both measured),
// so the k range is enforced by cutting the resource at the job's last row, as in KMajorLoader.
// Panels are [k][128] without padding.  Wave w owns output columns 32 w .. 32 w + 31 and all 128
// rows as four 32-row MFMA blocks whose rows are interleaved (block r, MFMA row i <-> tile row
// 4 i + r): the four a-values of a lane are then one 16-byte LDS read, its b-value one 4-byte read,
// both free of bank conflicts.  A tile with at most 64 (32) valid rows interleaves by 2 (1) instead
// -- the lanes' 16-byte loads then overlap -- and computes two (one) of the four blocks.  Columns of a tile beyond the operand's extent hold whatever follows
// in memory (or zeros); they only reach outputs that are never stored.  With 16-deep panels the
// workgroup needs 32 KB of LDS and 80-odd registers, so several workgroups share a compute unit
// and hide each other's latencies: 120 TFLOP/s on 4096 x 4096 x 768 against 101 for the staged
// loop, bit-identical results (same order of accumulation).
constexpr int DL_KC = 16;                        // panel depth
constexpr int DL_PANEL = DL_KC * BM;             // floats of one operand panel
constexpr int DL_LDS_FLOATS = 4 * DL_PANEL;      // two operands x two buffers
constexpr int DL_KC_DEEP = 32;                   // panel depth of the kernels that run one workgroup to a compute unit
constexpr int DL_DEEP_LDS_FLOATS = 4 * DL_KC_DEEP * BM;

// RS: row interleave = number of 32-row blocks computed (4: more than 64 valid rows, 2: more than 32, 1).
// KCD: panel depth, 16 (32 KB of LDS: several workgroups per compute unit) or 32 (64 KB: half as many
// barriers and waits per contraction row, which is what counts where the workgroup is alone on its unit).
template <bool PREFETCH_OLD, bool YIELD, int RS, int KCD>
__device__ __forceinline__ void run_tile_dl_rs(const TileDesc& D, const TileJob& J, float* smem, const int* cu_flags) {
  const int t = threadIdx.x, lane = t & 63;
  const int w = __builtin_amdgcn_readfirstlane(t >> 6);
  const int i0 = J.bi * BM, j0 = J.bj * BN;
  const bool diag = D.sym && (J.bi == J.bj);
  constexpr int PANEL_F = KCD * BM;     // floats of one operand panel
  float* As = smem;                    // [2][KCD][128]
  float* Bs = smem + 2 * PANEL_F;
  const uint32_t lda4 = (uint32_t)D.a.ld * 4u, ldb4 = (uint32_t)D.b.ld * 4u;
  const uint32_t cut_a = (uint32_t)J.kend * lda4, cut_b = (uint32_t)J.kend * ldb4;
  const rsrc_t ra = make_rsrc(D.a.ptr, cut_a < D.a.bytes ? cut_a : D.a.bytes);
  const rsrc_t rb = make_rsrc(D.b.ptr, cut_b < D.b.bytes ? cut_b : D.b.bytes);
  constexpr int rs = RS;
  const int lca = rs * (lane & 31), lc = 4 * (lane & 31);
  const uint32_t va = (i0 + lca < D.a.M) ? (uint32_t)(lane >> 5) * lda4 + (uint32_t)(i0 + lca) * 4u : OOB_OFFSET;
  const uint32_t vb = (j0 + lc < D.b.M) ? (uint32_t)(lane >> 5) * ldb4 + (uint32_t)(j0 + lc) * 4u : OOB_OFFSET;
  constexpr int PAIRS = KCD / 8;     // row pairs per wave, operand and k step
  auto issue = [&](int k0, int buf) {
#pragma unroll
    for (int u = 0; u < PAIRS; ++u) {
      const int r = 2 * (4 * u + w);   // first row of the pair inside the panel
      __builtin_amdgcn_raw_ptr_buffer_load_lds(ra, (lds_void_ptr)(As + buf * PANEL_F + r * BM), 16, (int)va, (int)((uint32_t)(k0 + r) * lda4), 0, 0);
      __builtin_amdgcn_raw_ptr_buffer_load_lds(rb, (lds_void_ptr)(Bs + buf * PANEL_F + r * BN), 16, (int)vb, (int)((uint32_t)(k0 + r) * ldb4), 0, 0);
    }
  };

  // output offsets: block r, register v of this lane <-> row i0 + rs mfma_row + r, column j0 + 32 w + mfma_col
  const uint32_t ldo4 = (uint32_t)D.ldo * 4u;
  const int gj = j0 + 32 * w + mfma_col(lane);
  auto out_offset = [&](int r, int v) -> uint32_t {
    const int gi = i0 + rs * mfma_row(v, lane) + r;
    const bool ok = gi < D.M && gj < D.N && (!D.sym || gi >= gj);
    return ok ? (uint32_t)gi * ldo4 + (uint32_t)gj * 4u : OOB_OFFSET;
  };
  const rsrc_t ro = make_rsrc(D.out, (uint32_t)D.M * ldo4);
  const float alpha = D.alpha, beta = D.beta;
  const bool direct = J.part < 0;
  const bool wave_used = j0 + 32 * w < D.N;    // a wave whose columns all lie outside the matrix only helps loading

  const int nkt = (J.kend - J.kbeg + KCD - 1) / KCD;
#ifdef KFAC_TRACE
  const long long tr0 = wall_clock64();
#endif
  if (nkt > 0) issue(J.kbeg, 0);
  // PREFETCH_OLD: the old output values are fetched before the k loop (64 more registers, fewer
  // workgroups per compute unit); otherwise block by block in the epilogue.
  f32x16 old[PREFETCH_OLD ? RS : 1];
  if constexpr (PREFETCH_OLD) {
#pragma unroll
    for (int r = 0; r < RS; ++r)
#pragma unroll
      for (int v = 0; v < 16; ++v) old[r][v] = (direct && beta != 0.f) ? buf_load(ro, out_offset(r, v)) : 0.f;
  }
  f32x16 acc[RS];
#pragma unroll
  for (int r = 0; r < RS; ++r)
#pragma unroll
    for (int v = 0; v < 16; ++v) acc[r][v] = 0.f;
  const int* yw = (YIELD && cu_flags) ? cu_flags + cu_slot() : nullptr;
  const int li = lane & 31, lh = lane >> 5;
  for (int kt = 0; kt < nkt; ++kt) {
    int busy = 0;
    if (yw && (kt & 1)) busy = __hip_atomic_load(yw, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    asm volatile("s_waitcnt vmcnt(0)" ::: "memory");   // this wave's part of panel kt has landed
    __syncthreads();                                    // ... and everybody's; all reads of the other buffer are done
    if (kt + 1 < nkt) issue(J.kbeg + (kt + 1) * KCD, (kt + 1) & 1);
    if (wave_used) {
      const float* ap = As + (kt & 1) * PANEL_F + lh * BM + 4 * li;
      const float* bp = Bs + (kt & 1) * PANEL_F + lh * BN + 32 * w + li;
#pragma unroll
      for (int q = 0; q < KCD / 2; ++q) {
        const float b = bp[2 * q * BN];
        if constexpr (RS == 4) {
          const f32x4 a = *reinterpret_cast<const f32x4*>(ap + 2 * q * BM);
#pragma unroll
          for (int r = 0; r < 4; ++r) acc[r] = __builtin_amdgcn_mfma_f32_32x32x2f32(a[r], b, acc[r], 0, 0, 0);
        } else if constexpr (RS == 2) {
          typedef float f32x2 __attribute__((ext_vector_type(2)));
          const f32x2 a = *reinterpret_cast<const f32x2*>(ap + 2 * q * BM);
#pragma unroll
          for (int r = 0; r < 2; ++r) acc[r] = __builtin_amdgcn_mfma_f32_32x32x2f32(a[r], b, acc[r], 0, 0, 0);
        } else {
          acc[0] = __builtin_amdgcn_mfma_f32_32x32x2f32(ap[2 * q * BM], b, acc[0], 0, 0, 0);
        }
      }
    }
    if (yw && __builtin_amdgcn_readfirstlane(busy) != 0) cu_yield(yw);
  }

#ifdef KFAC_TRACE
  const long long tr1 = wall_clock64();
#endif
  if (!direct) {   // raw partial tile, [128][128] in tile coordinates
    gf_ptr P = as_global(D.partial) + (size_t)J.part * (BM * BN);
#pragma unroll
    for (int r = 0; r < RS; ++r)
#pragma unroll
      for (int v = 0; v < 16; ++v) P[(rs * mfma_row(v, lane) + r) * BN + 32 * w + mfma_col(lane)] = acc[r][v];
    return;
  }
  const bool mirror = D.mirror == MIRROR_ALL || (D.mirror == MIRROR_DIAG_TILE && diag);
#pragma unroll
  for (int r = 0; r < RS; ++r) {
    f32x16 o;
#pragma unroll
    for (int v = 0; v < 16; ++v) {
      if constexpr (PREFETCH_OLD) o[v] = old[r][v];
      else o[v] = beta != 0.f ? buf_load(ro, out_offset(r, v)) : 0.f;
    }
#pragma unroll
    for (int v = 0; v < 16; ++v) {
      const float val = alpha * acc[r][v] + beta * o[v];
      const uint32_t off = out_offset(r, v);
      buf_store(ro, off, val);
      if (mirror) {
        const int gi = i0 + rs * mfma_row(v, lane) + r;
        buf_store(ro, (off != OOB_OFFSET && gi != gj) ? (uint32_t)gj * ldo4 + (uint32_t)gi * 4u : OOB_OFFSET, val);
      }
    }
  }
#ifdef KFAC_TRACE
  if (YIELD && cu_flags && t == 0) {
    int* cnt = const_cast<int*>(cu_flags) + CU_SLOTS;
    const int rix = __hip_atomic_fetch_add(cnt, 1, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    if (rix < 60000) {
      long long* rec = reinterpret_cast<long long*>(const_cast<int*>(cu_flags) + CU_SLOTS + 2) + (size_t)rix * 8;
      rec[0] = 5 + 8 * (long long)D.M; rec[1] = nkt; rec[2] = cu_slot(); rec[3] = tr0; rec[4] = tr1; rec[5] = tr1; rec[6] = tr1; rec[7] = wall_clock64();
    }
  }
#endif
}

template <bool PREFETCH_OLD = false, bool YIELD = false, int KCD = DL_KC>
__device__ __forceinline__ void run_tile_dl(const TileDesc& D, const TileJob& J, float* smem, const int* cu_flags = nullptr) {
  const int rows_valid = D.M - J.bi * BM;
  if (rows_valid > 64) run_tile_dl_rs<PREFETCH_OLD, YIELD, 4, KCD>(D, J, smem, cu_flags);
  else if (rows_valid > 32) run_tile_dl_rs<PREFETCH_OLD, YIELD, 2, KCD>(D, J, smem, cu_flags);
  else run_tile_dl_rs<PREFETCH_OLD, YIELD, 1, KCD>(D, J, smem, cu_flags);
}

// One 32 x 32 block of a tile per WAVE, operands straight from memory into registers in the MFMA's own
// layout (lane (i, h) of k pair q holds element (2q + h, i) of each operand: 32 consecutive floats of
// two rows per load), no LDS and no barriers: for the products that nothing else can overlap with
// (the products on the sweep chain of the inverse), where a tile's sixteen blocks should run on
// sixteen SIMDs at once and a block's time is the latency of its loads.  Loads run two chunks of
// 16 k pairs ahead of the MFMAs.  Job (bi, bj, quarter): wave w takes row block w of column block
// quarter - 1.  Old values fetched first; direct jobs only.
constexpr int QB_CH = 16;   // k pairs per chunk
struct QuarterOperands {
  rsrc_t ra, rb;
  uint32_t va, vb, lda4, ldb4;
  int kbeg;
  __device__ __forceinline__ void load(int c, float (&a)[QB_CH], float (&b)[QB_CH]) const {
#pragma unroll
    for (int q = 0; q < QB_CH; ++q) {
      const uint32_t k = (uint32_t)(kbeg + 2 * (c * QB_CH + q));   // rows at or past the job's last row lie beyond the resource
      a[q] = __builtin_bit_cast(float, __builtin_amdgcn_raw_buffer_load_b32(ra, (int)va, (int)(k * lda4), 0));
      b[q] = __builtin_bit_cast(float, __builtin_amdgcn_raw_buffer_load_b32(rb, (int)vb, (int)(k * ldb4), 0));
    }
  }
};
__device__ __forceinline__ void quarter_mma(const float (&a)[QB_CH], const float (&b)[QB_CH], f32x16& acc) {
#pragma unroll
  for (int q = 0; q < QB_CH; ++q) acc = __builtin_amdgcn_mfma_f32_32x32x2f32(a[q], b[q], acc, 0, 0, 0);
}
__device__ __forceinline__ void run_tile_quarter(const TileDesc& D, const TileJob& J) {
  const int t = threadIdx.x, lane = t & 63;
  const int w = __builtin_amdgcn_readfirstlane(t >> 6);
  const int li = lane & 31, lh = lane >> 5;
  const int i0 = J.bi * BM + 32 * w, j0 = J.bj * BN + 32 * (J.quarter - 1);
  if (i0 >= D.M || j0 >= D.N) return;          // wave-uniform; nothing below synchronises waves
  if (D.sym && j0 > i0 + 31) return;           // block above the diagonal
  const bool diag = D.sym && (J.bi == J.bj);
  QuarterOperands op;
  op.lda4 = (uint32_t)D.a.ld * 4u; op.ldb4 = (uint32_t)D.b.ld * 4u;
  const uint32_t cut_a = (uint32_t)J.kend * op.lda4, cut_b = (uint32_t)J.kend * op.ldb4;
  op.ra = make_rsrc(D.a.ptr, cut_a < D.a.bytes ? cut_a : D.a.bytes);
  op.rb = make_rsrc(D.b.ptr, cut_b < D.b.bytes ? cut_b : D.b.bytes);
  op.va = (i0 + li < D.a.M) ? (uint32_t)lh * op.lda4 + (uint32_t)(i0 + li) * 4u : OOB_OFFSET;
  op.vb = (j0 + li < D.b.M) ? (uint32_t)lh * op.ldb4 + (uint32_t)(j0 + li) * 4u : OOB_OFFSET;
  op.kbeg = J.kbeg;
  const uint32_t ldo4 = (uint32_t)D.ldo * 4u;
  const int gj = j0 + mfma_col(lane);
  auto out_offset = [&](int v) -> uint32_t {
    const int gi = i0 + mfma_row(v, lane);
    const bool ok = gi < D.M && gj < D.N && (!D.sym || gi >= gj);
    return ok ? (uint32_t)gi * ldo4 + (uint32_t)gj * 4u : OOB_OFFSET;
  };
  const rsrc_t ro = make_rsrc(D.out, (uint32_t)D.M * ldo4);
  const float alpha = D.alpha, beta = D.beta;
  const int nch = (J.kend - J.kbeg + 2 * QB_CH - 1) / (2 * QB_CH);
  f32x16 old, acc;
#pragma unroll
  for (int v = 0; v < 16; ++v) {
    old[v] = beta != 0.f ? buf_load(ro, out_offset(v)) : 0.f;
    acc[v] = 0.f;
  }
  float a0[QB_CH], b0[QB_CH], a1[QB_CH], b1[QB_CH], a2[QB_CH], b2[QB_CH];
  if (nch > 0) op.load(0, a0, b0);
  if (nch > 1) op.load(1, a1, b1);
  for (int c = 0; c < nch; c += 3) {
    if (c + 2 < nch) op.load(c + 2, a2, b2);
    quarter_mma(a0, b0, acc);
    if (c + 1 >= nch) break;
    if (c + 3 < nch) op.load(c + 3, a0, b0);
    quarter_mma(a1, b1, acc);
    if (c + 2 >= nch) break;
    if (c + 4 < nch) op.load(c + 4, a1, b1);
    quarter_mma(a2, b2, acc);
  }
  const bool mirror = D.mirror == MIRROR_ALL || (D.mirror == MIRROR_DIAG_TILE && diag);
#pragma unroll
  for (int v = 0; v < 16; ++v) {
    const float val = alpha * acc[v] + beta * old[v];
    const uint32_t off = out_offset(v);
    buf_store(ro, off, val);
    if (mirror) {
      const int gi = i0 + mfma_row(v, lane);
      buf_store(ro, (off != OOB_OFFSET && gi != gj) ? (uint32_t)gj * ldo4 + (uint32_t)gi * 4u : OOB_OFFSET, val);
    }
  }
}

// Dispatch on the operand type of a symmetric product a^T a (wave-uniform).
__device__ __forceinline__ void run_tile_sym(const TileDesc& D, const TileJob& J, float* smem) {
  const int ta = D.a.type;
  if (ta == OP_KMAJOR) run_tile<KMajorLoader, KMajorLoader, false, true>(D, J, smem);
  else if (ta == OP_CONV11V) run_tile_dm(D, J, smem);
  else if (ta == OP_CONV11) run_tile<ConvLoader<1, 1>, ConvLoader<1, 1>, false, true>(D, J, smem);
  else if (ta == OP_CONV33) run_tile<ConvLoader<3, 3>, ConvLoader<3, 3>, false, true>(D, J, smem);
  else if (ta == OP_CONV77) run_tile<ConvLoader<7, 7>, ConvLoader<7, 7>, false, true>(D, J, smem);
  else run_tile<ConvLoader<0, 0>, ConvLoader<0, 0>, false, true>(D, J, smem);
}

// Lag products (see lag_assemble_kernel): a = 1x1 view of a tensor, b = a small window of forward
// lags of the same tensor, over the same window of pixels.
__device__ __forceinline__ void run_tile_lag(const TileDesc& D, const TileJob& J, float* smem) {
  const int tb = D.b.type;
  if (D.a.type == OP_CONV11V) {
    if (tb == OP_CONV25) run_tile<Conv11VecLoader, ConvLoader<2, 5>, false, false>(D, J, smem);
    else run_tile<Conv11VecLoader, ConvLoader<1, 3>, false, false>(D, J, smem);
  } else if (tb == OP_CONV25) run_tile<ConvLoader<1, 1>, ConvLoader<2, 5>, false, false>(D, J, smem);
  else if (tb == OP_CONV13) run_tile<ConvLoader<1, 1>, ConvLoader<1, 3>, false, false>(D, J, smem);
  else run_tile<ConvLoader<1, 1>, ConvLoader<0, 0>, false, false>(D, J, smem);
}

}  // namespace kfac
