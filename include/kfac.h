/*
 * kfac.h -- C ABI of the MI355X (gfx950) K-FAC hot path.
 *
 * The library computes, for one data-parallel worker, the three per-iteration
 * K-FAC operations of Shi, Zhang, Li, "Accelerating Distributed K-FAC with Smart
 * Parallelism of Computing and Communication Tasks" (arXiv 2107.06533):
 *
 *   kfac_update_factors   Kronecker factors A = a a^T, G = g g^T   (Sec. II-B,
 *                         Eq. factorA / Eq. factorG), batch-averaged and folded
 *                         into a running average;
 *   kfac_invert_batch     f(T_i) = (T_i + gamma I)^-1 applied to a whole set of
 *                         symmetric tensors T_i in R^{d_i x d_i} (Sec. II-B damped
 *                         update rule; problem statement of Sec. IV-B);
 *   kfac_precondition     (A+gamma I)^-1 (x) (G+gamma I)^-1 applied to a layer's
 *                         gradient (Eq. kfacfinal), i.e.  G^-1 . V . A^-1.
 *
 * Conventions shared by every call
 *   - All DATA pointers are DEVICE pointers to fp32 buffers owned by the caller.
 *     The pointer ARRAYS (float* const*), the layer/dims arrays and every scalar
 *     are HOST memory; they are copied during the call and may be freed on return.
 *   - Matrices are dense row-major with leading dimension = number of columns.
 *   - Calls are asynchronous on `hip_stream` (a hipStream_t passed as void*, NULL
 *     = the default stream).  Calls on one context must be issued in stream
 *     order; a context is not thread-safe.
 *   - The context owns a device workspace that grows on demand (hipMalloc at the
 *     first call that needs more; query with kfac_workspace_bytes_*).
 *   - Errors are returned, never thrown.  Arguments are validated on the host
 *     before anything is launched; kfac_last_error() describes the last failure.
 *   - Arithmetic is fp32 throughout (fp32 MFMA, fp32 accumulation).
 *   - Limits (checked, KFAC_ERR_INVALID_ARG): every activation / gradient tensor holds at
 *     most 2^28 elements (1 GiB; operands are addressed with 32-bit byte offsets), convolution
 *     windows have at most 63 taps, every factor dimension (dA, dG, the d of a matrix to invert or
 *     to precondition with) is at most 16384.
 *   - kfac_invert_batch also launches on internal streams of the context (default priority),
 *     forked from and joined back into `hip_stream` with events before the call returns; the
 *     work is complete when `hip_stream` is.  The first call for a new set of shapes builds and
 *     uploads a schedule (it synchronises the device once); later calls with the same shapes only
 *     refresh a small pointer table.
 *   - Activation factors of 3x3 / stride 1 / pad 1 convolutions with >= 64 input channels are
 *     summed in a different order than the patch-matrix product (products over pixel lags,
 *     then assembled); the result is the same sum up to fp32 rounding.
 */
#ifndef KFAC_H_
#define KFAC_H_

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum {
  KFAC_OK = 0,
  KFAC_ERR_INVALID_ARG = 1, /* rejected on the host, nothing was launched        */
  KFAC_ERR_NOT_SPD = 2,     /* reported by kfac_check_info                        */
  KFAC_ERR_WORKSPACE = 3,   /* device workspace could not be (re)allocated        */
  KFAC_ERR_DEVICE = 4       /* HIP error, or a host-only context asked to launch  */
} kfac_status;

typedef struct kfac_ctx kfac_ctx; /* opaque: workspace + cached schedules only */

/* One preconditioned layer (one factor pair). */
typedef struct {
  int32_t kind;     /* 0 linear : act [rows, c_in],   gout [rows, c_out]   row-major
                       1 conv2d : act [n, c_in, h, w], gout [n, c_out, oh, ow] NCHW, dilation 1, groups 1 */
  int32_t n, c_in, h, w, c_out, kh, kw, stride, pad_h, pad_w; /* n,h,w,kh,kw,stride,pad_*: conv only;
                       zero padding of the height / of the width (they differ for 1x7-style windows) */
  int32_t rows;     /* linear only; a convolution has rows = n*oh*ow */
  int32_t has_bias; /* 1: a ones column is appended LAST to the activations,
                          dA = c_in*kh*kw + has_bias                           */
} kfac_layer;

/* Create a context on HIP device `device` (>= 0).  device = -1 creates a host-only
 * context: every call still validates its arguments and builds its schedule, then
 * returns KFAC_ERR_DEVICE instead of launching (used by CPU-only tests). */
kfac_status kfac_create(kfac_ctx** out, int device);
void kfac_destroy(kfac_ctx* ctx);
const char* kfac_last_error(const kfac_ctx* ctx); /* never NULL; ctx may be NULL */

/*
 * Tuning options of a context.  They change how the work is scheduled (launch structure, summation
 * order inside the stated tolerances), never what is computed; the defaults are the measured best on
 * the benchmark workloads.  A context reads no environment variable.  Setting an option discards the
 * cached schedules of the context (the next call of each kind plans again); set options between
 * calls, not while work of this context is in flight.
 * Returns INVALID_ARG for a NULL ctx, an unknown option or a value outside the stated range.
 */
typedef enum {
  KFAC_OPT_INV_GROUPS = 0,    /* 1..4   [2]     groups of matrices kfac_invert_batch sweeps concurrently           */
  KFAC_OPT_INV_AGG = 1,       /* 1..16  [4]     pivot blocks per outer block, throughput-bound group               */
  KFAC_OPT_INV_AGG_CHAIN = 2, /* 1..16  [6]     the same for a group bound by its chain of dependent launches      */
  KFAC_OPT_INV_FUSE = 3,      /* 0/1    [1]     pivot block applies the previous block's update to itself          */
  KFAC_OPT_INV_SIDE_PAD = 4,  /* 0..65536 [56000] bytes of LDS beyond 32 KB held by off-chain products (occupancy)      */
  KFAC_OPT_FACTOR_LAG = 5,    /* 0/1    [1]     3x3/stride 1/pad 1 activation factors from products over pixel lags */
  KFAC_OPT_FACTOR_VEC11 = 6,  /* 0/1    [1]     128-bit loads for 1x1 windows over whole images                    */
  KFAC_OPT_FACTOR_XCD = 7,    /* 0/1    [0]     factor jobs dealt to the 8 XCDs in contiguous segments             */
  KFAC_OPT_FACTOR_KJOB = 8,   /* 32..8192 [8192] longest run of rows one factor tile job accumulates               */
  KFAC_OPT_INV_CHAIN_PAD = 9, /* 0..65536 [0]   bytes of unused LDS added to the chain kernels of such a group              */
  KFAC_OPT_INV_SIDE = 10,     /* 0/1    [1]     off-chain work of a group on a second internal stream                  */
  KFAC_OPT_INV_SPLIT_LONG = 11, /* 0/1  [1]     the matrices with the longest chains form a group of their own         */
  KFAC_OPT_INV_YIELD = 12,    /* 0..65536 [64] sweep-chain kernels of at most this many workgroups make products give way   */
  KFAC_OPT_INV_QUARTER = 13,  /* 0/1    [1]     products on the sweep chain of the inverse on quarter tiles (four workgroups a tile) */
  KFAC_OPT_COUNT = 14
} kfac_option;
kfac_status kfac_set_option(kfac_ctx* ctx, int option, int value);
kfac_status kfac_get_option(const kfac_ctx* ctx, int option, int* value);

/* Factor dimensions implied by a layer (pure host). Return 0 for an invalid layer. */
int32_t kfac_layer_dA(const kfac_layer* layer);
int32_t kfac_layer_dG(const kfac_layer* layer);
int64_t kfac_layer_rows(const kfac_layer* layer);

/* Workspace each call needs for the given shapes (pure host; 0 on invalid input). */
size_t kfac_workspace_bytes_factors(const kfac_ctx* ctx, int n_layers, const kfac_layer* layers);
size_t kfac_workspace_bytes_invert(const kfac_ctx* ctx, int n_mats, const int32_t* dims);
size_t kfac_workspace_bytes_precondition(const kfac_ctx* ctx, int n_layers, const int32_t* dG, const int32_t* dA);

/*
 * Factor build with running average (Sec. II-B, Eq. factorA, Eq. factorG).
 * For every layer l:
 *     a-bar = [patches(act_l), 1]   [R, dA]  (patch expansion fused, never materialised;
 *                                              column q = (c*kh + i)*kw + j, ones column last)
 *     A_l <- xi * A_l + (1 - xi) * scale_a * a-bar^T a-bar
 *     G_l <- xi * G_l + (1 - xi) * scale_g * g-bar^T g-bar     g-bar [R, dG], one row per sample / output pixel
 * scale_a, scale_g <= 0 select the default 1/R (R = rows of a-bar).
 * act, gout: host arrays of n_layers device pointers; an array, or single entries,
 *     may be NULL to skip that factor (then the matching A / G entry is ignored).
 * A, G: in/out device matrices [dA,dA] / [dG,dG]; the result is written full and
 *     exactly symmetric.  Only the lower triangle of the old value is read.
 * Returns INVALID_ARG for: NULL ctx/layers, n_layers < 0, a malformed layer (non-positive
 * dimension, empty output, kind not 0/1, has_bias not 0/1), xi outside [0,1] or NaN, a
 * non-NULL act/gout entry whose factor pointer is NULL.  n_layers == 0 is a no-op.
 */
kfac_status kfac_update_factors(kfac_ctx* ctx, int n_layers, const kfac_layer* layers,
                                const float* const* act, const float* const* gout,
                                float* const* A, float* const* G,
                                float xi, float scale_a, float scale_g, void* hip_stream);

/*
 * The same call with a second output (Sec. IV-A: a worker communicates d(d+1)/2 elements per
 * symmetric factor; Sec. V-B: the upper triangle including the diagonal): `packed` (device buffer)
 * receives the packed upper triangles of the updated factors, all A_l in layer order followed by all
 * G_l -- the layout kfac_pack_triangles produces for the matrix list (A_0 .. A_{n-1}, G_0 .. G_{n-1}),
 * kfac_packed_elems over (dA_0 .. dA_{n-1}, dG_0 .. dG_{n-1}) floats -- written by the kernels that
 * write the factors, bit-identical to packing them afterwards.  The segment of a factor that is
 * skipped (NULL act / gout entry) is left untouched.  packed must not be NULL.
 */
kfac_status kfac_update_factors_packed(kfac_ctx* ctx, int n_layers, const kfac_layer* layers,
                                       const float* const* act, const float* const* gout,
                                       float* const* A, float* const* G,
                                       float xi, float scale_a, float scale_g, float* packed, void* hip_stream);

/*
 * Damped inverse of a heterogeneous set of symmetric positive-definite matrices
 * (Sec. II-B: Tikhonov term gamma I added before inverting; Sec. IV-B: N tensors
 * T_i in R^{d_i x d_i}, the same f applied to each):
 *     X_i = (F_i + gamma I)^-1,   i = 0 .. n_mats-1.
 * dims: host array of d_i >= 1.  F, X: host arrays of device pointers, [d_i, d_i];
 * only the lower triangle of F_i is read; X_i is written full and exactly symmetric;
 * X_i must not alias F_i (F_i is left untouched).
 * info_dev: optional DEVICE array of n_mats int32 (may be NULL).  Entry i is set to 0
 *     on success or to k > 0 when the leading minor of order k of F_i + gamma I is not
 *     positive (LAPACK convention); X_i is then unspecified, other matrices are still
 *     valid.  Read it after the stream has finished, e.g. with kfac_check_info.
 * Accuracy: the sweep runs in fp32 without pivoting, so the residual
 *     r = ||(F + gamma I) X - I||_F / sqrt(d)   grows with  kappa = cond(F + gamma I);
 *     measured on MI355X (d = 1153, eigenvalues log-spaced between 1 and kappa, the hardest spectrum):
 *     r = 9e-6 at kappa 1e2, 4e-5 at 3e2, 2.4e-4 at 1e3, 8.5e-3 at 1e4, below 4 kappa^1.75 2^-24 throughout.
 *     The bar r <= 1e-4 therefore holds for arbitrary spectra up to kappa = 3e2; K-FAC factors in steady state
 *     (a few large eigenvalues over a bulk near gamma) stay within it up to kappa of about 1e3 (1.4e-5 at
 *     kappa 914).  Past that, info stays 0 and r follows the envelope: raise gamma, or invert in fp64.
 * Returns INVALID_ARG for: NULL ctx/dims/F/X, n_mats < 0, d_i < 1, NULL or aliased
 * entries, gamma negative or NaN.  n_mats == 0 is a no-op.
 */
kfac_status kfac_invert_batch(kfac_ctx* ctx, int n_mats, const int32_t* dims,
                              const float* const* F, float* const* X,
                              float gamma, int32_t* info_dev, void* hip_stream);

/*
 * The same call with a second output: `packed` (device buffer of kfac_packed_elems(n_mats, dims)
 * floats, owned by the caller) receives the packed upper triangles of the inverses, in the layout of
 * kfac_pack_triangles (the form in which the paper sends an inverse to the other workers, Sec. V-B),
 * written by the kernels that write X_i: bit-identical to kfac_pack_triangles applied to X afterwards,
 * without the extra pass.  INVALID_ARG additionally for packed == NULL.
 */
kfac_status kfac_invert_batch_packed(kfac_ctx* ctx, int n_mats, const int32_t* dims,
                                     const float* const* F, float* const* X, float* packed,
                                     float gamma, int32_t* info_dev, void* hip_stream);

/* Synchronise `hip_stream`, copy info_dev[0..n) to info_host (may be NULL) and return
 * KFAC_ERR_NOT_SPD if any entry is non-zero, else KFAC_OK. */
kfac_status kfac_check_info(kfac_ctx* ctx, int n, const int32_t* info_dev, int32_t* info_host,
                            void* hip_stream);

/*
 * Two-sided preconditioning (Eq. kfacfinal with the inverses already formed):
 *     out_l = Ginv_l . gradW_l . Ainv_l        gradW_l, out_l : [dG_l, dA_l]
 * gradW_l is the layer's weight gradient flattened to [C_out, C_in*kh*kw] with the bias
 * gradient as last column when the layer has a bias.  Ginv_l [dG,dG], Ainv_l [dA,dA] are
 * used as stored (full matrices; they are symmetric when produced by kfac_invert_batch).
 * out_l may alias gradW_l; it must not alias the inverses.
 * Returns INVALID_ARG for NULL arrays/entries, n_layers < 0, non-positive dimensions.
 */
kfac_status kfac_precondition(kfac_ctx* ctx, int n_layers, const int32_t* dG, const int32_t* dA,
                              const float* const* Ginv, const float* const* Ainv,
                              const float* const* gradW, float* const* out, void* hip_stream);

/*
 * kfac_precondition for callers that cannot allocate device memory: code under HIP graph capture,
 * tight serving loops, harnesses that forbid hipMalloc.  Same arguments, same result (bit for bit),
 * but the call allocates nothing: descriptors, job lists and the intermediate Ginv . V live in one
 * static device array of KFAC_NOALLOC_SCRATCH_BYTES that every GPU the library runs on holds until the
 * process ends, and the call consists of three kernel launches on hip_stream (no copies, no memsets).
 * Limits per call (INVALID_ARG beyond them, with the figures in kfac_last_error): at most
 * KFAC_NOALLOC_MAX_LAYERS layers, KFAC_NOALLOC_MAX_ELEMS gradient elements (sum of dG*dA) and
 * KFAC_NOALLOC_MAX_TILES 128 x 128 output tiles (sum of ceil(dG/128)*ceil(dA/128)) over all layers.
 * All calls on one GPU share that GPU's array: two calls that overlap in time on one GPU (different
 * streams, different contexts or threads) race; issue them in one stream, or order them with events.
 * Nothing in the array has to start at zero, and nothing is kept between calls.
 */
#define KFAC_NOALLOC_MAX_LAYERS 32
#define KFAC_NOALLOC_MAX_ELEMS (7u << 20)
#define KFAC_NOALLOC_MAX_TILES 8192
#define KFAC_NOALLOC_SCRATCH_BYTES ((size_t)30 << 20) /* upper bound: tables (< 1 MiB) + 28 MiB of intermediates */
kfac_status kfac_precondition_noalloc(kfac_ctx* ctx, int n_layers, const int32_t* dG, const int32_t* dA,
                                      const float* const* Ginv, const float* const* Ainv,
                                      const float* const* gradW, float* const* out, void* hip_stream);

/*
 * Packed upper triangles: the form in which the paper communicates symmetric factors and
 * inverses between workers (Sec. IV-A: d(d+1)/2 communicated elements per factor; Sec. V-B: the
 * upper triangle including the diagonal).  The triangles of the n matrices are concatenated in one
 * device buffer, matrix after matrix, each row after row:
 *     packed[off_m + i*d - i*(i-1)/2 + (j - i)] = M_m[i][j],   0 <= i <= j < d_m.
 * kfac_packed_elems returns the total number of floats (0 on invalid input) and, if `offsets` is
 * not NULL, writes the n+1 float offsets off_0 .. off_n (host memory; pure host).
 * kfac_pack_triangles   reads only the upper triangle of every M_m (device, [d,d] row-major).
 * kfac_unpack_triangles writes every M_m full and exactly symmetric.
 * dims: host array, 1 <= d <= 46340.  M: host array of device pointers.  packed: device buffer of
 * kfac_packed_elems floats, owned by the caller.  Asynchronous on hip_stream.
 * Returns INVALID_ARG for NULL ctx/dims/M/packed, n_mats < 0, dims out of range, NULL entries.
 * n_mats == 0 is a no-op.
 */
size_t kfac_packed_elems(int n_mats, const int32_t* dims, int64_t* offsets);
kfac_status kfac_pack_triangles(kfac_ctx* ctx, int n_mats, const int32_t* dims, const float* const* M,
                                float* packed, void* hip_stream);
kfac_status kfac_unpack_triangles(kfac_ctx* ctx, int n_mats, const int32_t* dims, const float* packed,
                                  float* const* M, void* hip_stream);

/*
 * Load-balancing placement of the inversions on several workers (Sec. IV-B, Algorithm 1) with
 * the paper's two cost models; pure host, no context needed.
 *     t_comp(d) = alpha_inv * exp(beta_inv * d)              (Eq. inverting-model)
 *     t_comm(d) = alpha_bcast + beta_bcast * d (d + 1) / 2   (Eq. broadcast-model)
 * Tensors are visited in descending dimension (ties in input order).  One whose inverse is cheaper
 * to compute than to receive (t_comp < t_comm) is computed by every worker and not communicated:
 * owner[i] = -1, and every worker's bucket grows.  Otherwise it goes to the worker with the smallest
 * bucket (lowest index on ties): owner[i] = that worker.  A bucket grows by d ** weight_power
 * (1: as the algorithm is printed; 2: as the text describes the balance; 3: proportional to the
 * arithmetic of the inverse).
 * overall_time (may be NULL) receives the objective of the problem statement: the maximum over
 * workers of the summed t_comp of its tensors plus the summed t_comm of those it has to send.
 * Returns INVALID_ARG for NULL dims/model/owner, n_mats < 0, n_workers < 1, d < 1,
 * weight_power outside 1..3, negative or non-finite coefficients.  n_mats == 0 is a no-op.
 */
typedef struct {
  double alpha_inv, beta_inv;
  double alpha_bcast, beta_bcast;
  int32_t weight_power;
} kfac_cost_model;
kfac_status kfac_place_inversions(int n_mats, const int32_t* dims, int n_workers, const kfac_cost_model* model,
                                  int32_t* owner, double* overall_time);

/* Schedule statistics of the most recent call of each kind on this context (pure host;
 * for tests and benchmarks).  Fields that do not apply are 0. */
typedef struct {
  int64_t n_jobs;      /* tile jobs launched (all kernels of the call)          */
  int64_t n_launches;  /* kernel launches the call enqueues                     */
  int64_t n_split;     /* factors: tiles whose reduction is split along R       */
  int64_t mfma_flops;  /* flops the tile jobs execute (tile granularity)        */
  int64_t ws_bytes;    /* workspace the call uses                               */
} kfac_plan_stats;
void kfac_get_plan_stats(const kfac_ctx* ctx, int which /*0 factors, 1 invert, 2 precondition*/,
                         kfac_plan_stats* out);

/*
 * Optional per-kernel timing for benchmarks.  While bit k of `class_mask` is set, every launch of
 * kernel class k is bracketed by a pair of HIP events on the call's stream.  kfac_timing_read
 * waits for the recorded events, returns the summed duration and launch count of one class and,
 * if `reset` is non-zero, forgets that class's records.  Timing is off by default (mask 0).
 */
enum {
  KFAC_K_FACTOR_TILES = 0,  /* grouped factor build (patch expansion + MFMA + running average) */
  KFAC_K_FACTOR_REDUCE = 1, /* reduction of tiles whose row range was split                   */
  KFAC_K_INV_SMALL = 2,     /* whole-matrix in-register inverse, d <= 128                      */
  KFAC_K_INV_INIT = 3,
  KFAC_K_INV_PIVOT = 4,
  KFAC_K_INV_PANEL = 5,
  KFAC_K_INV_UPDATE = 6,    /* rank-128 MFMA update of the lower triangle                      */
  KFAC_K_INV_FINISH = 7,
  KFAC_K_PRECOND_LEFT = 8,  /* Ginv . V                                                        */
  KFAC_K_PRECOND_RIGHT = 9, /* (Ginv . V) . Ainv                                               */
  KFAC_K_TRI_PACK = 10,     /* packed upper triangles <-> full matrices                        */
  KFAC_K_COUNT = 11
};
void kfac_timing_enable(kfac_ctx* ctx, uint32_t class_mask);
kfac_status kfac_timing_read(kfac_ctx* ctx, int kclass, double* total_ms, int64_t* n_launches, int reset);

#ifdef __cplusplus
}
#endif
#endif /* KFAC_H_ */
