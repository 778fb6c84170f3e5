// C ABI of the K-FAC hot path: argument validation, schedule construction (host only) and
// kernel launches.  Everything that decides WHAT runs is here; the arithmetic is in the kernels.
#include "../../include/kfac.h"

#include <algorithm>
#include <cmath>
#include <cstdio>
#include <cstdlib>
#include <cstring>
#include <string>
#include <vector>

#include "common.h"
#include "launch.h"

using namespace kfac;

namespace {

struct MatJobH {
  int32_t mat, bi, bj, aux;
};

// The three update lists of an outer block (see schedule_invert).
enum { UPD_DIAG = 0, UPD_COL = 1, UPD_REST = 2 };

inline int ceil_div(int64_t a, int64_t b) { return int((a + b - 1) / b); }

// A device table that is re-uploaded whenever its host image changes.
struct DynTable {
  void* dev = nullptr;
  void* pin = nullptr;
  size_t cap = 0;
  hipEvent_t ev = nullptr;
  bool pending = false;
  std::vector<unsigned char> last;   // image currently on the device
};

// An activation factor that is assembled from lag products: descriptors desc0 .. desc0 + LAG_NMAT - 1
// write the small matrices at float offsets off[] of the lag scratch region.
struct LagLayer {
  int layer = 0, desc0 = 0;
  size_t off[LAG_NMAT] = {};
};

struct FactorPlan {
  bool valid = false;
  std::vector<kfac_layer> layers;
  std::vector<uint8_t> present;      // [2*l] A wanted, [2*l+1] G wanted
  std::vector<int> desc_of;          // [2*l + which] -> descriptor index or -1
  std::vector<TileDesc> descs;       // shape part filled at build time, pointers/scalars per call
  void* d_jobs = nullptr;
  void* d_rjobs = nullptr;
  void* d_ljobs = nullptr;   // mirror tiles of the lag-product factors
  void* d_pjobs = nullptr;   // their channel-pair tiles
  int njobs = 0, nrjobs = 0, nljobs = 0, npjobs = 0;
  size_t nslots = 0;
  std::vector<LagLayer> lags;        // activation factors built from lag products
  size_t lag_floats = 0;             // their scratch matrices, behind the split-reduction slots
  DynTable tab;                      // [TileDesc x descs][LagAsm x lags]
  kfac_plan_stats stats{};
};

// One group of matrices that is swept in lockstep on its own stream.
struct InvertGroup {
  std::vector<int> idx;              // caller indices of the group's matrices
  std::vector<int> order;            // sorted position -> position in idx (large first, descending d)
  int n_large = 0, n_small = 0, n_ob = 0, n_views = 0;
  int agg = 4;                       // pivot blocks per outer block in this group
  bool latency_bound = false;        // the chain of dependent launches outlasts the group's arithmetic
  std::vector<int> view_off, n_in_ob;            // [outer block]
  std::vector<int> sub_pivot_off, sub_panel_off, sub_upd_off;   // [outer block * (agg + 1) + sub-step (+1)]
  std::vector<int> qm_off, mv_off, bp_off;       // [outer block (+1)]
  std::vector<int> mv_mid, bp_mid;               // [outer block]: first job that does not belong to the next outer block's rows
  std::vector<int> upd_off[3];                   // [UPD_DIAG / UPD_COL / UPD_REST][outer block (+1)]
  std::vector<size_t> ws_off;        // per large matrix: float offset of its workspace inside the group's region
  void* d_init = nullptr; int n_init = 0;
  int n_init_first = 0;              // leading init jobs: the tiles of the first outer block's diagonal sub-matrix
  hipEvent_t ev_start = nullptr, ev_init = nullptr;   // side stream: fork at the start of a call, rest of the init done
  void* d_finish = nullptr; int n_finish = 0;
  void* d_sub_pivot = nullptr; void* d_sub_panel = nullptr; void* d_sub_upd = nullptr;
  void* d_qm = nullptr; void* d_mv = nullptr; void* d_bp = nullptr;
  void* d_upd[3] = {nullptr, nullptr, nullptr};
  void* d_chain_q = nullptr;         // quarter-tile jobs of the chain's products
  std::vector<int> cq_bp_off, cq_bp_end, cq_diag_end;
  std::vector<hipEvent_t> ev_gather, ev_chain, ev_col, ev_rest;   // [outer block], created on first use
  DynTable tab;                      // [InvMat x n][InvMat x views][PanelMove x 2 views][TileDesc x (2 views + n_large)]
  size_t ws_floats = 0, ws_base = 0;
};

struct InvertPlan {
  bool valid = false;
  std::vector<int32_t> dims;
  std::vector<InvertGroup> groups;
  size_t ws_floats = 0;
  kfac_plan_stats stats{};
};

struct PrecondPlan {
  bool valid = false;
  std::vector<int32_t> dG, dA;
  std::vector<size_t> t_off;         // per layer: float offset of the intermediate Ginv.V
  void* d_jobs1 = nullptr; void* d_jobs2 = nullptr;
  int njobs1 = 0, njobs2 = 0;
  DynTable tab;                      // [TileDesc x 2n]
  size_t ws_floats = 0;
  kfac_plan_stats stats{};
};

struct PackPlan {
  bool valid = false;
  std::vector<int32_t> dims;
  std::vector<uint64_t> off;         // float offset of every matrix's triangle
  void* d_jobs = nullptr;
  int njobs = 0;
  DynTable tab;                      // [PackMat x n]
};

}  // namespace

constexpr int MAX_INV_GROUPS = 4;

struct TimingRec {
  hipEvent_t a, b;
  int kclass;
};

struct kfac_ctx {
  uint32_t timing_mask = 0;
  std::vector<TimingRec> timing;
  int device = -1;
  bool host_only = true;
  std::string err;
  // one workspace per call kind (factors, inverse, preconditioning), so calls of different kinds
  // may run at the same time on different streams
  void* ws[3] = {nullptr, nullptr, nullptr};
  size_t ws_cap[3] = {0, 0, 0};
  // tuning options (kfac_set_option); the defaults are the measured best for the benchmark workloads
  int opt[KFAC_OPT_COUNT] = {
      /* INV_GROUPS     */ 2,       // lockstep groups of matrices swept concurrently
      /* INV_AGG        */ 4,       // pivot blocks per outer block (rank agg*128 updates), throughput-bound group
      /* INV_AGG_CHAIN  */ 6,       // the same for a latency-bound group (fewer outer steps on the critical path)
      /* INV_FUSE       */ 1,       // a pivot block applies the previous block's update to itself (one launch fewer per step)
      /* INV_SIDE_PAD   */ 56000,   // unused LDS beyond 32 KB in the off-chain products of a latency-bound group: one workgroup
                                    // per compute unit, so that the chain's kernels always find a free slot
      /* FACTOR_LAG     */ 1,       // lag products for 3x3 / stride 1 / pad 1 activation factors
      /* FACTOR_VEC11   */ 1,       // 128-bit loader for 1x1 windows over whole images
      /* FACTOR_XCD     */ 0,       // XCD-aware arrangement of the factor jobs (measured slower)
      /* FACTOR_KJOB    */ MAX_JOB_ROWS,   // longest contraction run of one factor tile job (rows)
      /* INV_CHAIN_PAD  */ 0,       // unused LDS added to the kernels of a latency-bound group's chain: with the side pad,
                                    // no workgroup of the call shares a compute unit with a chain workgroup
      /* INV_SIDE       */ 1,       // off-chain work of a group on a second stream (0: everything on the group's one stream)
      /* INV_SPLIT_LONG */ 1,       // the matrices with the longest chains form a group of their own
      /* INV_YIELD      */ 64,      // chain kernels of at most this many workgroups make the products on their compute
                                    // units give way while they run (0: off)
      /* INV_QUARTER    */ 1,       // the chain's two products of an outer block on quarter tiles (four workgroups a tile)
  };
  int* cu_flags = nullptr;          // per-compute-unit words of that protocol (device memory, zero when no kernel runs)
  hipStream_t inv_stream[MAX_INV_GROUPS] = {};   // sweep chain of groups 1.. (group 0 uses the caller's stream)
  hipStream_t inv_side[MAX_INV_GROUPS] = {};     // every group's side stream for the off-chain updates
  hipEvent_t inv_fork = nullptr, inv_join[MAX_INV_GROUPS] = {};
  FactorPlan fp;
  InvertPlan ip;
  PrecondPlan pp;
  PackPlan kp;
};

namespace {

std::string g_noctx_err = "no context";

kfac_status fail(kfac_ctx* ctx, kfac_status st, const std::string& msg) {
  if (ctx) ctx->err = msg; else g_noctx_err = msg;
  return st;
}

struct FactorOpts;
FactorOpts factor_opts(const kfac_ctx* c);

// Brackets the launches issued during its lifetime with a pair of events (when the class is enabled).
struct ScopedTiming {
  kfac_ctx* c;
  hipStream_t s;
  TimingRec r{};
  bool on = false;
  ScopedTiming(kfac_ctx* ctx, int kclass, hipStream_t stream) : c(ctx), s(stream) {
    if (!(ctx->timing_mask & (1u << kclass))) return;
    if (hipEventCreate(&r.a) != hipSuccess) return;
    if (hipEventCreate(&r.b) != hipSuccess) { (void)hipEventDestroy(r.a); return; }
    r.kclass = kclass;
    on = hipEventRecord(r.a, s) == hipSuccess;
  }
  ~ScopedTiming() {
    if (!on) return;
    (void)hipEventRecord(r.b, s);
    c->timing.push_back(r);
  }
};

#define HIP_TRY(ctx, expr)                                                                   \
  do {                                                                                       \
    hipError_t e_ = (expr);                                                                  \
    if (e_ != hipSuccess)                                                                    \
      return fail(ctx, KFAC_ERR_DEVICE, std::string(#expr) + ": " + hipGetErrorString(e_)); \
  } while (0)

struct DeviceGuard {
  int prev = -1;
  bool active = false;
  explicit DeviceGuard(const kfac_ctx* c) {
    if (!c->host_only && hipGetDevice(&prev) == hipSuccess && prev != c->device) {
      active = hipSetDevice(c->device) == hipSuccess;
    }
  }
  ~DeviceGuard() {
    if (active) (void)hipSetDevice(prev);
  }
};

void free_dev(void*& p) {
  if (p) { (void)hipFree(p); p = nullptr; }
}

void free_table(DynTable& t) {
  free_dev(t.dev);
  if (t.pin) { (void)hipHostFree(t.pin); t.pin = nullptr; }
  if (t.ev) { (void)hipEventDestroy(t.ev); t.ev = nullptr; }
  t.cap = 0; t.pending = false; t.last.clear();
}

kfac_status upload_static(kfac_ctx* ctx, void** dev, const void* src, size_t bytes) {
  free_dev(*dev);
  if (bytes == 0) return KFAC_OK;
  HIP_TRY(ctx, hipMalloc(dev, bytes));
  HIP_TRY(ctx, hipMemcpy(*dev, src, bytes, hipMemcpyHostToDevice));
  return KFAC_OK;
}

// Stream-ordered refresh of a device table; skipped when the image is unchanged.
kfac_status sync_table(kfac_ctx* ctx, DynTable& t, const void* img, size_t bytes, hipStream_t s) {
  if (bytes == 0) return KFAC_OK;
  if (t.last.size() == bytes && std::memcmp(t.last.data(), img, bytes) == 0) return KFAC_OK;
  if (bytes > t.cap) {
    if (t.pending) HIP_TRY(ctx, hipEventSynchronize(t.ev));
    HIP_TRY(ctx, hipDeviceSynchronize());
    free_dev(t.dev);
    if (t.pin) { (void)hipHostFree(t.pin); t.pin = nullptr; }
    HIP_TRY(ctx, hipMalloc(&t.dev, bytes));
    HIP_TRY(ctx, hipHostMalloc(&t.pin, bytes, hipHostMallocDefault));
    t.cap = bytes;
    if (!t.ev) HIP_TRY(ctx, hipEventCreateWithFlags(&t.ev, hipEventDisableTiming));
    t.pending = false;
  }
  if (t.pending) HIP_TRY(ctx, hipEventSynchronize(t.ev));
  std::memcpy(t.pin, img, bytes);
  HIP_TRY(ctx, hipMemcpyAsync(t.dev, t.pin, bytes, hipMemcpyHostToDevice, s));
  HIP_TRY(ctx, hipEventRecord(t.ev, s));
  t.pending = true;
  t.last.assign(static_cast<const unsigned char*>(img), static_cast<const unsigned char*>(img) + bytes);
  return KFAC_OK;
}

enum { WS_FACTORS = 0, WS_INVERT = 1, WS_PRECOND = 2 };
kfac_status ensure_ws(kfac_ctx* ctx, int which, size_t bytes) {
  if (bytes <= ctx->ws_cap[which]) return KFAC_OK;
  if (hipDeviceSynchronize() != hipSuccess) return fail(ctx, KFAC_ERR_DEVICE, "hipDeviceSynchronize failed");
  free_dev(ctx->ws[which]);
  ctx->ws_cap[which] = 0;
  if (hipMalloc(&ctx->ws[which], bytes) != hipSuccess) {
    ctx->ws[which] = nullptr;
    (void)hipGetLastError();
    return fail(ctx, KFAC_ERR_WORKSPACE, "cannot allocate " + std::to_string(bytes) + " bytes of device workspace");
  }
  ctx->ws_cap[which] = bytes;
  return KFAC_OK;
}

// ------------------------------------------------------------------------------- layers
bool layer_valid(const kfac_layer& L, std::string* why) {
  auto bad = [&](const char* m) { if (why) *why = m; return false; };
  if (L.kind != 0 && L.kind != 1) return bad("layer.kind must be 0 (linear) or 1 (conv2d)");
  if (L.has_bias != 0 && L.has_bias != 1) return bad("layer.has_bias must be 0 or 1");
  if (L.c_in < 1 || L.c_out < 1) return bad("layer.c_in and layer.c_out must be positive");
  const int64_t max_elems = (int64_t(1) << 28);   // operands are addressed with 32-bit byte offsets, at most 1 GiB each
  // factor dimensions: the kernels address a factor with 32-bit byte offsets, and the other two calls
  // accept matrices up to this order
  const int64_t max_dim = 16384;
  if (L.c_out > max_dim) return bad("factor dimension dG exceeds 16384");
  if (L.kind == 0) {
    if (int64_t(L.c_in) + L.has_bias > max_dim) return bad("factor dimension dA exceeds 16384");
    if (L.rows < 1) return bad("linear layer needs rows >= 1");
    if (int64_t(L.rows) * L.c_in > max_elems || int64_t(L.rows) * L.c_out > max_elems)
      return bad("linear layer tensor exceeds 1 GiB");
    return true;
  }
  if (L.n < 1 || L.h < 1 || L.w < 1) return bad("conv layer needs n, h, w >= 1");
  if (L.kh < 1 || L.kw < 1 || int64_t(L.kh) * L.kw > 63) return bad("conv window must have 1..63 taps");
  if (L.stride < 1) return bad("conv stride must be >= 1");
  if (L.pad_h < 0 || L.pad_h > 127 || L.pad_w < 0 || L.pad_w > 127) return bad("conv pads must be in 0..127");
  if (L.h + 2 * L.pad_h < L.kh || L.w + 2 * L.pad_w < L.kw) return bad("conv output is empty");
  const int64_t oh = (L.h + 2 * L.pad_h - L.kh) / L.stride + 1, ow = (L.w + 2 * L.pad_w - L.kw) / L.stride + 1;
  const int64_t lim = (int64_t(1) << 31) - 1;
  if (int64_t(L.n) * oh * ow > lim) return bad("conv rows n*oh*ow exceed 2^31-1");
  if (int64_t(L.c_in) * L.h * L.w > lim || int64_t(L.c_out) * oh * ow > lim) return bad("one sample exceeds 2^31-1 elements");
  if (int64_t(L.c_in) * L.kh * L.kw + L.has_bias > max_dim) return bad("factor dimension dA exceeds 16384");
  if (int64_t(L.n) * L.c_in * L.h * L.w > max_elems || int64_t(L.n) * L.c_out * oh * ow > max_elems)
    return bad("conv layer tensor exceeds 1 GiB");
  return true;
}

int conv_oh(const kfac_layer& L) { return (L.h + 2 * L.pad_h - L.kh) / L.stride + 1; }
int conv_ow(const kfac_layer& L) { return (L.w + 2 * L.pad_w - L.kw) / L.stride + 1; }
int64_t rows_of(const kfac_layer& L) { return L.kind == 0 ? L.rows : int64_t(L.n) * conv_oh(L) * conv_ow(L); }
int dA_of(const kfac_layer& L) { return (L.kind == 0 ? L.c_in : L.c_in * L.kh * L.kw) + L.has_bias; }

// The options that shape a factor schedule.
struct FactorOpts {
  int kjob = MAX_JOB_ROWS;
  bool lag = true, vec = true, xcd = false;
};

Operand act_operand(const kfac_layer& L, bool vec) {
  Operand o{};
  o.K = int32_t(rows_of(L));
  o.M = dA_of(L);
  o.bias = L.has_bias;
  if (L.kind == 0) {
    o.type = OP_KMAJOR;
    o.ld = L.c_in;
    o.bytes = uint32_t(int64_t(L.rows) * L.c_in * 4);
    return o;
  }
  o.bytes = uint32_t(int64_t(L.n) * L.c_in * L.h * L.w * 4);
  if (L.kh == 1 && L.kw == 1 && L.pad_h == 0 && L.pad_w == 0) o.type = (L.stride == 1 && vec && (L.h * L.w) % 4 == 0) ? OP_CONV11V : OP_CONV11;
  else if (L.kh == 3 && L.kw == 3) o.type = OP_CONV33;
  else if (L.kh == 7 && L.kw == 7) o.type = OP_CONV77;
  else o.type = OP_CONVGEN;
  o.C = L.c_in; o.H = L.h; o.W = L.w; o.OH = conv_oh(L); o.OW = conv_ow(L);
  o.stride = L.stride; o.pad_h = L.pad_h; o.pad_w = L.pad_w; o.KH = L.kh; o.KW = L.kw;
  o.dOW = make_fastdiv(uint32_t(o.OW));
  o.dOHW = make_fastdiv(uint32_t(o.OH) * uint32_t(o.OW));
  return o;
}

Operand gout_operand(const kfac_layer& L, bool vec) {
  Operand o{};
  o.K = int32_t(rows_of(L));
  o.M = L.c_out;
  o.bias = 0;
  if (L.kind == 0) {
    o.type = OP_KMAJOR;
    o.ld = L.c_out;
    o.bytes = uint32_t(int64_t(L.rows) * L.c_out * 4);
    return o;
  }
  o.bytes = uint32_t(o.K * int64_t(L.c_out) * 4);
  // [n, c_out, oh, ow] read through a 1x1 window: k = (n, oy, ox), m = channel
  o.C = L.c_out; o.H = conv_oh(L); o.W = conv_ow(L); o.OH = o.H; o.OW = o.W;
  o.type = (vec && (o.H * o.W) % 4 == 0) ? OP_CONV11V : OP_CONV11;
  o.stride = 1; o.pad_h = o.pad_w = 0; o.KH = 1; o.KW = 1;
  o.dOW = make_fastdiv(uint32_t(o.OW));
  o.dOHW = make_fastdiv(uint32_t(o.OH) * uint32_t(o.OW));
  return o;
}

Operand rowmajor_operand(const float* p, int K, int M, int ld) {   // element (k, m) at p[k*ld + m]
  Operand o{};
  o.ptr = p; o.type = OP_KMAJOR; o.K = K; o.M = M; o.bias = 0; o.ld = ld;
  o.bytes = uint32_t(int64_t(K) * ld * 4);
  return o;
}

Operand transposed_operand(const float* p, int K, int M) {   // element (k, m) at p[m*K + k]
  Operand o{};
  o.ptr = p; o.type = OP_CONV11; o.K = K; o.M = M; o.bias = 0;
  o.bytes = uint32_t(int64_t(K) * M * 4);
  o.C = M; o.H = 1; o.W = K; o.OH = 1; o.OW = K; o.stride = 1; o.pad_h = o.pad_w = 0; o.KH = 1; o.KW = 1;
  o.dOW = make_fastdiv(uint32_t(K));
  o.dOHW = make_fastdiv(uint32_t(K));
  return o;
}

// 32x32 MFMA blocks of a 128x128 tile that hold wanted outputs
int active_blocks(int M, int N, int bi, int bj, bool sym) {
  const int rb = std::min(4, ceil_div(std::min(BM, M - bi * BM), 32));
  const int cb = std::min(4, ceil_div(std::min(BN, N - bj * BN), 32));
  if (!(sym && bi == bj)) return rb * cb;
  int c = 0;
  for (int r = 0; r < rb; ++r)
    for (int q = 0; q < cb; ++q) c += r >= q;
  return c;
}

// XCD-aware arrangement of a grouped launch.  Workgroup g runs on XCD g % 8 (each XCD has its own
// L2) and the kernels map it to job (g % 8) * ceil(n / 8) + g / 8, i.e. XCD x walks segment x of the
// list in order.  Every group (one layer / one matrix, jobs in locality order, heaviest groups first)
// is cut into 8 contiguous pieces, one per XCD: the XCDs get equal work, and the jobs that run
// together on one XCD are neighbouring tiles of the same operand, which they then share in L2.
// Segments are padded to equal length with no-op jobs (desc = -1).
std::vector<TileJob> xcd_arrange(const std::vector<std::vector<TileJob>>& groups) {
  std::vector<TileJob> seg[8];
  for (const auto& g : groups) {
    const size_t L = g.size();
    for (int x = 0; x < 8; ++x)
      for (size_t i = x * L / 8; i < (x + 1) * L / 8; ++i) seg[x].push_back(g[i]);
  }
  size_t per = 0;
  for (int x = 0; x < 8; ++x) per = std::max(per, seg[x].size());
  TileJob nop{};
  nop.desc = -1;
  std::vector<TileJob> out;
  out.reserve(per * 8);
  for (int x = 0; x < 8; ++x) {
    out.insert(out.end(), seg[x].begin(), seg[x].end());
    out.insert(out.end(), per - seg[x].size(), nop);
  }
  return out;
}

// ------------------------------------------------------------------------------- factor plan
void release(FactorPlan& p) {
  free_dev(p.d_jobs); free_dev(p.d_rjobs); free_dev(p.d_ljobs); free_dev(p.d_pjobs); free_table(p.tab);
  p = FactorPlan{};
}
void release(InvertPlan& p) {
  for (InvertGroup& g : p.groups) {
    free_dev(g.d_init); free_dev(g.d_finish); free_dev(g.d_sub_pivot); free_dev(g.d_sub_panel); free_dev(g.d_sub_upd);
    free_dev(g.d_qm); free_dev(g.d_mv); free_dev(g.d_bp);
    for (int k = 0; k < 3; ++k) free_dev(g.d_upd[k]);
    free_dev(g.d_chain_q);
    free_table(g.tab);
    for (hipEvent_t e : g.ev_chain) if (e) (void)hipEventDestroy(e);
    for (hipEvent_t e : g.ev_gather) if (e) (void)hipEventDestroy(e);
    for (hipEvent_t e : g.ev_col) if (e) (void)hipEventDestroy(e);
    for (hipEvent_t e : g.ev_rest) if (e) (void)hipEventDestroy(e);
    if (g.ev_start) (void)hipEventDestroy(g.ev_start);
    if (g.ev_init) (void)hipEventDestroy(g.ev_init);
  }
  p = InvertPlan{};
}
void release(PackPlan& p) {
  free_dev(p.d_jobs); free_table(p.tab);
  p = PackPlan{};
}
void release(PrecondPlan& p) {
  free_dev(p.d_jobs1); free_dev(p.d_jobs2); free_table(p.tab);
  p = PrecondPlan{};
}

struct FactorSchedule {
  std::vector<TileDesc> descs;
  std::vector<int> desc_of;
  std::vector<TileJob> jobs;
  std::vector<ReduceJob> rjobs;
  std::vector<LagLayer> lags;
  std::vector<LagJob> ljobs, pjobs;   // mirror tiles; channel-pair tiles
  size_t nslots = 0, lag_floats = 0;
  kfac_plan_stats stats{};
};

// Activation factors of 3x3 / stride 1 / pad 1 convolutions with enough channels are built from
// lag products (about a third of the multiply-adds of the patch-matrix product, see LagAsm).
constexpr int LAG_MIN_C = 64;
bool lag_eligible(const kfac_layer& L) {
  return L.kind == 1 && L.kh == 3 && L.kw == 3 && L.stride == 1 && L.pad_h == 1 && L.pad_w == 1 && L.c_in >= LAG_MIN_C;
}

// View of the activations through a KH x KW window of lags over the pixel window [y0, y1] x [x0, x1]
Operand lag_operand(const kfac_layer& L, int type, int KH, int KW, int pad_h, int pad_w, int bias,
                    int y0, int y1, int x0, int x1) {
  Operand o{};
  o.type = type;
  o.C = L.c_in; o.H = L.h; o.W = L.w; o.OH = y1 - y0 + 1; o.OW = x1 - x0 + 1; o.oy0 = y0; o.ox0 = x0;
  o.stride = 1; o.pad_h = pad_h; o.pad_w = pad_w; o.KH = KH; o.KW = KW;
  o.K = int32_t(int64_t(L.n) * o.OH * o.OW);
  o.M = L.c_in * KH * KW + bias;
  o.bias = bias;
  o.bytes = uint32_t(int64_t(L.n) * L.c_in * L.h * L.w * 4);
  o.dOW = make_fastdiv(uint32_t(o.OW));
  o.dOHW = make_fastdiv(uint32_t(o.OH) * uint32_t(o.OW));
  return o;
}

FactorSchedule schedule_factors(int n, const kfac_layer* layers, const std::vector<uint8_t>& present, const FactorOpts& O) {
  const int kjob = O.kjob;
  FactorSchedule S;
  S.desc_of.assign(2 * n, -1);
  for (int l = 0; l < n; ++l)
    for (int which = 0; which < 2; ++which) {
      if (!present[2 * l + which]) continue;
      S.desc_of[2 * l + which] = int(S.descs.size());
      const kfac_layer& L = layers[l];
      if (which == 0 && O.lag && lag_eligible(L)) {
        LagLayer lg;
        lg.layer = l; lg.desc0 = int(S.descs.size());
        const int H = L.h, W = L.w, b = L.has_bias;
        const int win[LAG_NMAT][4] = {{0, H - 1, 0, W - 1}, {0, H - 1, 0, W - 1},
                                      {0, 0, 0, W - 1}, {H - 1, H - 1, 0, W - 1}, {0, H - 1, 0, 0}, {0, H - 1, W - 1, W - 1},
                                      {0, 0, 0, 0}, {0, 0, W - 1, W - 1}, {H - 1, H - 1, 0, 0}, {H - 1, H - 1, W - 1, W - 1}};
        for (int k = 0; k < LAG_NMAT; ++k) {
          TileDesc D{};
          const int* w = win[k];
          const bool whole = k <= LAG_G2 && O.vec && (H * W) % 4 == 0;   // whole images: four pixels per load
          D.a = lag_operand(L, whole ? OP_CONV11V : OP_CONV11, 1, 1, 0, 0, 0, w[0], w[1], w[2], w[3]);
          if (k == LAG_G1) D.b = lag_operand(L, OP_CONV25, 2, 5, -1, 2, 0, w[0], w[1], w[2], w[3]);
          else if (k == LAG_G2) D.b = lag_operand(L, OP_CONV13, 1, 3, 0, 0, b, w[0], w[1], w[2], w[3]);
          else {
            // A border row pairs with itself only: the tap in row i = 0 (which drops the bottom row) asks
            // for lags dy = i' - i >= 0, and below the bottom row there is nothing, so dy = 0 and the
            // lags along the row remain, of which the backward ones are transposes of the forward ones
            // (the row is closed under the shift): dx = 0, 1, 2.  Likewise a border column (dx = 0,
            // dy = 0, 1, 2) and a corner pixel (lag 0 only).
            static const int geo[LAG_NMAT][4] = {{0, 0, 0, 0}, {0, 0, 0, 0},                 // KH, KW, pad_h, pad_w
                                                 {1, 3, 0, 0}, {1, 3, 0, 0}, {3, 1, 0, 0}, {3, 1, 0, 0},
                                                 {1, 1, 0, 0}, {1, 1, 0, 0}, {1, 1, 0, 0}, {1, 1, 0, 0}};
            D.b = lag_operand(L, OP_CONVGEN, geo[k][0], geo[k][1], geo[k][2], geo[k][3], b, w[0], w[1], w[2], w[3]);
          }
          D.M = D.a.M; D.N = D.ldo = D.b.M;
          D.sym = 0; D.mirror = MIRROR_NONE; D.alpha = 1.f; D.beta = 0.f;
          lg.off[k] = S.lag_floats;
          S.lag_floats += size_t(D.M) * D.N;
          S.descs.push_back(D);
        }
        const int T = ceil_div(dA_of(L), 64);
        for (int bi = 0; bi < T; ++bi)
          for (int bj = 0; bj <= bi; ++bj) S.ljobs.push_back(LagJob{int(S.lags.size()), bi, bj, 0});
        {   // tiles of channel pairs (c, c2), c2 <= c, over the channels 0 .. C - 1 and the bias pseudo-channel C
          const int PR = lag_pair_rows(), PC = lag_pair_cols(), nch = L.c_in + (b ? 1 : 0);
          for (int bi = 0; bi < ceil_div(nch, PR); ++bi)
            for (int bj = 0; bj * PC <= std::min(nch - 1, bi * PR + PR - 1); ++bj) S.pjobs.push_back(LagJob{int(S.lags.size()), bi, bj, 0});
        }
        S.lags.push_back(lg);
        continue;
      }
      TileDesc D{};
      D.a = which == 0 ? act_operand(L, O.vec) : gout_operand(L, O.vec);
      D.b = D.a;
      D.M = D.N = D.ldo = D.a.M;
      D.sym = 1;
      D.mirror = MIRROR_ALL;
      S.descs.push_back(D);
    }
  struct Group { std::vector<TileJob> jobs; int64_t job_cost; };
  std::vector<Group> groups;
  for (size_t di = 0; di < S.descs.size(); ++di) {
    const TileDesc& D = S.descs[di];
    const bool sym = D.sym != 0;
    const int R = D.a.K, Tm = ceil_div(D.M, BM), Tn = ceil_div(D.N, BN);
    int nsplit = ceil_div(R, kjob);
    int chunk = ceil_div(ceil_div(R, nsplit), KC) * KC;
    nsplit = ceil_div(R, chunk);
    const int ntile = sym ? Tm * (Tm + 1) / 2 : Tm * Tn;
    const size_t slot0 = S.nslots;
    if (nsplit > 1) S.nslots += size_t(ntile) * nsplit;
    Group G;
    G.job_cost = int64_t(std::min(R, chunk)) * (sym ? 16 : active_blocks(D.M, D.N, 0, 0, false));
    // row chunk outermost: the jobs that run side by side read the same rows of the activations
    for (int sidx = 0; sidx < nsplit; ++sidx) {
      int tile = 0;
      for (int bi = 0; bi < Tm; ++bi)
        for (int bj = 0; bj < (sym ? bi + 1 : Tn); ++bj, ++tile) {
          const int ab = active_blocks(D.M, D.N, bi, bj, sym);
          if (nsplit > 1 && sidx == 0) {
            ReduceJob rj{};
            rj.desc = int(di); rj.bi = bi; rj.bj = bj; rj.part0 = int(slot0 + size_t(tile) * nsplit); rj.nsplit = nsplit;
            S.rjobs.push_back(rj);
            S.stats.n_split++;
          }
          TileJob j{};
          j.desc = int(di); j.bi = bi; j.bj = bj;
          j.kbeg = sidx * chunk; j.kend = std::min(R, (sidx + 1) * chunk);
          j.part = nsplit > 1 ? int(slot0 + size_t(tile) * nsplit + sidx) : -1;
          G.jobs.push_back(j);
          S.stats.mfma_flops += int64_t(j.kend - j.kbeg) * ab * 32 * 32 * 2;
        }
    }
    groups.push_back(std::move(G));
  }
  // longest jobs first: workgroups are dispatched in index order, so this is the list-scheduling
  // (largest-first) rule applied to compute units
  std::stable_sort(groups.begin(), groups.end(), [](const Group& x, const Group& y) { return x.job_cost > y.job_cost; });
  std::vector<std::vector<TileJob>> lists;
  for (auto& g : groups) lists.push_back(std::move(g.jobs));
  if (O.xcd) {
    S.jobs = xcd_arrange(lists);
  } else {
    for (auto& l : lists) S.jobs.insert(S.jobs.end(), l.begin(), l.end());
  }
  S.stats.n_jobs = int64_t(S.jobs.size() + S.rjobs.size() + S.ljobs.size() + S.pjobs.size());
  S.stats.n_launches = 1 + (S.rjobs.empty() ? 0 : 1) + (S.ljobs.empty() ? 0 : 2);
  S.stats.ws_bytes = int64_t((S.nslots * size_t(BM) * BN + S.lag_floats) * sizeof(float));
  return S;
}

// ------------------------------------------------------------------------------- invert plan
// Two-level blocked symmetric sweep.  A matrix is cut in outer blocks of `agg` pivot blocks
// (agg*128 rows).  For outer block b, with D its diagonal sub-matrix and Z the rest of its block
// column:
//   1. D is swept in place by the one-level algorithm (pivot, panel, rank-128 update, only on the
//      <= agg x agg tiles of D): D <- -D^-1.  With `fuse` the update of the next pivot block is left
//      to that block's own sweep kernel, which then shares a launch with the rest of the update;
//   2. QB = D^-1 as a full symmetric matrix;  Zt = Z^T gathered k-major;
//   3. Wt = QB Zt (one GEMM with K = agg*128), scattered back into the block column;
//   4. every tile outside the outer block gets  M_ij -= W_i Z_j^T  (K = agg*128), in three lists:
//      the diagonal sub-matrix of the NEXT outer block (UPD_DIAG), which step 1 of the next block
//      needs at once; the rest of the next block's rows/columns (UPD_COL), needed by its step 2;
//      and all the others (UPD_REST), which nothing touches before the next block's step 4.
//      UPD_COL and UPD_REST run on a second stream beside the next block's latency-bound step 1.
// The panel buffers of consecutive outer blocks alternate between two halves of the workspace so
// that the off-chain update can still read its panels while the next ones are written.
// All matrices of a group advance in lockstep: one launch per step covers every matrix that
// still has that step.
struct InvertSchedule {
  std::vector<int> order;
  int n_large = 0, n_small = 0, n_ob = 0, n_views = 0, n_init_first = 0;
  std::vector<int> nblk, ldp, nob;
  std::vector<size_t> ws_off;
  std::vector<int> view_off, n_in_ob, sub_pivot_off, sub_panel_off, sub_upd_off, qm_off, mv_off, bp_off, mv_mid, bp_mid;
  std::vector<int> upd_off[3];
  std::vector<MatJobH> init, finish, sub_pivot, sub_panel, qm, mv;
  std::vector<TileJob> sub_upd, bp, upd[3];
  // the chain's two product lists of every outer block (panel product for the next rows, update of the next
  // diagonal sub-matrix) cut into quarter tiles
  std::vector<TileJob> chain_q;
  std::vector<int> cq_bp_off, cq_bp_end, cq_diag_end;   // [outer block]: [off, bp_end) panel product, [bp_end, diag_end) update
  size_t ws_floats = 0;
  kfac_plan_stats stats{};
};

// workspace of one large matrix, offsets in floats
struct InvWsLayout {
  size_t wt, zt, swt, szt, q, qb, total;
};
// Outer blocks hold `agg` pivot blocks.  A last pivot block of at most TAIL_ROWS rows (the bias row of
// a factor whose other rows fill whole blocks) joins the outer block before it instead of forming
// one of its own, so an outer block spans at most agg + 1 pivot blocks.
constexpr int TAIL_ROWS = 32;
int inv_nob(int d, int agg) {
  const int nblk = ceil_div(d, NB);
  int nob = ceil_div(nblk, agg);
  if (nob > 1 && (nblk - 1) % agg == 0 && d - (nblk - 1) * NB <= TAIL_ROWS) --nob;
  return nob;
}
int inv_ob_end(int d, int agg, int b) {   // first pivot block behind outer block b
  return b >= inv_nob(d, agg) - 1 ? ceil_div(d, NB) : (b + 1) * agg;
}
InvWsLayout inv_ws_layout(int ldp, int agg) {
  InvWsLayout L{};
  const size_t aw = size_t(agg + 1) * NB;             // widest outer block
  const size_t big = 2 * aw * ldp;                    // two halves of panels
  const size_t sub = size_t(NB) * aw;                 // one panel of the diagonal sub-matrix
  L.wt = 0; L.zt = big; L.swt = 2 * big; L.szt = 2 * big + sub; L.q = 2 * big + 2 * sub;
  L.qb = L.q + size_t(NB) * NB;
  L.total = L.qb + aw * aw;
  return L;
}

InvertSchedule schedule_invert(int n, const int32_t* dims, int agg, bool fuse = false) {
  InvertSchedule S;
  S.order.resize(n);
  for (int i = 0; i < n; ++i) S.order[i] = i;
  std::stable_sort(S.order.begin(), S.order.end(), [&](int a, int b) { return dims[a] > dims[b]; });
  for (int i = 0; i < n; ++i) (dims[S.order[i]] > NB ? S.n_large : S.n_small)++;
  S.nblk.resize(S.n_large); S.ldp.resize(S.n_large); S.nob.resize(S.n_large); S.ws_off.resize(S.n_large);
  for (int m = 0; m < S.n_large; ++m) {
    const int d = dims[S.order[m]];
    S.nblk[m] = ceil_div(d, NB);
    S.ldp[m] = S.nblk[m] * NB;
    S.nob[m] = inv_nob(d, agg);
    S.ws_off[m] = S.ws_floats;
    S.ws_floats += inv_ws_layout(S.ldp[m], agg).total;
    S.n_ob = std::max(S.n_ob, S.nob[m]);
    const int tf = ceil_div(d, FINISH_TILE);
    for (int bi = 0; bi < tf; ++bi)
      for (int bj = 0; bj <= bi; ++bj) S.finish.push_back({m, bi, bj, 0});
  }
  // init jobs: the tiles of the first outer block's diagonal sub-matrix first (the sweep starts on
  // them; the others are copied on the side stream meanwhile)
  for (int pass = 0; pass < 2; ++pass) {
    for (int m = 0; m < S.n_large; ++m) {
      const int e0 = inv_ob_end(dims[S.order[m]], agg, 0);
      for (int bi = 0; bi < S.nblk[m]; ++bi)
        for (int bj = 0; bj <= bi; ++bj)
          if ((bi < e0) == (pass == 0)) S.init.push_back({m, bi, bj, 0});
    }
    if (pass == 0) S.n_init_first = int(S.init.size());
  }
  S.view_off.assign(S.n_ob + 1, 0); S.n_in_ob.assign(S.n_ob, 0);
  for (int b = 0; b < S.n_ob; ++b) {
    for (int m = 0; m < S.n_large; ++m) S.n_in_ob[b] += S.nob[m] > b;
    S.view_off[b + 1] = S.view_off[b] + S.n_in_ob[b];
  }
  S.n_views = S.view_off[S.n_ob];
  const int aw = agg + 1;   // sub-steps per outer block
  S.sub_pivot_off.assign(size_t(S.n_ob) * aw + 1, 0);
  S.sub_panel_off.assign(size_t(S.n_ob) * aw + 1, 0);
  S.sub_upd_off.assign(size_t(S.n_ob) * aw + 1, 0);
  S.qm_off.assign(S.n_ob + 1, 0); S.mv_off.assign(S.n_ob + 1, 0); S.bp_off.assign(S.n_ob + 1, 0);
  S.mv_mid.assign(S.n_ob, 0); S.bp_mid.assign(S.n_ob, 0);
  for (int k = 0; k < 3; ++k) S.upd_off[k].assign(S.n_ob + 1, 0);
  int64_t launches = 0;
  for (int b = 0; b < S.n_ob; ++b) {
    const int ob0 = b * agg;
    // ---- step 1: sweeps of the diagonal sub-matrices (views)
    for (int t = 0; t < aw; ++t) {
      const int st = b * aw + t;
      for (int m = 0; m < S.n_in_ob[b]; ++m) {
        const int v = S.view_off[b] + m;
        const int d = dims[S.order[m]];
        const int ob1 = inv_ob_end(d, agg, b);
        const int nsub = ob1 - ob0;
        const int dimB = std::min(d, ob1 * NB) - ob0 * NB;
        if (t >= nsub) continue;
        S.sub_pivot.push_back({v, 0, 0, 0});
        const int kb = std::min(NB, dimB - t * NB);
        for (int it = 0; it < nsub; ++it)
          if (it != t) S.sub_panel.push_back({v, it, 0, 0});
        for (int bi = 0; bi < nsub; ++bi)
          for (int bj = 0; bj <= bi; ++bj) {
            if (bi == t || bj == t) continue;
            S.stats.mfma_flops += int64_t(ceil_div(kb, KC) * KC) * active_blocks(dimB, dimB, bi, bj, true) * 32 * 32 * 2;
            if (fuse && bi == t + 1 && bj == t + 1) continue;   // the next pivot block: updated by its own sweep kernel
            TileJob j{};
            j.desc = v; j.bi = bi; j.bj = bj; j.kbeg = 0; j.kend = kb; j.part = -1;
            S.sub_upd.push_back(j);
          }
        S.stats.mfma_flops += int64_t(nsub - 1) * NB * 16 * 32 * 32 * 2;   // panel products
      }
      S.sub_pivot_off[st + 1] = int(S.sub_pivot.size());
      S.sub_panel_off[st + 1] = int(S.sub_panel.size());
      S.sub_upd_off[st + 1] = int(S.sub_upd.size());
    }
    for (int t = 0; t < aw; ++t) {   // fused: first pivot alone, panel, update together with the next pivot
      const int st = b * aw + t;
      const bool piv = S.sub_pivot_off[st + 1] > S.sub_pivot_off[st];
      const bool piv_next = t + 1 < aw && S.sub_pivot_off[st + 2] > S.sub_pivot_off[st + 1];
      const bool upd = S.sub_upd_off[st + 1] > S.sub_upd_off[st];
      launches += (S.sub_panel_off[st + 1] > S.sub_panel_off[st]);
      launches += fuse ? (t == 0 && piv) + (piv && (piv_next || upd)) : piv + upd;
    }
    // ---- steps 2-4 for the matrices that have more than one outer block.  The gather/scatter and
    // panel-product jobs of the rows of the NEXT outer block come first in their lists: the chain
    // needs only those, the others go to the side stream.
    std::vector<MatJobH> mv_rest;
    std::vector<TileJob> bp_rest;
    for (int m = 0; m < S.n_in_ob[b]; ++m) {
      if (S.nob[m] < 2) continue;
      const int v = S.view_off[b] + m;
      const int d = dims[S.order[m]];
      const int ob1 = inv_ob_end(d, agg, b), nb1 = b + 1 < S.nob[m] ? inv_ob_end(d, agg, b + 1) : ob1;
      const int dimB = std::min(d, ob1 * NB) - ob0 * NB;
      const int half = b & 1;
      auto in_ob = [&](int x) { return x >= ob0 && x < ob1; };
      auto in_next = [&](int x) { return x >= ob1 && x < nb1; };
      const int q32 = ceil_div(dimB, 32);
      for (int bi = 0; bi < q32; ++bi)
        for (int bj = 0; bj < q32; ++bj) S.qm.push_back({v, bi, bj, 0});
      for (int it = 0; it < S.nblk[m]; ++it) {
        if (in_ob(it)) continue;
        (in_next(it) ? S.mv : mv_rest).push_back({2 * v, it, 0, 0});
        for (int bi = 0; bi < ceil_div(dimB, BM); ++bi) {
          TileJob j{};
          j.desc = S.n_views + v; j.bi = bi; j.bj = it; j.kbeg = 0; j.kend = dimB; j.part = -1;
          (in_next(it) ? S.bp : bp_rest).push_back(j);
          S.stats.mfma_flops += int64_t(ceil_div(dimB, KC) * KC) * active_blocks(dimB, d, bi, it, false) * 32 * 32 * 2;
        }
      }
      for (int bi = 0; bi < S.nblk[m]; ++bi)
        for (int bj = 0; bj <= bi; ++bj) {
          if (in_ob(bi) || in_ob(bj)) continue;
          TileJob j{};
          j.desc = 2 * S.n_views + m; j.bi = bi; j.bj = bj; j.part = -1;
          j.kbeg = half * aw * NB; j.kend = j.kbeg + dimB;
          S.upd[(in_next(bi) && in_next(bj)) ? UPD_DIAG : (in_next(bi) || in_next(bj)) ? UPD_COL : UPD_REST].push_back(j);
          S.stats.mfma_flops += int64_t(ceil_div(dimB, KC) * KC) * active_blocks(d, d, bi, bj, true) * 32 * 32 * 2;
        }
    }
    S.mv_mid[b] = int(S.mv.size()); S.bp_mid[b] = int(S.bp.size());
    S.mv.insert(S.mv.end(), mv_rest.begin(), mv_rest.end());
    S.bp.insert(S.bp.end(), bp_rest.begin(), bp_rest.end());
    S.qm_off[b + 1] = int(S.qm.size()); S.mv_off[b + 1] = int(S.mv.size()); S.bp_off[b + 1] = int(S.bp.size());
    launches += (S.qm_off[b + 1] > S.qm_off[b]) + (S.mv_off[b + 1] > S.mv_off[b]) +
                (S.mv_mid[b] > S.mv_off[b]) * 2 + (S.mv_off[b + 1] > S.mv_mid[b]) * 2;
    for (int k = 0; k < 3; ++k) {
      S.upd_off[k][b + 1] = int(S.upd[k].size());
      launches += S.upd_off[k][b + 1] > S.upd_off[k][b];
    }
    // quarter tiles of the chain's products: every 32-column block of a tile that holds wanted columns
    auto quarters = [&](const TileJob& j, int ncols_total) {
      for (int q = 0; q < 4; ++q) {
        if (j.bj * BN + 32 * q >= ncols_total) break;
        TileJob x = j;
        x.quarter = q + 1;
        S.chain_q.push_back(x);
      }
    };
    S.cq_bp_off.push_back(int(S.chain_q.size()));
    for (int i = S.bp_off[b]; i < S.bp_mid[b]; ++i) quarters(S.bp[i], 1 << 30);   // panel buffers are padded to whole tiles
    S.cq_bp_end.push_back(int(S.chain_q.size()));
    for (int i = S.upd_off[UPD_DIAG][b]; i < S.upd_off[UPD_DIAG][b + 1]; ++i) {
      const TileJob& j = S.upd[UPD_DIAG][i];
      quarters(j, dims[S.order[j.desc - 2 * S.n_views]]);
    }
    S.cq_diag_end.push_back(int(S.chain_q.size()));
  }
  S.stats.n_jobs = int64_t(S.init.size() + S.finish.size() + S.sub_pivot.size() + S.sub_panel.size() + S.sub_upd.size() + S.qm.size() +
                           2 * S.mv.size() + S.bp.size() + S.upd[0].size() + S.upd[1].size() + S.upd[2].size()) + S.n_small;
  S.stats.n_launches = (S.n_small ? 1 : 0) + (S.n_large ? 2 + launches : 0);
  S.stats.ws_bytes = int64_t(S.ws_floats * sizeof(float));
  return S;
}

// ------------------------------------------------------------------------------- precondition plan
struct PrecondSchedule {
  std::vector<size_t> t_off;
  std::vector<TileJob> jobs1, jobs2;
  size_t ws_floats = 0;
  kfac_plan_stats stats{};
};

PrecondSchedule schedule_precond(int n, const int32_t* dG, const int32_t* dA) {
  PrecondSchedule S;
  S.t_off.resize(n);
  struct Tmp { TileJob j; int64_t cost; };
  std::vector<Tmp> t1, t2;
  for (int l = 0; l < n; ++l) {
    S.t_off[l] = S.ws_floats;
    S.ws_floats += size_t(dG[l]) * dA[l];
    const int Tm = ceil_div(dG[l], BM), Tn = ceil_div(dA[l], BN);
    for (int bi = 0; bi < Tm; ++bi)
      for (int bj = 0; bj < Tn; ++bj) {
        const int ab = active_blocks(dG[l], dA[l], bi, bj, false);
        TileJob j{};
        j.kbeg = 0; j.part = -1;
        j.bi = bj; j.bj = bi;              // first product: the intermediate is written transposed, [dA, dG]
        j.desc = 2 * l; j.kend = dG[l];
        t1.push_back({j, int64_t(dG[l]) * ab});
        j.bi = bi; j.bj = bj;
        j.desc = 2 * l + 1; j.kend = dA[l];
        t2.push_back({j, int64_t(dA[l]) * ab});
        S.stats.mfma_flops += (int64_t(ceil_div(dG[l], KC)) + ceil_div(dA[l], KC)) * KC * ab * 32 * 32 * 2;
      }
  }
  auto by_cost = [](const Tmp& x, const Tmp& y) { return x.cost > y.cost; };
  std::stable_sort(t1.begin(), t1.end(), by_cost);
  std::stable_sort(t2.begin(), t2.end(), by_cost);
  for (auto& t : t1) S.jobs1.push_back(t.j);
  for (auto& t : t2) S.jobs2.push_back(t.j);
  S.stats.n_jobs = int64_t(S.jobs1.size() + S.jobs2.size());
  S.stats.n_launches = n ? 2 : 0;
  S.stats.ws_bytes = int64_t(S.ws_floats * sizeof(float));
  return S;
}

bool finite_in(float v, float lo, float hi) { return v >= lo && v <= hi; }

FactorOpts factor_opts(const kfac_ctx* c) {
  FactorOpts O;
  O.kjob = c->opt[KFAC_OPT_FACTOR_KJOB];
  O.lag = c->opt[KFAC_OPT_FACTOR_LAG] != 0;
  O.vec = c->opt[KFAC_OPT_FACTOR_VEC11] != 0;
  O.xcd = c->opt[KFAC_OPT_FACTOR_XCD] != 0;
  return O;
}

}  // namespace

// =================================================================================== C ABI
extern "C" {

kfac_status kfac_create(kfac_ctx** out, int device) {
  if (!out) return fail(nullptr, KFAC_ERR_INVALID_ARG, "kfac_create: out is NULL");
  *out = nullptr;
  if (device < -1) return fail(nullptr, KFAC_ERR_INVALID_ARG, "kfac_create: device must be >= -1");
  kfac_ctx* c = new kfac_ctx();
  c->device = device;
  c->host_only = device < 0;
  if (!c->host_only) {
    int count = 0;
    if (hipGetDeviceCount(&count) != hipSuccess || device >= count) {
      (void)hipGetLastError();
      delete c;
      return fail(nullptr, KFAC_ERR_DEVICE, "kfac_create: no such HIP device");
    }
  }
  *out = c;
  return KFAC_OK;
}

void kfac_destroy(kfac_ctx* ctx) {
  if (!ctx) return;
  if (!ctx->host_only) {
    DeviceGuard g(ctx);
    (void)hipDeviceSynchronize();
    release(ctx->fp); release(ctx->ip); release(ctx->pp); release(ctx->kp);
    for (int k = 0; k < 3; ++k) free_dev(ctx->ws[k]);
    for (const TimingRec& r : ctx->timing) { (void)hipEventDestroy(r.a); (void)hipEventDestroy(r.b); }
    for (int g = 0; g < MAX_INV_GROUPS; ++g) {
      if (ctx->inv_stream[g]) (void)hipStreamDestroy(ctx->inv_stream[g]);
      if (ctx->inv_side[g]) (void)hipStreamDestroy(ctx->inv_side[g]);
      if (ctx->inv_join[g]) (void)hipEventDestroy(ctx->inv_join[g]);
    }
    if (ctx->inv_fork) (void)hipEventDestroy(ctx->inv_fork);
    if (ctx->cu_flags) (void)hipFree(ctx->cu_flags);
  }
  delete ctx;
}

const char* kfac_last_error(const kfac_ctx* ctx) { return ctx ? ctx->err.c_str() : g_noctx_err.c_str(); }

int32_t kfac_layer_dA(const kfac_layer* L) { return (L && layer_valid(*L, nullptr)) ? dA_of(*L) : 0; }
int32_t kfac_layer_dG(const kfac_layer* L) { return (L && layer_valid(*L, nullptr)) ? L->c_out : 0; }
int64_t kfac_layer_rows(const kfac_layer* L) { return (L && layer_valid(*L, nullptr)) ? rows_of(*L) : 0; }

size_t kfac_workspace_bytes_factors(const kfac_ctx* ctx, int n, const kfac_layer* layers) {
  if (n <= 0 || !layers) return 0;
  for (int l = 0; l < n; ++l)
    if (!layer_valid(layers[l], nullptr)) return 0;
  std::vector<uint8_t> present(2 * n, 1);
  return size_t(schedule_factors(n, layers, present, ctx ? factor_opts(ctx) : FactorOpts{}).stats.ws_bytes);
}

size_t kfac_workspace_bytes_invert(const kfac_ctx* ctx, int n, const int32_t* dims) {
  if (n <= 0 || !dims) return 0;
  for (int i = 0; i < n; ++i)
    if (dims[i] < 1) return 0;
  // independent of how the matrices are grouped, but not of the outer block size a group gets: the larger of the two
  const size_t a = size_t(schedule_invert(n, dims, ctx ? ctx->opt[KFAC_OPT_INV_AGG] : 4).stats.ws_bytes);
  const size_t b = size_t(schedule_invert(n, dims, ctx ? ctx->opt[KFAC_OPT_INV_AGG_CHAIN] : 6).stats.ws_bytes);
  return std::max(a, b);
}

size_t kfac_workspace_bytes_precondition(const kfac_ctx*, int n, const int32_t* dG, const int32_t* dA) {
  if (n <= 0 || !dG || !dA) return 0;
  for (int i = 0; i < n; ++i)
    if (dG[i] < 1 || dA[i] < 1) return 0;
  return size_t(schedule_precond(n, dG, dA).stats.ws_bytes);
}

kfac_status kfac_set_option(kfac_ctx* ctx, int option, int value) {
  if (!ctx) return fail(nullptr, KFAC_ERR_INVALID_ARG, "kfac_set_option: ctx is NULL");
  static const int lo[KFAC_OPT_COUNT] = {1, 1, 1, 0, 0, 0, 0, 0, KC, 0, 0, 0, 0, 0};
  static const int hi[KFAC_OPT_COUNT] = {MAX_INV_GROUPS, 16, 16, 1, 65536, 1, 1, 1, MAX_JOB_ROWS, 65536, 1, 1, 65536, 1};
  if (option < 0 || option >= KFAC_OPT_COUNT) return fail(ctx, KFAC_ERR_INVALID_ARG, "kfac_set_option: unknown option");
  if (value < lo[option] || value > hi[option])
    return fail(ctx, KFAC_ERR_INVALID_ARG, "kfac_set_option: value " + std::to_string(value) + " outside [" +
                                               std::to_string(lo[option]) + ", " + std::to_string(hi[option]) + "]");
  if (ctx->opt[option] == value) return KFAC_OK;
  ctx->opt[option] = value;
  // cached schedules were built under the old value: the next call of each kind plans again
  ctx->fp.valid = false;
  ctx->ip.valid = false;
  return KFAC_OK;
}

kfac_status kfac_get_option(const kfac_ctx* ctx, int option, int* value) {
  if (!ctx || !value || option < 0 || option >= KFAC_OPT_COUNT)
    return fail(nullptr, KFAC_ERR_INVALID_ARG, "kfac_get_option: bad arguments");
  *value = ctx->opt[option];
  return KFAC_OK;
}

void kfac_get_plan_stats(const kfac_ctx* ctx, int which, kfac_plan_stats* out) {
  if (!out) return;
  *out = kfac_plan_stats{};
  if (!ctx) return;
  if (which == 0) *out = ctx->fp.stats;
  else if (which == 1) *out = ctx->ip.stats;
  else if (which == 2) *out = ctx->pp.stats;
}

void kfac_timing_enable(kfac_ctx* ctx, uint32_t class_mask) {
  if (ctx) ctx->timing_mask = class_mask;
}

kfac_status kfac_timing_read(kfac_ctx* ctx, int kclass, double* total_ms, int64_t* n_launches, int reset) {
  if (!ctx) return fail(nullptr, KFAC_ERR_INVALID_ARG, "kfac_timing_read: ctx is NULL");
  if (kclass < 0 || kclass >= KFAC_K_COUNT) return fail(ctx, KFAC_ERR_INVALID_ARG, "kfac_timing_read: unknown kernel class");
  double sum = 0.0;
  int64_t cnt = 0;
  DeviceGuard guard(ctx);
  std::vector<TimingRec> keep;
  for (const TimingRec& r : ctx->timing) {
    if (r.kclass != kclass) { keep.push_back(r); continue; }
    HIP_TRY(ctx, hipEventSynchronize(r.b));
    float ms = 0.f;
    HIP_TRY(ctx, hipEventElapsedTime(&ms, r.a, r.b));
    sum += ms;
    ++cnt;
    if (reset) { (void)hipEventDestroy(r.a); (void)hipEventDestroy(r.b); }
    else keep.push_back(r);
  }
  ctx->timing.swap(keep);
  if (total_ms) *total_ms = sum;
  if (n_launches) *n_launches = cnt;
  return KFAC_OK;
}

// ----------------------------------------------------------------------------------- factors
// kfac_update_factors and kfac_update_factors_packed: `packed` (may be NULL) additionally receives the
// packed upper triangles of the updated factors (all A in layer order, then all G), written by the
// kernels that write the factors.
static kfac_status update_factors_impl(kfac_ctx* ctx, int n, const kfac_layer* layers,
                                       const float* const* act, const float* const* gout,
                                       float* const* A, float* const* G,
                                       float xi, float scale_a, float scale_g, float* packed, void* hip_stream) {
  if (!ctx) return fail(nullptr, KFAC_ERR_INVALID_ARG, "kfac_update_factors: ctx is NULL");
  if (n < 0) return fail(ctx, KFAC_ERR_INVALID_ARG, "kfac_update_factors: n_layers < 0");
  if (n == 0) return KFAC_OK;
  if (!layers) return fail(ctx, KFAC_ERR_INVALID_ARG, "kfac_update_factors: layers is NULL");
  if (!finite_in(xi, 0.f, 1.f)) return fail(ctx, KFAC_ERR_INVALID_ARG, "kfac_update_factors: xi must be in [0, 1]");
  if (std::isnan(scale_a) || std::isnan(scale_g) || std::isinf(scale_a) || std::isinf(scale_g))
    return fail(ctx, KFAC_ERR_INVALID_ARG, "kfac_update_factors: scale must be finite");
  std::vector<uint8_t> present(2 * n, 0);
  for (int l = 0; l < n; ++l) {
    std::string why;
    if (!layer_valid(layers[l], &why))
      return fail(ctx, KFAC_ERR_INVALID_ARG, "kfac_update_factors: layer " + std::to_string(l) + ": " + why);
    if (act && act[l]) {
      if (!A || !A[l]) return fail(ctx, KFAC_ERR_INVALID_ARG, "kfac_update_factors: act given but A is NULL for layer " + std::to_string(l));
      present[2 * l] = 1;
    }
    if (gout && gout[l]) {
      if (!G || !G[l]) return fail(ctx, KFAC_ERR_INVALID_ARG, "kfac_update_factors: gout given but G is NULL for layer " + std::to_string(l));
      present[2 * l + 1] = 1;
    }
  }

  FactorPlan& P = ctx->fp;
  const bool same = P.valid && int(P.layers.size()) == n && P.present == present &&
                    std::memcmp(P.layers.data(), layers, sizeof(kfac_layer) * n) == 0;
  DeviceGuard guard(ctx);
  if (!same) {
    FactorSchedule S = schedule_factors(n, layers, present, factor_opts(ctx));
    if (!ctx->host_only) {
      HIP_TRY(ctx, hipDeviceSynchronize());
      release(P);
    } else {
      P = FactorPlan{};
    }
    P.layers.assign(layers, layers + n);
    P.present = present;
    P.desc_of = S.desc_of;
    P.descs = S.descs;
    P.njobs = int(S.jobs.size());
    P.nrjobs = int(S.rjobs.size());
    P.nslots = S.nslots;
    P.lags = S.lags;
    P.lag_floats = S.lag_floats;
    P.nljobs = int(S.ljobs.size());
    P.npjobs = int(S.pjobs.size());
    P.stats = S.stats;
    if (!ctx->host_only) {
      kfac_status st = upload_static(ctx, &P.d_jobs, S.jobs.data(), S.jobs.size() * sizeof(TileJob));
      if (st != KFAC_OK) return st;
      st = upload_static(ctx, &P.d_rjobs, S.rjobs.data(), S.rjobs.size() * sizeof(ReduceJob));
      if (st != KFAC_OK) return st;
      st = upload_static(ctx, &P.d_ljobs, S.ljobs.data(), S.ljobs.size() * sizeof(LagJob));
      if (st == KFAC_OK) st = upload_static(ctx, &P.d_pjobs, S.pjobs.data(), S.pjobs.size() * sizeof(LagJob));
      if (st != KFAC_OK) return st;
    }
    P.valid = true;
  }
  if (ctx->host_only) return fail(ctx, KFAC_ERR_DEVICE, "host-only context: nothing launched");

  hipStream_t s = static_cast<hipStream_t>(hip_stream);
  const size_t slot_floats = P.nslots * size_t(BM) * BN;
  kfac_status st = ensure_ws(ctx, WS_FACTORS, (slot_floats + P.lag_floats) * sizeof(float));
  if (st != KFAC_OK) return st;
  float* lag_ws = static_cast<float*>(ctx->ws[WS_FACTORS]) + slot_floats;
  std::vector<size_t> packed_off(2 * size_t(n), 0);   // float offset of A_l (entry l) and G_l (entry n + l) in `packed`
  {
    size_t off = 0;
    for (int which = 0; which < 2; ++which)
      for (int l = 0; l < n; ++l) {
        const size_t d = size_t(which == 0 ? dA_of(P.layers[l]) : P.layers[l].c_out);
        packed_off[size_t(which) * n + l] = off;
        off += d * (d + 1) / 2;
      }
  }
  std::vector<uint8_t> is_lag(n, 0);
  for (const LagLayer& lg : P.lags) is_lag[lg.layer] = 1;
  for (int l = 0; l < n; ++l)
    for (int which = 0; which < 2; ++which) {
      const int di = P.desc_of[2 * l + which];
      if (di < 0 || (which == 0 && is_lag[l])) continue;
      TileDesc& D = P.descs[di];
      D.a.ptr = which == 0 ? act[l] : gout[l];
      D.b.ptr = D.a.ptr;
      D.out = which == 0 ? A[l] : G[l];
      D.packed = packed ? packed + packed_off[size_t(which) * n + l] : nullptr;
      D.partial = static_cast<float*>(ctx->ws[WS_FACTORS]);
      const float sc = which == 0 ? scale_a : scale_g;
      const float scale = sc > 0.f ? sc : float(1.0 / double(D.a.K));
      D.alpha = (1.f - xi) * scale;
      D.beta = xi;
    }
  std::vector<LagAsm> asms(P.lags.size());
  for (size_t i = 0; i < P.lags.size(); ++i) {
    const LagLayer& lg = P.lags[i];
    const kfac_layer& L = P.layers[lg.layer];
    LagAsm& Q = asms[i];
    for (int k = 0; k < LAG_NMAT; ++k) {
      TileDesc& D = P.descs[lg.desc0 + k];
      D.a.ptr = D.b.ptr = act[lg.layer];
      D.out = lag_ws + lg.off[k];
      D.partial = static_cast<float*>(ctx->ws[WS_FACTORS]);
      Q.G[k] = D.out;
    }
    const double rows = double(rows_of(L));
    Q.A = A[lg.layer];
    Q.P = packed ? packed + packed_off[lg.layer] : nullptr;
    Q.C = L.c_in; Q.bias = L.has_bias; Q.dA = dA_of(L);
    Q.alpha = (1.f - xi) * (scale_a > 0.f ? scale_a : float(1.0 / rows));
    Q.beta = xi;
    Q.rows = float(rows);
  }
  const size_t descs_bytes = P.descs.size() * sizeof(TileDesc), asms_bytes = asms.size() * sizeof(LagAsm);
  std::vector<unsigned char> img(descs_bytes + asms_bytes);
  std::memcpy(img.data(), P.descs.data(), descs_bytes);
  if (asms_bytes) std::memcpy(img.data() + descs_bytes, asms.data(), asms_bytes);
  st = sync_table(ctx, P.tab, img.data(), img.size(), s);
  if (st != KFAC_OK) return st;
  const TileDesc* d_descs = static_cast<const TileDesc*>(P.tab.dev);
  const LagAsm* d_asms = reinterpret_cast<const LagAsm*>(static_cast<const unsigned char*>(P.tab.dev) + descs_bytes);
  {
    ScopedTiming tm(ctx, KFAC_K_FACTOR_TILES, s);
    launch_tile_any(d_descs, static_cast<const TileJob*>(P.d_jobs), P.njobs, ctx->opt[KFAC_OPT_FACTOR_XCD] ? 1 : 0, s);
  }
  if (P.nrjobs || P.nljobs) {
    ScopedTiming tm(ctx, KFAC_K_FACTOR_REDUCE, s);
    launch_tile_reduce(d_descs, static_cast<const ReduceJob*>(P.d_rjobs), P.nrjobs, s);
    launch_lag_assemble(d_asms, static_cast<const LagJob*>(P.d_pjobs), P.npjobs, static_cast<const LagJob*>(P.d_ljobs), P.nljobs, s);
  }
  HIP_TRY(ctx, hipGetLastError());
  return KFAC_OK;
}

kfac_status kfac_update_factors(kfac_ctx* ctx, int n, const kfac_layer* layers,
                                const float* const* act, const float* const* gout,
                                float* const* A, float* const* G,
                                float xi, float scale_a, float scale_g, void* hip_stream) {
  return update_factors_impl(ctx, n, layers, act, gout, A, G, xi, scale_a, scale_g, nullptr, hip_stream);
}

kfac_status kfac_update_factors_packed(kfac_ctx* ctx, int n, const kfac_layer* layers,
                                       const float* const* act, const float* const* gout,
                                       float* const* A, float* const* G,
                                       float xi, float scale_a, float scale_g, float* packed, void* hip_stream) {
  if (ctx && n > 0 && !packed) return fail(ctx, KFAC_ERR_INVALID_ARG, "kfac_update_factors_packed: packed is NULL");
  return update_factors_impl(ctx, n, layers, act, gout, A, G, xi, scale_a, scale_g, packed, hip_stream);
}

// ----------------------------------------------------------------------------------- inverse
// kfac_invert_batch and kfac_invert_batch_packed: `packed` (may be NULL) additionally receives the
// packed upper triangles of the inverses, written by the kernels that write the inverses.
static kfac_status invert_batch_impl(kfac_ctx* ctx, int n, const int32_t* dims, const float* const* F,
                                     float* const* X, float gamma, int32_t* info_dev, float* packed, void* hip_stream) {
  if (!ctx) return fail(nullptr, KFAC_ERR_INVALID_ARG, "kfac_invert_batch: ctx is NULL");
  if (n < 0) return fail(ctx, KFAC_ERR_INVALID_ARG, "kfac_invert_batch: n_mats < 0");
  if (n == 0) return KFAC_OK;
  if (!dims || !F || !X) return fail(ctx, KFAC_ERR_INVALID_ARG, "kfac_invert_batch: dims, F or X is NULL");
  if (!(gamma >= 0.f) || std::isinf(gamma)) return fail(ctx, KFAC_ERR_INVALID_ARG, "kfac_invert_batch: gamma must be finite and >= 0");
  for (int i = 0; i < n; ++i) {
    if (dims[i] < 1 || dims[i] > 16384)   // sweep panels are addressed with 32-bit byte offsets (1 GiB)
      return fail(ctx, KFAC_ERR_INVALID_ARG, "kfac_invert_batch: dims[" + std::to_string(i) + "] out of range");
    if (!F[i] || !X[i]) return fail(ctx, KFAC_ERR_INVALID_ARG, "kfac_invert_batch: NULL matrix pointer at " + std::to_string(i));
    if (F[i] == X[i]) return fail(ctx, KFAC_ERR_INVALID_ARG, "kfac_invert_batch: X must not alias F at " + std::to_string(i));
  }

  InvertPlan& P = ctx->ip;
  const bool same = P.valid && int(P.dims.size()) == n && std::memcmp(P.dims.data(), dims, sizeof(int32_t) * n) == 0;
  DeviceGuard guard(ctx);
  if (!same) {
    if (!ctx->host_only) {
      HIP_TRY(ctx, hipDeviceSynchronize());
      release(P);
    } else {
      P = InvertPlan{};
    }
    P.dims.assign(dims, dims + n);
    // Placement of the matrices on the lockstep groups.  The matrices with the longest chains (more
    // than 0.6 of the largest number of pivot blocks) form group 0: they decide how long the call
    // takes, and kept apart they are not held back by the steps of the many shorter matrices, whose
    // groups finish early and fill the machine meanwhile.  The other matrices are spread over the
    // remaining groups by the paper's Algorithm 1 without its communication term and with the true
    // cost d^3 as weight: largest first, each to the lightest group.  Matrices that fit one pivot
    // block (d <= NB) need a single launch and all go to the last group.
    std::vector<int> by_size(n);
    for (int i = 0; i < n; ++i) by_size[i] = i;
    std::stable_sort(by_size.begin(), by_size.end(), [&](int a, int b) { return dims[a] > dims[b]; });
    int n_large = 0, max_nblk = 0, n_long = 0;
    for (int i = 0; i < n; ++i)
      if (dims[i] > NB) { ++n_large; max_nblk = std::max(max_nblk, ceil_div(dims[i], NB)); }
    auto is_long = [&](int i) { return dims[i] > NB && 5 * ceil_div(dims[i], NB) > 3 * max_nblk; };
    for (int i = 0; i < n; ++i) n_long += is_long(i);
    const int G = std::max(1, std::min(ctx->opt[KFAC_OPT_INV_GROUPS], n_large));
    const bool split = ctx->opt[KFAC_OPT_INV_SPLIT_LONG] && G >= 2 && n_long > 0 && n_long < n_large;   // otherwise: plain balancing over all groups
    P.groups.assign(G, InvertGroup{});
    std::vector<double> load(G, 0.0);
    for (int i : by_size) {
      int g = split ? G - 1 : 0;   // matrices of one pivot block: a single launch, kept off the long chain
      if (dims[i] > NB) {
        if (split) g = is_long(i) ? 0 : 1 + int(std::min_element(load.begin() + 1, load.end()) - (load.begin() + 1));
        else g = int(std::min_element(load.begin(), load.end()) - load.begin());
      }
      P.groups[g].idx.push_back(i);
      load[g] += double(dims[i]) * dims[i] * dims[i];
    }
    P.ws_floats = 0;
    P.stats = kfac_plan_stats{};
    for (InvertGroup& Gp : P.groups) {
      std::vector<int32_t> gd;
      for (int i : Gp.idx) gd.push_back(dims[i]);
      // Outer block size of the group.  A group whose longest chain of dependent launches outlasts
      // its arithmetic is latency-bound and gets the larger outer blocks (fewer outer steps, more
      // of the work in the diagonal sub-matrix sweeps); a throughput-bound group keeps the smaller
      // ones, whose rank-128 sub-updates are a smaller share of the work.  Estimates from timings
      // on MI355X: 90 us per pivot block, 300 us per outer block, 100 TFLOP/s for the products.
      {
        double flops = 0.0, chain = 0.0;
        for (int32_t d : gd) {
          if (d <= NB) continue;
          flops += double(d) * d * d;
          chain = std::max(chain, ceil_div(d, NB) * 90e-6 + inv_nob(d, ctx->opt[KFAC_OPT_INV_AGG]) * 300e-6);
        }
        Gp.latency_bound = chain > flops / 100e12;
        Gp.agg = Gp.latency_bound ? ctx->opt[KFAC_OPT_INV_AGG_CHAIN] : ctx->opt[KFAC_OPT_INV_AGG];
      }
      InvertSchedule S = schedule_invert(int(gd.size()), gd.data(), Gp.agg, ctx->opt[KFAC_OPT_INV_FUSE] != 0);
      Gp.order = S.order; Gp.n_large = S.n_large; Gp.n_small = S.n_small; Gp.n_ob = S.n_ob; Gp.n_views = S.n_views;
      Gp.view_off = S.view_off; Gp.n_in_ob = S.n_in_ob; Gp.sub_pivot_off = S.sub_pivot_off;
      Gp.sub_panel_off = S.sub_panel_off; Gp.sub_upd_off = S.sub_upd_off;
      Gp.qm_off = S.qm_off; Gp.mv_off = S.mv_off; Gp.bp_off = S.bp_off; Gp.mv_mid = S.mv_mid; Gp.bp_mid = S.bp_mid;
      for (int k = 0; k < 3; ++k) Gp.upd_off[k] = S.upd_off[k];
      Gp.cq_bp_off = S.cq_bp_off; Gp.cq_bp_end = S.cq_bp_end; Gp.cq_diag_end = S.cq_diag_end;
      Gp.ws_off = S.ws_off;
      Gp.ev_chain.assign(S.n_ob, nullptr); Gp.ev_col.assign(S.n_ob, nullptr); Gp.ev_rest.assign(S.n_ob, nullptr);
      Gp.ev_gather.assign(S.n_ob, nullptr);
      Gp.n_init = int(S.init.size()); Gp.n_init_first = S.n_init_first; Gp.n_finish = int(S.finish.size());
      Gp.ws_floats = S.ws_floats;
      Gp.ws_base = P.ws_floats;
      P.ws_floats += S.ws_floats;
      P.stats.n_jobs += S.stats.n_jobs; P.stats.n_launches += S.stats.n_launches;
      P.stats.mfma_flops += S.stats.mfma_flops; P.stats.ws_bytes += S.stats.ws_bytes;
      if (!ctx->host_only) {
        kfac_status st;
        auto up = [&](void** dev, const void* src, size_t bytes) { return upload_static(ctx, dev, src, bytes); };
        if ((st = up(&Gp.d_init, S.init.data(), S.init.size() * sizeof(MatJobH))) != KFAC_OK) return st;
        if ((st = up(&Gp.d_finish, S.finish.data(), S.finish.size() * sizeof(MatJobH))) != KFAC_OK) return st;
        if ((st = up(&Gp.d_sub_pivot, S.sub_pivot.data(), S.sub_pivot.size() * sizeof(MatJobH))) != KFAC_OK) return st;
        if ((st = up(&Gp.d_sub_panel, S.sub_panel.data(), S.sub_panel.size() * sizeof(MatJobH))) != KFAC_OK) return st;
        if ((st = up(&Gp.d_sub_upd, S.sub_upd.data(), S.sub_upd.size() * sizeof(TileJob))) != KFAC_OK) return st;
        if ((st = up(&Gp.d_qm, S.qm.data(), S.qm.size() * sizeof(MatJobH))) != KFAC_OK) return st;
        if ((st = up(&Gp.d_mv, S.mv.data(), S.mv.size() * sizeof(MatJobH))) != KFAC_OK) return st;
        if ((st = up(&Gp.d_bp, S.bp.data(), S.bp.size() * sizeof(TileJob))) != KFAC_OK) return st;
        for (int k = 0; k < 3; ++k)
          if ((st = up(&Gp.d_upd[k], S.upd[k].data(), S.upd[k].size() * sizeof(TileJob))) != KFAC_OK) return st;
        if ((st = up(&Gp.d_chain_q, S.chain_q.data(), S.chain_q.size() * sizeof(TileJob))) != KFAC_OK) return st;
      }
    }
    P.valid = true;
  }
  if (ctx->host_only) return fail(ctx, KFAC_ERR_DEVICE, "host-only context: nothing launched");

  std::vector<size_t> packed_off(n, 0);   // float offset of matrix i's triangle in `packed`
  for (int i = 1; i < n; ++i) packed_off[i] = packed_off[i - 1] + size_t(dims[i - 1]) * (size_t(dims[i - 1]) + 1) / 2;
  hipStream_t s = static_cast<hipStream_t>(hip_stream);
  kfac_status st = ensure_ws(ctx, WS_INVERT, P.ws_floats * sizeof(float));
  if (st != KFAC_OK) return st;
  const int G = int(P.groups.size());
  if (!ctx->cu_flags) {   // once per context: zeroed here, and every kernel that counts itself in also counts itself out
#ifdef KFAC_TRACE
    const size_t flag_bytes = sizeof(int) * (cu_flag_slots() + 2) + size_t(60000) * 64;
#else
    const size_t flag_bytes = sizeof(int) * cu_flag_slots();
#endif
    HIP_TRY(ctx, hipMalloc(reinterpret_cast<void**>(&ctx->cu_flags), flag_bytes));
    HIP_TRY(ctx, hipMemset(ctx->cu_flags, 0, flag_bytes));
  }
  const int yield_max = ctx->opt[KFAC_OPT_INV_YIELD];
  int* const yflags = yield_max > 0 ? ctx->cu_flags : nullptr;
  auto crit = [&](int nwg) { return nwg <= yield_max ? yflags : nullptr; };   // few workgroups: latency-critical
  // deep: the group's products run one workgroup to a compute unit (latency-bound group) and take the
  // 32-deep panels; the padding option counts from the 16-deep kernel's footprint
  auto bulk_gemm = [&](const TileDesc* dd, const TileJob* jj, int cnt, int pad, bool deep, hipStream_t st) {
    launch_tile_gemm_yield(dd, jj, cnt, deep ? std::max(0, pad - deep_lds_extra()) : pad, yflags, deep, st);
  };

  // Group 0 sweeps on the caller's stream; every further group on an internal stream forked from
  // it and joined back with events.  Each group also has a side stream for its off-chain updates.
  // All internal streams have the default priority.
  if (G > 1 && !ctx->inv_fork) HIP_TRY(ctx, hipEventCreateWithFlags(&ctx->inv_fork, hipEventDisableTiming));
  for (int g = 0; g < G; ++g) {
    if (g > 0 && !ctx->inv_stream[g]) HIP_TRY(ctx, hipStreamCreateWithFlags(&ctx->inv_stream[g], hipStreamNonBlocking));
    if (g > 0 && !ctx->inv_join[g]) HIP_TRY(ctx, hipEventCreateWithFlags(&ctx->inv_join[g], hipEventDisableTiming));
    if (!ctx->inv_side[g]) HIP_TRY(ctx, hipStreamCreateWithFlags(&ctx->inv_side[g], hipStreamNonBlocking));
  }
  if (G > 1) {
    HIP_TRY(ctx, hipEventRecord(ctx->inv_fork, s));
    for (int g = 1; g < G; ++g) HIP_TRY(ctx, hipStreamWaitEvent(ctx->inv_stream[g], ctx->inv_fork, 0));
  }
  auto gstream = [&](int g) { return g > 0 ? ctx->inv_stream[g] : s; };

  // per-call tables of every group: [InvMat x n_g][InvMat x views][PanelMove x 2 views][TileDesc x (2 views + n_large)]
  std::vector<const InvMat*> d_mats(G), d_views(G);
  std::vector<const PanelMove*> d_moves(G);
  std::vector<const TileDesc*> d_descs(G);
  float* wsf = static_cast<float*>(ctx->ws[WS_INVERT]);
  for (int g = 0; g < G; ++g) {
    InvertGroup& Gp = P.groups[g];
    const int agg = Gp.agg, aw = agg + 1;
    const int ng = int(Gp.idx.size()), nv = Gp.n_views;
    const size_t mats_bytes = sizeof(InvMat) * size_t(ng);
    const size_t views_bytes = sizeof(InvMat) * size_t(nv);
    const size_t moves_bytes = sizeof(PanelMove) * size_t(2 * nv);
    const size_t descs_bytes = sizeof(TileDesc) * size_t(2 * nv + Gp.n_large);
    const size_t tab_bytes = mats_bytes + views_bytes + moves_bytes + descs_bytes;
    std::vector<unsigned char> img(tab_bytes, 0);
    InvMat* hm = reinterpret_cast<InvMat*>(img.data());
    InvMat* hv = reinterpret_cast<InvMat*>(img.data() + mats_bytes);
    PanelMove* hp = reinterpret_cast<PanelMove*>(img.data() + mats_bytes + views_bytes);
    TileDesc* hd = reinterpret_cast<TileDesc*>(img.data() + mats_bytes + views_bytes + moves_bytes);
    for (int m = 0; m < ng; ++m) {
      const int o = Gp.idx[Gp.order[m]];
      InvMat& M = hm[m];
      M.F = F[o]; M.X = X[o]; M.d = M.ld = dims[o];
      M.info = info_dev ? info_dev + o : nullptr;
      M.P = packed ? packed + packed_off[o] : nullptr;
      M.xelems = uint32_t(M.d) * uint32_t(M.d);
      M.ldp = NB;
      if (m >= Gp.n_large) continue;
      const int d = M.d, nblk = ceil_div(d, NB), ldp = nblk * NB, nob = inv_nob(d, agg);
      const InvWsLayout L = inv_ws_layout(ldp, agg);
      float* base = wsf + Gp.ws_base + Gp.ws_off[m];
      M.ldp = ldp;
      TileDesc& DU = hd[2 * nv + m];    // step 4: X -= Wt^T Zt over one half of the panel buffers
      DU.a = rowmajor_operand(base + L.wt, 2 * aw * NB, ldp, ldp);
      DU.b = rowmajor_operand(base + L.zt, 2 * aw * NB, ldp, ldp);
      DU.out = M.X; DU.ldo = d; DU.M = DU.N = d;
      DU.sym = 1; DU.mirror = MIRROR_DIAG_TILE; DU.alpha = -1.f; DU.beta = 1.f;
      for (int b = 0; b < nob; ++b) {
        const int v = Gp.view_off[b] + m;
        const int c0 = b * agg * NB, dimB = std::min(d, inv_ob_end(d, agg, b) * NB) - c0, half = b & 1;
        InvMat& V = hv[v];              // step 1: the diagonal sub-matrix as a matrix of its own
        V.F = nullptr; V.X = M.X + size_t(c0) * d + c0; V.d = dimB; V.ld = d; V.ldp = aw * NB;
        V.Wt = base + L.swt; V.Zt = base + L.szt; V.Q = base + L.q; V.QB = base + L.qb;
        V.info = M.info; V.info_base = c0;
        V.xelems = uint32_t(size_t(d) * d - (size_t(c0) * d + c0));
        TileDesc& DS = hd[v];
        DS.a = rowmajor_operand(V.Wt, NB, aw * NB, aw * NB);
        DS.b = rowmajor_operand(V.Zt, NB, aw * NB, aw * NB);
        DS.out = V.X; DS.ldo = d; DS.M = DS.N = dimB;
        DS.sym = 1; DS.mirror = MIRROR_DIAG_TILE; DS.alpha = -1.f; DS.beta = 1.f;
        float* wt_half = base + L.wt + size_t(half) * aw * NB * ldp;
        float* zt_half = base + L.zt + size_t(half) * aw * NB * ldp;
        hp[2 * v] = PanelMove{M.X, zt_half, d, ldp, c0, dimB};       // step 2: gather Z
        hp[2 * v + 1] = PanelMove{M.X, wt_half, d, ldp, c0, dimB};   // step 3: scatter W
        TileDesc& DP = hd[nv + v];      // step 3: Wt = QB Zt
        DP.a = rowmajor_operand(V.QB, dimB, dimB, aw * NB);
        DP.b = rowmajor_operand(zt_half, dimB, ldp, ldp);
        DP.out = wt_half; DP.ldo = ldp; DP.M = dimB; DP.N = ldp;
        DP.sym = 0; DP.mirror = MIRROR_NONE; DP.alpha = 1.f; DP.beta = 0.f;
      }
    }
    st = sync_table(ctx, Gp.tab, img.data(), tab_bytes, gstream(g));
    if (st != KFAC_OK) return st;
    const unsigned char* dev = static_cast<const unsigned char*>(Gp.tab.dev);
    d_mats[g] = reinterpret_cast<const InvMat*>(dev);
    d_views[g] = reinterpret_cast<const InvMat*>(dev + mats_bytes);
    d_moves[g] = reinterpret_cast<const PanelMove*>(dev + mats_bytes + views_bytes);
    d_descs[g] = reinterpret_cast<const TileDesc*>(dev + mats_bytes + views_bytes + moves_bytes);
  }

  int max_ob = 0;
  for (int g = 0; g < G; ++g) {
    InvertGroup& Gp = P.groups[g];
    hipStream_t gs = gstream(g);
    max_ob = std::max(max_ob, Gp.n_ob);
    if (Gp.n_small) {
      ScopedTiming tm(ctx, KFAC_K_INV_SMALL, gs);
      launch_gj_pivot(d_mats[g], nullptr, Gp.n_large, Gp.n_small, 0, gamma, 1, gs);
    }
    if (Gp.n_large) {
      ScopedTiming tm(ctx, KFAC_K_INV_INIT, gs);
      launch_gj_init(d_mats[g], Gp.d_init, Gp.n_init_first, gamma, gs);
    }
    if (Gp.n_init > Gp.n_init_first) {   // the other tiles: on the side stream, beside the first diagonal sweep
      hipStream_t side = ctx->opt[KFAC_OPT_INV_SIDE] ? ctx->inv_side[g] : gs;
      if (!Gp.ev_start) HIP_TRY(ctx, hipEventCreateWithFlags(&Gp.ev_start, hipEventDisableTiming));
      if (!Gp.ev_init) HIP_TRY(ctx, hipEventCreateWithFlags(&Gp.ev_init, hipEventDisableTiming));
      HIP_TRY(ctx, hipEventRecord(Gp.ev_start, gs));
      HIP_TRY(ctx, hipStreamWaitEvent(side, Gp.ev_start, 0));
      {
        ScopedTiming tm(ctx, KFAC_K_INV_INIT, side);
        launch_gj_init(d_mats[g], static_cast<const MatJobH*>(Gp.d_init) + Gp.n_init_first, Gp.n_init - Gp.n_init_first, gamma, side);
      }
      HIP_TRY(ctx, hipEventRecord(Gp.ev_init, side));
    }
  }
  // The groups are issued outer block by outer block so that their kernels interleave in time.
  // Chain of a group (its main stream), per outer block b: sweep of the diagonal sub-matrix, QB,
  // gather of the block column, then only what the next diagonal sub-matrix needs: panel product
  // for the rows of the next outer block, update of the next diagonal sub-matrix.
  // Side stream: panel product for all other rows, every scatter, then the other two update lists.
  // Cross-stream order, by what the kernels touch:
  //   QB(b), gather(b)   rewrite QB, which the side's panel product (b-1) reads, and read tiles
  //                      that UPD_COL(b-1) wrote                        -> chain waits for ev_col[b-1]
  //   UPD_DIAG(b)        writes tiles that UPD_REST(b-1) also updates; gather(b+1) and the panel
  //                      products (b+1) reuse the buffer half it reads   -> chain waits for ev_rest[b-1]
  //   side panel product reads QB(b) and the gathered column            -> side waits for ev_gather[b]
  //   UPD_COL/REST(b)    read the chain's part of the W panel           -> side waits for ev_chain[b]
  std::vector<int> last_col(G, -1), last_rest(G, -1);    // outer block of the group's latest side-stream work
  auto ensure_event = [&](hipEvent_t& e) { return e ? hipSuccess : hipEventCreateWithFlags(&e, hipEventDisableTiming); };
  auto upd_launch = [&](int g, int kind, int b, hipStream_t st, int pad = 0) {
    InvertGroup& Gp = P.groups[g];
    const int o0 = Gp.upd_off[kind][b], cnt = Gp.upd_off[kind][b + 1] - o0;
    if (cnt <= 0) return;
    ScopedTiming tm(ctx, KFAC_K_INV_UPDATE, st);
    bulk_gemm(d_descs[g], static_cast<const TileJob*>(Gp.d_upd[kind]) + o0, cnt, pad, Gp.latency_bound, st);
  };
  for (int b = 0; b < max_ob; ++b)
    for (int g = 0; g < G; ++g) {
      InvertGroup& Gp = P.groups[g];
      if (b >= Gp.n_ob) continue;
      hipStream_t gs = gstream(g), side = ctx->opt[KFAC_OPT_INV_SIDE] ? ctx->inv_side[g] : gs;
      const InvMat* views = d_views[g];
      const int side_pad = Gp.latency_bound ? ctx->opt[KFAC_OPT_INV_SIDE_PAD] : 0;
      const int chain_pad = Gp.latency_bound ? ctx->opt[KFAC_OPT_INV_CHAIN_PAD] : 0;
      const int aw = Gp.agg + 1;
      // Sweep of the diagonal sub-matrices: pivot block t, its panel, then ONE launch holding both
      // the update by block t of every tile but the next pivot block and the sweep of pivot block
      // t + 1 (which applies that update to itself): the two are independent.
      for (int t = 0; t < aw; ++t) {
        const int stp = b * aw + t;
        const int npiv = Gp.sub_pivot_off[stp + 1] - Gp.sub_pivot_off[stp];
        if (npiv == 0) break;
        if (t == 0 || !ctx->opt[KFAC_OPT_INV_FUSE]) {
          ScopedTiming tm(ctx, KFAC_K_INV_PIVOT, gs);
          launch_gj_pivot(views, static_cast<const MatJobH*>(Gp.d_sub_pivot) + Gp.sub_pivot_off[stp], 0, npiv, t, gamma, 0, gs, chain_pad, crit(npiv));
        }
        if (Gp.sub_panel_off[stp + 1] > Gp.sub_panel_off[stp]) {
          ScopedTiming tm(ctx, KFAC_K_INV_PANEL, gs);
          launch_gj_panel(views, static_cast<const MatJobH*>(Gp.d_sub_panel) + Gp.sub_panel_off[stp],
                          Gp.sub_panel_off[stp + 1] - Gp.sub_panel_off[stp], t, gs, chain_pad,
                          crit(Gp.sub_panel_off[stp + 1] - Gp.sub_panel_off[stp]));
        }
        const int npiv_next = t + 1 < aw ? Gp.sub_pivot_off[stp + 2] - Gp.sub_pivot_off[stp + 1] : 0;
        const int nupd = Gp.sub_upd_off[stp + 1] - Gp.sub_upd_off[stp];
        const TileJob* uj = static_cast<const TileJob*>(Gp.d_sub_upd) + Gp.sub_upd_off[stp];
        if (ctx->opt[KFAC_OPT_INV_FUSE] && npiv_next > 0) {
          ScopedTiming tm(ctx, KFAC_K_INV_PIVOT, gs);
          launch_gj_pivot_update(views, static_cast<const MatJobH*>(Gp.d_sub_pivot) + Gp.sub_pivot_off[stp + 1], npiv_next, t + 1, gamma,
                                 d_descs[g], uj, nupd, gs, chain_pad, yflags, npiv_next <= yield_max);
        } else if (nupd > 0) {
          ScopedTiming tm(ctx, KFAC_K_INV_UPDATE, gs);
          bulk_gemm(d_descs[g], uj, nupd, chain_pad, Gp.latency_bound, gs);
        }
      }
      const MatJobH* mvj = static_cast<const MatJobH*>(Gp.d_mv);
      const TileJob* bpj = static_cast<const TileJob*>(Gp.d_bp);
      const TileJob* cqj = static_cast<const TileJob*>(Gp.d_chain_q);
      // only the group of the longest chains: its few tiles are what the call waits for; the other groups' chain
      // products are hundreds of tiles, which fill the machine as they are
      const bool quarter = ctx->opt[KFAC_OPT_INV_QUARTER] != 0 && g == 0 && Gp.latency_bound;
      const int mv0 = Gp.mv_off[b], mv1 = Gp.mv_mid[b], mv2 = Gp.mv_off[b + 1];
      const int bp0 = Gp.bp_off[b], bp1 = Gp.bp_mid[b], bp2 = Gp.bp_off[b + 1];
      const int kch = aw * NB / 32;
      const bool has_panel = Gp.qm_off[b + 1] > Gp.qm_off[b];
      if (has_panel) {
        if (b == 0 && Gp.n_init > Gp.n_init_first) HIP_TRY(ctx, hipStreamWaitEvent(gs, Gp.ev_init, 0));   // first touch of tiles outside D_0
        if (last_col[g] >= 0) HIP_TRY(ctx, hipStreamWaitEvent(gs, Gp.ev_col[last_col[g]], 0));
        {
          ScopedTiming tm(ctx, KFAC_K_INV_PANEL, gs);
          launch_gj_qmirror(views, static_cast<const MatJobH*>(Gp.d_qm) + Gp.qm_off[b], Gp.qm_off[b + 1] - Gp.qm_off[b], gs);
          launch_gj_move(d_moves[g], mvj + mv0, mv2 - mv0, kch, 0, gs);
        }
        HIP_TRY(ctx, ensure_event(Gp.ev_gather[b]));
        HIP_TRY(ctx, hipEventRecord(Gp.ev_gather[b], gs));
        if (bp1 > bp0) {
          ScopedTiming tm(ctx, KFAC_K_INV_PANEL, gs);
          if (quarter) launch_tile_gemm_quarter(d_descs[g], cqj + Gp.cq_bp_off[b], Gp.cq_bp_end[b] - Gp.cq_bp_off[b], Gp.latency_bound ? yflags : nullptr, gs);
          else bulk_gemm(d_descs[g], bpj + bp0, bp1 - bp0, chain_pad, Gp.latency_bound, gs);
        }
        if (bp1 > bp0) {   // the chain wrote part of the W panel
          HIP_TRY(ctx, ensure_event(Gp.ev_chain[b]));
          HIP_TRY(ctx, hipEventRecord(Gp.ev_chain[b], gs));
        }
      }
      const bool has_diag = Gp.upd_off[UPD_DIAG][b + 1] > Gp.upd_off[UPD_DIAG][b];
      const bool has_col = Gp.upd_off[UPD_COL][b + 1] > Gp.upd_off[UPD_COL][b];
      const bool has_rest = Gp.upd_off[UPD_REST][b + 1] > Gp.upd_off[UPD_REST][b];
      if (has_diag) {
        if (last_rest[g] >= 0) HIP_TRY(ctx, hipStreamWaitEvent(gs, Gp.ev_rest[last_rest[g]], 0));
        if (quarter) {
          ScopedTiming tm(ctx, KFAC_K_INV_UPDATE, gs);
          launch_tile_gemm_quarter(d_descs[g], cqj + Gp.cq_bp_end[b], Gp.cq_diag_end[b] - Gp.cq_bp_end[b], Gp.latency_bound ? yflags : nullptr, gs);
        } else {
          upd_launch(g, UPD_DIAG, b, gs, chain_pad);
        }
      }
      if (!has_panel) continue;
      HIP_TRY(ctx, hipStreamWaitEvent(side, Gp.ev_gather[b], 0));
      if (bp2 > bp1) {
        ScopedTiming tm(ctx, KFAC_K_INV_PANEL, side);
        bulk_gemm(d_descs[g], bpj + bp1, bp2 - bp1, side_pad, Gp.latency_bound, side);
        launch_gj_move(d_moves[g] + 1, mvj + mv1, mv2 - mv1, kch, 1, side);
      }
      if (bp1 > bp0) {
        HIP_TRY(ctx, hipStreamWaitEvent(side, Gp.ev_chain[b], 0));
        // its scatter into the matrix is read by nothing before the next outer block's gather
        // (which waits for ev_col[b]), so it leaves the chain
        ScopedTiming tm(ctx, KFAC_K_INV_PANEL, side);
        launch_gj_move(d_moves[g] + 1, mvj + mv0, mv1 - mv0, kch, 1, side);
      }
      upd_launch(g, UPD_COL, b, side, side_pad);
      HIP_TRY(ctx, ensure_event(Gp.ev_col[b]));
      HIP_TRY(ctx, hipEventRecord(Gp.ev_col[b], side));
      last_col[g] = b;
      if (has_rest) {
        upd_launch(g, UPD_REST, b, side, side_pad);
        HIP_TRY(ctx, ensure_event(Gp.ev_rest[b]));
        HIP_TRY(ctx, hipEventRecord(Gp.ev_rest[b], side));
        last_rest[g] = b;
      }
      (void)has_col;
    }
  for (int g = 0; g < G; ++g)   // everything on the side stream must be done before the finish
    if (last_col[g] >= 0) HIP_TRY(ctx, hipStreamWaitEvent(gstream(g), P.groups[g].ev_col[last_col[g]], 0));
  for (int g = 0; g < G; ++g) {
    InvertGroup& Gp = P.groups[g];
    if (!Gp.n_large) continue;
    if (last_rest[g] >= 0) HIP_TRY(ctx, hipStreamWaitEvent(gstream(g), Gp.ev_rest[last_rest[g]], 0));
    ScopedTiming tm(ctx, KFAC_K_INV_FINISH, gstream(g));
    launch_gj_finish(d_mats[g], Gp.d_finish, Gp.n_finish, gstream(g));
  }
  for (int g = 1; g < G; ++g) {
    HIP_TRY(ctx, hipEventRecord(ctx->inv_join[g], ctx->inv_stream[g]));
    HIP_TRY(ctx, hipStreamWaitEvent(s, ctx->inv_join[g], 0));
  }
  HIP_TRY(ctx, hipGetLastError());
  return KFAC_OK;
}

#ifdef KFAC_TRACE
extern "C" int kfac_debug_trace(kfac_ctx* ctx, long long* out, int max_recs, int reset) {
  if (!ctx || !ctx->cu_flags) return 0;
  (void)hipDeviceSynchronize();
  int n = 0;
  (void)hipMemcpy(&n, ctx->cu_flags + cu_flag_slots(), sizeof(int), hipMemcpyDeviceToHost);
  if (n > 60000) n = 60000;
  if (n > max_recs) n = max_recs;
  if (out && n > 0) (void)hipMemcpy(out, ctx->cu_flags + cu_flag_slots() + 2, size_t(n) * 64, hipMemcpyDeviceToHost);
  if (reset) (void)hipMemset(ctx->cu_flags + cu_flag_slots(), 0, sizeof(int));
  return n;
}
#endif

kfac_status kfac_invert_batch(kfac_ctx* ctx, int n, const int32_t* dims, const float* const* F,
                              float* const* X, float gamma, int32_t* info_dev, void* hip_stream) {
  return invert_batch_impl(ctx, n, dims, F, X, gamma, info_dev, nullptr, hip_stream);
}

kfac_status kfac_invert_batch_packed(kfac_ctx* ctx, int n, const int32_t* dims, const float* const* F,
                                     float* const* X, float* packed, float gamma, int32_t* info_dev, void* hip_stream) {
  if (ctx && n > 0 && !packed) return fail(ctx, KFAC_ERR_INVALID_ARG, "kfac_invert_batch_packed: packed is NULL");
  return invert_batch_impl(ctx, n, dims, F, X, gamma, info_dev, packed, hip_stream);
}

// ----------------------------------------------------------------------------- placement
kfac_status kfac_place_inversions(int n, const int32_t* dims, int n_workers, const kfac_cost_model* model,
                                  int32_t* owner, double* overall_time) {
  if (n < 0) return fail(nullptr, KFAC_ERR_INVALID_ARG, "kfac_place_inversions: n_mats < 0");
  if (n_workers < 1) return fail(nullptr, KFAC_ERR_INVALID_ARG, "kfac_place_inversions: n_workers < 1");
  if (!model) return fail(nullptr, KFAC_ERR_INVALID_ARG, "kfac_place_inversions: model is NULL");
  const double coef[4] = {model->alpha_inv, model->beta_inv, model->alpha_bcast, model->beta_bcast};
  for (double c : coef)
    if (!(c >= 0.0) || std::isinf(c)) return fail(nullptr, KFAC_ERR_INVALID_ARG, "kfac_place_inversions: coefficients must be finite and >= 0");
  if (model->weight_power < 1 || model->weight_power > 3)
    return fail(nullptr, KFAC_ERR_INVALID_ARG, "kfac_place_inversions: weight_power must be 1, 2 or 3");
  if (n == 0) {
    if (overall_time) *overall_time = 0.0;
    return KFAC_OK;
  }
  if (!dims || !owner) return fail(nullptr, KFAC_ERR_INVALID_ARG, "kfac_place_inversions: dims or owner is NULL");
  for (int i = 0; i < n; ++i)
    if (dims[i] < 1) return fail(nullptr, KFAC_ERR_INVALID_ARG, "kfac_place_inversions: dims[" + std::to_string(i) + "] < 1");
  auto comp = [&](int d) { return model->alpha_inv * std::exp(model->beta_inv * double(d)); };
  auto comm = [&](int d) { return model->alpha_bcast + model->beta_bcast * (double(d) * (double(d) + 1.0) / 2.0); };
  std::vector<int> order(n);
  for (int i = 0; i < n; ++i) order[i] = i;
  std::stable_sort(order.begin(), order.end(), [&](int a, int b) { return dims[a] > dims[b]; });
  std::vector<double> bucket(n_workers, 0.0), busy(n_workers, 0.0);
  for (int i : order) {
    const double w = std::pow(double(dims[i]), double(model->weight_power));
    if (comp(dims[i]) < comm(dims[i])) {
      owner[i] = -1;
      for (int p = 0; p < n_workers; ++p) { bucket[p] += w; busy[p] += comp(dims[i]); }
    } else {
      const int p = int(std::min_element(bucket.begin(), bucket.end()) - bucket.begin());
      owner[i] = p;
      bucket[p] += w;
      busy[p] += comp(dims[i]) + comm(dims[i]);
    }
  }
  if (overall_time) *overall_time = *std::max_element(busy.begin(), busy.end());
  return KFAC_OK;
}

// ----------------------------------------------------------------------------- packed triangles
size_t kfac_packed_elems(int n, const int32_t* dims, int64_t* offsets) {
  if (n <= 0 || !dims) return 0;
  size_t tot = 0;
  for (int i = 0; i < n; ++i) {
    if (dims[i] < 1) return 0;
    if (offsets) offsets[i] = int64_t(tot);
    tot += size_t(dims[i]) * (size_t(dims[i]) + 1) / 2;
  }
  if (offsets) offsets[n] = int64_t(tot);
  return tot;
}

namespace {
kfac_status pack_call(kfac_ctx* ctx, const char* who, int n, const int32_t* dims, const float* const* M,
                      const float* packed, int to_full, void* hip_stream) {
  const std::string name(who);
  if (!ctx) return fail(nullptr, KFAC_ERR_INVALID_ARG, name + ": ctx is NULL");
  if (n < 0) return fail(ctx, KFAC_ERR_INVALID_ARG, name + ": n_mats < 0");
  if (n == 0) return KFAC_OK;
  if (!dims || !M || !packed) return fail(ctx, KFAC_ERR_INVALID_ARG, name + ": dims, M or packed is NULL");
  for (int i = 0; i < n; ++i) {
    if (dims[i] < 1 || dims[i] > 46340)   // element offsets inside one matrix stay below 2^31
      return fail(ctx, KFAC_ERR_INVALID_ARG, name + ": dims[" + std::to_string(i) + "] out of range");
    if (!M[i]) return fail(ctx, KFAC_ERR_INVALID_ARG, name + ": NULL matrix pointer at " + std::to_string(i));
  }
  PackPlan& P = ctx->kp;
  const bool same = P.valid && int(P.dims.size()) == n && std::memcmp(P.dims.data(), dims, sizeof(int32_t) * n) == 0;
  DeviceGuard guard(ctx);
  if (!same) {
    if (!ctx->host_only) {
      HIP_TRY(ctx, hipDeviceSynchronize());
      release(P);
    } else {
      P = PackPlan{};
    }
    P.dims.assign(dims, dims + n);
    P.off.resize(n);
    std::vector<MatJobH> jobs;
    uint64_t tot = 0;
    for (int i = 0; i < n; ++i) {
      P.off[i] = tot;
      tot += uint64_t(dims[i]) * (uint64_t(dims[i]) + 1) / 2;
      const int T = ceil_div(dims[i], 64);   // 64 x 64 tiles of the upper triangle
      for (int bi = 0; bi < T; ++bi)
        for (int bj = bi; bj < T; ++bj) jobs.push_back({i, bi, bj, 0});
    }
    P.njobs = int(jobs.size());
    if (!ctx->host_only) {
      kfac_status st = upload_static(ctx, &P.d_jobs, jobs.data(), jobs.size() * sizeof(MatJobH));
      if (st != KFAC_OK) return st;
    }
    P.valid = true;
  }
  if (ctx->host_only) return fail(ctx, KFAC_ERR_DEVICE, "host-only context: nothing launched");
  hipStream_t s = static_cast<hipStream_t>(hip_stream);
  std::vector<PackMat> mats(n);
  for (int i = 0; i < n; ++i) mats[i] = PackMat{const_cast<float*>(M[i]), P.off[i], dims[i], 0};
  kfac_status st = sync_table(ctx, P.tab, mats.data(), mats.size() * sizeof(PackMat), s);
  if (st != KFAC_OK) return st;
  {
    ScopedTiming tm(ctx, KFAC_K_TRI_PACK, s);
    launch_tri_pack(static_cast<const PackMat*>(P.tab.dev), P.d_jobs, P.njobs, const_cast<float*>(packed), to_full, s);
  }
  HIP_TRY(ctx, hipGetLastError());
  return KFAC_OK;
}
}  // namespace

kfac_status kfac_pack_triangles(kfac_ctx* ctx, int n, const int32_t* dims, const float* const* M, float* packed,
                                void* hip_stream) {
  return pack_call(ctx, "kfac_pack_triangles", n, dims, M, packed, 0, hip_stream);
}

kfac_status kfac_unpack_triangles(kfac_ctx* ctx, int n, const int32_t* dims, const float* packed, float* const* M,
                                  void* hip_stream) {
  return pack_call(ctx, "kfac_unpack_triangles", n, dims, M, packed, 1, hip_stream);
}

kfac_status kfac_check_info(kfac_ctx* ctx, int n, const int32_t* info_dev, int32_t* info_host, void* hip_stream) {
  if (!ctx) return fail(nullptr, KFAC_ERR_INVALID_ARG, "kfac_check_info: ctx is NULL");
  if (n < 0 || (n > 0 && !info_dev)) return fail(ctx, KFAC_ERR_INVALID_ARG, "kfac_check_info: bad arguments");
  if (n == 0) return KFAC_OK;
  if (ctx->host_only) return fail(ctx, KFAC_ERR_DEVICE, "host-only context");
  DeviceGuard guard(ctx);
  std::vector<int32_t> tmp(n);
  HIP_TRY(ctx, hipStreamSynchronize(static_cast<hipStream_t>(hip_stream)));
  HIP_TRY(ctx, hipMemcpy(tmp.data(), info_dev, sizeof(int32_t) * n, hipMemcpyDeviceToHost));
  if (info_host) std::memcpy(info_host, tmp.data(), sizeof(int32_t) * n);
  for (int i = 0; i < n; ++i)
    if (tmp[i] != 0)
      return fail(ctx, KFAC_ERR_NOT_SPD, "matrix " + std::to_string(i) + ": leading minor of order " +
                                             std::to_string(tmp[i]) + " is not positive");
  return KFAC_OK;
}

// ----------------------------------------------------------------------------------- precondition
kfac_status kfac_precondition(kfac_ctx* ctx, int n, const int32_t* dG, const int32_t* dA,
                              const float* const* Ginv, const float* const* Ainv,
                              const float* const* gradW, float* const* out, void* hip_stream) {
  if (!ctx) return fail(nullptr, KFAC_ERR_INVALID_ARG, "kfac_precondition: ctx is NULL");
  if (n < 0) return fail(ctx, KFAC_ERR_INVALID_ARG, "kfac_precondition: n_layers < 0");
  if (n == 0) return KFAC_OK;
  if (!dG || !dA || !Ginv || !Ainv || !gradW || !out)
    return fail(ctx, KFAC_ERR_INVALID_ARG, "kfac_precondition: NULL array argument");
  for (int l = 0; l < n; ++l) {
    if (dG[l] < 1 || dA[l] < 1 || dG[l] > (1 << 20) || dA[l] > (1 << 20) ||
        int64_t(std::max(dG[l], dA[l])) * std::max(dG[l], dA[l]) > (int64_t(1) << 28))
      return fail(ctx, KFAC_ERR_INVALID_ARG, "kfac_precondition: dimension out of range at layer " + std::to_string(l));
    if (!Ginv[l] || !Ainv[l] || !gradW[l] || !out[l])
      return fail(ctx, KFAC_ERR_INVALID_ARG, "kfac_precondition: NULL matrix pointer at layer " + std::to_string(l));
    if (out[l] == Ginv[l] || out[l] == Ainv[l])
      return fail(ctx, KFAC_ERR_INVALID_ARG, "kfac_precondition: out aliases an inverse at layer " + std::to_string(l));
  }
  PrecondPlan& P = ctx->pp;
  const bool same = P.valid && int(P.dG.size()) == n && std::memcmp(P.dG.data(), dG, sizeof(int32_t) * n) == 0 &&
                    std::memcmp(P.dA.data(), dA, sizeof(int32_t) * n) == 0;
  DeviceGuard guard(ctx);
  if (!same) {
    PrecondSchedule S = schedule_precond(n, dG, dA);
    if (!ctx->host_only) {
      HIP_TRY(ctx, hipDeviceSynchronize());
      release(P);
    } else {
      P = PrecondPlan{};
    }
    P.dG.assign(dG, dG + n); P.dA.assign(dA, dA + n);
    P.t_off = S.t_off; P.ws_floats = S.ws_floats; P.stats = S.stats;
    P.njobs1 = int(S.jobs1.size()); P.njobs2 = int(S.jobs2.size());
    if (!ctx->host_only) {
      kfac_status st;
      if ((st = upload_static(ctx, &P.d_jobs1, S.jobs1.data(), S.jobs1.size() * sizeof(TileJob))) != KFAC_OK) return st;
      if ((st = upload_static(ctx, &P.d_jobs2, S.jobs2.data(), S.jobs2.size() * sizeof(TileJob))) != KFAC_OK) return st;
    }
    P.valid = true;
  }
  if (ctx->host_only) return fail(ctx, KFAC_ERR_DEVICE, "host-only context: nothing launched");

  hipStream_t s = static_cast<hipStream_t>(hip_stream);
  kfac_status st = ensure_ws(ctx, WS_PRECOND, P.ws_floats * sizeof(float));
  if (st != KFAC_OK) return st;
  std::vector<TileDesc> descs(2 * size_t(n));
  float* wsf = static_cast<float*>(ctx->ws[WS_PRECOND]);
  for (int l = 0; l < n; ++l) {
    float* T = wsf + P.t_off[l];
    TileDesc& D1 = descs[2 * l];       // T^T = V^T . Ginv^T : a(k, j) = V[k][j], b(k, i) = Ginv[i][k]
    D1 = TileDesc{};
    D1.a = rowmajor_operand(gradW[l], dG[l], dA[l], dA[l]);
    D1.b = transposed_operand(Ginv[l], dG[l], dG[l]);
    D1.out = T; D1.ldo = dG[l]; D1.M = dA[l]; D1.N = dG[l];
    D1.sym = 0; D1.mirror = MIRROR_NONE; D1.alpha = 1.f; D1.beta = 0.f;
    TileDesc& D2 = descs[2 * l + 1];   // out = T . Ainv : a(k, i) = T^T[k][i], b(k, j) = Ainv[k][j], both as stored
    D2 = TileDesc{};
    D2.a = rowmajor_operand(T, dA[l], dG[l], dG[l]);
    D2.b = rowmajor_operand(Ainv[l], dA[l], dA[l], dA[l]);
    D2.out = out[l]; D2.ldo = dA[l]; D2.M = dG[l]; D2.N = dA[l];
    D2.sym = 0; D2.mirror = MIRROR_NONE; D2.alpha = 1.f; D2.beta = 0.f;
  }
  st = sync_table(ctx, P.tab, descs.data(), descs.size() * sizeof(TileDesc), s);
  if (st != KFAC_OK) return st;
  const TileDesc* d_descs = static_cast<const TileDesc*>(P.tab.dev);
  {
    ScopedTiming tm(ctx, KFAC_K_PRECOND_LEFT, s);
    launch_tile_gemm(d_descs, static_cast<const TileJob*>(P.d_jobs1), P.njobs1, 0, s);
  }
  {
    ScopedTiming tm(ctx, KFAC_K_PRECOND_RIGHT, s);
    launch_tile_gemm_dl(d_descs, static_cast<const TileJob*>(P.d_jobs2), P.njobs2, s);   // both operands row-major
  }
  HIP_TRY(ctx, hipGetLastError());
  return KFAC_OK;
}

}  // extern "C"

// ----------------------------------------------------------------------------------- precondition, no allocation
// kfac_precondition for callers that cannot allocate device memory (HIP graph capture, tight serving
// loops): descriptors, job lists and the intermediate Ginv . V live in one file-scope device array;
// the tables are written by a small kernel from arguments passed by value, so the call issues three
// kernel launches and nothing else (no hipMalloc / hipFree / hipMemcpy / hipMemset).
namespace {

constexpr int NA_MAX_LAYERS = KFAC_NOALLOC_MAX_LAYERS;
constexpr size_t NA_MAX_ELEMS = KFAC_NOALLOC_MAX_ELEMS;           // floats of all intermediates together
constexpr int NA_MAX_JOBS = KFAC_NOALLOC_MAX_TILES;               // 128 x 128 output tiles of all layers together
constexpr size_t NA_DESC_BYTES = size_t(2) * NA_MAX_LAYERS * sizeof(TileDesc);
constexpr size_t NA_JOB_BYTES = size_t(2) * NA_MAX_JOBS * sizeof(TileJob);
constexpr size_t NA_T_OFFSET = ((NA_DESC_BYTES + NA_JOB_BYTES + 255) / 256) * 256;
constexpr size_t NA_SCRATCH_BYTES = NA_T_OFFSET + NA_MAX_ELEMS * sizeof(float);
static_assert(NA_SCRATCH_BYTES <= KFAC_NOALLOC_SCRATCH_BYTES, "the header states an upper bound of the array's size");

// One copy per GPU, held until the process ends.  In host code this name is only a handle for
// hipGetSymbolAddress: kernels get the device address looked up below, never the name.
static __device__ __align__(256) unsigned char scratch[NA_SCRATCH_BYTES];

constexpr int NA_MAX_DEVICES = 64;
unsigned char* g_scratch_ptr[NA_MAX_DEVICES] = {};               // per device: address of its copy of `scratch`

struct NoallocArgs {
  int32_t n;
  int32_t dG[NA_MAX_LAYERS], dA[NA_MAX_LAYERS];
  int32_t job_off[NA_MAX_LAYERS + 1];                             // first tile of every layer
  uint32_t t_off[NA_MAX_LAYERS];                                  // float offset of the layer's intermediate
  const float* Ginv[NA_MAX_LAYERS];
  const float* Ainv[NA_MAX_LAYERS];
  const float* gradW[NA_MAX_LAYERS];
  float* out[NA_MAX_LAYERS];
};
static_assert(sizeof(NoallocArgs) <= 3072, "passed by value as a kernel argument");

__device__ Operand dev_rowmajor_operand(const float* p, int K, int M, int ld) {
  Operand o{};
  o.ptr = p; o.type = OP_KMAJOR; o.K = K; o.M = M; o.bias = 0; o.ld = ld;
  o.bytes = uint32_t(K) * uint32_t(ld) * 4u;
  return o;
}
__device__ Operand dev_transposed_operand(const float* p, int K, int M) {
  Operand o{};
  o.ptr = p; o.type = OP_CONV11; o.K = K; o.M = M; o.bias = 0;
  o.bytes = uint32_t(K) * uint32_t(M) * 4u;
  o.C = M; o.H = 1; o.W = K; o.OH = 1; o.OW = K; o.stride = 1; o.pad_h = o.pad_w = 0; o.KH = 1; o.KW = 1;
  o.dOW = make_fastdiv(uint32_t(K));
  o.dOHW = make_fastdiv(uint32_t(K));
  return o;
}

// Block l writes the two descriptors and the tile jobs of layer l (the same descriptors
// kfac_precondition builds on the host; jobs in layer order).
__global__ void noalloc_tables_kernel(NoallocArgs a, TileDesc* descs, TileJob* jobs1, TileJob* jobs2, float* tbuf) {
  const int l = blockIdx.x;
  if (l >= a.n) return;
  const int dG = a.dG[l], dA = a.dA[l];
  float* T = tbuf + a.t_off[l];
  if (threadIdx.x == 0) {
    TileDesc D1{};     // T^T = V^T . Ginv^T
    D1.a = dev_rowmajor_operand(a.gradW[l], dG, dA, dA);
    D1.b = dev_transposed_operand(a.Ginv[l], dG, dG);
    D1.out = T; D1.ldo = dG; D1.M = dA; D1.N = dG;
    D1.sym = 0; D1.mirror = MIRROR_NONE; D1.alpha = 1.f; D1.beta = 0.f;
    descs[2 * l] = D1;
    TileDesc D2{};     // out = T . Ainv
    D2.a = dev_rowmajor_operand(T, dA, dG, dG);
    D2.b = dev_rowmajor_operand(a.Ainv[l], dA, dA, dA);
    D2.out = a.out[l]; D2.ldo = dA; D2.M = dG; D2.N = dA;
    D2.sym = 0; D2.mirror = MIRROR_NONE; D2.alpha = 1.f; D2.beta = 0.f;
    descs[2 * l + 1] = D2;
  }
  const int Tn = (dA + BN - 1) / BN, ntile = a.job_off[l + 1] - a.job_off[l];
  for (int e = threadIdx.x; e < ntile; e += blockDim.x) {
    const int bi = e / Tn, bj = e - bi * Tn;
    TileJob j{};
    j.kbeg = 0; j.part = -1;
    j.desc = 2 * l; j.bi = bj; j.bj = bi; j.kend = dG;
    jobs1[a.job_off[l] + e] = j;
    j.desc = 2 * l + 1; j.bi = bi; j.bj = bj; j.kend = dA;
    jobs2[a.job_off[l] + e] = j;
  }
}

}  // namespace

extern "C" kfac_status kfac_precondition_noalloc(kfac_ctx* ctx, int n, const int32_t* dG, const int32_t* dA,
                                                 const float* const* Ginv, const float* const* Ainv,
                                                 const float* const* gradW, float* const* out, void* hip_stream) {
  if (!ctx) return fail(nullptr, KFAC_ERR_INVALID_ARG, "kfac_precondition_noalloc: ctx is NULL");
  if (n < 0) return fail(ctx, KFAC_ERR_INVALID_ARG, "kfac_precondition_noalloc: n_layers < 0");
  if (n == 0) return KFAC_OK;
  if (!dG || !dA || !Ginv || !Ainv || !gradW || !out)
    return fail(ctx, KFAC_ERR_INVALID_ARG, "kfac_precondition_noalloc: NULL array argument");
  if (n > NA_MAX_LAYERS)
    return fail(ctx, KFAC_ERR_INVALID_ARG, "kfac_precondition_noalloc: " + std::to_string(n) + " layers exceed the maximum of " +
                                               std::to_string(NA_MAX_LAYERS) + " per call");
  NoallocArgs a{};
  a.n = n;
  size_t elems = 0;
  int64_t tiles = 0;
  for (int l = 0; l < n; ++l) {
    if (dG[l] < 1 || dA[l] < 1 || dG[l] > 16384 || dA[l] > 16384)
      return fail(ctx, KFAC_ERR_INVALID_ARG, "kfac_precondition_noalloc: dimension out of range at layer " + std::to_string(l));
    if (!Ginv[l] || !Ainv[l] || !gradW[l] || !out[l])
      return fail(ctx, KFAC_ERR_INVALID_ARG, "kfac_precondition_noalloc: NULL matrix pointer at layer " + std::to_string(l));
    if (out[l] == Ginv[l] || out[l] == Ainv[l])
      return fail(ctx, KFAC_ERR_INVALID_ARG, "kfac_precondition_noalloc: out aliases an inverse at layer " + std::to_string(l));
    a.dG[l] = dG[l]; a.dA[l] = dA[l];
    a.Ginv[l] = Ginv[l]; a.Ainv[l] = Ainv[l]; a.gradW[l] = gradW[l]; a.out[l] = out[l];
    a.job_off[l] = int32_t(tiles);
    a.t_off[l] = uint32_t(elems);
    tiles += int64_t(ceil_div(dG[l], BM)) * ceil_div(dA[l], BN);
    elems += size_t(dG[l]) * dA[l];
  }
  a.job_off[n] = int32_t(std::min<int64_t>(tiles, INT32_MAX));
  if (elems > NA_MAX_ELEMS)
    return fail(ctx, KFAC_ERR_INVALID_ARG, "kfac_precondition_noalloc: gradients of " + std::to_string(elems) +
                                               " elements exceed the static scratch (" + std::to_string(NA_MAX_ELEMS) + " elements per call)");
  if (tiles > NA_MAX_JOBS)
    return fail(ctx, KFAC_ERR_INVALID_ARG, "kfac_precondition_noalloc: " + std::to_string(tiles) + " output tiles exceed the maximum of " +
                                               std::to_string(NA_MAX_JOBS) + " per call");
  if (ctx->host_only) return fail(ctx, KFAC_ERR_DEVICE, "host-only context: nothing launched");
  if (ctx->device >= NA_MAX_DEVICES) return fail(ctx, KFAC_ERR_DEVICE, "kfac_precondition_noalloc: device index too large");
  DeviceGuard guard(ctx);
  unsigned char*& base = g_scratch_ptr[ctx->device];
  if (!base) {   // first call on this device: look up where this device holds its copy of the array
    void* p = nullptr;
    HIP_TRY(ctx, hipGetSymbolAddress(&p, HIP_SYMBOL(scratch)));
    if (!p) return fail(ctx, KFAC_ERR_DEVICE, "kfac_precondition_noalloc: the scratch array has no device address");
    base = static_cast<unsigned char*>(p);
  }
  TileDesc* d_descs = reinterpret_cast<TileDesc*>(base);
  TileJob* d_jobs1 = reinterpret_cast<TileJob*>(base + NA_DESC_BYTES);
  TileJob* d_jobs2 = d_jobs1 + NA_MAX_JOBS;
  float* d_t = reinterpret_cast<float*>(base + NA_T_OFFSET);
  hipStream_t s = static_cast<hipStream_t>(hip_stream);
  hipLaunchKernelGGL(noalloc_tables_kernel, dim3(n), dim3(256), 0, s, a, d_descs, d_jobs1, d_jobs2, d_t);
  launch_tile_gemm(d_descs, d_jobs1, int(tiles), 0, s);
  launch_tile_gemm_dl(d_descs, d_jobs2, int(tiles), s);
  HIP_TRY(ctx, hipGetLastError());
  return KFAC_OK;
}
