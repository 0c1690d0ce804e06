// Host orchestration behind the C ABI of include/bbmm.h: owns the workspaces, queues the
// kernels of kernels_vec.hip / kernels_mm.hip on the caller's stream in the order of the
// paper's algorithm (App. C preconditioner -> probes -> Alg. 2 -> SLQ / trace terms) and
// copies the scalar results back with a single stream synchronisation.
#include "bbmm.h"
#include "bbmm_dev.h"
#include "bbmm_plan.h"

#include <math.h>
#include <stdio.h>
#include <string.h>

#include <algorithm>
#include <mutex>
#include <string>
#include <vector>

// Work area of bbmm_tridiag_eig_batched_noalloc: device copies of the batch (diagonals,
// off-diagonals, eigenvalues, first rows: 4 x BBMM_EIG_NOALLOC_MAX doubles) followed by one status
// word per matrix.  Every GPU the library runs on holds its own copy of this array until the
// process ends.  In host code the name is only a handle for hipGetSymbolAddress: the address the
// kernels get is the one resolved per device in scratch_of().
#define BBMM_EIG_NOALLOC_MAX 16384
static __device__ __align__(256) double scratch[4 * BBMM_EIG_NOALLOC_MAX + BBMM_EIG_NOALLOC_MAX / 2];

namespace {

struct Buf {
  void* p = nullptr;
  size_t cap = 0;
};

// Work lists of a product that walks only the panels on and above the diagonal (see build_tri_lists).
struct TriLists {
  Buf pieces, first0, first1, base, tot;
  int wgs[2] = {0, 0};
  int np = 0;
  int max_slots = 0;
  int64_t tune = -1;
};

constexpr int kMaxVecBlocks = 512;   // at most 32 reduction groups of 16 blocks
constexpr int kMaxSplit = bbmm_plan::kMaxSplit;
// Measured, product in us (two-use / one-use form): n = 5 000: 88 / 60; 10 000: 125 / 121; 20 000: 312 / 331;
// 30 000: 630 / 696; 50 000: 1950 / 2630.
constexpr int kOtfSymMinRows = 12288;
constexpr int kDkStride = 2 * (BBMM_MAXD + 2);

}  // namespace

// Everything the launch sequence of the iteration loop depends on.
struct LoopKey {
  uint64_t alloc_epoch, tune_epoch;
  int mode, kernel, n, d, cc, ld, kp, maxit, m, tri, nls;
  bool operator==(const LoopKey& o) const {
    return alloc_epoch == o.alloc_epoch && tune_epoch == o.tune_epoch && mode == o.mode && kernel == o.kernel &&
           n == o.n && d == o.d && cc == o.cc && ld == o.ld && kp == o.kp && maxit == o.maxit && m == o.m &&
           tri == o.tri && nls == o.nls;
  }
};

struct bbmm_ctx {
  int device = 0;
  int num_cus = 256;          // compute units of the device (hipDeviceProp_t::multiProcessorCount)
  hipStream_t stream = nullptr;
  hipStream_t side = nullptr;            // second stream (default priority) for the SLQ eigensolves
  hipEvent_t ev_fork = nullptr, ev_join = nullptr;
  std::string err;

  // problem snapshot (valid after bbmm_setup)
  bool is_setup = false;
  bbmm_problem prob{};
  std::vector<double> ls;
  std::vector<int> forced;                  // replayed pivot order (empty = greedy rule)
  int n = 0, d = 0, t = 0, k = 0, kp = 0, np = 0, KK = 0, dp = 0, maxit = 0;
  int m = 0, mp = 0;                        // inducing inputs (SGPR), padded to 256
  HypArgs hyp{};
  bool khat_built = false, chol_done = false, pre_done = false, mbcg_done = false;
  bool sgpr = false, sgpr_built = false;
  int last_c = 0, last_ld = 0, last_t = 0;   // shape of the last mBCG run

  int64_t mat_wgs = 0, otf_split = 0;        // 0 = default
  int64_t sgpr_wgs[2] = {0, 0};              // workgroups of the two SGPR streaming products (0 = default)
  int64_t ur_blocks_cap = 0;
  int64_t zd_blocks = 0;
  int64_t khat_panel = 0;                    // column-panel width of the stored K_hat (0 = row-major)
  int khat_pw = 0;                           // layout of the K_hat currently in memory
  int64_t khat_sym = 0;                      // 1: keep only the upper triangle of K_hat (packed panels)
  bool khat_tri = false;                     // the K_hat currently in memory is such a triangle
  // work list of the product from the triangle
  TriLists sym;                              // ... from the stored triangle (panels of 1024 columns)
  TriLists otft;                             // ... on the fly from X (panels of 512 columns)
  int64_t otf_sym = 1;                       // on-the-fly product with each tile pair evaluated once (<= 16 columns, d <= 32): 0 never, 1 from kOtfSymMinRows rows on, 2 always
  // plans of the materialised product: 16- and 32-column blocks (index 0 / 1), 16-column block with at most 12 columns in use (2)
  int plan_np = 0, plan_wgs[3] = {0, 0, 0}, plan_slots[3] = {0, 0, 0};
  int64_t plan_tune = -1;
  // SGPR: plans of the two streaming products per block width: [v] = A (rows np, columns mp),
  // [2 + v] = A^T (rows mp, columns np)
  int sg_np = 0, sg_mp = 0, sg_wgs[4] = {0, 0, 0, 0}, sg_slots[4] = {0, 0, 0, 0};
  int64_t sg_tune[2] = {-1, -1};
  int64_t slq_eig = 0;                       // "slq_eig": 1 = SLQ terms through the eigen-decomposition of T
  int64_t eig_sweeps = 0;                    // trip budget of the tridiagonal eigen-solver per row (0 = default)
  // The mBCG iteration loop as a HIP graph: replayed when a run has the same launch sequence as an
  // earlier one (same sizes, mode, tuning values and buffers; the hyperparameters are read from the
  // device state, so a training loop replays one graph).
  int64_t use_graph = 0;                     // "loop_graph": 0 = always launch kernel by kernel
  uint64_t alloc_epoch = 0, tune_epoch = 0;  // bumped by every (re)allocation / bbmm_tune call
  hipStream_t cap = nullptr;                 // capture stream (the caller's may be the null stream)
  struct LoopGraph {
    LoopKey key;
    hipGraphExec_t exec = nullptr;           // NULL: key seen once, launched eagerly, not captured yet
    uint64_t used = 0;
  };
  std::vector<LoopGraph> graphs;
  uint64_t graph_clock = 0;
  int graph_replays = 0, graph_captures = 0; // statistics (bbmm_tune("loop_graph", -1) reads nothing; tests use timing)
  bool side_busy = false;                    // work was forked to `side` and its join has not been queued yet
  bool time_mm = false;                      // record HIP events around every product launch
  std::vector<hipEvent_t> ev;                // 2 per iteration, created on demand
  int ev_iters = 0;                          // iterations covered by the last timed run

  Buf Xa, Xb, Xs, X4, sq, Khat, L, delta, U, R, V, Z0, D4, Vp, partial, gpartial, alpha, beta, resid, st,
      tmpA, tmpB, SA, SB, u0v, dkpartial, eig, plan[3], nseg[3], 
      KUU, Gm, Ginv, Kux, AT, A, qdiag, Tp, T4, sgplan[4], sgnseg[4],
      Ua, Ub, Us, U4, usq, TU, TW, BU, BW, dkops;
  double* eig_static = nullptr;   // this device's address of `scratch`
  int* h_eig_status = nullptr;    // pinned, BBMM_EIG_NOALLOC_MAX ints
  DevState* h_st = nullptr;   // pinned
  double* h_hist = nullptr;   // pinned, 3 * MAXP * MAXC doubles
  size_t dk_rows_cap = 0;
};

namespace {

int fail(bbmm_ctx* c, int code, const std::string& msg) {
  if (c) c->err = msg;
  return code;
}

#define HIPCHK(ctx, expr)                                                              \
  do {                                                                                 \
    hipError_t e_ = (expr);                                                            \
    if (e_ != hipSuccess)                                                              \
      return fail(ctx, BBMM_EHIP, std::string(#expr) + ": " + hipGetErrorString(e_));  \
  } while (0)

int ensure(bbmm_ctx* c, Buf& b, size_t bytes) {
  if (bytes <= b.cap) return BBMM_OK;
  if (b.p) {
    hipError_t e = hipFree(b.p);
    b.p = nullptr;
    b.cap = 0;
    if (e != hipSuccess) return fail(c, BBMM_EHIP, std::string("hipFree: ") + hipGetErrorString(e));
  }
  void* p = nullptr;
  hipError_t e = hipMalloc(&p, bytes);
  if (e != hipSuccess) {
    (void)hipGetLastError();
    char msg[128];
    snprintf(msg, sizeof msg, "device allocation of %zu bytes failed", bytes);
    return fail(c, BBMM_ENOMEM, msg);
  }
  b.p = p;
  b.cap = bytes;
  if (c) ++c->alloc_epoch;
  return BBMM_OK;
}

template <typename T>
T* ptr(const Buf& b) {
  return reinterpret_cast<T*>(b.p);
}

// Device address of `scratch` on the CURRENT device `device`, resolved once per device.
constexpr int kMaxDevices = 64;
double* g_scratch_addr[kMaxDevices] = {};
std::mutex g_scratch_mu;

hipError_t scratch_of(int device, double** out) {
  std::lock_guard<std::mutex> lock(g_scratch_mu);
  if (device >= 0 && device < kMaxDevices && g_scratch_addr[device]) {
    *out = g_scratch_addr[device];
    return hipSuccess;
  }
  void* p = nullptr;
  hipError_t e = hipGetSymbolAddress(&p, HIP_SYMBOL(scratch));
  if (e != hipSuccess) return e;
  if (!p) return hipErrorInvalidSymbol;
  if (device >= 0 && device < kMaxDevices) g_scratch_addr[device] = reinterpret_cast<double*>(p);
  *out = reinterpret_cast<double*>(p);
  return hipSuccess;
}

int ld_for(int c) { return c <= 16 ? 16 : 32; }

// about two sweeps per eigenvalue are needed; 60 trips per row is far beyond any convergent case
int eig_sweeps_of(const bbmm_ctx* c) { return c->eig_sweeps > 0 ? (int)c->eig_sweeps : 60; }

// An error return between a fork to the second stream and the queued join leaves kernels running
// there that read and write context buffers; the next call that may free or refill those buffers
// waits for them first.
int drain_side(bbmm_ctx* c) {
  if (!c->side_busy) return BBMM_OK;
  c->side_busy = false;
  HIPCHK(c, hipStreamSynchronize(c->side));
  return BBMM_OK;
}

int vec_blocks(int n, int ld) {
  int rpp = BBMM_VEC_THREADS / ld;
  int nb = (n + rpp * 4 - 1) / (rpp * 4);
  if (nb < 1) nb = 1;
  if (nb > kMaxVecBlocks) nb = kMaxVecBlocks;
  return nb;
}

// blocks of the 1024-thread update kernel: at least two 4-row steps per wave, at most 128 partial rows
int ur_blocks(const bbmm_ctx* c, int n, int ld) {
  (void)ld;
  int rows_per_step = 16 * 4;               // 16 waves, 4 rows each
  int nb = (n + rows_per_step * 2 - 1) / (rows_per_step * 2);
  int cap = c->ur_blocks_cap > 0 ? (int)std::min<int64_t>(c->ur_blocks_cap, kMaxVecBlocks) : 128;
  return std::max(1, std::min(nb, cap));
}

int split_by_fill(const bbmm_ctx* c, int strips, int want_wgs, double min_fill) {
  return bbmm_plan::split_by_fill(c->np, c->num_cus, strips, want_wgs, min_fill);
}

int mat_wgs_of(const bbmm_ctx* c, int ld, bool narrow) {
  return bbmm_plan::mat_wgs_of(c->np, c->num_cus, c->mat_wgs, ld, narrow);
}

// Partial results of a product: `slots` blocks of np x ld doubles.  Grown on demand, per mode and
// block width (the largest user is the triangle product: up to one slot per panel).
int ensure_vp(bbmm_ctx* c, int slots, int ld) {
  size_t bytes = (size_t)std::max(slots, 1) * c->np * ld * sizeof(double);
  if (bytes <= c->Vp.cap) return BBMM_OK;
  HIPCHK(c, hipStreamSynchronize(c->stream));   // earlier launches may still use the old buffer
  return ensure(c, c->Vp, bytes);
}

// Lays out one plan on the host (bbmm_plan::lay_out_plan, which checks everything the kernel
// relies on) and uploads it.
int make_plan(bbmm_ctx* c, int rows_p, int cols_p, int ld, int wgs, int slot_cap, Buf& plan_buf,
              Buf& nseg_buf, int* max_slots) {
  std::vector<MmPlan> plan;
  std::vector<int> nseg;
  if (const char* what = bbmm_plan::lay_out_plan(rows_p, cols_p, ld, wgs, slot_cap, plan, nseg))
    return fail(c, BBMM_EINVAL, what);
  int rc = ensure(c, plan_buf, sizeof(MmPlan) * plan.size());
  if (rc) return rc;
  rc = ensure(c, nseg_buf, sizeof(int) * nseg.size());
  if (rc) return rc;
  HIPCHK(c, hipMemcpy(plan_buf.p, plan.data(), sizeof(MmPlan) * plan.size(), hipMemcpyHostToDevice));
  HIPCHK(c, hipMemcpy(nseg_buf.p, nseg.data(), sizeof(int) * nseg.size(), hipMemcpyHostToDevice));
  if (max_slots) *max_slots = *std::max_element(nseg.begin(), nseg.end());
  return BBMM_OK;
}

int ensure_mat_plans(bbmm_ctx* c) {
  if (c->plan_np == c->np && c->plan_tune == c->mat_wgs) return BBMM_OK;
  HIPCHK(c, hipStreamSynchronize(c->stream));   // earlier launches may still read the old plans
  // plans: 0 = 16-column block, 1 = 32-column block, 2 = 16-column block with at most 12 columns in use
  for (int v = 0; v < 3; ++v) {
    int ld = (v == 1) ? 32 : 16;
    int wgs = mat_wgs_of(c, ld, v == 2);
    int rc = make_plan(c, c->np, c->np, ld, wgs, kMaxSplit, c->plan[v], c->nseg[v], &c->plan_slots[v]);
    if (rc) return rc;
    c->plan_wgs[v] = wgs;
  }
  c->plan_np = c->np;
  c->plan_tune = c->mat_wgs;
  return BBMM_OK;
}

// Work lists of a product that visits only the panels (W columns each) on and above the diagonal
// (bbmm_plan::lay_out_triangle), uploaded.
int build_tri_lists(bbmm_ctx* c, int W, int want, int64_t tune, TriLists& L) {
  if (L.np == c->np && L.tune == tune) return BBMM_OK;
  HIPCHK(c, hipStreamSynchronize(c->stream));   // earlier launches may still read the old lists
  bbmm_plan::TriHost H;
  if (const char* what = bbmm_plan::lay_out_triangle(c->np, W, want, H)) return fail(c, BBMM_EINVAL, what);
  struct Up {
    Buf* b;
    const void* src;
    size_t bytes;
  } ups[] = {{&L.pieces, H.pieces.data(), sizeof(MmPiece) * H.pieces.size()},
             {&L.first0, H.first[0].data(), sizeof(int) * H.first[0].size()},
             {&L.first1, H.first[1].data(), sizeof(int) * H.first[1].size()},
             {&L.base, H.cnt.data(), sizeof(int) * H.cnt.size()},
             {&L.tot, H.tot.data(), sizeof(int) * H.tot.size()}};
  for (const Up& u : ups) {
    int rc = ensure(c, *u.b, std::max<size_t>(u.bytes, 16));
    if (rc) return rc;
    if (u.bytes) HIPCHK(c, hipMemcpy(u.b->p, u.src, u.bytes, hipMemcpyHostToDevice));
  }
  L.wgs[0] = H.wgs[0];
  L.wgs[1] = H.wgs[1];
  L.max_slots = H.max_slots;
  L.np = c->np;
  L.tune = tune;
  return BBMM_OK;
}

int ensure_sym_plan(bbmm_ctx* c) {
  return build_tri_lists(c, BBMM_SYM_PANEL, c->mat_wgs > 0 ? (int)c->mat_wgs : c->num_cus, c->mat_wgs, c->sym);
}

// two workgroups of the on-the-fly triangle kernel fit a compute unit
int ensure_otf_tri_plan(bbmm_ctx* c) {
  return build_tri_lists(c, BBMM_OTF_PANEL, c->otf_split > 0 ? (int)c->otf_split : 2 * c->num_cus, c->otf_split,
                         c->otft);
}

int rect_wgs_of(const bbmm_ctx* c, int rows_p, int cols_p, int ld, int slot_cap, int64_t tuned) {
  return bbmm_plan::rect_wgs_of(c->num_cus, rows_p, cols_p, ld, slot_cap, tuned);
}

constexpr int kSgprSlotCap = 1024;   // partial results of A^T D: one per workgroup when m <= 1024

int ensure_sgpr_plans(bbmm_ctx* c) {
  if (c->sg_np == c->np && c->sg_mp == c->mp && c->sg_tune[0] == c->sgpr_wgs[0] && c->sg_tune[1] == c->sgpr_wgs[1])
    return BBMM_OK;
  HIPCHK(c, hipStreamSynchronize(c->stream));
  for (int v = 0; v < 2; ++v) {
    int ld = v ? 32 : 16;
    int w1 = rect_wgs_of(c, c->np, c->mp, ld, kSgprSlotCap, c->sgpr_wgs[0]);
    int rc = make_plan(c, c->np, c->mp, ld, w1, kSgprSlotCap, c->sgplan[v], c->sgnseg[v], &c->sg_slots[v]);
    if (rc) return rc;
    c->sg_wgs[v] = w1;
    int w2 = rect_wgs_of(c, c->mp, c->np, ld, kMaxSplit, c->sgpr_wgs[1]);
    rc = make_plan(c, c->mp, c->np, ld, w2, kMaxSplit, c->sgplan[2 + v], c->sgnseg[2 + v], &c->sg_slots[2 + v]);
    if (rc) return rc;
    c->sg_wgs[2 + v] = w2;
  }
  size_t slots = (size_t)std::max(c->sg_slots[0], c->sg_slots[1]);
  int rc = ensure(c, c->Tp, slots * (size_t)c->mp * BBMM_MAXC * sizeof(double));
  if (rc) return rc;
  c->sg_np = c->np;
  c->sg_mp = c->mp;
  c->sg_tune[0] = c->sgpr_wgs[0];
  c->sg_tune[1] = c->sgpr_wgs[1];
  return BBMM_OK;
}

int otf_split_of(const bbmm_ctx* c) {
  if (c->otf_split > 0) return (int)std::min<int64_t>(c->otf_split, std::min(kMaxSplit, c->np / 16));
  int strips = (c->np / 16 + 31) / 32;          // 4 waves x 8 column blocks per workgroup
  // (at least four 16-row blocks per chunk: n = 1 000 runs 24 us with 16 chunks, 32 us with 64)
  return std::min(split_by_fill(c, strips, 4 * c->num_cus, 0.97), std::max(1, c->np / 64));
}

// the derivative pass skips the tiles below the diagonal, so its workgroups differ in length:
// many small ones even that out
int dk_split_of(const bbmm_ctx* c) {
  int strips = (c->np / 16 + 15) / 16;          // 4 waves x 4 column blocks per workgroup
  int s = (16 * c->num_cus + strips - 1) / strips;
  return std::max(1, std::min(s, std::min(kMaxSplit, c->np / 16)));
}

int check_ready(bbmm_ctx* c) {
  if (!c) return BBMM_EINVAL;
  if (!c->is_setup) return fail(c, BBMM_EINVAL, "bbmm_setup has not been called");
  hipError_t e = hipSetDevice(c->device);
  if (e != hipSuccess) return fail(c, BBMM_EHIP, std::string("hipSetDevice: ") + hipGetErrorString(e));
  return drain_side(c);
}

// Copies the device state to the pinned mirror and waits for the stream.
int fetch_state(bbmm_ctx* c, bool with_hist) {
  HIPCHK(c, hipMemcpyAsync(c->h_st, c->st.p, sizeof(DevState), hipMemcpyDeviceToHost, c->stream));
  if (with_hist) {
    size_t hb = sizeof(double) * BBMM_MAXP * BBMM_MAXC;
    HIPCHK(c, hipMemcpyAsync(c->h_hist, c->alpha.p, hb, hipMemcpyDeviceToHost, c->stream));
    HIPCHK(c, hipMemcpyAsync(c->h_hist + BBMM_MAXP * BBMM_MAXC, c->beta.p, hb, hipMemcpyDeviceToHost, c->stream));
    HIPCHK(c, hipMemcpyAsync(c->h_hist + 2 * BBMM_MAXP * BBMM_MAXC, c->resid.p, hb, hipMemcpyDeviceToHost, c->stream));
  }
  HIPCHK(c, hipStreamSynchronize(c->stream));
  HIPCHK(c, hipGetLastError());
  return BBMM_OK;
}

int device_status(bbmm_ctx* c) {
  int s = c->h_st->status;
  if (s == BBMM_ENOTPD)
    return fail(c, BBMM_ENOTPD, "capacitance matrix sigma^2 I + L^T L (or K_UU + jitter I) is not positive definite");
  if (s == BBMM_ENONFINITE) return fail(c, BBMM_ENONFINITE, "non-finite value in the log-determinant estimate");
  if (s == BBMM_ENOCONV)
    return fail(c, BBMM_ENOCONV, "the eigen-solver did not reduce a Lanczos tridiagonal within its sweep budget");
  if (s != 0) return fail(c, s, "device-side failure");
  return BBMM_OK;
}

// ---- stages on internal buffers -------------------------------------------------------------
int stage_build_khat(bbmm_ctx* c) {
  // column panels of 1024 (one 16-row step of a workgroup is then 64 KB of contiguous memory:
  // 1.515 -> 1.498 ms per product at n = 50,000); "khat_panel" = 1 keeps plain row-major
  int pw = c->khat_panel == 0 ? 1024 : (c->khat_panel == 1 ? 0 : (int)c->khat_panel);
  bool tri = c->khat_sym != 0;
  size_t cols_alloc = pw > 0 ? (size_t)((c->np + pw - 1) / pw) * pw : (size_t)c->np;
  size_t bytes = (size_t)c->np * cols_alloc * sizeof(float);
  if (tri) {
    // "khat_sym": the upper triangle in packed panels, all panels but the last being full height
    pw = BBMM_SYM_PANEL;
    size_t S = (size_t)((c->np + pw - 1) / pw);
    bytes = ((size_t)pw * pw * (S * (S - 1) / 2) + (size_t)c->np * pw) * sizeof(float);
  }
  int rc = ensure(c, c->Khat, bytes);
  if (rc) return rc;
  c->khat_pw = pw;
  c->khat_tri = tri;
  if (launch_build_khat(c->stream, c->prob.kernel, c->KK, ptr<float>(c->Xa), ptr<float>(c->Xb),
                        ptr<float>(c->sq), c->n, c->np, pw, tri ? 1 : 0, c->prob.outputscale, c->prob.noise,
                        ptr<float>(c->Khat)))
    return fail(c, BBMM_EINVAL, "unsupported input dimension");
  c->khat_built = true;
  return BBMM_OK;
}

// SGPR: K_UU (fp64) -> Cholesky factor G -> G^{-1}; K_UX (fp64); A^T = G^{-1} K_UX rounded to fp32,
// A by transposition, and the diagonal of Q = A A^T.
int stage_sgpr_build(bbmm_ctx* c) {
  if (!c->sgpr) return fail(c, BBMM_EINVAL, "the problem is not an SGPR problem");
  hipStream_t s = c->stream;
  size_t mp = (size_t)c->mp, np = (size_t)c->np;
  struct { Buf* b; size_t bytes; } want[] = {
      {&c->KUU, mp * mp * sizeof(double)}, {&c->Gm, mp * mp * sizeof(double)},
      {&c->Ginv, mp * mp * sizeof(double)}, {&c->Kux, mp * np * sizeof(double)},
      {&c->AT, mp * ((np + BBMM_SGPR_PANEL - 1) / BBMM_SGPR_PANEL) * BBMM_SGPR_PANEL * sizeof(float)},
      {&c->A, mp * np * sizeof(float)},
      {&c->qdiag, np * sizeof(double)}, {&c->T4, mp * BBMM_MAXC * sizeof(double)},
      {&c->Ua, mp * c->dp * sizeof(float)}, {&c->Ub, mp * c->dp * sizeof(float)},
      {&c->Us, mp * c->dp * sizeof(float)}, {&c->U4, mp * c->dp * sizeof(float)},
      {&c->usq, mp * sizeof(float)},
      {&c->TU, mp * BBMM_MAXC * sizeof(double)}, {&c->TW, mp * BBMM_MAXC * sizeof(double)},
      {&c->BU, mp * BBMM_MAXC * sizeof(double)}, {&c->BW, mp * BBMM_MAXC * sizeof(double)},
      {&c->dkops, mp * (3 * 64 + 2) * sizeof(float)},
  };
  for (auto& w : want) {
    int rc = ensure(c, *w.b, w.bytes);
    if (rc) return rc;
  }
  int rc = ensure_sgpr_plans(c);
  if (rc) return rc;
  DevState* st = ptr<DevState>(c->st);
  // K_UX (n m kernel values in fp64, one big launch) does not depend on the K_UU chain (about a
  // hundred small launches): it runs beside it on the context's second stream
  HIPCHK(c, hipEventRecord(c->ev_fork, s));
  HIPCHK(c, hipStreamWaitEvent(c->side, c->ev_fork, 0));
  c->side_busy = true;
  if (c->mp > c->m) launch_fill_f64(c->side, ptr<double>(c->Kux), mp * np, 0.0);   // padding rows of every panel
  if (launch_sgpr_kux(c->side, c->prob.X, c->prob.Uind, c->n, c->np, c->m, c->mp, c->dp, c->hyp,
                      ptr<double>(c->Kux)))
    return fail(c, BBMM_EINVAL, "unsupported input dimension");
  HIPCHK(c, hipEventRecord(c->ev_join, c->side));
  launch_fill_f64(s, ptr<double>(c->Gm), mp * mp, 0.0);
  launch_fill_f64(s, ptr<double>(c->Ginv), mp * mp, 0.0);
  launch_sgpr_kuu(s, c->prob.Uind, c->m, c->mp, c->hyp, c->prob.jitter_rel * c->prob.outputscale,
                  ptr<double>(c->KUU));
  launch_sgpr_chol(s, ptr<double>(c->KUU), ptr<double>(c->Gm), c->mp, 1e-13 * c->prob.outputscale, st);
  launch_sgpr_trinv(s, ptr<double>(c->Gm), ptr<double>(c->Ginv), c->mp);
  HIPCHK(c, hipStreamWaitEvent(s, c->ev_join, 0));
  c->side_busy = false;
  // the Cholesky work matrix is free again: it receives G^{-1} in MFMA operand order
  launch_sgpr_root(s, ptr<double>(c->Ginv), ptr<double>(c->KUU), ptr<double>(c->Kux), c->mp, c->np,
                   ptr<float>(c->AT));
  launch_root_transpose(s, ptr<float>(c->AT), c->mp, c->np, ptr<float>(c->A));
  launch_sgpr_qdiag(s, ptr<float>(c->A), c->n, c->mp, ptr<double>(c->qdiag));
  // inducing inputs in the centred, scaled coordinates of X (for the derivative pair sums)
  launch_prep_x(s, c->prob.Uind, c->m, c->d, c->mp, c->KK, c->hyp, st, ptr<float>(c->Ua), ptr<float>(c->Ub),
                ptr<float>(c->Us), ptr<float>(c->U4), ptr<float>(c->usq));
  c->sgpr_built = true;
  c->chol_done = c->pre_done = c->mbcg_done = false;
  return BBMM_OK;
}

// SGPR product, second half: Vp <- partial sums of A T with T (quad-swizzled, mp rows) in T4.
// cols: columns of the block in use (0 = all).
int sgpr_second_pass(bbmm_ctx* c, int ld, VpShape* shape, int cols = 0) {
  int v = (ld == 32) ? 1 : 0;
  int rc0 = ensure_vp(c, c->sg_slots[2 + v], ld);
  if (rc0) return rc0;
  if (launch_mm_mat(c->stream, ptr<float>(c->AT), ptr<double>(c->T4), ptr<double>(c->Vp), c->np, ld,
                    ptr<MmPlan>(c->sgplan[2 + v]), c->sg_wgs[2 + v], ptr<DevState>(c->st), BBMM_SGPR_PANEL,
                    c->mp, cols))
    return fail(c, BBMM_EINVAL, "unsupported block width");
  *shape = VpShape{0, ptr<int>(c->sgnseg[2 + v]), v ? 512 : 1024, c->sg_slots[2 + v]};
  return BBMM_OK;
}

// SGPR product, first half: Tp <- partial sums of A^T D with D (quad-swizzled, np rows) in `D4`.
int sgpr_first_pass(bbmm_ctx* c, int ld, const double* D4, VpShape* shape, int cols = 0) {
  int v = (ld == 32) ? 1 : 0;
  if (launch_mm_mat(c->stream, ptr<float>(c->A), D4, ptr<double>(c->Tp), c->mp, ld,
                    ptr<MmPlan>(c->sgplan[v]), c->sg_wgs[v], ptr<DevState>(c->st), 0, 0, cols))
    return fail(c, BBMM_EINVAL, "unsupported block width");
  *shape = VpShape{0, ptr<int>(c->sgnseg[v]), v ? 512 : 1024};
  return BBMM_OK;
}

// Vp <- partial products of K_hat with the block in D4; returns the split count and the
// (scale, add) pair that turns the partial sums into K_hat D.
int stage_mm(bbmm_ctx* c, int mode, int cc, int ld, VpShape* shape, double* scaleV, double* addD) {
  if ((mode == BBMM_MODE_SGPR) != c->sgpr)
    return fail(c, BBMM_EINVAL, "an SGPR problem takes mode SGPR, and only an SGPR problem does");
  if (mode == BBMM_MODE_SGPR) {
    if (!c->sgpr_built) return fail(c, BBMM_EINVAL, "SGPR product needs bbmm_sgpr_build first");
    if (ld != 16 && ld != 32) return fail(c, BBMM_EINVAL, "unsupported block width");
    VpShape sh1{0, nullptr, 1};
    int rc = sgpr_first_pass(c, ld, ptr<double>(c->D4), &sh1, cc);
    if (rc) return rc;
    launch_sgpr_mid(c->stream, ptr<double>(c->Tp), sh1, c->mp, ld, ptr<DevState>(c->st), ptr<double>(c->T4));
    rc = sgpr_second_pass(c, ld, shape, cc);
    if (rc) return rc;
    *scaleV = 1.0;
    *addD = c->prob.noise;
  } else if (mode == BBMM_MODE_MATERIALISED) {
    if (!c->khat_built) return fail(c, BBMM_EINVAL, "materialised product needs bbmm_build_khat first");
    if (ld != 16 && ld != 32) return fail(c, BBMM_EINVAL, "unsupported block width");
    if (c->khat_tri) {
      int rc = ensure_sym_plan(c);
      if (rc) return rc;
      rc = ensure_vp(c, c->sym.max_slots, ld);
      if (rc) return rc;
      if (launch_mm_sym(c->stream, ptr<float>(c->Khat), ptr<double>(c->D4), ptr<double>(c->Vp), c->np, ld, cc,
                        ptr<MmPiece>(c->sym.pieces), ptr<int>(c->sym.first0), c->sym.wgs[0],
                        ptr<int>(c->sym.first1), c->sym.wgs[1], ptr<int>(c->sym.base), ptr<DevState>(c->st)))
        return fail(c, BBMM_EINVAL, "unsupported block width");
      *shape = VpShape{0, ptr<int>(c->sym.tot), BBMM_SYM_PANEL};
      *scaleV = 1.0;
      *addD = 0.0;
      return BBMM_OK;
    }
    int rc = ensure_mat_plans(c);
    if (rc) return rc;
    int v = (ld == 32) ? 1 : (cc <= 12 ? 2 : 0);
    rc = ensure_vp(c, c->plan_slots[v], ld);
    if (rc) return rc;
    if (launch_mm_mat(c->stream, ptr<float>(c->Khat), ptr<double>(c->D4), ptr<double>(c->Vp), c->np, ld,
                      ptr<MmPlan>(c->plan[v]), c->plan_wgs[v], ptr<DevState>(c->st), c->khat_pw, c->np, cc))
      return fail(c, BBMM_EINVAL, "unsupported block width");
    *shape = VpShape{0, ptr<int>(c->nseg[v]), v == 1 ? 512 : 1024, c->plan_slots[v]};
    *scaleV = 1.0;
    *addD = 0.0;
  } else if (mode == BBMM_MODE_ONTHEFLY && (c->otf_sym == 2 || (c->otf_sym == 1 && c->np >= kOtfSymMinRows)) &&
             ld == 16 && c->KK <= 8) {
    // every pair of tiles (I, J), (J, I) evaluated once and used for both contributions (beyond 32
    // input dimensions the two-use form runs out of registers and the one-use form is the faster;
    // so it is for small n, where the pieces of the two-use form are short)
    int rc = ensure_otf_tri_plan(c);
    if (rc) return rc;
    rc = ensure_vp(c, c->otft.max_slots, ld);
    if (rc) return rc;
    if (launch_mm_otf_tri(c->stream, c->prob.kernel, c->KK, ptr<float>(c->Xa), ptr<float>(c->Xb), ptr<float>(c->sq),
                          ptr<double>(c->D4), ptr<double>(c->Vp), c->np, cc, ptr<MmPiece>(c->otft.pieces),
                          ptr<int>(c->otft.first0), c->otft.wgs[0], ptr<int>(c->otft.first1), c->otft.wgs[1],
                          ptr<int>(c->otft.base), ptr<DevState>(c->st)))
      return fail(c, BBMM_EINVAL, "unsupported input dimension");
    *shape = VpShape{0, ptr<int>(c->otft.tot), BBMM_OTF_PANEL};
    *scaleV = c->prob.outputscale;
    *addD = c->prob.noise;
  } else if (mode == BBMM_MODE_ONTHEFLY) {
    int ns = otf_split_of(c);
    int rc = ensure_vp(c, ns, ld);
    if (rc) return rc;
    if (launch_mm_otf(c->stream, c->prob.kernel, c->KK, ptr<float>(c->Xa), ptr<float>(c->Xb),
                      ptr<float>(c->sq), ptr<double>(c->D4), ptr<double>(c->Vp), c->np, ld, cc, ns,
                      ptr<DevState>(c->st)))
      return fail(c, BBMM_EINVAL, "unsupported block width or input dimension");
    *shape = VpShape{ns, nullptr, 1};
    *scaleV = c->prob.outputscale;
    *addD = c->prob.noise;
  } else {
    return fail(c, BBMM_EINVAL, "unknown mode");
  }
  return BBMM_OK;
}

int stage_pivchol(bbmm_ctx* c) {
  hipStream_t s = c->stream;
  int nb = vec_blocks(c->n, 16);
  if (c->kp > 0) launch_fill_f64(s, ptr<double>(c->L), (size_t)c->np * c->kp, 0.0);
  // pivot candidates alternate between two buffers (a step reads one and writes the other)
  double* arg[2] = {ptr<double>(c->partial), ptr<double>(c->partial) + 2 * kMaxVecBlocks};
  auto fpiv = [c](int m) { return (m < (int)c->forced.size()) ? c->forced[m] : -1; };
  if (c->sgpr) {
    // App. C, SoR case: the diagonal of Q is not constant and a row of Q costs one pass over the
    // root: row piv = A (A^T e_piv), the second streaming product applied to row piv of A.
    if (!c->sgpr_built) return fail(c, BBMM_EINVAL, "bbmm_sgpr_build must run first");
    DevState* st = ptr<DevState>(c->st);
    launch_fill_bytes0(s, &st->done, 2 * sizeof(int));
    launch_fill_f64(s, ptr<double>(c->D4), (size_t)c->np * 16, 0.0);
    launch_pc_init(s, c->n, c->hyp, ptr<double>(c->delta), st, arg[0], nb, ptr<double>(c->qdiag), fpiv(0));
    for (int m = 0; m < c->k; ++m) {
      launch_sgpr_pick(s, ptr<float>(c->A), c->mp, arg[m & 1], nb, ptr<double>(c->T4), fpiv(m));
      VpShape sh{0, nullptr, 1};
      int rc = sgpr_second_pass(c, 16, &sh, 1);
      if (rc) return rc;
      launch_vreduce(s, ptr<double>(c->Vp), sh, c->n, c->np, 16, 1.0, 0.0, ptr<double>(c->D4), ptr<double>(c->V));
      launch_pc_step(s, c->prob.X, c->n, m, c->kp, c->hyp, ptr<double>(c->delta), ptr<double>(c->L), st,
                     arg[m & 1], arg[(m + 1) & 1], nb, ptr<double>(c->V), 16, fpiv(m), fpiv(m + 1));
    }
    c->chol_done = true;
    c->pre_done = false;
    return BBMM_OK;
  }
  launch_pc_init(s, c->n, c->hyp, ptr<double>(c->delta), ptr<DevState>(c->st), arg[0], nb, nullptr, fpiv(0));
  for (int m = 0; m < c->k; ++m)
    launch_pc_step(s, c->prob.X, c->n, m, c->kp, c->hyp, ptr<double>(c->delta), ptr<double>(c->L),
                   ptr<DevState>(c->st), arg[m & 1], arg[(m + 1) & 1], nb, nullptr, 0, fpiv(m), fpiv(m + 1));
  c->chol_done = true;
  c->pre_done = false;
  return BBMM_OK;
}

int stage_pre_setup(bbmm_ctx* c) {
  if (!c->chol_done) return fail(c, BBMM_EINVAL, "bbmm_pivoted_cholesky must run first");
  int nb = std::min(kMaxVecBlocks, std::max(1, c->n / 64));
  launch_pre_setup(c->stream, ptr<double>(c->L), c->n, c->k, c->kp, c->prob.noise, ptr<DevState>(c->st),
                   ptr<double>(c->partial), ptr<double>(c->gpartial), nb);
  c->pre_done = true;
  return BBMM_OK;
}

// mBCG on the block held in R (padded row-major, stride ld); U, Z0, coefficient histories and the
// device state are left in the context.
// warm != NULL: column 0 starts from that solution (device, n floats) instead of zero.
int stage_mbcg(bbmm_ctx* c, int mode, int cc, int ld, const float* warm = nullptr) {
  if (!c->pre_done) return fail(c, BBMM_EINVAL, "bbmm_precond_setup must run first");
  hipStream_t s = c->stream;
  DevState* st = ptr<DevState>(c->st);
  int nb = vec_blocks(c->n, ld);
  // k_zd has no reduction, so its grid is not tied to the partial-sum layout: one 16-row trip per
  // wave where n allows it (a trip costs a memory round trip; more waves overlap more of them)
  int nb_zd = std::max(nb, std::min((c->n / 16 + 3) / 4, (c->zd_blocks > 0 ? (int)c->zd_blocks : 16) * c->num_cus));
  size_t blk = (size_t)c->np * ld;
  // U, D, the coefficient histories and done / iters_run (next to each other at the end of
  // DevState), zeroed by one launch
  {
    size_t hist = (size_t)2 * BBMM_MAXP * BBMM_MAXC;   // words of one history of doubles
    ZeroSegs z = {{c->U.p, c->D4.p, c->alpha.p, c->beta.p, c->resid.p, &st->done},
                  {2 * blk, 2 * blk, hist, hist, hist, 2}, 6};
    launch_fill_multi0(s, z);
  }
  double noise = c->prob.noise;
  int nb_ur = ur_blocks(c, c->n, ld);
  double* pdv = ptr<double>(c->gpartial);
  double* pur = ptr<double>(c->partial);
  launch_ur(s, 1, c->n, ld, cc, c->kp, noise, 0.0, ptr<double>(c->D4), ptr<double>(c->V), ptr<double>(c->U),
            ptr<double>(c->R), ptr<double>(c->L), st, pdv, nb, pur, nb_ur, 0, ptr<double>(c->alpha),
            ptr<double>(c->beta), ptr<double>(c->resid));
  if (warm) {
    // Alg. 1/2: r_0 = b - K_hat u_0 for the current solution u_0 -- one more product, of the block
    // [u_init, 0, ..]; the pass above has left |b| (the residuals stay relative to it), the second
    // pass redoes rho_0 for the new residual
    launch_warm_rhs(s, warm, c->n, ld, ptr<double>(c->D4));
    VpShape ns{0, nullptr, 1};
    double scaleV = 1.0, addD = 0.0;
    int rc = stage_mm(c, mode, cc, ld, &ns, &scaleV, &addD);
    if (rc) return rc;
    launch_vreduce(s, ptr<double>(c->Vp), ns, c->n, c->np, ld, scaleV, addD, ptr<double>(c->D4), ptr<double>(c->V));
    launch_warm_apply(s, warm, ptr<double>(c->V), c->n, ld, ptr<double>(c->U), ptr<double>(c->R));
    launch_fill_f64(s, ptr<double>(c->D4), blk, 0.0);
    launch_ur(s, 2, c->n, ld, cc, c->kp, noise, 0.0, ptr<double>(c->D4), ptr<double>(c->V), ptr<double>(c->U),
              ptr<double>(c->R), ptr<double>(c->L), st, pdv, nb, pur, nb_ur, 0, ptr<double>(c->alpha),
              ptr<double>(c->beta), ptr<double>(c->resid));
  }
  launch_zd(s, 1, c->n, ld, c->kp, noise, ptr<double>(c->R), ptr<double>(c->L), ptr<double>(c->D4),
            ptr<double>(c->Z0), st, nb);
  // the loop's kernels take noise, tolerance and the (scale, diagonal) pair of the product from the
  // device state, so their launches are the same for any hyperparameter values
  {
    double scaleV = 1.0, addD = 0.0;
    if (mode == BBMM_MODE_SGPR) addD = noise;
    else if (mode == BBMM_MODE_ONTHEFLY) {
      scaleV = c->prob.outputscale;
      addD = noise;
    }
    launch_set_loop_scalars(s, st, noise, c->prob.tol, scaleV, addD);
  }
  if (c->time_mm) {
    while ((int)c->ev.size() < 2 * c->maxit) {
      hipEvent_t e;
      HIPCHK(c, hipEventCreate(&e));
      c->ev.push_back(e);
    }
  }
  c->ev_iters = 0;
  // one pass over the maxit iterations on stream `ls`, kernel by kernel
  auto launch_loop = [&](hipStream_t ls, bool timed) -> int {
    hipStream_t user = c->stream;
    c->stream = ls;                       // stage_mm queues on the context's stream
    int rc = BBMM_OK;
    for (int j = 0; j < c->maxit && rc == BBMM_OK; ++j) {
      VpShape ns{0, nullptr, 1};
      double scaleV = 1.0, addD = 0.0;
      if (timed && hipEventRecord(c->ev[2 * j], ls) != hipSuccess) rc = fail(c, BBMM_EHIP, "hipEventRecord failed");
      if (rc == BBMM_OK) rc = stage_mm(c, mode, cc, ld, &ns, &scaleV, &addD);
      if (rc) break;
      if (timed) {
        if (hipEventRecord(c->ev[2 * j + 1], ls) != hipSuccess) {
          rc = fail(c, BBMM_EHIP, "hipEventRecord failed");
          break;
        }
        c->ev_iters = j + 1;
      }
      launch_dv(ls, ptr<double>(c->Vp), ns, c->n, c->np, ld, scaleV, -1.0, ptr<double>(c->D4),
                ptr<double>(c->V), st, pdv, nb);
      launch_ur(ls, 0, c->n, ld, cc, c->kp, -1.0, 0.0, ptr<double>(c->D4), ptr<double>(c->V),
                ptr<double>(c->U), ptr<double>(c->R), ptr<double>(c->L), st, pdv, nb, pur, nb_ur, j,
                ptr<double>(c->alpha), ptr<double>(c->beta), ptr<double>(c->resid));
      launch_zd(ls, 0, c->n, ld, c->kp, -1.0, ptr<double>(c->R), ptr<double>(c->L), ptr<double>(c->D4),
                ptr<double>(c->Z0), st, nb_zd);
    }
    c->stream = user;
    return rc;
  };
  bool replayed = false;
  if (c->use_graph && !c->time_mm && c->cap) {
    LoopKey key{c->alloc_epoch, c->tune_epoch, mode, c->prob.kernel, c->n, c->d, cc, ld, c->kp, c->maxit, c->m,
                c->khat_tri ? 1 : 0, (int)c->prob.n_lengthscale};
    // graphs recorded against buffers or tuning values that are gone can never be replayed again
    for (size_t i = 0; i < c->graphs.size();) {
      if (c->graphs[i].key.alloc_epoch != c->alloc_epoch || c->graphs[i].key.tune_epoch != c->tune_epoch) {
        if (c->graphs[i].exec) (void)hipGraphExecDestroy(c->graphs[i].exec);
        c->graphs.erase(c->graphs.begin() + (long)i);
      } else {
        ++i;
      }
    }
    bbmm_ctx::LoopGraph* g = nullptr;
    for (auto& e : c->graphs)
      if (e.key == key) g = &e;
    if (!g) {
      // first run with this launch sequence: kernel by kernel (it also lays out plans and grows
      // buffers, which a capture must not do); if nothing was allocated the next run captures it
      int rc = launch_loop(s, false);
      if (rc) return rc;
      replayed = true;
      if (key.alloc_epoch == c->alloc_epoch) {
        if (c->graphs.size() >= 8) {
          size_t old = 0;
          for (size_t i = 1; i < c->graphs.size(); ++i)
            if (c->graphs[i].used < c->graphs[old].used) old = i;
          if (c->graphs[old].exec) (void)hipGraphExecDestroy(c->graphs[old].exec);
          c->graphs.erase(c->graphs.begin() + (long)old);
        }
        c->graphs.push_back(bbmm_ctx::LoopGraph{key, nullptr, ++c->graph_clock});
      }
    } else {
      if (!g->exec) {
        hipGraph_t graph = nullptr;
        bool ok = hipStreamBeginCapture(c->cap, hipStreamCaptureModeThreadLocal) == hipSuccess;
        int rc = BBMM_OK;
        if (ok) {
          rc = launch_loop(c->cap, false);
          ok = hipStreamEndCapture(c->cap, &graph) == hipSuccess && graph != nullptr && rc == BBMM_OK;
        }
        if (ok) ok = hipGraphInstantiate(&g->exec, graph, nullptr, nullptr, 0) == hipSuccess;
        if (graph) (void)hipGraphDestroy(graph);
        if (!ok) {
          // no graph on this runtime / for this sequence: stay with kernel-by-kernel launches
          (void)hipGetLastError();
          g->exec = nullptr;
          c->use_graph = 0;
          if (rc) return rc;
        } else {
          ++c->graph_captures;
        }
      }
      if (g->exec) {
        HIPCHK(c, hipGraphLaunch(g->exec, s));
        g->used = ++c->graph_clock;
        ++c->graph_replays;
        replayed = true;
      }
    }
  }
  if (!replayed) {
    int rc = launch_loop(s, c->time_mm);
    if (rc) return rc;
  }
  c->mbcg_done = true;
  c->last_c = cc;
  c->last_ld = ld;
  c->last_t = cc - 1;
  return BBMM_OK;
}

int stage_slq(bbmm_ctx* c, hipStream_t s) {
  if (!c->mbcg_done || c->last_t < 1) return fail(c, BBMM_EINVAL, "bbmm_mbcg with at least one probe column must run first");
  launch_slq(s, ptr<double>(c->alpha), ptr<double>(c->beta), c->last_t, c->slq_eig ? 1 : 0, eig_sweeps_of(c),
             ptr<DevState>(c->st));
  return BBMM_OK;
}

int stage_dk_sgpr(bbmm_ctx* c, int ld, int t);

// Derivative pass on U (padded, stride ld; columns 0..t) and Z0 (columns 1..t = W).
int stage_dk(bbmm_ctx* c, int ld, int t) {
  if (c->sgpr) return stage_dk_sgpr(c, ld, t);
  hipStream_t s = c->stream;
  int ard = (c->prob.n_lengthscale > 1) ? 1 : 0;
  // S = (U W^T + W U^T) / (2t): operands [U, W] / (2t) and [W, U], so that S is symmetric and the
  // pass needs only the tiles on and above the diagonal
  int ncol = 2 * t;
  int TS = (ncol + 3) / 4;
  size_t opsz = (size_t)(c->np / 16) * TS * 64;
  float* SA = ptr<float>(c->SA);
  float* SB = ptr<float>(c->SB);
  {
    ZeroSegs z = {{SA, SB}, {opsz, opsz}, 2};
    launch_fill_multi0(s, z);
  }
  const double* U = ptr<double>(c->U);
  const double* Z0 = ptr<double>(c->Z0);
  float h = 0.5f / (float)t;
  launch_swizzle_cols(s, U, ld, c->n, c->np, 1, t, TS, 0, h, SA);
  launch_swizzle_cols(s, Z0, ld, c->n, c->np, 1, t, TS, t, h, SA);
  launch_swizzle_cols(s, Z0, ld, c->n, c->np, 1, t, TS, 0, 1.f, SB);
  launch_swizzle_cols(s, U, ld, c->n, c->np, 1, t, TS, t, 1.f, SB);
  launch_extract_col(s, U, ld, c->n, c->np, 0, ptr<float>(c->u0v));
  int ns = dk_split_of(c);
  if (launch_dk(s, c->prob.kernel, c->KK, ard, TS, ptr<float>(c->Xa), ptr<float>(c->Xb), ptr<float>(c->sq),
                ptr<float>(c->Xs), ptr<float>(c->X4), SA, SB, ptr<float>(c->u0v), c->np, ns,
                ptr<double>(c->dkpartial), kDkStride, (int)c->dk_rows_cap, ptr<DevState>(c->st)))
    return fail(c, BBMM_EINVAL, "derivative pass: unsupported configuration");
  int nls = ard ? c->dp : 1;
  launch_noise_terms(s, U, Z0, c->prob.y, c->n, ld, t, nls + 1, ptr<DevState>(c->st), ptr<double>(c->partial),
                     ptr<double>(c->gpartial), vec_blocks(c->n, ld));
  return BBMM_OK;
}

// Derivative terms of the SoR matrix on U (padded, stride ld; columns 0..t) and Z0 (columns 1..t = W).
int stage_dk_sgpr(bbmm_ctx* c, int ld, int t) {
  if (!c->sgpr_built) return fail(c, BBMM_EINVAL, "bbmm_sgpr_build must run first");
  hipStream_t s = c->stream;
  DevState* st = ptr<DevState>(c->st);
  int ard = (c->prob.n_lengthscale > 1) ? 1 : 0;
  int NT = (2 * t <= 32) ? 32 : 64;
  const double* U = ptr<double>(c->U);
  const double* Z0 = ptr<double>(c->Z0);
  // the streaming product skips its work when the stop flag is set; iters_run (next to it) stays
  launch_fill_bytes0(s, &st->done, sizeof(int));
  // T_U = A^T U, T_W = A^T Z0 (m x ld), then b = G^{-T} T = K_UU^{-1} K_UX (.)
  const double* blocks[2] = {U, Z0};
  double* tout[2] = {ptr<double>(c->TU), ptr<double>(c->TW)};
  double* bout[2] = {ptr<double>(c->BU), ptr<double>(c->BW)};
  for (int h = 0; h < 2; ++h) {
    launch_rows_to_d4(s, blocks[h], c->n, c->np, ld, ptr<double>(c->tmpA));
    VpShape sh{0, nullptr, 1};
    int rc = sgpr_first_pass(c, ld, ptr<double>(c->tmpA), &sh);
    if (rc) return rc;
    launch_sgpr_mid_rows(s, ptr<double>(c->Tp), sh, c->mp, ld, tout[h]);
    launch_sgpr_bsolve(s, ptr<double>(c->Ginv), tout[h], c->mp, ld, bout[h]);
  }
  float* PR = ptr<float>(c->SA);           // np x NT
  float* qr = ptr<float>(c->u0v);          // np
  size_t mp = (size_t)c->mp;
  float* PCx = ptr<float>(c->dkops);
  float* PRu = PCx + mp * 64;
  float* PCu = PRu + mp * 64;
  float* qcx = PCu + mp * 64;
  float* qru = qcx + mp;
  launch_sgpr_dk_ops(s, U, Z0, bout[0], bout[1], c->n, c->np, c->m, c->mp, ld, t, NT, PR, qr, PCx, qcx, PRu,
                     qru, PCu);
  double* partial = ptr<double>(c->dkpartial);
  // one partial row per block of each pair sum; the (U, U) rows follow the (X, U) rows
  int col_chunks = (c->m + 127) / 128;
  int nb1 = (c->np / 256) * col_chunks, nb2 = (c->mp / 256) * col_chunks;
  if ((size_t)(nb1 + nb2) > c->dk_rows_cap) return fail(c, BBMM_EINVAL, "internal: derivative partial rows");
  if (launch_dk_rect(s, c->prob.kernel, c->dp, NT, ard, ptr<float>(c->Xs), ptr<float>(c->Us), PR, qr, PCx, qcx,
                     c->np, c->m, partial, kDkStride) != nb1 ||
      launch_dk_rect(s, c->prob.kernel, c->dp, NT, ard, ptr<float>(c->Us), ptr<float>(c->Us), PRu, qru, PCu, qcx,
                     c->mp, c->m, partial + (size_t)nb1 * kDkStride, kDkStride) != nb2)
    return fail(c, BBMM_EINVAL, "SGPR derivative terms: unsupported configuration");
  int nls = ard ? c->dp : 1;
  launch_dk_finish(s, partial, nb1 + nb2, kDkStride, 2 * nls, st);
  launch_sgpr_sterm(s, tout[0], tout[1], c->mp, ld, t, c->prob.outputscale, nls, st);
  launch_noise_terms(s, U, Z0, c->prob.y, c->n, ld, t, nls + 1, st, ptr<double>(c->partial),
                     ptr<double>(c->gpartial), vec_blocks(c->n, ld));
  return BBMM_OK;
}

// Square of the factor (times 1/l) that the tile kernels' coordinates are scaled by, chosen so that
// the kernel function needs no constant on the distance: RBF k/s = 2^(-r2) with c0 = log2(e)/2,
// Matern-5/2 k/s = poly(a) 2^(-a), a = sqrt(r2), with c0 = 5 log2(e)^2.  Squared distances of the
// derivative pass come out c0 times (Delta/l)^2, which finish_dk divides out.
double coord_scale_sq(int kernel) {
  const double log2e = 1.4426950408889634074;
  return (kernel == BBMM_KERNEL_RBF) ? 0.5 * log2e : 5.0 * log2e * log2e;
}

// Turns the raw accumulators of the derivative pass into trace[h], quad[h] (host side).
void finish_dk(const bbmm_ctx* c, double* trace, double* quad) {
  const DevState* st = c->h_st;
  int nl = (int)c->prob.n_lengthscale;
  int ard = nl > 1;
  int nls_dev = ard ? c->dp : 1;
  double s = c->prob.outputscale;
  // inputs were scaled by sqrt(c0)/l, see coord_scale_sq and HypArgs::xscale
  double c0 = coord_scale_sq(c->prob.kernel);
  for (int h = 0; h < nl; ++h) {
    double f = s / (c0 * c->ls[h]);
    trace[h] = f * st->dk_out[2 * h];
    quad[h] = f * st->dk_out[2 * h + 1];
  }
  trace[nl] = st->dk_out[2 * nls_dev];
  quad[nl] = st->dk_out[2 * nls_dev + 1];
  trace[nl + 1] = st->dk_out[2 * (nls_dev + 1)];
  quad[nl + 1] = st->dk_out[2 * (nls_dev + 1) + 1];
}

int validate(bbmm_ctx* c, const bbmm_problem* in) {
  if (!in) return fail(c, BBMM_EINVAL, "problem is NULL");
  if (in->kernel != BBMM_KERNEL_RBF && in->kernel != BBMM_KERNEL_MATERN52)
    return fail(c, BBMM_EINVAL, "unknown kernel");
  if (in->mode != BBMM_MODE_MATERIALISED && in->mode != BBMM_MODE_ONTHEFLY && in->mode != BBMM_MODE_SGPR)
    return fail(c, BBMM_EINVAL, "unknown mode");
  if (in->mode == BBMM_MODE_SGPR) {
    if (in->m < 1 || in->m > 4096 || in->m > in->n) return fail(c, BBMM_EINVAL, "m must be in 1..min(n, 4096)");
    if (!in->Uind) return fail(c, BBMM_EINVAL, "Uind is NULL");
    if (in->d > 32) return fail(c, BBMM_EINVAL, "SGPR needs d <= 32");
    if (!(in->jitter_rel >= 0.0) || !isfinite(in->jitter_rel)) return fail(c, BBMM_EINVAL, "jitter_rel must be >= 0");
  }
  if (in->n < 1 || in->n > (int64_t)1 << 30) return fail(c, BBMM_EINVAL, "n out of range");
  if (in->d < 1 || in->d > BBMM_MAXD) return fail(c, BBMM_EINVAL, "d must be in 1..64");
  if (in->t < 1 || in->t > BBMM_MAXC - 1) return fail(c, BBMM_EINVAL, "t must be in 1..31");
  if (in->k < 0 || in->k > BBMM_MAXK) return fail(c, BBMM_EINVAL, "k must be in 0..32");
  if (in->k > in->n) return fail(c, BBMM_EINVAL, "k must not exceed n");
  if (in->max_iters < 1 || in->max_iters > BBMM_MAXP) return fail(c, BBMM_EINVAL, "max_iters must be in 1..256");
  if (in->n_lengthscale != 1 && in->n_lengthscale != in->d)
    return fail(c, BBMM_EINVAL, "n_lengthscale must be 1 or d");
  if (!in->lengthscale || !in->X || !in->y || !in->E2) return fail(c, BBMM_EINVAL, "NULL input pointer");
  if (in->k > 0 && !in->E1) return fail(c, BBMM_EINVAL, "E1 is NULL but k > 0");
  if (in->pivots_in)
    for (int64_t a = 0; a < in->k; ++a) {
      if (in->pivots_in[a] < 0 || in->pivots_in[a] >= in->n) return fail(c, BBMM_EINVAL, "pivots_in entry out of range");
      for (int64_t b = 0; b < a; ++b)
        if (in->pivots_in[a] == in->pivots_in[b]) return fail(c, BBMM_EINVAL, "pivots_in entries must be distinct");
    }
  for (int64_t h = 0; h < in->n_lengthscale; ++h)
    if (!(in->lengthscale[h] > 0.0) || !isfinite(in->lengthscale[h]))
      return fail(c, BBMM_EINVAL, "lengthscale must be positive and finite");
  if (!(in->outputscale > 0.0) || !isfinite(in->outputscale)) return fail(c, BBMM_EINVAL, "outputscale must be positive");
  if (!(in->noise > 0.0) || !isfinite(in->noise)) return fail(c, BBMM_EINVAL, "noise must be positive");
  return BBMM_OK;
}

}  // namespace

// ================================================================== public ABI
extern "C" {

int bbmm_create(bbmm_ctx** out, int device, void* hip_stream) {
  if (!out) return BBMM_EINVAL;
  *out = nullptr;
  int ndev = 0;
  if (hipGetDeviceCount(&ndev) != hipSuccess || device < 0 || device >= ndev) return BBMM_EHIP;
  if (hipSetDevice(device) != hipSuccess) return BBMM_EHIP;
  bbmm_ctx* c = new bbmm_ctx();
  c->device = device;
  int cus = 0;
  if (hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, device) == hipSuccess && cus > 0)
    c->num_cus = cus;
  c->stream = reinterpret_cast<hipStream_t>(hip_stream);
  if (scratch_of(device, &c->eig_static) != hipSuccess) {
    delete c;
    return BBMM_EHIP;
  }
  if (hipHostMalloc((void**)&c->h_eig_status, sizeof(int) * BBMM_EIG_NOALLOC_MAX, hipHostMallocDefault) != hipSuccess ||
      hipHostMalloc((void**)&c->h_st, sizeof(DevState), hipHostMallocDefault) != hipSuccess ||
      hipHostMalloc((void**)&c->h_hist, sizeof(double) * 3 * BBMM_MAXP * BBMM_MAXC, hipHostMallocDefault) != hipSuccess) {
    delete c;
    return BBMM_ENOMEM;
  }
  if (hipStreamCreateWithFlags(&c->cap, hipStreamNonBlocking) != hipSuccess) c->cap = nullptr;   // no graphs then
  if (hipStreamCreateWithFlags(&c->side, hipStreamNonBlocking) != hipSuccess ||
      hipEventCreateWithFlags(&c->ev_fork, hipEventDisableTiming) != hipSuccess ||
      hipEventCreateWithFlags(&c->ev_join, hipEventDisableTiming) != hipSuccess) {
    bbmm_destroy(c);
    return BBMM_EHIP;
  }
  *out = c;
  return BBMM_OK;
}

int bbmm_destroy(bbmm_ctx* c) {
  if (!c) return BBMM_OK;
  (void)hipSetDevice(c->device);
  (void)hipStreamSynchronize(c->stream);
  if (c->side) {
    (void)hipStreamSynchronize(c->side);
    (void)hipStreamDestroy(c->side);
  }
  for (auto& g : c->graphs)
    if (g.exec) (void)hipGraphExecDestroy(g.exec);
  if (c->cap) (void)hipStreamDestroy(c->cap);
  if (c->ev_fork) (void)hipEventDestroy(c->ev_fork);
  if (c->ev_join) (void)hipEventDestroy(c->ev_join);
  Buf* bufs[] = {&c->Xa, &c->Xb, &c->Xs, &c->X4, &c->sq, &c->Khat, &c->L, &c->delta, &c->U, &c->R, &c->V,
                 &c->Z0, &c->D4, &c->Vp, &c->partial, &c->gpartial, &c->alpha, &c->beta, &c->resid, &c->st, &c->sym.pieces, &c->sym.first0, &c->sym.first1, &c->sym.base, &c->sym.tot, &c->otft.pieces, &c->otft.first0,
                 &c->otft.first1, &c->otft.base, &c->otft.tot, &c->tmpA,
                 &c->tmpB, &c->SA, &c->SB, &c->u0v, &c->dkpartial, &c->eig, &c->plan[0], &c->plan[1], &c->plan[2], &c->nseg[0],
                 &c->nseg[1], &c->nseg[2], &c->KUU, &c->Gm, &c->Ginv, &c->Kux, &c->AT, &c->A, &c->qdiag, &c->Tp, &c->T4,
                 &c->sgplan[0], &c->sgplan[1], &c->sgplan[2], &c->sgplan[3], &c->sgnseg[0], &c->sgnseg[1],
                 &c->sgnseg[2], &c->sgnseg[3], &c->Ua, &c->Ub, &c->Us, &c->U4, &c->usq, &c->TU, &c->TW, &c->BU,
                 &c->BW, &c->dkops};
  for (Buf* b : bufs)
    if (b->p) (void)hipFree(b->p);
  for (hipEvent_t e : c->ev) (void)hipEventDestroy(e);
  if (c->h_eig_status) (void)hipHostFree(c->h_eig_status);
  if (c->h_st) (void)hipHostFree(c->h_st);
  if (c->h_hist) (void)hipHostFree(c->h_hist);
  delete c;
  return BBMM_OK;
}

const char* bbmm_last_error(const bbmm_ctx* c) { return c ? c->err.c_str() : "context is NULL"; }

int bbmm_tune(bbmm_ctx* c, const char* key, int64_t value) {
  if (!c || !key) return BBMM_EINVAL;
  ++c->tune_epoch;
  if (!strcmp(key, "loop_graph")) {
    c->use_graph = value != 0;
    return BBMM_OK;
  }
  if (!strcmp(key, "mat_wgs")) c->mat_wgs = value > 0 ? value : 0;
  else if (!strcmp(key, "otf_split")) c->otf_split = value > 0 ? value : 0;
  else if (!strcmp(key, "otf_sym")) c->otf_sym = value <= 0 ? 0 : (value == 1 ? 1 : 2);   // off / by size / always
  else if (!strcmp(key, "ur_blocks")) c->ur_blocks_cap = value > 0 ? value : 0;
  else if (!strcmp(key, "khat_sym")) {
    if (value != 0 && value != 1) return fail(c, BBMM_EINVAL, "khat_sym must be 0 or 1");
    if (c->khat_sym != value) c->khat_built = false;   // the stored matrix has the other layout
    c->khat_sym = value;
  } else if (!strcmp(key, "khat_panel")) {
    if (value > 1 && value % 256 != 0) return fail(c, BBMM_EINVAL, "khat_panel must be 1 or a multiple of 256");
    c->khat_panel = value > 0 ? value : 0;
    c->khat_built = false;
  } else if (!strcmp(key, "zd_blocks")) c->zd_blocks = value > 0 ? std::min<int64_t>(value, 64) : 0;
  else if (!strcmp(key, "sgpr_wgs1")) c->sgpr_wgs[0] = value > 0 ? value : 0;
  else if (!strcmp(key, "sgpr_wgs2")) c->sgpr_wgs[1] = value > 0 ? value : 0;
  else if (!strcmp(key, "slq_eig")) c->slq_eig = value > 0;
  else if (!strcmp(key, "eig_sweeps")) c->eig_sweeps = value > 0 ? std::min<int64_t>(value, 1000) : 0;
  else if (!strcmp(key, "time_mm")) c->time_mm = value > 0;
  else return fail(c, BBMM_EINVAL, std::string("unknown tuning key: ") + key);
  return BBMM_OK;
}

int bbmm_loop_graph_stats(bbmm_ctx* c, int64_t* captures, int64_t* replays) {
  if (!c) return BBMM_EINVAL;
  if (captures) *captures = c->graph_captures;
  if (replays) *replays = c->graph_replays;
  return BBMM_OK;
}

int bbmm_mm_timing(bbmm_ctx* c, double* avg_ms, double* total_ms, int64_t* launches) {
  if (!c) return BBMM_EINVAL;
  if (!c->time_mm || c->ev_iters == 0 || !c->h_st)
    return fail(c, BBMM_EINVAL, "no timed mBCG run: set bbmm_tune(\"time_mm\", 1) and run the solver first");
  HIPCHK(c, hipSetDevice(c->device));
  HIPCHK(c, hipStreamSynchronize(c->stream));
  int n_it = std::min(c->ev_iters, std::max(1, c->h_st->iters_run));
  double tot = 0.0;
  for (int j = 0; j < n_it; ++j) {
    float ms = 0.f;
    HIPCHK(c, hipEventElapsedTime(&ms, c->ev[2 * j], c->ev[2 * j + 1]));
    tot += (double)ms;
  }
  if (avg_ms) *avg_ms = tot / n_it;
  if (total_ms) *total_ms = tot;
  if (launches) *launches = n_it;
  return BBMM_OK;
}

int bbmm_setup(bbmm_ctx* c, const bbmm_problem* in) {
  if (!c) return BBMM_EINVAL;
  c->is_setup = false;
  int rc = validate(c, in);
  if (rc) return rc;
  HIPCHK(c, hipSetDevice(c->device));
  rc = drain_side(c);
  if (rc) return rc;
  c->prob = *in;
  c->ls.assign(in->lengthscale, in->lengthscale + in->n_lengthscale);
  c->prob.lengthscale = c->ls.data();
  c->forced.clear();
  if (in->pivots_in) c->forced.assign(in->pivots_in, in->pivots_in + in->k);
  c->prob.pivots_in = nullptr;              // the caller's array is not kept
  c->n = (int)in->n;
  c->d = (int)in->d;
  c->t = (int)in->t;
  c->k = (int)in->k;
  c->kp = ((c->k + 7) / 8) * 8;
  c->np = ((c->n + 255) / 256) * 256;
  c->maxit = (int)in->max_iters;
  int KK = 1;
  while (4 * KK < c->d) KK *= 2;
  c->KK = KK;
  c->dp = 4 * KK;
  c->khat_built = c->chol_done = c->pre_done = c->mbcg_done = false;
  c->sgpr = (in->mode == BBMM_MODE_SGPR);
  c->sgpr_built = false;
  c->m = c->sgpr ? (int)in->m : 0;
  c->mp = ((c->m + 255) / 256) * 256;

  memset(&c->hyp, 0, sizeof(HypArgs));
  double c0 = coord_scale_sq(in->kernel);
  for (int dim = 0; dim < c->d; ++dim) {
    double l = (in->n_lengthscale == 1) ? c->ls[0] : c->ls[dim];
    c->hyp.inv_ls[dim] = 1.0 / l;
    c->hyp.xscale[dim] = sqrt(c0) / l;
  }
  c->hyp.outputscale = in->outputscale;
  c->hyp.noise = in->noise;
  c->hyp.kernel = in->kernel;
  c->hyp.d = c->d;

  size_t np = (size_t)c->np;
  size_t blk = np * BBMM_MAXC * sizeof(double);
  size_t opx = np * c->dp * sizeof(float);
  struct { Buf* b; size_t bytes; } want[] = {
      {&c->Xa, opx}, {&c->Xb, opx}, {&c->Xs, opx}, {&c->X4, opx}, {&c->sq, np * sizeof(float)},
      {&c->L, np * std::max(c->kp, 8) * sizeof(double)}, {&c->delta, np * sizeof(double)},
      {&c->U, blk}, {&c->R, blk}, {&c->V, blk}, {&c->Z0, blk}, {&c->D4, blk},
      {&c->partial, sizeof(double) * (size_t)kMaxVecBlocks * (BBMM_MAXK * BBMM_MAXK + (BBMM_MAXK + 1) * BBMM_MAXC)},
      {&c->gpartial, sizeof(double) * 40 * (BBMM_MAXK * BBMM_MAXK + (BBMM_MAXK + 1) * BBMM_MAXC)},
      {&c->alpha, sizeof(double) * BBMM_MAXP * BBMM_MAXC}, {&c->beta, sizeof(double) * BBMM_MAXP * BBMM_MAXC},
      {&c->resid, sizeof(double) * BBMM_MAXP * BBMM_MAXC}, {&c->st, sizeof(DevState)},
      {&c->tmpA, blk}, {&c->tmpB, blk},
      {&c->SA, np * 64 * sizeof(float)}, {&c->SB, np * 64 * sizeof(float)}, {&c->u0v, np * sizeof(float)},
  };
  for (auto& w : want) {
    rc = ensure(c, *w.b, w.bytes);
    if (rc) return rc;
  }
  // one partial row per wave of the derivative pass
  size_t dk_rows = (size_t)((c->np / 16 + 15) / 16) * kMaxSplit * 4;
  rc = ensure(c, c->dkpartial, dk_rows * kDkStride * sizeof(double));
  if (rc) return rc;
  c->dk_rows_cap = dk_rows;

  hipStream_t s = c->stream;
  launch_fill_bytes0(s, c->st.p, sizeof(DevState));
  launch_colmean(s, in->X, c->n, c->d, ptr<DevState>(c->st), ptr<double>(c->partial), ptr<double>(c->gpartial));
  launch_prep_x(s, in->X, c->n, c->d, c->np, c->KK, c->hyp, ptr<DevState>(c->st), ptr<float>(c->Xa),
                ptr<float>(c->Xb), ptr<float>(c->Xs), ptr<float>(c->X4), ptr<float>(c->sq));
  HIPCHK(c, hipGetLastError());
  c->is_setup = true;
  return BBMM_OK;
}

int bbmm_build_khat(bbmm_ctx* c) {
  int rc = check_ready(c);
  if (rc) return rc;
  rc = stage_build_khat(c);
  if (rc) return rc;
  HIPCHK(c, hipGetLastError());
  return BBMM_OK;
}

int bbmm_sgpr_build(bbmm_ctx* c) {
  int rc = check_ready(c);
  if (rc) return rc;
  rc = stage_sgpr_build(c);
  if (rc) return rc;
  rc = fetch_state(c, false);
  if (rc) return rc;
  if (c->h_st->status == BBMM_ENOTPD) return fail(c, BBMM_ENOTPD, "K_UU + jitter I is not positive definite");
  return device_status(c);
}

int bbmm_sgpr_root_rows(bbmm_ctx* c, int64_t row0, int64_t nrows, float* out) {
  int rc = check_ready(c);
  if (rc) return rc;
  if (!c->sgpr_built) return fail(c, BBMM_EINVAL, "bbmm_sgpr_build must run first");
  if (!out || row0 < 0 || nrows < 0 || row0 + nrows > c->n || nrows * (int64_t)c->m > (int64_t)1 << 31)
    return fail(c, BBMM_EINVAL, "rows out of range");
  if (nrows == 0) return BBMM_OK;
  launch_copy_block(c->stream, ptr<float>(c->A), (size_t)c->mp, (size_t)c->np, 0, (int)row0, (int)nrows, 0, c->m, out);
  HIPCHK(c, hipGetLastError());
  return BBMM_OK;
}

int bbmm_khat_block(bbmm_ctx* c, int64_t row0, int64_t nrows, int64_t col0, int64_t ncols, float* out) {
  int rc = check_ready(c);
  if (rc) return rc;
  if (!c->khat_built) return fail(c, BBMM_EINVAL, "bbmm_build_khat must run first");
  if (!out || row0 < 0 || col0 < 0 || nrows < 0 || ncols < 0 || row0 + nrows > c->n || col0 + ncols > c->n ||
      nrows * ncols > (int64_t)1 << 31)
    return fail(c, BBMM_EINVAL, "block out of range");
  if (nrows * ncols == 0) return BBMM_OK;
  launch_copy_block(c->stream, ptr<float>(c->Khat), (size_t)(c->khat_pw > 0 ? c->khat_pw : c->np), (size_t)c->np,
                    c->khat_tri ? 1 : 0, (int)row0, (int)nrows, (int)col0, (int)ncols, out);
  HIPCHK(c, hipGetLastError());
  return BBMM_OK;
}

int bbmm_kernel_mm(bbmm_ctx* c, int32_t mode, const float* M, int64_t cc, float* V) {
  int rc = check_ready(c);
  if (rc) return rc;
  if (!M || !V || cc < 1 || cc > BBMM_MAXC) return fail(c, BBMM_EINVAL, "bad block");
  int ld = ld_for((int)cc);
  hipStream_t s = c->stream;
  launch_fill_bytes0(s, &ptr<DevState>(c->st)->done, 2 * sizeof(int));
  launch_pack_d4(s, M, c->n, (int)cc, c->np, ld, ptr<double>(c->D4));
  VpShape ns{0, nullptr, 1};
  double scaleV = 1.0, addD = 0.0;
  rc = stage_mm(c, mode, (int)cc, ld, &ns, &scaleV, &addD);
  if (rc) return rc;
  launch_vreduce(s, ptr<double>(c->Vp), ns, c->n, c->np, ld, scaleV, addD, ptr<double>(c->D4), ptr<double>(c->V));
  launch_unpack_rows(s, ptr<double>(c->V), ld, c->n, (int)cc, V);
  HIPCHK(c, hipGetLastError());
  return BBMM_OK;
}

int bbmm_pivoted_cholesky(bbmm_ctx* c, double* L, int64_t* pivots, int64_t* rank) {
  int rc = check_ready(c);
  if (rc) return rc;
  rc = stage_pivchol(c);
  if (rc) return rc;
  if (L && c->k > 0) launch_unpack_rows_f64(c->stream, ptr<double>(c->L), c->kp, c->n, c->k, L);
  rc = fetch_state(c, false);
  if (rc) return rc;
  if (pivots)
    for (int m = 0; m < c->k; ++m) pivots[m] = (m < c->h_st->rank) ? c->h_st->piv[m] : -1;
  if (rank) *rank = c->h_st->rank;
  return BBMM_OK;
}

int bbmm_precond_setup(bbmm_ctx* c, double* logdet_precond) {
  int rc = check_ready(c);
  if (rc) return rc;
  rc = stage_pre_setup(c);
  if (rc) return rc;
  rc = fetch_state(c, false);
  if (rc) return rc;
  rc = device_status(c);
  if (rc) return rc;
  if (logdet_precond) *logdet_precond = c->h_st->logdetP;
  return BBMM_OK;
}

int bbmm_precond_solve(bbmm_ctx* c, const float* R, int64_t cc, float* Z) {
  int rc = check_ready(c);
  if (rc) return rc;
  if (!c->pre_done) return fail(c, BBMM_EINVAL, "bbmm_precond_setup must run first");
  if (!R || !Z || cc < 1 || cc > BBMM_MAXC) return fail(c, BBMM_EINVAL, "bad block");
  int ld = ld_for((int)cc);
  hipStream_t s = c->stream;
  DevState* st = ptr<DevState>(c->st);
  int nb = vec_blocks(c->n, ld);
  launch_fill_bytes0(s, &st->done, 2 * sizeof(int));
  launch_pack_rows(s, R, c->n, (int)cc, ld, ptr<double>(c->tmpA));
  launch_ur(s, 1, c->n, ld, (int)cc, c->kp, c->prob.noise, 0.0, ptr<double>(c->D4), ptr<double>(c->V),
            ptr<double>(c->U), ptr<double>(c->tmpA), ptr<double>(c->L), st, ptr<double>(c->gpartial), nb,
            ptr<double>(c->partial), ur_blocks(c, c->n, ld), 0, ptr<double>(c->alpha), ptr<double>(c->beta),
            ptr<double>(c->resid));
  launch_psolve_apply(s, c->n, ld, c->kp, c->prob.noise, ptr<double>(c->tmpA), ptr<double>(c->L),
                      ptr<double>(c->tmpB), st, nb);
  launch_unpack_rows(s, ptr<double>(c->tmpB), ld, c->n, (int)cc, Z);
  c->mbcg_done = false;
  HIPCHK(c, hipGetLastError());
  return BBMM_OK;
}

int bbmm_make_probes(bbmm_ctx* c, float* B) {
  int rc = check_ready(c);
  if (rc) return rc;
  if (!c->chol_done) return fail(c, BBMM_EINVAL, "bbmm_pivoted_cholesky must run first");
  if (!B) return fail(c, BBMM_EINVAL, "B is NULL");
  int cc = c->t + 1, ld = ld_for(cc);
  launch_probes(c->stream, c->prob.y, c->prob.E1, c->prob.E2, ptr<double>(c->L), c->n, c->t, c->kp, ld,
                c->prob.noise, ptr<DevState>(c->st), ptr<double>(c->tmpA));
  launch_unpack_rows(c->stream, ptr<double>(c->tmpA), ld, c->n, cc, B);
  HIPCHK(c, hipGetLastError());
  return BBMM_OK;
}

int bbmm_mbcg(bbmm_ctx* c, int32_t mode, const float* B, int64_t cc, float* U, double* alpha, double* beta,
              double* resid, int64_t* iters_run) {
  int rc = check_ready(c);
  if (rc) return rc;
  if (!B || !U || cc < 1 || cc > BBMM_MAXC) return fail(c, BBMM_EINVAL, "bad block");
  int ld = ld_for((int)cc);
  launch_pack_rows(c->stream, B, c->n, (int)cc, ld, ptr<double>(c->R));
  rc = stage_mbcg(c, mode, (int)cc, ld, c->prob.u0_init);
  if (rc) return rc;
  launch_unpack_rows(c->stream, ptr<double>(c->U), ld, c->n, (int)cc, U);
  rc = fetch_state(c, true);
  if (rc) return rc;
  int it = c->h_st->iters_run;
  if (iters_run) *iters_run = it;
  double* dst[3] = {alpha, beta, resid};
  for (int a = 0; a < 3; ++a)
    if (dst[a])
      for (int j = 0; j < c->maxit; ++j)
        for (int q = 0; q < cc; ++q)
          dst[a][(size_t)j * cc + q] = c->h_hist[(size_t)a * BBMM_MAXP * BBMM_MAXC + (size_t)j * BBMM_MAXC + q];
  return BBMM_OK;
}

int bbmm_predict_mean(bbmm_ctx* c, const float* Xstar, int64_t ns, const float* u0, float* mean) {
  int rc = check_ready(c);
  if (rc) return rc;
  if (!Xstar || !u0 || !mean || ns < 1 || ns > (1 << 30)) return fail(c, BBMM_EINVAL, "bad test block");
  hipStream_t s = c->stream;
  if (c->sgpr) {
    // SoR prior: mean = k_{*U} K_UU^{-1} K_UX u0 = k_{*U} b0 with b0 = G^{-T} (A^T u0)
    if (!c->sgpr_built) return fail(c, BBMM_EINVAL, "bbmm_sgpr_build must run first");
    launch_fill_bytes0(s, &ptr<DevState>(c->st)->done, sizeof(int));
    launch_fill_f64(s, ptr<double>(c->tmpA), (size_t)c->np * 16, 0.0);
    launch_warm_rhs(s, u0, c->n, 16, ptr<double>(c->tmpA));
    VpShape sh{0, nullptr, 1};
    rc = sgpr_first_pass(c, 16, ptr<double>(c->tmpA), &sh);
    if (rc) return rc;
    launch_sgpr_mid_rows(s, ptr<double>(c->Tp), sh, c->mp, 16, ptr<double>(c->TU));
    launch_sgpr_bsolve(s, ptr<double>(c->Ginv), ptr<double>(c->TU), c->mp, 16, ptr<double>(c->BU));
    launch_cross_dot(s, c->prob.Uind, Xstar, c->m, (int)ns, c->hyp, ptr<double>(c->BU), 16, 0, 0.0, 1.0, mean);
    HIPCHK(c, hipGetLastError());
    return BBMM_OK;
  }
  launch_pack_rows(s, u0, c->n, 1, 16, ptr<double>(c->tmpB));
  launch_cross_dot(s, c->prob.X, Xstar, c->n, (int)ns, c->hyp, ptr<double>(c->tmpB), 16, 0, 0.0, 1.0, mean);
  HIPCHK(c, hipGetLastError());
  return BBMM_OK;
}

int bbmm_predict_var(bbmm_ctx* c, int32_t mode, const float* Xstar, int64_t ns, float* var,
                     int64_t* iters_run, double* max_resid) {
  int rc = check_ready(c);
  if (rc) return rc;
  if (!Xstar || !var || ns < 1 || ns > BBMM_MAXC)
    return fail(c, BBMM_EINVAL, "bad test block (1 <= ns <= 32 per call)");
  if (!c->pre_done) return fail(c, BBMM_EINVAL, "bbmm_precond_setup must run first");
  hipStream_t s = c->stream;
  int ld = ld_for((int)ns);
  if (c->sgpr) {
    // SoR prior: q(x*, x*) = |v|^2 and the right-hand sides Q_{X x*} = A v with v = G^{-1} k_{U x*}
    if (mode != BBMM_MODE_SGPR) return fail(c, BBMM_EINVAL, "an SGPR problem takes mode SGPR");
    size_t mb = (size_t)c->mp * ld;
    launch_fill_bytes0(s, &ptr<DevState>(c->st)->done, sizeof(int));
    launch_fill_f64(s, ptr<double>(c->TU), mb, 0.0);
    launch_cross_block(s, c->prob.Uind, Xstar, c->m, (int)ns, ld, c->hyp, ptr<double>(c->TU));
    launch_sgpr_fsolve(s, ptr<double>(c->Ginv), ptr<double>(c->TU), c->mp, ld, ptr<double>(c->BU));
    launch_colnorm2(s, ptr<double>(c->BU), c->mp, ld, ptr<double>(c->TW));
    launch_rows_to_d4(s, ptr<double>(c->BU), c->mp, c->mp, ld, ptr<double>(c->T4));
    VpShape sh{0, nullptr, 1};
    rc = sgpr_second_pass(c, ld, &sh);
    if (rc) return rc;
    launch_fill_f64(s, ptr<double>(c->D4), (size_t)c->np * ld, 0.0);
    launch_vreduce(s, ptr<double>(c->Vp), sh, c->n, c->np, ld, 1.0, 0.0, ptr<double>(c->D4), ptr<double>(c->R));
    HIPCHK(c, hipMemcpyAsync(c->tmpB.p, c->R.p, sizeof(double) * (size_t)c->np * ld, hipMemcpyDeviceToDevice, s));
    rc = stage_mbcg(c, mode, (int)ns, ld);
    if (rc) return rc;
    launch_coldot_var(s, ptr<double>(c->tmpB), ptr<double>(c->U), c->n, ld, (int)ns, ptr<double>(c->TW), var);
  } else {
    launch_cross_block(s, c->prob.X, Xstar, c->n, (int)ns, ld, c->hyp, ptr<double>(c->R));
    rc = stage_mbcg(c, mode, (int)ns, ld);
    if (rc) return rc;
    launch_cross_dot(s, c->prob.X, Xstar, c->n, (int)ns, c->hyp, ptr<double>(c->U), ld, 1,
                     c->prob.outputscale, -1.0, var);
  }
  rc = fetch_state(c, true);
  if (rc) return rc;
  rc = device_status(c);
  if (rc) return rc;
  int it = c->h_st->iters_run;
  if (iters_run) *iters_run = it;
  if (max_resid) {
    double m = 0.0;
    if (it > 0)
      for (int q = 0; q < (int)ns; ++q)
        m = std::max(m, c->h_hist[(size_t)2 * BBMM_MAXP * BBMM_MAXC + (size_t)(it - 1) * BBMM_MAXC + q]);
    *max_resid = m;
  }
  return BBMM_OK;
}

// Copies the batch to `work` (device, room for 3 nd + no doubles and `batch` ints), runs the
// eigen-solver there and copies values, first rows and the per-matrix status (to `status`, host,
// `batch` ints) back.
static int run_tridiag_eig(bbmm_ctx* c, double* work, int* status, const double* diag, const double* off,
                           int64_t m, int64_t batch, double* eigvals, double* first_row) {
  size_t nd = (size_t)batch * m, no = (size_t)batch * (m > 1 ? m - 1 : 1);
  double* d_diag = work;
  double* d_off = d_diag + nd;
  double* d_val = d_off + no;
  double* d_vec = d_val + nd;
  int* d_status = reinterpret_cast<int*>(d_vec + nd);
  HIPCHK(c, hipMemcpyAsync(d_diag, diag, sizeof(double) * nd, hipMemcpyHostToDevice, c->stream));
  if (m > 1) HIPCHK(c, hipMemcpyAsync(d_off, off, sizeof(double) * batch * (m - 1), hipMemcpyHostToDevice, c->stream));
  launch_tridiag_eig(c->stream, d_diag, d_off, (int)m, (int)batch, eig_sweeps_of(c), d_val, d_vec, d_status);
  HIPCHK(c, hipMemcpyAsync(eigvals, d_val, sizeof(double) * nd, hipMemcpyDeviceToHost, c->stream));
  HIPCHK(c, hipMemcpyAsync(first_row, d_vec, sizeof(double) * nd, hipMemcpyDeviceToHost, c->stream));
  HIPCHK(c, hipMemcpyAsync(status, d_status, sizeof(int) * (size_t)batch, hipMemcpyDeviceToHost, c->stream));
  HIPCHK(c, hipStreamSynchronize(c->stream));
  HIPCHK(c, hipGetLastError());
  for (int64_t b = 0; b < batch; ++b)
    if (status[b] != 0) {
      char msg[128];
      snprintf(msg, sizeof msg, "tridiagonal matrix %lld of the batch was not reduced within the sweep budget",
               (long long)b);
      return fail(c, BBMM_ENOCONV, msg);
    }
  return BBMM_OK;
}

int bbmm_tridiag_eig_batched(bbmm_ctx* c, const double* diag, const double* off, int64_t m, int64_t batch,
                             double* eigvals, double* first_row) {
  if (!c) return BBMM_EINVAL;
  if (!diag || !eigvals || !first_row || m < 1 || m > BBMM_MAXP || batch < 1 || batch > 65535 || (m > 1 && !off))
    return fail(c, BBMM_EINVAL, "bad tridiagonal batch");
  HIPCHK(c, hipSetDevice(c->device));
  size_t nd = (size_t)batch * m, no = (size_t)batch * (m > 1 ? m - 1 : 1);
  int rc = ensure(c, c->eig, sizeof(double) * (3 * nd + no) + sizeof(int) * (size_t)batch);
  if (rc) return rc;
  std::vector<int> status((size_t)batch, 0);
  return run_tridiag_eig(c, ptr<double>(c->eig), status.data(), diag, off, m, batch, eigvals, first_row);
}

int bbmm_tridiag_eig_batched_noalloc(bbmm_ctx* c, const double* diag, const double* off, int64_t m,
                                     int64_t batch, double* eigvals, double* first_row) {
  if (!c) return BBMM_EINVAL;
  if (!diag || !eigvals || !first_row || m < 1 || m > BBMM_MAXP || batch < 1 || (m > 1 && !off))
    return fail(c, BBMM_EINVAL, "bad tridiagonal batch");
  if (batch > BBMM_EIG_NOALLOC_MAX || batch * m > BBMM_EIG_NOALLOC_MAX)
    return fail(c, BBMM_EINVAL, "batch * m exceeds the 16384 entries of the static work area");
  HIPCHK(c, hipSetDevice(c->device));
  // same kernel and staging order as bbmm_tridiag_eig_batched; the work area is this device's
  // copy of `scratch`, every word the kernel or the copies read is written first
  return run_tridiag_eig(c, c->eig_static, c->h_eig_status, diag, off, m, batch, eigvals, first_row);
}

int bbmm_slq_from_coeffs(bbmm_ctx* c, const double* alpha, const double* beta, const double* rho0,
                         const int64_t* m_valid, int64_t p, int64_t t, double logdet_precond, double* logdet,
                         double* slq_terms) {
  if (!c) return BBMM_EINVAL;
  if (!alpha || !beta || !rho0 || p < 1 || p > BBMM_MAXP || t < 1 || t > BBMM_MAXC - 1 || (!logdet && !slq_terms))
    return fail(c, BBMM_EINVAL, "bad coefficient arrays (1 <= p <= 256, 1 <= t <= 31)");
  std::vector<int> mv((size_t)t, (int)p);
  if (m_valid)
    for (int64_t i = 0; i < t; ++i) {
      if (m_valid[i] < 0 || m_valid[i] > p) return fail(c, BBMM_EINVAL, "m_valid entry outside 0..p");
      mv[(size_t)i] = (int)m_valid[i];
    }
  HIPCHK(c, hipSetDevice(c->device));
  size_t np_ = (size_t)p * t;
  int rc = ensure(c, c->eig, sizeof(double) * (2 * np_ + 2 * (size_t)t) + sizeof(int) * 2 * (size_t)t);
  if (rc) return rc;
  double* d_alpha = ptr<double>(c->eig);
  double* d_beta = d_alpha + np_;
  double* d_rho0 = d_beta + np_;
  double* d_terms = d_rho0 + t;
  int* d_mv = reinterpret_cast<int*>(d_terms + t);
  int* d_status = d_mv + t;
  std::vector<double> terms((size_t)t, 0.0);
  std::vector<int> status((size_t)t, 0);
  hipStream_t s = c->stream;
  HIPCHK(c, hipMemcpyAsync(d_alpha, alpha, sizeof(double) * np_, hipMemcpyHostToDevice, s));
  HIPCHK(c, hipMemcpyAsync(d_beta, beta, sizeof(double) * np_, hipMemcpyHostToDevice, s));
  HIPCHK(c, hipMemcpyAsync(d_rho0, rho0, sizeof(double) * (size_t)t, hipMemcpyHostToDevice, s));
  HIPCHK(c, hipMemcpyAsync(d_mv, mv.data(), sizeof(int) * (size_t)t, hipMemcpyHostToDevice, s));
  launch_slq_coeffs(s, d_alpha, d_beta, d_rho0, d_mv, (int)t, c->slq_eig ? 1 : 0, eig_sweeps_of(c), d_terms, d_status);
  HIPCHK(c, hipMemcpyAsync(terms.data(), d_terms, sizeof(double) * (size_t)t, hipMemcpyDeviceToHost, s));
  HIPCHK(c, hipMemcpyAsync(status.data(), d_status, sizeof(int) * (size_t)t, hipMemcpyDeviceToHost, s));
  HIPCHK(c, hipStreamSynchronize(s));
  HIPCHK(c, hipGetLastError());
  double sum = 0.0;
  for (int64_t i = 0; i < t; ++i) {
    if (status[(size_t)i] == BBMM_ENOCONV)
      return fail(c, BBMM_ENOCONV, "the eigen-solver did not reduce a Lanczos tridiagonal within its sweep budget");
    if (status[(size_t)i] != 0) return fail(c, BBMM_ENONFINITE, "non-finite value in the log-determinant estimate");
    sum += terms[(size_t)i];
    if (slq_terms) slq_terms[i] = terms[(size_t)i];
  }
  if (logdet) *logdet = logdet_precond + sum / (double)t;
  return BBMM_OK;
}

int bbmm_slq_logdet(bbmm_ctx* c, double* logdet, double* slq_terms) {
  int rc = check_ready(c);
  if (rc) return rc;
  rc = stage_slq(c, c->stream);
  if (rc) return rc;
  rc = fetch_state(c, false);
  if (rc) return rc;
  rc = device_status(c);
  if (rc) return rc;
  if (logdet) *logdet = c->h_st->logdetP + c->h_st->slq_mean;
  if (slq_terms)
    for (int i = 0; i < c->last_t; ++i) slq_terms[i] = c->h_st->slq_terms[i];
  return BBMM_OK;
}

int bbmm_dk_traces(bbmm_ctx* c, const float* U, const float* W, double* trace, double* quad) {
  int rc = check_ready(c);
  if (rc) return rc;
  if (!U || !W || !trace || !quad) return fail(c, BBMM_EINVAL, "NULL pointer");
  int cc = c->t + 1, ld = ld_for(cc);
  hipStream_t s = c->stream;
  launch_pack_rows(s, U, c->n, cc, ld, ptr<double>(c->U));
  launch_fill_f64(s, ptr<double>(c->Z0), (size_t)c->np * ld, 0.0);
  launch_pack_cols_at(s, W, c->n, c->t, ld, 1, ptr<double>(c->Z0));
  c->mbcg_done = false;
  rc = stage_dk(c, ld, c->t);
  if (rc) return rc;
  rc = fetch_state(c, false);
  if (rc) return rc;
  finish_dk(c, trace, quad);
  return BBMM_OK;
}

int bbmm_solve_logdet_grad(bbmm_ctx* c, const bbmm_problem* in, bbmm_result* out) {
  if (!c) return BBMM_EINVAL;
  if (!out || !out->u0 || !out->trace || !out->quad || !out->grad_nlml)
    return fail(c, BBMM_EINVAL, "result struct, u0, trace, quad and grad_nlml are required");
  int rc = bbmm_setup(c, in);
  if (rc) return rc;
  hipStream_t s = c->stream;
  int cc = c->t + 1, ld = ld_for(cc);
  if (in->mode == BBMM_MODE_MATERIALISED) {
    rc = stage_build_khat(c);
    if (rc) return rc;
  } else if (in->mode == BBMM_MODE_SGPR) {
    rc = stage_sgpr_build(c);
    if (rc) return rc;
  }
  rc = stage_pivchol(c);
  if (rc) return rc;
  rc = stage_pre_setup(c);
  if (rc) return rc;
  launch_probes(s, in->y, in->E1, in->E2, ptr<double>(c->L), c->n, c->t, c->kp, ld, in->noise,
                ptr<DevState>(c->st), ptr<double>(c->R));
  rc = stage_mbcg(c, in->mode, cc, ld, in->u0_init);
  if (rc) return rc;
  // The eigensolves need only the coefficient histories and the derivative pass only the solves:
  // they run side by side, the SLQ kernel on the context's second stream.
  HIPCHK(c, hipEventRecord(c->ev_fork, s));
  HIPCHK(c, hipStreamWaitEvent(c->side, c->ev_fork, 0));
  c->side_busy = true;
  rc = stage_slq(c, c->side);
  if (rc) return rc;
  HIPCHK(c, hipEventRecord(c->ev_join, c->side));
  rc = stage_dk(c, ld, c->t);
  if (rc) return rc;
  launch_extract_col(s, ptr<double>(c->U), ld, c->n, c->n, 0, out->u0);
  if (out->U) launch_unpack_rows(s, ptr<double>(c->U), ld, c->n, cc, out->U);
  HIPCHK(c, hipStreamWaitEvent(s, c->ev_join, 0));
  c->side_busy = false;
  rc = fetch_state(c, true);
  if (rc) return rc;
  rc = device_status(c);
  if (rc) return rc;

  const DevState* st = c->h_st;
  int nl = (int)in->n_lengthscale;
  finish_dk(c, out->trace, out->quad);
  for (int h = 0; h < nl + 2; ++h) out->grad_nlml[h] = 0.5 * (out->trace[h] - out->quad[h]);
  out->logdet_precond = st->logdetP;
  out->logdet = st->logdetP + st->slq_mean;
  out->iters_run = st->iters_run;
  out->rank = st->rank;
  out->yKinvy = st->dk_out[2 * ((nl > 1 ? c->dp : 1) + 1) + 2];
  out->nlml = 0.5 * (out->yKinvy + out->logdet + (double)c->n * log(2.0 * M_PI));
  if (!isfinite(out->logdet) || !isfinite(out->yKinvy)) return fail(c, BBMM_ENONFINITE, "non-finite result");
  double* dst[3] = {out->alpha, out->beta, out->resid};
  for (int a = 0; a < 3; ++a)
    if (dst[a])
      for (int j = 0; j < c->maxit; ++j)
        for (int q = 0; q < cc; ++q)
          dst[a][(size_t)j * cc + q] = c->h_hist[(size_t)a * BBMM_MAXP * BBMM_MAXC + (size_t)j * BBMM_MAXC + q];
  if (out->pivots)
    for (int m = 0; m < c->k; ++m) out->pivots[m] = (m < st->rank) ? st->piv[m] : -1;
  if (out->slq_terms)
    for (int i = 0; i < c->t; ++i) out->slq_terms[i] = st->slq_terms[i];
  return BBMM_OK;
}

}  // extern "C"
