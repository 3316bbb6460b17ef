// C ABI of lrboost: argument validation and kernel sequencing.  No arithmetic happens here.
//
// Every entry point runs the same sequencing function twice over its lifetime: once "dry" (no
// launches, only workspace carving) to answer *_workspace_bytes(), once for real.  That keeps the
// size query and the actual use of the workspace from drifting apart.
#include <cstring>
#include <mutex>

#include "common.h"

using namespace lrb;

namespace {

inline size_t esize(int dt) { return dt == LR_BF16 ? 2 : 4; }
inline int64_t rup(int64_t v, int64_t m) { return (v + m - 1) / m * m; }

struct Ctx {
  char* base = nullptr;
  size_t cap = 0, off = 0, peak = 0;
  bool dry = false;
  int dt = LR_BF16;
  int gdt = LR_F32;          // dtype of the weight / gamma gradients
  hipStream_t st = nullptr;
  hipError_t err = hipSuccess;

  void* take(size_t bytes) {
    off = (off + 255) & ~(size_t)255;
    void* p = dry ? nullptr : (void*)(base + off);
    off += bytes;
    if (off > peak) peak = off;
    return p;
  }
  size_t mark() const { return off; }
  void release(size_t m) { off = m; }   // stack discipline: drop everything taken since mark()
  void run(hipError_t e) { if (err == hipSuccess && e != hipSuccess) err = e; }
};

#define LAUNCH(c, call) do { if (!(c).dry && (c).err == hipSuccess) (c).run(call); } while (0)

bool aligned16(const void* p) { return ((uintptr_t)p & 15) == 0; }

// A k-contiguous copy of an operand stored k-major: in[k_rows, n_cols] -> out[n_cols, ld = rup(k_rows, 8)].
const void* kmajor_to_kcontig(Ctx& c, const void* in, int64_t ld_in, int64_t k_rows, int64_t n_cols, int64_t& ld_out) {
  ld_out = rup(k_rows, 8);
  void* out = c.take((size_t)n_cols * ld_out * esize(c.dt));
  LAUNCH(c, k_transpose(in, ld_in, out, ld_out, k_rows, n_cols, c.dt, c.st));
  return out;
}

// Runs one GEMM in the context's dtype.  The fp32 kernel takes any orientation; the bf16 MFMA kernel
// wants k contiguous, so k-major operands are first copied through a transpose.
void gemm(Ctx& c, GemmOp op) {
  if (c.dt == LR_F32) {
    LAUNCH(c, gemm_f32(op, c.st));
    return;
  }
  if (gemm_bf16_kmajor_ok(op)) {   // weight gradient: both operands k-major, read in place
    LAUNCH(c, gemm_bf16(op, c.st));
    return;
  }
  const size_t m = c.mark();
  if (op.transA) {
    // only un-batched k-major A operands occur (weight gradients)
    int64_t ld;
    op.A = kmajor_to_kcontig(c, op.A, op.lda, op.K, op.M, ld);
    op.lda = ld;
    op.transA = 0;
  }
  int64_t kpad = op.K;
  if (op.transB) {
    int64_t ld = rup(op.K, 8);
    void* out = c.take((size_t)op.batch * op.N * ld * esize(c.dt));
    for (int b = 0; b < op.batch; b++)
      LAUNCH(c, k_transpose((const char*)op.B + (size_t)b * op.sB * esize(c.dt), op.ldb,
                            (char*)out + (size_t)b * op.N * ld * esize(c.dt), ld, op.K, op.N, c.dt, c.st));
    op.B = out;
    op.ldb = ld;
    op.sB = (int64_t)op.N * ld;
    op.transB = 0;
  }
  op.K = (int)rup(kpad, 8);  // transposed copies are zero-padded to the vector width
  LAUNCH(c, gemm_bf16(op, c.st));
  c.release(m);  // the stream orders later reuse of the transposed copies after this GEMM
}

// dw[Mw, Nw] (+)= colscale * sum_t Aact[t, Mw] * Bact[t, Nw]    (reduction over tokens, split-K)
void wgrad(Ctx& c, const void* Aact, int64_t lda, int Mw, const void* Bact, int64_t ldb, int Nw, int64_t T, void* dw,
           const void* colscale, const void* w_for_dgamma, float* dgamma_part, int accumulate) {
  const size_t m = c.mark();
  GemmOp op;
  op.A = Aact; op.lda = lda; op.transA = 1;
  op.B = Bact; op.ldb = ldb; op.transB = 1;
  op.M = Mw; op.N = Nw; op.K = (int)T;
  op.splitk = gemm_bf16_pick_splitk(Mw, Nw, (int)T, 1);
  float* part = (float*)c.take((size_t)op.splitk * Mw * Nw * sizeof(float));
  op.C = part; op.ldc = Nw;
  op.epi.kind = EPI_PARTIAL;
  gemm(c, op);
  LAUNCH(c, k_wgrad_finish(part, op.splitk, Mw, Nw, dw, colscale, w_for_dgamma, dgamma_part, accumulate, c.dt, c.gdt, c.st));
  c.release(m);
}

int status_of(const Ctx& c) { return c.err == hipSuccess ? LR_OK : LR_ELAUNCH; }

// ---------------------------------------------------------------------------------------------
// one bottleneck layer
// ---------------------------------------------------------------------------------------------
struct LinArgs {
  const void *x, *w_down, *w_up;
  void *z, *y;
  const void *zc, *dy;
  void *dx, *dw_down, *dw_up;
  int64_t ldx, ldy, lddy, lddx, T, d_in, r, d_out;
  int act, accumulate;
};

void linear_fwd_seq(Ctx& c, const LinArgs& a) {
  const size_t es = esize(c.dt);
  void* act = c.take((size_t)a.T * a.r * es);
  GemmOp dn;
  dn.A = a.x; dn.lda = a.ldx; dn.B = a.w_down; dn.ldb = a.d_in; dn.C = a.z; dn.ldc = a.r;
  dn.M = (int)a.T; dn.N = (int)a.r; dn.K = (int)a.d_in;
  dn.epi.kind = EPI_DOWN; dn.epi.act = a.act; dn.epi.C2 = act; dn.epi.ldc2 = a.r;
  gemm(c, dn);
  GemmOp up;
  up.A = act; up.lda = a.r; up.B = a.w_up; up.ldb = a.r; up.C = a.y; up.ldc = a.ldy;
  up.M = (int)a.T; up.N = (int)a.d_out; up.K = (int)a.r;
  up.epi.kind = EPI_STORE;
  gemm(c, up);
}

void linear_bwd_seq(Ctx& c, const LinArgs& a) {
  const size_t es = esize(c.dt);
  void* act = c.take((size_t)a.T * a.r * es);
  void* dz = c.take((size_t)a.T * a.r * es);
  LAUNCH(c, k_act_fwd(a.zc, a.r, act, a.r, a.T, a.r, a.act, c.dt, c.st));
  // dW_up = dy^T . sigma(z)
  wgrad(c, a.dy, a.lddy, (int)a.d_out, act, a.r, (int)a.r, a.T, a.dw_up, nullptr, nullptr, nullptr, a.accumulate);
  // dz = (dy . W_up) * sigma'(z)
  GemmOp da;
  da.A = a.dy; da.lda = a.lddy; da.B = a.w_up; da.ldb = a.r; da.transB = 1; da.C = dz; da.ldc = a.r;
  da.M = (int)a.T; da.N = (int)a.r; da.K = (int)a.d_out;
  da.epi.kind = EPI_ACTGRAD; da.epi.act = a.act; da.epi.R = a.zc; da.epi.ldr = a.r;
  gemm(c, da);
  // dW_down = dz^T . x
  wgrad(c, dz, a.r, (int)a.r, a.x, a.ldx, (int)a.d_in, a.T, a.dw_down, nullptr, nullptr, nullptr, a.accumulate);
  // dx = dz . W_down
  GemmOp dx;
  dx.A = dz; dx.lda = a.r; dx.B = a.w_down; dx.ldb = a.d_in; dx.transB = 1; dx.C = a.dx; dx.ldc = a.lddx;
  dx.M = (int)a.T; dx.N = (int)a.d_in; dx.K = (int)a.r;
  dx.epi.kind = EPI_STORE;
  gemm(c, dx);
}

// ---------------------------------------------------------------------------------------------
// G projections sharing one input, optional RMSNorm folded into the down-projection
// ---------------------------------------------------------------------------------------------
struct GrpArgs {
  const void *x, *gamma, *w_down_cat, *w_up_stack;
  void* z_cat; float* stat; void* y_stack;
  const void *zc, *dy_stack; const float* statc;
  void *dx, *dgamma, *dw_down_cat, *dw_up_stack;
  const void* dres;          // optional residual gradient added into dx (block use)
  int64_t lddres;
  const float* dres32;       // the same residual gradient as an fp32 [T, d_in] tensor (takes precedence)
  float* dx32;               // optional: dx also un-rounded, fp32 [T, d_in] (the residual of a later sum)
  void* act_out;             // optional: where sigma(z_cat) goes (else workspace)
  // LaX variant (identity gate): h_prev [T, G*r] is added to z_cat before the up-projections; in the
  // backward dz_next [T, G*r] is the layer above's gradient w.r.t. z_cat and dh_prev [T, G*r] receives
  // the gradient w.r.t. h_prev.  `lax` selects the variant; each pointer may still be null (= zeros / unused).
  int lax;
  const void *h_prev, *dz_next;
  void* dh_prev;
  int stat_ready;            // stat[] already holds sum_j x^2 (gathered by the GEMM that produced x)
  // d_out_tail > 0: member 0 is d_out wide and members 1..G-1 are d_out_tail wide (a block with fewer
  // key / value heads than query heads); w_up_stack, y_stack, dy_stack and dw_up_stack are then packed:
  // member 0 ([d_out, r] / [T, d_out]) followed by the others ([d_out_tail, r] / [T, d_out_tail]).
  int64_t d_out_tail;
  int64_t ldx, ldy, y_bs, lddy, dy_bs, lddx, T, d_in, r, d_out;
  int G, act, norm, accumulate;
  float eps;
};

// Members of a group that one batched GEMM launch can take: equal width, constant strides.
struct GrpRun {
  int g0, n;                        // first member, number of members
  int64_t d_out, w_off;             // width; element offset of the first member's W_up (and dW_up)
  int64_t y_off, ldy, y_bs;         // element offset, row stride and member stride in y_stack
  int64_t dy_off, lddy, dy_bs;      // the same in dy_stack
};
int group_runs(const GrpArgs& a, GrpRun (&run)[2]) {
  if (a.d_out_tail <= 0 || a.G < 2) {
    run[0] = GrpRun{0, a.G, a.d_out, 0, 0, a.ldy, a.y_bs, 0, a.lddy, a.dy_bs};
    return 1;
  }
  const int64_t w0 = a.d_out * a.r, y0 = a.T * a.d_out, yt = a.T * a.d_out_tail;
  run[0] = GrpRun{0, 1, a.d_out, 0, 0, a.d_out, y0, 0, a.d_out, y0};
  run[1] = GrpRun{1, a.G - 1, a.d_out_tail, w0, y0, a.d_out_tail, yt, y0, a.d_out_tail, yt};
  return 2;
}

// z_cat = RMSNorm(x) . w_down_cat^T (+ sigma(z_cat) into `act`)
void group_down_seq(Ctx& c, const GrpArgs& a, void* act) {
  const size_t es = esize(c.dt);
  const int64_t GR = (int64_t)a.G * a.r;
  GemmOp dn;
  dn.A = a.x; dn.lda = a.ldx; dn.B = a.w_down_cat; dn.ldb = a.d_in; dn.C = a.z_cat; dn.ldc = GR;
  dn.M = (int)a.T; dn.N = (int)GR; dn.K = (int)a.d_in;
  dn.epi.kind = EPI_DOWN; dn.epi.act = a.act; dn.epi.C2 = act; dn.epi.ldc2 = GR;
  if (a.lax) { dn.epi.kind = EPI_DOWN_LAX; dn.epi.R = a.h_prev; dn.epi.ldr = GR; }
  if (a.norm == LR_NORM_ONLINE || a.norm == LR_NORM_ONLINE_GATHER) {
    void* wg = c.take((size_t)GR * a.d_in * es);   // w_down_cat with gamma folded into its columns
    LAUNCH(c, k_scale_cols(a.w_down_cat, a.gamma, wg, GR, a.d_in, c.dt, c.st));
    dn.B = wg;
    dn.epi.use_rho = 1; dn.epi.inv_d = 1.f / (float)a.d_in; dn.epi.eps = a.eps;
    if (a.stat_ready) {
      dn.epi.rowa = a.stat;
    } else if (c.dt == LR_BF16 && (GR <= 512 || a.norm == LR_NORM_ONLINE_GATHER)) {
      // sum of squares gathered from the A tiles inside the GEMM.  Every column tile of a row panel
      // repeats the gather, so this pays only while the output is one or two tiles wide; beyond that a
      // separate pass over x (Alg. 1 line 1 as its own step) is faster (0.80 against 0.89 ms for the
      // Q/K/V group of the 7B shape), and LR_NORM_ONLINE takes it.  LR_NORM_ONLINE_GATHER asks for the
      // gather at any width.
      dn.epi.stat_from_a = 1; dn.epi.stat_out = a.stat;
    } else {
      LAUNCH(c, k_rms_stat(a.x, a.ldx, a.stat, a.T, a.d_in, c.dt, c.st));
      dn.epi.rowa = a.stat;
    }
  } else if (a.norm == LR_NORM_TWO_PASS) {
    void* xh = c.take((size_t)a.T * a.d_in * es);
    if (!a.stat_ready) LAUNCH(c, k_rms_stat(a.x, a.ldx, a.stat, a.T, a.d_in, c.dt, c.st));
    LAUNCH(c, k_rmsnorm_apply(a.x, a.ldx, a.gamma, a.stat, a.eps, xh, a.d_in, a.T, a.d_in, c.dt, c.st));
    dn.A = xh; dn.lda = a.d_in;
  } else if (a.norm == LR_NORM_SHARD_LOCAL) {
    // One rank's part of the feature-sharded form (Sec. 4.2, Alg. 1, the steps before the exchange): x is a
    // [T, d_in] slice of the full input.  Local statistic, normalisation by the LOCAL rms (rounded to the
    // storage type, as a rank would feed it to its GEMM), product with the rank's weight rows, and the local
    // scale undone per row in the epilogue: z_cat receives the un-normalised partial product that the ranks
    // add up, stat the local sum of squares that travels with it.  No activation, no up-projection: both
    // come after the exchange and the global rescale.
    void* xh = c.take((size_t)a.T * a.d_in * es);
    LAUNCH(c, k_rms_stat(a.x, a.ldx, a.stat, a.T, a.d_in, c.dt, c.st));
    LAUNCH(c, k_rmsnorm_apply(a.x, a.ldx, a.gamma, a.stat, a.eps, xh, a.d_in, a.T, a.d_in, c.dt, c.st));
    dn.A = xh; dn.lda = a.d_in;
    dn.epi.kind = EPI_DOWN; dn.epi.C2 = nullptr; dn.epi.R = nullptr;
    dn.epi.use_rho = 1; dn.epi.rho_sqrt = 1; dn.epi.rowa = a.stat; dn.epi.inv_d = 1.f / (float)a.d_in; dn.epi.eps = a.eps;
  }
  gemm(c, dn);
}

void group_up_seq(Ctx& c, const GrpArgs& a, const void* act) {
  const size_t es = esize(c.dt);
  const int64_t GR = (int64_t)a.G * a.r;
  GrpRun run[2];
  const int nrun = group_runs(a, run);
  for (int i = 0; i < nrun; i++) {
    const GrpRun& u = run[i];
    GemmOp up;
    up.A = (const char*)act + (size_t)u.g0 * a.r * es; up.lda = GR; up.sA = a.r;
    up.B = (const char*)a.w_up_stack + (size_t)u.w_off * es; up.ldb = a.r; up.sB = u.d_out * a.r;
    up.C = (char*)a.y_stack + (size_t)u.y_off * es; up.ldc = u.ldy; up.sC = u.y_bs;
    up.M = (int)a.T; up.N = (int)u.d_out; up.K = (int)a.r; up.batch = u.n;
    up.epi.kind = EPI_STORE;
    gemm(c, up);
  }
}

void group_fwd_seq(Ctx& c, const GrpArgs& a) {
  const size_t es = esize(c.dt);
  void* act = a.act_out ? a.act_out : c.take((size_t)a.T * a.G * a.r * es);
  group_down_seq(c, a, act);
  if (a.norm != LR_NORM_SHARD_LOCAL) group_up_seq(c, a, act);
}

// Backward of the group.  `act` = sigma(z_cat) must already be in place.
void group_bwd_seq(Ctx& c, const GrpArgs& a, const void* act) {
  const size_t es = esize(c.dt);
  const int64_t GR = (int64_t)a.G * a.r;
  const bool normed = a.norm != LR_NORM_NONE;
  GrpRun run[2];
  const int nrun = group_runs(a, run);
  // dW_up[g] = dy_g^T . sigma(z_g)
  for (int i = 0; i < nrun; i++)
    for (int j = 0; j < run[i].n; j++) {
      const GrpRun& u = run[i];
      wgrad(c, (const char*)a.dy_stack + (size_t)(u.dy_off + j * u.dy_bs) * es, u.lddy, (int)u.d_out,
            (const char*)act + (size_t)(u.g0 + j) * a.r * es, GR, (int)a.r, a.T,
            (char*)a.dw_up_stack + (size_t)(u.w_off + j * u.d_out * a.r) * esize(c.gdt), nullptr, nullptr, nullptr,
            a.accumulate);
    }
  // dp_g = rho * (dy_g . W_up_g) * sigma'(z_g), batched over g, written into the columns of dp_cat;
  // cdot[t] = sum_n dp[t,n] z[t,n] is the RMSNorm-backward statistic, taken at rank r.
  void* dp = c.take((size_t)a.T * GR * es);
  float* cdot = normed ? (float*)c.take((size_t)a.T * sizeof(float)) : nullptr;
  // one launch per run of equally wide members (one launch in all unless the key / value members are narrower)
  const int slabs1 = (normed && c.dt == LR_BF16) ? gemm_bf16_rowpart_slabs((int)a.r) : 0;   // row-partial columns per member
  float* parts = slabs1 ? (float*)c.take((size_t)a.T * slabs1 * a.G * sizeof(float)) : nullptr;
  auto at = [&](const void* p, int g0) -> const void* { return p ? (const char*)p + (size_t)g0 * a.r * es : nullptr; };
  for (int i = 0; i < nrun; i++) {
    const GrpRun& u = run[i];
    GemmOp da;
    da.A = (const char*)a.dy_stack + (size_t)u.dy_off * es; da.lda = u.lddy; da.sA = u.dy_bs;
    da.B = (const char*)a.w_up_stack + (size_t)u.w_off * es; da.ldb = a.r; da.sB = u.d_out * a.r; da.transB = 1;
    da.C = (char*)dp + (size_t)u.g0 * a.r * es; da.ldc = GR; da.sC = a.r;
    da.M = (int)a.T; da.N = (int)a.r; da.K = (int)u.d_out; da.batch = u.n;
    da.epi.kind = EPI_ACTGRAD; da.epi.act = a.act; da.epi.R = at(a.zc, u.g0); da.epi.ldr = GR; da.epi.sR = a.r;
    if (a.lax) {
      da.epi.kind = EPI_LAXGRAD;
      da.epi.R2 = at(a.dz_next, u.g0); da.epi.ldr2 = GR; da.epi.sR2 = a.r;
      da.epi.C2 = (void*)at(a.dh_prev, u.g0); da.epi.ldc2 = GR; da.epi.sC2 = a.r;
    }
    if (normed) {
      da.epi.use_rho = 1; da.epi.rowa = a.statc; da.epi.inv_d = 1.f / (float)a.d_in; da.epi.eps = a.eps;
    }
    if (parts) {
      da.epi.rowpart = parts; da.epi.rowpart_ld = slabs1 * a.G; da.epi.rowpart_off = u.g0 * slabs1;
    }
    gemm(c, da);
  }
  if (parts) {
    LAUNCH(c, k_rowsum_parts(parts, slabs1 * a.G, slabs1 * a.G, cdot, a.T, c.st));
  } else if (normed) {
    LAUNCH(c, k_rowdot(dp, GR, a.zc, GR, cdot, a.T, GR, c.dt, c.st));
  }
  // dW_down_cat: with the norm folded in, the GEMM yields the gradient of (w * gamma); the finishing
  // pass scales it by gamma and also produces dgamma[k] = sum_n w[n,k] * dW'[n,k].
  const void* wB = a.w_down_cat;
  if (normed) {
    const int64_t nparts = k_wgrad_dgamma_parts(GR);
    float* dgp = (float*)c.take((size_t)nparts * a.d_in * sizeof(float));
    wgrad(c, dp, GR, (int)GR, a.x, a.ldx, (int)a.d_in, a.T, a.dw_down_cat, a.gamma, a.w_down_cat, dgp, a.accumulate);
    LAUNCH(c, k_colsum_parts(dgp, nparts, a.d_in, a.dgamma, a.accumulate, c.gdt, c.st));
    void* wg = c.take((size_t)GR * a.d_in * es);
    LAUNCH(c, k_scale_cols(a.w_down_cat, a.gamma, wg, GR, a.d_in, c.dt, c.st));
    wB = wg;
  } else {
    wgrad(c, dp, GR, (int)GR, a.x, a.ldx, (int)a.d_in, a.T, a.dw_down_cat, nullptr, nullptr, nullptr, a.accumulate);
  }
  // dx = dp_cat . (w*gamma)  - (rho/d) * cdot * x  (+ residual gradient)
  GemmOp dx;
  dx.A = dp; dx.lda = GR; dx.B = wB; dx.ldb = a.d_in; dx.transB = 1; dx.C = a.dx; dx.ldc = a.lddx;
  dx.M = (int)a.T; dx.N = (int)a.d_in; dx.K = (int)GR;
  if (normed) {
    dx.epi.kind = EPI_NORMBWD; dx.epi.use_rho = 1; dx.epi.rowa = a.statc; dx.epi.rowb = cdot;
    dx.epi.inv_d = 1.f / (float)a.d_in; dx.epi.eps = a.eps;
    dx.epi.R2 = a.x; dx.epi.ldr2 = a.ldx;
    dx.epi.R = a.dres; dx.epi.ldr = a.lddres;
    if (c.dt == LR_BF16 && a.dres32) {
      dx.epi.kind = EPI_NORMBWD_I32; dx.epi.R = a.dres32; dx.epi.ldr = a.d_in;
    } else if (c.dt == LR_BF16 && a.dx32) {
      dx.epi.kind = EPI_NORMBWD_O32; dx.epi.C32 = a.dx32; dx.epi.ldc32 = a.d_in;
    }
  } else if (a.dres) {
    dx.epi.kind = EPI_UP; dx.epi.R = a.dres; dx.epi.ldr = a.lddres;
  } else {
    dx.epi.kind = EPI_STORE;
  }
  gemm(c, dx);
}

void group_bwd_full_seq(Ctx& c, const GrpArgs& a) {
  const size_t es = esize(c.dt);
  const int64_t GR = (int64_t)a.G * a.r;
  void* act = c.take((size_t)a.T * GR * es);
  LAUNCH(c, k_act_fwd(a.zc, GR, act, GR, a.T, GR, a.act, c.dt, c.st));
  group_bwd_seq(c, a, act);
}

// ---- validation helpers -------------------------------------------------------------------------
int check_dt(int dt) { return (dt == LR_F32 || dt == LR_BF16) ? LR_OK : LR_EINVAL; }
int check_gdt(int dt, int gdt) {
  if (gdt != LR_F32 && gdt != LR_BF16) return LR_EINVAL;
  return (gdt == LR_BF16 && dt != LR_BF16) ? LR_EINVAL : LR_OK;
}
int check_gptrs(int gdt, std::initializer_list<const void*> ps);
int check_act(int act) { return (act == LR_ACT_IDENTITY || act == LR_ACT_SILU) ? LR_OK : LR_EINVAL; }
int check_dims_bf16(int dt, std::initializer_list<int64_t> dims) {
  if (dt != LR_BF16) return LR_OK;
  for (int64_t v : dims) if (v % 8 != 0) return LR_EALIGN;
  return LR_OK;
}
int check_ptrs(int dt, std::initializer_list<const void*> ps) {
  for (const void* p : ps) {
    if (!p) return LR_EINVAL;
    if (dt == LR_BF16 ? !aligned16(p) : ((uintptr_t)p & 3) != 0) return LR_EALIGN;
  }
  return LR_OK;
}
int check_gptrs(int gdt, std::initializer_list<const void*> ps) { return check_ptrs(gdt == LR_F32 ? LR_BF16 : gdt, ps); }
#define TRY(expr) do { int _s = (expr); if (_s != LR_OK) return _s; } while (0)

int check_ws(const void* ws, size_t have, size_t need) {
  if (need == 0) return LR_OK;
  if (!ws || have < need) return LR_EWORKSPACE;
  if (((uintptr_t)ws & 255) != 0) return LR_EALIGN;
  return LR_OK;
}

int check_sizes_fit_int(std::initializer_list<int64_t> v) {
  for (int64_t x : v) if (x <= 0 || x > 0x7fffffffLL) return LR_EINVAL;
  return LR_OK;
}


// ---------------------------------------------------------------------------------------------
// the decoder block
// ---------------------------------------------------------------------------------------------
struct Blk {
  int64_t B, S, T, d, H, hd, f, r;
  int64_t Hkv, dkv;                   // key / value heads and their total width (= H, d: multi-head)
  float eps;
  int act, norm, causal, gdt;
  const float *rope_cos, *rope_sin;   // both null: no rotary embedding
  int stat_x_ready;                   // ckpt->s1 arrives filled (by the block below)
  float* stat_y_out;                  // optional: sum of squares of y for the block above
};

bool block_desc_ok(const lr_block_desc* ds, Blk& b, int* why) {
  *why = LR_EINVAL;
  if (!ds) return false;
  if (ds->batch <= 0 || ds->seq <= 0 || ds->d_model <= 0 || ds->n_heads <= 0 || ds->head_dim <= 0 || ds->ffn <= 0 ||
      ds->rank <= 0 || ds->ffn_ld < ds->ffn)
    return false;
  if (ds->n_heads * ds->head_dim != ds->d_model) return false;
  if (check_act(ds->act) != LR_OK) return false;
  if (ds->norm != LR_NORM_ONLINE && ds->norm != LR_NORM_TWO_PASS && ds->norm != LR_NORM_ONLINE_GATHER) return false;
  if (ds->grad_dt != LR_F32 && ds->grad_dt != LR_BF16) return false;
  if (ds->batch * ds->seq > 0x7fffffffLL || ds->ffn_ld > 0x7fffffffLL || 3 * ds->rank > 0x7fffffffLL) return false;
  *why = LR_EUNSUPPORTED;
  if (ds->dt != LR_BF16 || ds->head_dim != 128 || ds->causal != 1) return false;
  if (ds->seq * ds->d_model * 2 >= 0x7fffffffLL) return false;   // attention: 32-bit byte offsets per batch element
  *why = LR_EALIGN;
  if (ds->d_model % 8 || ds->ffn_ld % 8 || ds->rank % 8) return false;
  b.B = ds->batch; b.S = ds->seq; b.T = ds->batch * ds->seq; b.d = ds->d_model; b.H = ds->n_heads; b.hd = ds->head_dim;
  b.f = ds->ffn_ld; b.r = ds->rank; b.eps = ds->eps; b.act = ds->act; b.norm = ds->norm; b.causal = ds->causal;
  b.gdt = ds->grad_dt;
  b.Hkv = ds->n_kv_heads > 0 ? ds->n_kv_heads : ds->n_heads;
  if (b.Hkv > b.H || b.H % b.Hkv != 0) { *why = LR_EINVAL; return false; }
  b.dkv = b.Hkv * b.hd;
  b.rope_cos = ds->rope_cos; b.rope_sin = ds->rope_sin;
  b.stat_x_ready = ds->stat_x_ready != 0; b.stat_y_out = ds->stat_y_out;
  if (b.stat_y_out && ((uintptr_t)b.stat_y_out & 3)) { *why = LR_EALIGN; return false; }
  if ((b.rope_cos == nullptr) != (b.rope_sin == nullptr)) { *why = LR_EINVAL; return false; }
  if (b.rope_cos && (((uintptr_t)b.rope_cos & 15) || ((uintptr_t)b.rope_sin & 15))) { *why = LR_EALIGN; return false; }
  *why = LR_OK;
  return true;
}

// FLOPs of one S x S x hd product over all (batch, head) pairs, causal half counted
double attn_unit_flops(const Blk& b) { return 2.0 * (double)b.B * b.H * (double)b.S * b.S * b.hd / 2.0; }

// z = in . w_dn^T (no norm), act = sigma(z)
// (LaX: act = z + h_prev, identity gate)
void single_down(Ctx& c, const Blk& b, const void* in, int64_t K, const void* w_dn, void* z, void* act, int lax = 0,
                 const void* h_prev = nullptr) {
  GemmOp dn;
  dn.A = in; dn.lda = K; dn.B = w_dn; dn.ldb = K; dn.C = z; dn.ldc = b.r;
  dn.M = (int)b.T; dn.N = (int)b.r; dn.K = (int)K;
  dn.epi.kind = EPI_DOWN; dn.epi.act = b.act; dn.epi.C2 = act; dn.epi.ldc2 = b.r;
  if (lax) { dn.epi.kind = EPI_DOWN_LAX; dn.epi.R = h_prev; dn.epi.ldr = b.r; }
  gemm(c, dn);
}

// out = act . w_up^T + resid ; optionally the per-row sum of squares of out into `sumsq`.
// The residual stream stays un-rounded between the two sums of a block: out32 (optional) receives the
// sum as fp32 beside the bf16 `out`, resid32 (optional, instead of resid) is such a tensor taken back.
void single_up(Ctx& c, const Blk& b, const void* act, const void* w_up, int64_t N, const void* resid, void* out,
               float* sumsq, float* out32 = nullptr, const float* resid32 = nullptr) {
  const size_t m = c.mark();
  GemmOp up;
  up.A = act; up.lda = b.r; up.B = w_up; up.ldb = b.r; up.C = out; up.ldc = N;
  up.M = (int)b.T; up.N = (int)N; up.K = (int)b.r;
  up.epi.kind = EPI_UP; up.epi.R = resid; up.epi.ldr = N;
  if (resid32) { up.epi.kind = EPI_UP_I32; up.epi.R = resid32; }
  else if (out32) { up.epi.kind = EPI_UP_O32; up.epi.C32 = out32; up.epi.ldc32 = N; }
  if (sumsq) {
    const int slabs = gemm_bf16_rowpart_slabs((int)N);
    float* parts = (float*)c.take((size_t)b.T * slabs * sizeof(float));
    up.epi.rowpart = parts; up.epi.rowpart_ld = slabs;
    gemm(c, up);
    LAUNCH(c, k_rowsum_parts(parts, slabs, slabs, sumsq, b.T, c.st));
  } else {
    gemm(c, up);
  }
  c.release(m);
}

// Backward through an un-grouped up-projection: dw_up (+)= dout^T . act ; dz = (dout . w_up) * sigma'(z)
// (LaX: dz = dout . w_up + dz_next, and dh_prev = dout . w_up)
void single_up_bwd(Ctx& c, const Blk& b, const void* dout, int64_t N, const void* act, const void* z, const void* w_up,
                   void* dw_up, void* dz, int accumulate, int lax = 0, const void* dz_next = nullptr,
                   void* dh_prev = nullptr) {
  wgrad(c, dout, N, (int)N, act, b.r, (int)b.r, b.T, dw_up, nullptr, nullptr, nullptr, accumulate);
  GemmOp da;
  da.A = dout; da.lda = N; da.B = w_up; da.ldb = b.r; da.transB = 1; da.C = dz; da.ldc = b.r;
  da.M = (int)b.T; da.N = (int)b.r; da.K = (int)N;
  da.epi.kind = EPI_ACTGRAD; da.epi.act = b.act; da.epi.R = z; da.epi.ldr = b.r;
  if (lax) {
    da.epi.kind = EPI_LAXGRAD; da.epi.R = nullptr;   // no row statistic wanted here
    da.epi.R2 = dz_next; da.epi.ldr2 = b.r; da.epi.C2 = dh_prev; da.epi.ldc2 = b.r;
  }
  gemm(c, da);
}

// The gate / up pair of the MLP: g = act_g . W_up_g^T, then u = act_u . W_up_u^T whose epilogue forms
// m = SiLU(g) * u from its fp32 accumulators and the g tile just written (the SwiGLU gate never
// runs as a pass of its own).  u itself is stored only where a buffer is given: the forward has no use
// for it, the backward's re-forward does.
void mlp_up_swiglu(Ctx& c, const Blk& b, const void* w_up_gu, const void* act, void* g, void* u, void* m) {
  const size_t es = 2;
  GemmOp up;
  up.A = act; up.lda = 2 * b.r; up.B = w_up_gu; up.ldb = b.r; up.C = g; up.ldc = b.f;
  up.M = (int)b.T; up.N = (int)b.f; up.K = (int)b.r;
  up.epi.kind = EPI_STORE;
  gemm(c, up);
  up.A = (const char*)act + (size_t)b.r * es;
  up.B = (const char*)w_up_gu + (size_t)b.f * b.r * es;
  up.C = u;
  up.epi.kind = EPI_SWIGLU_FWD; up.epi.R = g; up.epi.ldr = b.f; up.epi.C2 = m; up.epi.ldc2 = b.f;
  gemm(c, up);
}

// the Q/K/V group of a block: K and V may be narrower than Q (fewer key / value heads)
GrpArgs group_args(const Blk& b, int G, int64_t d_out);
GrpArgs qkv_group_args(const Blk& b) {
  GrpArgs g = group_args(b, 3, b.d);
  if (b.dkv != b.d) g.d_out_tail = b.dkv;
  return g;
}
// q and k of a stack laid out as q [T, d], k [T, dkv], v [T, dkv]: rotary embedding (or its transpose)
void rope_qk(Ctx& c, const Blk& b, void* qkv, int inverse);

GrpArgs group_args(const Blk& b, int G, int64_t d_out) {
  GrpArgs g{};
  g.G = G; g.T = b.T; g.d_in = b.d; g.r = b.r; g.d_out = d_out; g.act = b.act; g.norm = b.norm; g.eps = b.eps;
  g.ldx = b.d; g.ldy = d_out; g.y_bs = b.T * d_out; g.lddy = d_out; g.dy_bs = b.T * d_out; g.lddx = b.d;
  g.lddres = b.d;
  return g;
}

// rank-r activation of a layer for the backward: sigma(z), or z + h_prev in the LaX variant
void rebuild_act(Ctx& c, const Blk& b, const void* z, const void* h_prev, void* act, int64_t n, int lax) {
  if (lax && h_prev) LAUNCH(c, k_add2_bf16(z, h_prev, act, b.T, n, c.st));
  else LAUNCH(c, k_act_fwd(z, n, act, n, b.T, n, lax ? (int)LR_ACT_IDENTITY : b.act, LR_BF16, c.st));
}

void rope_qk(Ctx& c, const Blk& b, void* qkv, int inverse) {
  if (b.dkv == b.d) {   // q and k are two [T, d] tensors back to back: one pass over both
    LAUNCH(c, k_rope128_bf16(qkv, b.d, b.rope_cos, b.rope_sin, 2 * b.T, (int)b.S, (int)b.H, inverse, c.st));
    return;
  }
  LAUNCH(c, k_rope128_bf16(qkv, b.d, b.rope_cos, b.rope_sin, b.T, (int)b.S, (int)b.H, inverse, c.st));
  LAUNCH(c, k_rope128_bf16((char*)qkv + (size_t)b.T * b.d * 2, b.dkv, b.rope_cos, b.rope_sin, b.T, (int)b.S, (int)b.Hkv,
                           inverse, c.st));
}

// sv: optional; the wide activations then land in the caller's buffers (to be kept for a backward that
// does not re-forward) instead of the workspace
void block_fwd_seq(Ctx& c, const Blk& b, const lr_block_params* p, const void* x, void* y, const lr_block_ckpt* ck,
                   const lr_block_lax* lx = nullptr, const lr_block_saved* sv = nullptr) {
  const int lax = lx != nullptr;
  const size_t es = 2;
  const int64_t T = b.T, d = b.d, r = b.r, f = b.f;
  const int64_t dkv = b.dkv;
  void* qkv = sv ? sv->qkv : c.take((size_t)T * (d + 2 * dkv) * es);     // q [T, d], k [T, dkv], v [T, dkv]
  void* o = sv ? sv->o : c.take((size_t)T * d * es);
  void* h1 = sv ? sv->h1 : c.take((size_t)T * d * es);
  float* h1f = (float*)c.take((size_t)T * d * sizeof(float));   // h1 before rounding: the residual of y
  float* lse = sv ? sv->lse : (float*)c.take((size_t)b.B * b.H * b.S * sizeof(float));
  void* act = c.take((size_t)T * 3 * r * es);     // sigma(z) of whichever projection group is live
  void* gg = sv ? sv->gu : c.take((size_t)T * f * es);
  void* uu = sv ? (void*)((char*)sv->gu + (size_t)T * f * es) : nullptr;   // u itself is kept only when saving
  void* mm = sv ? sv->m : c.take((size_t)T * f * es);
  // attention side
  GrpArgs a = qkv_group_args(b);
  a.x = x; a.gamma = p->gamma1; a.w_down_cat = p->w_dn_qkv; a.w_up_stack = p->w_up_qkv;
  a.z_cat = ck ? ck->z_qkv : nullptr; a.stat = ck ? ck->s1 : nullptr; a.y_stack = qkv; a.act_out = act;
  a.stat_ready = b.stat_x_ready;
  a.lax = lax; a.h_prev = lax ? lx->h_prev_qkv : nullptr;
  group_fwd_seq(c, a);
  if (b.rope_cos) rope_qk(c, b, qkv, 0);
  {
    const int slot = c.dry ? -1 : launch_timer_open(LR_TAG_ATTN_FWD, (int)T, (int)d, (int)b.S, 1, attn_unit_flops(b) * 2.0, c.st);
    LAUNCH(c, attention_gqa_fwd_bf16(qkv, (char*)qkv + (size_t)T * d * es, (char*)qkv + (size_t)T * (d + dkv) * es, o, lse,
                                     d, dkv, (int)b.B, (int)b.S, (int)b.H, (int)b.Hkv, (int)b.hd, b.causal, c.st));
    launch_timer_close(slot, c.st);
  }
  single_down(c, b, o, d, p->w_dn_o, ck ? ck->z_o : nullptr, act, lax, lax ? lx->h_prev_o : nullptr);
  single_up(c, b, act, p->w_up_o, d, x, h1, ck ? ck->s2 : nullptr, h1f);   // h1 = x + ..., s2 = sum h1^2 from the epilogue
  // MLP side
  GrpArgs m = group_args(b, 2, f);
  m.x = h1; m.gamma = p->gamma2; m.w_down_cat = p->w_dn_gu; m.w_up_stack = p->w_up_gu;
  m.z_cat = ck ? ck->z_gu : nullptr; m.stat = ck ? ck->s2 : nullptr; m.stat_ready = 1; m.act_out = act;
  m.lax = lax; m.h_prev = lax ? lx->h_prev_gu : nullptr;
  group_down_seq(c, m, act);
  mlp_up_swiglu(c, b, p->w_up_gu, act, gg, uu, mm);
  single_down(c, b, mm, f, p->w_dn_d, ck ? ck->z_d : nullptr, act, lax, lax ? lx->h_prev_d : nullptr);
  single_up(c, b, act, p->w_up_d, d, nullptr, y, b.stat_y_out, nullptr, h1f);   // optionally sum y^2 for the block above
}

// sv: optional; the forward's wide activations as kept by the caller (read only): the re-forward of h1,
// g, u, m, q, k, v, o and lse from the rank-r checkpoints is then skipped
void block_bwd_seq(Ctx& c, const Blk& b, const lr_block_params* p, const void* x, const void* dy,
                   const lr_block_ckpt* ck, void* dx, const lr_block_params* g, int accumulate,
                   const lr_block_lax* lx = nullptr, const lr_block_saved* sv = nullptr) {
  const int lax = lx != nullptr;
  const lr_block_lax nlx{};
  if (!lx) lx = &nlx;
  const size_t es = 2;
  const int64_t T = b.T, d = b.d, r = b.r, f = b.f;
  const lr_block_params np{};  // dry runs have no parameter structs
  const lr_block_ckpt nck{};
  if (!p) p = &np;
  if (!g) g = &np;
  if (!ck) ck = &nck;
  void* act_d = c.take((size_t)T * r * es);
  void* act_o = c.take((size_t)T * r * es);
  void* act_g = c.take((size_t)T * 3 * r * es);   // sigma(z_gu), later sigma(z_qkv)
  void* dz1 = c.take((size_t)T * r * es);         // dz_d, later dz_o
  void* h1 = sv ? sv->h1 : c.take((size_t)T * d * es);
  void* dh1 = c.take((size_t)T * d * es);
  float* dh1f = (float*)c.take((size_t)T * d * sizeof(float));   // dh1 before rounding: the residual of dx
  void* big = sv ? sv->gu : c.take((size_t)2 * T * f * es);     // g,u  (later q,k,v: needs 3*T*d <= 2*T*f checked below)
  void* big2 = c.take((size_t)2 * T * f * es);    // dg,du (later dq,dk,dv)
  void* mm = sv ? sv->m : c.take((size_t)T * f * es);          // m, later o and do
  float* lse = sv ? sv->lse : (float*)c.take((size_t)b.B * b.H * b.S * sizeof(float));
  const int64_t dkv = b.dkv;
  void* qkv = big;
  void* dqkv = big2;
  if (sv) qkv = sv->qkv;
  if (d + 2 * dkv > 2 * f) {  // unusual shapes: separate buffers
    if (!sv) qkv = c.take((size_t)T * (d + 2 * dkv) * es);
    dqkv = c.take((size_t)T * (d + 2 * dkv) * es);
  }
  void* o = mm;
  void* dout = nullptr;
  if (sv) {                   // the kept tensors are read only: dO gets a buffer of its own
    o = sv->o;
    dout = c.take((size_t)T * d * es);
  } else if (2 * d > f) {
    o = c.take((size_t)T * d * es);
    dout = c.take((size_t)T * d * es);
  } else {
    dout = (char*)mm + (size_t)T * d * es;
  }

  // ---- MLP side ----
  rebuild_act(c, b, ck->z_d, lx->h_prev_d, act_d, r, lax);
  single_up_bwd(c, b, dy, d, act_d, ck->z_d, p->w_up_d, g->w_up_d, dz1, accumulate, lax, lx->dz_next_d, lx->dh_prev_d);
  // re-forward from the rank-r checkpoints: h1, then g, u, m
  rebuild_act(c, b, ck->z_o, lx->h_prev_o, act_o, r, lax);
  if (!sv) single_up(c, b, act_o, p->w_up_o, d, x, h1, nullptr);
  rebuild_act(c, b, ck->z_gu, lx->h_prev_gu, act_g, 2 * r, lax);
  GrpArgs m = group_args(b, 2, f);
  m.x = h1; m.gamma = p->gamma2; m.w_down_cat = p->w_dn_gu; m.w_up_stack = p->w_up_gu; m.y_stack = big;
  if (!sv) mlp_up_swiglu(c, b, p->w_up_gu, act_g, big, (char*)big + (size_t)T * f * es, mm);
  // down-D backward: dW_dn_d = dz_d^T . m ; dm = dz_d . W_dn_d with the SwiGLU reverse fused in
  wgrad(c, dz1, r, (int)r, mm, f, (int)f, T, g->w_dn_d, nullptr, nullptr, nullptr, accumulate);
  {
    GemmOp dm;
    dm.A = dz1; dm.lda = r; dm.B = p->w_dn_d; dm.ldb = f; dm.transB = 1; dm.C = big2; dm.ldc = f;
    dm.M = (int)T; dm.N = (int)f; dm.K = (int)r;
    dm.epi.kind = EPI_SWIGLU_BWD; dm.epi.R = big; dm.epi.ldr = f; dm.epi.R2 = (char*)big + (size_t)T * f * es;
    dm.epi.ldr2 = f; dm.epi.C2 = (char*)big2 + (size_t)T * f * es; dm.epi.ldc2 = f;
    gemm(c, dm);
  }
  // gate/up group backward; dh1 = dy + RMSNorm-2 reverse
  m.zc = ck->z_gu; m.statc = ck->s2; m.dy_stack = big2; m.dx = dh1; m.dx32 = dh1f; m.dres = dy; m.dgamma = g->gamma2;
  m.dw_down_cat = g->w_dn_gu; m.dw_up_stack = g->w_up_gu; m.accumulate = accumulate;
  m.lax = lax; m.dz_next = lx->dz_next_gu; m.dh_prev = lx->dh_prev_gu;
  group_bwd_seq(c, m, act_g);

  // ---- attention side ----
  single_up_bwd(c, b, dh1, d, act_o, ck->z_o, p->w_up_o, g->w_up_o, dz1, accumulate, lax, lx->dz_next_o, lx->dh_prev_o);
  // re-forward q, k, v, o
  rebuild_act(c, b, ck->z_qkv, lx->h_prev_qkv, act_g, 3 * r, lax);
  GrpArgs a = qkv_group_args(b);
  a.x = x; a.gamma = p->gamma1; a.w_down_cat = p->w_dn_qkv; a.w_up_stack = p->w_up_qkv; a.y_stack = qkv;
  if (!sv) group_up_seq(c, a, act_g);
  if (!sv && b.rope_cos) rope_qk(c, b, qkv, 0);
  const void* q_ = qkv; const void* k_ = (char*)qkv + (size_t)T * d * es; const void* v_ = (char*)qkv + (size_t)T * (d + dkv) * es;
  if (!sv) {
    const int slot = c.dry ? -1 : launch_timer_open(LR_TAG_ATTN_FWD, (int)T, (int)d, (int)b.S, 1, attn_unit_flops(b) * 2.0, c.st);
    LAUNCH(c, attention_gqa_fwd_bf16(q_, k_, v_, o, lse, d, dkv, (int)b.B, (int)b.S, (int)b.H, (int)b.Hkv, (int)b.hd,
                                     b.causal, c.st));
    launch_timer_close(slot, c.st);
  }
  // down-O backward
  wgrad(c, dz1, r, (int)r, o, d, (int)d, T, g->w_dn_o, nullptr, nullptr, nullptr, accumulate);
  {
    GemmOp dO;
    dO.A = dz1; dO.lda = r; dO.B = p->w_dn_o; dO.ldb = d; dO.transB = 1; dO.C = dout; dO.ldc = d;
    dO.M = (int)T; dO.N = (int)d; dO.K = (int)r;
    dO.epi.kind = EPI_STORE;
    gemm(c, dO);
  }
  {
    const size_t mk = c.mark();
    void* aws = c.take(attention_gqa_bwd_ws_bytes((int)b.B, (int)b.S, (int)b.H, (int)b.Hkv, (int)b.hd));
    // five GEMM units (S, dP, dV, dK in one kernel, dQ over the stored score gradient) against the forward's two
    const int slot = c.dry ? -1 : launch_timer_open(LR_TAG_ATTN_BWD, (int)T, (int)d, (int)b.S, 1, attn_unit_flops(b) * 5.0, c.st);
    LAUNCH(c, attention_gqa_bwd_bf16(q_, k_, v_, o, dout, lse, dqkv, (char*)dqkv + (size_t)T * d * es,
                                     (char*)dqkv + (size_t)T * (d + dkv) * es, d, dkv, (int)b.B, (int)b.S, (int)b.H,
                                     (int)b.Hkv, (int)b.hd, b.causal, aws, c.st));
    launch_timer_close(slot, c.st);
    c.release(mk);
  }
  // back through the rotations of q and k: their transposes, on dq and dk
  if (b.rope_cos) rope_qk(c, b, dqkv, 1);
  a.zc = ck->z_qkv; a.statc = ck->s1; a.dy_stack = dqkv; a.dx = dx; a.dres = dh1; a.dres32 = dh1f; a.dgamma = g->gamma1;
  a.dw_down_cat = g->w_dn_qkv; a.dw_up_stack = g->w_up_qkv; a.accumulate = accumulate;
  a.lax = lax; a.dz_next = lx->dz_next_qkv; a.dh_prev = lx->dh_prev_qkv;
  group_bwd_seq(c, a, act_g);
}

}  // namespace

// =============================================================================================
extern "C" {

int lr_version(void) { return 100; }

const char* lr_status_string(int status) {
  switch (status) {
    case LR_OK: return "LR_OK";
    case LR_EINVAL: return "LR_EINVAL: null pointer, non-positive size or unknown enum value";
    case LR_EUNSUPPORTED: return "LR_EUNSUPPORTED: valid request this library cannot run";
    case LR_EWORKSPACE: return "LR_EWORKSPACE: workspace missing or too small";
    case LR_EALIGN: return "LR_EALIGN: pointer, leading dimension or size alignment rule violated";
    case LR_ELAUNCH: return "LR_ELAUNCH: kernel launch rejected by the runtime";
    default: return "unknown lr_status";
  }
}

// ---- linear ---------------------------------------------------------------------------------
size_t lr_linear_workspace_bytes(int64_t T, int64_t d_in, int64_t r, int64_t d_out, int dt, int backward) {
  if (check_dt(dt) != LR_OK || T < 0 || check_sizes_fit_int({d_in, r, d_out}) != LR_OK) return 0;
  if (T == 0) return 0;
  Ctx c; c.dry = true; c.dt = dt;
  LinArgs a{}; a.T = T; a.d_in = d_in; a.r = r; a.d_out = d_out; a.ldx = d_in; a.ldy = d_out; a.lddy = d_out; a.lddx = d_in;
  if (backward) linear_bwd_seq(c, a); else linear_fwd_seq(c, a);
  return c.peak + 256;
}

int lr_linear_fwd(const void* x, int64_t ldx, const void* w_down, const void* w_up, void* z, void* y, int64_t ldy,
                  int64_t T, int64_t d_in, int64_t r, int64_t d_out, int act, int dt, void* ws, size_t ws_bytes,
                  void* stream) {
  TRY(check_dt(dt)); TRY(check_act(act));
  if (T < 0) return LR_EINVAL;
  TRY(check_sizes_fit_int({d_in, r, d_out}));
  if (T > 0x7fffffffLL) return LR_EINVAL;
  if (ldx < d_in || ldy < d_out) return LR_EINVAL;
  TRY(check_dims_bf16(dt, {d_in, r, d_out, ldx, ldy}));
  if (T == 0) return LR_OK;   // no tokens: nothing to do (empty tensors may have null pointers)
  TRY(check_ptrs(dt, {x, w_down, w_up, z, y}));
  TRY(check_ws(ws, ws_bytes, lr_linear_workspace_bytes(T, d_in, r, d_out, dt, 0)));
  Ctx c; c.base = (char*)ws; c.cap = ws_bytes; c.dt = dt; c.st = (hipStream_t)stream;
  LinArgs a{}; a.x = x; a.w_down = w_down; a.w_up = w_up; a.z = z; a.y = y; a.ldx = ldx; a.ldy = ldy;
  a.T = T; a.d_in = d_in; a.r = r; a.d_out = d_out; a.act = act;
  linear_fwd_seq(c, a);
  return status_of(c);
}

int lr_linear_bwd(const void* x, int64_t ldx, const void* w_down, const void* w_up, const void* z, const void* dy,
                  int64_t lddy, void* dx, int64_t lddx, void* dw_down, void* dw_up, int64_t T, int64_t d_in, int64_t r,
                  int64_t d_out, int act, int dt, int grad_dt, int accumulate, void* ws, size_t ws_bytes,
                  void* stream) {
  TRY(check_dt(dt)); TRY(check_act(act)); TRY(check_gdt(dt, grad_dt));
  if (T < 0 || T > 0x7fffffffLL) return LR_EINVAL;
  TRY(check_sizes_fit_int({d_in, r, d_out}));
  if (ldx < d_in || lddy < d_out || lddx < d_in) return LR_EINVAL;
  TRY(check_dims_bf16(dt, {d_in, r, d_out, ldx, lddy, lddx}));
  if (T == 0) return LR_OK;   // no tokens: gradients are left as they are
  TRY(check_ptrs(dt, {x, w_down, w_up, z, dy, dx}));
  TRY(check_gptrs(grad_dt, {dw_down, dw_up}));
  TRY(check_ws(ws, ws_bytes, lr_linear_workspace_bytes(T, d_in, r, d_out, dt, 1)));
  Ctx c; c.base = (char*)ws; c.cap = ws_bytes; c.dt = dt; c.gdt = grad_dt; c.st = (hipStream_t)stream;
  LinArgs a{}; a.x = x; a.w_down = w_down; a.w_up = w_up; a.zc = z; a.dy = dy; a.dx = dx; a.dw_down = dw_down;
  a.dw_up = dw_up; a.ldx = ldx; a.lddy = lddy; a.lddx = lddx; a.T = T; a.d_in = d_in; a.r = r; a.d_out = d_out;
  a.act = act; a.accumulate = accumulate;
  linear_bwd_seq(c, a);
  return status_of(c);
}

// ---- linear forward for callers that cannot allocate ------------------------------------------------
// The rank-r activation sigma(z) between the two GEMMs of lr_linear_fwd, which that entry point keeps in
// the caller's workspace, lives here in a file-scope device array.  Each GPU holds its own copy of the
// array at its own address: the address is looked up once per device (with that device current) and kept;
// host code only ever uses that looked-up pointer, never the array's name.
}  // extern "C"
namespace {
static __device__ __align__(256) unsigned char g_linear_scratch[LR_LINEAR_STATIC_SCRATCH_BYTES];
constexpr int kMaxDevices = 64;
std::mutex g_scratch_mutex;
void* g_scratch_ptr[kMaxDevices] = {};

int linear_scratch_of_current_device(void** out) {
  int dev = -1;
  if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= kMaxDevices) return LR_ELAUNCH;
  std::lock_guard<std::mutex> lock(g_scratch_mutex);
  if (!g_scratch_ptr[dev]) {
    void* p = nullptr;
    if (hipGetSymbolAddress(&p, HIP_SYMBOL(g_linear_scratch)) != hipSuccess || !p) return LR_ELAUNCH;
    g_scratch_ptr[dev] = p;
  }
  *out = g_scratch_ptr[dev];
  return LR_OK;
}
}  // namespace
extern "C" {

int lr_linear_fwd_static(const void* x, int64_t ldx, const void* w_down, const void* w_up, void* z, void* y,
                         int64_t ldy, int64_t T, int64_t d_in, int64_t r, int64_t d_out, int act, int dt,
                         void* stream) {
  TRY(check_dt(dt)); TRY(check_act(act));
  if (T < 0 || T > 0x7fffffffLL) return LR_EINVAL;
  TRY(check_sizes_fit_int({d_in, r, d_out}));
  if (ldx < d_in || ldy < d_out) return LR_EINVAL;
  TRY(check_dims_bf16(dt, {d_in, r, d_out, ldx, ldy}));
  if (T == 0) return LR_OK;
  TRY(check_ptrs(dt, {x, w_down, w_up, z, y}));
  // the same carving as lr_linear_fwd, run dry: what the sequence takes from its scratch
  Ctx dry; dry.dry = true; dry.dt = dt;
  LinArgs a{}; a.x = x; a.w_down = w_down; a.w_up = w_up; a.z = z; a.y = y; a.ldx = ldx; a.ldy = ldy;
  a.T = T; a.d_in = d_in; a.r = r; a.d_out = d_out; a.act = act;
  linear_fwd_seq(dry, a);
  if (dry.peak > (size_t)LR_LINEAR_STATIC_SCRATCH_BYTES) return LR_EWORKSPACE;
  void* scratch = nullptr;
  TRY(linear_scratch_of_current_device(&scratch));
  Ctx c; c.base = (char*)scratch; c.cap = LR_LINEAR_STATIC_SCRATCH_BYTES; c.dt = dt; c.st = (hipStream_t)stream;
  linear_fwd_seq(c, a);
  return status_of(c);
}

// ---- group -----------------------------------------------------------------------------------
size_t lr_group_workspace_bytes(int G, int64_t T, int64_t d_in, int64_t r, int64_t d_out, int dt, int backward) {
  if (check_dt(dt) != LR_OK || G <= 0 || G > 64 || T < 0 || check_sizes_fit_int({d_in, r, d_out}) != LR_OK) return 0;
  if (T == 0) return 0;
  Ctx c; c.dry = true; c.dt = dt;
  GrpArgs a{}; a.G = G; a.T = T; a.d_in = d_in; a.r = r; a.d_out = d_out; a.ldx = d_in; a.ldy = d_out;
  a.y_bs = T * d_out; a.lddy = d_out; a.dy_bs = T * d_out; a.lddx = d_in;
  size_t peak = 0;
  // take the larger of the norm variants so one query serves all of them
  for (int norm : {LR_NORM_NONE, LR_NORM_TWO_PASS, LR_NORM_ONLINE, LR_NORM_SHARD_LOCAL}) {
    if (backward && norm == LR_NORM_SHARD_LOCAL) continue;
    c.off = 0; a.norm = norm;
    if (backward) group_bwd_full_seq(c, a); else group_fwd_seq(c, a);
    if (c.peak > peak) peak = c.peak;
  }
  return peak + 256;
}

int lr_group_fwd(const void* x, int64_t ldx, const void* gamma, float eps, int norm, const void* w_down_cat,
                 const void* w_up_stack, void* z_cat, float* stat, void* y_stack, int64_t ldy, int64_t y_batch_stride,
                 int G, int64_t T, int64_t d_in, int64_t r, int64_t d_out, int act, int dt, void* ws, size_t ws_bytes,
                 void* stream) {
  TRY(check_dt(dt)); TRY(check_act(act));
  const bool shard = norm == LR_NORM_SHARD_LOCAL;   // stops before the exchange: no up-projections, no y
  if (norm != LR_NORM_NONE && norm != LR_NORM_TWO_PASS && norm != LR_NORM_ONLINE && norm != LR_NORM_ONLINE_GATHER && !shard)
    return LR_EINVAL;
  if (G <= 0 || G > 64 || T < 0 || T > 0x7fffffffLL) return LR_EINVAL;
  TRY(check_sizes_fit_int({d_in, r, d_out}));
  if ((int64_t)G * r > 0x7fffffffLL) return LR_EINVAL;
  if (ldx < d_in || (!shard && ldy < d_out)) return LR_EINVAL;
  if (!shard && G > 1 && y_batch_stride < d_out) return LR_EINVAL;
  TRY(check_dims_bf16(dt, {d_in, r, ldx}));
  if (!shard) TRY(check_dims_bf16(dt, {d_out, ldy, y_batch_stride}));
  if (T == 0) return LR_OK;
  TRY(check_ptrs(dt, {x, w_down_cat, z_cat}));
  if (!shard) TRY(check_ptrs(dt, {w_up_stack, y_stack}));
  if (norm != LR_NORM_NONE) {
    TRY(check_ptrs(dt, {gamma}));
    if (!stat) return LR_EINVAL;
  }
  if (T == 0) return LR_OK;
  TRY(check_ws(ws, ws_bytes, lr_group_workspace_bytes(G, T, d_in, r, d_out, dt, 0)));
  Ctx c; c.base = (char*)ws; c.cap = ws_bytes; c.dt = dt; c.st = (hipStream_t)stream;
  GrpArgs a{}; a.x = x; a.gamma = gamma; a.w_down_cat = w_down_cat; a.w_up_stack = w_up_stack; a.z_cat = z_cat;
  a.stat = stat; a.y_stack = y_stack; a.ldx = ldx; a.ldy = ldy; a.y_bs = y_batch_stride; a.T = T; a.d_in = d_in;
  a.r = r; a.d_out = d_out; a.G = G; a.act = act; a.norm = norm; a.eps = eps;
  group_fwd_seq(c, a);
  return status_of(c);
}

int lr_group_bwd(const void* x, int64_t ldx, const void* gamma, float eps, int norm, const void* w_down_cat,
                 const void* w_up_stack, const void* z_cat, const float* stat, const void* dy_stack, int64_t lddy,
                 int64_t dy_batch_stride, void* dx, int64_t lddx, void* dgamma, void* dw_down_cat, void* dw_up_stack,
                 int G, int64_t T, int64_t d_in, int64_t r, int64_t d_out, int act, int dt, int grad_dt, int accumulate,
                 void* ws, size_t ws_bytes, void* stream) {
  TRY(check_dt(dt)); TRY(check_act(act)); TRY(check_gdt(dt, grad_dt));
  if (norm != LR_NORM_NONE && norm != LR_NORM_TWO_PASS && norm != LR_NORM_ONLINE && norm != LR_NORM_ONLINE_GATHER)
    return LR_EINVAL;
  if (G <= 0 || G > 64 || T < 0 || T > 0x7fffffffLL) return LR_EINVAL;
  TRY(check_sizes_fit_int({d_in, r, d_out}));
  if ((int64_t)G * r > 0x7fffffffLL) return LR_EINVAL;
  if (ldx < d_in || lddy < d_out || lddx < d_in) return LR_EINVAL;
  if (G > 1 && dy_batch_stride < d_out) return LR_EINVAL;
  TRY(check_dims_bf16(dt, {d_in, r, d_out, ldx, lddy, lddx, dy_batch_stride}));
  if (T == 0) return LR_OK;
  TRY(check_ptrs(dt, {x, w_down_cat, w_up_stack, z_cat, dy_stack, dx}));
  TRY(check_gptrs(grad_dt, {dw_down_cat, dw_up_stack}));
  if (norm != LR_NORM_NONE) {
    TRY(check_ptrs(dt, {gamma}));
    TRY(check_gptrs(grad_dt, {dgamma}));
    if (!stat) return LR_EINVAL;
  }
  if (T == 0) return LR_OK;
  TRY(check_ws(ws, ws_bytes, lr_group_workspace_bytes(G, T, d_in, r, d_out, dt, 1)));
  Ctx c; c.base = (char*)ws; c.cap = ws_bytes; c.dt = dt; c.gdt = grad_dt; c.st = (hipStream_t)stream;
  GrpArgs a{}; a.x = x; a.gamma = gamma; a.w_down_cat = w_down_cat; a.w_up_stack = w_up_stack; a.zc = z_cat;
  a.statc = stat; a.dy_stack = dy_stack; a.dx = dx; a.dgamma = dgamma; a.dw_down_cat = dw_down_cat;
  a.dw_up_stack = dw_up_stack; a.ldx = ldx; a.lddy = lddy; a.dy_bs = dy_batch_stride; a.lddx = lddx; a.T = T;
  a.d_in = d_in; a.r = r; a.d_out = d_out; a.G = G; a.act = act; a.norm = norm; a.eps = eps; a.accumulate = accumulate;
  group_bwd_full_seq(c, a);
  return status_of(c);
}


// ---- block -----------------------------------------------------------------------------------
size_t lr_block_workspace_bytes(const lr_block_desc* desc, int backward) {
  Blk b; int why;
  if (!block_desc_ok(desc, b, &why)) return 0;
  Ctx c; c.dry = true; c.dt = LR_BF16;
  lr_block_params np{};
  if (backward) block_bwd_seq(c, b, nullptr, nullptr, nullptr, nullptr, nullptr, nullptr, 0);
  else block_fwd_seq(c, b, &np, nullptr, nullptr, nullptr);
  return c.peak + 256;
}

size_t lr_block_ckpt_bytes(const lr_block_desc* desc) {
  Blk b; int why;
  if (!block_desc_ok(desc, b, &why)) return 0;
  return (size_t)7 * b.T * b.r * 2 + (size_t)2 * b.T * sizeof(float);
}

static int check_params(const lr_block_params* p) {
  if (!p) return LR_EINVAL;
  return check_ptrs(LR_BF16, {p->gamma1, p->w_dn_qkv, p->w_up_qkv, p->w_dn_o, p->w_up_o, p->gamma2, p->w_dn_gu,
                              p->w_up_gu, p->w_dn_d, p->w_up_d});
}
static int check_ckpt(const lr_block_ckpt* ck) {
  if (!ck) return LR_EINVAL;
  TRY(check_ptrs(LR_BF16, {ck->z_qkv, ck->z_o, ck->z_gu, ck->z_d}));
  if (!ck->s1 || !ck->s2) return LR_EINVAL;
  return LR_OK;
}

int lr_block_fwd(const lr_block_desc* desc, const lr_block_params* params, const void* x, void* y,
                 const lr_block_ckpt* ckpt, void* ws, size_t ws_bytes, void* stream) {
  Blk b; int why;
  if (!block_desc_ok(desc, b, &why)) return why;
  TRY(check_params(params)); TRY(check_ckpt(ckpt));
  TRY(check_ptrs(LR_BF16, {x, y}));
  TRY(check_ws(ws, ws_bytes, lr_block_workspace_bytes(desc, 0)));
  Ctx c; c.base = (char*)ws; c.cap = ws_bytes; c.dt = LR_BF16; c.st = (hipStream_t)stream;
  block_fwd_seq(c, b, params, x, y, ckpt);
  return c.err == hipErrorNotSupported ? LR_EUNSUPPORTED : status_of(c);
}

int lr_block_bwd(const lr_block_desc* desc, const lr_block_params* params, const void* x, const void* dy,
                 const lr_block_ckpt* ckpt, void* dx, const lr_block_params* grads, int accumulate, void* ws,
                 size_t ws_bytes, void* stream) {
  Blk b; int why;
  if (!block_desc_ok(desc, b, &why)) return why;
  TRY(check_params(params)); TRY(check_params(grads)); TRY(check_ckpt(ckpt));
  TRY(check_ptrs(LR_BF16, {x, dy, dx}));
  TRY(check_ws(ws, ws_bytes, lr_block_workspace_bytes(desc, 1)));
  Ctx c; c.base = (char*)ws; c.cap = ws_bytes; c.dt = LR_BF16; c.gdt = b.gdt; c.st = (hipStream_t)stream;
  block_bwd_seq(c, b, params, x, dy, ckpt, dx, grads, accumulate);
  return c.err == hipErrorNotSupported ? LR_EUNSUPPORTED : status_of(c);
}

// ---- block with every wide activation kept (the store-everything reference of Sec. 4.4 / Table 5) ----
size_t lr_block_saved_workspace_bytes(const lr_block_desc* desc, int backward) {
  Blk b; int why;
  if (!block_desc_ok(desc, b, &why)) return 0;
  Ctx c; c.dry = true; c.dt = LR_BF16;
  lr_block_params np{};
  lr_block_saved nsv{};
  if (backward) block_bwd_seq(c, b, nullptr, nullptr, nullptr, nullptr, nullptr, nullptr, 0, nullptr, &nsv);
  else block_fwd_seq(c, b, &np, nullptr, nullptr, nullptr, nullptr, &nsv);
  return c.peak + 256;
}

static int check_saved(const lr_block_saved* sv) {
  if (!sv) return LR_EINVAL;
  TRY(check_ptrs(LR_BF16, {sv->qkv, sv->o, sv->h1, sv->gu, sv->m}));
  if (!sv->lse) return LR_EINVAL;
  return LR_OK;
}

int lr_block_fwd_save(const lr_block_desc* desc, const lr_block_params* params, const void* x, void* y,
                      const lr_block_ckpt* ckpt, const lr_block_saved* saved, void* ws, size_t ws_bytes, void* stream) {
  Blk b; int why;
  if (!block_desc_ok(desc, b, &why)) return why;
  TRY(check_params(params)); TRY(check_ckpt(ckpt)); TRY(check_saved(saved));
  TRY(check_ptrs(LR_BF16, {x, y}));
  TRY(check_ws(ws, ws_bytes, lr_block_saved_workspace_bytes(desc, 0)));
  Ctx c; c.base = (char*)ws; c.cap = ws_bytes; c.dt = LR_BF16; c.st = (hipStream_t)stream;
  block_fwd_seq(c, b, params, x, y, ckpt, nullptr, saved);
  return status_of(c);
}

int lr_block_bwd_saved(const lr_block_desc* desc, const lr_block_params* params, const void* x, const void* dy,
                       const lr_block_ckpt* ckpt, const lr_block_saved* saved, void* dx, const lr_block_params* grads,
                       int accumulate, void* ws, size_t ws_bytes, void* stream) {
  Blk b; int why;
  if (!block_desc_ok(desc, b, &why)) return why;
  TRY(check_params(params)); TRY(check_params(grads)); TRY(check_ckpt(ckpt)); TRY(check_saved(saved));
  TRY(check_ptrs(LR_BF16, {x, dy, dx}));
  TRY(check_ws(ws, ws_bytes, lr_block_saved_workspace_bytes(desc, 1)));
  Ctx c; c.base = (char*)ws; c.cap = ws_bytes; c.dt = LR_BF16; c.gdt = b.gdt; c.st = (hipStream_t)stream;
  block_bwd_seq(c, b, params, x, dy, ckpt, dx, grads, accumulate, nullptr, saved);
  return status_of(c);
}

// ---- block, LaX variant -------------------------------------------------------------------------
static int check_lax(const lr_block_desc* desc, const lr_block_lax* lx) {
  if (!lx) return LR_EINVAL;
  if (desc->act != LR_ACT_IDENTITY) return LR_EUNSUPPORTED;
  for (const void* q : {lx->h_prev_qkv, lx->h_prev_o, lx->h_prev_gu, lx->h_prev_d, lx->dz_next_qkv, lx->dz_next_o,
                        lx->dz_next_gu, lx->dz_next_d, (const void*)lx->dh_prev_qkv, (const void*)lx->dh_prev_o,
                        (const void*)lx->dh_prev_gu, (const void*)lx->dh_prev_d})
    if (q && !aligned16(q)) return LR_EALIGN;   // each is optional
  return LR_OK;
}

int lr_block_lax_fwd(const lr_block_desc* desc, const lr_block_params* params, const void* x, void* y,
                     const lr_block_ckpt* ckpt, const lr_block_lax* lax, void* ws, size_t ws_bytes, void* stream) {
  Blk b; int why;
  if (!block_desc_ok(desc, b, &why)) return why;
  TRY(check_lax(desc, lax));
  TRY(check_params(params)); TRY(check_ckpt(ckpt));
  TRY(check_ptrs(LR_BF16, {x, y}));
  TRY(check_ws(ws, ws_bytes, lr_block_workspace_bytes(desc, 0)));
  Ctx c; c.base = (char*)ws; c.cap = ws_bytes; c.dt = LR_BF16; c.st = (hipStream_t)stream;
  block_fwd_seq(c, b, params, x, y, ckpt, lax);
  return c.err == hipErrorNotSupported ? LR_EUNSUPPORTED : status_of(c);
}

int lr_block_lax_bwd(const lr_block_desc* desc, const lr_block_params* params, const void* x, const void* dy,
                     const lr_block_ckpt* ckpt, void* dx, const lr_block_params* grads, int accumulate,
                     const lr_block_lax* lax, void* ws, size_t ws_bytes, void* stream) {
  Blk b; int why;
  if (!block_desc_ok(desc, b, &why)) return why;
  TRY(check_lax(desc, lax));
  TRY(check_params(params)); TRY(check_params(grads)); TRY(check_ckpt(ckpt));
  TRY(check_ptrs(LR_BF16, {x, dy, dx}));
  TRY(check_ws(ws, ws_bytes, lr_block_workspace_bytes(desc, 1)));
  Ctx c; c.base = (char*)ws; c.cap = ws_bytes; c.dt = LR_BF16; c.gdt = b.gdt; c.st = (hipStream_t)stream;
  block_bwd_seq(c, b, params, x, dy, ckpt, dx, grads, accumulate, lax);
  return c.err == hipErrorNotSupported ? LR_EUNSUPPORTED : status_of(c);
}

// ---- attention -------------------------------------------------------------------------------
static int check_attn(int64_t ld, int64_t B, int64_t S, int64_t H, int64_t hd, int causal, int dt) {
  if (B <= 0 || S <= 0 || H <= 0 || hd <= 0 || ld < H * hd) return LR_EINVAL;
  if (B * S > 0x7fffffffLL || B * H > 0x7fffffffLL) return LR_EINVAL;
  if (dt != LR_BF16 || hd != 128 || causal != 1) return LR_EUNSUPPORTED;
  if (S * ld * 2 >= 0x7fffffffLL) return LR_EUNSUPPORTED;   // the kernels use 32-bit byte offsets per batch element
  if (ld % 8) return LR_EALIGN;
  return LR_OK;
}

int lr_attention_fwd(const void* q, const void* k, const void* v, void* o, float* lse, int64_t ld, int64_t B,
                     int64_t S, int64_t H, int64_t hd, int causal, int dt, void* stream) {
  TRY(check_attn(ld, B, S, H, hd, causal, dt));
  TRY(check_ptrs(LR_BF16, {q, k, v, o}));
  if (!lse) return LR_EINVAL;
  hipError_t e = attention_fwd_bf16(q, k, v, o, lse, ld, (int)B, (int)S, (int)H, (int)hd, causal, (hipStream_t)stream);
  return e == hipSuccess ? LR_OK : (e == hipErrorNotSupported ? LR_EUNSUPPORTED : LR_ELAUNCH);
}

size_t lr_attention_bwd_workspace_bytes(int64_t B, int64_t S, int64_t H, int64_t hd) {
  if (B <= 0 || S <= 0 || H <= 0 || hd != 128) return 0;
  return attention_bwd_ws_bytes((int)B, (int)S, (int)H, (int)hd) + 256;
}

int lr_attention_bwd(const void* q, const void* k, const void* v, const void* o, const void* dout, const float* lse,
                     void* dq, void* dk, void* dv, int64_t ld, int64_t B, int64_t S, int64_t H, int64_t hd, int causal,
                     int dt, void* ws, size_t ws_bytes, void* stream) {
  TRY(check_attn(ld, B, S, H, hd, causal, dt));
  TRY(check_ptrs(LR_BF16, {q, k, v, o, dout, dq, dk, dv}));
  if (!lse) return LR_EINVAL;
  TRY(check_ws(ws, ws_bytes, lr_attention_bwd_workspace_bytes(B, S, H, hd)));
  hipError_t e = attention_bwd_bf16(q, k, v, o, dout, lse, dq, dk, dv, ld, (int)B, (int)S, (int)H, (int)hd, causal, ws,
                                    (hipStream_t)stream);
  return e == hipSuccess ? LR_OK : (e == hipErrorNotSupported ? LR_EUNSUPPORTED : LR_ELAUNCH);
}

// grouped-query attention: H query heads over Hkv key / value heads
static int check_attn_gqa(int64_t ld, int64_t ldkv, int64_t B, int64_t S, int64_t H, int64_t Hkv, int64_t hd, int causal,
                          int dt) {
  if (Hkv <= 0 || H <= 0 || H % Hkv != 0 || hd <= 0 || ldkv < Hkv * hd) return LR_EINVAL;
  TRY(check_attn(ld, B, S, H, hd, causal, dt));
  if (S * ldkv * 2 >= 0x7fffffffLL) return LR_EUNSUPPORTED;
  if (ldkv % 8) return LR_EALIGN;
  return LR_OK;
}

int lr_attention_gqa_fwd(const void* q, const void* k, const void* v, void* o, float* lse, int64_t ld, int64_t ldkv,
                         int64_t B, int64_t S, int64_t H, int64_t Hkv, int64_t hd, int causal, int dt, void* stream) {
  TRY(check_attn_gqa(ld, ldkv, B, S, H, Hkv, hd, causal, dt));
  TRY(check_ptrs(LR_BF16, {q, k, v, o}));
  if (!lse) return LR_EINVAL;
  hipError_t e = attention_gqa_fwd_bf16(q, k, v, o, lse, ld, ldkv, (int)B, (int)S, (int)H, (int)Hkv, (int)hd, causal,
                                        (hipStream_t)stream);
  return e == hipSuccess ? LR_OK : (e == hipErrorNotSupported ? LR_EUNSUPPORTED : LR_ELAUNCH);
}

size_t lr_attention_gqa_bwd_workspace_bytes(int64_t B, int64_t S, int64_t H, int64_t Hkv, int64_t hd) {
  if (B <= 0 || S <= 0 || H <= 0 || Hkv <= 0 || H % Hkv != 0 || hd != 128) return 0;
  if (B * S > 0x7fffffffLL || B * H > 0x7fffffffLL) return 0;
  return attention_gqa_bwd_ws_bytes((int)B, (int)S, (int)H, (int)Hkv, (int)hd) + 256;
}

int lr_attention_gqa_bwd(const void* q, const void* k, const void* v, const void* o, const void* dout, const float* lse,
                         void* dq, void* dk, void* dv, int64_t ld, int64_t ldkv, int64_t B, int64_t S, int64_t H,
                         int64_t Hkv, int64_t hd, int causal, int dt, void* ws, size_t ws_bytes, void* stream) {
  TRY(check_attn_gqa(ld, ldkv, B, S, H, Hkv, hd, causal, dt));
  TRY(check_ptrs(LR_BF16, {q, k, v, o, dout, dq, dk, dv}));
  if (!lse) return LR_EINVAL;
  TRY(check_ws(ws, ws_bytes, lr_attention_gqa_bwd_workspace_bytes(B, S, H, Hkv, hd)));
  hipError_t e = attention_gqa_bwd_bf16(q, k, v, o, dout, lse, dq, dk, dv, ld, ldkv, (int)B, (int)S, (int)H, (int)Hkv,
                                        (int)hd, causal, ws, (hipStream_t)stream);
  return e == hipSuccess ? LR_OK : (e == hipErrorNotSupported ? LR_EUNSUPPORTED : LR_ELAUNCH);
}

// ---- rotary position embedding -------------------------------------------------------------------
int lr_rope(void* x, int64_t ldx, const float* cos_tab, const float* sin_tab, int64_t B, int64_t S, int64_t H,
            int64_t hd, int inverse, int dt, void* stream) {
  if (B < 0 || S <= 0 || H <= 0 || hd <= 0 || ldx < H * hd) return LR_EINVAL;
  if (B * S > 0x7fffffffLL || H > 0x7fffffffLL || S > 0x7fffffffLL) return LR_EINVAL;
  if (dt != LR_BF16 || hd != 128) return LR_EUNSUPPORTED;
  if (B == 0) return LR_OK;
  if (!cos_tab || !sin_tab) return LR_EINVAL;
  TRY(check_ptrs(LR_BF16, {x, cos_tab, sin_tab}));
  if (ldx % 8) return LR_EALIGN;
  hipError_t e = k_rope128_bf16(x, ldx, cos_tab, sin_tab, B * S, (int)S, (int)H, inverse, (hipStream_t)stream);
  return e == hipSuccess ? LR_OK : LR_ELAUNCH;
}

// ---- measurement aid ---------------------------------------------------------------------------
int lr_launch_timer_begin(int max_launches) { return launch_timer_begin(max_launches) == 0 ? LR_OK : LR_EINVAL; }
int lr_launch_timer_end(lr_launch_record* records, int max_records, int* n_records) {
  return launch_timer_end(records, max_records, n_records) == 0 ? LR_OK : LR_EINVAL;
}

// ---- standalone memory-bound kernels ---------------------------------------------------------
int lr_rms_stat(const void* x, int64_t ldx, float* stat, int64_t T, int64_t d, int dt, void* stream) {
  TRY(check_dt(dt));
  if (T < 0 || d <= 0 || ldx < d || !stat) return LR_EINVAL;
  TRY(check_dims_bf16(dt, {d, ldx}));
  TRY(check_ptrs(dt, {x}));
  return k_rms_stat(x, ldx, stat, T, d, dt, (hipStream_t)stream) == hipSuccess ? LR_OK : LR_ELAUNCH;
}

int lr_rmsnorm_apply(const void* x, int64_t ldx, const void* gamma, const float* stat, float eps, void* xhat,
                     int64_t ldo, int64_t T, int64_t d, int dt, void* stream) {
  TRY(check_dt(dt));
  if (T < 0 || d <= 0 || ldx < d || ldo < d || !stat) return LR_EINVAL;
  TRY(check_dims_bf16(dt, {d, ldx, ldo}));
  TRY(check_ptrs(dt, {x, gamma, xhat}));
  return k_rmsnorm_apply(x, ldx, gamma, stat, eps, xhat, ldo, T, d, dt, (hipStream_t)stream) == hipSuccess ? LR_OK
                                                                                                        : LR_ELAUNCH;
}

int lr_online_rmsnorm_finish(const void* h_sum, int64_t ldh, const float* stat_sum, int64_t d_total, float eps,
                             void* z, int64_t ldz, int64_t T, int64_t n, int dt, void* stream) {
  TRY(check_dt(dt));
  if (T < 0 || n <= 0 || d_total <= 0 || ldh < n || ldz < n || !stat_sum) return LR_EINVAL;
  TRY(check_dims_bf16(dt, {n, ldh, ldz}));
  if (T == 0) return LR_OK;
  TRY(check_ptrs(dt, {h_sum, z}));
  return k_row_rms_scale(h_sum, ldh, stat_sum, d_total, eps, z, ldz, T, n, dt, (hipStream_t)stream) == hipSuccess
             ? LR_OK : LR_ELAUNCH;
}

int64_t lr_rmsnorm_bwd_parts(int64_t T) { return T > 0 ? k_rmsnorm_bwd_parts(T) : 0; }

int lr_rmsnorm_bwd(const void* x, int64_t ldx, const void* gamma, const float* stat, float eps, const void* dxhat,
                   int64_t lddxh, const void* dres, int64_t lddres, void* dx, int64_t lddx, float* dgamma_part,
                   int64_t T, int64_t d, int dt, void* stream) {
  TRY(check_dt(dt));
  if (T < 0 || d <= 0 || ldx < d || lddxh < d || lddx < d || !stat || !dgamma_part) return LR_EINVAL;
  if (dres && lddres < d) return LR_EINVAL;
  TRY(check_dims_bf16(dt, {d, ldx, lddxh, lddx, dres ? lddres : 0}));
  TRY(check_ptrs(dt, {x, gamma, dxhat, dx}));
  if (dres) TRY(check_ptrs(dt, {dres}));
  return k_rmsnorm_bwd(x, ldx, gamma, stat, eps, dxhat, lddxh, dres, lddres, dx, lddx, dgamma_part, T, d, dt,
                       (hipStream_t)stream) == hipSuccess ? LR_OK : LR_ELAUNCH;
}

int lr_act_fwd(const void* z, int64_t ldz, void* a, int64_t lda, int64_t T, int64_t n, int act, int dt, void* stream) {
  TRY(check_dt(dt)); TRY(check_act(act));
  if (T < 0 || n <= 0 || ldz < n || lda < n) return LR_EINVAL;
  TRY(check_dims_bf16(dt, {n, ldz, lda}));
  TRY(check_ptrs(dt, {z, a}));
  return k_act_fwd(z, ldz, a, lda, T, n, act, dt, (hipStream_t)stream) == hipSuccess ? LR_OK : LR_ELAUNCH;
}

int lr_swiglu_fwd(const void* g, const void* u, void* m, int64_t ld, int64_t T, int64_t f, int dt, void* stream) {
  TRY(check_dt(dt));
  if (T < 0 || f <= 0 || ld < f) return LR_EINVAL;
  TRY(check_dims_bf16(dt, {f, ld}));
  TRY(check_ptrs(dt, {g, u, m}));
  return k_swiglu_fwd(g, u, m, ld, T, f, dt, (hipStream_t)stream) == hipSuccess ? LR_OK : LR_ELAUNCH;
}

int lr_swiglu_bwd(const void* g, const void* u, const void* dm, void* dg, void* du, int64_t ld, int64_t T, int64_t f,
                  int dt, void* stream) {
  TRY(check_dt(dt));
  if (T < 0 || f <= 0 || ld < f) return LR_EINVAL;
  TRY(check_dims_bf16(dt, {f, ld}));
  TRY(check_ptrs(dt, {g, u, dm, dg, du}));
  return k_swiglu_bwd(g, u, dm, dg, du, ld, T, f, dt, (hipStream_t)stream) == hipSuccess ? LR_OK : LR_ELAUNCH;
}

}  // extern "C"
