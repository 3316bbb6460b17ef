/* lrboost -- C ABI of the low-rank bottleneck decoder-block hot path for one MI355X (gfx950).
 *
 * A linear map W[d_out, d_in] is replaced by  y = W_up . sigma(W_down . x)  with a rank-r
 * bottleneck (paper Sec. 2, "Low-Rank Matrix Factorization" / "Low-Rank Activation via
 * Auto-Encoder"; sigma = identity is the SVD variant of App. "Low-rank Training Algorithm").
 *
 * Conventions common to every entry point
 *  - Every pointer is a DEVICE pointer owned by the caller unless a comment says "host".  The
 *    library never allocates, frees or synchronises: each call validates its arguments on the
 *    host, enqueues kernels on `stream` (a hipStream_t passed as void*, NULL = default
 *    stream) and returns.  Scratch memory comes from the caller through (ws, ws_bytes); the
 *    matching *_workspace_bytes() call gives the size needed.
 *  - Matrices are row-major, activations token-major: x[T, d] with leading dimension ld (in
 *    elements).  Weights use the [out, in] layout: W_down[r, d_in], W_up[d_out, r], dense.
 *  - dt selects the storage type of activations, weights and gradients (LR_F32 or LR_BF16);
 *    accumulation is always fp32.  Per-token statistics are fp32 in either case.
 *  - LR_BF16 requires d_in, r, d_out and every leading dimension to be multiples of 8 and
 *    every pointer 16-byte aligned (LR_EALIGN otherwise).  T is arbitrary.
 *  - Return value: LR_OK or a negative lr_status.  Argument, alignment, workspace and
 *    "unsupported" errors (everything but LR_ELAUNCH) are detected on the host before any launch,
 *    so such a failed call has enqueued nothing.  LR_ELAUNCH reports that the runtime rejected a
 *    kernel launch midway through a call's sequence: the kernels before it have been enqueued and
 *    the outputs are then unspecified.  Faults inside kernels surface at the caller's next
 *    synchronisation.  Outputs must not alias inputs.
 *  - Weight and gamma gradients are written in grad_dt: LR_F32 (fp32 main-gradient buffers, the
 *    usual companion of bf16 weights; always the case when dt == LR_F32) or LR_BF16 (pure bf16,
 *    App. "Low-rank Training Algorithm", costs one more rounding).  accumulate != 0 adds them
 *    into the given buffers instead of overwriting.  Activation gradients (dx) use dt.
 */
#ifndef LRBOOST_H
#define LRBOOST_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum {
  LR_OK = 0,
  LR_EINVAL = -1,       /* null pointer, non-positive size, unknown enum value            */
  LR_EUNSUPPORTED = -2, /* valid request the library cannot run (e.g. fp32 block)         */
  LR_EWORKSPACE = -3,   /* ws is NULL or ws_bytes is smaller than *_workspace_bytes()     */
  LR_EALIGN = -4,       /* pointer / leading-dimension / size alignment rule violated     */
  LR_ELAUNCH = -5       /* a kernel launch was rejected by the runtime                    */
} lr_status;

typedef enum { LR_F32 = 0, LR_BF16 = 1 } lr_dtype;
typedef enum { LR_ACT_IDENTITY = 0, LR_ACT_SILU = 1 } lr_act;
/* LR_NORM_ONLINE: RMSNorm folded into the down-projection GEMM (sum of squares gathered
 * inside a GEMM, 1/rms applied as a per-row scale in the epilogue; single-GPU form of the
 * paper's Alg. 1).  LR_NORM_TWO_PASS: the unfused twin (statistic pass, normalise pass,
 * plain GEMM), i.e. what Alg. 1 falls back to (Sec. 4.5 "Configuration").               */
/* LR_NORM_ONLINE takes the sum of squares from the A tiles inside the down-projection while the
 * output is at most 512 columns wide and from one pass over x (Alg. 1, its first step) beyond
 * that, where the pass is the faster of the two.  LR_NORM_ONLINE_GATHER is the same computation
 * with the in-GEMM gather at every width (bf16; fp32 storage takes the pass): no pass over x at
 * all, at the price of every column tile repeating the gather.  Same outputs, same backward.  */
/* LR_NORM_SHARD_LOCAL (lr_group_fwd only): one tensor-parallel rank's part of Alg. 1, the steps
 * before the exchange.  x[T, d_in] is the rank's slice of the features (d_in = d / TP), gamma its
 * slice of the scale, w_down_cat[G*r, d_in] the matching columns of the weights.  The rank takes its
 * local sum of squares, normalises its slice by its LOCAL rms, multiplies by its weight slice and
 * undoes the local scale on the product: z_cat[T, G*r] receives that un-normalised partial product
 * (to be summed over the ranks), stat[T] the local sum of squares (summed with it).  sigma, the
 * up-projections and y come after the exchange: act, w_up_stack, y_stack, ldy, y_batch_stride and
 * d_out are ignored (pass NULL / 0 / any positive d_out).  lr_online_rmsnorm_finish applies the
 * global rescale to the summed product.  No backward form.                                  */
typedef enum { LR_NORM_NONE = 0, LR_NORM_TWO_PASS = 1, LR_NORM_ONLINE = 2, LR_NORM_SHARD_LOCAL = 3,
               LR_NORM_ONLINE_GATHER = 4 } lr_norm;

int lr_version(void);
/* Human-readable name of a status code; static storage, never freed. */
const char* lr_status_string(int status);

/* ---- one bottleneck layer (Sec. 2: B sigma(A x)) ------------------------------------- */
/* y[T, d_out] = W_up . act(W_down . x);  z[T, r] (dense) receives the rank-r pre-activation,
 * the only tensor the backward needs besides x (Sec. 4.4).                                */
size_t lr_linear_workspace_bytes(int64_t T, int64_t d_in, int64_t r, int64_t d_out, int dt,
                                 int backward);
int lr_linear_fwd(const void* x, int64_t ldx, const void* w_down, const void* w_up, void* z,
                  void* y, int64_t ldy, int64_t T, int64_t d_in, int64_t r, int64_t d_out,
                  int act, int dt, void* ws, size_t ws_bytes, void* stream);
/* From x, z and dy[T, d_out]: dx[T, d_in], dw_down[r, d_in], dw_up[d_out, r].              */
int lr_linear_bwd(const void* x, int64_t ldx, const void* w_down, const void* w_up,
                  const void* z, const void* dy, int64_t lddy, void* dx, int64_t lddx,
                  void* dw_down, void* dw_up, int64_t T, int64_t d_in, int64_t r,
                  int64_t d_out, int act, int dt, int grad_dt, int accumulate, void* ws,
                  size_t ws_bytes, void* stream);

/* lr_linear_fwd for callers that cannot allocate device memory or hand over a workspace: code under
 * HIP graph capture, tight serving loops, harnesses that forbid hipMalloc.  Same arguments, results and
 * error codes as lr_linear_fwd without (ws, ws_bytes): the rank-r activation between the two GEMMs is
 * kept in a device array that is part of the library image (LR_LINEAR_STATIC_SCRATCH_BYTES per GPU, held
 * from the moment the library is loaded on that GPU until the process ends).  The call allocates and
 * frees nothing.  Limit: T * r * (2 for LR_BF16, 4 for LR_F32) bytes must fit the array, otherwise
 * LR_EWORKSPACE and nothing is enqueued.  All calls on one GPU share the array: calls that may run
 * concurrently on one GPU (different streams, different host threads) race on it and must be serialised
 * by the caller.  Nothing in it needs clearing between calls (every element a call reads, it has
 * written).  The first call on a device looks up the array's address, which is a set-up step: make it
 * before a stream capture begins, not inside one.                                                    */
#define LR_LINEAR_STATIC_SCRATCH_BYTES (32u << 20)
int lr_linear_fwd_static(const void* x, int64_t ldx, const void* w_down, const void* w_up, void* z,
                         void* y, int64_t ldy, int64_t T, int64_t d_in, int64_t r, int64_t d_out,
                         int act, int dt, void* stream);

/* ---- G projections sharing one input (Sec. 4.3 and App. "Linear Grouping Details") ---- */
/* w_down_cat[G*r, d_in]: the G down-projection weights concatenated along the rank axis (one
 * GEMM); w_up_stack[G, d_out, r]: stacked up-projection weights (one batched GEMM over the
 * (input, weight) pairs).  Optional RMSNorm of x (Eq. 4; gamma[d_in], eps inside the root):
 *   z_cat[T, G*r] = RMSNorm(x) . w_down_cat^T     (dense, the rank-r checkpoint)
 *   y_g[T, d_out] = act(z_g) . w_up_g^T           at y_stack + g*y_batch_stride, ld = ldy
 *   stat[T] (fp32) = sum_j x[t,j]^2               (written when norm != LR_NORM_NONE)
 * gamma and stat may be NULL when norm == LR_NORM_NONE.                                     */
size_t lr_group_workspace_bytes(int G, int64_t T, int64_t d_in, int64_t r, int64_t d_out,
                                int dt, int backward);
int lr_group_fwd(const void* x, int64_t ldx, const void* gamma, float eps, int norm,
                 const void* w_down_cat, const void* w_up_stack, void* z_cat, float* stat,
                 void* y_stack, int64_t ldy, int64_t y_batch_stride, int G, int64_t T,
                 int64_t d_in, int64_t r, int64_t d_out, int act, int dt, void* ws,
                 size_t ws_bytes, void* stream);
/* dx[T, d_in] is the gradient w.r.t. the un-normalised x; dgamma[d_in] (grad_dt; ignored when
 * norm == LR_NORM_NONE).  stat is the forward's output.                                     */
int lr_group_bwd(const void* x, int64_t ldx, const void* gamma, float eps, int norm,
                 const void* w_down_cat, const void* w_up_stack, const void* z_cat,
                 const float* stat, const void* dy_stack, int64_t lddy,
                 int64_t dy_batch_stride, void* dx, int64_t lddx, void* dgamma,
                 void* dw_down_cat, void* dw_up_stack, int G, int64_t T, int64_t d_in,
                 int64_t r, int64_t d_out, int act, int dt, int grad_dt, int accumulate,
                 void* ws, size_t ws_bytes, void* stream);

/* ---- the decoder block ------------------------------------------------------------------
 * RMSNorm -> grouped low-rank Q/K/V -> causal attention -> low-rank O + residual -> RMSNorm
 * -> grouped low-rank gate/up -> SiLU(g)*u -> low-rank down + residual.  Seven factored
 * projections (App. "Communication volume analysis": 11dr + 3 d_ff r parameters).  Only the
 * rank-r pre-activations are kept for the backward, which re-forwards everything wider from
 * them and from x (Sec. 4.4).                                                              */
typedef struct {
  int64_t batch, seq, d_model, n_heads, head_dim;
  int64_t ffn;     /* logical MLP width                                                    */
  int64_t ffn_ld;  /* padded MLP width, multiple of 8, >= ffn; the pad rows/columns of the
                      ffn-sized weights must be zero (then their gradients stay zero)      */
  int64_t rank;
  float eps;
  int act;         /* lr_act at rank r                                                     */
  int norm;        /* LR_NORM_ONLINE, LR_NORM_ONLINE_GATHER or LR_NORM_TWO_PASS            */
  int dt;          /* LR_BF16                                                              */
  int grad_dt;     /* dtype of the weight / gamma gradient buffers: LR_F32 or LR_BF16      */
  int causal;      /* 1                                                                    */
  /* Optional rotary position embedding of q and k (LLaMA-style models, Sec. 5.2), applied
   * between the up-projections and the attention in the forward and in the re-forward, and
   * transposed on dq, dk in the backward.  DEVICE pointers to cos / sin tables [seq, 64] fp32
   * (16-byte aligned) of the angles of lr_rope below; both NULL: no rotary embedding.       */
  const float* rope_cos;
  const float* rope_sin;
  /* Chaining the norm statistic through a stack of blocks (Sec. 4.2: the sum of squares travels
   * with the GEMM that produces the normalised tensor).  stat_y_out, if not NULL: DEVICE [T] fp32,
   * receives sum_j y[t,j]^2, accumulated from the fp32 output tiles in the epilogue of the block's
   * last GEMM; it is the s1 of the block above.  stat_x_ready != 0: ckpt->s1 already holds
   * sum_j x[t,j]^2 (the stat_y_out of the block below) and the forward takes it as given instead
   * of computing it from x.                                                                    */
  int stat_x_ready;
  float* stat_y_out;
  /* Grouped-query attention (section "Discussion and Future Work": only the shapes of the K and V
   * projections change).  0 or n_heads: multi-head.  Otherwise a divisor of n_heads: the K and V
   * up-projections are [n_kv_heads * head_dim, rank], and w_up_qkv (and its gradient) is packed:
   * W_up,q [d_model, rank], then W_up,k, then W_up,v.  Everything else keeps its shape.          */
  int64_t n_kv_heads;
} lr_block_desc;

typedef struct {
  void* gamma1;    /* [d]                                                                  */
  void* w_dn_qkv;  /* [3r, d]   q, k, v concatenated along the rank axis                   */
  void* w_up_qkv;  /* [3, d, r]  (n_kv_heads < n_heads: [d + 2 n_kv_heads head_dim, r])     */
  void* w_dn_o;    /* [r, d]                                                               */
  void* w_up_o;    /* [d, r]                                                               */
  void* gamma2;    /* [d]                                                                  */
  void* w_dn_gu;   /* [2r, d]   gate, up concatenated                                      */
  void* w_up_gu;   /* [2, ffn_ld, r]                                                       */
  void* w_dn_d;    /* [r, ffn_ld]                                                          */
  void* w_up_d;    /* [d, r]                                                               */
} lr_block_params;  /* the same struct, pointing at grad_dt buffers, receives the grads    */

typedef struct {
  void* z_qkv;     /* [T, 3r]                                                              */
  void* z_o;       /* [T, r]                                                               */
  void* z_gu;      /* [T, 2r]                                                              */
  void* z_d;       /* [T, r]                                                               */
  float* s1;       /* [T] sum of squares of x                                              */
  float* s2;       /* [T] sum of squares of h1 = x + attention branch                      */
} lr_block_ckpt;    /* rank-r checkpoints, written by fwd, read by bwd; caller-allocated    */

/* 0 when the descriptor is invalid or unsupported. */
size_t lr_block_workspace_bytes(const lr_block_desc* desc, int backward);
/* Bytes of all six checkpoint buffers together (information only; the caller allocates
 * each buffer of lr_block_ckpt separately, with the shapes given above).                  */
size_t lr_block_ckpt_bytes(const lr_block_desc* desc);
/* desc, params, ckpt are HOST structs holding device pointers.  x, y: [T, d], dense.      */
int lr_block_fwd(const lr_block_desc* desc, const lr_block_params* params, const void* x,
                 void* y, const lr_block_ckpt* ckpt, void* ws, size_t ws_bytes, void* stream);
/* x must be unchanged since the forward.  dy, dx: [T, d] dense.                           */
int lr_block_bwd(const lr_block_desc* desc, const lr_block_params* params, const void* x,
                 const void* dy, const lr_block_ckpt* ckpt, void* dx,
                 const lr_block_params* grads, int accumulate, void* ws, size_t ws_bytes,
                 void* stream);

/* ---- the block with every wide activation kept ---------------------------------------------
 * The reference point of the checkpointing comparison (Sec. 4.4, Table 5: memory saved against time
 * added by keeping only rank-r activations): lr_block_fwd_save also leaves every d-wide and ffn-wide
 * activation of the forward in caller-owned buffers, and lr_block_bwd_saved reads them instead of
 * re-forwarding from the rank-r checkpoints (which it still takes: sigma and sigma' are rebuilt from z at
 * rank r).  Results equal those of lr_block_fwd / lr_block_bwd bit for bit (recomputed = stored).  Dense
 * bf16 unless noted; the backward only reads them:
 *   qkv  q [T, d], then k [T, d_kv], then v [T, d_kv], back to back (after the rotary embedding, if any)
 *   o    [T, d]        lse  [batch, n_heads, seq] fp32        h1  [T, d]
 *   gu   g [T, ffn_ld], then u [T, ffn_ld]                    m   [T, ffn_ld]
 * 2.4 GB at the 7B shape (batch 4 x seq 4096) against 0.24 GB of rank-r checkpoints.                 */
typedef struct {
  void *qkv, *o;
  float* lse;
  void *h1, *gu, *m;
} lr_block_saved;
size_t lr_block_saved_workspace_bytes(const lr_block_desc* desc, int backward);
int lr_block_fwd_save(const lr_block_desc* desc, const lr_block_params* params, const void* x,
                      void* y, const lr_block_ckpt* ckpt, const lr_block_saved* saved, void* ws,
                      size_t ws_bytes, void* stream);
int lr_block_bwd_saved(const lr_block_desc* desc, const lr_block_params* params, const void* x,
                       const void* dy, const lr_block_ckpt* ckpt, const lr_block_saved* saved,
                       void* dx, const lr_block_params* grads, int accumulate, void* ws,
                       size_t ws_bytes, void* stream);

/* ---- the LaX variant of the block (App. "LaX variant (residual low-rank)") ----------------
 * Identity gate at rank r, and every bottleneck layer adds the rank-r activation h_{i-1} of the
 * same projection in the decoder layer below before its up-projection: y_i = B_i (h_i + h_{i-1}),
 * h_i = A_i x_i.  A block's own h_i are its checkpoints z_* (lr_block_ckpt), which the caller
 * hands to the block above as h_prev_*.  In the backward, dz_next_* is the block above's
 * gradient w.r.t. this block's z_* (its dh_prev_*), and dh_prev_* receives this block's gradient
 * w.r.t. its h_prev_*.  Layouts as the checkpoints: qkv [T, 3r], o [T, r], gu [T, 2r], d [T, r],
 * bf16, dense.  Each pointer may be NULL: an absent h_prev / dz_next counts as zeros (first /
 * last block of a stack), an absent dh_prev is not written.  desc->act must be
 * LR_ACT_IDENTITY (else LR_EUNSUPPORTED); everything else as lr_block_fwd / lr_block_bwd
 * (grouped key / value heads included), same workspace sizes.                               */
typedef struct {
  const void *h_prev_qkv, *h_prev_o, *h_prev_gu, *h_prev_d;       /* forward and backward inputs  */
  const void *dz_next_qkv, *dz_next_o, *dz_next_gu, *dz_next_d;   /* backward inputs              */
  void *dh_prev_qkv, *dh_prev_o, *dh_prev_gu, *dh_prev_d;         /* backward outputs             */
} lr_block_lax;
int lr_block_lax_fwd(const lr_block_desc* desc, const lr_block_params* params, const void* x,
                     void* y, const lr_block_ckpt* ckpt, const lr_block_lax* lax, void* ws,
                     size_t ws_bytes, void* stream);
int lr_block_lax_bwd(const lr_block_desc* desc, const lr_block_params* params, const void* x,
                     const void* dy, const lr_block_ckpt* ckpt, void* dx,
                     const lr_block_params* grads, int accumulate, const lr_block_lax* lax,
                     void* ws, size_t ws_bytes, void* stream);

/* ---- rotary position embedding (optional step of the block; the paper does not describe
 * it, LLaMA-style attention has it) -------------------------------------------------------
 * In place on x[B*S, ldx] (bf16, H heads of hd = 128 from column 0): inside every head the pair
 * (v[i], v[i + 64]), i < 64, of the token at position p of its sequence becomes
 * (v[i] c - v[i+64] s, v[i+64] c + v[i] s) with c = cos_tab[p, i], s = sin_tab[p, i]
 * (DEVICE tables [S, 64] fp32).  inverse != 0 uses -s: the transpose of the rotation, which
 * is its backward.  Other dtypes / head sizes: LR_EUNSUPPORTED.                             */
int lr_rope(void* x, int64_t ldx, const float* cos_tab, const float* sin_tab, int64_t B,
            int64_t S, int64_t H, int64_t hd, int inverse, int dt, void* stream);

/* ---- causal multi-head attention (the sharded-safe op between the chunks, Sec. 4.2) ---- */
/* q, k, v, o: [B*S, H*hd] token-major, head h in columns h*hd..; lse[B, H, S] fp32.
 * bf16 only, hd = 128, and S * ld * 2 < 2^31 bytes (the kernels address one batch element with
 * 32-bit buffer offsets); otherwise LR_EUNSUPPORTED.  The backward workspace holds two [B, H, S]
 * fp32 arrays (sum_h dO*O and lse * log2(e)) and, when S is a multiple of 8 and it stays under
 * 24 GiB, the score gradient scale * dS^T as bf16 [B, H, S, S] (4.3 GB at B 4, H 32, S 4096):
 * the key / value gradient kernel writes it and the query gradient is one GEMM over it, which
 * saves recomputing the scores a second time.  Other shapes take the recomputing form.        */
int lr_attention_fwd(const void* q, const void* k, const void* v, void* o, float* lse,
                     int64_t ld, int64_t B, int64_t S, int64_t H, int64_t hd, int causal,
                     int dt, void* stream);
size_t lr_attention_bwd_workspace_bytes(int64_t B, int64_t S, int64_t H, int64_t hd);
int lr_attention_bwd(const void* q, const void* k, const void* v, const void* o,
                     const void* dout, const float* lse, void* dq, void* dk, void* dv,
                     int64_t ld, int64_t B, int64_t S, int64_t H, int64_t hd, int causal,
                     int dt, void* ws, size_t ws_bytes, void* stream);

/* Grouped-query form (the extension named in the section "Discussion and Future Work": only the
 * shapes of the K and V projections change).  Hkv key / value heads, H % Hkv == 0; query head h
 * attends over key / value head h / (H / Hkv).  q, o, dout, dq: [B*S, ld] with H heads of hd columns;
 * k, v, dk, dv: [B*S, ldkv] with Hkv heads; lse [B, H, S].  dk and dv are the sums over the query
 * heads of each group.  Same restrictions and error behaviour as the multi-head calls, which are the
 * case Hkv = H, ldkv = ld; for Hkv < H the backward workspace additionally holds one dK and one dV
 * contribution per query head (2 * B*S*H*hd bf16), added up by a last kernel.               */
int lr_attention_gqa_fwd(const void* q, const void* k, const void* v, void* o, float* lse,
                         int64_t ld, int64_t ldkv, int64_t B, int64_t S, int64_t H, int64_t Hkv,
                         int64_t hd, int causal, int dt, void* stream);
size_t lr_attention_gqa_bwd_workspace_bytes(int64_t B, int64_t S, int64_t H, int64_t Hkv,
                                            int64_t hd);
int lr_attention_gqa_bwd(const void* q, const void* k, const void* v, const void* o,
                         const void* dout, const float* lse, void* dq, void* dk, void* dv,
                         int64_t ld, int64_t ldkv, int64_t B, int64_t S, int64_t H, int64_t Hkv,
                         int64_t hd, int causal, int dt, void* ws, size_t ws_bytes, void* stream);

/* ---- measurement aid (not on the compute path) ------------------------------------------ */
/* Between begin and end every bf16 MFMA GEMM launch the library makes, and each attention forward /
 * backward call of the block, is bracketed by two HIP events on its stream.  end waits for the last one
 * and writes one record per bracketed launch, in launch order, into records[0 .. max_records) (HOST
 * memory; *n_records receives the number of launches seen, which may exceed max_records).  begin creates
 * max_launches event pairs and end destroys them: the one place where the library creates runtime
 * objects, and only on request.  Process-global and not thread-safe: one measuring thread, no compute
 * calls from other threads meanwhile.  Used by the benchmark for the per-class GEMM and attention rates
 * (Sec. 5.3 of the paper measures the same quantity per linear layer: kernel time and utilisation).
 * tag: the GEMM's epilogue class (0 store, 1 down-projection: row scale + sigma, 2 / 10 / 11 up-projection
 * + residual, 3 sigma' (+ row statistic), 4 / 12 / 13 RMSNorm backward, 5 split-K weight-gradient partial,
 * 6 SwiGLU backward, 7 SwiGLU forward, 8 / 9 the LaX forms), or LR_TAG_ATTN_FWD / LR_TAG_ATTN_BWD.
 * flops: 2 M N K batch for a GEMM; causal-halved 2 S^2 hd per (batch, head) and product for attention
 * (2 products forward, 5 backward).                                                               */
#define LR_TAG_ATTN_FWD 32
#define LR_TAG_ATTN_BWD 33
typedef struct {
  int tag, M, N, K, batch;
  float ms;
  double flops;
} lr_launch_record;
int lr_launch_timer_begin(int max_launches);
int lr_launch_timer_end(lr_launch_record* records, int max_records, int* n_records);
/* Sustained rate of the bf16 matrix pipes fed from registers alone (no LDS, no memory traffic):
 * 2048 wavefronts, 8 independent 32x32x16 accumulator tiles each, iters instructions per tile and
 * launch, `launches` timed launches after up to 4 untimed ones, on `stream`; *tflops (HOST pointer)
 * receives the rate.  random_operands = 0 uses smooth operand values, otherwise pseudo-random ones in
 * (-1, 1): the clock the chip holds under matrix load depends on how much the operand bits toggle,
 * so the second figure is the ceiling for a GEMM on trained-weight-like data.  Creates and destroys
 * two HIP events and waits for the launches.  iters in 1..2^20, launches in 1..1000, else
 * LR_EINVAL.  The utilisation of Sec. 5.3 is read against this figure and the published peak.    */
int lr_mfma_probe(int random_operands, int iters, int launches, double* tflops, void* stream);

/* ---- standalone memory-bound kernels: the unfused twins of the fused epilogues ---------- */
/* stat[t] = sum_j x[t,j]^2  (Alg. 1 line 1).                                               */
int lr_rms_stat(const void* x, int64_t ldx, float* stat, int64_t T, int64_t d, int dt,
                void* stream);
/* xhat = x * gamma / sqrt(stat/d + eps)  (Eq. 4).                                          */
int lr_rmsnorm_apply(const void* x, int64_t ldx, const void* gamma, const float* stat,
                     float eps, void* xhat, int64_t ldo, int64_t T, int64_t d, int dt,
                     void* stream);
/* The steps of Alg. 1 after the exchange: z[t, j] = h_sum[t, j] / sqrt(stat_sum[t] / d_total + eps) for
 * j < n, where h_sum[T, n] is the sum over the ranks of the partial products of LR_NORM_SHARD_LOCAL calls,
 * stat_sum[T] (fp32) the sum of their local statistics and d_total the full feature width (Eq. 5: the
 * result equals RMSNorm over the full width followed by the full projection).                  */
int lr_online_rmsnorm_finish(const void* h_sum, int64_t ldh, const float* stat_sum, int64_t d_total,
                             float eps, void* z, int64_t ldz, int64_t T, int64_t n, int dt,
                             void* stream);
/* Reverse mode of Eq. 4: dx = (dn - n*c)/rms [+ dres], dn = dxhat*gamma, n = x/rms,
 * c = mean_j(dn*n); dgamma_part[nparts, d] fp32 partial column sums of dxhat*n, where
 * nparts = lr_rmsnorm_bwd_parts(T) (the caller, or lr_colsum, adds them up).  dres may be
 * NULL.                                                                                    */
int64_t lr_rmsnorm_bwd_parts(int64_t T);
int lr_rmsnorm_bwd(const void* x, int64_t ldx, const void* gamma, const float* stat, float eps,
                   const void* dxhat, int64_t lddxh, const void* dres, int64_t lddres,
                   void* dx, int64_t lddx, float* dgamma_part, int64_t T, int64_t d, int dt,
                   void* stream);
/* a = act(z) elementwise on a [T, n] tensor.                                               */
int lr_act_fwd(const void* z, int64_t ldz, void* a, int64_t lda, int64_t T, int64_t n,
               int act, int dt, void* stream);
/* m = SiLU(g) * u    and its reverse  dg = dm*u*SiLU'(g), du = dm*SiLU(g).                 */
int lr_swiglu_fwd(const void* g, const void* u, void* m, int64_t ld, int64_t T, int64_t f,
                  int dt, void* stream);
int lr_swiglu_bwd(const void* g, const void* u, const void* dm, void* dg, void* du, int64_t ld,
                  int64_t T, int64_t f, int dt, void* stream);

#ifdef __cplusplus
}
#endif
#endif /* LRBOOST_H */
