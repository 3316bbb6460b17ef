// Internal declarations shared by the kernel files and the C-ABI layer of lrboost.
#pragma once
#include <hip/hip_runtime.h>
#include <stddef.h>
#include <stdint.h>

#include "lrboost.h"

namespace lrb {

// ---------------------------------------------------------------------------------------------
// Epilogue of C[M,N] = sum_k A(m,k) B(n,k): what happens to the fp32 accumulator tile before it
// is rounded and stored.  Row scalars (rowa, rowb) are final per-row values, not partials.
// ---------------------------------------------------------------------------------------------
enum EpiKind : int {
  EPI_STORE = 0,    // C = acc
  EPI_DOWN = 1,     // v = acc * rho_m (rho = rsqrt(rowa/d + eps) if norm) ; C = v ; C2 = act(v)
  EPI_UP = 2,       // v = acc + R ; C = v ; rowpart = sum_n v^2
  EPI_ACTGRAD = 3,  // v = acc * act'(R) * rho_m ; C = v ; rowpart = sum_n v * R      (R = z)
  EPI_NORMBWD = 4,  // v = acc - (rho_m/d) * rowb_m * R2 + R ; C = v     (R2 = x, R = residual grad)
  EPI_PARTIAL = 5,  // fp32 store of a split-K partial: Cpart[split][M][N]
  EPI_SWIGLU_BWD = 6,  // v = acc (= dm); C = v*R2*silu'(R) (dg), C2 = v*silu(R) (du); R=g, R2=u
  EPI_SWIGLU_FWD = 7,  // v = acc (= u); C = v (skipped when C is null), C2 = silu(R)*v (m); R = g
  // LaX variant (identity gate, rank-r residual from the layer below; App. "LaX variant"):
  EPI_DOWN_LAX = 8,    // v = acc * rho_m ; C = v (= h_i) ; C2 = v + R (R = h_{i-1}; absent R reads as zero)
  EPI_LAXGRAD = 9,     // C2 = acc (gradient w.r.t. h_{i-1}) ; v = (acc + R2) * rho_m (R2 = the layer above's
                       // gradient w.r.t. h_i) ; C = v ; rowpart = sum_n v * R (R = h_i)
  // The residual stream in fp32 (bf16 kernel only).  A residual sum x + f(x) stored in bf16 and added to
  // once more carries the rounding of the large term twice; these forms keep the un-rounded sum beside
  // the bf16 copy that the next GEMM consumes (O32: C32 = v as fp32, in addition to C) and take it back
  // as the residual of the next sum (I32: R is an fp32 tile).  Formulas as EPI_UP / EPI_NORMBWD.
  EPI_UP_O32 = 10,
  EPI_UP_I32 = 11,
  EPI_NORMBWD_O32 = 12,
  EPI_NORMBWD_I32 = 13
};
// the formula an epilogue kind applies (the fp32-residual forms share EPI_UP's and EPI_NORMBWD's)
constexpr int epi_base(int kind) {
  return (kind == EPI_UP_O32 || kind == EPI_UP_I32) ? (int)EPI_UP
         : (kind == EPI_NORMBWD_O32 || kind == EPI_NORMBWD_I32) ? (int)EPI_NORMBWD : kind;
}
constexpr bool epi_r_is_f32(int kind) { return kind == EPI_UP_I32 || kind == EPI_NORMBWD_I32; }
constexpr bool epi_writes_f32(int kind) { return kind == EPI_UP_O32 || kind == EPI_NORMBWD_O32; }

struct Epilogue {
  int kind = EPI_STORE;
  int act = LR_ACT_IDENTITY;
  int use_rho = 0;            // multiply rows by rho_m
  int rho_sqrt = 0;           // rho_m = sqrt(rowa/d + eps) instead of its reciprocal (un-scaling a local norm)
  int stat_from_a = 0;        // rowa is gathered from the A tiles in the main loop (bf16 kernel)
  const float* rowa = nullptr;  // [M] sum of squares
  const float* rowb = nullptr;  // [M]
  float inv_d = 0.f, eps = 0.f;
  float* stat_out = nullptr;  // [M] final sum of squares, written by the n-tile 0 blocks
  void* C2 = nullptr;
  int64_t ldc2 = 0, sC2 = 0;
  float* C32 = nullptr;       // O32 kinds: fp32 copy of the primary output (un-batched)
  int64_t ldc32 = 0;
  const void* R = nullptr;
  int64_t ldr = 0, sR = 0;
  const void* R2 = nullptr;
  int64_t ldr2 = 0, sR2 = 0;
  float* rowpart = nullptr;   // [M, rowpart_ld] per-(n-slab) partial row sums
  int64_t rowpart_ld = 0;
  int rowpart_off = 0;        // column offset (batched launches: g * slabs per batch)
};

struct GemmOp {
  const void* A = nullptr;
  const void* B = nullptr;
  void* C = nullptr;
  int64_t lda = 0, ldb = 0, ldc = 0;  // elements
  int64_t sA = 0, sB = 0, sC = 0;     // batch strides, elements
  int transA = 0, transB = 0;  // 0: operand(i,k) at p[i*ld + k]; 1: at p[k*ld + i]
  int M = 0, N = 0, K = 0, batch = 1;
  int splitk = 1;              // > 1: EPI_PARTIAL into fp32 C[batch][split][M][N] (ldc = N)
  // Two-level batches (bf16 kernel, A, B and C only): batch index = outer * batch_inner + inner, the
  // operand of that entry starts at outer * s?o + inner * s?.  batch_inner = 0: one level.
  int batch_inner = 0;
  int64_t sAo = 0, sBo = 0, sCo = 0;
  // k-major bf16 form only: the rows m0.. of a row tile use k < m0 + (tile height) only, i.e. A is
  // known to be zero where k > m (the causal structure of an attention gradient)
  int causal_k = 0;
  Epilogue epi;
};

// Number of n-slabs the bf16 kernel emits row partials for (rowpart_ld must be >= this * batch).
int gemm_bf16_rowpart_slabs(int N);
// Chooses a split-K factor for a weight-gradient GEMM with K = T.
int gemm_bf16_pick_splitk(int M, int N, int K, int batch);
hipError_t gemm_bf16(const GemmOp& op, hipStream_t st);
// the same launch, never counted by the benchmark timer below (launches that are not projection GEMMs)
hipError_t gemm_bf16_untimed(const GemmOp& op, hipStream_t st);
// true when gemm_bf16 can run `op` with both operands k-major (no transposed copies needed)
bool gemm_bf16_kmajor_ok(const GemmOp& op);
hipError_t gemm_f32(const GemmOp& op, hipStream_t st);
// Benchmark aid: launches bracketed by HIP events on their stream (every gemm_bf16 launch, tagged with
// its epilogue kind, and whatever the sequencing code opens and closes itself, tags >= LR_TAG_ATTN_FWD).
int launch_timer_begin(int max_launches);
int launch_timer_open(int tag, int M, int N, int K, int batch, double flops, hipStream_t st);   // -1: not recording
void launch_timer_close(int slot, hipStream_t st);
int launch_timer_end(lr_launch_record* out, int max_records, int* n_records);

// ---- streaming kernels (stream_kernels.hip) ---------------------------------------------------
hipError_t k_rms_stat(const void* x, int64_t ldx, float* stat, int64_t T, int64_t d, int dt, hipStream_t);
hipError_t k_rmsnorm_apply(const void* x, int64_t ldx, const void* gamma, const float* stat, float eps,
                           void* xhat, int64_t ldo, int64_t T, int64_t d, int dt, hipStream_t);
// out[t, j] = h[t, j] * rsqrt(stat[t] / d_total + eps), j < n  (the global rescale of a sharded projection)
hipError_t k_row_rms_scale(const void* h, int64_t ldh, const float* stat, int64_t d_total, float eps, void* out,
                           int64_t ldo, int64_t T, int64_t n, int dt, hipStream_t);
int64_t k_rmsnorm_bwd_parts(int64_t T);
hipError_t k_rmsnorm_bwd(const void* x, int64_t ldx, const void* gamma, const float* stat, float eps,
                         const void* dxhat, int64_t lddxh, const void* dres, int64_t lddres, void* dx,
                         int64_t lddx, float* dgamma_part, int64_t T, int64_t d, int dt, hipStream_t);
hipError_t k_act_fwd(const void* z, int64_t ldz, void* a, int64_t lda, int64_t T, int64_t n, int act,
                     int dt, hipStream_t);
hipError_t k_swiglu_fwd(const void* g, const void* u, void* m, int64_t ld, int64_t T, int64_t f, int dt,
                        hipStream_t);
// rotary embedding in place on x[rows, ld] (bf16, H heads of 128 from column 0, position = row % S);
// cos / sin tables [S, 64] fp32; inverse = the transposed rotation
hipError_t k_rope128_bf16(void* x, int64_t ld, const float* cos_tab, const float* sin_tab, int64_t rows, int S, int H,
                          int inverse, hipStream_t);
// out = a + b, dense bf16 [T, n] (n a multiple of 8)
hipError_t k_add2_bf16(const void* a, const void* b, void* out, int64_t T, int64_t n, hipStream_t);
hipError_t k_swiglu_bwd(const void* g, const void* u, const void* dm, void* dg, void* du, int64_t ld,
                        int64_t T, int64_t f, int dt, hipStream_t);
// out[r, c] = in[c, r] for in[rows, cols] (ld_in) -> out[cols, rows] (ld_out)
hipError_t k_transpose(const void* in, int64_t ld_in, void* out, int64_t ld_out, int64_t rows,
                       int64_t cols, int dt, hipStream_t);
// out[m] = sum_p part[m, p], p < nparts
hipError_t k_rowsum_parts(const float* part, int64_t ld, int nparts, float* out, int64_t M, hipStream_t);
// out[m] = sum_n a[m,n] * b[m,n]
hipError_t k_rowdot(const void* a, int64_t lda, const void* b, int64_t ldb, float* out, int64_t M,
                    int64_t N, int dt, hipStream_t);
// wout[n, k] = w[n, k] * gamma[k]
hipError_t k_scale_cols(const void* w, const void* gamma, void* wout, int64_t rows, int64_t cols, int dt,
                        hipStream_t);
// Sum `nsplit` fp32 partials [nsplit][count] (batch-major outside) and write / accumulate into dw.
//   dw[i] (+)= colscale[i % cols] * sum_s part[s][i]      (colscale optional)
// With wg_for_dgamma (the un-scaled weight) also emits dgamma_part[row_block][cols] partial sums of
// w * sum_s part (dgamma = sum over all rows).
hipError_t k_wgrad_finish(const float* part, int nsplit, int64_t rows, int64_t cols, void* dw,
                          const void* colscale, const void* w_for_dgamma, float* dgamma_part,
                          int accumulate, int dt, int out_dt, hipStream_t);
int64_t k_wgrad_dgamma_parts(int64_t rows);
// out[c] (+)= sum_p part[p, c]; out has dtype out_dt
hipError_t k_colsum_parts(const float* part, int64_t nparts, int64_t cols, void* out, int accumulate,
                          int out_dt, hipStream_t);

// ---- attention (attention.hip) ---------------------------------------------------------------
hipError_t attention_fwd_bf16(const void* q, const void* k, const void* v, void* o, float* lse, int64_t ld,
                              int B, int S, int H, int hd, int causal, hipStream_t);
size_t attention_bwd_ws_bytes(int B, int S, int H, int hd);
hipError_t attention_bwd_bf16(const void* q, const void* k, const void* v, const void* o, const void* dout,
                              const float* lse, void* dq, void* dk, void* dv, int64_t ld, int B, int S, int H,
                              int hd, int causal, void* ws, hipStream_t);
// grouped-query form: Hkv key / value heads (k, v, dk, dv rows of ldkv elements), H % Hkv == 0
hipError_t attention_gqa_fwd_bf16(const void* q, const void* k, const void* v, void* o, float* lse, int64_t ld,
                                  int64_t ldkv, int B, int S, int H, int Hkv, int hd, int causal, hipStream_t);
size_t attention_gqa_bwd_ws_bytes(int B, int S, int H, int Hkv, int hd);
hipError_t attention_gqa_bwd_bf16(const void* q, const void* k, const void* v, const void* o, const void* dout,
                                  const float* lse, void* dq, void* dk, void* dv, int64_t ld, int64_t ldkv, int B,
                                  int S, int H, int Hkv, int hd, int causal, void* ws, hipStream_t);

// ---------------------------------------------------------------------------------------------
// device helpers
// ---------------------------------------------------------------------------------------------
typedef __bf16 bf16_t;
typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef __bf16 bf16x4 __attribute__((ext_vector_type(4)));
typedef float f32x4 __attribute__((ext_vector_type(4)));
typedef float f32x16 __attribute__((ext_vector_type(16)));

__device__ __forceinline__ float bf16_bits_to_f32(uint32_t lo16) { return __uint_as_float(lo16 << 16); }
typedef __bf16 bf16x2 __attribute__((ext_vector_type(2)));
typedef float f32x2 __attribute__((ext_vector_type(2)));
// fp32 -> bf16, round to nearest even, through the hardware conversion (v_cvt_pk_bf16_f32)
__device__ __forceinline__ uint32_t pack_bf16x2(float lo, float hi) {
  f32x2 v = {lo, hi};
  return __builtin_bit_cast(uint32_t, __builtin_convertvector(v, bf16x2));
}
__device__ __forceinline__ uint32_t f32_to_bf16_bits(float f) { return pack_bf16x2(f, 0.f) & 0xffffu; }
// the value a float has once stored as bf16 (round to nearest even) and read back
__device__ __forceinline__ float bf16_round_f(float f) { return bf16_bits_to_f32(f32_to_bf16_bits(f)); }
__device__ __forceinline__ void unpack8(const uint4& q, float* v) {
  v[0] = __uint_as_float(q.x << 16); v[1] = __uint_as_float(q.x & 0xffff0000u);
  v[2] = __uint_as_float(q.y << 16); v[3] = __uint_as_float(q.y & 0xffff0000u);
  v[4] = __uint_as_float(q.z << 16); v[5] = __uint_as_float(q.z & 0xffff0000u);
  v[6] = __uint_as_float(q.w << 16); v[7] = __uint_as_float(q.w & 0xffff0000u);
}
__device__ __forceinline__ uint4 pack8(const float* v) {
  uint4 q;
  q.x = pack_bf16x2(v[0], v[1]); q.y = pack_bf16x2(v[2], v[3]);
  q.z = pack_bf16x2(v[4], v[5]); q.w = pack_bf16x2(v[6], v[7]);
  return q;
}
// 1 / (1 + e^-z) with the hardware reciprocal (1 ulp) instead of an IEEE division, which costs ten
// instructions per element: in the GEMM epilogues that apply sigma or the SwiGLU gate these divisions
// were 40 % of all instructions.
__device__ __forceinline__ float logistic_f(float z) { return __builtin_amdgcn_rcpf(1.f + __expf(-z)); }
__device__ __forceinline__ float silu_f(float z) { return z * logistic_f(z); }
__device__ __forceinline__ float silu_prime_f(float z) {
  float s = logistic_f(z);
  return s * (1.f + z * (1.f - s));
}
__device__ __forceinline__ float act_f(float z, int act) { return act == LR_ACT_SILU ? silu_f(z) : z; }
__device__ __forceinline__ float act_prime_f(float z, int act) { return act == LR_ACT_SILU ? silu_prime_f(z) : 1.f; }

}  // namespace lrb
