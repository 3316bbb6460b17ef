// Memory-bound kernels: per-token statistics, RMSNorm apply / backward, sigma at rank r, SwiGLU
// forward / backward, transposes and the small reductions that finish weight gradients.
// bf16 tensors move as 16-byte vectors (8 elements per lane, 1 KB per wavefront instruction);
// fp32 tensors (precision path, arbitrary sizes) move element-wise.  All arithmetic is fp32.
// The forms the block uses (dense bf16 tensors, rows of at most 4096 elements) reach memory through
// buffer resources sized to what a workgroup or a row owns, so that they need no bounds branches: with
// a test per vector the compiler puts a full memory wait inside every branch and a lane's loads go one
// round trip after the other.  Also here: the rotary embedding and the LaX variant's rank-r sum.
#include "epilogue.h"

namespace lrb {
namespace {

template <int DT> struct St;
template <> struct St<LR_F32> { using T = float; static constexpr int NV = 1; };
template <> struct St<LR_BF16> { using T = bf16_t; static constexpr int NV = 8; };

__device__ __forceinline__ float wave_sum(float v) {
#pragma unroll
  for (int o = 32; o >= 1; o >>= 1) v += __shfl_xor(v, o);
  return v;
}

// ---- S[t] = sum_j x[t,j]^2 : one wavefront per row ---------------------------------------------
// (Many short wavefronts read faster here than fewer wavefronts with more rows or vectors each.)
template <int DT>
__global__ __launch_bounds__(256) void rms_stat_kernel(const void* x, int64_t ldx, float* stat, int64_t T, int64_t d) {
  using S = St<DT>;
  using IO = VecIO<typename S::T, S::NV>;
  const int lane = threadIdx.x & 63;
  const int64_t row = (int64_t)blockIdx.x * 4 + (threadIdx.x >> 6);
  if (row >= T) return;
  float s = 0.f;
  // four vectors per lane in flight before the arithmetic
  constexpr int U = 4;
  for (int64_t c0 = 0; c0 < d; c0 += U * 64 * S::NV) {
    float v[U][S::NV];
#pragma unroll
    for (int j = 0; j < U; j++) {
      const int64_t c = c0 + (j * 64 + lane) * S::NV;
      if (c < d) IO::load_nt(x, row * ldx + c, v[j]);
    }
#pragma unroll
    for (int j = 0; j < U; j++) {
      const int64_t c = c0 + (j * 64 + lane) * S::NV;
      if (c < d) {
#pragma unroll
        for (int i = 0; i < S::NV; i++) s = fmaf(v[j][i], v[j][i], s);
      }
    }
  }
  s = wave_sum(s);
  if (lane == 0) stat[row] = s;
}

template <int DT>
__global__ __launch_bounds__(256) void rmsnorm_apply_kernel(const void* x, int64_t ldx, const void* gamma,
                                                            const float* stat, float eps, void* out, int64_t ldo,
                                                            int64_t T, int64_t d, int64_t d_div) {
  // d: row width; d_div: the width the statistic was taken over (differs from d when the rows are the
  // summed partial products of a feature-sharded projection); gamma may be null (no scale)
  using S = St<DT>;
  using IO = VecIO<typename S::T, S::NV>;
  const int lane = threadIdx.x & 63;
  const int64_t row = (int64_t)blockIdx.x * 4 + (threadIdx.x >> 6);
  if (row >= T) return;
  const float rho = rsqrtf(stat[row] / (float)d_div + eps);
  for (int64_t c = lane * S::NV; c < d; c += 64 * S::NV) {
    float v[S::NV], g[S::NV];
    IO::load(x, row * ldx + c, v);
#pragma unroll
    for (int i = 0; i < S::NV; i++) g[i] = 1.f;
    if (gamma) IO::load(gamma, c, g);
#pragma unroll
    for (int i = 0; i < S::NV; i++) v[i] = v[i] * g[i] * rho;
    IO::store(out, row * ldo + c, v);
  }
}

// ---- reverse mode of RMSNorm ----------------------------------------------------------------------
// One workgroup owns RB consecutive rows.  Phase A: each wavefront reduces c = mean_j(dn*n) for its
// rows.  Phase B: column super-chunks of 64*NV*IT columns; each lane keeps the column partial sums
// of dxhat*n for its columns across the workgroup's rows, writes dx, and the four wavefronts'
// partials are added through LDS into dgamma_part[blockIdx][.].
constexpr int NB_RB = 64;
constexpr int NB_IT = 4;

template <int DT>
__global__ __launch_bounds__(256) void rmsnorm_bwd_kernel(const void* x, int64_t ldx, const void* gamma,
                                                          const float* stat, float eps, const void* dxh,
                                                          int64_t lddxh, const void* dres, int64_t lddres, void* dx,
                                                          int64_t lddx, float* dgpart, int64_t T, int64_t d) {
  using S = St<DT>;
  using IO = VecIO<typename S::T, S::NV>;
  constexpr int NV = S::NV;
  __shared__ float sc[NB_RB];
  __shared__ float sred[4][64 * NV];  // one it-slice of a super-chunk at a time
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int64_t row0 = (int64_t)blockIdx.x * NB_RB;
  const float inv_d = 1.f / (float)d;
  for (int r = wave; r < NB_RB; r += 4) {
    const int64_t row = row0 + r;
    if (row >= T) break;
    const float rho = rsqrtf(stat[row] * inv_d + eps);
    float s = 0.f;
    for (int64_t c = lane * NV; c < d; c += 64 * NV) {
      float xv[NV], gv[NV], dv[NV];
      IO::load(x, row * ldx + c, xv);
      IO::load(gamma, c, gv);
      IO::load(dxh, row * lddxh + c, dv);
#pragma unroll
      for (int i = 0; i < NV; i++) s = fmaf(dv[i] * gv[i], xv[i] * rho, s);
    }
    s = wave_sum(s);
    if (lane == 0) sc[r] = s * inv_d;
  }
  __syncthreads();
  constexpr int SUPER = 64 * NV * NB_IT;
  for (int64_t cb = 0; cb < d; cb += SUPER) {
    float acc[NB_IT][NV];
#pragma unroll
    for (int it = 0; it < NB_IT; it++)
#pragma unroll
      for (int i = 0; i < NV; i++) acc[it][i] = 0.f;
    for (int r = wave; r < NB_RB; r += 4) {
      const int64_t row = row0 + r;
      if (row >= T) break;
      const float rho = rsqrtf(stat[row] * inv_d + eps);
      const float c = sc[r];
#pragma unroll
      for (int it = 0; it < NB_IT; it++) {
        const int64_t col = cb + (int64_t)it * 64 * NV + lane * NV;
        if (col < d) {
          float xv[NV], gv[NV], dv[NV], o[NV];
          IO::load(x, row * ldx + col, xv);
          IO::load(gamma, col, gv);
          IO::load(dxh, row * lddxh + col, dv);
#pragma unroll
          for (int i = 0; i < NV; i++) {
            const float n = xv[i] * rho;
            o[i] = (dv[i] * gv[i] - n * c) * rho;
            acc[it][i] = fmaf(dv[i], n, acc[it][i]);
          }
          if (dres) {
            float rv[NV];
            IO::load(dres, row * lddres + col, rv);
#pragma unroll
            for (int i = 0; i < NV; i++) o[i] += rv[i];
          }
          IO::store(dx, row * lddx + col, o);
        }
      }
    }
    // add the four wavefronts' column partials, one it-slice at a time
#pragma unroll
    for (int it = 0; it < NB_IT; it++) {
#pragma unroll
      for (int i = 0; i < NV; i++) sred[wave][lane * NV + i] = acc[it][i];
      __syncthreads();
      for (int e = threadIdx.x; e < 64 * NV; e += 256) {
        const int64_t col = cb + (int64_t)it * 64 * NV + e;
        if (col < d) dgpart[(int64_t)blockIdx.x * d + col] = sred[0][e] + sred[1][e] + sred[2][e] + sred[3][e];
      }
      __syncthreads();
    }
  }
}

// bf16, d <= 512 * NIT: a wavefront holds a whole row of x, dxhat and the residual gradient in
// registers (packed, as loaded), so every tensor is read exactly once: reduce c, then write dx and add
// the row into the lane's column partials of dgamma.  Same partial layout as the kernel above; the rows
// of a workgroup are interleaved with those of the others, so that the workgroups in flight together
// sweep one contiguous window of each tensor.
// All global accesses of the row loop go through buffer resources that span exactly one row (and
// nothing, for an absent residual): columns past d read as zeros and are dropped on store without a
// branch, so the loop body is straight-line code and all of a row's loads are in flight together.  (With a
// bounds test per vector the compiler had put a full wait for memory between the vectors of the
// second phase: 4.5 instead of the rate below.)
template <int NIT>
__global__ __launch_bounds__(256, 2) void rmsnorm_bwd_row_kernel(const uint16_t* x, int64_t ldx, const uint16_t* gamma,
                                                              const float* stat, float eps, const uint16_t* dxh,
                                                              int64_t lddxh, const uint16_t* dres, int64_t lddres,
                                                              uint16_t* dx, int64_t lddx, float* dgpart, int64_t T,
                                                              int64_t d, int rows_per_wg, int64_t nparts) {
  // LDS: gamma (staged once per workgroup: re-reading it here costs no registers and, unlike a global
  // re-read, does not queue behind the row's stores), then each wavefront's column partials of dgamma
  // (kept here rather than in 64 registers per lane, which the row data needs)
  extern __shared__ __align__(16) unsigned char rn_smem[];
  uint4* sgam = reinterpret_cast<uint4*>(rn_smem);                           // [NIT * 64]
  float4* sacc = reinterpret_cast<float4*>(rn_smem + NIT * 64 * 16);          // [4][NIT * 64][2]
  const int lane = threadIdx.x & 63, wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
  const float inv_d = 1.f / (float)d;
  const uint32_t row_bytes = (uint32_t)d * 2u;
  // cache policy of the streamed tensors: non-temporal loads; the stores with the default policy (measured:
  // 5.8 against 5.6 TB/s with non-temporal stores, and the reverse for the loads)
  constexpr int NT_ = 2, ST_ = 0;
  auto row_rsrc = [&](const uint16_t* base, int64_t row, int64_t ld) {
    return __builtin_amdgcn_make_buffer_rsrc((void*)(base ? base + row * ld : nullptr), 0, base ? row_bytes : 0u,
                                             0x00020000);
  };
  for (int e = threadIdx.x; e < NIT * 64; e += 256)
    sgam[e] = (int64_t)e * 8 < d ? *reinterpret_cast<const uint4*>(gamma + (int64_t)e * 8) : make_uint4(0, 0, 0, 0);
  float4* myacc = sacc + (wave * NIT * 64 + lane) * 2;      // + it * 128: this lane's 8 columns of slice it
#pragma unroll
  for (int it = 0; it < NIT; it++) {
    myacc[it * 128] = make_float4(0.f, 0.f, 0.f, 0.f);
    myacc[it * 128 + 1] = make_float4(0.f, 0.f, 0.f, 0.f);
  }
  __syncthreads();
  auto u4 = [](const u32x4_t& t) { return make_uint4(t.x, t.y, t.z, t.w); };
  for (int r = 0; r < rows_per_wg / 4; r++) {
    const int64_t row = ((int64_t)r * gridDim.x + blockIdx.x) * 4 + wave;
    if (row >= T) break;
    const float rho = rsqrtf(stat[row] * inv_d + eps);
    const __amdgpu_buffer_rsrc_t rsX = row_rsrc(x, row, ldx), rsD = row_rsrc(dxh, row, lddxh),
                                 rsR = row_rsrc(dres, row, lddres), rsO = row_rsrc(dx, row, lddx);
    u32x4_t xq[NIT], dq[NIT], rq[NIT];
#pragma unroll
    for (int it = 0; it < NIT; it++) {
      const int off = (it * 64 + lane) * 16;
      xq[it] = __builtin_amdgcn_raw_buffer_load_b128(rsX, off, 0, NT_);
      dq[it] = __builtin_amdgcn_raw_buffer_load_b128(rsD, off, 0, NT_);
    }
#pragma unroll
    for (int it = 0; it < NIT; it++) rq[it] = __builtin_amdgcn_raw_buffer_load_b128(rsR, (it * 64 + lane) * 16, 0, NT_);
    float s = 0.f;
#pragma unroll
    for (int it = 0; it < NIT; it++) {
      float xv[8], gv[8], dv[8];
      unpack8(u4(xq[it]), xv); unpack8(sgam[it * 64 + lane], gv); unpack8(u4(dq[it]), dv);
#pragma unroll
      for (int i = 0; i < 8; i++) s = fmaf(dv[i] * gv[i], xv[i] * rho, s);
      // keeps the compiler from fetching and unpacking every slice's gamma at once (registers)
      if (it % 2 == 1) __builtin_amdgcn_sched_barrier(0);
    }
    const float c = wave_sum(s) * inv_d;
#pragma unroll
    for (int it = 0; it < NIT; it++) {
      float xv[8], gv[8], dv[8], rv[8], o[8];
      if (it % 2 == 0) __builtin_amdgcn_sched_barrier(0);
      unpack8(u4(xq[it]), xv); unpack8(sgam[it * 64 + lane], gv); unpack8(u4(dq[it]), dv); unpack8(u4(rq[it]), rv);
      float4 a0 = myacc[it * 128], a1 = myacc[it * 128 + 1];
      float a[8] = {a0.x, a0.y, a0.z, a0.w, a1.x, a1.y, a1.z, a1.w};
#pragma unroll
      for (int i = 0; i < 8; i++) {
        const float n = xv[i] * rho;
        o[i] = (dv[i] * gv[i] - n * c) * rho + rv[i];
        a[i] = fmaf(dv[i], n, a[i]);
      }
      myacc[it * 128] = make_float4(a[0], a[1], a[2], a[3]);
      myacc[it * 128 + 1] = make_float4(a[4], a[5], a[6], a[7]);
      const uint4 ov = pack8(o);
      __builtin_amdgcn_raw_buffer_store_b128(u32x4_t{ov.x, ov.y, ov.z, ov.w}, rsO, (it * 64 + lane) * 16, 0, ST_);
    }
  }
  // add the four wavefronts' column partials
  __syncthreads();
  const float* fa = reinterpret_cast<const float*>(sacc);
  for (int e = threadIdx.x; e < NIT * 512; e += 256) {
    if (e < d) {
      dgpart[(int64_t)blockIdx.x * d + e] = fa[e] + fa[NIT * 512 + e] + fa[2 * NIT * 512 + e] + fa[3 * NIT * 512 + e];
      // the caller adds up nparts rows of partials: those that no workgroup owns hold zeros
      for (int64_t pr = (int64_t)blockIdx.x + gridDim.x; pr < nparts; pr += gridDim.x) dgpart[pr * d + e] = 0.f;
    }
  }
}
constexpr int RN_ROW_LDS = 8 * 64 * 16 + 4 * 8 * 512 * 4;   // rmsnorm_bwd_row_kernel<8>: gamma + four partial sets

// ---- elementwise on [T, n] with leading dimensions -------------------------------------------
// Each workgroup owns one contiguous run of EW_U x 256 vectors and issues all of its loads before the
// arithmetic; loads and stores are non-temporal.  (Measured on this chip: 6.3 TB/s for a two-input,
// one-output kernel, against 5.2 TB/s for a grid-stride loop with one vector in flight per lane.)
constexpr int EW_U = 4;
template <int DT>
__global__ __launch_bounds__(256) void act_fwd_kernel(const void* z, int64_t ldz, void* a, int64_t lda, int64_t T,
                                                      int64_t n, int act) {
  using S = St<DT>;
  using IO = VecIO<typename S::T, S::NV>;
  const int64_t cpr = n / S::NV;  // vectors per row
  const int64_t total = T * cpr;
  const int64_t base = (int64_t)blockIdx.x * (256 * EW_U) + threadIdx.x;
  float v[EW_U][S::NV];
#pragma unroll
  for (int j = 0; j < EW_U; j++) {
    const int64_t i = base + j * 256;
    if (i < total) IO::load_nt(z, (i / cpr) * ldz + (i % cpr) * S::NV, v[j]);
  }
#pragma unroll
  for (int j = 0; j < EW_U; j++) {
    const int64_t i = base + j * 256;
    if (i < total) {
#pragma unroll
      for (int k = 0; k < S::NV; k++) v[j][k] = act_f(v[j][k], act);
      IO::store_nt(a, (i / cpr) * lda + (i % cpr) * S::NV, v[j]);
    }
  }
}

template <int DT>
__global__ __launch_bounds__(256) void swiglu_fwd_kernel(const void* g, const void* u, void* m, int64_t ld, int64_t T,
                                                         int64_t f) {
  using S = St<DT>;
  using IO = VecIO<typename S::T, S::NV>;
  const int64_t cpr = f / S::NV, total = T * cpr;
  const int64_t base = (int64_t)blockIdx.x * (256 * EW_U) + threadIdx.x;
  float gv[EW_U][S::NV], uv[EW_U][S::NV];
#pragma unroll
  for (int j = 0; j < EW_U; j++) {
    const int64_t i = base + j * 256;
    if (i < total) {
      const int64_t off = (i / cpr) * ld + (i % cpr) * S::NV;
      IO::load_nt(g, off, gv[j]);
      IO::load_nt(u, off, uv[j]);
    }
  }
#pragma unroll
  for (int j = 0; j < EW_U; j++) {
    const int64_t i = base + j * 256;
    if (i < total) {
#pragma unroll
      for (int k = 0; k < S::NV; k++) gv[j][k] = silu_f(gv[j][k]) * uv[j][k];
      IO::store_nt(m, (i / cpr) * ld + (i % cpr) * S::NV, gv[j]);
    }
  }
}

constexpr int EW_U3 = 2;   // three inputs, two outputs: fewer vectors per lane keep the register count down
template <int DT>
__global__ __launch_bounds__(256) void swiglu_bwd_kernel(const void* g, const void* u, const void* dm, void* dg,
                                                         void* du, int64_t ld, int64_t T, int64_t f) {
  using S = St<DT>;
  using IO = VecIO<typename S::T, S::NV>;
  const int64_t cpr = f / S::NV, total = T * cpr;
  const int64_t base = (int64_t)blockIdx.x * (256 * EW_U3) + threadIdx.x;
  float gv[EW_U3][S::NV], uv[EW_U3][S::NV], dv[EW_U3][S::NV];
#pragma unroll
  for (int j = 0; j < EW_U3; j++) {
    const int64_t i = base + j * 256;
    if (i < total) {
      const int64_t off = (i / cpr) * ld + (i % cpr) * S::NV;
      IO::load_nt(g, off, gv[j]);
      IO::load_nt(u, off, uv[j]);
      IO::load_nt(dm, off, dv[j]);
    }
  }
#pragma unroll
  for (int j = 0; j < EW_U3; j++) {
    const int64_t i = base + j * 256;
    if (i < total) {
      const int64_t off = (i / cpr) * ld + (i % cpr) * S::NV;
      float o1[S::NV], o2[S::NV];
#pragma unroll
      for (int k = 0; k < S::NV; k++) {
        o1[k] = dv[j][k] * uv[j][k] * silu_prime_f(gv[j][k]);
        o2[k] = dv[j][k] * silu_f(gv[j][k]);
      }
      IO::store_nt(dg, off, o1);
      IO::store_nt(du, off, o2);
    }
  }
}

// ---- the same three maps for dense bf16 tensors (row pitch = row length), the form the block uses ------
// The tensor is one flat array; a workgroup owns the 256 * U vectors from byte blockIdx.x * CHUNK on and
// reaches them through a buffer resource that starts there and ends at the chunk's or the tensor's end,
// whichever comes first: the tail needs no bounds test, the body is straight-line code, and all loads of
// a lane are in flight before the first is used.  (With a test per vector the compiler waits for each
// vector's load inside its branch, one memory round trip after the other.)
constexpr int DENSE_U = 4, DENSE_U3 = 4;   // vectors per lane: one / two inputs, three inputs (measured best)
constexpr int NT_POLICY = 2;   // buffer cache policy: non-temporal, loads and stores (for these kernels default-policy
                               // stores measured 4 - 5 % slower, unlike the row kernel above)
__device__ __forceinline__ __amdgpu_buffer_rsrc_t chunk_rsrc(const void* p, int64_t total_bytes, int64_t chunk_bytes) {
  const int64_t start = (int64_t)blockIdx.x * chunk_bytes;
  const int64_t left = total_bytes - start;
  return __builtin_amdgcn_make_buffer_rsrc((void*)((const char*)p + start), 0,
                                           (uint32_t)(left < chunk_bytes ? left : chunk_bytes), 0x00020000);
}
__device__ __forceinline__ void unpack8v(const u32x4_t& t, float* v) { unpack8(make_uint4(t.x, t.y, t.z, t.w), v); }
__device__ __forceinline__ u32x4_t pack8v(const float* v) {
  const uint4 q = pack8(v);
  return u32x4_t{q.x, q.y, q.z, q.w};
}

template <int U>
__global__ __launch_bounds__(256) void act_fwd_dense_kernel(const void* z, void* a, int64_t total_bytes, int act) {
  constexpr int64_t CHUNK = 256 * U * 16;
  const __amdgpu_buffer_rsrc_t rz = chunk_rsrc(z, total_bytes, CHUNK), ra = chunk_rsrc(a, total_bytes, CHUNK);
  u32x4_t q[U];
#pragma unroll
  for (int j = 0; j < U; j++) q[j] = __builtin_amdgcn_raw_buffer_load_b128(rz, (j * 256 + (int)threadIdx.x) * 16, 0, NT_POLICY);
#pragma unroll
  for (int j = 0; j < U; j++) {
    float v[8];
    unpack8v(q[j], v);
#pragma unroll
    for (int k = 0; k < 8; k++) v[k] = act_f(v[k], act);
    __builtin_amdgcn_raw_buffer_store_b128(pack8v(v), ra, (j * 256 + (int)threadIdx.x) * 16, 0, NT_POLICY);
  }
}

// out = a + b: the LaX variant's rank-r activation h_i + h_{i-1}, rebuilt in the backward
template <int U>
__global__ __launch_bounds__(256) void add2_dense_kernel(const void* a, const void* b, void* out, int64_t total_bytes) {
  constexpr int64_t CHUNK = 256 * U * 16;
  const __amdgpu_buffer_rsrc_t ra = chunk_rsrc(a, total_bytes, CHUNK), rb = chunk_rsrc(b, total_bytes, CHUNK),
                               ro = chunk_rsrc(out, total_bytes, CHUNK);
  u32x4_t aq[U], bq[U];
#pragma unroll
  for (int j = 0; j < U; j++) {
    const int off = (j * 256 + (int)threadIdx.x) * 16;
    aq[j] = __builtin_amdgcn_raw_buffer_load_b128(ra, off, 0, NT_POLICY);
    bq[j] = __builtin_amdgcn_raw_buffer_load_b128(rb, off, 0, NT_POLICY);
  }
#pragma unroll
  for (int j = 0; j < U; j++) {
    float av[8], bv[8];
    unpack8v(aq[j], av);
    unpack8v(bq[j], bv);
#pragma unroll
    for (int k = 0; k < 8; k++) av[k] += bv[k];
    __builtin_amdgcn_raw_buffer_store_b128(pack8v(av), ro, (j * 256 + (int)threadIdx.x) * 16, 0, NT_POLICY);
  }
}

template <int U>
__global__ __launch_bounds__(256) void swiglu_fwd_dense_kernel(const void* g, const void* u, void* m, int64_t total_bytes) {
  constexpr int64_t CHUNK = 256 * U * 16;
  const __amdgpu_buffer_rsrc_t rg = chunk_rsrc(g, total_bytes, CHUNK), ru = chunk_rsrc(u, total_bytes, CHUNK),
                               rm = chunk_rsrc(m, total_bytes, CHUNK);
  u32x4_t gq[U], uq[U];
#pragma unroll
  for (int j = 0; j < U; j++) {
    const int off = (j * 256 + (int)threadIdx.x) * 16;
    gq[j] = __builtin_amdgcn_raw_buffer_load_b128(rg, off, 0, NT_POLICY);
    uq[j] = __builtin_amdgcn_raw_buffer_load_b128(ru, off, 0, NT_POLICY);
  }
#pragma unroll
  for (int j = 0; j < U; j++) {
    float gv[8], uv[8];
    unpack8v(gq[j], gv);
    unpack8v(uq[j], uv);
#pragma unroll
    for (int k = 0; k < 8; k++) gv[k] = silu_f(gv[k]) * uv[k];
    __builtin_amdgcn_raw_buffer_store_b128(pack8v(gv), rm, (j * 256 + (int)threadIdx.x) * 16, 0, NT_POLICY);
  }
}

template <int U>
__global__ __launch_bounds__(256) void swiglu_bwd_dense_kernel(const void* g, const void* u, const void* dm, void* dg,
                                                               void* du, int64_t total_bytes) {
  constexpr int64_t CHUNK = 256 * U * 16;
  const __amdgpu_buffer_rsrc_t rg = chunk_rsrc(g, total_bytes, CHUNK), ru = chunk_rsrc(u, total_bytes, CHUNK),
                               rd = chunk_rsrc(dm, total_bytes, CHUNK), rdg = chunk_rsrc(dg, total_bytes, CHUNK),
                               rdu = chunk_rsrc(du, total_bytes, CHUNK);
  u32x4_t gq[U], uq[U], dq[U];
#pragma unroll
  for (int j = 0; j < U; j++) {
    const int off = (j * 256 + (int)threadIdx.x) * 16;
    gq[j] = __builtin_amdgcn_raw_buffer_load_b128(rg, off, 0, NT_POLICY);
    uq[j] = __builtin_amdgcn_raw_buffer_load_b128(ru, off, 0, NT_POLICY);
    dq[j] = __builtin_amdgcn_raw_buffer_load_b128(rd, off, 0, NT_POLICY);
  }
#pragma unroll
  for (int j = 0; j < U; j++) {
    float gv[8], uv[8], dv[8], o1[8], o2[8];
    unpack8v(gq[j], gv);
    unpack8v(uq[j], uv);
    unpack8v(dq[j], dv);
#pragma unroll
    for (int k = 0; k < 8; k++) {
      o1[k] = dv[k] * uv[k] * silu_prime_f(gv[k]);
      o2[k] = dv[k] * silu_f(gv[k]);
    }
    const int off = (j * 256 + (int)threadIdx.x) * 16;
    __builtin_amdgcn_raw_buffer_store_b128(pack8v(o1), rdg, off, 0, NT_POLICY);
    __builtin_amdgcn_raw_buffer_store_b128(pack8v(o2), rdu, off, 0, NT_POLICY);
  }
}

// ---- rotary position embedding, in place, heads of 128 (rotate-half form) -----------------------
// x[rows, ld], head h in columns 128 h ..; the pair (v[i], v[i + 64]) of the row at position p = row % S
// is turned by the angle whose cosine and sine the caller tabulated as cs[p, i], sn[p, i] ([S, 64] fp32).
// One lane owns 8 consecutive i of one head: two 16-byte loads, two 16-byte stores.  sgn = -1 applies the
// transpose (the backward of the rotation).
__global__ __launch_bounds__(256) void rope128_kernel(uint16_t* x, int64_t ld, const float* __restrict__ cs,
                                                      const float* __restrict__ sn, int64_t rows, int S, int H, float sgn) {
  const int64_t idx = (int64_t)blockIdx.x * 256 + threadIdx.x;
  if (idx >= rows * H * 8) return;
  const int c8 = (int)(idx & 7) * 8;
  const int64_t rh = idx >> 3;
  const int h = (int)(rh % H);
  const int64_t row = rh / H;
  const int p = (int)(row % S);
  uint16_t* ptr = x + row * ld + (int64_t)h * 128 + c8;
  float lo[8], hi[8], c[8], s[8];
  unpack8(*reinterpret_cast<const uint4*>(ptr), lo);
  unpack8(*reinterpret_cast<const uint4*>(ptr + 64), hi);
  const float4* cp = reinterpret_cast<const float4*>(cs + (int64_t)p * 64 + c8);
  const float4* sp = reinterpret_cast<const float4*>(sn + (int64_t)p * 64 + c8);
  const float4 c0 = cp[0], c1 = cp[1], s0 = sp[0], s1 = sp[1];
  c[0] = c0.x; c[1] = c0.y; c[2] = c0.z; c[3] = c0.w; c[4] = c1.x; c[5] = c1.y; c[6] = c1.z; c[7] = c1.w;
  s[0] = s0.x; s[1] = s0.y; s[2] = s0.z; s[3] = s0.w; s[4] = s1.x; s[5] = s1.y; s[6] = s1.z; s[7] = s1.w;
  float olo[8], ohi[8];
#pragma unroll
  for (int i = 0; i < 8; i++) {
    const float si = s[i] * sgn;
    olo[i] = lo[i] * c[i] - hi[i] * si;
    ohi[i] = hi[i] * c[i] + lo[i] * si;
  }
  *reinterpret_cast<uint4*>(ptr) = pack8(olo);
  *reinterpret_cast<uint4*>(ptr + 64) = pack8(ohi);
}

// ---- transpose: out[c, r] = in[r, c]; 64x64 tiles through LDS.  Output columns rows..pad_to-1
// are written as zeros, so a transposed activation can serve as a k-contiguous GEMM operand whose
// k extent is rounded up to the 16-byte vector.
template <typename E>
__global__ __launch_bounds__(256) void transpose_kernel(const E* in, int64_t ld_in, E* out, int64_t ld_out,
                                                        int64_t rows, int64_t cols, int64_t pad_to) {
  __shared__ E tile[64][64 + 2];
  const int64_t r0 = (int64_t)blockIdx.y * 64, c0 = (int64_t)blockIdx.x * 64;
  const int tx = threadIdx.x & 63, ty = threadIdx.x >> 6;
  for (int i = ty; i < 64; i += 4) {
    const int64_t r = r0 + i, c = c0 + tx;
    if (r < rows && c < cols) tile[i][tx] = in[r * ld_in + c];
  }
  __syncthreads();
  for (int i = ty; i < 64; i += 4) {
    const int64_t c = c0 + i, r = r0 + tx;
    if (c < cols) {
      if (r < rows) out[c * ld_out + r] = tile[tx][i];
      else if (r < pad_to) out[c * ld_out + r] = (E)0;
    }
  }
}

// 16-bit elements, all extents and pitches multiples of 8: global accesses are 16-byte vectors on both
// sides (a 2-byte-per-lane access moves 128 bytes per wavefront instruction, a 16-byte one 1 KB); the
// element shuffle happens between LDS and registers.  Tile: 64 input rows x 64 input columns.
__global__ __launch_bounds__(256) void transpose16_vec_kernel(const uint16_t* in, int64_t ld_in, uint16_t* out,
                                                              int64_t ld_out, int64_t rows, int64_t cols, int64_t pad_to) {
  __shared__ uint16_t tile[64][64 + 8];   // pitch 144 bytes: 16-byte aligned rows, column walks spread over banks
  const int64_t r0 = (int64_t)blockIdx.y * 64, c0 = (int64_t)blockIdx.x * 64;
  const int t = threadIdx.x;
#pragma unroll
  for (int k = 0; k < 2; k++) {           // 64 rows x 8 vectors
    const int v = t + k * 256, i = v >> 3, cv = (v & 7) * 8;
    const int64_t r = r0 + i, c = c0 + cv;
    uint4 q = make_uint4(0, 0, 0, 0);
    if (r < rows && c < cols) q = *reinterpret_cast<const uint4*>(in + r * ld_in + c);
    *reinterpret_cast<uint4*>(&tile[i][cv]) = q;
  }
  __syncthreads();
#pragma unroll
  for (int k = 0; k < 2; k++) {           // 64 output rows (input columns) x 8 vectors of 8 input rows
    const int v = t + k * 256, i = v >> 3, rv = (v & 7) * 8;
    const int64_t c = c0 + i, r = r0 + rv;
    if (c < cols && r < pad_to) {
      uint16_t e[8];
#pragma unroll
      for (int j = 0; j < 8; j++) e[j] = tile[rv + j][i];   // rows past `rows` were staged as zeros
      uint4 q;
      q.x = e[0] | ((uint32_t)e[1] << 16); q.y = e[2] | ((uint32_t)e[3] << 16);
      q.z = e[4] | ((uint32_t)e[5] << 16); q.w = e[6] | ((uint32_t)e[7] << 16);
      *reinterpret_cast<uint4*>(out + c * ld_out + r) = q;
    }
  }
}

__global__ __launch_bounds__(256) void rowsum_parts_kernel(const float* part, int64_t ld, int nparts, float* out,
                                                           int64_t M) {
  const int64_t m = (int64_t)blockIdx.x * 256 + threadIdx.x;
  if (m >= M) return;
  float s = 0.f;
  for (int p = 0; p < nparts; p++) s += part[m * ld + p];
  out[m] = s;
}

template <int DT>
__global__ __launch_bounds__(256) void rowdot_kernel(const void* a, int64_t lda, const void* b, int64_t ldb,
                                                     float* out, int64_t M, int64_t N) {
  using S = St<DT>;
  using IO = VecIO<typename S::T, S::NV>;
  const int lane = threadIdx.x & 63;
  const int64_t row = (int64_t)blockIdx.x * 4 + (threadIdx.x >> 6);
  if (row >= M) return;
  float s = 0.f;
  for (int64_t c = lane * S::NV; c < N; c += 64 * S::NV) {
    float av[S::NV], bv[S::NV];
    IO::load(a, row * lda + c, av);
    IO::load(b, row * ldb + c, bv);
#pragma unroll
    for (int i = 0; i < S::NV; i++) s = fmaf(av[i], bv[i], s);
  }
  s = wave_sum(s);
  if (lane == 0) out[row] = s;
}

template <int DT>
__global__ __launch_bounds__(256) void scale_cols_kernel(const void* w, const void* gamma, void* wout, int64_t rows,
                                                         int64_t cols) {
  using S = St<DT>;
  using IO = VecIO<typename S::T, S::NV>;
  const int64_t cpr = cols / S::NV, total = rows * cpr;
  for (int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x; i < total; i += (int64_t)gridDim.x * 256) {
    const int64_t c = (i % cpr) * S::NV, off = (i / cpr) * cols + c;
    float wv[S::NV], gv[S::NV];
    IO::load(w, off, wv);
    IO::load(gamma, c, gv);
#pragma unroll
    for (int k = 0; k < S::NV; k++) wv[k] *= gv[k];
    IO::store(wout, off, wv);
  }
}

// ---- finish a split-K weight gradient ------------------------------------------------------------
// One thread per 8-column (bf16) / 1-column (fp32) vector of one row: sums the nsplit fp32 partials,
// scales, accumulates, stores.  When dgamma partials are wanted a workgroup covers WF_RB rows of a
// 64-vector column strip: its 4 wavefronts take rows r, r+4, ... and add their column sums through LDS.
constexpr int WF_RB = 32;  // rows per dgamma partial

// NS > 0: the number of split-K partials is known at compile time, so their loads are issued
// together instead of one dependent round trip per partial; NS = 0 takes any count.
template <int DT, typename OT, bool DG, int NS>
__global__ __launch_bounds__(256) void wgrad_finish_kernel(const float* part, int nsplit, int64_t rows, int64_t cols,
                                                           void* dw, const void* colscale, const void* wdg,
                                                           float* dgpart, int accumulate) {
  using S = St<DT>;
  using IO = VecIO<typename S::T, S::NV>;
  using OIO = VecIO<OT, S::NV>;
  using PIO = VecIO<float, S::NV>;
  constexpr int NV = S::NV;
  __shared__ float sred[DG ? 4 * 64 * NV : 1];
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int64_t count = rows * cols;
  float cs[NV], dg[NV];
#pragma unroll
  for (int i = 0; i < NV; i++) { cs[i] = 1.f; dg[i] = 0.f; }
  auto one = [&](int64_t r, int64_t c) {
    float s[NV];
    if constexpr (NS > 0) {
      float t[NS][NV];
#pragma unroll
      for (int sp = 0; sp < NS; sp++) PIO::load(part, (int64_t)sp * count + r * cols + c, t[sp]);
#pragma unroll
      for (int i = 0; i < NV; i++) s[i] = t[0][i];
#pragma unroll
      for (int sp = 1; sp < NS; sp++)
#pragma unroll
        for (int i = 0; i < NV; i++) s[i] += t[sp][i];
    } else {
      PIO::load(part, r * cols + c, s);
      for (int sp = 1; sp < nsplit; sp++) {
        float t[NV];
        PIO::load(part, (int64_t)sp * count + r * cols + c, t);
#pragma unroll
        for (int i = 0; i < NV; i++) s[i] += t[i];
      }
    }
    if constexpr (DG) {
      float wv[NV];
      IO::load(wdg, r * cols + c, wv);
#pragma unroll
      for (int i = 0; i < NV; i++) dg[i] = fmaf(wv[i], s[i], dg[i]);
    }
#pragma unroll
    for (int i = 0; i < NV; i++) s[i] *= cs[i];
    if (accumulate) {
      float old[NV];
      OIO::load(dw, r * cols + c, old);
#pragma unroll
      for (int i = 0; i < NV; i++) s[i] += old[i];
    }
    OIO::store(dw, r * cols + c, s);
  };
  if constexpr (!DG) {
    const int64_t vpr = cols / NV;                               // vectors per row
    const int64_t v = (int64_t)blockIdx.x * 256 + threadIdx.x;
    if (v >= rows * vpr) return;
    const int64_t r = v / vpr, c = (v % vpr) * NV;
    if (colscale) IO::load(colscale, c, cs);
    one(r, c);
  } else {
    const int64_t c = ((int64_t)blockIdx.x * 64 + lane) * NV;
    const bool cok = c < cols;
    if (cok && colscale) IO::load(colscale, c, cs);
    const int64_t rbeg = (int64_t)blockIdx.y * WF_RB, rend = min(rows, rbeg + WF_RB);
    if (cok)
      for (int64_t r = rbeg + wave; r < rend; r += 4) one(r, c);
#pragma unroll
    for (int i = 0; i < NV; i++) sred[(wave * 64 + lane) * NV + i] = dg[i];
    __syncthreads();
    if (wave == 0 && cok) {
#pragma unroll
      for (int i = 0; i < NV; i++)
        dgpart[(int64_t)blockIdx.y * cols + c + i] = sred[lane * NV + i] + sred[(64 + lane) * NV + i] +
                                                     sred[(128 + lane) * NV + i] + sred[(192 + lane) * NV + i];
    }
  }
}

template <typename OT>
__global__ __launch_bounds__(256) void colsum_parts_kernel(const float* part, int64_t nparts, int64_t cols, void* out,
                                                           int accumulate) {
  using IO = VecIO<OT, 1>;
  const int64_t c = (int64_t)blockIdx.x * 256 + threadIdx.x;
  if (c >= cols) return;
  float s = 0.f;
  for (int64_t p = 0; p < nparts; p++) s += part[p * cols + c];
  if (accumulate) {
    float o;
    IO::load(out, c, &o);
    s += o;
  }
  IO::store(out, c, &s);
}

// one workgroup per run of `per` items
inline unsigned grid_chunks(int64_t total, int per) { return (unsigned)((total + per - 1) / per); }
inline int grid1d(int64_t total, int cap = 256 * 32) {
  int64_t g = (total + 255) / 256;
  if (g > cap) g = cap;
  if (g < 1) g = 1;
  return (int)g;
}

}  // namespace

#define DISPATCH_DT(dt, KERNEL, grid, block, st, ...)                                              \
  do {                                                                                             \
    if ((dt) == LR_F32) hipLaunchKernelGGL(KERNEL<LR_F32>, grid, block, 0, st, __VA_ARGS__);       \
    else hipLaunchKernelGGL(KERNEL<LR_BF16>, grid, block, 0, st, __VA_ARGS__);                     \
    return hipGetLastError();                                                                      \
  } while (0)

hipError_t k_rms_stat(const void* x, int64_t ldx, float* stat, int64_t T, int64_t d, int dt, hipStream_t st) {
  if (T <= 0) return hipSuccess;
  DISPATCH_DT(dt, rms_stat_kernel, dim3((T + 3) / 4), dim3(256), st, x, ldx, stat, T, d);
}
hipError_t k_rmsnorm_apply(const void* x, int64_t ldx, const void* gamma, const float* stat, float eps, void* xhat,
                           int64_t ldo, int64_t T, int64_t d, int dt, hipStream_t st) {
  if (T <= 0) return hipSuccess;
  DISPATCH_DT(dt, rmsnorm_apply_kernel, dim3((T + 3) / 4), dim3(256), st, x, ldx, gamma, stat, eps, xhat, ldo, T, d, d);
}
hipError_t k_row_rms_scale(const void* h, int64_t ldh, const float* stat, int64_t d_total, float eps, void* out,
                           int64_t ldo, int64_t T, int64_t n, int dt, hipStream_t st) {
  if (T <= 0) return hipSuccess;
  DISPATCH_DT(dt, rmsnorm_apply_kernel, dim3((T + 3) / 4), dim3(256), st, h, ldh, (const void*)nullptr, stat, eps, out, ldo,
              T, n, d_total);
}
int64_t k_rmsnorm_bwd_parts(int64_t T) { return (T + NB_RB - 1) / NB_RB; }
hipError_t k_rmsnorm_bwd(const void* x, int64_t ldx, const void* gamma, const float* stat, float eps,
                         const void* dxhat, int64_t lddxh, const void* dres, int64_t lddres, void* dx, int64_t lddx,
                         float* dgamma_part, int64_t T, int64_t d, int dt, hipStream_t st) {
  if (T <= 0) return hipSuccess;
  if (dt == LR_BF16 && d <= 4096) {   // a row fits a wavefront's registers: single pass over every tensor
    // one-time opt-in to more than 64 KB of dynamic LDS (thread-safe static initialisation)
    static const hipError_t attr_err = hipFuncSetAttribute((const void*)rmsnorm_bwd_row_kernel<8>,
                                                           hipFuncAttributeMaxDynamicSharedMemorySize, RN_ROW_LDS);
    if (attr_err != hipSuccess) return attr_err;
    // Rows per workgroup: a multiple of NB_RB chosen so that the launch is about one workgroup per CU
    // (measured at T = 32768: 6.1 TB/s with 256 workgroups of 128 rows against 5.8 with 512 of 64; 128
    // workgroups of 256 rows leave half the chip idle, 4.7).  The partial buffer keeps one row per NB_RB
    // rows of the input, whatever the launch.
    const int64_t nparts = k_rmsnorm_bwd_parts(T);
    int64_t mult = T / ((int64_t)NB_RB * 256);
    if (mult < 1) mult = 1;
    const int rows_per_wg = (int)(mult * NB_RB);
    const unsigned grid = (unsigned)((T + rows_per_wg - 1) / rows_per_wg);
    hipLaunchKernelGGL(rmsnorm_bwd_row_kernel<8>, dim3(grid), dim3(256), RN_ROW_LDS, st,
                       (const uint16_t*)x, ldx, (const uint16_t*)gamma, stat, eps, (const uint16_t*)dxhat, lddxh,
                       (const uint16_t*)dres, lddres, (uint16_t*)dx, lddx, dgamma_part, T, d, rows_per_wg, nparts);
    return hipGetLastError();
  }
  DISPATCH_DT(dt, rmsnorm_bwd_kernel, dim3(k_rmsnorm_bwd_parts(T)), dim3(256), st, x, ldx, gamma, stat, eps, dxhat,
              lddxh, dres, lddres, dx, lddx, dgamma_part, T, d);
}
hipError_t k_act_fwd(const void* z, int64_t ldz, void* a, int64_t lda, int64_t T, int64_t n, int act, int dt,
                     hipStream_t st) {
  if (T <= 0 || n <= 0) return hipSuccess;
  if (dt == LR_BF16 && ldz == n && lda == n) {
    const int64_t bytes = T * n * 2;
    hipLaunchKernelGGL(act_fwd_dense_kernel<DENSE_U>, dim3(grid_chunks(bytes / 16, 256 * DENSE_U)), dim3(256), 0, st, z, a, bytes, act);
    return hipGetLastError();
  }
  const int nv = dt == LR_BF16 ? 8 : 1;
  DISPATCH_DT(dt, act_fwd_kernel, dim3(grid_chunks(T * (n / nv), 256 * EW_U)), dim3(256), st, z, ldz, a, lda, T, n, act);
}
hipError_t k_rope128_bf16(void* x, int64_t ld, const float* cos_tab, const float* sin_tab, int64_t rows, int S, int H,
                          int inverse, hipStream_t st) {
  if (rows <= 0 || H <= 0) return hipSuccess;
  const int64_t items = rows * H * 8;
  hipLaunchKernelGGL(rope128_kernel, dim3((unsigned)((items + 255) / 256)), dim3(256), 0, st, (uint16_t*)x, ld, cos_tab,
                     sin_tab, rows, S, H, inverse ? -1.f : 1.f);
  return hipGetLastError();
}
hipError_t k_add2_bf16(const void* a, const void* b, void* out, int64_t T, int64_t n, hipStream_t st) {
  if (T <= 0 || n <= 0) return hipSuccess;
  const int64_t bytes = T * n * 2;
  hipLaunchKernelGGL(add2_dense_kernel<DENSE_U>, dim3(grid_chunks(bytes / 16, 256 * DENSE_U)), dim3(256), 0, st, a, b, out, bytes);
  return hipGetLastError();
}
hipError_t k_swiglu_fwd(const void* g, const void* u, void* m, int64_t ld, int64_t T, int64_t f, int dt,
                        hipStream_t st) {
  if (T <= 0 || f <= 0) return hipSuccess;
  if (dt == LR_BF16 && ld == f) {
    const int64_t bytes = T * f * 2;
    hipLaunchKernelGGL(swiglu_fwd_dense_kernel<DENSE_U>, dim3(grid_chunks(bytes / 16, 256 * DENSE_U)), dim3(256), 0, st, g, u, m, bytes);
    return hipGetLastError();
  }
  const int nv = dt == LR_BF16 ? 8 : 1;
  DISPATCH_DT(dt, swiglu_fwd_kernel, dim3(grid_chunks(T * (f / nv), 256 * EW_U)), dim3(256), st, g, u, m, ld, T, f);
}
hipError_t k_swiglu_bwd(const void* g, const void* u, const void* dm, void* dg, void* du, int64_t ld, int64_t T,
                        int64_t f, int dt, hipStream_t st) {
  if (T <= 0 || f <= 0) return hipSuccess;
  if (dt == LR_BF16 && ld == f) {
    const int64_t bytes = T * f * 2;
    hipLaunchKernelGGL(swiglu_bwd_dense_kernel<DENSE_U3>, dim3(grid_chunks(bytes / 16, 256 * DENSE_U3)), dim3(256), 0, st, g, u, dm, dg, du, bytes);
    return hipGetLastError();
  }
  const int nv = dt == LR_BF16 ? 8 : 1;
  DISPATCH_DT(dt, swiglu_bwd_kernel, dim3(grid_chunks(T * (f / nv), 256 * EW_U3)), dim3(256), st, g, u, dm, dg, du, ld, T, f);
}
hipError_t k_transpose(const void* in, int64_t ld_in, void* out, int64_t ld_out, int64_t rows, int64_t cols, int dt,
                       hipStream_t st) {
  if (rows <= 0 || cols <= 0) return hipSuccess;
  const int64_t pad_to = ld_out;  // the whole output row is owned by the destination buffer
  dim3 grid((cols + 63) / 64, (pad_to + 63) / 64);
  if (dt == LR_F32)
    hipLaunchKernelGGL(transpose_kernel<float>, grid, dim3(256), 0, st, (const float*)in, ld_in, (float*)out, ld_out,
                       rows, cols, pad_to);
  else if (rows % 8 == 0 && cols % 8 == 0 && ld_in % 8 == 0 && ld_out % 8 == 0 && ((uintptr_t)in & 15) == 0 &&
           ((uintptr_t)out & 15) == 0)
    hipLaunchKernelGGL(transpose16_vec_kernel, grid, dim3(256), 0, st, (const uint16_t*)in, ld_in, (uint16_t*)out, ld_out,
                       rows, cols, pad_to);
  else
    hipLaunchKernelGGL(transpose_kernel<uint16_t>, grid, dim3(256), 0, st, (const uint16_t*)in, ld_in, (uint16_t*)out,
                       ld_out, rows, cols, pad_to);
  return hipGetLastError();
}
hipError_t k_rowsum_parts(const float* part, int64_t ld, int nparts, float* out, int64_t M, hipStream_t st) {
  if (M <= 0) return hipSuccess;
  hipLaunchKernelGGL(rowsum_parts_kernel, dim3((M + 255) / 256), dim3(256), 0, st, part, ld, nparts, out, M);
  return hipGetLastError();
}
hipError_t k_rowdot(const void* a, int64_t lda, const void* b, int64_t ldb, float* out, int64_t M, int64_t N, int dt,
                    hipStream_t st) {
  if (M <= 0) return hipSuccess;
  DISPATCH_DT(dt, rowdot_kernel, dim3((M + 3) / 4), dim3(256), st, a, lda, b, ldb, out, M, N);
}
hipError_t k_scale_cols(const void* w, const void* gamma, void* wout, int64_t rows, int64_t cols, int dt,
                        hipStream_t st) {
  if (rows <= 0 || cols <= 0) return hipSuccess;
  const int nv = dt == LR_BF16 ? 8 : 1;
  DISPATCH_DT(dt, scale_cols_kernel, dim3(grid1d(rows * (cols / nv))), dim3(256), st, w, gamma, wout, rows, cols);
}
int64_t k_wgrad_dgamma_parts(int64_t rows) { return (rows + WF_RB - 1) / WF_RB; }
hipError_t k_wgrad_finish(const float* part, int nsplit, int64_t rows, int64_t cols, void* dw, const void* colscale,
                          const void* w_for_dgamma, float* dgamma_part, int accumulate, int dt, int out_dt,
                          hipStream_t st) {
  if (rows <= 0 || cols <= 0) return hipSuccess;
  const int nv = dt == LR_BF16 ? 8 : 1;
  const bool dg = w_for_dgamma != nullptr && dgamma_part != nullptr;
  dim3 grid = dg ? dim3((unsigned)((cols / nv + 63) / 64), (unsigned)((rows + WF_RB - 1) / WF_RB))
                 : dim3((unsigned)((rows * (cols / nv) + 255) / 256));
#define LRB_WF2(DT_, OT_, NS_)                                                                                   \
  do {                                                                                                           \
    if (dg)                                                                                                      \
      hipLaunchKernelGGL((wgrad_finish_kernel<DT_, OT_, true, NS_>), grid, dim3(256), 0, st, part, nsplit, rows, cols, dw, \
                         colscale, w_for_dgamma, dgamma_part, accumulate);                                      \
    else                                                                                                         \
      hipLaunchKernelGGL((wgrad_finish_kernel<DT_, OT_, false, NS_>), grid, dim3(256), 0, st, part, nsplit, rows, cols, dw, \
                         colscale, w_for_dgamma, dgamma_part, accumulate);                                      \
  } while (0)
#define LRB_WF(DT_, OT_)                                                                                         \
  do {                                                                                                           \
    switch (nsplit) {                                                                                            \
      case 2: LRB_WF2(DT_, OT_, 2); break;                                                                       \
      case 3: LRB_WF2(DT_, OT_, 3); break;                                                                       \
      case 4: LRB_WF2(DT_, OT_, 4); break;                                                                       \
      case 8: LRB_WF2(DT_, OT_, 8); break;                                                                       \
      default: LRB_WF2(DT_, OT_, 0); break;                                                                      \
    }                                                                                                            \
  } while (0)
  if (dt == LR_F32) LRB_WF(LR_F32, float);
  else if (out_dt == LR_F32) LRB_WF(LR_BF16, float);
  else LRB_WF(LR_BF16, bf16_t);
#undef LRB_WF
#undef LRB_WF2
  return hipGetLastError();
}
hipError_t k_colsum_parts(const float* part, int64_t nparts, int64_t cols, void* out, int accumulate, int out_dt,
                          hipStream_t st) {
  if (cols <= 0) return hipSuccess;
  if (out_dt == LR_F32)
    hipLaunchKernelGGL(colsum_parts_kernel<float>, dim3((cols + 255) / 256), dim3(256), 0, st, part, nparts, cols, out,
                       accumulate);
  else
    hipLaunchKernelGGL(colsum_parts_kernel<bf16_t>, dim3((cols + 255) / 256), dim3(256), 0, st, part, nparts, cols,
                       out, accumulate);
  return hipGetLastError();
}

}  // namespace lrb
