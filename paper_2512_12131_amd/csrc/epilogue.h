// Device-side epilogue shared by the bf16 MFMA GEMM and the fp32 GEMM: takes NV consecutive
// accumulator columns of one output row, applies the fused elementwise work in fp32, rounds once
// and stores.  See EpiKind in common.h for the formulas.
#pragma once
#include <type_traits>

#include "common.h"

namespace lrb {

template <typename ST, int NV>
struct VecIO;

template <>
struct VecIO<float, 1> {
  static __device__ __forceinline__ void load(const void* p, int64_t off, float* v) { v[0] = ((const float*)p)[off]; }
  static __device__ __forceinline__ void store(void* p, int64_t off, const float* v) { ((float*)p)[off] = v[0]; }
  static __device__ __forceinline__ void load_nt(const void* p, int64_t off, float* v) { load(p, off, v); }
  static __device__ __forceinline__ void store_nt(void* p, int64_t off, const float* v) { store(p, off, v); }
};
template <>
struct VecIO<float, 8> {
  static __device__ __forceinline__ void load(const void* p, int64_t off, float* v) {
    const float4 a = *reinterpret_cast<const float4*>((const float*)p + off);
    const float4 b = *reinterpret_cast<const float4*>((const float*)p + off + 4);
    v[0] = a.x; v[1] = a.y; v[2] = a.z; v[3] = a.w; v[4] = b.x; v[5] = b.y; v[6] = b.z; v[7] = b.w;
  }
  static __device__ __forceinline__ void store(void* p, int64_t off, const float* v) {
    *reinterpret_cast<float4*>((float*)p + off) = make_float4(v[0], v[1], v[2], v[3]);
    *reinterpret_cast<float4*>((float*)p + off + 4) = make_float4(v[4], v[5], v[6], v[7]);
  }
};
typedef unsigned int u32x4_t __attribute__((ext_vector_type(4)));
template <>
struct VecIO<bf16_t, 8> {
  static __device__ __forceinline__ void load(const void* p, int64_t off, float* v) {
    uint4 q = *reinterpret_cast<const uint4*>((const uint16_t*)p + off);
    unpack8(q, v);
  }
  static __device__ __forceinline__ void store(void* p, int64_t off, const float* v) {
    *reinterpret_cast<uint4*>((uint16_t*)p + off) = pack8(v);
  }
  // streaming forms for data touched once: non-temporal, so it does not displace reusable lines
  static __device__ __forceinline__ void load_nt(const void* p, int64_t off, float* v) {
    const u32x4_t t = __builtin_nontemporal_load(reinterpret_cast<const u32x4_t*>((const uint16_t*)p + off));
    unpack8(make_uint4(t.x, t.y, t.z, t.w), v);
  }
  static __device__ __forceinline__ void store_nt(void* p, int64_t off, const float* v) {
    const uint4 q = pack8(v);
    const u32x4_t t = {q.x, q.y, q.z, q.w};
    __builtin_nontemporal_store(t, reinterpret_cast<u32x4_t*>((uint16_t*)p + off));
  }
};

template <>
struct VecIO<bf16_t, 1> {
  static __device__ __forceinline__ void load(const void* p, int64_t off, float* v) {
    v[0] = bf16_bits_to_f32(((const uint16_t*)p)[off]);
  }
  static __device__ __forceinline__ void store(void* p, int64_t off, const float* v) {
    ((uint16_t*)p)[off] = (uint16_t)f32_to_bf16_bits(v[0]);
  }
};

// Which auxiliary tiles an epilogue kind reads (same shape as C): R and / or R2.
template <int KIND>
__device__ __forceinline__ bool epi_reads_r(const Epilogue& e) {
  if constexpr (KIND == EPI_UP || KIND == EPI_NORMBWD || KIND == EPI_DOWN_LAX || KIND == EPI_LAXGRAD) return e.R != nullptr;
  return KIND == EPI_ACTGRAD || KIND == EPI_SWIGLU_BWD || KIND == EPI_SWIGLU_FWD;
}
template <int KIND>
__device__ __forceinline__ bool epi_reads_r2(const Epilogue& e) {
  if constexpr (KIND == EPI_LAXGRAD) return e.R2 != nullptr;
  return KIND == EPI_NORMBWD || KIND == EPI_SWIGLU_BWD;
}

// The arithmetic of an epilogue kind on NV consecutive columns of one row.  v[NV]: accumulators in,
// primary output out; v2[NV]: secondary output (EPI_DOWN with want2, EPI_SWIGLU_BWD); r[NV], r2[NV]:
// the matching entries of the auxiliary tiles (zeros where a kind's tile is absent: adding them is
// harmless).  rho / rowb: per-row scalars resolved by the caller (rho = 1 when unused).  fp32 throughout;
// returns this thread's contribution to the row partial (0 if the kind has none).
// STORE_BF16: the primary output is stored as bf16.  The rank-r activation (sigma(z), or z + h_prev in the
// LaX form) is then formed from z AS STORED, so that the backward, which rebuilds it from the bf16
// checkpoint, gets the forward's activation bit for bit (Sec. 4.4: recomputed = stored).
template <int NV, int KIND, bool STORE_BF16>
__device__ __forceinline__ float epi_math(int act, float inv_d, bool want2, float* v, float* v2, float rho, float rowb,
                                          const float* r, const float* r2) {
  float part = 0.f;
  if constexpr (KIND == EPI_DOWN) {
#pragma unroll
    for (int i = 0; i < NV; i++) v[i] *= rho;
    if (want2) {
#pragma unroll
      for (int i = 0; i < NV; i++) v2[i] = act_f(STORE_BF16 ? bf16_round_f(v[i]) : v[i], act);
    }
  } else if constexpr (KIND == EPI_UP) {
#pragma unroll
    for (int i = 0; i < NV; i++) {
      v[i] += r[i];
      part += v[i] * v[i];
    }
  } else if constexpr (KIND == EPI_ACTGRAD) {
#pragma unroll
    for (int i = 0; i < NV; i++) {
      v[i] = v[i] * act_prime_f(r[i], act) * rho;
      part += v[i] * r[i];
    }
  } else if constexpr (KIND == EPI_NORMBWD) {
    const float coef = rho * inv_d * rowb;
#pragma unroll
    for (int i = 0; i < NV; i++) v[i] = v[i] - coef * r2[i] + r[i];
  } else if constexpr (KIND == EPI_SWIGLU_BWD) {
#pragma unroll
    for (int i = 0; i < NV; i++) {
      const float dm = v[i];
      v2[i] = dm * silu_f(r[i]);
      v[i] = dm * r2[i] * silu_prime_f(r[i]);
    }
  } else if constexpr (KIND == EPI_SWIGLU_FWD) {
#pragma unroll
    for (int i = 0; i < NV; i++) v2[i] = silu_f(r[i]) * v[i];
  } else if constexpr (KIND == EPI_DOWN_LAX) {
#pragma unroll
    for (int i = 0; i < NV; i++) {
      v[i] *= rho;
      v2[i] = (STORE_BF16 ? bf16_round_f(v[i]) : v[i]) + r[i];
    }
  } else if constexpr (KIND == EPI_LAXGRAD) {
#pragma unroll
    for (int i = 0; i < NV; i++) {
      v2[i] = v[i];
      v[i] = (v[i] + r2[i]) * rho;
      part += v[i] * r[i];
    }
  }
  return part;
}

// epi_math, then the stores through plain pointers (the fp32 kernel's epilogue).
template <typename ST, int NV, int KIND>
__device__ __forceinline__ float epi_compute(const Epilogue& e, void* C, int64_t ldc, int64_t sC, int b, int64_t m,
                                             int64_t n, float* v, float rho, float rowb, const float* r,
                                             const float* r2) {
  using IO = VecIO<ST, NV>;
  float v2[NV];
  const bool want2 = KIND == EPI_SWIGLU_BWD || KIND == EPI_SWIGLU_FWD || KIND == EPI_DOWN_LAX || KIND == EPI_LAXGRAD ||
                     (KIND == EPI_DOWN && e.C2 != nullptr);
  const float part = epi_math<NV, KIND, std::is_same<ST, bf16_t>::value>(e.act, e.inv_d, want2, v, v2, rho, rowb, r, r2);
  if (KIND != EPI_SWIGLU_FWD || C != nullptr) IO::store(C, (int64_t)b * sC + m * ldc + n, v);
  if (want2 && e.C2 != nullptr) IO::store(e.C2, (int64_t)b * e.sC2 + m * e.ldc2 + n, v2);
  return part;
}

// Load the auxiliary entries, then epi_compute.
template <typename ST, int NV, int KIND>
__device__ __forceinline__ float epi_apply(const Epilogue& e, void* C, int64_t ldc, int64_t sC, int b, int64_t m,
                                           int64_t n, float* v, float rho, float rowb) {
  using IO = VecIO<ST, NV>;
  float r[NV], r2[NV];
#pragma unroll
  for (int i = 0; i < NV; i++) { r[i] = 0.f; r2[i] = 0.f; }
  if (epi_reads_r<KIND>(e)) IO::load(e.R, (int64_t)b * e.sR + m * e.ldr + n, r);
  if (epi_reads_r2<KIND>(e)) IO::load(e.R2, (int64_t)b * e.sR2 + m * e.ldr2 + n, r2);
  return epi_compute<ST, NV, KIND>(e, C, ldc, sC, b, m, n, v, rho, rowb, r, r2);
}

__device__ __forceinline__ float rho_of(const Epilogue& e, float sumsq) {
  const float t = sumsq * e.inv_d + e.eps;
  return e.rho_sqrt ? sqrtf(t) : rsqrtf(t);
}

}  // namespace lrb
