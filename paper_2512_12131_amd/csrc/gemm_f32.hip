// fp32 reference-precision GEMM: C[M,N] = epi(sum_k A(m,k) B(n,k)) for any operand orientation and
// any sizes.  This is the precision path (max|err|/RMS <= 1e-4 against the fp64 oracle), not a
// throughput path: 64x64 output tile, 16-deep k slices through LDS, 4x4 outputs per thread, plain
// fp32 FMA.  Split-K and every epilogue kind of the bf16 kernel are available, except row partials
// (callers run k_rowdot / k_rms_stat instead).
#include "epilogue.h"

namespace lrb {
namespace {

constexpr int TBM = 64, TBN = 64, TBK = 16;

template <int KIND>
__global__ __launch_bounds__(256) void gemm_f32_kernel(GemmOp op, int kper) {
  __shared__ float sA[TBK][TBM + 4];
  __shared__ float sB[TBK][TBN + 4];
  const int tid = threadIdx.x;
  const int tx = tid % 16, ty = tid / 16;
  const int m0 = blockIdx.y * TBM, n0 = blockIdx.x * TBN;
  const int bz = blockIdx.z;
  const int b = bz / op.splitk, ks = bz % op.splitk;
  const int kbeg = ks * kper;
  const int kend = min(op.K, kbeg + kper);
  const float* A = (const float*)op.A + (int64_t)b * op.sA;
  const float* B = (const float*)op.B + (int64_t)b * op.sB;
  const int64_t sAm = op.transA ? 1 : op.lda, sAk = op.transA ? op.lda : 1;
  const int64_t sBn = op.transB ? 1 : op.ldb, sBk = op.transB ? op.ldb : 1;

  float acc[4][4] = {};
  for (int k0 = kbeg; k0 < kend; k0 += TBK) {
    // 64x16 elements per operand, 256 threads -> 4 each.  Pick the thread->element map so that the
    // fastest-varying thread index walks the contiguous memory axis.
#pragma unroll
    for (int i = 0; i < 4; i++) {
      int e = tid + i * 256;
      int mm, kk;
      if (op.transA) { mm = e % TBM; kk = e / TBM; } else { kk = e % TBK; mm = e / TBK; }
      int gm = m0 + mm, gk = k0 + kk;
      sA[kk][mm] = (gm < op.M && gk < kend) ? A[gm * sAm + gk * sAk] : 0.f;
      int nn;
      if (op.transB) { nn = e % TBN; kk = e / TBN; } else { kk = e % TBK; nn = e / TBK; }
      int gn = n0 + nn;
      gk = k0 + kk;
      sB[kk][nn] = (gn < op.N && gk < kend) ? B[gn * sBn + gk * sBk] : 0.f;
    }
    __syncthreads();
#pragma unroll
    for (int kk = 0; kk < TBK; kk++) {
      float a[4], bb[4];
#pragma unroll
      for (int i = 0; i < 4; i++) a[i] = sA[kk][ty * 4 + i];
#pragma unroll
      for (int j = 0; j < 4; j++) bb[j] = sB[kk][tx * 4 + j];
#pragma unroll
      for (int i = 0; i < 4; i++)
#pragma unroll
        for (int j = 0; j < 4; j++) acc[i][j] = fmaf(a[i], bb[j], acc[i][j]);
    }
    __syncthreads();
  }

  const Epilogue& e = op.epi;
#pragma unroll
  for (int i = 0; i < 4; i++) {
    int64_t gm = m0 + ty * 4 + i;
    if (gm >= op.M) continue;
    float rho = 1.f, rowb = 0.f;
    if constexpr (KIND != EPI_PARTIAL) {
      if (e.use_rho) rho = rho_of(e, e.rowa[gm]);
      if (e.rowb) rowb = e.rowb[gm];
    }
#pragma unroll
    for (int j = 0; j < 4; j++) {
      int64_t gn = n0 + tx * 4 + j;
      if (gn >= op.N) continue;
      float v = acc[i][j];
      if constexpr (KIND == EPI_PARTIAL) {
        ((float*)op.C)[((int64_t)bz * op.M + gm) * op.N + gn] = v;
      } else {
        epi_apply<float, 1, KIND>(e, op.C, op.ldc, op.sC, b, gm, gn, &v, rho, rowb);
      }
    }
  }
}

}  // namespace

hipError_t gemm_f32(const GemmOp& op, hipStream_t st) {
  if (op.M <= 0 || op.N <= 0 || op.batch <= 0) return hipSuccess;
  dim3 grid((op.N + TBN - 1) / TBN, (op.M + TBM - 1) / TBM, op.batch * op.splitk);
  dim3 block(256);
  int kper = (op.K + op.splitk - 1) / op.splitk;
  kper = (kper + TBK - 1) / TBK * TBK;
  const int kind = op.splitk > 1 ? (int)EPI_PARTIAL : op.epi.kind;
  switch (kind) {
#define CASE(KD) \
  case KD: hipLaunchKernelGGL(gemm_f32_kernel<KD>, grid, block, 0, st, op, kper); break;
    CASE(EPI_STORE)
    CASE(EPI_DOWN)
    CASE(EPI_UP)
    CASE(EPI_ACTGRAD)
    CASE(EPI_NORMBWD)
    CASE(EPI_PARTIAL)
    CASE(EPI_SWIGLU_BWD)
    CASE(EPI_SWIGLU_FWD)
    CASE(EPI_DOWN_LAX)
    CASE(EPI_LAXGRAD)
#undef CASE
    default: return hipErrorInvalidValue;
  }
  return hipGetLastError();
}

}  // namespace lrb
