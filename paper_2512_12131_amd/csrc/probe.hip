// Measurement aid, not on the compute path: the rate the matrix pipes of this chip sustain when they
// are fed from registers alone (no LDS, no memory traffic).  It bounds what any bf16 GEMM kernel can
// reach on the machine it runs on, which is what a utilisation figure (Sec. 5.3 reports kernel
// utilisation per linear layer) has to be read against: the sustained clock under matrix load
// depends on how much the operand bits toggle, so the probe runs with smooth and with pseudo-random
// operands.
#include <hip/hip_runtime.h>

#include "common.h"
#include "lrboost.h"

// Externally visible on purpose: stores to a file-local variable that nothing reads would be removed,
// and the probe's loop with them.
__device__ float lr_probe_sink[256];

namespace {

typedef __bf16 bf16x8_t __attribute__((ext_vector_type(8)));
typedef float f32x16_t __attribute__((ext_vector_type(16)));

constexpr int PROBE_ACC = 8;          // independent accumulator tiles per wavefront
constexpr int PROBE_THREADS = 256;    // 4 wavefronts, one per SIMD (the sink above has as many slots)
constexpr int PROBE_BLOCKS = 512;     // 2 workgroups per CU on 256 CUs: 2 wavefronts per SIMD

__device__ __forceinline__ float probe_uniform(uint32_t x) {   // (-1, 1) from a 32-bit mix
  x ^= x >> 16; x *= 0x7feb352dU; x ^= x >> 15; x *= 0x846ca68bU; x ^= x >> 16;
  return (float)(int32_t)x * (1.0f / 2147483648.0f);
}

// Every wavefront issues iters * PROBE_ACC v_mfma_f32_32x32x16_bf16 on PROBE_ACC independent
// accumulators; the two operands change places from one instruction to the next so that the operand
// buses toggle.  The result is folded into a store that a never-true comparison guards, so the loop
// cannot be removed and nothing is written.
template <bool RANDOM>
__global__ __launch_bounds__(PROBE_THREADS) void mfma_probe_kernel(int iters) {
  bf16x8_t a, b;
  for (int e = 0; e < 8; e++) {
    if (RANDOM) {
      const uint32_t id = (blockIdx.x * PROBE_THREADS + threadIdx.x) * 16 + e;
      a[e] = (__bf16)probe_uniform(id);
      b[e] = (__bf16)probe_uniform(id + 8);
    } else {
      a[e] = (__bf16)(threadIdx.x * 0.001f + e);
      b[e] = (__bf16)(1.0f + e * 0.01f);
    }
  }
  f32x16_t acc[PROBE_ACC];
  for (int i = 0; i < PROBE_ACC; i++)
    for (int e = 0; e < 16; e++) acc[i][e] = 0.f;
  for (int it = 0; it < iters; it++) {
#pragma unroll
    for (int i = 0; i < PROBE_ACC; i++)
      acc[i] = (i & 1) ? __builtin_amdgcn_mfma_f32_32x32x16_bf16(b, a, acc[i], 0, 0, 0)
                       : __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, b, acc[i], 0, 0, 0);
  }
  float s = 0.f;
  for (int i = 0; i < PROBE_ACC; i++)
    for (int e = 0; e < 16; e++) s += acc[i][e];
  if (s == 12345.678f) lr_probe_sink[threadIdx.x] = s;
}

}  // namespace

int lr_mfma_probe(int random_operands, int iters, int launches, double* tflops, void* stream) {
  if (!tflops || iters <= 0 || iters > (1 << 20) || launches <= 0 || launches > 1000) return LR_EINVAL;
  hipStream_t st = (hipStream_t)stream;
  hipEvent_t e0 = nullptr, e1 = nullptr;
  if (hipEventCreate(&e0) != hipSuccess) return LR_ELAUNCH;
  if (hipEventCreate(&e1) != hipSuccess) { (void)hipEventDestroy(e0); return LR_ELAUNCH; }
  auto launch = [&]() {
    if (random_operands) hipLaunchKernelGGL(mfma_probe_kernel<true>, dim3(PROBE_BLOCKS), dim3(PROBE_THREADS), 0, st, iters);
    else hipLaunchKernelGGL(mfma_probe_kernel<false>, dim3(PROBE_BLOCKS), dim3(PROBE_THREADS), 0, st, iters);
  };
  const int warm = launches < 4 ? launches : 4;   // lets the clock settle under the load
  for (int i = 0; i < warm; i++) launch();
  bool ok = hipEventRecord(e0, st) == hipSuccess;
  for (int i = 0; i < launches; i++) launch();
  ok = ok && hipEventRecord(e1, st) == hipSuccess && hipGetLastError() == hipSuccess &&
       hipEventSynchronize(e1) == hipSuccess;
  float ms = 0.f;
  ok = ok && hipEventElapsedTime(&ms, e0, e1) == hipSuccess && ms > 0.f;
  (void)hipEventDestroy(e0);
  (void)hipEventDestroy(e1);
  if (!ok) return LR_ELAUNCH;
  const double flop = 2.0 * 32 * 32 * 16 * PROBE_ACC * (double)iters * (PROBE_BLOCKS * (PROBE_THREADS / 64)) *
                      (double)launches;
  *tflops = flop / (ms * 1e-3) * 1e-12;
  return LR_OK;
}
