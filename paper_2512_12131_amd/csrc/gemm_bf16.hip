// bf16 MFMA GEMM for gfx950:  C[M,N] = epi( sum_k A[m,k] * B[n,k] ), fp32 accumulate.
//
// Both operands are read with k contiguous ("NT" form: the forward projections x.W^T, and the
// data-gradient GEMMs after the small weight matrices have been transposed once).  A k-major
// operand (weight gradients reduce over tokens) is staged through the same LDS layout by the
// transposing loader further down.
//
// Work decomposition: one workgroup owns a BM x BN output tile, WM x WN wavefronts each own a
// (BM/WM) x (BN/WN) sub-tile built from 32x32x16 MFMA blocks.  The k loop moves 64-wide slices
// global -> registers -> LDS with two LDS stages (one barrier per slice); LDS rows are 128 bytes
// with the 16-byte chunk index XOR-swizzled by the row so that both the row-wise stores and the
// MFMA-operand reads (32 rows x one chunk) are conflict free.  The accumulator tile leaves through
// LDS as well, so that every global access of the epilogue (C, the auxiliary tiles it reads, the
// secondary output) is a row-contiguous 16-byte vector.
#include <type_traits>

#include "epilogue.h"

namespace lrb {
namespace {

constexpr int BK = 64;          // k elements per slice (128 bytes per LDS row)
constexpr int NXCD = 8;

template <int BM_, int BN_, int WM_, int WN_>
struct Tile {
  static constexpr int BM = BM_, BN = BN_, WM = WM_, WN = WN_;
  static constexpr int NT = WM * WN * 64;
  static constexpr int TM = BM / WM, TN = BN / WN;
  static constexpr int FM = TM / 32, FN = TN / 32;
  static constexpr int A_BYTES = BM * 128, B_BYTES = BN * 128, STAGE = A_BYTES + B_BYTES;
  static constexpr int ACH = BM * 8 / NT, BCH = BN * 8 / NT;
  static constexpr int CS = TN + 8;  // fp32 row stride of the epilogue staging tile
  static constexpr int EPI_BYTES = WM * WN * 32 * CS * 4;
  static constexpr int STAT_BYTES = BM * 4;
  static constexpr int MAIN_BYTES = 2 * STAGE;
  static constexpr int LDS_BYTES = (MAIN_BYTES > EPI_BYTES ? MAIN_BYTES : EPI_BYTES) + STAT_BYTES;
  static_assert(ACH >= 1 && BCH >= 1 && FM >= 1 && FN >= 1, "tile too small for the thread count");
};

// Compile-time loop: the body receives std::integral_constant indices, so register arrays indexed
// by them never turn into scratch memory, whatever the unroller decides.
template <int N, class F, int I = 0>
__device__ __forceinline__ void static_for(F&& f) {
  if constexpr (I < N) {
    f(std::integral_constant<int, I>{});
    static_for<N, F, I + 1>(static_cast<F&&>(f));
  }
}

__device__ __forceinline__ uint4 ldg16(const uint16_t* p, bool ok) {
  uint4 z = make_uint4(0, 0, 0, 0);
  return ok ? *reinterpret_cast<const uint4*>(p) : z;
}

__device__ __forceinline__ float sumsq8(const uint4& q) {
  float v[8];
  unpack8(q, v);
  float s = 0.f;
#pragma unroll
  for (int i = 0; i < 8; i++) s = fmaf(v[i], v[i], s);
  return s;
}

// Maps the linear workgroup id to an output tile so that (a) the workgroups that the hardware
// deals round-robin to one XCD form a contiguous range of tiles, and (b) consecutive tiles of that
// range form compact panels (PM tiles tall), keeping the A rows and B rows they share in that
// XCD's L2.
__device__ __forceinline__ void tile_of_block(int bid, int total, int tiles_m, int tiles_n, int& tm, int& tn) {
  const int xcd = bid % NXCD, loc = bid / NXCD;
  const int base = total / NXCD, rem = total % NXCD;
  const int nid = xcd * base + (xcd < rem ? xcd : rem) + loc;
  constexpr int PM = 8;
  const int per_panel = PM * tiles_n;
  const int panel = nid / per_panel, within = nid % per_panel;
  const int pm_eff = min(PM, tiles_m - panel * PM);
  tn = within / pm_eff;
  tm = panel * PM + within % pm_eff;
}

template <class T, int KIND, bool STAT_A>
__global__ __launch_bounds__(T::NT) void gemm_bf16_kernel(GemmOp op, int kper, int tiles_m, int tiles_n) {
  extern __shared__ __attribute__((aligned(16))) unsigned char smem[];
  float* sStat = reinterpret_cast<float*>(smem + T::LDS_BYTES - T::STAT_BYTES);

  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int wm = wave / T::WN, wn = wave % T::WN;
  int tm, tn;
  tile_of_block(blockIdx.x, gridDim.x, tiles_m, tiles_n, tm, tn);
  const int m0 = tm * T::BM, n0 = tn * T::BN;
  const int bz = blockIdx.y;
  const int b = bz / op.splitk, ks = bz % op.splitk;
  const int kbeg = ks * kper, kend = min(op.K, kbeg + kper);
  const int nk = kend > kbeg ? (kend - kbeg + BK - 1) / BK : 0;

  const uint16_t* A = (const uint16_t*)op.A + (int64_t)b * op.sA;
  const uint16_t* B = (const uint16_t*)op.B + (int64_t)b * op.sB;

  // ---- global -> register staging -------------------------------------------------------------
  const int kc = tid & 7;          // 16-byte chunk of the 128-byte k slice this thread moves
  const int r0 = tid >> 3;         // first tile row this thread moves; further rows every NT/8
  const uint16_t* ap[T::ACH];
  const uint16_t* bp[T::BCH];
  bool aok[T::ACH], bok[T::BCH];
#pragma unroll
  for (int i = 0; i < T::ACH; i++) {
    int row = r0 + i * (T::NT / 8);
    aok[i] = (m0 + row) < op.M;
    ap[i] = A + (int64_t)(aok[i] ? m0 + row : 0) * op.lda + kbeg + kc * 8;
  }
#pragma unroll
  for (int i = 0; i < T::BCH; i++) {
    int row = r0 + i * (T::NT / 8);
    bok[i] = (n0 + row) < op.N;
    bp[i] = B + (int64_t)(bok[i] ? n0 + row : 0) * op.ldb + kbeg + kc * 8;
  }
  uint4 ra[T::ACH], rb[T::BCH];
  float ssq[T::ACH];
#pragma unroll
  for (int i = 0; i < T::ACH; i++) ssq[i] = 0.f;

  auto load_slice = [&](int kt) {
    const bool kok = (kbeg + kt * BK + kc * 8) < kend;
#pragma unroll
    for (int i = 0; i < T::ACH; i++) ra[i] = ldg16(ap[i] + kt * BK, aok[i] && kok);
#pragma unroll
    for (int i = 0; i < T::BCH; i++) rb[i] = ldg16(bp[i] + kt * BK, bok[i] && kok);
  };
  auto store_slice = [&](int stage) {
    unsigned char* sa = smem + stage * T::STAGE;
    unsigned char* sb = sa + T::A_BYTES;
#pragma unroll
    for (int i = 0; i < T::ACH; i++) {
      int row = r0 + i * (T::NT / 8);
      *reinterpret_cast<uint4*>(sa + row * 128 + ((kc ^ (row & 7)) << 4)) = ra[i];
      if constexpr (STAT_A) ssq[i] += sumsq8(ra[i]);
    }
#pragma unroll
    for (int i = 0; i < T::BCH; i++) {
      int row = r0 + i * (T::NT / 8);
      *reinterpret_cast<uint4*>(sb + row * 128 + ((kc ^ (row & 7)) << 4)) = rb[i];
    }
  };

  f32x16 acc[T::FM][T::FN];
#pragma unroll
  for (int i = 0; i < T::FM; i++)
#pragma unroll
    for (int j = 0; j < T::FN; j++)
#pragma unroll
      for (int v = 0; v < 16; v++) acc[i][j][v] = 0.f;

  const int frow = lane & 31, fk = lane >> 5, fsw = lane & 7;

  if (nk > 0) {
    load_slice(0);
    store_slice(0);
  }
  __syncthreads();
  for (int kt = 0; kt < nk; kt++) {
    const bool more = kt + 1 < nk;
    if (more) load_slice(kt + 1);
    const unsigned char* sa = smem + (kt & 1) * T::STAGE + (wm * T::TM + frow) * 128;
    const unsigned char* sb = smem + (kt & 1) * T::STAGE + T::A_BYTES + (wn * T::TN + frow) * 128;
#pragma unroll
    for (int kk = 0; kk < BK / 16; kk++) {
      const int coff = ((kk * 2 + fk) ^ fsw) << 4;
      bf16x8 af[T::FM], bf[T::FN];
#pragma unroll
      for (int i = 0; i < T::FM; i++) af[i] = *reinterpret_cast<const bf16x8*>(sa + i * 32 * 128 + coff);
#pragma unroll
      for (int j = 0; j < T::FN; j++) bf[j] = *reinterpret_cast<const bf16x8*>(sb + j * 32 * 128 + coff);
#pragma unroll
      for (int i = 0; i < T::FM; i++)
#pragma unroll
        for (int j = 0; j < T::FN; j++)
          acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(af[i], bf[j], acc[i][j], 0, 0, 0);
    }
    if (more) store_slice((kt + 1) & 1);
    __syncthreads();
  }

  // ---- per-row sum of squares gathered from the A slices ---------------------------------------
  if constexpr (STAT_A) {
#pragma unroll
    for (int i = 0; i < T::ACH; i++) {
      float s = ssq[i];
      s += __shfl_xor(s, 1);
      s += __shfl_xor(s, 2);
      s += __shfl_xor(s, 4);
      if (kc == 0) sStat[r0 + i * (T::NT / 8)] = s;
    }
  }
  __syncthreads();  // main-loop LDS is dead from here on; sStat is visible

  // ---- epilogue: accumulators -> LDS (per-wave region) -> row-contiguous 8-wide vectors ---------
  const Epilogue& e = op.epi;
  float* sC = reinterpret_cast<float*>(smem) + wave * (32 * T::CS);
  constexpr int LPR = T::TN / 8;            // lanes per output row
  constexpr int RPP = 64 / LPR;             // rows per pass
  const int cg = lane % LPR, rsub = lane / LPR;
  static_for<T::FM>([&](auto I) {
    constexpr int i = decltype(I)::value;
    static_for<T::FN>([&](auto J) {
      constexpr int j = decltype(J)::value;
#pragma unroll
      for (int v = 0; v < 16; v++) {
        int rl = 8 * (v >> 2) + 4 * (lane >> 5) + (v & 3);
        sC[rl * T::CS + j * 32 + (lane & 31)] = acc[i][j][v];
      }
    });
    __syncthreads();
#pragma unroll
    for (int p = 0; p < 32 / RPP; p++) {
      const int rl = p * RPP + rsub;
      const int lm = wm * T::TM + i * 32 + rl;      // row inside the block tile
      const int64_t gm = (int64_t)m0 + lm;
      const int64_t gn = (int64_t)n0 + wn * T::TN + cg * 8;
      float v[8];
      {
        const float4 lo = *reinterpret_cast<const float4*>(sC + rl * T::CS + cg * 8);
        const float4 hi = *reinterpret_cast<const float4*>(sC + rl * T::CS + cg * 8 + 4);
        v[0] = lo.x; v[1] = lo.y; v[2] = lo.z; v[3] = lo.w;
        v[4] = hi.x; v[5] = hi.y; v[6] = hi.z; v[7] = hi.w;
      }
      const bool ok = gm < op.M && gn < op.N;
      float part = 0.f;
      if constexpr (KIND == EPI_PARTIAL) {
        if (ok) {
          float* cp = (float*)op.C + ((int64_t)bz * op.M + gm) * op.N + gn;
          *reinterpret_cast<float4*>(cp) = make_float4(v[0], v[1], v[2], v[3]);
          *reinterpret_cast<float4*>(cp + 4) = make_float4(v[4], v[5], v[6], v[7]);
        }
      } else {
        if (ok) {
          float rho = 1.f, rowb = 0.f;
          if (e.use_rho) {
            float ss;
            if constexpr (STAT_A) ss = sStat[lm]; else ss = e.rowa[gm];
            rho = rho_of(e, ss);
          }
          if (e.rowb) rowb = e.rowb[gm];
          part = epi_apply<bf16_t, 8, KIND>(e, op.C, op.ldc, op.sC, b, gm, gn, v, rho, rowb);
        }
        if constexpr (KIND == EPI_UP || KIND == EPI_ACTGRAD) {
          if (e.rowpart) {
#pragma unroll
            for (int o = 1; o < LPR; o <<= 1) part += __shfl_xor(part, o);
            if (cg == 0 && gm < op.M)
              e.rowpart[gm * e.rowpart_ld + e.rowpart_off + b * (tiles_n * T::WN) + tn * T::WN + wn] = part;
          }
        }
        if constexpr (STAT_A) {
          if (e.stat_out && tn == 0 && wn == 0 && b == 0 && cg == 0 && gm < op.M) e.stat_out[gm] = sStat[lm];
        }
      }
    }
    __syncthreads();
  });
}

// ---------------------------------------------------------------------------------------------
template <class T, int KIND, bool STAT_A>
hipError_t launch(const GemmOp& op, hipStream_t st) {
  static bool attr_set = false;  // one-time opt-in to > 64 KB of dynamic LDS for this instantiation
  auto kern = gemm_bf16_kernel<T, KIND, STAT_A>;
  if (!attr_set) {
    hipError_t err = hipFuncSetAttribute((const void*)kern, hipFuncAttributeMaxDynamicSharedMemorySize, T::LDS_BYTES);
    if (err != hipSuccess) return err;
    attr_set = true;
  }
  const int tiles_m = (op.M + T::BM - 1) / T::BM, tiles_n = (op.N + T::BN - 1) / T::BN;
  int kper = (op.K + op.splitk - 1) / op.splitk;
  kper = (kper + BK - 1) / BK * BK;
  dim3 grid(tiles_m * tiles_n, op.batch * op.splitk);
  hipLaunchKernelGGL(kern, grid, dim3(T::NT), T::LDS_BYTES, st, op, kper, tiles_m, tiles_n);
  return hipGetLastError();
}

using TileBig = Tile<256, 256, 2, 2>;   // 4 waves, 128x128 per wave
using TileMid = Tile<256, 128, 2, 2>;   // 4 waves, 128x64 per wave (narrow N, weight gradients)

template <class T>
hipError_t dispatch(const GemmOp& op, hipStream_t st) {
  const int kind = op.splitk > 1 ? (int)EPI_PARTIAL : op.epi.kind;
  switch (kind) {
    case EPI_STORE: return launch<T, EPI_STORE, false>(op, st);
    case EPI_DOWN:
      return op.epi.stat_from_a ? launch<T, EPI_DOWN, true>(op, st) : launch<T, EPI_DOWN, false>(op, st);
    case EPI_UP: return launch<T, EPI_UP, false>(op, st);
    case EPI_ACTGRAD: return launch<T, EPI_ACTGRAD, false>(op, st);
    case EPI_NORMBWD: return launch<T, EPI_NORMBWD, false>(op, st);
    case EPI_PARTIAL: return launch<T, EPI_PARTIAL, false>(op, st);
    case EPI_SWIGLU_BWD: return launch<T, EPI_SWIGLU_BWD, false>(op, st);
    default: return hipErrorInvalidValue;
  }
}

bool use_big_tile(int N) { return N > 128 && (N % 256 == 0 || N > 512); }

}  // namespace

int gemm_bf16_rowpart_slabs(int N) {
  if (use_big_tile(N)) return (N + TileBig::BN - 1) / TileBig::BN * TileBig::WN;
  return (N + TileMid::BN - 1) / TileMid::BN * TileMid::WN;
}

int gemm_bf16_pick_splitk(int M, int N, int K, int batch) {
  const int bm = 256, bn = use_big_tile(N) ? 256 : 128;
  const long tiles = (long)((M + bm - 1) / bm) * ((N + bn - 1) / bn) * batch;
  int s = (int)((2 * 256 + tiles - 1) / tiles);   // aim at >= 2 workgroups per CU
  const int maxs = (K + 4 * BK - 1) / (4 * BK);   // at least 4 slices per split
  if (s > maxs) s = maxs;
  if (s > 64) s = 64;
  if (s < 1) s = 1;
  return s;
}

hipError_t gemm_bf16(const GemmOp& op, hipStream_t st) {
  if (op.M <= 0 || op.N <= 0 || op.batch <= 0) return hipSuccess;
  if (op.transA || op.transB) return hipErrorInvalidValue;
  if (op.epi.stat_from_a && op.splitk > 1) return hipErrorInvalidValue;
  if (use_big_tile(op.N)) return dispatch<TileBig>(op, st);
  return dispatch<TileMid>(op, st);
}

}  // namespace lrb
