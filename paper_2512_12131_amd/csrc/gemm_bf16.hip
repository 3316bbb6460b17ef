// bf16 MFMA GEMM for gfx950:  C[M,N] = epi( sum_k A[m,k] * B[n,k] ), fp32 accumulate.
//
// Two operand forms.  k-contiguous ("NT": the forward projections x.W^T, and the data-gradient GEMMs
// after the small weight matrices have been transposed once): slices land in LDS as [row][k] and the
// MFMA operands are plain 16-byte reads.  k-major (weight gradients, which reduce over tokens): slices
// land as [k][column] and the operands are gathered with the LDS transpose read.  The k-major form with
// a plain bf16 store, batched with two-level strides and with the k range of a row tile cut at its last
// row, also computes the attention's query gradient from the stored score gradient.
//
// Work decomposition: one workgroup owns a BM x BN output tile, WM x WN wavefronts each own a
// (BM/WM) x (BN/WN) sub-tile built from 32x32x16 MFMA blocks (256x256 by 8 wavefronts, two per SIMD,
// or 256x128 by 4).  The k loop moves 64-wide slices straight from global memory into LDS
// (buffer_load ... lds, no register staging, whole 128-byte cache lines per row) through a ring of
// three A slots and two B slots, one workgroup barrier per slice, the loads of a slice spread over
// its four k16 steps; the 16-byte chunk index of a row is XOR-swizzled so that the MFMA-operand reads
// spread over all banks.  The accumulator tile (held transposed: the MFMAs are issued with their
// operands exchanged) leaves through LDS as well, so that every global access of the epilogue (C, the
// auxiliary tiles it reads, the secondary output) is a row-contiguous 16-byte vector through a per-tile
// buffer resource, without branches.  Workgroups map to tiles XCD by XCD in compact panels and all walk k front to back, so that
// the tiles resident in one XCD share operand slices in its L2.
#include <type_traits>
#include <vector>

#include "epilogue.h"

namespace lrb {
namespace {

constexpr int BK = 64;          // k elements per LDS stage: 128-byte rows, i.e. whole cache lines per request
constexpr int NSA = 3;          // LDS slots of the A operand's slices: loads get two slices of lead
constexpr int NSB = 2;          // LDS slots of the B operand's slices: loads get one slice of lead
constexpr int NXCD = 8;

template <int BM_, int BN_, int WM_, int WN_>
struct Tile {
  static constexpr int BM = BM_, BN = BN_, WM = WM_, WN = WN_;
  static constexpr int NW = WM * WN, NT = NW * 64;
  static constexpr int TM = BM / WM, TN = BN / WN;
  static constexpr int FM = TM / 32, FN = TN / 32;
  static constexpr int A_BYTES = BM * 128, B_BYTES = BN * 128, STAGE = A_BYTES + B_BYTES;
  static constexpr int WLOADS = (BM + BN) / 8 / NW;   // 1 KB wavefront loads (8 rows x 128 B) per wavefront per stage
  static constexpr int WLOADS_A = BM / 8 / NW;        // the first WLOADS_A of them fetch A rows, the rest B rows
  // fp32 row stride of the epilogue staging tile: = 4 (mod 64), so the 16 rows that one cycle of a
  // 16-byte-per-lane write touches fall on 16 different groups of four banks
  static constexpr int CS = TN + 4;
  static constexpr int EPI_BYTES = NW * 32 * CS * 4;
  static constexpr int STAT_BYTES = BM * 4;
  static constexpr int MAIN_BYTES = NSA * A_BYTES + NSB * B_BYTES;
  // The per-row statistic is written after the main loop, into main-loop space the epilogue staging
  // does not reach (the 256x256 tile uses all 160 KB of LDS for its slices).
  static constexpr int STAT_OFF = EPI_BYTES;
  static constexpr int LDS_BYTES = MAIN_BYTES > EPI_BYTES + STAT_BYTES ? MAIN_BYTES : EPI_BYTES + STAT_BYTES;
  static_assert(BM / 8 % NW == 0 && BN / 8 % NW == 0 && FM >= 1 && FN >= 1 && BM <= NT,
                "tile / wavefront layout mismatch");
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

__device__ __forceinline__ float sumsq8(const uint4& q) {
  float v[8];
  unpack8(q, v);
  float s = 0.f;
#pragma unroll
  for (int i = 0; i < 8; i++) s = fmaf(v[i], v[i], s);
  return s;
}

// s_waitcnt vmcnt(N) with the other counters left alone (gfx9 encoding: vmcnt in bits 3:0 and 15:14).
template <int N>
__device__ __forceinline__ void wait_vmcnt() {
  __builtin_amdgcn_s_waitcnt((N & 15) | ((N >> 4) << 14) | 0x0f70);
}
__device__ __forceinline__ void wait_lgkmcnt0() { __builtin_amdgcn_s_waitcnt(0xc07f); }

// Sum over aligned groups of N = 8 or 16 consecutive lanes, every lane receiving the total, with
// data-parallel-primitive moves (register file only): neighbours inside a quad, then the mirror image
// inside 8 lanes, then inside 16.  (A butterfly of __shfl_xor goes through the LDS crossbar: four
// dependent round trips per row partial.)
template <int N>
__device__ __forceinline__ float lane_group_sum(float x) {
  static_assert(N == 8 || N == 16, "lane group size");
  auto dpp = [](float v, auto CTRL) {
    return __int_as_float(__builtin_amdgcn_update_dpp(0, __float_as_int(v), decltype(CTRL)::value, 0xf, 0xf, false));
  };
  x += dpp(x, std::integral_constant<int, 0xB1>{});    // quad_perm [1,0,3,2]
  x += dpp(x, std::integral_constant<int, 0x4E>{});    // quad_perm [2,3,0,1]
  x += dpp(x, std::integral_constant<int, 0x141>{});   // row_half_mirror: lane i <-> 7 - i
  if constexpr (N == 16) x += dpp(x, std::integral_constant<int, 0x140>{});   // row_mirror: lane i <-> 15 - i
  return x;
}

// Maps the linear workgroup id to an output tile so that (a) the workgroups that the hardware
// deals round-robin to one XCD form a contiguous range of tiles, and (b) consecutive tiles of that
// range form compact panels (PM tiles tall), keeping the A rows and B rows they share in that
// XCD's L2.
// The range runs over the whole launch, (batch member, k split) slowest: an XCD then works on tiles of
// one batch member and one k range at a time, which is what lets its workgroups share operand slices.
__device__ __forceinline__ void tile_of_block(int bid, int total, int tiles_m, int tiles_n, int& tm, int& tn, int& bz) {
  const int xcd = bid % NXCD, loc = bid / NXCD;
  const int base = total / NXCD, rem = total % NXCD;
  const int nid = xcd * base + (xcd < rem ? xcd : rem) + loc;
  const int tiles = tiles_m * tiles_n;
  bz = nid / tiles;
  const int tid_ = nid % tiles;
  constexpr int PM = 8;
  const int per_panel = PM * tiles_n;
  const int panel = tid_ / per_panel, within = tid_ % per_panel;
  const int pm_eff = min(PM, tiles_m - panel * PM);
  tn = within / pm_eff;
  tm = panel * PM + within % pm_eff;
}

#define LRB_LDS_PTR(p) ((__attribute__((address_space(3))) void*)(p))

// KM = false: operands k-contiguous, A[m][k], B[n][k].
// KM = true:  operands k-major,      A[k][m], B[k][n]  (weight gradients: k runs over tokens).  The
//             slices are stored in LDS as they arrive, [k][m], and the MFMA operands are gathered
//             with the LDS transpose read, so no transposed copy of an activation is ever written.
template <class T, int KIND, bool STAT_A, bool KM>
__global__ __launch_bounds__(T::NT) void gemm_bf16_kernel(GemmOp op, int kper, int tiles_m, int tiles_n) {
  static_assert(!KM || ((KIND == EPI_PARTIAL || KIND == EPI_STORE) && !STAT_A && T::BM == 256 && T::BN % 128 == 0),
                "the k-major form serves split-K weight gradients and plain stores");
  extern __shared__ __attribute__((aligned(16))) unsigned char smem[];
  float* sStat = reinterpret_cast<float*>(smem + T::STAT_OFF);

  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int wm = wave / T::WN, wn = wave % T::WN;
  int tm, tn, bz;
  tile_of_block(blockIdx.x + gridDim.x * blockIdx.y, gridDim.x * gridDim.y, tiles_m, tiles_n, tm, tn, bz);
  const int m0 = tm * T::BM, n0 = tn * T::BN;
  const int b = bz / op.splitk, ks = bz % op.splitk;
  const int kbeg = ks * kper;
  int kend = min(op.K, kbeg + kper);
  if (KM && op.causal_k) kend = min(kend, m0 + T::BM);
  // element offsets of this batch entry's operands
  const int bo = op.batch_inner > 0 ? b / op.batch_inner : 0, bi = op.batch_inner > 0 ? b % op.batch_inner : b;
  const int nk = kend > kbeg ? (kend - kbeg + BK - 1) / BK : 0;

  const uint16_t* A = (const uint16_t*)op.A + (int64_t)bi * op.sA + (int64_t)bo * op.sAo;
  const uint16_t* B = (const uint16_t*)op.B + (int64_t)bi * op.sB + (int64_t)bo * op.sBo;

  // ---- global -> LDS, without passing through registers ---------------------------------------
  // One buffer_load_dwordx4 ... lds per wavefront moves 8 tile rows x 128 bytes (1 KB, eight whole
  // cache lines): lane L's 16 bytes land at LDS base + 16 L, i.e. tile row L/8, physical chunk L%8.
  // The 16-byte chunks of a row are stored XOR-swizzled by (row/2)%8, so each lane fetches the logical
  // chunk that belongs in its slot; MFMA operand reads (32 rows x one logical chunk) then spread over
  // all banks.  A lane whose chunk lies outside the matrix (row tail, k tail) uses an offset past the
  // resource size: the load returns zeros and zeros are what reaches LDS.
  constexpr uint32_t OOB = 0x80000000u;
  const __amdgpu_buffer_rsrc_t rsA = __builtin_amdgcn_make_buffer_rsrc(
      (void*)(KM ? A + (int64_t)kbeg * op.lda + m0 : A + (int64_t)m0 * op.lda + kbeg), 0, 0x7fffffff, 0x00020000);
  const __amdgpu_buffer_rsrc_t rsB = __builtin_amdgcn_make_buffer_rsrc(
      (void*)(KM ? B + (int64_t)kbeg * op.ldb + n0 : B + (int64_t)n0 * op.ldb + kbeg), 0, 0x7fffffff, 0x00020000);
  // k-contiguous form: 8 rows x 128 B per wavefront load; k-major form: 2 k-rows x 512 B (BM = 256
  // columns) or 4 k-rows x 256 B (128 columns).  In both, the 16-byte chunk index inside a row is
  // XOR-swizzled so that the operand reads spread over the banks.
  // Swizzle of the k-contiguous form: physical chunk = logical chunk ^ ((row / 2) % 8).  An LDS row is
  // 128 bytes, half of the 64 x 4-byte banks, so rows 2i and 2i+1 lie side by side in one bank line;
  // with this term the 16 rows that one cycle of a 16-byte-per-lane read touches (16 lanes) fall on
  // 16 different 16-byte bank groups.  The 1 KB group index g = wave + NW * i keeps its parity over i
  // (NW is even), so one swizzle value per lane serves all of its loads.
  static_assert(T::NW % 2 == 0 && (T::BM / 8) % 2 == 0, "row parity of a lane must not depend on the load index");
  const int lrow = KM ? 0 : lane >> 3;
  const int lchunk = KM ? 0 : (lane & 7) ^ (((wave & 1) << 2) | (lrow >> 1));
  uint32_t goff[T::WLOADS];
  int kml_a = 0, kml_b = 0;          // KM: k-row (inside the slice, modulo the per-load stride) of this lane
#pragma unroll
  for (int i = 0; i < T::WLOADS; i++) {
    const int g = wave + T::NW * i;                        // 1 KB group: A groups first, then B
    if constexpr (!KM) {
      if (i < T::WLOADS_A) {
        const int row = g * 8 + lrow;
        goff[i] = (m0 + row) < op.M ? (uint32_t)(row * (int)op.lda + lchunk * 8) * 2u : OOB;
      } else {
        const int row = (g - T::BM / 8) * 8 + lrow;
        goff[i] = (n0 + row) < op.N ? (uint32_t)(row * (int)op.ldb + lchunk * 8) * 2u : OOB;
      }
    } else {
      if (i < T::WLOADS_A) {
        constexpr int CPR = T::BM / 8, RPL = 64 / CPR;       // chunks per k-row, k-rows per wavefront load
        const int krow = g * RPL + lane / CPR;
        const int lc = (lane % CPR) ^ ((krow & 7) << 2);
        goff[i] = (m0 + lc * 8) < op.M ? (uint32_t)(krow * (int)op.lda + lc * 8) * 2u : OOB;
        if (i == 0) kml_a = krow;
      } else {
        constexpr int CPR = T::BN / 8, RPL = 64 / CPR;
        const int krow = (g - T::BM / 8) * RPL + lane / CPR;
        const int lc = (lane % CPR) ^ (((krow & 7) << 2) & (CPR - 1));
        goff[i] = (n0 + lc * 8) < op.N ? (uint32_t)(krow * (int)op.ldb + lc * 8) * 2u : OOB;
        if (i == T::WLOADS_A) kml_b = krow;
      }
    }
  }
  // Every workgroup walks its k range in the same order, front to back.  The workgroups of an XCD
  // that share A rows or B rows (one panel of tiles) then want the same k slice at about the same time,
  // and all but the first request for it hit in that XCD's L2: walking from staggered starting slices
  // instead multiplied the traffic out of L2 by 3.6 and cost 12-18% of the GEMM rate.  The fixed order
  // also makes the summation order of a token row independent of how sequences are batched.
  // slot addresses: A slices cycle through NSA slots at the bottom of LDS, B slices through NSB above
  auto a_slot = [&](int kt) -> unsigned char* { return smem + (kt % NSA) * T::A_BYTES; };
  auto b_slot = [&](int kt) -> unsigned char* { return smem + NSA * T::A_BYTES + (kt % NSB) * T::B_BYTES; };
  constexpr int WLOADS_B = T::WLOADS - T::WLOADS_A;
  // issue_ab(kt, IS_A, HALF): HALF = 0 / 1 issues the first / second half of the operand's loads of
  // slice kt, HALF = 2 all of them
  auto issue_ab = [&](int kt, auto IS_A, auto HALF) {
    constexpr bool isA = decltype(IS_A)::value;
    constexpr int half = decltype(HALF)::value;
    const int kte = kt;
    unsigned char* dst = (isA ? a_slot(kt) : b_slot(kt)) + wave * 1024;
    constexpr int F0 = isA ? 0 : T::WLOADS_A, F1 = isA ? T::WLOADS_A : T::WLOADS;   // the operand's loads
    constexpr int I0 = half == 1 ? (F0 + F1) / 2 : F0, I1 = half == 0 ? (F0 + F1) / 2 : F1;
    if constexpr (!KM) {
      const uint32_t kmask = (kt < nk && (kbeg + kte * BK + lchunk * 8) < kend) ? 0u : OOB;
      const uint32_t ktoff = (uint32_t)kte * (BK * 2);
#pragma unroll
      for (int i = I0; i < I1; i++)
        __builtin_amdgcn_raw_ptr_buffer_load_lds(isA ? rsA : rsB, LRB_LDS_PTR(dst + (i - F0) * (T::NW * 1024)), 16,
                                                 (int)((goff[i] + ktoff) | kmask), 0, 0, 0);
    } else {
      // k-rows of load i: kml + i * (NW * rows-per-load); rows at or past the end of k read as zeros
      constexpr int RPL = 64 / ((isA ? T::BM : T::BN) / 8);
      const int krem = kt < nk ? (kend - kbeg) - kte * BK : 0;      // valid k-rows left from this slice's start
      const uint32_t off = (uint32_t)kte * BK * (uint32_t)(isA ? op.lda : op.ldb) * 2u;
      const int kml = isA ? kml_a : kml_b;
#pragma unroll
      for (int i = I0; i < I1; i++) {
        const uint32_t km = (kml + (i - F0) * T::NW * RPL) < krem ? 0u : OOB;
        __builtin_amdgcn_raw_ptr_buffer_load_lds(isA ? rsA : rsB, LRB_LDS_PTR(dst + (i - F0) * (T::NW * 1024)), 16,
                                                 (int)((goff[i] + off) | km), 0, 0, 0);
      }
    }
  };
  using Half0 = std::integral_constant<int, 0>;
  using Half1 = std::integral_constant<int, 1>;
  using Whole = std::integral_constant<int, 2>;

  f32x16 acc[T::FM][T::FN];
#pragma unroll
  for (int i = 0; i < T::FM; i++)
#pragma unroll
    for (int j = 0; j < T::FN; j++)
#pragma unroll
      for (int v = 0; v < 16; v++) acc[i][j][v] = 0.f;

  // MFMA operand addressing: row = lane%32 of a 32-row block, logical chunk kk*2 + lane/32
  const int frow = lane & 31, fk = lane >> 5, fsw = (frow >> 1) & 7;
  bf16x8 af[2][T::FM], bf[2][T::FN];
  // k-major form, transpose reads.  Inside each group of 16 lanes, lane s supplies the address of 4
  // consecutive columns of k-row (s/4) and receives column s of the 4 x 16 block; two reads (k-rows +0 and
  // +8) give the 8 k slots of a lane: slot (half, e) -> k = kk*16 + (e/4)*8 + half*4 + e%4, the same
  // assignment for both operands.  The lane-dependent part of every fragment address (k-row inside a
  // k16 step, swizzled column chunk) does not change over the main loop and is computed once; the slot
  // of the slice is added per fragment, the k16 step and the +8 rows ride in the instruction's offset.
  uint32_t troffA[KM ? T::FM : 1], troffB[KM ? T::FN : 1];
  if constexpr (KM) {
    const int g = lane >> 4, sl = lane & 15;
    const int krow0 = (g >> 1) * 4 + (sl >> 2);
    const int ksw = (krow0 & 7) << 2;                     // (krow0 + 8 n) & 7 is the same
    const int cin = (g & 1) * 16 + (sl & 3) * 4;          // column inside the 32-column block
    auto lane_off = [&](int pitch, int col, int swz) {
      return (uint32_t)(krow0 * pitch + ((((col >> 3) ^ swz) << 4) + (col & 7) * 2));
    };
#pragma unroll
    for (int i = 0; i < T::FM; i++) troffA[i] = lane_off(T::BM * 2, wm * T::TM + i * 32 + cin, ksw);
#pragma unroll
    for (int j2 = 0; j2 < T::FN; j2++) troffB[j2] = lane_off(T::BN * 2, wn * T::TN + j2 * 32 + cin, ksw & (T::BN / 8 - 1));
  }
  auto load_frags = [&](int buf, int kt, auto KKc) {
    constexpr int kk = decltype(KKc)::value;
    if constexpr (!KM) {
      const unsigned char* sa = a_slot(kt) + (wm * T::TM + frow) * 128;
      const unsigned char* sb = b_slot(kt) + (wn * T::TN + frow) * 128;
      const int coff = ((kk * 2 + fk) ^ fsw) << 4;
#pragma unroll
      for (int i = 0; i < T::FM; i++) af[buf][i] = *reinterpret_cast<const bf16x8*>(sa + i * 32 * 128 + coff);
#pragma unroll
      for (int j = 0; j < T::FN; j++) bf[buf][j] = *reinterpret_cast<const bf16x8*>(sb + j * 32 * 128 + coff);
    } else {
      typedef short s16x4 __attribute__((ext_vector_type(4)));
      typedef short s16x8 __attribute__((ext_vector_type(8)));
      // The transpose reads are issued as inline assembly.  Through the builtin, the compiler cannot
      // tell them from a read of the slot that the global->LDS loads in flight are writing, and puts a
      // wait for ALL outstanding global loads in front of each group of reads (which throws away the
      // two slices of load lead).  The price: the compiler does not wait for their results either, so
      // every k16 step of this form ends with an explicit wait for the LDS counter behind a scheduling
      // barrier (see the main loop).
      const uint32_t slotA = (uint32_t)(uintptr_t)LRB_LDS_PTR(a_slot(kt));
      const uint32_t slotB = (uint32_t)(uintptr_t)LRB_LDS_PTR(b_slot(kt));
      auto tr_pair = [&](uint32_t addr, auto PITCH) -> bf16x8 {
        constexpr int o0 = kk * 16 * decltype(PITCH)::value, o1 = o0 + 8 * decltype(PITCH)::value;
        static_assert(o1 < 65536, "LDS instruction offset field");
        s16x4 lo, hi;
        asm volatile("ds_read_b64_tr_b16 %0, %1 offset:%2" : "=v"(lo) : "v"(addr), "n"(o0) : "memory");
        asm volatile("ds_read_b64_tr_b16 %0, %1 offset:%2" : "=v"(hi) : "v"(addr), "n"(o1) : "memory");
        s16x8 r = {lo[0], lo[1], lo[2], lo[3], hi[0], hi[1], hi[2], hi[3]};
        return __builtin_bit_cast(bf16x8, r);
      };
#pragma unroll
      for (int i = 0; i < T::FM; i++) af[buf][i] = tr_pair(slotA + troffA[i], std::integral_constant<int, T::BM * 2>{});
#pragma unroll
      for (int j = 0; j < T::FN; j++) bf[buf][j] = tr_pair(slotB + troffB[j], std::integral_constant<int, T::BN * 2>{});
    }
  };
  auto mfma_step = [&](int buf) {
#pragma unroll
    for (int i = 0; i < T::FM; i++)
#pragma unroll
      for (int j = 0; j < T::FN; j++)
        acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(bf[buf][j], af[buf][i], acc[i][j], 0, 0, 0);
  };
  float ssq = 0.f;   // STAT_A: thread t accumulates the sum of squares of tile row t from the LDS copy
  auto stat_row = [&](int kt, int half) {
    if constexpr (STAT_A) {
      if (tid < T::BM) {
        const unsigned char* sr = a_slot(kt) + tid * 128 + half * 64;
#pragma unroll
        for (int c = 0; c < 4; c++) ssq += sumsq8(*reinterpret_cast<const uint4*>(sr + c * 16));
      }
    }
  };

  // ---- main loop ---------------------------------------------------------------------------------
  // Slice kt (64 wide) is multiplied in four k16 steps.  While step s runs, the operands of step s+1
  // are read from LDS.  Before step 3 a barrier establishes that every wavefront's part of slice
  // kt+1 has landed and that nobody reads slice kt's slots any more (the step-3 operands are in
  // registers).
  // The global->LDS loads are spread evenly over the four steps, because the CU's address/texture
  // path accepts about one 1 KB wavefront load per 23 cycles: issued in one burst they block the
  // issuing wavefronts (and with them their MFMAs) for most of a step.  LDS holds 3 slots for A
  // slices and 2 for B slices (5 x 32 KB), which allows this order inside iteration kt:
  //   step 0: second half of B(kt+1)      -> the slot B(kt-1) left at the previous barrier
  //   step 1, 2: the halves of A(kt+2)    -> the slot A(kt-1) left at the previous barrier
  //   barrier (needs A(kt+1), B(kt+1); loads retire in order, so A(kt+2) alone may stay in flight)
  //   step 3: first half of B(kt+2)       -> the slot B(kt) just left
  // The loop body is branch free: slices past the end of k are "loaded" with every lane out of range
  // (zeros into a slot nobody reads again), so the wait counts are compile-time constants.
  // Instruction interleave: a wavefront issues in order, and an MFMA occupies the matrix pipe for
  // 32 cycles during which the same wavefront may issue other work.  The scheduler is therefore
  // told to thread the LDS reads and global->LDS loads between the MFMAs instead of issuing them
  // in a burst while the matrix pipe idles.
  constexpr int MPR = (T::FM * T::FN) / (T::FM + T::FN);   // MFMAs per LDS operand read
  constexpr int HLA = T::WLOADS_A / 2, HLB = WLOADS_B / 2; // loads per half slice of A, of B
  constexpr std::true_type OPA{};
  constexpr std::false_type OPB{};
  issue_ab(0, OPA, Whole{});
  issue_ab(0, OPB, Whole{});
  issue_ab(1, OPA, Whole{});
  issue_ab(1, OPB, Half0{});
  wait_vmcnt<T::WLOADS_A + HLB>();   // A(0), B(0) landed; A(1) and half of B(1) may fly
  __builtin_amdgcn_s_barrier();
  load_frags(0, 0, std::integral_constant<int, 0>{});
  if constexpr (KM) {
    wait_lgkmcnt0();
    __builtin_amdgcn_sched_barrier(0);
  }
  for (int kt = 0; kt < nk; kt++) {
    static_for<3>([&](auto KK) {
      constexpr int kk = decltype(KK)::value;
      load_frags((kk + 1) & 1, kt, std::integral_constant<int, kk + 1>{});
      if constexpr (kk == 0) issue_ab(kt + 1, OPB, Half1{});
      if constexpr (kk == 1) issue_ab(kt + 2, OPA, Half0{});
      if constexpr (kk == 2) issue_ab(kt + 2, OPA, Half1{});
      if constexpr (kk < 2) stat_row(kt, kk);
      mfma_step(kk & 1);
      constexpr int NL = kk == 0 ? HLB : HLA;
#pragma unroll
      for (int i = 0; i < T::FM + T::FN; i++) {
        __builtin_amdgcn_sched_group_barrier(0x008, MPR, 0);   // MFMA
        __builtin_amdgcn_sched_group_barrier(0x100, KM ? 2 : 1, 0);     // DS read
        if (i * NL / (T::FM + T::FN) != (i + 1) * NL / (T::FM + T::FN))
          __builtin_amdgcn_sched_group_barrier(0x020, 1, 0);   // VMEM read (global -> LDS)
      }
      if constexpr (KM) {
        __builtin_amdgcn_sched_barrier(0);
        wait_lgkmcnt0();                   // the next step's operands (inline-assembly reads) have arrived
      }
      __builtin_amdgcn_sched_barrier(0);
    });
    wait_vmcnt<T::WLOADS_A>();             // A(kt+1), B(kt+1) of this wavefront landed; A(kt+2) may fly
    wait_lgkmcnt0();                       // and its reads of slice kt's slots are complete
    __builtin_amdgcn_s_barrier();
    __builtin_amdgcn_sched_barrier(0);
    issue_ab(kt + 2, OPB, Half0{});
    load_frags(0, kt + 1, std::integral_constant<int, 0>{});
    mfma_step(1);
#pragma unroll
    for (int i = 0; i < T::FM + T::FN; i++) {
      __builtin_amdgcn_sched_group_barrier(0x008, MPR, 0);   // MFMA
      __builtin_amdgcn_sched_group_barrier(0x100, KM ? 2 : 1, 0);     // DS read
      if (i * HLB / (T::FM + T::FN) != (i + 1) * HLB / (T::FM + T::FN))
        __builtin_amdgcn_sched_group_barrier(0x020, 1, 0);   // VMEM read (global -> LDS)
    }
    if constexpr (KM) {
      __builtin_amdgcn_sched_barrier(0);
      wait_lgkmcnt0();
    }
    __builtin_amdgcn_sched_barrier(0);
  }
  wait_vmcnt<0>();

  // ---- per-row sum of squares gathered from the A slices ---------------------------------------
  __syncthreads();  // main-loop LDS is dead from here on
  if constexpr (STAT_A) {
    if (tid < T::BM) sStat[tid] = ssq;
    __syncthreads();
  }

  // ---- epilogue: accumulators -> LDS (per-wave region) -> row-contiguous 8-wide vectors ---------
  // The wavefront's sub-tile leaves in FM x (32/RPP) passes of RPP rows.  Everything the passes touch
  // in global memory goes through buffer resources that start at the tile's first row and end after
  // its last valid row: rows past M (and, by an out-of-range offset, columns past N) read as zeros and
  // are dropped on store, an absent auxiliary tile is a resource of size zero.  The pass code is
  // therefore free of branches, which is what lets the compiler count the loads in flight exactly: the
  // auxiliary tiles an epilogue reads (residual, z, x, g, u) are fetched PF passes ahead into a small
  // register ring, and each pass waits only for its own.
  const Epilogue& e = op.epi;
  float* sC = reinterpret_cast<float*>(smem) + wave * (32 * T::CS);
  constexpr int LPR = T::TN / 8;            // lanes per output row
  constexpr int RPP = 64 / LPR;             // rows per pass
  constexpr int PPB = 32 / RPP;             // passes per 32-row block
  constexpr int NQ = T::FM * PPB;           // passes per wavefront
  // which auxiliary tiles a kind can read at all, and the prefetch distance in passes: kinds with one
  // auxiliary tile keep eight of its 16-byte vectors in flight per lane, kinds with two keep four of each
  // BASE: the formula; R_F32: the R tile is fp32 (two 16-byte vectors per lane and pass); O32: the primary
  // output is also written un-rounded, as fp32, into C32
  constexpr int BASE = epi_base(KIND);
  constexpr bool R_F32 = epi_r_is_f32(KIND), O32 = epi_writes_f32(KIND);
  constexpr bool HAS_R = BASE == EPI_UP || BASE == EPI_ACTGRAD || BASE == EPI_NORMBWD || BASE == EPI_SWIGLU_BWD ||
                         BASE == EPI_SWIGLU_FWD || BASE == EPI_DOWN_LAX || BASE == EPI_LAXGRAD;
  constexpr bool HAS_R2 = BASE == EPI_NORMBWD || BASE == EPI_SWIGLU_BWD || BASE == EPI_LAXGRAD;
  constexpr int PF = (HAS_R2 || R_F32) ? 4 : 8;
  constexpr uint32_t EOOB = 0x80000000u;
  const int cg = lane % LPR, rsub = lane / LPR;
  const int rows_valid = min(T::BM, op.M - m0);
  const int coln = n0 + wn * T::TN + cg * 8;                         // first of this lane's 8 columns
  const bool col_ok = coln < op.N;
  auto tile_rsrc = [&](const void* base, int64_t batch_off, int64_t ld, int esz) {
    const char* p = base ? (const char*)base + (batch_off + (int64_t)m0 * ld) * esz : nullptr;
    return __builtin_amdgcn_make_buffer_rsrc((void*)p, 0, base ? (uint32_t)rows_valid * (uint32_t)ld * (uint32_t)esz : 0u,
                                             0x00020000);
  };
  auto row_rsrc = [&](const float* base) {   // per-row fp32 scalars of the tile's rows
    return __builtin_amdgcn_make_buffer_rsrc((void*)(base ? base + m0 : nullptr), 0, base ? (uint32_t)rows_valid * 4u : 0u,
                                             0x00020000);
  };
  constexpr bool PARTIAL = KIND == EPI_PARTIAL;
  // C: bf16 [batch][M][ldc]; fp32 split-K partials: [batch * split][M][N]
  const __amdgpu_buffer_rsrc_t rsC = PARTIAL
      ? __builtin_amdgcn_make_buffer_rsrc((void*)((char*)op.C + ((int64_t)bz * op.M + m0) * op.N * 4), 0,
                                          (uint32_t)rows_valid * (uint32_t)op.N * 4u, 0x00020000)
      : tile_rsrc(op.C, (int64_t)bi * op.sC + (int64_t)bo * op.sCo, op.ldc, 2);
  const __amdgpu_buffer_rsrc_t rsC2 = tile_rsrc(PARTIAL ? nullptr : e.C2, (int64_t)b * e.sC2, e.ldc2, 2);
  const bool use_r = !PARTIAL && epi_reads_r<BASE>(e), use_r2 = !PARTIAL && epi_reads_r2<BASE>(e);
  const __amdgpu_buffer_rsrc_t rsR = tile_rsrc(use_r ? e.R : nullptr, (int64_t)b * e.sR, e.ldr, R_F32 ? 4 : 2);
  const __amdgpu_buffer_rsrc_t rsC32 = tile_rsrc(O32 ? e.C32 : nullptr, 0, e.ldc32, 4);
  const __amdgpu_buffer_rsrc_t rsR2 = tile_rsrc(use_r2 ? e.R2 : nullptr, (int64_t)b * e.sR2, e.ldr2, 2);
  const __amdgpu_buffer_rsrc_t rsRowA = row_rsrc((!PARTIAL && e.use_rho && !STAT_A) ? e.rowa : nullptr);
  const __amdgpu_buffer_rsrc_t rsRowB = row_rsrc(!PARTIAL ? e.rowb : nullptr);
  const int ldC = PARTIAL ? op.N * 4 : (int)op.ldc * 2;               // row pitches in bytes
  const int ldC2 = (int)e.ldc2 * 2, ldR = (int)e.ldr * (R_F32 ? 4 : 2), ldR2 = (int)e.ldr2 * 2, ldC32 = (int)e.ldc32 * 4;
  const uint32_t colC = col_ok ? (uint32_t)coln * (PARTIAL ? 4u : 2u) : EOOB, col2 = col_ok ? (uint32_t)coln * 2u : EOOB;
  const uint32_t col4 = col_ok ? (uint32_t)coln * 4u : EOOB;      // this lane's columns in an fp32 tile
  const bool want2 = KIND == EPI_SWIGLU_BWD || KIND == EPI_SWIGLU_FWD || KIND == EPI_DOWN_LAX || KIND == EPI_LAXGRAD ||
                     (KIND == EPI_DOWN && e.C2 != nullptr);
  const bool use_rho = !PARTIAL && e.use_rho;
  const bool rho_sqrt = e.rho_sqrt != 0;
  // row partials [M, rowpart_ld] and the statistic [M]: one lane per row writes, the others (and rows
  // past M) are given an out-of-range offset
  constexpr bool ROWPART = BASE == EPI_UP || BASE == EPI_ACTGRAD || BASE == EPI_LAXGRAD;
  const __amdgpu_buffer_rsrc_t rsPart = __builtin_amdgcn_make_buffer_rsrc(
      (void*)((ROWPART && e.rowpart) ? e.rowpart + (int64_t)m0 * e.rowpart_ld : nullptr), 0,
      (ROWPART && e.rowpart) ? (uint32_t)rows_valid * (uint32_t)e.rowpart_ld * 4u : 0u, 0x00020000);
  const int ldPart = ROWPART ? (int)e.rowpart_ld * 4 : 0;
  const uint32_t colPart = cg == 0 ? (uint32_t)(e.rowpart_off + b * (tiles_n * T::WN) + tn * T::WN + wn) * 4u : EOOB;
  const bool write_stat = STAT_A && e.stat_out && tn == 0 && wn == 0 && b == 0;
  const __amdgpu_buffer_rsrc_t rsStat = row_rsrc(write_stat ? e.stat_out : nullptr);
  const uint32_t colStat = cg == 0 ? 0u : EOOB;
  const int act = e.act;
  const float inv_d = e.inv_d, eps = e.eps;
  typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
  u32x4 auxr[PF], auxr2[PF], auxr3[R_F32 ? PF : 1];   // auxr3: columns 4..7 of an fp32 R tile
  auto row_of = [&](int q) { return wm * T::TM + (q / PPB) * 32 + (q % PPB) * RPP + rsub; };   // row inside the tile
  auto fetch = [&](int q, u32x4& ar, u32x4& ar2, u32x4& ar3) {
    const int lm = row_of(q);
    if constexpr (R_F32) {
      ar = __builtin_amdgcn_raw_buffer_load_b128(rsR, (int)((uint32_t)(lm * ldR) + col4), 0, 0);
      ar3 = __builtin_amdgcn_raw_buffer_load_b128(rsR, (int)((uint32_t)(lm * ldR) + col4 + 16u), 0, 0);
    } else if constexpr (HAS_R) {
      ar = __builtin_amdgcn_raw_buffer_load_b128(rsR, (int)((uint32_t)(lm * ldR) + col2), 0, 0);
    }
    if constexpr (HAS_R2) ar2 = __builtin_amdgcn_raw_buffer_load_b128(rsR2, (int)((uint32_t)(lm * ldR2) + col2), 0, 0);
  };
  static_for<PF>([&](auto Q) {
    constexpr int q = decltype(Q)::value;
    auxr[q] = u32x4{0u, 0u, 0u, 0u};
    auxr2[q] = u32x4{0u, 0u, 0u, 0u};
    if constexpr (R_F32) auxr3[q] = u32x4{0u, 0u, 0u, 0u};
    if constexpr (q < NQ) fetch(q, auxr[q], auxr2[q], auxr3[R_F32 ? q : 0]);
  });
  // per-row scalars of all passes, requested before the first pass
  float ssv[NQ], rbv[NQ];
  static_for<NQ>([&](auto Q) {
    constexpr int q = decltype(Q)::value;
    ssv[q] = 0.f;
    rbv[q] = 0.f;
    if constexpr (!PARTIAL && !STAT_A) {
      if (use_rho) ssv[q] = __uint_as_float(__builtin_amdgcn_raw_buffer_load_b32(rsRowA, row_of(q) * 4, 0, 0));
    }
    if constexpr (BASE == EPI_NORMBWD)
      rbv[q] = __uint_as_float(__builtin_amdgcn_raw_buffer_load_b32(rsRowB, row_of(q) * 4, 0, 0));
  });
  static_for<NQ>([&](auto Q) {
    constexpr int q = decltype(Q)::value;
    constexpr int i = q / PPB, p = q % PPB;
    if constexpr (p == 0) {
      static_for<T::FN>([&](auto J) {
        constexpr int j = decltype(J)::value;
        // the accumulators hold the transposed 32x32 block (the MFMA is issued with its operands
        // exchanged): lane -> row lane%32, registers 4g..4g+3 -> columns 8g + 4*(lane/32) + 0..3, so a lane
        // stages four consecutive columns with one 16-byte write
#pragma unroll
        for (int g = 0; g < 4; g++)
          *reinterpret_cast<float4*>(sC + (lane & 31) * T::CS + j * 32 + 8 * g + 4 * (lane >> 5)) =
              make_float4(acc[i][j][4 * g], acc[i][j][4 * g + 1], acc[i][j][4 * g + 2], acc[i][j][4 * g + 3]);
      });
      // No barrier: the staging region belongs to this wavefront alone and a wavefront's LDS
      // operations complete in order.
    }
    const int rl = p * RPP + rsub;
    const int lm = wm * T::TM + i * 32 + rl;      // row inside the block tile
    float v[8];
    {
      const float4 lo = *reinterpret_cast<const float4*>(sC + rl * T::CS + cg * 8);
      const float4 hi = *reinterpret_cast<const float4*>(sC + rl * T::CS + cg * 8 + 4);
      v[0] = lo.x; v[1] = lo.y; v[2] = lo.z; v[3] = lo.w;
      v[4] = hi.x; v[5] = hi.y; v[6] = hi.z; v[7] = hi.w;
    }
    if constexpr (PARTIAL) {
      const uint32_t off = (uint32_t)(lm * ldC) + colC;
      const u32x4 lo = {__float_as_uint(v[0]), __float_as_uint(v[1]), __float_as_uint(v[2]), __float_as_uint(v[3])};
      const u32x4 hi = {__float_as_uint(v[4]), __float_as_uint(v[5]), __float_as_uint(v[6]), __float_as_uint(v[7])};
      __builtin_amdgcn_raw_buffer_store_b128(lo, rsC, (int)off, 0, 0);
      __builtin_amdgcn_raw_buffer_store_b128(hi, rsC, (int)(off + 16u), 0, 0);
    } else {
      float rho = 1.f, rowb = 0.f;
      if (use_rho) {
        float ss;
        if constexpr (STAT_A) ss = sStat[lm];
        else ss = ssv[q];
        rho = rho_sqrt ? sqrtf(ss * inv_d + eps) : rsqrtf(ss * inv_d + eps);
      }
      if constexpr (BASE == EPI_NORMBWD) rowb = rbv[q];
      float r[8], r2[8], v2[8];
      if constexpr (R_F32) {
        const u32x4 a0 = auxr[q % PF], a1 = auxr3[q % PF];
        r[0] = __uint_as_float(a0.x); r[1] = __uint_as_float(a0.y); r[2] = __uint_as_float(a0.z); r[3] = __uint_as_float(a0.w);
        r[4] = __uint_as_float(a1.x); r[5] = __uint_as_float(a1.y); r[6] = __uint_as_float(a1.z); r[7] = __uint_as_float(a1.w);
      } else {
        unpack8(make_uint4(auxr[q % PF].x, auxr[q % PF].y, auxr[q % PF].z, auxr[q % PF].w), r);
      }
      unpack8(make_uint4(auxr2[q % PF].x, auxr2[q % PF].y, auxr2[q % PF].z, auxr2[q % PF].w), r2);
      float part = epi_math<8, BASE, true>(act, inv_d, want2, v, v2, rho, rowb, r, r2);
      if constexpr (O32) {
        const u32x4 lo = {__float_as_uint(v[0]), __float_as_uint(v[1]), __float_as_uint(v[2]), __float_as_uint(v[3])};
        const u32x4 hi = {__float_as_uint(v[4]), __float_as_uint(v[5]), __float_as_uint(v[6]), __float_as_uint(v[7])};
        const uint32_t off = (uint32_t)(lm * ldC32) + col4;
        __builtin_amdgcn_raw_buffer_store_b128(lo, rsC32, (int)off, 0, 0);
        __builtin_amdgcn_raw_buffer_store_b128(hi, rsC32, (int)(off + 16u), 0, 0);
      }
      {
        const uint4 o = pack8(v);
        const u32x4 ov = {o.x, o.y, o.z, o.w};
        __builtin_amdgcn_raw_buffer_store_b128(ov, rsC, (int)((uint32_t)(lm * ldC) + colC), 0, 0);
      }
      if (want2) {
        const uint4 o = pack8(v2);
        const u32x4 ov = {o.x, o.y, o.z, o.w};
        __builtin_amdgcn_raw_buffer_store_b128(ov, rsC2, (int)((uint32_t)(lm * ldC2) + col2), 0, 0);
      }
      if constexpr (q + PF < NQ) fetch(q + PF, auxr[q % PF], auxr2[q % PF], auxr3[R_F32 ? q % PF : 0]);
      if constexpr (ROWPART) {
        part = lane_group_sum<LPR>(part);
        __builtin_amdgcn_raw_buffer_store_b32(__float_as_uint(part), rsPart, (int)((uint32_t)(lm * ldPart) + colPart), 0, 0);
      }
      if constexpr (STAT_A)
        __builtin_amdgcn_raw_buffer_store_b32(__float_as_uint(sStat[lm]), rsStat, (int)((uint32_t)(lm * 4) + colStat), 0, 0);
    }
  });
}

// ---------------------------------------------------------------------------------------------
template <class T, int KIND, bool STAT_A, bool KM = false>
hipError_t launch(const GemmOp& op, hipStream_t st) {
  // one-time opt-in to > 64 KB of dynamic LDS for this instantiation (a function-local static: its
  // initialisation is thread-safe and runs once per process; a failure is reported by every launch)
  auto kern = gemm_bf16_kernel<T, KIND, STAT_A, KM>;
  static const hipError_t attr_err =
      hipFuncSetAttribute((const void*)kern, hipFuncAttributeMaxDynamicSharedMemorySize, T::LDS_BYTES);
  if (attr_err != hipSuccess) return attr_err;
  const int tiles_m = (op.M + T::BM - 1) / T::BM, tiles_n = (op.N + T::BN - 1) / T::BN;
  int kper = (op.K + op.splitk - 1) / op.splitk;
  kper = (kper + BK - 1) / BK * BK;
  dim3 grid(tiles_m * tiles_n, op.batch * op.splitk);
  hipLaunchKernelGGL(kern, grid, dim3(T::NT), T::LDS_BYTES, st, op, kper, tiles_m, tiles_n);
  return hipGetLastError();
}

using TileBig = Tile<256, 256, 4, 2>;   // 8 waves, 64x128 per wave
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
    case EPI_SWIGLU_FWD: return launch<T, EPI_SWIGLU_FWD, false>(op, st);
    case EPI_DOWN_LAX:
      return op.epi.stat_from_a ? launch<T, EPI_DOWN_LAX, true>(op, st) : launch<T, EPI_DOWN_LAX, false>(op, st);
    case EPI_LAXGRAD: return launch<T, EPI_LAXGRAD, false>(op, st);
    case EPI_UP_O32: return launch<T, EPI_UP_O32, false>(op, st);
    case EPI_UP_I32: return launch<T, EPI_UP_I32, false>(op, st);
    case EPI_NORMBWD_O32: return launch<T, EPI_NORMBWD_O32, false>(op, st);
    case EPI_NORMBWD_I32: return launch<T, EPI_NORMBWD_I32, false>(op, st);
    default: return hipErrorInvalidValue;
  }
}

// (A 128x128 tile of four wavefronts needs 80 KB of LDS, so two workgroups share a CU and one's epilogue
// could run under the other's main loop.  Measured on the 7B block it loses everywhere, 6-30 % per launch
// class, the classes with tile-reading epilogues included: it moves twice the operand bytes per FLOP
// through L2 and LDS, and that costs more than the overlap returns.)
bool use_big_tile(int N) { return N > 128 && (N % 256 == 0 || N > 512); }

}  // namespace

int gemm_bf16_rowpart_slabs(int N) {
  if (use_big_tile(N)) return (N + TileBig::BN - 1) / TileBig::BN * TileBig::WN;
  return (N + TileMid::BN - 1) / TileMid::BN * TileMid::WN;
}

int gemm_bf16_pick_splitk(int M, int N, int K, int batch) {
  // One workgroup per CU is resident at a time (LDS), so a launch runs in ceil(workgroups / 256)
  // rounds, each as long as one workgroup: its k-slices plus a fixed cost (pipeline fill, the fp32
  // partial tile it writes, its share of the fold) worth about 8 slices.  Pick the split count with
  // the smallest estimate; ties go to fewer splits (less partial traffic).
  const int bm = 256, bn = use_big_tile(N) ? 256 : 128;
  const long tiles = (long)((M + bm - 1) / bm) * ((N + bn - 1) / bn) * batch;
  const int nk = (K + BK - 1) / BK;
  const int maxs = nk >= 16 ? (nk / 8 < 64 ? nk / 8 : 64) : 1;   // at least 8 slices per split
  int best = 1;
  long best_cost = -1;
  for (int s = 1; s <= maxs; s++) {
    const long rounds = (tiles * s + 255) / 256;
    const long cost = rounds * ((nk + s - 1) / s + 8) * 16 + s;   // "+ s": the tie-break
    if (best_cost < 0 || cost < best_cost) { best_cost = cost; best = s; }
  }
  return best;
}

// ---- optional timing of launches (for the benchmark's roofline figures) --------------------------
// When enabled, every gemm_bf16 launch (and whatever else the sequencing code brackets with
// launch_timer_open / close) sits between two HIP events on its stream; the elapsed time between them is
// the time the stream spent in that launch.  Off by default; the events are created by launch_timer_begin
// and released when the session is read out, never on the compute path.  Process-global and not
// thread-safe: a measurement aid for a single-threaded benchmark, not part of the compute contract.
namespace {
struct LaunchTimer {
  bool on = false;
  std::vector<hipEvent_t> ev;
  std::vector<lr_launch_record> rec;
  size_t used = 0;
} g_timer;

void timer_release() {
  for (auto& e : g_timer.ev)
    if (e) (void)hipEventDestroy(e);
  g_timer.ev.clear();
  g_timer.rec.clear();
  g_timer.used = 0;
  g_timer.on = false;
}
}  // namespace

int launch_timer_begin(int max_launches) {
  if (g_timer.on || max_launches <= 0) return -1;
  g_timer.ev.assign((size_t)max_launches * 2, nullptr);
  for (auto& e : g_timer.ev)
    if (hipEventCreate(&e) != hipSuccess) {
      e = nullptr;
      timer_release();          // destroys the events created so far
      return -1;
    }
  g_timer.rec.assign((size_t)max_launches, lr_launch_record{});
  g_timer.used = 0;
  g_timer.on = true;
  return 0;
}

int launch_timer_open(int tag, int M, int N, int K, int batch, double flops, hipStream_t st) {
  if (!g_timer.on || g_timer.used >= g_timer.rec.size()) return -1;
  const int slot = (int)g_timer.used++;
  lr_launch_record& r = g_timer.rec[slot];
  r.tag = tag; r.M = M; r.N = N; r.K = K; r.batch = batch; r.flops = flops; r.ms = 0.f;
  (void)hipEventRecord(g_timer.ev[2 * slot], st);
  return slot;
}

void launch_timer_close(int slot, hipStream_t st) {
  if (slot >= 0 && g_timer.on) (void)hipEventRecord(g_timer.ev[2 * slot + 1], st);
}

int launch_timer_end(lr_launch_record* out, int max_records, int* n_records) {
  if (!g_timer.on) return -1;
  const size_t n = g_timer.used;
  if (n > 0) (void)hipEventSynchronize(g_timer.ev[2 * n - 1]);
  int w = 0;
  for (size_t i = 0; i < n; i++) {
    float ms = 0.f;
    (void)hipEventElapsedTime(&ms, g_timer.ev[2 * i], g_timer.ev[2 * i + 1]);
    g_timer.rec[i].ms = ms;
    if (out && w < max_records) out[w++] = g_timer.rec[i];
  }
  if (n_records) *n_records = (int)n;
  timer_release();
  return 0;
}

hipError_t gemm_bf16(const GemmOp& op, hipStream_t st) {
  if (!g_timer.on || op.M <= 0 || op.N <= 0 || op.batch <= 0) return gemm_bf16_untimed(op, st);
  const int tag = op.splitk > 1 ? (int)EPI_PARTIAL : op.epi.kind;
  const int slot = launch_timer_open(tag, op.M, op.N, op.K, op.batch, 2.0 * op.M * op.N * (double)op.K * op.batch, st);
  hipError_t e = gemm_bf16_untimed(op, st);
  launch_timer_close(slot, st);
  return e;
}

bool gemm_bf16_kmajor_ok(const GemmOp& op) {
  // both operands k-major, fp32 partial output, offsets within the 2 GB a buffer resource addresses
  const bool wgrad = op.batch == 1 && op.epi.kind == EPI_PARTIAL;
  const bool plain = op.splitk == 1 && op.epi.kind == EPI_STORE;
  return op.transA && op.transB && (wgrad || plain) && op.M % 8 == 0 && op.N % 8 == 0 &&
         (int64_t)op.K * op.lda * 2 < 0x7fffffffLL && (int64_t)op.K * op.ldb * 2 < 0x7fffffffLL;
}

hipError_t gemm_bf16_untimed(const GemmOp& op, hipStream_t st) {
  if (op.M <= 0 || op.N <= 0 || op.batch <= 0) return hipSuccess;
  if (op.transA && op.transB) {
    if (!gemm_bf16_kmajor_ok(op)) return hipErrorInvalidValue;
    if (op.epi.kind == EPI_STORE && op.splitk == 1) {
      if (use_big_tile(op.N)) return launch<TileBig, EPI_STORE, false, true>(op, st);
      return launch<TileMid, EPI_STORE, false, true>(op, st);
    }
    if (use_big_tile(op.N)) return launch<TileBig, EPI_PARTIAL, false, true>(op, st);
    return launch<TileMid, EPI_PARTIAL, false, true>(op, st);
  }
  if (op.transA || op.transB) return hipErrorInvalidValue;
  if (op.epi.stat_from_a && op.splitk > 1) return hipErrorInvalidValue;
  if (use_big_tile(op.N)) return dispatch<TileBig>(op, st);
  return dispatch<TileMid>(op, st);
}

}  // namespace lrb
