// Causal multi-head attention, head_dim 128, bf16 in / fp32 softmax, for gfx950.
//
// Forward (one workgroup = 4 wavefronts x 32 queries of one (batch, head), for one query block and
// its causal mirror; K/V stream through LDS in 64-key tiles, double buffered):
//   S^T = K Q^T      MFMA, A = K rows from LDS, B = Q rows kept in registers for the whole kernel
//   online softmax   per query = per lane column of the S^T accumulators (one cross-half shuffle)
//   O^T += V^T P^T   MFMA, B = P^T straight from the softmax registers, A = V^T through the LDS
//                    transpose read (ds_read_b64_tr_b16), so V is stored as it arrives: [key][h]
// Working on the transposed problem is what lets the probabilities feed the second MFMA without
// leaving registers: the 32x32 accumulator layout (lane = column, 16 rows in 4-row groups) is, up
// to a fixed permutation of the k slots that the V^T loads follow, the B-operand layout.
//
// Backward, free of atomics and therefore deterministic, with D[q] = sum_h dO[q,h] O[q,h] and
// lse * log2(e) from a small preprocessing kernel:
//   dkv kernel - workgroup owns 128 keys, streams 64-query tiles from the diagonal on:
//                S = Q K^T, dP = dO V^T, dV^T += dO^T P, dK^T += Q^T dS;
//                in its usual form it also stores scale * dS^T (bf16, [key][query] per (batch, head)),
//                and dQ = (scale dS^T)^T K is then one causal k-major GEMM (gemm_bf16.hip): the scores
//                are formed once, 5 GEMM units in all
//   dq kernel  - the form without that workspace (S not a multiple of 8, or too large): same walk as the
//                forward (workgroup owns queries, streams keys): S^T, dP^T = V dO^T,
//                dS^T = P^T*(dP^T - D), dQ^T += K^T dS^T; 7 units together with the dkv kernel
//
// Grouped-query form (fewer key / value heads than query heads, H / Hkv consecutive query heads per
// key / value head): the same kernels with K and V addressed by head / group and their own row stride.
// The dkv kernel then writes one dK and one dV contribution per query head into the workspace and a
// last kernel adds up each group; the dQ GEMM runs per batch element with (key / value head, head in
// group) as its two batch levels.  Multi-head attention is the case of groups of one.
#include "common.h"

namespace lrb {
namespace {

constexpr int HD = 128;
constexpr int KT = 64;            // keys (or queries, in the dkv kernel) per streamed tile
constexpr float LOG2E = 1.4426950408889634f;

typedef short s16x4 __attribute__((ext_vector_type(4)));

// raw v_exp_f32 (2^x): the arguments here are differences to a running maximum, never denormal-critical
__device__ __forceinline__ float fast_exp2(float x) { return __builtin_amdgcn_exp2f(x); }

__device__ __forceinline__ bf16x8 lds_b128(const unsigned char* p) { return *reinterpret_cast<const bf16x8*>(p); }

// 8 consecutive accumulator values (v = t*8 .. t*8+7) packed as the bf16 B operand of one k16 step.
__device__ __forceinline__ bf16x8 pack_acc_half(const f32x16& a, int t) {
  uint4 q;
  q.x = pack_bf16x2(a[t * 8 + 0], a[t * 8 + 1]);
  q.y = pack_bf16x2(a[t * 8 + 2], a[t * 8 + 3]);
  q.z = pack_bf16x2(a[t * 8 + 4], a[t * 8 + 5]);
  q.w = pack_bf16x2(a[t * 8 + 6], a[t * 8 + 7]);
  return __builtin_bit_cast(bf16x8, q);
}

// Row index of accumulator element v inside a 32-row block.
__device__ __forceinline__ int acc_row(int v, int lane) { return 8 * (v >> 2) + 4 * (lane >> 5) + (v & 3); }

// Query-row fragments kept in registers: B operand (rows = queries) for all 8 k16 steps over h.
template <int MB>
__device__ __forceinline__ void load_row_frags(bf16x8 (&f)[MB][8], const uint16_t* base, int64_t ld, int row0,
                                               int nrows, int lane) {
#pragma unroll
  for (int mb = 0; mb < MB; mb++) {
    const int row = row0 + mb * 32 + (lane & 31);
    const bool ok = row < nrows;
#pragma unroll
    for (int ks = 0; ks < 8; ks++) {
      uint4 q = ok ? *reinterpret_cast<const uint4*>(base + (int64_t)row * ld + ks * 16 + (lane >> 5) * 8)
                   : make_uint4(0, 0, 0, 0);
      f[mb][ks] = __builtin_bit_cast(bf16x8, q);
    }
  }
}

// Writes a transposed accumulator block set acc[hb][.] (rows = h, column = the lane's token) as
// out[token][h], 4 consecutive h (8 bytes) at a time, scaled by `mul`.
__device__ __forceinline__ void store_acc_T(uint16_t* out_row, const f32x16 (&acc)[4], float mul, int lane) {
#pragma unroll
  for (int hb = 0; hb < 4; hb++)
#pragma unroll
    for (int g4 = 0; g4 < 4; g4++) {
      const int h = hb * 32 + 8 * g4 + 4 * (lane >> 5);
      uint2 w;
      w.x = pack_bf16x2(acc[hb][g4 * 4 + 0] * mul, acc[hb][g4 * 4 + 1] * mul);
      w.y = pack_bf16x2(acc[hb][g4 * 4 + 2] * mul, acc[hb][g4 * 4 + 3] * mul);
      *reinterpret_cast<uint2*>(out_row + h) = w;
    }
}

// ----------------------------------------------------------------------------------------------
// 64-row x 128-column bf16 tiles moved global -> LDS without passing through registers.
// One buffer_load_dwordx4 ... lds per wavefront writes 1 KB = 4 tile rows of 256 bytes; lane L's 16
// bytes land at base + 16 L, i.e. row L/16, physical chunk L%16.  Rows are not padded; instead the
// 16-byte chunks of a row are XOR-swizzled and each lane fetches the logical chunk that belongs in its
// slot.  Two swizzles, one per read pattern:
//   SWZ_ROW16  chunk ^ (row % 16)        16 consecutive rows x one logical chunk (ds_read_b128 of
//                                        MFMA operand rows) cover all 64 banks
//   SWZ_ROW4   chunk ^ ((row % 4) * 4)   4 consecutive rows x 64 bytes (the LDS transpose read)
//                                        cover all 64 banks
// Rows at or past `nrows` are fetched with an out-of-range offset: the load returns zeros.
// ----------------------------------------------------------------------------------------------
constexpr int TILE_BYTES = KT * HD * 2;
constexpr uint32_t DMA_OOB = 0x80000000u;
enum { SWZ_ROW16 = 0, SWZ_ROW4 = 1, SWZ_BOTH = 2 };
//   SWZ_BOTH   chunk ^ ((row % 4) * 4 + (row / 4) % 4)   serves both read patterns of a tile that is
//                                        needed row-wise and transposed: 16 consecutive rows see 16
//                                        different terms, 4 consecutive rows 4 different 64-byte groups
#define LRB_LDS_PTR(p) ((__attribute__((address_space(3))) void*)(p))

// Buffer resource as four scalar words: base address, stride 0, size in bytes, data format word.
typedef uint32_t rsrc_t __attribute__((ext_vector_type(4)));
__device__ __forceinline__ rsrc_t make_rsrc(const void* base, uint32_t bytes) {
  const uint64_t a = (uint64_t)(uintptr_t)base;
  rsrc_t r = {(uint32_t)a, (uint32_t)(a >> 32) & 0xffffu, bytes, 0x00020000u};
  return r;
}
__device__ __forceinline__ rsrc_t tile_rsrc(const uint16_t* base) { return make_rsrc(base, 0x7fffffffu); }

// One global -> LDS load of BYTES (4 or 16) per lane: lane L's data lands at lds + BYTES * L.  Issued
// as inline assembly on purpose: through the builtin the compiler treats every later LDS read as a
// possible read of this load's destination and makes it wait for ALL global loads in flight, i.e. the
// tile being worked on would wait for the next tile's loads.  Completion is tracked by hand instead
// (wait_vm0 before the barrier that publishes a tile).  `lds` must be wavefront-uniform.
template <int BYTES>
__device__ __forceinline__ void lds_dma(rsrc_t rs, const unsigned char* lds, uint32_t voff) {
  const uint32_t m0v = __builtin_amdgcn_readfirstlane((uint32_t)(uintptr_t)LRB_LDS_PTR(lds));
  if constexpr (BYTES == 16)
    asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tbuffer_load_dwordx4 %1, %2, 0 offen lds" ::"s"(m0v), "v"(voff), "s"(rs) : "memory");
  else
    asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tbuffer_load_dword %1, %2, 0 offen lds" ::"s"(m0v), "v"(voff), "s"(rs) : "memory");
}

// Per-lane byte offsets (row * ld + logical chunk) of the 16 / NW wavefront loads that a wavefront of
// an NW-wavefront workgroup contributes to one tile.
template <int SWZ, int NL>
__device__ __forceinline__ void dma_lane_offsets(uint32_t (&off)[NL], int (&row)[NL], int64_t ld, int wave, int lane) {
  constexpr int NW = 16 / NL;
#pragma unroll
  for (int i = 0; i < NL; i++) {
    const int r = (i * NW + wave) * 4 + (lane >> 4);
    const int pc = lane & 15;
    const int lc = SWZ == SWZ_ROW16 ? (pc ^ (r & 15))
                 : SWZ == SWZ_ROW4 ? (pc ^ ((r & 3) << 2))
                                   : (pc ^ (((r & 3) << 2) | ((r >> 2) & 3)));
    row[i] = r;
    off[i] = (uint32_t)(r * (int)ld + lc * 8) * 2u;
  }
}
template <int NL>
__device__ __forceinline__ void dma_tile(rsrc_t rs, unsigned char* tile, const uint32_t (&off)[NL],
                                         const int (&row)[NL], int row0, int nrows, int64_t ld, int wave) {
  constexpr int NW = 16 / NL;
  const uint32_t base = (uint32_t)row0 * (uint32_t)ld * 2u;
#pragma unroll
  for (int i = 0; i < NL; i++) {
    const uint32_t o = (row0 + row[i]) < nrows ? base + off[i] : DMA_OOB;
    lds_dma<16>(rs, tile + (i * NW + wave) * 1024, o);
  }
}
// s_waitcnt vmcnt(0) alone (gfx9 encoding), and lgkmcnt(0) alone
__device__ __forceinline__ void wait_vm0() { __builtin_amdgcn_s_waitcnt(0x0f70); }
// s_waitcnt vmcnt(N) alone, N < 64: bits 3:0 and 15:14 hold vmcnt, the other counters stay at "no wait"
template <int N>
__device__ __forceinline__ void wait_vm() {
  static_assert(N >= 0 && N < 64, "vmcnt is a 6-bit counter");
  __builtin_amdgcn_s_waitcnt(0x0f70 | (N & 15) | ((N >> 4) << 14));
}

// A operand (32 rows = tile rows r0 + lane%32, k slots = logical chunk ks*2 + lane/32) from a
// SWZ_ROW16 tile.  r0 is a multiple of 16, so the swizzle term depends on the lane only.
__device__ __forceinline__ bf16x8 swz_row_frag(const unsigned char* tile, int r0, int ks, int lane) {
  const int row = r0 + (lane & 31);
  return lds_b128(tile + row * 256 + (((ks * 2 + (lane >> 5)) ^ (lane & 15)) << 4));
}
// Transposed A operand from a SWZ_ROW4 tile stored [k][col]: rows = columns c0..c0+31 (c0 a multiple
// of 32), k slots (half = lane / 32, e = 0..7) = tile rows k0 + (e/4)*8 + half*4 + e%4 (k0 a multiple
// of 16), which is the row order of a 32x32 accumulator.  Inside each group of 16 lanes the transpose
// read hands lane i the i-th 16-bit column of the 4 x 16 block that the 16 lanes fetched as 4 rows x
// 4 lanes x 8 bytes.
__device__ __forceinline__ bf16x8 swz_tr_frag(const unsigned char* tile, int k0, int c0, int lane) {
  const int g = lane >> 4, s = lane & 15;
  const int rl = (g >> 1) * 4 + (s >> 2);                       // row inside the 16-row group; rl % 4 = s / 4
  const int chunk = (c0 >> 3) + (g & 1) * 2 + ((s & 3) >> 1);   // logical 16-byte chunk
  const unsigned char* p0 = tile + (k0 + rl) * 256 + ((chunk ^ ((s >> 2) << 2)) << 4) + (s & 1) * 8;
  const unsigned char* p1 = p0 + 8 * 256;
  s16x4 lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16((s16x4 __attribute__((address_space(3)))*)(p0));
  s16x4 hi = __builtin_amdgcn_ds_read_tr16_b64_v4i16((s16x4 __attribute__((address_space(3)))*)(p1));
  typedef short s16x8 __attribute__((ext_vector_type(8)));
  s16x8 r = {lo[0], lo[1], lo[2], lo[3], hi[0], hi[1], hi[2], hi[3]};
  return __builtin_bit_cast(bf16x8, r);
}

// The same two operand reads for a SWZ_BOTH tile (r0 and k0 multiples of 16, c0 a multiple of 32).
__device__ __forceinline__ bf16x8 both_row_frag(const unsigned char* tile, int r0, int ks, int lane) {
  const int l31 = lane & 31;
  const int f = ((l31 & 3) << 2) | ((l31 >> 2) & 3);
  return lds_b128(tile + (r0 + l31) * 256 + (((ks * 2 + (lane >> 5)) ^ f) << 4));
}
__device__ __forceinline__ bf16x8 both_tr_frag(const unsigned char* tile, int k0, int c0, int lane) {
  const int g = lane >> 4, s = lane & 15;
  const int rl = (g >> 1) * 4 + (s >> 2);
  const int f0 = ((s >> 2) << 2) | (g >> 1);                    // rows k0 + rl; rows + 8 flip bit 1 of the term
  const int chunk = (c0 >> 3) + (g & 1) * 2 + ((s & 3) >> 1);
  const unsigned char* rowp = tile + (k0 + rl) * 256 + (s & 1) * 8;
  s16x4 lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16((s16x4 __attribute__((address_space(3)))*)(rowp + ((chunk ^ f0) << 4)));
  s16x4 hi = __builtin_amdgcn_ds_read_tr16_b64_v4i16(
      (s16x4 __attribute__((address_space(3)))*)(rowp + 8 * 256 + ((chunk ^ f0 ^ 2) << 4)));
  typedef short s16x8 __attribute__((ext_vector_type(8)));
  s16x8 r = {lo[0], lo[1], lo[2], lo[3], hi[0], hi[1], hi[2], hi[3]};
  return __builtin_bit_cast(bf16x8, r);
}

// The hardware deals consecutive workgroup ids to the 8 XCDs in rotation.  This maps the id back so
// that each XCD works through a contiguous range of (batch, head, block) triples, block fastest: the
// workgroups that stream the same head's K / V (or Q / dO) tiles then share one XCD's L2 instead of
// every XCD fetching every head.
struct WgCoord { int x, head, b; };
__device__ __forceinline__ WgCoord wg_coord() {
  const int nx = gridDim.x, H = gridDim.y;
  const int total = nx * H * (int)gridDim.z;
  const int lin = (int)blockIdx.x + nx * ((int)blockIdx.y + H * (int)blockIdx.z);
  const int xcd = lin % 8, loc = lin / 8;
  const int base = total / 8, rem = total % 8;
  const int v = xcd * base + (xcd < rem ? xcd : rem) + loc;
  WgCoord c;
  c.x = v % nx;
  c.head = (v / nx) % H;
  c.b = v / (nx * H);
  return c;
}

constexpr int FWD_LDS = 4 * TILE_BYTES;   // K and V, double buffered

// ----------------------------------------------------------------------------------------------
// forward
// ----------------------------------------------------------------------------------------------
template <int MB>
__global__ __launch_bounds__(256, 2) void attn_fwd_kernel(const uint16_t* __restrict__ q, const uint16_t* __restrict__ k,
                                                       const uint16_t* __restrict__ v, uint16_t* __restrict__ o,
                                                       float* __restrict__ lse, int64_t ld, int64_t ldkv, int grp, int S,
                                                       int H, float scale) {
  static_assert(MB == 1, "one 32-query block per wavefront");
  extern __shared__ __attribute__((aligned(16))) unsigned char smem[];
  constexpr int BQ = 4 * MB * 32;
  // (here the wavefront index stays a vector value: as a scalar it costs this kernel 13 more spilled
  // registers; only the LDS destinations of the global->LDS loads use a scalar copy)
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int wave_s = __builtin_amdgcn_readfirstlane(wave);
  const int nqb = (S + BQ - 1) / BQ;
  const WgCoord wg = wg_coord();
  const int head = wg.head, b = wg.b;
  const int64_t tok0 = (int64_t)b * S;
  const uint16_t* qb = q + tok0 * ld + head * HD;
  // grouped-query attention: grp consecutive query heads share key / value head head / grp (rows of ldkv)
  const int kvh = head / grp;
  const rsrc_t rsK = tile_rsrc(k + tok0 * ldkv + kvh * HD);
  const rsrc_t rsV = tile_rsrc(v + tok0 * ldkv + kvh * HD);
  const float c = scale * LOG2E;
  uint32_t offK[4], offV[4];
  int rowK[4], rowV[4];
  dma_lane_offsets<SWZ_ROW16, 4>(offK, rowK, ldkv, wave, lane);
  dma_lane_offsets<SWZ_ROW4, 4>(offV, rowV, ldkv, wave, lane);
  unsigned char* sK = smem;                              // 2 tiles
  unsigned char* sV = smem + 2 * TILE_BYTES;             // 2 tiles

  // Causal work grows linearly with the query block index.  Every workgroup takes one block from the
  // late end and its mirror image from the early end, so that all workgroups of the launch do the
  // same amount of work (the hardware deals workgroups to the XCDs in strict rotation: unequal
  // workgroups leave most of the chip waiting for the XCD that drew the heavy ones).
  for (int pass = 0; pass < 2; pass++) {
  const int qblk = pass == 0 ? nqb - 1 - wg.x : wg.x;
  if (pass == 1 && qblk >= nqb - 1 - wg.x) break;   // odd block count: the middle block has no mirror
  const int q0 = qblk * BQ;
  const int qw0 = q0 + wave * MB * 32;                   // first query of this wavefront

  bf16x8 qf[MB][8];
  load_row_frags<MB>(qf, qb, ld, qw0, S, lane);

  f32x16 oacc[4];
  float mrun = -INFINITY, lrun = 0.f;
#pragma unroll
  for (int hb = 0; hb < 4; hb++)
#pragma unroll
    for (int e = 0; e < 16; e++) oacc[hb][e] = 0.f;

  const int kv_end = min(S, q0 + BQ);                    // causal: keys up to the block's last query
  const int ntiles = (kv_end + KT - 1) / KT;

  dma_tile(rsK, sK, offK, rowK, 0, S, ldkv, wave_s);
  dma_tile(rsV, sV, offV, rowV, 0, S, ldkv, wave_s);
  wait_vm0();
  __syncthreads();

  for (int j = 0; j < ntiles; j++) {
    const int cur = j & 1;
    if (j + 1 < ntiles) {                                // next tiles land while this one is worked on
      dma_tile(rsK, sK + (cur ^ 1) * TILE_BYTES, offK, rowK, (j + 1) * KT, S, ldkv, wave_s);
      dma_tile(rsV, sV + (cur ^ 1) * TILE_BYTES, offV, rowV, (j + 1) * KT, S, ldkv, wave_s);
    }
    const int key0 = j * KT;
    const unsigned char* sKc = sK + cur * TILE_BYTES;
    const unsigned char* sVc = sV + cur * TILE_BYTES;
    if (key0 <= qw0 + MB * 32 - 1) {                     // this wavefront still has unmasked keys here
      // ---- S^T[n][m] for 64 keys x 32 queries: all 16 operand reads are issued up front, so the LDS
      //      latency is paid once per tile and not once per MFMA pair ----
      bf16x8 kf[8][2];
#pragma unroll
      for (int ks = 0; ks < 8; ks++)
#pragma unroll
        for (int nb = 0; nb < 2; nb++) kf[ks][nb] = swz_row_frag(sKc, nb * 32, ks, lane);
      __builtin_amdgcn_sched_barrier(0);
      f32x16 st[2];
#pragma unroll
      for (int nb = 0; nb < 2; nb++)
#pragma unroll
        for (int e = 0; e < 16; e++) st[nb][e] = 0.f;
#pragma unroll
      for (int ks = 0; ks < 8; ks++)
#pragma unroll
        for (int nb = 0; nb < 2; nb++)
          st[nb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(kf[ks][nb], qf[0][ks], st[nb], 0, 0, 0);
      // first half of the V^T operands: in flight during the softmax
      bf16x8 vf[2][4];
#pragma unroll
      for (int t = 0; t < 2; t++)
#pragma unroll
        for (int hb = 0; hb < 4; hb++) vf[t][hb] = swz_tr_frag(sVc, t * 16, hb * 32, lane);
      __builtin_amdgcn_sched_barrier(0);
      if ((key0 + KT - 1 > qw0) || (key0 + KT > S)) {    // wavefront-uniform: diagonal / tail tile
        asm volatile("" ::: "memory");                   // a real branch: the selects are not to be speculated
        const int qi = qw0 + (lane & 31);
#pragma unroll
        for (int nb = 0; nb < 2; nb++)
#pragma unroll
          for (int e = 0; e < 16; e++) {
            const int key = key0 + nb * 32 + acc_row(e, lane);
            st[nb][e] = (key > qi || key >= S) ? -INFINITY : st[nb][e];
          }
      }
      float mx = -INFINITY;
#pragma unroll
      for (int nb = 0; nb < 2; nb++)
#pragma unroll
        for (int e = 0; e < 16; e++) mx = fmaxf(mx, st[nb][e]);
      mx = fmaxf(mx, __shfl_xor(mx, 32));
      const float mnew = fmaxf(mrun, mx);                // finite: key 0 is visible to every query
      const float alpha = fast_exp2((mrun - mnew) * c);
      mrun = mnew;
      const float mc = mnew * c;
      float rs = 0.f;
#pragma unroll
      for (int nb = 0; nb < 2; nb++)
#pragma unroll
        for (int e = 0; e < 16; e++) {
          const float p = fast_exp2(fmaf(st[nb][e], c, -mc));
          st[nb][e] = p;
          rs += p;
        }
      lrun = lrun * alpha + rs;
      // the running maximum settles after the first tiles: skip the rescale when no lane needs it
      if (__builtin_amdgcn_ballot_w64(alpha != 1.f) != 0) {
#pragma unroll
        for (int hb = 0; hb < 4; hb++)
#pragma unroll
          for (int e = 0; e < 16; e++) oacc[hb][e] *= alpha;
      }
      // ---- O^T += V^T P^T ----
#pragma unroll
      for (int nb = 0; nb < 2; nb++) {
        bf16x8 vn[2][4];
        if (nb == 0) {                                   // second half of the operands, during the first half's MFMAs
#pragma unroll
          for (int t = 0; t < 2; t++)
#pragma unroll
            for (int hb = 0; hb < 4; hb++) vn[t][hb] = swz_tr_frag(sVc, 32 + t * 16, hb * 32, lane);
        }
#pragma unroll
        for (int t = 0; t < 2; t++) {
          const bf16x8 pf = pack_acc_half(st[nb], t);
#pragma unroll
          for (int hb = 0; hb < 4; hb++)
            oacc[hb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(vf[t][hb], pf, oacc[hb], 0, 0, 0);
        }
        if (nb == 0) {
#pragma unroll
          for (int t = 0; t < 2; t++)
#pragma unroll
            for (int hb = 0; hb < 4; hb++) vf[t][hb] = vn[t][hb];
        }
      }
    }
    wait_vm0();
    __syncthreads();
  }

  {
    const int qi = qw0 + (lane & 31);
    const float l = lrun + __shfl_xor(lrun, 32);
    if (qi < S) {
      store_acc_T(o + (tok0 + qi) * ld + head * HD, oacc, 1.f / l, lane);
      if (lane < 32) lse[((int64_t)b * H + head) * S + qi] = mrun * scale + logf(l);
    }
  }
  }  // pass
}

// ----------------------------------------------------------------------------------------------
// D[b, head, q] = sum_h dO[q, h] * O[q, h] : 16 lanes per (token, head); also lse2 = lse * log2(e)
// ----------------------------------------------------------------------------------------------
__global__ __launch_bounds__(256) void attn_dot_kernel(const uint16_t* __restrict__ dout, const uint16_t* __restrict__ o,
                                                       const float* __restrict__ lse, float* __restrict__ D,
                                                       float* __restrict__ lse2, int64_t ld, int S, int H,
                                                       int64_t total) {
  const int64_t item = ((int64_t)blockIdx.x * 256 + threadIdx.x) >> 4;   // (token, head) pair
  const int sub = threadIdx.x & 15;
  float s = 0.f;
  int64_t tok = 0;
  int head = 0;
  if (item < total) {
    tok = item / H;
    head = (int)(item % H);
    const int64_t off = tok * ld + head * HD + sub * 8;
    float a[8], bb[8];
    unpack8(*reinterpret_cast<const uint4*>(dout + off), a);
    unpack8(*reinterpret_cast<const uint4*>(o + off), bb);
#pragma unroll
    for (int i = 0; i < 8; i++) s = fmaf(a[i], bb[i], s);
  }
  s += __shfl_xor(s, 1);
  s += __shfl_xor(s, 2);
  s += __shfl_xor(s, 4);
  s += __shfl_xor(s, 8);
  if (item < total && sub == 0) {
    const int64_t bidx = tok / S, qi = tok % S;
    D[(bidx * H + head) * S + qi] = s;
    lse2[(bidx * H + head) * S + qi] = lse[(bidx * H + head) * S + qi] * LOG2E;   // exponent offset in base 2
  }
}

// ----------------------------------------------------------------------------------------------
// backward, dQ: workgroup owns 4 x 32 queries, streams 64-key tiles of K and V
// ----------------------------------------------------------------------------------------------
template <int MB>
__global__ __launch_bounds__(256) void attn_bwd_dq_kernel(const uint16_t* __restrict__ q, const uint16_t* __restrict__ k,
                                                          const uint16_t* __restrict__ v,
                                                          const uint16_t* __restrict__ dout,
                                                          const float* __restrict__ lse2, const float* __restrict__ D,
                                                          uint16_t* __restrict__ dq, int64_t ld, int64_t ldkv, int grp, int S, int H,
                                                          float scale) {
  extern __shared__ __attribute__((aligned(16))) unsigned char smem[];
  constexpr int BQ = 4 * MB * 32;
  // the wavefront index as a scalar: everything derived from it (LDS slots, tile rows) is scalar arithmetic
  const int tid = threadIdx.x, lane = tid & 63, wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int nqb = (S + BQ - 1) / BQ;
  const WgCoord wg = wg_coord();
  const int head = wg.head, b = wg.b;
  const int64_t tok0 = (int64_t)b * S;
  const int64_t hoff = head * HD;
  const float c = scale * LOG2E;
  // K is needed row-wise (S^T) and transposed (dQ^T), V row-wise (dP^T): one LDS copy each, in the
  // swizzle that serves both reads, written by direct-to-LDS loads.
  const int64_t kvoff = (head / grp) * HD;     // the key / value head this query head's group shares
  const rsrc_t rsK = tile_rsrc(k + tok0 * ldkv + kvoff);
  const rsrc_t rsV = tile_rsrc(v + tok0 * ldkv + kvoff);
  uint32_t offT[4];
  int rowT[4];
  dma_lane_offsets<SWZ_BOTH, 4>(offT, rowT, ldkv, wave, lane);
  // one query block from the late end and its mirror image from the early end: equal work per workgroup
  for (int pass = 0; pass < 2; pass++) {
  const int qblk = pass == 0 ? nqb - 1 - wg.x : wg.x;
  if (pass == 1 && qblk >= nqb - 1 - wg.x) break;
  const int q0 = qblk * BQ;
  const int qw0 = q0 + wave * MB * 32;

  // Q and dO rows of this wavefront stay in registers (B operands); every K / V fragment read from
  // LDS then feeds MB MFMAs.
  bf16x8 qf[MB][8], dof[MB][8];
  load_row_frags<MB>(qf, q + tok0 * ld + hoff, ld, qw0, S, lane);
  load_row_frags<MB>(dof, dout + tok0 * ld + hoff, ld, qw0, S, lane);
  float lsq[MB], Dq[MB];
#pragma unroll
  for (int mb = 0; mb < MB; mb++) {
    const int qi = qw0 + mb * 32 + (lane & 31);
    const int64_t sidx = ((int64_t)b * H + head) * S + min(qi, S - 1);
    lsq[mb] = lse2[sidx];
    Dq[mb] = D[sidx];
  }

  f32x16 acc[MB][4];
#pragma unroll
  for (int mb = 0; mb < MB; mb++)
#pragma unroll
    for (int hb = 0; hb < 4; hb++)
#pragma unroll
      for (int e = 0; e < 16; e++) acc[mb][hb][e] = 0.f;

  constexpr int STAGE = 2 * TILE_BYTES;                  // K, V
  const int kv_end = min(S, q0 + BQ);
  const int ntiles = (kv_end + KT - 1) / KT;
  dma_tile<4>(rsK, smem, offT, rowT, 0, S, ldkv, wave);
  dma_tile<4>(rsV, smem + TILE_BYTES, offT, rowT, 0, S, ldkv, wave);
  wait_vm0();
  __syncthreads();

  for (int j = 0; j < ntiles; j++) {
    const int cur = j & 1;
    if (j + 1 < ntiles) {                                // lands while this tile is worked on
      dma_tile<4>(rsK, smem + (cur ^ 1) * STAGE, offT, rowT, (j + 1) * KT, S, ldkv, wave);
      dma_tile<4>(rsV, smem + (cur ^ 1) * STAGE + TILE_BYTES, offT, rowT, (j + 1) * KT, S, ldkv, wave);
    }
    const unsigned char* sK = smem + cur * STAGE;
    const unsigned char* sVb = sK + TILE_BYTES;
    const int key0 = j * KT;
    // one 32-key block at a time; blocks entirely after this wavefront's queries are skipped
#pragma unroll 1
    for (int nb = 0; nb < 2; nb++) {
      const int kb0 = key0 + nb * 32;
      if (kb0 > qw0 + MB * 32 - 1 || kb0 >= S) continue;
      f32x16 st[MB], dp[MB];
#pragma unroll
      for (int mb = 0; mb < MB; mb++)
#pragma unroll
        for (int e = 0; e < 16; e++) { st[mb][e] = 0.f; dp[mb][e] = 0.f; }
#pragma unroll
      for (int ks = 0; ks < 8; ks++) {
        const bf16x8 kfr = both_row_frag(sK, nb * 32, ks, lane), vfr = both_row_frag(sVb, nb * 32, ks, lane);
#pragma unroll
        for (int mb = 0; mb < MB; mb++) {
          st[mb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(kfr, qf[mb][ks], st[mb], 0, 0, 0);
          dp[mb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(vfr, dof[mb][ks], dp[mb], 0, 0, 0);
        }
      }
      // dS^T = P^T * (dP^T - D), masked on the diagonal / tail blocks only
      const bool need_mask = (kb0 + 31 > qw0) || (kb0 + 32 > S);
      auto elements = [&](auto MASKED) {   // one wavefront-uniform branch around two copies of the loop
#pragma unroll
        for (int mb = 0; mb < MB; mb++) {
          const int qi = qw0 + mb * 32 + (lane & 31);
#pragma unroll
          for (int e = 0; e < 16; e++) {
            float p = fast_exp2(fmaf(st[mb][e], c, -lsq[mb]));
            if constexpr (decltype(MASKED)::value) {
              const int key = kb0 + acc_row(e, lane);
              p = (key > qi || key >= S) ? 0.f : p;
            }
            st[mb][e] = p * (dp[mb][e] - Dq[mb]);
          }
        }
      };
      if (need_mask) {
        asm volatile("" ::: "memory");
        elements(std::true_type{});
      } else {
        elements(std::false_type{});
      }
#pragma unroll
      for (int t = 0; t < 2; t++) {
        bf16x8 dsf[MB];
#pragma unroll
        for (int mb = 0; mb < MB; mb++) dsf[mb] = pack_acc_half(st[mb], t);
#pragma unroll
        for (int hb = 0; hb < 4; hb++) {
          const bf16x8 ktf = both_tr_frag(sK, nb * 32 + t * 16, hb * 32, lane);
#pragma unroll
          for (int mb = 0; mb < MB; mb++)
            acc[mb][hb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(ktf, dsf[mb], acc[mb][hb], 0, 0, 0);
        }
      }
    }
    wait_vm0();
    __syncthreads();
  }
#pragma unroll
  for (int mb = 0; mb < MB; mb++) {
    const int qi = qw0 + mb * 32 + (lane & 31);
    if (qi < S) store_acc_T(dq + (tok0 + qi) * ld + hoff, acc[mb], scale, lane);
  }
  }  // pass
}
constexpr int DQ_LDS = 4 * TILE_BYTES;   // K and V, double buffered

// ----------------------------------------------------------------------------------------------
// backward, dK and dV: workgroup owns 4 x 32 keys, streams 64-query tiles of Q and dO
// ----------------------------------------------------------------------------------------------
constexpr int DKV_STAGE = 2 * TILE_BYTES + 2 * KT * 4;     // Q tile, dO tile, lse2[64], D[64]
constexpr int DKV_LDS = 2 * DKV_STAGE;

// NB 32-key blocks per wavefront: every Q / dO operand read from LDS feeds NB MFMAs.  With NB = 1 the
// four wavefronts together need 128 bytes of LDS operands per clock to keep the matrix pipes busy,
// which is all the LDS delivers; NB = 2 halves that (the accumulators then fill the AGPR file).
// WRITE_DS: the kernel also leaves scale * dS^T, as bf16 [key][query] per (batch, head), in `dst`; the
// query gradient is then one k-major GEMM dQ = (scale dS^T)^T K over it, instead of a second kernel
// that forms S, dP and dS all over again.  Everything a row tile of that GEMM reads is written here:
// key k's row holds every query from 256 * floor(k / 256) on, zeros where the query precedes the key.
template <int NB, bool WRITE_DS>
__global__ __launch_bounds__(256) void attn_bwd_dkv_kernel(const uint16_t* __restrict__ q, const uint16_t* __restrict__ k,
                                                           const uint16_t* __restrict__ v,
                                                           const uint16_t* __restrict__ dout,
                                                           const float* __restrict__ lse2, const float* __restrict__ D,
                                                           uint16_t* __restrict__ dk, uint16_t* __restrict__ dv,
                                                           uint16_t* __restrict__ dst, int64_t ld, int64_t ldkv, int64_t lddkv, int grp, int S, int H,
                                                           float scale) {
  extern __shared__ __attribute__((aligned(16))) unsigned char smem[];
  constexpr int BN = 4 * NB * 32;
  // the wavefront index as a scalar: everything derived from it (LDS slots, tile rows) is scalar arithmetic
  const int tid = threadIdx.x, lane = tid & 63, wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int nkb = (S + BN - 1) / BN;
  const WgCoord wg = wg_coord();
  const int head = wg.head, b = wg.b;
  const int64_t tok0 = (int64_t)b * S;
  const int64_t hoff = head * HD;
  const float c = scale * LOG2E;
  // Q and dO tiles are needed row-wise (S, dP) and transposed (dK^T, dV^T): one LDS copy each, in the
  // swizzle that serves both reads, written by direct-to-LDS loads.
  const rsrc_t rsQ = tile_rsrc(q + tok0 * ld + hoff);
  const rsrc_t rsO = tile_rsrc(dout + tok0 * ld + hoff);
  const rsrc_t rsL = make_rsrc(lse2 + ((int64_t)b * H + head) * S, (uint32_t)S * 4u);
  const rsrc_t rsD = make_rsrc(D + ((int64_t)b * H + head) * S, (uint32_t)S * 4u);
  uint32_t offT[4];
  int rowT[4];
  dma_lane_offsets<SWZ_BOTH, 4>(offT, rowT, ld, wave, lane);
  // all loads of one 64-query tile: 4 + 4 tile loads per wavefront; wavefronts 0 and 1 also fetch the
  // tile's 64 row scalars (out-of-range rows read as zeros: the resource ends at S)
  auto dma_stage = [&](int st, int j) {
    unsigned char* p = smem + st * DKV_STAGE;
    dma_tile<4>(rsQ, p, offT, rowT, j * KT, S, ld, wave);
    dma_tile<4>(rsO, p + TILE_BYTES, offT, rowT, j * KT, S, ld, wave);
    if (wave == 0)
      lds_dma<4>(rsL, p + 2 * TILE_BYTES, (uint32_t)(j * KT + lane) * 4u);
    if (wave == 1)
      lds_dma<4>(rsD, p + 2 * TILE_BYTES + KT * 4, (uint32_t)(j * KT + lane) * 4u);
  };

  // one key block from the early end (most queries) and its mirror image from the late end: equal
  // work per workgroup
  // dS^T of this (batch, head): S rows of S bf16.  A packed k16 fragment holds, for the lane's key row,
  // queries 4h..4h+3 and 8+4h..8+4h+3 (h = lane / 32); lanes l and l + 32 exchange one half each, after
  // which a lane owns 8 consecutive queries and stores them with one 16-byte access.  Rows past S fall
  // outside the resource, queries past S (a multiple of 8) are given an offset that does.
  const __amdgpu_buffer_rsrc_t rsS = __builtin_amdgcn_make_buffer_rsrc(
      (void*)(WRITE_DS ? dst + ((int64_t)b * H + head) * S * S : nullptr), 0, WRITE_DS ? (uint32_t)S * (uint32_t)S * 2u : 0u,
      0x00020000);
  typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
  auto store_ds = [&](const bf16x8& f, int key, int q16) {
    const uint4 w = __builtin_bit_cast(uint4, f);
    // swap(a, b): lanes 32..63 of a <-> lanes 0..31 of b
    const auto sx = __builtin_amdgcn_permlane32_swap(w.x, w.z, false, false);
    const auto sy = __builtin_amdgcn_permlane32_swap(w.y, w.w, false, false);
    const int q0 = q16 + 8 * (lane >> 5);
    const uint32_t o = q0 < S ? (uint32_t)key * (uint32_t)S * 2u + (uint32_t)q0 * 2u : DMA_OOB;
    __builtin_amdgcn_raw_buffer_store_b128(u32x4{sx[0], sy[0], sx[1], sy[1]}, rsS, (int)o, 0, 0);
  };
  const bf16x8 zero_frag = __builtin_bit_cast(bf16x8, make_uint4(0, 0, 0, 0));

  for (int pass = 0; pass < 2; pass++) {
  const int kblk = pass == 0 ? wg.x : nkb - 1 - wg.x;
  if (pass == 1 && kblk <= wg.x) break;
  const int n0 = kblk * BN;
  const int nw0 = n0 + wave * NB * 32;
  if constexpr (WRITE_DS) {
    // queries between the start of the enclosing 256-row tile and this key block: zeros
    for (int qz = (n0 / 256) * 256; qz < n0; qz += 16)
#pragma unroll
      for (int nb = 0; nb < NB; nb++) store_ds(zero_frag, nw0 + nb * 32 + (lane & 31), qz);
  }

  // K and V rows of this wavefront stay in registers (B operands).
  bf16x8 kf[NB][8], vf[NB][8];
  // (grouped-query attention: the group's shared key / value head, rows of ldkv; dk and dv below are
  // this query head's contribution, laid out like q)
  load_row_frags<NB>(kf, k + tok0 * ldkv + (head / grp) * HD, ldkv, nw0, S, lane);
  load_row_frags<NB>(vf, v + tok0 * ldkv + (head / grp) * HD, ldkv, nw0, S, lane);

  f32x16 akv[2][NB][4];                                    // [0] = dK^T, [1] = dV^T
#pragma unroll
  for (int w = 0; w < 2; w++)
#pragma unroll
    for (int nb = 0; nb < NB; nb++)
#pragma unroll
      for (int hb = 0; hb < 4; hb++)
#pragma unroll
        for (int e = 0; e < 16; e++) akv[w][nb][hb][e] = 0.f;

  const int jbeg = n0 / KT;                                // causal: first query tile that sees key n0
  const int jend = (S + KT - 1) / KT;
  dma_stage(0, jbeg);
  wait_vm0();
  __syncthreads();

  for (int j = jbeg; j < jend; j++) {
    const int cur = (j - jbeg) & 1;
    if (j + 1 < jend) dma_stage(cur ^ 1, j + 1);           // lands while this tile is worked on
    const unsigned char* sQ = smem + cur * DKV_STAGE;
    const unsigned char* sO = sQ + TILE_BYTES;
    const float* sl = reinterpret_cast<const float*>(sO + TILE_BYTES);
    const float* sd = sl + KT;
    const int qt0 = j * KT;
    // one 32-query block at a time; blocks entirely before this wavefront's keys are skipped, blocks
    // entirely after them need no mask
#pragma unroll 1
    for (int qb2 = 0; qb2 < 2; qb2++) {
      const int qb0 = qt0 + qb2 * 32;
      if (qb0 + 31 < nw0 || qb0 >= S) {
        if constexpr (WRITE_DS) {   // not computed, but a row tile of the dQ GEMM reads it: zeros
#pragma unroll
          for (int t = 0; t < 2; t++)
#pragma unroll
            for (int nb = 0; nb < NB; nb++) store_ds(zero_frag, nw0 + nb * 32 + (lane & 31), qb0 + t * 16);
        }
        continue;
      }
      f32x16 st[NB], dp[NB];                               // rows = queries, column = key
#pragma unroll
      for (int nb = 0; nb < NB; nb++)
#pragma unroll
        for (int e = 0; e < 16; e++) { st[nb][e] = 0.f; dp[nb][e] = 0.f; }
#pragma unroll
      for (int ks = 0; ks < 8; ks++) {
        const bf16x8 qfr = both_row_frag(sQ, qb2 * 32, ks, lane), dfr = both_row_frag(sO, qb2 * 32, ks, lane);
#pragma unroll
        for (int nb = 0; nb < NB; nb++) {
          st[nb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(qfr, kf[nb][ks], st[nb], 0, 0, 0);
          dp[nb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(dfr, vf[nb][ks], dp[nb], 0, 0, 0);
        }
      }
      float4 slv[4], sdv[4];                               // rows 8 g + 4 (lane / 32) + 0..3, g = 0..3
#pragma unroll
      for (int g4 = 0; g4 < 4; g4++) {
        slv[g4] = *reinterpret_cast<const float4*>(sl + qb2 * 32 + 8 * g4 + 4 * (lane >> 5));
        sdv[g4] = *reinterpret_cast<const float4*>(sd + qb2 * 32 + 8 * g4 + 4 * (lane >> 5));
      }
      const bool need_mask = (qb0 < nw0 + NB * 32 - 1) || (qb0 + 32 > S);
      // the element loop exists twice, with and without the mask, under one wavefront-uniform branch
      // (left to the compiler, the test was repeated per element and split the loop into 16 blocks)
      auto elements = [&](auto MASKED) {
#pragma unroll
        for (int nb = 0; nb < NB; nb++) {
          const int ni = nw0 + nb * 32 + (lane & 31);
#pragma unroll
          for (int e = 0; e < 16; e++) {
            const float lv = e % 4 == 0 ? slv[e / 4].x : e % 4 == 1 ? slv[e / 4].y : e % 4 == 2 ? slv[e / 4].z : slv[e / 4].w;
            const float dvv = e % 4 == 0 ? sdv[e / 4].x : e % 4 == 1 ? sdv[e / 4].y : e % 4 == 2 ? sdv[e / 4].z : sdv[e / 4].w;
            float p = fast_exp2(fmaf(st[nb][e], c, -lv));
            if constexpr (decltype(MASKED)::value) {
              const int qi = qb0 + acc_row(e, lane);
              p = (ni > qi || qi >= S) ? 0.f : p;
            }
            st[nb][e] = p;                                   // P
            if constexpr (WRITE_DS) dp[nb][e] = (p * scale) * (dp[nb][e] - dvv);   // scale * dS
            else dp[nb][e] = p * (dp[nb][e] - dvv);          // dS
          }
        }
      };
      if (need_mask) {
        asm volatile("" ::: "memory");
        elements(std::true_type{});
      } else {
        elements(std::false_type{});
      }
#pragma unroll
      for (int t = 0; t < 2; t++) {
        bf16x8 pf[NB], dsf[NB];
#pragma unroll
        for (int nb = 0; nb < NB; nb++) { pf[nb] = pack_acc_half(st[nb], t); dsf[nb] = pack_acc_half(dp[nb], t); }
        if constexpr (WRITE_DS) {
#pragma unroll
          for (int nb = 0; nb < NB; nb++) store_ds(dsf[nb], nw0 + nb * 32 + (lane & 31), qb0 + t * 16);
        }
#pragma unroll
        for (int hb = 0; hb < 4; hb++) {
          const bf16x8 dtf = both_tr_frag(sO, qb2 * 32 + t * 16, hb * 32, lane);
          const bf16x8 qtf = both_tr_frag(sQ, qb2 * 32 + t * 16, hb * 32, lane);
#pragma unroll
          for (int nb = 0; nb < NB; nb++) {
            akv[1][nb][hb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(dtf, pf[nb], akv[1][nb][hb], 0, 0, 0);
            akv[0][nb][hb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(qtf, dsf[nb], akv[0][nb][hb], 0, 0, 0);
          }
        }
      }
    }
    // The next tile's loads were issued before this tile's dS^T stores (4 * NB per wavefront, issued on
    // every path) and memory operations retire in order: waiting until at most that many are
    // outstanding covers the loads without waiting for the stores to be acknowledged.
    if constexpr (WRITE_DS) wait_vm<4 * NB>();
    else wait_vm0();
    __syncthreads();
  }
#pragma unroll
  for (int nb = 0; nb < NB; nb++) {
    const int ni = nw0 + nb * 32 + (lane & 31);
    if (ni < S) {
      store_acc_T(dk + (tok0 + ni) * lddkv + hoff, akv[0][nb], WRITE_DS ? 1.f : scale, lane);
      store_acc_T(dv + (tok0 + ni) * lddkv + hoff, akv[1][nb], 1.f, lane);
    }
  }
  }  // pass
}

// Grouped-query attention: a key / value head's gradient is the sum of the contributions of the grp
// query heads that share it.  part: two [T, H * HD] bf16 tensors (dK, then dV contributions, one per
// query head), out: dk / dv [T, ldkv].  One thread adds grp 16-byte vectors in fp32.
__global__ __launch_bounds__(256) void attn_group_sum_kernel(const uint16_t* __restrict__ part, int64_t part_elems,
                                                             uint16_t* __restrict__ dk, uint16_t* __restrict__ dv,
                                                             int64_t ldkv, int grp, int H, int64_t T) {
  const int Hkv = H / grp;
  const int64_t item = (int64_t)blockIdx.x * 256 + threadIdx.x;   // (token, kv head, 16-byte chunk)
  if (item >= T * Hkv * (HD / 8)) return;
  const int ch = (int)(item % (HD / 8));
  const int kvh = (int)((item / (HD / 8)) % Hkv);
  const int64_t t = item / ((int64_t)(HD / 8) * Hkv);
  const uint16_t* src = part + (int64_t)blockIdx.y * part_elems + t * ((int64_t)H * HD) + (int64_t)kvh * grp * HD + ch * 8;
  float acc[8] = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};
  for (int g = 0; g < grp; g++) {
    float v[8];
    unpack8(*reinterpret_cast<const uint4*>(src + g * HD), v);
#pragma unroll
    for (int e = 0; e < 8; e++) acc[e] += v[e];
  }
  uint16_t* dst = (blockIdx.y == 0 ? dk : dv) + t * ldkv + kvh * HD + ch * 8;
  *reinterpret_cast<uint4*>(dst) = pack8(acc);
}

template <class K>
hipError_t set_lds(K kern, int bytes) {
  return hipFuncSetAttribute((const void*)kern, hipFuncAttributeMaxDynamicSharedMemorySize, bytes);
}

}  // namespace

hipError_t attention_fwd_bf16(const void* q, const void* k, const void* v, void* o, float* lse, int64_t ld, int B,
                              int S, int H, int hd, int causal, hipStream_t st) {
  return attention_gqa_fwd_bf16(q, k, v, o, lse, ld, ld, B, S, H, H, hd, causal, st);
}

// Hkv key / value heads (rows of ldkv elements) serve H query heads, H / Hkv consecutive ones each.
hipError_t attention_gqa_fwd_bf16(const void* q, const void* k, const void* v, void* o, float* lse, int64_t ld,
                                  int64_t ldkv, int B, int S, int H, int Hkv, int hd, int causal, hipStream_t st) {
  if (hd != HD || !causal) return hipErrorNotSupported;
  if (Hkv <= 0 || H % Hkv != 0) return hipErrorInvalidValue;
  const int grp = H / Hkv;
  // 32-bit buffer offsets per (batch, head)
  if ((int64_t)S * ld * 2 >= (int64_t)0x7fffffff || (int64_t)S * ldkv * 2 >= (int64_t)0x7fffffff) return hipErrorNotSupported;
  constexpr int MB = 1;
  constexpr int BQ = 4 * MB * 32;
  // one-time opt-in to more than 64 KB of dynamic LDS (thread-safe static initialisation)
  static const hipError_t attr_err = set_lds(attn_fwd_kernel<MB>, FWD_LDS);
  if (attr_err != hipSuccess) return attr_err;
  const int nqb = (S + BQ - 1) / BQ;
  dim3 grid((nqb + 1) / 2, H, B);                        // each workgroup: one query block and its mirror
  hipLaunchKernelGGL(attn_fwd_kernel<MB>, grid, dim3(256), FWD_LDS, st, (const uint16_t*)q, (const uint16_t*)k,
                     (const uint16_t*)v, (uint16_t*)o, lse, ld, ldkv, grp, S, H, 1.f / sqrtf((float)hd));
  return hipGetLastError();
}

// The backward runs in one of two forms.  With the score gradient kept (S a multiple of 8, and
// B * H * S^2 bf16 values within the cap below): the dK / dV kernel also writes scale * dS^T and dQ is
// one k-major GEMM over it, 5 GEMM units in all.  Otherwise: a second kernel recomputes S, dP and dS for
// dQ, 7 units and no large workspace.
constexpr size_t DS_WS_CAP = (size_t)24 << 30;
static bool keep_ds(int B, int S, int H) {
  return S % 8 == 0 && (int64_t)S * S * 2 < (int64_t)0x7fffffff && (size_t)B * H * S * S * 2 <= DS_WS_CAP;
}
// D and the base-2 exponent offsets lse * log2(e), both [B, H, S] fp32; then dS^T [B, H, S, S] bf16
size_t attention_bwd_ws_bytes(int B, int S, int H, int hd) { return attention_gqa_bwd_ws_bytes(B, S, H, H, hd); }
// ... and, with fewer key / value heads than query heads, the per-query-head contributions to dK and dV
// (two [B * S, H * hd] bf16 tensors) that a last kernel adds up group by group
static size_t ds_bytes(int B, int S, int H) { return keep_ds(B, S, H) ? ((size_t)B * H * S * S * 2 + 255) / 256 * 256 : 0; }
size_t attention_gqa_bwd_ws_bytes(int B, int S, int H, int Hkv, int hd) {
  const size_t small = (2 * (size_t)B * H * S * sizeof(float) + 255) / 256 * 256;
  return small + ds_bytes(B, S, H) + (Hkv < H ? 2 * (size_t)B * S * H * HD * 2 : 0);
}

constexpr int DQ_MB = 2;    // 32-query blocks per wavefront in the dQ kernel
constexpr int DKV_NB = 1;   // 32-key blocks per wavefront in the dK/dV kernel

hipError_t attention_bwd_bf16(const void* q, const void* k, const void* v, const void* o, const void* dout,
                              const float* lse, void* dq, void* dk, void* dv, int64_t ld, int B, int S, int H, int hd,
                              int causal, void* ws, hipStream_t st) {
  return attention_gqa_bwd_bf16(q, k, v, o, dout, lse, dq, dk, dv, ld, ld, B, S, H, H, hd, causal, ws, st);
}

hipError_t attention_gqa_bwd_bf16(const void* q, const void* k, const void* v, const void* o, const void* dout,
                                  const float* lse, void* dq, void* dk, void* dv, int64_t ld, int64_t ldkv, int B, int S,
                                  int H, int Hkv, int hd, int causal, void* ws, hipStream_t st) {
  if (hd != HD || !causal) return hipErrorNotSupported;
  if (Hkv <= 0 || H % Hkv != 0) return hipErrorInvalidValue;
  const int grp = H / Hkv;
  // 32-bit buffer offsets per (batch, head)
  if ((int64_t)S * ld * 2 >= (int64_t)0x7fffffff || (int64_t)S * ldkv * 2 >= (int64_t)0x7fffffff) return hipErrorNotSupported;
  static const hipError_t attr_err = [] {
    hipError_t e = set_lds(attn_bwd_dq_kernel<DQ_MB>, DQ_LDS);
    if (e == hipSuccess) e = set_lds(attn_bwd_dkv_kernel<DKV_NB, false>, DKV_LDS);
    if (e == hipSuccess) e = set_lds(attn_bwd_dkv_kernel<DKV_NB, true>, DKV_LDS);
    return e;
  }();
  if (attr_err != hipSuccess) return attr_err;
  float* D = (float*)ws;
  const int64_t items = (int64_t)B * S * H;
  float* lse2 = D + items;
  hipLaunchKernelGGL(attn_dot_kernel, dim3((unsigned)((items * 16 + 255) / 256)), dim3(256), 0, st,
                     (const uint16_t*)dout, (const uint16_t*)o, lse, D, lse2, ld, S, H, items);
  const float scale = 1.f / sqrtf((float)hd);
  const dim3 kv_grid(((S + DKV_NB * 128 - 1) / (DKV_NB * 128) + 1) / 2, H, B);
  const size_t small = (2 * (size_t)items * sizeof(float) + 255) / 256 * 256;
  // where the dK / dV kernel writes: the outputs themselves, or (fewer key / value heads than query
  // heads) one contribution per query head, added up at the end
  const int64_t T = (int64_t)B * S, part_elems = T * H * HD;
  uint16_t* part = (uint16_t*)((char*)ws + small + ds_bytes(B, S, H));
  uint16_t* dk_w = grp > 1 ? part : (uint16_t*)dk;
  uint16_t* dv_w = grp > 1 ? part + part_elems : (uint16_t*)dv;
  const int64_t lddkv = grp > 1 ? (int64_t)H * HD : ldkv;
  auto group_sum = [&]() -> hipError_t {
    if (grp == 1) return hipSuccess;
    const int64_t n = T * Hkv * (HD / 8);
    hipLaunchKernelGGL(attn_group_sum_kernel, dim3((unsigned)((n + 255) / 256), 2), dim3(256), 0, st, (const uint16_t*)part,
                       part_elems, (uint16_t*)dk, (uint16_t*)dv, ldkv, grp, H, T);
    return hipGetLastError();
  };
  if (keep_ds(B, S, H)) {
    uint16_t* dst = (uint16_t*)((char*)ws + small);
    hipLaunchKernelGGL((attn_bwd_dkv_kernel<DKV_NB, true>), kv_grid, dim3(256), DKV_LDS, st, (const uint16_t*)q,
                       (const uint16_t*)k, (const uint16_t*)v, (const uint16_t*)dout, lse2, D, dk_w, dv_w, dst, ld, ldkv,
                       lddkv, grp, S, H, scale);
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) return e;
    // dQ[q, :] = sum_key (scale dS^T)[key, q] * K[key, :], per (batch, head): both operands k-major, the
    // key range of a row tile cut at its last query
    GemmOp op;
    op.lda = S; op.transA = 1; op.ldb = ldkv; op.transB = 1; op.ldc = ld;
    op.M = S; op.N = HD; op.K = S; op.causal_k = 1;
    op.epi.kind = EPI_STORE;
    if (grp == 1) {   // one launch: batch index = (batch element, head)
      op.A = dst; op.sA = (int64_t)S * S; op.sAo = (int64_t)H * S * S;
      op.B = k; op.sB = HD; op.sBo = (int64_t)S * ldkv;
      op.C = dq; op.sC = HD; op.sCo = (int64_t)S * ld;
      op.batch = B * H; op.batch_inner = H;
      return gemm_bf16_untimed(op, st);
    }
    // one launch per batch element: batch index = (key / value head, query head inside its group)
    for (int b = 0; b < B; b++) {
      op.A = dst + (int64_t)b * H * S * S; op.sA = (int64_t)S * S; op.sAo = (int64_t)grp * S * S;
      op.B = (const uint16_t*)k + (int64_t)b * S * ldkv; op.sB = 0; op.sBo = HD;
      op.C = (uint16_t*)dq + (int64_t)b * S * ld; op.sC = HD; op.sCo = (int64_t)grp * HD;
      op.batch = H; op.batch_inner = grp;
      e = gemm_bf16_untimed(op, st);
      if (e != hipSuccess) return e;
    }
    return group_sum();
  }
  hipLaunchKernelGGL(attn_bwd_dq_kernel<DQ_MB>, dim3(((S + DQ_MB * 128 - 1) / (DQ_MB * 128) + 1) / 2, H, B), dim3(256), DQ_LDS, st, (const uint16_t*)q,
                     (const uint16_t*)k, (const uint16_t*)v, (const uint16_t*)dout, lse2, D, (uint16_t*)dq, ld, ldkv, grp,
                     S, H, scale);
  hipLaunchKernelGGL((attn_bwd_dkv_kernel<DKV_NB, false>), kv_grid, dim3(256), DKV_LDS, st, (const uint16_t*)q,
                     (const uint16_t*)k, (const uint16_t*)v, (const uint16_t*)dout, lse2, D, dk_w, dv_w,
                     (uint16_t*)nullptr, ld, ldkv, lddkv, grp, S, H, scale);
  hipError_t e = hipGetLastError();
  if (e != hipSuccess) return e;
  return group_sum();
}

}  // namespace lrb
