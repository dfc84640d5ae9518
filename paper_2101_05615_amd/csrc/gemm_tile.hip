// Large-tile quantized GEMM for compute-bound shapes.
//
// One launch does everything the paper fuses around the GEMM (Sec. 2.1-2.2):
//   - A is read once from HBM, straight into LDS (global_load_lds, no register
//     staging); when a fragment is fetched from LDS for the matrix cores it is
//     shifted from uint8 to int8 (xor 0x80 == subtract 128: the int8 MFMA is
//     signed x signed) and its row offsets are accumulated with v_sad_u8 -- the row
//     offsets are a by-product of the staged block, never a second pass over A
//     (Appendix B, "PackingWithRowOffset");
//   - int32 accumulation on v_mfma_i32_32x32x32_i8, LDS multi-buffered;
//   - the output pipeline (zero-point corrections of Eq. (2), bias, fp32 scale,
//     round-to-nearest-even, clamp/ReLU) runs on the accumulators in registers and
//     stores uint8 directly: there is no int32 C in memory.  The same pipeline can
//     instead leave the result in fp32 (Appendix B: any output processing).
//
// Shift algebra: with A_s = A_u - 128, rowsum_s = rowsum_u - 128 K and
// acc_s = acc_u - 128 colsum, the corrected accumulator of Eq. (2) is
//   x = acc_s - (theta_A - 128) * (colsum - K theta_B) - theta_B * rowsum_s + bias,
// i.e. "replace theta_A by theta_A - 128" with the folded column offsets.
//
// The MFMA is issued transposed (first operand = B fragment, second = A fragment) so that a
// lane ends up with 16 consecutive columns of one row (one 16-byte store); the packed-B column
// permutation makes those columns consecutive.
//
// One template, a family of tile shapes (Appendix C: a few shape-specific kernels, every
// problem mapped to one of them): 256 x 256, 128 x 256 and 128 x 128 with a hand-scheduled loop (one
// generator, three register tiles; four LDS stages, three for 128 x 256 so that two workgroups share a CU),
// and 64 x 64 with a compiler-scheduled three-stage loop, several workgroups per CU, for shapes that would
// leave most CUs idle at the larger tiles; the compiler-scheduled loop also serves the dense convolution and
// K below the pipeline depth of the hand-scheduled one.  The 64 x 64 workgroup has two or four sets of four
// waves that take alternate k tiles and add their accumulators at the end.
#include "qg_internal.h"
#include <type_traits>
#include "tile_loop_asm.inc"

namespace {

typedef int v4i __attribute__((ext_vector_type(4)));
typedef int v16i __attribute__((ext_vector_type(16)));

constexpr int BK = 64;      // k extent of one LDS stage = one packed fragment deep
constexpr int NSTAGE = 4;   // LDS stages of the hand-scheduled loop: three tiles in flight behind the one being consumed
// (three stages, two tiles in flight, for the 128 x 256 tile, so that two workgroups fit the LDS of a CU)
constexpr int asm_stages(int blocks) { return blocks == 8 ? 3 : NSTAGE; }
// LDS stages of the compiler-scheduled loop, by 32 x 32 blocks per wave.  Three everywhere: measured with 3 to 8
// stages, a thin grid's k step (0.28 us at 64 x 64) does not get shorter with more tiles in flight -- it is the
// barrier / LDS read / MFMA chain of a lone workgroup -- while deeper buffers cost occupancy on full grids.
constexpr int pipe_stages(int) { return 3; }

// main-loop flavours
constexpr int PATH_ASM = 1;      // 256 x 256, hand-scheduled, four stages
constexpr int PATH_PIPE = 2;     // any tile shape, compiler-scheduled, three stages

template <int N>
__device__ __forceinline__ void wait_vmcnt() {
  asm volatile("s_waitcnt vmcnt(%0)" ::"n"(N) : "memory");
}
// wait until at most min(younger, I) tiles of N_DMA requests each are still in flight
template <int I, int N_DMA>
__device__ __forceinline__ void wait_tiles(int younger) {
  if constexpr (I == 0) {
    wait_vmcnt<0>();
  } else {
    if (younger >= I)
      wait_vmcnt<I * N_DMA>();
    else
      wait_tiles<I - 1, N_DMA>(younger);
  }
}
// 16 bytes per lane from global memory into LDS at lds_base + lane*16 (lds_base wave-uniform)
__device__ __forceinline__ void dma16(const void* gptr, unsigned char* lds_base) {
  __builtin_amdgcn_global_load_lds((const __attribute__((address_space(1))) void*)gptr,
                                   (__attribute__((address_space(3))) void*)lds_base, 16, 0, 0);
}

// Chunk swizzle of row r of an A stage (rows are 64 B = four 16-byte chunks).  A 16-byte read of one chunk
// index is served sixteen rows at a time out of 256 B of banks (eight rows and 128 B on older parts): the
// four rows 4 apart that share a 64-byte bank window must then hold that chunk at four different places.
__device__ __forceinline__ int a_swz(int r) { return ((r >> 1) & 3) ^ ((r >> 3) & 1); }
// swizzled byte offset of 16-byte chunk kc (0..3) of row r in an A stage
__device__ __forceinline__ int a_lds_off(int r, int kc) { return r * BK + ((kc ^ a_swz(r)) << 4); }

// operand list shared by the two generated loop variants (gen_tile_loop.py)
#define QG_TILE_LOOP_OPERANDS \
                 : [c0] "+a"(acc[0][0]), [c1] "+a"(acc[0][1]), [c2] "+a"(acc[0][2]), [c3] "+a"(acc[0][3]), \
                   [c4] "+a"(acc[1][0]), [c5] "+a"(acc[1][1]), [c6] "+a"(acc[1][2]), [c7] "+a"(acc[1][3]), \
                   [c8] "+a"(acc[2][0]), [c9] "+a"(acc[2][1]), [c10] "+a"(acc[2][2]), [c11] "+a"(acc[2][3]), \
                   [c12] "+a"(acc[3][0]), [c13] "+a"(acc[3][1]), [c14] "+a"(acc[3][2]), [c15] "+a"(acc[3][3]), \
                   [rs01] "=v"(rs01), [rs23] "=v"(rs23) \
                 : [av01] "v"(av01), [av23] "v"(av23), [bv01] "v"(bv01), [bv23] "v"(bv23), [ard] "v"(ard), \
                   [brd] "v"(brd), [aptr] "s"(A - (A_DMA - 1) * 1024), [bptr] "s"(b_tile0), [kt] "s"(KTF), [ldsdma] "s"(lds_dma), \
                   [lds] "s"(lds_base), [bstep] "s"(b_step) \
                 : QG_TILE_LOOP_CLOBBERS

#define QG_TILE_LOOP_OPERANDS_2X2 \
                 : [c0] "+a"(acc[0][0]), [c1] "+a"(acc[0][1]), [c2] "+a"(acc[1][0]), [c3] "+a"(acc[1][1]), \
                   [rs01] "=v"(rs01) \
                 : [av01] "v"(av01), [bv01] "v"(bv01), [ard] "v"(ard), [brd] "v"(brd), \
                   [aptr] "s"(A - (A_DMA - 1) * 1024), [bptr] "s"(b_tile0), [kt] "s"(KTF), [ldsdma] "s"(lds_dma), \
                   [lds] "s"(lds_base), [bstep] "s"(b_step) \
                 : QG_TILE_LOOP_CLOBBERS_2X2

#define QG_TILE_LOOP_OPERANDS_2X4 \
                 : [c0] "+a"(acc[0][0]), [c1] "+a"(acc[0][1]), [c2] "+a"(acc[0][2]), [c3] "+a"(acc[0][3]), \
                   [c4] "+a"(acc[1][0]), [c5] "+a"(acc[1][1]), [c6] "+a"(acc[1][2]), [c7] "+a"(acc[1][3]), \
                   [rs01] "=v"(rs01) \
                 : [av01] "v"(av01), [bv01] "v"(bv01), [ard] "v"(ard), [brd] "v"(brd), \
                   [aptr] "s"(A - (A_DMA - 1) * 1024), [bptr] "s"(b_tile0), [kt] "s"(KTF), [ldsdma] "s"(lds_dma), \
                   [lds] "s"(lds_base), [bstep] "s"(b_step), [bofs] "s"(A_STAGE + wave * ((B_DMA - A_DMA) * 1024)) \
                 : QG_TILE_LOOP_CLOBBERS_2X4

// the convolution variants: image base, per-lane pixel offsets and tap-validity bits, the row of theta_A bytes
#define QG_TILE_LOOP_OPERANDS_CONV_2X2 \
                 : [c0] "+a"(acc[0][0]), [c1] "+a"(acc[0][1]), [c2] "+a"(acc[1][0]), [c3] "+a"(acc[1][1]), \
                   [rs01] "=v"(rs01) \
                 : [apix01] "v"(apix01), [amask01] "v"(amask01), [bv01] "v"(bv01), [ard] "v"(ard), [brd] "v"(brd), \
                   [aptr] "s"(A), [tab] "s"(azp_row), [nc] "s"(cv_nc), [fs] "s"(cv_fs), [rowjump] "s"(cv_rowjump), [tapjump] "s"(cv_tapjump), \
                   [bptr] "s"(b_tile0), [kt] "s"(KTF), [ldsdma] "s"(lds_dma), [lds] "s"(lds_base), [bstep] "s"(b_step) \
                 : QG_TILE_LOOP_CLOBBERS_CONV_2X2

#define QG_TILE_LOOP_OPERANDS_CONV_2X4 \
                 : [c0] "+a"(acc[0][0]), [c1] "+a"(acc[0][1]), [c2] "+a"(acc[0][2]), [c3] "+a"(acc[0][3]), \
                   [c4] "+a"(acc[1][0]), [c5] "+a"(acc[1][1]), [c6] "+a"(acc[1][2]), [c7] "+a"(acc[1][3]), \
                   [rs01] "=v"(rs01) \
                 : [apix01] "v"(apix01), [amask01] "v"(amask01), [bv01] "v"(bv01), [ard] "v"(ard), [brd] "v"(brd), \
                   [aptr] "s"(A), [tab] "s"(azp_row), [nc] "s"(cv_nc), [fs] "s"(cv_fs), [rowjump] "s"(cv_rowjump), [tapjump] "s"(cv_tapjump), \
                   [bptr] "s"(b_tile0), [kt] "s"(KTF), [ldsdma] "s"(lds_dma), [lds] "s"(lds_base), [bstep] "s"(b_step), \
                   [bofs] "s"(A_STAGE + wave * ((B_DMA - A_DMA) * 1024)) \
                 : QG_TILE_LOOP_CLOBBERS_CONV_2X4

// NWM x NWN waves, each TM x TN blocks of 32 x 32.
// Both loops take any pointer, lda and K (PATH_ASM: K >= 256): every whole 64-deep tile is requested with
// global_load_lds -- the requests are 16 bytes per lane from any address -- and the loop is software-pipelined; a
// ragged last tile (K % 64 != 0) is staged once through registers with a byte mask and bounds checks.
// ROWSUM: row offsets are needed (some theta_B != 0, or the test hook asks for them); without it the
// loop skips the byte sums and the output pipeline skips the theta_B * rowsum term of Eq. (2).
//
// Workgroups per CU the register budget must allow: the hand-scheduled loop owns a SIMD per wave (256
// accumulator registers); the compiler-scheduled shapes rely on neighbours to hide latency, as many as
// their LDS stages allow (72 / 48 / 24 KB per workgroup).
constexpr int min_wg_per_cu(int path, int blocks) {
  if (path != PATH_PIPE) return blocks >= 16 ? 1 : 2;  // hand-scheduled: 128 / 64 KiB of LDS stages
  return blocks >= 8 ? 2 : (blocks >= 4 ? 3 : 4);
}

// CONV: dense convolution with the im2col folded into the addressing.  Row m of "A" is
// output pixel m of the NHWC result; the 64-deep k tile kt is 64 input channels of ONE filter tap
// (Cin % 64 == 0), so staging a tile is the same request as in the GEMM with the row base moved by the
// tap's pixel offset.  A tap outside the image must read as theta_A (zero in the real domain): a lane whose
// chunk lies outside the image requests its 16 bytes from a constant row of theta_A bytes instead
// (qg_byte_rows), so what lands in the stage is the im2col row itself and row sums, shift and MFMAs are the GEMM's.
// CONV == 2: any Cin % 16 == 0.  A 64-deep tile is then four 16-channel chunks that may belong to different
// taps (and, in the last tile, lie past K = R*S*Cin), so the tap of the chunk a lane requests is per-lane state
// (channel chunk, kw, kh), advanced by four chunks per tile.  A chunk past K is requested from the row of 0x80
// bytes, the K padding of every A stage (zero after the shift).
// KS (PATH_PIPE only): wave groups that split K inside the workgroup.  With KS = 2 the workgroup has two sets of
// NWM x NWN waves; set g consumes the k tiles g, g + 2, ... from its own LDS stages (a lone workgroup's k
// step is a barrier / LDS read / MFMA chain, so two chains side by side halve the time of a thin grid), and the
// two partial accumulators are added through LDS before the output pipeline, which set 0 runs.
// EPI: the form of the uint8 output pipeline, fixed per launch by the host (one copy of the pipeline per kernel: the
// large tiles sit at the edge of the register budget): EPI_CLAMP the explicit clamp of the definition, EPI_SAT the
// saturating convert doing the clamp (no ReLU, or theta_C == 0), EPI_SAT0 the same with theta_C == 0, where the
// convert also does the rounding (v_cvt_pk_u8_f32 rounds to nearest even: checked on 4 M values, ties included).
//
// The leading scalar arguments repeat the fields of p that a wave needs before its first tile request: the file is
// compiled with kernel-argument preloading, so they arrive in scalar registers with the wave instead of costing a
// cold trip to memory.
constexpr int EPI_CLAMP = 0, EPI_SAT = 1, EPI_SAT0 = 2;

// SPLIT (hand-scheduled 128 x 128 tile only): K split ACROSS workgroups, as in the streaming kernels (the role of the
// paper's caller-provided C_buffer, Appendix A).  blockIdx.y is the slice: p.ks_per k tiles from tile blockIdx.y *
// p.ks_per on.  A slice hands its int32 accumulators and row offsets to its slot of the caller's workspace with
// device-coherent stores, waits for their acknowledgement and takes a ticket; the workgroup that draws the last
// ticket adds the other slices' slots to its registers (integer sums: every split gives the same bytes), puts the
// counter back to zero and runs the output pipeline.  For a few hundred rows and a long K, where the tiles of the
// problem are fewer than the CUs and each would walk all of K alone.
template <int MODE, int PATH, bool ROWSUM, int NWM, int NWN, int TM, int TN, int CONV = 0, int KS = 1, int EPI = EPI_CLAMP,
          bool SPLIT = false>
__global__ __launch_bounds__(NWM * NWN * KS * 64, min_wg_per_cu(PATH, TM * TN) / KS) void qg_gemm_tile_kernel(
    const uint8_t* A0, const int8_t* Bp, const int M, const int N, const int K0, const int nb16_total, const int lda,
    const int tiles_m, const int tiles_n, const qg_gemm_args p) {
  static_assert(!SPLIT || (PATH == PATH_ASM && TM == 2 && TN == 2 && CONV == 0 && KS == 1), "the cross-workgroup K split is built for the 128 x 128 tile");
  // this workgroup's part of K (all of it unless SPLIT; K0 stays the K of the whole product)
  const int k_first = SPLIT ? (int)blockIdx.y * p.ks_per : 0;  // in 64-deep tiles
  const uint8_t* const A = A0 + (SPLIT ? k_first * BK : 0);
  const int K = SPLIT ? min(K0 - k_first * BK, p.ks_per * BK) : K0;
  static_assert(KS == 1 || ((KS == 2 || KS == 4 || KS == 8) && PATH == PATH_PIPE), "K split: wave sets on the pipelined path");
  constexpr bool CVG = CONV == 2;  // per-chunk taps
  constexpr int NW = NWM * NWN, NT = NW * KS * 64;  // NW: waves of one set; NT: threads of the workgroup
  constexpr int BM = NWM * TM * 32, BN = NWN * TN * 32;
  constexpr int A_STAGE = BM * BK, B_STAGE = BN * BK, STAGE = A_STAGE + B_STAGE;
  constexpr int A_DMA = A_STAGE / 1024 / NW;  // 1 KiB wave-loads per wave per tile
  constexpr int B_DMA = B_STAGE / 1024 / NW;
  constexpr int N_DMA = A_DMA + B_DMA;
  static_assert(A_STAGE % (1024 * NW) == 0 && B_STAGE % (1024 * NW) == 0, "tile/wave mismatch");
  constexpr int NS = pipe_stages(TM * TN);  // PATH_PIPE
  static_assert((PATH == PATH_PIPE ? NS - 2 : 2) * N_DMA <= 63, "vmcnt is a 6-bit counter");
  extern __shared__ __align__(16) unsigned char smem[];

  const int tid = threadIdx.x;
  const int lane = tid & 63;
  const int wave_all = __builtin_amdgcn_readfirstlane(tid >> 6);  // wave-uniform, kept in an SGPR
  const int kg = wave_all / NW;      // wave set (0 unless KS > 1)
  const int wave = wave_all % NW;    // position inside the set
  const int wave_m = wave % NWM, wave_n = wave / NWM;
  const int l32 = lane & 31, lg = lane >> 5;

  // ---- workgroup -> tile.  Consecutive workgroup ids go to different XCDs
  // (8 of them, each with its own L2), so give every XCD one contiguous chunk of
  // the tile sequence, and walk that sequence in bands of 8 tile-rows so that
  // the tiles resident on an XCD at one time share A and B panels in its L2.
  const int total = tiles_m * tiles_n;
  int lin = blockIdx.x;
  if ((total & 7) == 0) lin = (lin & 7) * (total >> 3) + (lin >> 3);
  constexpr int BAND = 8;
  const int band_sz = BAND * tiles_n;
  const int band = lin / band_sz;
  const int first_m = band * BAND;
  const int rows_in_band = min(tiles_m - first_m, BAND);
  const int in_band = lin - band * band_sz;
  const int tm = first_m + in_band % rows_in_band;
  const int tn = in_band / rows_in_band;
  const int m0 = tm * BM, n0 = tn * BN;

  // ---- staging.  A: one wave-load fills 1 KiB of LDS = 16 rows x 64 B; lane l lands at row l/4,
  // physical chunk l%4, so it fetches the logical chunk that the swizzle maps there.  B: the tile is
  // BN/16 fragments of 1 KiB, one contiguous run of the packed buffer.  Addresses are a wave-uniform
  // base (advanced per tile on the scalar unit) plus a fixed 32-bit per-lane offset.
  unsigned a_voff[A_DMA], b_voff[B_DMA];
  int a_pix[A_DMA];  // CONV: byte offset of the chunk this lane requests, at tap (0, 0) (may be negative)
  int a_h[A_DMA], a_w[A_DMA];  // CONV: image row and column of that tap
#pragma unroll
  for (int q = 0; q < A_DMA; ++q) {
    const int r = (wave * A_DMA + q) * 16 + (lane >> 2);
    const int kc = (lane & 3) ^ a_swz(r);
    const int rg = min(m0 + r, M - 1);  // rows past M re-read the last row; never stored
    if (CONV) {
      const int wo = rg % p.cv_Wo, t = rg / p.cv_Wo;
      const int ho = t % p.cv_Ho, n = t / p.cv_Ho;
      // byte offset of this lane's chunk at tap (0, 0), channel slice 0; a tap adds a workgroup-uniform offset
      a_pix[q] = ((n * p.cv_H + ho * p.cv_stride - p.cv_pad) * p.cv_W + wo * p.cv_stride - p.cv_pad) * p.cv_pix +
                 (CVG ? 0 : kc * 16);
      a_voff[q] = kc * 16;  // CVG: the chunk of the tile this lane requests
      a_h[q] = ho * p.cv_stride - p.cv_pad;
      a_w[q] = wo * p.cv_stride - p.cv_pad;
      continue;
    }
    // hand-scheduled loop: it uses instruction offset q*1024 (it moves the LDS slot AND the global address, so one
    // M0 serves a group of requests) against a base of A - (A_DMA-1) KiB; the per-lane offset absorbs the difference
    a_voff[q] = (unsigned)rg * (unsigned)lda + kc * 16 + (PATH == PATH_ASM ? (A_DMA - 1 - q) * 1024 : 0);
  }
#pragma unroll
  for (int q = 0; q < B_DMA; ++q)
    b_voff[q] = (unsigned)(wave * B_DMA + q) * QG_FRAG_BYTES + lane * 16;
  const unsigned b_step = (unsigned)nb16_total * QG_FRAG_BYTES;  // one 64-deep slab of the packed buffer
  const int8_t* b_tile0 = Bp + (size_t)(n0 / QG_FRAG_COLS) * QG_FRAG_BYTES + (SPLIT ? (size_t)k_first * b_step : 0);

  // ---- fragment fetch (LDS -> registers): per-lane base offsets, everything else is an immediate
  int a_rd[2];  // k-step 0 / 1 of block mb = 0; block mb is 32 rows = 2 KiB further
#pragma unroll
  for (int ks = 0; ks < 2; ++ks) a_rd[ks] = a_lds_off(wave_m * TM * 32 + l32, ks * 2 + lg);
  // slot i = l32 -> fragment (i >> 4) of the super-block, nl = i & 15; k-half lg is 256 B further
  const int b_rd = A_STAGE + ((wave_n * TN) * 2 + (l32 >> 4)) * QG_FRAG_BYTES + (l32 & 15) * 16 + lg * 256;
  auto fetch = [&](int stage, int ks, v4i (&af)[TM], v4i (&bf)[TN]) {
    const unsigned char* base = smem + (stage * KS + kg) * STAGE;
#pragma unroll
    for (int mb = 0; mb < TM; ++mb)
      af[mb] = *reinterpret_cast<const v4i*>(base + a_rd[ks] + mb * (32 * BK));
#pragma unroll
    for (int nb = 0; nb < TN; ++nb)
      bf[nb] = *reinterpret_cast<const v4i*>(base + b_rd + nb * (2 * QG_FRAG_BYTES) + ks * 512);
  };

  v16i acc[TM][TN];
#pragma unroll
  for (int i = 0; i < TM; ++i)
#pragma unroll
    for (int j = 0; j < TN; ++j)
#pragma unroll
      for (int r = 0; r < 16; ++r) acc[i][j][r] = 0;
  unsigned rs[TM];  // sums of raw uint8 bytes, K padding (stored as 0x80) included
#pragma unroll
  for (int i = 0; i < TM; ++i) rs[i] = 0;

  // Row-offset partial sums on the raw uint8 bytes (v_sad_u8 against 0 adds the four bytes of a
  // dword in one plain VALU op; v_dot4 would contend with the MFMAs for the dot-product pipeline),
  // then uint8 -> int8 in place (xor 0x80 == minus 128).
  auto prep = [&](v4i (&af)[TM]) {
#pragma unroll
    for (int mb = 0; mb < TM; ++mb) {
      if (ROWSUM) {
        rs[mb] = __builtin_amdgcn_sad_u8(af[mb].x, 0u, rs[mb]);
        rs[mb] = __builtin_amdgcn_sad_u8(af[mb].y, 0u, rs[mb]);
        rs[mb] = __builtin_amdgcn_sad_u8(af[mb].z, 0u, rs[mb]);
        rs[mb] = __builtin_amdgcn_sad_u8(af[mb].w, 0u, rs[mb]);
      }
      af[mb] = af[mb] ^ (int)0x80808080;
    }
  };
  auto mma = [&](const v4i (&af)[TM], const v4i (&bf)[TN]) {
#pragma unroll
    for (int mb = 0; mb < TM; ++mb)
#pragma unroll
      for (int nb = 0; nb < TN; ++nb)
        acc[mb][nb] = __builtin_amdgcn_mfma_i32_32x32x32_i8(bf[nb], af[mb], acc[mb][nb], 0, 0, 0);
  };
  const int KT = (K + BK - 1) / BK;  // tiles that hold real data
  // the pipelined loops run the KTF whole tiles; a ragged last tile (K % 64 bytes of A) is staged through
  // registers afterwards, once per workgroup
  const int KTF = CVG ? KT : K / BK;  // (CVG: chunks past K are replaced like taps outside the image)
  v4i a0[TM], b0[TN], a1[TM], b1[TN];
  if constexpr (PATH == PATH_ASM) {
    // Tile kt lives in stage kt % 4.  In iteration kt: the first k-step runs while the fragments of
    // the second are fetched; then every wave waits until ITS requests for tile kt+1 have landed
    // (two younger tiles may still be in flight) and until its own reads of tile kt are done, the
    // workgroup meets at one barrier, stage kt % 4 is handed to the request for tile kt+4, and the
    // second k-step runs while the first fragments of tile kt+1 are fetched.  The loop is one
    // hand-scheduled asm statement (gen_tile_loop.py): behind every MFMA sit at most seven other
    // instructions, so LDS reads, row sums, shifts and tile requests issue in the MFMA's shadow.
    static_assert(PATH != PATH_ASM || (NWM == 2 && NWN == 2 && BK == 64 && NSTAGE == 4 &&
                                       ((TM == 4 && TN == 4) || (TM == 2 && TN == 2) || (TM == 2 && TN == 4))),
                  "the scheduled loop is generated for these configurations");
    const unsigned long long av01 = a_voff[0] | ((unsigned long long)a_voff[1] << 32);
    const unsigned long long bv01 = b_voff[0] | ((unsigned long long)b_voff[1] << 32);
    const unsigned long long ard = (unsigned)a_rd[0] | ((unsigned long long)(unsigned)a_rd[1] << 32);
    const unsigned long long brd = (unsigned)b_rd;
    const unsigned lds_base = (unsigned)(uintptr_t)((__attribute__((address_space(3))) unsigned char*)smem);
    const unsigned lds_dma = lds_base + wave * (A_DMA * 1024);
    unsigned long long rs01;
    if constexpr (TM == 4) {
      const unsigned long long av23 = a_voff[2] | ((unsigned long long)a_voff[3] << 32);
      const unsigned long long bv23 = b_voff[2] | ((unsigned long long)b_voff[3] << 32);
      unsigned long long rs23;
      if (ROWSUM)
        asm volatile(QG_TILE_LOOP_ASM QG_TILE_LOOP_OPERANDS);
      else
        asm volatile(QG_TILE_LOOP_ASM_NOROWSUM QG_TILE_LOOP_OPERANDS);
      rs[2] = (unsigned)rs23;
      rs[3] = (unsigned)(rs23 >> 32);
    } else if constexpr (CONV != 0) {
      // the convolution's requests: pixel offsets pre-biased like the table rows, one validity bit per filter tap
      static_assert(CONV == 1 && TM == 2 && A_DMA == 2, "generated for 64 channels per tile and two requests per wave");
      unsigned amask[A_DMA];
#pragma unroll
      for (int q = 0; q < A_DMA; ++q) {
        amask[q] = 0;
        for (int kh = 0, tap = 0; kh < p.cv_R; ++kh)
          for (int kw = 0; kw < p.cv_S; ++kw, ++tap)
            if ((unsigned)(a_h[q] + kh) < (unsigned)p.cv_H && (unsigned)(a_w[q] + kw) < (unsigned)p.cv_W) amask[q] |= 1u << tap;
      }
      const unsigned long long apix01 = (unsigned)a_pix[0] | ((unsigned long long)(unsigned)(a_pix[1] - 1024) << 32);
      const unsigned long long amask01 = amask[0] | ((unsigned long long)amask[1] << 32);
      const uint8_t* const azp_row = qg_byte_rows.b[p.cv_azp];
      const int cv_nc = p.cv_Cin / BK, cv_fs = p.cv_S, cv_rowjump = (p.cv_W - p.cv_S) * p.cv_pix;
      const int cv_tapjump = p.cv_pix - p.cv_Cin;
      if constexpr (TN == 2) {
        if (ROWSUM)
          asm volatile(QG_TILE_LOOP_ASM_CONV_2X2 QG_TILE_LOOP_OPERANDS_CONV_2X2);
        else
          asm volatile(QG_TILE_LOOP_ASM_CONV_NOROWSUM_2X2 QG_TILE_LOOP_OPERANDS_CONV_2X2);
      } else {
        if (ROWSUM)
          asm volatile(QG_TILE_LOOP_ASM_CONV_2X4 QG_TILE_LOOP_OPERANDS_CONV_2X4);
        else
          asm volatile(QG_TILE_LOOP_ASM_CONV_NOROWSUM_2X4 QG_TILE_LOOP_OPERANDS_CONV_2X4);
      }
    } else if constexpr (TN == 2) {
      if (ROWSUM)
        asm volatile(QG_TILE_LOOP_ASM_2X2 QG_TILE_LOOP_OPERANDS_2X2);
      else
        asm volatile(QG_TILE_LOOP_ASM_NOROWSUM_2X2 QG_TILE_LOOP_OPERANDS_2X2);
    } else {
      if (ROWSUM)
        asm volatile(QG_TILE_LOOP_ASM_2X4 QG_TILE_LOOP_OPERANDS_2X4);
      else
        asm volatile(QG_TILE_LOOP_ASM_NOROWSUM_2X4 QG_TILE_LOOP_OPERANDS_2X4);
    }
    rs[0] = (unsigned)rs01;
    rs[1] = (unsigned)(rs01 >> 32);
  } else if constexpr (PATH == PATH_PIPE) {
    // Tile kt lives in stage kt % NS; NS-2 tiles are in flight behind the one being consumed.  At the top of
    // iteration kt a wave waits until ITS requests for tile kt have landed (younger ones may still be in
    // flight: requests complete in order), the workgroup meets at one barrier -- which also says that
    // every wave is done with tile kt-1 -- and that tile's stage is handed to the request for tile kt+NS-1.
    // Instruction order inside the iteration is the compiler's; latency is hidden by the other
    // workgroups on the CU.
    // CONV: filter tap (kh, kw) and 64-channel slice cc of a k tile, advanced incrementally
    const int cv_nc = CONV ? p.cv_Cin / BK : 1;
    int rq_kh = 0, rq_kw = 0, rq_cc = 0;  // of the next tile to request
    // CVG: the same per lane, in 16-channel chunks, for the chunk of request q.  A step of n tiles is 4 n chunks;
    // at most cv_wraps taps are crossed by it.
    const int cv_nc16 = CVG ? p.cv_Cin / 16 : 1;
    const int cv_wraps = CVG ? (4 * KS + cv_nc16 - 1) / cv_nc16 : 0;
    int rqv_c[A_DMA], rqv_kw[A_DMA], rqv_kh[A_DMA];
    const uint8_t* const azp_row = qg_byte_rows.b[CONV ? p.cv_azp : 0];
    auto cvg_init = [&](int chunk, int& c, int& kw, int& kh) {  // chunk: index along K in units of 16
      const int tap = chunk / cv_nc16;
      c = chunk - tap * cv_nc16;
      kh = tap / p.cv_S;
      kw = tap - kh * p.cv_S;
    };
    auto cvg_advance = [&](int& c, int& kw, int& kh) {
      c += 4 * KS;
      for (int j = 0; j < cv_wraps; ++j)
        if (c >= cv_nc16) {
          c -= cv_nc16;
          if (++kw == p.cv_S) kw = 0, ++kh;
        }
    };
    if (CVG) {
#pragma unroll
      for (int q = 0; q < A_DMA; ++q) cvg_init(kg * 4 + (int)(a_voff[q] >> 4), rqv_c[q], rqv_kw[q], rqv_kh[q]);
    }
    // n tiles on (wave-uniform, scalar unit): a wave set starts at tile kg and takes every KS-th
    auto cv_advance = [&](int& kh, int& kw, int& cc, int n) {
      for (int j = 0; j < n; ++j)
        if (++cc == cv_nc) {
          cc = 0;
          if (++kw == p.cv_S) kw = 0, ++kh;
        }
    };
    if (CONV == 1 && KS > 1) cv_advance(rq_kh, rq_kw, rq_cc, kg);
    auto request = [&](int kt, int stage) {
      const uint8_t* ab = A + (size_t)kt * BK;
      const int8_t* bb = b_tile0 + (size_t)kt * b_step;
      unsigned char* st = smem + (stage * KS + kg) * STAGE;
      if (CVG) {
#pragma unroll
        for (int q = 0; q < A_DMA; ++q) {
          const int off = a_pix[q] + (rqv_kh[q] * p.cv_W + rqv_kw[q]) * p.cv_pix + rqv_c[q] * 16;
          const bool in_k = rqv_kh[q] < p.cv_R;
          const bool in_image = (unsigned)(a_h[q] + rqv_kh[q]) < (unsigned)p.cv_H && (unsigned)(a_w[q] + rqv_kw[q]) < (unsigned)p.cv_W;
          const uint8_t* src = !in_k ? qg_byte_rows.b[128] : (in_image ? A + off : azp_row);
          dma16(src, st + (wave * A_DMA + q) * 1024);
          cvg_advance(rqv_c[q], rqv_kw[q], rqv_kh[q]);
        }
      } else if (CONV) {
        const int tap_off = (rq_kh * p.cv_W + rq_kw) * p.cv_pix + rq_cc * BK;
#pragma unroll
        for (int q = 0; q < A_DMA; ++q) {
          const bool in_image = (unsigned)(a_h[q] + rq_kh) < (unsigned)p.cv_H && (unsigned)(a_w[q] + rq_kw) < (unsigned)p.cv_W;
          dma16(in_image ? A + (a_pix[q] + tap_off) : azp_row, st + (wave * A_DMA + q) * 1024);
        }
        cv_advance(rq_kh, rq_kw, rq_cc, KS);
      } else
#pragma unroll
      for (int q = 0; q < A_DMA; ++q) dma16(ab + a_voff[q], st + (wave * A_DMA + q) * 1024);
#pragma unroll
      for (int q = 0; q < B_DMA; ++q) dma16(bb + b_voff[q], st + A_STAGE + (wave * B_DMA + q) * 1024);
    };
    // this wave set's tiles are kg, kg + KS, ...: KTg of them, in KT2 common steps (sets share the barriers)
    const int KTg = (KTF - kg + KS - 1) / KS, KT2 = (KTF + KS - 1) / KS;
#pragma unroll
    for (int t = 0; t < NS - 1; ++t)
      if (t < KTg) request(t * KS + kg, t);
    int stage = 0;
    // one common step: `consume` says whether this wave set has a tile in it (always, except in the last step
    // of the other set when the number of tiles is odd)
    auto step = [&](int i, bool consume) {
      wait_tiles<NS - 2, N_DMA>(KTg - 1 - i);  // this set's tile i has landed; up to NS-2 younger ones may be in flight
      asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");
      __builtin_amdgcn_s_barrier();
      asm volatile("" ::: "memory");
      if (i + NS - 1 < KTg) request((i + NS - 1) * KS + kg, stage == 0 ? NS - 1 : stage - 1);
      if (consume) {
        fetch(stage, 0, a0, b0);
        fetch(stage, 1, a1, b1);
        prep(a0);
        mma(a0, b0);
        prep(a1);
        mma(a1, b1);
      }
      stage = stage == NS - 1 ? 0 : stage + 1;
    };
    // the steps in which every set has a tile run unconditionally: a conditional MFMA inside the loop makes the
    // compiler copy the accumulators every iteration
    const int KTall = KTF / KS;
    for (int i = 0; i < KTall; ++i) step(i, true);
    if (KS > 1 && KT2 > KTall) step(KTall, KTall < KTg);
  }

  // ---- ragged last tile of the pipelined paths: bytes past K are staged as 0x80 (int8 zero after the shift)
  if (KTF < KT) {
    const int k0 = KTF * BK;
    __syncthreads();  // every wave is done with the stages
    if (kg == 0) {
      const size_t a_end = (size_t)(M - 1) * (size_t)lda + (size_t)K;  // one past the last byte A is known to have
#pragma unroll
      for (int q = 0; q < A_DMA; ++q) {
        const int r = (wave * A_DMA + q) * 16 + (lane >> 2);
        const int kc = (lane & 3) ^ a_swz(r);
        const size_t off = (size_t)min(m0 + r, M - 1) * (size_t)lda + (size_t)(kc * 16 + k0);
        *reinterpret_cast<v4i*>(smem + (wave * A_DMA + q) * 1024 + lane * 16) =
            qg_load_a_chunk(A + off, K - (k0 + kc * 16), off + 16 <= a_end);
      }
      const int8_t* b_base = b_tile0 + (size_t)KTF * b_step;
#pragma unroll
      for (int q = 0; q < B_DMA; ++q)
        *reinterpret_cast<v4i*>(smem + A_STAGE + (wave * B_DMA + q) * 1024 + lane * 16) =
            *reinterpret_cast<const v4i*>(b_base + b_voff[q]);
    }
    __syncthreads();
    if (kg == 0) {
      // (a convolution has no ragged tile: Cin % 64 == 0, or its last tile went through the loop above)
      fetch(0, 0, a0, b0);
      fetch(0, 1, a1, b1);
      prep(a0);
      prep(a1);
      mma(a0, b0);
      mma(a1, b1);
    }
  }

  // ---- K split: the other wave sets hand their accumulators and byte sums to the first through LDS
  if constexpr (KS > 1) {
    constexpr int PER_LANE = TM * TN * 16 + TM;
    constexpr int SET = PER_LANE * NW * 64;  // ints per handing set
    static_assert(4096 + (KS - 1) * SET * 4 <= NS * KS * STAGE, "partials must fit the stage memory");
    __syncthreads();  // every wave is done with the stages
    int* red = reinterpret_cast<int*>(smem) + 1024;  // past the per-column constants staged below
    if (kg != 0) {
      int* mine = red + (kg - 1) * SET;
#pragma unroll
      for (int mb = 0; mb < TM; ++mb) {
#pragma unroll
        for (int nb = 0; nb < TN; ++nb)
#pragma unroll
          for (int r = 0; r < 16; ++r) mine[((mb * TN + nb) * 16 + r) * (NW * 64) + wave * 64 + lane] = acc[mb][nb][r];
        mine[(TM * TN * 16 + mb) * (NW * 64) + wave * 64 + lane] = (int)rs[mb];
      }
    }
    __syncthreads();
    if (kg == 0) {
#pragma unroll
      for (int g = 0; g < KS - 1; ++g) {
        const int* theirs = red + g * SET;
#pragma unroll
        for (int mb = 0; mb < TM; ++mb) {
#pragma unroll
          for (int nb = 0; nb < TN; ++nb)
#pragma unroll
            for (int r = 0; r < 16; ++r) acc[mb][nb][r] += theirs[((mb * TN + nb) * 16 + r) * (NW * 64) + wave * 64 + lane];
          rs[mb] += (unsigned)theirs[(TM * TN * 16 + mb) * (NW * 64) + wave * 64 + lane];
        }
      }
    }
  }

  // ---- row offsets: lane (m, k-half) holds half of row m's byte sum; every one of the KT*64 bytes
  // summed (padding reads as 0x80) is 128 above its int8 value
  int rsum_s[TM];
#pragma unroll
  for (int mb = 0; mb < TM; ++mb)
    rsum_s[mb] = (int)(rs[mb] + (unsigned)__shfl_xor((int)rs[mb], 32)) - 128 * (KT * BK);

  // ---- K split across workgroups: hand the partial tile in, the last slice to arrive carries on
  if constexpr (SPLIT) {
    constexpr int PER = TM * TN * 16 + TM;  // ints per thread and slot
    const int unit = tm * tiles_n + tn, ks = p.ksplit;
    int* const cnt = p.ws_cnt + unit;
    int* const slots = p.ws_slots + (size_t)unit * ks * (PER * NT);
    int* const mine = slots + (size_t)blockIdx.y * (PER * NT) + tid;
#pragma unroll
    for (int mb = 0; mb < TM; ++mb) {
#pragma unroll
      for (int nb = 0; nb < TN; ++nb)
#pragma unroll
        for (int r = 0; r < 16; ++r)
          __hip_atomic_store(mine + ((mb * TN + nb) * 16 + r) * NT, acc[mb][nb][r], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
      __hip_atomic_store(mine + (TM * TN * 16 + mb) * NT, rsum_s[mb], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    }
    asm volatile("s_waitcnt vmcnt(0)" ::: "memory");  // the write-through stores above have been acknowledged
    __syncthreads();                                   // ... those of every wave (and every wave is done with the stages)
    int* const ticket_s = reinterpret_cast<int*>(smem);
    if (tid == 0) *ticket_s = __hip_atomic_fetch_add(cnt, 1, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    __syncthreads();
    if (*ticket_s != ks - 1) return;
    // every other slice's stores were acknowledged before it took its ticket
    for (int ss = 0; ss < ks; ++ss) {
      if (ss == (int)blockIdx.y) continue;
      const int* const theirs = slots + (size_t)ss * (PER * NT) + tid;
#pragma unroll
      for (int mb = 0; mb < TM; ++mb) {
#pragma unroll
        for (int nb = 0; nb < TN; ++nb)
#pragma unroll
          for (int r = 0; r < 16; ++r)
            acc[mb][nb][r] += __hip_atomic_load(theirs + ((mb * TN + nb) * 16 + r) * NT, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        rsum_s[mb] += __hip_atomic_load(theirs + (TM * TN * 16 + mb) * NT, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
      }
    }
    if (tid == 0) __hip_atomic_store(cnt, 0, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);  // ready for the next call
  }

  // ---- per-column constants of the output pipeline, staged once per workgroup
  __syncthreads();
  int* cj_s = reinterpret_cast<int*>(smem);
  int* bz_s = cj_s + BN;
  float* sc_s = reinterpret_cast<float*>(bz_s + BN);
  for (int t = tid; t < BN; t += NT) {
    const int col = n0 + t;  // col_off / bzp are padded to N_pad, bias / scales are not
    const int co = p.col_off[col], bz = p.bzp[col];
    if (MODE != QG_MODE_ACC32) {
      const int b = (p.bias != nullptr && col < N) ? p.bias[col] : 0;
      cj_s[t] = b - p.a_zp_m128 * co;
      sc_s[t] = (col < N) ? p.scales[(size_t)col * p.scale_stride] : 1.0f;
    } else {
      cj_s[t] = 128 * (co + K0 * bz);  // acc_u = acc_s + 128 * colsum
    }
    bz_s[t] = -bz;  // negated: x = acc + cj + (-theta_B) * rowsum
  }
  __syncthreads();
  if (KS > 1 && kg != 0) return;  // the first wave set holds the sums and runs the output pipeline

  // ---- epilogue straight from the accumulators.  Lane (l32, lg) of block (mb, nb) holds row
  // 32*mb + l32 and the 16 consecutive columns 32*nb + 16*lg .. +15; the per-column constants of a
  // column block are fetched once and reused for the wave's TM row blocks.
  if (MODE != QG_MODE_ACC32) {
    const bool full_cols = p.c_vec && (n0 + BN <= N);  // uniform: every 16-byte store is in range
    const float czp_f = (float)p.c_zp;
#pragma unroll
    for (int nb = 0; nb < TN; ++nb) {
      const int col_l = (wave_n * TN + nb) * 32 + lg * 16;
      const int col = n0 + col_l;
      int cj[16], nbz[16];
      float sc[16];
#pragma unroll
      for (int q = 0; q < 4; ++q) {
        *reinterpret_cast<v4i*>(&cj[4 * q]) = *reinterpret_cast<const v4i*>(&cj_s[col_l + 4 * q]);
        *reinterpret_cast<v4i*>(&nbz[4 * q]) = *reinterpret_cast<const v4i*>(&bz_s[col_l + 4 * q]);
        *reinterpret_cast<float4*>(&sc[4 * q]) = *reinterpret_cast<const float4*>(&sc_s[col_l + 4 * q]);
      }
#pragma unroll
      for (int mb = 0; mb < TM; ++mb) {
        const int row = m0 + (wave_m * TM + mb) * 32 + l32;
        const int rsum = rsum_s[mb];
        if (MODE == QG_MODE_REQUANT) {
          unsigned out[4];
#pragma unroll
          for (int q = 0; q < 4; ++q) {
            unsigned w = 0;
#pragma unroll
            for (int t = 0; t < 4; ++t) {
              const int i = 4 * q + t;
              const int x = acc[mb][nb][i] + cj[i] + (ROWSUM ? __mul24(nbz[i], rsum) : 0);
              if constexpr (EPI == EPI_SAT0)
                w = qg_requant_pack0(x, sc[i], t, w);
              else
                w = qg_requant_pack<EPI == EPI_CLAMP>(x, sc[i], p.clamp_lo, p.clamp_hi, czp_f, t, w);
            }
            out[q] = w;
          }
          if (row < M) {
            uint8_t* dst = p.C + (size_t)row * p.ldc + col;
            if (full_cols) {
              *reinterpret_cast<uint4*>(dst) = make_uint4(out[0], out[1], out[2], out[3]);
            } else if (col + 16 <= N) {
              // any address: one 16-byte store all the same
              *reinterpret_cast<qg_v4i_unaligned*>(dst) = (v4i){(int)out[0], (int)out[1], (int)out[2], (int)out[3]};
            } else {
              // the lanes whose 16 columns N cuts
#pragma unroll
              for (int i = 0; i < 16; ++i)
                if (col + i < N) dst[i] = (uint8_t)(out[i >> 2] >> ((i & 3) * 8));
            }
          }
        } else {
          // fp32 output: 16 consecutive floats per lane, four 16-byte stores
          float out[16];
#pragma unroll
          for (int i = 0; i < 16; ++i) {
            const int x = acc[mb][nb][i] + cj[i] + (ROWSUM ? __mul24(nbz[i], rsum) : 0);
            out[i] = qg_dequant_one(x, sc[i], p.relu_lo);
          }
          if (row < M) {
            float* dst = p.Cf + (size_t)row * p.ldc + col;
            if (full_cols) {
#pragma unroll
              for (int q = 0; q < 4; ++q)
                *reinterpret_cast<float4*>(dst + 4 * q) = make_float4(out[4 * q], out[4 * q + 1], out[4 * q + 2], out[4 * q + 3]);
            } else if (col + 16 <= N) {
#pragma unroll
              for (int q = 0; q < 4; ++q)
                *reinterpret_cast<qg_v4i_unaligned*>(dst + 4 * q) =
                    (v4i){__float_as_int(out[4 * q]), __float_as_int(out[4 * q + 1]), __float_as_int(out[4 * q + 2]),
                          __float_as_int(out[4 * q + 3])};
            } else {
#pragma unroll
              for (int i = 0; i < 16; ++i)
                if (col + i < N) dst[i] = out[i];
            }
          }
        }
      }
    }
  } else {
#pragma unroll
    for (int mb = 0; mb < TM; ++mb) {
      const int row = m0 + (wave_m * TM + mb) * 32 + l32;
      if (row >= M) continue;
      if (p.rowsum_out != nullptr && tn == 0 && wave_n == 0 && lg == 0)
        p.rowsum_out[row] = rsum_s[mb] + 128 * K0;
#pragma unroll
      for (int nb = 0; nb < TN; ++nb) {
        const int col_l = (wave_n * TN + nb) * 32 + lg * 16;
        const int col = n0 + col_l;
        int32_t* dst = p.C32 + (size_t)row * p.ldc + col;
#pragma unroll
        for (int i = 0; i < 16; ++i)
          if (col + i < N) dst[i] = acc[mb][nb][i] + cj_s[col_l + i];
      }
    }
  }
}

template <int MODE, int PATH, bool ROWSUM, int NWM, int NWN, int TM, int TN, int KS = 1, int EPI = EPI_CLAMP>
hipError_t launch(const qg_gemm_args& a, hipStream_t s) {
  constexpr int BM = NWM * TM * 32, BN = NWN * TN * 32;
  constexpr int STAGES = (PATH == PATH_ASM ? asm_stages(TM * TN) : pipe_stages(TM * TN)) * KS;
  // the output pipeline's per-column constants (12 B per column) reuse the stage memory
  constexpr int SMEM = STAGES * (BM + BN) * BK > 12 * BN ? STAGES * (BM + BN) * BK : 12 * BN;
  const int tiles_m = (a.M + BM - 1) / BM;
  const int tiles_n = (a.N + BN - 1) / BN;
  if constexpr (PATH == PATH_ASM && TM == 2 && TN == 2 && KS == 1) {
    if (a.ksplit > 1) {  // K split across workgroups: the slices are the second grid dimension
      if (a.ws_cnt == nullptr || a.ws_slots == nullptr || a.ksplit > 65535 || a.K % BK != 0 ||
          a.K / BK - (a.ksplit - 1) * a.ks_per < NSTAGE || a.ks_per < NSTAGE)
        return hipErrorInvalidValue;
      constexpr auto fns = qg_gemm_tile_kernel<MODE, PATH, ROWSUM, NWM, NWN, TM, TN, 0, KS, EPI, true>;
      hipError_t es = qg_allow_smem<fns>(SMEM);
      if (es != hipSuccess) return es;
      hipLaunchKernelGGL(fns, dim3((unsigned)(tiles_m * tiles_n), (unsigned)a.ksplit), dim3(NWM * NWN * KS * 64), SMEM, s, a.A, a.Bp,
                         a.M, a.N, a.K, a.nb16, a.lda, tiles_m, tiles_n, a);
      return hipGetLastError();
    }
  }
  if (a.ksplit > 1) return hipErrorInvalidValue;
  constexpr auto fn = qg_gemm_tile_kernel<MODE, PATH, ROWSUM, NWM, NWN, TM, TN, false, KS, EPI>;
  hipError_t e = qg_allow_smem<fn>(SMEM);
  if (e != hipSuccess) return e;
  hipLaunchKernelGGL(fn, dim3((unsigned)(tiles_m * tiles_n)), dim3(NWM * NWN * KS * 64), SMEM, s, a.A, a.Bp, a.M, a.N, a.K,
                     a.nb16, a.lda, tiles_m, tiles_n, a);
  return hipGetLastError();
}

// which form of the uint8 output pipeline this launch needs (see EPI above).  The one-block waves take the short
// forms too: their pipeline is only 16 values per lane, but a short K with many rows is little else.
template <int BLOCKS>
int epi_form(const qg_gemm_args& a) {
  if (qg_requant_needs_lo_host(a.clamp_lo, a.c_zp)) return EPI_CLAMP;
  return a.c_zp == 0 ? EPI_SAT0 : EPI_SAT;
}
template <int PATH, bool ROWSUM, int NWM, int NWN, int TM, int TN, int KS>
hipError_t launch_requant(const qg_gemm_args& a, hipStream_t s) {
  switch (epi_form<TM * TN>(a)) {
    case EPI_SAT0: return launch<QG_MODE_REQUANT, PATH, ROWSUM, NWM, NWN, TM, TN, KS, EPI_SAT0>(a, s);
    case EPI_SAT: return launch<QG_MODE_REQUANT, PATH, ROWSUM, NWM, NWN, TM, TN, KS, EPI_SAT>(a, s);
    default: return launch<QG_MODE_REQUANT, PATH, ROWSUM, NWM, NWN, TM, TN, KS, EPI_CLAMP>(a, s);
  }
}

// requant mode with / without the row-offset term; the int32 test hook always carries the row sums
template <int PATH, int NWM, int NWN, int TM, int TN, int KS = 1>
hipError_t launch_cfg(const qg_gemm_args& a, int mode, hipStream_t s) {
  if (mode == QG_MODE_REQUANT)
    return a.has_bzp ? launch_requant<PATH, true, NWM, NWN, TM, TN, KS>(a, s)
                     : launch_requant<PATH, false, NWM, NWN, TM, TN, KS>(a, s);
  if (mode == QG_MODE_DEQUANT)
    return a.has_bzp ? launch<QG_MODE_DEQUANT, PATH, true, NWM, NWN, TM, TN, KS>(a, s)
                     : launch<QG_MODE_DEQUANT, PATH, false, NWM, NWN, TM, TN, KS>(a, s);
  return launch<QG_MODE_ACC32, PATH, true, NWM, NWN, TM, TN, KS>(a, s);
}

template <bool ROWSUM, int NWM, int NWN, int TM, int TN, int KS, int EPI, int CONV = 1, int PATH = PATH_PIPE>
hipError_t launch_conv_path(const qg_gemm_args& a, hipStream_t s) {
  constexpr int BM = NWM * TM * 32, BN = NWN * TN * 32;
  constexpr int SMEM = (PATH == PATH_ASM ? asm_stages(TM * TN) : pipe_stages(TM * TN)) * KS * (BM + BN) * BK;
  const int tiles_m = (a.M + BM - 1) / BM, tiles_n = (a.N + BN - 1) / BN;
  const dim3 grid((unsigned)(tiles_m * tiles_n)), block(NWM * NWN * KS * 64);
  constexpr auto fn = qg_gemm_tile_kernel<QG_MODE_REQUANT, PATH, ROWSUM, NWM, NWN, TM, TN, CONV, KS, EPI>;
  hipError_t e = qg_allow_smem<fn>(SMEM);
  if (e != hipSuccess) return e;
  hipLaunchKernelGGL(fn, grid, block, SMEM, s, a.A, a.Bp, a.M, a.N, a.K, a.nb16, a.lda, tiles_m, tiles_n, a);
  return hipGetLastError();
}
// The 128-row tiles take the hand-scheduled loop when it applies: whole 64-channel slices, at most 32 filter taps
// (one validity bit each), enough k tiles to fill its stages, and an image that -- with the 1 KiB the second
// request of a wave is biased by -- lies inside one 4 GiB window (the loop forms the low address word alone).
template <bool ROWSUM, int NWM, int NWN, int TM, int TN, int KS, int EPI>
hipError_t launch_conv_epi(const qg_gemm_args& a, hipStream_t s) {
  if constexpr (TM == 2 && KS == 1) {
    const uintptr_t lo = (uintptr_t)a.A - 1024, hi = (uintptr_t)a.A + (uintptr_t)a.cv_in_bytes - 1;
    if (a.cv_R * a.cv_S <= 32 && a.K / BK >= asm_stages(TM * TN) && (lo >> 32) == (hi >> 32))
      return launch_conv_path<ROWSUM, NWM, NWN, TM, TN, KS, EPI, 1, PATH_ASM>(a, s);
  }
  return launch_conv_path<ROWSUM, NWM, NWN, TM, TN, KS, EPI, 1, PATH_PIPE>(a, s);
}
template <bool ROWSUM, int NWM, int NWN, int TM, int TN, int KS>
hipError_t launch_conv_rs(const qg_gemm_args& a, hipStream_t s) {
  // channel counts that are not a multiple of 64: the per-chunk variant, with the one always-correct output form
  if (a.cv_Cin % BK != 0) return launch_conv_path<ROWSUM, NWM, NWN, TM, TN, KS, EPI_CLAMP, 2>(a, s);
  switch (epi_form<TM * TN>(a)) {
    case EPI_SAT0: return launch_conv_epi<ROWSUM, NWM, NWN, TM, TN, KS, EPI_SAT0>(a, s);
    case EPI_SAT: return launch_conv_epi<ROWSUM, NWM, NWN, TM, TN, KS, EPI_SAT>(a, s);
    default: return launch_conv_epi<ROWSUM, NWM, NWN, TM, TN, KS, EPI_CLAMP>(a, s);
  }
}
template <int NWM, int NWN, int TM, int TN, int KS = 1>
hipError_t launch_conv(const qg_gemm_args& a, hipStream_t s) {
  return a.has_bzp ? launch_conv_rs<true, NWM, NWN, TM, TN, KS>(a, s) : launch_conv_rs<false, NWM, NWN, TM, TN, KS>(a, s);
}

}  // namespace

// Dense convolution: a.A is the NHWC image, a.M the number of output pixels, a.K = R*S*Cin with Cin % 16 == 0.
hipError_t qg_launch_conv_dense(const qg_gemm_args& a, int kernel, hipStream_t s) {
  switch (kernel) {
    case QG_KERNEL_TILE64K1: return launch_conv<2, 2, 1, 1>(a, s);
    case QG_KERNEL_TILE64: return launch_conv<2, 2, 1, 1, 2>(a, s);
    case QG_KERNEL_TILE64K4: return launch_conv<2, 2, 1, 1, 4>(a, s);
    case QG_KERNEL_TILE64X32K8: return launch_conv<2, 1, 1, 1, 8>(a, s);
    case QG_KERNEL_TILE128: return launch_conv<2, 2, 2, 2>(a, s);
    case QG_KERNEL_TILE128X256: return launch_conv<2, 2, 2, 4>(a, s);
    default: return hipErrorInvalidValue;
  }
}

hipError_t qg_launch_gemm_tile(const qg_gemm_args& a, int mode, int kernel, hipStream_t s) {
  // any pointer, lda and K; every byte offset into A fits 32 bits (the caller splits larger matrices by rows)
  switch (kernel) {
    case QG_KERNEL_TILE64: return launch_cfg<PATH_PIPE, 2, 2, 1, 1, 2>(a, mode, s);  // two wave sets split K
    case QG_KERNEL_TILE128:
      if (a.K >= NSTAGE * BK) return launch_cfg<PATH_ASM, 2, 2, 2, 2>(a, mode, s);
      return launch_cfg<PATH_PIPE, 2, 2, 2, 2>(a, mode, s);
    case QG_KERNEL_TILE128X256:
      if (a.K >= asm_stages(8) * BK) return launch_cfg<PATH_ASM, 2, 2, 2, 4>(a, mode, s);
      return launch_cfg<PATH_PIPE, 2, 2, 2, 4>(a, mode, s);
    case QG_KERNEL_TILE64K4: return launch_cfg<PATH_PIPE, 2, 2, 1, 1, 4>(a, mode, s);
    case QG_KERNEL_TILE64K1: return launch_cfg<PATH_PIPE, 2, 2, 1, 1>(a, mode, s);
    case QG_KERNEL_TILE64X32K8: return launch_cfg<PATH_PIPE, 2, 1, 1, 1, 8>(a, mode, s);  // two waves per set
    case QG_KERNEL_TILE256:
      if (a.K >= NSTAGE * BK) return launch_cfg<PATH_ASM, 2, 2, 4, 4>(a, mode, s);
      return launch_cfg<PATH_PIPE, 2, 2, 2, 4>(a, mode, s);
    default: return hipErrorInvalidValue;
  }
}
