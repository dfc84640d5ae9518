// Dense "same" convolution (stride 1, 2*pad == R-1 == S-1, Cin a multiple of 32) with the input PATCH resident in
// LDS.  The paper only names convolution (Sec. 1); the arithmetic is Eq. (2) and the requantization pipeline of the
// GEMM, with out-of-image taps carrying theta_A (real zero).
//
// The im2col matrix of such a layer repeats every input byte R*S times.  The GEMM-shaped kernels fetch each repeat
// from L2 again (R*S times the image through L2 -> LDS, one stage of latency per 64-deep step).  Here a workgroup
// owns TP consecutive output pixels of the linear NHWC pixel sequence: the input pixel of tap (kh, kw) of output
// pixel q is pixel q + (kh-pad)*W + (kw-pad) of the same sequence, so ONE contiguous run of TP + (R-1)*W + (S-1)
// pixels holds every tap of the tile.  It is requested in one burst (one memory latency per workgroup); the A
// operand of an MFMA is then 16 consecutive channel bytes of a patch pixel, read from LDS at a per-lane address:
// pixel base + tap offset (scalar) + channel offset.  Taps outside the image are redirected, by address, to a row
// of theta_A bytes in LDS, so the consume path has no select.  Only the weights stream: 64-deep slabs of the packed
// GEMM matrix through a ring of LDS stages, the same bytes for every workgroup (L2 hits).
//
// Patch layout: pixel pp at pp * PS bytes, PS = Cin rounded up to an ODD number of 16-byte chunks: the 16 consecutive
// pixels that a quarter-wave reads at one channel offset then fall into 16 different 16-byte bank groups with no
// swizzle, which keeps the channel offset an address immediate.  The pad chunk is requested from the table of
// constant rows like every out-of-buffer chunk (a request always writes 64 consecutive chunks).
#include "qg_internal.h"
#include <type_traits>
#include <utility>

namespace {

typedef int v4i __attribute__((ext_vector_type(4)));
typedef int v16i __attribute__((ext_vector_type(16)));

// ring of weight slabs: one consumed, the next landed, one being freed, the others in flight (an L2 hit takes about as
// long as four slabs of MFMAs: the deep ring is as deep as 48 KiB of LDS allow).  The shallow ring is for the launches
// in which it lets a CU hold one more workgroup and there are workgroups to fill the places: the other workgroups'
// waves then cover the latency that the ring no longer does.
constexpr int ring_slabs(int tn, bool deep) { return deep ? (tn <= 64 ? 8 : 6) : (tn <= 64 ? 4 : 3); }

// slab(0) && slab(1) && ... && slab(N-1): the ring, unrolled
template <class F, int... Is>
__device__ __forceinline__ bool once_round_the_ring(F& slab, std::integer_sequence<int, Is...>) {
  return (... && slab(std::integral_constant<int, Is>{}, std::false_type{}));
}
// slab(1) && ... && slab(N)
template <class F, int... Is>
__device__ __forceinline__ bool rest_of_the_ring(F& slab, std::integer_sequence<int, Is...>) {
  return (... && slab(std::integral_constant<int, Is + 1>{}, std::false_type{}));
}

// The requests (global memory straight into LDS, 16 or 4 bytes per lane, at lds + lane * size; lds wave-uniform) are
// written out: the compiler orders every LDS read behind every request of its own that may still be in flight
// (s_waitcnt vmcnt(0) in front of the fragment reads, i.e. one full memory latency per slab), so it must not see
// them; the waits that order the reads behind the requests they depend on are written out too (they complete in
// order).
__device__ __forceinline__ unsigned lds_addr(const void* p) {
  return (unsigned)(uintptr_t)((__attribute__((address_space(3))) const unsigned char*)p);
}
// per-lane 64-bit address
__device__ __forceinline__ void request16(const void* addr, unsigned lds) {
  asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %1, off" ::"s"(lds), "v"(addr) : "memory");
}
__device__ __forceinline__ void request4(const void* addr, unsigned lds) {
  asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tglobal_load_lds_dword %1, off" ::"s"(lds), "v"(addr) : "memory");
}
// N consecutive KiB: wave-uniform base (scalar registers) + per-lane byte offset
template <int N>
__device__ __forceinline__ void request_kib(const void* base, unsigned voff, unsigned lds) {
  static_assert(N == 1 || N == 2, "one or two fragments per wave and slab");
  if (N == 1)
    asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %1, %2" ::"s"(lds), "v"(voff), "s"(base) : "memory");
  else
    asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %1, %2\n\tglobal_load_lds_dwordx4 %1, %2 offset:1024"
                 ::"s"(lds), "v"(voff), "s"(base) : "memory");
}

template <int N>
__device__ __forceinline__ void wait_vmcnt() {
  asm volatile("s_waitcnt vmcnt(%0)" ::"n"(N) : "memory");
}

// WM x WN waves of MB x NBW blocks of 32 x 32: the workgroup owns TP = WM*MB*32 pixels x TN = WN*NBW*32 channels.
// C64: Cin is a multiple of 64, so every 64-deep weight slab lies inside one filter tap.  (Inside: ps = bytes per
// patch pixel in LDS; patch_chunks = 16-byte chunks requested for the patch, a multiple of the workgroup size, the
// same formula as the host's LDS sizing; halo = pad*W + pad = pixels in front of the tile's first.)
//
// A wave alone on its SIMD issues one instruction every four cycles or so, an MFMA of this shape occupies the pipe
// for 32: whatever the main loop does per MFMA beyond its operand reads costs time.  So the uint8 -> int8 shift
// (xor 0x80) and the byte sums for the row offsets are NOT done per fragment: once the patch has landed, every
// thread flips the bytes of whole patch pixels in place and leaves each pixel's channel sum in LDS; the row offset
// of an output pixel is then the sum of R*S of those (or Cin * theta_A for a tap outside the image).
template <int WM, int WN, int MB, int NBW, bool HAS_BZP, bool C64, bool DEEP>
__global__ __launch_bounds__(WM* WN * 64) void qg_conv_patch_kernel(
    const uint8_t* const in, const int8_t* const Bp, const int npix, const int W, const int H, const int N, const int nb16,
    const int cpix, const int geom, const qg_gemm_args p) {
  // The leading scalar arguments repeat what the request burst needs (cpix = Cin | bytes per image pixel << 16,
  // geom = R | S << 8 | pad << 16 | theta_A << 24): the file is compiled with kernel-argument preloading, so they
  // arrive in scalar registers with the wave (the first 14 dwords do), and the cold trip to the argument buffer
  // for the rest of p (first used after the burst) overlaps the patch's own.
  constexpr int NW = WM * WN, NT = NW * 64;
  constexpr int TP = WM * MB * 32, TN = WN * NBW * 32;
  constexpr int STAGE = TN * QG_FRAG_K;           // bytes of one 64-deep slab of TN columns
  constexpr int NSTAGE = ring_slabs(TN, DEEP);
  constexpr int FPS = TN / QG_FRAG_COLS;          // fragments per slab
  // Requests per wave: the same number for every wave that requests at all, so the waits are constant counts; with
  // more waves than requests the first waves issue one each and the others' waits are satisfied trivially.
  static_assert(FPS % NW == 0 || NW % FPS == 0, "whole requests per wave");
  constexpr int RPW = FPS >= NW ? FPS / NW : 1;   // requests per (requesting) wave and slab
  constexpr int PARTS = TN / 64;                  // requests per array of column constants
  static_assert((4 * PARTS) % NW == 0 || NW % (4 * PARTS) == 0, "whole requests per wave");
  constexpr int CPW = 4 * PARTS >= NW ? 4 * PARTS / NW : 1;  // constant requests per (requesting) wave

  const int tid = threadIdx.x, lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int wave_m = wave % WM, wave_n = wave / WM;
  const int l32 = lane & 31, lg = lane >> 5;
  const int R = geom & 255, S = (geom >> 8) & 255, pad = (geom >> 16) & 255, azp = (geom >> 24) & 255;
  const int Cin = cpix & 0xFFFF, pix = (int)((unsigned)cpix >> 16), K = R * S * Cin;
  const int nc = Cin >> 4, psc = nc | 1, ps = psc << 4;  // an odd number of 16-byte chunks per patch pixel
  const int npp = TP + (R - 1) * W + (S - 1);            // patch pixels
  const int patch_chunks = (npp * psc + NT - 1) / NT * NT;
  const int halo = pad * W + pad;

  extern __shared__ __align__(16) unsigned char smem[];
  const int theta_bytes = (ps + 63) & ~63;
  unsigned char* const theta_s = smem;                         // ps bytes of theta_A (flipped)
  unsigned char* const patch = smem + theta_bytes;
  unsigned char* const ring = patch + patch_chunks * 16;
  int* const cj_s = reinterpret_cast<int*>(ring + NSTAGE * STAGE);  // lands as bias, becomes bias - (theta_A - 128) * col_off
  int* const nbz_s = cj_s + TN;                                     // lands as theta_B, becomes -theta_B
  float* const sc_s = reinterpret_cast<float*>(nbz_s + TN);
  int* const coff_s = reinterpret_cast<int*>(sc_s + TN);            // column offsets
  int* const psum_s = coff_s + TN;                                  // npp channel sums of the patch pixels

  // Workgroup -> (pixel tile, channel slice).  Workgroup ids go round-robin over the 8 XCDs: each XCD walks its own
  // contiguous eighth of the pixel tiles (neighbouring tiles share their halo rows in one L2), the channel slices
  // of a tile back to back on the same XCD.
  int tile, slice;
  {
    const int ntile = (npix + TP - 1) / TP, id = blockIdx.x;
    if (N <= TN) {  // one slice: no division
      slice = 0;
      tile = (ntile & 7) == 0 ? (id & 7) * (ntile >> 3) + (id >> 3) : id;
    } else {
      const int nslice = (N + TN - 1) / TN;
      if ((ntile & 7) == 0) {
        const int j = id >> 3;
        slice = j % nslice;
        tile = (id & 7) * (ntile >> 3) + j / nslice;
      } else {
        slice = id % nslice;
        tile = id / nslice;
      }
    }
  }
  const int m0 = tile * TP, n0 = slice * TN;
  const int lin0 = m0 - halo;  // linear index of patch pixel 0 (may be negative)

  // ---- the requests of the patch, one burst
  {
    const int c = wave * 64 + lane;
    int pp = (int)((float)c / (float)psc);  // c < 2^16 and psc < 2^8: the rounded quotient is off by one at most
    int ch = c - pp * psc;
    if (ch < 0) ch += psc, --pp;
    if (ch >= psc) ch -= psc, ++pp;
    const int dpp = NT / psc, dch = NT - dpp * psc;
    const uint8_t* const theta_row = qg_byte_rows.b[azp];
    const unsigned patch_lds = lds_addr(patch);
    for (int c0 = wave * 64; c0 < patch_chunks; c0 += NT) {
      const int lin = lin0 + pp;
      const bool ok = ch < nc && (unsigned)lin < (unsigned)npix;
      const uint8_t* src = ok ? in + (size_t)lin * pix + (ch << 4) : theta_row;
      request16(src, patch_lds + c0 * 16);
      pp += dpp;
      ch += dch;
      if (ch >= psc) ch -= psc, ++pp;
    }
  }
  const int nkb = (K + QG_FRAG_K - 1) / QG_FRAG_K;  // 64-deep slabs that hold weights
  const size_t b_step = (size_t)nb16 * QG_FRAG_BYTES;
  // Requests the next slab (they are requested in order, each into the next slot of the ring).  A slab past the last
  // is requested again from the last one, into a slot nobody reads any more: every iteration issues the same number
  // of requests, so the wait counts below are constants.
  const int8_t* req_src = Bp + ((size_t)(n0 / QG_FRAG_COLS) + wave * RPW) * QG_FRAG_BYTES;  // wave-uniform
  int req_kb = 0;
  const unsigned ring_w = lds_addr(ring) + wave * RPW * QG_FRAG_BYTES;
  auto request_slab = [&](int slot) {
    if (FPS >= NW || wave < FPS) request_kib<RPW>(req_src, (unsigned)(lane * 16), ring_w + slot * STAGE);
    req_src += ++req_kb < nkb ? b_step : 0;
  };
  // the row of (flipped) theta_A bytes
  for (int c = tid; c < (ps >> 2); c += NT)
    reinterpret_cast<unsigned*>(theta_s)[c] = ((unsigned)azp * 0x01010101u) ^ 0x80808080u;

  // ---- this lane's pixels: patch address of tap (0, 0), and which taps lie inside the image.  The wave's first
  // pixel is divided once (wave-uniform), the lanes walk on from there.
  unsigned pixaddr[MB], tapok[MB];  // tapok: bit t = tap t (row major) lies inside the image
  {
    const int mw = min(m0 + wave_m * MB * 32, npix - 1);
    const int wo0 = mw % W, ho0 = (mw / W) % H;
#pragma unroll
    for (int mb = 0; mb < MB; ++mb) {
      const int lp = (wave_m * MB + mb) * 32 + l32;
      int wo = wo0 + mb * 32 + l32, ho = ho0;
      while (wo >= W) {
        wo -= W;
        ho = ho + 1 == H ? 0 : ho + 1;
      }
      // filter rows kh with 0 <= ho + kh - pad < H: bits [max(pad - ho, 0), min(H + pad - ho, R)); columns alike
      const unsigned rows = ((1u << min(H + pad - ho, R)) - 1u) & ~((1u << max(pad - ho, 0)) - 1u);
      const unsigned cols = ((1u << min(W + pad - wo, S)) - 1u) & ~((1u << max(pad - wo, 0)) - 1u);
      unsigned mask = 0;
      for (int kh = 0; kh < R; ++kh) mask |= ((rows >> kh) & 1u ? cols : 0u) << (kh * S);
      tapok[mb] = m0 + lp < npix ? mask : 0u;  // rows past the last pixel read the theta row
      pixaddr[mb] = (unsigned)(theta_bytes + lp * ps + lg * 16);
    }
  }

  // The first NSTAGE - 1 weight slabs: behind the pixel set-up, which ran while the texture addresser worked through
  // the patch requests (a wave cannot issue past a full request queue).
#pragma unroll
  for (int u = 0; u < NSTAGE - 1; ++u) request_slab(u);
  // The column constants of the output pipeline (first use of the arguments that are not preloaded): four arrays of
  // TN entries, 64 per request, straight to LDS like everything else, so every wait below is a constant count.
  // They are needed after the main loop.
#pragma unroll
  for (int i = 0; i < CPW; ++i) {
    if (FPS < NW && wave >= FPS) break;
    const int q = wave + i * NW, arr = q / PARTS, part = q % PARTS;
    const int oc = min(n0 + part * 64 + lane, N - 1);  // columns past N read a valid entry that is never used
    const void* src = arr == 0 ? (const void*)((p.bias ? p.bias : p.col_off) + oc)
                    : arr == 1 ? (const void*)(p.bzp + oc)
                    : arr == 2 ? (const void*)(p.scales + (size_t)oc * p.scale_stride)
                               : (const void*)(p.col_off + oc);
    request4(src, lds_addr(cj_s + arr * TN + part * 64));
  }

  // ---- the patch has landed (weights and constants may still be in flight): flip its bytes, sum its pixels
  static_assert(4 * PARTS == FPS, "the waves that request weights are the ones that request constants");
  if (FPS >= NW || wave < FPS)
    wait_vmcnt<(NSTAGE - 1) * RPW + CPW>();
  else
    wait_vmcnt<0>();  // a wave without weight and constant requests has only its patch requests in flight
  __syncthreads();
  for (int pp = tid; pp < npp; pp += NT) {
    unsigned char* const px = patch + pp * ps;
    unsigned sum = 0;
#pragma unroll 4
    for (int c = 0; c < nc; ++c) {
      v4i v = *reinterpret_cast<const v4i*>(px + c * 16);
      if (HAS_BZP) {
        sum = __builtin_amdgcn_sad_u8(v.x, 0u, sum);
        sum = __builtin_amdgcn_sad_u8(v.y, 0u, sum);
        sum = __builtin_amdgcn_sad_u8(v.z, 0u, sum);
        sum = __builtin_amdgcn_sad_u8(v.w, 0u, sum);
      }
      *reinterpret_cast<v4i*>(px + c * 16) = v ^ (int)0x80808080;
    }
    if (HAS_BZP) psum_s[pp] = (int)sum;
  }
  // everything requested so far has landed; the column constants become what the output pipeline uses
  wait_vmcnt<0>();
  __syncthreads();  // flipped patch, pixel sums, everybody's constants
  static_assert(TN <= NT, "one column constant per thread");
  if (tid < TN) {
    cj_s[tid] = (p.bias ? cj_s[tid] : 0) - p.a_zp_m128 * coff_s[tid];
    nbz_s[tid] = -nbz_s[tid];
  }
  // row offsets of this lane's pixels, int8 domain: sum over the taps of (channel sum, or Cin * theta_A outside) - 128 K.
  // A filter row's reads are issued together (up to five columns; a column the filter does not have reads the last
  // one again and counts nothing), so the loop pays one LDS latency per filter row.
  int rsum[MB];
  if (HAS_BZP) {
    const int outside = Cin * azp;
#pragma unroll
    for (int mb = 0; mb < MB; ++mb) rsum[mb] = -128 * K;
    const int* const ps0 = psum_s + (wave_m * MB) * 32 + l32;
    for (int kh = 0; kh < R; ++kh) {
      int v[MB][5];
#pragma unroll
      for (int mb = 0; mb < MB; ++mb)
#pragma unroll
        for (int j = 0; j < 5; ++j) v[mb][j] = ps0[mb * 32 + kh * W + min(j, S - 1)];
#pragma unroll
      for (int mb = 0; mb < MB; ++mb)
#pragma unroll
        for (int j = 0; j < 5; ++j) {
          const int here = (tapok[mb] >> (kh * S + min(j, S - 1))) & 1u ? v[mb][j] : outside;
          rsum[mb] += j < S ? here : 0;
        }
    }
  }
  __syncthreads();  // cj_s, nbz_s
  // The accumulators start at bias - (theta_A - 128) * column offset: it is the C operand of the first step's MFMAs
  // (no instruction to initialise them, nothing to add in the output pipeline).
  v16i cj0[NBW];
#pragma unroll
  for (int nb = 0; nb < NBW; ++nb)
#pragma unroll
    for (int q = 0; q < 4; ++q) {
      const v4i cj = *reinterpret_cast<const v4i*>(&cj_s[(wave_n * NBW + nb) * 32 + 16 * lg + 4 * q]);
#pragma unroll
      for (int r = 0; r < 4; ++r) cj0[nb][4 * q + r] = cj[r];
    }
  v16i acc[MB][NBW];

  // ---- main loop: one weight slab (two MFMA k steps of 32) per barrier.  The operand fragments of a step are read
  // from LDS one step ahead of their MFMAs, so slab kb + 1 must have landed when slab kb is consumed: one slab
  // consumed, the next landed, one being freed, NSTAGE - 3 in flight.  The loop is unrolled over the ring, so that
  // every ring address is an immediate: a wave alone on its SIMD pays for every instruction.
  const unsigned b_lane = (unsigned)((wave_n * NBW * 2 + (l32 >> 4)) * QG_FRAG_BYTES + (l32 & 15) * 16 + lg * 256) +
                          (unsigned)(ring - smem);
  // the walk along k: tap index, its patch offset, 64- (C64) or 32-channel block of the tap
  int tap = 0, kw = 0, cc = 0;
  unsigned tapoff = 0;
  unsigned abase[MB];  // LDS address of the walk's channel block (+ this lane's half) in the walk's tap, or in the theta row
  auto set_tap = [&]() {
#pragma unroll
    for (int mb = 0; mb < MB; ++mb) {
      const unsigned in = (unsigned)__builtin_amdgcn_sbfe((int)tapok[mb], tap, 1);  // all ones if the tap is inside the image
      abase[mb] = (in & (pixaddr[mb] + tapoff)) | (~in & (unsigned)(lg * 16));
    }
  };
  constexpr int CSTEP = C64 ? 64 : 32;
  const int ncc = Cin / CSTEP;
  const unsigned row_step = (unsigned)((W - S + 1) * ps);
  auto advance = [&]() {  // on to the next channel block, or the next tap
    if (++cc == ncc) {
      cc = 0;
      ++tap;
      const bool wrap = ++kw == S;
      kw = wrap ? 0 : kw;
      tapoff += wrap ? row_step : (unsigned)ps;
      set_tap();
    } else {
#pragma unroll
      for (int mb = 0; mb < MB; ++mb) abase[mb] += CSTEP;
    }
  };
  auto read_a = [&](v4i(&af)[MB], int off) {
#pragma unroll
    for (int mb = 0; mb < MB; ++mb) af[mb] = *reinterpret_cast<const v4i*>(smem + abase[mb] + off);
  };
  auto read_b = [&](v4i(&bf)[NBW], int slot, int ks) {
#pragma unroll
    for (int nb = 0; nb < NBW; ++nb)
      bf[nb] = *reinterpret_cast<const v4i*>(smem + b_lane + slot * STAGE + ks * 512 + nb * 2 * QG_FRAG_BYTES);
  };
  auto mfmas = [&](const v4i(&af)[MB], const v4i(&bf)[NBW], auto first_tag) {
#pragma unroll
    for (int mb = 0; mb < MB; ++mb)
#pragma unroll
      for (int nb = 0; nb < NBW; ++nb)
        acc[mb][nb] = __builtin_amdgcn_mfma_i32_32x32x32_i8(bf[nb], af[mb], decltype(first_tag)::value ? cj0[nb] : acc[mb][nb], 0, 0, 0);
  };
  set_tap();
  v4i a0[MB], b0[NBW], a1[MB], b1[NBW];
  read_a(a0, 0);
  read_b(b0, 0, 0);
  if (!C64) advance();
  int kb = 0;
  // one slab, in ring slot U; false after the last
  auto slab = [&](auto u_tag, auto first_tag) {
    constexpr int U = decltype(u_tag)::value, U1 = (U + 1) % NSTAGE, UR = (U + NSTAGE - 1) % NSTAGE;
    // slab kb + 1 has landed (this wave's share, then everybody's); every fragment of slab kb - 1 has been consumed
    wait_vmcnt<(NSTAGE - 3) * RPW>();
    __syncthreads();
    request_slab(UR);  // slab kb + NSTAGE - 1, into the slot of slab kb - 1
    // No branch around the reads: a wait behind a join of paths with different numbers of reads in flight waits
    // for all of them.  Past the end of K the reads fetch bytes nobody uses (the walk stands on a tap that does not
    // exist: the theta row; the next slot holds the last slab again), and a second step that K does not have
    // multiplies the zero rows that pad the packed weights to whole slabs.
    if (C64) {
      read_a(a1, 32);
      read_b(b1, U, 1);
      mfmas(a0, b0, first_tag);
      advance();
      read_a(a0, 0);
      read_b(b0, U1, 0);
      mfmas(a1, b1, std::false_type{});
    } else {
      read_a(a1, 0);
      read_b(b1, U, 1);
      advance();
      mfmas(a0, b0, first_tag);
      read_a(a0, 0);
      read_b(b0, U1, 0);
      advance();
      mfmas(a1, b1, std::false_type{});
    }
    ++kb;
    return kb < nkb;
  };
  // the first slab starts the accumulators; then the rest of the first round of the ring, then whole rounds
  if (slab(std::integral_constant<int, 0>{}, std::true_type{}) &&
      rest_of_the_ring(slab, std::make_integer_sequence<int, NSTAGE - 1>{})) {
    while (once_round_the_ring(slab, std::make_integer_sequence<int, NSTAGE>{})) {
    }
  }
  wait_vmcnt<0>();  // the requests past the last slab: nothing may be in flight into LDS when the workgroup ends

  // ---- output pipeline: lane (pixel l32, half lg) holds 16 consecutive output channels of its pixel per block
  const float czp_f = (float)p.c_zp;
  // form 0: explicit lower clamp (ReLU with theta_C != 0); 1: the saturating convert clamps; 2: theta_C == 0, the
  // saturating convert also rounds (qg_requant_pack0)
  auto pipeline = [&](auto form_tag) {
    constexpr int FORM = decltype(form_tag)::value;
    constexpr bool LO = FORM == 0;
#pragma unroll
    for (int mb = 0; mb < MB; ++mb) {
      const int lp = (wave_m * MB + mb) * 32 + l32;
      const int row = m0 + lp;
      const int rs = HAS_BZP ? rsum[mb] : 0;
      if (row >= npix) continue;
#pragma unroll
      for (int nb = 0; nb < NBW; ++nb) {
        const int c_l = (wave_n * NBW + nb) * 32 + 16 * lg;
        const int col = n0 + c_l;
        if (col >= N) continue;
        unsigned out[4];
#pragma unroll
        for (int q = 0; q < 4; ++q) {
          const float4 sc = *reinterpret_cast<const float4*>(&sc_s[c_l + 4 * q]);
          int x0 = acc[mb][nb][4 * q + 0], x1 = acc[mb][nb][4 * q + 1], x2 = acc[mb][nb][4 * q + 2], x3 = acc[mb][nb][4 * q + 3];
          if (HAS_BZP) {
            const v4i nbz = *reinterpret_cast<const v4i*>(&nbz_s[c_l + 4 * q]);
            x0 += __mul24(nbz.x, rs);  // |theta_B| <= 255, |row offset| <= 128 * K < 2^23
            x1 += __mul24(nbz.y, rs);
            x2 += __mul24(nbz.z, rs);
            x3 += __mul24(nbz.w, rs);
          }
          unsigned w;
          if (FORM == 2) {
            w = qg_requant_pack0(x0, sc.x, 0, 0);
            w = qg_requant_pack0(x1, sc.y, 1, w);
            w = qg_requant_pack0(x2, sc.z, 2, w);
            out[q] = qg_requant_pack0(x3, sc.w, 3, w);
          } else {
            w = qg_requant_pack<LO>(x0, sc.x, p.clamp_lo, p.clamp_hi, czp_f, 0, 0);
            w = qg_requant_pack<LO>(x1, sc.y, p.clamp_lo, p.clamp_hi, czp_f, 1, w);
            w = qg_requant_pack<LO>(x2, sc.z, p.clamp_lo, p.clamp_hi, czp_f, 2, w);
            out[q] = qg_requant_pack<LO>(x3, sc.w, p.clamp_lo, p.clamp_hi, czp_f, 3, w);
          }
        }
        uint8_t* dst = p.C + (size_t)row * p.ldc + col;
        if (p.c_vec && col + 16 <= N) {
          *reinterpret_cast<uint4*>(dst) = make_uint4(out[0], out[1], out[2], out[3]);
        } else {
#pragma unroll
          for (int i = 0; i < 16; ++i)
            if (col + i < N) dst[i] = (uint8_t)(out[i >> 2] >> (8 * (i & 3)));
        }
      }
    }
  };
  if (qg_requant_needs_lo(p.clamp_lo, czp_f))
    pipeline(std::integral_constant<int, 0>{});
  else if (p.c_zp != 0)
    pipeline(std::integral_constant<int, 1>{});
  else
    pipeline(std::integral_constant<int, 2>{});
}

constexpr int k_lds_limit = 160 * 1024;

// LDS bytes of a workgroup with the deep or the shallow ring, or 0 when the patch does not fit
template <int WM, int WN, int MB, int NBW>
int patch_smem(const qg_gemm_args& a, bool deep) {
  constexpr int NT = WM * WN * 64, TP = WM * MB * 32, TN = WN * NBW * 32;
  const int nc = a.cv_Cin / 16, psc = nc | 1, ps = psc * 16;
  const long long pixels = (long long)TP + (long long)(a.cv_R - 1) * a.cv_W + (a.cv_S - 1);
  const long long chunks = (pixels * psc + NT - 1) / NT * NT;
  const long long bytes = ((ps + 63) & ~63) + chunks * 16 + (long long)ring_slabs(TN, deep) * TN * QG_FRAG_K + 16 * TN + 4 * pixels;
  return bytes > k_lds_limit ? 0 : (int)bytes;
}

// What a launch of one tiling looks like: which ring, its LDS bytes (0 = the patch does not fit), the workgroups a CU
// holds side by side.  The shallow ring where it raises that number and the grid has workgroups for the places (or
// where only it fits).
struct patch_plan {
  bool deep;
  int lds, per_cu;
};
template <int WM, int WN, int MB, int NBW>
patch_plan plan(const qg_gemm_args& a) {
  constexpr int NT = WM * WN * 64, TP = WM * MB * 32, TN = WN * NBW * 32;
  const int lds_d = patch_smem<WM, WN, MB, NBW>(a, true), lds_s = patch_smem<WM, WN, MB, NBW>(a, false);
  if (lds_s == 0) return {true, 0, 0};
  // the registers of a SIMD hold 4 waves of the four-wave kernels (90 to 100 registers each, with the accumulators),
  // 7 of the eight-wave one-block-row kernel (up to 72), 4 of the 2 x 2 kernel (up to 121), 2 of the 4 x 2 kernel
  // (up to 218): the compiler's report, and tests/test_kernel_resources.py holds it to these
  constexpr int waves_per_simd = MB * NBW >= 8 ? 2 : (MB * NBW == 2 && NT == 512 ? 7 : 4);
  const int by_threads = waves_per_simd * 256 / NT;
  const int cu_d = lds_d ? min(k_lds_limit / lds_d, by_threads) : 0, cu_s = min(k_lds_limit / lds_s, by_threads);
  const long long wgs = (long long)((a.M + TP - 1) / TP) * ((a.N + TN - 1) / TN);
  if (lds_d != 0 && (cu_s <= cu_d || wgs <= 256ll * cu_d)) return {true, lds_d, cu_d};
  return {false, lds_s, cu_s};
}

template <int WM, int WN, int MB, int NBW>
hipError_t launch(const qg_gemm_args& a, hipStream_t s) {
  constexpr int TP = WM * MB * 32, TN = WN * NBW * 32;
  const patch_plan pl = plan<WM, WN, MB, NBW>(a);
  const int smem = pl.lds;
  if (smem == 0) return hipErrorInvalidValue;
  const unsigned grid = (unsigned)((a.M + TP - 1) / TP) * (unsigned)((a.N + TN - 1) / TN);
  auto go3 = [&](auto bzp_tag, auto c64_tag, auto deep_tag) {
    constexpr bool BZP = decltype(bzp_tag)::value, C64 = decltype(c64_tag)::value, DEEP = decltype(deep_tag)::value;
    const hipError_t e = qg_allow_smem<qg_conv_patch_kernel<WM, WN, MB, NBW, BZP, C64, DEEP>>(smem);
    if (e != hipSuccess) return e;
    const int geom = (int)((unsigned)a.cv_R | (unsigned)a.cv_S << 8 | (unsigned)a.cv_pad << 16 | ((unsigned)a.cv_azp & 255u) << 24);
    const int cpix = (int)((unsigned)a.cv_Cin | (unsigned)a.cv_pix << 16);
    hipLaunchKernelGGL((qg_conv_patch_kernel<WM, WN, MB, NBW, BZP, C64, DEEP>), dim3(grid), dim3(WM * WN * 64), smem, s, a.A, a.Bp,
                       a.M, a.cv_W, a.cv_H, a.N, a.nb16, cpix, geom, a);
    return hipGetLastError();
  };
  auto go = [&](auto bzp_tag, auto c64_tag) {
    return pl.deep ? go3(bzp_tag, c64_tag, std::true_type{}) : go3(bzp_tag, c64_tag, std::false_type{});
  };
  const bool c64 = a.cv_Cin % 64 == 0;
  if (a.has_bzp) return c64 ? go(std::true_type{}, std::true_type{}) : go(std::true_type{}, std::false_type{});
  return c64 ? go(std::false_type{}, std::true_type{}) : go(std::false_type{}, std::false_type{});
}

}  // namespace

// Whether the patch kernel takes this convolution (geometry and LDS); `form` selects the workgroup's tile and waves:
// 0 = 64 pixels x 128 channels, 1 = 128 x 64, 2 = 256 x 64 (eight waves), 3 = 256 x 128 (eight waves, 2 x 2 blocks each),
// 4 = 512 x 128 (eight waves, 4 x 2 blocks each).
// Workgroups of the launch that a CU holds side by side; 0 = the kernel does not take the layer.
int qg_conv_patch_per_cu(const qg_gemm_args& a, int form) {
  // a bit per tap, and a few taps past the last
  if (a.cv_stride != 1 || a.cv_R != a.cv_S || a.cv_R % 2 == 0 || 2 * a.cv_pad != a.cv_R - 1 || a.cv_R * a.cv_S > 28) return 0;
  if (a.cv_Ho != a.cv_H || a.cv_Wo != a.cv_W || a.cv_Cin % 32 != 0 || a.cv_pix % 16 != 0 || a.cv_pix >= 65536) return 0;
  if (((uintptr_t)a.A & 15) != 0 || a.K != a.cv_R * a.cv_S * a.cv_Cin) return 0;
  switch (form) {
    case 0: return plan<2, 2, 1, 2>(a).per_cu;
    case 1: return plan<4, 1, 1, 2>(a).per_cu;
    case 2: return plan<8, 1, 1, 2>(a).per_cu;
    case 3: return plan<4, 2, 2, 2>(a).per_cu;
    case 4: return plan<4, 2, 4, 2>(a).per_cu;
  }
  return 0;
}

bool qg_conv_patch_applies(const qg_gemm_args& a, int form) { return qg_conv_patch_per_cu(a, form) != 0; }

hipError_t qg_launch_conv_patch(const qg_gemm_args& a, int form, hipStream_t s) {
  if (!qg_conv_patch_applies(a, form)) return hipErrorInvalidValue;
  switch (form) {
    case 0: return launch<2, 2, 1, 2>(a, s);
    case 1: return launch<4, 1, 1, 2>(a, s);
    case 2: return launch<8, 1, 1, 2>(a, s);
    case 3: return launch<4, 2, 2, 2>(a, s);
    default: return launch<4, 2, 4, 2>(a, s);
  }
}
