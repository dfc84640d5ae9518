// Group-wise convolution (4 input and 4 output channels per group) as one small
// GEMM per group with the im2col addressing fused into the operand fetch: the
// K = R*S*4 vector of an output pixel is gathered tap by tap from the NHWC image
// and never written anywhere.  The paper only names convolution (Sec. 1); the
// arithmetic is the same Eq. (2) + requantization pipeline as the GEMM, with
// out-of-image taps carrying theta_A (real zero).
//
// Two kernels:
//  * matrix-core kernel (C a multiple of 32).  For one tap, 32 adjacent channels (8 groups) of 32 pixels
//    against the 32 matching output channels is a 32 x 32 x 32 product whose weight matrix is block
//    diagonal (8 blocks of 4 x 4): one v_mfma_i32_32x32x32_i8 per tap, 9 per 3x3 filter.  7/8 of the MACs
//    multiply zeros, but the shape is HBM-bound (36 op/byte) and the MFMA time stays far below the
//    memory time, while the VALU is left to the output pipeline.  The activation operand is simply the 16
//    contiguous channel bytes of a pixel per lane -- NHWC needs no gather -- and the column permutation
//    of the packed weights leaves each lane with 16 consecutive output channels (one 16-byte store).
//  * dot4 kernel (any C = 4 G): thread = (pixel, group), one tap of one group is one dword = one
//    v_dot4_i32_i8 operand, the 36 x 4 weight block lives in 36 registers.
#include "qg_internal.h"
#include <type_traits>

namespace {

typedef int v4i __attribute__((ext_vector_type(4)));
typedef int v16i __attribute__((ext_vector_type(16)));

// Byte sums of a lane's four dwords (16 input channels of one pixel) -> per dword, the sum over the whole group the
// dword belongs to: groups of 4 channels are the dwords themselves, of 8 pairs of dwords, of 16 the lane's four, of 32
// those of both lanes of the pixel (lanes 32 apart).  lcg = log2(channels per group), uniform.
__device__ __forceinline__ void group_sums(unsigned (&rs)[4], int lcg) {
  if (lcg <= 2) return;
  const unsigned a = rs[0] + rs[1], b = rs[2] + rs[3];
  if (lcg == 3) {
    rs[0] = rs[1] = a;
    rs[2] = rs[3] = b;
    return;
  }
  unsigned t = a + b;
  if (lcg == 5) t += (unsigned)__shfl_xor((int)t, 32);
  rs[0] = rs[1] = rs[2] = rs[3] = t;
}

// Groups of 1 or 2 channels (depthwise and its neighbour) have no dword of their own to sum bytes over: their row
// offsets come from the matrix cores too, as the product with the block-diagonal matrix of ONES of the same group
// structure (RS_MFMA): one more MFMA per tap, on operands that are already in registers, and the sums arrive per
// output channel, in the int8 domain, padding included.  This lane's 16 bytes of that matrix (the same for every tap):
__device__ __forceinline__ v4i ones_fragment(int lane, int lcg) {
  const int oc_l = qg_slot_to_col(lane & 31), g = lane >> 5;
  v4i f;
#pragma unroll
  for (int j = 0; j < 4; ++j) {
    unsigned w = 0;
#pragma unroll
    for (int b = 0; b < 4; ++b)
      if (((16 * g + 4 * j + b) >> lcg) == (oc_l >> lcg)) w |= 1u << (8 * b);
    f[j] = (int)w;
  }
  return f;
}

// NCB 32-channel blocks per wave pass; the workgroup (4 waves) shares their weights in LDS and each wave
// walks over blocks of 32 consecutive output pixels.
template <int R, int S, int NCB, bool HAS_BZP, bool RS_MFMA = false>
__global__ __launch_bounds__(256, HAS_BZP ? 2 : 4) void qg_conv_group_mfma_kernel(const qg_conv_args p) {
  static_assert(!RS_MFMA || HAS_BZP, "row sums are only needed with a nonzero theta_B");
  constexpr int RS = R * S;
  constexpr int NCH = NCB * 32;
  extern __shared__ __align__(16) unsigned char smem[];  // [cb][tap] 1 KiB fragments, then constants
  int* cj_s = reinterpret_cast<int*>(smem + NCB * RS * QG_FRAG_BYTES);
  int* nbz_s = cj_s + NCH;
  float* sc_s = reinterpret_cast<float*>(nbz_s + NCH);

  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int ch0 = blockIdx.y * NCH;  // first channel (input and output) of this workgroup

  // ---- weights of this channel group and per-channel constants into LDS, once per workgroup
  {
    const int8_t* src = p.Wfrag + (size_t)blockIdx.y * NCB * RS * QG_FRAG_BYTES;
    for (int c = tid; c < NCB * RS * 64; c += 256)
      *reinterpret_cast<v4i*>(smem + c * 16) = *reinterpret_cast<const v4i*>(src + (size_t)c * 16);
    for (int c = tid; c < NCH; c += 256) {
      const int oc = ch0 + c;
      cj_s[c] = (p.bias ? p.bias[oc] : 0) - (p.a_zp - 128) * p.col_off[oc];
      nbz_s[c] = -p.bzp[oc];
      sc_s[c] = p.scales[(size_t)oc * p.scale_stride];
    }
  }
  __syncthreads();

  const int pl = lane & 31, g = lane >> 5;  // pixel inside the block, channel half (k half of the MFMA)
  const int npix = p.Nb * p.Ho * p.Wo;
  const int nblk = (npix + 31) / 32;
  const unsigned azp_word = (unsigned)p.a_zp * 0x01010101u;
  const float czp_f = (float)p.c_zp;
  const v4i ones = RS_MFMA ? ones_fragment(lane, p.lcg) : (v4i){0, 0, 0, 0};

  for (int blk = blockIdx.x * 4 + wave; blk < nblk; blk += gridDim.x * 4) {
    const int px = blk * 32 + pl;
    const int pxc = min(px, npix - 1);  // lanes past the end recompute the last pixel; never stored
    const int wo = pxc % p.Wo;
    const int t1 = pxc / p.Wo;
    const int ho = t1 % p.Ho;
    const int n = t1 / p.Ho;

    v16i acc[NCB];
#pragma unroll
    for (int cb = 0; cb < NCB; ++cb)
#pragma unroll
      for (int r = 0; r < 16; ++r) acc[cb][r] = 0;
    unsigned rs[NCB][4];  // byte sums per (block, group inside this lane's 16 channels)
#pragma unroll
    for (int cb = 0; cb < NCB; ++cb)
#pragma unroll
      for (int j = 0; j < 4; ++j) rs[cb][j] = 0;
    v16i racc[RS_MFMA ? NCB : 1];  // RS_MFMA: row offsets per output channel (int8 domain)
    if (RS_MFMA) {
#pragma unroll
      for (int cb = 0; cb < NCB; ++cb)
#pragma unroll
        for (int r = 0; r < 16; ++r) racc[cb][r] = 0;
    }

    // taps one at a time, the next tap's 16-byte loads in flight while this tap's MFMAs run; the
    // scheduling barriers stop the compiler from hoisting all R*S*NCB loads (and their registers) up front
    v4i xn[NCB];
    unsigned keep_n, flip_n;
    auto issue = [&](int tap) {
      const int kh = tap / S, kw = tap % S;
      const int hi = ho * p.stride + kh - p.pad, wi = wo * p.stride + kw - p.pad;
      const bool ok = hi >= 0 && hi < p.H && wi >= 0 && wi < p.W;
      const int hc = min(max(hi, 0), p.H - 1), wc = min(max(wi, 0), p.W - 1);
      const uint8_t* src = p.in + ((size_t)(n * p.H + hc) * p.W + wc) * p.C + ch0 + 16 * g;
      keep_n = ok ? 0xFFFFFFFFu : 0u;
      // in-image: x ^ 0x80 (uint8 -> int8); out of image: theta_A - 128 in every byte
      flip_n = ok ? 0x80808080u : (azp_word ^ 0x80808080u);
#pragma unroll
      for (int cb = 0; cb < NCB; ++cb) xn[cb] = *reinterpret_cast<const v4i*>(src + cb * 32);
    };
    issue(0);
#pragma unroll
    for (int tap = 0; tap < RS; ++tap) {
      v4i x[NCB];
#pragma unroll
      for (int cb = 0; cb < NCB; ++cb) x[cb] = xn[cb];
      const unsigned keep = keep_n, flip = flip_n;
      __builtin_amdgcn_sched_barrier(0);
      if (tap + 1 < RS) issue(tap + 1);
      __builtin_amdgcn_sched_barrier(0);
#pragma unroll
      for (int cb = 0; cb < NCB; ++cb) {
        if (HAS_BZP && !RS_MFMA) {
#pragma unroll
          for (int j = 0; j < 4; ++j) {
            const unsigned y = __builtin_amdgcn_bitop3_b32((unsigned)x[cb][j], keep, azp_word, 0xe2);  // keep ? x : theta_A bytes
            rs[cb][j] = __builtin_amdgcn_sad_u8(y, 0u, rs[cb][j]);
          }
        }
#pragma unroll
        for (int j = 0; j < 4; ++j) x[cb][j] = (int)__builtin_amdgcn_bitop3_b32((unsigned)x[cb][j], keep, flip, 0x6a);  // (x & keep) ^ flip
        const v4i wf = *reinterpret_cast<const v4i*>(smem + (cb * RS + tap) * QG_FRAG_BYTES + lane * 16);
        acc[cb] = __builtin_amdgcn_mfma_i32_32x32x32_i8(wf, x[cb], acc[cb], 0, 0, 0);
        if (RS_MFMA) racc[cb] = __builtin_amdgcn_mfma_i32_32x32x32_i8(ones, x[cb], racc[cb], 0, 0, 0);
      }
    }

    // ---- output pipeline: lane (pixel pl, half g) holds channels 32 cb + 16 g .. + 15 of its pixel
    if (HAS_BZP && !RS_MFMA) {
#pragma unroll
      for (int cb = 0; cb < NCB; ++cb) group_sums(rs[cb], p.lcg);
    }
    if (px < npix) {
      auto pipeline = [&](auto lo_tag) {
      constexpr bool LO = decltype(lo_tag)::value;
#pragma unroll
      for (int cb = 0; cb < NCB; ++cb) {
        const int c_l = cb * 32 + 16 * g;
        unsigned out[4];
#pragma unroll
        for (int q = 0; q < 4; ++q) {
          const v4i cj = *reinterpret_cast<const v4i*>(&cj_s[c_l + 4 * q]);
          const v4i nbz = *reinterpret_cast<const v4i*>(&nbz_s[c_l + 4 * q]);
          const float4 sc = *reinterpret_cast<const float4*>(&sc_s[c_l + 4 * q]);
          // row offset of the group of dword q of this half, in the int8 domain: every one of its RS*Cg bytes is 128 high
          const int rsum = HAS_BZP ? (int)rs[cb][q] - ((128 * RS) << p.lcg) : 0;
          const int r0 = RS_MFMA ? racc[RS_MFMA ? cb : 0][4 * q + 0] : rsum, r1 = RS_MFMA ? racc[RS_MFMA ? cb : 0][4 * q + 1] : rsum;
          const int r2 = RS_MFMA ? racc[RS_MFMA ? cb : 0][4 * q + 2] : rsum, r3 = RS_MFMA ? racc[RS_MFMA ? cb : 0][4 * q + 3] : rsum;
          const int x0 = acc[cb][4 * q + 0] + cj.x + (HAS_BZP ? __mul24(nbz.x, r0) : 0);
          const int x1 = acc[cb][4 * q + 1] + cj.y + (HAS_BZP ? __mul24(nbz.y, r1) : 0);
          const int x2 = acc[cb][4 * q + 2] + cj.z + (HAS_BZP ? __mul24(nbz.z, r2) : 0);
          const int x3 = acc[cb][4 * q + 3] + cj.w + (HAS_BZP ? __mul24(nbz.w, r3) : 0);
          unsigned w = qg_requant_pack<LO>(x0, sc.x, p.clamp_lo, p.clamp_hi, czp_f, 0, 0);
          w = qg_requant_pack<LO>(x1, sc.y, p.clamp_lo, p.clamp_hi, czp_f, 1, w);
          w = qg_requant_pack<LO>(x2, sc.z, p.clamp_lo, p.clamp_hi, czp_f, 2, w);
          out[q] = qg_requant_pack<LO>(x3, sc.w, p.clamp_lo, p.clamp_hi, czp_f, 3, w);
        }
        *reinterpret_cast<uint4*>(p.out + (size_t)px * p.Cout + ch0 + c_l) =
            make_uint4(out[0], out[1], out[2], out[3]);
      }
      };
      if (qg_requant_needs_lo(p.clamp_lo, czp_f))
        pipeline(std::true_type{});
      else
        pipeline(std::false_type{});
    }
  }
}

// 16 bytes per lane from global memory into LDS at lds_base + lane*16 (lds_base wave-uniform)
__device__ __forceinline__ void dma16(const void* gptr, unsigned char* lds_base) {
  __builtin_amdgcn_global_load_lds((const __attribute__((address_space(1))) void*)gptr,
                                   (__attribute__((address_space(3))) void*)lds_base, 16, 0, 0);
}

// "Same" convolution (stride 1, 2*pad == R-1 == S-1): the input pixel of tap (kh, kw) of output pixel q
// is pixel q + (kh-pad)*W + (kw-pad) of the same linear NHWC pixel sequence.  A workgroup owns 128
// consecutive output pixels of one group of NCB*32 channels; it requests its whole input patch (the 128
// pixels plus pad*W+pad on either side) and its weights with global_load_lds in one burst -- one memory
// latency per workgroup -- and every tap then comes from LDS.  Pixel p's 16-byte channel chunks are
// stored swizzled so that the 32 consecutive pixels a half-wave reads hit different banks.
template <int R, int S, int NCB, bool HAS_BZP, bool RS_MFMA = false>
__global__ __launch_bounds__(256, HAS_BZP ? 2 : 3) void qg_conv_same_mfma_kernel(
    const uint8_t* in, const int8_t* Wfrag, const int Nb, const int H, const int W, const int C, const int halo,
    const int nchunks_pad, const qg_conv_args p) {
  static_assert(!RS_MFMA || HAS_BZP, "row sums are only needed with a nonzero theta_B");
  // the leading scalar arguments repeat the fields of p that the request burst needs: the file is compiled with
  // kernel-argument preloading, so they arrive in scalar registers with the wave
  constexpr int RS = R * S;
  constexpr int NCH = NCB * 32;
  constexpr int CP = NCH / 16;       // 16-byte chunks per pixel
  constexpr int PAD_H = (R - 1) / 2, PAD_W = (S - 1) / 2;
  // chunk swizzle of patch pixel pp: the 16 consecutive pixels whose chunk of one index is read in one cycle
  // (8 on parts with 128 B of banks) must fall into different 16-byte bank groups; period 16 pixels
  auto swz = [](int pp) {
    return CP == 8 ? ((pp & 7) ^ ((pp >> 3) & 1)) : (CP == 4 ? (((pp >> 1) & 3) ^ ((pp >> 3) & 1)) : ((pp >> 3) & 1));
  };
  extern __shared__ __align__(16) unsigned char smem[];
  unsigned char* w_s = smem;                                        // [cb][tap] fragments
  int* cj_s = reinterpret_cast<int*>(smem + NCB * RS * QG_FRAG_BYTES);
  int* nbz_s = cj_s + NCH;
  float* sc_s = reinterpret_cast<float*>(nbz_s + NCH);
  unsigned char* patch = smem + NCB * RS * QG_FRAG_BYTES + NCH * 12;

  const int tid = threadIdx.x, lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  // Workgroup -> (pixel tile, channel slice).  Workgroup ids go round-robin over the 8 XCDs.  The slices of one
  // pixel tile touch the two halves of the same 128-byte input and output lines, so they are given ids 8 apart:
  // same XCD, dispatched back to back, and its L2 fetches each input line once and merges the output halves.
  // Each XCD walks its own contiguous eighth of the tile sequence, so neighbouring tiles, whose input patches
  // overlap by the halo rows, also meet in one L2.
  int tile, slice;
  {
    const int nslice = C / NCH, ntile = gridDim.x / nslice, id = blockIdx.x;
    if ((ntile & 7) == 0) {
      const int j = id >> 3;
      slice = j % nslice;
      tile = (id & 7) * (ntile >> 3) + j / nslice;
    } else {
      slice = id % nslice;
      tile = id / nslice;
    }
  }
  const int ch0 = slice * NCH;
  const int q0 = tile * 128;  // first output pixel of the workgroup
  const int npix = Nb * H * W;
  const int lin0 = q0 - halo;       // linear index of patch pixel 0 (may be negative; clamped per chunk)

  // ---- one burst of requests: weights, then the input patch
  {
    const int8_t* wsrc = Wfrag + (size_t)slice * NCB * RS * QG_FRAG_BYTES + lane * 16;
    for (int f = wave; f < NCB * RS; f += 4) dma16(wsrc + (size_t)f * QG_FRAG_BYTES, w_s + f * QG_FRAG_BYTES);
    if (lin0 >= 0 && lin0 + nchunks_pad / CP <= npix) {
      // the whole patch lies inside the buffer: one address per lane, then 256 chunks = 256 / CP pixels further
      // per request (the swizzle has period 16 pixels or less, so it is the same for every request of a lane)
      const int c = wave * 64 + lane;
      const int pp = c / CP, phys = c % CP;
      const uint8_t* src = in + (size_t)(lin0 + pp) * C + ch0 + ((phys ^ swz(pp)) << 4);
      const int step = 256 / CP * C;
      for (int c0 = wave * 64; c0 < nchunks_pad; c0 += 256, src += step) dma16(src, patch + c0 * 16);
    } else {
      for (int c0 = wave * 64; c0 < nchunks_pad; c0 += 256) {
        const int c = c0 + lane;
        const int pp = c / CP, phys = c % CP;
        const int lin = min(max(lin0 + pp, 0), npix - 1);
        dma16(in + (size_t)lin * C + ch0 + ((phys ^ swz(pp)) << 4), patch + c0 * 16);
      }
    }
    for (int c = tid; c < NCH; c += 256) {
      const int oc = ch0 + c;
      cj_s[c] = (p.bias ? p.bias[oc] : 0) - (p.a_zp - 128) * p.col_off[oc];
      nbz_s[c] = -p.bzp[oc];
      sc_s[c] = p.scales[(size_t)oc * p.scale_stride];
    }
  }
  asm volatile("s_waitcnt vmcnt(0)" ::: "memory");  // every request of this wave has landed in LDS ...
  __syncthreads();                                   // ... before any wave reads the others' slots

  const int pl = lane & 31, g = lane >> 5;
  const int px = q0 + wave * 32 + pl;
  // image position of this lane's pixel: the wave's first pixel is divided on the scalar unit, the lane walks
  // pl pixels on from there (a lane past the last pixel gets a position that is never used for a store)
  const int pw0 = q0 + wave * 32;
  int wo = pw0 % W + pl;
  int ho = (pw0 / W) % H;
  for (int i = 31 / W + 1; i > 0; --i) {
    const bool wrap = wo >= W;
    wo -= wrap ? W : 0;
    ho += wrap ? 1 : 0;
    ho = ho == H ? 0 : ho;
  }
  bool row_ok[R], col_ok[S];
#pragma unroll
  for (int kh = 0; kh < R; ++kh) row_ok[kh] = (unsigned)(ho + kh - PAD_H) < (unsigned)H;
#pragma unroll
  for (int kw = 0; kw < S; ++kw) col_ok[kw] = (unsigned)(wo + kw - PAD_W) < (unsigned)W;
  const unsigned azp_word = (unsigned)p.a_zp * 0x01010101u;
  const float czp_f = (float)p.c_zp;
  const int pp_c = wave * 32 + pl + halo;  // patch index of this lane's centre pixel

  // the accumulators start at bias - (theta_A - 128) * column offset, so the output pipeline adds nothing
  v16i acc[NCB];
#pragma unroll
  for (int cb = 0; cb < NCB; ++cb)
#pragma unroll
    for (int q = 0; q < 4; ++q) {
      const v4i cj = *reinterpret_cast<const v4i*>(&cj_s[cb * 32 + 16 * g + 4 * q]);
#pragma unroll
      for (int r = 0; r < 4; ++r) acc[cb][4 * q + r] = cj[r];
    }
  unsigned rs[NCB][4];
#pragma unroll
  for (int cb = 0; cb < NCB; ++cb)
#pragma unroll
    for (int j = 0; j < 4; ++j) rs[cb][j] = 0;
  v16i racc[RS_MFMA ? NCB : 1];  // RS_MFMA: row offsets per output channel (int8 domain)
  const v4i ones = RS_MFMA ? ones_fragment(lane, p.lcg) : (v4i){0, 0, 0, 0};
  if (RS_MFMA) {
#pragma unroll
    for (int cb = 0; cb < NCB; ++cb)
#pragma unroll
      for (int r = 0; r < 16; ++r) racc[cb][r] = 0;
  }

#pragma unroll
  for (int kh = 0; kh < R; ++kh) {
#pragma unroll
    for (int kw = 0; kw < S; ++kw) {
      const bool ok = row_ok[kh] && col_ok[kw];
      const int pp = pp_c + (kh - PAD_H) * W + (kw - PAD_W);
      const unsigned keep = ok ? 0xFFFFFFFFu : 0u;
      // in-image: x ^ 0x80 (uint8 -> int8); out of image: theta_A - 128 in every byte
      const unsigned flip = ok ? 0x80808080u : (azp_word ^ 0x80808080u);
      const unsigned char* src = patch + pp * NCH;
#pragma unroll
      for (int cb = 0; cb < NCB; ++cb) {
        v4i x = *reinterpret_cast<const v4i*>(src + (((cb * 2 + g) ^ swz(pp)) << 4));
        if (HAS_BZP && !RS_MFMA) {
#pragma unroll
          for (int j = 0; j < 4; ++j) {
            const unsigned y = __builtin_amdgcn_bitop3_b32((unsigned)x[j], keep, azp_word, 0xe2);  // keep ? x : theta_A bytes
            rs[cb][j] = __builtin_amdgcn_sad_u8(y, 0u, rs[cb][j]);
          }
        }
#pragma unroll
        for (int j = 0; j < 4; ++j) x[j] = (int)__builtin_amdgcn_bitop3_b32((unsigned)x[j], keep, flip, 0x6a);  // (x & keep) ^ flip
        const v4i wf = *reinterpret_cast<const v4i*>(w_s + (cb * RS + kh * S + kw) * QG_FRAG_BYTES + lane * 16);
        acc[cb] = __builtin_amdgcn_mfma_i32_32x32x32_i8(wf, x, acc[cb], 0, 0, 0);
        if (RS_MFMA) racc[cb] = __builtin_amdgcn_mfma_i32_32x32x32_i8(ones, x, racc[cb], 0, 0, 0);
      }
    }
  }

  // ---- output pipeline: lane (pixel pl, half g) holds channels 32 cb + 16 g .. + 15 of its pixel
  if (HAS_BZP && !RS_MFMA) {
#pragma unroll
    for (int cb = 0; cb < NCB; ++cb) group_sums(rs[cb], p.lcg);
  }
  if (px < npix) {
    auto pipeline = [&](auto lo_tag) {
    constexpr bool LO = decltype(lo_tag)::value;
#pragma unroll
    for (int cb = 0; cb < NCB; ++cb) {
      const int c_l = cb * 32 + 16 * g;
      unsigned out[4];
#pragma unroll
      for (int q = 0; q < 4; ++q) {
        const float4 sc = *reinterpret_cast<const float4*>(&sc_s[c_l + 4 * q]);
        int x0 = acc[cb][4 * q + 0], x1 = acc[cb][4 * q + 1], x2 = acc[cb][4 * q + 2], x3 = acc[cb][4 * q + 3];
        if (HAS_BZP) {
          const v4i nbz = *reinterpret_cast<const v4i*>(&nbz_s[c_l + 4 * q]);
          const int rsum = (int)rs[cb][q] - ((128 * RS) << p.lcg);
          x0 += __mul24(nbz.x, RS_MFMA ? racc[RS_MFMA ? cb : 0][4 * q + 0] : rsum);
          x1 += __mul24(nbz.y, RS_MFMA ? racc[RS_MFMA ? cb : 0][4 * q + 1] : rsum);
          x2 += __mul24(nbz.z, RS_MFMA ? racc[RS_MFMA ? cb : 0][4 * q + 2] : rsum);
          x3 += __mul24(nbz.w, RS_MFMA ? racc[RS_MFMA ? cb : 0][4 * q + 3] : rsum);
        }
        unsigned w = qg_requant_pack<LO>(x0, sc.x, p.clamp_lo, p.clamp_hi, czp_f, 0, 0);
        w = qg_requant_pack<LO>(x1, sc.y, p.clamp_lo, p.clamp_hi, czp_f, 1, w);
        w = qg_requant_pack<LO>(x2, sc.z, p.clamp_lo, p.clamp_hi, czp_f, 2, w);
        out[q] = qg_requant_pack<LO>(x3, sc.w, p.clamp_lo, p.clamp_hi, czp_f, 3, w);
      }
      *reinterpret_cast<uint4*>(p.out + (size_t)px * p.Cout + ch0 + c_l) =
          make_uint4(out[0], out[1], out[2], out[3]);
    }
    };
    if (qg_requant_needs_lo(p.clamp_lo, czp_f))
      pipeline(std::true_type{});
    else
      pipeline(std::false_type{});
  }
}

template <int R, int S>
__global__ __launch_bounds__(256) void qg_conv_group_kernel(const qg_conv_args p, int ppb) {
  constexpr int RS = R * S;
  const int g = threadIdx.x % p.G;
  const int pl = threadIdx.x / p.G;  // pixel slot inside the block
  if (pl >= ppb) return;

  int w[RS][4];
  const int* wp = reinterpret_cast<const int*>(p.Wp) + (size_t)g * RS * 4;
#pragma unroll
  for (int t = 0; t < RS; ++t)
#pragma unroll
    for (int co = 0; co < 4; ++co) w[t][co] = wp[t * 4 + co];

  int cj[4], bz[4];
  float sc[4];
#pragma unroll
  for (int co = 0; co < 4; ++co) {
    const int oc = g * 4 + co;
    bz[co] = p.bzp[oc];
    cj[co] = (p.bias ? p.bias[oc] : 0) - (p.a_zp - 128) * p.col_off[oc];
    sc[co] = p.scales[(size_t)oc * p.scale_stride];
  }
  const int pad_word = ((p.a_zp * 0x01010101) ^ 0x80808080);  // theta_A - 128 in every byte

  const long long npix = (long long)p.Nb * p.Ho * p.Wo;
  const long long step = (long long)gridDim.x * ppb;
  for (long long px = (long long)blockIdx.x * ppb + pl; px < npix; px += step) {
    const int wo = (int)(px % p.Wo);
    const int ho = (int)((px / p.Wo) % p.Ho);
    const int n = (int)(px / ((long long)p.Wo * p.Ho));
    int acc[4] = {0, 0, 0, 0};
    int rsum = 0;
#pragma unroll
    for (int kh = 0; kh < R; ++kh) {
      const int hi = ho * p.stride + kh - p.pad;
#pragma unroll
      for (int kw = 0; kw < S; ++kw) {
        const int wi = wo * p.stride + kw - p.pad;
        int a = pad_word;
        if (hi >= 0 && hi < p.H && wi >= 0 && wi < p.W) {
          a = *reinterpret_cast<const int*>(p.in + (((size_t)n * p.H + hi) * p.W + wi) * p.C + 4 * g);
          a ^= 0x80808080;
        }
        rsum = __builtin_amdgcn_sdot4(a, 0x01010101, rsum, false);
#pragma unroll
        for (int co = 0; co < 4; ++co)
          acc[co] = __builtin_amdgcn_sdot4(a, w[kh * S + kw][co], acc[co], false);
      }
    }
    unsigned out = 0;
#pragma unroll
    for (int co = 0; co < 4; ++co) {
      const int x = acc[co] + cj[co] - bz[co] * rsum;
      out |= (unsigned)qg_requant_one(x, sc[co], p.clamp_lo, p.clamp_hi, p.c_zp) << (8 * co);
    }
    *reinterpret_cast<unsigned*>(p.out + (size_t)px * p.Cout + 4 * g) = out;
  }
}

// Any group shape (G groups of Cg input and Og output channels, any filter): thread = (pixel, output channel),
// output channels fastest so that the bytes of a pixel are stored side by side; the K = R*S*Cg inputs of the
// thread's group are read tap by tap, whole dwords against the [Cout][R*S][Cg4] weight layout (v_dot4_i32_i8)
// when Cg and C are multiples of 4, byte by byte otherwise.  Nothing is tiled: this is the kernel for the
// shapes no other one takes.
template <bool DWORDS>
__global__ __launch_bounds__(256) void qg_conv_group_any_kernel(const qg_conv_args p) {
  const int RS = p.R * p.S, Cg4 = (p.Cg + 3) / 4 * 4;
  const long long total = (long long)p.Nb * p.Ho * p.Wo * p.Cout;
  const int azp_s = p.a_zp - 128;
  const int pad_word = (p.a_zp * 0x01010101) ^ 0x80808080;  // theta_A - 128 in every byte
  for (long long idx = (long long)blockIdx.x * 256 + threadIdx.x; idx < total; idx += (long long)gridDim.x * 256) {
    const int oc = (int)(idx % p.Cout);
    const long long px = idx / p.Cout;
    const int g = oc / p.Og;
    const int wo = (int)(px % p.Wo);
    const int ho = (int)((px / p.Wo) % p.Ho);
    const int n = (int)(px / ((long long)p.Wo * p.Ho));
    const int8_t* w = p.Wany + (size_t)oc * RS * Cg4;
    int acc = 0, rsum = 0;  // both on A - 128
    for (int kh = 0; kh < p.R; ++kh) {
      const int hi = ho * p.stride + kh - p.pad;
      for (int kw = 0; kw < p.S; ++kw, w += Cg4) {
        const int wi = wo * p.stride + kw - p.pad;
        const bool ok = hi >= 0 && hi < p.H && wi >= 0 && wi < p.W;
        const uint8_t* src = p.in + (((size_t)n * p.H + (ok ? hi : 0)) * p.W + (ok ? wi : 0)) * p.C + (size_t)g * p.Cg;
        if (DWORDS) {
          for (int c = 0; c < p.Cg; c += 4) {
            const int a = ok ? (*reinterpret_cast<const int*>(src + c) ^ (int)0x80808080) : pad_word;
            acc = __builtin_amdgcn_sdot4(a, *reinterpret_cast<const int*>(w + c), acc, false);
            rsum = __builtin_amdgcn_sdot4(a, 0x01010101, rsum, false);
          }
        } else {
          for (int c = 0; c < p.Cg; ++c) {
            const int a = ok ? (int)src[c] - 128 : azp_s;
            acc += a * (int)w[c];
            rsum += a;
          }
        }
      }
    }
    const int x = acc + (p.bias ? p.bias[oc] : 0) - azp_s * p.col_off[oc] - p.bzp[oc] * rsum;
    p.out[idx] = (uint8_t)qg_requant_one(x, p.scales[(size_t)oc * p.scale_stride], p.clamp_lo, p.clamp_hi, p.c_zp);
  }
}

// Dense convolution for the extents no requested staging takes (channel counts that are not a multiple of 16 -- the
// three channels of a first layer --, an image that is not 16-byte aligned): the im2col tile is GATHERED, byte by
// byte, into LDS.  Workgroup = 64 output pixels x 64 output channels, four waves of one 32 x 32 block each; per
// 64-deep k chunk every thread gathers 16 consecutive k of one pixel row (walking (channel, kw, kh) as it goes; a tap
// outside the image reads as theta_A, k past K as 0x80, the K padding of every A stage) and copies 16 bytes of the
// packed weights, then two MFMAs per wave.  One stage, two barriers per chunk: K is short where this kernel is used.
// Weights: the packed (R*S*C) x Cout matrix of a GEMM descriptor.
__device__ __forceinline__ int gather_swz(int r) { return ((r >> 1) & 3) ^ ((r >> 3) & 1); }

// GW = bytes per gathered piece: 4 when the channel count is a multiple of 4 and the image 4-byte aligned (a piece is
// then four channels of one tap: a first layer with its RGB input padded to four channels), else 1.
template <bool HAS_BZP, int GW>
__global__ __launch_bounds__(256) void qg_conv_dense_gather_kernel(const qg_conv_args p) {
  __shared__ __align__(16) unsigned char a_s[64 * 64];
  __shared__ __align__(16) unsigned char b_s[4 * QG_FRAG_BYTES];
  __shared__ int cj_s[64], nbz_s[64];
  __shared__ float sc_s[64];
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int wave_m = wave & 1, wave_n = wave >> 1;
  const int l32 = lane & 31, lg = lane >> 5;
  const int npix = p.Nb * p.Ho * p.Wo;
  const int m0 = blockIdx.x * 64, n0 = blockIdx.y * 64;
  const int K = p.R * p.S * p.C, KT = (K + 63) / 64;

  // the row this thread gathers for: pixel position of tap (0, 0)
  const int gr = tid >> 2, gc = tid & 3;
  const int gm = min(m0 + gr, npix - 1);
  const int gwo = gm % p.Wo, gt = gm / p.Wo;
  const int h0 = (gt % p.Ho) * p.stride - p.pad, w0 = gwo * p.stride - p.pad;
  // byte offset of pixel (h0, w0) of this row's image, as if it existed (the image is smaller than 2 GiB)
  const int pix0 = (((gt / p.Ho) * p.H + h0) * p.W + w0) * p.C;
  const int row_step = (p.W - p.S) * p.C;  // from the end of one filter row to the start of the next
  const int8_t* const bsrc = p.Bp + (size_t)(n0 / QG_FRAG_COLS) * QG_FRAG_BYTES + tid * 16;  // 4 KiB per chunk: 256 threads x 16 B
  const size_t b_step = (size_t)p.nb16 * QG_FRAG_BYTES;
  // whole fragments past N_pad do not exist: clamp the copy to the last fragment of the slab (its columns are never stored)
  const int frag_ok = min(4, p.nb16 - n0 / QG_FRAG_COLS);
  const int8_t* const bsrc_c = (tid >> 6) < frag_ok ? bsrc : p.Bp + (size_t)(p.nb16 - 1) * QG_FRAG_BYTES + lane * 16;

  v16i acc;
#pragma unroll
  for (int r = 0; r < 16; ++r) acc[r] = 0;
  unsigned rs = 0;
  if (tid < 64) {  // column constants of the output pipeline (visible behind the barriers of the first chunk)
    const int col = blockIdx.y * 64 + tid;
    const bool in = col < p.Cout;
    cj_s[tid] = in ? (p.bias ? p.bias[col] : 0) - (p.a_zp - 128) * p.col_off[col] : 0;
    nbz_s[tid] = in && HAS_BZP ? -p.bzp[col] : 0;
    sc_s[tid] = in ? p.scales[(size_t)col * p.scale_stride] : 0.0f;
  }

  for (int kc = 0; kc < KT; ++kc) {
    // ---- gather 16 bytes of the im2col row, copy 16 bytes of weights
    struct {
      v4i v;
    } u;
    {
      // (channel, kw, kh) and byte offset of this thread's first k of the chunk, then one byte per step.  Written
      // without branches: every byte is loaded (from offset 0 when its tap lies outside the image) and selected, the
      // walk advances by masks; a branch per byte costs more than the load it saves.
      const int k0 = kc * 64 + gc * 16, tap = k0 / p.C;
      int ci = k0 - tap * p.C, kh = tap / p.S, kw = tap - kh * p.S;
      int off = pix0 + (kh * p.W + kw) * p.C + ci;
      const int nvalid = K - k0;  // bytes of this chunk that belong to the matrix; the rest is the K padding, 0x80
      unsigned w[4] = {0, 0, 0, 0};
#pragma unroll
      for (int i = 0; i < 16; i += GW) {
        const unsigned ok = -(unsigned)((int)(i < nvalid) & (int)((unsigned)(h0 + kh) < (unsigned)p.H) & (int)((unsigned)(w0 + kw) < (unsigned)p.W));
        // (masks, not ?: -- the compiler turns a selected load back into a branch)
        if (GW == 4) {  // K is a multiple of 4 as well: a piece lies inside the matrix or in its padding as a whole
          const unsigned piece = *reinterpret_cast<const unsigned*>(p.in + (off & ok));
          const unsigned other = i < nvalid ? (unsigned)p.a_zp * 0x01010101u : 0x80808080u;
          w[i >> 2] = (piece & ok) | (other & ~ok);
        } else {
          const unsigned byte = p.in[off & ok];
          const unsigned other = i < nvalid ? (unsigned)p.a_zp : 0x80u;
          w[i >> 2] |= ((byte & ok) | (other & ~ok)) << (8 * (i & 3));
        }
        off += GW;
        ci += GW;
        const int wrapc = -(int)(ci == p.C);             // all ones behind the last channel of a pixel
        ci &= ~wrapc;
        kw -= wrapc;
        const int wrapw = wrapc & -(int)(kw == p.S);     // ... of the last pixel of a filter row
        kw &= ~wrapw;
        kh -= wrapw;
        off += wrapw & row_step;
      }
      u.v = (v4i){(int)w[0], (int)w[1], (int)w[2], (int)w[3]};
    }
    const v4i bw = *reinterpret_cast<const v4i*>(bsrc_c + (size_t)kc * b_step);
    __syncthreads();  // the previous chunk's fragments have been read
    *reinterpret_cast<v4i*>(a_s + gr * 64 + ((gc ^ gather_swz(gr)) << 4)) = u.v;
    *reinterpret_cast<v4i*>(b_s + tid * 16) = bw;
    __syncthreads();
#pragma unroll
    for (int ks = 0; ks < 2; ++ks) {
      const int r = wave_m * 32 + l32;
      v4i af = *reinterpret_cast<const v4i*>(a_s + r * 64 + (((ks * 2 + lg) ^ gather_swz(r)) << 4));
      const v4i bf = *reinterpret_cast<const v4i*>(b_s + (wave_n * 2 + (l32 >> 4)) * QG_FRAG_BYTES + (l32 & 15) * 16 + lg * 256 + ks * 512);
      if (HAS_BZP) {
        rs = __builtin_amdgcn_sad_u8(af.x, 0u, rs);
        rs = __builtin_amdgcn_sad_u8(af.y, 0u, rs);
        rs = __builtin_amdgcn_sad_u8(af.z, 0u, rs);
        rs = __builtin_amdgcn_sad_u8(af.w, 0u, rs);
      }
      af = af ^ (int)0x80808080;
      acc = __builtin_amdgcn_mfma_i32_32x32x32_i8(bf, af, acc, 0, 0, 0);
    }
  }

  // ---- output pipeline: lane (row l32, half lg) holds 16 consecutive output channels of its pixel; the column
  // constants were staged by the first 64 threads while the first chunk was gathered
  const int rsum = HAS_BZP ? (int)(rs + (unsigned)__shfl_xor((int)rs, 32)) - 128 * (KT * 64) : 0;
  const int row = m0 + wave_m * 32 + l32;
  const int c_l = wave_n * 32 + lg * 16, col0 = n0 + c_l;
  if (row < npix && col0 < p.Cout) {
    unsigned out[4];
#pragma unroll
    for (int q = 0; q < 4; ++q) {
      unsigned w = 0;
#pragma unroll
      for (int r = 0; r < 4; ++r) {
        const int i = 4 * q + r;
        const int x = acc[i] + cj_s[c_l + i] + (HAS_BZP ? nbz_s[c_l + i] * rsum : 0);
        w |= (unsigned)qg_requant_one(x, sc_s[c_l + i], p.clamp_lo, p.clamp_hi, p.c_zp) << (8 * r);
      }
      out[q] = w;
    }
    uint8_t* dst = p.out + (size_t)row * p.Cout + col0;
    if (col0 + 16 <= p.Cout && (((uintptr_t)p.out | (uintptr_t)p.Cout) & 15) == 0) {
      *reinterpret_cast<uint4*>(dst) = make_uint4(out[0], out[1], out[2], out[3]);
    } else {
#pragma unroll
      for (int i = 0; i < 16; ++i)
        if (col0 + i < p.Cout) dst[i] = (uint8_t)(out[i >> 2] >> (8 * (i & 3)));
    }
  }
}

}  // namespace

hipError_t qg_launch_conv_dense_plain(const qg_conv_args& a, hipStream_t s) {
  const int npix = a.Nb * a.Ho * a.Wo;
  const dim3 grid((unsigned)((npix + 63) / 64), (unsigned)((a.Cout + 63) / 64));
  const bool words = a.C % 4 == 0 && ((uintptr_t)a.in & 3) == 0;
  if (a.has_bzp) {
    if (words)
      hipLaunchKernelGGL((qg_conv_dense_gather_kernel<true, 4>), grid, dim3(256), 0, s, a);
    else
      hipLaunchKernelGGL((qg_conv_dense_gather_kernel<true, 1>), grid, dim3(256), 0, s, a);
  } else {
    if (words)
      hipLaunchKernelGGL((qg_conv_dense_gather_kernel<false, 4>), grid, dim3(256), 0, s, a);
    else
      hipLaunchKernelGGL((qg_conv_dense_gather_kernel<false, 1>), grid, dim3(256), 0, s, a);
  }
  return hipGetLastError();
}

template <int R, int S, int NCB>
hipError_t launch_mfma(const qg_conv_args& a, hipStream_t s) {
  constexpr int RS = R * S;
  const int smem = NCB * RS * QG_FRAG_BYTES + NCB * 32 * 12;
  const int nblk = (a.Nb * a.Ho * a.Wo + 31) / 32;
  const dim3 grid((unsigned)min((nblk + 3) / 4, 2048), (unsigned)(a.C / (NCB * 32)));
  if (a.has_bzp && a.lcg < 2) {  // groups of 1 or 2 channels: row offsets from the matrix cores
    if (hipError_t e = qg_allow_smem<qg_conv_group_mfma_kernel<R, S, NCB, true, true>>(smem); e != hipSuccess) return e;
    hipLaunchKernelGGL((qg_conv_group_mfma_kernel<R, S, NCB, true, true>), grid, dim3(256), smem, s, a);
  } else if (a.has_bzp) {
    if (hipError_t e = qg_allow_smem<qg_conv_group_mfma_kernel<R, S, NCB, true>>(smem); e != hipSuccess) return e;
    hipLaunchKernelGGL((qg_conv_group_mfma_kernel<R, S, NCB, true>), grid, dim3(256), smem, s, a);
  } else {
    if (hipError_t e = qg_allow_smem<qg_conv_group_mfma_kernel<R, S, NCB, false>>(smem); e != hipSuccess) return e;
    hipLaunchKernelGGL((qg_conv_group_mfma_kernel<R, S, NCB, false>), grid, dim3(256), smem, s, a);
  }
  return hipGetLastError();
}

template <int R, int S, int NCB>
hipError_t launch_same(const qg_conv_args& a, int smem, int halo, int nchunks_pad, hipStream_t s) {
  const int npix = a.Nb * a.H * a.W;
  const dim3 grid((unsigned)(((npix + 127) / 128) * (a.C / (NCB * 32))));
  if (a.has_bzp && a.lcg < 2) {  // groups of 1 or 2 channels: row offsets from the matrix cores
    if (hipError_t e = qg_allow_smem<qg_conv_same_mfma_kernel<R, S, NCB, true, true>>(smem); e != hipSuccess) return e;
    hipLaunchKernelGGL((qg_conv_same_mfma_kernel<R, S, NCB, true, true>), grid, dim3(256), smem, s, a.in, a.Wfrag, a.Nb, a.H, a.W, a.C,
                       halo, nchunks_pad, a);
  } else if (a.has_bzp) {
    if (hipError_t e = qg_allow_smem<qg_conv_same_mfma_kernel<R, S, NCB, true>>(smem); e != hipSuccess) return e;
    hipLaunchKernelGGL((qg_conv_same_mfma_kernel<R, S, NCB, true>), grid, dim3(256), smem, s, a.in, a.Wfrag, a.Nb, a.H, a.W, a.C, halo,
                       nchunks_pad, a);
  } else {
    if (hipError_t e = qg_allow_smem<qg_conv_same_mfma_kernel<R, S, NCB, false>>(smem); e != hipSuccess) return e;
    hipLaunchKernelGGL((qg_conv_same_mfma_kernel<R, S, NCB, false>), grid, dim3(256), smem, s, a.in, a.Wfrag, a.Nb, a.H, a.W, a.C, halo,
                       nchunks_pad, a);
  }
  return hipGetLastError();
}

hipError_t qg_launch_conv_group(const qg_conv_args& a, int RS, hipStream_t s) {
  // the matrix-core kernels: block-diagonal 32 x 32 weight fragments exist (Cg == Og in {4, 8, 16, 32}, 1 x 1 or 3 x 3)
  const bool mfma_ok = a.Wfrag != nullptr && ((a.R == 3 && a.S == 3) || (a.R == 1 && a.S == 1)) && a.C % 32 == 0 && a.Cout == a.C &&
                       reinterpret_cast<uintptr_t>(a.in) % 16 == 0 && reinterpret_cast<uintptr_t>(a.out) % 16 == 0;
  // "same" convolution: whole input patch staged in LDS, if it fits
  const int R = RS == 9 ? 3 : 1;
  if (mfma_ok && a.stride == 1 && 2 * a.pad == R - 1 && a.Ho == a.H && a.Wo == a.W) {
    // 64 channels per workgroup: about 35 KB of LDS at W = 56, so four workgroups share a CU and one's
    // request burst overlaps the others' arithmetic (128 channels halve the weight traffic but leave two)
    const int ncb = a.C % 64 == 0 ? 2 : 1;
    const int halo = a.pad * a.W + a.pad;
    const int cp = ncb * 2;
    const int nchunks_pad = ((128 + 2 * halo) * cp + 255) / 256 * 256;
    const int smem = ncb * RS * QG_FRAG_BYTES + ncb * 32 * 12 + nchunks_pad * 16;
    if (smem <= 160 * 1024) {
      if (ncb == 2) return RS == 9 ? launch_same<3, 3, 2>(a, smem, halo, nchunks_pad, s)
                                   : launch_same<1, 1, 2>(a, smem, halo, nchunks_pad, s);
      return RS == 9 ? launch_same<3, 3, 1>(a, smem, halo, nchunks_pad, s)
                     : launch_same<1, 1, 1>(a, smem, halo, nchunks_pad, s);
    }
  }
  // matrix-core kernel with taps fetched from global memory: needs whole 32-channel blocks and 16-byte aligned pixels
  if (mfma_ok && a.C % 32 == 0 && a.Cout == a.C &&
      reinterpret_cast<uintptr_t>(a.in) % 16 == 0 && reinterpret_cast<uintptr_t>(a.out) % 16 == 0) {
    if (a.C % 128 == 0) return RS == 9 ? launch_mfma<3, 3, 4>(a, s) : launch_mfma<1, 1, 4>(a, s);
    return RS == 9 ? launch_mfma<3, 3, 1>(a, s) : launch_mfma<1, 1, 1>(a, s);
  }
  if (a.Wany != nullptr) {
    // the general kernel: one thread per output byte
    const long long total = (long long)a.Nb * a.Ho * a.Wo * a.Cout;
    const unsigned blocks = (unsigned)((total + 255) / 256 < 256LL * 64 ? (total + 255) / 256 : 256LL * 64);
    const bool dwords = a.Cg % 4 == 0 && a.C % 4 == 0 && reinterpret_cast<uintptr_t>(a.in) % 4 == 0;
    if (dwords)
      hipLaunchKernelGGL(qg_conv_group_any_kernel<true>, dim3(blocks), dim3(256), 0, s, a);
    else
      hipLaunchKernelGGL(qg_conv_group_any_kernel<false>, dim3(blocks), dim3(256), 0, s, a);
    return hipGetLastError();
  }
  const int ppb = a.G >= 256 ? 1 : 256 / a.G;
  const int threads = ppb * a.G;
  const long long npix = (long long)a.Nb * a.Ho * a.Wo;
  long long blocks = (npix + ppb - 1) / ppb;
  const long long cap = 256LL * 16;  // a few workgroups per CU; each thread then loops over pixels
  if (blocks > cap) blocks = cap;
  if (RS == 9)
    hipLaunchKernelGGL((qg_conv_group_kernel<3, 3>), dim3((unsigned)blocks), dim3(threads), 0, s, a, ppb);
  else
    hipLaunchKernelGGL((qg_conv_group_kernel<1, 1>), dim3((unsigned)blocks), dim3(threads), 0, s, a, ppb);
  return hipGetLastError();
}
