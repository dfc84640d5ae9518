// Group-wise convolution (4 input and 4 output channels per group) as one small
// GEMM per group with the im2col addressing fused into the operand fetch: the
// K = R*S*4 vector of an output pixel is gathered tap by tap from the NHWC image
// and never written anywhere.  The paper only names convolution (Sec. 1); the
// arithmetic is the same Eq. (2) + requantization pipeline as the GEMM, with
// out-of-image taps carrying theta_A (real zero).
//
// With 4 channels per group one tap of one group is exactly one dword, i.e. one
// v_dot4_i32_i8 operand, and a 36 x 4 weight block fits in 36 registers.  The
// shape is HBM-bound (36 op/byte), so the matrix cores are not needed to reach
// the memory roofline; the work per pixel is 36 dot4 + the output pipeline.
//
// Thread = (pixel, group): the 32 groups of a pixel are 32 adjacent lanes reading
// one contiguous 128-byte pixel; every thread keeps its group's weights and
// per-channel constants in registers and walks over pixels grid-stride.
#include "qg_internal.h"

namespace {

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

}  // namespace

hipError_t qg_launch_conv_group(const qg_conv_args& a, int RS, hipStream_t s) {
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
