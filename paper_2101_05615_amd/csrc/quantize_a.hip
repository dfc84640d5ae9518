// Activation quantization fp32 -> uint8 (paper Sec. 2.1 Eq. (1) solved for the quantized value; Appendix B:
// a packing routine for A with a simple compute step folded into the bandwidth-bound pass).  The fp32
// matrix is read once and a quarter of its bytes are written; the GEMM then stages the uint8 copy like
// any other activation matrix and takes its row offsets from the staged tiles as usual.
//
// Why this is a pass of its own rather than part of the GEMM's staging: the GEMM requests its tiles with
// global_load_lds, which moves bytes and cannot convert them; a tile of A is staged once per tile COLUMN
// of C, so a conversion inside the staging would be repeated N / tile-width times; and five VALU
// operations per element next to the matrix cores would make the compute-bound shapes VALU-bound.
#include "qg_internal.h"

namespace {

// One thread per 4 consecutive elements of a row (16 bytes in, 4 bytes out), grid-stride.
__global__ __launch_bounds__(256) void qg_quantize_a_kernel(const float* __restrict__ A, int M, int K, int lda,
                                                            float inv, float lo, float hi, float zp_f,
                                                            uint8_t* __restrict__ Aq, int ldq, int vec) {
  const int k4 = (K + 3) >> 2;
  const long long total = (long long)M * k4;
  const long long step = (long long)gridDim.x * blockDim.x;
  for (long long t = (long long)blockIdx.x * blockDim.x + threadIdx.x; t < total; t += step) {
    const int row = (int)(t / k4);
    const int k = (int)(t - (long long)row * k4) * 4;
    const float* src = A + (size_t)row * lda + k;
    uint8_t* dst = Aq + (size_t)row * ldq + k;
    if (vec && k + 4 <= K) {
      const float4 v = *reinterpret_cast<const float4*>(src);
      unsigned w = qg_quantize_pack(v.x, inv, lo, hi, zp_f, 0, 0);
      w = qg_quantize_pack(v.y, inv, lo, hi, zp_f, 1, w);
      w = qg_quantize_pack(v.z, inv, lo, hi, zp_f, 2, w);
      w = qg_quantize_pack(v.w, inv, lo, hi, zp_f, 3, w);
      *reinterpret_cast<unsigned*>(dst) = w;
    } else {
      for (int i = 0; i < 4 && k + i < K; ++i) dst[i] = (uint8_t)qg_quantize_pack(src[i], inv, lo, hi, zp_f, 0, 0);
    }
  }
}

}  // namespace

hipError_t qg_launch_quantize_a(const float* A, int M, int K, int lda, float inv_scale, int a_zp, uint8_t* Aq,
                                int ldq, hipStream_t s) {
  const int vec = (reinterpret_cast<uintptr_t>(A) % 16 == 0) && (lda % 4 == 0) &&
                  (reinterpret_cast<uintptr_t>(Aq) % 4 == 0) && (ldq % 4 == 0);
  const long long total = (long long)M * ((K + 3) / 4);
  long long blocks = (total + 255) / 256;
  if (blocks > 256 * 32) blocks = 256 * 32;  // a few thousand resident waves; the loop covers the rest
  hipLaunchKernelGGL(qg_quantize_a_kernel, dim3((unsigned)blocks), dim3(256), 0, s, A, M, K, lda, inv_scale,
                     (float)(0 - a_zp), (float)(255 - a_zp), (float)a_zp, Aq, ldq, vec);
  return hipGetLastError();
}
