// Measurement probes of bench.py (built into libbench_probes.so beside it; not part of libqgemm): what this
// machine sustains on the two resources the kernels are priced against, measured with the same clocks, power
// management and operand statistics as the kernels themselves.  bench.py reports them next to the published peaks.
//
// bp_mfma_i8: a register-only loop of v_mfma_i32_32x32x32_i8 on a 4 x 4 block register tile per wave; `workgroups`
// workgroups of 4 waves run `iters` rounds of 16 matrix instructions each, i.e. workgroups * 4 * iters * 16 * 65536
// operations.  The operands are the first 32 KiB at operands_dev (16-byte aligned, any content: the clock the chip
// holds depends on how many operand bits toggle, so pass bytes distributed like the data of interest).  sink_dev
// receives workgroups * 256 int32 (contents meaningless).
// bp_read: reads `bytes` (a multiple of 16) from src_dev (16-byte aligned) once with `workgroups` workgroups of 256
// threads; sink_dev: one int32.  Both return 0 on success, -1 on a bad argument, -2 if the launch failed.
#include <hip/hip_runtime.h>
#include <stddef.h>
#include <stdint.h>

namespace {

typedef int v4i __attribute__((ext_vector_type(4)));
typedef int v16i __attribute__((ext_vector_type(16)));

// Register-only int8 matrix-core loop: 4 x 4 accumulator blocks per wave (the register tile of the large
// GEMM kernel), operands taken once from memory so that their bit statistics are the caller's -- the power
// the matrix cores draw, and with it the clock the chip holds, depends on how many operand bits toggle.
__global__ __launch_bounds__(256, 1) void bp_mfma_kernel(const v4i* __restrict__ operands, int32_t* __restrict__ sink,
                                                               int iters) {
  v16i acc[4][4];
#pragma unroll
  for (int i = 0; i < 4; ++i)
#pragma unroll
    for (int j = 0; j < 4; ++j)
#pragma unroll
      for (int r = 0; r < 16; ++r) acc[i][j][r] = 0;
  v4i a[4], b[4];
  const int t = threadIdx.x;  // 256 lanes x 8 fragments x 16 B = 32 KiB of operands, the same for every workgroup
#pragma unroll
  for (int i = 0; i < 4; ++i) {
    a[i] = operands[(i * 256) + t];
    b[i] = operands[((4 + i) * 256) + t];
  }
  for (int it = 0; it < iters; ++it) {
#pragma unroll
    for (int i = 0; i < 4; ++i)
#pragma unroll
      for (int j = 0; j < 4; ++j) acc[i][j] = __builtin_amdgcn_mfma_i32_32x32x32_i8(b[j], a[i], acc[i][j], 0, 0, 0);
    a[it & 3].x ^= it;  // keeps the operands from being loop-invariant
  }
  int s = 0;
#pragma unroll
  for (int i = 0; i < 4; ++i)
#pragma unroll
    for (int j = 0; j < 4; ++j)
#pragma unroll
      for (int r = 0; r < 16; ++r) s += acc[i][j][r];
  sink[blockIdx.x * 256 + t] = s;
}

// Streaming read: every 16-byte word of the buffer once, grid-stride, nothing written unless a checksum matches.
__global__ __launch_bounds__(256) void bp_read_kernel(const v4i* __restrict__ src, size_t n16, int32_t* __restrict__ sink) {
  size_t i = (size_t)blockIdx.x * 256 + threadIdx.x;
  const size_t stride = (size_t)gridDim.x * 256;
  int s = 0;
  for (; i < n16; i += stride) {
    const v4i v = src[i];
    s += v.x ^ v.y ^ v.z ^ v.w;
  }
  if (s == 0x12345678) sink[0] = s;
}

}  // namespace

extern "C" {

int bp_mfma_i8(const void* operands_dev, int32_t* sink_dev, int workgroups, int iters, void* stream) {
  if (!operands_dev || !sink_dev || workgroups <= 0 || workgroups > 65535 || iters <= 0) return -1;
  if (((uintptr_t)operands_dev & 15) != 0) return -1;
  hipLaunchKernelGGL(bp_mfma_kernel, dim3((unsigned)workgroups), dim3(256), 0, static_cast<hipStream_t>(stream),
                     static_cast<const v4i*>(operands_dev), sink_dev, iters);
  return hipGetLastError() == hipSuccess ? 0 : -2;
}

int bp_read(const void* src_dev, size_t bytes, int32_t* sink_dev, int workgroups, void* stream) {
  if (!src_dev || !sink_dev || bytes == 0 || bytes % 16 != 0 || workgroups <= 0 || workgroups > 1048576) return -1;
  if (((uintptr_t)src_dev & 15) != 0) return -1;
  hipLaunchKernelGGL(bp_read_kernel, dim3((unsigned)workgroups), dim3(256), 0, static_cast<hipStream_t>(stream),
                     static_cast<const v4i*>(src_dev), bytes / 16, sink_dev);
  return hipGetLastError() == hipSuccess ? 0 : -2;
}

}  // extern "C"
