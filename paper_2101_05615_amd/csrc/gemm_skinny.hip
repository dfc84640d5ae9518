// Small-batch quantized GEMM (M <= 64): the bandwidth-bound case the paper
// stresses ("M is sometimes very small", Appendix C; int32 accumulation for the
// bandwidth-bound shapes, Sec. 4).  Every byte of B is used exactly once, so B
// fragments go STRAIGHT from HBM into MFMA operand registers: the packed layout
// makes each wave load one contiguous KiB (16 B per lane).  LDS is used only to
// combine the partial sums of the 16 waves that split K.
//
// One workgroup (1024 threads) owns one 16-column fragment column of B over all
// of K; wave w takes a contiguous range of 64-deep k blocks and issues all of its
// loads before the first MFMA so that the whole weight matrix is in flight at
// once.  A (at most 64 rows) is read from L2 in MFMA operand order, shifted to
// int8 (xor 0x80) and row-summed with v_dot4 on the way, as in the large kernel.
#include "qg_internal.h"

namespace {

typedef int v4i __attribute__((ext_vector_type(4)));

constexpr int NWAVES = 16;
constexpr int NTHREADS = NWAVES * 64;

__device__ __forceinline__ v4i load_a_chunk_slow(const uint8_t* p, int kvalid) {
  union {
    v4i v;
    uint8_t b[16];
  } u;
#pragma unroll
  for (int i = 0; i < 16; ++i) u.b[i] = (i < kvalid) ? p[i] : (uint8_t)0x80;
  return u.v;
}

template <int MODE, int MB>
__global__ __launch_bounds__(NTHREADS) void qg_gemm_skinny_kernel(const qg_gemm_args p) {
  extern __shared__ __align__(16) unsigned char smem[];
  v4i* part = reinterpret_cast<v4i*>(smem);                              // [wave][mb][lane]
  int* rsp = reinterpret_cast<int*>(smem + NWAVES * MB * 64 * sizeof(v4i));  // [wave][mb][16]

  const int nb16 = blockIdx.x;
  const int sb = nb16 >> 1, sfrag = nb16 & 1;
  // columns held by this fragment: sb*32 + 16*(u&1) + 8*sfrag + 4*(u>>1) + r, u<4, r<4
  if (sb * 32 + 8 * sfrag >= p.N) return;  // nothing but padding (uniform for the workgroup)

  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int ml = lane & 15, g = lane >> 4;

  const int per = (p.kb64 + NWAVES - 1) / NWAVES;
  const int kb_begin = wave * per;
  const int kb_end = min(p.kb64, kb_begin + per);

  v4i acc[MB];
  int rs[MB];
  const uint8_t* a_row[MB];
#pragma unroll
  for (int mb = 0; mb < MB; ++mb) {
    acc[mb] = (v4i){0, 0, 0, 0};
    rs[mb] = 0;
    a_row[mb] = p.A + (size_t)min(mb * 16 + ml, p.M - 1) * p.lda + g * 16;
  }
  const int8_t* bcol = p.Bp + (size_t)nb16 * p.kb64 * QG_FRAG_BYTES + lane * 16;

  for (int kb = kb_begin; kb < kb_end; kb += 4) {
    v4i bf[4];
#pragma unroll
    for (int j = 0; j < 4; ++j)
      if (kb + j < kb_end) bf[j] = *reinterpret_cast<const v4i*>(bcol + (size_t)(kb + j) * QG_FRAG_BYTES);
    v4i af[MB][4];
#pragma unroll
    for (int mb = 0; mb < MB; ++mb)
#pragma unroll
      for (int j = 0; j < 4; ++j)
        if (kb + j < kb_end) {
          const int k = (kb + j) * QG_FRAG_K + g * 16;
          const int kvalid = p.K - k;
          if (p.a_vec && kvalid >= 16)
            af[mb][j] = *reinterpret_cast<const v4i*>(a_row[mb] + (kb + j) * QG_FRAG_K);
          else
            af[mb][j] = load_a_chunk_slow(a_row[mb] + (kb + j) * QG_FRAG_K, kvalid);
        }
#pragma unroll
    for (int j = 0; j < 4; ++j)
      if (kb + j < kb_end) {
#pragma unroll
        for (int mb = 0; mb < MB; ++mb) {
          const v4i a = af[mb][j] ^ (int)0x80808080;
          rs[mb] = __builtin_amdgcn_sdot4(a.x, 0x01010101, rs[mb], false);
          rs[mb] = __builtin_amdgcn_sdot4(a.y, 0x01010101, rs[mb], false);
          rs[mb] = __builtin_amdgcn_sdot4(a.z, 0x01010101, rs[mb], false);
          rs[mb] = __builtin_amdgcn_sdot4(a.w, 0x01010101, rs[mb], false);
          acc[mb] = __builtin_amdgcn_mfma_i32_16x16x64_i8(bf[j], a, acc[mb], 0, 0, 0);
        }
      }
  }

  // ---- combine the 16 K-slices through LDS
#pragma unroll
  for (int mb = 0; mb < MB; ++mb) {
    part[(wave * MB + mb) * 64 + lane] = acc[mb];
    int v = rs[mb];
    v += __shfl_xor(v, 16);
    v += __shfl_xor(v, 32);
    if (g == 0) rsp[(wave * MB + mb) * 16 + ml] = v;
  }
  __syncthreads();
  if (wave >= MB) return;
  const int mb = wave;
  v4i sum = (v4i){0, 0, 0, 0};
  int rsum = 0;
#pragma unroll
  for (int w = 0; w < NWAVES; ++w) {
    sum += part[(w * MB + mb) * 64 + lane];
    rsum += rsp[(w * MB + mb) * 16 + ml];
  }

  // ---- output pipeline; lane (ml, u = g) holds row mb*16+ml, 4 consecutive columns
  const int row = mb * 16 + ml;
  const int c0 = sb * 32 + 16 * (g & 1) + 8 * sfrag + 4 * (g >> 1);
  if (row >= p.M || c0 >= p.N) return;
  if (MODE == QG_MODE_REQUANT) {
    unsigned out = 0;
#pragma unroll
    for (int r = 0; r < 4; ++r) {
      const int col = c0 + r;  // col_off / bzp are padded, bias / scales are not
      const int co = p.col_off[col], bz = p.bzp[col];
      const int b = (p.bias != nullptr && col < p.N) ? p.bias[col] : 0;
      const float sc = (col < p.N) ? p.scales[(size_t)col * p.scale_stride] : 1.0f;
      const int x = sum[r] + b - p.a_zp_m128 * co - bz * rsum;
      out |= (unsigned)qg_requant_one(x, sc, p.clamp_lo, p.clamp_hi, p.c_zp) << (8 * r);
    }
    uint8_t* dst = p.C + (size_t)row * p.ldc + c0;
    if (p.c_vec && c0 + 4 <= p.N) {
      *reinterpret_cast<unsigned*>(dst) = out;
    } else {
#pragma unroll
      for (int r = 0; r < 4; ++r)
        if (c0 + r < p.N) dst[r] = (uint8_t)(out >> (8 * r));
    }
  } else {
#pragma unroll
    for (int r = 0; r < 4; ++r) {
      const int col = c0 + r;
      if (col < p.N)
        p.C32[(size_t)row * p.ldc + col] = sum[r] + 128 * (p.col_off[col] + p.K * p.bzp[col]);
    }
    if (p.rowsum_out != nullptr && nb16 == 0 && g == 0) p.rowsum_out[row] = rsum + 128 * p.K;
  }
}

template <int MODE, int MB>
hipError_t launch(const qg_gemm_args& a, hipStream_t s) {
  const int smem = NWAVES * MB * 64 * (int)sizeof(v4i) + NWAVES * MB * 16 * (int)sizeof(int);
  hipError_t e = hipFuncSetAttribute((const void*)qg_gemm_skinny_kernel<MODE, MB>,
                                     hipFuncAttributeMaxDynamicSharedMemorySize, smem);
  if (e != hipSuccess) return e;
  const int nfrag = ((a.N + 31) / 32) * 2;
  hipLaunchKernelGGL((qg_gemm_skinny_kernel<MODE, MB>), dim3(nfrag), dim3(NTHREADS), smem, s, a);
  return hipGetLastError();
}

template <int MODE>
hipError_t launch_mb(const qg_gemm_args& a, hipStream_t s) {
  if (a.M <= 16) return launch<MODE, 1>(a, s);
  if (a.M <= 32) return launch<MODE, 2>(a, s);
  return launch<MODE, 4>(a, s);
}

}  // namespace

hipError_t qg_launch_gemm_skinny(const qg_gemm_args& a, int mode, hipStream_t s) {
  return mode == QG_MODE_REQUANT ? launch_mb<QG_MODE_REQUANT>(a, s) : launch_mb<QG_MODE_ACC32>(a, s);
}
