// Large-tile quantized GEMM for compute-bound shapes.
//
// One launch does everything the paper fuses around the GEMM (Sec. 2.1-2.2):
//   - A is read once; while a tile is staged on its way to LDS it is shifted from
//     uint8 to int8 (xor 0x80 == subtract 128, the int8 MFMA is signed x signed)
//     and its row offsets are accumulated with v_dot4 ("row offsets are computed
//     for the block being packed", Appendix B);
//   - int32 accumulation on v_mfma_i32_32x32x32_i8, LDS double-buffered;
//   - the output pipeline (zero-point corrections of Eq. (2), bias, fp32 scale,
//     round-to-nearest-even, clamp/ReLU) runs on the accumulators in registers and
//     stores uint8 directly: there is no int32 C in memory.
//
// Shift algebra: with A_s = A_u - 128, rowsum_s = rowsum_u - 128 K and
// acc_s = acc_u - 128 colsum, the corrected accumulator of Eq. (2) is
//   x = acc_s - (theta_A - 128) * (colsum - K theta_B) - theta_B * rowsum_s + bias,
// i.e. "replace theta_A by theta_A - 128" with the folded column offsets.
//
// Workgroup: 512 threads = 8 waves as 4 (M) x 2 (N); tile 256 x 256 x 128;
// each wave owns 64 x 128 = 2 x 4 MFMA blocks of 32 x 32 (128 accumulator VGPRs).
// The MFMA is issued transposed (first operand = B fragment, second = A fragment)
// so that a lane ends up with 16 consecutive columns of one row.
#include "qg_internal.h"

namespace {

typedef int v4i __attribute__((ext_vector_type(4)));
typedef int v16i __attribute__((ext_vector_type(16)));

constexpr int BM = 256, BN = 256, BK = 128;
constexpr int NTHREADS = 512;
constexpr int A_STAGE_BYTES = BM * BK;                 // 32 KiB
constexpr int B_STAGE_BYTES = BN * BK;                 // 32 KiB
constexpr int STAGE_BYTES = A_STAGE_BYTES + B_STAGE_BYTES;
constexpr int ROWSUM_OFF = 2 * STAGE_BYTES;            // 256 int32 after the two stages
constexpr int SMEM_BYTES = ROWSUM_OFF + BM * 4;
// epilogue constants live in stage 0 once the main loop is over
constexpr int EP_CJ_OFF = 0, EP_BZ_OFF = 1024, EP_SC_OFF = 2048;

// swizzled byte offset of 16-byte chunk kc (0..7) of row r in an A stage
__device__ __forceinline__ int a_lds_off(int r, int kc) { return r * BK + ((kc ^ ((r >> 1) & 7)) << 4); }

__device__ __forceinline__ v4i load_a_chunk_slow(const uint8_t* p, int kvalid) {
  // byte-wise, bounds-checked; bytes past K read as 0x80 (int8 zero after the shift)
  union {
    v4i v;
    uint8_t b[16];
  } u;
#pragma unroll
  for (int i = 0; i < 16; ++i) u.b[i] = (i < kvalid) ? p[i] : (uint8_t)0x80;
  return u.v;
}

__device__ __forceinline__ int requant_one(int x, float sc, float lo, float hi, int czp) {
  float f = (float)x;                 // v_cvt_f32_i32, round to nearest even
  float p = f * sc;                   // one fp32 multiply
  float r = __builtin_rintf(p);       // v_rndne_f32
  r = __builtin_fminf(__builtin_fmaxf(r, lo), hi);
  return (int)r + czp;
}

template <int MODE>
__global__ __launch_bounds__(NTHREADS) void qg_gemm_tile_kernel(const qg_gemm_args p, int tiles_m,
                                                               int tiles_n) {
  extern __shared__ __align__(16) unsigned char smem[];
  const int tid = threadIdx.x;
  const int lane = tid & 63;
  const int wave = tid >> 6;
  const int wave_m = wave & 3, wave_n = wave >> 2;

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

  // ---- staging assignment: thread -> (row, 16-byte chunk) of the A tile, 4 passes
  const int a_row = tid >> 3;  // + 64 * pass
  const int a_kc = tid & 7;
  const uint8_t* a_src[4];
  int a_dst[4];
#pragma unroll
  for (int q = 0; q < 4; ++q) {
    const int r = a_row + 64 * q;
    const int rg = min(m0 + r, p.M - 1);  // rows past M re-read the last row; never stored
    a_src[q] = p.A + (size_t)rg * p.lda + a_kc * 16;
    a_dst[q] = a_lds_off(r, a_kc);
  }
  // B tile: 16 fragments-pairs of 2 KiB, a straight copy
  const int8_t* b_src[4];
  int b_dst[4];
#pragma unroll
  for (int q = 0; q < 4; ++q) {
    const int c = q * NTHREADS + tid;  // 16-byte chunk 0..2047
    const int nbl = c >> 7, within = c & 127;
    b_src[q] = p.Bp + ((size_t)(n0 / QG_FRAG_COLS + nbl) * p.kb64) * QG_FRAG_BYTES + within * 16;
    b_dst[q] = A_STAGE_BYTES + c * 16;
  }

  v4i a_reg[4], b_reg[4];
  int rs[4] = {0, 0, 0, 0};

  auto load_global = [&](int kt) {
    const int k0 = kt * BK;
    if (p.a_vec && k0 + BK <= p.K) {
#pragma unroll
      for (int q = 0; q < 4; ++q) a_reg[q] = *reinterpret_cast<const v4i*>(a_src[q] + k0);
    } else {
      const int kvalid = p.K - (k0 + a_kc * 16);
#pragma unroll
      for (int q = 0; q < 4; ++q) a_reg[q] = load_a_chunk_slow(a_src[q] + k0, kvalid);
    }
#pragma unroll
    for (int q = 0; q < 4; ++q)
      b_reg[q] = *reinterpret_cast<const v4i*>(b_src[q] + (size_t)kt * (2 * QG_FRAG_BYTES));
  };

  auto store_lds = [&](int stage) {
    unsigned char* base = smem + stage * STAGE_BYTES;
#pragma unroll
    for (int q = 0; q < 4; ++q) {
      v4i v = a_reg[q] ^ (int)0x80808080;  // uint8 -> int8 (minus 128)
      rs[q] = __builtin_amdgcn_sdot4(v.x, 0x01010101, rs[q], false);
      rs[q] = __builtin_amdgcn_sdot4(v.y, 0x01010101, rs[q], false);
      rs[q] = __builtin_amdgcn_sdot4(v.z, 0x01010101, rs[q], false);
      rs[q] = __builtin_amdgcn_sdot4(v.w, 0x01010101, rs[q], false);
      *reinterpret_cast<v4i*>(base + a_dst[q]) = v;
    }
#pragma unroll
    for (int q = 0; q < 4; ++q) *reinterpret_cast<v4i*>(base + b_dst[q]) = b_reg[q];
  };

  v16i acc[2][4];
#pragma unroll
  for (int i = 0; i < 2; ++i)
#pragma unroll
    for (int j = 0; j < 4; ++j)
#pragma unroll
      for (int r = 0; r < 16; ++r) acc[i][j][r] = 0;

  // fragment read offsets (constant over the k loop)
  const int l32 = lane & 31, lg = lane >> 5;
  int a_frag_row[2];
#pragma unroll
  for (int mb = 0; mb < 2; ++mb) a_frag_row[mb] = wave_m * 64 + mb * 32 + l32;
  // B fragment: slot i = l32 -> fragment (i >> 4) of the super-block, nl = i & 15
  int b_frag_base[4];
#pragma unroll
  for (int nb = 0; nb < 4; ++nb) {
    const int nbl = (wave_n * 4 + nb) * 2 + (l32 >> 4);
    b_frag_base[nb] = A_STAGE_BYTES + nbl * (2 * QG_FRAG_BYTES) + (l32 & 15) * 16;
  }

  const int KT = p.kb64 >> 1;
  load_global(0);
  store_lds(0);
  __syncthreads();

  for (int kt = 0; kt < KT; ++kt) {
    const bool more = kt + 1 < KT;
    if (more) load_global(kt + 1);
    const unsigned char* base = smem + (kt & 1) * STAGE_BYTES;
#pragma unroll
    for (int ks = 0; ks < 4; ++ks) {
      v4i af[2], bf[4];
#pragma unroll
      for (int mb = 0; mb < 2; ++mb)
        af[mb] = *reinterpret_cast<const v4i*>(base + a_lds_off(a_frag_row[mb], ks * 2 + lg));
#pragma unroll
      for (int nb = 0; nb < 4; ++nb)
        bf[nb] = *reinterpret_cast<const v4i*>(base + b_frag_base[nb] + (ks >> 1) * QG_FRAG_BYTES +
                                               (((ks & 1) * 2 + lg) * 16) * 16);
#pragma unroll
      for (int mb = 0; mb < 2; ++mb)
#pragma unroll
        for (int nb = 0; nb < 4; ++nb)
          acc[mb][nb] = __builtin_amdgcn_mfma_i32_32x32x32_i8(bf[nb], af[mb], acc[mb][nb], 0, 0, 0);
    }
    if (more) store_lds((kt + 1) & 1);
    __syncthreads();
  }

  // ---- row offsets: the 8 threads that staged one row hold its partial sums
  int* rowsum_s = reinterpret_cast<int*>(smem + ROWSUM_OFF);
#pragma unroll
  for (int q = 0; q < 4; ++q) {
    int v = rs[q];
    v += __shfl_xor(v, 1);
    v += __shfl_xor(v, 2);
    v += __shfl_xor(v, 4);
    if (a_kc == 0) rowsum_s[a_row + 64 * q] = v;
  }
  // ---- per-column constants of the output pipeline, staged once per workgroup
  int* cj_s = reinterpret_cast<int*>(smem + EP_CJ_OFF);
  int* bz_s = reinterpret_cast<int*>(smem + EP_BZ_OFF);
  float* sc_s = reinterpret_cast<float*>(smem + EP_SC_OFF);
  if (tid < BN) {
    const int col = n0 + tid;  // col_off / bzp are padded to N_pad, bias / scales are not
    const int co = p.col_off[col], bz = p.bzp[col];
    if (MODE == QG_MODE_REQUANT) {
      const int b = (p.bias != nullptr && col < p.N) ? p.bias[col] : 0;
      cj_s[tid] = b - p.a_zp_m128 * co;
      sc_s[tid] = (col < p.N) ? p.scales[(size_t)col * p.scale_stride] : 1.0f;
    } else {
      cj_s[tid] = 128 * (co + p.K * bz);  // acc_u = acc_s + 128 * colsum
    }
    bz_s[tid] = bz;
  }
  __syncthreads();

  // ---- epilogue straight from the accumulators
#pragma unroll
  for (int mb = 0; mb < 2; ++mb) {
    const int row_l = wave_m * 64 + mb * 32 + l32;
    const int row = m0 + row_l;
    const int rsum = rowsum_s[row_l];
    if (MODE == QG_MODE_ACC32 && p.rowsum_out != nullptr && tn == 0 && wave_n == 0 && lg == 0 &&
        row < p.M)
      p.rowsum_out[row] = rsum + 128 * p.K;
#pragma unroll
    for (int nb = 0; nb < 4; ++nb) {
      const int col_l = wave_n * 128 + nb * 32 + lg * 16;
      const int col = n0 + col_l;
      if (row >= p.M || col >= p.N) continue;
      if (MODE == QG_MODE_REQUANT) {
        unsigned out[4];
#pragma unroll
        for (int q = 0; q < 4; ++q) {
          const v4i cj = *reinterpret_cast<const v4i*>(&cj_s[col_l + 4 * q]);
          const v4i bz = *reinterpret_cast<const v4i*>(&bz_s[col_l + 4 * q]);
          const float4 sc = *reinterpret_cast<const float4*>(&sc_s[col_l + 4 * q]);
          const int x0 = acc[mb][nb][4 * q + 0] + cj.x - bz.x * rsum;
          const int x1 = acc[mb][nb][4 * q + 1] + cj.y - bz.y * rsum;
          const int x2 = acc[mb][nb][4 * q + 2] + cj.z - bz.z * rsum;
          const int x3 = acc[mb][nb][4 * q + 3] + cj.w - bz.w * rsum;
          const unsigned q0 = (unsigned)requant_one(x0, sc.x, p.clamp_lo, p.clamp_hi, p.c_zp);
          const unsigned q1 = (unsigned)requant_one(x1, sc.y, p.clamp_lo, p.clamp_hi, p.c_zp);
          const unsigned q2 = (unsigned)requant_one(x2, sc.z, p.clamp_lo, p.clamp_hi, p.c_zp);
          const unsigned q3 = (unsigned)requant_one(x3, sc.w, p.clamp_lo, p.clamp_hi, p.c_zp);
          out[q] = q0 | (q1 << 8) | (q2 << 16) | (q3 << 24);
        }
        uint8_t* dst = p.C + (size_t)row * p.ldc + col;
        if (p.c_vec && col + 16 <= p.N) {
          *reinterpret_cast<uint4*>(dst) = make_uint4(out[0], out[1], out[2], out[3]);
        } else {
#pragma unroll
          for (int i = 0; i < 16; ++i)
            if (col + i < p.N) dst[i] = (uint8_t)(out[i >> 2] >> ((i & 3) * 8));
        }
      } else {
        int32_t* dst = p.C32 + (size_t)row * p.ldc + col;
#pragma unroll
        for (int i = 0; i < 16; ++i)
          if (col + i < p.N) dst[i] = acc[mb][nb][i] + cj_s[col_l + i];
      }
    }
  }
}

}  // namespace

hipError_t qg_launch_gemm_tile(const qg_gemm_args& a, int mode, hipStream_t s) {
  const int tiles_m = (a.M + BM - 1) / BM;
  const int tiles_n = (a.N + BN - 1) / BN;
  const void* fn = mode == QG_MODE_REQUANT ? (const void*)qg_gemm_tile_kernel<QG_MODE_REQUANT>
                                           : (const void*)qg_gemm_tile_kernel<QG_MODE_ACC32>;
  hipError_t e = hipFuncSetAttribute(fn, hipFuncAttributeMaxDynamicSharedMemorySize, SMEM_BYTES);
  if (e != hipSuccess) return e;
  const dim3 grid((unsigned)(tiles_m * tiles_n)), block(NTHREADS);
  if (mode == QG_MODE_REQUANT)
    hipLaunchKernelGGL(qg_gemm_tile_kernel<QG_MODE_REQUANT>, grid, block, SMEM_BYTES, s, a, tiles_m,
                       tiles_n);
  else
    hipLaunchKernelGGL(qg_gemm_tile_kernel<QG_MODE_ACC32>, grid, block, SMEM_BYTES, s, a, tiles_m,
                       tiles_n);
  return hipGetLastError();
}
