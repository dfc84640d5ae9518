// Offline weight packing (paper Sec. 2.2: the constant matrix is packed once and
// reused) fused with the column-offset computation (Sec. 2.1: column offsets, with
// the constant K*theta_A*theta_B folded into the offsets of the constant matrix).
// Packing only moves data, so the column sums ride along for free.
#include "qg_internal.h"

namespace {

__global__ void qg_fill_i32(int32_t* p, int n, int32_t v) {
  int i = blockIdx.x * blockDim.x + threadIdx.x;
  if (i < n) p[i] = v;
}

// One thread produces one 16-byte chunk of the packed buffer: 16 consecutive k of
// one column.  Threads are ordered with the column fastest so that the 16 row
// reads are coalesced across the wave.
// TRANSPOSED: the source is B^T (N x K row-major, leading dimension ldb >= K, the layout deep-learning
// frameworks keep weights in): the 16 k values of a chunk are then 16 consecutive bytes.
template <bool TRANSPOSED>
__global__ __launch_bounds__(256) void qg_pack_b_kernel(const int8_t* __restrict__ B, int K, int N,
                                                        int ldb, int K_pad, int N_pad,
                                                        int8_t* __restrict__ packed,
                                                        int32_t* __restrict__ colsum) {
  const long long gid = (long long)blockIdx.x * blockDim.x + threadIdx.x;
  const long long total = (long long)N_pad * (K_pad / 16);
  if (gid >= total) return;
  const int n = (int)(gid % N_pad);
  const int kc16 = (int)(gid / N_pad);
  const int k0 = kc16 * 16;

  union {
    int4 v;
    int8_t b[16];
  } u;
  int sum = 0;
#pragma unroll
  for (int i = 0; i < 16; ++i) {
    int8_t x = 0;
    if (n < N && k0 + i < K) x = TRANSPOSED ? B[(size_t)n * ldb + k0 + i] : B[(size_t)(k0 + i) * ldb + n];
    u.b[i] = x;
    sum += x;
  }
  const int sb = n >> 5, c = n & 31;
  const int slot = qg_col_to_slot(c);
  const int nb16 = sb * 2 + (slot >> 4), nl = slot & 15;
  const int kb = kc16 >> 2, g = kc16 & 3;
  const size_t dst = ((size_t)kb * (N_pad / QG_FRAG_COLS) + nb16) * QG_FRAG_BYTES + (g * 16 + nl) * 16;
  *reinterpret_cast<int4*>(packed + dst) = u.v;
  if (n < N && sum != 0) atomicAdd(&colsum[n], sum);
}

// col_offsets[j] = colsum[j] - K * theta_B[j]
__global__ void qg_fold_offsets(int32_t* col_off, const int32_t* __restrict__ bzp, int n, int K) {
  int j = blockIdx.x * blockDim.x + threadIdx.x;
  if (j < n) col_off[j] = col_off[j] - K * bzp[j];
}

// ---- outlier split (Sec. 2.2): B = B' + B_sparse, B' in 4 bits, B_sparse per fragment -------------------
__device__ __forceinline__ bool is_outlier(int b) { return b < -8 || b > 7; }

// one thread per 16 consecutive columns of a row (one 16-byte load when the row allows it), grid-stride
__global__ __launch_bounds__(256) void qg_count_outliers_kernel(const int8_t* __restrict__ B, int K, int N, int ldb,
                                                                int vec, unsigned long long* __restrict__ count) {
  const int n16 = (N + 15) >> 4;
  const long long total = (long long)K * n16;
  const long long step = (long long)gridDim.x * blockDim.x;
  unsigned n = 0;
  for (long long t = (long long)blockIdx.x * blockDim.x + threadIdx.x; t < total; t += step) {
    const int k = (int)(t / n16), j0 = (int)(t - (long long)k * n16) * 16;
    const int8_t* src = B + (size_t)k * ldb + j0;
    if (vec && j0 + 16 <= N) {
      union {
        int4 v;
        int8_t b[16];
      } u;
      u.v = *reinterpret_cast<const int4*>(src);
#pragma unroll
      for (int i = 0; i < 16; ++i) n += is_outlier(u.b[i]);
    } else {
      for (int i = 0; i < 16 && j0 + i < N; ++i) n += is_outlier(src[i]);
    }
  }
  for (int o = 32; o > 0; o >>= 1) n += __shfl_xor((int)n, o);
  if ((threadIdx.x & 63) == 0 && n) atomicAdd(count, (unsigned long long)n);
}

// As qg_pack_b_kernel, writing 8 bytes of nibbles (U = B' + 8) per thread; the column sums are those of
// the WHOLE matrix B (the output pipeline corrects A B, not A B'), and the thread counts its outliers
// into the bucket of its fragment (fragment column nb16, 64-deep k block kb: bucket nb16 * kb64 + kb).
__global__ __launch_bounds__(256) void qg_pack_b_split_kernel(const int8_t* __restrict__ B, int K, int N, int ldb,
                                                              int K_pad, int N_pad, uint8_t* __restrict__ packed4,
                                                              int32_t* __restrict__ colsum,
                                                              int32_t* __restrict__ frag_cnt) {
  const long long gid = (long long)blockIdx.x * blockDim.x + threadIdx.x;
  const long long total = (long long)N_pad * (K_pad / 16);
  if (gid >= total) return;
  const int n = (int)(gid % N_pad);
  const int kc16 = (int)(gid / N_pad);
  const int k0 = kc16 * 16;
  int sum = 0, nout = 0;
  unsigned w[2] = {0, 0};
#pragma unroll
  for (int i = 0; i < 16; ++i) {
    int x = 0;
    if (n < N && k0 + i < K) x = B[(size_t)(k0 + i) * ldb + n];
    sum += x;
    const bool big = is_outlier(x);
    nout += big;
    const unsigned u = (unsigned)((big ? 0 : x) + 8);  // 0..15
    // value i of the chunk: dword i/8, byte i%4, high nibble for i%8 >= 4
    w[i >> 3] |= u << (8 * (i & 3) + 4 * ((i >> 2) & 1));
  }
  const int sb = n >> 5, c = n & 31;
  const int slot = qg_col_to_slot(c);
  const int nb16 = sb * 2 + (slot >> 4), nl = slot & 15;
  const int kb = kc16 >> 2, g = kc16 & 3;
  // one 1 KiB unit per pair of k blocks: lane (g*16 + nl) owns 16 bytes, 8 for the even and 8 for the odd block
  const size_t dst = ((size_t)(kb >> 1) * (N_pad / QG_FRAG_COLS) + nb16) * QG_FRAG_BYTES + (g * 16 + nl) * 16 + (kb & 1) * 8;
  *reinterpret_cast<uint2*>(packed4 + dst) = make_uint2(w[0], w[1]);
  if (n < N && sum != 0) atomicAdd(&colsum[n], sum);
  if (nout) atomicAdd(&frag_cnt[(size_t)nb16 * (K_pad / QG_FRAG_K) + kb], nout);
}

// exclusive prefix sum of the per-bucket counts (in place: cnt[i] -> offset of bucket i, cnt[n] = total)
// and zeroing of the fill cursors; one workgroup
__global__ __launch_bounds__(1024) void qg_scan_frag_kernel(int32_t* __restrict__ cnt, int32_t* __restrict__ cursor,
                                                            int n) {
  __shared__ int part[1024];
  const int t = threadIdx.x;
  const int per = (n + 1023) / 1024;
  const int lo = t * per, hi = min(n, lo + per);
  int s = 0;
  for (int i = lo; i < hi; ++i) s += cnt[i];
  part[t] = s;
  __syncthreads();
  for (int o = 1; o < 1024; o <<= 1) {
    const int v = t >= o ? part[t - o] : 0;
    __syncthreads();
    part[t] += v;
    __syncthreads();
  }
  int run = t ? part[t - 1] : 0;
  for (int i = lo; i < hi; ++i) {
    const int c = cnt[i];
    cnt[i] = run;
    cursor[i] = 0;
    run += c;
  }
  if (t == 1023) cnt[n] = part[1023];
}

// every outlier takes the next free entry of its bucket (order inside a bucket is arbitrary: the sparse term
// is an integer sum)
__global__ __launch_bounds__(256) void qg_fill_outliers_kernel(const int8_t* __restrict__ B, int K, int N, int ldb,
                                                               int kb64, const int32_t* __restrict__ frag_ptr,
                                                               int32_t* __restrict__ cursor,
                                                               int32_t* __restrict__ entries) {
  const long long total = (long long)K * N;
  const long long step = (long long)gridDim.x * blockDim.x;
  for (long long t = (long long)blockIdx.x * blockDim.x + threadIdx.x; t < total; t += step) {
    const int k = (int)(t / N), j = (int)(t - (long long)k * N);
    const int x = B[(size_t)k * ldb + j];
    if (!is_outlier(x)) continue;
    const int slot = qg_col_to_slot(j & 31);
    const int nb16 = (j >> 5) * 2 + (slot >> 4), nl = slot & 15;
    const int bucket = nb16 * kb64 + k / QG_FRAG_K;
    const int pos = atomicAdd(&cursor[bucket], 1);
    entries[frag_ptr[bucket] + pos] = (int32_t)((unsigned)k | ((unsigned)nl << 16) | ((unsigned)(x & 0xFF) << 24));
  }
}

// Conv weights [G][RS][4 ci][4 co] -> [G][RS][4 co][4 ci]: one dword per (tap, co)
// holding the group's 4 input channels, the operand shape of v_dot4_i32_i8.
// One thread per output channel; it also forms that channel's folded offset.
__global__ void qg_pack_conv_w_kernel(const int8_t* __restrict__ W, int G, int RS,
                                      int8_t* __restrict__ packed, int32_t* __restrict__ col_off,
                                      const int32_t* __restrict__ bzp) {
  const int oc = blockIdx.x * blockDim.x + threadIdx.x;
  if (oc >= G * 4) return;
  const int g = oc >> 2, co = oc & 3;
  int sum = 0;
  for (int tap = 0; tap < RS; ++tap)
    for (int ci = 0; ci < 4; ++ci) {
      const int8_t w = W[(((size_t)g * RS + tap) * 4 + ci) * 4 + co];
      packed[(((size_t)g * RS + tap) * 4 + co) * 4 + ci] = w;
      sum += w;
    }
  col_off[oc] = sum - RS * 4 * bzp[oc];
}

// Conv weights for the matrix-core kernel: for every 32-channel block cb and tap, one 1 KiB fragment in
// v_mfma_i32_32x32x32_i8 operand order holding the block-diagonal 32 x 32 matrix W[oc][ic] (32 / Cg groups of
// Cg x Cg, Cg = 1 << lcg in {4, 8, 16, 32}; everything off the diagonal blocks is zero).  Lane (i + 32 g) owns
// W[oc(i)][16 g .. 16 g + 15], oc(i) being the column permutation that leaves each lane of the result with 16
// consecutive channels.
__global__ void qg_pack_conv_w_mfma_kernel(const int8_t* __restrict__ W, int RS, int nfrag, int lcg,
                                           int8_t* __restrict__ frags) {
  const int gid = blockIdx.x * blockDim.x + threadIdx.x;  // one 16-byte chunk per thread
  if (gid >= nfrag * 64) return;
  const int frag = gid >> 6, lane = gid & 63;
  const int cb = frag / RS, tap = frag % RS;
  const int i = lane & 31, g = lane >> 5;
  const int oc_l = qg_slot_to_col(i);
  union {
    int4 v;
    int8_t b[16];
  } u;
#pragma unroll
  for (int b = 0; b < 16; ++b) {
    const int ic_l = 16 * g + b;
    int8_t w = 0;
    if ((ic_l >> lcg) == (oc_l >> lcg)) {
      const int cg = 1 << lcg;
      const int grp = cb * (32 >> lcg) + (oc_l >> lcg);
      w = W[(((size_t)grp * RS + tap) * cg + (ic_l & (cg - 1))) * cg + (oc_l & (cg - 1))];
    }
    u.b[b] = w;
  }
  *reinterpret_cast<int4*>(frags + (size_t)frag * QG_FRAG_BYTES + lane * 16) = u.v;
}

// Conv weights [G][RS][Cg][Og] -> [Cout][RS][Cg4] (Cg4 = Cg rounded up to 4, zero filled): the input channels of
// one (output channel, tap) are consecutive bytes, whole dwords, the operand shape of v_dot4_i32_i8.  One thread
// per byte of the result.
__global__ void qg_pack_conv_w_any_kernel(const int8_t* __restrict__ W, int G, int RS, int Cg, int Og, int Cg4,
                                          int8_t* __restrict__ packed) {
  const long long total = (long long)G * Og * RS * Cg4;
  for (long long i = (long long)blockIdx.x * blockDim.x + threadIdx.x; i < total; i += (long long)gridDim.x * blockDim.x) {
    const int ci = (int)(i % Cg4);
    const int tap = (int)((i / Cg4) % RS);
    const int oc = (int)(i / ((long long)Cg4 * RS));
    const int g = oc / Og, co = oc - g * Og;
    packed[i] = ci < Cg ? W[(((size_t)g * RS + tap) * Cg + ci) * Og + co] : (int8_t)0;
  }
}
// Folded offsets of the general layout: col_off[oc] = sum of the output channel's weights - R*S*Cg * theta_B[oc]
__global__ void qg_conv_any_offsets_kernel(const int8_t* __restrict__ packed, int Cout, int RS, int Cg, int Cg4,
                                           int32_t* __restrict__ col_off, const int32_t* __restrict__ bzp) {
  const int oc = blockIdx.x * blockDim.x + threadIdx.x;
  if (oc >= Cout) return;
  const int8_t* w = packed + (size_t)oc * RS * Cg4;
  int sum = 0;
  for (int i = 0; i < RS * Cg4; ++i) sum += w[i];
  col_off[oc] = sum - RS * Cg * bzp[oc];
}

}  // namespace

hipError_t qg_launch_pack_b(const int8_t* B, int K, int N, int ldb, int transposed, int K_pad, int N_pad,
                            int8_t* packed, int32_t* col_off, const int32_t* bzp_dev,
                            hipStream_t s) {
  hipLaunchKernelGGL(qg_fill_i32, dim3((N_pad + 255) / 256), dim3(256), 0, s, col_off, N_pad, 0);
  const long long total = (long long)N_pad * (K_pad / 16);
  const dim3 grid((unsigned)((total + 255) / 256));
  if (transposed)
    hipLaunchKernelGGL(qg_pack_b_kernel<true>, grid, dim3(256), 0, s, B, K, N, ldb, K_pad, N_pad, packed, col_off);
  else
    hipLaunchKernelGGL(qg_pack_b_kernel<false>, grid, dim3(256), 0, s, B, K, N, ldb, K_pad, N_pad, packed, col_off);
  hipLaunchKernelGGL(qg_fold_offsets, dim3((N_pad + 255) / 256), dim3(256), 0, s, col_off, bzp_dev,
                     N_pad, K);
  return hipGetLastError();
}

hipError_t qg_launch_count_outliers(const int8_t* B, int K, int N, int ldb, unsigned long long* count_dev, hipStream_t s) {
  hipLaunchKernelGGL(qg_fill_i32, dim3(1), dim3(64), 0, s, reinterpret_cast<int32_t*>(count_dev), 2, 0);
  const long long total = (long long)K * ((N + 15) / 16);
  const unsigned blocks = (unsigned)((total + 255) / 256 < 8192 ? (total + 255) / 256 : 8192);
  const int vec = reinterpret_cast<uintptr_t>(B) % 16 == 0 && ldb % 16 == 0;
  hipLaunchKernelGGL(qg_count_outliers_kernel, dim3(blocks), dim3(256), 0, s, B, K, N, ldb, vec, count_dev);
  return hipGetLastError();
}

hipError_t qg_launch_pack_b_split_count(const int8_t* B, int K, int N, int ldb, int K_pad, int N_pad, uint8_t* packed4,
                                        int32_t* col_off, const int32_t* bzp_dev, int32_t* frag_ptr, int32_t* cursor,
                                        hipStream_t s) {
  const int nbucket = (N_pad / QG_FRAG_COLS) * (K_pad / QG_FRAG_K);
  hipLaunchKernelGGL(qg_fill_i32, dim3((N_pad + 255) / 256), dim3(256), 0, s, col_off, N_pad, 0);
  hipLaunchKernelGGL(qg_fill_i32, dim3((nbucket + 1 + 255) / 256), dim3(256), 0, s, frag_ptr, nbucket + 1, 0);
  const long long total = (long long)N_pad * (K_pad / 16);
  hipLaunchKernelGGL(qg_pack_b_split_kernel, dim3((unsigned)((total + 255) / 256)), dim3(256), 0, s, B, K, N, ldb,
                     K_pad, N_pad, packed4, col_off, frag_ptr);
  hipLaunchKernelGGL(qg_fold_offsets, dim3((N_pad + 255) / 256), dim3(256), 0, s, col_off, bzp_dev, N_pad, K);
  hipLaunchKernelGGL(qg_scan_frag_kernel, dim3(1), dim3(1024), 0, s, frag_ptr, cursor, nbucket);
  return hipGetLastError();
}

hipError_t qg_launch_pack_b_split_fill(const int8_t* B, int K, int N, int ldb, int K_pad, const int32_t* frag_ptr,
                                       int32_t* cursor, int32_t* entries, hipStream_t s) {
  const long long total = (long long)K * N;
  const unsigned blocks = (unsigned)((total + 255) / 256 < 8192 ? (total + 255) / 256 : 8192);
  hipLaunchKernelGGL(qg_fill_outliers_kernel, dim3(blocks), dim3(256), 0, s, B, K, N, ldb, K_pad / QG_FRAG_K, frag_ptr, cursor,
                     entries);
  return hipGetLastError();
}

hipError_t qg_launch_pack_conv_w(const int8_t* W, int G, int RS, int8_t* packed, int32_t* col_off,
                                 const int32_t* bzp_dev, int8_t* mfma_frags, hipStream_t s) {
  hipLaunchKernelGGL(qg_pack_conv_w_kernel, dim3((G * 4 + 63) / 64), dim3(64), 0, s, W, G, RS, packed,
                     col_off, bzp_dev);
  if (mfma_frags != nullptr) {  // C = 4 G is a multiple of 32
    const int nfrag = (G / 8) * RS;
    hipLaunchKernelGGL(qg_pack_conv_w_mfma_kernel, dim3((nfrag * 64 + 255) / 256), dim3(256), 0, s, W, RS,
                       nfrag, 2, mfma_frags);
  }
  return hipGetLastError();
}

// any group shape: the general layout, its folded offsets and, when lcg >= 0 (Cg == Og == 1 << lcg, C a multiple of
// 32), the matrix-core fragments
hipError_t qg_launch_pack_conv_w_any(const int8_t* W, int G, int RS, int Cg, int Og, int8_t* packed, int32_t* col_off,
                                     const int32_t* bzp_dev, int8_t* mfma_frags, int lcg, hipStream_t s) {
  const int Cg4 = (Cg + 3) / 4 * 4, Cout = G * Og;
  const long long total = (long long)Cout * RS * Cg4;
  const unsigned blocks = (unsigned)((total + 255) / 256 < 65535 ? (total + 255) / 256 : 65535);
  hipLaunchKernelGGL(qg_pack_conv_w_any_kernel, dim3(blocks), dim3(256), 0, s, W, G, RS, Cg, Og, Cg4, packed);
  hipLaunchKernelGGL(qg_conv_any_offsets_kernel, dim3((Cout + 63) / 64), dim3(64), 0, s, packed, Cout, RS, Cg, Cg4, col_off,
                     bzp_dev);
  if (mfma_frags != nullptr) {
    const int nfrag = (G * Cg / 32) * RS;
    hipLaunchKernelGGL(qg_pack_conv_w_mfma_kernel, dim3((nfrag * 64 + 255) / 256), dim3(256), 0, s, W, RS, nfrag, lcg,
                       mfma_frags);
  }
  return hipGetLastError();
}
