// Internal declarations shared by the HIP translation units of libqgemm.
// Not part of the public interface.
#pragma once

#include <hip/hip_runtime.h>
#include <stddef.h>
#include <stdint.h>

#include "qgemm.h"

// ---------------------------------------------------------------------------
// Packed-B layout ("fragment-linear", version 1)
//
// B (K x N, int8) is zero-padded to K_pad x N_pad (multiples of 128 and 256) and
// cut into fragments of 16 columns x 64 k = 1 KiB.  A fragment is stored in the
// exact order in which one 64-lane wave feeds it to v_mfma_i32_16x16x64_i8:
// lane (nl + 16 g), nl = 0..15, g = 0..3, owns the 16 consecutive bytes
//     B[kb*64 + g*16 + 0..15][column(nl)]
// at byte offset (g*16 + nl)*16, so a wave loads a fragment with ONE fully
// coalesced 16-byte-per-lane load and no shuffling.  Two vertically adjacent
// half-fragments (g pair) of two fragments of one 32-column super-block are
// what v_mfma_i32_32x32x32_i8 wants, so the same bytes serve both MFMA shapes.
//
// Fragments are ordered [kb64][nb16]: one 64-deep slab of K for all columns is contiguous, so
// a k-tile of any width is one contiguous run and the workgroups of the small-batch kernel,
// which walk down K side by side, stream adjacent KiBs (all HBM channels busy at once).
//
// Columns are permuted inside each 32-column super-block so that the 32x32
// MFMA leaves every lane holding 16 CONSECUTIVE output columns (one 16-byte
// store).  Column c = 16h + 4q + t (h<2, q<4, t<4) sits in slot i = 8q + 4h + t;
// slot i lives in fragment 2*sb + (i >> 4) at nl = i & 15.
// ---------------------------------------------------------------------------
#define QG_FRAG_COLS 16
#define QG_FRAG_K 64
#define QG_FRAG_BYTES 1024
#define QG_KPAD 128
#define QG_NPAD 256
#define QG_LAYOUT_VERSION 1

// ---------------------------------------------------------------------------
// Outlier-split layout (paper Sec. 2.2: B = B' + B_sparse)
//
// B' (entries -8..7, zero where B holds a larger number) is stored as U = B' + 8 in 4 bits, same
// fragment order as above at half the size: a fragment is 512 B, lane (nl + 16 g) owns 8 bytes = two
// dwords; byte b of dword d holds U[k0 + 8d + b] in its low and U[k0 + 8d + 4 + b] in its high nibble
// (k0 = kb*64 + g*16), so "x & 0x0F0F0F0F" and "(x >> 4) & 0x0F0F0F0F" are two consecutive operand
// dwords.  Two fragments of consecutive k blocks (2p, 2p+1) are interleaved into one 1 KiB unit, lane by
// lane (8 bytes of block 2p, then 8 of block 2p+1), so that one 16-byte-per-lane request fetches both:
// unit (p, nb16) sits at (p * (N_pad/16) + nb16) * 1024.
// The +8 is undone with the row offsets: A_s B' = A_s U - 8 rowsum(A_s).  Padding is U = 8.
// B_sparse: one bucket per fragment (fragment column nb16, 64-deep k block kb), bucket index
// nb16 * kb64 + kb, holding entries [frag_ptr[bucket], frag_ptr[bucket+1]) of one int32 each:
// bits 0..14 row k, bits 16..19 slot of the column inside the fragment, bits 24..31 the int8 value.
// The buckets of one fragment column are consecutive, so any run of k blocks of a column is one run of
// entries.  The sparse buffer is [frag_ptr: nbucket+1][cursor: nbucket] int32, rounded up to 256 B, then
// the entries.
// ---------------------------------------------------------------------------

static inline __host__ __device__ int qg_round_up(int x, int m) { return (x + m - 1) / m * m; }

// column within a super-block -> slot (MFMA row index of the 32x32 shape)
static inline __host__ __device__ int qg_col_to_slot(int c) {
  return ((c >> 2) & 3) * 8 + (c >> 4) * 4 + (c & 3);
}
static inline __host__ __device__ int qg_slot_to_col(int i) {
  return ((i >> 2) & 1) * 16 + (i >> 3) * 4 + (i & 3);
}

enum qg_kind { QG_KIND_GEMM = 1, QG_KIND_CONV = 2 };

struct qg_packed_b {
  int kind;
  int version;
  int K, N;          // logical extents (conv: K = R*S*Cg, N = Cout)
  int K_pad, N_pad;  // padded extents of the packed buffer (gemm only)
  int has_bzp;       // any theta_B != 0
  int n_b_zp;
  const int8_t* packed;   // device
  const int32_t* col_off; // device: [0, N) col_offsets
  const int32_t* bzp;     // device: per-column theta_B (inside the col_offsets buffer)
  // conv only
  int G, R, S, Cg, Og;
  const int8_t* conv_frags;  // device: matrix-core layout of the conv weights, or null (no such layout for these extents)
  const int8_t* conv_any;    // device: [Cout][R*S][Cg rounded up to 4] layout of the general kernel, or null (4 -> 4 groups)
  const int8_t* conv_gemm;   // device: one packed (R*S*Cg) x Og GEMM matrix per group (groups of a multiple of 16 channels), or null
  const int32_t* conv_gemm_off;  // device: per group [N_pad col_offsets][N_pad theta_B]
  int conv_gemm_kpad, conv_gemm_npad;
  // outlier split only
  int split;                 // packed holds 4-bit B', the sparse part is below
  const int32_t* frag_ptr;   // device: nbucket + 1 offsets into entries
  const int32_t* entries;    // device
  long long nnz;             // number of outliers
};

// Arguments of the GEMM kernels (by value).  The first 64 bytes hold everything a wave needs before it can issue
// its first loads, so that one line of the kernel-argument segment (cold at every launch) gets it going.
struct qg_gemm_args {
  const uint8_t* A;
  const int8_t* Bp;
  int M, N, K;
  int kb64;              // K_pad / 64
  int nb16;              // N_pad / 16: fragments per 64-deep slab of the packed buffer
  int lda, ldc;
  int ksplit;            // streaming kernels: slices of K that run as separate workgroups (>= 1)
  int ks_per;            // 64-deep blocks of K per slice (ceil; even for 4-bit weights)
  int a_vec;             // A base and lda are multiples of 16 (the streaming kernels keep a variant for that case)
  int c_vec;             // output base and row pitch are multiples of 16 bytes (uint8 output of the streaming kernels: 4)
  int has_bzp;           // some theta_B != 0: the row-offset term of Eq. (2) is needed
  // ---- 64 bytes
  const int32_t* col_off;
  const int32_t* bzp;
  const int32_t* bias;   // may be null
  const float* scales;
  uint8_t* C;            // requant output
  int32_t* C32;          // acc32 output
  float* Cf;             // fp32 output (dequant mode)
  int32_t* rowsum_out;   // acc32 mode, may be null
  int scale_stride;      // 0 per tensor, 1 per channel
  int a_zp_m128;         // theta_A - 128
  int c_zp;
  float clamp_lo, clamp_hi;  // lo - theta_C, 255 - theta_C
  float relu_lo;         // dequant mode: 0 with ReLU, -inf without
  int c_wt;              // streaming kernels: write the (small) uint8 output through to memory instead of leaving it dirty in L2
  // K split across workgroups (streaming kernels): the caller's workspace (tickets, partial tiles)
  int32_t* ws_cnt;       // one ticket counter per (row block of 16, fragment column); zero between calls
  int32_t* ws_slots;     // ksplit slots of 272 int32 per counter
  float q_inv, q_lo, q_hi, q_zp;  // fp32 activations quantized while staged: 1/alpha_A, -theta_A, 255 - theta_A, theta_A
  const int32_t* sp_ptr;      // outlier split: per-bucket offsets, or null for a dense 8-bit B
  const int32_t* sp_entries;  // outlier split: entries
  int sp_total;               // outlier split: number of entries (the buffer holds at least one)
  // dense convolution through the tiled kernel (A = NHWC image, rows = output pixels, K = (kh, kw, ci)):
  int cv_H, cv_W, cv_Cin, cv_Ho, cv_Wo, cv_R, cv_S, cv_stride, cv_pad;
  int cv_pix;  // bytes per pixel of the image (>= cv_Cin: the channels may be a slice of wider pixels, a group)
  int cv_azp;                 // theta_A: what a tap outside the image reads as
  int cv_in_bytes;            // size of the image buffer
};

struct qg_conv_args {
  const uint8_t* in;
  const int8_t* Wp;
  const int8_t* Wfrag;  // matrix-core layout, or null
  const int8_t* Wany;   // general layout [Cout][R*S][Cg4], or null
  const int8_t* Bp;     // dense convolution on the byte-gathering kernel: the packed (R*S*C) x Cout matrix; nb16 = N_pad / 16
  int nb16;
  const int32_t* col_off;
  const int32_t* bzp;
  const int32_t* bias;
  const float* scales;
  uint8_t* out;
  int Nb, H, W, C, Ho, Wo, Cout, G;
  int Cg, Og, R, S;   // channels per group in / out, filter extents
  int lcg;            // log2(Cg) when the matrix-core layout is used (Cg == Og in {4, 8, 16, 32})
  int pad, stride;
  int scale_stride;
  int a_zp;       // theta_A
  int c_zp;
  float clamp_lo, clamp_hi;
  int has_bzp;
};

#ifdef __HIPCC__
// Row v holds 16 bytes of value v: where a convolution's requests go for chunks that are not in the image.  The
// hand-scheduled loop addresses a row minus 1 KiB with a 32-bit subtraction (its second request carries an
// instruction offset of 1 KiB): the rows sit 4 KiB into an 8 KiB-aligned object, so that cannot borrow.
struct alignas(8192) qg_byte_rows_t {
  uint8_t lead[4096];
  uint8_t b[256][16];
};
constexpr qg_byte_rows_t qg_make_byte_rows() {
  qg_byte_rows_t r{};
  for (int v = 0; v < 256; ++v)
    for (int i = 0; i < 16; ++i) r.b[v][i] = (uint8_t)v;
  return r;
}
static __device__ const qg_byte_rows_t qg_byte_rows = qg_make_byte_rows();  // one copy per source file that uses it

typedef int qg_v4i __attribute__((ext_vector_type(4)));
typedef qg_v4i qg_v4i_unaligned __attribute__((aligned(1)));  // a 16-byte load from any address (one instruction)

// 16 bytes of a row of A of which the first `kvalid` belong to the matrix; the rest reads as 0x80 (the int8
// zero after the uint8 -> int8 shift).  `safe`: all 16 bytes lie inside the caller's buffer, so one vector
// load and a byte mask do; otherwise byte by byte with bounds checks.  Any address.
__device__ __forceinline__ qg_v4i qg_load_a_chunk(const uint8_t* p, int kvalid, bool safe) {
  if (kvalid <= 0) return (qg_v4i){(int)0x80808080, (int)0x80808080, (int)0x80808080, (int)0x80808080};
  if (!safe) {
    union {
      qg_v4i v;
      uint8_t b[16];
    } u;
#pragma unroll
    for (int i = 0; i < 16; ++i) u.b[i] = (i < kvalid) ? p[i] : (uint8_t)0x80;
    return u.v;
  }
  qg_v4i v = *reinterpret_cast<const qg_v4i_unaligned*>(p);
#pragma unroll
  for (int j = 0; j < 4; ++j) {
    const int nb = min(max(kvalid - 4 * j, 0), 4);  // valid bytes of this dword
    const unsigned keep = nb == 4 ? 0xFFFFFFFFu : ((1u << (8 * nb)) - 1u);
    v[j] = (int)(((unsigned)v[j] & keep) | (0x80808080u & ~keep));
  }
  return v;
}

// Requantization of one corrected int32 accumulator, the fixed fp32 sequence of the output pipeline
// (paper Sec. 2.1, requantization remark): int32 -> fp32 (round to nearest even), ONE fp32 multiply,
// round to nearest even, clamp in float (so the conversion back can never be out of range), add theta_C.
__device__ __forceinline__ int qg_requant_one(int x, float sc, float lo, float hi, int czp) {
  const float f = (float)x;                          // v_cvt_f32_i32
  const float p = f * sc;                            // v_mul_f32
  const float r = __builtin_rintf(p);                // v_rndne_f32
  const float c = __builtin_amdgcn_fmed3f(r, lo, hi);  // lo <= hi, r is never NaN for finite scales
  return (int)c + czp;
}
// Same result, inserted as byte `pos` of `word`, in fewer instructions.  v_cvt_pk_u8_f32 converts with
// saturation to [0, 255] (and an integer-valued input exactly), so the clamp is done by the convert itself:
// with r the rounded product, min(max(r, lo), hi) + theta_C == sat_u8(max(r + theta_C, lo + theta_C)).
// r + theta_C is exact while |r| < 2^24 and stays far outside [0, 255], on the same side, beyond that.
// Without ReLU the lower bound lo + theta_C is 0, which the saturation covers; with ReLU it is theta_C and
// needs the explicit max unless theta_C == 0.  LO says whether that max is needed; `lo`, `hi` are the bounds of
// qg_requant_one (lo - theta_C <= 0 <= 255 - theta_C), used only when LO.
template <bool LO>
__device__ __forceinline__ unsigned qg_requant_pack(int x, float sc, float lo, float hi, float czp_f,
                                                    unsigned pos, unsigned word) {
  const float f = (float)x;
  const float p = f * sc;
  float r = __builtin_rintf(p);
  if (LO) r = __builtin_amdgcn_fmed3f(r, lo, hi);
  return __builtin_amdgcn_cvt_pk_u8_f32(r + czp_f, pos, word);
}
// whether the explicit lower clamp is needed: ReLU (lo == 0 in the shifted domain) with a nonzero theta_C
__device__ __forceinline__ bool qg_requant_needs_lo(float lo, float czp_f) { return lo == 0.0f && czp_f != 0.0f; }
// theta_C == 0 and no explicit lower clamp: the saturating convert also does the rounding (v_cvt_pk_u8_f32 rounds to
// nearest even), so sat_u8(rne(x * s)) is the convert of the product itself
__device__ __forceinline__ unsigned qg_requant_pack0(int x, float sc, unsigned pos, unsigned word) {
  const float f = (float)x;
  const float p = f * sc;
  return __builtin_amdgcn_cvt_pk_u8_f32(p, pos, word);
}
// Quantization of one fp32 activation, Eq. (1) solved for the quantized value: ONE fp32 multiply, round to nearest
// even, clamp in float to [-theta, 255 - theta], add theta; v_cvt_pk_u8_f32 converts the (exact, in-range) integer
// and inserts it as byte `pos` of `word`.
__device__ __forceinline__ unsigned qg_quantize_pack(float a, float inv, float lo, float hi, float zp_f, unsigned pos,
                                                     unsigned word) {
  const float pr = a * inv;
  const float r = __builtin_rintf(pr);
  const float c = __builtin_amdgcn_fmed3f(r, lo, hi) + zp_f;
  return __builtin_amdgcn_cvt_pk_u8_f32(c, pos, word);
}
// fp32 output of one corrected accumulator: int32 -> fp32 (nearest even), ONE fp32 multiply, optional
// max(., 0) (lo = 0 with ReLU, -inf without; a select, so no NaN-canonicalising extra instruction).
__device__ __forceinline__ float qg_dequant_one(int x, float sc, float lo) {
  const float v = (float)x * sc;
  return v < lo ? lo : v;
}
#endif

// host side of qg_requant_needs_lo (clamp_lo == 0 means ReLU: lo - theta_C with lo = theta_C)
static inline bool qg_requant_needs_lo_host(float clamp_lo, int c_zp) { return clamp_lo == 0.0f && c_zp != 0; }

#ifdef __HIPCC__
// Raises kernel Fn's dynamic-LDS limit to `bytes` on the current device unless that was already done: the
// runtime call costs about as much host time as the launch itself, which matters for microsecond kernels.
// (Concurrent callers may both make the call; it is idempotent.)
template <auto Fn>
inline hipError_t qg_allow_smem(int bytes) {
  static int allowed[64] = {0};  // per kernel, indexed by device
  int dev = 0;
  hipError_t e = hipGetDevice(&dev);
  if (e != hipSuccess) return e;
  if (dev >= 0 && dev < 64 && allowed[dev] >= bytes) return hipSuccess;
  e = hipFuncSetAttribute((const void*)Fn, hipFuncAttributeMaxDynamicSharedMemorySize, bytes);
  if (e == hipSuccess && dev >= 0 && dev < 64) allowed[dev] = bytes;
  if (e != hipSuccess) (void)hipGetLastError();  // reported through the return value; not left for the next call to find
  return e;
}
#endif

// launchers (each returns a hipError_t from hipGetLastError after the launch)
hipError_t qg_launch_pack_b(const int8_t* B, int K, int N, int ldb, int transposed, int K_pad, int N_pad,
                            int8_t* packed, int32_t* col_off, const int32_t* bzp_dev, hipStream_t s);
hipError_t qg_launch_count_outliers(const int8_t* B, int K, int N, int ldb, unsigned long long* count_dev, hipStream_t s);
hipError_t qg_launch_pack_b_split_count(const int8_t* B, int K, int N, int ldb, int K_pad, int N_pad, uint8_t* packed4,
                                        int32_t* col_off, const int32_t* bzp_dev, int32_t* frag_ptr, int32_t* cursor,
                                        hipStream_t s);
hipError_t qg_launch_pack_b_split_fill(const int8_t* B, int K, int N, int ldb, int K_pad, const int32_t* frag_ptr,
                                       int32_t* cursor, int32_t* entries, hipStream_t s);
hipError_t qg_launch_pack_conv_w(const int8_t* W, int G, int RS, int8_t* packed, int32_t* col_off,
                                 const int32_t* bzp_dev, int8_t* mfma_frags, hipStream_t s);
hipError_t qg_launch_pack_conv_w_any(const int8_t* W, int G, int RS, int Cg, int Og, int8_t* packed, int32_t* col_off,
                                     const int32_t* bzp_dev, int8_t* mfma_frags, int lcg, hipStream_t s);
// `kernel` is one of the QG_KERNEL_* ids of qgemm.h (never QG_KERNEL_AUTO: selection happens in api.hip)
hipError_t qg_launch_gemm_tile(const qg_gemm_args& a, int mode, int kernel, hipStream_t s);
// kernel: QG_KERNEL_TILE64 / TILE64K4 / TILE64K1 / TILE128 / TILE128X256
hipError_t qg_launch_conv_dense(const qg_gemm_args& a, int kernel, hipStream_t s);
hipError_t qg_launch_gemm_skinny(const qg_gemm_args& a, int mode, int kernel, hipStream_t s);
hipError_t qg_launch_gemm_skinny_f32(const qg_gemm_args& a, int mode, int kernel, hipStream_t s);
hipError_t qg_launch_conv_skinny(const qg_gemm_args& a, int kernel, hipStream_t s);
hipError_t qg_launch_quantize_a(const float* A, int M, int K, int lda, float inv_scale, int a_zp, uint8_t* Aq,
                                int ldq, hipStream_t s);
hipError_t qg_launch_conv_group(const qg_conv_args& a, int RS, hipStream_t s);
hipError_t qg_launch_conv_dense_plain(const qg_conv_args& a, hipStream_t s);
// the kernels with the input patch in LDS ("same" convolutions); form 0 = 64 pixels x 128 channels, 1 = 128 x 64, 2 = 256 x 64, 3 = 256 x 128, 4 = 512 x 128
bool qg_conv_patch_applies(const qg_gemm_args& a, int form);
int qg_conv_patch_per_cu(const qg_gemm_args& a, int form);  // workgroups a CU holds side by side; 0 = does not apply
hipError_t qg_launch_conv_patch(const qg_gemm_args& a, int form, hipStream_t s);

#define QG_MODE_REQUANT 0
#define QG_MODE_ACC32 1
#define QG_MODE_DEQUANT 2
