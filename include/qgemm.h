/*
 * qgemm -- quantized matrix multiply  C_u8 = requant(A_u8 * B_s8)  for AMD MI355X
 * (gfx950), with the pre- and post-processing of the FBGEMM paper
 * (arXiv 2101.05615) fused in.  C ABI, plain pointers and sizes.
 *
 * Conventions taken from the paper's statement of the problem (Sec. 2.1,
 * Eq. (1)-(2), and the interface of Appendix A):
 *   - C = A B with A: M x K (uint8 activations), B: K x N (int8 weights),
 *     C: M x N (uint8), all row-major with leading dimensions in elements.
 *   - every matrix is affinely quantized, X = alpha_X (X^q - theta_X)   (Eq. 1);
 *     theta_A and theta_C are per tensor, theta_B and the combined multiplier
 *     alpha_A alpha_B / alpha_C are per tensor or per output channel (column of B).
 *   - B is the constant matrix: it is packed ONCE, ahead of time, never at run
 *     time (Sec. 2.2; Appendix A "packB.pack is never called").
 *   - the library creates no streams, allocates no device memory and never
 *     synchronises: device buffers, including scratch, are caller-allocated
 *     (Appendix A: preallocated C_buffer, no threads created internally).
 *
 * "dev" pointers are device (HBM) addresses valid on the current HIP device;
 * "host" pointers are ordinary host memory.  `stream` is a hipStream_t passed
 * as void* (NULL = the default stream).  Every run-time call is asynchronous:
 * a 0 return means "enqueued on `stream`".  The run-time calls (the GEMMs, the
 * convolutions, qg_quantize_a_f32) enqueue kernels and nothing else -- no copy,
 * no memset, no allocation -- so they may be recorded into a HIP graph and
 * replayed; call each once outside the capture first (the first launch of a
 * kernel raises its LDS limit with a runtime call).  The offline packing and
 * counting calls wait once for `stream` (they stage host values through it) and
 * cannot be recorded.
 *
 * Errors: every function returns 0 on success or one of the negative QG_E*
 * codes; nothing is printed, nothing aborts.  On error no output is written.
 * An empty batch (M == 0, or Nb == 0 for a convolution) is a valid request:
 * its data pointers (A, C, image, workspace) are not referenced and may be NULL,
 * the other arguments are checked as usual, nothing is enqueued and the return
 * is QG_OK; negative counts are QG_EINVAL.
 */
#ifndef QGEMM_H
#define QGEMM_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

#define QG_OK 0
#define QG_ENULL (-1)      /* a required pointer is NULL                               */
#define QG_EINVAL (-2)     /* a size, leading dimension, zero point or count is invalid */
#define QG_EALIGN (-3)     /* a device pointer violates a documented alignment          */
#define QG_EWORKSPACE (-4) /* workspace needed but NULL                                 */
#define QG_ELAUNCH (-5)    /* the HIP runtime refused a launch or copy                  */
#define QG_ENOMEM (-6)     /* host allocation of the descriptor failed                  */
#define QG_EUNSUPPORTED (-7) /* valid request outside what this build implements        */
#define QG_ECAPACITY (-8)  /* more outliers than the caller's sparse buffer can hold       */

/* Largest K accepted: with |A| <= 255 and |B - theta_B| <= 255 the int32
 * accumulator and the zero-point terms of Eq. (2) together stay within
 * 255 * 255 * K <= 2 130 739 200 < 2^31 (Eq. (2) never discusses overflow).
 * The int32 bias is added on top in 32-bit arithmetic, so the caller must keep
 *     |bias[j]| <= 2^31 - 1 - 255 * 255 * K
 * (16 744 447 at K = 32768, about 2^31 for short K); beyond that the corrected
 * accumulator may wrap and the result is unspecified. */
#define QG_MAX_K 32768

/* Opaque HOST-side descriptor of a packed weight matrix.  It owns no device
 * memory: it records K, N, the padded extents, the layout version and the
 * caller's two device buffers, which must outlive it and all enqueued work. */
typedef struct qg_packed_b qg_packed_b;

/* Run-time parameters of the output pipeline (Sec. 2.1 requantization remark;
 * Sec. 2.2 "bias addition, nonlinearities, requantization"):
 *   x      = acc - theta_A*colsum_B[j] - theta_B[j]*rowsum_A[i] + K*theta_A*theta_B[j] + bias[j]
 *   C[i,j] = clamp(rne((float)x * scale[j]), lo - theta_C, 255 - theta_C) + theta_C
 * with lo = theta_C when relu != 0, else 0; rne = round to nearest even; the
 * product is ONE IEEE fp32 multiply.  scales must be finite and > 0. */
typedef struct {
  int32_t a_zp;          /* theta_A, 0..255                                   */
  const int32_t* bias;   /* dev, N entries in accumulator units, or NULL;
                            |bias[j]| <= 2^31 - 1 - 255*255*K (see QG_MAX_K)  */
  const float* scales;   /* dev, n_scales entries                             */
  int32_t n_scales;      /* 1 (per tensor) or N (per output channel)          */
  int32_t c_zp;          /* theta_C, 0..255                                   */
  int32_t relu;          /* 0 or 1                                            */
} qg_requant_params;

/* ---- offline: weight packing with column-offset precompute --------------- */

/* Bytes the caller must allocate for qg_pack_b: `packed_bytes` for the
 * reordered, zero-padded int8 weights and `col_offsets_bytes` for the int32
 * side buffer.  Both buffers must be 256-byte aligned. */
int qg_pack_b_sizes(int K, int N, size_t* packed_bytes, size_t* col_offsets_bytes);

/* Pack B (Sec. 2.2: prepack the constant matrix once) and compute the column
 * offsets with the constant term of Eq. (2) folded in (Sec. 2.1, second remark):
 *     col_offsets[j] = sum_k B[k][j] - K * theta_B[j],   j = 0..N-1
 * which occupy the first N int32 of col_offsets_dev; the rest of that buffer
 * is private to the library (a per-channel copy of theta_B).
 *   B_dev      dev, int8, row-major K x N, leading dimension ldb >= N
 *   b_zp_host  HOST, n_b_zp entries (1 = per tensor, N = per channel), each -128..127
 *   packed_dev, col_offsets_dev  dev, caller-allocated, sizes from qg_pack_b_sizes
 *   out        receives the descriptor; release with qg_packed_b_destroy
 * 1 <= K <= QG_MAX_K, N >= 1. */
int qg_pack_b(const int8_t* B_dev, int K, int N, int ldb, const int32_t* b_zp_host, int n_b_zp,
              void* packed_dev, int32_t* col_offsets_dev, void* stream, qg_packed_b** out);

/* As qg_pack_b from the TRANSPOSED weight matrix, the layout deep-learning
 * frameworks store (the paper's row-wise quantization speaks of the rows of
 * that matrix = output channels = columns of B):
 *   Bt_dev  dev, int8, row-major N x K, leading dimension ldbt >= K; Bt[n][k] = B[k][n]
 * The descriptor is indistinguishable from qg_pack_b's. */
int qg_pack_b_transposed(const int8_t* Bt_dev, int K, int N, int ldbt, const int32_t* b_zp_host,
                         int n_b_zp, void* packed_dev, int32_t* col_offsets_dev, void* stream,
                         qg_packed_b** out);

/* Frees the host descriptor only.  NULL is allowed. */
void qg_packed_b_destroy(qg_packed_b* p);

/* K, N of a descriptor (0 on NULL). */
int qg_packed_b_k(const qg_packed_b* p);
int qg_packed_b_n(const qg_packed_b* p);

/* ---- run time ------------------------------------------------------------ */

/* Scratch for the GEMM calls: the role of the paper's caller-preallocated C_buffer
 * (Appendix A).  A shape with few columns and a long K is split over K ACROSS
 * workgroups so that the whole chip streams the weights; the int32 partial
 * tiles meet in this workspace and the slice that arrives last runs the output
 * pipeline.  Integer sums: every split gives the same bytes as no split.
 *
 * qg_gemm_workspace_bytes: bytes qg_gemm_u8s8_requant / _acc32 / _dequant_f32
 * (and their _kernel forms with QG_KERNEL_AUTO) want for this M; 0 when the
 * built-in choice does not split, in which case workspace_dev may be NULL.
 * Passing NULL is always allowed: the call then never splits.
 *
 * Protocol: allocate (16-byte aligned), call qg_gemm_workspace_init ONCE (it
 * enqueues a kernel that zero-fills it; no copy, no memset, so it may be
 * recorded into a graph), then pass it to any number of calls that run one
 * after another on one stream: every call leaves the workspace as it found it.
 * Calls that may overlap in time (different streams) need different
 * workspaces.  A workspace of qg_gemm_workspace_bytes(M, Bp) also serves any
 * smaller M with the same Bp. */
size_t qg_gemm_workspace_bytes(int M, const qg_packed_b* Bp);
int qg_gemm_workspace_init(void* workspace_dev, size_t bytes, void* stream);

/* The fused hot path (Sec. 2.1 Eq. (2) + requantization; Sec. 2.2 fusion of
 * row-offset computation into the A staging pass and of the output pipeline
 * into the GEMM): one launch reads A once, computes row offsets from the
 * staged tile, accumulates in int32 and writes uint8 C from the accumulators.
 *   A_dev  dev, uint8, row-major M x K (K from Bp), lda >= K
 *   C_dev  dev, uint8, row-major M x N, ldc >= N; must not alias A
 * No alignment is required and K need not be a multiple of anything: A is staged
 * with 16-byte requests from any address, a last partial 64-deep slice of K with a
 * byte mask; C is written with 16-byte stores to any address, byte by byte only
 * where N cuts a lane's 16 columns.  A may exceed 4 GiB: the kernels
 * address it with 32-bit offsets from a base, so the call then enqueues several
 * launches over consecutive row ranges.  Identical inputs give identical bytes
 * on every run. */
int qg_gemm_u8s8_requant(const uint8_t* A_dev, int M, int lda, const qg_packed_b* Bp,
                         const qg_requant_params* p, uint8_t* C_dev, int ldc, void* workspace_dev,
                         void* stream);

/* Test hook for the first term of Eq. (2): C32[i][j] = sum_k A_u8[i][k]*B_s8[k][j]
 * (the accumulator in the uint8 domain, exactly), through the same main loop as
 * the fused call.  rowsum_dev (optional, M int32) receives sum_k A_u8[i][k]. */
int qg_gemm_u8s8_acc32(const uint8_t* A_dev, int M, int lda, const qg_packed_b* Bp, int32_t* C32_dev,
                       int ldc, int32_t* rowsum_dev, void* workspace_dev, void* stream);

/* ---- shape-specific kernels (Appendix C) ----------------------------------- */

/* The paper's observation: inference GEMMs are tall, skinny or small, so a few
 * kernels specialised by shape beat one kernel tuned for large squares; the
 * library asks "is there a kernel for this M" and maps every other size to the
 * nearest one.  Here the family is a table of pre-instantiated configurations;
 * every one of them computes every shape (bit-identical results), they differ
 * only in speed:
 *   SKINNY16/32/64  one workgroup per 16 columns of B and per block of 16/32/64
 *                   rows, K split over the waves of the workgroup; B streams from
 *                   HBM straight into operand registers (bandwidth-bound shapes)
 *   TILE64          64 x 64 workgroup tile, three LDS stages, K split over two wave sets
 *   TILE128         128 x 128, four LDS stages, hand-scheduled loop (K >= 256; else like TILE128X256)
 *   TILE128X256     128 x 256, three LDS stages, hand-scheduled loop, two workgroups per CU (K >= 192)
 *   TILE256         256 x 256, four LDS stages, hand-scheduled loop (large shapes)
 *   TILE64K4        64 x 64 with K split over four wave sets (1024 threads; a few
 *                   tiles and a long K)
 *   TILE64K1        64 x 64 without a K split (256 threads, 24 KB of LDS: six small
 *                   workgroups per CU; many tiles and a short K)
 *   TILE64X32K8     64 x 32 with K split over eight sets of two waves (1024 threads;
 *                   at most one workgroup per CU and a long K: M up to 128 with N = K = 4096)
 * QG_KERNEL_AUTO picks by (M, N, K): first the rules installed with
 * qg_dispatch_set_rules (an offline autotune writes them), then a built-in
 * rule of thumb derived from the same measurements. */
#define QG_KERNEL_AUTO 0
#define QG_KERNEL_SKINNY16 1
#define QG_KERNEL_SKINNY32 2
#define QG_KERNEL_SKINNY64 3
#define QG_KERNEL_TILE64 4
#define QG_KERNEL_TILE128 5
#define QG_KERNEL_TILE128X256 6
#define QG_KERNEL_TILE256 7
#define QG_KERNEL_TILE64K4 8
#define QG_KERNEL_TILE64K1 9
#define QG_KERNEL_TILE64X32K8 10
#define QG_KERNEL_LAST 10
/* Dense convolution only (qg_conv_dense_u8s8_requant): the kernels that keep the input patch of a pixel tile in LDS;
 * workgroup = 64 pixels x 128 channels, 128 x 64, 256 x 64 (eight waves), 256 x 128 (eight waves), 512 x 128 (eight
 * waves of 128 x 64: the form for many pixels and at least 96 output channels). */
#define QG_KERNEL_PATCH64X128 11
#define QG_KERNEL_PATCH128X64 12
#define QG_KERNEL_PATCH256X64 13
#define QG_KERNEL_PATCH256 14
#define QG_KERNEL_PATCH512 15
#define QG_KERNEL_CONV_LAST 15

/* Name of a kernel id ("skinny16", "tile128x256", "patch128x64", ...; "auto" for 0), NULL if invalid. */
const char* qg_kernel_name(int kernel);

/* The id QG_KERNEL_AUTO resolves to for this shape (never QG_KERNEL_AUTO);
 * QG_EINVAL (negative) if a size is not positive. */
int qg_kernel_select(int M, int N, int K);

/* One line of the dispatch table: shapes with m_lo <= M <= m_hi, n_lo <= N <= n_hi
 * and k_lo <= K <= k_hi run `kernel` (QG_KERNEL_SKINNY16..QG_KERNEL_LAST). */
typedef struct {
  int32_t m_lo, m_hi, n_lo, n_hi, k_lo, k_hi;
  int32_t kernel;
} qg_dispatch_rule;
#define QG_MAX_DISPATCH_RULES 256

/* Replace the table by n rules (HOST array, copied); the first matching rule
 * wins, shapes no rule matches use the built-in choice; n == 0 empties the
 * table.  Process-wide; must not run concurrently with other qg_ calls.
 * QG_EINVAL if n is out of range or a rule is malformed (then nothing changes). */
int qg_dispatch_set_rules(const qg_dispatch_rule* rules_host, int n);

/* qg_gemm_u8s8_requant / qg_gemm_u8s8_acc32 with the kernel chosen by the caller
 * (the autotuner and the tests use these); QG_KERNEL_AUTO behaves like the plain
 * calls.  QG_EINVAL for an unknown id or when M needs more than 65535 row blocks
 * of a SKINNY kernel. */
int qg_gemm_u8s8_requant_kernel(const uint8_t* A_dev, int M, int lda, const qg_packed_b* Bp,
                                const qg_requant_params* p, uint8_t* C_dev, int ldc,
                                void* workspace_dev, void* stream, int kernel);
int qg_gemm_u8s8_acc32_kernel(const uint8_t* A_dev, int M, int lda, const qg_packed_b* Bp,
                              int32_t* C32_dev, int ldc, int32_t* rowsum_dev, void* workspace_dev,
                              void* stream, int kernel);

/* The K split chosen by the caller (the tests compare every factor with the
 * oracle; the autotuner times them).  Appendix A: the caller's C_buffer.
 *   kernel  QG_KERNEL_AUTO or QG_KERNEL_SKINNY16/32/64, or QG_KERNEL_TILE128 (the
 *           caller's ksplit only: 0 does not split it; slices of at least four
 *           64-deep tiles, K a multiple of 64, dense weights -- otherwise the
 *           factor used is 1); another TILE kernel with ksplit > 1 is
 *           QG_EUNSUPPORTED
 *   ksplit  0 = built-in choice, 1 = no split, up to 64 slices of K; the factor
 *           actually used (qg_gemm_splitk_factor) never leaves a slice without a
 *           64-deep block of K
 *   workspace_dev / workspace_bytes  as above, at least
 *           qg_gemm_splitk_workspace_bytes(M, Bp, kernel, ksplit) bytes:
 *           QG_EWORKSPACE when NULL or too small while the factor used exceeds 1. */
size_t qg_gemm_splitk_workspace_bytes(int M, const qg_packed_b* Bp, int kernel, int ksplit);
int qg_gemm_splitk_factor(int M, const qg_packed_b* Bp, int kernel, int ksplit);
int qg_gemm_u8s8_requant_splitk(const uint8_t* A_dev, int M, int lda, const qg_packed_b* Bp,
                                const qg_requant_params* p, uint8_t* C_dev, int ldc, void* workspace_dev,
                                size_t workspace_bytes, void* stream, int kernel, int ksplit);
int qg_gemm_u8s8_acc32_splitk(const uint8_t* A_dev, int M, int lda, const qg_packed_b* Bp, int32_t* C32_dev,
                              int ldc, int32_t* rowsum_dev, void* workspace_dev, size_t workspace_bytes,
                              void* stream, int kernel, int ksplit);

/* For callers that cannot allocate device memory or hand a workspace through:
 * code under HIP graph capture, tight serving loops, harnesses that forbid
 * allocation.  qg_gemm_u8s8_requant_splitk with the workspace replaced by a
 * scratch array built into the library (QG_NOALLOC_SCRATCH_BYTES per GPU, held
 * from the first use of the library on that GPU until the process ends).  The
 * call allocates nothing and enqueues kernels only.
 *   kernel, ksplit  as qg_gemm_u8s8_requant_splitk (QG_KERNEL_AUTO / 0 = built-in choices)
 * QG_EWORKSPACE when the split in use needs more than QG_NOALLOC_SCRATCH_BYTES
 * (qg_gemm_splitk_workspace_bytes tells; pass ksplit = 1 to run without any).
 * All calls on one GPU share that GPU's array: calls that may overlap in time
 * (different streams, different threads) race on it and must not be made; one
 * after another on a stream they are safe, since every call leaves the array
 * ready for the next (a call that was killed mid-flight does not: the process
 * must then stop using this entry point on that GPU). */
#define QG_NOALLOC_SCRATCH_BYTES (2u << 20)
int qg_gemm_u8s8_requant_noalloc(const uint8_t* A_dev, int M, int lda, const qg_packed_b* Bp,
                                 const qg_requant_params* p, uint8_t* C_dev, int ldc, void* stream, int kernel,
                                 int ksplit);

/* ---- the other ends of the pipeline (Appendix B) --------------------------- */

/* The paper builds a pipeline from any packing routine for A and any output
 * processing around the same core kernels.  Two more ends are provided here:
 * fp32 activations that are quantized by the library, and an fp32 result. */

/* Output pipeline that leaves the result in fp32: the real-domain value of
 * Eq. (2), alpha_A alpha_B[j] * x, with x the corrected accumulator of
 * qg_requant_params (zero-point terms and bias included):
 *   C[i,j] = (float)x * scale[j]        ONE IEEE fp32 multiply after the
 *                                       int32 -> fp32 conversion (nearest even)
 *   relu != 0:  C[i,j] = max(C[i,j], 0) */
typedef struct {
  int32_t a_zp;          /* theta_A, 0..255                                   */
  const int32_t* bias;   /* dev, N entries in accumulator units, or NULL      */
  const float* scales;   /* dev, n_scales entries: alpha_A * alpha_B[j]       */
  int32_t n_scales;      /* 1 or N                                            */
  int32_t relu;          /* 0 or 1                                            */
} qg_dequant_params;

/* As qg_gemm_u8s8_requant, with the fp32 output pipeline above.
 *   C_dev  dev, float, row-major M x N, ldc >= N in ELEMENTS; must not alias A
 * 16-byte aligned C_dev with ldc a multiple of 4 takes the vector store path.
 * kernel: QG_KERNEL_AUTO or a kernel id. */
int qg_gemm_u8s8_dequant_f32(const uint8_t* A_dev, int M, int lda, const qg_packed_b* Bp,
                             const qg_dequant_params* p, float* C_dev, int ldc, void* workspace_dev,
                             void* stream, int kernel);

/* Quantization of fp32 activations, Eq. (1) solved for the quantized value:
 *   Aq[i,k] = clamp(rne(A[i,k] * inv_scale), -theta_A, 255 - theta_A) + theta_A
 * (inv_scale = 1 / alpha_A passed by the caller; ONE fp32 multiply; rne = round
 * to nearest even; the clamp happens in float).  A must hold no NaN; +-inf
 * saturate.  The fp32 matrix is read once; this is the bandwidth-bound
 * "packing" pass of the pipeline, one launch.
 *   A_dev   dev, float, row-major M x K, lda >= K (elements)
 *   Aq_dev  dev, uint8, row-major M x K, ldq >= K; must not alias A
 * No alignment required; 16-byte aligned A_dev with lda % 4 == 0 and 4-byte
 * aligned Aq_dev with ldq % 4 == 0 take the vector path. */
int qg_quantize_a_f32(const float* A_dev, int M, int K, int lda, float inv_scale, int a_zp,
                      uint8_t* Aq_dev, int ldq, void* stream);

/* fp32 activations in, either output; p->a_zp is the zero point of the quantization
 * and of Eq. (2).  Two forms, the same bytes either way:
 *  - with a workspace (qg_gemm_f32_workspace_bytes(M, Bp) bytes, 16-byte
 *    aligned): qg_quantize_a_f32 into the workspace, then the GEMM on the
 *    quantized copy, two launches on `stream`.  The quantized copy stays in
 *    the workspace.  This is the fast form on every shape measured: a tile of A
 *    is staged once per tile column of C, so converting while staging repeats
 *    the conversion for every column block.
 *  - workspace_dev == NULL and a streaming kernel (kernel, or what QG_KERNEL_AUTO
 *    resolves to, is QG_KERNEL_SKINNY*; dense descriptor): ONE launch, nothing
 *    written but C.  The kernel quantizes the block of A it stages, with the
 *    sequence of qg_quantize_a_f32, and takes row offsets from the staged block
 *    in the same pass (Appendix B: row offsets computed while packing A).
 *    A_dev 4-byte aligned; 16-byte aligned rows (A_dev % 16 == 0, lda % 4 == 0)
 *    take the vector loads.  For callers that cannot provide a workspace; it
 *    costs about 2 us more than the two launches at 16 x 4096 x 4096.
 *    workspace_dev == NULL with a tiled kernel is QG_EWORKSPACE. */
size_t qg_gemm_f32_workspace_bytes(int M, const qg_packed_b* Bp);
int qg_gemm_f32s8_requant(const float* A_dev, int M, int lda, float a_inv_scale, const qg_packed_b* Bp,
                          const qg_requant_params* p, uint8_t* C_dev, int ldc, void* workspace_dev,
                          void* stream, int kernel);
int qg_gemm_f32s8_dequant_f32(const float* A_dev, int M, int lda, float a_inv_scale,
                              const qg_packed_b* Bp, const qg_dequant_params* p, float* C_dev, int ldc,
                              void* workspace_dev, void* stream, int kernel);

/* ---- outlier-aware split of the weights (Sec. 2.2) ------------------------- */

/* The paper's sample pipeline splits the constant matrix into B = B' + B_sparse:
 * B' keeps the small-magnitude numbers, the few big ones go to B_sparse in a
 * compressed sparse column format, both prepared once offline, and
 * A B = A B' + A B_sparse with the sparse product fused into the output
 * processing.  There the point is a cheaper accumulation for B'; on this GPU
 * the point is bandwidth: B' (here: -8 <= b <= 7) is stored in 4 bits, which
 * halves the bytes the small-batch kernels stream.  Results are bit-identical
 * to the same call on a dense descriptor of B.
 *
 * A split descriptor runs on the streaming kernels only (QG_KERNEL_SKINNY*,
 * any M through row blocks); naming a TILE kernel returns QG_EUNSUPPORTED.
 *
 * Protocol: qg_count_outliers -> allocate -> qg_pack_b_outlier.  Both calls
 * wait for `stream`. */

/* Number of entries of B outside -8..7.  scratch_dev: 8 bytes of device memory,
 * 8-byte aligned. */
int qg_count_outliers(const int8_t* B_dev, int K, int N, int ldb, void* scratch_dev, size_t* nnz_host,
                      void* stream);

/* Buffer sizes for a split descriptor holding up to max_nnz outliers. */
int qg_pack_b_outlier_sizes(int K, int N, size_t max_nnz, size_t* packed_bytes,
                            size_t* col_offsets_bytes, size_t* sparse_bytes);

/* As qg_pack_b; packed_dev receives the 4-bit B', sparse_dev (256-byte aligned)
 * the sparse part; col_offsets are those of the whole B.  QG_ECAPACITY when B
 * holds more than max_nnz outliers (nothing usable is left in the buffers). */
int qg_pack_b_outlier(const int8_t* B_dev, int K, int N, int ldb, const int32_t* b_zp_host,
                      int n_b_zp, size_t max_nnz, void* packed_dev, int32_t* col_offsets_dev,
                      void* sparse_dev, void* stream, qg_packed_b** out);

/* Outliers held by a split descriptor (0 for a dense one or NULL). */
size_t qg_packed_b_nnz(const qg_packed_b* p);

/* ---- group-wise convolution with fused im2col ----------------------------- */

/* The paper names convolution without describing it; the definition used is the
 * real-domain one implied by Eq. (1): NHWC uint8 input with zero point theta_A,
 * zero padding in the real domain (= theta_A in the quantized domain), G groups,
 * each an independent GEMM with rows = output pixels, K = R*S*(C/G) ordered
 * (kh, kw, c_in), N = Cout/G.  The im2col matrix is never materialised.
 *   W_dev      dev, int8, [G][R][S][C/G][Cout/G]
 *   b_zp_host  HOST, 1 or Cout entries
 * Any G, R, S, C/G and Cout/G (R*S*C/G <= QG_MAX_K).  Groups of 4 -> 4 channels
 * with a 1 x 1 or 3 x 3 filter have the kernels this library is tuned for (one
 * dword per tap, or block-diagonal matrix-core tiles when C % 32 == 0); square
 * groups of 1 (a depthwise convolution), 2, 8, 16 or 32 channels with those
 * filters and C % 32 == 0 run the same matrix-core kernels on their own
 * block-diagonal tiles; other groups of a
 * multiple of 16 input channels (up to 64 groups, 16-byte aligned image) run one
 * dense convolution per group on the group's channel slice; every other shape
 * runs a plain one-thread-per-output kernel (correct for any extents, not tuned). */
int qg_pack_conv_w_sizes(int G, int R, int S, int Cg, int Og, size_t* packed_bytes,
                         size_t* col_offsets_bytes);
int qg_pack_conv_w(const int8_t* W_dev, int G, int R, int S, int Cg, int Og, const int32_t* b_zp_host,
                   int n_b_zp, void* packed_dev, int32_t* col_offsets_dev, void* stream,
                   qg_packed_b** out);

/* in_nhwc: dev uint8 [Nb][H][W][C]; out_nhwc: dev uint8 [Nb][Ho][Wo][Cout],
 * Ho = (H + 2*pad - R)/stride + 1 (same for Wo); both 4-byte aligned for the
 * 4 -> 4 groups (QG_EALIGN otherwise), any address for other group shapes.
 * p->n_scales is 1 or Cout, p->bias has Cout entries or is NULL. */
int qg_conv_groupwise_u8s8_requant(const uint8_t* in_nhwc, int Nb, int H, int W, int C, int pad,
                                   int stride, const qg_packed_b* Wp, const qg_requant_params* p,
                                   uint8_t* out_nhwc, void* stream);

/* ---- dense convolution with fused im2col ---------------------------------- */

/* Ordinary (one group) convolution as the same quantized GEMM: rows = output
 * pixels, K = R*S*Cin ordered (kh, kw, c_in), N = Cout; definition as for the
 * group-wise call (zero padding in the real domain).  The weights are packed
 * with qg_pack_b from the row-major (R*S*Cin) x Cout matrix W[kh][kw][ci][co];
 * the im2col matrix is never materialised: a 64-deep k tile is requested
 * straight from the image, as 64 channels of one filter tap when Cin % 64 == 0
 * and as four 16-channel pieces that may belong to different taps otherwise.  A 1 x 1 filter with
 * stride 1 and no padding IS the GEMM over the pixel rows and runs as
 * qg_gemm_u8s8_requant_kernel(in, Nb*H*W, Cin, ...) with the same kernel id.
 *   in_nhwc  dev uint8 [Nb][H][W][Cin]; 16-byte aligned with Cin % 16 == 0 for the staged
 *            kernels below -- any other image runs, under QG_KERNEL_AUTO only, on a kernel
 *            that gathers the im2col rows into LDS byte by byte -- four bytes at a time when
 *            Cin % 4 == 0 and the image is 4-byte aligned -- and multiplies them on the
 *            matrix cores (any extents; a 3- or 4-channel first layer is its case)
 *   out_nhwc dev uint8 [Nb][Ho][Wo][Cout], Ho = (H + 2*pad - R)/stride + 1
 *   kernel   QG_KERNEL_AUTO (chosen from the extents by a cost model fitted to 3 x 3 and
 *            5 x 5 layers, the patch kernels below included), or QG_KERNEL_TILE64 / TILE64K4 / TILE64X32K8 / TILE64K1 /
 *            TILE128 / TILE128X256; every choice gives the same bytes.  The 128-row tiles run
 *            their hand-scheduled loop when Cin % 64 == 0, R*S <= 32 and K >= 256.  With
 *            Cin % 64 == 0 and R*S <= 32 the streaming kernels QG_KERNEL_SKINNY16 / 32 / 64
 *            are taken too (few output pixels and a long K; QG_EUNSUPPORTED otherwise).
 *            QG_KERNEL_PATCH64X128 / PATCH128X64 / PATCH256X64 / PATCH256 / PATCH512 keep the input patch of a tile
 *            of 64 to 512 consecutive output pixels in LDS and stream only the weights: "same" convolutions
 *            (stride 1, R == S odd, 2*pad == R - 1, R*S <= 28) with Cin % 32 == 0, pixels less
 *            than 64 KiB apart and a patch that fits the LDS; QG_EUNSUPPORTED otherwise.
 * QG_EUNSUPPORTED for QG_KERNEL_TILE256, or an explicit kernel id with such an image;
 * QG_EINVAL when R*S*Cin differs from the K of Wp or the id is unknown. */
int qg_conv_dense_u8s8_requant(const uint8_t* in_nhwc, int Nb, int H, int W, int Cin, int R, int S,
                               int pad, int stride, const qg_packed_b* Wp, const qg_requant_params* p,
                               uint8_t* out_nhwc, void* stream, int kernel);

const char* qg_status_string(int code);

#ifdef __cplusplus
}
#endif
#endif /* QGEMM_H */
