// Host side of the C ABI declared in qgemm.h: argument checks, descriptor
// bookkeeping and kernel selection by shape.  No device allocation, no stream
// creation, no synchronisation happens here (paper Appendix A: the library works
// on caller-provided buffers and leaves parallelism to the caller).
#include <math.h>

#include <new>
#include <vector>

#include "qg_internal.h"

namespace {

inline bool aligned(const void* p, size_t a) { return (reinterpret_cast<uintptr_t>(p) % a) == 0; }

int check_requant(const qg_requant_params* p, int N) {
  if (!p) return QG_ENULL;
  if (!p->scales) return QG_ENULL;
  if (p->a_zp < 0 || p->a_zp > 255 || p->c_zp < 0 || p->c_zp > 255) return QG_EINVAL;
  if (p->n_scales != 1 && p->n_scales != N) return QG_EINVAL;
  if (p->relu != 0 && p->relu != 1) return QG_EINVAL;
  return QG_OK;
}

// Builds the padded per-column theta_B array on the host and enqueues its upload
// into the second half of the caller's col_offsets buffer.
int upload_bzp(const int32_t* b_zp_host, int n_b_zp, int N, int N_pad, int32_t* dst_dev, hipStream_t s,
               int* has_bzp) {
  std::vector<int32_t> tmp;
  try {
    tmp.assign((size_t)N_pad, 0);
  } catch (const std::bad_alloc&) {
    return QG_ENOMEM;
  }
  int any = 0;
  for (int j = 0; j < N; ++j) {
    const int32_t z = b_zp_host[n_b_zp == 1 ? 0 : j];
    if (z < -128 || z > 127) return QG_EINVAL;
    tmp[j] = z;
    any |= (z != 0);
  }
  *has_bzp = any;
  // pageable source: the runtime stages it before returning, so tmp may die here
  if (hipMemcpyAsync(dst_dev, tmp.data(), sizeof(int32_t) * (size_t)N_pad, hipMemcpyHostToDevice, s) !=
      hipSuccess)
    return QG_ELAUNCH;
  if (hipStreamSynchronize(s) != hipSuccess) return QG_ELAUNCH;  // offline path; keeps tmp's lifetime trivially safe
  return QG_OK;
}

// ---- kernel selection by shape (paper Appendix C) --------------------------------------------
qg_dispatch_rule g_rules[QG_MAX_DISPATCH_RULES];
int g_nrules = 0;

inline int ceil_div(int a, int b) { return (a + b - 1) / b; }

// Built-in choice: a small cost model of every kernel, fitted to timings of the whole family over a grid of
// shapes on MI355X (256 CUs), evaluated for the shape at hand; the cheapest estimate wins.
//
// Tiled kernels.  A workgroup alone on the chip needs `lat` us per 64-deep k step (one barrier plus request
// latency) and `fix` us of launch, prologue and output pipeline.  With the chip full, each of the
// ceil(workgroups / 256) workgroups a CU has to run costs `thr` us per k step and `epi` us of output
// pipeline: a big tile moves the fewest LDS bytes per multiply (small `thr` per unit of work) but pays for
// it with few, long workgroups.  The estimate is the larger of the two regimes; a grid of at most one
// workgroup per CU is in the first by definition.
// Streaming kernels.  One workgroup per 16 columns and per row block; alone it takes fix + K * lat_k us, with
// the chip full each workgroup costs wg + K * wg_k nanoseconds; a third bound covers tall, narrow shapes.
struct tile_cost {
  int kernel, bm, bn;
  double fix, lat, thr, epi;
  double out = 0.0;  // output bytes per microsecond that the kernel sustains when K is short; 0 = never the bound
};
struct stream_cost {
  int kernel, rows;
  double fix, lat_k, wg, wg_k;
};
const tile_cost k_tile_cost[] = {
    {QG_KERNEL_TILE64, 64, 64, 3.169, 0.1296, 0.1046, 0.6015},
    {QG_KERNEL_TILE128, 128, 128, 3.401, 0.242, 0.2725, 1.102, 2.88e6},
    {QG_KERNEL_TILE128X256, 128, 256, 5.288, 0.3543, 0.4409, 2.253},
    {QG_KERNEL_TILE256, 256, 256, 7.789, 0.6867, 0.8478, 6.549},
    {QG_KERNEL_TILE64K4, 64, 64, 3.617, 0.1035, 0.1077, 2.38},
    {QG_KERNEL_TILE64K1, 64, 64, 2.714, 0.2482, 0.1361, 0.1909, 2.35e6},
    {QG_KERNEL_TILE64X32K8, 64, 32, 3.817, 0.05427, 0.0602, 2.585},
};
// The dense convolution runs the same tile loops with the im2col addressing folded into the requests; the same
// formula, constants fitted to 56 layers (3 x 3 and 5 x 5, stride 1 and 2, 1 .. 32 images, Cin % 64 == 0; graph-replay
// times): the choice is within 5 % of the measured best on 54 of them, worst 1.07x.  The 64 x 64 tile comes without a
// K split and with two or four wave sets that share K, the 64 x 32 tile with eight.
const tile_cost k_conv_cost[] = {
    {QG_KERNEL_TILE64K1, 64, 64, 2.55, 0.412, 0.136, 0.432},
    {QG_KERNEL_TILE64, 64, 64, 3.95, 0.167, 0.115, 1.24},
    {QG_KERNEL_TILE64K4, 64, 64, 5.36, 0.118, 0.112, 3.74},
    {QG_KERNEL_TILE64X32K8, 64, 32, 6.28, 0.0686, 0.0682, 4.43},
    {QG_KERNEL_TILE128, 128, 128, 5.68, 0.279, 0.229, 2.36},
    {QG_KERNEL_TILE128X256, 128, 256, 11.1, 0.261, 0.353, 4.01},
};
// "Same" convolutions (stride 1, output as large as the input) with Cin % 32 == 0 also have the kernels that keep the
// input patch of a pixel tile in LDS; same formula, fitted to 80 layers (3 x 3 and 5 x 5, 1 .. 32 images, 32 .. 512
// channels; the 512 x 128 form to the layers of the autotuner's convolution grid).  Over the 100 layers of that grid
// the automatic choice among all of these kernels is within 5 % of the measured best on 91 (geometric mean 1.009x,
// worst 1.10x), and the best kernel is one of these on 49 (up to 1.74x faster than the best of the others).
const tile_cost k_conv_patch_cost[] = {
    {QG_KERNEL_PATCH64X128, 64, 128, 4.86, 0.137, 0.119, 1.4},
    {QG_KERNEL_PATCH128X64, 128, 64, 4.83, 0.148, 0.135, 1.32},
    {QG_KERNEL_PATCH256X64, 256, 64, 5.5, 0.196, 0.25, 1.84},
    {QG_KERNEL_PATCH256, 256, 128, 5.78, 0.381, 0.642, 0.756},
    {QG_KERNEL_PATCH512, 512, 128, 10.0, 0.603, 0.973, 3.72},
};
const stream_cost k_stream_cost[] = {
    {QG_KERNEL_SKINNY16, 16, 3.826, 3.664e-06, 5.429, 0.002625},
    {QG_KERNEL_SKINNY32, 32, 3.918, 2.404e-05, 8.639, 0.0005841},
    {QG_KERNEL_SKINNY64, 64, 3.821, 0.0004905, 9.136, 0.002971},
};
// The 16-row kernel's four-wave form (more than 128 super-blocks of 16 rows x 32 columns, K a multiple of 2048,
// dense weights): the same formula per super-block.
const stream_cost k_stream_wide_cost = {QG_KERNEL_SKINNY16, 16, 3.191, 0.0002712, 4.302e-05, 0.001958};
// A streaming workgroup re-reads its rows of A for every 16 columns; with few columns to share them that
// traffic comes from far memory, row piece by row piece, at about this many bytes per microsecond.
const double k_stream_a_rate = 2.0e6;
const double k_stream_a_near = 1048576.0;     // bytes of A that the L2s keep
const double k_stream_a_far_rate = 1.0e7;     // bytes per microsecond, all workgroups together

double stream_estimate(const stream_cost& c, int M, int N, int K, bool dense) {
  double a_bound = 2.5 + (double)M * (double)K / k_stream_a_rate;
  const double blocks32 = (double)ceil_div(M, c.rows) * (double)ceil_div(N, 32);
  if (dense && c.kernel == QG_KERNEL_SKINNY16 && blocks32 > 128.0 && K % 2048 == 0) {
    const stream_cost& w = k_stream_wide_cost;
    return fmax(fmax(w.fix + K * w.lat_k, a_bound), 2.5 + blocks32 * (w.wg + K * w.wg_k) * 1e-3);
  }
  const double wgs = 2.0 * blocks32;
  // an A too large to stay in the L2s is fetched from far memory once per 16 columns
  if ((double)M * (double)K > k_stream_a_near)
    a_bound = fmax(a_bound, 2.5 + (double)M * (double)K * (double)ceil_div(N, 16) / k_stream_a_far_rate);
  const double alone = fmax(c.fix + K * c.lat_k, a_bound);
  if (wgs <= 256.0) return alone;  // at most one workgroup per CU: each runs as if alone
  return fmax(alone, 2.5 + wgs * (c.wg + K * c.wg_k) * 1e-3);
}

double tile_estimate(const tile_cost& c, int M, int N, int K) {
  const double kt = (double)ceil_div(K, 64);
  const double wgs = (double)ceil_div(M, c.bm) * (double)ceil_div(N, c.bn);
  const double alone = c.fix + kt * c.lat;
  if (wgs <= 256.0) return alone;
  double us = fmax(alone, 2.5 + ceil(wgs / 256.0) * (kt * c.thr + c.epi));
  // many rows and a K of one or two tiles (the 1 x 1 layers of a convolutional network as GEMMs): little but output,
  // at a rate measured on 30 such shapes (without this bound the 64 x 64 tile was chosen for 100352 x 256 x 64,
  // 1.15x behind the 128 x 128 tile)
  if (c.out > 0.0) us = fmax(us, 2.5 + (double)M * (double)N / c.out);
  return us;
}

int builtin_select(int M, int N, int K) {
  int best = QG_KERNEL_TILE64;
  double best_us = 1e300;
  for (const stream_cost& c : k_stream_cost) {
    const long long blocks = ceil_div(M, c.rows);
    if (blocks > 65535) continue;
    const double us = stream_estimate(c, M, N, K, true);
    if (us < best_us) best_us = us, best = c.kernel;
  }
  for (const tile_cost& c : k_tile_cost) {
    const double us = tile_estimate(c, M, N, K);
    if (us < best_us) best_us = us, best = c.kernel;
  }
  return best;
}

// cheapest streaming kernel (outlier-split descriptors run on these only, always in the 16-wave form: the constants
// fitted when every shape ran that form, large column counts included)
const stream_cost k_stream_cost_16wave[] = {
    {QG_KERNEL_SKINNY16, 16, 3.58, 7.3e-5, 7.55, 0.74e-3},
    {QG_KERNEL_SKINNY32, 32, 4.13, 1.99e-4, 10.33, 1.28e-3},
    {QG_KERNEL_SKINNY64, 64, 4.96, 3.88e-4, 14.26, 2.23e-3},
};
// The same kernels with the convolution's per-lane tap addressing in their requests: the streaming formula with
// constants of their own, fitted to 72 layers (Cin % 64 == 0; 3 x 3 and 5 x 5, stride 1 and 2, 1 .. 32 images).
const stream_cost k_conv_stream_cost[] = {
    {QG_KERNEL_SKINNY16, 16, 5.24, 2.1e-4, 12.0, 1.4e-3},
    {QG_KERNEL_SKINNY32, 32, 5.74, 4.39e-4, 18.2, 1.85e-3},
    {QG_KERNEL_SKINNY64, 64, 7.35, 6.52e-4, 24.4, 4.24e-3},
};

int select_stream_kernel(int M, int N, int K) {
  int best = QG_KERNEL_SKINNY64;
  double best_us = 1e300;
  for (const stream_cost& c : k_stream_cost_16wave) {
    const long long blocks = ceil_div(M, c.rows);
    if (blocks > 65535) continue;
    const double us = stream_estimate(c, M, N, K, false);
    if (us < best_us) best_us = us, best = c.kernel;
  }
  return best;
}

int select_kernel(int M, int N, int K) {
  for (int i = 0; i < g_nrules; ++i) {
    const qg_dispatch_rule& r = g_rules[i];
    if (M >= r.m_lo && M <= r.m_hi && N >= r.n_lo && N <= r.n_hi && K >= r.k_lo && K <= r.k_hi) return r.kernel;
  }
  return builtin_select(M, N, K);
}

hipError_t launch_rows(const qg_gemm_args& a, int mode, int kernel, hipStream_t s) {
  if (kernel <= QG_KERNEL_SKINNY64) return qg_launch_gemm_skinny(a, mode, kernel, s);
  return qg_launch_gemm_tile(a, mode, kernel, s);
}

// The kernels address A with 32-bit byte offsets from its base.  An A beyond that reach is run as several
// launches over consecutive row ranges (whole 256-row tiles where possible, so the tiling is that of one launch),
// each with its own base pointers; rows are independent, the result is the same.
hipError_t launch_gemm(const qg_gemm_args& a, int mode, int kernel, hipStream_t s) {
  const uint64_t reach = (1ull << 32) - (uint64_t)a.K - 4096;
  if ((uint64_t)(a.M - 1) * (uint64_t)a.lda < reach) return launch_rows(a, mode, kernel, s);
  int rows = (int)(reach / (uint64_t)a.lda);  // >= 1: lda is an int
  if (rows >= 256) rows = rows / 256 * 256;
  for (int r0 = 0; r0 < a.M; r0 += rows) {
    qg_gemm_args b = a;
    b.M = a.M - r0 < rows ? a.M - r0 : rows;
    b.A = a.A + (size_t)r0 * (size_t)a.lda;
    if (a.C) b.C = a.C + (size_t)r0 * (size_t)a.ldc;
    if (a.Cf) b.Cf = a.Cf + (size_t)r0 * (size_t)a.ldc;
    if (a.C32) b.C32 = a.C32 + (size_t)r0 * (size_t)a.ldc;
    if (a.rowsum_out) b.rowsum_out = a.rowsum_out + r0;
    const hipError_t e = launch_rows(b, mode, kernel, s);
    if (e != hipSuccess) return e;
  }
  return hipSuccess;
}

// resolves QG_KERNEL_AUTO for a descriptor and checks an explicit choice against it: QG_OK, or
// QG_EINVAL (unknown id / too many row blocks), QG_EUNSUPPORTED (tiled kernel on a split descriptor)
int resolve_kernel(const qg_packed_b* Bp, int M, int* kernel);

// kernel id valid for this M (the streaming kernels put row blocks on the 16-bit grid dimension)
bool kernel_ok(int kernel, int M) {
  if (kernel < QG_KERNEL_AUTO || kernel > QG_KERNEL_LAST) return false;
  if (kernel >= QG_KERNEL_SKINNY16 && kernel <= QG_KERNEL_SKINNY64)
    return ceil_div(M, 16 << (kernel - QG_KERNEL_SKINNY16)) <= 65535;
  return true;
}

int resolve_kernel(const qg_packed_b* Bp, int M, int* kernel) {
  if (!kernel_ok(*kernel, M)) return QG_EINVAL;
  if (Bp->split) {
    if (*kernel == QG_KERNEL_AUTO) *kernel = select_stream_kernel(M, Bp->N, Bp->K);
    if (*kernel > QG_KERNEL_SKINNY64) return QG_EUNSUPPORTED;
    return kernel_ok(*kernel, M) ? QG_OK : QG_EINVAL;
  }
  if (*kernel == QG_KERNEL_AUTO) {
    *kernel = select_kernel(M, Bp->N, Bp->K);
    if (!kernel_ok(*kernel, M)) *kernel = builtin_select(M, Bp->N, Bp->K);
  }
  return QG_OK;
}

// ---- K split across workgroups (streaming kernels; the caller's workspace is the paper's C_buffer, Appendix A)
constexpr int kSlotInts = 64 * 4 + 16;   // one (K slice, row block of 16) slot: 64 lanes x 4 partial sums + 16 row sums
constexpr int kMaxKsplit = 64;

struct splitk_layout {
  size_t cnt_ints, slot_ints;
  size_t bytes() const { return (cnt_ints + slot_ints) * sizeof(int32_t); }
};
// counters first (one per row block of 16 and fragment column, rounded up to 256 bytes), then the slots
splitk_layout splitk_ws(int kernel, int M, int N, int ksplit) {
  if (kernel == QG_KERNEL_TILE128) {  // one counter per 128 x 128 tile; a slot is 256 threads x (64 sums + 2 row offsets)
    const size_t tiles = (size_t)ceil_div(M, 128) * (size_t)ceil_div(N, 128);
    return {(tiles + 63) / 64 * 64, tiles * (size_t)ksplit * (66 * 256)};
  }
  const int rows = 16 << (kernel - QG_KERNEL_SKINNY16);
  const size_t units = (size_t)ceil_div(M, rows) * (size_t)(2 * ceil_div(N, 32)) * (size_t)(rows / 16);
  return {(units + 63) / 64 * 64, units * (size_t)ksplit * kSlotInts};
}
// slices that are all non-empty: at most one per 64-deep block of K (a pair of blocks for 4-bit weights)
int clamp_ksplit(const qg_packed_b* Bp, int ksplit) {
  const int blocks = Bp->K_pad / QG_FRAG_K / (Bp->split ? 2 : 1);
  if (ksplit > blocks) ksplit = blocks;
  const int per = ceil_div(blocks, ksplit);
  return ceil_div(blocks, per);
}
// Built-in choice of the split, from timings of 16 x {16..512} x {4096..32768} and 64 x {64, 256} x {8192, 16384}
// (cold weights): handing a partial tile through the workspace costs 1.5 - 2 us, so a split pays only where it
// removes several batches of weight loads from every wave's chain.  Give each wave of a slice four 64-deep blocks
// (one batch of loads); take the split from 4 slices up (from 2 for 64-row blocks, whose waves do four times the
// work per block), and never more slices than there are idle CUs to take them.
// The 128 x 128 tile: slices of whole 64-deep tiles, at least four each (the depth of the hand-scheduled loop's
// pipeline), K a multiple of 64, dense weights.  -> the number of slices that `ksplit` gives, 1 if it cannot be split
int clamp_ksplit_tile128(const qg_packed_b* Bp, int ksplit) {
  if (Bp->split || Bp->K % QG_FRAG_K != 0) return 1;
  const int blocks = Bp->K / QG_FRAG_K;
  if (ksplit > blocks / 4) ksplit = blocks / 4;
  while (ksplit > 1) {
    const int per = ceil_div(blocks, ksplit), s = ceil_div(blocks, per);
    if (blocks - (s - 1) * per >= 4) return s;
    --ksplit;
  }
  return 1;
}
int auto_ksplit(int kernel, int M, const qg_packed_b* Bp) {
  if (kernel < QG_KERNEL_SKINNY16 || kernel > QG_KERNEL_SKINNY64) return 1;
  const int rows = 16 << (kernel - QG_KERNEL_SKINNY16);
  const long long wgs = (long long)ceil_div(M, rows) * (2 * ceil_div(Bp->N, 32));
  if (wgs * 2 > 256) return 1;
  int s = Bp->K_pad / QG_FRAG_K / (16 * 4);  // 16 waves x 4 blocks
  if (s > 256 / wgs) s = (int)(256 / wgs);
  if (s > 16) s = 16;
  if (s < (rows == 64 ? 2 : 4)) return 1;
  return clamp_ksplit(Bp, s);
}
// ksplit_req: 0 = built-in choice (1 without a workspace), otherwise the caller's.  Fills the workspace fields of `a`.
int resolve_ksplit(const qg_packed_b* Bp, int M, int kernel, int ksplit_req, void* workspace_dev, size_t workspace_bytes,
                   bool bytes_known, qg_gemm_args* a) {
  a->ksplit = 1;
  a->ks_per = Bp->K_pad / QG_FRAG_K;
  a->ws_cnt = a->ws_slots = nullptr;
  if (ksplit_req < 0 || ksplit_req > kMaxKsplit) return QG_EINVAL;
  if (M == 0) return QG_OK;
  int s = ksplit_req;
  if (kernel == QG_KERNEL_TILE128 && s > 1) {
    // the caller's split on the 128 x 128 tile (never the built-in choice)
    s = clamp_ksplit_tile128(Bp, s);
    if (s <= 1) return QG_OK;
    if (!workspace_dev) return QG_EWORKSPACE;
    if (!aligned(workspace_dev, 16)) return QG_EALIGN;
    const splitk_layout w = splitk_ws(kernel, M, Bp->N, s);
    if (bytes_known && workspace_bytes < w.bytes()) return QG_EWORKSPACE;
    a->ksplit = s;
    a->ks_per = ceil_div(Bp->K / QG_FRAG_K, s);
    a->ws_cnt = static_cast<int32_t*>(workspace_dev);
    a->ws_slots = a->ws_cnt + w.cnt_ints;
    return QG_OK;
  }
  if (kernel > QG_KERNEL_SKINNY64) {
    if (s > 1) return QG_EUNSUPPORTED;  // the other tiled kernels keep K inside the workgroup
    return QG_OK;
  }
  if (s == 0) s = workspace_dev ? auto_ksplit(kernel, M, Bp) : 1;
  s = clamp_ksplit(Bp, s);
  if (s <= 1) return QG_OK;
  if (!workspace_dev) return QG_EWORKSPACE;
  if (!aligned(workspace_dev, 16)) return QG_EALIGN;
  const splitk_layout w = splitk_ws(kernel, M, Bp->N, s);
  if (bytes_known && workspace_bytes < w.bytes()) return QG_EWORKSPACE;
  a->ksplit = s;
  {
    const int unit = Bp->split ? 2 : 1, blocks = Bp->K_pad / QG_FRAG_K / unit;
    a->ks_per = ceil_div(blocks, s) * unit;
  }
  a->ws_cnt = static_cast<int32_t*>(workspace_dev);
  a->ws_slots = a->ws_cnt + w.cnt_ints;
  return QG_OK;
}

// ---- built-in scratch for callers that cannot allocate (qg_gemm_u8s8_requant_noalloc) -------------------------
// The K-split workspace as a file-scope device array: every GPU the library runs on holds its own copy, at its own
// address, from the moment the code object is loaded until the process ends.  Zero-initialised at load, and every
// call leaves the ticket counters at zero, so no clearing pass is needed between calls.  In host code the array's
// name is only a handle: the device address comes from hipGetSymbolAddress, once per device.
static __device__ __align__(256) int32_t qg_noalloc_scratch[QG_NOALLOC_SCRATCH_BYTES / sizeof(int32_t)];
void* g_scratch_ptr[64] = {nullptr};  // per device; concurrent first calls may both look it up (same answer)

int noalloc_scratch(void** out) {
  int dev = 0;
  if (hipGetDevice(&dev) != hipSuccess) return QG_ELAUNCH;
  if (dev < 0 || dev >= 64) return QG_EUNSUPPORTED;
  if (!g_scratch_ptr[dev]) {
    void* ptr = nullptr;
    if (hipGetSymbolAddress(&ptr, HIP_SYMBOL(qg_noalloc_scratch)) != hipSuccess || !ptr) {
      (void)hipGetLastError();
      return QG_ELAUNCH;
    }
    g_scratch_ptr[dev] = ptr;
  }
  *out = g_scratch_ptr[dev];
  return QG_OK;
}

__global__ void qg_fill_zero_kernel(int32_t* p, size_t n) {
  size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
  const size_t stride = (size_t)gridDim.x * blockDim.x;
  for (; i < n; i += stride) p[i] = 0;
}

}  // namespace

extern "C" {

const char* qg_kernel_name(int kernel) {
  static const char* const names[] = {"auto",   "skinny16", "skinny32",    "skinny64",
                                      "tile64", "tile128",  "tile128x256", "tile256",
                                      "tile64k4", "tile64k1", "tile64x32k8",
                                      "patch64x128", "patch128x64", "patch256x64", "patch256", "patch512"};
  return (kernel >= 0 && kernel <= QG_KERNEL_CONV_LAST) ? names[kernel] : nullptr;
}

int qg_kernel_select(int M, int N, int K) {
  if (M <= 0 || N <= 0 || K <= 0) return QG_EINVAL;
  int k = select_kernel(M, N, K);
  if (!kernel_ok(k, M)) k = builtin_select(M, N, K);
  return k;
}

int qg_dispatch_set_rules(const qg_dispatch_rule* rules_host, int n) {
  if (n < 0 || n > QG_MAX_DISPATCH_RULES) return QG_EINVAL;
  if (n > 0 && !rules_host) return QG_ENULL;
  for (int i = 0; i < n; ++i) {
    const qg_dispatch_rule& r = rules_host[i];
    if (r.m_lo > r.m_hi || r.n_lo > r.n_hi || r.k_lo > r.k_hi) return QG_EINVAL;
    if (r.kernel < QG_KERNEL_SKINNY16 || r.kernel > QG_KERNEL_LAST) return QG_EINVAL;
  }
  for (int i = 0; i < n; ++i) g_rules[i] = rules_host[i];
  g_nrules = n;
  return QG_OK;
}

const char* qg_status_string(int code) {
  switch (code) {
    case QG_OK: return "ok";
    case QG_ENULL: return "required pointer is NULL";
    case QG_EINVAL: return "invalid size, leading dimension, zero point or count";
    case QG_EALIGN: return "device pointer alignment violated";
    case QG_EWORKSPACE: return "workspace required but not provided";
    case QG_ELAUNCH: return "HIP runtime refused the launch or copy";
    case QG_ENOMEM: return "host allocation failed";
    case QG_EUNSUPPORTED: return "configuration not implemented in this build";
    case QG_ECAPACITY: return "more outliers than the sparse buffer holds";
    default: return "unknown status";
  }
}

int qg_pack_b_sizes(int K, int N, size_t* packed_bytes, size_t* col_offsets_bytes) {
  if (!packed_bytes || !col_offsets_bytes) return QG_ENULL;
  if (K <= 0 || N <= 0 || K > QG_MAX_K) return QG_EINVAL;
  const size_t K_pad = (size_t)qg_round_up(K, QG_KPAD), N_pad = (size_t)qg_round_up(N, QG_NPAD);
  *packed_bytes = K_pad * N_pad;
  *col_offsets_bytes = 2 * N_pad * sizeof(int32_t);
  return QG_OK;
}

static int pack_b_any(const int8_t* B_dev, int K, int N, int ldb, int transposed, const int32_t* b_zp_host,
                      int n_b_zp, void* packed_dev, int32_t* col_offsets_dev, void* stream, qg_packed_b** out);

int qg_pack_b(const int8_t* B_dev, int K, int N, int ldb, const int32_t* b_zp_host, int n_b_zp,
              void* packed_dev, int32_t* col_offsets_dev, void* stream, qg_packed_b** out) {
  return pack_b_any(B_dev, K, N, ldb, 0, b_zp_host, n_b_zp, packed_dev, col_offsets_dev, stream, out);
}

int qg_pack_b_transposed(const int8_t* Bt_dev, int K, int N, int ldbt, const int32_t* b_zp_host, int n_b_zp,
                         void* packed_dev, int32_t* col_offsets_dev, void* stream, qg_packed_b** out) {
  return pack_b_any(Bt_dev, K, N, ldbt, 1, b_zp_host, n_b_zp, packed_dev, col_offsets_dev, stream, out);
}

static int pack_b_any(const int8_t* B_dev, int K, int N, int ldb, int transposed, const int32_t* b_zp_host,
                      int n_b_zp, void* packed_dev, int32_t* col_offsets_dev, void* stream, qg_packed_b** out) {
  if (!B_dev || !b_zp_host || !packed_dev || !col_offsets_dev || !out) return QG_ENULL;
  if (K <= 0 || N <= 0 || K > QG_MAX_K || ldb < (transposed ? K : N)) return QG_EINVAL;
  if (n_b_zp != 1 && n_b_zp != N) return QG_EINVAL;
  if (!aligned(packed_dev, 256) || !aligned(col_offsets_dev, 256)) return QG_EALIGN;
  hipStream_t s = static_cast<hipStream_t>(stream);
  const int K_pad = qg_round_up(K, QG_KPAD), N_pad = qg_round_up(N, QG_NPAD);

  qg_packed_b* h = new (std::nothrow) qg_packed_b();
  if (!h) return QG_ENOMEM;
  h->kind = QG_KIND_GEMM;
  h->version = QG_LAYOUT_VERSION;
  h->K = K;
  h->N = N;
  h->K_pad = K_pad;
  h->N_pad = N_pad;
  h->n_b_zp = n_b_zp;
  h->packed = static_cast<const int8_t*>(packed_dev);
  h->col_off = col_offsets_dev;
  h->bzp = col_offsets_dev + N_pad;
  h->G = h->R = h->S = h->Cg = h->Og = 0;
  h->conv_frags = nullptr;
  h->split = 0;
  h->frag_ptr = h->entries = nullptr;
  h->nnz = 0;

  int rc = upload_bzp(b_zp_host, n_b_zp, N, N_pad, col_offsets_dev + N_pad, s, &h->has_bzp);
  if (rc != QG_OK) {
    delete h;
    return rc;
  }
  if (qg_launch_pack_b(B_dev, K, N, ldb, transposed, K_pad, N_pad, static_cast<int8_t*>(packed_dev), col_offsets_dev,
                       col_offsets_dev + N_pad, s) != hipSuccess) {
    delete h;
    return QG_ELAUNCH;
  }
  *out = h;
  return QG_OK;
}

void qg_packed_b_destroy(qg_packed_b* p) { delete p; }

int qg_packed_b_k(const qg_packed_b* p) { return p ? p->K : 0; }
int qg_packed_b_n(const qg_packed_b* p) { return p ? p->N : 0; }

int qg_count_outliers(const int8_t* B_dev, int K, int N, int ldb, void* scratch_dev, size_t* nnz_host, void* stream) {
  if (!B_dev || !scratch_dev || !nnz_host) return QG_ENULL;
  if (K <= 0 || N <= 0 || K > QG_MAX_K || ldb < N) return QG_EINVAL;
  if (!aligned(scratch_dev, 8)) return QG_EALIGN;
  hipStream_t s = static_cast<hipStream_t>(stream);
  unsigned long long* cnt = static_cast<unsigned long long*>(scratch_dev);
  if (qg_launch_count_outliers(B_dev, K, N, ldb, cnt, s) != hipSuccess) return QG_ELAUNCH;
  unsigned long long host = 0;
  if (hipMemcpyAsync(&host, cnt, sizeof(host), hipMemcpyDeviceToHost, s) != hipSuccess) return QG_ELAUNCH;
  if (hipStreamSynchronize(s) != hipSuccess) return QG_ELAUNCH;
  *nnz_host = (size_t)host;
  return QG_OK;
}

// [frag_ptr: nbucket+1][cursor: nbucket] int32, rounded up to 256 B; one bucket per fragment of the packed matrix
static size_t sparse_buckets(int K_pad, int N_pad) { return (size_t)(N_pad / QG_FRAG_COLS) * (size_t)(K_pad / QG_FRAG_K); }
static size_t sparse_header_bytes(int K_pad, int N_pad) {
  return ((2 * sparse_buckets(K_pad, N_pad) + 1) * sizeof(int32_t) + 255) / 256 * 256;
}

int qg_pack_b_outlier_sizes(int K, int N, size_t max_nnz, size_t* packed_bytes, size_t* col_offsets_bytes,
                            size_t* sparse_bytes) {
  if (!packed_bytes || !col_offsets_bytes || !sparse_bytes) return QG_ENULL;
  if (K <= 0 || N <= 0 || K > QG_MAX_K) return QG_EINVAL;
  if (max_nnz > (size_t)0x7FFFFFFF) return QG_EINVAL;
  const size_t K_pad = (size_t)qg_round_up(K, QG_KPAD), N_pad = (size_t)qg_round_up(N, QG_NPAD);
  *packed_bytes = K_pad * N_pad / 2;
  *col_offsets_bytes = 2 * N_pad * sizeof(int32_t);
  *sparse_bytes = sparse_header_bytes((int)K_pad, (int)N_pad) + (max_nnz ? max_nnz : 1) * sizeof(int32_t);
  return QG_OK;
}

int qg_pack_b_outlier(const int8_t* B_dev, int K, int N, int ldb, const int32_t* b_zp_host, int n_b_zp,
                      size_t max_nnz, void* packed_dev, int32_t* col_offsets_dev, void* sparse_dev, void* stream,
                      qg_packed_b** out) {
  if (!B_dev || !b_zp_host || !packed_dev || !col_offsets_dev || !sparse_dev || !out) return QG_ENULL;
  if (K <= 0 || N <= 0 || K > QG_MAX_K || ldb < N) return QG_EINVAL;
  if (n_b_zp != 1 && n_b_zp != N) return QG_EINVAL;
  if (max_nnz > (size_t)0x7FFFFFFF) return QG_EINVAL;
  if (!aligned(packed_dev, 256) || !aligned(col_offsets_dev, 256) || !aligned(sparse_dev, 256)) return QG_EALIGN;
  hipStream_t s = static_cast<hipStream_t>(stream);
  const int K_pad = qg_round_up(K, QG_KPAD), N_pad = qg_round_up(N, QG_NPAD);
  const size_t nbucket = sparse_buckets(K_pad, N_pad);
  int32_t* frag_ptr = static_cast<int32_t*>(sparse_dev);
  int32_t* cursor = frag_ptr + nbucket + 1;
  int32_t* entries =
      reinterpret_cast<int32_t*>(static_cast<unsigned char*>(sparse_dev) + sparse_header_bytes(K_pad, N_pad));

  qg_packed_b* h = new (std::nothrow) qg_packed_b();
  if (!h) return QG_ENOMEM;
  h->kind = QG_KIND_GEMM;
  h->version = QG_LAYOUT_VERSION;
  h->K = K;
  h->N = N;
  h->K_pad = K_pad;
  h->N_pad = N_pad;
  h->n_b_zp = n_b_zp;
  h->packed = static_cast<const int8_t*>(packed_dev);
  h->col_off = col_offsets_dev;
  h->bzp = col_offsets_dev + N_pad;
  h->G = h->R = h->S = h->Cg = h->Og = 0;
  h->conv_frags = nullptr;
  h->split = 1;
  h->frag_ptr = frag_ptr;
  h->entries = entries;
  h->nnz = 0;

  int rc = upload_bzp(b_zp_host, n_b_zp, N, N_pad, col_offsets_dev + N_pad, s, &h->has_bzp);
  int32_t total = 0;
  if (rc == QG_OK && qg_launch_pack_b_split_count(B_dev, K, N, ldb, K_pad, N_pad, static_cast<uint8_t*>(packed_dev),
                                                  col_offsets_dev, col_offsets_dev + N_pad, frag_ptr, cursor,
                                                  s) != hipSuccess)
    rc = QG_ELAUNCH;
  // the total decides whether the fill may run: it must not write past the caller's capacity
  if (rc == QG_OK && (hipMemcpyAsync(&total, frag_ptr + nbucket, sizeof(total), hipMemcpyDeviceToHost, s) != hipSuccess ||
                      hipStreamSynchronize(s) != hipSuccess))
    rc = QG_ELAUNCH;
  if (rc == QG_OK && (total < 0 || (size_t)total > max_nnz)) rc = QG_ECAPACITY;
  if (rc == QG_OK && total > 0 &&
      qg_launch_pack_b_split_fill(B_dev, K, N, ldb, K_pad, frag_ptr, cursor, entries, s) != hipSuccess)
    rc = QG_ELAUNCH;
  if (rc != QG_OK) {
    delete h;
    return rc;
  }
  h->nnz = total;
  *out = h;
  return QG_OK;
}

size_t qg_packed_b_nnz(const qg_packed_b* p) { return (p && p->split) ? (size_t)p->nnz : 0; }

size_t qg_gemm_workspace_bytes(int M, const qg_packed_b* Bp) {
  if (!Bp || M <= 0 || Bp->kind != QG_KIND_GEMM) return 0;
  int kernel = QG_KERNEL_AUTO;
  if (resolve_kernel(Bp, M, &kernel) != QG_OK) return 0;
  const int s = auto_ksplit(kernel, M, Bp);
  return s > 1 ? splitk_ws(kernel, M, Bp->N, s).bytes() : 0;
}

size_t qg_gemm_splitk_workspace_bytes(int M, const qg_packed_b* Bp, int kernel, int ksplit) {
  if (!Bp || M <= 0 || Bp->kind != QG_KIND_GEMM || ksplit < 0 || ksplit > kMaxKsplit) return 0;
  if (resolve_kernel(Bp, M, &kernel) != QG_OK) return 0;
  if (kernel == QG_KERNEL_TILE128) {
    const int s = ksplit > 1 ? clamp_ksplit_tile128(Bp, ksplit) : 1;
    return s > 1 ? splitk_ws(kernel, M, Bp->N, s).bytes() : 0;
  }
  if (kernel > QG_KERNEL_SKINNY64) return 0;
  const int s = ksplit == 0 ? auto_ksplit(kernel, M, Bp) : clamp_ksplit(Bp, ksplit);
  return s > 1 ? splitk_ws(kernel, M, Bp->N, s).bytes() : 0;
}

int qg_gemm_splitk_factor(int M, const qg_packed_b* Bp, int kernel, int ksplit) {
  if (!Bp || Bp->kind != QG_KIND_GEMM) return QG_ENULL;
  if (M <= 0 || ksplit < 0 || ksplit > kMaxKsplit) return QG_EINVAL;
  const int rc = resolve_kernel(Bp, M, &kernel);
  if (rc != QG_OK) return rc;
  if (kernel == QG_KERNEL_TILE128) return ksplit > 1 ? clamp_ksplit_tile128(Bp, ksplit) : 1;
  if (kernel > QG_KERNEL_SKINNY64) return 1;
  return ksplit == 0 ? auto_ksplit(kernel, M, Bp) : clamp_ksplit(Bp, ksplit);
}

int qg_gemm_workspace_init(void* workspace_dev, size_t bytes, void* stream) {
  if (bytes == 0) return QG_OK;
  if (!workspace_dev) return QG_ENULL;
  if (!aligned(workspace_dev, 16) || bytes % 4 != 0) return QG_EALIGN;
  const size_t n = bytes / 4;
  const unsigned blocks = (unsigned)((n + 255) / 256 < 2048 ? (n + 255) / 256 : 2048);
  hipLaunchKernelGGL(qg_fill_zero_kernel, dim3(blocks), dim3(256), 0, static_cast<hipStream_t>(stream),
                     static_cast<int32_t*>(workspace_dev), n);
  return hipGetLastError() == hipSuccess ? QG_OK : QG_ELAUNCH;
}

static int gemm_common(const uint8_t* A_dev, int M, int lda, const qg_packed_b* Bp, qg_gemm_args* a) {
  if (!Bp || (!A_dev && M != 0)) return QG_ENULL;  // the data pointers of an empty batch are not referenced
  if (Bp->kind != QG_KIND_GEMM || Bp->version != QG_LAYOUT_VERSION) return QG_EINVAL;
  if (M < 0 || lda < Bp->K) return QG_EINVAL;
  a->A = A_dev;
  a->Bp = Bp->packed;
  a->col_off = Bp->col_off;
  a->bzp = Bp->bzp;
  a->M = M;
  a->N = Bp->N;
  a->K = Bp->K;
  a->kb64 = Bp->K_pad / QG_FRAG_K;
  a->nb16 = Bp->N_pad / QG_FRAG_COLS;
  a->has_bzp = Bp->has_bzp;
  a->sp_ptr = Bp->split ? Bp->frag_ptr : nullptr;
  a->sp_entries = Bp->entries;
  a->sp_total = (int)Bp->nnz;
  a->lda = lda;
  a->a_vec = aligned(A_dev, 16) && (lda % 16 == 0);
  a->ksplit = 1;
  a->ks_per = a->kb64;
  return QG_OK;
}

static int gemm_requant(const uint8_t* A_dev, int M, int lda, const qg_packed_b* Bp, const qg_requant_params* p,
                        uint8_t* C_dev, int ldc, void* workspace_dev, size_t workspace_bytes, bool bytes_known,
                        void* stream, int kernel, int ksplit) {
  qg_gemm_args a = {};
  int rc = gemm_common(A_dev, M, lda, Bp, &a);
  if (rc != QG_OK) return rc;
  rc = resolve_kernel(Bp, M, &kernel);
  if (rc != QG_OK) return rc;
  if (!C_dev && M != 0) return QG_ENULL;
  rc = check_requant(p, Bp->N);
  if (rc != QG_OK) return rc;
  if (ldc < Bp->N) return QG_EINVAL;
  rc = resolve_ksplit(Bp, M, kernel, ksplit, workspace_dev, workspace_bytes, bytes_known, &a);
  if (rc != QG_OK) return rc;
  a.bias = p->bias;
  a.scales = p->scales;
  a.scale_stride = p->n_scales == 1 ? 0 : 1;
  a.a_zp_m128 = p->a_zp - 128;
  a.c_zp = p->c_zp;
  const int lo = p->relu ? p->c_zp : 0;
  a.clamp_lo = (float)(lo - p->c_zp);
  a.clamp_hi = (float)(255 - p->c_zp);
  a.C = C_dev;
  a.ldc = ldc;
  hipStream_t s = static_cast<hipStream_t>(stream);
  // 4-byte stores in the streaming kernels, 16-byte stores in the tiled ones
  a.c_vec = kernel <= QG_KERNEL_SKINNY64 ? (aligned(C_dev, 4) && (ldc % 4 == 0)) : (aligned(C_dev, 16) && (ldc % 16 == 0));
  a.c_wt = (long long)M * Bp->N <= (1 << 18);
  if (M == 0) return QG_OK;  // an empty batch: checked like any other, nothing to enqueue
  const hipError_t e = launch_gemm(a, QG_MODE_REQUANT, kernel, s);
  return e == hipSuccess ? QG_OK : QG_ELAUNCH;
}

int qg_gemm_u8s8_requant(const uint8_t* A_dev, int M, int lda, const qg_packed_b* Bp,
                         const qg_requant_params* p, uint8_t* C_dev, int ldc, void* workspace_dev,
                         void* stream) {
  return gemm_requant(A_dev, M, lda, Bp, p, C_dev, ldc, workspace_dev, 0, false, stream, QG_KERNEL_AUTO, 0);
}

int qg_gemm_u8s8_requant_kernel(const uint8_t* A_dev, int M, int lda, const qg_packed_b* Bp,
                                const qg_requant_params* p, uint8_t* C_dev, int ldc, void* workspace_dev,
                                void* stream, int kernel) {
  return gemm_requant(A_dev, M, lda, Bp, p, C_dev, ldc, workspace_dev, 0, false, stream, kernel, 0);
}

int qg_gemm_u8s8_requant_splitk(const uint8_t* A_dev, int M, int lda, const qg_packed_b* Bp,
                                const qg_requant_params* p, uint8_t* C_dev, int ldc, void* workspace_dev,
                                size_t workspace_bytes, void* stream, int kernel, int ksplit) {
  return gemm_requant(A_dev, M, lda, Bp, p, C_dev, ldc, workspace_dev, workspace_bytes, true, stream, kernel, ksplit);
}

int qg_gemm_u8s8_requant_noalloc(const uint8_t* A_dev, int M, int lda, const qg_packed_b* Bp,
                                 const qg_requant_params* p, uint8_t* C_dev, int ldc, void* stream, int kernel,
                                 int ksplit) {
  if (!Bp) return QG_ENULL;
  if (Bp->kind != QG_KIND_GEMM || Bp->version != QG_LAYOUT_VERSION || M < 0) return QG_EINVAL;
  // the split this call would use with a workspace at hand, and what it needs of the built-in scratch
  const size_t need = M > 0 ? qg_gemm_splitk_workspace_bytes(M, Bp, kernel, ksplit) : 0;
  if (need > QG_NOALLOC_SCRATCH_BYTES) return QG_EWORKSPACE;
  void* scratch = nullptr;
  const int rc = noalloc_scratch(&scratch);
  if (rc != QG_OK) return rc;
  return gemm_requant(A_dev, M, lda, Bp, p, C_dev, ldc, scratch, QG_NOALLOC_SCRATCH_BYTES, true, stream, kernel, ksplit);
}

static int gemm_acc32(const uint8_t* A_dev, int M, int lda, const qg_packed_b* Bp, int32_t* C32_dev, int ldc,
                      int32_t* rowsum_dev, void* workspace_dev, size_t workspace_bytes, bool bytes_known, void* stream,
                      int kernel, int ksplit) {
  qg_gemm_args a = {};
  int rc = gemm_common(A_dev, M, lda, Bp, &a);
  if (rc != QG_OK) return rc;
  rc = resolve_kernel(Bp, M, &kernel);
  if (rc != QG_OK) return rc;
  if (!C32_dev && M != 0) return QG_ENULL;
  if (ldc < Bp->N) return QG_EINVAL;
  rc = resolve_ksplit(Bp, M, kernel, ksplit, workspace_dev, workspace_bytes, bytes_known, &a);
  if (rc != QG_OK) return rc;
  a.C32 = C32_dev;
  a.rowsum_out = rowsum_dev;
  a.ldc = ldc;
  if (M == 0) return QG_OK;
  const hipError_t e = launch_gemm(a, QG_MODE_ACC32, kernel, static_cast<hipStream_t>(stream));
  return e == hipSuccess ? QG_OK : QG_ELAUNCH;
}

int qg_gemm_u8s8_acc32(const uint8_t* A_dev, int M, int lda, const qg_packed_b* Bp, int32_t* C32_dev,
                       int ldc, int32_t* rowsum_dev, void* workspace_dev, void* stream) {
  return gemm_acc32(A_dev, M, lda, Bp, C32_dev, ldc, rowsum_dev, workspace_dev, 0, false, stream, QG_KERNEL_AUTO, 0);
}

int qg_gemm_u8s8_acc32_kernel(const uint8_t* A_dev, int M, int lda, const qg_packed_b* Bp, int32_t* C32_dev,
                              int ldc, int32_t* rowsum_dev, void* workspace_dev, void* stream, int kernel) {
  return gemm_acc32(A_dev, M, lda, Bp, C32_dev, ldc, rowsum_dev, workspace_dev, 0, false, stream, kernel, 0);
}

int qg_gemm_u8s8_acc32_splitk(const uint8_t* A_dev, int M, int lda, const qg_packed_b* Bp, int32_t* C32_dev,
                              int ldc, int32_t* rowsum_dev, void* workspace_dev, size_t workspace_bytes, void* stream,
                              int kernel, int ksplit) {
  return gemm_acc32(A_dev, M, lda, Bp, C32_dev, ldc, rowsum_dev, workspace_dev, workspace_bytes, true, stream, kernel,
                    ksplit);
}

static int check_dequant(const qg_dequant_params* p, int N) {
  if (!p) return QG_ENULL;
  if (!p->scales) return QG_ENULL;
  if (p->a_zp < 0 || p->a_zp > 255) return QG_EINVAL;
  if (p->n_scales != 1 && p->n_scales != N) return QG_EINVAL;
  if (p->relu != 0 && p->relu != 1) return QG_EINVAL;
  return QG_OK;
}

int qg_gemm_u8s8_dequant_f32(const uint8_t* A_dev, int M, int lda, const qg_packed_b* Bp,
                             const qg_dequant_params* p, float* C_dev, int ldc, void* workspace_dev,
                             void* stream, int kernel) {
  qg_gemm_args a = {};
  int rc = gemm_common(A_dev, M, lda, Bp, &a);
  if (rc != QG_OK) return rc;
  rc = resolve_kernel(Bp, M, &kernel);
  if (rc != QG_OK) return rc;
  if (!C_dev && M != 0) return QG_ENULL;
  rc = check_dequant(p, Bp->N);
  if (rc != QG_OK) return rc;
  if (ldc < Bp->N) return QG_EINVAL;
  if (!aligned(C_dev, 4)) return QG_EALIGN;
  rc = resolve_ksplit(Bp, M, kernel, 0, workspace_dev, 0, false, &a);
  if (rc != QG_OK) return rc;
  a.bias = p->bias;
  a.scales = p->scales;
  a.scale_stride = p->n_scales == 1 ? 0 : 1;
  a.a_zp_m128 = p->a_zp - 128;
  a.relu_lo = p->relu ? 0.0f : -INFINITY;
  a.Cf = C_dev;
  a.ldc = ldc;
  a.c_vec = aligned(C_dev, 16) && (ldc % 4 == 0);
  if (M == 0) return QG_OK;
  const hipError_t e = launch_gemm(a, QG_MODE_DEQUANT, kernel, static_cast<hipStream_t>(stream));
  return e == hipSuccess ? QG_OK : QG_ELAUNCH;
}

int qg_quantize_a_f32(const float* A_dev, int M, int K, int lda, float inv_scale, int a_zp, uint8_t* Aq_dev,
                      int ldq, void* stream) {
  if ((!A_dev || !Aq_dev) && M != 0) return QG_ENULL;
  if (M < 0 || K <= 0 || lda < K || ldq < K) return QG_EINVAL;
  if (a_zp < 0 || a_zp > 255 || !(inv_scale > 0.0f) || !isfinite(inv_scale)) return QG_EINVAL;
  if (!aligned(A_dev, 4)) return QG_EALIGN;
  if (M == 0) return QG_OK;
  const hipError_t e =
      qg_launch_quantize_a(A_dev, M, K, lda, inv_scale, a_zp, Aq_dev, ldq, static_cast<hipStream_t>(stream));
  return e == hipSuccess ? QG_OK : QG_ELAUNCH;
}

// row pitch of the quantized copy in the workspace: whole 16-byte chunks, so the copy takes the vector paths
static int f32_ldq(const qg_packed_b* Bp) { return qg_round_up(Bp->K, 16); }

size_t qg_gemm_f32_workspace_bytes(int M, const qg_packed_b* Bp) {
  if (!Bp || M <= 0 || Bp->kind != QG_KIND_GEMM) return 0;
  return (size_t)M * (size_t)f32_ldq(Bp);  // what a tiled kernel needs; a streaming kernel needs none
}

static int quantize_into_workspace(const float* A_dev, int M, int lda, float a_inv_scale, const qg_packed_b* Bp,
                                   int a_zp, void* workspace_dev, void* stream) {
  if (!Bp || (!A_dev && M != 0)) return QG_ENULL;
  if (Bp->kind != QG_KIND_GEMM || Bp->version != QG_LAYOUT_VERSION) return QG_EINVAL;
  if (M == 0)  // an empty batch needs no workspace; the remaining arguments are still checked
    return (lda < Bp->K || a_zp < 0 || a_zp > 255 || !(a_inv_scale > 0.0f) || !isfinite(a_inv_scale)) ? QG_EINVAL : QG_OK;
  if (!workspace_dev) return QG_EWORKSPACE;
  if (!aligned(workspace_dev, 16)) return QG_EALIGN;
  return qg_quantize_a_f32(A_dev, M, Bp->K, lda, a_inv_scale, a_zp, static_cast<uint8_t*>(workspace_dev),
                           f32_ldq(Bp), stream);
}

// fp32 activations on a streaming kernel for a caller without a workspace: ONE launch -- the kernel quantizes the block it stages
// (Appendix B: any packing routine for A; row offsets come from the staged block in the same pass).  Fills the
// common fields of `a`; returns QG_OK with *fused = false when the kernel in use is a tiled one.
static int f32_fused_common(const float* A_dev, int M, int lda, float a_inv_scale, int a_zp, const qg_packed_b* Bp,
                            int kernel, const void* workspace_dev, qg_gemm_args* a, bool* fused) {
  *fused = false;
  // With a workspace at hand the separate quantization pass is the faster form even here (every 16-column
  // workgroup of a streaming kernel would convert all of A again: 16 x 4096 x 4096 7.8 us fused, 5.8 us in two
  // launches), so the one-launch form serves the caller that has none.
  if (kernel > QG_KERNEL_SKINNY64 || Bp->split || workspace_dev != nullptr) return QG_OK;
  if (!A_dev && M != 0) return QG_ENULL;
  if (lda < Bp->K || a_zp < 0 || a_zp > 255 || !(a_inv_scale > 0.0f) || !isfinite(a_inv_scale)) return QG_EINVAL;
  if (!aligned(A_dev, 4)) return QG_EALIGN;
  int rc = gemm_common(reinterpret_cast<const uint8_t*>(A_dev), M, lda, Bp, a);
  if (rc != QG_OK) return rc;
  a->a_vec = aligned(A_dev, 16) && (lda % 4 == 0);  // rows of floats that 16-byte loads may take
  a->q_inv = a_inv_scale;
  a->q_lo = (float)(0 - a_zp);
  a->q_hi = (float)(255 - a_zp);
  a->q_zp = (float)a_zp;
  *fused = true;
  return QG_OK;
}

int qg_gemm_f32s8_requant(const float* A_dev, int M, int lda, float a_inv_scale, const qg_packed_b* Bp,
                          const qg_requant_params* p, uint8_t* C_dev, int ldc, void* workspace_dev,
                          void* stream, int kernel) {
  // every check of the second stage first, so that an error leaves nothing enqueued
  if (!Bp || !p || (!C_dev && M != 0)) return QG_ENULL;
  if (Bp->kind != QG_KIND_GEMM || Bp->version != QG_LAYOUT_VERSION) return QG_EINVAL;
  int rc = check_requant(p, Bp->N);
  if (rc != QG_OK) return rc;
  if (M < 0 || ldc < Bp->N) return QG_EINVAL;
  rc = resolve_kernel(Bp, M, &kernel);
  if (rc != QG_OK) return rc;
  {
    qg_gemm_args a = {};
    bool fused = false;
    rc = f32_fused_common(A_dev, M, lda, a_inv_scale, p->a_zp, Bp, kernel, workspace_dev, &a, &fused);
    if (rc != QG_OK) return rc;
    if (fused) {
      a.bias = p->bias;
      a.scales = p->scales;
      a.scale_stride = p->n_scales == 1 ? 0 : 1;
      a.a_zp_m128 = p->a_zp - 128;
      a.c_zp = p->c_zp;
      const int lo = p->relu ? p->c_zp : 0;
      a.clamp_lo = (float)(lo - p->c_zp);
      a.clamp_hi = (float)(255 - p->c_zp);
      a.C = C_dev;
      a.ldc = ldc;
      a.c_vec = aligned(C_dev, 4) && (ldc % 4 == 0);
      a.c_wt = (long long)M * Bp->N <= (1 << 18);
      if (M == 0) return QG_OK;
      const hipError_t e = qg_launch_gemm_skinny_f32(a, QG_MODE_REQUANT, kernel, static_cast<hipStream_t>(stream));
      return e == hipSuccess ? QG_OK : QG_ELAUNCH;
    }
  }
  rc = quantize_into_workspace(A_dev, M, lda, a_inv_scale, Bp, p->a_zp, workspace_dev, stream);
  if (rc != QG_OK || M == 0) return rc;
  return qg_gemm_u8s8_requant_kernel(static_cast<const uint8_t*>(workspace_dev), M, f32_ldq(Bp), Bp, p, C_dev, ldc,
                                     nullptr, stream, kernel);
}

int qg_gemm_f32s8_dequant_f32(const float* A_dev, int M, int lda, float a_inv_scale, const qg_packed_b* Bp,
                              const qg_dequant_params* p, float* C_dev, int ldc, void* workspace_dev,
                              void* stream, int kernel) {
  if (!Bp || !p || (!C_dev && M != 0)) return QG_ENULL;
  if (Bp->kind != QG_KIND_GEMM || Bp->version != QG_LAYOUT_VERSION) return QG_EINVAL;
  int rc = check_dequant(p, Bp->N);
  if (rc != QG_OK) return rc;
  if (M < 0 || ldc < Bp->N) return QG_EINVAL;
  rc = resolve_kernel(Bp, M, &kernel);
  if (rc != QG_OK) return rc;
  if (!aligned(C_dev, 4)) return QG_EALIGN;
  {
    qg_gemm_args a = {};
    bool fused = false;
    rc = f32_fused_common(A_dev, M, lda, a_inv_scale, p->a_zp, Bp, kernel, workspace_dev, &a, &fused);
    if (rc != QG_OK) return rc;
    if (fused) {
      a.bias = p->bias;
      a.scales = p->scales;
      a.scale_stride = p->n_scales == 1 ? 0 : 1;
      a.a_zp_m128 = p->a_zp - 128;
      a.relu_lo = p->relu ? 0.0f : -INFINITY;
      a.Cf = C_dev;
      a.ldc = ldc;
      a.c_vec = aligned(C_dev, 16) && (ldc % 4 == 0);
      if (M == 0) return QG_OK;
      const hipError_t e = qg_launch_gemm_skinny_f32(a, QG_MODE_DEQUANT, kernel, static_cast<hipStream_t>(stream));
      return e == hipSuccess ? QG_OK : QG_ELAUNCH;
    }
  }
  rc = quantize_into_workspace(A_dev, M, lda, a_inv_scale, Bp, p->a_zp, workspace_dev, stream);
  if (rc != QG_OK || M == 0) return rc;
  return qg_gemm_u8s8_dequant_f32(static_cast<const uint8_t*>(workspace_dev), M, f32_ldq(Bp), Bp, p, C_dev, ldc,
                                  nullptr, stream, kernel);
}

namespace {
// One convolution as a GEMM with the im2col folded into the requests: Cin channels starting at `in` of pixels that
// are `pix` bytes apart (a whole image, or the channel slice of one group), weights as a packed K x N matrix with
// K = R*S*Cin; output channel j goes to out[pixel * ldc + j]; bias and scales (when per channel) start at entry ch0.
int launch_conv_gemm(const uint8_t* in, int in_bytes, int Nb, int H, int W, int Cin, int pix, int R, int S, int pad, int stride,
                     int Ho, int Wo, const int8_t* packed, const int32_t* col_off, const int32_t* bzp, int K, int K_pad, int N,
                     int N_pad, int has_bzp, const qg_requant_params* p, int ch0, uint8_t* out, int ldc, int kernel,
                     hipStream_t stream) {
  qg_gemm_args a = {};
  a.A = in;
  a.Bp = packed;
  a.col_off = col_off;
  a.bzp = bzp;
  a.M = Nb * Ho * Wo;
  a.N = N;
  a.K = K;
  a.kb64 = K_pad / QG_FRAG_K;
  a.nb16 = N_pad / QG_FRAG_COLS;
  a.has_bzp = has_bzp;
  a.lda = 0;
  a.bias = p->bias ? p->bias + ch0 : nullptr;
  a.scales = p->n_scales == 1 ? p->scales : p->scales + ch0;
  a.scale_stride = p->n_scales == 1 ? 0 : 1;
  a.a_zp_m128 = p->a_zp - 128;
  a.c_zp = p->c_zp;
  const int lo = p->relu ? p->c_zp : 0;
  a.clamp_lo = (float)(lo - p->c_zp);
  a.clamp_hi = (float)(255 - p->c_zp);
  a.C = out;
  a.ldc = ldc;
  a.c_vec = aligned(out, 16) && (ldc % 16 == 0);
  a.cv_H = H;
  a.cv_W = W;
  a.cv_Cin = Cin;
  a.cv_pix = pix;
  a.cv_Ho = Ho;
  a.cv_Wo = Wo;
  a.cv_R = R;
  a.cv_S = S;
  a.cv_stride = stride;
  a.cv_pad = pad;
  a.cv_azp = p->a_zp;
  a.cv_in_bytes = in_bytes;
  // the tiled kernels, chosen by the same cost formula as a GEMM's; few pixels and a long K go to the 16-row streaming
  // kernel where it applies (whole 64-channel slices, at most 32 taps), priced with the streaming formula and the
  // constants measured for the convolution's requests
  const bool stream_ok = Cin % QG_FRAG_K == 0 && R * S <= 32;
  if (kernel == QG_KERNEL_AUTO) {
    double best_us = 1e300;
    for (const tile_cost& c : k_conv_cost) {
      const double us = tile_estimate(c, a.M, a.N, a.K);
      if (us < best_us) best_us = us, kernel = c.kernel;
    }
    for (const tile_cost& c : k_conv_patch_cost) {
      const int per_cu = qg_conv_patch_per_cu(a, c.kernel - QG_KERNEL_PATCH64X128);
      if (per_cu == 0) continue;
      double us = tile_estimate(c, a.M, a.N, a.K);
      // A wide patch leaves room for few workgroups per CU: what does not run side by side runs one after the
      // other, each pass at the pace of a workgroup alone.
      const double wgs = (double)ceil_div(a.M, c.bm) * (double)ceil_div(a.N, c.bn);
      const double passes = ceil(wgs / (256.0 * per_cu));
      us = fmax(us, 2.5 + passes * (c.fix + ceil_div(a.K, 64) * c.lat - 2.5));
      if (us < best_us) best_us = us, kernel = c.kernel;
    }
    if (stream_ok)
      for (const stream_cost& c : k_conv_stream_cost) {
        const double us = stream_estimate(c, a.M, a.N, a.K, false);
        if (ceil_div(a.M, c.rows) <= 65535 && us < best_us) best_us = us, kernel = c.kernel;
      }
  }
  if (kernel >= QG_KERNEL_PATCH64X128) {
    const int form = kernel - QG_KERNEL_PATCH64X128;
    if (!qg_conv_patch_applies(a, form)) return QG_EUNSUPPORTED;
    return qg_launch_conv_patch(a, form, stream) == hipSuccess ? QG_OK : QG_ELAUNCH;
  }
  if (kernel <= QG_KERNEL_SKINNY64) {
    if (!stream_ok) return QG_EUNSUPPORTED;
    a.ksplit = 1;
    a.ks_per = a.kb64;
    a.a_vec = 1;
    a.c_vec = aligned(out, 4) && (ldc % 4 == 0);
    a.c_wt = (long long)a.M * N <= (1 << 18);
    const hipError_t e = qg_launch_conv_skinny(a, kernel, stream);
    return e == hipSuccess ? QG_OK : QG_ELAUNCH;
  }
  const hipError_t e = qg_launch_conv_dense(a, kernel, stream);
  return e == hipSuccess ? QG_OK : QG_ELAUNCH;
}
}  // namespace

int qg_conv_dense_u8s8_requant(const uint8_t* in_nhwc, int Nb, int H, int W, int Cin, int R, int S, int pad,
                               int stride, const qg_packed_b* Wp, const qg_requant_params* p, uint8_t* out_nhwc,
                               void* stream, int kernel) {
  if (!Wp || ((!in_nhwc || !out_nhwc) && Nb != 0)) return QG_ENULL;
  if (Wp->kind != QG_KIND_GEMM || Wp->version != QG_LAYOUT_VERSION) return QG_EINVAL;
  if (kernel < QG_KERNEL_AUTO || kernel > QG_KERNEL_CONV_LAST) return QG_EINVAL;
  if (kernel == QG_KERNEL_TILE256) return QG_EUNSUPPORTED;
  if (Nb < 0 || H <= 0 || W <= 0 || Cin <= 0 || R <= 0 || S <= 0 || pad < 0 || stride <= 0) return QG_EINVAL;
  if ((long long)R * S * Cin != Wp->K) return QG_EINVAL;
  int rc = check_requant(p, Wp->N);
  if (rc != QG_OK) return rc;
  if (H + 2 * pad < R || W + 2 * pad < S) return QG_EINVAL;
  const int Ho = (H + 2 * pad - R) / stride + 1, Wo = (W + 2 * pad - S) / stride + 1;
  if (Wp->split) return QG_EUNSUPPORTED;
  if (Cin % 16 != 0 || !aligned(in_nhwc, 16)) {
    // no staged kernel takes these extents: the byte-gathering kernel, under the automatic choice only
    if (kernel != QG_KERNEL_AUTO) return QG_EUNSUPPORTED;
    if ((uint64_t)Nb * H * W * Cin >= (1ull << 31) || (uint64_t)Nb * Ho * Wo * Wp->N >= (1ull << 31)) return QG_EUNSUPPORTED;
    qg_conv_args c = {};
    c.in = in_nhwc;
    c.Bp = Wp->packed;
    c.nb16 = Wp->N_pad / QG_FRAG_COLS;
    c.col_off = Wp->col_off;
    c.bzp = Wp->bzp;
    c.bias = p->bias;
    c.scales = p->scales;
    c.out = out_nhwc;
    c.Nb = Nb;
    c.H = H;
    c.W = W;
    c.C = Cin;
    c.Ho = Ho;
    c.Wo = Wo;
    c.Cout = Wp->N;
    c.G = 1;
    c.Cg = Cin;
    c.Og = Wp->N;
    c.R = R;
    c.S = S;
    c.pad = pad;
    c.stride = stride;
    c.scale_stride = p->n_scales == 1 ? 0 : 1;
    c.a_zp = p->a_zp;
    c.c_zp = p->c_zp;
    const int lo = p->relu ? p->c_zp : 0;
    c.clamp_lo = (float)(lo - p->c_zp);
    c.clamp_hi = (float)(255 - p->c_zp);
    c.has_bzp = Wp->has_bzp;
    if (Nb == 0) return QG_OK;
    return qg_launch_conv_dense_plain(c, static_cast<hipStream_t>(stream)) == hipSuccess ? QG_OK : QG_ELAUNCH;
  }
  // 32-bit byte offsets into the image (tap offsets included) and 32-bit pixel counts
  if ((uint64_t)Nb * H * W * Cin >= (1ull << 30) || (uint64_t)Nb * Ho * Wo >= (1ull << 31) / 4) return QG_EUNSUPPORTED;
  // A 1 x 1 filter with unit stride and no padding is the plain GEMM over the pixel rows (lda = Cin): it takes
  // the GEMM's own kernels and choice, hand-scheduled loops included; the bytes are the same either way.
  if (R == 1 && S == 1 && pad == 0 && stride == 1) {
    if (kernel > QG_KERNEL_LAST) return QG_EUNSUPPORTED;  // the patch kernels have nothing to keep for a single tap
    return qg_gemm_u8s8_requant_kernel(in_nhwc, Nb * H * W, Cin, Wp, p, out_nhwc, Wp->N, nullptr, stream, kernel);
  }
  if (Nb == 0) return QG_OK;  // an empty batch
  return launch_conv_gemm(in_nhwc, Nb * H * W * Cin, Nb, H, W, Cin, Cin, R, S, pad, stride, Ho, Wo, Wp->packed, Wp->col_off,
                          Wp->bzp, Wp->K, Wp->K_pad, Wp->N, Wp->N_pad, Wp->has_bzp, p, 0, out_nhwc, Wp->N, kernel,
                          static_cast<hipStream_t>(stream));
}

namespace {
// the groups of 4 -> 4 channels with a 1 x 1 or 3 x 3 filter have a layout (and kernels) of their own
bool conv_is_4to4(int G, int R, int S, int Cg, int Og) {
  return Cg == 4 && Og == 4 && ((R == 1 && S == 1) || (R == 3 && S == 3)) && G <= 256;
}
// log2(Cg) when the block-diagonal matrix-core fragments exist for a general group shape (square groups of 1 -- a
// depthwise convolution --, 2, 8, 16 or 32 channels -- or of 4 in more than 256 groups --, 1 x 1 or 3 x 3, whole
// 32-channel blocks), else -1
int conv_mfma_lcg(int G, int R, int S, int Cg, int Og) {
  if (Cg != Og || !((R == 1 && S == 1) || (R == 3 && S == 3)) || (G * Cg) % 32 != 0) return -1;
  return Cg == 1 ? 0 : Cg == 2 ? 1 : Cg == 4 ? 2 : Cg == 8 ? 3 : Cg == 16 ? 4 : Cg == 32 ? 5 : -1;
}
// groups of a multiple of 16 channels without block-diagonal tiles: each group is a dense convolution of its own
// channel slice (one launch per group), with its weights packed as a GEMM matrix
bool conv_is_wide(int G, int R, int S, int Cg, int Og) {
  return !conv_is_4to4(G, R, S, Cg, Og) && conv_mfma_lcg(G, R, S, Cg, Og) < 0 && Cg % 16 == 0 && G <= 64;
}
}  // namespace

static int conv_sizes_without_gemms(int G, int R, int S, int Cg, int Og, size_t* packed_bytes, size_t* col_offsets_bytes);

int qg_pack_conv_w_sizes(int G, int R, int S, int Cg, int Og, size_t* packed_bytes,
                         size_t* col_offsets_bytes) {
  if (!packed_bytes || !col_offsets_bytes) return QG_ENULL;
  if (G <= 0 || R <= 0 || S <= 0 || Cg <= 0 || Og <= 0) return QG_EINVAL;
  if ((long long)R * S * Cg > QG_MAX_K || (long long)G * Cg >= (1 << 24) || (long long)G * Og >= (1 << 24)) return QG_EINVAL;
  const int rc = conv_sizes_without_gemms(G, R, S, Cg, Og, packed_bytes, col_offsets_bytes);
  if (rc != QG_OK) return rc;
  if (conv_is_wide(G, R, S, Cg, Og)) {
    const size_t kp = (size_t)qg_round_up(R * S * Cg, QG_KPAD), np = (size_t)qg_round_up(Og, QG_NPAD);
    *packed_bytes += (size_t)G * kp * np;
    *col_offsets_bytes += (size_t)G * 2 * np * sizeof(int32_t);
  }
  return QG_OK;
}

// the layouts every group shape has: the general (or 4 -> 4) weights, the block-diagonal tiles, the folded offsets
static int conv_sizes_without_gemms(int G, int R, int S, int Cg, int Og, size_t* packed_bytes, size_t* col_offsets_bytes) {
  if (conv_is_4to4(G, R, S, Cg, Og)) {
    // dot4 layout, then (when C = 4 G is a multiple of 32) the matrix-core fragments
    *packed_bytes = (size_t)qg_round_up(G * R * S * Cg * Og, 256) +
                    ((G % 8 == 0) ? (size_t)(G / 8) * R * S * QG_FRAG_BYTES : 0);
  } else {
    // general layout [Cout][R*S][Cg rounded up to 4], then the matrix-core fragments where they exist
    const size_t any = (size_t)G * Og * R * S * (size_t)qg_round_up(Cg, 4);
    if (any >= (1ull << 31)) return QG_EUNSUPPORTED;
    *packed_bytes = (any + 255) / 256 * 256 +
                    (conv_mfma_lcg(G, R, S, Cg, Og) >= 0 ? (size_t)(G * Cg / 32) * R * S * QG_FRAG_BYTES : 0);
  }
  *col_offsets_bytes = (size_t)qg_round_up(2 * G * Og * (int)sizeof(int32_t), 256);
  return QG_OK;
}

int qg_pack_conv_w(const int8_t* W_dev, int G, int R, int S, int Cg, int Og, const int32_t* b_zp_host,
                   int n_b_zp, void* packed_dev, int32_t* col_offsets_dev, void* stream,
                   qg_packed_b** out) {
  if (!W_dev || !b_zp_host || !packed_dev || !col_offsets_dev || !out) return QG_ENULL;
  size_t pb, cb;
  int rc = qg_pack_conv_w_sizes(G, R, S, Cg, Og, &pb, &cb);
  if (rc != QG_OK) return rc;
  const int Cout = G * Og;
  if (n_b_zp != 1 && n_b_zp != Cout) return QG_EINVAL;
  if (!aligned(packed_dev, 256) || !aligned(col_offsets_dev, 256)) return QG_EALIGN;
  hipStream_t s = static_cast<hipStream_t>(stream);
  qg_packed_b* h = new (std::nothrow) qg_packed_b();
  if (!h) return QG_ENOMEM;
  h->kind = QG_KIND_CONV;
  h->version = QG_LAYOUT_VERSION;
  h->K = R * S * Cg;
  h->N = Cout;
  h->K_pad = h->K;
  h->N_pad = Cout;
  h->n_b_zp = n_b_zp;
  h->packed = static_cast<const int8_t*>(packed_dev);
  h->col_off = col_offsets_dev;
  h->bzp = col_offsets_dev + Cout;
  h->G = G;
  h->R = R;
  h->S = S;
  h->Cg = Cg;
  h->Og = Og;
  h->split = 0;
  h->frag_ptr = h->entries = nullptr;
  h->nnz = 0;
  const bool four = conv_is_4to4(G, R, S, Cg, Og);
  const int lcg = four ? 2 : conv_mfma_lcg(G, R, S, Cg, Og);
  int8_t* frags = nullptr;
  if (four)
    frags = (G % 8 == 0) ? static_cast<int8_t*>(packed_dev) + qg_round_up(G * R * S * Cg * Og, 256) : nullptr;
  else if (lcg >= 0)
    frags = static_cast<int8_t*>(packed_dev) + ((size_t)Cout * R * S * (size_t)qg_round_up(Cg, 4) + 255) / 256 * 256;
  h->conv_frags = frags;
  h->conv_any = four ? nullptr : static_cast<const int8_t*>(packed_dev);
  rc = upload_bzp(b_zp_host, n_b_zp, Cout, Cout, col_offsets_dev + Cout, s, &h->has_bzp);
  if (rc != QG_OK) {
    delete h;
    return rc;
  }
  const hipError_t e = four ? qg_launch_pack_conv_w(W_dev, G, R * S, static_cast<int8_t*>(packed_dev), col_offsets_dev,
                                                    col_offsets_dev + Cout, frags, s)
                            : qg_launch_pack_conv_w_any(W_dev, G, R * S, Cg, Og, static_cast<int8_t*>(packed_dev),
                                                        col_offsets_dev, col_offsets_dev + Cout, frags, lcg, s);
  if (e != hipSuccess) {
    delete h;
    return QG_ELAUNCH;
  }
  h->conv_gemm = nullptr;
  h->conv_gemm_off = nullptr;
  if (conv_is_wide(G, R, S, Cg, Og)) {
    const int K = R * S * Cg, kp = qg_round_up(K, QG_KPAD), np = qg_round_up(Og, QG_NPAD);
    size_t pb0, cb0;
    conv_sizes_without_gemms(G, R, S, Cg, Og, &pb0, &cb0);
    int8_t* gp = static_cast<int8_t*>(packed_dev) + pb0;
    int32_t* go = col_offsets_dev + cb0 / sizeof(int32_t);
    for (int g = 0; g < G; ++g) {
      int unused;
      rc = upload_bzp(n_b_zp == 1 ? b_zp_host : b_zp_host + (size_t)g * Og, n_b_zp == 1 ? 1 : Og, Og, np,
                      go + (size_t)g * 2 * np + np, s, &unused);
      if (rc == QG_OK && qg_launch_pack_b(W_dev + (size_t)g * K * Og, K, Og, Og, 0, kp, np, gp + (size_t)g * kp * np,
                                          go + (size_t)g * 2 * np, go + (size_t)g * 2 * np + np, s) != hipSuccess)
        rc = QG_ELAUNCH;
      if (rc != QG_OK) {
        delete h;
        return rc;
      }
    }
    h->conv_gemm = gp;
    h->conv_gemm_off = go;
    h->conv_gemm_kpad = kp;
    h->conv_gemm_npad = np;
  }
  *out = h;
  return QG_OK;
}

int qg_conv_groupwise_u8s8_requant(const uint8_t* in_nhwc, int Nb, int H, int W, int C, int pad,
                                   int stride, const qg_packed_b* Wp, const qg_requant_params* p,
                                   uint8_t* out_nhwc, void* stream) {
  if (!Wp || ((!in_nhwc || !out_nhwc) && Nb != 0)) return QG_ENULL;
  if (Wp->kind != QG_KIND_CONV || Wp->version != QG_LAYOUT_VERSION) return QG_EINVAL;
  if (Nb < 0 || H <= 0 || W <= 0 || C <= 0 || pad < 0 || stride <= 0) return QG_EINVAL;
  if (C != Wp->G * Wp->Cg) return QG_EINVAL;
  int rc = check_requant(p, Wp->N);
  if (rc != QG_OK) return rc;
  const int Ho = (H + 2 * pad - Wp->R) / stride + 1;
  const int Wo = (W + 2 * pad - Wp->S) / stride + 1;
  if (H + 2 * pad < Wp->R || W + 2 * pad < Wp->S || Ho <= 0 || Wo <= 0) return QG_EINVAL;
  if (Wp->conv_any == nullptr && (!aligned(in_nhwc, 4) || !aligned(out_nhwc, 4))) return QG_EALIGN;
  if ((uint64_t)Nb * H * W * C >= (1ull << 31) || (uint64_t)Nb * Ho * Wo * Wp->N >= (1ull << 31)) return QG_EUNSUPPORTED;
  qg_conv_args a = {};
  a.in = in_nhwc;
  a.Wp = Wp->packed;
  a.Wfrag = Wp->conv_frags;
  a.col_off = Wp->col_off;
  a.bzp = Wp->bzp;
  a.bias = p->bias;
  a.scales = p->scales;
  a.out = out_nhwc;
  a.Nb = Nb;
  a.H = H;
  a.W = W;
  a.C = C;
  a.Ho = Ho;
  a.Wo = Wo;
  a.Cout = Wp->N;
  a.G = Wp->G;
  a.Wany = Wp->conv_any;
  a.Cg = Wp->Cg;
  a.Og = Wp->Og;
  a.R = Wp->R;
  a.S = Wp->S;
  a.lcg = Wp->conv_any == nullptr ? 2 : (Wp->conv_frags != nullptr ? conv_mfma_lcg(Wp->G, Wp->R, Wp->S, Wp->Cg, Wp->Og) : 0);
  a.pad = pad;
  a.stride = stride;
  a.scale_stride = p->n_scales == 1 ? 0 : 1;
  a.a_zp = p->a_zp;
  a.c_zp = p->c_zp;
  const int lo = p->relu ? p->c_zp : 0;
  a.clamp_lo = (float)(lo - p->c_zp);
  a.clamp_hi = (float)(255 - p->c_zp);
  a.has_bzp = Wp->has_bzp;
  if (Nb == 0) return QG_OK;  // an empty batch
  // wide groups: every group is a dense convolution of its own channel slice (16-byte chunks need aligned pixels)
  if (Wp->conv_gemm != nullptr && C % 16 == 0 && aligned(in_nhwc, 16) && (uint64_t)Nb * H * W * C < (1ull << 30) &&
      (uint64_t)Nb * Ho * Wo < (1ull << 31) / 4) {
    const size_t kp = (size_t)Wp->conv_gemm_kpad, np = (size_t)Wp->conv_gemm_npad;
    for (int g = 0; g < Wp->G; ++g) {
      const int32_t* off = Wp->conv_gemm_off + (size_t)g * 2 * np;
      rc = launch_conv_gemm(in_nhwc + (size_t)g * Wp->Cg, Nb * H * W * C - g * Wp->Cg, Nb, H, W, Wp->Cg, C, Wp->R, Wp->S, pad,
                            stride, Ho, Wo, Wp->conv_gemm + (size_t)g * kp * np, off, off + np, Wp->K, (int)kp, Wp->Og, (int)np,
                            Wp->has_bzp, p, g * Wp->Og, out_nhwc + (size_t)g * Wp->Og, Wp->N, QG_KERNEL_AUTO,
                            static_cast<hipStream_t>(stream));
      if (rc != QG_OK) return rc;
    }
    return QG_OK;
  }
  hipError_t e = qg_launch_conv_group(a, Wp->R * Wp->S, static_cast<hipStream_t>(stream));
  return e == hipSuccess ? QG_OK : QG_ELAUNCH;
}

}  // extern "C"
