// Small-batch quantized GEMM (row blocks of 16, 32 or 64): the bandwidth-bound case the paper
// stresses ("M is sometimes very small", Appendix C; int32 accumulation for the
// bandwidth-bound shapes, Sec. 4).  Every byte of B is used exactly once, so B
// fragments go STRAIGHT from HBM into MFMA operand registers: the packed layout
// makes each wave load one contiguous KiB (16 B per lane).  LDS is used only to
// combine the partial sums of the 16 waves that split K.
//
// One workgroup owns one 16-column fragment column of B over all of K; wave w
// takes a contiguous range of 64-deep k blocks and issues a whole batch of loads
// before the first MFMA so that the whole weight matrix is in flight at once; the next
// batch's weights are requested before the wave waits for the current batch's activations.
// A (the row block, at most 64 rows) comes from L2, is row-summed on its raw bytes (v_sad_u8) and
// shifted to int8 (xor 0x80) on the way, as in the large kernel.  Each wave stages its own K-slice of
// the row block, batch by batch, through a private 4 or 8 KiB of LDS with global_load_lds: a request
// reads whole 128- or 256-byte row segments (MFMA operand order would touch 16 rows x 64 B per load,
// half-used lines, which cost more than the weight stream itself at 64 rows), and the fragments are then
// fetched from LDS in operand order.  Unaligned A, ragged K and partial batches take the same route
// with the lanes copying the bytes themselves.
//
// Outlier-split weights (Sec. 2.2, B = B' + B_sparse): B' streams in at 4 bits per weight -- half the bytes
// of the shape this kernel exists for -- and is widened to int8 operand dwords with two bit operations
// per eight weights; the sparse term A B_sparse is added while the block of C is still on chip (the paper
// fuses it into the output processing while the block is cache-resident): a wave that has just consumed a
// batch of k blocks adds the products of that batch's entries, one (row, entry) pair per lane, into an LDS
// tile that joins the K-split reduction.  The A bytes come from the wave's staged LDS copy of the batch
// when there is one (a gather from memory would cost one L1 line per lane).
//
// M larger than the row block is covered by the second grid dimension: every row block streams
// B again (from L2 / the memory-side cache when the blocks run close together), which beats the
// tiled kernel only while there are too few tiles to occupy the chip.
//
// K split ACROSS workgroups (third grid dimension, p.ksplit slices of K; the role of the paper's caller-provided
// C_buffer, Appendix A): a shape with few fragment columns and a long K would leave most of the chip idle, so the
// slices of one fragment column run as separate workgroups.  Each adds up its own waves through LDS as usual; the
// wave that would run the output pipeline instead writes its int32 partial tile and row offsets into its slot of
// the caller's workspace with device-coherent (write-through) stores, waits for their acknowledgement and takes
// a ticket from a counter; the wave that draws the last ticket reads the other slices' slots, adds them in slice
// order -- integer sums, so every split factor gives the same bytes -- runs the output pipeline and puts the
// counter back to zero for the next call.  No fence instruction is used: a release fence at device scope writes
// back the whole L2 of the XCD, which was measured at 20 - 80 us per workgroup.
#include "qg_internal.h"
#include <type_traits>

namespace {

typedef int v4i __attribute__((ext_vector_type(4)));

// ints of one (K slice, row block of 16) slot of the cross-workgroup workspace: 64 lanes x 4 partial sums, 16 row sums
constexpr int SLOT_INTS = 64 * 4 + 16;

// One activation request: 16 bytes per lane from a_base + voff (a_base wave-uniform, in scalar registers; voff a
// per-lane byte offset) into LDS at lds + lane * 16 (lds wave-uniform).  Written out instead of the compiler's
// builtin because that one forms the 64-bit address in a temporary vector register, and the register it picked
// was the destination of a weight load still in flight: the request then waited for weights from HBM before it
// could even be issued.  Here the address registers are never the target of a load.
__device__ __forceinline__ void request_a(const uint8_t* a_base, unsigned voff, unsigned lds) {
  asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %1, %2" ::"s"(lds), "v"(voff), "s"(a_base) : "memory");
}

// The same with a 64-bit per-lane address (the convolution's requests go to the image or to a table row).
__device__ __forceinline__ void request_a64(const uint8_t* addr, unsigned lds) {
  asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %1, off" ::"s"(lds), "v"(addr) : "memory");
}

// Explicit wait: at most LEFT vector-memory operations of this wave still in flight (they complete in order).
// The compiler's own bookkeeping does not see the activation requests (they are issued by request_a), so the
// waits that order LDS reads behind them are written out.
template <int LEFT>
__device__ __forceinline__ void wait_vm() {
  asm volatile("s_waitcnt vmcnt(%0)" ::"n"(LEFT) : "memory");
}

// ANYALIGN: rows of A that are not 16-byte aligned.  The requests and vector loads take any address; the variant
// exists so that the aligned one keeps its code (and its timing) to the instruction.
// SIMPLE: the straight-line variant for the common case the host has checked -- 8-bit weights, 16-byte aligned
// rows, K a whole number of 64-deep blocks and every wave of every slice a whole number of batches: no partial
// batch, no lane-copied staging, every request issued by hand in a known order.
// CPW (straight-line variant only): fragment columns per wave.  With two, a workgroup of four waves covers a whole
// 32-column super-block: every activation fragment feeds two MFMAs, the workgroup stages half as many activation
// bytes per weight byte, and few fat waves (16 weight loads in flight each) keep a large matrix streaming at the
// rate of a plain read -- the shape for weights of tens of MiB, where the 16-wave form pays for its A traffic.
// AF32: the activations are fp32 and are quantized to uint8 while they are staged (Appendix B: any packing routine for
// A; Eq. (1) solved for the quantized value, the fixed sequence of the stand-alone quantization pass): the lanes load
// 16 floats per 16-byte chunk of the staged block, convert and write the chunk to LDS, where row offsets and
// fragments are taken from it as from any uint8 block.  A then points to floats and lda counts floats.
// ACONV: the rows are the output pixels of a dense convolution and A is its NHWC image (the paper names convolution in
// Sec. 1; im2col folded into the requests as in the tiled kernels): the K = R*S*Cin bytes of a row are R*S runs of
// Cin channels (Cin a multiple of 64, so every 64-deep k block lies inside one filter tap), and the 16-byte chunk a
// lane requests comes from its pixel at that tap, or from a constant row of theta_A bytes when the tap lies outside
// the image (a k block past K: of 0x80 bytes, the K padding).  A request here covers ONE k block for 16 rows (lane =
// row, 16-byte piece of the block), so the tap of a request is wave-uniform and lives on the scalar unit, moved on
// block by block; a lane carries its pixel's byte offset and one validity bit per tap (R*S <= 32) per row block.
// The staged batch is therefore laid out [k block][row block][16 rows][64 bytes] instead of whole row segments.
template <int MODE, int MB, int NWAVES, int BATCH, bool B4, bool ANYALIGN, bool SIMPLE = false, int CPW = 1, bool AF32 = false,
          bool ACONV = false>
__global__ __launch_bounds__(NWAVES * 64) void qg_gemm_skinny_kernel(const uint8_t* A, const int8_t* Bp, const int M, const int N, const int K, const int kb64,
                                                                   const int nb16_total, const int lda, const int ks_per, const int ksplit,
                                                                   const qg_gemm_args p) {
  // The leading scalar arguments repeat what a wave needs before it can issue its first loads (the fields of the same
  // names in p): the file is compiled with kernel-argument preloading, so they arrive in scalar registers with the
  // wave instead of costing a cold trip to memory (measured: 0.4 us of a 5 us launch).
  static_assert(!SIMPLE || (!B4 && !ANYALIGN), "the straight-line variant takes dense 8-bit weights and aligned rows");
  static_assert(CPW == 1 || SIMPLE, "several fragment columns per wave: straight-line variant only");
  static_assert(!AF32 || (!SIMPLE && !B4 && ANYALIGN), "fp32 activations: the lane-copied staging of the general variant");
  static_assert(!ACONV || (!SIMPLE && !B4 && !ANYALIGN && !AF32), "convolution: the requested staging of the general variant");
  static_assert(MB * CPW <= NWAVES && CPW <= BATCH, "one wave per (row block, fragment column) runs the output pipeline");
  const bool a_vec = ANYALIGN || p.a_vec;  // whole 16-byte chunks may be moved as such
  using chunk_t = typename std::conditional<ANYALIGN, qg_v4i_unaligned, v4i>::type;
  // A through LDS (see the file header): per wave and batch, ROWS rows x ROWB bytes
  constexpr int ROWS = MB * 16, ROWB = BATCH * QG_FRAG_K, NCHUNK = ROWB / 16;
  constexpr int REGION = ROWS * ROWB, NREQ = REGION / 1024, RPR = 64 / NCHUNK;  // requests per batch, rows per request
  static_assert(NCHUNK == 8 || NCHUNK == 16 || NCHUNK == 32, "a request covers whole rows of 128, 256 or 512 bytes");
  constexpr int PART_BYTES = NWAVES * MB * CPW * 64 * (int)sizeof(v4i);
  constexpr int RSP_BYTES = NWAVES * MB * 16 * (int)sizeof(int);
  constexpr int STAGE_BYTES = NWAVES * REGION;
  // every wave leaves its K-split partial sums (MB * CPW KiB) at the start of its OWN staging region (MB * BATCH KiB) once
  // it is done with it: no wave waits for the others before it may write
  static_assert(PART_BYTES <= STAGE_BYTES, "a wave's partial tile fits its staging region");
  constexpr int UNION_BYTES = STAGE_BYTES;
  extern __shared__ __align__(16) unsigned char smem[];
  int* rsp = reinterpret_cast<int*>(smem + UNION_BYTES);    // [mb][row][wave]
  int* sp = reinterpret_cast<int*>(smem + UNION_BYTES + RSP_BYTES);  // B4: [row][slot] sparse term

  const int nb16 = blockIdx.x * CPW;  // first fragment column of this workgroup
  // columns held by fragment f: (f>>1)*32 + 16*(u&1) + 8*(f&1) + 4*(u>>1) + r, u<4, r<4
  if ((nb16 >> 1) * 32 + 8 * (nb16 & 1) >= N) return;  // nothing but padding (uniform for the workgroup)

  const int tid = threadIdx.x, lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int ml = lane & 15, g = lane >> 4;
  const int m_base = blockIdx.y * (MB * 16);  // first row of this workgroup's row block

  // The waves that run the output pipeline fetch its per-column constants early, not after the reduction -- but
  // BEHIND the first batch's weight loads and activation requests (load_ep is called from the first batch): cold,
  // they take a trip to HBM, and nothing on the request path may end up waiting for them (the compiler had paired
  // a pending constant with an address computation and stalled the requests of exactly the wave the others wait for).
  // wave w < MB * CPW runs the output pipeline of row block w / CPW, fragment column nb16 + w % CPW
  const int red_mb = wave / CPW, red_c = wave % CPW;
  const int c0 = ((nb16 + red_c) >> 1) * 32 + 16 * (g & 1) + 8 * ((nb16 + red_c) & 1) + 4 * (g >> 1);  // this lane's 4 output columns
  int ep_co[4] = {0, 0, 0, 0}, ep_bz[4] = {0, 0, 0, 0}, ep_bias[4] = {0, 0, 0, 0};
  float ep_sc[4] = {1.0f, 1.0f, 1.0f, 1.0f};
  auto load_ep = [&]() {
    if (wave < MB * CPW) {
#pragma unroll
      for (int r = 0; r < 4; ++r) {
        const int col = c0 + r;  // col_off / bzp are padded to N_pad, bias / scales are not
        ep_co[r] = p.col_off[col];
        ep_bz[r] = p.bzp[col];
        ep_bias[r] = (MODE != QG_MODE_ACC32 && p.bias != nullptr && col < N) ? p.bias[col] : 0;
        ep_sc[r] = (MODE != QG_MODE_ACC32 && col < N) ? p.scales[(size_t)col * p.scale_stride] : 1.0f;
      }
    }
  };

  if (B4) {
    for (int t = tid; t < MB * 256; t += NWAVES * 64) sp[t] = 0;
    __syncthreads();
  }

  // K slices are dealt to the waves rotated by the workgroup index, so that at any instant the workgroups
  // of an XCD read DIFFERENT lines of A (all of them read all of A; unrotated they would all hit the same
  // L2 channel at the same time)
  // (4-bit weights come in pairs of k blocks, so their slices hold an even number of blocks)
  // (ksplit > 1: this workgroup owns slice blockIdx.z of K, whole k blocks, an even number of them for 4-bit weights)
  const int ks_begin = min(kb64, (int)blockIdx.z * ks_per), ks_end = min(kb64, ks_begin + ks_per);
  const int ks_len = ks_end - ks_begin;
  const int per = B4 ? ((ks_len + 2 * NWAVES - 1) / (2 * NWAVES)) * 2 : (ks_len + NWAVES - 1) / NWAVES;
  const int kb_begin = min(ks_end, ks_begin + ((wave + nb16) % NWAVES) * per);
  const int kb_end = min(ks_end, kb_begin + per);

  // outlier split: the entry offsets of all of this wave's batches, one per lane (batch b: lanes b and b+1), are
  // requested before anything else so that no batch waits for an offset before it can ask for its entries
  int sp_offs = 0;
  if (B4 && kb_begin < kb_end) {
    const int32_t* col = p.sp_ptr + (size_t)nb16 * kb64;
    sp_offs = col[min(kb_begin + BATCH * lane, kb_end)];
  }

  v4i acc[MB][CPW];
  unsigned rs[MB];  // sums of raw uint8 bytes (K padding reads as 0x80)
#pragma unroll
  for (int mb = 0; mb < MB; ++mb) {
#pragma unroll
    for (int c = 0; c < CPW; ++c) acc[mb][c] = (v4i){0, 0, 0, 0};
    rs[mb] = 0;
  }
  // 8-bit: one 1 KiB fragment per k block, 16 bytes per lane.  4-bit: one 1 KiB unit per PAIR of k blocks, 16 bytes
  // per lane (8 for each block), so that a request moves as many bytes as in the 8-bit layout.
  const int8_t* bcol = Bp + (size_t)nb16 * QG_FRAG_BYTES;  // wave-uniform; the lane's 16 bytes are at + lane * 16
  const unsigned lane16 = lane * 16;
  const size_t b_step = (size_t)nb16_total * QG_FRAG_BYTES;  // one slab (8-bit: 64 deep, 4-bit: 128 deep) of the packed buffer

  // per-lane byte offsets of the NREQ activation requests of a batch (a.a_vec: they fit 32 bits); with them the
  // request address is a wave-uniform base plus a register that is never the target of a load, so issuing
  // the requests never has to wait for loads in flight
  unsigned a_off[NREQ];
  // ACONV: of the piece a lane requests for row block mb: byte offset of its pixel at tap (0, 0), channel slice 0 (may
  // be negative) and the taps of that pixel that lie inside the image; wave-uniform: the tap of the next k block
  int cv_pix[MB];
  unsigned cv_mask[MB];
  int cv_cc = 0, cv_kw = 0, cv_kh = 0;
  const int cv_nc = ACONV ? p.cv_Cin / QG_FRAG_K : 1;  // k blocks per tap
  const uint8_t* const cv_azp_row = qg_byte_rows.b[ACONV ? p.cv_azp : 0];
  if (ACONV) {
#pragma unroll
    for (int mb = 0; mb < MB; ++mb) {
      const int r = mb * 16 + (lane >> 2);
      const int m = min(m_base + r, M - 1);
      const int wo = m % p.cv_Wo, t = m / p.cv_Wo;
      const int ho = t % p.cv_Ho, n = t / p.cv_Ho;
      const int h0 = ho * p.cv_stride - p.cv_pad, w0 = wo * p.cv_stride - p.cv_pad;
      // the lane's 16 bytes land at piece lane % 4 of its row's 64-byte block; that place holds logical piece (lane % 4) ^ (row / 4 % 4)
      cv_pix[mb] = ((n * p.cv_H + h0) * p.cv_W + w0) * p.cv_pix + ((((lane & 3) ^ (lane >> 4)) & 3) << 4);
      cv_mask[mb] = 0;
      for (int kh = 0, tap = 0; kh < p.cv_R; ++kh)
        for (int kw = 0; kw < p.cv_S; ++kw, ++tap)
          if ((unsigned)(h0 + kh) < (unsigned)p.cv_H && (unsigned)(w0 + kw) < (unsigned)p.cv_W) cv_mask[mb] |= 1u << tap;
    }
    const int tap = kb_begin / cv_nc;
    cv_cc = kb_begin - tap * cv_nc;
    cv_kh = tap / p.cv_S;
    cv_kw = tap - cv_kh * p.cv_S;
  }
#pragma unroll
  for (int jj = 0; jj < NREQ; ++jj) {
    const int r = jj * RPR + lane / NCHUNK;
    a_off[jj] = (unsigned)min(m_base + r, M - 1) * (unsigned)lda + ((unsigned)((lane ^ r) & (NCHUNK - 1)) << 4);
  }

  // Weight requests of one batch: NLOAD loads of 16 bytes per lane, kept RAW (the 4-bit units are widened only
  // when they are consumed, so that nothing waits for them before the activations have been requested too).
  constexpr int NLOAD = B4 ? BATCH / 2 : BATCH;
  static_assert(!B4 || BATCH % 2 == 0, "4-bit weights are fetched in pairs of k blocks");
  // (every element is loaded unconditionally -- blocks past the end of the slice re-read its last block and are
  // never used -- so that the loaded registers are plain values and no copy has to wait for them)
  auto load_b = [&](int kb0, v4i (&raw)[NLOAD]) {
#pragma unroll
    for (int i = 0; i < NLOAD; ++i) {
      const int kbi = min(kb0 + (B4 ? 2 * i : i), kb_end - 1);  // B4: kb0 and kb_end are even
      raw[i] = *reinterpret_cast<const v4i*>(bcol + (size_t)(B4 ? kbi >> 1 : kbi) * b_step + lane16);
    }
  };
  auto operand = [&](const v4i (&raw)[NLOAD], int j) -> v4i {
    if (!B4) return raw[j];
    const v4i w = raw[j >> 1];
    const unsigned lo = (unsigned)((j & 1) ? w.z : w.x), hi = (unsigned)((j & 1) ? w.w : w.y);
    return (v4i){(int)(lo & 0x0F0F0F0Fu), (int)((lo >> 4) & 0x0F0F0F0Fu), (int)(hi & 0x0F0F0F0Fu),
                 (int)((hi >> 4) & 0x0F0F0F0Fu)};
  };

  // One batch: its weights were requested one batch earlier (into `cur`); request its activations and the NEXT
  // batch's weights (into `nxt`), then wait for the activations only.  Requests complete in order, so
  // "at most NLOAD outstanding" means that everything older than the next batch's weights has arrived.
  auto batch = [&](int kb, const v4i (&cur)[NLOAD], v4i (&nxt)[NLOAD], const bool has_next, auto first_tag) {
    constexpr bool FIRST = decltype(first_tag)::value;
    // whole rows of BATCH k blocks are requested even when the slice ends earlier: the surplus lies inside the
    // row (it is the next wave's slice) and is simply not consumed
    const bool staged = ACONV || (!AF32 && a_vec && (kb + BATCH) * QG_FRAG_K <= K);
    unsigned char* region = smem + wave * REGION;
    // outlier split: this batch's entries are one run; the first 64 are requested one per lane right behind the
    // activations (always exactly one request, clamped into the buffer, so that the wait below can count it)
    int sp_e0 = 0, sp_ne = 0, sp_first = 0;
    auto sparse_request = [&]() {
      if (B4) {
        const int b = (kb - kb_begin) / BATCH;  // at most 64 batches per wave: K <= 32768 gives 32 blocks per wave
        sp_e0 = __shfl(sp_offs, b);
        sp_ne = __shfl(sp_offs, b + 1) - sp_e0;
        sp_first = p.sp_entries[min(sp_e0 + lane, max(p.sp_total, 1) - 1)];
      }
    };
    v4i af[MB][BATCH];
    if (staged) {
      // ROWS rows x ROWB bytes of A: NREQ requests of RPR whole rows into this wave's LDS region, chunk c of
      // row r stored at chunk c ^ r so that the operand-order reads below are bank-conflict free
      const uint8_t* a_base = A + (size_t)kb * QG_FRAG_K;  // wave-uniform
      const unsigned region_lds = (unsigned)(uintptr_t)((__attribute__((address_space(3))) unsigned char*)region);
      if (ACONV) {
#pragma unroll
        for (int j = 0; j < BATCH; ++j) {
          // (wave-uniform) a k block past K -- the zero padding of the packed weights -- is staged as 0x80 bytes like
          // all K padding, a tap outside the image as theta_A bytes
          const bool in_k = cv_kh < p.cv_R;
          const unsigned tapbit = in_k ? 1u << (cv_kh * p.cv_S + cv_kw) : 0u;
          const int toff = (cv_kh * p.cv_W + cv_kw) * p.cv_pix + cv_cc * QG_FRAG_K;
          const uint8_t* const other = in_k ? cv_azp_row : qg_byte_rows.b[128];
#pragma unroll
          for (int mb = 0; mb < MB; ++mb)
            request_a64((cv_mask[mb] & tapbit) != 0 ? A + (cv_pix[mb] + toff) : other, region_lds + (j * MB + mb) * 1024);
          if (++cv_cc == cv_nc) {
            cv_cc = 0;
            if (++cv_kw == p.cv_S) cv_kw = 0, ++cv_kh;
          }
        }
      } else
#pragma unroll
      for (int jj = 0; jj < NREQ; ++jj) request_a(a_base, a_off[jj], region_lds + jj * 1024);
      asm volatile("" ::: "memory");
      if (FIRST) load_ep();
      sparse_request();
      asm volatile("" ::: "memory");
      if (has_next) {
        load_b(kb + BATCH, nxt);
        asm volatile("s_waitcnt vmcnt(%0)" ::"n"(NLOAD) : "memory");
      } else {
        asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
      }
    } else {
      // any pointer, lda and K, partial batches: the lanes copy the block into the region themselves, 16-byte
      // chunk by chunk (bytes past K as 0x80, the int8 zero after the shift), in the same swizzled layout
      const int nchunk = min(BATCH, kb_end - kb) * 4;  // 16-byte chunks per row that this batch will consume
      if constexpr (AF32) {
        const float* Af = reinterpret_cast<const float*>(A);
        constexpr int CH = ROWS * NCHUNK / 64;  // chunks per lane of a full batch
        if (p.a_vec && nchunk == NCHUNK && (kb + BATCH) * QG_FRAG_K <= K) {
          // whole batch inside K, rows of floats 16-byte aligned: two chunks' loads at a time (8 x 16 bytes per lane in
          // flight; more would not fit the 128 registers of a 16-wave workgroup), then convert
          constexpr int GRP = (CH >= 2 && MB == 1) ? 2 : 1;
#pragma unroll 1
          for (int t0 = 0; t0 < CH; t0 += GRP) {
            float4 v[GRP][4];
#pragma unroll
            for (int t = 0; t < GRP; ++t) {
              const int i = lane + 64 * (t0 + t), r = i / NCHUNK, lc = i % NCHUNK;
              const float4* src = reinterpret_cast<const float4*>(Af + (size_t)min(m_base + r, M - 1) * lda + kb * QG_FRAG_K + (lc << 4));
#pragma unroll
              for (int e = 0; e < 4; ++e) v[t][e] = src[e];
            }
#pragma unroll
            for (int t = 0; t < GRP; ++t) {
              const int i = lane + 64 * (t0 + t), r = i / NCHUNK, lc = i % NCHUNK;
              v4i w;
#pragma unroll
              for (int e = 0; e < 4; ++e) {
                unsigned d = qg_quantize_pack(v[t][e].x, p.q_inv, p.q_lo, p.q_hi, p.q_zp, 0, 0);
                d = qg_quantize_pack(v[t][e].y, p.q_inv, p.q_lo, p.q_hi, p.q_zp, 1, d);
                d = qg_quantize_pack(v[t][e].z, p.q_inv, p.q_lo, p.q_hi, p.q_zp, 2, d);
                w[e] = (int)qg_quantize_pack(v[t][e].w, p.q_inv, p.q_lo, p.q_hi, p.q_zp, 3, d);
              }
              *reinterpret_cast<v4i*>(region + (r * NCHUNK + ((lc ^ r) & (NCHUNK - 1))) * 16) = w;
            }
          }
        } else {
          // any pointer, lda and K, partial batches: element by element, positions past K as 0x80
#pragma unroll 1
          for (int i = lane; i < ROWS * nchunk; i += 64) {
            const int r = i / nchunk, lc = i % nchunk;
            const int k0 = kb * QG_FRAG_K + (lc << 4);
            const float* src = Af + (size_t)min(m_base + r, M - 1) * lda + k0;
            v4i w;
#pragma unroll
            for (int e = 0; e < 4; ++e) {
              unsigned d = 0x80808080u;
#pragma unroll
              for (int b = 0; b < 4; ++b)
                if (k0 + 4 * e + b < K) d = qg_quantize_pack(src[4 * e + b], p.q_inv, p.q_lo, p.q_hi, p.q_zp, b, d);
              w[e] = (int)d;
            }
            *reinterpret_cast<v4i*>(region + (r * NCHUNK + ((lc ^ r) & (NCHUNK - 1))) * 16) = w;
          }
        }
      } else
#pragma unroll 1
      for (int i = lane; i < ROWS * nchunk; i += 64) {
        const int r = i / nchunk, lc = i % nchunk;     // row, logical chunk
        const int c = r * NCHUNK + ((lc ^ r) & (NCHUNK - 1));
        const int k0 = kb * QG_FRAG_K + (lc << 4);
        const uint8_t* src = A + (size_t)min(m_base + r, M - 1) * lda + k0;
        v4i v;
        if (a_vec && k0 + 16 <= K)
          v = *reinterpret_cast<const chunk_t*>(src);
        else
          v = qg_load_a_chunk(src, K - k0, false);  // byte by byte, bytes past K as 0x80
        *reinterpret_cast<v4i*>(region + c * 16) = v;
      }
      if (FIRST) load_ep();
      sparse_request();
      if (has_next) load_b(kb + BATCH, nxt);
    }
#pragma unroll
    for (int mb = 0; mb < MB; ++mb)
#pragma unroll
      for (int j = 0; j < BATCH; ++j) {
        const int r = mb * 16 + ml;
        if (ACONV)  // [k block][row block][row][piece ^ (row / 4 % 4)]
          af[mb][j] = *reinterpret_cast<const v4i*>(region + (j * MB + mb) * 1024 + ml * QG_FRAG_K + (((g ^ (ml >> 2)) & 3) << 4));
        else
          af[mb][j] = *reinterpret_cast<const v4i*>(region + r * ROWB + ((((4 * j + g) ^ r) & (NCHUNK - 1)) << 4));
      }
#pragma unroll
    for (int j = 0; j < BATCH; ++j)
      if (kb + j < kb_end) {
        const v4i bfj = operand(cur, j);
#pragma unroll
        for (int mb = 0; mb < MB; ++mb) {
          rs[mb] = __builtin_amdgcn_sad_u8(af[mb][j].x, 0u, rs[mb]);
          rs[mb] = __builtin_amdgcn_sad_u8(af[mb][j].y, 0u, rs[mb]);
          rs[mb] = __builtin_amdgcn_sad_u8(af[mb][j].z, 0u, rs[mb]);
          rs[mb] = __builtin_amdgcn_sad_u8(af[mb][j].w, 0u, rs[mb]);
          const v4i a = af[mb][j] ^ (int)0x80808080;
          acc[mb][0] = __builtin_amdgcn_mfma_i32_16x16x64_i8(bfj, a, acc[mb][0], 0, 0, 0);
        }
      }
    if (B4) {
      // sparse term of this batch: pair idx = (entry idx / ROWS, row idx % ROWS); A_s = A_u - 128.  Entries are
      // held one per lane, 64 at a time, and handed to the lanes that need them with a shuffle.
      for (int c0 = 0; c0 < sp_ne; c0 += 64) {
        const int held = c0 == 0 ? sp_first : (c0 + lane < sp_ne ? p.sp_entries[sp_e0 + c0 + lane] : 0);
        const int pairs = min(sp_ne - c0, 64) * ROWS;
        for (int idx = lane; idx < ((pairs + 63) & ~63); idx += 64) {
          const int ent = __shfl(held, idx / ROWS);  // every lane takes part in the shuffle
          if (idx >= pairs) continue;
          const int r = idx % ROWS;
          const int k = ent & 0x7FFF, slot = (ent >> 16) & 15, v = ent >> 24;
          const int kk = k - kb * QG_FRAG_K;  // inside the staged ROWS x ROWB block (chunk c of row r at c ^ r)
          const int a = region[r * ROWB + ((((kk >> 4) ^ r) & (NCHUNK - 1)) << 4) + (kk & 15)];
          atomicAdd(&sp[r * 16 + slot], (a - 128) * v);
        }
      }
    }
  };

  if constexpr (SIMPLE) {
    // per is a multiple of BATCH and at least BATCH (host-checked); everything below is wave-uniform control flow
    const int nbatch = per / BATCH;
    const int8_t* bptr = bcol + (size_t)kb_begin * b_step;
    const uint8_t* aptr = A + (size_t)kb_begin * QG_FRAG_K;
    unsigned char* region = smem + wave * REGION;
    const unsigned region_lds = (unsigned)(uintptr_t)((__attribute__((address_space(3))) unsigned char*)region);
    auto issue_w = [&](int b, v4i (&raw)[BATCH * CPW]) {
      const int8_t* bp = bptr + (size_t)b * BATCH * b_step;
#pragma unroll
      for (int i = 0; i < BATCH; ++i)
#pragma unroll
        for (int c = 0; c < CPW; ++c)  // the CPW fragments of one k block are adjacent KiBs
          raw[i * CPW + c] = *reinterpret_cast<const v4i*>(bp + (size_t)i * b_step + c * QG_FRAG_BYTES + lane16);
    };
    // batch b: its weights were requested one batch earlier; request its activations, (first batch) the constants of
    // the output pipeline, the next batch's weights; wait for everything older than those; consume
    auto step = [&](int b, v4i (&cur)[BATCH * CPW], v4i (&nxt)[BATCH * CPW], auto first_tag) {
      const uint8_t* ab = aptr + (size_t)b * (BATCH * QG_FRAG_K);
#pragma unroll
      for (int jj = 0; jj < NREQ; ++jj) request_a(ab, a_off[jj], region_lds + jj * 1024);
      if (decltype(first_tag)::value) load_ep();
      asm volatile("" ::: "memory");
      if (b + 1 < nbatch) {
        issue_w(b + 1, nxt);
        wait_vm<BATCH * CPW>();
      } else {
        wait_vm<0>();
      }
      v4i af[MB][BATCH];
#pragma unroll
      for (int mb = 0; mb < MB; ++mb)
#pragma unroll
        for (int j = 0; j < BATCH; ++j) {
          const int r = mb * 16 + ml;
          af[mb][j] = *reinterpret_cast<const v4i*>(region + r * ROWB + ((((4 * j + g) ^ r) & (NCHUNK - 1)) << 4));
        }
#pragma unroll
      for (int j = 0; j < BATCH; ++j)
#pragma unroll
        for (int mb = 0; mb < MB; ++mb) {
          rs[mb] = __builtin_amdgcn_sad_u8(af[mb][j].x, 0u, rs[mb]);
          rs[mb] = __builtin_amdgcn_sad_u8(af[mb][j].y, 0u, rs[mb]);
          rs[mb] = __builtin_amdgcn_sad_u8(af[mb][j].z, 0u, rs[mb]);
          rs[mb] = __builtin_amdgcn_sad_u8(af[mb][j].w, 0u, rs[mb]);
          const v4i a = af[mb][j] ^ (int)0x80808080;
#pragma unroll
          for (int c = 0; c < CPW; ++c)
            acc[mb][c] = __builtin_amdgcn_mfma_i32_16x16x64_i8(cur[j * CPW + c], a, acc[mb][c], 0, 0, 0);
        }
      asm volatile("" ::: "memory");  // the fragment reads stay in front of the next batch's requests into the same region
    };
    v4i w0[BATCH * CPW], w1[BATCH * CPW];
    issue_w(0, w0);
    step(0, w0, w1, std::true_type{});
    for (int b = 1; b < nbatch; b += 2) {
      step(b, w1, w0, std::false_type{});
      if (b + 1 < nbatch) step(b + 1, w0, w1, std::false_type{});
    }
  } else
  // two register sets alternate; the first batch is peeled (it also requests the output-pipeline constants)
  if (kb_begin < kb_end) {
    v4i braw0[NLOAD], braw1[NLOAD];
    load_b(kb_begin, braw0);
    batch(kb_begin, braw0, braw1, kb_begin + BATCH < kb_end, std::true_type{});
    for (int kb = kb_begin + BATCH; kb < kb_end; kb += 2 * BATCH) {
      batch(kb, braw1, braw0, kb + BATCH < kb_end, std::false_type{});
      if (kb + BATCH < kb_end) batch(kb + BATCH, braw0, braw1, kb + 2 * BATCH < kb_end, std::false_type{});
    }
  } else {
    load_ep();
  }

  // ---- combine the 16 K-slices through LDS (a wave's fragment reads of its region are complete: the MFMAs consumed them)
#pragma unroll
  for (int mb = 0; mb < MB; ++mb) {
#pragma unroll
    for (int c = 0; c < CPW; ++c) reinterpret_cast<v4i*>(smem + wave * REGION)[(mb * CPW + c) * 64 + lane] = acc[mb][c];
    // the four lanes (ml, g = 0..3) of a row hold its byte sums over different k: add them with two lane swaps
    // (v_permlane32_swap / v_permlane16_swap; a shuffle through the LDS crossbar costs about 100 cycles each)
    const unsigned v = rs[mb];
    const auto h = __builtin_amdgcn_permlane32_swap(v, v, false, false);
    const unsigned v2 = h[0] + h[1];
    const auto q = __builtin_amdgcn_permlane16_swap(v2, v2, false, false);
    if (g == 0) rsp[((mb * 16 + ml) * NWAVES) + wave] = (int)(q[0] + q[1]);  // [mb][row][wave]: the reader takes a row's 16 sums in four reads
  }
  __syncthreads();
  if (wave >= MB * CPW) return;
  const int mb = red_mb;
  v4i sum = (v4i){0, 0, 0, 0};
  int rsum = -128 * (ks_len * QG_FRAG_K);  // every staged byte (padding included) is 128 above its int8 value
  {
    // every read is issued before the first sum (a sum per read would serialise on the LDS latency, 16 times over)
    static_assert(NWAVES % 4 == 0, "row sums are fetched four waves at a time");
    v4i t[NWAVES], tr[NWAVES / 4];
#pragma unroll
    for (int w = 0; w < NWAVES; ++w) t[w] = reinterpret_cast<const v4i*>(smem + w * REGION)[(mb * CPW + red_c) * 64 + lane];
#pragma unroll
    for (int w = 0; w < NWAVES / 4; ++w) tr[w] = reinterpret_cast<const v4i*>(rsp + (mb * 16 + ml) * NWAVES)[w];
#pragma unroll
    for (int w = 0; w < NWAVES; ++w) sum += t[w];
#pragma unroll
    for (int w = 0; w < NWAVES / 4; ++w) rsum += tr[w].x + tr[w].y + tr[w].z + tr[w].w;
  }
  if (B4) {
    // A_s B = (A_s U - 8 rowsum(A_s)) + A_s B_sparse; lane (ml, g) register r is slot 4 g + r of the fragment
#pragma unroll
    for (int r = 0; r < 4; ++r) sum[r] += sp[(mb * 16 + ml) * 16 + 4 * g + r] - 8 * rsum;
  }

  // ---- K split across workgroups: hand the partial tile in, the last slice to arrive carries on
  if (ksplit > 1) {
    // one counter per (row block of 16, fragment column)
    const int unit = (((int)blockIdx.y * (int)gridDim.x + (int)blockIdx.x) * CPW + red_c) * MB + mb;
    int* cnt = p.ws_cnt + unit;
    int* slots = p.ws_slots + (size_t)unit * ksplit * SLOT_INTS;
    int* mine = slots + (size_t)blockIdx.z * SLOT_INTS;
#pragma unroll
    for (int r = 0; r < 4; ++r) __hip_atomic_store(mine + lane * 4 + r, sum[r], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    if (g == 0) __hip_atomic_store(mine + 256 + ml, rsum, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    asm volatile("s_waitcnt vmcnt(0)" ::: "memory");  // the write-through stores above have been acknowledged
    int ticket = 0;
    if (lane == 0) ticket = __hip_atomic_fetch_add(cnt, 1, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    ticket = __builtin_amdgcn_readfirstlane(ticket);
    if (ticket != ksplit - 1) return;
    asm volatile("" ::: "memory");
    // every other slice's stores were acknowledged before it took its ticket; add all slots in slice order
    sum = (v4i){0, 0, 0, 0};
    rsum = 0;
#pragma unroll 4  // the loads of four slots are in flight together
    for (int ss = 0; ss < ksplit; ++ss) {
      const int* theirs = slots + (size_t)ss * SLOT_INTS;
#pragma unroll
      for (int r = 0; r < 4; ++r) sum[r] += __hip_atomic_load(theirs + lane * 4 + r, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
      rsum += __hip_atomic_load(theirs + 256 + ml, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    }
    if (lane == 0) __hip_atomic_store(cnt, 0, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);  // ready for the next call
  }

  // ---- output pipeline; lane (ml, u = g) holds row m_base+mb*16+ml, 4 consecutive columns
  const int row = m_base + mb * 16 + ml;
  if (row >= M || c0 >= N) return;
  if (MODE == QG_MODE_REQUANT) {
    unsigned out = 0;
#pragma unroll
    for (int r = 0; r < 4; ++r) {
      const int x = sum[r] + ep_bias[r] - p.a_zp_m128 * ep_co[r] - ep_bz[r] * rsum;
      out |= (unsigned)qg_requant_one(x, ep_sc[r], p.clamp_lo, p.clamp_hi, p.c_zp) << (8 * r);
    }
    uint8_t* dst = p.C + (size_t)row * p.ldc + c0;
    if (p.c_vec && c0 + 4 <= N) {
      // a small output goes out write-through: the end of the kernel then finds no dirty lines to write back
      // (measured: 0.3 us of a 5 us launch)
      if (p.c_wt)
        __hip_atomic_store(reinterpret_cast<unsigned*>(dst), out, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_SYSTEM);
      else
        *reinterpret_cast<unsigned*>(dst) = out;
    } else {
#pragma unroll
      for (int r = 0; r < 4; ++r)
        if (c0 + r < N) dst[r] = (uint8_t)(out >> (8 * r));
    }
  } else if (MODE == QG_MODE_DEQUANT) {
    float out[4];
#pragma unroll
    for (int r = 0; r < 4; ++r) {
      const int x = sum[r] + ep_bias[r] - p.a_zp_m128 * ep_co[r] - ep_bz[r] * rsum;
      out[r] = qg_dequant_one(x, ep_sc[r], p.relu_lo);
    }
    float* dst = p.Cf + (size_t)row * p.ldc + c0;
    if (p.c_vec && c0 + 4 <= N) {
      *reinterpret_cast<float4*>(dst) = make_float4(out[0], out[1], out[2], out[3]);
    } else {
#pragma unroll
      for (int r = 0; r < 4; ++r)
        if (c0 + r < N) dst[r] = out[r];
    }
  } else {
#pragma unroll
    for (int r = 0; r < 4; ++r) {
      const int col = c0 + r;
      if (col < N) p.C32[(size_t)row * p.ldc + col] = sum[r] + 128 * (ep_co[r] + K * ep_bz[r]);
    }
    if (p.rowsum_out != nullptr && nb16 + red_c == 0 && g == 0) p.rowsum_out[row] = rsum + 128 * K;
  }
}

template <int MODE, int MB, int NWAVES, int BATCH, bool B4, bool ANYALIGN>
hipError_t launch(const qg_gemm_args& a, hipStream_t s) {
  const int part = NWAVES * MB * 64 * (int)sizeof(v4i), stage = NWAVES * (MB * 16) * (BATCH * QG_FRAG_K);
  const int smem = (stage > part ? stage : part) + NWAVES * MB * 16 * (int)sizeof(int) +
                   (B4 ? MB * 256 * (int)sizeof(int) : 0);
  const int nfrag = ((a.N + 31) / 32) * 2;
  const int mblocks = (a.M + MB * 16 - 1) / (MB * 16);
  if (mblocks > 65535 || a.ksplit < 1 || a.ksplit > 65535) return hipErrorInvalidValue;
  if (a.ksplit > 1 && (a.ws_cnt == nullptr || a.ws_slots == nullptr)) return hipErrorInvalidValue;
  const dim3 grid(nfrag, mblocks, a.ksplit), block(NWAVES * 64);
  if constexpr (!B4 && !ANYALIGN) {
    // More 32-column super-blocks than half the CUs: few fat waves per workgroup, each streaming two fragment columns
    // (four waves and batches of eight k blocks; eight waves and batches of four at 64 rows, whose staged batch is
    // four times as large).  The 16-wave form would put two or more workgroups on a CU there, and a second
    // one costs about as much as the first (80 x 1536 x 2048: 6.7 -> 3.4 us cold, 640 x 128 x 2048: 6.7 -> 3.7,
    // 80 x 1024 x 4096: 6.9 -> 5.7).  Cold, 16 rows: 8192 x 4096 11.4 -> 9.4 us, 8192 x 8192 18.2 -> 15.0 (a plain
    // read of the weights in the same launch shape: 14.4), 16384 x 16384 59.2 -> 48.7; 32 rows, 8192 x 8192:
    // 21.0 -> 16.9; 64 rows: 8192 x 8192 26.3 -> 19.7, 2048 x 8192 10.8 -> 7.7, 128 x 8192 x 4096 27.7 -> 19.8 --
    // every activation fragment feeds two MFMAs, so the workgroup stages half the activation bytes per weight byte,
    // which at 64 rows is most of the traffic.  With 128 super-blocks or fewer half the CUs would idle and the
    // 16-wave form stays ahead (16 x 4096 x 8192: 9.6 vs 10.9 us; 64 x 4096 x 4096: 8.1 vs 9.5).
    constexpr int WN = MB == 4 ? 8 : 4, WB = MB == 4 ? 4 : 8, WC = 2;
    if ((long long)((a.N + 31) / 32) * mblocks > 128 && a.K == a.kb64 * QG_FRAG_K && a.kb64 % a.ks_per == 0 &&
        a.ks_per % (WN * WB) == 0) {
      constexpr auto fn = qg_gemm_skinny_kernel<MODE, MB, WN, WB, false, false, true, WC>;
      const int wpart = WN * MB * WC * 64 * (int)sizeof(v4i), wstage = WN * (MB * 16) * (WB * QG_FRAG_K);
      const int wsmem = (wstage > wpart ? wstage : wpart) + WN * MB * 16 * (int)sizeof(int);
      hipError_t e = qg_allow_smem<fn>(wsmem);
      if (e != hipSuccess) return e;
      hipLaunchKernelGGL(fn, dim3((a.N + 31) / 32, mblocks, a.ksplit), dim3(WN * 64), wsmem, s, a.A, a.Bp, a.M, a.N, a.K, a.kb64,
                         a.nb16, a.lda, a.ks_per, a.ksplit, a);
      return hipGetLastError();
    }
  }
  if constexpr (!B4 && !ANYALIGN) {
    // the straight-line variant: K is a whole number of blocks, all slices are equal and give every wave whole batches
    if (a.K == a.kb64 * QG_FRAG_K && a.kb64 % a.ks_per == 0 && a.ks_per % (NWAVES * BATCH) == 0) {
      constexpr auto fn = qg_gemm_skinny_kernel<MODE, MB, NWAVES, BATCH, false, false, true>;
      hipError_t e = qg_allow_smem<fn>(smem);
      if (e != hipSuccess) return e;
      hipLaunchKernelGGL(fn, grid, block, smem, s, a.A, a.Bp, a.M, a.N, a.K, a.kb64, a.nb16, a.lda, a.ks_per, a.ksplit, a);
      return hipGetLastError();
    }
  }
  hipError_t e = qg_allow_smem<qg_gemm_skinny_kernel<MODE, MB, NWAVES, BATCH, B4, ANYALIGN>>(smem);
  if (e != hipSuccess) return e;
  hipLaunchKernelGGL((qg_gemm_skinny_kernel<MODE, MB, NWAVES, BATCH, B4, ANYALIGN>), grid, block, smem, s, a.A, a.Bp, a.M, a.N,
                     a.K, a.kb64, a.nb16, a.lda, a.ks_per, a.ksplit, a);
  return hipGetLastError();
}

// fp32 activations: the general variant with the converting staging (any alignment; a.a_vec says whether the rows of
// floats are 16-byte aligned)
template <int MODE, int MB, int NWAVES, int BATCH>
hipError_t launch_af32(const qg_gemm_args& a, hipStream_t s) {
  const int part = NWAVES * MB * 64 * (int)sizeof(v4i), stage = NWAVES * (MB * 16) * (BATCH * QG_FRAG_K);
  const int smem = (stage > part ? stage : part) + NWAVES * MB * 16 * (int)sizeof(int);
  const int nfrag = ((a.N + 31) / 32) * 2;
  const int mblocks = (a.M + MB * 16 - 1) / (MB * 16);
  if (mblocks > 65535 || a.ksplit < 1 || a.ksplit > 65535) return hipErrorInvalidValue;
  if (a.ksplit > 1 && (a.ws_cnt == nullptr || a.ws_slots == nullptr)) return hipErrorInvalidValue;
  constexpr auto fn = qg_gemm_skinny_kernel<MODE, MB, NWAVES, BATCH, false, true, false, 1, true>;
  hipError_t e = qg_allow_smem<fn>(smem);
  if (e != hipSuccess) return e;
  hipLaunchKernelGGL(fn, dim3(nfrag, mblocks, a.ksplit), dim3(NWAVES * 64), smem, s, a.A, a.Bp, a.M, a.N, a.K, a.kb64, a.nb16,
                     a.lda, a.ks_per, a.ksplit, a);
  return hipGetLastError();
}

// dense convolution (a.cv_* describe it, a.A is the image): the general variant with the convolution's requests
template <int MB, int NWAVES, int BATCH>
hipError_t launch_conv(const qg_gemm_args& a, hipStream_t s) {
  const int part = NWAVES * MB * 64 * (int)sizeof(v4i), stage = NWAVES * (MB * 16) * (BATCH * QG_FRAG_K);
  const int smem = (stage > part ? stage : part) + NWAVES * MB * 16 * (int)sizeof(int);
  const int nfrag = ((a.N + 31) / 32) * 2;
  const int mblocks = (a.M + MB * 16 - 1) / (MB * 16);
  if (mblocks > 65535) return hipErrorInvalidValue;
  constexpr auto fn = qg_gemm_skinny_kernel<QG_MODE_REQUANT, MB, NWAVES, BATCH, false, false, false, 1, false, true>;
  hipError_t e = qg_allow_smem<fn>(smem);
  if (e != hipSuccess) return e;
  hipLaunchKernelGGL(fn, dim3(nfrag, mblocks, 1), dim3(NWAVES * 64), smem, s, a.A, a.Bp, a.M, a.N, a.K, a.kb64, a.nb16, a.lda,
                     a.kb64, 1, a);
  return hipGetLastError();
}

// waves per workgroup and k blocks a wave requests at once, per row-block height
template <int MODE, bool B4, bool ANYALIGN>
hipError_t launch_mb(const qg_gemm_args& a, int kernel, hipStream_t s) {
  switch (kernel) {
    case QG_KERNEL_SKINNY16: return launch<MODE, 1, 16, 4, B4, ANYALIGN>(a, s);
    case QG_KERNEL_SKINNY32: return launch<MODE, 2, 16, 4, B4, ANYALIGN>(a, s);
    case QG_KERNEL_SKINNY64: return launch<MODE, 4, 16, 2, B4, ANYALIGN>(a, s);
    default: return hipErrorInvalidValue;
  }
}

template <bool B4, bool ANYALIGN>
hipError_t launch_mode(const qg_gemm_args& a, int mode, int kernel, hipStream_t s) {
  if (mode == QG_MODE_REQUANT) return launch_mb<QG_MODE_REQUANT, B4, ANYALIGN>(a, kernel, s);
  if (mode == QG_MODE_DEQUANT) return launch_mb<QG_MODE_DEQUANT, B4, ANYALIGN>(a, kernel, s);
  return launch_mb<QG_MODE_ACC32, B4, ANYALIGN>(a, kernel, s);
}

}  // namespace

// Dense convolution on the streaming kernels: few output pixels and a long K.  Cin % 64 == 0, R*S <= 32.
hipError_t qg_launch_conv_skinny(const qg_gemm_args& a, int kernel, hipStream_t s) {
  if (a.sp_ptr != nullptr || a.cv_Cin % QG_FRAG_K != 0 || a.cv_R * a.cv_S > 32 || a.ksplit != 1) return hipErrorInvalidValue;
  switch (kernel) {
    case QG_KERNEL_SKINNY16: return launch_conv<1, 16, 4>(a, s);
    case QG_KERNEL_SKINNY32: return launch_conv<2, 16, 4>(a, s);
    case QG_KERNEL_SKINNY64: return launch_conv<4, 16, 2>(a, s);
    default: return hipErrorInvalidValue;
  }
}

// a.A points to fp32 activations (a.lda in floats, a.q_*: the quantization); mode: QG_MODE_REQUANT or QG_MODE_DEQUANT
hipError_t qg_launch_gemm_skinny_f32(const qg_gemm_args& a, int mode, int kernel, hipStream_t s) {
  if (a.sp_ptr != nullptr || mode == QG_MODE_ACC32) return hipErrorInvalidValue;
  if (mode == QG_MODE_REQUANT) {
    switch (kernel) {
      case QG_KERNEL_SKINNY16: return launch_af32<QG_MODE_REQUANT, 1, 16, 4>(a, s);
      case QG_KERNEL_SKINNY32: return launch_af32<QG_MODE_REQUANT, 2, 16, 4>(a, s);
      case QG_KERNEL_SKINNY64: return launch_af32<QG_MODE_REQUANT, 4, 16, 2>(a, s);
      default: return hipErrorInvalidValue;
    }
  }
  switch (kernel) {
    case QG_KERNEL_SKINNY16: return launch_af32<QG_MODE_DEQUANT, 1, 16, 4>(a, s);
    case QG_KERNEL_SKINNY32: return launch_af32<QG_MODE_DEQUANT, 2, 16, 4>(a, s);
    case QG_KERNEL_SKINNY64: return launch_af32<QG_MODE_DEQUANT, 4, 16, 2>(a, s);
    default: return hipErrorInvalidValue;
  }
}

hipError_t qg_launch_gemm_skinny(const qg_gemm_args& a, int mode, int kernel, hipStream_t s) {
  // a.sp_ptr != null: Bp holds the 4-bit part of an outlier-split matrix
  if (a.a_vec) return a.sp_ptr != nullptr ? launch_mode<true, false>(a, mode, kernel, s) : launch_mode<false, false>(a, mode, kernel, s);
  return a.sp_ptr != nullptr ? launch_mode<true, true>(a, mode, kernel, s) : launch_mode<false, true>(a, mode, kernel, s);
}
