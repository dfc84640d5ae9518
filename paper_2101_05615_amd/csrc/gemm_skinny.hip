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
#include "qg_internal.h"
#include <type_traits>

namespace {

typedef int v4i __attribute__((ext_vector_type(4)));

// ANYALIGN: rows of A that are not 16-byte aligned.  The requests and vector loads take any address; the variant
// exists so that the aligned one keeps its code (and its timing) to the instruction.
template <int MODE, int MB, int NWAVES, int BATCH, bool B4, bool ANYALIGN>
__global__ __launch_bounds__(NWAVES * 64) void qg_gemm_skinny_kernel(const qg_gemm_args p) {
  const bool a_vec = ANYALIGN || p.a_vec;  // whole 16-byte chunks may be moved as such
  using chunk_t = typename std::conditional<ANYALIGN, qg_v4i_unaligned, v4i>::type;
  // A through LDS (see the file header): per wave and batch, ROWS rows x ROWB bytes
  constexpr int ROWS = MB * 16, ROWB = BATCH * QG_FRAG_K, NCHUNK = ROWB / 16;
  constexpr int REGION = ROWS * ROWB, NREQ = REGION / 1024, RPR = 64 / NCHUNK;  // requests per batch, rows per request
  static_assert(NCHUNK == 8 || NCHUNK == 16, "a request covers whole rows of 128 or 256 bytes");
  constexpr int PART_BYTES = NWAVES * MB * 64 * (int)sizeof(v4i);
  constexpr int RSP_BYTES = NWAVES * MB * 16 * (int)sizeof(int);
  constexpr int STAGE_BYTES = NWAVES * REGION;
  // the K-split partial sums reuse the staging regions once the main loop is over
  constexpr int UNION_BYTES = STAGE_BYTES > PART_BYTES ? STAGE_BYTES : PART_BYTES;
  extern __shared__ __align__(16) unsigned char smem[];
  v4i* part = reinterpret_cast<v4i*>(smem);                 // [wave][mb][lane]
  int* rsp = reinterpret_cast<int*>(smem + UNION_BYTES);    // [wave][mb][16]
  int* sp = reinterpret_cast<int*>(smem + UNION_BYTES + RSP_BYTES);  // B4: [row][slot] sparse term

  const int nb16 = blockIdx.x;
  const int sb = nb16 >> 1, sfrag = nb16 & 1;
  // columns held by this fragment: sb*32 + 16*(u&1) + 8*sfrag + 4*(u>>1) + r, u<4, r<4
  if (sb * 32 + 8 * sfrag >= p.N) return;  // nothing but padding (uniform for the workgroup)

  const int tid = threadIdx.x, lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int ml = lane & 15, g = lane >> 4;
  const int m_base = blockIdx.y * (MB * 16);  // first row of this workgroup's row block

  // the waves that run the output pipeline fetch its per-column constants now, not after the reduction
  const int c0 = sb * 32 + 16 * (g & 1) + 8 * sfrag + 4 * (g >> 1);  // this lane's 4 output columns
  int ep_co[4], ep_bz[4], ep_bias[4];
  float ep_sc[4];
  if (wave < MB) {
#pragma unroll
    for (int r = 0; r < 4; ++r) {
      const int col = c0 + r;  // col_off / bzp are padded to N_pad, bias / scales are not
      ep_co[r] = p.col_off[col];
      ep_bz[r] = p.bzp[col];
      ep_bias[r] = (MODE != QG_MODE_ACC32 && p.bias != nullptr && col < p.N) ? p.bias[col] : 0;
      ep_sc[r] = (MODE != QG_MODE_ACC32 && col < p.N) ? p.scales[(size_t)col * p.scale_stride] : 1.0f;
    }
  }

  if (B4) {
    for (int t = tid; t < MB * 256; t += NWAVES * 64) sp[t] = 0;
    __syncthreads();
  }

  // K slices are dealt to the waves rotated by the workgroup index, so that at any instant the workgroups
  // of an XCD read DIFFERENT lines of A (all of them read all of A; unrotated they would all hit the same
  // L2 channel at the same time)
  // (4-bit weights come in pairs of k blocks, so their slices hold an even number of blocks)
  const int per = B4 ? ((p.kb64 + 2 * NWAVES - 1) / (2 * NWAVES)) * 2 : (p.kb64 + NWAVES - 1) / NWAVES;
  const int kb_begin = ((wave + nb16) % NWAVES) * per;
  const int kb_end = min(p.kb64, kb_begin + per);

  // outlier split: the entry offsets of all of this wave's batches, one per lane (batch b: lanes b and b+1), are
  // requested before anything else so that no batch waits for an offset before it can ask for its entries
  int sp_offs = 0;
  if (B4 && kb_begin < kb_end) {
    const int32_t* col = p.sp_ptr + (size_t)nb16 * p.kb64;
    sp_offs = col[min(kb_begin + BATCH * lane, kb_end)];
  }

  v4i acc[MB];
  unsigned rs[MB];  // sums of raw uint8 bytes (K padding reads as 0x80)
#pragma unroll
  for (int mb = 0; mb < MB; ++mb) {
    acc[mb] = (v4i){0, 0, 0, 0};
    rs[mb] = 0;
  }
  // 8-bit: one 1 KiB fragment per k block, 16 bytes per lane.  4-bit: one 1 KiB unit per PAIR of k blocks, 16 bytes
  // per lane (8 for each block), so that a request moves as many bytes as in the 8-bit layout.
  const int8_t* bcol = p.Bp + (size_t)nb16 * QG_FRAG_BYTES + lane * 16;
  const size_t b_step = (size_t)p.nb16 * QG_FRAG_BYTES;  // one slab (8-bit: 64 deep, 4-bit: 128 deep) of the packed buffer

  // per-lane byte offsets of the NREQ activation requests of a batch (a.a_vec: they fit 32 bits); with them the
  // request address is a wave-uniform base plus a register that is never the target of a load, so issuing
  // the requests never has to wait for loads in flight
  unsigned a_off[NREQ];
#pragma unroll
  for (int jj = 0; jj < NREQ; ++jj) {
    const int r = jj * RPR + lane / NCHUNK;
    a_off[jj] = (unsigned)min(m_base + r, p.M - 1) * (unsigned)p.lda + ((unsigned)((lane ^ r) & (NCHUNK - 1)) << 4);
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
      raw[i] = *reinterpret_cast<const v4i*>(bcol + (size_t)(B4 ? kbi >> 1 : kbi) * b_step);
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
  auto batch = [&](int kb, const v4i (&cur)[NLOAD], v4i (&nxt)[NLOAD], const bool has_next) {
    // whole rows of BATCH k blocks are requested even when the slice ends earlier: the surplus lies inside the
    // row (it is the next wave's slice) and is simply not consumed
    const bool staged = a_vec && (kb + BATCH) * QG_FRAG_K <= p.K;
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
      const uint8_t* a_base = p.A + (size_t)kb * QG_FRAG_K;  // wave-uniform
#pragma unroll
      for (int jj = 0; jj < NREQ; ++jj)
        __builtin_amdgcn_global_load_lds((const __attribute__((address_space(1))) void*)(a_base + a_off[jj]),
                                         (__attribute__((address_space(3))) void*)(region + jj * 1024), 16, 0, 0);
      asm volatile("" ::: "memory");
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
#pragma unroll 1
      for (int i = lane; i < ROWS * nchunk; i += 64) {
        const int r = i / nchunk, lc = i % nchunk;     // row, logical chunk
        const int c = r * NCHUNK + ((lc ^ r) & (NCHUNK - 1));
        const int k0 = kb * QG_FRAG_K + (lc << 4);
        const uint8_t* src = p.A + (size_t)min(m_base + r, p.M - 1) * p.lda + k0;
        v4i v;
        if (a_vec && k0 + 16 <= p.K)
          v = *reinterpret_cast<const chunk_t*>(src);
        else
          v = qg_load_a_chunk(src, p.K - k0, false);  // byte by byte, bytes past K as 0x80
        *reinterpret_cast<v4i*>(region + c * 16) = v;
      }
      sparse_request();
      if (has_next) load_b(kb + BATCH, nxt);
    }
#pragma unroll
    for (int mb = 0; mb < MB; ++mb)
#pragma unroll
      for (int j = 0; j < BATCH; ++j) {
        const int r = mb * 16 + ml;
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
          acc[mb] = __builtin_amdgcn_mfma_i32_16x16x64_i8(bfj, a, acc[mb], 0, 0, 0);
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

  // two register sets alternate
  if (kb_begin < kb_end) {
    v4i braw0[NLOAD], braw1[NLOAD];
    load_b(kb_begin, braw0);
    for (int kb = kb_begin; kb < kb_end; kb += 2 * BATCH) {
      batch(kb, braw0, braw1, kb + BATCH < kb_end);
      if (kb + BATCH < kb_end) batch(kb + BATCH, braw1, braw0, kb + 2 * BATCH < kb_end);
    }
  }

  // ---- combine the 16 K-slices through LDS (the partial sums overwrite the staging regions: every wave must
  // be done with its own first)
  __syncthreads();
#pragma unroll
  for (int mb = 0; mb < MB; ++mb) {
    part[(wave * MB + mb) * 64 + lane] = acc[mb];
    int v = (int)rs[mb];
    v += __shfl_xor(v, 16);
    v += __shfl_xor(v, 32);
    if (g == 0) rsp[(wave * MB + mb) * 16 + ml] = v;
  }
  __syncthreads();
  if (wave >= MB) return;
  const int mb = wave;
  v4i sum = (v4i){0, 0, 0, 0};
  int rsum = -128 * (p.kb64 * QG_FRAG_K);  // every staged byte (padding included) is 128 above its int8 value
#pragma unroll
  for (int w = 0; w < NWAVES; ++w) {
    sum += part[(w * MB + mb) * 64 + lane];
    rsum += rsp[(w * MB + mb) * 16 + ml];
  }
  if (B4) {
    // A_s B = (A_s U - 8 rowsum(A_s)) + A_s B_sparse; lane (ml, g) register r is slot 4 g + r of the fragment
#pragma unroll
    for (int r = 0; r < 4; ++r) sum[r] += sp[(mb * 16 + ml) * 16 + 4 * g + r] - 8 * rsum;
  }

  // ---- output pipeline; lane (ml, u = g) holds row m_base+mb*16+ml, 4 consecutive columns
  const int row = m_base + mb * 16 + ml;
  if (row >= p.M || c0 >= p.N) return;
  if (MODE == QG_MODE_REQUANT) {
    unsigned out = 0;
#pragma unroll
    for (int r = 0; r < 4; ++r) {
      const int x = sum[r] + ep_bias[r] - p.a_zp_m128 * ep_co[r] - ep_bz[r] * rsum;
      out |= (unsigned)qg_requant_one(x, ep_sc[r], p.clamp_lo, p.clamp_hi, p.c_zp) << (8 * r);
    }
    uint8_t* dst = p.C + (size_t)row * p.ldc + c0;
    if (p.c_vec && c0 + 4 <= p.N) {
      *reinterpret_cast<unsigned*>(dst) = out;
    } else {
#pragma unroll
      for (int r = 0; r < 4; ++r)
        if (c0 + r < p.N) dst[r] = (uint8_t)(out >> (8 * r));
    }
  } else if (MODE == QG_MODE_DEQUANT) {
    float out[4];
#pragma unroll
    for (int r = 0; r < 4; ++r) {
      const int x = sum[r] + ep_bias[r] - p.a_zp_m128 * ep_co[r] - ep_bz[r] * rsum;
      out[r] = qg_dequant_one(x, ep_sc[r], p.relu_lo);
    }
    float* dst = p.Cf + (size_t)row * p.ldc + c0;
    if (p.c_vec && c0 + 4 <= p.N) {
      *reinterpret_cast<float4*>(dst) = make_float4(out[0], out[1], out[2], out[3]);
    } else {
#pragma unroll
      for (int r = 0; r < 4; ++r)
        if (c0 + r < p.N) dst[r] = out[r];
    }
  } else {
#pragma unroll
    for (int r = 0; r < 4; ++r) {
      const int col = c0 + r;
      if (col < p.N) p.C32[(size_t)row * p.ldc + col] = sum[r] + 128 * (ep_co[r] + p.K * ep_bz[r]);
    }
    if (p.rowsum_out != nullptr && nb16 == 0 && g == 0) p.rowsum_out[row] = rsum + 128 * p.K;
  }
}

template <int MODE, int MB, int NWAVES, int BATCH, bool B4, bool ANYALIGN>
hipError_t launch(const qg_gemm_args& a, hipStream_t s) {
  const int part = NWAVES * MB * 64 * (int)sizeof(v4i), stage = NWAVES * (MB * 16) * (BATCH * QG_FRAG_K);
  const int smem = (stage > part ? stage : part) + NWAVES * MB * 16 * (int)sizeof(int) +
                   (B4 ? MB * 256 * (int)sizeof(int) : 0);
  hipError_t e = qg_allow_smem<qg_gemm_skinny_kernel<MODE, MB, NWAVES, BATCH, B4, ANYALIGN>>(smem);
  if (e != hipSuccess) return e;
  const int nfrag = ((a.N + 31) / 32) * 2;
  const int mblocks = (a.M + MB * 16 - 1) / (MB * 16);
  if (mblocks > 65535) return hipErrorInvalidValue;
  hipLaunchKernelGGL((qg_gemm_skinny_kernel<MODE, MB, NWAVES, BATCH, B4, ANYALIGN>), dim3(nfrag, mblocks), dim3(NWAVES * 64), smem,
                     s, a);
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

hipError_t qg_launch_gemm_skinny(const qg_gemm_args& a, int mode, int kernel, hipStream_t s) {
  // a.sp_ptr != null: Bp holds the 4-bit part of an outlier-split matrix
  if (a.a_vec) return a.sp_ptr != nullptr ? launch_mode<true, false>(a, mode, kernel, s) : launch_mode<false, false>(a, mode, kernel, s);
  return a.sp_ptr != nullptr ? launch_mode<true, true>(a, mode, kernel, s) : launch_mode<false, true>(a, mode, kernel, s);
}
