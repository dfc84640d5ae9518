#!/usr/bin/env python3
"""Writes tile_loop_asm.inc: the software-pipelined main loop of the large-tile GEMM kernel as one
inline-asm string.

Why assembly: with one wave per SIMD (256 accumulator registers per wave) nothing but the order of the
instruction stream hides LDS and memory latency, and the compiler's scheduler clusters LDS reads, VALU
work and tile requests instead of spreading them behind the MFMAs.  Measured on MI355X, each
v_mfma_i32_32x32x32_i8 occupies the matrix pipe for 32 cycles, in whose shadow up to seven other
instructions of the same wave can issue for free; v_dot4 is NOT free (it shares the pipe), v_sad_u8 is.

Fixed register plan (all clobbered by the asm statement):
  v[160:175] A fragments set 0   v[176:191] B fragments set 0
  v[192:207] A fragments set 1   v[208:223] B fragments set 1
  v[224:227] row-sum accumulators (raw uint8 byte sums)
  v[228:231] per-lane byte offsets of the 4 A tile requests, v[232:235] of the 4 B tile requests
  v236/v237  per-lane LDS offsets of the A fragment for k-step 0 / 1, v238 of the B fragment
  v240/v241  LDS read addresses (stage base added)
  s84 xor mask, s[86:87] A request base, s[88:89] B request base, s90 loop counter, s91 LDS base of
  this wave's request slots, s92 LDS base, s99 bytes per 64-deep slab of packed B, s93 stage index, s96 request stage base, s97/s98 read
  stage bases (current / next), s94/s95 temporaries
Operands: 16 accumulators c0..c15 ("+a", acc[mb][nb] = c{4*mb+nb}), packed 64-bit VGPR inputs
av01 av23 bv01 bv23 ard brd, SGPR inputs aptr bptr kt ldsdma lds bstep, 64-bit VGPR outputs rs01 rs23.

Two configurations are generated from the same schedule: TM x TN = 4 x 4 blocks per wave (256 x 256 workgroup
tile, the plan above) and 2 x 2 (128 x 128 tile: 4 accumulators c0..c3, inputs av01 bv01 ard brd, output rs01,
fixed registers from v96, 16 KiB stages).  With only four MFMAs per k-step the LDS reads sit behind the first
two and the row sums and shifts of both A fragments behind the last two.  A third one, 2 x 4 blocks (128 x 256
tile: 8 accumulators, three 24 KiB stages so that two workgroups share a CU, fixed registers from v56, one more
SGPR input bofs = distance from a wave's A request slots to its B request slots), has eight MFMAs per k-step.

CONV variants (2 x 2 and 2 x 4): the A side of a dense convolution with the im2col folded into the requests.
Tile kt is 64 channels of one filter tap (Cin % 64 == 0, at most 32 taps); a lane's chunk comes from the image at
(its pixel's byte offset at tap (0, 0)) + (tap offset, kept on the scalar unit), or, when that tap of its pixel
lies outside the image, from a constant row of theta_A bytes -- so the tile that lands in the stage is the im2col
tile itself and everything behind the request is the GEMM's loop.  Requests take a 64-bit per-lane address
(v[lo:hi], off): lo = image_lo + offset or row_lo, hi = image_hi or row_hi (the host checks that the image does
not straddle a 4 GiB line, the row table is aligned so that it cannot).  Per request: add, and, compare, two
selects.  Extra fixed registers (after VB): CT..CT+3 address temporaries (two even-aligned pairs), APIX, APIX+1
per-lane pixel offsets (request q pre-biased by -q KiB, like the table rows: the instruction offset q*1024 moves
the global address too), AMASK, AMASK+1 per-lane tap-validity bits, TABLO, TABLO+1, TABHI, IMGHI wave-uniform
address parts.  Extra SGPRs s72..s81: image_lo + tap offset, channel slice, slices per tap, kw, S, row jump
((W - S) pixels), tap bit, temporary, tap jump (pixel bytes - Cin), temporary.  Inputs apix01 amask01 (64-bit
VGPR), aptr = image, tab = row of theta_A bytes (64-bit SGPR), nc, fs (S), rowjump, tapjump (SGPR); av01 is not used.
"""
import os

def configure(tm, tn, nstage=4, conv=False):
    """sets the module-level plan for TM x TN blocks of 32 x 32 per wave (2 x 2 waves per workgroup)"""
    global TM, TN, NM, A, B, RS, AV, BV, ARD0, ARD1, BRD, VA, VB, STAGE_BYTES, A_STAGE, A_DMA, N_DMA, NREAD, RSLOTS
    global FIRST_VGPR, LAST_VGPR, NSTAGE, CT, APIX, AMASK, TABLO, TABHI, IMGHI
    assert (tm, tn) in ((4, 4), (2, 2), (2, 4)) and nstage in (3, 4)
    TM, TN, NM, NSTAGE = tm, tn, tm * tn, nstage
    # (two waves per SIMD split the register file into 128 vector and 128 accumulator registers: v127 is the last
    # one, so the convolution variants, with twelve more fixed registers, start lower)
    base = {16: 160, 4: 66 if conv else 76, 8: 50 if conv else 56}[tm * tn]
    A = [base, base + 4 * (tm + tn)]
    B = [base + 4 * tm, base + 4 * (tm + tn) + 4 * tm]
    RS = base + 8 * (tm + tn)                       # TM row-sum accumulators
    AV = RS + 4                                     # per-lane offsets of the A requests
    BV = AV + 4                                     # ... of the B requests (only the first is used: B is contiguous)
    ARD0, ARD1, BRD = BV + 4, BV + 5, BV + 6        # BRD is moved as a 64-bit pair
    VA, VB = BV + 8, BV + 9
    FIRST_VGPR, LAST_VGPR = base, 255 if tm == 4 else VB
    CT = VB + 1 + ((VB + 1) & 1)                    # CONV: even-aligned address pairs of the two A requests
    APIX, AMASK, TABLO, TABHI, IMGHI = CT + 4, CT + 6, CT + 8, CT + 10, CT + 11
    A_STAGE = tm * 4096                             # 64 * TM rows of 64 bytes
    STAGE_BYTES = (tm + tn) * 4096
    A_DMA = tm                                      # 1 KiB requests per wave and tile: TM for A, then TN for B
    N_DMA = tm + tn
    NREAD = tm + tn                                 # LDS reads per k-step
    RSLOTS = (NREAD + 1) // 2                       # slots that carry them, two each


configure(4, 4)


def vr(base, n=4):
    return f"v[{base}:{base + n - 1}]"


class Emit:
    def __init__(self):
        self.lines = []

    def __call__(self, s):
        self.lines.append(s)

    def text(self):
        return "".join(f'    "{l}\\n"\n' for l in self.lines)


def dma(e, q):
    """one tile request: q = 0..A_DMA-1 A, then B; m0 = request stage base + slot"""
    # The instruction offset is added to the global address AND to the LDS address, so one M0 value serves the
    # four requests of a group; the per-lane A offsets come in pre-biased by -q*1024 (B is contiguous anyway).
    if q == 0:
        e("s_mov_b32 m0, s96")
        e("s_nop 0")
    if q == A_DMA:
        # B slots of this wave: A_STAGE further when a wave requests as many KiB of B as of A; otherwise the
        # distance is wave dependent and comes in as an operand (s85)
        e(f"s_add_u32 m0, s96, {A_STAGE}" if TM == TN else "s_add_u32 m0, s96, s85")
        e("s_nop 0")
    if q < A_DMA and CONV:
        lo, hi = CT + 2 * q, CT + 2 * q + 1
        e(f"v_add_u32 v{lo}, s72, v{APIX + q}")
        e(f"v_and_b32 v{hi}, s78, v{AMASK + q}")
        e(f"v_cmp_ne_u32 vcc, 0, v{hi}")
        e(f"v_cndmask_b32 v{lo}, v{TABLO + q}, v{lo}, vcc")
        e(f"v_cndmask_b32 v{hi}, v{TABHI}, v{IMGHI}, vcc")
        e(f"global_load_lds_dwordx4 v[{lo}:{hi}], off" + (f" offset:{q * 1024}" if q else ""))
    elif q < A_DMA:
        e(f"global_load_lds_dwordx4 v{AV + q}, s[86:87]" + (f" offset:{q * 1024}" if q else ""))
    else:
        e(f"global_load_lds_dwordx4 v{BV}, s[88:89]" + (f" offset:{(q - A_DMA) * 1024}" if q > A_DMA else ""))


def advance_request_pointers(e):
    if CONV:
        # next 64-channel slice; past the last slice of a tap the next tap of the filter row is (pixel bytes - Cin)
        # further (0 unless the channels are a slice of wider pixels), past the last tap of a filter row the next
        # image row (W - S) pixels further
        e("s_add_u32 s72, s72, 64")
        e("s_add_u32 s73, s73, 1")
        e("s_cmp_eq_u32 s73, s74")
        e("s_cselect_b32 s79, 1, 0")
        e("s_cselect_b32 s73, 0, s73")
        e("s_cselect_b32 s81, s80, 0")
        e("s_add_u32 s72, s72, s81")
        e("s_lshl_b32 s78, s78, s79")
        e("s_add_u32 s75, s75, s79")
        e("s_cmp_eq_u32 s75, s76")
        e("s_cselect_b32 s75, 0, s75")
        e("s_cselect_b32 s79, s77, 0")
        e("s_add_u32 s72, s72, s79")
    else:
        e("s_add_u32 s86, s86, 64")
        e("s_addc_u32 s87, s87, 0")
    e("s_add_u32 s88, s88, s99")
    e("s_addc_u32 s89, s89, 0")


def mfma(e, i, use):
    mb, nb = i // TN, i % TN
    e(f"v_mfma_i32_32x32x32_i8 %[c{i}], {vr(B[use] + 4 * nb)}, {vr(A[use] + 4 * mb)}, %[c{i}]")


def reads(e, slot, ld, ks):
    """the two LDS reads of slot 0..RSLOTS-1: A fragments first (they are needed first), then B"""
    for j in (2 * slot, 2 * slot + 1):
        if j >= NREAD:
            continue
        if j < TM:
            e(f"ds_read_b128 {vr(A[ld] + 4 * j)}, v{VA} offset:{j * 2048}")
        else:
            nb = j - TM
            e(f"ds_read_b128 {vr(B[ld] + 4 * nb)}, v{VB} offset:{nb * 2048 + ks * 512}")


ROWSUM = True  # False: variant for weights whose zero points are all 0 (no row offsets needed)
CONV = False   # True: the A requests of a dense convolution (see the module text)


def prep_slots():
    """(first slot, slots per A fragment) of the row-sum / shift work of a k-step: the last 2*TM slots with the
    byte sums and the xor of a fragment in separate slots, or -- when the reads leave fewer -- the last TM slots
    with both in one"""
    per = 2 if NM - RSLOTS >= 2 * TM else 1
    return NM - per * TM, per


def prep(e, slot, ld):
    """fragment f = (slot - first) // per; two slots per fragment: byte sums, then xor; one slot: both"""
    first, per = prep_slots()
    f, part = (slot - first) // per, (slot - first) % per
    base = A[ld] + 4 * f
    if part == 0:
        e(f"s_waitcnt lgkmcnt({NREAD - 1 - f})")
        for c in range(4):
            if ROWSUM:
                e(f"v_sad_u8 v{RS + f}, v{base + c}, 0, v{RS + f}")
    if part == per - 1:
        for c in range(4):
            e(f"v_xor_b32 v{base + c}, s84, v{base + c}")


def step(e, use, ks_load, request, next_va, load=True):
    """TM*TN MFMAs on fragment set `use`; meanwhile fetch the next k-step's fragments into the other set
    (k-step ks_load of the stage VA/VB point at), row-sum and shift its A fragments, and optionally
    issue the tile requests.  next_va: which A offset (0/1) the NEXT step's reads use."""
    ld = 1 - use
    for slot in range(NM):
        mfma(e, slot, use)
        if load and slot < RSLOTS:
            reads(e, slot, ld, ks_load)
        if request and slot < N_DMA:
            dma(e, slot)
        if load and slot >= prep_slots()[0]:
            prep(e, slot, ld)
        if slot == RSLOTS + 1 and next_va is not None:
            # all reads of this step are issued: point v240/v241 at the next step's fragments
            e(f"v_add_u32 v{VA}, s98, v{ARD0 if next_va == 0 else ARD1}")
            if next_va == 0:
                e(f"v_add_u32 v{VB}, s98, v{BRD}")


def wrap_stage(e, reg):
    """reg = reg mod NSTAGE for reg in 0..NSTAGE"""
    if NSTAGE == 4:
        e(f"s_and_b32 {reg}, {reg}, 3")
    else:
        e(f"s_cmp_eq_u32 {reg}, {NSTAGE}")
        e(f"s_cselect_b32 {reg}, 0, {reg}")


def stage_offset(e, dst, src):
    """dst = src * STAGE_BYTES"""
    if STAGE_BYTES & (STAGE_BYTES - 1) == 0:
        e(f"s_lshl_b32 {dst}, {src}, {STAGE_BYTES.bit_length() - 1}")
    else:
        e(f"s_mul_i32 {dst}, {src}, {STAGE_BYTES}")


def rotate_stage(e):
    """end of a tile: stage index += 1 (mod NSTAGE); recompute the read bases"""
    e("s_add_u32 s93, s93, 1")
    wrap_stage(e, "s93")
    e("s_mov_b32 s97, s98")
    e("s_add_u32 s94, s93, 1")
    wrap_stage(e, "s94")
    stage_offset(e, "s94", "s94")
    e("s_add_u32 s98, s92, s94")


def tile(e, wait_vm, request, last=False):
    # k-step 0 of tile t: consume set 0, fetch (t, 1) into set 1 from the current stage
    step(e, use=0, ks_load=1, request=False, next_va=None if last else 0)
    if last:
        e("s_waitcnt lgkmcnt(0)")
        step(e, use=1, ks_load=0, request=False, next_va=None, load=False)
        return
    # every wave: its requests for tile t+1 have landed, its reads of tile t are done
    e(f"s_waitcnt vmcnt({wait_vm}) lgkmcnt(0)")
    e("s_barrier")
    if request:
        stage_offset(e, "s94", "s93")
        e("s_add_u32 s96, s91, s94")
    # k-step 1 of tile t: consume set 1, fetch (t+1, 0) into set 0 from the next stage
    step(e, use=1, ks_load=0, request=request, next_va=1)
    if request:
        advance_request_pointers(e)
    rotate_stage(e)
    e("s_waitcnt lgkmcnt(0)")


def generate_loop(rowsum, conv=False):
    global ROWSUM, CONV
    ROWSUM, CONV = rowsum, conv
    assert not conv or TM == 2
    e = Emit()
    # ---- unpack operands into the fixed registers
    if conv:
        e(f"v_mov_b64 v[{APIX}:{APIX + 1}], %[apix01]")
        e(f"v_mov_b64 v[{AMASK}:{AMASK + 1}], %[amask01]")
        e("s_mov_b64 s[72:73], %[tab]")
        e(f"v_mov_b32 v{TABLO}, s72")
        e("s_sub_u32 s72, s72, 1024")
        e(f"v_mov_b32 v{TABLO + 1}, s72")
        e(f"v_mov_b32 v{TABHI}, s73")
        e("s_mov_b64 s[72:73], %[aptr]")
        e(f"v_mov_b32 v{IMGHI}, s73")
        e("s_mov_b32 s73, 0")
        e("s_mov_b32 s74, %[nc]")
        e("s_mov_b32 s75, 0")
        e("s_mov_b32 s76, %[fs]")
        e("s_mov_b32 s77, %[rowjump]")
        e("s_mov_b32 s78, 1")
        e("s_mov_b32 s80, %[tapjump]")
    else:
        e(f"v_mov_b64 v[{AV}:{AV + 1}], %[av01]")
    if TM == 4:
        e(f"v_mov_b64 v[{AV + 2}:{AV + 3}], %[av23]")
    e(f"v_mov_b64 v[{BV}:{BV + 1}], %[bv01]")
    if TM == 4:
        e(f"v_mov_b64 v[{BV + 2}:{BV + 3}], %[bv23]")
    e(f"v_mov_b64 v[{ARD0}:{ARD1}], %[ard]")
    e(f"v_mov_b64 v[{BRD}:{BRD + 1}], %[brd]")
    e("s_mov_b32 s84, 0x80808080")
    if TM != TN:
        e("s_mov_b32 s85, %[bofs]")
    if not conv:
        e("s_mov_b64 s[86:87], %[aptr]")
    e("s_mov_b64 s[88:89], %[bptr]")
    e(f"s_sub_u32 s90, %[kt], {NSTAGE}")
    e("s_mov_b32 s91, %[ldsdma]")
    e("s_mov_b32 s92, %[lds]")
    e("s_mov_b32 s99, %[bstep]")
    for f in range(TM):
        e(f"v_mov_b32 v{RS + f}, 0")
    # ---- request tiles 0..NSTAGE-1 into stages 0..NSTAGE-1
    for st in range(NSTAGE):
        e(f"s_add_u32 s96, s91, {st * STAGE_BYTES}")
        for q in range(N_DMA):
            dma(e, q)
        advance_request_pointers(e)
    e("s_mov_b32 s93, 0")
    e("s_mov_b32 s97, s92")
    e(f"s_add_u32 s98, s92, {STAGE_BYTES}")
    e(f"s_waitcnt vmcnt({(NSTAGE - 1) * N_DMA})")
    e("s_barrier")
    # ---- fragments (0, 0) into set 0
    e(f"v_add_u32 v{VA}, s97, v{ARD0}")
    e(f"v_add_u32 v{VB}, s97, v{BRD}")
    for slot in range(RSLOTS):
        reads(e, slot, 0, 0)
    for f in range(TM):
        e(f"s_waitcnt lgkmcnt({NREAD - 1 - f})")
        for c in range(4):
            if ROWSUM:
                e(f"v_sad_u8 v{RS + f}, v{A[0] + 4 * f + c}, 0, v{RS + f}")
        for c in range(4):
            e(f"v_xor_b32 v{A[0] + 4 * f + c}, s84, v{A[0] + 4 * f + c}")
    e("s_waitcnt lgkmcnt(0)")
    e(f"v_add_u32 v{VA}, s97, v{ARD1}")
    e("s_nop 1")
    # ---- steady state: KT-NSTAGE tiles, each requesting tile t+NSTAGE
    e("s_cmp_eq_u32 s90, 0")
    e("s_cbranch_scc1 2f")
    e("1:")
    tile(e, (NSTAGE - 2) * N_DMA, request=True)
    e("s_sub_u32 s90, s90, 1")
    e("s_cmp_lg_u32 s90, 0")
    e("s_cbranch_scc1 1b")
    e("2:")
    # ---- drain: nothing left to request; the tiles still in flight are fewer with every tile
    for younger in range(NSTAGE - 2, -1, -1):
        tile(e, younger * N_DMA, request=False)
    tile(e, 0, request=False, last=True)
    # ---- results: let the last MFMAs retire, hand the row sums back
    e("s_nop 15")
    e("s_nop 15")
    e("s_nop 15")
    e(f"v_mov_b64 %[rs01], v[{RS}:{RS + 1}]")
    if TM == 4:
        e(f"v_mov_b64 %[rs23], v[{RS + 2}:{RS + 3}]")
    return e.lines


def generate():
    out = "// GENERATED by gen_tile_loop.py -- do not edit.\n"
    for tm, tn, nstage, suffix in ((4, 4, 4, ""), (2, 2, 4, "_2X2"), (2, 4, 3, "_2X4")):
        configure(tm, tn, nstage)
        clob = [f'"v{i}"' for i in range(FIRST_VGPR, LAST_VGPR + 1)] + [f'"s{i}"' for i in range(84, 100)] + \
               ['"scc"', '"memory"']
        for name, rowsum in (("QG_TILE_LOOP_ASM", True), ("QG_TILE_LOOP_ASM_NOROWSUM", False)):
            out += (f"#define {name}{suffix} \\\n" +
                    "".join(f'  "{l}\\n" \\\n' for l in generate_loop(rowsum)) + "  \"\"\n")
        out += f"#define QG_TILE_LOOP_CLOBBERS{suffix} " + ", ".join(clob) + "\n"
        if tm == 2:
            configure(tm, tn, nstage, conv=True)
            clob = [f'"v{i}"' for i in range(FIRST_VGPR, IMGHI + 1)] + [f'"s{i}"' for i in range(72, 82)] + \
                   [f'"s{i}"' for i in range(84, 100)] + ['"vcc"', '"scc"', '"memory"']
            for name, rowsum in (("QG_TILE_LOOP_ASM_CONV", True), ("QG_TILE_LOOP_ASM_CONV_NOROWSUM", False)):
                out += (f"#define {name}{suffix} \\\n" +
                        "".join(f'  "{l}\\n" \\\n' for l in generate_loop(rowsum, conv=True)) + "  \"\"\n")
            out += f"#define QG_TILE_LOOP_CLOBBERS_CONV{suffix} " + ", ".join(clob) + "\n"
    configure(4, 4)
    return out


if __name__ == "__main__":
    here = os.path.dirname(os.path.abspath(__file__))
    with open(os.path.join(here, "tile_loop_asm.inc"), "w") as f:
        f.write(generate())
    print("wrote tile_loop_asm.inc")
