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
"""
import os

ABL = set(filter(None, os.environ.get("QG_GEN_ABL", "").split(",")))

A = [160, 192]
B = [176, 208]
RS, AV, BV, ARD0, ARD1, BRD, VA, VB = 224, 228, 232, 236, 237, 238, 240, 241
STAGE_BYTES = 32768      # A 256x64 + B 256x64
A_STAGE = 16384
N_DMA = 8                # tile requests per wave per tile


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
    """one tile request: q = 0..3 A, 4..7 B; m0 = request stage base + slot"""
    if "nodma" in ABL:
        return
    if "m0each" in ABL:
        if q < 4:
            e(f"s_add_u32 m0, s96, {q * 1024}")
            e("s_nop 0")
            e(f"global_load_lds_dwordx4 v{AV + q}, s[86:87]")
        else:
            e(f"s_add_u32 m0, s96, {A_STAGE + (q - 4) * 1024}")
            e("s_nop 0")
            e(f"global_load_lds_dwordx4 v{BV + q - 4}, s[88:89]")
        return
    # The instruction offset is added to the global address AND to the LDS address, so one M0 value serves the
    # four requests of a group; the per-lane A offsets come in pre-biased by -q*1024 (B is contiguous anyway).
    if q == 0:
        e("s_mov_b32 m0, s96")
        e("s_nop 0")
    if q == 4:
        e(f"s_add_u32 m0, s96, {A_STAGE}")
        e("s_nop 0")
    if q < 4:
        e(f"global_load_lds_dwordx4 v{AV + q}, s[86:87]" + (f" offset:{q * 1024}" if q else ""))
    else:
        e(f"global_load_lds_dwordx4 v{BV}, s[88:89]" + (f" offset:{(q - 4) * 1024}" if q > 4 else ""))


def advance_request_pointers(e):
    e("s_add_u32 s86, s86, 64")
    e("s_addc_u32 s87, s87, 0")
    e("s_add_u32 s88, s88, s99")
    e("s_addc_u32 s89, s89, 0")


def mfma(e, i, use):
    mb, nb = i // 4, i % 4
    if "nomfma" in ABL:
        return
    e(f"v_mfma_i32_32x32x32_i8 %[c{i}], {vr(B[use] + 4 * nb)}, {vr(A[use] + 4 * mb)}, %[c{i}]")


def reads(e, slot, ld, ks):
    """the two LDS reads of slot 0..3: A fragments first (they are needed first), then B"""
    for j in (2 * slot, 2 * slot + 1):
        if "nolds" in ABL:
            continue
        if j < 4:
            e(f"ds_read_b128 {vr(A[ld] + 4 * j)}, v{VA} offset:{j * 2048}")
        else:
            nb = j - 4
            e(f"ds_read_b128 {vr(B[ld] + 4 * nb)}, v{VB} offset:{nb * 2048 + ks * 512}")


ROWSUM = True  # False: variant for weights whose zero points are all 0 (no row offsets needed)


def prep(e, slot, ld):
    """slots 8..15: fragment f = (slot-8)//2; even slot: byte sums, odd slot: xor"""
    f, odd = (slot - 8) // 2, (slot - 8) % 2
    if "novalu" in ABL:
        return
    base = A[ld] + 4 * f
    if not odd:
        e(f"s_waitcnt lgkmcnt({7 - f})")
        for c in range(4):
            if ROWSUM:
                e(f"v_sad_u8 v{RS + f}, v{base + c}, 0, v{RS + f}")
    else:
        for c in range(4):
            e(f"v_xor_b32 v{base + c}, s84, v{base + c}")


def step(e, use, ks_load, request, next_va, load=True):
    """16 MFMAs on fragment set `use`; meanwhile fetch the next k-step's fragments into the other set
    (k-step ks_load of the stage v240/v241 point at), row-sum and shift its A fragments, and optionally
    issue the 8 tile requests.  next_va: which A offset (0/1) the NEXT step's reads use."""
    ld = 1 - use
    for slot in range(16):
        mfma(e, slot, use)
        if load and slot < 4:
            reads(e, slot, ld, ks_load)
        if request and slot < 8:
            dma(e, slot)
        if load and slot >= 8:
            prep(e, slot, ld)
        if slot == 5 and next_va is not None:
            # all reads of this step are issued: point v240/v241 at the next step's fragments
            e(f"v_add_u32 v{VA}, s98, v{ARD0 if next_va == 0 else ARD1}")
            if next_va == 0:
                e(f"v_add_u32 v{VB}, s98, v{BRD}")


def rotate_stage(e):
    """end of a tile: stage index += 1 (mod 4); recompute the read bases"""
    e("s_add_u32 s93, s93, 1")
    e("s_and_b32 s93, s93, 3")
    e("s_mov_b32 s97, s98")
    e("s_add_u32 s94, s93, 1")
    e("s_and_b32 s94, s94, 3")
    e("s_lshl_b32 s94, s94, 15")
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
    if "nobar" not in ABL:
        e("s_barrier")
    if request:
        e("s_lshl_b32 s94, s93, 15")
        e("s_add_u32 s96, s91, s94")
    # k-step 1 of tile t: consume set 1, fetch (t+1, 0) into set 0 from the next stage
    step(e, use=1, ks_load=0, request=request, next_va=1)
    if request:
        advance_request_pointers(e)
    rotate_stage(e)
    e("s_waitcnt lgkmcnt(0)")


def generate_loop(rowsum):
    global ROWSUM
    ROWSUM = rowsum
    e = Emit()
    # ---- unpack operands into the fixed registers
    e(f"v_mov_b64 v[{AV}:{AV + 1}], %[av01]")
    e(f"v_mov_b64 v[{AV + 2}:{AV + 3}], %[av23]")
    e(f"v_mov_b64 v[{BV}:{BV + 1}], %[bv01]")
    e(f"v_mov_b64 v[{BV + 2}:{BV + 3}], %[bv23]")
    e(f"v_mov_b64 v[{ARD0}:{ARD1}], %[ard]")
    e(f"v_mov_b64 v[{BRD}:{BRD + 1}], %[brd]")
    e("s_mov_b32 s84, 0x80808080")
    e("s_mov_b64 s[86:87], %[aptr]")
    e("s_mov_b64 s[88:89], %[bptr]")
    e("s_sub_u32 s90, %[kt], 4")
    e("s_mov_b32 s91, %[ldsdma]")
    e("s_mov_b32 s92, %[lds]")
    e("s_mov_b32 s99, %[bstep]")
    for f in range(4):
        e(f"v_mov_b32 v{RS + f}, 0")
    # ---- request tiles 0..3 into stages 0..3
    for st in range(4):
        e(f"s_add_u32 s96, s91, {st * STAGE_BYTES}")
        for q in range(N_DMA):
            dma(e, q)
        advance_request_pointers(e)
    e("s_mov_b32 s93, 0")
    e("s_mov_b32 s97, s92")
    e(f"s_add_u32 s98, s92, {STAGE_BYTES}")
    e(f"s_waitcnt vmcnt({3 * N_DMA})")
    e("s_barrier")
    # ---- fragments (0, 0) into set 0
    e(f"v_add_u32 v{VA}, s97, v{ARD0}")
    e(f"v_add_u32 v{VB}, s97, v{BRD}")
    for slot in range(4):
        reads(e, slot, 0, 0)
    for f in range(4):
        e(f"s_waitcnt lgkmcnt({7 - f})")
        for c in range(4):
            if ROWSUM:
                e(f"v_sad_u8 v{RS + f}, v{A[0] + 4 * f + c}, 0, v{RS + f}")
        for c in range(4):
            e(f"v_xor_b32 v{A[0] + 4 * f + c}, s84, v{A[0] + 4 * f + c}")
    e("s_waitcnt lgkmcnt(0)")
    e(f"v_add_u32 v{VA}, s97, v{ARD1}")
    e("s_nop 1")
    # ---- steady state: KT-4 tiles, each requesting tile t+4
    e("s_cmp_eq_u32 s90, 0")
    e("s_cbranch_scc1 2f")
    e("1:")
    tile(e, 2 * N_DMA, request=True)
    e("s_sub_u32 s90, s90, 1")
    e("s_cmp_lg_u32 s90, 0")
    e("s_cbranch_scc1 1b")
    e("2:")
    # ---- drain: nothing left to request
    tile(e, 2 * N_DMA, request=False)
    tile(e, N_DMA, request=False)
    tile(e, 0, request=False)
    tile(e, 0, request=False, last=True)
    # ---- results: let the last MFMAs retire, hand the row sums back
    e("s_nop 15")
    e("s_nop 15")
    e("s_nop 15")
    e(f"v_mov_b64 %[rs01], v[{RS}:{RS + 1}]")
    e(f"v_mov_b64 %[rs23], v[{RS + 2}:{RS + 3}]")
    return e.lines


def generate():
    clob = [f'"v{i}"' for i in range(160, 256)] + [f'"s{i}"' for i in range(84, 100)] + \
           ['"scc"', '"memory"']
    out = "// GENERATED by gen_tile_loop.py -- do not edit.\n"
    for name, rowsum in (("QG_TILE_LOOP_ASM", True), ("QG_TILE_LOOP_ASM_NOROWSUM", False)):
        out += (f"#define {name} \\\n" +
                "".join(f'  "{l}\\n" \\\n' for l in generate_loop(rowsum)) + "  \"\"\n")
    out += "#define QG_TILE_LOOP_CLOBBERS " + ", ".join(clob) + "\n"
    return out


if __name__ == "__main__":
    here = os.path.dirname(os.path.abspath(__file__))
    with open(os.environ.get("QG_GEN_OUT", os.path.join(here, "tile_loop_asm.inc")), "w") as f:
        f.write(generate())
    print("wrote tile_loop_asm.inc")
