"""GPU parity of the shape-specific kernel family (paper Appendix C): every kernel id must compute every
shape, bit-identical to the CPU oracle; the dispatch table only chooses which one runs."""
import numpy as np
import pytest

from paper_2101_05615_amd import workloads as wl
from gpu_util import assert_same, dev_case, oracle_gemm, say

pytestmark = pytest.mark.gpu

KERNELS = ["skinny16", "skinny32", "skinny64", "tile64", "tile128", "tile128x256", "tile256", "tile64k4", "tile64k1", "tile64x32k8"]

# (M, N, K): 1, 2, 3, 4 and many 64-deep tiles on the pipelined paths (K % 64 == 0), ragged M and N that
# span several tiles of every shape, and a ragged K that takes the general path
SHAPES = [(257, 130, 64), (130, 257, 128), (70, 64, 192), (100, 300, 256), (300, 520, 1024), (515, 260, 448),
          (130, 100, 100), (1, 1, 64)]


@pytest.fixture(scope="module")
def env():
    import torch
    assert torch.cuda.is_available(), "these tests need the MI355X"
    from paper_2101_05615_amd import qgemm as q
    import oracle
    oracle.build()
    return q, torch, torch.device("cuda:0"), oracle


@pytest.fixture(scope="module")
def cases(env):
    """One seeded case per shape with its oracle results, shared by all kernels."""
    _, _, _, oracle = env
    out = {}
    for (M, N, K) in SHAPES:
        c = wl.unsaturated(wl.random_gemm(1000 + M + 3 * N + 7 * K, M, N, K, per_channel=True, with_bias=True,
                                          wide_zp=True))
        out[(M, N, K)] = (c, oracle_gemm(c, oracle), oracle.acc32(c.A, c.B), oracle.rowsum(c.A))
    return out


def test_kernel_names(env):
    q = env[0]
    names = q.kernel_names()
    assert names[0] == "auto" and [names[i] for i in range(1, q.KERNEL_LAST + 1)] == KERNELS
    assert q.lib.qg_kernel_name(q.KERNEL_CONV_LAST + 1) is None and q.lib.qg_kernel_name(-1) is None


@pytest.mark.parametrize("shape", SHAPES, ids=lambda s: "x".join(map(str, s)))
@pytest.mark.parametrize("kernel", KERNELS)
def test_every_kernel_bit_exact_on_every_shape(env, cases, kernel, shape):
    q, torch, dev, oracle = env
    c, want, want_acc, want_rs = cases[shape]
    say(f"kernel {kernel} shape {shape}")
    A, B, bias, scales, C, c_store = dev_case(c, torch, dev)
    Bp = q.pack_b(B, c.b_zp)
    q.gemm_u8s8_requant(A, c.a_zp, Bp, bias, scales, c.c_zp, c.relu, out=C, kernel=kernel)
    acc, rs = q.gemm_u8s8_acc32(A, Bp, want_rowsum=True, kernel=kernel)
    torch.cuda.synchronize()
    assert_same(C.cpu().numpy(), want, f"{kernel} requant")
    assert_same(acc.cpu().numpy(), want_acc, f"{kernel} acc32")
    assert_same(rs.cpu().numpy(), want_rs, f"{kernel} rowsum")
    tail = c_store.cpu().numpy()[c.M * c.N:]
    assert (tail == 0xEE).all(), "bytes past C were written"


@pytest.mark.parametrize("kernel", KERNELS)
def test_every_kernel_without_row_offsets(env, kernel):
    """theta_B == 0 everywhere: the variants that skip the row-offset term."""
    q, torch, dev, oracle = env
    c = wl.unsaturated(wl.random_gemm(5, 200, 264, 512, per_channel=True, with_bias=True))
    c.b_zp[:] = 0
    want = oracle_gemm(c, oracle)
    A, B, bias, scales, C, _ = dev_case(c, torch, dev)
    Bp = q.pack_b(B, c.b_zp)
    q.gemm_u8s8_requant(A, c.a_zp, Bp, bias, scales, c.c_zp, c.relu, out=C, kernel=kernel)
    torch.cuda.synchronize()
    assert_same(C.cpu().numpy(), want, f"{kernel} requant, theta_B = 0")


@pytest.mark.parametrize("kernel", KERNELS)
def test_every_kernel_unaligned(env, kernel):
    q, torch, dev, oracle = env
    c = wl.unsaturated(wl.random_gemm(6, 150, 140, 256, per_channel=False, with_bias=False, wide_zp=True))
    want = oracle_gemm(c, oracle)
    A, B, bias, scales, C, _ = dev_case(c, torch, dev, lda_pad=3, ldc_pad=5, a_off=1, c_off=3)
    Bp = q.pack_b(B, c.b_zp)
    q.gemm_u8s8_requant(A, c.a_zp, Bp, bias, scales, c.c_zp, c.relu, out=C, kernel=kernel)
    torch.cuda.synchronize()
    assert_same(C.cpu().numpy(), want, f"{kernel} unaligned")


@pytest.mark.parametrize("M,N,K,lda_pad", [(257, 130, 100, 12), (150, 200, 1000, 8), (70, 64, 37, 11),
                                           (300, 260, 464, 0), (130, 96, 336, 16), (40, 48, 4, 12)])
@pytest.mark.parametrize("kernel", KERNELS)
def test_every_kernel_ragged_k_on_aligned_rows(env, kernel, M, N, K, lda_pad):
    """16-byte aligned rows with K % 64 != 0 (whole 16-byte chunks past K, a chunk cut by K, K below one tile):
    the pipelined kernels run the whole tiles as usual and stage the ragged last tile with a byte mask."""
    q, torch, dev, oracle = env
    assert (K + lda_pad) % 16 == 0
    say(f"kernel {kernel} ragged K {M}x{N}x{K} lda {K + lda_pad}")
    c = wl.unsaturated(wl.random_gemm(7000 + M + K, M, N, K, per_channel=True, with_bias=True, wide_zp=True))
    want = oracle_gemm(c, oracle)
    A, B, bias, scales, C, _ = dev_case(c, torch, dev, lda_pad=lda_pad)
    Bp = q.pack_b(B, c.b_zp)
    q.gemm_u8s8_requant(A, c.a_zp, Bp, bias, scales, c.c_zp, c.relu, out=C, kernel=kernel)
    acc, rs = q.gemm_u8s8_acc32(A, Bp, want_rowsum=True, kernel=kernel)
    torch.cuda.synchronize()
    assert_same(C.cpu().numpy(), want, f"{kernel} requant")
    assert_same(acc.cpu().numpy(), oracle.acc32(c.A, c.B), f"{kernel} acc32")
    assert_same(rs.cpu().numpy(), oracle.rowsum(c.A), f"{kernel} rowsum")


def test_dispatch_rules_choose_the_kernel_and_never_the_result(env, cases):
    q, torch, dev, oracle = env
    shape = (300, 520, 1024)
    c, want, _, _ = cases[shape]
    A, B, bias, scales, C, _ = dev_case(c, torch, dev)
    Bp = q.pack_b(B, c.b_zp)
    builtin = q.kernel_select(*shape)
    try:
        for name in KERNELS:
            q.dispatch_set_rules([(257, 1000, 1, 1 << 30, 1, 1 << 30, name)])
            assert q.kernel_names()[q.kernel_select(*shape)] == name
            assert q.kernel_select(256, 520, 1024) == q.kernel_id(q.kernel_names()[q.kernel_select(256, 520, 1024)])
            C.fill_(0xEE)
            q.gemm_u8s8_requant(A, c.a_zp, Bp, bias, scales, c.c_zp, c.relu, out=C)  # auto
            torch.cuda.synchronize()
            assert_same(C.cpu().numpy(), want, f"auto -> {name}")
    finally:
        q.dispatch_set_rules([])
    assert q.kernel_select(*shape) == builtin


def test_unknown_kernel_id_is_rejected(env, cases):
    import ctypes
    q, torch, dev, oracle = env
    c, _, _, _ = cases[(70, 64, 192)]
    A, B, bias, scales, C, _ = dev_case(c, torch, dev)
    Bp = q.pack_b(B, c.b_zp)
    p = q.RequantParams(c.a_zp, None, scales.data_ptr(), scales.numel(), c.c_zp, 0)
    for bad in (-1, q.KERNEL_LAST + 1, 100):
        rc = q.lib.qg_gemm_u8s8_requant_kernel(A.data_ptr(), c.M, A.stride(0), Bp.handle, ctypes.byref(p),
                                               C.data_ptr(), C.stride(0), None, None, bad)
        assert rc == q.EINVAL
    torch.cuda.synchronize()


@pytest.mark.parametrize("M,N,K,ksplit", [(16, 8192, 2048, 1), (5, 8200, 4096, 1), (1, 8192, 2048, 1), (40, 2752, 2048, 1),
                                          (16, 8200, 4096, 2), (9, 8192, 6144, 3), (16, 4128, 2048, 1),
                                          (70, 1000, 2048, 1), (640, 100, 4096, 2)])
def test_streaming_kernel_with_two_fragment_columns_per_wave(env, M, N, K, ksplit):
    """More than 128 super-blocks of 16 rows x 32 columns (and aligned rows, K a multiple of 2048): the 16-row
    streaming kernel runs its four-wave form with two fragment columns per wave.  N that cuts a super-block, several
    row blocks, one row, the smallest count that takes this form (129), many row blocks of few columns, and the K
    split across workgroups on top."""
    q, torch, dev, oracle = env
    say(f"wide streaming form {M}x{N}x{K} ksplit {ksplit}")
    c = wl.unsaturated(wl.random_gemm(8100 + M + N + K, M, N, K, per_channel=True, with_bias=True, wide_zp=True))
    want = oracle_gemm(c, oracle)
    A, B, bias, scales, C, c_store = dev_case(c, torch, dev)
    Bp = q.pack_b(B, c.b_zp)
    ws = q.gemm_workspace(M, Bp, "skinny16", ksplit)
    assert (ws is None) == (ksplit == 1)
    for rep in range(2):
        C.fill_(0xEE)
        q.gemm_u8s8_requant_splitk(A, c.a_zp, Bp, bias, scales, c.c_zp, c.relu, ws, "skinny16", ksplit, out=C)
        acc, rs = q.gemm_u8s8_acc32_splitk(A, Bp, ws, "skinny16", ksplit, want_rowsum=True)
        torch.cuda.synchronize()
        assert_same(C.cpu().numpy(), want, f"requant (call {rep})")
        assert_same(acc.cpu().numpy(), oracle.acc32(c.A, c.B), f"acc32 (call {rep})")
        assert_same(rs.cpu().numpy(), oracle.rowsum(c.A), f"rowsum (call {rep})")
    assert (c_store.cpu().numpy()[M * N:] == 0xEE).all(), "bytes past C were written"


@pytest.mark.parametrize("kernel,M,N,K,ksplit", [("skinny32", 32, 8192, 2048, 1), ("skinny32", 19, 4140, 4096, 1), ("skinny32", 70, 2100, 2048, 1),
                                                 ("skinny32", 32, 8200, 4096, 2), ("skinny64", 64, 8192, 2048, 1), ("skinny64", 33, 4128, 4096, 1),
                                                 ("skinny64", 200, 1100, 2048, 1), ("skinny64", 64, 4200, 6144, 3), ("skinny64", 2200, 100, 4096, 2)])
def test_taller_streaming_kernels_with_two_fragment_columns_per_wave(env, kernel, M, N, K, ksplit):
    """The same form of the 32- and 64-row streaming kernels (four waves with batches of eight k blocks, eight waves
    with batches of four): more than 128 super-blocks, N that cuts a super-block, ragged and several row blocks, the
    smallest count that takes the form, and the K split across workgroups on top."""
    q, torch, dev, oracle = env
    say(f"wide streaming form {kernel} {M}x{N}x{K} ksplit {ksplit}")
    c = wl.unsaturated(wl.random_gemm(8300 + M + N + K, M, N, K, per_channel=True, with_bias=True, wide_zp=True))
    want = oracle_gemm(c, oracle)
    A, B, bias, scales, C, c_store = dev_case(c, torch, dev)
    Bp = q.pack_b(B, c.b_zp)
    ws = q.gemm_workspace(M, Bp, kernel, ksplit)
    assert (ws is None) == (ksplit == 1)
    for rep in range(2):
        C.fill_(0xEE)
        q.gemm_u8s8_requant_splitk(A, c.a_zp, Bp, bias, scales, c.c_zp, c.relu, ws, kernel, ksplit, out=C)
        acc, rs = q.gemm_u8s8_acc32_splitk(A, Bp, ws, kernel, ksplit, want_rowsum=True)
        torch.cuda.synchronize()
        assert_same(C.cpu().numpy(), want, f"requant (call {rep})")
        assert_same(acc.cpu().numpy(), oracle.acc32(c.A, c.B), f"acc32 (call {rep})")
        assert_same(rs.cpu().numpy(), oracle.rowsum(c.A), f"rowsum (call {rep})")
    assert (c_store.cpu().numpy()[M * N:] == 0xEE).all(), "bytes past C were written"
