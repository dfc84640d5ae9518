"""GPU parity of the K split ACROSS workgroups of the streaming kernels (the role of the paper's caller-provided
C_buffer, Appendix A): int32 partial tiles meet in a caller workspace, the last slice to arrive runs the output
pipeline.  Integer sums: every split factor must give the oracle's bytes, and every call must leave the workspace
ready for the next one."""
import ctypes

import numpy as np
import pytest

from paper_2101_05615_amd import workloads as wl
from gpu_util import assert_same, dev_case, oracle_gemm, say

pytestmark = pytest.mark.gpu

STREAMING = ["skinny16", "skinny32", "skinny64"]

# (M, N, K): few fragment columns and a long K (what the split is for), ragged K, N that cuts a fragment, M over
# several row blocks, the longest K the library takes
SHAPES = [(16, 64, 4096), (7, 100, 3000), (40, 36, 8192), (130, 48, 2500), (3, 16, 32768), (16, 256, 1024)]


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
    _, _, _, oracle = env
    out = {}
    for (M, N, K) in SHAPES:
        c = wl.unsaturated(wl.random_gemm(4000 + M + 3 * N + 7 * K, M, N, K, per_channel=True, with_bias=True,
                                          wide_zp=True))
        out[(M, N, K)] = (c, oracle_gemm(c, oracle), oracle.acc32(c.A, c.B), oracle.rowsum(c.A))
    return out


@pytest.mark.parametrize("shape", SHAPES, ids=lambda s: "x".join(map(str, s)))
@pytest.mark.parametrize("kernel", STREAMING)
def test_every_split_factor_gives_the_oracle_bytes(env, cases, kernel, shape):
    q, torch, dev, oracle = env
    c, want, want_acc, want_rs = cases[shape]
    A, B, bias, scales, C, c_store = dev_case(c, torch, dev)
    Bp = q.pack_b(B, c.b_zp)
    seen = set()
    for ksplit in (1, 2, 3, 4, 7, 16, 64):
        used = q.gemm_splitk_factor(c.M, Bp, kernel, ksplit)
        assert 1 <= used <= ksplit
        if used in seen:
            continue
        seen.add(used)
        say(f"kernel {kernel} shape {shape} ksplit {ksplit} -> {used}")
        ws = q.gemm_workspace(c.M, Bp, kernel, ksplit)
        assert (ws is None) == (used == 1)
        # twice on the same workspace: the first call must leave it as it found it
        for rep in range(2):
            C.fill_(0xEE)
            q.gemm_u8s8_requant_splitk(A, c.a_zp, Bp, bias, scales, c.c_zp, c.relu, ws, kernel, ksplit, out=C)
            acc, rs = q.gemm_u8s8_acc32_splitk(A, Bp, ws, kernel, ksplit, want_rowsum=True)
            torch.cuda.synchronize()
            assert_same(C.cpu().numpy(), want, f"{kernel} ksplit {used} requant (call {rep})")
            assert_same(acc.cpu().numpy(), want_acc, f"{kernel} ksplit {used} acc32 (call {rep})")
            assert_same(rs.cpu().numpy(), want_rs, f"{kernel} ksplit {used} rowsum (call {rep})")
        if ws is not None:
            assert int(ws.view(torch.int32)[:64].abs().sum().item()) == 0, "ticket counters not back at zero"
        tail = c_store.cpu().numpy()[c.M * c.N:]
        assert (tail == 0xEE).all(), "bytes past C were written"


def test_a_workspace_sized_for_a_large_batch_serves_a_smaller_one(env):
    q, torch, dev, oracle = env
    big = wl.unsaturated(wl.random_gemm(77, 48, 80, 4096, per_channel=True, with_bias=True, wide_zp=True))
    A, B, bias, scales, C, _ = dev_case(big, torch, dev)
    Bp = q.pack_b(B, big.b_zp)
    ws = q.gemm_workspace(big.M, Bp, "skinny16", 4)
    assert ws is not None
    want = oracle_gemm(big, oracle)
    q.gemm_u8s8_requant_splitk(A, big.a_zp, Bp, bias, scales, big.c_zp, big.relu, ws, "skinny16", 4, out=C)
    torch.cuda.synchronize()
    assert_same(C.cpu().numpy(), want, "48 rows")
    for m in (5, 17):
        out = q.gemm_u8s8_requant_splitk(A[:m], big.a_zp, Bp, bias, scales, big.c_zp, big.relu, ws, "skinny16", 4)
        torch.cuda.synchronize()
        assert_same(out.cpu().numpy(), want[:m], f"{m} rows on the larger workspace")


def test_unaligned_activations_and_output_with_a_split(env):
    q, torch, dev, oracle = env
    c = wl.unsaturated(wl.random_gemm(78, 20, 52, 3001, per_channel=False, with_bias=False, wide_zp=True))
    want = oracle_gemm(c, oracle)
    A, B, bias, scales, C, c_store = dev_case(c, torch, dev, lda_pad=3, ldc_pad=5, a_off=1, c_off=3)
    Bp = q.pack_b(B, c.b_zp)
    for kernel in STREAMING:
        ws = q.gemm_workspace(c.M, Bp, kernel, 5)
        q.gemm_u8s8_requant_splitk(A, c.a_zp, Bp, bias, scales, c.c_zp, c.relu, ws, kernel, 5, out=C)
        torch.cuda.synchronize()
        assert_same(C.cpu().numpy(), want, f"{kernel} unaligned, 5 slices")


def test_outlier_split_weights_with_a_k_split(env):
    """4-bit B' + sparse part (Sec. 2.2) and the K split together: slices hold whole pairs of 64-deep blocks."""
    q, torch, dev, oracle = env
    K, N, M = 4096 + 64, 72, 16
    Bn = wl.outlier_weights(5, K, N, outlier_frac=0.01)
    c = wl.random_gemm(79, M, N, K, per_channel=True, with_bias=True, wide_zp=True)
    c.B = Bn
    c = wl.unsaturated(c)
    want = oracle_gemm(c, oracle)
    A, _, bias, scales, C, _ = dev_case(c, torch, dev)
    Bp = q.pack_b_outlier(torch.from_numpy(Bn).to(dev), c.b_zp)
    for kernel in STREAMING:
        for ksplit in (2, 5):
            ws = q.gemm_workspace(M, Bp, kernel, ksplit)
            C.fill_(0xEE)
            q.gemm_u8s8_requant_splitk(A, c.a_zp, Bp, bias, scales, c.c_zp, c.relu, ws, kernel, ksplit, out=C)
            torch.cuda.synchronize()
            assert_same(C.cpu().numpy(), want, f"{kernel} split descriptor, {ksplit} slices")


def test_plain_call_splits_only_with_a_workspace_and_matches(env):
    """The plain entry point: NULL workspace never splits; with the workspace of qg_gemm_workspace_bytes the
    built-in choice may split; the bytes are the same."""
    q, torch, dev, oracle = env
    c = wl.unsaturated(wl.random_gemm(80, 16, 64, 16384, per_channel=True, with_bias=True, wide_zp=True))
    want = oracle_gemm(c, oracle)
    A, B, bias, scales, C, _ = dev_case(c, torch, dev)
    Bp = q.pack_b(B, c.b_zp)
    nbytes = q.gemm_workspace_bytes(c.M, Bp)
    say(f"auto workspace for 16x64x16384: {nbytes} bytes, split {q.gemm_splitk_factor(c.M, Bp)}")
    assert nbytes > 0 and q.gemm_splitk_factor(c.M, Bp) > 1
    q.gemm_u8s8_requant(A, c.a_zp, Bp, bias, scales, c.c_zp, c.relu, out=C)
    torch.cuda.synchronize()
    assert_same(C.cpu().numpy(), want, "no workspace")
    ws = torch.empty(nbytes, dtype=torch.uint8, device=dev)
    q._check(q.lib.qg_gemm_workspace_init(ws.data_ptr(), nbytes, None), "init")
    for rep in range(3):
        C.fill_(0xEE)
        q.gemm_u8s8_requant(A, c.a_zp, Bp, bias, scales, c.c_zp, c.relu, out=C, workspace=ws)
        torch.cuda.synchronize()
        assert_same(C.cpu().numpy(), want, f"auto split, call {rep}")


def test_split_argument_errors(env):
    q, torch, dev, oracle = env
    c = wl.random_gemm(81, 16, 64, 1024)
    A, B, bias, scales, C, _ = dev_case(c, torch, dev)
    Bp = q.pack_b(B, c.b_zp)
    p = q.RequantParams(c.a_zp, None, scales.data_ptr(), scales.numel(), c.c_zp, 0)

    def call(ws, nbytes, kernel, ksplit):
        return q.lib.qg_gemm_u8s8_requant_splitk(A.data_ptr(), c.M, A.stride(0), Bp.handle, ctypes.byref(p), C.data_ptr(),
                                                 C.stride(0), ws, nbytes, None, kernel, ksplit)

    need = q.lib.qg_gemm_splitk_workspace_bytes(c.M, Bp.handle, 1, 4)
    assert need > 0
    ws = torch.zeros(need, dtype=torch.uint8, device=dev)
    assert call(None, 0, 1, 4) == q.EWORKSPACE                      # needed, not given
    assert call(ws.data_ptr(), need - 4, 1, 4) == q.EWORKSPACE      # too small
    assert call(ws.data_ptr() + 4, need, 1, 4) == q.EALIGN
    assert call(ws.data_ptr(), need, 1, -1) == q.EINVAL
    assert call(ws.data_ptr(), need, 1, 65) == q.EINVAL
    assert call(ws.data_ptr(), need, q.kernel_id("tile64"), 2) == q.EUNSUPPORTED
    assert call(None, 0, 1, 1) == q.OK                               # one slice needs no workspace
    assert call(ws.data_ptr(), need, 1, 4) == q.OK
    torch.cuda.synchronize()
    assert q.lib.qg_gemm_splitk_workspace_bytes(c.M, Bp.handle, q.kernel_id("tile64"), 4) == 0
    # K = 1024 has 16 blocks of 64: a request for 64 slices is served with 16
    assert q.gemm_splitk_factor(c.M, Bp, "skinny16", 64) == 16


@pytest.mark.parametrize("M,N,K,ksplit,served", [(128, 128, 512, 2, 2), (300, 200, 1024, 4, 4), (130, 520, 2048, 3, 3), (256, 256, 640, 2, 2),
                                                 (64, 100, 8192, 8, 8), (200, 300, 768, 64, 3), (100, 64, 576, 2, 2)])
def test_k_split_across_workgroups_on_the_128_tile(env, M, N, K, ksplit, served):
    """The 128 x 128 tile with its K split over the second grid dimension (caller's choice only): slices of at least
    four 64-deep tiles, a last slice that is shorter, ragged M and N, more slices asked for than K has; twice per
    case (the counters go back to zero), uint8 result, raw accumulators and row sums against the oracle."""
    q, torch, dev, oracle = env
    say(f"tile128 K split {M}x{N}x{K} / {ksplit}")
    c = wl.unsaturated(wl.random_gemm(8500 + M + N + K, M, N, K, per_channel=True, with_bias=True, wide_zp=True))
    want = oracle_gemm(c, oracle)
    A, B, bias, scales, C, c_store = dev_case(c, torch, dev)
    Bp = q.pack_b(B, c.b_zp)
    assert q.gemm_splitk_factor(M, Bp, "tile128", ksplit) == served
    ws = q.gemm_workspace(M, Bp, "tile128", ksplit)
    for rep in range(2):
        C.fill_(0xEE)
        q.gemm_u8s8_requant_splitk(A, c.a_zp, Bp, bias, scales, c.c_zp, c.relu, ws, "tile128", ksplit, out=C)
        acc, rs = q.gemm_u8s8_acc32_splitk(A, Bp, ws, "tile128", ksplit, want_rowsum=True)
        torch.cuda.synchronize()
        assert_same(C.cpu().numpy(), want, f"requant (call {rep})")
        assert_same(acc.cpu().numpy(), oracle.acc32(c.A, c.B), f"acc32 (call {rep})")
        assert_same(rs.cpu().numpy(), oracle.rowsum(c.A), f"rowsum (call {rep})")
    assert (c_store.cpu().numpy()[M * N:] == 0xEE).all(), "bytes past C were written"


def test_128_tile_split_argument_errors(env):
    q, torch, dev, oracle = env
    c = wl.random_gemm(82, 130, 140, 1024)
    A, B, bias, scales, C, _ = dev_case(c, torch, dev)
    Bp = q.pack_b(B, c.b_zp)
    p = q.RequantParams(c.a_zp, None, scales.data_ptr(), scales.numel(), c.c_zp, 0)
    t128 = q.kernel_id("tile128")

    def call(ws, nbytes, kernel, ksplit):
        return q.lib.qg_gemm_u8s8_requant_splitk(A.data_ptr(), c.M, A.stride(0), Bp.handle, ctypes.byref(p), C.data_ptr(),
                                                 C.stride(0), ws, nbytes, None, kernel, ksplit)

    need = q.lib.qg_gemm_splitk_workspace_bytes(c.M, Bp.handle, t128, 4)
    assert need == (64 + 4 * 4 * 66 * 256) * 4      # 4 tiles: 64 counters, 4 slots of 256 x 66 int32 each
    ws = torch.zeros(need, dtype=torch.uint8, device=dev)
    assert call(None, 0, t128, 4) == q.EWORKSPACE
    assert call(ws.data_ptr(), need - 4, t128, 4) == q.EWORKSPACE
    assert call(ws.data_ptr() + 4, need, t128, 4) == q.EALIGN
    assert call(ws.data_ptr(), need, q.kernel_id("tile256"), 2) == q.EUNSUPPORTED
    assert call(None, 0, t128, 0) == q.OK           # the built-in choice never splits this kernel
    assert call(ws.data_ptr(), need, t128, 4) == q.OK
    torch.cuda.synchronize()
    # K = 1024 has 16 tiles: at most four slices of four
    assert q.gemm_splitk_factor(c.M, Bp, "tile128", 64) == 4
    # a K that is not a whole number of 64-deep tiles is not split
    c2 = wl.random_gemm(83, 130, 140, 1000)
    Bp2 = q.pack_b(torch.from_numpy(c2.B).to(dev), c2.b_zp)
    assert q.gemm_splitk_factor(c2.M, Bp2, "tile128", 4) == 1
    assert q.lib.qg_gemm_splitk_workspace_bytes(c2.M, Bp2.handle, t128, 4) == 0
