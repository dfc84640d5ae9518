"""The entry point that allocates nothing (qg_gemm_u8s8_requant_noalloc): its K-split workspace is a scratch array
built into the library.  Its bytes must equal those of qg_gemm_u8s8_requant_splitk with a caller workspace (and the
oracle's), on calls made one after another on the same GPU, the later ones smaller than the first."""
import ctypes

import numpy as np
import pytest

from paper_2101_05615_amd import workloads as wl
from gpu_util import assert_same, dev_case, oracle_gemm, say

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def env():
    import torch
    assert torch.cuda.is_available(), "these tests need the MI355X"
    from paper_2101_05615_amd import qgemm as q
    import oracle
    oracle.build()
    return q, torch, torch.device("cuda:0"), oracle


def run_pair(q, torch, dev, oracle, case, kernel, ksplit, tag):
    """Both entry points on the same inputs; returns the split factor in use."""
    A, B, bias, scales, C, c_store = dev_case(case, torch, dev)
    Bp = q.pack_b(B, case.b_zp)
    used = q.gemm_splitk_factor(case.M, Bp, kernel, ksplit)
    ws = q.gemm_workspace(case.M, Bp, kernel, ksplit)
    ref = q.gemm_u8s8_requant_splitk(A, case.a_zp, Bp, bias, scales, case.c_zp, case.relu, ws, kernel, ksplit)
    C.fill_(0xEE)
    q.gemm_u8s8_requant_noalloc(A, case.a_zp, Bp, bias, scales, case.c_zp, case.relu, C, kernel, ksplit)
    torch.cuda.synchronize()
    say(f"{tag}: {case.M}x{case.N}x{case.K} kernel {kernel} ksplit {ksplit} -> {used}")
    assert_same(C.cpu().numpy(), ref.cpu().numpy(), f"{tag}: built-in scratch vs caller workspace")
    assert_same(C.cpu().numpy(), oracle_gemm(case, oracle), f"{tag}: built-in scratch vs oracle")
    assert (c_store.cpu().numpy()[case.M * case.N:] == 0xEE).all(), "bytes past C were written"
    return used


def test_two_calls_in_a_row_the_second_smaller(env):
    q, torch, dev, oracle = env
    first = wl.unsaturated(wl.random_gemm(9100, 40, 200, 8192, per_channel=True, with_bias=True, wide_zp=True))
    second = wl.unsaturated(wl.random_gemm(9101, 7, 72, 3000, per_channel=True, with_bias=True, wide_zp=True))
    assert run_pair(q, torch, dev, oracle, first, "skinny16", 8, "first call") == 8
    assert run_pair(q, torch, dev, oracle, second, "skinny16", 3, "second, smaller call") == 3
    # and again the larger one: the scratch must be as the first call found it
    assert run_pair(q, torch, dev, oracle, first, "skinny32", 5, "third call") == 5


def test_built_in_choices_and_no_split(env):
    q, torch, dev, oracle = env
    c = wl.unsaturated(wl.random_gemm(9102, 16, 64, 16384, per_channel=False, with_bias=False, wide_zp=True))
    assert run_pair(q, torch, dev, oracle, c, "auto", 0, "auto kernel, auto split") > 1
    run_pair(q, torch, dev, oracle, c, "auto", 1, "auto kernel, no split")
    big = wl.unsaturated(wl.random_gemm(9103, 300, 260, 512, per_channel=True, with_bias=True))
    run_pair(q, torch, dev, oracle, big, "tile128", 0, "a tiled kernel (needs no scratch)")


def test_a_request_beyond_the_scratch_is_refused(env):
    q, torch, dev, oracle = env
    c = wl.random_gemm(9104, 64, 4096, 4096, per_channel=False, with_bias=False)
    A, B, bias, scales, C, _ = dev_case(c, torch, dev)
    Bp = q.pack_b(B, c.b_zp)
    need = q.lib.qg_gemm_splitk_workspace_bytes(c.M, Bp.handle, q.kernel_id("skinny16"), 8)
    assert need > q.NOALLOC_SCRATCH_BYTES
    p = q.RequantParams(c.a_zp, None, scales.data_ptr(), scales.numel(), c.c_zp, 0)
    C.fill_(0xEE)
    rc = q.lib.qg_gemm_u8s8_requant_noalloc(A.data_ptr(), c.M, A.stride(0), Bp.handle, ctypes.byref(p), C.data_ptr(),
                                            C.stride(0), None, q.kernel_id("skinny16"), 8)
    assert rc == q.EWORKSPACE
    torch.cuda.synchronize()
    assert (C.cpu().numpy() == 0xEE).all(), "a refused call wrote output"
    # the same call without a split runs
    rc = q.lib.qg_gemm_u8s8_requant_noalloc(A.data_ptr(), c.M, A.stride(0), Bp.handle, ctypes.byref(p), C.data_ptr(),
                                            C.stride(0), None, q.kernel_id("skinny16"), 1)
    assert rc == q.OK
    torch.cuda.synchronize()
    assert_same(C.cpu().numpy(), oracle_gemm(c, oracle), "no split")
