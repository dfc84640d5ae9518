"""GPU parity of the outlier-aware split B = B' + B_sparse (paper Sec. 2.2): a split descriptor must give the
same bytes as the plain definition on the whole matrix B, for every streaming kernel, any outlier density."""
import ctypes

import numpy as np
import pytest

from paper_2101_05615_amd import workloads as wl
from gpu_util import assert_same, dev_case, oracle_gemm, say

pytestmark = pytest.mark.gpu

STREAM = ["auto", "skinny16", "skinny32", "skinny64"]


@pytest.fixture(scope="module")
def env():
    import torch
    assert torch.cuda.is_available(), "these tests need the MI355X"
    from paper_2101_05615_amd import qgemm as q
    import oracle
    oracle.build()
    return q, torch, torch.device("cuda:0"), oracle


def split_case(seed, M, N, K, frac, **kw):
    c = wl.random_gemm(seed, M, N, K, wide_zp=True, **kw)
    c.B = wl.outlier_weights(seed + 1, K, N, outlier_frac=frac, outlier_sigma=50.0)
    return wl.unsaturated(c)


@pytest.mark.parametrize("K,N,frac", [(64, 16, 0.0), (300, 100, 0.02), (4224, 64, 0.01), (1000, 520, 0.2), (128, 257, 1.0)])
def test_outlier_count_and_offsets(env, K, N, frac):
    q, torch, dev, oracle = env
    B = wl.outlier_weights(K + N, K, N, outlier_frac=frac, outlier_sigma=50.0)
    if frac == 1.0:
        B = np.where((B >= -8) & (B <= 7), np.int8(100), B).astype(np.int8)   # every entry an outlier
    _, _, want = oracle.split_outliers(B, -8, 7)
    Bd = torch.from_numpy(B).to(dev)
    assert q.count_outliers(Bd) == want
    b_zp = np.arange(N, dtype=np.int32) % 17 - 8
    Bp = q.pack_b_outlier(Bd, b_zp)
    torch.cuda.synchronize()
    assert Bp.nnz == want
    assert_same(Bp.col_offsets.cpu().numpy(), oracle.col_offsets(B, b_zp), "col_offsets of the whole B")


SHAPES = [(16, 100, 300), (5, 64, 4224), (40, 260, 1024), (130, 257, 128), (64, 512, 1000), (1, 1, 1), (300, 48, 192)]


@pytest.mark.parametrize("frac", [0.0, 0.01, 0.3])
@pytest.mark.parametrize("shape", SHAPES, ids=lambda s: "x".join(map(str, s)))
def test_split_descriptor_bit_exact_all_outputs(env, shape, frac):
    q, torch, dev, oracle = env
    M, N, K = shape
    say(f"split shape {shape} frac {frac}")
    c = split_case(M + 2 * N + 3 * K, M, N, K, frac, per_channel=True, with_bias=True)
    A, B, bias, scales, C, c_store = dev_case(c, torch, dev)
    Bp = q.pack_b_outlier(B, c.b_zp)
    want = oracle_gemm(c, oracle)
    want_acc, want_rs = oracle.acc32(c.A, c.B), oracle.rowsum(c.A)
    want_f = oracle.gemm_u8s8_dequant_f32(c.A, c.a_zp, c.B, c.b_zp, c.bias, c.scales, False)
    for kernel in STREAM:
        C.fill_(0xEE)
        q.gemm_u8s8_requant(A, c.a_zp, Bp, bias, scales, c.c_zp, c.relu, out=C, kernel=kernel)
        acc, rs = q.gemm_u8s8_acc32(A, Bp, want_rowsum=True, kernel=kernel)
        f = q.gemm_u8s8_dequant_f32(A, c.a_zp, Bp, bias, scales, False, kernel=kernel)
        torch.cuda.synchronize()
        assert_same(C.cpu().numpy(), want, f"{kernel} requant")
        assert_same(acc.cpu().numpy(), want_acc, f"{kernel} acc32")
        assert_same(rs.cpu().numpy(), want_rs, f"{kernel} rowsum")
        assert_same(f.cpu().numpy().view(np.uint32), want_f.view(np.uint32), f"{kernel} fp32 output")
    assert (c_store.cpu().numpy()[c.M * c.N:] == 0xEE).all()


def test_split_equals_dense_descriptor_on_config2_shape(env):
    """The bandwidth-bound small-batch shape the split is for, full size, against the oracle."""
    q, torch, dev, oracle = env
    c = split_case(21, 16, 4096, 4096, 0.01, per_channel=False, with_bias=False, relu=True)
    A, B, bias, scales, C, _ = dev_case(c, torch, dev)
    Bp = q.pack_b_outlier(B, c.b_zp)
    q.gemm_u8s8_requant(A, c.a_zp, Bp, bias, scales, c.c_zp, c.relu, out=C)
    torch.cuda.synchronize()
    assert 0.005 < Bp.nnz / (4096 * 4096) < 0.03
    assert_same(C.cpu().numpy(), oracle_gemm(c, oracle), "split, 16 x 4096 x 4096")


def test_split_at_the_largest_k(env):
    """K = 32768: 32 k blocks per wave, eight batches, entry offsets of nine batch boundaries per wave."""
    q, torch, dev, oracle = env
    c = split_case(33, 16, 40, q.MAX_K, 0.004, per_channel=True, with_bias=True)
    A, B, bias, scales, C, _ = dev_case(c, torch, dev)
    Bp = q.pack_b_outlier(B, c.b_zp)
    for kernel in STREAM:
        C.fill_(0xEE)
        q.gemm_u8s8_requant(A, c.a_zp, Bp, bias, scales, c.c_zp, c.relu, out=C, kernel=kernel)
        acc = q.gemm_u8s8_acc32(A, Bp, kernel=kernel)
        torch.cuda.synchronize()
        assert_same(acc.cpu().numpy(), oracle.acc32(c.A, c.B), f"{kernel} acc32 at K = 32768")
        assert_same(C.cpu().numpy(), oracle_gemm(c, oracle), f"{kernel} requant at K = 32768")


def test_split_with_fp32_activations(env):
    q, torch, dev, oracle = env
    M, N, K, zp = 16, 256, 1024, 90
    Af, inv = wl.random_fp32_activations(5, M, K, alpha=0.02, zp=zp)
    c = split_case(6, M, N, K, 0.02, per_channel=True, with_bias=True, a_zp=zp)
    Bp = q.pack_b_outlier(torch.from_numpy(c.B).to(dev), c.b_zp)
    got = q.gemm_f32s8_requant(torch.from_numpy(Af).to(dev), inv, zp, Bp, torch.from_numpy(c.bias).to(dev),
                               torch.from_numpy(c.scales).to(dev), c.c_zp, c.relu)
    torch.cuda.synchronize()
    Aq = oracle.quantize_f32(Af, inv, zp)
    assert_same(got.cpu().numpy(), oracle.gemm_u8s8_requant(Aq, zp, c.B, c.b_zp, c.bias, c.scales, c.c_zp, c.relu),
                "fp32 in, split weights")


def test_split_errors(env):
    q, torch, dev, oracle = env
    c = split_case(9, 16, 64, 128, 0.1)
    A, B, bias, scales, C, _ = dev_case(c, torch, dev)
    nnz = q.count_outliers(B)
    assert nnz > 1
    with pytest.raises(q.QGemmError) as ei:
        q.pack_b_outlier(B, c.b_zp, max_nnz=nnz - 1)
    assert ei.value.code == q.ECAPACITY
    Bp = q.pack_b_outlier(B, c.b_zp, max_nnz=nnz + 100)     # spare capacity is fine
    assert Bp.nnz == nnz
    p = q.RequantParams(c.a_zp, None, scales.data_ptr(), scales.numel(), c.c_zp, 0)
    for tile in (4, 5, 6, 7):
        rc = q.lib.qg_gemm_u8s8_requant_kernel(A.data_ptr(), c.M, A.stride(0), Bp.handle, ctypes.byref(p), C.data_ptr(),
                                               C.stride(0), None, None, tile)
        assert rc == q.EUNSUPPORTED
    n = ctypes.c_size_t()
    scratch = torch.empty(2, dtype=torch.int64, device=dev)
    assert q.lib.qg_count_outliers(B.data_ptr(), 128, 64, 63, scratch.data_ptr(), ctypes.byref(n), None) == q.EINVAL
    assert q.lib.qg_count_outliers(B.data_ptr(), 128, 64, 64, scratch.data_ptr() + 4, ctypes.byref(n), None) == q.EALIGN
    assert q.lib.qg_count_outliers(B.data_ptr(), 128, 64, 64, None, ctypes.byref(n), None) == q.ENULL
    assert q.lib.qg_packed_b_nnz(None) == 0
    torch.cuda.synchronize()
