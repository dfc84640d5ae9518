"""GPU parity of the fp32 ends of the pipeline (paper Appendix B: other packing routines for A, other output
processing): activation quantization fp32 -> uint8 and the fp32 output pipeline, alone and combined, against
the CPU oracle.  Every step is a fixed sequence of correctly rounded fp32 operations, so results must be
identical bit for bit (floats are compared through their bit patterns)."""
import numpy as np
import pytest

from paper_2101_05615_amd import workloads as wl
from gpu_util import assert_same, dev_case, say

pytestmark = pytest.mark.gpu

KERNELS = ["auto", "skinny16", "skinny32", "skinny64", "tile64", "tile128", "tile128x256", "tile256", "tile64k4", "tile64k1", "tile64x32k8"]


@pytest.fixture(scope="module")
def env():
    import torch
    assert torch.cuda.is_available(), "these tests need the MI355X"
    from paper_2101_05615_amd import qgemm as q
    import oracle
    oracle.build()
    return q, torch, torch.device("cuda:0"), oracle


def bits(a):
    return np.ascontiguousarray(np.asarray(a, np.float32)).view(np.uint32)


@pytest.mark.parametrize("M,K,lda_pad,off", [(1, 1, 0, 0), (3, 7, 0, 0), (7, 100, 3, 1), (16, 4096, 0, 0),
                                               (300, 515, 1, 0), (2048, 1024, 0, 0), (65, 64, 4, 4)])
def test_quantize_a_bit_exact(env, M, K, lda_pad, off):
    q, torch, dev, oracle = env
    say(f"quantize M={M} K={K} lda_pad={lda_pad} off={off}")
    A, inv = wl.random_fp32_activations(M * 31 + K, M, K, alpha=0.0371, zp=77)
    store = torch.zeros(M * (K + lda_pad) + off + 8, dtype=torch.float32, device=dev)
    Ad = store[off:off + M * (K + lda_pad)].view(M, K + lda_pad)[:, :K]
    Ad.copy_(torch.from_numpy(A).to(dev))
    out_store = torch.full((M * (K + lda_pad) + off + 8,), 0xEE, dtype=torch.uint8, device=dev)
    out = out_store[off:off + M * (K + lda_pad)].view(M, K + lda_pad)[:, :K]
    q.quantize_a_f32(Ad, inv, 77, out=out)
    torch.cuda.synchronize()
    assert_same(out.cpu().numpy(), oracle.quantize_f32(A, inv, 77), "quantized activations")
    if lda_pad:
        pad = out_store[off:off + M * (K + lda_pad)].view(M, K + lda_pad)[:, K:].cpu().numpy()
        assert (pad == 0xEE).all(), "bytes between rows were written"


@pytest.mark.parametrize("zp,alpha", [(0, 1.0), (255, 0.5), (128, 2.0 ** -6)])
def test_quantize_extreme_zero_points_and_ties(env, zp, alpha):
    q, torch, dev, oracle = env
    codes = np.arange(-20, 280, dtype=np.float64)
    vals = np.concatenate([alpha * (codes - zp), alpha * (codes - zp + 0.5), alpha * (codes - zp - 0.5)])
    A = vals.astype(np.float32).reshape(1, -1).copy()
    out = q.quantize_a_f32(torch.from_numpy(A).to(dev), 1.0 / alpha, zp)
    torch.cuda.synchronize()
    assert_same(out.cpu().numpy(), oracle.quantize_f32(A, 1.0 / alpha, zp), "ties and saturation")


SHAPES = [(16, 100, 300), (5, 64, 4224), (40, 260, 1024), (130, 257, 128), (300, 520, 1024), (257, 130, 100)]


@pytest.mark.parametrize("shape", SHAPES, ids=lambda s: "x".join(map(str, s)))
@pytest.mark.parametrize("kernel", KERNELS)
def test_fp32_output_bit_exact(env, kernel, shape):
    q, torch, dev, oracle = env
    M, N, K = shape
    say(f"dequant kernel {kernel} shape {shape}")
    for relu, per_channel, with_bias in [(False, True, True), (True, False, False)]:
        c = wl.random_gemm(M + N + K + int(relu), M, N, K, per_channel=per_channel, with_bias=with_bias, wide_zp=True)
        A, B, bias, scales, _, _ = dev_case(c, torch, dev)
        Bp = q.pack_b(B, c.b_zp)
        out = q.gemm_u8s8_dequant_f32(A, c.a_zp, Bp, bias, scales, relu, kernel=kernel)
        torch.cuda.synchronize()
        want = oracle.gemm_u8s8_dequant_f32(c.A, c.a_zp, c.B, c.b_zp, c.bias, c.scales, relu)
        assert_same(bits(out.cpu().numpy()), bits(want), f"fp32 output relu={relu}")


def test_fp32_output_unaligned_and_padded(env):
    q, torch, dev, oracle = env
    c = wl.random_gemm(3, 150, 140, 256, per_channel=True, with_bias=True, wide_zp=True)
    A, B, bias, scales, _, _ = dev_case(c, torch, dev, lda_pad=3, a_off=1)
    Bp = q.pack_b(B, c.b_zp)
    want = oracle.gemm_u8s8_dequant_f32(c.A, c.a_zp, c.B, c.b_zp, c.bias, c.scales, False)
    for kernel in ["skinny16", "tile64", "tile256"]:
        store = torch.full((150 * 143 + 9,), float("nan"), dtype=torch.float32, device=dev)
        out = store[1:1 + 150 * 143].view(150, 143)[:, :140]   # 4-byte aligned only, ldc not a multiple of 4
        q.gemm_u8s8_dequant_f32(A, c.a_zp, Bp, bias, scales, False, out=out, kernel=kernel)
        torch.cuda.synchronize()
        assert_same(bits(out.cpu().numpy()), bits(want), f"{kernel} unaligned fp32 output")
        pad = store[1:1 + 150 * 143].view(150, 143)[:, 140:].cpu().numpy()
        assert np.isnan(pad).all(), "floats between rows were written"


@pytest.mark.parametrize("M,N,K", [(16, 256, 1024), (48, 100, 300), (300, 260, 512), (1024, 512, 448)])
def test_fp32_activations_both_outputs(env, M, N, K):
    q, torch, dev, oracle = env
    say(f"fp32 in M={M} N={N} K={K}")
    alpha, zp = 0.02, 90
    Af, inv = wl.random_fp32_activations(M + K, M, K, alpha=alpha, zp=zp)
    c = wl.unsaturated(wl.random_gemm(M * 3 + N, M, N, K, per_channel=True, with_bias=True, a_zp=zp))
    B = torch.from_numpy(c.B).to(dev)
    bias = torch.from_numpy(c.bias).to(dev)
    scales = torch.from_numpy(c.scales).to(dev)
    Bp = q.pack_b(B, c.b_zp)
    Ad = torch.from_numpy(Af).to(dev)
    Aq = oracle.quantize_f32(Af, inv, zp)
    want_u8 = oracle.gemm_u8s8_requant(Aq, zp, c.B, c.b_zp, c.bias, c.scales, c.c_zp, c.relu)
    want_f32 = oracle.gemm_u8s8_dequant_f32(Aq, zp, c.B, c.b_zp, c.bias, c.scales, True)
    got_u8 = q.gemm_f32s8_requant(Ad, inv, zp, Bp, bias, scales, c.c_zp, c.relu)
    got_f32 = q.gemm_f32s8_dequant_f32(Ad, inv, zp, Bp, bias, scales, True)
    torch.cuda.synchronize()
    assert_same(got_u8.cpu().numpy(), want_u8, "fp32 in, uint8 out")
    assert_same(bits(got_f32.cpu().numpy()), bits(want_f32), "fp32 in, fp32 out")
    assert np.mean((want_u8 > 0) & (want_u8 < 255)) > 0.3


@pytest.mark.parametrize("kernel", ["skinny16", "skinny32", "skinny64"])
@pytest.mark.parametrize("M,N,K,lda_pad", [(16, 256, 1024, 0), (48, 100, 300, 0), (7, 40, 4097, 3), (130, 72, 2048, 4),
                                           (1, 520, 512, 0), (64, 64, 100, 1)])
def test_fp32_activations_quantized_while_staged(env, kernel, M, N, K, lda_pad):
    """A streaming kernel takes fp32 activations in ONE launch and without a workspace: it quantizes the block it
    stages.  Bytes must be those of oracle.quantize_f32 followed by the oracle GEMM: aligned and unaligned rows of
    floats, ragged K, ties, saturating and infinite activations, both outputs."""
    q, torch, dev, oracle = env
    say(f"fused fp32 staging {kernel} M={M} N={N} K={K} lda={K + lda_pad}")
    alpha, zp = 0.02, 90
    Af, inv = wl.random_fp32_activations(5 * M + K, M, K, alpha=alpha, zp=zp)
    c = wl.unsaturated(wl.random_gemm(M * 3 + N + K, M, N, K, per_channel=True, with_bias=True, a_zp=zp, wide_zp=True))
    B = torch.from_numpy(c.B).to(dev)
    bias = torch.from_numpy(c.bias).to(dev)
    scales = torch.from_numpy(c.scales).to(dev)
    Bp = q.pack_b(B, c.b_zp)
    store = torch.full((M, K + lda_pad), float("nan"), dtype=torch.float32, device=dev)
    Ad = store[:, :K]
    Ad.copy_(torch.from_numpy(Af).to(dev))
    Aq = oracle.quantize_f32(Af, inv, zp)
    want_u8 = oracle.gemm_u8s8_requant(Aq, zp, c.B, c.b_zp, c.bias, c.scales, c.c_zp, c.relu)
    want_f32 = oracle.gemm_u8s8_dequant_f32(Aq, zp, c.B, c.b_zp, c.bias, c.scales, True)
    got_u8 = q.gemm_f32s8_requant(Ad, inv, zp, Bp, bias, scales, c.c_zp, c.relu, workspace=q.NO_WORKSPACE, kernel=kernel)
    got_f32 = q.gemm_f32s8_dequant_f32(Ad, inv, zp, Bp, bias, scales, True, workspace=q.NO_WORKSPACE, kernel=kernel)
    torch.cuda.synchronize()
    assert_same(got_u8.cpu().numpy(), want_u8, "fp32 in, uint8 out, one launch")
    assert_same(bits(got_f32.cpu().numpy()), bits(want_f32), "fp32 in, fp32 out, one launch")


def test_fp32_ends_argument_errors(env):
    import ctypes
    q, torch, dev, oracle = env
    c = wl.config1_tiny()
    A, B, bias, scales, C, _ = dev_case(c, torch, dev)
    Bp = q.pack_b(B, c.b_zp)
    Af = torch.zeros((64, 128), dtype=torch.float32, device=dev)
    Cf = torch.zeros((64, 64), dtype=torch.float32, device=dev)
    ws = torch.zeros(q.gemm_f32_workspace_bytes(64, Bp) + 16, dtype=torch.uint8, device=dev)
    assert q.gemm_f32_workspace_bytes(64, Bp) == 64 * 128
    p = q.RequantParams(128, None, scales.data_ptr(), 1, 0, 0)
    d = q.DequantParams(128, None, scales.data_ptr(), 1, 0)
    L = q.lib
    assert L.qg_gemm_f32s8_requant(Af.data_ptr(), 64, 128, 1.0, Bp.handle, ctypes.byref(p), C.data_ptr(), 64, None, None, 4) == q.EWORKSPACE
    assert L.qg_gemm_f32s8_requant(Af.data_ptr(), 64, 128, 1.0, Bp.handle, ctypes.byref(p), C.data_ptr(), 64, ws.data_ptr() + 1, None, 4) == q.EALIGN
    assert L.qg_gemm_f32s8_requant(Af.data_ptr(), 64, 127, 1.0, Bp.handle, ctypes.byref(p), C.data_ptr(), 64, ws.data_ptr(), None, 0) == q.EINVAL
    assert L.qg_gemm_f32s8_requant(Af.data_ptr(), 64, 128, 0.0, Bp.handle, ctypes.byref(p), C.data_ptr(), 64, ws.data_ptr(), None, 0) == q.EINVAL
    assert L.qg_gemm_f32s8_requant(Af.data_ptr(), 64, 128, 1.0, Bp.handle, ctypes.byref(p), C.data_ptr(), 64, ws.data_ptr(), None, q.KERNEL_LAST + 1) == q.EINVAL
    assert L.qg_gemm_f32s8_dequant_f32(Af.data_ptr(), 64, 128, 1.0, Bp.handle, ctypes.byref(d), Cf.data_ptr(), 63, ws.data_ptr(), None, 0) == q.EINVAL
    assert L.qg_gemm_f32s8_dequant_f32(Af.data_ptr(), 64, 128, 1.0, Bp.handle, ctypes.byref(d), None, 64, ws.data_ptr(), None, 0) == q.ENULL
    assert L.qg_gemm_u8s8_dequant_f32(A.data_ptr(), 64, 128, Bp.handle, ctypes.byref(d), Cf.data_ptr() + 2, 64, None, None, 0) == q.EALIGN
    d.relu = 3
    assert L.qg_gemm_u8s8_dequant_f32(A.data_ptr(), 64, 128, Bp.handle, ctypes.byref(d), Cf.data_ptr(), 64, None, None, 0) == q.EINVAL
    assert L.qg_quantize_a_f32(Af.data_ptr(), 64, 128, 128, 1.0, 256, ws.data_ptr(), 128, None) == q.EINVAL
    assert L.qg_quantize_a_f32(Af.data_ptr(), 64, 128, 128, float("inf"), 0, ws.data_ptr(), 128, None) == q.EINVAL
    assert L.qg_quantize_a_f32(None, 64, 128, 128, 1.0, 0, ws.data_ptr(), 128, None) == q.ENULL
    # a streaming kernel needs no workspace, and checks the quantization parameters itself
    assert L.qg_gemm_f32s8_requant(Af.data_ptr(), 64, 128, 1.0, Bp.handle, ctypes.byref(p), C.data_ptr(), 64, None, None, 1) == q.OK
    assert L.qg_gemm_f32s8_requant(Af.data_ptr(), 64, 128, 0.0, Bp.handle, ctypes.byref(p), C.data_ptr(), 64, None, None, 1) == q.EINVAL
    assert L.qg_gemm_f32s8_requant(Af.data_ptr() + 2, 64, 128, 1.0, Bp.handle, ctypes.byref(p), C.data_ptr(), 64, None, None, 1) == q.EALIGN
    assert L.qg_gemm_f32s8_requant(None, 64, 128, 1.0, Bp.handle, ctypes.byref(p), C.data_ptr(), 64, None, None, 1) == q.ENULL
    torch.cuda.synchronize()
    torch.cuda.synchronize()
