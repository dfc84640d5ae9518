"""The run-time calls only enqueue kernels on the caller's stream (no allocation, no copy, no memset, no
synchronisation), so a caller may record them into a HIP graph.  A graph of several calls is replayed a few
times, with fresh inputs written by ordinary eager work and synchronisations in between, and every replay is
compared with the CPU oracle."""
import numpy as np
import pytest

from paper_2101_05615_amd import workloads as wl
from gpu_util import assert_same, say

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def env():
    import torch
    assert torch.cuda.is_available(), "these tests need the MI355X"
    from paper_2101_05615_amd import qgemm as q
    import oracle
    oracle.build()
    return q, torch, torch.device("cuda:0"), oracle


def test_recorded_calls_replay_bit_exact(env):
    q, torch, dev, oracle = env
    rng = np.random.default_rng(77)
    # a small-batch layer (streaming kernel), a tiled layer fed by the first one's output, a group convolution,
    # and the fp32-in composite (quantize pass + GEMM through the caller's workspace)
    c1 = wl.unsaturated(wl.random_gemm(31, 16, 512, 1024, per_channel=True, with_bias=True))
    c2 = wl.unsaturated(wl.random_gemm(32, 16, 256, 512, per_channel=False, with_bias=True, relu=True))
    c3 = wl.unsaturated(wl.random_gemm(33, 300, 384, 256, per_channel=True, with_bias=False))
    cv = wl.random_conv(34, Nb=2, H=9, W=7, C=128, G=32)
    alpha, zp = 0.05, 100
    inv = np.float32(1.0 / alpha)

    def up(x):
        return torch.from_numpy(x).to(dev)

    A1 = up(c1.A)
    B1, B2, B3 = q.pack_b(up(c1.B), c1.b_zp), q.pack_b(up(c2.B), c2.b_zp), q.pack_b(up(c3.B), c3.b_zp)
    bias1, bias2 = up(c1.bias), up(c2.bias)
    s1, s2, s3 = up(c1.scales), up(c2.scales), up(c3.scales)
    H1 = torch.empty((16, 512), dtype=torch.uint8, device=dev)
    H2 = torch.empty((16, 256), dtype=torch.uint8, device=dev)
    Af = torch.empty((300, 256), dtype=torch.float32, device=dev)
    ws = torch.empty(q.gemm_f32_workspace_bytes(300, B3), dtype=torch.uint8, device=dev)
    C3 = torch.empty((300, 384), dtype=torch.uint8, device=dev)
    Wp = q.pack_conv_w(up(cv.wgt), cv.b_zp)
    cbias, cs = up(cv.bias), up(cv.scales)
    X = up(cv.inp)
    Y = torch.empty_like(X)

    def enqueue():
        q.gemm_u8s8_requant(A1, c1.a_zp, B1, bias1, s1, c1.c_zp, c1.relu, out=H1)
        q.gemm_u8s8_requant(H1, c2.a_zp, B2, bias2, s2, c2.c_zp, c2.relu, out=H2, kernel="tile64")
        q.gemm_f32s8_requant(Af, inv, zp, B3, None, s3, c3.c_zp, c3.relu, out=C3, workspace=ws)
        q.conv_groupwise_u8s8_requant(X, Wp, cv.a_zp, cbias, cs, cv.c_zp, cv.relu, cv.pad, cv.stride, out=Y)

    def expected(a1, af, x):
        h1 = oracle.gemm_u8s8_requant(a1, c1.a_zp, c1.B, c1.b_zp, c1.bias, c1.scales, c1.c_zp, c1.relu)
        h2 = oracle.gemm_u8s8_requant(h1, c2.a_zp, c2.B, c2.b_zp, c2.bias, c2.scales, c2.c_zp, c2.relu)
        aq = oracle.quantize_f32(af, inv, zp)
        o3 = oracle.gemm_u8s8_requant(aq, zp, c3.B, c3.b_zp, None, c3.scales, c3.c_zp, c3.relu)
        y = oracle.conv_groupwise_direct(x, cv.G, cv.wgt, cv.a_zp, cv.b_zp, cv.bias, cv.scales, cv.c_zp, cv.relu,
                                         cv.pad, cv.stride)
        return h1, h2, o3, y

    af0, _ = wl.random_fp32_activations(35, 300, 256, alpha, zp)
    Af.copy_(up(af0))
    # eager once on a side stream (the usual warm-up before a capture), then record
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):
        enqueue()
    torch.cuda.current_stream().wait_stream(side)
    torch.cuda.synchronize()
    eager = [t.cpu().numpy().copy() for t in (H1, H2, C3, Y)]
    for got, want, what in zip(eager, expected(c1.A, af0, cv.inp), ("fc1", "fc2", "f32 in", "conv")):
        assert_same(got, want, "eager " + what)

    g = torch.cuda.CUDAGraph()
    say("recording")
    with torch.cuda.graph(g):
        enqueue()
    for rep in range(3):
        say(f"replay {rep}")
        a1 = rng.integers(0, 256, size=c1.A.shape, dtype=np.uint8)
        af, _ = wl.random_fp32_activations(100 + rep, 300, 256, alpha, zp)
        x = rng.integers(0, 256, size=cv.inp.shape, dtype=np.uint8)
        A1.copy_(up(a1))
        Af.copy_(up(af))
        X.copy_(up(x))
        for t in (H1, H2, C3, Y):
            t.fill_(0xEE)          # eager work between replays; a stale result cannot pass
        torch.cuda.synchronize()
        g.replay()
        torch.cuda.synchronize()
        got = [t.cpu().numpy() for t in (H1, H2, C3, Y)]
        for gt, want, what in zip(got, expected(a1, af, x), ("fc1", "fc2", "f32 in", "conv")):
            assert_same(gt, want, f"replay {rep} {what}")
