"""Seeded random sweep: shapes around every tile and fragment boundary, leading-dimension paddings and base
offsets, every kernel of the family, per-tensor / per-channel parameters, the three output modes -- each case
against the CPU oracle, and the bytes around C must stay untouched."""
import numpy as np
import pytest

from paper_2101_05615_amd import workloads as wl
from gpu_util import dev_case, say

pytestmark = pytest.mark.gpu

MS = [1, 2, 15, 16, 17, 31, 33, 64, 65, 100, 128, 129, 200, 257, 300, 513]
NS = [1, 3, 4, 15, 16, 17, 32, 33, 63, 64, 65, 100, 128, 130, 255, 256, 260, 300, 520]
KS = [1, 3, 4, 16, 36, 63, 64, 65, 100, 127, 128, 129, 192, 200, 256, 257, 320, 448, 500, 512, 1000, 1024, 1100]


@pytest.fixture(scope="module")
def env():
    import torch
    assert torch.cuda.is_available(), "these tests need the MI355X"
    from paper_2101_05615_amd import qgemm as q
    import oracle
    oracle.build()
    return q, torch, torch.device("cuda:0"), oracle


@pytest.mark.parametrize("seed", [11, 12, 13])
def test_random_gemm_cases(env, seed):
    q, torch, dev, oracle = env
    names = q.kernel_names()
    rng = np.random.default_rng(seed)
    for it in range(400):
        M, N, K = int(rng.choice(MS)), int(rng.choice(NS)), int(rng.choice(KS))
        lda_pad, ldc_pad = int(rng.choice([0, 0, 1, 3, 4, 12, 16])), int(rng.choice([0, 0, 1, 5, 16]))
        a_off, c_off = int(rng.choice([0, 0, 1, 4, 16])), int(rng.choice([0, 0, 3, 4, 16]))
        kern = names[int(rng.integers(0, q.KERNEL_LAST + 1))]
        pc, wb, relu = bool(rng.integers(0, 2)), bool(rng.integers(0, 2)), bool(rng.integers(0, 2))
        c = wl.unsaturated(wl.random_gemm(int(rng.integers(1, 1 << 30)), M, N, K, per_channel=pc, with_bias=wb,
                                          wide_zp=True))
        c.relu = relu
        if rng.integers(0, 4) == 0:
            c.b_zp[:] = 0
        if relu and rng.integers(0, 2):
            c.c_zp = 0
        tag = (f"seed {seed} case {it}: {M}x{N}x{K} lda+{lda_pad} ldc+{ldc_pad} a_off {a_off} c_off {c_off} {kern} "
               f"per_channel={pc} bias={wb} relu={relu} c_zp={c.c_zp}")
        if it % 50 == 0:
            say(tag)
        want = oracle.gemm_u8s8_requant(c.A, c.a_zp, c.B, c.b_zp, c.bias, c.scales, c.c_zp, c.relu)
        A, B, bias, scales, C, c_store = dev_case(c, torch, dev, lda_pad=lda_pad, ldc_pad=ldc_pad, a_off=a_off,
                                                  c_off=c_off)
        Bp = q.pack_b(B, c.b_zp)
        q.gemm_u8s8_requant(A, c.a_zp, Bp, bias, scales, c.c_zp, c.relu, out=C, kernel=kern)
        mode = int(rng.integers(0, 3))
        acc = rs = f32 = None
        if mode == 1:
            acc, rs = q.gemm_u8s8_acc32(A, Bp, want_rowsum=True, kernel=kern)
        if mode == 2:
            f32 = q.gemm_u8s8_dequant_f32(A, c.a_zp, Bp, bias, scales, relu, kernel=kern)
        torch.cuda.synchronize()
        got = C.cpu().numpy()
        assert np.array_equal(got, want), tag
        expect_store = np.full(c_store.numel(), 0xEE, np.uint8)
        idx = c_off + np.arange(M)[:, None] * (N + ldc_pad) + np.arange(N)[None, :]
        expect_store[idx.reshape(-1)] = want.reshape(-1)
        assert np.array_equal(c_store.cpu().numpy(), expect_store), tag + " (bytes around C)"
        if acc is not None:
            assert np.array_equal(acc.cpu().numpy(), oracle.acc32(c.A, c.B)), tag + " (acc32)"
            assert np.array_equal(rs.cpu().numpy(), oracle.rowsum(c.A)), tag + " (row sums)"
        if f32 is not None:
            wf = oracle.gemm_u8s8_dequant_f32(c.A, c.a_zp, c.B, c.b_zp, c.bias, c.scales, relu)
            assert np.array_equal(f32.cpu().numpy().view(np.uint32), wf.view(np.uint32)), tag + " (fp32 out)"


@pytest.mark.parametrize("seed", [21, 22])
def test_random_convolution_cases(env, seed):
    q, torch, dev, oracle = env
    rng = np.random.default_rng(seed)

    def up(x):
        return None if x is None else torch.from_numpy(x).to(dev)

    for it in range(200):
        dense = bool(rng.integers(0, 2))
        pc, wb, relu = bool(rng.integers(0, 2)), bool(rng.integers(0, 2)), bool(rng.integers(0, 2))
        Nb, H, W = int(rng.integers(1, 4)), int(rng.integers(1, 15)), int(rng.integers(1, 15))
        stride = int(rng.choice([1, 1, 2]))
        if dense:
            C, Cout, G = int(rng.choice([64, 128, 192])), int(rng.choice([8, 16, 40, 64, 100, 130])), 1
            R, S, pad = int(rng.choice([1, 3, 5])), int(rng.choice([1, 3])), int(rng.integers(0, 3))
        else:
            G = int(rng.choice([1, 2, 3, 8, 16, 32, 64]))
            C = Cout = 4 * G
            R = S = int(rng.choice([1, 3]))
            pad = int(rng.integers(0, 3)) if R == 3 else 0
        if H + 2 * pad < R or W + 2 * pad < S:
            continue
        c = wl.random_conv(int(rng.integers(1, 1 << 30)), Nb=Nb, H=H, W=W, C=C, G=G, Cout=Cout, R=R, S=S, pad=pad,
                           stride=stride, per_channel=pc, with_bias=wb, relu=relu)
        if rng.integers(0, 3) == 0:
            c.b_zp[:] = 0
        tag = (f"seed {seed} case {it}: {'dense' if dense else 'group'} {Nb}x{H}x{W}x{C}->{Cout} G={G} {R}x{S} "
               f"pad={pad} stride={stride} per_channel={pc} bias={wb} relu={relu}")
        if it % 50 == 0:
            say(tag)
        if dense:
            Wp = q.pack_conv_dense_w(up(np.ascontiguousarray(c.wgt[0])), c.b_zp)
            kern = ["auto", "tile64k1", "tile64", "tile64k4", "tile128", "tile128x256"][int(rng.integers(0, 6))]
            tag += f" kernel={kern}"
            got = q.conv_dense_u8s8_requant(up(c.inp), Wp, c.a_zp, up(c.bias), up(c.scales), c.c_zp, c.relu, pad=pad,
                                            stride=stride, kernel=kern)
        else:
            Wp = q.pack_conv_w(up(c.wgt), c.b_zp)
            got = q.conv_groupwise_u8s8_requant(up(c.inp), Wp, c.a_zp, up(c.bias), up(c.scales), c.c_zp, c.relu, pad,
                                                stride)
        torch.cuda.synchronize()
        want = oracle.conv_groupwise_direct(c.inp, G, c.wgt, c.a_zp, c.b_zp, c.bias, c.scales, c.c_zp, c.relu, pad,
                                            stride)
        assert np.array_equal(got.cpu().numpy(), want), tag
