"""GPU parity of the group-wise convolution for group shapes beyond 4 -> 4 channels (the paper names convolution
in Sec. 1 without describing it; the definition is the real-domain one of Eq. (1), one GEMM per group) against the
CPU oracle's direct 7-loop convolution: identical bytes.  Square groups of 8, 16 and 32 channels with a 1 x 1 or
3 x 3 filter -- and of 1 (depthwise) and 2 -- run the matrix-core kernels on block-diagonal tiles; groups of a multiple of
16 channels run one dense convolution per group; every other shape runs the plain kernel."""
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


def run(c, q, torch, dev):
    Wp = q.pack_conv_w(torch.from_numpy(c.wgt).to(dev), c.b_zp)
    bias = None if c.bias is None else torch.from_numpy(c.bias).to(dev)
    out = q.conv_groupwise_u8s8_requant(torch.from_numpy(c.inp).to(dev), Wp, c.a_zp, bias, torch.from_numpy(c.scales).to(dev),
                                        c.c_zp, c.relu, pad=c.pad, stride=c.stride)
    torch.cuda.synchronize()
    return out.cpu().numpy()


def want(c, oracle):
    return oracle.conv_groupwise_direct(c.inp, c.G, c.wgt, c.a_zp, c.b_zp, c.bias, c.scales, c.c_zp, c.relu, c.pad, c.stride)


@pytest.mark.parametrize("cfg", [
    # matrix-core kernels on block-diagonal tiles (C % 32 == 0, square groups, 1 x 1 / 3 x 3)
    dict(Nb=2, H=9, W=7, C=64, G=8),                               # 8 -> 8, "same" 3 x 3: the staged-patch kernel
    dict(Nb=1, H=12, W=10, C=128, G=8),                            # 16 -> 16
    dict(Nb=2, H=6, W=6, C=64, G=2),                               # 32 -> 32: row sums across the two lanes of a pixel
    dict(Nb=1, H=9, W=9, C=32, G=4, stride=2),                     # taps from memory (stride 2), one 32-channel block
    dict(Nb=2, H=8, W=8, C=256, G=16, R=1, S=1, pad=0),            # 1 x 1, 16 -> 16
    dict(Nb=1, H=7, W=7, C=96, G=12, pad=0),                       # 8 -> 8 without padding, three blocks
    dict(Nb=1, H=5, W=5, C=2048, G=512),                           # 4 -> 4 in more groups than the dword kernel takes
    dict(Nb=2, H=9, W=7, C=64, G=64),                              # depthwise (1 -> 1): row offsets from the matrix cores
    dict(Nb=1, H=11, W=10, C=32, G=32, stride=2),                  # depthwise, taps from memory
    dict(Nb=2, H=8, W=8, C=128, G=128, R=1, S=1, pad=0),           # depthwise 1 x 1: a per-channel scale
    dict(Nb=1, H=7, W=9, C=64, G=32),                              # 2 -> 2
    # everything else: the plain kernel
    dict(Nb=2, H=7, W=9, C=32, G=4, Cout=16),                      # 8 -> 4
    dict(Nb=1, H=8, W=8, C=24, G=2, Cout=40, R=5, S=5, pad=2),     # 12 -> 20, 5 x 5
    dict(Nb=2, H=6, W=5, C=9, G=3, Cout=6, R=2, S=3, pad=1),       # 3 -> 2: byte path, odd channel counts
    dict(Nb=1, H=9, W=9, C=7, G=7, Cout=7, R=3, S=3),              # depthwise, 1 -> 1
    dict(Nb=1, H=6, W=6, C=20, G=5, Cout=20, R=1, S=7, pad=3),     # 4 -> 4 with a filter the tuned kernels do not take
    dict(Nb=2, H=10, W=10, C=64, G=1, Cout=48, stride=3),          # one group: a dense convolution through this call
    # groups of a multiple of 16 channels without block-diagonal tiles: one dense convolution per group on its channel slice
    dict(Nb=1, H=4, W=4, C=128, G=2, Cout=128, R=3, S=3),          # 64 -> 64: too wide for one block-diagonal tile
    dict(Nb=2, H=9, W=8, C=144, G=3, Cout=60),                     # 48 -> 20: 16-channel chunks, taps inside a k tile
    dict(Nb=1, H=10, W=10, C=64, G=4, Cout=32, stride=2),          # 16 -> 8
    dict(Nb=2, H=14, W=14, C=384, G=3, Cout=384),                  # 128 -> 128: the hand-scheduled loop on a channel slice
    dict(Nb=1, H=8, W=9, C=256, G=2, Cout=96, R=5, S=5, pad=2),    # 128 -> 48, 5 x 5
])
@pytest.mark.parametrize("per_channel,with_bias,relu", [(True, True, False), (False, False, True)])
def test_group_conv_any_group_shape_bit_exact(env, cfg, per_channel, with_bias, relu):
    q, torch, dev, oracle = env
    say(f"group conv {cfg} per_channel={per_channel}")
    c = wl.random_conv(21, per_channel=per_channel, with_bias=with_bias, relu=relu, **cfg)
    assert_same(run(c, q, torch, dev), want(c, oracle), f"group conv {cfg}")


def test_group_conv_zero_weight_zero_points(env):
    """theta_B == 0 everywhere: the kernels without row offsets."""
    q, torch, dev, oracle = env
    for cfg in (dict(Nb=2, H=9, W=7, C=64, G=8), dict(Nb=1, H=7, W=7, C=18, G=3, Cout=12), dict(Nb=2, H=9, W=7, C=64, G=64)):
        c = wl.random_conv(22, **cfg)
        c.b_zp[:] = 0
        assert_same(run(c, q, torch, dev), want(c, oracle), f"group conv {cfg}, theta_B = 0")


def test_group_conv_resnext_like_layer(env):
    """56 x 56 x 256 in 32 groups of 8 -> 8 channels, 3 x 3, batch 2: the staged-patch matrix-core kernel at a real size."""
    q, torch, dev, oracle = env
    c = wl.random_conv(23, Nb=2, H=56, W=56, C=256, G=32)
    assert_same(run(c, q, torch, dev), want(c, oracle), "32 groups of 8 -> 8 at 56 x 56")
