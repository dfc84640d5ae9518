"""GPU parity of the dense (one group) convolution with fused im2col against the CPU oracle's direct
7-loop convolution: identical bytes."""
import ctypes
import dataclasses

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


CONV_KERNELS = ["auto", "tile64k1", "tile64", "tile64k4", "tile64x32k8", "tile128", "tile128x256"]


def run(c, q, torch, dev, kernel="auto"):
    Wp = q.pack_conv_dense_w(torch.from_numpy(np.ascontiguousarray(c.wgt[0])).to(dev), c.b_zp)
    bias = None if c.bias is None else torch.from_numpy(c.bias).to(dev)
    out = q.conv_dense_u8s8_requant(torch.from_numpy(c.inp).to(dev), Wp, c.a_zp, bias, torch.from_numpy(c.scales).to(dev),
                                    c.c_zp, c.relu, pad=c.pad, stride=c.stride, kernel=kernel)
    torch.cuda.synchronize()
    return out.cpu().numpy()


def want(c, oracle):
    return oracle.conv_groupwise_direct(c.inp, 1, c.wgt, c.a_zp, c.b_zp, c.bias, c.scales, c.c_zp, c.relu, c.pad, c.stride)


@pytest.mark.parametrize("cfg", [
    dict(Nb=2, H=7, W=9, C=64, Cout=64),                          # ragged pixel count, one channel slice per tap
    dict(Nb=1, H=3, W=3, C=64, Cout=16),                          # every pixel but the centre sees padding
    dict(Nb=1, H=12, W=10, C=128, Cout=40),                       # two channel slices per tap, ragged Cout
    dict(Nb=3, H=9, W=9, C=64, Cout=96, stride=2),
    dict(Nb=2, H=8, W=8, C=192, Cout=64, R=1, S=1, pad=0),        # 1 x 1: a plain GEMM over pixels
    dict(Nb=1, H=10, W=11, C=64, Cout=64, R=5, S=5, pad=2),
    dict(Nb=1, H=9, W=12, C=64, Cout=32, R=3, S=1, pad=1),        # non-square filter, padding wider than the filter needs
    dict(Nb=2, H=14, W=14, C=256, Cout=300, pad=0),               # no padding, several column tiles
    dict(Nb=1, H=6, W=6, C=64, Cout=64, pad=3),                   # padding beyond the filter's reach
    dict(Nb=1, H=9, W=9, C=64, Cout=64, R=6, S=6, pad=2),         # 36 taps: more than the hand-scheduled loop's validity bits
    dict(Nb=2, H=11, W=13, C=128, Cout=130, R=2, S=4, pad=1, stride=2),  # even filter extents, two slices per tap
    # channel counts that are not a multiple of 64: a 64-deep k tile spans taps, the last one may end past K
    dict(Nb=2, H=7, W=9, C=96, Cout=64),                          # K = 864: 13 whole tiles and a half one
    dict(Nb=1, H=5, W=6, C=16, Cout=48),                          # four taps per tile, K = 144
    dict(Nb=2, H=9, W=8, C=48, Cout=72, stride=2),                # K = 432, three chunks per tap
    dict(Nb=1, H=8, W=8, C=80, Cout=64, R=5, S=5, pad=2),         # K = 2000
    dict(Nb=2, H=6, W=7, C=32, Cout=40, R=1, S=1, pad=0, stride=2),  # 1 x 1 with a stride: not a plain GEMM
    dict(Nb=1, H=6, W=6, C=160, Cout=64, pad=3),                  # padding beyond the filter's reach, K = 1440
    dict(Nb=2, H=8, W=8, C=96, Cout=64, R=1, S=1, pad=0),         # 1 x 1: the plain GEMM with a ragged K
])
@pytest.mark.parametrize("per_channel,with_bias,relu", [(True, True, False), (False, False, True)])
def test_dense_conv_bit_exact(env, cfg, per_channel, with_bias, relu):
    q, torch, dev, oracle = env
    say(f"dense conv {cfg} per_channel={per_channel}")
    c = wl.random_conv(11, G=1, per_channel=per_channel, with_bias=with_bias, relu=relu, **cfg)
    ref = want(c, oracle)
    for kernel in CONV_KERNELS:
        assert_same(run(c, q, torch, dev, kernel), ref, f"dense conv, kernel {kernel}")
    if cfg["C"] % 64 == 0 and cfg.get("R", 3) * cfg.get("S", 3) <= 32:   # the streaming kernels' conditions
        for kernel in ("skinny16", "skinny32", "skinny64"):
            assert_same(run(c, q, torch, dev, kernel), ref, f"dense conv, kernel {kernel}")


def test_dense_conv_zero_weight_zero_points(env):
    q, torch, dev, oracle = env
    c = wl.random_conv(12, Nb=2, H=9, W=7, C=64, G=1, Cout=48)
    c.b_zp[:] = 0
    assert_same(run(c, q, torch, dev), want(c, oracle), "dense conv, theta_B = 0")


def test_dense_conv_resnet_block_shape(env):
    """56 x 56 x 64 -> 64, 3 x 3, the first residual stage of a ResNet at batch 4: 12544 pixel rows, K = 576."""
    q, torch, dev, oracle = env
    c = wl.random_conv(13, Nb=4, H=56, W=56, C=64, G=1, Cout=64)
    ref = want(c, oracle)
    for kernel in CONV_KERNELS:
        assert_same(run(c, q, torch, dev, kernel), ref, f"dense conv 4x56x56x64, kernel {kernel}")
    assert np.mean((ref > 0) & (ref < 255)) > 0.5


def test_dense_conv_few_pixels_long_k(env):
    """7 x 7 x 512 -> 128, 3 x 3: 98 pixel rows and K = 4608, the shape the K-split wave sets are for (72 k tiles:
    an even and an odd share per set, taps that change inside a set's stride)."""
    q, torch, dev, oracle = env
    c = wl.random_conv(15, Nb=2, H=7, W=7, C=512, G=1, Cout=128)
    ref = want(c, oracle)
    for kernel in CONV_KERNELS:
        assert_same(run(c, q, torch, dev, kernel), ref, f"dense conv 2x7x7x512, kernel {kernel}")
    c = wl.random_conv(16, Nb=1, H=5, W=6, C=192, G=1, Cout=64)   # 27 k tiles: odd, and not a multiple of four
    ref = want(c, oracle)
    for kernel in CONV_KERNELS:
        assert_same(run(c, q, torch, dev, kernel), ref, f"dense conv 1x5x6x192, kernel {kernel}")


def test_dense_conv_errors(env):
    q, torch, dev, oracle = env
    c = wl.random_conv(14, Nb=1, H=5, W=5, C=64, G=1, Cout=64)
    Wp = q.pack_conv_dense_w(torch.from_numpy(np.ascontiguousarray(c.wgt[0])).to(dev), c.b_zp)
    inp = torch.from_numpy(c.inp).to(dev)
    out = torch.empty((1, 5, 5, 64), dtype=torch.uint8, device=dev)
    sc = torch.from_numpy(c.scales).to(dev)
    p = q.RequantParams(c.a_zp, None, sc.data_ptr(), sc.numel(), c.c_zp, 0)
    L = q.lib.qg_conv_dense_u8s8_requant
    assert L(inp.data_ptr(), 1, 5, 5, 64, 3, 3, 1, 1, Wp.handle, ctypes.byref(p), None, None, 0) == q.ENULL
    assert L(inp.data_ptr(), 1, 5, 5, 64, 1, 1, 0, 1, Wp.handle, ctypes.byref(p), out.data_ptr(), None, 0) == q.EINVAL  # K mismatch
    # extents no staged kernel takes: fine under the automatic choice (the byte-gathering kernel), refused with an explicit kernel id
    t64 = q.kernel_id("tile64")
    assert L(inp.data_ptr(), 1, 5, 5, 8, 9, 8, 4, 1, Wp.handle, ctypes.byref(p), out.data_ptr(), None, t64) == q.EUNSUPPORTED  # Cin % 16
    assert L(inp.data_ptr() + 4, 1, 5, 5, 64, 3, 3, 1, 1, Wp.handle, ctypes.byref(p), out.data_ptr(), None, t64) == q.EUNSUPPORTED
    assert L(inp.data_ptr(), 1, 1, 1, 64, 3, 3, 0, 1, Wp.handle, ctypes.byref(p), out.data_ptr(), None, 0) == q.EINVAL  # filter larger than image
    ok = (inp.data_ptr(), 1, 5, 5, 64, 3, 3, 1, 1, Wp.handle, ctypes.byref(p), out.data_ptr(), None)
    assert L(*ok, q.KERNEL_CONV_LAST + 1) == q.EINVAL and L(*ok, -1) == q.EINVAL
    assert L(*ok, q.kernel_id("tile256")) == q.EUNSUPPORTED
    torch.cuda.synchronize()


PATCH_KERNELS = ["patch64x128", "patch128x64", "patch256x64", "patch256", "patch512"]


@pytest.mark.parametrize("cfg", [
    dict(Nb=2, H=7, W=9, C=64, Cout=64),                          # ragged pixel count, borders on every side
    dict(Nb=1, H=3, W=3, C=64, Cout=16),                          # every pixel but the centre sees padding
    dict(Nb=1, H=12, W=10, C=128, Cout=40),                       # two slabs per tap, ragged Cout
    dict(Nb=3, H=9, W=9, C=32, Cout=96),                          # 32 channels: a slab holds two taps, K = 288 ends mid-slab
    dict(Nb=2, H=20, W=17, C=96, Cout=200),                       # 96 channels: taps change mid-slab; several tiles and slices
    dict(Nb=1, H=9, W=8, C=64, Cout=64, R=5, S=5, pad=2),         # 5 x 5
    dict(Nb=5, H=14, W=14, C=256, Cout=256),                      # images end inside tiles
    dict(Nb=1, H=1, W=1, C=32, Cout=1),                           # one pixel, one channel: only the centre tap is inside
    dict(Nb=1, H=40, W=70, C=160, Cout=130, R=5, S=5, pad=2),     # a wide image: the patch is several times the tile
])
@pytest.mark.parametrize("variant", range(4))
def test_dense_conv_patch_kernels(env, cfg, variant):
    """The kernels that keep a pixel tile's input patch in LDS, every form, against the oracle's direct convolution;
    the variants cover the three output forms (saturating convert with and without theta_C, explicit lower clamp) and
    weights without zero points (no row offsets)."""
    q, torch, dev, oracle = env
    say(f"dense conv, patch kernels {cfg}, variant {variant}")
    c = wl.random_conv(15100 + variant, G=1, per_channel=variant != 1, with_bias=variant != 2, relu=variant in (1, 3), **cfg)
    if variant == 2:
        c.b_zp[:] = 0
    c = dataclasses.replace(c, c_zp=[c.c_zp, 0, 0, 7][variant])
    ref = want(c, oracle)
    ran = 0
    for kernel in PATCH_KERNELS:
        try:
            got = run(c, q, torch, dev, kernel)
        except q.QGemmError as e:   # a form whose patch does not fit the LDS
            assert e.code == q.EUNSUPPORTED, f"{kernel} {cfg}"
            continue
        assert_same(got, ref, f"dense conv {cfg}, kernel {kernel}")
        ran += 1
    assert ran >= 3


@pytest.mark.parametrize("seed", range(16))
def test_dense_conv_patch_kernels_random_same_layers(env, seed):
    """Random "same" layers (3 x 3 and 5 x 5, any multiple of 32 channels, images from one pixel to wider than a tile)
    through every patch form and the automatic choice."""
    q, torch, dev, oracle = env
    rng = np.random.default_rng(15300 + seed)
    R = int(rng.choice([3, 3, 5]))
    cfg = dict(Nb=int(rng.integers(1, 4)), H=int(rng.integers(1, 24)), W=int(rng.integers(1, 90)), C=32 * int(rng.integers(1, 11)),
               Cout=int(rng.integers(1, 300)), R=R, S=R, pad=R // 2)
    say(f"dense conv, patch kernels, random layer {cfg}")
    c = wl.random_conv(15300 + seed, G=1, per_channel=bool(seed & 1), with_bias=bool(seed & 2), relu=bool(seed & 4), **cfg)
    if seed % 5 == 0:
        c.b_zp[:] = 0
    if seed % 3 == 0:
        c = dataclasses.replace(c, c_zp=0)
    ref = want(c, oracle)
    ran = 0
    for kernel in PATCH_KERNELS + ["auto"]:
        try:
            got = run(c, q, torch, dev, kernel)
        except q.QGemmError as e:   # a form whose patch does not fit the LDS
            assert e.code == q.EUNSUPPORTED and kernel != "auto", f"{kernel} {cfg}"
            continue
        assert_same(got, ref, f"dense conv {cfg}, kernel {kernel}")
        ran += 1
    assert ran >= 3


def test_dense_conv_patch_kernels_refuse_other_geometries(env):
    q, torch, dev, oracle = env
    for cfg in [dict(Nb=1, H=8, W=8, C=64, Cout=32, stride=2), dict(Nb=1, H=8, W=8, C=64, Cout=32, pad=0),
                dict(Nb=1, H=8, W=8, C=48, Cout=32), dict(Nb=1, H=8, W=8, C=64, Cout=32, R=3, S=5, pad=1),
                dict(Nb=1, H=9, W=9, C=32, Cout=32, R=7, S=7, pad=3), dict(Nb=1, H=8, W=8, C=64, Cout=32, R=1, S=1, pad=0)]:
        c = wl.random_conv(15200, G=1, **cfg)
        for kernel in PATCH_KERNELS:
            with pytest.raises(q.QGemmError) as err:
                run(c, q, torch, dev, kernel)
            assert err.value.code == q.EUNSUPPORTED, f"{kernel} {cfg}"


@pytest.mark.parametrize("seed", range(12))
def test_dense_conv_random_extents_any_multiple_of_16_channels(env, seed):
    """Random small layers: channel counts over the multiples of 16, filters 1..5 in each direction, padding 0..3,
    stride 1..2, every kernel id."""
    q, torch, dev, oracle = env
    rng = np.random.default_rng(9000 + seed)
    R, S = int(rng.integers(1, 6)), int(rng.integers(1, 6))
    pad, stride = int(rng.integers(0, 4)), int(rng.integers(1, 3))
    H = int(rng.integers(max(1, R - 2 * pad), 13))
    W = int(rng.integers(max(1, S - 2 * pad), 13))
    cfg = dict(Nb=int(rng.integers(1, 4)), H=H, W=W, C=16 * int(rng.integers(1, 14)), Cout=int(rng.integers(4, 100)),
               R=R, S=S, pad=pad, stride=stride)
    say(f"dense conv, random extents {cfg}")
    c = wl.random_conv(9100 + seed, G=1, per_channel=bool(seed & 1), with_bias=bool(seed & 2), relu=bool(seed & 4), **cfg)
    ref = want(c, oracle)
    for kernel in CONV_KERNELS:
        assert_same(run(c, q, torch, dev, kernel), ref, f"dense conv {cfg}, kernel {kernel}")


@pytest.mark.parametrize("cfg", [
    dict(Nb=2, H=9, W=11, C=3, Cout=32, stride=2),                 # a first layer: three channels
    dict(Nb=1, H=8, W=8, C=24, Cout=24),
    dict(Nb=2, H=7, W=6, C=70, Cout=33, R=2, S=5, pad=2),          # K = 700 crosses several 64-deep blocks of the packed matrix
    dict(Nb=1, H=6, W=6, C=1, Cout=5, R=1, S=1, pad=0),
    dict(Nb=3, H=19, W=17, C=3, Cout=150, R=7, S=7, pad=3, stride=2),   # several pixel and channel blocks, both ragged
    dict(Nb=2, H=13, W=13, C=5, Cout=70, R=3, S=3, pad=0, stride=3),    # taps that straddle the 16-byte pieces
    dict(Nb=1, H=10, W=12, C=17, Cout=64, R=3, S=1, pad=1),             # 17 channels: every piece starts mid-pixel
    dict(Nb=1, H=1, W=1, C=3, Cout=1, R=1, S=1, pad=0),                 # one output byte
    dict(Nb=2, H=19, W=15, C=4, Cout=64, R=7, S=7, pad=3, stride=2),    # RGB padded to four channels: gathered in 4-byte pieces
    dict(Nb=1, H=9, W=10, C=12, Cout=40, R=3, S=3, pad=1),              # 12 channels: taps change inside a thread's 16 bytes
    dict(Nb=2, H=6, W=7, C=20, Cout=33, R=5, S=3, pad=1, stride=2),     # K = 300: the last block ends mid-thread
    dict(Nb=1, H=5, W=5, C=8, Cout=16, R=1, S=1, pad=0),                # 1 x 1 on 8 channels
])
@pytest.mark.parametrize("variant", range(3))
def test_dense_conv_any_channel_count_on_the_gathering_kernel(env, cfg, variant):
    q, torch, dev, oracle = env
    say(f"dense conv, byte-gathering kernel {cfg}, variant {variant}")
    c = wl.random_conv(15 + variant, G=1, per_channel=variant != 1, with_bias=variant != 2, relu=variant == 1, **cfg)
    if variant == 2:   # all weight zero points zero: the variant without row offsets
        c.b_zp[:] = 0
    assert_same(run(c, q, torch, dev, "auto"), want(c, oracle), f"dense conv {cfg}")


def test_dense_conv_four_channel_image_off_a_4_byte_boundary(env):
    """Cin = 4 with the image 2 bytes off a 4-byte boundary: the gathering kernel's byte form, not its 4-byte form."""
    q, torch, dev, oracle = env
    c = wl.random_conv(17, Nb=2, H=9, W=8, C=4, G=1, Cout=32, R=5, S=5, pad=2)
    Wp = q.pack_conv_dense_w(torch.from_numpy(np.ascontiguousarray(c.wgt[0])).to(dev), c.b_zp)
    store = torch.zeros(c.inp.size + 16, dtype=torch.uint8, device=dev)
    store[2:2 + c.inp.size] = torch.from_numpy(c.inp.reshape(-1)).to(dev)
    out = torch.empty((2, 9, 8, 32), dtype=torch.uint8, device=dev)
    sc = torch.from_numpy(c.scales).to(dev)
    bias = torch.from_numpy(c.bias).to(dev)
    p = q.RequantParams(c.a_zp, bias.data_ptr(), sc.data_ptr(), sc.numel(), c.c_zp, int(c.relu))
    rc = q.lib.qg_conv_dense_u8s8_requant(store.data_ptr() + 2, 2, 9, 8, 4, 5, 5, c.pad, c.stride, Wp.handle, ctypes.byref(p),
                                          out.data_ptr(), None, 0)
    assert rc == q.OK
    torch.cuda.synchronize()
    assert_same(out.cpu().numpy(), want(c, oracle), "four channels, image 2 bytes off a 4-byte boundary")


def test_dense_conv_unaligned_image_on_the_gathering_kernel(env):
    q, torch, dev, oracle = env
    c = wl.random_conv(16, Nb=1, H=7, W=7, C=64, G=1, Cout=48)
    Wp = q.pack_conv_dense_w(torch.from_numpy(np.ascontiguousarray(c.wgt[0])).to(dev), c.b_zp)
    store = torch.zeros(c.inp.size + 16, dtype=torch.uint8, device=dev)
    store[4:4 + c.inp.size] = torch.from_numpy(c.inp.reshape(-1)).to(dev)
    inp = store[4:4 + c.inp.size].view(c.inp.shape)
    out = torch.empty((1, 7, 7, 48), dtype=torch.uint8, device=dev)
    sc = torch.from_numpy(c.scales).to(dev)
    bias = torch.from_numpy(c.bias).to(dev)
    p = q.RequantParams(c.a_zp, bias.data_ptr(), sc.data_ptr(), sc.numel(), c.c_zp, int(c.relu))
    rc = q.lib.qg_conv_dense_u8s8_requant(inp.data_ptr(), 1, 7, 7, 64, 3, 3, c.pad, c.stride, Wp.handle, ctypes.byref(p),
                                          out.data_ptr(), None, 0)
    assert rc == q.OK
    torch.cuda.synchronize()
    assert_same(out.cpu().numpy(), want(c, oracle), "image 4 bytes off a 16-byte boundary")
