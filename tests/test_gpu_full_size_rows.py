"""Full-size parity of the widening rows in the launch configurations bench.py times: fp32 output and fp32
activations at 8192^3 (sampled complete rows, one in every 256-row tile), the outlier split at 16 x 8192 x 8192,
the dense convolution layers at batch 32 (sampled images)."""
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


def _rows(M, tile, seed, extra):
    rng = np.random.default_rng(seed)
    rows = [t * tile + int(rng.integers(0, min(tile, M - t * tile))) for t in range((M + tile - 1) // tile)]
    rows += [0, M - 1] + [int(v) for v in rng.integers(0, M, extra)]
    return np.array(sorted(set(rows)))


def test_fp32_ends_at_the_headline_size(env):
    q, torch, dev, oracle = env
    c = wl.unsaturated(wl.config3_square())
    say("fp32 ends, 8192^3")
    rows = _rows(c.M, 256, 7, 8)
    A, B = torch.from_numpy(c.A).to(dev), torch.from_numpy(c.B).to(dev)
    bias, scales = torch.from_numpy(c.bias).to(dev), torch.from_numpy(c.scales).to(dev)
    Bp = q.pack_b(B, c.b_zp)
    # uint8 in, fp32 out
    out = q.gemm_u8s8_dequant_f32(A, c.a_zp, Bp, bias, scales, True)
    torch.cuda.synchronize()
    want = oracle.gemm_u8s8_dequant_f32(np.ascontiguousarray(c.A[rows]), c.a_zp, c.B, c.b_zp, c.bias, c.scales, True)
    assert_same(out[torch.from_numpy(rows).to(dev)].cpu().numpy().view(np.uint32), want.view(np.uint32), "fp32 out rows")
    del out
    # fp32 in (quantized by the library), uint8 out
    alpha, zp = 0.03, c.a_zp
    Af, inv = wl.random_fp32_activations(11, c.M, c.K, alpha=alpha, zp=zp, special=False)
    got = q.gemm_f32s8_requant(torch.from_numpy(Af).to(dev), inv, zp, Bp, bias, scales, c.c_zp, c.relu)
    torch.cuda.synchronize()
    Aq = oracle.quantize_f32(Af[rows], inv, zp)
    want8 = oracle.gemm_u8s8_requant(Aq, zp, c.B, c.b_zp, c.bias, c.scales, c.c_zp, c.relu)
    assert_same(got[torch.from_numpy(rows).to(dev)].cpu().numpy(), want8, "fp32 in rows")
    assert np.mean((want8 > 0) & (want8 < 255)) > 0.3


def test_outlier_split_at_the_benchmark_size(env):
    q, torch, dev, oracle = env
    say("outlier split, 16 x 8192 x 8192")
    M, N, K = 16, 8192, 8192
    c = wl.random_gemm(41, M, N, K, per_channel=False, with_bias=False)
    c.B = wl.outlier_weights(31, K, N, outlier_frac=0.01)
    c = wl.unsaturated(c)
    A, B = torch.from_numpy(c.A).to(dev), torch.from_numpy(c.B).to(dev)
    Bp = q.pack_b_outlier(B, c.b_zp)
    got = q.gemm_u8s8_requant(A, c.a_zp, Bp, None, torch.from_numpy(c.scales).to(dev), c.c_zp, c.relu)
    torch.cuda.synchronize()
    want = oracle.gemm_u8s8_requant(c.A, c.a_zp, c.B, c.b_zp, None, c.scales, c.c_zp, c.relu)
    assert_same(got.cpu().numpy(), want, "split 16 x 8192 x 8192")
    _, _, nnz = oracle.split_outliers(c.B, -8, 7)
    assert Bp.nnz == nnz


@pytest.mark.parametrize("H,C", [(56, 64), (28, 128), (14, 256)])
def test_dense_conv_layers_at_batch_32(env, H, C):
    q, torch, dev, oracle = env
    say(f"dense conv 32x{H}x{H}x{C}")
    c = wl.random_conv(40 + C, Nb=32, H=H, W=H, C=C, G=1, Cout=C)
    Wp = q.pack_conv_dense_w(torch.from_numpy(np.ascontiguousarray(c.wgt[0])).to(dev), c.b_zp)
    got = q.conv_dense_u8s8_requant(torch.from_numpy(c.inp).to(dev), Wp, c.a_zp, torch.from_numpy(c.bias).to(dev),
                                    torch.from_numpy(c.scales).to(dev), c.c_zp, c.relu).cpu().numpy()
    # images are independent: the oracle recomputes the first, the last and one in the middle
    for n in (0, 17, 31):
        want = oracle.conv_groupwise_direct(c.inp[n:n + 1], 1, c.wgt, c.a_zp, c.b_zp, c.bias, c.scales, c.c_zp, c.relu,
                                            c.pad, c.stride)
        assert_same(got[n:n + 1], want, f"image {n}")


@pytest.mark.parametrize("H,C,Cout", [(56, 64, 64), (56, 64, 128), (14, 512, 512)])
def test_patch_kernels_with_more_workgroups_than_places(env, H, C, Cout):
    """Batch 32: grids of several hundred workgroups, where the patch kernels run the build with the shallow weight
    ring (one more workgroup per CU); every form that takes the layer, three images against the oracle."""
    q, torch, dev, oracle = env
    say(f"dense conv 32x{H}x{H}x{C}->{Cout}, patch kernels")
    c = wl.random_conv(45 + C, Nb=32, H=H, W=H, C=C, G=1, Cout=Cout)
    Wp = q.pack_conv_dense_w(torch.from_numpy(np.ascontiguousarray(c.wgt[0])).to(dev), c.b_zp)
    x, b, sc = torch.from_numpy(c.inp).to(dev), torch.from_numpy(c.bias).to(dev), torch.from_numpy(c.scales).to(dev)
    want = {n: oracle.conv_groupwise_direct(c.inp[n:n + 1], 1, c.wgt, c.a_zp, c.b_zp, c.bias, c.scales, c.c_zp, c.relu,
                                            c.pad, c.stride) for n in (0, 17, 31)}
    ran = 0
    for kernel in ["patch64x128", "patch128x64", "patch256x64", "patch256", "patch512"]:
        try:
            got = q.conv_dense_u8s8_requant(x, Wp, c.a_zp, b, sc, c.c_zp, c.relu, pad=c.pad, stride=c.stride, kernel=kernel)
        except q.QGemmError:
            continue   # the patch does not fit the LDS at this tile and channel count
        torch.cuda.synchronize()
        got = got.cpu().numpy()
        for n, w in want.items():
            assert_same(got[n:n + 1], w, f"kernel {kernel}, image {n}")
        ran += 1
    assert ran >= 2


@pytest.mark.parametrize("cfg,kernels", [
    (dict(Nb=8, H=56, W=56, C=128, Cout=128), ["auto", "tile128", "tile128x256", "tile64k1", "patch64x128", "patch256", "patch512"]),   # the hand-scheduled loops, the patch kernels
    (dict(Nb=8, H=56, W=56, C=96, Cout=96), ["auto", "tile128", "patch128x64"]),                    # 16-channel chunks; taps that change mid-slab
    (dict(Nb=8, H=56, W=56, C=64, Cout=64), ["auto", "patch256x64", "tile64k1"]),
    (dict(Nb=2, H=7, W=7, C=512, Cout=128), ["auto", "skinny16", "skinny32", "tile64x32k8"]),    # few pixels, K = 4608
    (dict(Nb=4, H=14, W=14, C=256, Cout=256, stride=2), ["auto", "skinny64", "tile64"]),
    (dict(Nb=2, H=224, W=224, C=3, Cout=32, stride=2), ["auto"]),                               # first layers: the byte-gathering kernel
    (dict(Nb=1, H=224, W=224, C=3, Cout=64, R=7, S=7, pad=3, stride=2), ["auto"]),
])
def test_dense_conv_layers_on_every_competing_kernel(env, cfg, kernels):
    """Real layer sizes through the kernels that compete for them, the whole output against the oracle's direct convolution."""
    q, torch, dev, oracle = env
    say(f"dense conv {cfg}")
    c = wl.random_conv(50 + cfg["C"], G=1, **cfg)
    want = oracle.conv_groupwise_direct(c.inp, 1, c.wgt, c.a_zp, c.b_zp, c.bias, c.scales, c.c_zp, c.relu, c.pad, c.stride)
    Wp = q.pack_conv_dense_w(torch.from_numpy(np.ascontiguousarray(c.wgt[0])).to(dev), c.b_zp)
    x, b, sc = torch.from_numpy(c.inp).to(dev), torch.from_numpy(c.bias).to(dev), torch.from_numpy(c.scales).to(dev)
    for kernel in kernels:
        got = q.conv_dense_u8s8_requant(x, Wp, c.a_zp, b, sc, c.c_zp, c.relu, pad=c.pad, stride=c.stride, kernel=kernel)
        torch.cuda.synchronize()
        assert_same(got.cpu().numpy(), want, f"kernel {kernel}")


@pytest.mark.parametrize("cfg", [
    dict(Nb=32, H=56, W=56, C=128, G=128),             # depthwise
    dict(Nb=32, H=28, W=28, C=512, G=32),              # 16 -> 16
    dict(Nb=8, H=56, W=56, C=128, G=2),                # 64 -> 64: one dense convolution per group
    dict(Nb=2, H=28, W=28, C=40, G=5, Cout=60),        # 8 -> 12: the one-thread-per-output kernel
])
def test_group_conv_shapes_at_layer_sizes(env, cfg):
    q, torch, dev, oracle = env
    say(f"group conv {cfg}")
    c = wl.random_conv(60 + cfg["G"], **cfg)
    Wp = q.pack_conv_w(torch.from_numpy(c.wgt).to(dev), c.b_zp)
    got = q.conv_groupwise_u8s8_requant(torch.from_numpy(c.inp).to(dev), Wp, c.a_zp, torch.from_numpy(c.bias).to(dev),
                                        torch.from_numpy(c.scales).to(dev), c.c_zp, c.relu).cpu().numpy()
    # images are independent: the oracle recomputes the first, the last and one in the middle
    for n in sorted({0, cfg["Nb"] // 2, cfg["Nb"] - 1}):
        want = oracle.conv_groupwise_direct(c.inp[n:n + 1], c.G, c.wgt, c.a_zp, c.b_zp, c.bias, c.scales, c.c_zp, c.relu,
                                            c.pad, c.stride)
        assert_same(got[n:n + 1], want, f"image {n}")


@pytest.mark.parametrize("shape,kernels", [
    ((128, 4096, 4096), ["auto", "tile64", "tile64k4", "tile64x32k8", "skinny64"]),
    ((2048, 2048, 2048), ["auto", "tile128", "tile128x256"]),
    ((4096, 1024, 1024), ["auto", "tile128", "tile256"]),
    ((16384, 256, 512), ["auto", "tile64", "tile256"]),
])
def test_kernel_family_at_the_benchmark_shapes(env, shape, kernels):
    """The shapes of bench.py's kernel-family rows, through the automatic choice and the kernels that compete for
    them: sampled complete rows (one per 64-row block of a sample of blocks, first and last row) against the oracle,
    and all kernels byte-identical to each other on the whole output."""
    q, torch, dev, oracle = env
    M, N, K = shape
    say(f"kernel family {shape}")
    c = wl.unsaturated(wl.random_gemm(900 + M % 97 + N % 89, M, N, K, per_channel=True, with_bias=True, relu=True))
    rows = _rows(M, 64, 13, 4)
    if rows.size > 48:
        rows = np.unique(np.concatenate([rows[:: rows.size // 40], rows[-2:]]))
    A, B = torch.from_numpy(c.A).to(dev), torch.from_numpy(c.B).to(dev)
    bias, scales = torch.from_numpy(c.bias).to(dev), torch.from_numpy(c.scales).to(dev)
    Bp = q.pack_b(B, c.b_zp)
    want = oracle.gemm_u8s8_requant(np.ascontiguousarray(c.A[rows]), c.a_zp, c.B, c.b_zp, c.bias, c.scales, c.c_zp,
                                    c.relu)
    assert np.mean((want > 0) & (want < 255)) > 0.3
    first = None
    for kernel in kernels:
        got = q.gemm_u8s8_requant(A, c.a_zp, Bp, bias, scales, c.c_zp, c.relu, kernel=kernel)
        torch.cuda.synchronize()
        assert_same(got[torch.from_numpy(rows).to(dev)].cpu().numpy(), want, f"{kernel} rows of {shape}")
        if first is None:
            first = got
        else:
            assert torch.equal(first, got), f"{kernel} differs from {kernels[0]} on {shape}"


def test_activations_beyond_32_bit_offsets(env):
    """An A of more than 4 GiB: the kernels address A with 32-bit offsets from a base, so the library runs it as
    several launches over row ranges.  Rows around the seam, the first and the last row against the oracle, for
    the automatic choice, a tiled and a streaming kernel."""
    q, torch, dev, oracle = env
    M, N, K = 1_050_000, 32, 4096
    say(f"large A {M} x {K}")
    rng = np.random.default_rng(2024)
    B = rng.integers(-128, 128, size=(K, N), dtype=np.int8)
    b_zp = rng.integers(-4, 5, size=N).astype(np.int32)
    bias = rng.integers(-1000, 1001, size=N).astype(np.int32)
    scales = (40.0 / (np.sqrt(K) * 74.0 * 74.0) * 2.0 ** rng.uniform(-1, 1, size=N)).astype(np.float32)
    a_zp, c_zp = 131, 120
    A = torch.empty((M, K), dtype=torch.uint8, device=dev)
    seam = ((1 << 32) - K - 4096) // K // 256 * 256
    rows = np.array(sorted({0, 1, 255, seam - 256, seam - 1, seam, seam + 1, seam + 255, M - 257, M - 2, M - 1}))
    # seeded fill, block by block (host memory stays small); the sampled rows are kept for the oracle
    kept = {}
    blk = 65536
    for r0 in range(0, M, blk):
        n = min(blk, M - r0)
        a = np.random.default_rng(5000 + r0 // blk).integers(0, 256, size=(n, K), dtype=np.uint8)
        A[r0:r0 + n].copy_(torch.from_numpy(a).to(dev))
        for r in rows[(rows >= r0) & (rows < r0 + n)]:
            kept[int(r)] = a[r - r0].copy()
    Arows = np.stack([kept[int(r)] for r in rows])
    want = oracle.gemm_u8s8_requant(Arows, a_zp, B, b_zp, bias, scales, c_zp, False)
    assert np.mean((want > 0) & (want < 255)) > 0.3
    Bp = q.pack_b(torch.from_numpy(B).to(dev), b_zp)
    d_bias, d_scales = torch.from_numpy(bias).to(dev), torch.from_numpy(scales).to(dev)
    idx = torch.from_numpy(rows).to(dev)
    first = None
    for kernel in ("auto", "tile256", "skinny64"):
        say(f"  kernel {kernel}")
        got = q.gemm_u8s8_requant(A, a_zp, Bp, d_bias, d_scales, c_zp, False, kernel=kernel)
        torch.cuda.synchronize()
        assert_same(got[idx].cpu().numpy(), want, f"{kernel} rows of the large A")
        if first is None:
            first = got
        else:
            assert torch.equal(first, got), f"{kernel} differs from the automatic choice"
