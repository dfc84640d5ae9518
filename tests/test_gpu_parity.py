"""GPU parity: the HIP path, called through the C ABI, against the CPU oracle, bit for bit.

Integer results (column offsets, row sums, int32 accumulators) and requantized uint8 outputs must be
identical: every step is integer arithmetic or a fixed sequence of correctly rounded fp32 operations, so
exactly one result is right and the tolerance is zero.
"""
import numpy as np
import pytest

from paper_2101_05615_amd import workloads as wl
from gpu_util import assert_same, dev_case, oracle_gemm, run_gemm, say

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def env():
    import torch
    assert torch.cuda.is_available(), "these tests need the MI355X"
    from paper_2101_05615_amd import qgemm as q
    import oracle
    oracle.build()
    return q, torch, torch.device("cuda:0"), oracle


# ---------------------------------------------------------------- sub-results
@pytest.mark.parametrize("K,N,per_channel", [(128, 64, False), (36, 4, True), (100, 100, True), (4097, 257, True),
                                             (1, 1, False), (4096, 512, True)])
def test_col_offsets_match_oracle(env, K, N, per_channel):
    q, torch, dev, oracle = env
    say(f"col_offsets K={K} N={N}")
    c = wl.random_gemm(K + N, 2, N, K, per_channel=per_channel, wide_zp=True)
    Bp = q.pack_b(torch.from_numpy(c.B).to(dev), c.b_zp)
    torch.cuda.synchronize()
    assert_same(Bp.col_offsets.cpu().numpy(), oracle.col_offsets(c.B, c.b_zp), "col_offsets")


def test_pack_b_accepts_strided_b(env):
    q, torch, dev, oracle = env
    c = wl.random_gemm(77, 20, 50, 90, wide_zp=True)
    big = torch.zeros((90, 64), dtype=torch.int8, device=dev)
    big[:, :50] = torch.from_numpy(c.B).to(dev)
    Bp = q.pack_b(big[:, :50], c.b_zp)
    acc = q.gemm_u8s8_acc32(torch.from_numpy(c.A).to(dev), Bp)
    torch.cuda.synchronize()
    assert_same(Bp.col_offsets.cpu().numpy(), oracle.col_offsets(c.B, c.b_zp), "col_offsets strided")
    assert_same(acc.cpu().numpy(), oracle.acc32(c.A, c.B), "acc32 strided B")


@pytest.mark.parametrize("K,N", [(128, 64), (100, 100), (4097, 257), (1, 1), (512, 300)])
def test_pack_from_the_transposed_weight_matrix(env, K, N):
    """Packing B^T (N x K, the layout frameworks keep weights in) gives the same bytes as packing B."""
    q, torch, dev, oracle = env
    c = wl.random_gemm(K + N, 40, N, K, wide_zp=True)
    B = torch.from_numpy(c.B).to(dev)
    store = torch.zeros((N, K + 5), dtype=torch.int8, device=dev)   # padded rows: ldbt > K
    store[:, :K] = B.t()
    p1, p2 = q.pack_b(B, c.b_zp), q.pack_b_transposed(store[:, :K], c.b_zp)
    torch.cuda.synchronize()
    assert torch.equal(p1.packed, p2.packed), "packed bytes differ"
    assert torch.equal(p1.aux, p2.aux), "col_offsets / theta_B differ"
    assert_same(p2.col_offsets.cpu().numpy(), oracle.col_offsets(c.B, c.b_zp), "col_offsets")
    A, _, bias, scales, C, _ = dev_case(c, torch, dev)
    q.gemm_u8s8_requant(A, c.a_zp, p2, bias, scales, c.c_zp, c.relu, out=C)
    torch.cuda.synchronize()
    assert_same(C.cpu().numpy(), oracle_gemm(c, oracle), "GEMM on the transposed-packed weights")


ACC_SHAPES = [  # (M, N, K): both kernels (M <= 64 skinny, above: large tile), ragged in every dimension
    (1, 1, 1), (1, 16, 64), (16, 16, 64), (16, 32, 128), (16, 100, 300), (17, 40, 36), (33, 257, 4097),
    (64, 64, 128), (5, 4, 36), (48, 512, 1024),
    (65, 64, 128), (255, 100, 100), (256, 256, 128), (257, 300, 129), (300, 4, 36), (512, 512, 512),
    (700, 520, 4097), (1024, 256, 2048),
    # aligned shapes that take the pipelined paths: 4 / 5 / many 64-deep tiles, several batches per wave
    (300, 512, 256), (512, 256, 320), (260, 256, 192), (16, 256, 8448), (5, 64, 4224), (16, 512, 12288),
    (40, 128, 4096),
]


@pytest.mark.parametrize("M,N,K", ACC_SHAPES)
def test_int32_accumulators_and_row_sums_bit_exact(env, M, N, K):
    q, torch, dev, oracle = env
    say(f"acc32 M={M} N={N} K={K}")
    c = wl.random_gemm(M * 7 + N * 3 + K, M, N, K, wide_zp=True)
    Bp = q.pack_b(torch.from_numpy(c.B).to(dev), c.b_zp)
    acc, rs = q.gemm_u8s8_acc32(torch.from_numpy(c.A).to(dev), Bp, want_rowsum=True)
    torch.cuda.synchronize()
    assert_same(acc.cpu().numpy(), oracle.acc32(c.A, c.B), "acc32")
    assert_same(rs.cpu().numpy(), oracle.rowsum(c.A), "rowsum")


def test_accumulator_extremes_do_not_saturate(env):
    # all-255 activations against all -128 / +127 weights at the largest K: |acc| ~ 1.07e9, still exact int32
    q, torch, dev, oracle = env
    K = q.MAX_K
    for M in (16, 80):
        for b in (-128, 127):
            say(f"extremes M={M} b={b}")
            A = np.full((M, K), 255, np.uint8)
            B = np.full((K, 20), b, np.int8)
            Bp = q.pack_b(torch.from_numpy(B).to(dev), np.zeros(1, np.int32))
            acc, rs = q.gemm_u8s8_acc32(torch.from_numpy(A).to(dev), Bp, want_rowsum=True)
            torch.cuda.synchronize()
            assert np.all(acc.cpu().numpy() == 255 * b * K)
            assert np.all(rs.cpu().numpy() == 255 * K)


# ------------------------------------------------------------ requantized C
REQ_SHAPES = [
    (1, 1, 1), (1, 4, 36), (16, 64, 128), (16, 100, 100), (17, 100, 100), (31, 33, 65), (64, 257, 4097),
    (65, 64, 128), (100, 4, 36), (255, 100, 100), (256, 256, 256), (257, 255, 127), (300, 300, 300),
    (513, 264, 1000),
    (300, 512, 256), (512, 256, 320), (260, 256, 192), (16, 256, 8448), (5, 64, 4224), (640, 384, 1024),
]


@pytest.mark.parametrize("M,N,K", REQ_SHAPES)
@pytest.mark.parametrize("per_channel,relu,with_bias", [(True, False, True), (False, True, False)])
def test_requant_bit_exact_on_ragged_shapes(env, M, N, K, per_channel, relu, with_bias):
    q, torch, dev, oracle = env
    say(f"requant M={M} N={N} K={K} pc={per_channel} relu={relu} bias={with_bias}")
    c = wl.random_gemm(M + 2 * N + 3 * K, M, N, K, per_channel=per_channel, with_bias=with_bias, relu=relu)
    got, _, _ = run_gemm(c, q, torch, dev)
    want = oracle_gemm(c, oracle)
    assert_same(got, want, c.name)
    if M * N >= 4096:
        inside = np.mean((want > 0) & (want < 255))
        assert inside > 0.3, f"parity case is mostly saturated ({inside:.2f} unsaturated)"


@pytest.mark.parametrize("M,N,K", [(16, 100, 100), (40, 260, 300), (200, 100, 100), (300, 260, 300)])
def test_unaligned_pointers_and_padded_leading_dimensions(env, M, N, K):
    # lda/ldc not multiples of 16 and odd base addresses: the byte-wise load/store paths; and the guard bytes
    # around C must stay untouched
    q, torch, dev, oracle = env
    c = wl.random_gemm(M + N + K, M, N, K)
    want = oracle_gemm(c, oracle)
    for (lp, cp, ao, co) in [(3, 5, 1, 3), (16, 16, 0, 0), (0, 0, 16, 16), (12, 4, 4, 8)]:
        say(f"unaligned M={M} N={N} K={K} lda+{lp} ldc+{cp} a_off={ao} c_off={co}")
        got, store, _ = run_gemm(c, q, torch, dev, lda_pad=lp, ldc_pad=cp, a_off=ao, c_off=co)
        assert_same(got, want, f"{c.name} lda+{lp} ldc+{cp}")
        guard = store.copy()
        view = guard[co:co + M * (N + cp)].reshape(M, N + cp)
        view[:, :N] = 0xEE
        assert np.all(guard == 0xEE), "bytes outside C were written"


@pytest.mark.parametrize("a_zp,b_zp,c_zp", [(0, -128, 0), (255, 127, 255), (0, 127, 128), (255, -128, 1), (128, 0, 0)])
@pytest.mark.parametrize("M", [16, 130])
def test_extreme_zero_points(env, a_zp, b_zp, c_zp, M):
    q, torch, dev, oracle = env
    say(f"zp extremes M={M} a_zp={a_zp} b_zp={b_zp} c_zp={c_zp}")
    c = wl.random_gemm(a_zp + c_zp + M, M, 72, 500, per_channel=False, a_zp=a_zp, c_zp=c_zp, unsat=False)
    c.b_zp = np.array([b_zp], np.int32)
    c.scales = np.array([2.0 ** -12], np.float32)
    got, _, _ = run_gemm(c, q, torch, dev)
    assert_same(got, oracle_gemm(c, oracle), c.name)


ALL_KERNELS = ["skinny16", "skinny32", "skinny64", "tile64", "tile128", "tile128x256", "tile256", "tile64k4", "tile64k1",
               "tile64x32k8"]


def _hand_rows():
    import os
    rows = []
    with open(os.path.join(os.path.dirname(__file__), "golden", "requant_hand_cases.txt")) as f:
        for line in f:
            line = line.split("#")[0].strip()
            if line:
                x, s, z, r, e = line.split()
                rows.append((int(x), float(s), int(z), int(r), int(e)))
    return rows


@pytest.mark.parametrize("relu,c_zp", [(0, 0), (0, 10), (1, 0), (1, 10), (0, 255)])
@pytest.mark.parametrize("kernel", ["auto"] + ALL_KERNELS)
def test_hand_worked_rounding_cases_through_every_kernel(env, kernel, relu, c_zp):
    """The hand-worked ties, saturation rows and +-2^31 accumulators of tests/golden/requant_hand_cases.txt through
    every kernel's output pipeline -- both forms of it: the explicit clamp (ReLU with theta_C != 0) and the saturating
    convert -- at K = 256, so that the hand-scheduled tiles run their own loop.  x is injected through the bias of a
    column whose accumulator is zero (A = theta_A everywhere), one column per (x, scale) pair; theta_C and ReLU are per
    call, so every pair is also run under the other combinations, where the expected byte is the oracle's per-element
    function (itself pinned to the hand-worked values on the CPU)."""
    q, torch, dev, oracle = env
    rows = _hand_rows()
    pairs = sorted({(x, s) for x, s, _, _, _ in rows})
    M, K, N = 130, 256, len(pairs)
    A = np.full((M, K), 7, np.uint8)
    B = np.ones((K, N), np.int8)
    bias = np.array([x for x, _ in pairs], np.int32)
    scales = np.array([s for _, s in pairs], np.float32)
    c = wl.GemmCase("hand", A, 7, B, np.zeros(1, np.int32), bias, scales, c_zp, bool(relu))
    want = np.array([oracle.requant_one(x, s, c_zp, relu) for x, s in pairs], np.uint8)
    n_golden = 0
    for x, s, z, r, e in rows:  # the rows worked by hand for exactly this (theta_C, ReLU)
        if z == c_zp and r == relu:
            assert want[pairs.index((x, s))] == e
            n_golden += 1
    say(f"hand cases: kernel {kernel} relu {relu} c_zp {c_zp}: {N} columns, {n_golden} of them hand-worked for this combination")
    Ad, Bd, biasd, scalesd, C, _ = dev_case(c, torch, dev)
    Bp = q.pack_b(Bd, c.b_zp)
    q.gemm_u8s8_requant(Ad, c.a_zp, Bp, biasd, scalesd, c.c_zp, c.relu, out=C, kernel=kernel)
    torch.cuda.synchronize()
    got = C.cpu().numpy()
    assert_same(got, np.broadcast_to(want, (M, N)), f"{kernel} hand cases")


# ---------------------------------------------------- the five stated configs
@pytest.mark.parametrize("kernel", ["auto"] + ALL_KERNELS)
def test_config1_tiny(env, kernel):
    q, torch, dev, oracle = env
    c = wl.config1_tiny()
    for case in (c, wl.unsaturated(c)):
        Ad, Bd, biasd, scalesd, C, _ = dev_case(case, torch, dev)
        Bp = q.pack_b(Bd, case.b_zp)
        q.gemm_u8s8_requant(Ad, case.a_zp, Bp, biasd, scalesd, case.c_zp, case.relu, out=C, kernel=kernel)
        torch.cuda.synchronize()
        assert_same(C.cpu().numpy(), oracle_gemm(case, oracle), f"{case.name} {kernel}")


@pytest.mark.parametrize("relu,c_zp", [(0, 0), (1, 10)])
@pytest.mark.parametrize("kernel", ALL_KERNELS)
def test_tie_rich_scale_at_a_depth_the_hand_scheduled_loops_take(env, kernel, relu, c_zp):
    """Config 1's scale 2^-10 makes the product exact and exact .5 ties frequent (about one output in a thousand);
    here at K = 512 and over several tiles, so that the 128- and 256-row kernels run their hand-scheduled loops."""
    q, torch, dev, oracle = env
    c = wl.random_gemm(4242, 200, 330, 512, per_channel=False, with_bias=True, relu=bool(relu), a_zp=128, c_zp=c_zp)
    c.scales = np.array([2.0 ** -10], np.float32)
    c.b_zp = np.zeros(1, np.int32)
    want, x = oracle.gemm_u8s8_requant(c.A, c.a_zp, c.B, c.b_zp, c.bias, c.scales, c.c_zp, c.relu, return_x=True)
    ties = int(np.sum(np.abs(x) % 1024 == 512))
    assert ties >= 20, ties
    Ad, Bd, biasd, scalesd, C, _ = dev_case(c, torch, dev)
    Bp = q.pack_b(Bd, c.b_zp)
    q.gemm_u8s8_requant(Ad, c.a_zp, Bp, biasd, scalesd, c.c_zp, c.relu, out=C, kernel=kernel)
    torch.cuda.synchronize()
    assert_same(C.cpu().numpy(), want, f"{kernel} ties ({ties} exact halves)")


@pytest.mark.parametrize("with_bias", [False, True])
def test_config2_small_batch_fc_full(env, with_bias):
    q, torch, dev, oracle = env
    c = wl.config2_small_batch_fc(with_bias=with_bias)
    say(c.name)
    got, _, _ = run_gemm(c, q, torch, dev)
    assert_same(got, oracle_gemm(c, oracle), c.name)
    u = wl.unsaturated(c)
    got, _, _ = run_gemm(u, q, torch, dev)
    want = oracle_gemm(u, oracle)
    assert_same(got, want, u.name)
    assert np.mean((want > 0) & (want < 255)) > 0.5


def _sampled_rows(M, tile, rng, extra):
    rows = [t * tile + int(rng.integers(0, min(tile, M - t * tile))) for t in range((M + tile - 1) // tile)]
    rows += [0, M - 1] + [int(v) for v in rng.integers(0, M, extra)]
    return np.array(sorted(set(rows)))


def test_config3_square_full_size_sampled_rows(env):
    # the launch configuration bench.py times; the oracle recomputes complete rows (all 8192 columns), at
    # least one in every 256-row tile, so every workgroup tile of the grid is checked
    q, torch, dev, oracle = env
    c = wl.config3_square()
    say(c.name)
    rows = _sampled_rows(c.M, 256, np.random.default_rng(0), 16)
    for case in (c, wl.unsaturated(c)):
        got, _, Bp = run_gemm(case, q, torch, dev)
        assert_same(got[rows], oracle_gemm(case, oracle, rows), case.name + " sampled rows")
        assert_same(Bp.col_offsets.cpu().numpy(), oracle.col_offsets(case.B, case.b_zp), "col_offsets")
    # properties that hold at any size: determinism, and ReLU lower bound = theta_C
    got2, _, _ = run_gemm(c, q, torch, dev)
    got1, _, _ = run_gemm(c, q, torch, dev)
    assert np.array_equal(got1, got2)
    assert got1.min() >= c.c_zp


def test_config4_recsys_mlp_full_output(env):
    """All 32768 x 512 outputs of config 4 (and of its unsaturated variant) against the oracle: every one of the 128
    row tiles, through the variant without row offsets (theta_B = 0)."""
    q, torch, dev, oracle = env
    c = wl.config4_recsys_mlp()
    say(c.name)
    for case in (c, wl.unsaturated(c)):
        got, _, _ = run_gemm(case, q, torch, dev)
        assert_same(got, oracle_gemm(case, oracle), case.name + " all rows")


def test_determinism_and_independence_of_m_padding(env):
    # the same rows give the same bytes whether they are computed alone (small-batch kernel) or as part
    # of a larger batch (large-tile kernel): any K split or tile order must produce identical integers
    q, torch, dev, oracle = env
    c = wl.random_gemm(99, 300, 200, 700)
    full, _, _ = run_gemm(c, q, torch, dev)
    sub = wl.GemmCase("sub", np.ascontiguousarray(c.A[:16]), c.a_zp, c.B, c.b_zp, c.bias, c.scales, c.c_zp, c.relu)
    part, _, _ = run_gemm(sub, q, torch, dev)
    assert_same(part, full[:16], "skinny vs tile kernel")


# ------------------------------------------------------------------ group conv
def _run_conv(c, q, torch, dev):
    Wp = q.pack_conv_w(torch.from_numpy(c.wgt).to(dev), c.b_zp)
    bias = None if c.bias is None else torch.from_numpy(c.bias).to(dev)
    out = q.conv_groupwise_u8s8_requant(torch.from_numpy(c.inp).to(dev), Wp, c.a_zp, bias,
                                        torch.from_numpy(c.scales).to(dev), c.c_zp, c.relu, c.pad, c.stride)
    torch.cuda.synchronize()
    return out.cpu().numpy(), Wp


def _oracle_conv(c, oracle):
    return oracle.conv_groupwise_direct(c.inp, c.G, c.wgt, c.a_zp, c.b_zp, c.bias, c.scales, c.c_zp, c.relu,
                                        c.pad, c.stride)


@pytest.mark.parametrize("cfg", [
    dict(Nb=1, H=3, W=3, C=4, G=1), dict(Nb=2, H=5, W=7, C=16, G=4), dict(Nb=1, H=9, W=6, C=128, G=32),
    dict(Nb=3, H=8, W=8, C=32, G=8, stride=2), dict(Nb=1, H=6, W=6, C=8, G=2, pad=0),
    dict(Nb=1, H=5, W=5, C=12, G=3, pad=2), dict(Nb=2, H=4, W=4, C=16, G=4, R=1, S=1, pad=0),
    dict(Nb=1, H=1, W=1, C=4, G=1),
    # matrix-core kernels: one and several 32-channel blocks, two channel groups, 1x1, an image too wide for the
    # LDS-staged patch (falls back to taps from global memory), a pixel count that is not a multiple of 32 or 128
    dict(Nb=2, H=7, W=9, C=64, G=16), dict(Nb=1, H=5, W=5, C=256, G=64), dict(Nb=3, H=6, W=6, C=128, G=32, R=1, S=1, pad=0),
    dict(Nb=1, H=3, W=600, C=128, G=32), dict(Nb=2, H=13, W=11, C=128, G=32), dict(Nb=1, H=8, W=8, C=32, G=8, pad=0),
    dict(Nb=2, H=9, W=9, C=128, G=32, stride=2),
])
@pytest.mark.parametrize("per_channel,with_bias,relu", [(True, True, False), (False, False, True)])
def test_group_conv_bit_exact_small(env, cfg, per_channel, with_bias, relu):
    q, torch, dev, oracle = env
    say(f"conv {cfg}")
    c = wl.random_conv(5, per_channel=per_channel, with_bias=with_bias, relu=relu, **cfg)
    got, Wp = _run_conv(c, q, torch, dev)
    assert_same(got, _oracle_conv(c, oracle), c.name)


def test_group_conv_zero_weight_zero_point_variant(env):
    # theta_B == 0 selects the kernel variants without row offsets
    q, torch, dev, oracle = env
    for cfg in (dict(Nb=2, H=8, W=8, C=128, G=32), dict(Nb=1, H=6, W=7, C=32, G=8), dict(Nb=1, H=5, W=5, C=8, G=2)):
        c = wl.random_conv(11, **cfg)
        c.b_zp = np.zeros(1, np.int32)
        got, _ = _run_conv(c, q, torch, dev)
        assert_same(got, _oracle_conv(c, oracle), c.name + "_bzp0")


def test_config5_group_conv_full(env):
    q, torch, dev, oracle = env
    c = wl.config5_group_conv()
    say(c.name)
    got, _ = _run_conv(c, q, torch, dev)
    want = _oracle_conv(c, oracle)
    assert_same(got, want, c.name)
    # parity-sensitive variant: scales sized so most outputs are unsaturated
    c.scales = (c.scales * 0 + 40.0 / (6.0 * 74.0 * 74.0)).astype(np.float32)
    got, _ = _run_conv(c, q, torch, dev)
    want = _oracle_conv(c, oracle)
    assert_same(got, want, c.name + "_unsat")
    assert np.mean((want > 0) & (want < 255)) > 0.5


# ------------------------------------------------------------- error handling
def test_runtime_argument_errors(env):
    import ctypes
    q, torch, dev, oracle = env
    c = wl.config1_tiny()
    A, B, bias, scales, C, _ = dev_case(c, torch, dev)
    Bp = q.pack_b(B, c.b_zp)
    bad = [dict(a_zp=256), dict(a_zp=-1), dict(c_zp=256), dict(n_scales=2), dict(relu=2)]
    for kw in bad:
        p = q.RequantParams(128, None, scales.data_ptr(), 1, 0, 0)
        for k, v in kw.items():
            setattr(p, k, v)
        rc = q.lib.qg_gemm_u8s8_requant(A.data_ptr(), 64, 128, Bp.handle, ctypes.byref(p), C.data_ptr(), 64, None, None)
        assert rc == q.EINVAL, kw
    p = q.RequantParams(128, None, scales.data_ptr(), 1, 0, 0)
    assert q.lib.qg_gemm_u8s8_requant(A.data_ptr(), 64, 127, Bp.handle, ctypes.byref(p), C.data_ptr(), 64, None, None) == q.EINVAL
    assert q.lib.qg_gemm_u8s8_requant(A.data_ptr(), 64, 128, Bp.handle, ctypes.byref(p), C.data_ptr(), 63, None, None) == q.EINVAL
    assert q.lib.qg_gemm_u8s8_requant(A.data_ptr(), -1, 128, Bp.handle, ctypes.byref(p), C.data_ptr(), 64, None, None) == q.EINVAL
    assert q.lib.qg_gemm_u8s8_requant(A.data_ptr(), 64, 128, Bp.handle, ctypes.byref(p), None, 64, None, None) == q.ENULL
    p.scales = None
    assert q.lib.qg_gemm_u8s8_requant(A.data_ptr(), 64, 128, Bp.handle, ctypes.byref(p), C.data_ptr(), 64, None, None) == q.ENULL
    with pytest.raises(q.QGemmError) as ei:
        q.pack_b(B, np.array([200], np.int32))  # theta_B outside int8
    assert ei.value.code == q.EINVAL
    # a conv descriptor is not a GEMM descriptor
    cc = wl.random_conv(1, Nb=1, H=4, W=4, C=8, G=2)
    Wp = q.pack_conv_w(torch.from_numpy(cc.wgt).to(dev), cc.b_zp)
    p = q.RequantParams(128, None, scales.data_ptr(), 1, 0, 0)
    assert q.lib.qg_gemm_u8s8_requant(A.data_ptr(), 64, 128, Wp.handle, ctypes.byref(p), C.data_ptr(), 64, None, None) == q.EINVAL
    torch.cuda.synchronize()


def test_empty_batch_is_a_checked_no_op(env):
    """M == 0 (Nb == 0 for the convolutions): QG_OK, nothing written; the other arguments are still checked."""
    import ctypes
    q, torch, dev, oracle = env
    c = wl.config1_tiny()
    A, B, bias, scales, C, _ = dev_case(c, torch, dev)
    Bp = q.pack_b(B, c.b_zp)
    L = q.lib
    C.fill_(0x5A)
    C32 = torch.full((64, 64), 77, dtype=torch.int32, device=dev)
    Cf = torch.full((64, 64), 7.0, dtype=torch.float32, device=dev)
    Af = torch.zeros((64, 128), dtype=torch.float32, device=dev)
    p = q.RequantParams(128, None, scales.data_ptr(), 1, 0, 0)
    d = q.DequantParams(128, None, scales.data_ptr(), 1, 0)
    assert L.qg_gemm_u8s8_requant(A.data_ptr(), 0, 128, Bp.handle, ctypes.byref(p), C.data_ptr(), 64, None, None) == q.OK
    assert L.qg_gemm_u8s8_acc32(A.data_ptr(), 0, 128, Bp.handle, C32.data_ptr(), 64, None, None, None) == q.OK
    assert L.qg_gemm_u8s8_dequant_f32(A.data_ptr(), 0, 128, Bp.handle, ctypes.byref(d), Cf.data_ptr(), 64, None, None, 0) == q.OK
    assert L.qg_quantize_a_f32(Af.data_ptr(), 0, 128, 128, 1.0, 128, A.data_ptr(), 128, None) == q.OK
    assert L.qg_gemm_f32s8_requant(Af.data_ptr(), 0, 128, 1.0, Bp.handle, ctypes.byref(p), C.data_ptr(), 64, None, None, 0) == q.OK
    assert L.qg_gemm_f32s8_dequant_f32(Af.data_ptr(), 0, 128, 1.0, Bp.handle, ctypes.byref(d), Cf.data_ptr(), 64, None, None, 0) == q.OK
    # the data pointers of an empty batch are not referenced (an empty tensor has none)
    assert L.qg_gemm_u8s8_requant(None, 0, 128, Bp.handle, ctypes.byref(p), None, 64, None, None) == q.OK
    assert L.qg_gemm_f32s8_requant(None, 0, 128, 1.0, Bp.handle, ctypes.byref(p), None, 64, None, None, 0) == q.OK
    # still checked: a short leading dimension, a bad zero point, a missing descriptor or parameter block
    assert L.qg_gemm_u8s8_requant(A.data_ptr(), 0, 127, Bp.handle, ctypes.byref(p), C.data_ptr(), 64, None, None) == q.EINVAL
    assert L.qg_gemm_u8s8_requant(A.data_ptr(), 0, 128, None, ctypes.byref(p), C.data_ptr(), 64, None, None) == q.ENULL
    assert L.qg_gemm_u8s8_requant(A.data_ptr(), 0, 128, Bp.handle, None, C.data_ptr(), 64, None, None) == q.ENULL
    assert L.qg_gemm_f32s8_requant(Af.data_ptr(), 0, 127, 1.0, Bp.handle, ctypes.byref(p), C.data_ptr(), 64, None, None, 0) == q.EINVAL
    bad = q.RequantParams(300, None, scales.data_ptr(), 1, 0, 0)
    assert L.qg_gemm_u8s8_requant(A.data_ptr(), 0, 128, Bp.handle, ctypes.byref(bad), C.data_ptr(), 64, None, None) == q.EINVAL
    # convolutions with no image
    cg = wl.random_conv(3, Nb=1, H=5, W=5, C=64, G=16)
    Wg = q.pack_conv_w(torch.from_numpy(cg.wgt).to(dev), cg.b_zp)
    cd = wl.random_conv(4, Nb=1, H=5, W=5, C=64, G=1, Cout=64)
    Wd = q.pack_conv_dense_w(torch.from_numpy(np.ascontiguousarray(cd.wgt[0])).to(dev), cd.b_zp)
    x = torch.zeros((1, 5, 5, 64), dtype=torch.uint8, device=dev)
    y = torch.full((1, 5, 5, 64), 0x5A, dtype=torch.uint8, device=dev)
    sg = torch.from_numpy(cg.scales).to(dev)
    pg = q.RequantParams(cg.a_zp, None, sg.data_ptr(), sg.numel(), cg.c_zp, 0)
    assert L.qg_conv_groupwise_u8s8_requant(x.data_ptr(), 0, 5, 5, 64, 1, 1, Wg.handle, ctypes.byref(pg), y.data_ptr(), None) == q.OK
    sd = torch.from_numpy(cd.scales).to(dev)
    pd = q.RequantParams(cd.a_zp, None, sd.data_ptr(), sd.numel(), cd.c_zp, 0)
    assert L.qg_conv_dense_u8s8_requant(x.data_ptr(), 0, 5, 5, 64, 3, 3, 1, 1, Wd.handle, ctypes.byref(pd), y.data_ptr(), None, 0) == q.OK
    assert L.qg_conv_dense_u8s8_requant(x.data_ptr(), -1, 5, 5, 64, 3, 3, 1, 1, Wd.handle, ctypes.byref(pd), y.data_ptr(), None, 0) == q.EINVAL
    # through the binding: empty tensors in, empty tensors out
    e = q.gemm_u8s8_requant(torch.empty((0, 128), dtype=torch.uint8, device=dev), 128, Bp, None, scales, 0, False)
    assert tuple(e.shape) == (0, 64)
    ec = q.conv_dense_u8s8_requant(torch.empty((0, 5, 5, 64), dtype=torch.uint8, device=dev), Wd, cd.a_zp, None, sd,
                                   cd.c_zp, False)
    assert tuple(ec.shape) == (0, 5, 5, 64)
    torch.cuda.synchronize()
    assert bool((C == 0x5A).all()) and bool((C32 == 77).all()) and bool((Cf == 7.0).all()) and bool((y == 0x5A).all())


def test_measurement_probes_run(env):
    """bench.py's probes (a library of their own, not part of the path): they must launch, finish and leave their
    inputs alone."""
    import ctypes
    import os
    q, torch, dev, oracle = env
    say("probes")
    root = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
    bp = ctypes.CDLL(os.path.join(root, "libbench_probes.so"))
    vp = ctypes.c_void_p
    bp.bp_mfma_i8.argtypes = [vp, vp, ctypes.c_int, ctypes.c_int, vp]
    bp.bp_read.argtypes = [vp, ctypes.c_size_t, vp, ctypes.c_int, vp]
    operands = torch.arange(32768, dtype=torch.int32, device=dev).to(torch.uint8)
    before = operands.clone()
    sink = torch.zeros(4 * 256, dtype=torch.int32, device=dev)
    st = torch.cuda.current_stream().cuda_stream
    assert bp.bp_mfma_i8(operands.data_ptr(), sink.data_ptr(), 4, 3, st) == 0
    src = torch.ones(1 << 20, dtype=torch.uint8, device=dev)
    assert bp.bp_read(src.data_ptr(), src.numel(), sink.data_ptr(), 64, st) == 0
    assert bp.bp_read(src.data_ptr(), 24, sink.data_ptr(), 64, st) == -1 and bp.bp_mfma_i8(None, sink.data_ptr(), 4, 3, st) == -1
    torch.cuda.synchronize()
    assert torch.equal(operands, before) and int(src.sum().item()) == 1 << 20
