"""Seeded synthetic inputs for the quantized GEMM / group-conv path.

This module only draws numbers.  It holds none of the method's arithmetic and
imports neither the HIP binding nor the oracle, so both sides can be fed from
it.  Everything is numpy `default_rng(seed)` (PCG64); arrays are drawn in the
fixed order A, A_zp, B, B_zp, bias, scales.

The shapes and value distributions stand in for the production GEMM shapes the
paper benchmarks (small-batch fully connected layers, square compute-bound
GEMMs, recommender MLP layers, group convolution); the paper names no public
dataset, so nothing external is needed.
"""
from dataclasses import dataclass, field
from typing import Optional

import numpy as np


@dataclass
class GemmCase:
    name: str
    A: np.ndarray                 # uint8  [M, K]
    a_zp: int                     # 0..255
    B: np.ndarray                 # int8   [K, N]
    b_zp: np.ndarray              # int32  [1] or [N], each -128..127
    bias: Optional[np.ndarray]    # int32  [N] or None
    scales: np.ndarray            # float32 [1] or [N]
    c_zp: int                     # 0..255
    relu: bool
    note: dict = field(default_factory=dict)

    @property
    def M(self):
        return self.A.shape[0]

    @property
    def K(self):
        return self.A.shape[1]

    @property
    def N(self):
        return self.B.shape[1]


@dataclass
class ConvCase:
    name: str
    inp: np.ndarray               # uint8 NHWC
    a_zp: int
    wgt: np.ndarray               # int8 [G][R][S][C/G][Cout/G]
    G: int
    b_zp: np.ndarray              # int32 [1] or [Cout]
    bias: Optional[np.ndarray]    # int32 [Cout] or None
    scales: np.ndarray            # float32 [1] or [Cout]
    c_zp: int
    relu: bool
    pad: int = 1
    stride: int = 1
    note: dict = field(default_factory=dict)


def _u8_uniform(rng, shape):
    return rng.integers(0, 256, size=shape, dtype=np.uint8)


def _s8_uniform(rng, shape):
    return rng.integers(-128, 128, size=shape, dtype=np.int8)


def _log_uniform(rng, n, lo=-14.0, hi=-8.0):
    return np.float32(2.0) ** rng.uniform(lo, hi, size=n).astype(np.float32)


def config1_tiny(seed=0):
    """M=64,N=64,K=128; A_zp=128, B_zp=0, bias U[-1000,1000], scale 2^-10."""
    rng = np.random.default_rng(seed)
    M, N, K = 64, 64, 128
    A = _u8_uniform(rng, (M, K))
    B = _s8_uniform(rng, (K, N))
    bias = rng.integers(-1000, 1001, size=N).astype(np.int32)
    return GemmCase("c1_tiny_64x64x128", A, 128, B, np.zeros(1, np.int32), bias,
                    np.array([2.0 ** -10], np.float32), 0, False)


def config2_small_batch_fc(seed=1, with_bias=False, M=16, N=4096, K=4096):
    """M=16,N=K=4096; A_zp U{0..255}; B_zp U{-4..4}; per-tensor scale; C_zp=10; ReLU."""
    rng = np.random.default_rng(seed)
    A = _u8_uniform(rng, (M, K))
    a_zp = int(rng.integers(0, 256))
    B = _s8_uniform(rng, (K, N))
    b_zp = rng.integers(-4, 5, size=1).astype(np.int32)
    bias = rng.integers(-1000, 1001, size=N).astype(np.int32)  # always drawn, used on request
    scales = _log_uniform(rng, 1)
    return GemmCase(f"c2_fc_{M}x{N}x{K}", A, a_zp, B, b_zp, bias if with_bias else None, scales, 10, True)


def config3_square(seed=2, M=8192, N=8192, K=8192):
    """M=N=K=8192; per-channel B_zp U{-8..8} and scales; bias; ReLU; A_zp=128; C_zp=0."""
    rng = np.random.default_rng(seed)
    A = _u8_uniform(rng, (M, K))
    B = _s8_uniform(rng, (K, N))
    b_zp = rng.integers(-8, 9, size=N).astype(np.int32)
    bias = rng.integers(-1000, 1001, size=N).astype(np.int32)
    scales = _log_uniform(rng, N)
    return GemmCase(f"c3_square_{M}x{N}x{K}", A, 128, B, b_zp, bias, scales, 0, True)


def config4_recsys_mlp(seed=3, M=32768, N=512, K=1024):
    """M=32768,N=512,K=1024; A clipped half-normal(std 40), A_zp=0; B normal(0,30) clipped."""
    rng = np.random.default_rng(seed)
    A = np.minimum(255.0, np.rint(np.abs(rng.normal(0.0, 40.0, size=(M, K))))).astype(np.uint8)
    B = np.clip(np.rint(rng.normal(0.0, 30.0, size=(K, N))), -128, 127).astype(np.int8)
    scales = _log_uniform(rng, N)
    return GemmCase(f"c4_mlp_{M}x{N}x{K}", A, 0, B, np.zeros(1, np.int32), None, scales, 0, False)


def config5_group_conv(seed=4, Nb=32, H=56, W=56, C=128, G=32):
    """NHWC 32x56x56x128, 3x3 s1 p1, 32 groups of 4->4; A_zp=128; per-group scale; C_zp=128."""
    rng = np.random.default_rng(seed)
    Cg = C // G
    inp = _u8_uniform(rng, (Nb, H, W, C))
    wgt = _s8_uniform(rng, (G, 3, 3, Cg, Cg))
    scales = np.repeat(_log_uniform(rng, G), Cg).astype(np.float32)
    return ConvCase(f"c5_gconv_{Nb}x{H}x{W}x{C}_g{G}", inp, 128, wgt, G, np.zeros(1, np.int32), None,
                    scales, 128, False)


def unsaturated(case: GemmCase) -> GemmCase:
    """Parity-only variant of a GEMM case: same A and B, but C_zp=128, no ReLU and
    scales sized so that most outputs land strictly inside (0,255), which makes
    the comparison sensitive to rounding instead of to the clamp."""
    a_std = float(np.std(case.A[: min(case.M, 256)].astype(np.float64) - case.a_zp)) + 1.0
    b_std = float(np.std(case.B[: min(case.K, 256)].astype(np.float64))) + 1.0
    base = 40.0 / (np.sqrt(case.K) * a_std * b_std)
    rng = np.random.default_rng(12345)
    n = case.scales.size
    s = (base * 2.0 ** rng.uniform(-0.5, 0.5, size=n)).astype(np.float32)
    return GemmCase(case.name + "_unsat", case.A, case.a_zp, case.B, case.b_zp, case.bias, s, 128, False)


def random_gemm(seed, M, N, K, per_channel=True, with_bias=True, relu=False, a_zp=None, c_zp=None,
                unsat=True, wide_zp=False):
    """Generic seeded case for ragged / edge shapes."""
    rng = np.random.default_rng(seed)
    A = _u8_uniform(rng, (M, K))
    # zero points near the data means keep the mean of x near 0 so that the `unsat` scales work;
    # extreme zero points are covered by passing a_zp / wide_zp explicitly
    a_draw = int(rng.integers(0, 256)) if wide_zp else int(rng.integers(120, 137))
    a_zp = a_draw if a_zp is None else int(a_zp)
    B = _s8_uniform(rng, (K, N))
    nz = N if per_channel else 1
    b_zp = (rng.integers(-128, 128, size=nz) if wide_zp else rng.integers(-4, 5, size=nz)).astype(np.int32)
    bias = rng.integers(-1000, 1001, size=N).astype(np.int32) if with_bias else None
    if unsat:
        base = 40.0 / (np.sqrt(K) * 74.0 * 74.0)
        scales = (base * 2.0 ** rng.uniform(-1.0, 1.0, size=nz)).astype(np.float32)
    else:
        scales = _log_uniform(rng, nz)
    c_draw = int(rng.integers(0, 256)) if wide_zp else int(rng.integers(96, 161))
    c_zp = c_draw if c_zp is None else int(c_zp)
    return GemmCase(f"rand_{M}x{N}x{K}_s{seed}", A, a_zp, B, b_zp, bias, scales, c_zp, relu)


def random_conv(seed, Nb, H, W, C, G, Cout=None, R=3, S=3, pad=1, stride=1, per_channel=True,
                with_bias=True, relu=False):
    rng = np.random.default_rng(seed)
    Cout = C if Cout is None else Cout
    Cg, Og = C // G, Cout // G
    inp = _u8_uniform(rng, (Nb, H, W, C))
    a_zp = int(rng.integers(0, 256))
    wgt = _s8_uniform(rng, (G, R, S, Cg, Og))
    nz = Cout if per_channel else 1
    b_zp = rng.integers(-16, 17, size=nz).astype(np.int32)
    bias = rng.integers(-1000, 1001, size=Cout).astype(np.int32) if with_bias else None
    base = 40.0 / (np.sqrt(R * S * Cg) * 74.0 * 74.0)
    scales = (base * 2.0 ** rng.uniform(-1.0, 1.0, size=nz)).astype(np.float32)
    c_zp = int(rng.integers(0, 256))
    return ConvCase(f"randconv_{Nb}x{H}x{W}x{C}_g{G}_s{seed}", inp, a_zp, wgt, G, b_zp, bias, scales,
                    c_zp, relu, pad, stride)


def random_fp32_activations(seed, M, K, alpha=0.05, zp=100, special=True):
    """fp32 activations around the range an (alpha, zp) uint8 quantizer represents: most values inside the
    range, some beyond either end, and -- with `special` -- exact half-way points, zeros, huge values and
    infinities sprinkled in.  Returns (A float32 [M, K], inv_scale float32)."""
    rng = np.random.default_rng(seed)
    lo, hi = alpha * (0 - zp), alpha * (255 - zp)
    span = hi - lo
    A = rng.uniform(lo - 0.1 * span, hi + 0.1 * span, size=(M, K)).astype(np.float32)
    if special and A.size >= 16:
        flat = A.reshape(-1)
        idx = rng.choice(flat.size, size=max(8, flat.size // 16), replace=False)
        codes = rng.integers(0, 255, size=idx.size)
        flat[idx] = (alpha * (codes - zp + 0.5)).astype(np.float32)   # near or exactly on a tie
        extra = np.array([0.0, -0.0, 1e30, -1e30, np.inf, -np.inf, 1e-30, -1e-30], np.float32)
        flat[idx[:8]] = extra
    return A, np.float32(1.0 / alpha)


def outlier_weights(seed, K, N, sigma=2.5, outlier_frac=0.01, outlier_sigma=40.0):
    """int8 weights as outlier-aware quantization produces them: a narrow bulk (rounded normal, sigma a few
    quantization steps) and a small fraction of large-magnitude entries."""
    rng = np.random.default_rng(seed)
    B = np.rint(rng.normal(0.0, sigma, size=(K, N)))
    big = rng.random(size=(K, N)) < outlier_frac
    B[big] = np.rint(rng.normal(0.0, outlier_sigma, size=int(big.sum())))
    return np.clip(B, -128, 127).astype(np.int8)
