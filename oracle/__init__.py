"""ctypes face of the CPU oracle (oracle/qgemm_oracle.c).

TEST INFRASTRUCTURE ONLY: imported by tests/, by the smoke check and by the
benchmark's cpu_baseline leg.  The product package never imports this module
and this module never imports the product package.

Every function takes and returns numpy arrays; all arithmetic happens in the C
file, whose header states which passage of the paper each routine follows.
"""
import ctypes
import os
import subprocess

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "qgemm_oracle.c")
_LIB = os.path.join(_HERE, "liboracle.so")

OK, EINVAL, EOVERFLOW, ENOMEM = 0, -1, -2, -3


def build(force=False):
    """Compile the oracle with gcc.  No fast-math, no FMA contraction."""
    if not force and os.path.exists(_LIB) and os.path.getmtime(_LIB) >= os.path.getmtime(_SRC):
        return _LIB
    cmd = ["gcc", "-O2", "-fopenmp", "-ffp-contract=off", "-fno-fast-math", "-std=c11",
           "-shared", "-fPIC", "-o", _LIB, _SRC, "-lm"]
    subprocess.run(cmd, check=True)
    return _LIB


_lib = None


def _load():
    global _lib
    if _lib is None:
        build()
        lib = ctypes.CDLL(_LIB)
        lib.orc_requant_one.restype = ctypes.c_uint8
        lib.orc_requant_one.argtypes = [ctypes.c_int32, ctypes.c_float, ctypes.c_int32, ctypes.c_int]
        lib.orc_dequant_one.restype = ctypes.c_float
        lib.orc_dequant_one.argtypes = [ctypes.c_int32, ctypes.c_float, ctypes.c_int]
        lib.orc_quantize_one.restype = ctypes.c_uint8
        lib.orc_quantize_one.argtypes = [ctypes.c_float, ctypes.c_float, ctypes.c_int32]
        vp, i = ctypes.c_void_p, ctypes.c_int
        lib.orc_quantize_f32.argtypes = [vp, i, i, i, ctypes.c_float, ctypes.c_int32, vp, i]
        lib.orc_dequant_f32.argtypes = [vp, i, i, vp, i, i, vp]
        lib.orc_split_outliers.restype = ctypes.c_long
        lib.orc_split_outliers.argtypes = [vp, i, i, i, i, i, vp, vp]
        lib.orc_csc_from_dense.argtypes = [vp, i, i, vp, vp, vp, ctypes.c_long]
        _lib = lib
    return _lib


def _p(a):
    return None if a is None else a.ctypes.data_as(ctypes.c_void_p)


def _check(rc, what):
    if rc != OK:
        raise OracleError(rc, what)


class OracleError(RuntimeError):
    def __init__(self, code, what):
        super().__init__(f"oracle {what} failed with code {code}")
        self.code = code


def _u8(a):
    a = np.asarray(a)
    assert a.dtype == np.uint8 and a.ndim == 2 and a.strides[1] == 1
    return a


def _s8(a):
    a = np.asarray(a)
    assert a.dtype == np.int8 and a.ndim == 2 and a.strides[1] == 1
    return a


def _zp_vec(z):
    return np.ascontiguousarray(np.atleast_1d(np.asarray(z)).astype(np.int32))


def num_threads():
    return int(_load().orc_num_threads())


def colsum(B):
    B = _s8(B)
    K, N = B.shape
    out = np.empty(N, np.int32)
    _check(_load().orc_colsum(_p(B), K, N, B.strides[0], _p(out)), "colsum")
    return out


def rowsum(A):
    A = _u8(A)
    M, K = A.shape
    out = np.empty(M, np.int32)
    _check(_load().orc_rowsum(_p(A), M, K, A.strides[0], _p(out)), "rowsum")
    return out


def col_offsets(B, b_zp):
    B = _s8(B)
    K, N = B.shape
    z = _zp_vec(b_zp)
    out = np.empty(N, np.int32)
    _check(_load().orc_col_offsets(_p(B), K, N, B.strides[0], _p(z), z.size, _p(out)), "col_offsets")
    return out


def acc32(A, B):
    A, B = _u8(A), _s8(B)
    M, K = A.shape
    K2, N = B.shape
    assert K == K2
    out = np.empty((M, N), np.int32)
    _check(_load().orc_acc32(_p(A), M, K, A.strides[0], _p(B), N, B.strides[0], _p(out), N), "acc32")
    return out


def requant_one(x, scale, c_zp, relu):
    return int(_load().orc_requant_one(int(x), float(np.float32(scale)), int(c_zp), int(bool(relu))))


def gemm_u8s8_requant(A, a_zp, B, b_zp, bias, scales, c_zp, relu, return_x=False):
    """C_u8 (and optionally the corrected int32 accumulator x) for one GEMM."""
    A, B = _u8(A), _s8(B)
    M, K = A.shape
    K2, N = B.shape
    assert K == K2
    z = _zp_vec(b_zp)
    s = np.ascontiguousarray(np.atleast_1d(np.asarray(scales)).astype(np.float32))
    bias_c = None if bias is None else np.ascontiguousarray(np.asarray(bias).astype(np.int32))
    if bias_c is not None:
        assert bias_c.shape == (N,)
    C = np.empty((M, N), np.uint8)
    x = np.empty((M, N), np.int32) if return_x else None
    rc = _load().orc_gemm_u8s8_requant(_p(A), M, K, A.strides[0], int(a_zp), _p(B), N, B.strides[0],
                                       _p(z), z.size, _p(bias_c), _p(s), s.size, int(c_zp),
                                       int(bool(relu)), _p(C), N, _p(x))
    _check(rc, "gemm_u8s8_requant")
    return (C, x) if return_x else C


def dequant_one(x, scale, relu):
    return float(_load().orc_dequant_one(int(x), float(np.float32(scale)), int(bool(relu))))


def quantize_one(a, inv_scale, zp):
    return int(_load().orc_quantize_one(float(np.float32(a)), float(np.float32(inv_scale)), int(zp)))


def quantize_f32(A, inv_scale, zp):
    """uint8 quantization of an fp32 matrix (Eq. (1) solved for the quantized value)."""
    A = np.ascontiguousarray(np.asarray(A, dtype=np.float32))
    assert A.ndim == 2
    M, K = A.shape
    out = np.empty((M, K), np.uint8)
    _check(_load().orc_quantize_f32(_p(A), M, K, K, float(np.float32(inv_scale)), int(zp), _p(out), K),
           "quantize_f32")
    return out


def gemm_u8s8_dequant_f32(A, a_zp, B, b_zp, bias, scales, relu):
    """fp32 output: the corrected accumulator x of Eq. (2) times scale[j] = alpha_A * alpha_B[j]."""
    N = np.asarray(B).shape[1]
    one = np.ones(1, np.float32)
    _, x = gemm_u8s8_requant(A, a_zp, B, b_zp, bias, one, 0, False, return_x=True)
    s = np.ascontiguousarray(np.atleast_1d(np.asarray(scales)).astype(np.float32))
    out = np.empty(x.shape, np.float32)
    _check(_load().orc_dequant_f32(_p(x), x.shape[0], N, _p(s), s.size, int(bool(relu)), _p(out)), "dequant_f32")
    return out


def split_outliers(B, lo=-8, hi=7):
    """B = B_small + B_sparse (both dense int8 [K, N]); returns (B_small, B_sparse, number of outliers)."""
    B = _s8(B)
    K, N = B.shape
    small, sparse = np.empty((K, N), np.int8), np.empty((K, N), np.int8)
    nnz = _load().orc_split_outliers(_p(B), K, N, B.strides[0], int(lo), int(hi), _p(small), _p(sparse))
    if nnz < 0:
        raise OracleError(int(nnz), "split_outliers")
    return small, sparse, int(nnz)


def csc_from_dense(S):
    """(col_ptr int32 [N+1], row_idx int32 [nnz], val int8 [nnz]) of a dense int8 [K, N] matrix."""
    S = _s8(S)
    K, N = S.shape
    cap = int(np.count_nonzero(S))
    col_ptr = np.empty(N + 1, np.int32)
    row_idx, val = np.empty(max(cap, 1), np.int32), np.empty(max(cap, 1), np.int8)
    _check(_load().orc_csc_from_dense(_p(S), K, N, _p(col_ptr), _p(row_idx), _p(val), cap), "csc_from_dense")
    return col_ptr, row_idx[:cap], val[:cap]


def acc32_split(A, B_small, csc):
    """A B_small + A B_sparse with B_sparse in CSC form."""
    A, B_small = _u8(A), _s8(B_small)
    M, K = A.shape
    N = B_small.shape[1]
    col_ptr, row_idx, val = csc
    row_idx = np.ascontiguousarray(row_idx if row_idx.size else np.zeros(1, np.int32))
    val = np.ascontiguousarray(val if val.size else np.zeros(1, np.int8))
    out = np.empty((M, N), np.int32)
    _check(_load().orc_acc32_split(_p(A), M, K, A.strides[0], _p(np.ascontiguousarray(B_small)), N, _p(col_ptr),
                                   _p(row_idx), _p(val), _p(out)), "acc32_split")
    return out


def conv_out_hw(H, W, R, S, pad, stride):
    return (H + 2 * pad - R) // stride + 1, (W + 2 * pad - S) // stride + 1


def conv_groupwise_direct(inp, G, wgt, a_zp, b_zp, bias, scales, c_zp, relu, pad=1, stride=1,
                          return_x=False):
    """inp: NHWC uint8; wgt: [G][R][S][C/G][Cout/G] int8.  Returns NHWC uint8."""
    inp = np.ascontiguousarray(inp)
    wgt = np.ascontiguousarray(wgt)
    assert inp.dtype == np.uint8 and inp.ndim == 4 and wgt.dtype == np.int8 and wgt.ndim == 5
    Nb, H, W, C = inp.shape
    G2, R, S, Cg, Og = wgt.shape
    assert G2 == G and Cg * G == C
    Cout = G * Og
    z = _zp_vec(b_zp)
    s = np.ascontiguousarray(np.atleast_1d(np.asarray(scales)).astype(np.float32))
    bias_c = None if bias is None else np.ascontiguousarray(np.asarray(bias).astype(np.int32))
    Ho, Wo = conv_out_hw(H, W, R, S, pad, stride)
    out = np.empty((Nb, Ho, Wo, Cout), np.uint8)
    x = np.empty((Nb, Ho, Wo, Cout), np.int32) if return_x else None
    rc = _load().orc_conv_groupwise_direct(_p(inp), Nb, H, W, C, G, Cout, R, S, pad, stride, int(a_zp),
                                           _p(wgt), _p(z), z.size, _p(bias_c), _p(s), s.size,
                                           int(c_zp), int(bool(relu)), _p(out), _p(x))
    _check(rc, "conv_groupwise_direct")
    return (out, x) if return_x else out


def im2col_group(inp, G, g, R, S, pad, stride, a_zp):
    inp = np.ascontiguousarray(inp)
    Nb, H, W, C = inp.shape
    Ho, Wo = conv_out_hw(H, W, R, S, pad, stride)
    cols = np.empty((Nb * Ho * Wo, R * S * (C // G)), np.uint8)
    _check(_load().orc_im2col_group(_p(inp), Nb, H, W, C, G, g, R, S, pad, stride, int(a_zp), _p(cols)),
           "im2col_group")
    return cols
