"""Thin ctypes binding of libqgemm.so (the C ABI in include/qgemm.h).

Argument marshalling only: every step of the path runs in the HIP kernels.
PyTorch supplies device memory (`tensor.data_ptr()`) and the stream.  There is
no CPU fallback: if the library is not built, importing this module raises.
"""
import ctypes
import os

import torch  # noqa: F401  (imported first so that libqgemm binds to the HIP runtime torch loaded)

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libqgemm.so")

OK, ENULL, EINVAL, EALIGN, EWORKSPACE, ELAUNCH, ENOMEM, EUNSUPPORTED, ECAPACITY = 0, -1, -2, -3, -4, -5, -6, -7, -8
MAX_K = 32768

EXPORTS = [
    "qg_pack_b_sizes", "qg_pack_b", "qg_packed_b_destroy", "qg_packed_b_k", "qg_packed_b_n",
    "qg_gemm_workspace_bytes", "qg_gemm_u8s8_requant", "qg_gemm_u8s8_acc32",
    "qg_pack_conv_w_sizes", "qg_pack_conv_w", "qg_conv_groupwise_u8s8_requant", "qg_status_string",
    "qg_kernel_name", "qg_kernel_select", "qg_dispatch_set_rules", "qg_gemm_u8s8_requant_kernel",
    "qg_gemm_u8s8_acc32_kernel", "qg_gemm_u8s8_dequant_f32", "qg_quantize_a_f32", "qg_gemm_f32_workspace_bytes",
    "qg_gemm_f32s8_requant", "qg_gemm_f32s8_dequant_f32",
    "qg_count_outliers", "qg_pack_b_outlier_sizes", "qg_pack_b_outlier", "qg_packed_b_nnz",
    "qg_conv_dense_u8s8_requant", "qg_pack_b_transposed",
    "qg_gemm_workspace_init", "qg_gemm_splitk_workspace_bytes", "qg_gemm_splitk_factor",
    "qg_gemm_u8s8_requant_splitk", "qg_gemm_u8s8_acc32_splitk", "qg_gemm_u8s8_requant_noalloc",
]

KERNEL_AUTO, KERNEL_LAST = 0, 10
KERNEL_CONV_LAST = 15   # the ids above KERNEL_LAST are kernels of the dense convolution only
MAX_DISPATCH_RULES = 256


class RequantParams(ctypes.Structure):
    _fields_ = [("a_zp", ctypes.c_int32), ("bias", ctypes.c_void_p), ("scales", ctypes.c_void_p),
                ("n_scales", ctypes.c_int32), ("c_zp", ctypes.c_int32), ("relu", ctypes.c_int32)]


class DequantParams(ctypes.Structure):
    _fields_ = [("a_zp", ctypes.c_int32), ("bias", ctypes.c_void_p), ("scales", ctypes.c_void_p),
                ("n_scales", ctypes.c_int32), ("relu", ctypes.c_int32)]


class DispatchRule(ctypes.Structure):
    _fields_ = [(n, ctypes.c_int32) for n in ("m_lo", "m_hi", "n_lo", "n_hi", "k_lo", "k_hi", "kernel")]


def _load():
    if not os.path.exists(LIB_PATH):
        raise ImportError(f"{LIB_PATH} is not built; run `python -c 'import __graft_entry__ as g; g.build()'` "
                          "or `python paper_2101_05615_amd/build.py` (there is no CPU fallback)")
    lib = ctypes.CDLL(LIB_PATH)
    vp, i, sz = ctypes.c_void_p, ctypes.c_int, ctypes.c_size_t
    lib.qg_pack_b_sizes.argtypes = [i, i, ctypes.POINTER(sz), ctypes.POINTER(sz)]
    lib.qg_pack_b.argtypes = [vp, i, i, i, vp, i, vp, vp, vp, ctypes.POINTER(vp)]
    lib.qg_pack_b_transposed.argtypes = lib.qg_pack_b.argtypes
    lib.qg_packed_b_destroy.argtypes = [vp]
    lib.qg_packed_b_destroy.restype = None
    lib.qg_packed_b_k.argtypes = [vp]
    lib.qg_packed_b_n.argtypes = [vp]
    lib.qg_gemm_workspace_bytes.argtypes = [i, vp]
    lib.qg_gemm_workspace_bytes.restype = sz
    lib.qg_gemm_u8s8_requant.argtypes = [vp, i, i, vp, ctypes.POINTER(RequantParams), vp, i, vp, vp]
    lib.qg_gemm_u8s8_acc32.argtypes = [vp, i, i, vp, vp, i, vp, vp, vp]
    lib.qg_pack_conv_w_sizes.argtypes = [i, i, i, i, i, ctypes.POINTER(sz), ctypes.POINTER(sz)]
    lib.qg_pack_conv_w.argtypes = [vp, i, i, i, i, i, vp, i, vp, vp, vp, ctypes.POINTER(vp)]
    lib.qg_conv_groupwise_u8s8_requant.argtypes = [vp, i, i, i, i, i, i, vp, ctypes.POINTER(RequantParams),
                                                   vp, vp]
    lib.qg_status_string.argtypes = [i]
    lib.qg_status_string.restype = ctypes.c_char_p
    lib.qg_kernel_name.argtypes = [i]
    lib.qg_kernel_name.restype = ctypes.c_char_p
    lib.qg_kernel_select.argtypes = [i, i, i]
    lib.qg_dispatch_set_rules.argtypes = [ctypes.POINTER(DispatchRule), i]
    lib.qg_gemm_u8s8_requant_kernel.argtypes = lib.qg_gemm_u8s8_requant.argtypes + [i]
    lib.qg_gemm_u8s8_acc32_kernel.argtypes = lib.qg_gemm_u8s8_acc32.argtypes + [i]
    f = ctypes.c_float
    lib.qg_gemm_u8s8_dequant_f32.argtypes = [vp, i, i, vp, ctypes.POINTER(DequantParams), vp, i, vp, vp, i]
    lib.qg_quantize_a_f32.argtypes = [vp, i, i, i, f, i, vp, i, vp]
    lib.qg_gemm_f32_workspace_bytes.argtypes = [i, vp]
    lib.qg_gemm_f32_workspace_bytes.restype = sz
    lib.qg_gemm_f32s8_requant.argtypes = [vp, i, i, f, vp, ctypes.POINTER(RequantParams), vp, i, vp, vp, i]
    lib.qg_gemm_f32s8_dequant_f32.argtypes = [vp, i, i, f, vp, ctypes.POINTER(DequantParams), vp, i, vp, vp, i]
    lib.qg_count_outliers.argtypes = [vp, i, i, i, vp, ctypes.POINTER(sz), vp]
    lib.qg_pack_b_outlier_sizes.argtypes = [i, i, sz, ctypes.POINTER(sz), ctypes.POINTER(sz), ctypes.POINTER(sz)]
    lib.qg_pack_b_outlier.argtypes = [vp, i, i, i, vp, i, sz, vp, vp, vp, vp, ctypes.POINTER(vp)]
    lib.qg_packed_b_nnz.argtypes = [vp]
    lib.qg_conv_dense_u8s8_requant.argtypes = [vp, i, i, i, i, i, i, i, i, vp, ctypes.POINTER(RequantParams), vp, vp, i]
    lib.qg_packed_b_nnz.restype = sz
    lib.qg_gemm_workspace_init.argtypes = [vp, sz, vp]
    lib.qg_gemm_splitk_workspace_bytes.argtypes = [i, vp, i, i]
    lib.qg_gemm_splitk_workspace_bytes.restype = sz
    lib.qg_gemm_splitk_factor.argtypes = [i, vp, i, i]
    lib.qg_gemm_u8s8_requant_splitk.argtypes = [vp, i, i, vp, ctypes.POINTER(RequantParams), vp, i, vp, sz, vp, i, i]
    lib.qg_gemm_u8s8_acc32_splitk.argtypes = [vp, i, i, vp, vp, i, vp, vp, sz, vp, i, i]
    lib.qg_gemm_u8s8_requant_noalloc.argtypes = [vp, i, i, vp, ctypes.POINTER(RequantParams), vp, i, vp, i, i]
    return lib


lib = _load()


class QGemmError(RuntimeError):
    def __init__(self, code, where):
        super().__init__(f"{where}: {lib.qg_status_string(code).decode()} ({code})")
        self.code = code


def _check(rc, where):
    if rc != OK:
        raise QGemmError(rc, where)


def _stream():
    return ctypes.c_void_p(torch.cuda.current_stream().cuda_stream)


def _host_i32(z):
    import numpy as np
    a = np.ascontiguousarray(np.atleast_1d(np.asarray(z)).astype(np.int32))
    return a, a.ctypes.data_as(ctypes.c_void_p)


class PackedB:
    """Owner of the two device buffers and of the host descriptor of a packed weight matrix."""

    def __init__(self, handle, packed, aux, n):
        self.handle, self.packed, self.aux, self._n = handle, packed, aux, n

    @property
    def col_offsets(self):
        return self.aux[: self._n]

    @property
    def K(self):
        return lib.qg_packed_b_k(self.handle)

    @property
    def N(self):
        return lib.qg_packed_b_n(self.handle)

    def close(self):
        if self.handle:
            lib.qg_packed_b_destroy(self.handle)
            self.handle = None

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass


def pack_b_sizes(K, N):
    pb, cb = ctypes.c_size_t(), ctypes.c_size_t()
    _check(lib.qg_pack_b_sizes(K, N, ctypes.byref(pb), ctypes.byref(cb)), "qg_pack_b_sizes")
    return pb.value, cb.value


def pack_b(B, b_zp):
    """B: int8 cuda tensor [K, N] (row stride arbitrary, unit column stride); b_zp: 1 or N ints (host)."""
    assert B.is_cuda and B.dtype == torch.int8 and B.dim() == 2 and B.stride(1) == 1
    K, N = B.shape
    pb, cb = pack_b_sizes(K, N)
    packed = torch.empty(pb, dtype=torch.int8, device=B.device)
    aux = torch.empty(cb // 4, dtype=torch.int32, device=B.device)
    z, zp = _host_i32(b_zp)
    h = ctypes.c_void_p()
    _check(lib.qg_pack_b(B.data_ptr(), K, N, B.stride(0), zp, z.size, packed.data_ptr(), aux.data_ptr(),
                         _stream(), ctypes.byref(h)), "qg_pack_b")
    return PackedB(h, packed, aux, N)


def count_outliers(B):
    """Entries of B (int8 cuda [K, N]) outside -8..7."""
    assert B.is_cuda and B.dtype == torch.int8 and B.dim() == 2 and B.stride(1) == 1
    K, N = B.shape
    scratch = torch.empty(1, dtype=torch.int64, device=B.device)
    n = ctypes.c_size_t()
    _check(lib.qg_count_outliers(B.data_ptr(), K, N, B.stride(0), scratch.data_ptr(), ctypes.byref(n), _stream()),
           "qg_count_outliers")
    return n.value


def pack_b_outlier(B, b_zp, max_nnz=None):
    """Outlier-split descriptor of B: 4-bit B' plus the sparse part (capacity max_nnz, default: exactly enough)."""
    assert B.is_cuda and B.dtype == torch.int8 and B.dim() == 2 and B.stride(1) == 1
    K, N = B.shape
    if max_nnz is None:
        max_nnz = count_outliers(B)
    pb, cb, sb = ctypes.c_size_t(), ctypes.c_size_t(), ctypes.c_size_t()
    _check(lib.qg_pack_b_outlier_sizes(K, N, max_nnz, ctypes.byref(pb), ctypes.byref(cb), ctypes.byref(sb)),
           "qg_pack_b_outlier_sizes")
    packed = torch.empty(pb.value, dtype=torch.int8, device=B.device)
    aux = torch.empty(cb.value // 4, dtype=torch.int32, device=B.device)
    sparse = torch.empty(sb.value // 4, dtype=torch.int32, device=B.device)
    z, zp = _host_i32(b_zp)
    h = ctypes.c_void_p()
    _check(lib.qg_pack_b_outlier(B.data_ptr(), K, N, B.stride(0), zp, z.size, max_nnz, packed.data_ptr(),
                                 aux.data_ptr(), sparse.data_ptr(), _stream(), ctypes.byref(h)), "qg_pack_b_outlier")
    pk = PackedB(h, packed, aux, N)
    pk.sparse = sparse
    pk.nnz = lib.qg_packed_b_nnz(h)
    return pk


def pack_b_transposed(Bt, b_zp):
    """Bt: int8 cuda tensor [N, K] (the transposed weight matrix, unit stride along K); b_zp: 1 or N ints (host)."""
    assert Bt.is_cuda and Bt.dtype == torch.int8 and Bt.dim() == 2 and Bt.stride(1) == 1
    N, K = Bt.shape
    pb, cb = pack_b_sizes(K, N)
    packed = torch.empty(pb, dtype=torch.int8, device=Bt.device)
    aux = torch.empty(cb // 4, dtype=torch.int32, device=Bt.device)
    z, zp = _host_i32(b_zp)
    h = ctypes.c_void_p()
    _check(lib.qg_pack_b_transposed(Bt.data_ptr(), K, N, Bt.stride(0), zp, z.size, packed.data_ptr(), aux.data_ptr(),
                                    _stream(), ctypes.byref(h)), "qg_pack_b_transposed")
    return PackedB(h, packed, aux, N)


def _params(a_zp, bias, scales, c_zp, relu):
    assert scales.is_cuda and scales.dtype == torch.float32 and scales.is_contiguous()
    if bias is not None:
        assert bias.is_cuda and bias.dtype == torch.int32 and bias.is_contiguous()
    return RequantParams(int(a_zp), bias.data_ptr() if bias is not None else None, scales.data_ptr(),
                         scales.numel(), int(c_zp), int(bool(relu)))


def kernel_names():
    """id -> name of every kernel of the shape-specific family (0 is "auto")."""
    return {k: lib.qg_kernel_name(k).decode() for k in range(KERNEL_LAST + 1)}


def kernel_id(kernel):
    """Accepts an id or a name."""
    if isinstance(kernel, str):
        for k in range(KERNEL_CONV_LAST + 1):
            if lib.qg_kernel_name(k).decode() == kernel:
                return k
        raise ValueError(f"unknown kernel {kernel!r}")
    return int(kernel)


def kernel_select(M, N, K):
    k = lib.qg_kernel_select(M, N, K)
    if k < 0:
        raise QGemmError(k, "qg_kernel_select")
    return k


def dispatch_set_rules(rules):
    """rules: iterable of (m_lo, m_hi, n_lo, n_hi, k_lo, k_hi, kernel id or name); first match wins."""
    rules = [tuple(r[:6]) + (kernel_id(r[6]),) for r in rules]
    arr = (DispatchRule * max(len(rules), 1))(*[DispatchRule(*r) for r in rules])
    _check(lib.qg_dispatch_set_rules(arr, len(rules)), "qg_dispatch_set_rules")


def gemm_workspace_bytes(M, Bp):
    return lib.qg_gemm_workspace_bytes(M, Bp.handle)


def gemm_workspace(M, Bp, kernel=KERNEL_AUTO, ksplit=0):
    """A zero-initialised workspace for the K split across workgroups (None when the split factor is 1)."""
    n = lib.qg_gemm_splitk_workspace_bytes(M, Bp.handle, kernel_id(kernel), ksplit)
    if n == 0:
        return None
    ws = torch.empty(n, dtype=torch.uint8, device=Bp.packed.device)
    _check(lib.qg_gemm_workspace_init(ws.data_ptr(), n, _stream()), "qg_gemm_workspace_init")
    return ws


def gemm_splitk_factor(M, Bp, kernel=KERNEL_AUTO, ksplit=0):
    s = lib.qg_gemm_splitk_factor(M, Bp.handle, kernel_id(kernel), ksplit)
    if s < 0:
        raise QGemmError(s, "qg_gemm_splitk_factor")
    return s


def gemm_u8s8_requant_splitk(A, a_zp, Bp, bias, scales, c_zp, relu, workspace, kernel=KERNEL_AUTO, ksplit=0, out=None):
    """As gemm_u8s8_requant with the K split across workgroups chosen by the caller (0 = built-in choice): a streaming
    kernel, or "tile128" (the caller's factor only; slices of at least four 64-deep tiles)."""
    assert A.is_cuda and A.dtype == torch.uint8 and A.dim() == 2 and A.stride(1) == 1 and A.shape[1] == Bp.K
    M = A.shape[0]
    if out is None:
        out = torch.empty((M, Bp.N), dtype=torch.uint8, device=A.device)
    assert out.is_cuda and out.dtype == torch.uint8 and out.stride(1) == 1 and out.shape == (M, Bp.N)
    p = _params(a_zp, bias, scales, c_zp, relu)
    wp, wn = (workspace.data_ptr(), workspace.numel() * workspace.element_size()) if workspace is not None else (None, 0)
    _check(lib.qg_gemm_u8s8_requant_splitk(A.data_ptr(), M, A.stride(0), Bp.handle, ctypes.byref(p), out.data_ptr(),
                                           out.stride(0), wp, wn, _stream(), kernel_id(kernel), ksplit),
           "qg_gemm_u8s8_requant_splitk")
    return out


NOALLOC_SCRATCH_BYTES = 2 << 20


def gemm_u8s8_requant_noalloc(A, a_zp, Bp, bias, scales, c_zp, relu, out, kernel=KERNEL_AUTO, ksplit=0):
    """qg_gemm_u8s8_requant_noalloc: the K-split workspace is the library's built-in scratch; `out` is the caller's."""
    assert A.is_cuda and A.dtype == torch.uint8 and A.dim() == 2 and A.stride(1) == 1 and A.shape[1] == Bp.K
    assert out.is_cuda and out.dtype == torch.uint8 and out.stride(1) == 1 and out.shape == (A.shape[0], Bp.N)
    p = _params(a_zp, bias, scales, c_zp, relu)
    _check(lib.qg_gemm_u8s8_requant_noalloc(A.data_ptr(), A.shape[0], A.stride(0), Bp.handle, ctypes.byref(p),
                                            out.data_ptr(), out.stride(0), _stream(), kernel_id(kernel), ksplit),
           "qg_gemm_u8s8_requant_noalloc")
    return out


def gemm_u8s8_acc32_splitk(A, Bp, workspace, kernel=KERNEL_AUTO, ksplit=0, want_rowsum=False):
    assert A.is_cuda and A.dtype == torch.uint8 and A.dim() == 2 and A.stride(1) == 1
    M = A.shape[0]
    out = torch.empty((M, Bp.N), dtype=torch.int32, device=A.device)
    rs = torch.empty(M, dtype=torch.int32, device=A.device) if want_rowsum else None
    wp, wn = (workspace.data_ptr(), workspace.numel() * workspace.element_size()) if workspace is not None else (None, 0)
    _check(lib.qg_gemm_u8s8_acc32_splitk(A.data_ptr(), M, A.stride(0), Bp.handle, out.data_ptr(), out.stride(0),
                                         rs.data_ptr() if rs is not None else None, wp, wn, _stream(),
                                         kernel_id(kernel), ksplit), "qg_gemm_u8s8_acc32_splitk")
    return (out, rs) if want_rowsum else out


def gemm_u8s8_requant(A, a_zp, Bp, bias, scales, c_zp, relu, out=None, workspace=None, kernel=KERNEL_AUTO):
    """C_u8 = requant(A_u8 . B_s8): A uint8 cuda [M, K]; returns / fills uint8 [M, N]."""
    assert A.is_cuda and A.dtype == torch.uint8 and A.dim() == 2 and A.stride(1) == 1
    M = A.shape[0]
    assert A.shape[1] == Bp.K
    if out is None:
        out = torch.empty((M, Bp.N), dtype=torch.uint8, device=A.device)
    assert out.is_cuda and out.dtype == torch.uint8 and out.stride(1) == 1 and out.shape == (M, Bp.N)
    p = _params(a_zp, bias, scales, c_zp, relu)
    ws = workspace.data_ptr() if workspace is not None else None
    _check(lib.qg_gemm_u8s8_requant_kernel(A.data_ptr(), M, A.stride(0), Bp.handle, ctypes.byref(p), out.data_ptr(),
                                           out.stride(0), ws, _stream(), kernel_id(kernel)), "qg_gemm_u8s8_requant")
    return out


class PreparedGemm:
    """All arguments of one qg_gemm_u8s8_requant call marshalled once; `launch()` is a single ctypes call on
    the stream that was current when the object was made.  For loops that repeat the same call."""

    def __init__(self, A, a_zp, Bp, bias, scales, c_zp, relu, out, kernel=KERNEL_AUTO, workspace=None):
        assert A.is_cuda and A.dtype == torch.uint8 and A.dim() == 2 and A.stride(1) == 1 and A.shape[1] == Bp.K
        assert out.is_cuda and out.dtype == torch.uint8 and out.stride(1) == 1 and out.shape == (A.shape[0], Bp.N)
        self._keep = (A, Bp, bias, scales, out, workspace)
        self._p = _params(a_zp, bias, scales, c_zp, relu)
        self._args = (A.data_ptr(), A.shape[0], A.stride(0), Bp.handle, ctypes.byref(self._p), out.data_ptr(),
                      out.stride(0), workspace.data_ptr() if workspace is not None else None, _stream(),
                      kernel_id(kernel))
        self.out = out

    def launch(self):
        rc = lib.qg_gemm_u8s8_requant_kernel(*self._args)
        if rc != OK:
            raise QGemmError(rc, "qg_gemm_u8s8_requant")

    def rebind(self):
        """Later launches go to the stream that is current now (e.g. the capturing stream of a graph)."""
        self._args = self._args[:8] + (_stream(),) + self._args[9:]
        return self


class PreparedConv:
    """Same for qg_conv_groupwise_u8s8_requant."""

    def __init__(self, inp, Wp, a_zp, bias, scales, c_zp, relu, pad, stride, out):
        assert inp.is_cuda and inp.dtype == torch.uint8 and inp.dim() == 4 and inp.is_contiguous()
        assert out.is_cuda and out.dtype == torch.uint8 and out.is_contiguous()
        Nb, H, W, C = inp.shape
        self._keep = (inp, Wp, bias, scales, out)
        self._p = _params(a_zp, bias, scales, c_zp, relu)
        self._args = (inp.data_ptr(), Nb, H, W, C, pad, stride, Wp.handle, ctypes.byref(self._p), out.data_ptr(),
                      _stream())
        self.out = out

    def launch(self):
        rc = lib.qg_conv_groupwise_u8s8_requant(*self._args)
        if rc != OK:
            raise QGemmError(rc, "qg_conv_groupwise_u8s8_requant")

    def rebind(self):
        """Later launches go to the stream that is current now (e.g. the capturing stream of a graph)."""
        self._args = self._args[:-1] + (_stream(),)
        return self


class PreparedConvDense:
    """Same for qg_conv_dense_u8s8_requant (Wp from pack_conv_dense_w)."""

    def __init__(self, inp, Wp, a_zp, bias, scales, c_zp, relu, pad, stride, out, kernel=KERNEL_AUTO):
        assert inp.is_cuda and inp.dtype == torch.uint8 and inp.dim() == 4 and inp.is_contiguous()
        assert out.is_cuda and out.dtype == torch.uint8 and out.is_contiguous()
        Nb, H, W, C = inp.shape
        self._keep = (inp, Wp, bias, scales, out)
        self._p = _params(a_zp, bias, scales, c_zp, relu)
        self._args = (inp.data_ptr(), Nb, H, W, C, Wp.R, Wp.S, pad, stride, Wp.handle, ctypes.byref(self._p), out.data_ptr(),
                      _stream(), kernel_id(kernel))
        self.out = out

    def launch(self):
        rc = lib.qg_conv_dense_u8s8_requant(*self._args)
        if rc != OK:
            raise QGemmError(rc, "qg_conv_dense_u8s8_requant")

    def rebind(self):
        """Later launches go to the stream that is current now (e.g. the capturing stream of a graph)."""
        self._args = self._args[:12] + (_stream(),) + self._args[13:]
        return self


def gemm_u8s8_acc32(A, Bp, want_rowsum=False, kernel=KERNEL_AUTO):
    assert A.is_cuda and A.dtype == torch.uint8 and A.dim() == 2 and A.stride(1) == 1
    M = A.shape[0]
    out = torch.empty((M, Bp.N), dtype=torch.int32, device=A.device)
    rs = torch.empty(M, dtype=torch.int32, device=A.device) if want_rowsum else None
    _check(lib.qg_gemm_u8s8_acc32_kernel(A.data_ptr(), M, A.stride(0), Bp.handle, out.data_ptr(), out.stride(0),
                                         rs.data_ptr() if rs is not None else None, None, _stream(),
                                         kernel_id(kernel)), "qg_gemm_u8s8_acc32")
    return (out, rs) if want_rowsum else out


def _dq_params(a_zp, bias, scales, relu):
    assert scales.is_cuda and scales.dtype == torch.float32 and scales.is_contiguous()
    if bias is not None:
        assert bias.is_cuda and bias.dtype == torch.int32 and bias.is_contiguous()
    return DequantParams(int(a_zp), bias.data_ptr() if bias is not None else None, scales.data_ptr(),
                         scales.numel(), int(bool(relu)))


def _f32_out(out, M, N, dev):
    if out is None:
        out = torch.empty((M, N), dtype=torch.float32, device=dev)
    assert out.is_cuda and out.dtype == torch.float32 and out.stride(1) == 1 and out.shape == (M, N)
    return out


def gemm_u8s8_dequant_f32(A, a_zp, Bp, bias, scales, relu, out=None, kernel=KERNEL_AUTO):
    """fp32 C = (alpha_A alpha_B) * corrected accumulator: A uint8 cuda [M, K]; returns / fills float32 [M, N]."""
    assert A.is_cuda and A.dtype == torch.uint8 and A.dim() == 2 and A.stride(1) == 1 and A.shape[1] == Bp.K
    M = A.shape[0]
    out = _f32_out(out, M, Bp.N, A.device)
    p = _dq_params(a_zp, bias, scales, relu)
    _check(lib.qg_gemm_u8s8_dequant_f32(A.data_ptr(), M, A.stride(0), Bp.handle, ctypes.byref(p), out.data_ptr(),
                                        out.stride(0), None, _stream(), kernel_id(kernel)), "qg_gemm_u8s8_dequant_f32")
    return out


def quantize_a_f32(A, inv_scale, a_zp, out=None):
    """uint8 copy of an fp32 activation matrix (cuda [M, K], unit column stride)."""
    assert A.is_cuda and A.dtype == torch.float32 and A.dim() == 2 and A.stride(1) == 1
    M, K = A.shape
    if out is None:
        out = torch.empty((M, K), dtype=torch.uint8, device=A.device)
    assert out.is_cuda and out.dtype == torch.uint8 and out.stride(1) == 1 and out.shape == (M, K)
    _check(lib.qg_quantize_a_f32(A.data_ptr(), M, K, A.stride(0), float(inv_scale), int(a_zp), out.data_ptr(),
                                 out.stride(0), _stream()), "qg_quantize_a_f32")
    return out


def gemm_f32_workspace_bytes(M, Bp):
    return lib.qg_gemm_f32_workspace_bytes(M, Bp.handle)


class _NoWorkspace:
    """Stands for a NULL workspace pointer (the one-launch form on a streaming kernel needs none)."""

    @staticmethod
    def data_ptr():
        return None


NO_WORKSPACE = _NoWorkspace()


def _f32_ws(A, Bp, workspace):
    assert A.is_cuda and A.dtype == torch.float32 and A.dim() == 2 and A.stride(1) == 1 and A.shape[1] == Bp.K
    if workspace is None:
        workspace = torch.empty(gemm_f32_workspace_bytes(A.shape[0], Bp), dtype=torch.uint8, device=A.device)
    return workspace


def gemm_f32s8_requant(A, a_inv_scale, a_zp, Bp, bias, scales, c_zp, relu, out=None, workspace=None,
                       kernel=KERNEL_AUTO):
    """fp32 activations, quantized by the library, uint8 out."""
    ws = _f32_ws(A, Bp, workspace)
    M = A.shape[0]
    if out is None:
        out = torch.empty((M, Bp.N), dtype=torch.uint8, device=A.device)
    assert out.is_cuda and out.dtype == torch.uint8 and out.stride(1) == 1 and out.shape == (M, Bp.N)
    p = _params(a_zp, bias, scales, c_zp, relu)
    _check(lib.qg_gemm_f32s8_requant(A.data_ptr(), M, A.stride(0), float(a_inv_scale), Bp.handle, ctypes.byref(p),
                                     out.data_ptr(), out.stride(0), ws.data_ptr(), _stream(), kernel_id(kernel)),
           "qg_gemm_f32s8_requant")
    return out


def gemm_f32s8_dequant_f32(A, a_inv_scale, a_zp, Bp, bias, scales, relu, out=None, workspace=None,
                           kernel=KERNEL_AUTO):
    """fp32 activations in, fp32 result out."""
    ws = _f32_ws(A, Bp, workspace)
    M = A.shape[0]
    out = _f32_out(out, M, Bp.N, A.device)
    p = _dq_params(a_zp, bias, scales, relu)
    _check(lib.qg_gemm_f32s8_dequant_f32(A.data_ptr(), M, A.stride(0), float(a_inv_scale), Bp.handle,
                                         ctypes.byref(p), out.data_ptr(), out.stride(0), ws.data_ptr(), _stream(),
                                         kernel_id(kernel)), "qg_gemm_f32s8_dequant_f32")
    return out


def pack_conv_w(Wt, b_zp):
    """Wt: int8 cuda [G][R][S][C/G][Cout/G], contiguous."""
    assert Wt.is_cuda and Wt.dtype == torch.int8 and Wt.dim() == 5 and Wt.is_contiguous()
    G, R, S, Cg, Og = Wt.shape
    pb, cb = ctypes.c_size_t(), ctypes.c_size_t()
    _check(lib.qg_pack_conv_w_sizes(G, R, S, Cg, Og, ctypes.byref(pb), ctypes.byref(cb)), "qg_pack_conv_w_sizes")
    packed = torch.empty(pb.value, dtype=torch.int8, device=Wt.device)
    aux = torch.empty(cb.value // 4, dtype=torch.int32, device=Wt.device)
    z, zp = _host_i32(b_zp)
    h = ctypes.c_void_p()
    _check(lib.qg_pack_conv_w(Wt.data_ptr(), G, R, S, Cg, Og, zp, z.size, packed.data_ptr(), aux.data_ptr(),
                              _stream(), ctypes.byref(h)), "qg_pack_conv_w")
    pk = PackedB(h, packed, aux, G * Og)
    pk.R, pk.S = R, S
    return pk


def conv_groupwise_u8s8_requant(inp, Wp, a_zp, bias, scales, c_zp, relu, pad=1, stride=1, out=None):
    """inp: uint8 cuda NHWC contiguous; returns uint8 NHWC."""
    assert inp.is_cuda and inp.dtype == torch.uint8 and inp.dim() == 4 and inp.is_contiguous()
    Nb, H, W, C = inp.shape
    Ho = (H + 2 * pad - Wp.R) // stride + 1
    Wo = (W + 2 * pad - Wp.S) // stride + 1
    if out is None:
        out = torch.empty((Nb, Ho, Wo, Wp.N), dtype=torch.uint8, device=inp.device)
    assert out.is_contiguous() and out.shape == (Nb, Ho, Wo, Wp.N)
    p = _params(a_zp, bias, scales, c_zp, relu)
    _check(lib.qg_conv_groupwise_u8s8_requant(inp.data_ptr(), Nb, H, W, C, pad, stride, Wp.handle,
                                              ctypes.byref(p), out.data_ptr(), _stream()),
           "qg_conv_groupwise_u8s8_requant")
    return out


def pack_conv_dense_w(Wt, b_zp):
    """Dense-convolution weights int8 cuda [R][S][Cin][Cout] -> GEMM descriptor of the (R*S*Cin) x Cout matrix."""
    assert Wt.is_cuda and Wt.dtype == torch.int8 and Wt.dim() == 4 and Wt.is_contiguous()
    R, S, Cin, Cout = Wt.shape
    pk = pack_b(Wt.view(R * S * Cin, Cout), b_zp)
    pk.R, pk.S = R, S
    return pk


def conv_dense_u8s8_requant(inp, Wp, a_zp, bias, scales, c_zp, relu, pad=1, stride=1, out=None, kernel="auto"):
    """inp: uint8 cuda NHWC contiguous (Cin % 16 == 0 for the staged kernels, anything under kernel="auto"); Wp from pack_conv_dense_w; returns uint8 NHWC.
    kernel: "auto", one of the 64- and 128-row tiled kernels or streaming kernels (name or id; not the 256 x 256 tile), or
    "patch64x128" / "patch128x64" / "patch256x64" / "patch256" / "patch512" (stride-1 "same" layers with Cin % 32 == 0: the input patch stays in LDS)."""
    assert inp.is_cuda and inp.dtype == torch.uint8 and inp.dim() == 4 and inp.is_contiguous()
    Nb, H, W, C = inp.shape
    Ho = (H + 2 * pad - Wp.R) // stride + 1
    Wo = (W + 2 * pad - Wp.S) // stride + 1
    if out is None:
        out = torch.empty((Nb, Ho, Wo, Wp.N), dtype=torch.uint8, device=inp.device)
    assert out.is_contiguous() and out.shape == (Nb, Ho, Wo, Wp.N)
    p = _params(a_zp, bias, scales, c_zp, relu)
    _check(lib.qg_conv_dense_u8s8_requant(inp.data_ptr(), Nb, H, W, C, Wp.R, Wp.S, pad, stride, Wp.handle,
                                          ctypes.byref(p), out.data_ptr(), _stream(), kernel_id(kernel)),
           "qg_conv_dense_u8s8_requant")
    return out
