"""Host-side checks that need no GPU: the library loads, exports every symbol the header declares,
and rejects bad arguments before touching the device."""
import ctypes
import os
import re

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
HEADER = os.path.join(ROOT, "include", "qgemm.h")
LIB = os.path.join(ROOT, "paper_2101_05615_amd", "libqgemm.so")


@pytest.fixture(scope="module")
def lib():
    if not os.path.exists(LIB):
        import __graft_entry__ as g
        g.build()
    from paper_2101_05615_amd import qgemm
    return qgemm.lib


def declared_symbols():
    text = open(HEADER).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(qg_[a-z0-9_]+)\s*\(", text)))


def test_header_declares_the_expected_entry_points():
    syms = declared_symbols()
    for must in ["qg_pack_b", "qg_pack_b_sizes", "qg_gemm_u8s8_requant", "qg_gemm_u8s8_acc32",
                 "qg_conv_groupwise_u8s8_requant", "qg_packed_b_destroy", "qg_status_string"]:
        assert must in syms


def test_library_exports_every_declared_symbol(lib):
    raw = ctypes.CDLL(LIB)
    for s in declared_symbols():
        assert hasattr(raw, s), f"{s} declared in qgemm.h but not exported"
    from paper_2101_05615_amd import qgemm
    assert sorted(qgemm.EXPORTS) == declared_symbols()


def test_no_torch_types_in_the_boundary():
    text = open(HEADER).read()
    assert "torch" not in text.lower() and "at::" not in text and "#include <hip" not in text


def test_pack_sizes_and_padding(lib):
    pb, cb = ctypes.c_size_t(), ctypes.c_size_t()
    assert lib.qg_pack_b_sizes(4096, 4096, ctypes.byref(pb), ctypes.byref(cb)) == 0
    assert pb.value == 4096 * 4096 and cb.value == 2 * 4096 * 4
    assert lib.qg_pack_b_sizes(36, 4, ctypes.byref(pb), ctypes.byref(cb)) == 0
    assert pb.value == 128 * 256 and cb.value == 2 * 256 * 4
    assert lib.qg_pack_b_sizes(1, 257, ctypes.byref(pb), ctypes.byref(cb)) == 0
    assert pb.value == 128 * 512


def test_size_query_rejects_bad_arguments(lib):
    from paper_2101_05615_amd import qgemm as q
    pb, cb = ctypes.c_size_t(), ctypes.c_size_t()
    assert lib.qg_pack_b_sizes(0, 4, ctypes.byref(pb), ctypes.byref(cb)) == q.EINVAL
    assert lib.qg_pack_b_sizes(4, -1, ctypes.byref(pb), ctypes.byref(cb)) == q.EINVAL
    assert lib.qg_pack_b_sizes(q.MAX_K + 1, 4, ctypes.byref(pb), ctypes.byref(cb)) == q.EINVAL
    assert lib.qg_pack_b_sizes(q.MAX_K, 4, ctypes.byref(pb), ctypes.byref(cb)) == q.OK
    assert lib.qg_pack_b_sizes(4, 4, None, ctypes.byref(cb)) == q.ENULL
    assert lib.qg_pack_conv_w_sizes(32, 3, 3, 4, 4, ctypes.byref(pb), ctypes.byref(cb)) == q.OK
    assert pb.value >= 32 * 36 * 4
    # any group shape: [Cout][R*S][Cg rounded up to 4] bytes, plus block-diagonal tiles where they exist
    assert lib.qg_pack_conv_w_sizes(32, 3, 3, 8, 4, ctypes.byref(pb), ctypes.byref(cb)) == q.OK
    assert pb.value == 32 * 4 * 9 * 8 and cb.value >= 2 * 128 * 4
    assert lib.qg_pack_conv_w_sizes(32, 5, 5, 4, 4, ctypes.byref(pb), ctypes.byref(cb)) == q.OK
    assert pb.value == 32 * 4 * 25 * 4
    assert lib.qg_pack_conv_w_sizes(8, 3, 3, 8, 8, ctypes.byref(pb), ctypes.byref(cb)) == q.OK
    assert pb.value == 64 * 9 * 8 + 2 * 9 * 1024            # 64 channels: two 32-channel blocks of nine tiles
    assert lib.qg_pack_conv_w_sizes(3, 2, 5, 3, 7, ctypes.byref(pb), ctypes.byref(cb)) == q.OK
    assert pb.value == (21 * 10 * 4 + 255) // 256 * 256
    assert lib.qg_pack_conv_w_sizes(1, 64, 64, 16, 4, ctypes.byref(pb), ctypes.byref(cb)) == q.EINVAL   # K beyond the bound
    assert lib.qg_pack_conv_w_sizes(0, 3, 3, 4, 4, ctypes.byref(pb), ctypes.byref(cb)) == q.EINVAL


def test_null_and_range_checks_happen_before_any_device_work(lib):
    from paper_2101_05615_amd import qgemm as q
    h = ctypes.c_void_p()
    fake = ctypes.c_void_p(256)  # never dereferenced: the checks below fail first
    assert lib.qg_pack_b(None, 4, 4, 4, fake, 1, fake, fake, None, ctypes.byref(h)) == q.ENULL
    assert lib.qg_pack_b(fake, 4, 4, 4, None, 1, fake, fake, None, ctypes.byref(h)) == q.ENULL
    assert lib.qg_pack_b(fake, 4, 4, 3, fake, 1, fake, fake, None, ctypes.byref(h)) == q.EINVAL   # ldb < N
    assert lib.qg_pack_b(fake, 4, 4, 4, fake, 2, fake, fake, None, ctypes.byref(h)) == q.EINVAL   # n_b_zp
    assert lib.qg_pack_b(fake, q.MAX_K + 1, 4, 4, fake, 1, fake, fake, None, ctypes.byref(h)) == q.EINVAL
    assert lib.qg_pack_b(fake, 4, 4, 4, fake, 1, ctypes.c_void_p(260), fake, None, ctypes.byref(h)) == q.EALIGN
    p = q.RequantParams(0, None, 256, 1, 0, 0)
    assert lib.qg_gemm_u8s8_requant(fake, 4, 4, None, ctypes.byref(p), fake, 4, None, None) == q.ENULL
    assert lib.qg_gemm_u8s8_acc32(None, 4, 4, None, fake, 4, None, None, None) == q.ENULL
    assert lib.qg_conv_groupwise_u8s8_requant(fake, 1, 4, 4, 4, 1, 1, None, ctypes.byref(p), fake, None) == q.ENULL
    lib.qg_packed_b_destroy(None)
    assert lib.qg_packed_b_k(None) == 0 and lib.qg_gemm_workspace_bytes(16, None) == 0


def test_status_strings(lib):
    for code in range(0, -9, -1):
        s = lib.qg_status_string(code)
        assert s and (code == 0) == (s == b"ok")
    assert lib.qg_status_string(-99) == b"unknown status"


def test_column_permutation_is_a_bijection_with_16_contiguous_columns_per_lane():
    # host model of the packed layout rule stated in the header of the packing code:
    # column c = 16h + 4q + t of a 32-column super-block sits in slot 8q + 4h + t
    slot = lambda c: ((c >> 2) & 3) * 8 + (c >> 4) * 4 + (c & 3)
    assert sorted(slot(c) for c in range(32)) == list(range(32))
    # the 32x32 MFMA gives lane-half h, register r = 4q + t the row 8q + 4h + t:
    for h in range(2):
        cols = []
        for r in range(16):
            q, t = r >> 2, r & 3
            i = 8 * q + 4 * h + t
            cols.append([c for c in range(32) if slot(c) == i][0])
        assert cols == list(range(16 * h, 16 * h + 16))


def test_kernel_selection_is_host_logic(lib):
    """The shape -> kernel map of the shape-specific family: ids, names, built-in choice, rule table."""
    from paper_2101_05615_amd import qgemm as q
    names = q.kernel_names()
    assert names[0] == "auto" and len(set(names.values())) == q.KERNEL_LAST + 1
    # the ids above the GEMM family's are kernels of the dense convolution only
    assert [lib.qg_kernel_name(k) for k in range(q.KERNEL_LAST + 1, q.KERNEL_CONV_LAST + 1)] == [b"patch64x128", b"patch128x64", b"patch256x64", b"patch256", b"patch512"]
    assert q.kernel_id("patch256x64") == q.KERNEL_LAST + 3
    assert lib.qg_kernel_name(q.KERNEL_CONV_LAST + 1) is None
    # small batches go to the streaming kernels, one row block when M fits the smallest
    assert names[q.kernel_select(1, 4096, 4096)] == "skinny16"
    assert names[q.kernel_select(16, 4096, 4096)] == "skinny16"
    for M in (17, 32, 33, 48, 64):
        assert names[q.kernel_select(M, 4096, 4096)].startswith("skinny")
    # the large shapes go to the large tiles, thin grids to the small ones
    assert names[q.kernel_select(8192, 8192, 8192)] == "tile256"
    assert names[q.kernel_select(32768, 512, 1024)] in ("tile256", "tile128x256")
    assert names[q.kernel_select(2048, 2048, 2048)] == "tile128"
    assert names[q.kernel_select(128, 8192, 1024)] in ("tile64", "tile64k4")
    # the choice is always a concrete kernel
    for shape in [(65, 64, 64), (128, 4096, 4096), (2048, 2048, 2048), (32768, 512, 1024), (1 << 20, 16, 64)]:
        assert 1 <= q.kernel_select(*shape) <= q.KERNEL_LAST
    for bad in [(0, 1, 1), (1, 0, 1), (1, 1, 0), (-5, 4, 4)]:
        assert lib.qg_kernel_select(*bad) == q.EINVAL


def test_dispatch_rule_table(lib):
    from paper_2101_05615_amd import qgemm as q
    big = 1 << 30
    before = q.kernel_select(500, 500, 512)
    try:
        q.dispatch_set_rules([(400, 600, 1, big, 1, big, "tile64"), (1, big, 1, big, 1, big, "tile128")])
        assert q.kernel_names()[q.kernel_select(500, 500, 512)] == "tile64"     # first match wins
        assert q.kernel_names()[q.kernel_select(700, 500, 512)] == "tile128"
        # malformed tables change nothing
        R = q.DispatchRule
        for bad in [R(5, 4, 1, 2, 1, 2, 4), R(1, 2, 1, 2, 1, 2, 0), R(1, 2, 1, 2, 1, 2, q.KERNEL_LAST + 1), R(1, 2, 3, 2, 1, 2, 4)]:
            arr = (R * 1)(bad)
            assert lib.qg_dispatch_set_rules(arr, 1) == q.EINVAL
        assert lib.qg_dispatch_set_rules(None, 1) == q.ENULL
        assert lib.qg_dispatch_set_rules(None, -1) == q.EINVAL
        assert lib.qg_dispatch_set_rules(None, q.MAX_DISPATCH_RULES + 1) == q.EINVAL
        assert q.kernel_names()[q.kernel_select(500, 500, 512)] == "tile64"
        # a streaming kernel that would need more row blocks than the grid allows falls back to the built-in choice
        q.dispatch_set_rules([(1, big, 1, big, 1, big, "skinny16")])
        assert q.kernel_names()[q.kernel_select(16 * 65535, 64, 64)] == "skinny16"
        assert q.kernel_names()[q.kernel_select(16 * 65535 + 1, 64, 64)] != "skinny16"
    finally:
        q.dispatch_set_rules([])
    assert q.kernel_select(500, 500, 512) == before


def test_bench_refuses_more_than_one_gpu():
    """This build shows one GPU's share; bench.py says so and exits before touching a device."""
    import subprocess
    import sys
    root = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
    r = subprocess.run([sys.executable, os.path.join(root, "bench.py"), "--gpus", "2"], capture_output=True, text=True,
                       timeout=120)
    assert r.returncode != 0 and "ONE GPU" in r.stderr and r.stdout.strip() == ""


def test_workload_biases_respect_the_documented_bound():
    """qgemm.h: |bias[j]| <= 2^31 - 1 - 255 * 255 * K, outside of which the 32-bit corrected accumulator may wrap (the
    oracle then reports an overflow).  The seeded generators must stay inside it."""
    from paper_2101_05615_amd import workloads as wl
    cases = [wl.config1_tiny(), wl.config2_small_batch_fc(with_bias=True), wl.random_gemm(1, 40, 50, 1000),
             wl.random_gemm(2, 3, 16, 32768), wl.unsaturated(wl.random_gemm(3, 17, 33, 4097))]
    for c in cases:
        if c.bias is not None:
            bound = 2 ** 31 - 1 - 255 * 255 * c.K
            assert bound > 0 and int(abs(c.bias.astype("int64")).max()) <= bound, c.name
