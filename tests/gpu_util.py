"""Helpers for the GPU parity tests: run a seeded case through the C ABI (via the binding) and
compare with the CPU oracle element by element."""
import sys

import numpy as np


def say(msg):
    print(msg, flush=True)
    sys.stdout.flush()


def assert_same(got, want, what):
    got = np.asarray(got)
    want = np.asarray(want)
    assert got.shape == want.shape, f"{what}: shape {got.shape} vs {want.shape}"
    if not np.array_equal(got, want):
        bad = np.argwhere(got != want)
        first = tuple(int(v) for v in bad[0])
        raise AssertionError(f"{what}: {len(bad)} of {want.size} elements differ; first at {first}: "
                             f"got {got[first]} want {want[first]}")


def dev_case(case, torch, dev, lda_pad=0, ldc_pad=0, a_off=0, c_off=0):
    """Upload a GemmCase; optional leading-dimension padding and byte offsets exercise the unaligned paths."""
    M, K, N = case.M, case.K, case.N
    a_store = torch.full((M * (K + lda_pad) + a_off + 64,), 0x5A, dtype=torch.uint8, device=dev)  # padding is garbage
    A = a_store[a_off:a_off + M * (K + lda_pad)].view(M, K + lda_pad)[:, :K]
    A.copy_(torch.from_numpy(case.A).to(dev))
    c_store = torch.full((M * (N + ldc_pad) + c_off + 64,), 0xEE, dtype=torch.uint8, device=dev)
    C = c_store[c_off:c_off + M * (N + ldc_pad)].view(M, N + ldc_pad)[:, :N]
    B = torch.from_numpy(case.B).to(dev)
    bias = None if case.bias is None else torch.from_numpy(case.bias).to(dev)
    scales = torch.from_numpy(case.scales).to(dev)
    return A, B, bias, scales, C, c_store


def run_gemm(case, q, torch, dev, **kw):
    A, B, bias, scales, C, c_store = dev_case(case, torch, dev, **kw)
    Bp = q.pack_b(B, case.b_zp)
    q.gemm_u8s8_requant(A, case.a_zp, Bp, bias, scales, case.c_zp, case.relu, out=C)
    torch.cuda.synchronize()
    return C.cpu().numpy(), c_store.cpu().numpy(), Bp


def oracle_gemm(case, oracle, rows=None):
    A = case.A if rows is None else np.ascontiguousarray(case.A[rows])
    return oracle.gemm_u8s8_requant(A, case.a_zp, case.B, case.b_zp, case.bias, case.scales, case.c_zp,
                                    case.relu)
