"""Offline autotune of the shape-specific kernel family (paper Appendix C).

Times every kernel of the family on the given shapes (seeded synthetic operands, resident in HBM) and
writes a dispatch table: one rule per shape naming the fastest kernel.  `load_table()` installs such a
table with qg_dispatch_set_rules, after which QG_KERNEL_AUTO follows it; shapes that no rule covers keep
the library's built-in choice.

    python -m paper_2101_05615_amd.autotune --shapes 128x4096x4096,2048x2048x2048 --out table.json
    python -m paper_2101_05615_amd.autotune --grid --out table.json

    python -m paper_2101_05615_amd.autotune --cold --shapes 64x8192x8192 --out table.json

    python -m paper_2101_05615_amd.autotune --conv-grid

Every kernel returns identical bytes for a given input, so the table affects speed only.  Times are warm
(back-to-back launches on one set of buffers, weights in the memory-side cache when they fit) unless --cold is given.  --conv-grid times every
kernel id of the dense convolution (tiled, streaming and patch-resident kernels) and the automatic choice on a
built-in list of layers and reports what the choice loses against the measured best (the convolution has no rule
table: its built-in cost constants were fitted to such a run).
"""
import argparse
import json
import sys

GRID_M = [65, 96, 128, 192, 256, 384, 512, 1024, 2048, 4096, 8192, 32768]
GRID_N = [64, 256, 512, 1024, 2048, 4096, 8192]
GRID_K = [256, 1024, 4096]
MAX_OPS = 2.5e12  # skip grid points larger than the headline square
# the small-batch shapes the paper stresses (Appendix C: M = 1 .. 64, N sometimes very small)
SMALL_M = [1, 2, 4, 8, 16, 32, 64]
SMALL_N = [4, 16, 64, 256, 1024, 4096]
SMALL_K = [256, 1024, 4096]


def time_shape(q, torch, M, N, K, kernels, min_ms=3.0, seed=0, spin_ms=15.0):
    """-> {kernel name: microseconds per launch}; operands drawn on the device from a seeded generator.
    Each kernel first runs untimed for spin_ms of wall time, so that it is timed at settled clocks."""
    import time
    dev = torch.device("cuda:0")
    g = torch.Generator(device=dev)
    g.manual_seed(seed)
    A = torch.randint(0, 256, (M, K), dtype=torch.uint8, device=dev, generator=g)
    B = torch.randint(-128, 128, (K, N), dtype=torch.int8, device=dev, generator=g)
    b_zp = torch.randint(-8, 9, (N,), generator=torch.Generator().manual_seed(seed)).numpy()
    scales = torch.full((N,), 2.0 ** -12, dtype=torch.float32, device=dev)
    Bp = q.pack_b(B, b_zp)
    C = torch.empty((M, N), dtype=torch.uint8, device=dev)
    out = {}
    for name in kernels:
        call = q.PreparedGemm(A, 128, Bp, None, scales, 0, True, C, kernel=name)
        t_end = time.perf_counter() + spin_ms * 1e-3
        while True:
            for _ in range(8):
                call.launch()
            torch.cuda.synchronize()
            if time.perf_counter() >= t_end:
                break
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        n, best = 4, None
        while True:
            e0.record()
            for _ in range(n):
                call.launch()
            e1.record()
            torch.cuda.synchronize()
            ms = e0.elapsed_time(e1)
            best = ms / n if best is None else min(best, ms / n)
            if ms >= min_ms or n >= 4096:
                break
            n *= 4
        out[name] = best * 1e3
    Bp.close()
    return out


def time_cold_kernels(q, torch, M, N, K, kernels, seed=0, reps=3):
    """Microseconds per launch with COLD weights, per kernel: the launches rotate over enough packed copies of B
    (more than 1 GB together, at most 256) that the 256 MB memory-side cache cannot hold them, recorded as one graph
    per kernel and replayed (no host cost per launch).  -> ({kernel name: us}, copies)"""
    dev = torch.device("cuda:0")
    g = torch.Generator(device=dev)
    g.manual_seed(seed)
    A = torch.randint(0, 256, (M, K), dtype=torch.uint8, device=dev, generator=g)
    B = torch.randint(-128, 128, (K, N), dtype=torch.int8, device=dev, generator=g)
    scales = torch.full((N,), 2.0 ** -12, dtype=torch.float32, device=dev)
    b_zp = torch.randint(-8, 9, (N,), generator=torch.Generator().manual_seed(seed)).numpy()
    ncopy = int(max(2, min(256, 1.2e9 // (K * N))))
    packed = [q.pack_b(B, b_zp) for _ in range(ncopy)]
    acts = [A.clone() for _ in range(ncopy)]
    outs = [torch.empty((M, N), dtype=torch.uint8, device=dev) for _ in range(ncopy)]
    result = {}
    for kernel in kernels:
        calls = [q.PreparedGemm(acts[i], 128, packed[i], None, scales, 0, True, outs[i], kernel=kernel) for i in range(ncopy)]
        for c in calls:
            c.launch()
        torch.cuda.synchronize()
        graph = torch.cuda.CUDAGraph()
        with torch.cuda.graph(graph):
            for c in calls:
                c.rebind().launch()
        for _ in range(3):
            graph.replay()
        torch.cuda.synchronize()
        best = None
        for _ in range(reps):
            e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            e0.record()
            graph.replay()
            e1.record()
            torch.cuda.synchronize()
            t = e0.elapsed_time(e1) * 1e3 / ncopy
            best = t if best is None else min(best, t)
        result[kernel] = best
        del graph, calls
    for Bp in packed:
        Bp.close()
    return result, ncopy


def time_cold(q, torch, M, N, K, kernel="auto", seed=0, reps=3):
    """One kernel with cold weights -> (us, copies)."""
    t, ncopy = time_cold_kernels(q, torch, M, N, K, [kernel], seed, reps)
    return t[kernel], ncopy


# dense convolution layers (H = W, Cin, Cout, filter, stride), each at 1, 4, 8 and 32 images
CONV_LAYERS = [(56, 64, 64, 3, 1), (56, 64, 128, 3, 1), (56, 128, 128, 3, 1), (56, 96, 96, 3, 1), (28, 128, 128, 3, 1),
               (28, 256, 256, 3, 1), (28, 192, 192, 3, 1), (28, 64, 64, 5, 1), (14, 256, 256, 3, 1), (14, 512, 512, 3, 1),
               (7, 512, 512, 3, 1), (112, 64, 64, 3, 1), (112, 32, 32, 3, 1), (56, 32, 64, 3, 1), (28, 128, 256, 3, 1),
               (56, 256, 64, 3, 1), (224, 32, 32, 3, 1), (56, 128, 32, 3, 1), (14, 160, 320, 3, 1), (28, 128, 128, 5, 1),
               (56, 64, 128, 3, 2), (28, 128, 256, 3, 2), (14, 256, 512, 3, 2), (112, 128, 128, 3, 1), (56, 256, 256, 3, 1)]
CONV_BATCHES = [1, 4, 8, 32]


def time_conv_layer(q, torch, Nb, H, Cin, Cout, R, stride, kernels, seed=0, spin_ms=10.0):
    """-> {kernel name: microseconds per launch} for the kernels that take the layer; a recorded graph of 20 launches,
    replayed after spin_ms of untimed replays (settled clocks)."""
    import time
    dev = torch.device("cuda:0")
    g = torch.Generator(device=dev)
    g.manual_seed(seed)
    x = torch.randint(0, 256, (Nb, H, H, Cin), dtype=torch.uint8, device=dev, generator=g)
    w = torch.randint(-127, 128, (R, R, Cin, Cout), dtype=torch.int8, device=dev, generator=g)
    b_zp = torch.randint(-8, 9, (Cout,), generator=torch.Generator().manual_seed(seed)).tolist()
    Wd = q.pack_conv_dense_w(w, b_zp)
    sc = torch.full((Cout,), 1e-4, dtype=torch.float32, device=dev)
    Ho = (H + 2 * (R // 2) - R) // stride + 1
    y = torch.empty((Nb, Ho, Ho, Cout), dtype=torch.uint8, device=dev)
    out = {}
    for k in kernels:
        call = lambda: q.conv_dense_u8s8_requant(x, Wd, 3, None, sc, 5, False, pad=R // 2, stride=stride, out=y, kernel=k)
        try:
            call()
        except q.QGemmError:
            continue   # the kernel does not take this layer
        torch.cuda.synchronize()
        gr = torch.cuda.CUDAGraph()
        with torch.cuda.graph(gr):
            for _ in range(20):
                call()
        t_end = time.perf_counter() + spin_ms * 1e-3
        while time.perf_counter() < t_end:
            gr.replay()
            torch.cuda.synchronize()
        best = float("inf")
        for _ in range(4):
            e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            e0.record()
            gr.replay()
            e1.record()
            torch.cuda.synchronize()
            best = min(best, e0.elapsed_time(e1) * 1e3 / 20)
        out[k] = best
        del gr
    return out


def tune_conv(q, torch, log=None):
    names = [q.lib.qg_kernel_name(k).decode() for k in range(1, q.KERNEL_CONV_LAST + 1)]
    names = [n for n in names if n != "tile256"]
    rows = []
    for Nb in CONV_BATCHES:
        for (H, Cin, Cout, R, stride) in CONV_LAYERS:
            if Nb * H * H * max(Cin, Cout) > 64e6:
                continue
            t = time_conv_layer(q, torch, Nb, H, Cin, Cout, R, stride, names + ["auto"])
            auto = t.pop("auto")
            best = min(t, key=t.get)
            rows.append({"Nb": Nb, "H": H, "Cin": Cin, "Cout": Cout, "R": R, "stride": stride, "best": best, "auto_us": auto, "us": t})
            if log:
                log(f"{Nb:3d} x {H:3d}^2 x {Cin:3d} -> {Cout:3d}, {R}x{R} s{stride}: best {best:12s} {t[best]:7.2f} us, auto {auto:7.2f} us "
                    f"({auto / t[best]:4.2f}x), best without the patch kernels {min(v for k, v in t.items() if not k.startswith('patch')):7.2f} us")
    return rows


def conv_summary(rows):
    import math
    wins = {}
    for r in rows:
        wins[r["best"]] = wins.get(r["best"], 0) + 1
    loss = [r["auto_us"] / r["us"][r["best"]] for r in rows]
    gain = [min(v for k, v in r["us"].items() if not k.startswith("patch")) / r["us"][r["best"]] for r in rows]
    gm = lambda v: math.exp(sum(map(math.log, v)) / len(v))
    out = [f"layers: {len(rows)}",
           "fastest kernel, number of layers: " + ", ".join(f"{k} {v}" for k, v in sorted(wins.items())),
           f"automatic choice vs measured best: geometric mean {gm(loss):.4f}x, within 5 % on {sum(l <= 1.05 for l in loss)} layers, "
           f"worst {max(loss):.2f}x",
           f"best kernel vs best of the kernels without a resident patch: geometric mean {gm(gain):.3f}x faster, at most {max(gain):.2f}x"]
    return "\n".join(out)


def tune(q, torch, shapes, kernels=None, log=None, cold=False):
    names = q.kernel_names()
    kernels = kernels or [names[k] for k in range(1, q.KERNEL_LAST + 1)]
    rows = []
    for (M, N, K) in shapes:
        t = time_cold_kernels(q, torch, M, N, K, kernels)[0] if cold else time_shape(q, torch, M, N, K, kernels)
        best = min(t, key=t.get)
        auto = names[q.kernel_select(M, N, K)]
        rows.append({"M": M, "N": N, "K": K, "best": best, "auto": auto, "us": t})
        if log:
            line = " ".join(f"{k}={v:9.1f}" for k, v in t.items())
            log(f"{M:6d} {N:6d} {K:6d}  best {best:12s} auto {auto:12s} loss {t[auto] / t[best]:5.2f}x  {line}")
    return rows


def summary(rows):
    """A few lines: how often each kernel wins, and what the automatic choice loses against the measured best."""
    import math
    wins = {}
    for r in rows:
        wins[r["best"]] = wins.get(r["best"], 0) + 1
    loss = [r["us"][r["auto"]] / r["us"][r["best"]] for r in rows]
    worst = sorted(zip(loss, rows), key=lambda t: -t[0])[:5]
    out = [f"shapes: {len(rows)}",
           "fastest kernel, number of shapes: " + ", ".join(f"{k} {v}" for k, v in sorted(wins.items())),
           f"automatic choice vs measured best: geometric mean {math.exp(sum(map(math.log, loss)) / len(loss)):.4f}x, "
           f"within 5 % on {sum(l <= 1.05 for l in loss)} shapes, worst {max(loss):.2f}x"]
    for l, r in worst:
        out.append(f"  worst: {r['M']}x{r['N']}x{r['K']} auto {r['auto']} {r['us'][r['auto']]:.1f} us, "
                   f"best {r['best']} {r['us'][r['best']]:.1f} us ({l:.2f}x)")
    return "\n".join(out)


def table_from_rows(rows):
    """Exact-shape rules naming the measured winner."""
    return [[r["M"], r["M"], r["N"], r["N"], r["K"], r["K"], r["best"]] for r in rows]


def load_table(q, path):
    with open(path) as f:
        doc = json.load(f)
    q.dispatch_set_rules([tuple(r) for r in doc["rules"]])
    return len(doc["rules"])


def main(argv=None):
    ap = argparse.ArgumentParser(description=__doc__.split("\n")[0])
    ap.add_argument("--shapes", default="", help="comma-separated MxNxK")
    ap.add_argument("--grid", action="store_true", help="the built-in grid of inference-like shapes")
    ap.add_argument("--small-grid", action="store_true",
                    help="the small-batch grid (M 1..64 x N 4..4096 x K 256..4096); also times the automatic choice "
                         "with cold weights and reports its fraction of the 8 TB/s HBM peak")
    ap.add_argument("--conv-grid", action="store_true",
                    help="dense convolution: every kernel id and the automatic choice on the built-in list of layers")
    ap.add_argument("--cold", action="store_true",
                    help="time every kernel with cold weights (launches rotate over more than 1 GB of packed copies): the "
                         "table for a model whose weights do not stay in the memory-side cache between layers")
    ap.add_argument("--out", default="", help="write the dispatch table (JSON) here")
    ap.add_argument("--quiet", action="store_true", help="print only the summary")
    a = ap.parse_args(argv)
    import torch
    from . import qgemm as q
    shapes = [tuple(int(v) for v in s.split("x")) for s in a.shapes.split(",") if s]
    if a.grid:
        shapes += [(M, N, K) for M in GRID_M for N in GRID_N for K in GRID_K if 2.0 * M * N * K <= MAX_OPS]
    if a.small_grid:
        shapes += [(M, N, K) for M in SMALL_M for N in SMALL_N for K in SMALL_K]
    if a.conv_grid:
        rows = tune_conv(q, torch, log=None if a.quiet else (lambda s: print(s, flush=True)))
        print(conv_summary(rows), flush=True)
        if a.out:
            with open(a.out, "w") as f:
                json.dump({"device": torch.cuda.get_device_name(0), "measured": rows}, f, indent=1)
        return 0
    if not shapes:
        ap.error("no shapes given")
    rows = tune(q, torch, shapes, log=None if a.quiet else (lambda s: print(s, flush=True)), cold=a.cold)
    if a.small_grid:
        for r in rows:
            us, ncopy = time_cold(q, torch, r["M"], r["N"], r["K"])
            nbytes = r["M"] * r["K"] + r["K"] * r["N"] + r["M"] * r["N"] + 4 * r["N"]
            r["cold_us"], r["cold_copies"], r["cold_frac_hbm_peak"] = us, ncopy, nbytes / (us * 1e-6) / 8e12
    print(summary(rows), flush=True)
    if a.out:
        with open(a.out, "w") as f:
            json.dump({"device": torch.cuda.get_device_name(0), "rules": table_from_rows(rows), "measured": rows}, f,
                      indent=1)
    return 0


if __name__ == "__main__":
    sys.exit(main())
