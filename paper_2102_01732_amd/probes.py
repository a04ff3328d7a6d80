"""Re-runnable measurements behind design decisions (one MI355X).  Each probe times two ways of doing the same
work through the library's public entry points and prints a table; none of them is on the product path.

    python -m paper_2102_01732_amd.probes [stream] [fused_update] [batch_tiling] [row_balance] [graph] [--out FILE]

stream        what plain streaming kernels (torch copy and add) reach at the byte volumes of the small sweep points:
              the ceiling a short kernel with a third of its traffic in writes can be held against
fused_update  eq. (1) inside the backward kernels (sparse_layer_set_fused_update mode 1) against the separate update
              launch, on the 10^6-neuron network
batch_tiling  one forward pass over 128 batch columns against four passes over 32 columns each (a quarter of the
              operand per pass), on a 10^6 x 10^6 layer
row_balance   an Erdos-Renyi layer against a layer with the same number of connections in which every row and every
              column has exactly the same length: what perfectly balanced rows would buy
graph         a training step of the FashionMNIST-shaped network replayed from a captured HIP graph against eager
              launches
"""
from __future__ import annotations

import argparse
import time

import numpy as np
import torch

from . import binding, workloads as wl


def _time(fn, reps=20, warm=3):
    for _ in range(warm):
        fn()
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(reps):
        fn()
    torch.cuda.synchronize()
    return (time.perf_counter() - t0) / reps * 1e3


def _kernel_ms(layer, fn, reps=10):
    for _ in range(3):
        fn()
    layer.profile_begin()
    for _ in range(reps):
        fn()
    return {k: ms / n for k, (n, ms) in layer.profile_end().items()}


def probe_stream():
    rows = ["| bytes moved | kernel | ms | GB/s |", "|---|---|---|---|"]
    for mb in (32, 128, 512):
        n = mb * 2 ** 20 // 4
        a, b, c = (torch.randn(n, device="cuda") for _ in range(3))
        ev0, ev1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        for name, fn, moved in (("copy (1 read, 1 write)", lambda: c.copy_(a), 2 * 4 * n),
                                ("add (2 reads, 1 write)", lambda: torch.add(a, b, out=c), 3 * 4 * n)):
            for _ in range(5):
                fn()
            ts = []
            for _ in range(20):
                ev0.record()
                fn()
                ev1.record()
                ev1.synchronize()
                ts.append(ev0.elapsed_time(ev1))
            t = sorted(ts)[len(ts) // 2]
            rows.append(f"| {moved / 1e6:.0f} MB | {name}, {mb} MB arrays | {t:.4f} | {moved / t / 1e6:.0f} |")
    return "## stream: plain streaming kernels (torch), median of 20 event-timed launches\n" + "\n".join(rows)


def probe_fused_update():
    w = wl.WORKLOADS["set_mlp_1m"]
    B = w.batch
    net = binding.SparseMLP(w.layers, alpha=w.alpha, lr=w.lr, momentum=w.momentum, seed=w.seed, max_batch=B)
    x = torch.randn((w.dims[0], B), device="cuda")
    y = torch.randint(0, 2, (B,), device="cuda", dtype=torch.int32)
    rows = ["| update | ms per step | fused backward of a 10^6 x 10^6 layer, ms | update launch, ms |", "|---|---|---|---|"]
    for mode, name in ((0, "separate launch for all layers"), (1, "inside the backward kernels")):
        net.fused_update = mode
        step = lambda: net.train_step(x, y, B)
        ms = _time(step, reps=20)
        for layer in net.layers:
            layer.profile_begin()
        for _ in range(5):
            step()
        prof = [layer.profile_end() for layer in net.layers]
        bwd = prof[1]["backward_fused"][1] / prof[1]["backward_fused"][0]
        upd = prof[0]["update"][1] / prof[0]["update"][0]
        rows.append(f"| {name} | {ms:.3f} | {bwd:.3f} | {upd:.3f} |")
    net.close()
    return "## fused_update: set_mlp_1m, B = 128, 20 steps\n" + "\n".join(rows)


def probe_batch_tiling():
    n, nnz, B = 1000000, 20000000, 128
    L = binding.SparseLayer(binding.make_config(n, n, nnz=nnz, act_kind=1, act_parity=0, alpha=0.6, init_limit=0.5,
                                                seed=wl.DEFAULT_SEED, layer_id=1, max_batch=B, need_input_grad=False))
    x = torch.randn((n, B), device="cuda")
    a = torch.empty((n, B), device="cuda")
    one = _time(lambda: L.infer(x, B, a))

    def tiled():
        for t in range(4):
            L.infer(x[:, 32 * t:32 * t + 32], 32, a[:, 32 * t:32 * t + 32])

    four = _time(tiled)
    L.close()
    return ("## batch_tiling: forward of a 10^6 x 10^6 layer (2e7 connections), 128 batch columns\n"
            "| traversal | ms |\n|---|---|\n"
            f"| one pass, rows of 512 bytes gathered from a 512 MB operand | {one:.3f} |\n"
            f"| four passes of 32 columns (rows of 128 bytes, stride 512; the connections are read four times) | {four:.3f} |")


def _regular_pattern(n, per_row, seed):
    """Every row and every column holds exactly per_row entries: row r connects to (r + off_k) mod n for per_row
    distinct random offsets."""
    rng = np.random.Generator(np.random.PCG64(seed))
    off = np.sort(rng.choice(n, size=per_row, replace=False)).astype(np.int64)
    cols = (np.arange(n, dtype=np.int64)[:, None] + off[None, :]) % n
    cols.sort(axis=1)
    rowptr = (np.arange(n + 1, dtype=np.int64) * per_row).astype(np.int32)
    return rowptr, cols.reshape(-1).astype(np.int32)


def probe_row_balance():
    n, eps = wl.SWEEP_N, 16
    spec = wl.sweep_layer(eps)
    rows = ["| B | pattern | forward ms | fused backward ms |", "|---|---|---|---|"]
    for B in (32, 128):
        x = torch.randn((n, B), device="cuda")
        ga = torch.randn((n, B), device="cuda")
        a, gx = torch.empty((n, B), device="cuda"), torch.empty((n, B), device="cuda")
        for regular in (False, True):
            L = binding.SparseLayer(binding.make_config(n, n, nnz=spec.nnz, act_kind=1, act_parity=0, alpha=0.6,
                                                        init_limit=spec.init_limit, seed=wl.DEFAULT_SEED, layer_id=0,
                                                        max_batch=B, need_input_grad=True))
            if regular:
                rowptr, colidx = _regular_pattern(n, spec.nnz // n, 3)
                L.import_csr(rowptr, colidx, L.export_csr()[2])

            def fb():
                L.forward(x, B, a)
                L.backward(x, ga, B, gx)

            k = _kernel_ms(L, fb)
            rows.append(f"| {B} | {'every row and column of length %d' % (spec.nnz // n) if regular else 'Erdos-Renyi'} | "
                        f"{k['forward_spmm']:.4f} | {k['backward_fused']:.4f} |")
            L.close()
    return f"## row_balance: one {n} x {n} layer, {spec.nnz} connections\n" + "\n".join(rows)


def probe_graph():
    w = wl.WORKLOADS["set_mlp_fmnist"]
    B = w.batch
    X, y = wl.dataset(w, B)
    x = torch.from_numpy(wl.to_batch_blocks(X, B)[0]).cuda()
    yd = torch.from_numpy(y).cuda()
    net = binding.SparseMLP(w.layers, alpha=w.alpha, lr=w.lr, momentum=w.momentum, seed=w.seed, max_batch=B)
    eager = _time(lambda: net.train_step(x, yd, B), reps=200, warm=20)
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):
        net.train_step(x, yd, B)
    torch.cuda.current_stream().wait_stream(side)
    torch.cuda.synchronize()
    g = torch.cuda.CUDAGraph()
    with torch.cuda.graph(g):
        net.train_step(x, yd, B)
    replay = _time(g.replay, reps=200, warm=20)
    net.close()
    return ("## graph: one training step of set_mlp_fmnist (11 kernel launches), B = 128\n| launch | ms per step |\n|---|---|\n"
            f"| eager | {eager:.4f} |\n| replay of a captured HIP graph | {replay:.4f} |")


PROBES = dict(stream=probe_stream, fused_update=probe_fused_update, batch_tiling=probe_batch_tiling,
              row_balance=probe_row_balance, graph=probe_graph)


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("probes", nargs="*", default=list(PROBES))
    ap.add_argument("--out", default=None)
    args = ap.parse_args()
    binding.lib()
    parts = ["# design probes on one MI355X\n# command: python -m paper_2102_01732_amd.probes " + " ".join(args.probes)]
    for name in args.probes:
        print(f"probe {name} ...", flush=True)
        parts.append(PROBES[name]())
        print(parts[-1], flush=True)
    if args.out:
        open(args.out, "w").write("\n\n".join(parts) + "\n")


if __name__ == "__main__":
    main()
