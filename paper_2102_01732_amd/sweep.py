"""Single-layer kernel sweep: one n x n Erdos-Renyi layer (n = 262 144), epsilon in {1,4,16,64},
batch in {32,128,512,1024}; times the forward SpMM, the fused backward (transposed SpMM + SDDMM),
the SDDMM alone and one SET evolution, each against the HBM roofline.

    python -m paper_2102_01732_amd.sweep [--n 262144] [--reps 20] [--out profiles/sweep.md]
"""
from __future__ import annotations

import argparse
import json
import time

import torch

from . import binding, workloads as wl

PEAK = 8000.0


def bytes_model(kernel: str, nnz: int, n: int, B: int):
    """(gather-model bytes, compulsory bytes) of one launch: every stored connection fetches its own 4*B-byte
    operand row / every operand moved once."""
    row = 4 * B
    if kernel == "forward_spmm":
        fixed = 8 * nnz + n * (row + B // 4 + 8)
    elif kernel == "backward_fused":
        fixed = 12 * nnz + n * (2 * row + 4)
    else:  # sddmm
        fixed = 8 * nnz + n * (row + 4)
    return fixed + row * nnz, fixed + row * n


def evolve_bytes(nnz: int) -> int:
    """threshold read (4) + compaction (12 read, 12 written) + rebuild of the transposed view (16) per connection"""
    return 44 * nnz


def _layers(n, eps, max_batch):
    spec = wl.sweep_layer(eps, n)
    mk = lambda need: binding.SparseLayer(binding.make_config(
        n, n, nnz=spec.nnz, act_kind=1, act_parity=0, alpha=0.6, init_limit=spec.init_limit, seed=wl.DEFAULT_SEED,
        layer_id=0, max_batch=max_batch, need_input_grad=need))
    return spec, mk(True), mk(False)


def _time_point(spec, full, first, n, eps, B, reps, x, ga, a, gx):
    rows = []
    for layer in (full, first):
        for it in range(3 + reps):
            if it == 3:
                layer.profile_begin()
            layer.forward(x, B, a)
            layer.backward(x, ga, B, gx if layer is full else None)
        prof = layer.profile_end()
        for name in (("forward_spmm", "backward_fused") if layer is full else ("sddmm",)):
            cnt, ms = prof[name]
            t = ms / cnt
            gather, comp = bytes_model(name, spec.nnz, n, B)
            rows.append(dict(eps=eps, B=B, kernel=name, nnz=spec.nnz, ms=t, gather_model_gbs=gather / t / 1e6,
                             gather_model_frac=gather / t / 1e6 / PEAK, compulsory_gbs=comp / t / 1e6,
                             compulsory_frac=comp / t / 1e6 / PEAK))
    return rows


def _time_evolve(spec, full, eps):
    gen, ts = 0, []
    for it in range(1 + 3):
        gen += 1
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        full.evolve(0.3, gen)
        torch.cuda.synchronize()
        ts.append((time.perf_counter() - t0) * 1e3)
    t = sorted(ts[1:])[1]
    b = evolve_bytes(spec.nnz)
    return dict(eps=eps, B=0, kernel="evolve(zeta=0.3)", nnz=spec.nnz, ms=t, mconn_per_s=spec.nnz / t / 1e3,
                model_gbs=b / t / 1e6, model_frac=b / t / 1e6 / PEAK)


def run_points(n: int, reps: int, points, with_evolve: bool = True):
    """Times the (epsilon, B) points given; one evolve row per distinct epsilon."""
    rows = []
    maxB = max(B for _, B in points)
    x = torch.randn((n, maxB), device="cuda")
    ga = torch.randn((n, maxB), device="cuda")
    a = torch.empty((n, maxB), device="cuda")
    gx = torch.empty((n, maxB), device="cuda")
    for eps in sorted({e for e, _ in points}):
        spec, full, first = _layers(n, eps, maxB)
        for e, B in points:
            if e == eps:
                rows += _time_point(spec, full, first, n, eps, B, reps, x, ga, a, gx)
        if with_evolve:
            rows.append(_time_evolve(spec, full, eps))
        full.close()
        first.close()
    return rows


def run(n: int, reps: int, eps_list, batch_list):
    return run_points(n, reps, [(e, B) for e in eps_list for B in batch_list])


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--n", type=int, default=wl.SWEEP_N)
    ap.add_argument("--reps", type=int, default=20)
    ap.add_argument("--eps", type=int, nargs="*", default=list(wl.SWEEP_EPSILON))
    ap.add_argument("--batch", type=int, nargs="*", default=list(wl.SWEEP_BATCH))
    ap.add_argument("--out", default=None)
    args = ap.parse_args()
    rows = run(args.n, args.reps, args.eps, args.batch)
    lines = [f"# single-layer sweep, n_in = n_out = {args.n}, one MI355X, {args.reps} timed repeats (HIP events per kernel)",
             "# command: python -m paper_2102_01732_amd.sweep --out <this file>",
             "# gather-model GB/s = (bytes if each stored connection fetches its own 4*B-byte row) / time;",
             "# compulsory GB/s = (bytes if each operand moves once) / time; fractions are of 8 TB/s.",
             "# evolve (radix select, scans, compaction, sampler, sorts, merge, transposed-view rebuild; host wall clock of",
             "# one call): time, million connections per second, and 44 bytes per connection / time as a fraction of 8 TB/s.",
             "| eps | B | kernel | nnz | ms | gather-model GB/s | frac | compulsory GB/s | frac |", "|---|---|---|---|---|---|---|---|---|"]
    for r in rows:
        if "gather_model_gbs" in r:
            lines.append(f"| {r['eps']} | {r['B']} | {r['kernel']} | {r['nnz']} | {r['ms']:.4f} | {r['gather_model_gbs']:.0f} | "
                         f"{r['gather_model_frac']:.3f} | {r['compulsory_gbs']:.0f} | {r['compulsory_frac']:.3f} |")
        else:
            lines.append(f"| {r['eps']} | - | {r['kernel']} | {r['nnz']} | {r['ms']:.4f} | {r['mconn_per_s']:.0f} Mconn/s | - | "
                         f"{r['model_gbs']:.0f} | {r['model_frac']:.3f} |")
    text = "\n".join(lines) + "\n"
    print(text)
    if args.out:
        open(args.out, "w").write(text)
    print(json.dumps(rows))


if __name__ == "__main__":
    main()
