#!/usr/bin/env python3
"""Benchmark of the truly sparse SET-MLP training hot path on one MI355X.

A "step" is one minibatch through the whole path: forward SpMM + All-ReLU of every layer, softmax
cross-entropy, backward (transposed SpMM + SDDMM) of every layer, momentum-SGD update; after every
`steps_per_epoch` steps the SET prune/regrow evolution of every layer runs inside the timed region.
Inputs are synthetic and already resident in HBM when the clock starts.

Prints ONE JSON line: throughput in samples/s, the HBM roofline of the dominant kernel (measured
live with HIP events on the launch stream) and the CPU oracle timed on this host for context.
"""
import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0


def byte_counts(kernel, spec, B, has_csc):
    """(compulsory_bytes, gather_model_bytes) of one launch.  compulsory: every operand moved once.  gather
    model: every stored connection fetches its own 4*B-byte operand row (no reuse of gathered rows), which is
    what an Erdos-Renyi pattern of density 2e-5 leaves a kernel to work with."""
    nnz, n_in, n_out = spec.nnz, spec.n_in, spec.n_out
    row = 4 * B
    if kernel == "forward_spmm":
        fixed = 8 * nnz + 4 * (n_out + 1) + 4 * n_out + row * n_out + (B // 4) * n_out * (1 if spec.act_kind else 0)
        return fixed + row * n_in, fixed + row * nnz
    if kernel == "backward_fused":
        fixed = 8 * nnz + 4 * (n_in + 1) + 2 * row * n_in + 4 * nnz
        return fixed + row * n_out, fixed + row * nnz
    if kernel == "sddmm":
        fixed = 4 * nnz + 4 * (n_out + 1) + row * n_out + 4 * nnz
        return fixed + row * n_in, fixed + row * nnz
    if kernel == "act_grad":
        b = 2 * row * n_out + (B // 4) * n_out + 4 * n_out
        return b, b
    if kernel == "update":
        b = (28 if has_csc else 20) * nnz + 20 * n_out
        return b, b
    return 0, 0


def evolve_bytes(spec, has_csc):
    """One prune / regrow cycle of a layer: one read of |w| for the threshold (4), compaction of column, weight and
    velocity (12 read + 12 written, survivors and new connections together), and the rebuild of the transposed
    view (16: row index, position, weight and velocity in the other order) per stored connection."""
    return (44 if has_csc else 28) * spec.nnz


def run_small(name, torch, np, binding, wl, dev, with_cpu):
    """One epoch (all minibatches, last one partial) plus one evolution of a small workload."""
    w = wl.WORKLOADS[name]
    B, nb = w.batch, w.steps_per_epoch
    X, y = wl.dataset(w)
    host_blocks = wl.to_batch_blocks(X, B)
    blocks = torch.from_numpy(host_blocks).to(dev)
    ypad = np.zeros(nb * B, np.int32)
    ypad[: y.size] = y
    labels = torch.from_numpy(ypad.reshape(nb, B)).to(dev)
    sizes = [min(B, w.n_samples - k * B) for k in range(nb)]
    net = binding.SparseMLP(w.layers, alpha=w.alpha, lr=w.lr, momentum=w.momentum, seed=w.seed, max_batch=B)
    for k in range(3):
        net.train_step(blocks[k], labels[k], sizes[k])
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for k in range(nb):
        net.train_step(blocks[k], labels[k], sizes[k])
    net.evolve(w.zeta, 1)
    torch.cuda.synchronize()
    dt = time.perf_counter() - t0
    # one step = a forward launch per layer (+ the fix-up of the split output layer), the loss, a backward launch
    # per layer and one update launch: these small networks are bound by the latency between dependent launches
    launches = 2 * len(w.layers) + 3
    # the bytes one step would move if every connection fetched its own operand row (forward, backward, update of
    # every layer); the operands of these networks fit an L2, so this is an upper bound of what crosses the fabric
    step_bytes = 0
    for li, spec in enumerate(w.layers):
        step_bytes += byte_counts("forward_spmm", spec, B, li > 0)[1]
        step_bytes += byte_counts("backward_fused" if li > 0 else "sddmm", spec, B, li > 0)[1]
        step_bytes += byte_counts("update", spec, B, li > 0)[1]
    ms_step = dt / nb * 1e3
    rec = dict(workload=name, dims=list(w.dims), steps=nb, value=w.n_samples / dt, unit="samples/s",
               ms_per_step=ms_step, includes="one epoch + one SET evolution", launches_per_step=launches,
               us_per_launch=dt / nb * 1e6 / launches, bound="latency between dependent kernel launches",
               gather_model_bytes_per_step=step_bytes, gather_model_gbs=step_bytes / ms_step / 1e6,
               gather_model_frac=step_bytes / ms_step / 1e6 / HBM_PEAK_GBS)
    net.close()
    if with_cpu:
        from oracle import oracle as orc
        olayers = [orc.OracleLayer(s.n_in, s.n_out, s.nnz, s.act_kind, s.act_parity, w.alpha, s.init_limit, w.lr,
                                   w.momentum, 0.0, w.seed, s.layer_id) for s in w.layers]
        onet = orc.OracleMLP(olayers)
        ns = min(8, nb)
        cores = orc.set_threads(0)
        c0 = time.perf_counter()
        for k in range(ns):
            onet.train_step(host_blocks[k][:, : sizes[k]], ypad[k * B: k * B + sizes[k]])
        c1 = time.perf_counter()
        rec["cpu_baseline"] = dict(value=sum(sizes[:ns]) / (c1 - c0), unit="samples/s", cores=cores, kind="oracle",
                                   sample=f"first {ns} training steps")
    return rec


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=None)
    ap.add_argument("--warmup", type=int, default=3)
    ap.add_argument("--workload", default="set_mlp_1m")
    ap.add_argument("--profile-steps", type=int, default=8)
    ap.add_argument("--cpu-samples", type=int, default=16, help="samples of the single-thread oracle timing")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-sweep", action="store_true", help="skip the single-layer sweep points")
    ap.add_argument("--extra-workloads", default="set_mlp_madelon,set_mlp_fmnist,set_mlp_cifar",
                    help="comma list of further workloads timed for one epoch each and reported under `other_workloads`")
    ap.add_argument("--evolve-only", type=int, default=0, metavar="N",
                    help="build the network, run N prune/regrow cycles of every layer, print their times and exit "
                         "(the command behind the per-kernel evolve profile)")
    ap.add_argument("--calibrate-copy", action="store_true",
                    help="also run one plain 1 GiB device copy (reference point for rocprofv3 byte counters)")
    args = ap.parse_args()
    if args.gpus != 1 or int(os.environ.get("WORLD_SIZE", "1")) != 1:
        print("bench.py: this build runs on ONE GPU only (no collectives, no sharding); use --gpus 1", file=sys.stderr)
        sys.exit(2)

    import numpy as np
    import torch
    from paper_2102_01732_amd import binding, workloads as wl

    binding.lib()
    assert torch.cuda.is_available(), "bench.py needs a GPU"
    dev = torch.device("cuda:0")
    w = wl.WORKLOADS[args.workload]
    B = w.batch
    K = args.steps if args.steps is not None else w.steps_per_epoch
    n_blocks = w.steps_per_epoch
    n_in = w.dims[0]

    if args.evolve_only > 0:
        net = binding.SparseMLP(w.layers, alpha=w.alpha, lr=w.lr, momentum=w.momentum, seed=w.seed, max_batch=B)
        times, serial = [], []
        for g in range(args.evolve_only):
            torch.cuda.synchronize()
            q0 = time.perf_counter()
            net.evolve(w.zeta, 2 * g + 1)
            torch.cuda.synchronize()
            times.append((time.perf_counter() - q0) * 1e3)
            q0 = time.perf_counter()
            for layer in net.layers:
                layer.evolve(w.zeta, 2 * g + 2)
            torch.cuda.synchronize()
            serial.append((time.perf_counter() - q0) * 1e3)
        print(json.dumps(dict(workload=args.workload, evolve_ms_all_layers=times, evolve_ms_layer_after_layer=serial,
                              connections=sum(s.nnz for s in w.layers))))
        return

    # ---- synthetic data, resident in HBM, feature-major minibatch blocks [n_blocks][n_in][B]
    if w.n_samples * n_in > 2 ** 28:
        gen = torch.Generator(device=dev)
        gen.manual_seed(w.seed)
        blocks = torch.empty((n_blocks, n_in, B), dtype=torch.float32, device=dev)
        h = torch.randn(n_in, generator=gen, device=dev)
        labels = torch.empty((n_blocks, B), dtype=torch.int32, device=dev)
        for k in range(n_blocks):
            blocks[k].normal_(generator=gen)
            labels[k] = (h @ blocks[k] > 0).to(torch.int32)
        sizes = [B] * n_blocks
        data_note = "synthetic N(0,1) features generated on the device, labels from a seeded random hyperplane"
    else:
        X, y = wl.dataset(w)
        blocks = torch.from_numpy(wl.to_batch_blocks(X, B)).to(dev)
        ypad = np.zeros(n_blocks * B, np.int32)
        ypad[: y.size] = y
        labels = torch.from_numpy(ypad.reshape(n_blocks, B)).to(dev)
        sizes = [min(B, w.n_samples - k * B) for k in range(n_blocks)]
        data_note = f"synthetic {w.feature_law} features, labels from a seeded random linear teacher"

    if args.calibrate_copy:
        src = torch.ones(2 ** 28, dtype=torch.float32, device=dev)
        dst = torch.empty_like(src)
        dst.copy_(src)
        torch.cuda.synchronize()
        del src, dst

    net = binding.SparseMLP(w.layers, alpha=w.alpha, lr=w.lr, momentum=w.momentum, seed=w.seed, max_batch=B)
    generation = [0]

    def step(i):
        k = i % n_blocks
        net.train_step(blocks[k], labels[k], sizes[k])
        if (i + 1) % n_blocks == 0:
            generation[0] += 1
            net.evolve(w.zeta, generation[0])

    for i in range(args.warmup):
        net.train_step(blocks[i % n_blocks], labels[i % n_blocks], sizes[i % n_blocks])
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    samples = 0
    for i in range(K):
        step(i)
        samples += sizes[i % n_blocks]
    torch.cuda.synchronize()
    t1 = time.perf_counter()
    elapsed = t1 - t0
    value = samples / elapsed

    # ---- evolution alone (one generation, all layers): time, bytes of the per-connection count above, fraction
    torch.cuda.synchronize()
    te0 = time.perf_counter()
    generation[0] += 1
    net.evolve(w.zeta, generation[0])
    torch.cuda.synchronize()
    evolve_ms = (time.perf_counter() - te0) * 1e3
    generation[0] += 1
    ts0 = time.perf_counter()
    for layer in net.layers:
        layer.evolve(w.zeta, generation[0])
    torch.cuda.synchronize()
    evolve_serial_ms = (time.perf_counter() - ts0) * 1e3
    ev_bytes = sum(evolve_bytes(spec, li > 0) for li, spec in enumerate(w.layers))
    evolve = dict(ms_all_layers=evolve_ms, connections=sum(s.nnz for s in w.layers), model_bytes=ev_bytes,
                  model_gbs=ev_bytes / evolve_ms / 1e6, frac=ev_bytes / evolve_ms / 1e6 / HBM_PEAK_GBS,
                  share_of_an_epoch=evolve_ms / (evolve_ms + n_blocks * elapsed / K * 1e3),
                  ms_layer_after_layer=evolve_serial_ms,
                  note="host wall clock around sparse_layers_evolve (the layers' cycles run concurrently, one stream each), "
                       "synchronisations included; ms_layer_after_layer: one sparse_layer_evolve call per layer instead")

    # ---- per-kernel durations with HIP events on the launch stream
    for layer in net.layers:
        layer.profile_begin()
    P = max(1, args.profile_steps)
    for i in range(P):
        net.train_step(blocks[i % n_blocks], labels[i % n_blocks], sizes[i % n_blocks])
    torch.cuda.synchronize()
    kernels = []
    for li, (layer, spec) in enumerate(zip(net.layers, w.layers)):
        for name, (n, ms) in layer.profile_end().items():
            if name == "update":
                # one launch updates every layer (sparse_layers_update); it is timed on the first layer's handle
                pairs = [byte_counts(name, sp_, B, k > 0) for k, sp_ in enumerate(w.layers)]
                comp, gather = sum(p[0] for p in pairs), sum(p[1] for p in pairs)
                label, where = "update (all layers, one launch)", "all"
            else:
                comp, gather = byte_counts(name, spec, B, li > 0)
                label, where = name, li
            avg_ms = ms / n
            kernels.append(dict(layer=where, kernel=label, launches_per_step=n / P, avg_ms=avg_ms,
                                compulsory_bytes=comp, gather_model_bytes=gather,
                                compulsory_gbs=comp / avg_ms / 1e6 if comp else 0.0,
                                gather_model_gbs=gather / avg_ms / 1e6 if gather else 0.0,
                                compulsory_frac=comp / avg_ms / 1e6 / HBM_PEAK_GBS if comp else 0.0,
                                gather_model_frac=gather / avg_ms / 1e6 / HBM_PEAK_GBS if gather else 0.0))
    kernels.sort(key=lambda r: -r["avg_ms"] * r["launches_per_step"])
    dom = kernels[0]
    traffic = None
    tfile = os.path.join(ROOT, "profiles", "traffic.json")
    if os.path.exists(tfile):
        try:
            t = json.load(open(tfile))
            traffic = t.get(args.workload, {}).get(f"{dom['kernel']}:L{dom['layer']}")
        except Exception:
            traffic = None
    # `achieved` / `frac` count the gather-model bytes (every stored connection fetches its own 4*B-byte operand
    # row); the each-operand-once count and its fraction stand beside them.  `traffic` is NOT measured by this
    # run: it is the rocprofv3 reading of the same kernel and workload kept under profiles/.
    roofline = dict(bound="hbm", bound_note="L2 <-> fabric traffic (the L2 counters cannot separate Infinity Cache hits from HBM)",
                    kernel=dom["kernel"], layer=dom["layer"], achieved=dom["gather_model_gbs"], peak=HBM_PEAK_GBS,
                    unit="GB/s", frac=dom["gather_model_frac"], traffic=traffic,
                    traffic_source="profiles/traffic.json (rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE runs of this command; not measured in this run)",
                    avg_ms=dom["avg_ms"], gather_model_bytes=dom["gather_model_bytes"],
                    compulsory_bytes=dom["compulsory_bytes"], compulsory_achieved=dom["compulsory_gbs"],
                    compulsory_frac=dom["compulsory_frac"])

    # ---- CPU oracle on this host (reported baseline, not the target): one full minibatch at all host cores,
    # and a smaller sample on one thread
    cpu = None
    if not args.no_cpu_baseline:
        from oracle import oracle as orc
        olayers = [orc.OracleLayer(s.n_in, s.n_out, s.nnz, s.act_kind, s.act_parity, w.alpha, s.init_limit, w.lr,
                                   w.momentum, 0.0, w.seed, s.layer_id) for s in w.layers]
        onet = orc.OracleMLP(olayers)
        cores = orc.set_threads(0)
        ns = sizes[0]
        xs = blocks[0][:, :ns].contiguous().cpu().numpy()
        ys = labels[0][:ns].cpu().numpy()
        c0 = time.perf_counter()
        onet.train_step(xs, ys)
        c1 = time.perf_counter()
        n1 = max(1, min(args.cpu_samples, ns))
        orc.set_threads(1)
        d0 = time.perf_counter()
        onet.train_step(np.ascontiguousarray(xs[:, :n1]), ys[:n1])
        d1 = time.perf_counter()
        orc.set_threads(cores)
        e0 = time.perf_counter()
        olayers[0].evolve(w.zeta, 1)
        e1 = time.perf_counter()
        cpu = dict(value=ns / (c1 - c0), unit="samples/s", cores=cores, kind="oracle",
                   sample=f"one training step (forward, loss, backward, update) on minibatch 0 ({ns} samples) at the full "
                          f"layer shapes, rows shared among {cores} threads: {c1 - c0:.1f} s",
                   single_thread=dict(value=n1 / (d1 - d0), unit="samples/s", cores=1,
                                      sample=f"the same step on the first {n1} samples, one thread: {d1 - d0:.1f} s"),
                   evolve_first_layer_s=e1 - e0,
                   evolve_note=f"one prune / regrow cycle of the first layer only ({w.layers[0].nnz} of "
                               f"{sum(s.nnz for s in w.layers)} connections), one thread (sort-based)")

    # ---- forward only (inference): the whole network on every minibatch block, no sign masks kept
    def time_inference(model, xs, b, reps):
        model.infer(xs[0], b, model.acts)
        torch.cuda.synchronize()
        q0 = time.perf_counter()
        for r in range(reps):
            model.infer(xs[r % len(xs)], b, model.acts)
        torch.cuda.synchronize()
        dt = time.perf_counter() - q0
        return dict(batch=b, batches=reps, samples_per_s=reps * b / dt, ms_per_batch=dt / reps * 1e3)

    inference = [time_inference(net, blocks, B, n_blocks)]

    # ---- sparse averaging of two replicas (eq. 2 + magnitude re-pruning) of the first 10^6 x 10^6 layer
    average = None
    if len(net.layers) > 1:
        spec1 = w.layers[1]
        twin = binding.SparseLayer(binding.make_config(
            spec1.n_in, spec1.n_out, nnz=spec1.nnz, act_kind=spec1.act_kind, act_parity=spec1.act_parity, alpha=w.alpha,
            init_limit=spec1.init_limit, lr=w.lr, momentum=w.momentum, seed=w.seed + 1, layer_id=spec1.layer_id,
            max_batch=B, need_input_grad=True), scratch=net.layers[1].scratch)
        torch.cuda.synchronize()
        ta0 = time.perf_counter()
        binding.average_layers(twin, [twin, net.layers[1]])
        torch.cuda.synchronize()
        average = dict(layer=1, replicas=2, ms=(time.perf_counter() - ta0) * 1e3, nnz_after=twin.nnz)
        twin.close()
        del twin
        torch.cuda.empty_cache()

    # ---- Importance Pruning (eq. 4 + Algorithm 2) on the first 10^6 x 10^6 layer: weakest 10 % of the neurons
    L1 = net.layers[1] if len(net.layers) > 1 else net.layers[0]
    torch.cuda.synchronize()
    ti0 = time.perf_counter()
    imp = L1.importance()
    ti1 = time.perf_counter()
    thr = float(np.quantile(imp.astype(np.float64), 0.10))
    removed = L1.importance_prune(thr)
    torch.cuda.synchronize()
    ti2 = time.perf_counter()
    importance = dict(layer=1, importance_ms=(ti1 - ti0) * 1e3, prune_ms=(ti2 - ti1) * 1e3, threshold=thr,
                      removed_connections=removed, nnz_after=L1.nnz)

    # ---- the smaller workloads, one epoch (+ evolution) each, for the record
    others = []
    net.close()
    del net, blocks, labels
    torch.cuda.empty_cache()
    extra = [n for n in args.extra_workloads.split(",") if n in wl.WORKLOADS and n != args.workload]
    if extra:
        # the same network sized for minibatches of 1024 samples (batch tiles of 256 columns in the forward kernel)
        wide = binding.SparseMLP(w.layers, alpha=w.alpha, lr=w.lr, momentum=w.momentum, seed=w.seed, max_batch=1024)
        gen = torch.Generator(device=dev)
        gen.manual_seed(w.seed + 7)
        xs = [torch.randn((n_in, 1024), generator=gen, device=dev) for _ in range(2)]
        inference.append(time_inference(wide, xs, 1024, 16))
        wide.close()
        del wide, xs
        torch.cuda.empty_cache()
    for name in extra:
        others.append(run_small(name, torch, np, binding, wl, dev, not args.no_cpu_baseline))

    # ---- the single-layer sweep (one 262 144 x 262 144 layer): B = 128 at every density and the weakest corners
    sweep = None
    if not args.no_sweep:
        from paper_2102_01732_amd import sweep as sw
        sweep = sw.run_points(wl.SWEEP_N, 10, [(1, 128), (4, 128), (16, 128), (64, 128), (1, 32), (1, 1024), (4, 512), (64, 32)])

    out = dict(metric="sparse-MLP train samples/s", value=value, unit="samples/s", n_gpus=1, steps=K,
               warmup=args.warmup, ms_per_step=elapsed / K * 1e3, higher_is_better=True, scaling="weak",
               vs_baseline=None, dtype="f32", data=data_note,
               config=dict(workload=args.workload, dims=list(w.dims), epsilon=w.epsilon, batch=B,
                           nnz=[s.nnz for s in w.layers], alpha=w.alpha, zeta=w.zeta,
                           evolutions_in_timed_region=K // n_blocks, parallelism="single GPU"),
               roofline=roofline, cpu_baseline=cpu, evolve=evolve, kernels=kernels[:12], sweep=sweep,
               inference=inference, importance_pruning=importance, sparse_average=average, other_workloads=others)
    print(json.dumps(out))


if __name__ == "__main__":
    main()
