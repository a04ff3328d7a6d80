"""Writes tests/golden/set_mlp_1m_step.json: digests and sampled values of ONE evolution, of the
first training step and of the states after FOUR, after SIXTEEN and after all 128 training steps of
an epoch of the one-million-neuron workload, computed by the CPU oracle alone (about an hour on
eight cores).  Nothing from the GPU path is read or stored.

    python tests/golden/make_1m_golden.py
    python tests/golden/make_1m_golden.py --perturbed    # adds "after_epoch_perturbed" to the stored file (another hour)

--perturbed repeats the epoch with the oracle alone from initial weights of which a seeded random half was moved by
one unit in the last place, and stores the same samples: how far two evaluations of the method that differ only
by rounding are apart after 128 minibatches of this workload.
"""
import hashlib
import json
import os
import sys
import time

import numpy as np

ROOT = os.path.dirname(os.path.dirname(os.path.dirname(os.path.abspath(__file__))))
sys.path.insert(0, ROOT)
from oracle import oracle as orc                       # noqa: E402
from paper_2102_01732_amd import workloads as wl      # noqa: E402

ROW_SAMPLES = 48       # sampled neurons per layer (full batch rows are stored)
VAL_STRIDE = 8192      # every VAL_STRIDE-th stored connection
STEPS = 4              # training steps (minibatches 0..3) behind the "after_steps" values
MORE_STEPS = 16        # ... and behind the "after_more_steps" values
EPOCH_STEPS = 128      # ... and behind the "after_epoch" values (the whole epoch of the workload)


def digest(a):
    return hashlib.sha256(np.ascontiguousarray(a).tobytes()).hexdigest()


def sample_rows(n, layer_id):
    rng = np.random.Generator(np.random.PCG64(1000 + layer_id))
    return np.sort(rng.choice(n, size=min(ROW_SAMPLES, n), replace=False))


def main():
    w = wl.WORKLOADS["set_mlp_1m"]
    t0 = time.time()
    X, y = wl.dataset(w, EPOCH_STEPS * w.batch)
    blocks = wl.to_batch_blocks(X, w.batch)
    x0, y_all, y = blocks[0], y, y[: w.batch]
    layers = [orc.OracleLayer(s.n_in, s.n_out, s.nnz, s.act_kind, s.act_parity, w.alpha, s.init_limit, w.lr,
                              w.momentum, 0.0, w.seed, s.layer_id) for s in w.layers]
    print("init", time.time() - t0, flush=True)
    out = {"workload": w.name, "row_samples": ROW_SAMPLES, "val_stride": VAL_STRIDE, "layers": []}
    for L in layers:
        out["layers"].append({"init": {"rowptr": digest(L.rowptr), "colidx": digest(L.colidx), "val": digest(L.val)}})
    # one evolution straight from the initial state (identical bits on both sides), on copies
    for li, L in enumerate(layers):
        E = orc.OracleLayer.__new__(orc.OracleLayer)
        E.__dict__.update(L.__dict__)
        E.set_state(L.rowptr, L.colidx, L.val, L.vel, L.bias, L.bias_vel)
        k = E.evolve(w.zeta, 1)
        out["layers"][li]["evolved"] = {"k": k, "rowptr": digest(E.rowptr), "colidx": digest(E.colidx),
                                        "val": digest(E.val), "vel": digest(E.vel)}
        print("evolve", li, time.time() - t0, flush=True)
    # one training step from the initial state
    net = orc.OracleMLP(layers)
    loss = net.train_step(x0, y)
    print("step", time.time() - t0, flush=True)
    out["loss_mean"] = loss
    for li, L in enumerate(layers):
        rows = sample_rows(L.n_out, li)
        idx = np.arange(0, L.nnz, VAL_STRIDE)
        out["layers"][li]["step"] = {
            "rows": rows.tolist(),
            "act": net.acts[li + 1][rows].astype(np.float64).round(9).tolist(),
            "act_absmax": float(np.abs(net.acts[li + 1]).max()),
            "grad_val": L.grad_val[idx].astype(np.float64).tolist(),
            "grad_val_absmax": float(np.abs(L.grad_val).max()),
            "val": L.val[idx].astype(np.float64).tolist(),
            "vel": L.vel[idx].astype(np.float64).tolist(),
            "vel_absmax": float(np.abs(L.vel).max()),
            "bias": L.bias[rows].astype(np.float64).tolist(),
            "bias_absmax": float(np.abs(L.bias).max()),
        }
    # more steps on the next minibatches; the states after the fourth and the sixteenth are sampled the same way
    losses = [loss]

    def sampled_state():
        rec = []
        for li, L in enumerate(layers):
            rows = sample_rows(L.n_out, li)
            idx = np.arange(0, L.nnz, VAL_STRIDE)
            rec.append({
                "val": L.val[idx].astype(np.float64).tolist(), "val_absmax": float(np.abs(L.val).max()),
                "vel": L.vel[idx].astype(np.float64).tolist(), "vel_absmax": float(np.abs(L.vel).max()),
                "bias": L.bias[rows].astype(np.float64).tolist(), "bias_absmax": float(np.abs(L.bias).max()),
            })
        return rec

    for k in range(1, EPOCH_STEPS):
        losses.append(net.train_step(blocks[k], y_all[k * w.batch:(k + 1) * w.batch]))
        print("step", k + 1, time.time() - t0, flush=True)
        if k + 1 == STEPS:
            out["after_steps"] = {"steps": STEPS, "loss_means": list(losses), "layers": sampled_state()}
        if k + 1 == MORE_STEPS:
            out["after_more_steps"] = {"steps": MORE_STEPS, "loss_means": list(losses), "layers": sampled_state()}
    out["after_epoch"] = {"steps": EPOCH_STEPS, "loss_means": list(losses), "layers": sampled_state()}
    path = os.path.join(os.path.dirname(os.path.abspath(__file__)), os.environ.get("GOLDEN_OUT", "set_mlp_1m_step.json"))
    json.dump(out, open(path, "w"))
    print("wrote", path, os.path.getsize(path), "bytes in", time.time() - t0, "s")


def perturbed():
    w = wl.WORKLOADS["set_mlp_1m"]
    t0 = time.time()
    X, y = wl.dataset(w, EPOCH_STEPS * w.batch)
    blocks = wl.to_batch_blocks(X, w.batch)
    layers = [orc.OracleLayer(s.n_in, s.n_out, s.nnz, s.act_kind, s.act_parity, w.alpha, s.init_limit, w.lr,
                              w.momentum, 0.0, w.seed, s.layer_id) for s in w.layers]
    rng = np.random.Generator(np.random.PCG64(20210201))
    for L in layers:                       # one unit in the last place, up, on a random half of the weights
        val = L.val.copy()
        pick = rng.random(L.nnz) < 0.5
        val[pick] = np.nextafter(val[pick], np.float32(np.inf))
        L.set_state(L.rowptr, L.colidx, val, L.vel, L.bias, L.bias_vel)
    net = orc.OracleMLP(layers)
    losses = []
    for k in range(EPOCH_STEPS):
        losses.append(net.train_step(blocks[k], y[k * w.batch:(k + 1) * w.batch]))
        print("perturbed step", k + 1, time.time() - t0, flush=True)
    rec = []
    for li, L in enumerate(layers):
        rows = sample_rows(L.n_out, li)
        idx = np.arange(0, L.nnz, VAL_STRIDE)
        rec.append({"val": L.val[idx].astype(np.float64).tolist(), "vel": L.vel[idx].astype(np.float64).tolist(),
                    "bias": L.bias[rows].astype(np.float64).tolist()})
    path = os.path.join(os.path.dirname(os.path.abspath(__file__)), "set_mlp_1m_step.json")
    out = json.load(open(path))
    out["after_epoch_perturbed"] = {"steps": EPOCH_STEPS, "loss_means": losses, "layers": rec,
                                    "perturbation": "a seeded random half of the initial weights of every layer moved up by one unit in the last place"}
    json.dump(out, open(path, "w"))
    print("added after_epoch_perturbed to", path, "in", time.time() - t0, "s")


if __name__ == "__main__":
    if "--perturbed" in sys.argv[1:]:
        perturbed()
    else:
        main()
