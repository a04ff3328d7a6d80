"""Full-size parity: the one-million-neuron workload in exactly the launch configuration that
bench.py times (B = 128, all four layers on one GPU), against digests and sampled values that
tests/golden/make_1m_golden.py computed with the CPU oracle alone.  Topology, indices and fresh
weights are compared bit for bit over ALL entries (sha256); fp32 tensors on sampled neurons and
every 8192nd connection, within 1e-4 of the tensor's largest oracle magnitude after the first step and
within 1e-3 after four and after sixteen steps; after the whole epoch of 128 steps against the distance between
two roundings of the oracle itself (see test_one_million_neuron_whole_epoch).

The last tests run the oracle itself at full size next to the GPU (it shares its rows among the host's cores;
results do not depend on the thread count): four minibatches, each from the ORACLE's state, with every
activation, gradient, weight and velocity of all 5.3 * 10^7 connections compared element by element at 1e-4; then
the prune / regrow cycle of Algorithm 2 from the oracle's TRAINED state (non-zero velocities, trained magnitudes),
in both prune modes, bit for bit over all entries."""
import hashlib
import json
import os

import numpy as np
import pytest

from paper_2102_01732_amd import workloads as wl
from stepwise import make_oracle_net, run_stepwise_oracle_only

pytestmark = pytest.mark.gpu
GOLDEN = os.path.join(os.path.dirname(__file__), "golden", "set_mlp_1m_step.json")


def digest(a):
    return hashlib.sha256(np.ascontiguousarray(a).tobytes()).hexdigest()


def near(got, ref, absmax, tol, what):
    got, ref = np.asarray(got, np.float64), np.asarray(ref, np.float64)
    assert got.shape == ref.shape, what
    err = np.abs(got - ref).max()
    assert np.all(np.isfinite(got)) and err <= tol * absmax, f"{what}: max abs err {err:.3e} > {tol} * {absmax:.3e}"


@pytest.fixture(scope="module")
def setup():
    import torch
    if not torch.cuda.is_available():
        pytest.skip("no GPU")
    from paper_2102_01732_amd import binding
    binding.lib()
    return binding, json.load(open(GOLDEN)), wl.WORKLOADS["set_mlp_1m"]


def make_net(binding, w):
    return binding.SparseMLP(w.layers, alpha=w.alpha, lr=w.lr, momentum=w.momentum, seed=w.seed, max_batch=w.batch)


def test_one_million_neuron_init_and_evolution_bit_exact(setup):
    binding, golden, w = setup
    net = make_net(binding, w)
    for li, (G, g) in enumerate(zip(net.layers, golden["layers"])):
        rowptr, colidx, val, vel, bias, _ = G.export_csr()
        assert G.nnz == w.layers[li].nnz
        assert digest(rowptr) == g["init"]["rowptr"], f"layer {li} rowptr"
        assert digest(colidx) == g["init"]["colidx"], f"layer {li} colidx"
        assert digest(val) == g["init"]["val"], f"layer {li} val"
        assert not vel.any() and not bias.any()
    net.evolve(w.zeta, 1)
    for li, (G, g) in enumerate(zip(net.layers, golden["layers"])):
        rowptr, colidx, val, vel, _, _ = G.export_csr()
        assert G.nnz == w.layers[li].nnz
        assert int((vel == 0).sum()) == w.layers[li].nnz          # zero velocities everywhere (fresh network)
        assert digest(rowptr) == g["evolved"]["rowptr"], f"layer {li} rowptr after evolution"
        assert digest(colidx) == g["evolved"]["colidx"], f"layer {li} colidx after evolution"
        assert digest(val) == g["evolved"]["val"], f"layer {li} val after evolution"
        assert digest(vel) == g["evolved"]["vel"]
    net.close()


def test_one_million_neuron_training_step(setup):
    import torch
    binding, golden, w = setup
    B = w.batch
    X, y = wl.dataset(w, B)
    x0 = torch.from_numpy(wl.to_batch_blocks(X, B)[0]).cuda()
    yd = torch.from_numpy(y).cuda()
    net = make_net(binding, w)
    zL = net.forward(x0, B)
    binding.softmax_ce(zL, yd, B, net.n_classes, net.grad_out, net.loss_sum)
    net.backward(x0, B)
    stride = golden["val_stride"]
    grads = [G.export_grad() for G in net.layers]
    for G in net.layers:
        G.update()
    torch.cuda.synchronize()
    loss = net.loss_sum.item() / B
    assert abs(loss - golden["loss_mean"]) <= 1e-4 * abs(golden["loss_mean"])
    for li, (G, g) in enumerate(zip(net.layers, golden["layers"])):
        s = g["step"]
        rows = torch.tensor(s["rows"], device="cuda")
        act = net.acts[li][rows][:, :B].cpu().numpy()
        near(act, s["act"], s["act_absmax"], 1e-4, f"layer {li} activations")
        idx = np.arange(0, G.nnz, stride)
        near(grads[li][0][idx], s["grad_val"], s["grad_val_absmax"], 1e-4, f"layer {li} weight gradient")
        _, _, val, vel, bias, _ = G.export_csr()
        near(val[idx], s["val"], np.abs(s["val"]).max(), 1e-4, f"layer {li} weights")
        near(vel[idx], s["vel"], s["vel_absmax"], 1e-4, f"layer {li} velocities")
        near(bias[np.asarray(s["rows"])], s["bias"], s["bias_absmax"], 1e-4, f"layer {li} biases")
    net.close()


def test_one_million_neuron_four_training_steps(setup):
    """Four steps of the training loop that bench.py times (fused loss, chained backward, one update launch for
    all layers) on minibatches 0..3, against the oracle's state after the same four steps."""
    import torch
    binding, golden, w = setup
    after = golden["after_steps"]
    steps, B = after["steps"], w.batch
    X, y = wl.dataset(w, steps * B)
    blocks = torch.from_numpy(wl.to_batch_blocks(X, B)).cuda()
    yd = torch.from_numpy(y).cuda()
    net = make_net(binding, w)
    losses = []
    for k in range(steps):
        net.loss_sum.zero_()
        net.train_step(blocks[k], yd[k * B:(k + 1) * B], B)
        losses.append(net.loss_sum.item() / B)
    for k, (got, ref) in enumerate(zip(losses, after["loss_means"])):
        assert abs(got - ref) <= 1e-3 * abs(ref), f"loss of step {k + 1}: {got} vs {ref}"
    stride = golden["val_stride"]
    for li, (G, g, s1) in enumerate(zip(net.layers, after["layers"], golden["layers"])):
        idx = np.arange(0, G.nnz, stride)
        _, _, val, vel, bias, _ = G.export_csr()
        near(val[idx], g["val"], g["val_absmax"], 1e-3, f"layer {li} weights after {steps} steps")
        near(vel[idx], g["vel"], g["vel_absmax"], 1e-3, f"layer {li} velocities after {steps} steps")
        near(bias[np.asarray(s1["step"]["rows"])], g["bias"], g["bias_absmax"], 1e-3, f"layer {li} biases after {steps} steps")
    net.close()


def steps_against_the_golden_state(setup, key, strict=True):
    """The GPU trains on its own for the steps of golden block `key`; strict: every minibatch loss and every sampled
    weight, velocity and bias within 1e-3.  Returns the losses and, per layer and tensor, (largest error / largest
    magnitude, normwise error) against the block's values."""
    import torch
    binding, golden, w = setup
    if key not in golden:
        pytest.skip(f"tests/golden/set_mlp_1m_step.json has no {key!r} block (re-run make_1m_golden.py)")
    after = golden[key]
    steps, B = after["steps"], w.batch
    X, y = wl.dataset(w, steps * B)
    blocks = torch.from_numpy(wl.to_batch_blocks(X, B)).cuda()
    yd = torch.from_numpy(y).cuda()
    net = make_net(binding, w)
    losses = []
    for k in range(steps):
        net.loss_sum.zero_()
        net.train_step(blocks[k], yd[k * B:(k + 1) * B], B)
        losses.append(net.loss_sum.item() / B)
    rel = [abs(got - ref) / abs(ref) for got, ref in zip(losses, after["loss_means"])]
    print(f"{steps} steps: largest relative difference of a minibatch loss {max(rel):.3e} (step {int(np.argmax(rel)) + 1}), "
          f"of the mean loss {abs(np.mean(losses) - np.mean(after['loss_means'])) / np.mean(after['loss_means']):.3e}", flush=True)
    if strict:
        for k, (got, ref) in enumerate(zip(losses, after["loss_means"])):
            assert abs(got - ref) <= 1e-3 * abs(ref), f"loss of step {k + 1}: {got} vs {ref}"
    stride = golden["val_stride"]
    dist = {}
    for li, (G, g, s1) in enumerate(zip(net.layers, after["layers"], golden["layers"])):
        idx = np.arange(0, G.nnz, stride)
        _, _, val, vel, bias, _ = G.export_csr()
        for what, got, ref, scale in (("val", val[idx], g["val"], g["val_absmax"]), ("vel", vel[idx], g["vel"], g["vel_absmax"]),
                                      ("bias", bias[np.asarray(s1["step"]["rows"])], g["bias"], g["bias_absmax"])):
            d = np.abs(np.asarray(got, np.float64) - np.asarray(ref, np.float64))
            dist[(li, what)] = (d.max() / scale, np.linalg.norm(d) / max(np.linalg.norm(np.asarray(ref, np.float64)), 1e-300))
            print(f"layer {li} {what}: largest error / largest magnitude = {dist[(li, what)][0]:.3e}, normwise "
                  f"{dist[(li, what)][1]:.3e}", flush=True)
            if strict:
                near(got, ref, scale, 1e-3, f"layer {li} {what} after {steps} steps")
    net.close()
    return losses, dist


def test_one_million_neuron_sixteen_training_steps(setup):
    """Sixteen steps of the loop that bench.py times, against the oracle's state after the same sixteen steps."""
    steps_against_the_golden_state(setup, "after_more_steps")


def test_one_million_neuron_whole_epoch(setup):
    """All 128 minibatches of the epoch that bench.py times, the GPU training on its own, against the oracle's own
    epoch.  This workload does not damp differences: its loss climbs from 0.85 into the thousands, and the ORACLE
    ITSELF, restarted from initial weights of which half were moved by one unit in the last place, ends the epoch
    4-5 % away from its first run in the velocities, 3e-4 .. 9e-4 in the weights and up to 1.1 % in single
    minibatch losses (block "after_epoch_perturbed" of the golden file, written by the oracle alone).  A 1e-3
    bound on every tensor after the epoch is therefore not a property that any second evaluation of the method
    has here; what is asserted is that the GPU is no farther from the oracle than that second rounding of the
    oracle is (twice its normwise distance, per tensor), that the first 64 minibatch losses agree to 1e-3 and all
    of them to twice the perturbed run's largest difference, and that the epoch's mean loss agrees to 1e-3."""
    binding, golden, w = setup
    if "after_epoch_perturbed" not in golden:
        pytest.skip("tests/golden/set_mlp_1m_step.json has no 'after_epoch_perturbed' block (make_1m_golden.py --perturbed)")
    ref, other = golden["after_epoch"], golden["after_epoch_perturbed"]
    losses, dist = steps_against_the_golden_state(setup, "after_epoch", strict=False)
    l_ref, l_other = np.asarray(ref["loss_means"]), np.asarray(other["loss_means"])
    rel = np.abs(np.asarray(losses) - l_ref) / np.abs(l_ref)
    rel_other = np.abs(l_other - l_ref) / np.abs(l_ref)
    assert rel[:64].max() <= 1e-3, f"loss of step {int(rel[:64].argmax()) + 1} differs by {rel[:64].max():.3e}"
    assert rel.max() <= 2 * rel_other.max(), (rel.max(), rel_other.max())
    assert abs(np.mean(losses) - l_ref.mean()) <= 1e-3 * l_ref.mean()
    for li, (a, b) in enumerate(zip(ref["layers"], other["layers"])):
        for what in ("val", "vel", "bias"):
            r, q = np.asarray(a[what]), np.asarray(b[what])
            own = np.linalg.norm(r - q) / np.linalg.norm(r)      # the oracle against its perturbed self
            print(f"layer {li} {what}: GPU - oracle {dist[(li, what)][1]:.3e}, perturbed oracle - oracle {own:.3e}", flush=True)
            assert dist[(li, what)][1] <= 2 * own + 1e-4, f"layer {li} {what}: {dist[(li, what)][1]:.3e} vs {own:.3e}"


LIVE_STEPS = 4
_live = {}


def live_state(setup, oracle):
    """The oracle's one-million-neuron network and the GPU network that follows it (built once per session)."""
    if not _live:
        binding, _, w = setup
        print("oracle: initialising 5.3e7 connections ...", flush=True)
        _live["oracle_net"] = make_oracle_net(oracle, w)
        _live["net"] = make_net(binding, w)
        _live["done"] = 0
    return _live


@pytest.mark.parametrize("step", range(LIVE_STEPS))
def test_one_million_neuron_minibatch_from_the_oracles_state(setup, oracle, step):
    binding, _, w = setup
    st = live_state(setup, oracle)
    if st["done"] > step:
        pytest.skip("already covered")
    _, _, _, stats = run_stepwise_oracle_only(binding, oracle, w, step + 1, net=st["net"], oracle_net=st["oracle_net"],
                                              first_step=st["done"], oracle_logits=True)
    st["done"] = step + 1
    for t in stats["tally"]:
        assert t["needed"] <= 1e-3 * t["checked"], stats


@pytest.mark.parametrize("mode", [0, 1])
def test_one_million_neuron_evolution_of_the_trained_network(setup, oracle, mode):
    """Algorithm 2's prune / regrow cycle applied to the oracle's state after LIVE_STEPS training steps, on both
    sides; every array of every layer must come out identical."""
    binding, _, w = setup
    st = live_state(setup, oracle)
    if st["done"] < LIVE_STEPS:       # run alone: train the oracle first (no comparison needed here)
        X, y = wl.dataset(w, LIVE_STEPS * w.batch)
        blocks = wl.to_batch_blocks(X, w.batch)
        for k in range(st["done"], LIVE_STEPS):
            st["oracle_net"][0].train_step(blocks[k], y[k * w.batch:(k + 1) * w.batch])
        st["done"] = LIVE_STEPS
    onet, olayers = st["oracle_net"]
    net = binding.SparseMLP(w.layers, alpha=w.alpha, lr=w.lr, momentum=w.momentum, seed=w.seed, max_batch=w.batch,
                            prune_mode=mode)
    for li, (G, O) in enumerate(zip(net.layers, olayers)):
        assert np.count_nonzero(O.vel) > 0.9 * O.nnz
        G.import_csr(O.rowptr, O.colidx, O.val, O.vel, O.bias, O.bias_vel)
        E = oracle.OracleLayer.__new__(oracle.OracleLayer)
        E.__dict__.update(O.__dict__)
        E.set_state(O.rowptr, O.colidx, O.val, O.vel, O.bias, O.bias_vel)
        E.prune_mode = mode
        print(f"mode {mode} layer {li}: oracle evolve ...", flush=True)
        k = E.evolve(w.zeta, 1)
        G.evolve(w.zeta, 1)
        rowptr, colidx, val, vel, _, _ = G.export_csr()
        assert G.nnz == O.nnz and abs(k - w.zeta * O.nnz) <= 1
        assert np.array_equal(rowptr, E.rowptr) and np.array_equal(colidx, E.colidx), f"layer {li} pattern"
        assert np.array_equal(val.view(np.uint32), E.val.view(np.uint32)), f"layer {li} weights"
        assert np.array_equal(vel.view(np.uint32), E.vel.view(np.uint32)), f"layer {li} velocities"
    net.close()
