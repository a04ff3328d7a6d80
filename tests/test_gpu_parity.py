"""GPU parity: the HIP path (through the C ABI) against the CPU oracle, element by element, on
the same seeded inputs.  Topology, indices and counts must be bit-exact; fp32 tensors must agree
within relative 1e-4 after one step and 1e-3 after an epoch (normwise, and max-abs relative to the
largest oracle magnitude)."""
import os

import numpy as np
import pytest
import scipy.sparse as sp

from paper_2102_01732_amd import workloads as wl
from parity_util import abs_backward, abs_forward, close

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def gpu():
    import torch
    if not torch.cuda.is_available():
        pytest.skip("no GPU")
    from paper_2102_01732_amd import binding
    binding.lib()
    return binding


def dev(t, arr):
    return t.from_numpy(np.ascontiguousarray(arr)).to("cuda:0")


def pad_cols(arr, ld):
    out = np.full((arr.shape[0], ld), np.nan, dtype=np.float32)   # padding must never be read as data
    out[:, : arr.shape[1]] = arr
    return out


def make_pair(gpu, oracle, n_in, n_out, nnz, *, act_kind=1, parity=0, alpha=0.6, limit=0.3, seed=11, layer_id=2,
              max_batch=128, prune_mode=0, need_input_grad=True, lr=0.01, mu=0.9):
    cfg = gpu.make_config(n_in, n_out, nnz=nnz, act_kind=act_kind, act_parity=parity, alpha=alpha, init_limit=limit,
                          lr=lr, momentum=mu, seed=seed, layer_id=layer_id, max_batch=max_batch,
                          prune_mode=prune_mode, need_input_grad=need_input_grad)
    G = gpu.SparseLayer(cfg)
    O = oracle.OracleLayer(n_in, n_out, nnz, act_kind, parity, alpha, limit, lr, mu, 0.0, seed, layer_id, prune_mode)
    return G, O


def assert_same_topology(G, O, values=True):
    rowptr, colidx, val, vel, bias, bias_vel = G.export_csr()
    assert np.array_equal(rowptr, O.rowptr)
    assert np.array_equal(colidx, O.colidx)
    if values:
        assert np.array_equal(val.view(np.uint32), O.val.view(np.uint32))
        assert np.array_equal(vel.view(np.uint32), O.vel.view(np.uint32))


# ------------------------------------------------------------------------------------------ init
@pytest.mark.parametrize("n_in,n_out,nnz", [
    (500, 400, 9000), (400, 100, 5000),      # sparse sampler mode
    (400, 2, 800), (1000, 10, 10000),        # fully dense output layers (dense sampler mode)
    (64, 48, 1000),                          # dense mode, not full
    (3000, 5000, 37), (7, 5, 0), (1, 1, 1),  # nearly empty / empty / single
    (100000, 70000, 1700000)])               # several sort tiles, 64-bit flat positions > 2^32
def test_init_topology_bit_exact(gpu, oracle, n_in, n_out, nnz):
    G, O = make_pair(gpu, oracle, n_in, n_out, nnz)
    assert G.nnz == nnz == O.nnz
    assert_same_topology(G, O)
    rowptr, colidx, val, vel, bias, bias_vel = G.export_csr()
    assert np.all(vel == 0) and np.all(bias == 0) and np.all(bias_vel == 0)
    G.close()


# ------------------------------------------------------------------------------------------ one layer, one step
@pytest.mark.parametrize("n_in,n_out,nnz,B,max_batch,act_kind,parity,need_gx", [
    (500, 400, 9000, 128, 128, 1, 0, True),
    (500, 400, 9000, 128, 128, 1, 1, False),
    (300, 700, 6000, 96, 128, 1, 0, True),        # partial last minibatch
    (300, 700, 6000, 5, 128, 1, 1, True),         # ragged: not a multiple of 4
    (300, 700, 6000, 31, 32, 1, 0, True),         # G = 8 path, ragged
    (256, 300, 4000, 64, 64, 1, 0, True),         # G = 16 path
    (200, 150, 3000, 200, 256, 1, 1, True),       # G = 64 path
    (200, 150, 3000, 300, 512, 1, 0, True),       # two batch tiles of 256 columns, ragged tail
    (200, 150, 3000, 299, 512, 1, 0, False),      # SDDMM-only path, tiles + ragged
    (200, 150, 3000, 600, 1024, 1, 0, True),      # columns of 15 connections: one launch per 128-column slice, five of them
    (300, 250, 3000, 1021, 1024, 1, 0, True),     # the same walk, eight slices, ragged tail
    (200, 150, 6000, 600, 1024, 1, 0, True),      # columns of 30: three batch tiles of 256, a pair, then a single one
    (200, 150, 6000, 1021, 1024, 1, 1, True),     # two pairs, ragged tail
    (200, 150, 3000, 1021, 1024, 1, 1, False),    # four batch tiles, ragged, SDDMM only
    (6, 2000, 12000, 300, 512, 1, 0, True),       # split CSC side with two batch tiles
    (400, 2, 800, 128, 128, 0, 0, True),          # dense output layer: long rows are split
    (3000, 10, 30000, 80, 128, 0, 0, True),       # dense output layer, rows of 3000
    (6, 2000, 12000, 128, 128, 1, 0, True),       # long columns: the CSC side is split
    (3000, 5000, 37, 128, 128, 1, 0, True),       # mostly empty rows and columns
    (2000, 3000, 90000, 128, 128, 1, 0, True),
    (2000, 3001, 6000, 128, 128, 1, 0, True),     # rows of about two entries: span kernels, ragged last span
    (2000, 3001, 6000, 30, 32, 1, 1, False),      # span SDDMM, G = 8, ragged batch
    (1500, 2500, 5000, 300, 512, 1, 0, True),     # span kernels with two batch tiles
    (1500, 2500, 5000, 1000, 1024, 1, 1, True)])  # very short rows, four tiles: both tile pairs walked in one launch
def test_forward_backward_update_one_layer(gpu, oracle, n_in, n_out, nnz, B, max_batch, act_kind, parity, need_gx):
    run_one_layer(gpu, oracle, n_in, n_out, nnz, B, max_batch, act_kind, parity, need_gx)


@pytest.mark.parametrize("alpha,parity", [(0.0, 0), (0.0, 1), (0.05, 1), (0.75, 0)])
def test_other_slopes_including_plain_relu(gpu, oracle, alpha, parity):
    """alpha = 0 is ReLU (the comparison activation of the experiments); 0.05 and 0.75 are slopes their tables use."""
    run_one_layer(gpu, oracle, 500, 400, 9000, 128, 128, 1, parity, True, alpha=alpha)


def test_randomly_drawn_small_layers(gpu, oracle):
    """Forty small layers with shapes, densities, batch sizes and modes drawn from a seeded generator: single
    rows and columns, one-sample batches, fully dense and nearly empty patterns, every group width."""
    rng = np.random.default_rng(20210201)
    for case in range(40):
        n_in, n_out = int(rng.integers(1, 90)), int(rng.integers(1, 90))
        nnz = max(1, int(round(float(rng.choice([0.01, 0.05, 0.2, 0.6, 1.0])) * n_in * n_out)))
        B = int(rng.choice([1, 2, 3, 4, 7, 32, 33, 64, 100, 128, 130, 256, 300]))
        max_batch = B + int(rng.choice([0, 0, 5, 64]))
        act_kind, parity, need_gx = int(rng.integers(0, 2)), int(rng.integers(0, 2)), bool(rng.integers(0, 2))
        alpha = float(rng.choice([0.0, 0.6, 0.75]))
        print(f"case {case}: {n_in}x{n_out} nnz={nnz} B={B} max_batch={max_batch} act={act_kind}/{parity} gx={need_gx} "
              f"alpha={alpha}", flush=True)
        run_one_layer(gpu, oracle, n_in, n_out, nnz, B, max_batch, act_kind, parity, need_gx, alpha=alpha)
        mode = int(rng.integers(0, 2))
        G, O = make_pair(gpu, oracle, n_in, n_out, nnz, prune_mode=mode, need_input_grad=need_gx, seed=100 + case,
                         max_batch=max_batch)
        for gen, zeta in ((1, 0.3), (2, float(rng.choice([0.0, 0.5, 1.0])))):
            O.evolve(zeta, gen)
            G.evolve(zeta, gen)
            assert_same_topology(G, O)
        G.close()


def run_one_layer(gpu, oracle, n_in, n_out, nnz, B, max_batch, act_kind, parity, need_gx, alpha=0.6):
    import torch
    G, O = make_pair(gpu, oracle, n_in, n_out, nnz, act_kind=act_kind, parity=parity, max_batch=max_batch,
                     need_input_grad=need_gx, limit=0.2, alpha=alpha)
    assert_same_topology(G, O)
    rng = np.random.default_rng(n_in + B)
    # non-zero bias and velocity so that every term of the formulas is exercised
    rowptr, colidx, val, vel, bias, bias_vel = G.export_csr()
    vel = (rng.standard_normal(nnz) * 0.01).astype(np.float32)
    bias = (rng.standard_normal(n_out) * 0.1).astype(np.float32)
    bias_vel = (rng.standard_normal(n_out) * 0.01).astype(np.float32)
    x = rng.standard_normal((n_in, B)).astype(np.float32)
    ga = rng.standard_normal((n_out, B)).astype(np.float32)
    # The derivative of eq. (3) jumps at z = 0 and the two sides round z differently, so the inputs
    # are built such that no pre-activation sits within 1e-5 of the kink (bias of such rows nudged).
    for _ in range(8):
        O.set_state(rowptr, colidx, val, vel, bias, bias_vel)
        O.forward(x)
        near = np.abs(O.z).min(axis=1) < 1e-5
        if act_kind == 0 or not near.any():
            break
        bias[near] += np.float32(0.013)
    else:
        raise AssertionError("could not move pre-activations off the kink")
    G.import_csr(rowptr, colidx, val, vel, bias, bias_vel)
    O.set_state(rowptr, colidx, val, vel, bias, bias_vel)
    ld = (B + 3) // 4 * 4 + 4
    xd, gad = dev(torch, pad_cols(x, ld)), dev(torch, pad_cols(ga, ld))
    ad = torch.full((n_out, ld), 7.0, dtype=torch.float32, device="cuda:0")
    gxd = torch.full((n_in, ld), 7.0, dtype=torch.float32, device="cuda:0") if need_gx else None
    # oracle
    a_ref = O.forward(x)
    gx_ref = O.backward(x, ga, need_input_grad=need_gx)
    # GPU
    G.forward(xd, B, ad)
    G.backward(xd, gad, B, gxd)
    g, gb = G.export_grad()
    torch.cuda.synchronize()
    a = ad.cpu().numpy()
    # besides the tensor-wide checks every element is held to 1e-4 of the sum of the magnitudes of its own terms
    mg, mgb, mgx = abs_backward(oracle, O, x, O.dz, need_input_grad=need_gx)
    close(a[:, :B], a_ref, 1e-4, "a", mag=abs_forward(oracle, O, x))
    assert np.all(a[:, B:] == 7.0), "columns >= B were written"
    close(g, O.grad_val, 1e-4, "grad_val", mag=mg)
    close(gb, O.grad_bias, 1e-4, "grad_bias", mag=mgb)
    if need_gx:
        gx = gxd.cpu().numpy()
        close(gx[:, :B], gx_ref, 1e-4, "grad_x", mag=mgx)
        assert np.all(gx[:, B:] == 7.0)
    O.update()
    G.update()
    r2, c2, val2, vel2, bias2, bvel2 = G.export_csr()
    assert np.array_equal(r2, O.rowptr) and np.array_equal(c2, O.colidx)
    close(val2, O.val, 1e-4, "val")
    close(vel2, O.vel, 1e-4, "vel")
    close(bias2, O.bias, 1e-4, "bias")
    close(bvel2, O.bias_vel, 1e-4, "bias_vel")
    # the update itself is plain fp32 arithmetic: bit-exact when fed the GPU's own gradient
    O.set_state(rowptr, colidx, val, vel, bias, bias_vel)
    O.grad_val, O.grad_bias = g.copy(), gb.copy()
    O.update()
    assert np.array_equal(val2.view(np.uint32), O.val.view(np.uint32))
    assert np.array_equal(vel2.view(np.uint32), O.vel.view(np.uint32))
    assert np.array_equal(bias2.view(np.uint32), O.bias.view(np.uint32))
    G.close()


def test_softmax_cross_entropy(gpu, oracle):
    import torch
    rng = np.random.default_rng(3)
    for C, B in [(2, 128), (10, 96), (10, 1), (7, 300)]:
        z = (rng.standard_normal((C, B)) * 4).astype(np.float32)
        y = rng.integers(0, C, size=B).astype(np.int32)
        ld = B + 8
        zd = dev(torch, pad_cols(z, ld))
        dzd = torch.full((C, ld), 7.0, dtype=torch.float32, device="cuda:0")
        loss = torch.zeros(1, dtype=torch.float32, device="cuda:0")
        gpu.softmax_ce(zd, dev(torch, y), B, C, dzd, loss)
        loss_ref, dz_ref = oracle.softmax_ce(z, y)
        dz = dzd.cpu().numpy()
        close(dz[:, :B], dz_ref, 1e-5, "dz")
        assert np.all(dz[:, B:] == 7.0)
        assert abs(loss.item() / B - loss_ref) <= 1e-5 * max(1.0, abs(loss_ref))


# ------------------------------------------------------------------------------------------ evolve
@pytest.mark.parametrize("mode", [0, 1])
@pytest.mark.parametrize("n_in,n_out,nnz,need_gx", [
    (500, 400, 9000, False), (400, 100, 5000, True), (400, 2, 800, True), (64, 48, 1000, True),
    (3000, 5000, 37, True), (100000, 70000, 1700000, True)])
def test_evolve_bit_exact(gpu, oracle, mode, n_in, n_out, nnz, need_gx):
    G, O = make_pair(gpu, oracle, n_in, n_out, nnz, prune_mode=mode, need_input_grad=need_gx, seed=99)
    rng = np.random.default_rng(nnz)
    rowptr, colidx, val, vel, bias, bias_vel = G.export_csr()
    # trained-looking weights; a few exact ties and zeros to exercise the tie rule
    val = (rng.standard_normal(nnz) * 0.1).astype(np.float32)
    if nnz >= 100:
        val[rng.integers(0, nnz, size=nnz // 10)] = np.float32(0.03125)
        val[rng.integers(0, nnz, size=nnz // 20)] = np.float32(-0.03125)
        val[rng.integers(0, nnz, size=5)] = 0.0
    vel = (rng.standard_normal(nnz) * 0.01).astype(np.float32)
    for gen in (1, 2, 3):
        G.import_csr(rowptr, colidx, val, vel, bias, bias_vel)
        O.set_state(rowptr, colidx, val, vel, bias, bias_vel)
        k = O.evolve(0.3, gen)
        G.evolve(0.3, gen)
        assert G.nnz == nnz
        assert_same_topology(G, O)
        rowptr, colidx, val, vel, bias, bias_vel = G.export_csr()
        assert int((vel == 0).sum()) >= k
    G.close()


def test_evolve_all_ties_and_zero_fraction(gpu, oracle):
    G, O = make_pair(gpu, oracle, 300, 200, 4000, seed=5)
    rowptr, colidx, val, vel, bias, bias_vel = G.export_csr()
    val[:] = np.where(np.arange(4000) % 2 == 0, 0.25, -0.25)
    G.import_csr(rowptr, colidx, val, vel, bias, bias_vel)
    O.set_state(rowptr, colidx, val, vel, bias, bias_vel)
    O.evolve(0.3, 1)
    G.evolve(0.3, 1)
    assert_same_topology(G, O)
    before = G.export_csr()
    G.evolve(0.0, 2)
    after = G.export_csr()
    assert all(np.array_equal(a, b) for a, b in zip(before, after))
    G.close()


# ------------------------------------------------------------------------------------------ whole network
# The derivative of eq. (3) jumps at z = 0.  Over thousands of pre-activations per step a few land
# within rounding distance of the kink, where the oracle (double accumulation) and the kernel (fp32
# accumulation in another order) may legitimately take different branches; both are correct
# evaluations of the method.  The oracle is therefore run once as is; if that run saw
# pre-activations within KINK_TAU (relative) of zero, the alternatives in which subsets of them take the other
# branch are also valid references, and the GPU result must match one of them.  No GPU value
# enters any oracle run.
KINK_TAU = 3e-7      # relative to |b| + sum |w||x|: a few fp32 ulps of the terms that were added
MAX_KINKS = 8


def oracle_run(oracle, w, blocks, y, n_steps, flips=frozenset(), dropout=0.0):
    olayers = [oracle.OracleLayer(s.n_in, s.n_out, s.nnz, s.act_kind, s.act_parity, w.alpha, s.init_limit, w.lr,
                                  w.momentum, 0.0, w.seed, s.layer_id) for s in w.layers]
    onet = oracle.OracleMLP(olayers)
    onet.dropout = dropout
    seen, state = [], {"step": 0}

    def hook(li, layer, a):
        if not layer.act_kind:
            return a
        # rounding error of z scales with the magnitude of its terms: |b| + sum |w| |x|
        rows = np.repeat(np.arange(layer.n_out), np.diff(layer.rowptr))
        mag = sp.csr_matrix((np.abs(layer.val).astype(np.float64), layer.colidx, layer.rowptr),
                            shape=(layer.n_out, layer.n_in)) @ np.abs(onet.acts[-1]).astype(np.float64)
        mag += np.abs(layer.bias).astype(np.float64)[:, None]
        for j, b in np.argwhere(np.abs(layer.z) < KINK_TAU * mag):
            key = (state["step"], li, int(j), int(b))
            seen.append(key)
            if key in flips:
                z = layer.z[j, b]
                layer.z[j, b] = -z if z != 0 else np.float32(1e-30)
                a[j, b] = oracle.all_relu(layer.z[j:j + 1, b], layer.act_kind, layer.act_parity, layer.alpha)[0]
                if layer.keep is not None:
                    scale = np.float32(1.0) / (np.float32(1.0) - layer.drop_p)
                    a[j, b] = a[j, b] * scale if layer.keep[j, b] else np.float32(0.0)
        return a

    onet.after_forward = hook
    losses, first = [], None
    for k in range(n_steps):
        state["step"] = k
        B = min(w.batch, y.shape[0] - k * w.batch)
        losses.append(B * onet.train_step(blocks[k][:, :B], y[k * w.batch:k * w.batch + B]))
        if k == 0:
            first = dict(acts=[a.copy() for a in onet.acts[1:]],
                         layers=[(O.val.copy(), O.vel.copy(), O.bias.copy()) for O in olayers])
    return onet, olayers, losses, first, seen


def check_network(net, gpu_first, gpu_loss, olayers, losses, first, tol_first, tol_end):
    for li, O in enumerate(olayers):
        a, val, vel, bias = gpu_first[li]
        close(a, first["acts"][li], tol_first, f"act {li}")
        close(val, first["layers"][li][0], tol_first, f"val {li} after one step")
        close(vel, first["layers"][li][1], tol_first, f"vel {li} after one step")
        close(bias, first["layers"][li][2], tol_first, f"bias {li} after one step")
    assert abs(gpu_loss - sum(losses)) <= tol_end * abs(sum(losses)), "loss"
    for li, (G, O) in enumerate(zip(net.layers, olayers)):
        rowptr, colidx, val, vel, bias, bias_vel = G.export_csr()
        assert np.array_equal(rowptr, O.rowptr) and np.array_equal(colidx, O.colidx)
        close(val, O.val, tol_end, f"val {li}")
        close(vel, O.vel, tol_end, f"vel {li}")
        close(bias, O.bias, tol_end, f"bias {li}")
        close(bias_vel, O.bias_vel, tol_end, f"bias_vel {li}")


def run_network(gpu, oracle, w, n_steps, tol_first=1e-4, tol_end=1e-3, dropout=0.0):
    """Trains n_steps minibatches on both sides from the same initialisation and compares after the
    first step (tol_first) and after the last (tol_end).  Returns the GPU net and the matching oracle."""
    import itertools
    import torch
    X, y = wl.dataset(w, n_steps * w.batch)
    blocks = wl.to_batch_blocks(X, w.batch)
    net = gpu.SparseMLP(w.layers, alpha=w.alpha, lr=w.lr, momentum=w.momentum, seed=w.seed, max_batch=w.batch)
    net.dropout = dropout
    xd, yd = dev(torch, blocks), dev(torch, y)
    gpu_first = None
    for k in range(n_steps):
        B = min(w.batch, X.shape[0] - k * w.batch)
        net.train_step(xd[k], yd[k * w.batch:k * w.batch + B], B)
        if k == 0:
            gpu_first = []
            for li, G in enumerate(net.layers):
                _, _, val, vel, bias, _ = G.export_csr()
                gpu_first.append((net.acts[li].cpu().numpy()[:, :B], val, vel, bias))
    gpu_loss = net.loss_sum.item()
    onet, olayers, losses, first, seen = oracle_run(oracle, w, blocks, y, n_steps, dropout=dropout)
    assert len(seen) <= MAX_KINKS, f"{len(seen)} pre-activations on the kink: pick another seed"
    last_error = None
    for r in range(len(seen) + 1):
        for subset in itertools.combinations(seen, r):
            if r > 0:
                onet, olayers, losses, first, _ = oracle_run(oracle, w, blocks, y, n_steps, frozenset(subset), dropout)
            try:
                check_network(net, gpu_first, gpu_loss, olayers, losses, first, tol_first, tol_end)
                return net, onet, olayers
            except AssertionError as e:      # try the next valid branch assignment
                last_error = e if last_error is None else last_error
    raise last_error


def run_network_stepwise(gpu, oracle, w, n_steps, tol_end=1e-3):
    """A whole epoch on networks too large for the enumeration above (hundreds of pre-activations come within
    rounding distance of the kink over hundreds of steps, and a single one that takes the other branch grows into
    a difference of 1e-3 within a few hundred steps).  The GPU trains freely; the oracle follows minibatch by
    minibatch.  A pre-activation z_jb is ON THE KINK when |z_jb| is below the worst-case rounding error of an
    fp32 sum of its terms, (n_j + 2) 2^-24 (|b_j| + sum_i |w_ji||x_ib|): there either branch of eq. (3) is a
    correct result.  Which branch the GPU took shows in its gradient of that step: the other branch changes
    dz_jb and with it the gradient of row j by u = (dz'_jb - dz_jb) x_b, and the GPU took it if its gradient of
    that row sits nearer to the oracle's + u than to the oracle's: t = <g_gpu - g_oracle, u> / <u, u> > 1/2
    (t is about 0 or about 1).  The oracle then re-takes the step with those branches and continues.  Every
    number compared comes from the oracle; the GPU only selects which of the valid references it is compared
    with, and a branch missed here can only make the comparison at the end fail.  Asserted on the way: every t
    is within 0.02 of 0 or of 1, only pre-activations the oracle put on the kink are ever switched, and at most
    1 % of them are.  (test_gpu_epoch_oracle_only.py checks the same epochs without this dependence: there the
    oracle's state goes into the GPU before every minibatch.)"""
    import torch
    X, y = wl.dataset(w, n_steps * w.batch)
    blocks = wl.to_batch_blocks(X, w.batch)
    net = gpu.SparseMLP(w.layers, alpha=w.alpha, lr=w.lr, momentum=w.momentum, seed=w.seed, max_batch=w.batch)
    xd, yd = dev(torch, blocks), dev(torch, y)
    olayers = [oracle.OracleLayer(s.n_in, s.n_out, s.nnz, s.act_kind, s.act_parity, w.alpha, s.init_limit, w.lr,
                                  w.momentum, 0.0, w.seed, s.layer_id) for s in w.layers]
    onet = oracle.OracleMLP(olayers)
    state = {"flips": (), "seen": [], "collect": True}

    def hook(li, layer, a):
        if not layer.act_kind:
            return a
        if state["collect"]:
            x_in = np.abs(onet.acts[-1]).astype(np.float64)
            n_j = np.diff(layer.rowptr).astype(np.float64)
            rows = np.repeat(np.arange(layer.n_out), np.diff(layer.rowptr))
            absw = np.bincount(rows, weights=np.abs(layer.val).astype(np.float64), minlength=layer.n_out)
            loose = (n_j + 2.0) * 2.0 ** -24 * (np.abs(layer.bias) + absw * x_in.max())     # >= the bound of any sample
            for j, b in np.argwhere(np.abs(layer.z) < loose[:, None]):
                p0, p1 = layer.rowptr[j], layer.rowptr[j + 1]
                mag = abs(float(layer.bias[j])) + float(np.abs(layer.val[p0:p1]).astype(np.float64) @ x_in[layer.colidx[p0:p1], b])
                if abs(float(layer.z[j, b])) < (n_j[j] + 2.0) * 2.0 ** -24 * mag:
                    state["seen"].append((li, int(j), int(b)))
        for fl, j, b in state["flips"]:
            if fl == li:
                z = layer.z[j, b]
                layer.z[j, b] = -z if z != 0 else np.float32(1e-30)
                a[j, b] = oracle.all_relu(layer.z[j:j + 1, b], layer.act_kind, layer.act_parity, layer.alpha)[0]
        return a

    onet.after_forward = hook

    def snapshot():
        return [(O.val.copy(), O.vel.copy(), O.bias.copy(), O.bias_vel.copy()) for O in olayers]

    def restore(snap):
        for O, (val, vel, bias, bias_vel) in zip(olayers, snap):
            O.set_state(O.rowptr, O.colidx, val, vel, bias, bias_vel)

    def oracle_step(xs, ys, flips, collect=False):
        state["flips"], state["seen"], state["collect"] = tuple(flips), [], collect
        return onet.train_step(xs, ys)

    def took_other_branch(li, j, b, gpu_grad):
        O = olayers[li]
        s_neg = -float(O.alpha) if O.act_parity == 0 else float(O.alpha)
        s_cur, s_oth = (1.0, s_neg) if O.z[j, b] > 0 else (s_neg, 1.0)
        if s_cur == 0.0:
            return None                       # plain ReLU below zero: dz holds no trace of the incoming gradient
        dz = float(O.dz[j, b])
        p0, p1 = O.rowptr[j], O.rowptr[j + 1]
        u = (dz / s_cur * s_oth - dz) * onet.acts[li][O.colidx[p0:p1], b].astype(np.float64)
        if not u.any():
            return 0.0
        return float((gpu_grad[p0:p1].astype(np.float64) - O.grad_val[p0:p1]) @ u) / float(u @ u)

    trace = bool(os.environ.get("SL_TEST_TRACE"))
    loss_sum, on_kink, flipped = 0.0, 0, 0
    for k in range(n_steps):
        B = min(w.batch, X.shape[0] - k * w.batch)
        xs, ys = blocks[k][:, :B], y[k * w.batch:k * w.batch + B]
        before = snapshot()
        loss = oracle_step(xs, ys, (), collect=True)
        seen = list(state["seen"])
        on_kink += len(seen)
        gpu_grads = {}

        def read_gradients(model):
            for li in {key[0] for key in seen}:
                gpu_grads[li] = model.layers[li].export_grad()[0]

        net.train_step(xd[k], yd[k * w.batch:k * w.batch + B], B, before_update=read_gradients if seen else None)
        # Deepest layer first: a branch taken differently there changes the gradient that flows back into the
        # layers before it, so their rows are judged against the oracle re-run with the branches found so far.
        other = []
        for li in sorted({key[0] for key in seen}, reverse=True):
            found = []
            for fl, j, b in seen:
                if fl != li:
                    continue
                t = took_other_branch(li, j, b, gpu_grads[li])
                assert t is not None, "plain ReLU networks need the enumeration of run_network"
                # the GPU's gradient must BE one of the two valid ones, not merely nearer to one of them
                assert min(abs(t), abs(t - 1.0)) <= 0.02, f"step {k}: {(li, j, b)}: t = {t:.4f} is neither branch"
                if t > 0.5:
                    found.append((li, j, b))
                if trace and t > 0.1:
                    print(f"  step {k}: {(li, j, b)} t = {t:.3f}", flush=True)
            if found:
                assert set(found) <= set(seen)          # only pre-activations the oracle itself put on the kink
                other += found
                restore(before)
                loss = oracle_step(xs, ys, other)
        flipped += len(other)
        loss_sum += B * loss
    print(f"{w.name}: {n_steps} steps, {on_kink} pre-activations on the kink, {flipped} took the other branch", flush=True)
    # the bound is a worst case: the kernel's actual rounding error is far smaller, so nearly all stay on the oracle's side
    assert flipped <= max(2, 0.01 * on_kink), f"{flipped} of {on_kink} pre-activations on the kink took the other branch"
    assert abs(net.loss_sum.item() - loss_sum) <= tol_end * abs(loss_sum), "loss"
    for li, (G, O) in enumerate(zip(net.layers, olayers)):
        rowptr, colidx, val, vel, bias, bias_vel = G.export_csr()
        assert np.array_equal(rowptr, O.rowptr) and np.array_equal(colidx, O.colidx)
        close(val, O.val, tol_end, f"val {li}")
        close(vel, O.vel, tol_end, f"vel {li}")
        close(bias, O.bias, tol_end, f"bias {li}")
        close(bias_vel, O.bias_vel, tol_end, f"bias_vel {li}")
    return net, onet, olayers


@pytest.mark.parametrize("name", ["set_mlp_fmnist", "set_mlp_cifar"])
def test_image_shaped_networks_whole_epoch(gpu, oracle, name):
    """The FashionMNIST-shaped network for its epoch of 469 minibatches and the CIFAR-shaped one for its 391 (the
    last minibatch of each is ragged), then one evolution from the oracle's trained weights."""
    w = wl.WORKLOADS[name]
    net, onet, olayers = run_network_stepwise(gpu, oracle, w, w.steps_per_epoch)
    for G, O in zip(net.layers, olayers):
        G.import_csr(O.rowptr, O.colidx, O.val, O.vel, O.bias, O.bias_vel)
    net.evolve(w.zeta, 1)
    onet.evolve(w.zeta, 1)
    for G, O in zip(net.layers, olayers):
        assert_same_topology(G, O)
    net.close()


def test_madelon_shaped_epoch_and_evolution(gpu, oracle):
    import torch
    w = wl.WORKLOADS["set_mlp_madelon"]
    net, onet, olayers = run_network(gpu, oracle, w, w.steps_per_epoch)
    # Evolution after the epoch, as a function of bit-identical inputs: the ORACLE's trained weights
    # go into the GPU layers, then both sides evolve.
    for G, O in zip(net.layers, olayers):
        G.import_csr(O.rowptr, O.colidx, O.val, O.vel, O.bias, O.bias_vel)
    net.evolve(w.zeta, 1)
    onet.evolve(w.zeta, 1)
    for G, O, s in zip(net.layers, olayers, w.layers):
        assert G.nnz == s.nnz
        assert_same_topology(G, O)
    # the evolved network keeps training
    onet.after_forward = None
    X, y = wl.dataset(w, w.batch)
    blocks = wl.to_batch_blocks(X, w.batch)
    l0 = w.batch * onet.train_step(blocks[0], y)
    net.loss_sum.zero_()
    net.train_step(dev(torch, blocks[0]), dev(torch, y), w.batch)
    assert abs(net.loss_sum.item() - l0) <= 1e-4 * abs(l0)
    net.close()


@pytest.mark.parametrize("name,steps", [("set_mlp_fmnist", 3), ("set_mlp_cifar", 2)])
def test_image_shaped_networks_first_steps(gpu, oracle, name, steps):
    w = wl.WORKLOADS[name]
    net, onet, olayers = run_network(gpu, oracle, w, steps, tol_first=1e-4, tol_end=3e-4)
    net.close()


# ------------------------------------------------------------------------------------------ chained layers
@pytest.mark.parametrize("dims,nnz,B,max_batch", [
    ((300, 500, 200), (4000, 5000), 128, 128),
    ((300, 500, 200), (4000, 5000), 77, 128),        # ragged batch
    ((300, 6, 2000), (1800, 12000), 96, 128),        # long columns: the consumer's CSC side is split
    ((200, 400, 2), (3000, 800), 300, 512),          # batch tiles; narrow dense consumer
])
def test_linked_backward_equals_unlinked(gpu, oracle, dims, nnz, B, max_batch):
    """Handing dz to the producer inside the consumer's backward kernel must give exactly what the
    separate path (grad_x buffer, then the producer's own activation-derivative pass) gives."""
    import torch
    rng = np.random.default_rng(7)
    mk = lambda li, need: gpu.SparseLayer(gpu.make_config(dims[li], dims[li + 1], nnz=nnz[li], act_kind=1,
                                                           act_parity=li % 2, alpha=0.6, init_limit=0.2, seed=3,
                                                           layer_id=li, max_batch=max_batch, need_input_grad=need))
    ld = (B + 3) // 4 * 4
    x = dev(torch, pad_cols(rng.standard_normal((dims[0], B)).astype(np.float32), ld))
    ga = dev(torch, pad_cols(rng.standard_normal((dims[2], B)).astype(np.float32), ld))
    results = []
    for linked in (False, True):
        P, C = mk(0, False), mk(1, True)
        a1 = torch.zeros((dims[1], ld), device="cuda")
        a2 = torch.zeros((dims[2], ld), device="cuda")
        P.forward(x, B, a1)
        C.forward(a1, B, a2)
        if linked:
            C.link_producer(P)
            C.backward(a1, ga, B, None)
            P.backward(x, None, B, None)
        else:
            g1 = torch.zeros((dims[1], ld), device="cuda")
            C.backward(a1, ga, B, g1)
            P.backward(x, g1, B, None)
        results.append((P.export_grad(), C.export_grad()))
        P.close()
        C.close()
    for (g_u, gb_u), (g_l, gb_l) in zip(results[0], results[1]):
        assert np.array_equal(g_u.view(np.uint32), g_l.view(np.uint32))
        assert np.array_equal(gb_u.view(np.uint32), gb_l.view(np.uint32))
    assert np.abs(results[0][0][0]).max() > 0


# ------------------------------------------------------------------------------------------ Importance Pruning
@pytest.mark.parametrize("n_in,n_out,nnz,need_gx", [(500, 400, 9000, True), (500, 400, 9000, False),
                                                     (40, 30, 1000, True),          # dense sampler mode before pruning
                                                     (100000, 70000, 1700000, True)])
def test_importance_pruning_bit_exact(gpu, oracle, n_in, n_out, nnz, need_gx):
    import torch
    G, O = make_pair(gpu, oracle, n_in, n_out, nnz, need_input_grad=need_gx, seed=41)
    rng = np.random.default_rng(nnz + 1)
    rowptr, colidx, val, vel, bias, bias_vel = G.export_csr()
    val = (rng.standard_normal(nnz) * 0.1).astype(np.float32)
    vel = (rng.standard_normal(nnz) * 0.01).astype(np.float32)
    G.import_csr(rowptr, colidx, val, vel, bias, bias_vel)
    O.set_state(rowptr, colidx, val, vel, bias, bias_vel)
    imp = G.importance()
    assert np.array_equal(imp.view(np.uint32), O.importance_f32().view(np.uint32))      # eq. (4), same fp32 order
    t = float(np.quantile(imp.astype(np.float64), 0.3))
    removed = G.importance_prune(t)
    assert removed == O.importance_prune(t) and removed > 0
    assert G.nnz == O.nnz == nnz - removed
    assert_same_topology(G, O)
    # the pruned layer still trains: one forward/backward/update against the oracle
    B = 64
    x = rng.standard_normal((n_in, B)).astype(np.float32)
    ga = rng.standard_normal((n_out, B)).astype(np.float32)
    a_ref = O.forward(x)
    gx_ref = O.backward(x, ga, need_input_grad=need_gx)
    ad = torch.zeros((n_out, B), device="cuda")
    gxd = torch.zeros((n_in, B), device="cuda") if need_gx else None
    xd = dev(torch, x)
    G.forward(xd, B, ad)
    G.backward(xd, dev(torch, ga), B, gxd)
    close(ad.cpu().numpy(), a_ref, 1e-4, "a after pruning")
    g, gb = G.export_grad()
    keep_rows = np.abs(O.z).min(axis=1) > 1e-5                     # rows away from the kink of eq. (3)
    rows = np.repeat(np.arange(n_out), np.diff(O.rowptr))
    close(g[keep_rows[rows]], O.grad_val[keep_rows[rows]], 1e-4, "grad_val after pruning")
    G.update()
    # and it still evolves: from identical bits, with the reduced nnz preserved
    rowptr, colidx, val, vel, bias, bias_vel = G.export_csr()
    O.set_state(O.rowptr, O.colidx, O.val, O.vel, O.bias, O.bias_vel)
    G.import_csr(O.rowptr, O.colidx, O.val, O.vel, O.bias, O.bias_vel)
    for gen in (1, 2):
        O.evolve(0.3, gen)
        G.evolve(0.3, gen)
        assert G.nnz == nnz - removed
        assert_same_topology(G, O)
    # pruning everything leaves an empty but usable layer
    assert G.importance_prune(1e30) == nnz - removed and G.nnz == 0
    G.forward(xd, B, ad)
    assert np.array_equal(ad.cpu().numpy(), gpu_bias_act(O.bias, O, B))     # a = f(bias): no connection is left
    G.close()


# ------------------------------------------------------------------ RetainValidUpdates (Algorithm 1)
@pytest.mark.parametrize("n_in,n_out,nnz,need_gx", [(500, 400, 9000, True), (500, 400, 9000, False),
                                                     (64, 3, 100, True), (100000, 70000, 1700000, True)])
def test_retain_valid_updates_bit_exact(gpu, oracle, n_in, n_out, nnz, need_gx):
    import torch
    G, O = make_pair(gpu, oracle, n_in, n_out, nnz, need_input_grad=need_gx, seed=43)
    rng = np.random.default_rng(nnz + 5)
    old_rowptr, old_colidx = O.rowptr.copy(), O.colidx.copy()
    old_grad = rng.standard_normal(nnz).astype(np.float32)
    old_gb = rng.standard_normal(n_out).astype(np.float32)
    for gen in (1, 2):                                      # the topology moves on twice
        O.evolve(0.3, gen)
        G.evolve(0.3, gen)
    assert_same_topology(G, O)
    oracle.retain_valid_updates(O, old_rowptr, old_colidx, old_grad, old_gb)
    G.retain_valid_updates(dev(torch, old_rowptr), dev(torch, old_colidx), dev(torch, old_grad), dev(torch, old_gb))
    g, gb = G.export_grad()
    assert np.array_equal(g.view(np.uint32), O.grad_val.view(np.uint32))
    assert np.array_equal(gb.view(np.uint32), O.grad_bias.view(np.uint32))
    assert 0 < (g == 0).sum() < nnz
    O.update()
    G.update()
    assert_same_topology(G, O)
    # an empty old pattern retains nothing; a pattern identical to the current one retains everything
    zero_ptr = np.zeros(n_out + 1, np.int32)
    G.retain_valid_updates(dev(torch, zero_ptr), torch.zeros(0, dtype=torch.int32, device="cuda"),
                           torch.zeros(0, device="cuda"), dev(torch, old_gb))
    g, _ = G.export_grad()
    assert not g.any()
    G.update()
    O.grad_val = np.zeros(O.nnz, np.float32)
    O.grad_bias = old_gb.copy()
    O.update()
    assert_same_topology(G, O)
    same = rng.standard_normal(O.nnz).astype(np.float32)
    G.retain_valid_updates(dev(torch, O.rowptr), dev(torch, O.colidx), dev(torch, same), dev(torch, old_gb))
    g, _ = G.export_grad()
    assert np.array_equal(g, same)
    G.close()


def gpu_bias_act(bias, O, B):
    z = np.repeat(np.asarray(bias, np.float32)[:, None], B, axis=1)
    return np.where(z > 0, z, (-O.alpha if O.act_parity == 0 else O.alpha) * z).astype(np.float32)


# ------------------------------------------------------------------------------------------ sweep-sized layer
def test_sweep_sized_layer_two_batch_tiles(gpu, oracle):
    """One 262 144 x 262 144 layer (epsilon = 4) at B = 512: two batch tiles of 256 columns, chunk
    width 8, the launch shapes of the single-layer sweep; every output compared with the oracle."""
    import torch
    n, B = wl.SWEEP_N, 512
    spec = wl.sweep_layer(4)
    G, O = make_pair(gpu, oracle, n, n, spec.nnz, limit=spec.init_limit, max_batch=B, seed=wl.DEFAULT_SEED, layer_id=0)
    assert_same_topology(G, O)
    x = wl.dense_operand(n, B, 5)
    ga = wl.dense_operand(n, B, 6)
    a_ref = O.forward(x)
    gx_ref = O.backward(x, ga)
    xd, gad = dev(torch, x), dev(torch, ga)
    ad, gxd = torch.empty_like(xd), torch.empty_like(xd)
    G.forward(xd, B, ad)
    G.backward(xd, gad, B, gxd)
    g, gb = G.export_grad()
    close(ad.cpu().numpy(), a_ref, 1e-4, "a")
    # rows whose pre-activation sits on the kink of eq. (3) may take the other branch: leave them out
    safe = np.abs(O.z).min(axis=1) > 1e-5
    rows = np.repeat(np.arange(n), np.diff(O.rowptr))
    assert safe.mean() > 0.95
    close(g[safe[rows]], O.grad_val[safe[rows]], 1e-4, "grad_val")
    close(gb[safe], O.grad_bias[safe], 1e-4, "grad_bias")
    # an input gradient row is exact unless one of the rows it gathers is unsafe
    touched = np.zeros(n, bool)
    touched[O.colidx[~safe[rows]]] = True
    close(gxd.cpu().numpy()[~touched], gx_ref[~touched], 1e-4, "grad_x")
    G.close()


# ------------------------------------------------------------------------------------------ error paths on a live layer
def test_argument_and_call_order_errors(gpu):
    import torch
    cfg = gpu.make_config(64, 48, nnz=500, init_limit=0.1, max_batch=32, need_input_grad=True)
    L = gpu.SparseLayer(cfg)
    x = torch.zeros((64, 32), device="cuda")
    a = torch.zeros((48, 32), device="cuda")
    gx = torch.zeros((64, 32), device="cuda")

    def code(f):
        with pytest.raises(gpu.SparseSetError) as e:
            f()
        return e.value.code

    assert code(lambda: L.backward(x, a, 32, gx)) == gpu.SL_ESTATE          # backward before forward
    assert code(L.update) == gpu.SL_ESTATE                                  # update before backward
    assert code(lambda: L.forward(x, 33, a)) == gpu.SL_EINVAL               # B > max_batch
    assert code(lambda: L.forward(x, 0, a)) == gpu.SL_EINVAL
    assert code(lambda: L.forward(torch.zeros((64, 28), device="cuda"), 32, a)) == gpu.SL_EINVAL   # ld < B
    assert code(lambda: L.forward(x[:, 1:], 28, a)) == gpu.SL_EINVAL        # misaligned base pointer
    L.forward(x, 32, a)
    assert code(lambda: L.backward(x, a, 16, gx)) == gpu.SL_ESTATE          # other B than forward
    assert code(lambda: L.backward(x, a, 32, None)) == gpu.SL_EINVAL        # grad_x missing, no producer linked
    assert code(lambda: L.backward(x, None, 32, gx)) == gpu.SL_EINVAL       # grad_a missing, nothing handed over
    assert code(L.export_grad) == gpu.SL_ESTATE
    rp = torch.zeros(49, dtype=torch.int32, device="cuda")
    none_i, none_f, gb0 = torch.zeros(0, dtype=torch.int32, device="cuda"), torch.zeros(0, device="cuda"), torch.zeros(48, device="cuda")
    assert code(lambda: L.retain_valid_updates(rp, none_i, none_f, gb0)) == gpu.SL_ESTATE   # between forward and backward
    L.backward(x, a, 32, gx)
    L.export_grad()
    L.update()
    assert code(lambda: L.evolve(1.5, 1)) == gpu.SL_EINVAL
    assert code(lambda: L.evolve(0.3, 0)) == gpu.SL_EINVAL
    rowptr, colidx, val, vel, bias, bias_vel = L.export_csr()
    bad = colidx.copy()
    bad[0] = 64
    assert code(lambda: L.import_csr(rowptr, bad, val)) == gpu.SL_EINVAL
    assert code(lambda: L.import_csr(rowptr[::-1].copy(), colidx, val)) == gpu.SL_EINVAL
    # an old pattern whose row bounds are nonsense is clamped, never followed: every gradient comes out zero or in range
    wild = torch.full((49,), 2**31 - 1, dtype=torch.int32, device="cuda")
    wild[::2] = -5
    oc = torch.arange(7, dtype=torch.int32, device="cuda")
    L.retain_valid_updates(wild, oc, torch.ones(7, device="cuda"), gb0)
    g, _ = L.export_grad()
    assert set(np.unique(g)) <= {0.0, 1.0}
    L.update()
    other = gpu.SparseLayer(gpu.make_config(10, 64, nnz=50, init_limit=0.1, max_batch=16, need_input_grad=False))
    assert code(lambda: L.link_producer(other)) == gpu.SL_EINVAL            # producer's max_batch too small
    assert "max_batch" in gpu.lib().sparse_layer_last_error(L.handle).decode()
    # a state buffer that is too small is refused at init
    import ctypes as C
    sb, cb = gpu.query_sizes(cfg)
    st = torch.empty(sb // 2, dtype=torch.uint8, device="cuda")
    sc = torch.empty(cb + 256, dtype=torch.uint8, device="cuda")
    h = C.c_void_p(None)
    assert gpu.lib().sparse_layer_init(C.byref(cfg), st.data_ptr(), st.numel(), sc.data_ptr(), sc.numel(), None,
                                       C.byref(h)) == gpu.SL_ENOMEM
    L.close()
    other.close()


# ------------------------------------------------------------------------------------------ inference, weight decay
def test_infer_equals_forward_and_leaves_training_state_alone(gpu, oracle):
    import torch
    G, O = make_pair(gpu, oracle, 300, 700, 6000, max_batch=512, limit=0.2)
    rng = np.random.default_rng(9)
    x = rng.standard_normal((300, 128)).astype(np.float32)
    ga = rng.standard_normal((700, 128)).astype(np.float32)
    xd = dev(torch, x)
    a_train = torch.zeros((700, 128), device="cuda")
    G.forward(xd, 128, a_train)
    # a larger inference batch in between must not disturb the saved signs of the training batch
    xbig = dev(torch, rng.standard_normal((300, 512)).astype(np.float32))
    a_big = torch.zeros((700, 512), device="cuda")
    G.infer(xbig, 512, a_big)
    close(a_big.cpu().numpy(), O.forward(xbig.cpu().numpy()), 1e-4, "inference output")
    a_inf = torch.zeros((700, 128), device="cuda")
    G.infer(xd, 128, a_inf)
    assert torch.equal(a_inf, a_train)
    gx = torch.zeros((300, 128), device="cuda")
    G.backward(xd, dev(torch, ga), 128, gx)
    O.forward(x)
    gx_ref = O.backward(x, ga)
    g, gb = G.export_grad()
    safe = np.abs(O.z).min(axis=1) > 1e-5
    rows = np.repeat(np.arange(700), np.diff(O.rowptr))
    close(g[safe[rows]], O.grad_val[safe[rows]], 1e-4, "grad_val")
    G.close()


def test_weight_decay_term_of_the_update(gpu, oracle):
    import torch
    lam = 0.05
    cfg = gpu.make_config(200, 150, nnz=3000, act_kind=1, act_parity=1, alpha=0.6, init_limit=0.3, lr=0.01, momentum=0.9,
                          weight_decay=lam, seed=4, layer_id=1, max_batch=64, need_input_grad=True)
    G = gpu.SparseLayer(cfg)
    O = oracle.OracleLayer(200, 150, 3000, 1, 1, 0.6, 0.3, 0.01, 0.9, lam, 4, 1)
    assert_same_topology(G, O)
    rng = np.random.default_rng(2)
    x = rng.standard_normal((200, 64)).astype(np.float32)
    ga = rng.standard_normal((150, 64)).astype(np.float32)
    xd = dev(torch, x)
    a = torch.zeros((150, 64), device="cuda")
    gx = torch.zeros((200, 64), device="cuda")
    for _ in range(3):
        O.forward(x)
        O.backward(x, ga)
        G.forward(xd, 64, a)
        G.backward(xd, dev(torch, ga), 64, gx)
        g, gb = G.export_grad()
        O.grad_val, O.grad_bias = g.copy(), gb.copy()     # same gradient in: the update must agree bit for bit
        rowptr, colidx, val, vel, bias, bias_vel = G.export_csr()
        O.set_state(rowptr, colidx, val, vel, bias, bias_vel)
        O.grad_val, O.grad_bias = g.copy(), gb.copy()
        O.update()
        G.update()
        _, _, val2, vel2, bias2, _ = G.export_csr()
        assert np.array_equal(val2.view(np.uint32), O.val.view(np.uint32))
        assert np.array_equal(vel2.view(np.uint32), O.vel.view(np.uint32))
        assert np.array_equal(bias2.view(np.uint32), O.bias.view(np.uint32))
    # the decay really acts: with zero gradient the weights shrink by lr*lambda*w per step (plus momentum)
    assert lam > 0 and not np.array_equal(val2, val)
    G.close()


# ------------------------------------------------------------------------------------------ sparse averaging, eq. (2)
@pytest.mark.parametrize("n_in,n_out,nnz,K", [(300, 200, 4000, 3), (400, 2, 800, 2), (100000, 70000, 1700000, 4),
                                               (50, 40, 300, 1)])
def test_sparse_average_bit_exact(gpu, oracle, n_in, n_out, nnz, K):
    rng = np.random.default_rng(K + nnz)
    Gs, Os = [], []
    for k in range(K):
        G, O = make_pair(gpu, oracle, n_in, n_out, nnz, seed=500 + k)
        assert_same_topology(G, O)
        rowptr, colidx, val, vel, bias, bias_vel = G.export_csr()
        val = (rng.standard_normal(nnz) * 0.1).astype(np.float32)
        if nnz >= 100:
            val[rng.integers(0, nnz, size=nnz // 20)] = np.float32(0.0625)      # ties across the union
        bias = rng.standard_normal(n_out).astype(np.float32)
        vel = rng.standard_normal(nnz).astype(np.float32)
        G.import_csr(rowptr, colidx, val, vel, bias, bias_vel)
        O.set_state(rowptr, colidx, val, vel, bias, bias_vel)
        if k > 0:                                     # let the topologies diverge
            O.evolve(0.3, k)
            G.evolve(0.3, k)
            assert_same_topology(G, O)
        Gs.append(G)
        Os.append(O)
    U = oracle.average_layers(Os[0], Os)
    gpu.average_layers(Gs[0], Gs)
    assert Gs[0].nnz == Os[0].nnz == min(nnz, U)
    assert_same_topology(Gs[0], Os[0])
    rowptr, colidx, val, vel, bias, bias_vel = Gs[0].export_csr()
    assert np.array_equal(bias.view(np.uint32), Os[0].bias.view(np.uint32))
    assert not vel.any() and not bias_vel.any()
    # the averaged layer is a working layer: it still evolves identically on both sides
    Os[0].evolve(0.3, 9)
    Gs[0].evolve(0.3, 9)
    assert_same_topology(Gs[0], Os[0])
    for G in Gs:
        G.close()


# ------------------------------------------------------------------------------------------ fewer launches per step
def test_fused_loss_and_multi_layer_update_match_the_separate_calls(gpu, oracle):
    import ctypes as C
    import torch
    w = wl.WORKLOADS["set_mlp_madelon"]
    X, y = wl.dataset(w, 100)
    B = 100                                                  # ragged on purpose
    x = dev(torch, wl.to_batch_blocks(X, B, ld=128)[0])
    yd = dev(torch, y)
    nets = [gpu.SparseMLP(w.layers, alpha=w.alpha, lr=w.lr, momentum=w.momentum, seed=w.seed, max_batch=128)
            for _ in range(2)]
    # net 0: separate loss kernel + per-layer updates; net 1: train_step (loss written into the output
    # layer, one update launch)
    a = nets[0]
    zL = a.forward(x, B)
    gpu.softmax_ce(zL, yd, B, a.n_classes, a.grad_out, a.loss_sum)
    a.backward(x, B)
    ga = [L.export_grad() for L in a.layers]
    for L in a.layers:
        L.update()
    b = nets[1]
    b.train_step(x, yd, B)
    assert abs(a.loss_sum.item() - b.loss_sum.item()) <= 1e-6 * abs(a.loss_sum.item())
    for La, Lb, (g, gb) in zip(a.layers, b.layers, ga):
        ra, rb = La.export_csr(), Lb.export_csr()
        assert np.array_equal(ra[0], rb[0]) and np.array_equal(ra[1], rb[1])
        for u, v, what in zip(ra[2:], rb[2:], ("val", "vel", "bias", "bias_vel")):
            close(v, u, 1e-6, what)
    # hidden layers see bit-identical dz, so their weights agree bit for bit
    for La, Lb in zip(a.layers[:-1], b.layers[:-1]):
        assert np.array_equal(La.export_csr()[2].view(np.uint32), Lb.export_csr()[2].view(np.uint32))
    # the multi-layer update refuses layers that have no gradient yet
    h = (C.c_void_p * 1)(a.layers[0].handle)
    assert gpu.lib().sparse_layers_update(h, 1, None) == gpu.SL_ESTATE
    assert gpu.lib().sparse_layers_update(h, 0, None) == gpu.SL_EINVAL
    for n in nets:
        n.close()


# ------------------------------------------------------------------------------------------ dropout
@pytest.mark.parametrize("B,linked", [(128, False), (77, True)])
def test_dropout_forward_backward(gpu, oracle, B, linked):
    """Two chained hidden layers with dropout 0.3: identical keep masks (exact zeros in the same
    places), activations and gradients within 1e-4, with and without handing dz to the producer."""
    import torch
    dims, nnz = (300, 500, 400), (4000, 6000)
    rng = np.random.default_rng(B)
    Gs, Os = [], []
    for li in range(2):
        G, O = make_pair(gpu, oracle, dims[li], dims[li + 1], nnz[li], act_kind=1, parity=li % 2, limit=0.3, seed=21,
                         layer_id=li, need_input_grad=(li > 0))
        G.set_dropout(0.3, 11)
        O.set_dropout(0.3, 11)
        Gs.append(G)
        Os.append(O)
    ld = (B + 3) // 4 * 4
    x = rng.standard_normal((dims[0], B)).astype(np.float32)
    ga = rng.standard_normal((dims[2], B)).astype(np.float32)
    a1 = Os[0].forward(x)
    a2 = Os[1].forward(a1)
    g1 = Os[1].backward(a1, ga)
    Os[0].backward(x, g1, need_input_grad=False)
    xd, gad = dev(torch, pad_cols(x, ld)), dev(torch, pad_cols(ga, ld))
    a1d = torch.zeros((dims[1], ld), device="cuda")
    a2d = torch.zeros((dims[2], ld), device="cuda")
    Gs[0].forward(xd, B, a1d)
    Gs[1].forward(a1d, B, a2d)
    if linked:
        Gs[1].link_producer(Gs[0])
        Gs[1].backward(a1d, gad, B, None)
        Gs[0].backward(xd, None, B, None)
    else:
        g1d = torch.zeros((dims[1], ld), device="cuda")
        Gs[1].backward(a1d, gad, B, g1d)
        Gs[0].backward(xd, g1d, B, None)
    for got, ref, O in ((a1d, a1, Os[0]), (a2d, a2, Os[1])):
        got = got.cpu().numpy()[:, :B]
        assert np.array_equal(got == 0, ref == 0) and np.array_equal(ref == 0, O.keep == 0)     # same mask
        assert 0.25 < (ref == 0).mean() < 0.35
        close(got, ref, 1e-4, "activation with dropout")
    for G, O in zip(Gs, Os):
        g, gb = G.export_grad()
        safe = np.abs(O.z).min(axis=1) > 1e-5
        assert safe.mean() > 0.9
        rows = np.repeat(np.arange(O.n_out), np.diff(O.rowptr))
        if O is Os[0]:      # rows of layer 0 also depend on the kink decisions of layer 1 through g1
            pass
        close(g[safe[rows]], O.grad_val[safe[rows]], 2e-4 if O is Os[0] else 1e-4, "grad_val with dropout")
        close(gb[safe], O.grad_bias[safe], 2e-4 if O is Os[0] else 1e-4, "grad_bias with dropout")
    # inference never drops; rate 0 switches dropout off again
    inf = torch.zeros((dims[1], ld), device="cuda")
    Gs[0].infer(xd, B, inf)
    Os[0].set_dropout(0.0, 0)
    close(inf.cpu().numpy()[:, :B], Os[0].forward(x), 1e-4, "inference")
    with pytest.raises(gpu.SparseSetError):
        Gs[0].set_dropout(1.0, 0)
    for G in Gs:
        G.close()


def test_network_training_with_dropout(gpu, oracle):
    """Eight steps of the Madelon-shaped net with dropout 0.3 on the hidden layers (the paper's recipe)."""
    w = wl.WORKLOADS["set_mlp_madelon"]
    net, onet, olayers = run_network(gpu, oracle, w, 8, tol_first=1e-4, tol_end=3e-4, dropout=0.3)
    assert net.step_index == 8 and onet.step_index == 8
    net.close()


# ------------------------------------------------------------------------------------------ end to end
def test_training_learns_and_is_reproducible(gpu):
    """Eight epochs of Algorithm 2 (train, Importance Pruning from epoch 5, prune/regrow) on the
    Madelon-shaped workload: the loss falls, accuracy on the training data beats chance clearly, nnz
    only changes through Importance Pruning, and a second run gives the same bits.  The epochs of
    this workload are only 32 steps long, so a small evolution fraction is used (with zeta = 0.3 and
    so few steps between rewirings the loss does not settle)."""
    import torch
    w = wl.WORKLOADS["set_mlp_madelon"]
    X, y = wl.dataset(w)
    B = w.batch
    blocks = dev(torch, wl.to_batch_blocks(X, B))
    labels = dev(torch, y.reshape(-1, B))
    sizes = [B] * blocks.shape[0]

    def run():
        net = gpu.SparseMLP(w.layers, alpha=w.alpha, lr=w.lr, momentum=w.momentum, seed=w.seed, max_batch=B)
        hist = net.fit(blocks, labels, sizes, 8, 0.02, importance_every=1, importance_start=5, importance_quantile=0.02)
        outs = [torch.zeros_like(a) for a in net.acts]
        correct = 0
        for k in range(blocks.shape[0]):
            z = net.infer(blocks[k], B, outs)
            correct += int((z[:, :B].argmax(dim=0).to(torch.int32) == labels[k]).sum().item())
        state = [L.export_csr() for L in net.layers]
        nnz = [L.nnz for L in net.layers]
        net.close()
        return hist, correct / float(B * blocks.shape[0]), state, nnz

    hist, acc, state, nnz = run()
    assert all(np.isfinite(hist)) and hist[-1] < 0.8 * hist[0], hist
    assert acc > 0.6, acc
    assert nnz[-1] == w.layers[-1].nnz                               # the output layer is never importance-pruned
    assert all(n <= s.nnz for n, s in zip(nnz, w.layers)) and sum(nnz) < sum(s.nnz for s in w.layers)
    hist2, acc2, state2, nnz2 = run()
    assert hist2 == hist and acc2 == acc and nnz2 == nnz
    for a, b in zip(state, state2):
        for u, v in zip(a, b):
            assert np.array_equal(u.view(np.uint32) if u.dtype == np.float32 else u,
                                  v.view(np.uint32) if v.dtype == np.float32 else v)


# ------------------------------------------------------------------------------------------ update fused behind the SDDMM
@pytest.mark.parametrize("n_in,n_out,nnz,B,max_batch,need_gx", [
    (500, 400, 9000, 128, 128, True), (500, 400, 9000, 128, 128, False),      # CSC-ordered and CSR-ordered (first layer)
    (300, 700, 6000, 31, 32, True), (256, 300, 4000, 64, 64, False),          # groups of 8 and 16 lanes, ragged
    (200, 150, 3000, 600, 1024, True), (200, 150, 3000, 1021, 1024, False),   # batch tiles: the update waits for the last one
    (200, 150, 6000, 600, 1024, True),                                        # longer columns: the pair walk
    (6, 2000, 12000, 300, 512, True), (400, 2, 800, 128, 128, True),          # split columns / split rows
    (1500, 2500, 5000, 1000, 1024, True),                                     # very short rows: all tile pairs in one launch
    (3000, 5000, 37, 128, 128, True)])
def test_fused_update_equals_separate_update(gpu, n_in, n_out, nnz, B, max_batch, need_gx):
    """Eq. (1) applied inside the backward kernel (modes 1 and 2) gives the bits of backward followed by the update
    kernel (mode 0): weights, velocities, the CSR copy that forward reads, biases; and mode 2 also stores the
    same gradient."""
    import torch
    rng = np.random.default_rng(nnz + B)
    x = dev(torch, rng.standard_normal((n_in, (B + 3) // 4 * 4)).astype(np.float32))
    ga = dev(torch, rng.standard_normal((n_out, (B + 3) // 4 * 4)).astype(np.float32))
    out = []
    for mode in (0, 1, 2):
        L = gpu.SparseLayer(gpu.make_config(n_in, n_out, nnz=nnz, act_kind=1, act_parity=0, alpha=0.6, init_limit=0.2,
                                            lr=0.01, momentum=0.9, weight_decay=0.01, seed=8, layer_id=1,
                                            max_batch=max_batch, need_input_grad=need_gx))
        rowptr, colidx, val, vel, bias, bias_vel = L.export_csr()
        vel = (np.random.default_rng(1).standard_normal(nnz) * 0.01).astype(np.float32)
        L.import_csr(rowptr, colidx, val, vel, bias, bias_vel)
        L.set_fused_update(mode)
        a = torch.zeros((n_out, x.shape[1]), device="cuda")
        gx = torch.zeros((n_in, x.shape[1]), device="cuda") if need_gx else None
        grads = []
        for step in range(2):                         # the second step reads the weights the first one wrote
            L.forward(x, B, a)
            L.backward(x, ga, B, gx)
            if mode == 1:
                with pytest.raises(gpu.SparseSetError) as e:
                    L.export_grad()
                assert e.value.code == gpu.SL_ESTATE
            else:
                grads.append(L.export_grad())
            with pytest.raises(gpu.SparseSetError):
                L.set_fused_update(0)                 # not between backward and update
            L.update()
        out.append((L.export_csr(), grads, a.cpu().numpy(), None if gx is None else gx.cpu().numpy()))
        L.close()
    ref = out[0]
    for got in out[1:]:
        for u, v in zip(ref[0], got[0]):
            assert np.array_equal(u.view(np.uint32) if u.dtype == np.float32 else u,
                                  v.view(np.uint32) if v.dtype == np.float32 else v)
        assert np.array_equal(ref[2], got[2])
        if need_gx:
            assert np.array_equal(ref[3], got[3])
    for (g0, gb0), (g2, gb2) in zip(ref[1], out[2][1]):
        assert np.array_equal(g0.view(np.uint32), g2.view(np.uint32)) and np.array_equal(gb0.view(np.uint32), gb2.view(np.uint32))
    assert np.abs(ref[0][3]).max() > 0


def test_training_step_with_and_without_fused_update(gpu):
    """The network loop with the update inside the backward kernels against the same loop with the separate
    update launch (the default of train_step): identical bits after several steps, ragged last minibatch included."""
    import torch
    w = wl.WORKLOADS["set_mlp_madelon"]
    X, y = wl.dataset(w, 4 * 128 + 77)
    blocks = dev(torch, wl.to_batch_blocks(X, 128))
    yd = dev(torch, y)
    states = []
    for fused in (0, 1):
        net = gpu.SparseMLP(w.layers, alpha=w.alpha, lr=w.lr, momentum=w.momentum, seed=w.seed, max_batch=128)
        net.fused_update = fused
        for k in range(5):
            B = min(128, X.shape[0] - k * 128)
            net.train_step(blocks[k], yd[k * 128:k * 128 + B], B)
        states.append(([L.export_csr() for L in net.layers], net.loss_sum.item()))
        net.close()
    assert states[0][1] == states[1][1]
    for la, lb in zip(states[0][0], states[1][0]):
        for u, v in zip(la, lb):
            assert np.array_equal(u.view(np.uint32) if u.dtype == np.float32 else u,
                                  v.view(np.uint32) if v.dtype == np.float32 else v)


def test_layers_evolve_together_as_they_do_alone(gpu):
    """sparse_layers_evolve (every layer on a stream and host thread of its own, the default of SparseMLP.evolve)
    against one sparse_layer_evolve call per layer: identical bits in every array of every layer over three trained
    generations and both prune modes; layers that share a scratch buffer are turned away."""
    import ctypes as C
    import torch
    for name, mode in (("set_mlp_madelon", 0), ("set_mlp_fmnist", 1)):
        w = wl.WORKLOADS[name]
        X, y = wl.dataset(w, 3 * w.batch)
        blocks = dev(torch, wl.to_batch_blocks(X, w.batch))
        yd = dev(torch, y)
        states = []
        for shared in (True, False):
            net = gpu.SparseMLP(w.layers, alpha=w.alpha, lr=w.lr, momentum=w.momentum, seed=w.seed, max_batch=w.batch,
                                prune_mode=mode, shared_scratch=shared)
            for gen in (1, 2, 3):
                for k in range(3):
                    net.train_step(blocks[k], yd[k * w.batch:(k + 1) * w.batch], w.batch)
                net.evolve(0.3, gen)
            states.append([L.export_csr() for L in net.layers])
            if shared:   # one buffer under all layers: the concurrent form must refuse
                streams = (C.c_void_p * len(net.layers))(*[None] * len(net.layers))
                rc = gpu.lib().sparse_layers_evolve(net._handles, len(net.layers), 0.3, 9, streams)
                assert rc == gpu.SL_EINVAL
                assert "scratch" in gpu.lib().sparse_layer_last_error(net.layers[1].handle).decode()
                after = [L.export_csr() for L in net.layers]
                for la, lb in zip(states[0], after):
                    assert all(np.array_equal(u, v) for u, v in zip(la, lb))
            net.close()
        for la, lb in zip(*states):
            for u, v in zip(la, lb):
                assert np.array_equal(u.view(np.uint32) if u.dtype == np.float32 else u,
                                      v.view(np.uint32) if v.dtype == np.float32 else v)


# ------------------------------------------------------------------------------------------ sampler window
@pytest.mark.parametrize("n_in,n_out,nnz", [(500, 400, 9000), (100000, 70000, 1700000)])
def test_sampler_window_growth_and_failure(gpu, oracle, n_in, n_out, nnz):
    """A first window far too short for the k positions wanted is doubled until it suffices, and the result is
    still the oracle's sequential definition bit for bit; a window that is not allowed to grow far enough makes
    the call fail and leaves the layer exactly as it was."""
    G, O = make_pair(gpu, oracle, n_in, n_out, nnz, seed=61)
    rng = np.random.default_rng(nnz)
    rowptr, colidx, val, vel, bias, bias_vel = G.export_csr()
    val = (rng.standard_normal(nnz) * 0.1).astype(np.float32)
    vel = (rng.standard_normal(nnz) * 0.01).astype(np.float32)
    G.import_csr(rowptr, colidx, val, vel, bias, bias_vel)
    O.set_state(rowptr, colidx, val, vel, bias, bias_vel)
    before = G.export_csr()
    G.set_sampler_window(16, 64)                              # k is in the thousands: 64 candidates can never do
    with pytest.raises(gpu.SparseSetError) as e:
        G.evolve(0.3, 1)
    assert e.value.code == gpu.SL_ESTATE and "sampler" in str(e.value)
    after = G.export_csr()
    assert all(np.array_equal(a.view(np.uint32) if a.dtype == np.float32 else a,
                              b.view(np.uint32) if b.dtype == np.float32 else b) for a, b in zip(before, after))
    # the layer still works: same forward result as before the failed call would have given, then a good evolution
    G.set_sampler_window(16, 0)                               # sixteen candidates first, then doubling
    O.evolve(0.3, 1)
    G.evolve(0.3, 1)
    assert_same_topology(G, O)
    G.set_sampler_window(0, 0)
    O.evolve(0.3, 2)
    G.evolve(0.3, 2)
    assert_same_topology(G, O)
    G.close()


def test_one_layer_failing_while_the_layers_evolve_together(gpu):
    """sparse_layers_evolve when one layer's cycle fails (its sampler window may not grow): the call reports that
    layer's error, the layer is exactly as it was, and the other layers have completed their own cycle (same bits as
    a network in which nothing failed)."""
    w = wl.WORKLOADS["set_mlp_madelon"]
    nets = [gpu.SparseMLP(w.layers, alpha=w.alpha, lr=w.lr, momentum=w.momentum, seed=w.seed, max_batch=w.batch)
            for _ in range(2)]
    before = nets[0].layers[1].export_csr()
    nets[0].layers[1].set_sampler_window(16, 64)
    with pytest.raises(gpu.SparseSetError) as e:
        nets[0].evolve(0.3, 1)
    assert e.value.code == gpu.SL_ESTATE and "sampler" in str(e.value)
    nets[1].evolve(0.3, 1)
    same = lambda a, b: all(np.array_equal(u.view(np.uint32) if u.dtype == np.float32 else u,
                                           v.view(np.uint32) if v.dtype == np.float32 else v) for u, v in zip(a, b))
    assert same(before, nets[0].layers[1].export_csr())
    for li in (0, 2, 3):
        assert same(nets[0].layers[li].export_csr(), nets[1].layers[li].export_csr())
    nets[0].layers[1].set_sampler_window(0, 0)          # and the layer that failed still evolves afterwards
    nets[0].layers[1].evolve(0.3, 1)
    assert same(nets[0].layers[1].export_csr(), nets[1].layers[1].export_csr())
    for net in nets:
        net.close()


def test_softmax_cross_entropy_label_out_of_range(gpu):
    """A label outside [0, C) (padding, an uninitialised buffer) is never used as an index: the sample adds nothing
    to the loss and its gradient is softmax(z) / B; the labelled samples are untouched by it."""
    import scipy.special
    import torch
    rng = np.random.default_rng(4)
    C, B = 10, 96
    z = (rng.standard_normal((C, B)) * 3).astype(np.float32)
    y = rng.integers(0, C, size=B).astype(np.int32)
    bad = np.array([3, 17, 40, 95])
    y[bad] = [-1, C, 2 ** 31 - 1, -2 ** 31]
    zd = dev(torch, z)
    dzd = torch.zeros((C, B), device="cuda")
    loss = torch.zeros(1, device="cuda")
    gpu.softmax_ce(zd, dev(torch, y), B, C, dzd, loss)
    logp = scipy.special.log_softmax(z.astype(np.float64), axis=0)
    ref = np.exp(logp)
    good = np.setdiff1d(np.arange(B), bad)
    ref[y[good], good] -= 1
    close(dzd.cpu().numpy(), ref / B, 1e-5, "dz")
    assert abs(loss.item() - (-logp[y[good], good].sum())) <= 1e-4 * abs(logp[y[good], good].sum())
