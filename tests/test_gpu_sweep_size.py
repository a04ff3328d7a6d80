"""The single-layer sweep (one 262 144 x 262 144 Erdos-Renyi layer) at its real size: every group width and
kernel path the sweep times is compared with the oracle, all outputs element by element.

  epsilon  B      paths
  1        32     span forward, groups of 8 lanes, chunks of 2
  1        1024   span forward over four batch tiles, pair backward walking all tile pairs in one launch
  16       128    groups of 32 lanes, chunks of 8 (the shape of the 10^6-neuron layers)
  64       32     groups of 8 lanes, long rows
  64       512    two batch tiles, pair backward, 3.4 * 10^7 connections
plus the SDDMM-only form (a first layer, no input gradient) at two of them, and the prune / regrow cycle at
epsilon = 64 from trained-looking weights, bit for bit."""
import numpy as np
import pytest

from paper_2102_01732_amd import workloads as wl
from parity_util import abs_backward, band, close, forward_bounds, kink_delta

pytestmark = pytest.mark.gpu
N = wl.SWEEP_N
_oracle_layers = {}


@pytest.fixture(scope="module")
def gpu():
    import torch
    if not torch.cuda.is_available():
        pytest.skip("no GPU")
    from paper_2102_01732_amd import binding
    binding.lib()
    return binding


def oracle_layer(orc, eps):
    if eps not in _oracle_layers:
        spec = wl.sweep_layer(eps)
        _oracle_layers[eps] = orc.OracleLayer(N, N, spec.nnz, 1, 0, 0.6, spec.init_limit, 0.01, 0.9, 0.0,
                                              wl.DEFAULT_SEED, 0)
    return _oracle_layers[eps]


def gpu_layer(gpu, eps, max_batch, need_gx=True, prune_mode=0):
    spec = wl.sweep_layer(eps)
    return gpu.SparseLayer(gpu.make_config(N, N, nnz=spec.nnz, act_kind=1, act_parity=0, alpha=0.6,
                                           init_limit=spec.init_limit, lr=0.01, momentum=0.9, seed=wl.DEFAULT_SEED,
                                           layer_id=0, max_batch=max_batch, need_input_grad=need_gx,
                                           prune_mode=prune_mode))


@pytest.mark.parametrize("eps,B,need_gx", [(1, 32, True), (1, 1024, True), (16, 128, True), (64, 32, True),
                                           (64, 512, True), (1, 32, False), (64, 512, False)])
def test_sweep_point_against_the_oracle(gpu, oracle, eps, B, need_gx):
    import torch
    O = oracle_layer(oracle, eps)
    G = gpu_layer(gpu, eps, B, need_gx)
    rowptr, colidx, val, _, _, _ = G.export_csr()
    assert np.array_equal(rowptr, O.rowptr) and np.array_equal(colidx, O.colidx)
    assert np.array_equal(val.view(np.uint32), O.val.view(np.uint32))
    x = wl.dense_operand(N, B, 5)
    ga = wl.dense_operand(N, B, 6)
    print(f"eps {eps} B {B}: oracle forward/backward ...", flush=True)
    a_ref = O.forward(x)
    gx_ref = O.backward(x, ga, need_input_grad=need_gx)
    mag_z, err_z = forward_bounds(oracle, O, np.abs(x), None)
    in_band = band(O, err_z)
    allow_dz = kink_delta(O, in_band, np.abs(ga), np.zeros_like(ga))
    mg, mgb, mgx = abs_backward(oracle, O, x, O.dz, need_input_grad=need_gx)
    ag, agb, agx = abs_backward(oracle, O, x, allow_dz, need_input_grad=need_gx)
    print(f"eps {eps} B {B}: {int(in_band.sum())} pre-activations in the rounding band of the kink; GPU ...", flush=True)
    xd, gad = torch.from_numpy(x).cuda(), torch.from_numpy(ga).cuda()
    ad = torch.empty_like(xd)
    gxd = torch.empty_like(xd) if need_gx else None
    G.forward(xd, B, ad)
    G.backward(xd, gad, B, gxd)
    g, gb = G.export_grad()
    worst = close(ad.cpu().numpy(), a_ref, 1e-4, "a", mag=mag_z)
    tally = {}
    worst = max(worst, close(g, O.grad_val, 1e-4, "grad_val", mag=mg, allow=ag, tally=tally))
    worst = max(worst, close(gb, O.grad_bias, 1e-4, "grad_bias", mag=mgb, allow=agb, tally=tally))
    if need_gx:
        worst = max(worst, close(gxd.cpu().numpy(), gx_ref, 1e-4, "grad_x", mag=mgx, allow=agx, tally=tally))
    # the band is a worst-case bound: all but a sliver of the elements meet 1e-4 without any kink allowance
    assert tally["needed"] <= 1e-3 * tally["checked"], tally
    print(f"eps {eps} B {B}: largest error / allowed = {worst:.4f}", flush=True)
    G.close()


@pytest.mark.parametrize("mode", [0, 1])
def test_evolution_at_the_densest_sweep_point(gpu, oracle, mode):
    """epsilon = 64: 3.4 * 10^7 connections with trained-looking weights (ties and zeros included) and non-zero
    velocities go through one prune / regrow cycle on both sides; pattern, weights and velocities agree bit for bit."""
    eps = 64
    base = oracle_layer(oracle, eps)
    O = oracle.OracleLayer.__new__(oracle.OracleLayer)
    O.__dict__.update(base.__dict__)
    O.prune_mode = mode
    nnz = base.nnz
    rng = np.random.default_rng(640 + mode)
    val = (rng.standard_normal(nnz) * 0.1).astype(np.float32)
    val[rng.integers(0, nnz, size=nnz // 10)] = np.float32(0.03125)
    val[rng.integers(0, nnz, size=nnz // 20)] = np.float32(-0.03125)
    val[rng.integers(0, nnz, size=50)] = 0.0
    vel = (rng.standard_normal(nnz) * 0.01).astype(np.float32)
    bias = np.zeros(N, np.float32)
    O.set_state(base.rowptr, base.colidx, val, vel, bias, bias)
    G = gpu_layer(gpu, eps, 32, True, prune_mode=mode)
    G.import_csr(base.rowptr, base.colidx, val, vel, bias, bias)
    print(f"mode {mode}: oracle evolve ...", flush=True)
    k = O.evolve(0.3, 1)
    G.evolve(0.3, 1)
    rowptr, colidx, gval, gvel, _, _ = G.export_csr()
    assert G.nnz == nnz and abs(k - 0.3 * nnz) <= 1
    assert np.array_equal(rowptr, O.rowptr) and np.array_equal(colidx, O.colidx)
    assert np.array_equal(gval.view(np.uint32), O.val.view(np.uint32))
    assert np.array_equal(gvel.view(np.uint32), O.vel.view(np.uint32))
    G.close()
