"""Whole epochs of the three small networks, minibatch by minibatch, with the oracle training on its own: before
every minibatch the ORACLE's state goes into the GPU network, both take the step, and everything the step
produces is compared at 1e-4 (see stepwise.py).  No value computed on the GPU reaches the oracle."""
import numpy as np
import pytest

from paper_2102_01732_amd import workloads as wl
from stepwise import run_stepwise_oracle_only

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def gpu():
    import torch
    if not torch.cuda.is_available():
        pytest.skip("no GPU")
    from paper_2102_01732_amd import binding
    binding.lib()
    return binding


@pytest.mark.parametrize("name", ["set_mlp_madelon", "set_mlp_fmnist", "set_mlp_cifar"])
def test_every_minibatch_of_an_epoch_from_the_oracles_state(gpu, oracle, name):
    w = wl.WORKLOADS[name]
    net, onet, olayers, stats = run_stepwise_oracle_only(gpu, oracle, w, w.steps_per_epoch)
    assert stats["steps"] == w.steps_per_epoch
    # The band is a worst-case bound, so nearly all pre-activations in it still take the oracle's branch: all but a
    # sliver of the gradient elements must meet the plain 1e-4 bound without any kink allowance.
    for t in stats["tally"]:
        assert t["needed"] <= 0.002 * t["checked"], stats
    # then the evolution of Algorithm 2, from the oracle's trained state on both sides
    for G, O in zip(net.layers, olayers):
        G.import_csr(O.rowptr, O.colidx, O.val, O.vel, O.bias, O.bias_vel)
    net.evolve(w.zeta, 1)
    onet.evolve(w.zeta, 1)
    for G, O in zip(net.layers, olayers):
        rowptr, colidx, val, vel, _, _ = G.export_csr()
        assert np.array_equal(rowptr, O.rowptr) and np.array_equal(colidx, O.colidx)
        assert np.array_equal(val.view(np.uint32), O.val.view(np.uint32))
        assert np.array_equal(vel.view(np.uint32), O.vel.view(np.uint32))
    net.close()
