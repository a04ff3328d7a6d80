"""Minibatch-by-minibatch parity in which NO value of the GPU ever reaches the oracle.

The oracle trains freely.  Before every minibatch its state (pattern, weights, velocities, biases) is imported
into the GPU network, both sides take the same training step, and activations, gradients, and the updated
weights, velocities and biases are compared at the one-step tolerance, element by element.  Where a
pre-activation lies in the rounding band of eq. (3)'s kink (see parity_util; decided from oracle values only), the
elements its delta reaches get the corresponding allowance on top of the tolerance."""
import numpy as np

from paper_2102_01732_amd import workloads as wl
from parity_util import abs_backward, band, close, forward_bounds, kink_delta, slope_magnitude


def make_oracle_net(orc, w):
    olayers = [orc.OracleLayer(s.n_in, s.n_out, s.nnz, s.act_kind, s.act_parity, w.alpha, s.init_limit, w.lr,
                               w.momentum, 0.0, w.seed, s.layer_id) for s in w.layers]
    return orc.OracleMLP(olayers), olayers


def run_stepwise_oracle_only(gpu, orc, w, n_steps, tol=1e-4, net=None, oracle_net=None, log=print, first_step=0,
                             oracle_logits=False):
    """Minibatches first_step .. n_steps-1 (pass the same `net` and `oracle_net` to continue an earlier call).

    oracle_logits: after the GPU's forward pass (whose activations and logits are compared as always) the ORACLE's
    logits replace the GPU's before the loss is taken.  Needed where the softmax is ill-conditioned: the
    10^6-neuron network's logits are sums of a million terms and reach thousands, so a rounding difference that is
    1e-6 of such a sum can move a probability by O(1) when two logits happen to be close, and with it that sample's
    whole backward pass -- a property of the workload, not of either implementation."""
    import torch
    X, y = wl.dataset(w, n_steps * w.batch)
    blocks = wl.to_batch_blocks(X, w.batch)
    if net is None:
        net = gpu.SparseMLP(w.layers, alpha=w.alpha, lr=w.lr, momentum=w.momentum, seed=w.seed, max_batch=w.batch)
    onet, olayers = oracle_net if oracle_net is not None else make_oracle_net(orc, w)
    yd = torch.from_numpy(y).cuda()
    n_layers = len(olayers)
    bands, mags = [None] * n_layers, [None] * n_layers
    chain = {}

    def hook(li, layer, a):
        if li == 0:
            chain["mag"], chain["err"] = np.abs(onet.acts[0]), None     # the inputs are the same bits on both sides
        mags[li], chain["err"] = forward_bounds(orc, layer, chain["mag"], chain["err"])
        chain["mag"] = mags[li]
        bands[li] = band(layer, chain["err"])
        return a

    onet.after_forward = hook
    stats = dict(steps=0, band=0, worst=0.0, tally=[dict(checked=0, needed=0) for _ in range(n_layers)])
    for k in range(first_step, n_steps):
        B = min(w.batch, X.shape[0] - k * w.batch)
        xs, ys = blocks[k][:, :B], y[k * w.batch:k * w.batch + B]
        for G, O in zip(net.layers, olayers):
            G.import_csr(O.rowptr, O.colidx, O.val, O.vel, O.bias, O.bias_vel)
        before = [(O.val.copy(), O.vel.copy(), O.bias.copy(), O.bias_vel.copy()) for O in olayers]
        loss_ref = onet.train_step(xs, ys)
        got = {}

        def read(model):
            got["grads"] = [L.export_grad() for L in model.layers]

        def after_forward(model):
            got["acts"] = [a[:, :B].cpu().numpy() for a in model.acts]
            if oracle_logits:
                model.acts[-1][:, :B] = torch.from_numpy(onet.acts[-1]).to(model.acts[-1].device)

        net.loss_sum.zero_()
        net.train_step(torch.from_numpy(np.ascontiguousarray(blocks[k])).cuda(), yd[k * w.batch:k * w.batch + B], B,
                       before_update=read, after_forward=after_forward)
        loss = net.loss_sum.item() / B
        assert abs(loss - loss_ref) <= tol * max(abs(loss_ref), 1e-30), f"step {k}: loss {loss} vs {loss_ref}"
        stats["band"] += int(sum(b.sum() for b in bands))
        worst = 0.0
        top = olayers[-1]
        mag_dz = np.abs(top.dz)                      # magnitude bound of every delta, layer by layer
        allow_dz = np.zeros_like(mag_dz)             # how far a correct delta may lie from the oracle's (kink)
        for li in range(n_layers - 1, -1, -1):
            G, O = net.layers[li], olayers[li]
            tag = f"step {k} layer {li}"
            # a = f(z) is continuous at the kink: every activation is compared without allowance
            worst = max(worst, close(got["acts"][li], onet.acts[li + 1], tol, tag + " activations", mag=mags[li]))
            x_mag = np.abs(onet.acts[0]) if li == 0 else mags[li - 1]
            val0, vel0, bias0, bvel0 = before[li]                # the backward pass saw the weights before the update
            mg, mgb, mgx = abs_backward(orc, O, x_mag, mag_dz, need_input_grad=li > 0, val=val0)
            if allow_dz.any():
                ag, agb, agx = abs_backward(orc, O, x_mag, allow_dz, need_input_grad=li > 0, val=val0)
            else:
                ag, agb = np.zeros_like(mg), np.zeros_like(mgb)
                agx = np.zeros_like(mgx) if mgx is not None else None
            g, gb = got["grads"][li]
            worst = max(worst, close(g, O.grad_val, tol, tag + " weight gradient", mag=mg, allow=ag, tally=stats["tally"][li]))
            worst = max(worst, close(gb, O.grad_bias, tol, tag + " bias gradient", mag=mgb, allow=agb, tally=stats["tally"][li]))
            _, _, val, vel, bias, bias_vel = G.export_csr()
            lr = float(O.lr)
            worst = max(worst, close(vel, O.vel, tol, tag + " velocities", mag=np.abs(vel0) + lr * mg, allow=lr * ag))
            worst = max(worst, close(val, O.val, tol, tag + " weights", mag=np.abs(val0) + np.abs(vel0) + lr * mg,
                                     allow=lr * ag))
            worst = max(worst, close(bias_vel, O.bias_vel, tol, tag + " bias velocities", mag=np.abs(bvel0) + lr * mgb,
                                     allow=lr * agb))
            worst = max(worst, close(bias, O.bias, tol, tag + " biases", mag=np.abs(bias0) + np.abs(bvel0) + lr * mgb,
                                     allow=lr * agb))
            if li > 0:
                below = olayers[li - 1]
                allow_dz = kink_delta(below, bands[li - 1], mgx, agx)
                slope = slope_magnitude(below)
                slope[bands[li - 1]] = 1.0                 # in the band either branch may have been taken
                mag_dz = mgx * slope
        stats["steps"] += 1
        stats["worst"] = max(stats["worst"], worst)
        if log and (k % 50 == 0 or k == n_steps - 1):
            needed = sum(t["needed"] for t in stats["tally"])
            log(f"{w.name}: step {k}: loss {loss_ref:.6g}, {stats['band']} pre-activations in the band so far, "
                f"{needed} gradient elements needed their kink allowance, largest error / allowed = {stats['worst']:.3f}",
                flush=True)
    onet.after_forward = None
    return net, onet, olayers, stats
