"""ctypes binding of libsparse_set.so: argument marshalling only.

Every step of the training path runs in the library's HIP kernels; torch is used for device
buffers and for the current stream handle.  There is no CPU fallback: ``lib()`` raises if the
shared library has not been built (``python -m paper_2102_01732_amd.build``).
"""
from __future__ import annotations

import ctypes as C
import os
from typing import List, Optional, Sequence

import numpy as np
import torch

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libsparse_set.so")
_lib = None

SL_OK, SL_EINVAL, SL_ESTATE, SL_ENOMEM, SL_EHIP, SL_EOVERFLOW = 0, -1, -2, -3, -4, -5
SL_FLAG_NEED_INPUT_GRAD = 1

EXPORTS = [
    "sparse_layer_query_sizes", "sparse_layer_init", "sparse_layer_forward", "sparse_layer_backward",
    "sparse_layer_update", "sparse_layer_evolve", "sparse_layer_destroy", "sparse_loss_softmax_ce",
    "sparse_layer_nnz", "sparse_layer_export_csr", "sparse_layer_import_csr", "sparse_layer_export_grad",
    "sparse_layer_set_lr", "sparse_layer_last_error", "sparse_layer_profile_begin", "sparse_layer_profile_end",
    "sparse_kernel_name", "sparse_layer_link_producer", "sparse_layer_importance", "sparse_layer_importance_prune",
    "sparse_layer_infer", "sparse_layers_average_query", "sparse_layers_average",
    "sparse_loss_softmax_ce_into", "sparse_layers_update", "sparse_layer_set_dropout",
    "sparse_layer_retain_valid_updates", "sparse_layer_infer_static",
    "sparse_layer_set_fused_update", "sparse_layer_set_sampler_window", "sparse_layers_evolve",
]
N_KERNEL_IDS = 7


class SlConfig(C.Structure):
    _fields_ = [
        ("n_in", C.c_int64), ("n_out", C.c_int64), ("epsilon", C.c_double), ("nnz_override", C.c_int64),
        ("act_kind", C.c_int32), ("act_parity", C.c_int32), ("alpha", C.c_float), ("init_limit", C.c_float),
        ("lr", C.c_float), ("momentum", C.c_float), ("weight_decay", C.c_float), ("seed", C.c_uint64),
        ("layer_id", C.c_uint32), ("max_batch", C.c_int32), ("prune_mode", C.c_int32), ("flags", C.c_uint32),
    ]


class SparseSetError(RuntimeError):
    def __init__(self, code: int, where: str, text: str = ""):
        super().__init__(f"{where} failed with code {code}" + (f": {text}" if text else ""))
        self.code = code


def lib():
    """Loads libsparse_set.so; raises if it is missing (there is no other implementation)."""
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise RuntimeError(f"{LIB_PATH} not found: build it with `python -m paper_2102_01732_amd.build`")
        L = C.CDLL(LIB_PATH)
        vp, i64, i32, f32p, i32p = C.c_void_p, C.c_int64, C.c_int32, C.c_void_p, C.c_void_p
        L.sparse_layer_query_sizes.argtypes = [C.POINTER(SlConfig), C.POINTER(C.c_size_t), C.POINTER(C.c_size_t)]
        L.sparse_layer_init.argtypes = [C.POINTER(SlConfig), vp, C.c_size_t, vp, C.c_size_t, vp, C.POINTER(vp)]
        L.sparse_layer_forward.argtypes = [vp, f32p, i64, i32, f32p, i64, vp]
        L.sparse_layer_infer.argtypes = [vp, f32p, i64, i32, f32p, i64, vp]
        L.sparse_layer_infer_static.argtypes = [vp, f32p, i64, i32, f32p, i64, vp]
        L.sparse_layer_backward.argtypes = [vp, f32p, i64, f32p, i64, i32, f32p, i64, vp]
        L.sparse_layer_update.argtypes = [vp, vp]
        L.sparse_layer_set_fused_update.argtypes = [vp, i32]
        L.sparse_layer_set_sampler_window.argtypes = [vp, i64, i64]
        L.sparse_layer_evolve.argtypes = [vp, C.c_double, C.c_uint64, vp]
        L.sparse_layer_destroy.argtypes = [vp]
        L.sparse_loss_softmax_ce.argtypes = [f32p, i64, i32p, i32, i32, f32p, i64, f32p, vp]
        L.sparse_layer_nnz.argtypes = [vp, C.POINTER(i64)]
        L.sparse_layer_export_csr.argtypes = [vp, vp, vp, vp, vp, vp, vp]
        L.sparse_layer_import_csr.argtypes = [vp, vp, vp, vp, vp, vp, vp]
        L.sparse_layer_export_grad.argtypes = [vp, vp, vp]
        L.sparse_layer_set_lr.argtypes = [vp, C.c_float]
        L.sparse_layer_last_error.argtypes = [vp]
        L.sparse_layer_last_error.restype = C.c_char_p
        L.sparse_layer_link_producer.argtypes = [vp, vp]
        L.sparse_layers_average_query.argtypes = [i64, C.POINTER(C.c_size_t)]
        L.sparse_layers_average.argtypes = [vp, C.POINTER(vp), i32, vp, C.c_size_t, vp]
        L.sparse_loss_softmax_ce_into.argtypes = [vp, f32p, i64, i32p, i32, f32p, vp]
        L.sparse_layers_update.argtypes = [C.POINTER(vp), i32, vp]
        L.sparse_layers_evolve.argtypes = [C.POINTER(vp), i32, C.c_double, C.c_uint64, C.POINTER(vp)]
        L.sparse_layer_set_dropout.argtypes = [vp, C.c_float, C.c_uint64]
        L.sparse_layer_importance.argtypes = [vp, vp]
        L.sparse_layer_retain_valid_updates.argtypes = [vp, i32p, i32p, f32p, i64, f32p, vp]
        L.sparse_layer_importance_prune.argtypes = [vp, C.c_float, C.POINTER(i64), vp]
        L.sparse_layer_profile_begin.argtypes = [vp]
        L.sparse_layer_profile_end.argtypes = [vp, vp, vp, i32]
        L.sparse_kernel_name.argtypes = [i32]
        L.sparse_kernel_name.restype = C.c_char_p
        for name in EXPORTS:
            if name not in ("sparse_layer_last_error", "sparse_kernel_name"):
                getattr(L, name).restype = C.c_int
        _lib = L
    return _lib


def make_config(n_in, n_out, *, epsilon=0.0, nnz=-1, act_kind=1, act_parity=0, alpha=0.6, init_limit=0.1, lr=0.01,
                momentum=0.9, weight_decay=0.0, seed=0, layer_id=0, max_batch=128, prune_mode=0,
                need_input_grad=True) -> SlConfig:
    return SlConfig(n_in, n_out, float(epsilon), int(nnz), act_kind, act_parity, float(alpha), float(init_limit),
                    float(lr), float(momentum), float(weight_decay), int(seed), int(layer_id), int(max_batch),
                    int(prune_mode), SL_FLAG_NEED_INPUT_GRAD if need_input_grad else 0)


def query_sizes(cfg: SlConfig):
    sb, cb = C.c_size_t(0), C.c_size_t(0)
    rc = lib().sparse_layer_query_sizes(C.byref(cfg), C.byref(sb), C.byref(cb))
    if rc != SL_OK:
        raise SparseSetError(rc, "sparse_layer_query_sizes")
    return sb.value, cb.value


def _stream() -> int:
    return torch.cuda.current_stream().cuda_stream


def _ptr(t: Optional[torch.Tensor]):
    return None if t is None else t.data_ptr()


class SparseLayer:
    """One sparse layer living in caller-owned torch buffers."""

    def __init__(self, cfg: SlConfig, device="cuda:0", scratch: Optional[torch.Tensor] = None):
        self.cfg = cfg
        self.device = torch.device(device)
        sb, cb = query_sizes(cfg)
        self.state = torch.empty(sb + 256, dtype=torch.uint8, device=self.device)
        if scratch is None or scratch.numel() < cb:
            scratch = torch.empty(cb + 256, dtype=torch.uint8, device=self.device)
        self.scratch = scratch
        assert self.state.data_ptr() % 256 == 0 and self.scratch.data_ptr() % 256 == 0
        self.handle = C.c_void_p(None)
        rc = lib().sparse_layer_init(C.byref(cfg), self.state.data_ptr(), self.state.numel(), self.scratch.data_ptr(),
                                     self.scratch.numel(), _stream(), C.byref(self.handle))
        if rc != SL_OK:
            raise SparseSetError(rc, "sparse_layer_init")
        n = C.c_int64(0)
        lib().sparse_layer_nnz(self.handle, C.byref(n))
        self.nnz = n.value
        self.n_in, self.n_out = cfg.n_in, cfg.n_out

    def _check(self, rc: int, where: str):
        if rc != SL_OK:
            raise SparseSetError(rc, where, lib().sparse_layer_last_error(self.handle).decode())

    def forward(self, x: torch.Tensor, B: int, a: torch.Tensor):
        self._check(lib().sparse_layer_forward(self.handle, x.data_ptr(), x.stride(0), B, a.data_ptr(), a.stride(0),
                                               _stream()), "sparse_layer_forward")

    def infer(self, x: torch.Tensor, B: int, a: torch.Tensor):
        self._check(lib().sparse_layer_infer(self.handle, x.data_ptr(), x.stride(0), B, a.data_ptr(), a.stride(0),
                                             _stream()), "sparse_layer_infer")

    def infer_static(self, x: torch.Tensor, B: int, a: torch.Tensor):
        self._check(lib().sparse_layer_infer_static(self.handle, x.data_ptr(), x.stride(0), B, a.data_ptr(), a.stride(0),
                                                    _stream()), "sparse_layer_infer_static")

    def set_dropout(self, p: float, step: int):
        self._check(lib().sparse_layer_set_dropout(self.handle, float(p), int(step)), "sparse_layer_set_dropout")

    def link_producer(self, producer: Optional["SparseLayer"]):
        self._check(lib().sparse_layer_link_producer(self.handle, producer.handle if producer else None),
                    "sparse_layer_link_producer")
        self._producer = producer      # keeps the producer alive as long as the link

    def backward(self, x: torch.Tensor, grad_a: Optional[torch.Tensor], B: int, grad_x: Optional[torch.Tensor]):
        self._check(lib().sparse_layer_backward(self.handle, x.data_ptr(), x.stride(0), _ptr(grad_a),
                                                grad_a.stride(0) if grad_a is not None else 0, B, _ptr(grad_x),
                                                grad_x.stride(0) if grad_x is not None else 0, _stream()),
                    "sparse_layer_backward")

    def update(self):
        self._check(lib().sparse_layer_update(self.handle, _stream()), "sparse_layer_update")

    def set_fused_update(self, mode: int):
        """0: backward stores the gradient, update applies eq. (1); 1: backward applies it to the connections itself
        (gradient not stored), update finishes the biases; 2: as 1, gradient stored as well."""
        self._check(lib().sparse_layer_set_fused_update(self.handle, int(mode)), "sparse_layer_set_fused_update")

    def evolve(self, zeta: float, generation: int):
        self._check(lib().sparse_layer_evolve(self.handle, float(zeta), int(generation), _stream()),
                    "sparse_layer_evolve")

    def set_sampler_window(self, first_window: int = 0, max_window: int = 0):
        self._check(lib().sparse_layer_set_sampler_window(self.handle, int(first_window), int(max_window)),
                    "sparse_layer_set_sampler_window")

    def retain_valid_updates(self, old_rowptr: torch.Tensor, old_colidx: torch.Tensor, old_grad: torch.Tensor,
                             old_grad_bias: torch.Tensor):
        """Device tensors: int32 CSR pattern of an older topology, its gradient in that order, the bias gradient."""
        assert old_rowptr.dtype == torch.int32 and old_colidx.dtype == torch.int32 and old_rowptr.numel() == self.n_out + 1
        assert old_grad.dtype == torch.float32 and old_grad.numel() == old_colidx.numel()
        assert old_grad_bias.dtype == torch.float32 and old_grad_bias.numel() == self.n_out
        assert all(t.is_cuda and t.is_contiguous() for t in (old_rowptr, old_colidx, old_grad, old_grad_bias))
        self._check(lib().sparse_layer_retain_valid_updates(self.handle, old_rowptr.data_ptr(), old_colidx.data_ptr(),
                                                            old_grad.data_ptr(), old_colidx.numel(),
                                                            old_grad_bias.data_ptr(), _stream()),
                    "sparse_layer_retain_valid_updates")

    def importance(self) -> np.ndarray:
        out = np.zeros(self.n_out, np.float32)
        self._check(lib().sparse_layer_importance(self.handle, out.ctypes.data), "sparse_layer_importance")
        return out

    def importance_prune(self, threshold: float) -> int:
        removed = C.c_int64(0)
        self._check(lib().sparse_layer_importance_prune(self.handle, float(threshold), C.byref(removed), _stream()),
                    "sparse_layer_importance_prune")
        self.nnz -= removed.value
        return removed.value

    def set_lr(self, lr: float):
        self._check(lib().sparse_layer_set_lr(self.handle, float(lr)), "sparse_layer_set_lr")

    def export_csr(self):
        rowptr = np.zeros(self.n_out + 1, np.int32)
        colidx = np.zeros(max(self.nnz, 1), np.int32)
        val = np.zeros(max(self.nnz, 1), np.float32)
        vel = np.zeros(max(self.nnz, 1), np.float32)
        bias = np.zeros(self.n_out, np.float32)
        bias_vel = np.zeros(self.n_out, np.float32)
        self._check(lib().sparse_layer_export_csr(self.handle, rowptr.ctypes.data, colidx.ctypes.data, val.ctypes.data,
                                                  vel.ctypes.data, bias.ctypes.data, bias_vel.ctypes.data),
                    "sparse_layer_export_csr")
        n = self.nnz
        return rowptr, colidx[:n], val[:n], vel[:n], bias, bias_vel

    def import_csr(self, rowptr, colidx, val, vel=None, bias=None, bias_vel=None):
        arrs = [np.ascontiguousarray(rowptr, np.int32), np.ascontiguousarray(colidx, np.int32),
                np.ascontiguousarray(val, np.float32)]
        opt = [None if a is None else np.ascontiguousarray(a, np.float32) for a in (vel, bias, bias_vel)]
        self._check(lib().sparse_layer_import_csr(self.handle, *[a.ctypes.data for a in arrs],
                                                  *[None if a is None else a.ctypes.data for a in opt]),
                    "sparse_layer_import_csr")

    def export_grad(self):
        g = np.zeros(max(self.nnz, 1), np.float32)
        gb = np.zeros(self.n_out, np.float32)
        self._check(lib().sparse_layer_export_grad(self.handle, g.ctypes.data, gb.ctypes.data),
                    "sparse_layer_export_grad")
        return g[: self.nnz], gb

    def profile_begin(self):
        self._check(lib().sparse_layer_profile_begin(self.handle), "sparse_layer_profile_begin")

    def profile_end(self):
        """{kernel name: (launches, total ms)} since profile_begin."""
        n = (C.c_int32 * N_KERNEL_IDS)()
        ms = (C.c_float * N_KERNEL_IDS)()
        self._check(lib().sparse_layer_profile_end(self.handle, n, ms, N_KERNEL_IDS), "sparse_layer_profile_end")
        return {lib().sparse_kernel_name(i).decode(): (n[i], ms[i]) for i in range(N_KERNEL_IDS) if n[i]}

    def close(self):
        if self.handle:
            lib().sparse_layer_destroy(self.handle)
            self.handle = C.c_void_p(None)

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass


def average_layers(dst: SparseLayer, replicas: Sequence[SparseLayer]):
    """dst <- sparse average of the replicas (eq. 2), re-pruned by magnitude to dst's number of connections."""
    total = sum(r.nnz for r in replicas)
    need = C.c_size_t(0)
    rc = lib().sparse_layers_average_query(total, C.byref(need))
    if rc != SL_OK:
        raise SparseSetError(rc, "sparse_layers_average_query")
    scratch = torch.empty(need.value + 256, dtype=torch.uint8, device=dst.device)
    arr = (C.c_void_p * len(replicas))(*[r.handle for r in replicas])
    dst._check(lib().sparse_layers_average(dst.handle, arr, len(replicas), scratch.data_ptr(), scratch.numel(),
                                           _stream()), "sparse_layers_average")
    n = C.c_int64(0)
    lib().sparse_layer_nnz(dst.handle, C.byref(n))
    dst.nnz = n.value


def softmax_ce(z: torch.Tensor, y: torch.Tensor, B: int, n_classes: int, dz: torch.Tensor,
               loss_sum: Optional[torch.Tensor] = None):
    rc = lib().sparse_loss_softmax_ce(z.data_ptr(), z.stride(0), y.data_ptr(), B, n_classes, dz.data_ptr(),
                                      dz.stride(0), _ptr(loss_sum), _stream())
    if rc != SL_OK:
        raise SparseSetError(rc, "sparse_loss_softmax_ce")


class SparseMLP:
    """Chain of sparse layers + softmax cross-entropy: the training loop of Algorithm 2 (train for
    an epoch of minibatches, then prune and regrow every sparse layer).  Only calls into the
    library; activations and gradients are preallocated feature-major buffers [n][ld]."""

    def __init__(self, layer_specs: Sequence, *, alpha: float, lr: float, momentum: float, seed: int, max_batch: int,
                 prune_mode: int = 0, weight_decay: float = 0.0, device="cuda:0", shared_scratch: bool = False):
        """shared_scratch: one scratch buffer (the largest layer's) serves all layers and `evolve` takes the
        layers one after the other; by default every layer has its own and they evolve concurrently."""
        self.device = torch.device(device)
        self.max_batch = max_batch
        self.ld = (max_batch + 31) // 32 * 32
        cfgs = [make_config(s.n_in, s.n_out, nnz=s.nnz, act_kind=s.act_kind, act_parity=s.act_parity, alpha=alpha,
                            init_limit=s.init_limit, lr=lr, momentum=momentum, weight_decay=weight_decay, seed=seed,
                            layer_id=s.layer_id, max_batch=max_batch, prune_mode=prune_mode,
                            need_input_grad=(li > 0)) for li, s in enumerate(layer_specs)]
        self.shared_scratch = shared_scratch
        if shared_scratch:
            scratch_bytes = max(query_sizes(c)[1] for c in cfgs)
            self.scratch = torch.empty(scratch_bytes + 256, dtype=torch.uint8, device=self.device)
            self.layers: List[SparseLayer] = [SparseLayer(c, device, self.scratch) for c in cfgs]
        else:
            self.layers = [SparseLayer(c, device) for c in cfgs]
            self._evolve_streams = [torch.cuda.Stream(device=self.device) for _ in cfgs]
        self.acts = [torch.zeros((s.n_out, self.ld), dtype=torch.float32, device=self.device) for s in layer_specs]
        # Layers are chained: each backward hands dz to the layer below inside its own kernel, so only
        # the output layer needs a gradient buffer.
        for li in range(1, len(self.layers)):
            self.layers[li].link_producer(self.layers[li - 1])
        self.grad_out = torch.zeros((layer_specs[-1].n_out, self.ld), dtype=torch.float32, device=self.device)
        self._handles = (C.c_void_p * len(self.layers))(*[l.handle for l in self.layers])
        self.loss_sum = torch.zeros(1, dtype=torch.float32, device=self.device)
        self.n_classes = layer_specs[-1].n_out
        self.fused_update = 0       # train_step: 0 = one update launch for all layers (faster, see set_fused_update), 1 = eq. (1) inside the backward kernels
        self._fuse_mode = 0
        self.dropout = 0.0          # rate applied to the hidden layers by train_step (0 = off)
        self.step_index = 0         # selects the dropout masks; advanced by train_step

    def forward(self, x: torch.Tensor, B: int) -> torch.Tensor:
        cur = x
        for layer, a in zip(self.layers, self.acts):
            layer.forward(cur, B, a)
            cur = a
        return cur

    def infer(self, x: torch.Tensor, B: int, outs: Sequence[torch.Tensor]) -> torch.Tensor:
        """Forward only, into caller-provided activation buffers (B may differ from training)."""
        cur = x
        for layer, a in zip(self.layers, outs):
            layer.infer(cur, B, a)
            cur = a
        return cur

    def backward(self, x: torch.Tensor, B: int):
        """Backward through all layers; self.grad_out must hold dLoss/dz of the output layer."""
        last = len(self.layers) - 1
        for li in range(last, -1, -1):
            xin = x if li == 0 else self.acts[li - 1]
            self.layers[li].backward(xin, self.grad_out if li == last else None, B, None)

    def train_step(self, x: torch.Tensor, y: torch.Tensor, B: int, before_update=None, after_forward=None):
        """x [n_in][ld>=B] feature-major, y int32 [B].  Forward, loss written into the output layer,
        chained backward, one update launch for all layers.  `before_update(self)`, if given, runs between
        the backward pass and the update (the gradients can be read with SparseLayer.export_grad there);
        `after_forward(self)` runs between the forward pass and the loss (self.acts[-1] holds the logits there)."""
        if self.dropout > 0.0:
            for layer in self.layers[:-1]:
                layer.set_dropout(self.dropout, self.step_index)
        self.step_index += 1
        # with fused_update = 1 eq. (1) is applied inside the backward kernels, unless somebody wants to look at the gradients first
        mode = self.fused_update if before_update is None else 0
        if mode != self._fuse_mode:
            for layer in self.layers:
                layer.set_fused_update(mode)
            self._fuse_mode = mode
        zL = self.forward(x, B)
        if after_forward is not None:
            after_forward(self)
        last = self.layers[-1]
        last._check(lib().sparse_loss_softmax_ce_into(last.handle, zL.data_ptr(), zL.stride(0), y.data_ptr(), B,
                                                      self.loss_sum.data_ptr(), _stream()), "sparse_loss_softmax_ce_into")
        n = len(self.layers)
        for li in range(n - 1, -1, -1):
            self.layers[li].backward(x if li == 0 else self.acts[li - 1], None, B, None)
        if before_update is not None:
            before_update(self)
        last._check(lib().sparse_layers_update(self._handles, n, _stream()), "sparse_layers_update")

    def evolve(self, zeta: float, generation: int):
        if self.shared_scratch or len(self.layers) == 1:
            for layer in self.layers:
                layer.evolve(zeta, generation)
            return
        cur = torch.cuda.current_stream()
        for st in self._evolve_streams:
            st.wait_stream(cur)
        streams = (C.c_void_p * len(self.layers))(*[st.cuda_stream for st in self._evolve_streams])
        rc = lib().sparse_layers_evolve(self._handles, len(self.layers), float(zeta), int(generation), streams)
        if rc != SL_OK:   # the layer that failed holds the message
            msgs = [lib().sparse_layer_last_error(l.handle).decode() for l in self.layers]
            raise SparseSetError(rc, "sparse_layers_evolve", "; ".join(m for m in msgs if m))

    def fit(self, blocks: torch.Tensor, labels: torch.Tensor, sizes: Sequence[int], epochs: int, zeta: float, *,
            importance_every: int = 0, importance_start: int = 0, importance_quantile: float = 0.0,
            first_generation: int = 1):
        """The training loop of Algorithm 2 over library calls: per epoch, every minibatch block is
        trained on; then (optionally, every `importance_every` epochs from epoch `importance_start`
        on) Importance Pruning removes the incoming connections of the hidden neurons whose
        importance lies below the `importance_quantile` quantile of their layer; then every layer goes
        through the prune / regrow cycle.  blocks [n_blocks][n_in][ld], labels int32 [n_blocks][ld>=B],
        sizes[k] = number of samples in block k.  Returns the mean loss of every epoch."""
        history = []
        for e in range(epochs):
            self.loss_sum.zero_()
            for k in range(blocks.shape[0]):
                self.train_step(blocks[k], labels[k], sizes[k])
            history.append(self.loss_sum.item() / float(sum(sizes)))
            if importance_every > 0 and e >= importance_start and (e - importance_start) % importance_every == 0:
                for layer in self.layers[:-1]:
                    imp = layer.importance()
                    alive = imp[imp > 0]
                    if alive.size:
                        layer.importance_prune(float(np.quantile(alive.astype(np.float64), importance_quantile)))
            self.evolve(zeta, first_generation + e)
        return history

    def close(self):
        for layer in self.layers:
            layer.close()
