"""CPU oracle for truly sparse MLP training with SET -- TEST INFRASTRUCTURE ONLY.

Thin numpy front end over ``set_oracle.c`` (same directory).  The C file holds the arithmetic of
every step; this module only owns the arrays of a layer (CSR pattern, weights, velocities,
biases), calls the C routines in the order the paper's training loop prescribes (Algorithm 2:
train for an epoch, then prune and regrow every sparse layer) and rebuilds the CSR after an
evolution with library sorts.

Nothing here is part of the product: only tests, the smoke check and the benchmark's
``cpu_baseline`` leg import it, and it imports nothing from the GPU package.

Orientation: the stored matrix is the transpose of the paper's W^(l): ``Wt[n_out, n_in]`` in CSR,
row j = incoming connections of neuron j.  Dense operands are feature-major ``[n, B]``.
"""
from __future__ import annotations

import ctypes
import os
import subprocess
from typing import List, Optional, Sequence

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "set_oracle.c")
_LIB = os.path.join(_HERE, "liboracle.so")
_lib = None

_f32p = np.ctypeslib.ndpointer(dtype=np.float32, flags="C_CONTIGUOUS")
_i32p = np.ctypeslib.ndpointer(dtype=np.int32, flags="C_CONTIGUOUS")
_u64p = np.ctypeslib.ndpointer(dtype=np.uint64, flags="C_CONTIGUOUS")
_u32p = np.ctypeslib.ndpointer(dtype=np.uint32, flags="C_CONTIGUOUS")
_u8p = np.ctypeslib.ndpointer(dtype=np.uint8, flags="C_CONTIGUOUS")


def build(force: bool = False) -> str:
    """Compile set_oracle.c with gcc (no fast-math, no FMA contraction; OpenMP only shares loops whose
    iterations own disjoint outputs, so results do not depend on the thread count)."""
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        subprocess.check_call(
            ["gcc", "-O2", "-ffp-contract=off", "-fopenmp", "-fPIC", "-shared", "-std=c11", _SRC, "-o", _LIB, "-lm"]
        )
    return _LIB


def lib():
    global _lib
    if _lib is None:
        # ORACLE_LIB: another build of the same source (the sanitizer run of the pins uses it)
        path = os.environ.get("ORACLE_LIB") or build()
        L = ctypes.CDLL(path)
        c = ctypes
        L.or_set_threads.argtypes = [c.c_int]
        L.or_set_threads.restype = c.c_int
        L.or_philox4x32_10.argtypes = [_u32p, _u32p, _u32p]
        L.or_philox4x32_10.restype = None
        L.or_weight_value.argtypes = [c.c_uint64, c.c_uint32, c.c_uint32, c.c_uint64, c.c_float]
        L.or_weight_value.restype = c.c_float
        L.or_weight_values.argtypes = [c.c_uint64, c.c_uint32, c.c_uint32, _u64p, c.c_int64, c.c_float, _f32p]
        L.or_weight_values.restype = None
        L.or_sample_positions.argtypes = [c.c_int64, c.c_int64, c.c_int64, _u64p, c.c_int64, c.c_uint64,
                                          c.c_uint32, c.c_uint32, _u64p]
        L.or_sample_positions.restype = c.c_int
        L.or_all_relu.argtypes = [_f32p, c.c_int64, c.c_int, c.c_int, c.c_float, _f32p]
        L.or_all_relu.restype = None
        L.or_forward.argtypes = [c.c_int64, _i32p, _i32p, _f32p, _f32p, _f32p, c.c_int64, c.c_int32, c.c_int,
                                 c.c_int, c.c_float, _f32p, _f32p, c.c_int64]
        L.or_forward.restype = None
        L.or_backward.argtypes = [c.c_int64, c.c_int64, _i32p, _i32p, _f32p, _f32p, c.c_int64, _f32p, _f32p,
                                  c.c_int64, c.c_int32, c.c_int, c.c_int, c.c_float, _f32p, _f32p, _f32p,
                                  c.c_void_p, c.c_int64]
        L.or_backward.restype = c.c_int
        L.or_update.argtypes = [c.c_int64, _f32p, _f32p, _f32p, c.c_float, c.c_float, c.c_float]
        L.or_update.restype = None
        L.or_prune_select.argtypes = [c.c_int64, _f32p, _u64p, c.c_double, c.c_int, _u8p]
        L.or_prune_select.restype = c.c_int64
        L.or_softmax_ce.argtypes = [_f32p, c.c_int64, _i32p, c.c_int32, c.c_int32, _f32p, c.c_int64]
        L.or_softmax_ce.restype = c.c_double
        L.or_importance.argtypes = [c.c_int64, _i32p, _f32p, _f32p]
        L.or_importance.restype = None
        L.or_importance_f32.argtypes = [c.c_int64, _i32p, _f32p, _f32p]
        L.or_importance_f32.restype = None
        L.or_dropout_keep.argtypes = [c.c_uint64, c.c_uint32, c.c_uint32, c.c_int64, c.c_int32, c.c_uint32, _u8p]
        L.or_dropout_keep.restype = None
        L.or_dropout_apply.argtypes = [_f32p, _u8p, c.c_int64, c.c_float]
        L.or_dropout_apply.restype = None
        L.or_average_sorted.argtypes = [c.c_int64, _u64p, _f32p, c.c_int32, _u64p, _f32p]
        L.or_average_sorted.restype = c.c_int64
        L.or_keep_largest.argtypes = [c.c_int64, _f32p, _u64p, c.c_int64, _u8p]
        L.or_keep_largest.restype = c.c_int64
        _lib = L
    return _lib


# ----------------------------------------------------------------------------------------------
# small helpers
# ----------------------------------------------------------------------------------------------
def set_threads(n: int = 0) -> int:
    """Threads for the row-parallel loops of forward / backward / update (0: OpenMP's default, i.e.
    OMP_NUM_THREADS or all cores).  Returns the number in use.  Results never depend on it."""
    return int(lib().or_set_threads(int(n)))


def philox(ctr: Sequence[int], key: Sequence[int]) -> np.ndarray:
    out = np.zeros(4, dtype=np.uint32)
    lib().or_philox4x32_10(np.asarray(ctr, dtype=np.uint32), np.asarray(key, dtype=np.uint32), out)
    return out


def nnz_from_epsilon(n_in: int, n_out: int, epsilon: float) -> int:
    """Erdos-Renyi connection count: epsilon*(n_in+n_out), rounded half away from zero and capped
    at the size of the matrix (the extreme-scale table's parameter counts are exactly
    epsilon * sum(n_in+n_out))."""
    want = int(np.floor(float(epsilon) * float(n_in + n_out) + 0.5))
    return min(want, n_in * n_out)


def sample_positions(n_in: int, n_out: int, k: int, occupied: np.ndarray, seed: int, layer_id: int,
                     generation: int) -> np.ndarray:
    occupied = np.ascontiguousarray(occupied, dtype=np.uint64)
    out = np.zeros(max(k, 1), dtype=np.uint64)
    rc = lib().or_sample_positions(n_in, n_out, k, occupied if occupied.size else np.zeros(1, np.uint64),
                                   occupied.size, seed, layer_id, generation, out)
    if rc != 0:
        raise RuntimeError(f"or_sample_positions failed: {rc}")
    return out[:k]


def weight_values(seed: int, layer_id: int, generation: int, pos: np.ndarray, init_limit: float) -> np.ndarray:
    pos = np.ascontiguousarray(pos, dtype=np.uint64)
    out = np.zeros(max(pos.size, 1), dtype=np.float32)
    lib().or_weight_values(seed, layer_id, generation, pos if pos.size else np.zeros(1, np.uint64), pos.size,
                           np.float32(init_limit), out)
    return out[: pos.size]


def all_relu(z: np.ndarray, act_kind: int, parity: int, alpha: float) -> np.ndarray:
    z = np.ascontiguousarray(z, dtype=np.float32)
    a = np.empty_like(z)
    lib().or_all_relu(z.reshape(-1), z.size, act_kind, parity, np.float32(alpha), a.reshape(-1))
    return a


def softmax_ce(z: np.ndarray, y: np.ndarray):
    """z [C, B] float32, y [B] int32 -> (loss, dz [C, B])."""
    z = np.ascontiguousarray(z, dtype=np.float32)
    y = np.ascontiguousarray(y, dtype=np.int32)
    C, B = z.shape
    dz = np.zeros_like(z)
    loss = lib().or_softmax_ce(z, B, y, B, C, dz, B)
    return float(loss), dz


def csr_from_flat(flat: np.ndarray, n_in: int, n_out: int):
    """flat: ascending uint64 positions j*n_in+i -> (rowptr int32[n_out+1], colidx int32[nnz])."""
    rows = (flat // np.uint64(n_in)).astype(np.int64)
    cols = (flat % np.uint64(n_in)).astype(np.int32)
    counts = np.bincount(rows, minlength=n_out)
    rowptr = np.zeros(n_out + 1, dtype=np.int64)
    np.cumsum(counts, out=rowptr[1:])
    return rowptr.astype(np.int32), cols


def flat_from_csr(rowptr: np.ndarray, colidx: np.ndarray, n_in: int) -> np.ndarray:
    n_out = rowptr.size - 1
    rows = np.repeat(np.arange(n_out, dtype=np.uint64), np.diff(rowptr.astype(np.int64)))
    return rows * np.uint64(n_in) + colidx.astype(np.uint64)


# ----------------------------------------------------------------------------------------------
# one sparse layer
# ----------------------------------------------------------------------------------------------
class OracleLayer:
    def __init__(self, n_in: int, n_out: int, nnz: int, act_kind: int, act_parity: int, alpha: float,
                 init_limit: float, lr: float, momentum: float, weight_decay: float, seed: int,
                 layer_id: int, prune_mode: int = 0):
        self.n_in, self.n_out = int(n_in), int(n_out)
        self.act_kind, self.act_parity, self.alpha = int(act_kind), int(act_parity), np.float32(alpha)
        self.init_limit = np.float32(init_limit)
        self.lr, self.momentum, self.weight_decay = np.float32(lr), np.float32(momentum), np.float32(weight_decay)
        self.seed, self.layer_id, self.prune_mode = int(seed), int(layer_id), int(prune_mode)
        # Erdos-Renyi topology with exactly nnz distinct connections, generation 0.
        flat = sample_positions(self.n_in, self.n_out, int(nnz), np.zeros(0, np.uint64), self.seed,
                                self.layer_id, 0)
        self.rowptr, self.colidx = csr_from_flat(flat, self.n_in, self.n_out)
        self.val = weight_values(self.seed, self.layer_id, 0, flat, self.init_limit)
        self.vel = np.zeros_like(self.val)
        self.bias = np.zeros(self.n_out, dtype=np.float32)
        self.bias_vel = np.zeros(self.n_out, dtype=np.float32)
        self.grad_val = np.zeros_like(self.val)
        self.grad_bias = np.zeros(self.n_out, dtype=np.float32)
        self.z: Optional[np.ndarray] = None
        self.dz: Optional[np.ndarray] = None
        self.drop_p, self.drop_step = np.float32(0.0), 0
        self.keep: Optional[np.ndarray] = None

    def set_dropout(self, p: float, step: int):
        """Dropout rate for the next forward/backward pair of this (hidden) layer and the step index
        that selects the mask."""
        self.drop_p, self.drop_step = np.float32(p), int(step) & 0xFFFFFFFF

    def dropout_keep(self, B: int) -> np.ndarray:
        thr = int(np.floor(float(self.drop_p) * 4294967296.0))
        keep = np.zeros((self.n_out, B), dtype=np.uint8)
        lib().or_dropout_keep(self.seed, self.layer_id, self.drop_step, self.n_out, B, thr, keep)
        return keep

    @property
    def nnz(self) -> int:
        return int(self.val.size)

    def flat(self) -> np.ndarray:
        return flat_from_csr(self.rowptr, self.colidx, self.n_in)

    def set_state(self, rowptr, colidx, val, vel, bias, bias_vel):
        self.rowptr = np.ascontiguousarray(rowptr, dtype=np.int32).copy()
        self.colidx = np.ascontiguousarray(colidx, dtype=np.int32).copy()
        self.val = np.ascontiguousarray(val, dtype=np.float32).copy()
        self.vel = np.ascontiguousarray(vel, dtype=np.float32).copy()
        self.bias = np.ascontiguousarray(bias, dtype=np.float32).copy()
        self.bias_vel = np.ascontiguousarray(bias_vel, dtype=np.float32).copy()
        self.grad_val = np.zeros_like(self.val)
        self.grad_bias = np.zeros(self.n_out, dtype=np.float32)

    def forward(self, x: np.ndarray) -> np.ndarray:
        x = np.ascontiguousarray(x, dtype=np.float32)
        assert x.shape[0] == self.n_in
        B = x.shape[1]
        z = np.zeros((self.n_out, B), dtype=np.float32)
        a = np.zeros((self.n_out, B), dtype=np.float32)
        lib().or_forward(self.n_out, self.rowptr, self.colidx, self.val, self.bias, x, B, B, self.act_kind,
                         self.act_parity, self.alpha, z, a, B)
        self.z = z
        self.keep = None
        if self.drop_p > 0 and self.act_kind != 0:
            self.keep = self.dropout_keep(B)
            scale = np.float32(1.0) / (np.float32(1.0) - self.drop_p)
            lib().or_dropout_apply(a.reshape(-1), self.keep.reshape(-1), a.size, scale)
        return a

    def backward(self, x: np.ndarray, grad_a: np.ndarray, need_input_grad: bool = True) -> Optional[np.ndarray]:
        x = np.ascontiguousarray(x, dtype=np.float32)
        grad_a = np.ascontiguousarray(grad_a, dtype=np.float32)
        B = x.shape[1]
        assert self.z is not None and self.z.shape == (self.n_out, B) and grad_a.shape == (self.n_out, B)
        if self.keep is not None:              # the factor of the forward pass multiplies the gradient
            grad_a = grad_a.copy()
            scale = np.float32(1.0) / (np.float32(1.0) - self.drop_p)
            lib().or_dropout_apply(grad_a.reshape(-1), self.keep.reshape(-1), grad_a.size, scale)
        self.dz = np.zeros((self.n_out, B), dtype=np.float32)
        gx = np.zeros((self.n_in, B), dtype=np.float32) if need_input_grad else None
        rc = lib().or_backward(self.n_in, self.n_out, self.rowptr, self.colidx, self.val, x, B, self.z, grad_a,
                               B, B, self.act_kind, self.act_parity, self.alpha, self.dz, self.grad_val,
                               self.grad_bias, gx.ctypes.data if gx is not None else None, B)
        if rc != 0:
            raise MemoryError("or_backward")
        return gx

    def update(self):
        lib().or_update(self.nnz, self.val, self.vel, self.grad_val, self.lr, self.momentum, self.weight_decay)
        lib().or_update(self.n_out, self.bias, self.bias_vel, self.grad_bias, self.lr, self.momentum,
                        np.float32(0.0))

    def prune_flags(self, zeta: float) -> np.ndarray:
        remove = np.zeros(max(self.nnz, 1), dtype=np.uint8)
        k = lib().or_prune_select(self.nnz, self.val if self.nnz else np.zeros(1, np.float32),
                                  self.flat() if self.nnz else np.zeros(1, np.uint64), float(zeta),
                                  self.prune_mode, remove)
        if k < 0:
            raise MemoryError("or_prune_select")
        return remove[: self.nnz].astype(bool)

    def evolve(self, zeta: float, generation: int) -> int:
        """Algorithm 2's prune/regrow cycle for this layer.  Survivors keep weight and velocity;
        new connections get a fresh weight and zero velocity; nnz is unchanged.  Returns k."""
        flat = self.flat()
        remove = self.prune_flags(zeta)
        k = int(remove.sum())
        keep = ~remove
        s_flat, s_val, s_vel = flat[keep], self.val[keep], self.vel[keep]
        new_flat = sample_positions(self.n_in, self.n_out, k, s_flat, self.seed, self.layer_id, generation)
        new_val = weight_values(self.seed, self.layer_id, generation, new_flat, self.init_limit)
        all_flat = np.concatenate([s_flat, new_flat])
        order = np.argsort(all_flat, kind="stable")
        all_flat = all_flat[order]
        self.val = np.concatenate([s_val, new_val])[order].astype(np.float32)
        self.vel = np.concatenate([s_vel, np.zeros(k, dtype=np.float32)])[order].astype(np.float32)
        self.rowptr, self.colidx = csr_from_flat(all_flat, self.n_in, self.n_out)
        self.grad_val = np.zeros_like(self.val)
        self.z = None
        return k

    def importance(self) -> np.ndarray:
        out = np.zeros(self.n_out, dtype=np.float32)
        lib().or_importance(self.n_out, self.rowptr, self.val, out)
        return out

    def importance_f32(self) -> np.ndarray:
        out = np.zeros(self.n_out, dtype=np.float32)
        lib().or_importance_f32(self.n_out, self.rowptr, self.val if self.nnz else np.zeros(1, np.float32), out)
        return out

    def importance_prune(self, threshold: float) -> int:
        """Algorithm 2, Importance Pruning: remove all incoming connections of neurons whose importance
        (eq. 4) is below the threshold.  nnz shrinks; returns the number of removed connections."""
        gone_rows = self.importance_f32() < np.float32(threshold)
        rows = np.repeat(np.arange(self.n_out), np.diff(self.rowptr))
        keep = ~gone_rows[rows]
        removed = int((~keep).sum())
        counts = np.diff(self.rowptr).astype(np.int64)
        counts[gone_rows] = 0
        rowptr = np.zeros(self.n_out + 1, dtype=np.int64)
        np.cumsum(counts, out=rowptr[1:])
        self.rowptr = rowptr.astype(np.int32)
        self.colidx = np.ascontiguousarray(self.colidx[keep])
        self.val = np.ascontiguousarray(self.val[keep])
        self.vel = np.ascontiguousarray(self.vel[keep])
        self.grad_val = np.zeros_like(self.val)
        self.z = None
        return removed

    def dense(self) -> np.ndarray:
        """Wt as a dense float64 matrix with zeros (for brute-force checks only)."""
        W = np.zeros((self.n_out, self.n_in), dtype=np.float64)
        rows = np.repeat(np.arange(self.n_out), np.diff(self.rowptr))
        W[rows, self.colidx] = self.val
        return W


def average_layers(dst: OracleLayer, replicas: Sequence[OracleLayer]) -> int:
    """Last step of Algorithm 1: dst <- average of the K replicas (eq. 2; a connection missing from a
    replica counts as zero), re-pruned by magnitude to dst's current number of connections; biases
    are averaged, velocities reset.  Returns the size of the union of the patterns."""
    K = len(replicas)
    n_keep = dst.nnz
    flat = np.concatenate([r.flat() for r in replicas])
    val = np.concatenate([r.val for r in replicas]).astype(np.float32)
    order = np.argsort(flat, kind="stable")                  # equal positions stay in replica order
    T = flat.size
    uflat = np.zeros(max(T, 1), np.uint64)
    uval = np.zeros(max(T, 1), np.float32)
    U = lib().or_average_sorted(T, np.ascontiguousarray(flat[order]) if T else np.zeros(1, np.uint64),
                                np.ascontiguousarray(val[order]) if T else np.zeros(1, np.float32), K, uflat, uval)
    uflat, uval = uflat[:U].copy(), uval[:U].copy()
    remove = np.zeros(max(U, 1), np.uint8)
    rc = lib().or_keep_largest(U, uval if U else np.zeros(1, np.float32), uflat if U else np.zeros(1, np.uint64),
                               n_keep, remove)
    if rc < 0:
        raise MemoryError("or_keep_largest")
    keep = ~remove[:U].astype(bool)
    bias = replicas[0].bias.copy()
    for r in replicas[1:]:
        bias = (bias + r.bias).astype(np.float32)
    bias = (bias / np.float32(K)).astype(np.float32)
    rowptr, colidx = csr_from_flat(uflat[keep], dst.n_in, dst.n_out)
    dst.set_state(rowptr, colidx, uval[keep], np.zeros(int(keep.sum()), np.float32), bias,
                  np.zeros(dst.n_out, np.float32))
    return int(U)


def retain_valid_updates(layer: OracleLayer, old_rowptr: np.ndarray, old_colidx: np.ndarray, old_grad: np.ndarray,
                         old_grad_bias: np.ndarray):
    """RetainValidUpdates of Algorithm 1: a gradient that a worker computed on an older topology is
    restricted to the connections that still exist; connections created since then get a zero
    gradient.  The result becomes the layer's pending gradient (layer.update() applies it)."""
    old_flat = flat_from_csr(np.asarray(old_rowptr, np.int32), np.asarray(old_colidx, np.int32), layer.n_in)
    new_flat = layer.flat()
    g = np.zeros(layer.nnz, dtype=np.float32)
    if old_flat.size and new_flat.size:
        pos = np.searchsorted(old_flat, new_flat)
        pos_c = np.minimum(pos, old_flat.size - 1)
        hit = old_flat[pos_c] == new_flat
        g[hit] = np.asarray(old_grad, np.float32)[pos_c[hit]]
    layer.grad_val = g
    layer.grad_bias = np.asarray(old_grad_bias, np.float32).copy()


# ----------------------------------------------------------------------------------------------
# a sparse MLP = chain of layers + softmax cross-entropy
# ----------------------------------------------------------------------------------------------
class OracleMLP:
    def __init__(self, layers: List[OracleLayer]):
        self.layers = layers
        self.acts: List[np.ndarray] = []
        # optional callable(layer_index, layer, a) -> a, run after each layer's forward.  Tests use
        # it to look at pre-activations that sit on the kink of eq. (3), where the branch taken is
        # decided by rounding, and to evaluate the other branch.
        self.after_forward = None
        self.dropout, self.step_index = 0.0, 0

    def forward(self, x: np.ndarray) -> np.ndarray:
        self.acts = [np.ascontiguousarray(x, dtype=np.float32)]
        for li, layer in enumerate(self.layers):
            a = layer.forward(self.acts[-1])
            if self.after_forward is not None:
                a = self.after_forward(li, layer, a)
            self.acts.append(a)
        return self.acts[-1]

    def train_step(self, x: np.ndarray, y: np.ndarray) -> float:
        if self.dropout > 0.0:
            for layer in self.layers[:-1]:
                layer.set_dropout(self.dropout, self.step_index)
        self.step_index += 1
        zL = self.forward(x)
        loss, grad = softmax_ce(zL, y)
        self.grads = [None] * (len(self.layers) + 1)
        self.grads[-1] = grad
        for li in range(len(self.layers) - 1, -1, -1):
            grad = self.layers[li].backward(self.acts[li], grad, need_input_grad=(li > 0))
            self.grads[li] = grad
        for layer in self.layers:
            layer.update()
        return loss

    def evolve(self, zeta: float, generation: int):
        return [layer.evolve(zeta, generation) for layer in self.layers]
