"""Host-side checks that need no GPU: the shared library loads, exports every symbol the header
declares, sizes its buffers sensibly and rejects bad arguments with error codes."""
import ctypes as C
import os
import re

import pytest

from paper_2102_01732_amd import binding, workloads as wl

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


@pytest.fixture(scope="module")
def lib():
    if not os.path.exists(binding.LIB_PATH):
        from paper_2102_01732_amd import build
        build.build()
    return binding.lib()


def test_exports_match_header(lib):
    header = open(os.path.join(ROOT, "include", "sparse_set.h")).read()
    declared = set(re.findall(r"\b(sparse_(?:layers?|loss|kernel)_\w+)\s*\(", header))
    assert declared == set(binding.EXPORTS)
    for name in declared:
        assert hasattr(lib, name), name


def test_config_struct_layout_matches_header():
    # int64 x2, double, int64, int32 x2, float x5, (pad) uint64, uint32, int32 x2, uint32
    assert C.sizeof(binding.SlConfig) == 88
    assert binding.SlConfig.seed.offset == 64 and binding.SlConfig.flags.offset == 84


def test_query_sizes_and_argument_errors(lib):
    cfg = binding.make_config(500, 400, epsilon=10, init_limit=0.1)
    sb, cb = binding.query_sizes(cfg)
    assert sb > 9000 * 4 * 8 and cb > 0
    # nnz from epsilon, capped at the matrix size
    for (a, b, e) in [(500, 400, 10), (400, 2, 10), (1000, 10, 20)]:
        c1 = binding.make_config(a, b, epsilon=e, init_limit=0.1)
        c2 = binding.make_config(a, b, nnz=wl.er_nnz(a, b, e), init_limit=0.1)
        assert binding.query_sizes(c1) == binding.query_sizes(c2)
    bad = [dict(n_in=0), dict(n_out=-3), dict(max_batch=0), dict(act_kind=2), dict(act_parity=3), dict(prune_mode=5),
           dict(init_limit=0.0), dict(epsilon=-1.0)]
    for kw in bad:
        args = dict(n_in=10, n_out=10, epsilon=1.0, init_limit=0.1)
        args.update(kw)
        n_in, n_out = args.pop("n_in"), args.pop("n_out")
        with pytest.raises(binding.SparseSetError) as e:
            binding.query_sizes(binding.make_config(n_in, n_out, **args))
        assert e.value.code == binding.SL_EINVAL
    with pytest.raises(binding.SparseSetError) as e:
        binding.query_sizes(binding.make_config(2 ** 31, 10, epsilon=1.0))
    assert e.value.code == binding.SL_EOVERFLOW
    with pytest.raises(binding.SparseSetError) as e:
        binding.query_sizes(binding.make_config(2 ** 20, 2 ** 20, nnz=2 ** 30))
    assert e.value.code == binding.SL_EOVERFLOW
    # null handles are rejected, not dereferenced
    assert lib.sparse_layer_forward(None, None, 0, 0, None, 0, None) == binding.SL_EINVAL
    assert lib.sparse_layer_backward(None, None, 0, None, 0, 0, None, 0, None) == binding.SL_EINVAL
    assert lib.sparse_layer_update(None, None) == binding.SL_EINVAL
    assert lib.sparse_layer_evolve(None, 0.3, 1, None) == binding.SL_EINVAL
    assert lib.sparse_layer_destroy(None) == binding.SL_EINVAL
    assert lib.sparse_layer_infer_static(None, None, 0, 0, None, 0, None) == binding.SL_EINVAL
    assert lib.sparse_layer_set_fused_update(None, 1) == binding.SL_EINVAL
    assert lib.sparse_layer_set_sampler_window(None, 0, 0) == binding.SL_EINVAL
    assert lib.sparse_layers_evolve(None, 1, 0.3, 1, None) == binding.SL_EINVAL
    none = (C.c_void_p * 2)(None, None)
    assert lib.sparse_layers_evolve(none, 2, 0.3, 1, none) == binding.SL_EINVAL
    assert lib.sparse_loss_softmax_ce(None, 0, None, 1, 2, None, 0, None, None) == binding.SL_EINVAL
    out = C.c_void_p(None)
    assert lib.sparse_layer_init(C.byref(cfg), None, 0, None, 0, None, C.byref(out)) == binding.SL_EINVAL


def test_one_million_neuron_layer_fits_one_gpu():
    total = 0
    w = wl.WORKLOADS["set_mlp_1m"]
    scratch = 0
    for li, s in enumerate(w.layers):
        cfg = binding.make_config(s.n_in, s.n_out, nnz=s.nnz, init_limit=s.init_limit, max_batch=128,
                                  need_input_grad=li > 0)
        sb, cb = binding.query_sizes(cfg)
        total += sb
        scratch = max(scratch, cb)
    assert total + scratch < 8 * 2 ** 30      # a few GB of the 288 GB of one MI355X
