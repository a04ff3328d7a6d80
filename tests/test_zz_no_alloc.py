"""sparse_layer_infer_static (the entry point for callers that cannot allocate: partial sums in a buffer built into
the library) against sparse_layer_infer, through the C ABI: same bits, on two calls in a row, the second with a
smaller input; layers without split rows pass straight through; partial sums beyond the built-in buffer are
refused with an error and nothing is launched."""
import numpy as np
import pytest

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def gpu():
    import torch
    if not torch.cuda.is_available():
        pytest.skip("no GPU")
    from paper_2102_01732_amd import binding
    binding.lib()
    return binding


def make(gpu, n_in, n_out, nnz, max_batch, act_kind=0):
    return gpu.SparseLayer(gpu.make_config(n_in, n_out, nnz=nnz, act_kind=act_kind, act_parity=0, alpha=0.6,
                                           init_limit=0.05, seed=77, layer_id=3, max_batch=max_batch,
                                           need_input_grad=True))


def test_infer_static_equals_infer_twice_in_a_row(gpu):
    import torch
    torch.manual_seed(5)
    # fully dense output layers: every row is cut into virtual rows, so the partial-sum buffer is really used
    big = make(gpu, 30000, 10, 300000, 128)          # 10 rows of 30 000 entries
    small = make(gpu, 3000, 2, 6000, 64)             # 2 rows of 3 000 entries
    calls = [(big, 128), (small, 37), (big, 5), (small, 64)]       # a smaller input after a larger one, and back
    for L, B in calls:
        ld = (B + 3) // 4 * 4
        x = torch.randn((L.n_in, ld), device="cuda")
        ref = torch.full((L.n_out, ld), 7.0, device="cuda")
        got = torch.full((L.n_out, ld), 7.0, device="cuda")
        L.infer(x, B, ref)
        L.infer_static(x, B, got)
        torch.cuda.synchronize()
        assert torch.equal(got, ref), (L.n_in, B)
        assert bool((got[:, :B] != 7.0).all()) and bool((got[:, B:] == 7.0).all())
    # a hidden layer whose rows are not split needs no partial sums at all
    plain = make(gpu, 500, 400, 9000, 128, act_kind=1)
    x = torch.randn((500, 128), device="cuda")
    ref, got = torch.zeros((400, 128), device="cuda"), torch.zeros((400, 128), device="cuda")
    plain.infer(x, 128, ref)
    plain.infer_static(x, 128, got)
    assert torch.equal(got, ref)
    # interleaved with training calls of the same layer: the training state is left alone
    a = torch.zeros((10, 128), device="cuda")
    xb = torch.randn((30000, 128), device="cuda")
    big.forward(xb, 128, a)
    big.infer_static(xb, 128, got[:10])
    assert torch.equal(got[:10], a)
    for L in (big, small, plain):
        L.close()


def test_infer_static_refuses_what_does_not_fit(gpu):
    import torch
    # 2 rows of 10^6 entries at max_batch 1024: about 8200 virtual rows x 1024 floats = 32 MiB of partial sums
    L = make(gpu, 1000000, 2, 2000000, 1024)
    x = torch.zeros((1000000, 32), device="cuda")
    a = torch.full((2, 32), 3.0, device="cuda")
    with pytest.raises(gpu.SparseSetError) as e:
        L.infer_static(x, 32, a)
    assert e.value.code == gpu.SL_ENOMEM and "built-in buffer" in str(e.value)
    torch.cuda.synchronize()
    assert bool((a == 3.0).all())                     # nothing was launched
    L.infer(x, 32, a)                                 # the ordinary entry point still serves it
    torch.cuda.synchronize()
    assert bool((a[:, :32] == 0.0).all())
    with pytest.raises(gpu.SparseSetError) as e:
        L.infer_static(x, 2048, a)
    assert e.value.code == gpu.SL_EINVAL
    L.profile_begin()
    with pytest.raises(gpu.SparseSetError) as e:
        L.infer_static(x, 32, a)
    assert e.value.code == gpu.SL_ESTATE
    L.profile_end()
    L.close()
