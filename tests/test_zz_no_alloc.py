"""The entry point that allocates nothing (speca_verify_static) against speca_verify: same kernels and
summation order, so the same bits, on two calls in a row, the second with a smaller input (the shared
file-scope scratch keeps the first call's partial sums); sizes beyond the scratch are rejected."""
import numpy as np
import pytest

pytestmark = pytest.mark.gpu
torch = pytest.importorskip("torch")


def _ctx(metric=None):
    import paper_2509_11628_amd as sp
    from paper_2509_11628_amd import binding as bd
    ctx = sp.Context(sp.cache_only_desc(1, 1, 8, bd.BF16))
    if metric is not None:
        ctx.init_cache(sp.make_cfg(order=0, interval=1, metric=metric), 1)
    return ctx


def _pair(rows, E, dtype, seed):
    g = torch.Generator(device="cuda").manual_seed(seed)
    truth = torch.randn((rows, E), generator=g, device="cuda", dtype=torch.float32)
    pred = truth + torch.randn((rows, E), generator=g, device="cuda", dtype=torch.float32) * torch.linspace(0.01, 0.2, rows, device="cuda")[:, None]
    return pred.to(dtype).contiguous(), truth.to(dtype).contiguous()


@pytest.mark.parametrize("dtype", [torch.bfloat16, torch.float32])
def test_verify_static_matches_verify_twice(dtype):
    from paper_2509_11628_amd import binding as bd
    ctx = _ctx()
    before = torch.cuda.memory_allocated()
    # first a large call (many chunks, ragged tail, more rows than one launch takes), then a smaller one
    for rows, E, tau in ((70, 100003 * 8, 0.08), (3, 8192 * 2 + 40, 0.05), (5, 16, 0.1)):
        pred, truth = _pair(rows, E, dtype, rows)
        err_ref, acc_ref = ctx.verify(pred, truth, tau=tau)
        err = torch.full((rows,), -1.0, device="cuda"); acc = torch.full((rows,), 7, device="cuda", dtype=torch.uint8)
        tau_d = torch.full((rows,), tau, device="cuda")
        ctx.verify_static(pred, truth, err, tau=tau_d, accept_out=acc)
        torch.cuda.synchronize()
        assert np.array_equal(err.cpu().numpy().view(np.uint32), err_ref.view(np.uint32)), (rows, E)
        assert np.array_equal(acc.cpu().numpy().astype(bool), acc_ref), (rows, E)
        assert acc_ref.any() and not acc_ref.all() or rows == 5
        # without thresholds the verdicts are left alone
        acc2 = torch.full((rows,), 9, device="cuda", dtype=torch.uint8)
        ctx.verify_static(pred, truth, err)
        torch.cuda.synchronize()
        assert int(acc2.min()) == 9 and np.array_equal(err.cpu().numpy().view(np.uint32), err_ref.view(np.uint32))
        del pred, truth
    assert torch.cuda.memory_allocated() >= before          # torch's own tensors only; the library allocated nothing it could see
    ctx.close()


def test_verify_static_other_metric_and_limits():
    import paper_2509_11628_amd as sp
    from paper_2509_11628_amd import binding as bd
    ctx = _ctx(bd.METRIC_L1)
    pred, truth = _pair(4, 50000, torch.float32, 1)
    err_ref, _ = ctx.verify(pred, truth)
    err = torch.zeros(4, device="cuda")
    ctx.verify_static(pred, truth, err)
    torch.cuda.synchronize()
    assert np.array_equal(err.cpu().numpy().view(np.uint32), err_ref.view(np.uint32))
    # beyond the static scratch: rejected with a message, nothing launched (64 rows x 1025 chunks > 65536)
    big = torch.zeros((64, 8192 * 1025), dtype=torch.bfloat16, device="cuda")
    err64 = torch.full((64,), -2.0, device="cuda")
    with pytest.raises(sp.SpecaError) as e:
        ctx.verify_static(big, big, err64)
    assert e.value.code == bd.EINVAL and "static scratch" in e.value.msg
    torch.cuda.synchronize()
    assert float(err64.max()) == -2.0
    # one row of the same width fits (1025 chunks)
    ctx.verify_static(big[:1], big[:1], err64)
    torch.cuda.synchronize()
    assert float(err64[0]) == 0.0 and float(err64[1]) == -2.0
    with pytest.raises(sp.SpecaError):
        ctx.verify_static(pred, truth, err, tau=torch.zeros(4, device="cuda"))      # thresholds without a verdict array
    ctx.close()
