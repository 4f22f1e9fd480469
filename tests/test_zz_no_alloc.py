"""The allocation-free launch of the row-sum graph against the allocating entry points it is a variant of
(etc_graph_* + etc_graph_launch, static scheduler): same kernels, so the same bits, on two calls in a row,
the second with a smaller input (every call shares one device array and must not see the previous one)."""
import numpy as np
import pytest

pytestmark = pytest.mark.gpu


def _graph_result(etc, A_np):
    """C of the row-sum graph through the allocating entry points."""
    import torch
    from paper_2604_13327_amd import binding as b
    n = A_np.shape[0] // 32
    g = etc.EventGraph(kind=etc.SCHED_STATIC, spin_budget=400000)
    ns = g.dim(sym=0, mul=1, add=0)
    ev = g.add_event([ns])
    g.add_call(b.FN_ROWSUM_PARTIAL, [ns, g.dim(add=4)], out_edges=[g.edge(ev, [(b.MAP_DIM, 0, 1)])])
    g.add_call(b.FN_ROWSUM_FINAL, [ns], in_edges=[g.edge(ev, [(b.MAP_DIM, 0, 1)])])
    dA = torch.from_numpy(A_np).cuda()
    dB = torch.full((n * 32, 4), float("nan"), device="cuda")
    dC = torch.full((n * 32,), float("nan"), device="cuda")
    for slot, t in enumerate((dA, dB, dC)):
        g.bind_buffer(slot, t)
    g.bind_shape([n])
    g.launch()
    torch.cuda.synchronize()
    assert (g.event_counters() == 0).all()
    out = dC.cpu().numpy()
    g.close()
    return out


def test_allocation_free_rowsum_matches_the_graph_launch_twice():
    import torch
    import paper_2604_13327_amd as etc
    rng = np.random.default_rng(5)
    first = True
    for n in (300, 7):                      # several tasks per queue, then fewer tasks than queues
        A = rng.standard_normal((n * 32, 128)).astype(np.float32)       # order of the sums matters: bits must agree
        ref = _graph_result(etc, A)
        dA = torch.from_numpy(A).cuda()
        dC = torch.full((n * 32,), float("nan"), device="cuda")
        torch.cuda.synchronize()
        before = torch.cuda.memory_allocated()
        etc.rowsum_launch_noalloc(dA, dC, n)
        if not first:                       # a second launch right behind, on the array the first one left
            etc.rowsum_launch_noalloc(dA, dC, n)
        torch.cuda.synchronize()
        assert torch.cuda.memory_allocated() == before
        got = dC.cpu().numpy()
        np.testing.assert_array_equal(got, ref)
        # and the plain definition, within fp32 summation error
        np.testing.assert_allclose(got, A.astype(np.float64).sum(1), rtol=0, atol=2e-4)
        first = False
    # integer-valued input: exact against the closed form whatever the order; the largest size, then a small one
    for n in (etc.ROWSUM_NOALLOC_MAX_N, 1):
        A = rng.integers(-8, 9, size=(n * 32, 128)).astype(np.float32)
        dA = torch.from_numpy(A).cuda()
        dC = torch.full((n * 32,), float("nan"), device="cuda")
        etc.rowsum_launch_noalloc(dA, dC, n)
        torch.cuda.synchronize()
        np.testing.assert_array_equal(dC.cpu().numpy(), A.astype(np.float64).sum(1))


def test_allocation_free_rowsum_rejects_sizes_beyond_its_array():
    import torch
    import paper_2604_13327_amd as etc
    dA = torch.zeros(32, 128, device="cuda")
    dC = torch.zeros(32, device="cuda")
    for bad in (0, -1, etc.ROWSUM_NOALLOC_MAX_N + 1):
        with pytest.raises(etc.EtcError) as ei:
            etc.rowsum_launch_noalloc(dA, dC, bad)
        assert ei.value.status == -1
