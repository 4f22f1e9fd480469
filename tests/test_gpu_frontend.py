"""Generated-dispatch graphs on the GPU: libraries the front end built from graph descriptions (user-written device
functions), run through the C ABI under the three schedulers, against the definition of what they compute (sums of
small integers: exact in fp32 in any order)."""
import numpy as np
import pytest

pytestmark = pytest.mark.gpu
SPIN = 400000
KINDS = [0, 1, 2]                              # static, dynamic, unfused


def _compiled(name, kind):
    import os
    import paper_2604_13327_amd as etc
    from paper_2604_13327_amd import frontend
    g = frontend.EXAMPLES[name]()
    lib = frontend.library_path(g)
    assert os.path.exists(lib), f"{lib} is missing: run `python -c 'import __graft_entry__ as g; g.build()'` first"
    return frontend.CompiledGraph(g, lib, kind=kind, debug_flags=etc.DEBUG_EXEC_COUNT, spin_budget=SPIN)


@pytest.mark.parametrize("kind", KINDS)
@pytest.mark.parametrize("name", ["rowsum", "sumsq"])
def test_generated_graph_symbolic_n(name, kind):
    import torch
    cg = _compiled(name, kind)
    rng = np.random.default_rng(3)
    for n in (1, 5, 300):                      # one generated library, three bound shapes, nothing rebuilt
        A = rng.integers(-8, 9, size=(n * 32, 128)).astype(np.float32)
        dA = torch.from_numpy(A).cuda()
        dB = torch.full((n * 32, 4), float("nan"), device="cuda")
        dC = torch.full((n * 32,), float("nan"), device="cuda")
        dY = torch.full((n * 32, 128), float("nan"), device="cuda")
        for slot, t in ((0, dA), (1, dB), (2, dC), (3, dY)):
            cg.bind_buffer(slot, t)
        cg.bind_shape(n=n)
        want = (A.astype(np.float64) ** (2 if name == "sumsq" else 1)).sum(1)
        for rep in range(2):                   # the second launch runs on the re-armed event tensors
            dC.fill_(float("nan"))
            cg.launch()
            torch.cuda.synchronize()
            np.testing.assert_array_equal(dC.cpu().numpy(), want)
            assert (cg.error_word() == 0).all()
            assert (cg.event_counters() == 0).all()
            assert (cg.exec_counts() == rep + 1).all()          # counted per bound shape: once per launch and task
        info = cg.step_info()
        assert info.n_tasks == (9 if name == "sumsq" else 5) * n
        if name == "sumsq":
            np.testing.assert_array_equal(dY.cpu().numpy(), A * A)


def test_front_end_refuses_buffers_too_small_for_the_bound_shape():
    import torch
    cg = _compiled("rowsum", 0)
    cg.bind_buffer(0, torch.zeros(64, 128, device="cuda"))
    cg.bind_buffer(1, torch.zeros(64, 4, device="cuda"))
    with pytest.raises(ValueError, match="not bound"):
        cg.bind_shape(n=2)
    cg.bind_buffer(2, torch.zeros(64, device="cuda"))
    cg.bind_shape(n=2)
    with pytest.raises(ValueError, match="touches"):
        cg.bind_shape(n=3)


def test_stock_library_refuses_generated_function_ids():
    import paper_2604_13327_amd as etc
    g = etc.EventGraph(kind=0)
    ev = g.add_event([g.dim(sym=0, mul=1)])
    with pytest.raises(etc.EtcError):
        g.add_call(100, [g.dim(sym=0, mul=1)], out_edges=[g.edge(ev, [(0, 0, 1)])])


@pytest.mark.parametrize("kind", KINDS)
def test_generated_graph_with_data_dependent_edges(kind):
    """Sec. 2.4 through generated dispatch: run-time routed notifies (the event's count comes with the table) and
    events that release ranges of a grouped grid; surplus tasks of the grid write nothing (and under the ready queue
    never run).  Whatever the routing, C is the plain row sum of A."""
    import torch
    n_max, m = 24, 5
    cg = _compiled("routed_rowsum", kind)
    rng = np.random.default_rng(17)
    for rep, n_rows in enumerate((24, 7, 1, 19)):
        A = rng.integers(-8, 9, size=(n_rows * 32, 128)).astype(np.float32)
        route = rng.integers(0, m, size=n_rows).astype(np.int32)
        if rep == 1:
            route[:] = 2                                   # everything to one group
        perm = np.argsort(route, kind="stable").astype(np.int32)
        per_group = np.bincount(route, minlength=m)
        indptr = np.concatenate([[0], np.cumsum(per_group)]).astype(np.int32)
        count = (4 * per_group).astype(np.int32)
        perm_full = np.concatenate([perm, np.zeros(n_max - n_rows, np.int32)])
        dA = torch.from_numpy(A).cuda()
        dB = torch.full((n_rows * 32, 4), float("nan"), device="cuda")
        dC = torch.full((n_max * 32,), float("nan"), device="cuda")
        tabs = [torch.from_numpy(x).cuda() for x in (route, indptr, count, perm_full)]
        for slot, t in enumerate([dA, dB, dC] + tabs):
            cg.bind_buffer(slot, t)
        cg.bind_shape(n=n_rows)
        for launches in (1, 2):
            dC.fill_(float("nan"))
            cg.launch()
            torch.cuda.synchronize()
            got = dC.cpu().numpy()
            np.testing.assert_array_equal(got[: n_rows * 32], A.astype(np.float64).sum(1))
            assert np.isnan(got[n_rows * 32:]).all()
            assert (cg.error_word() == 0).all() and (cg.event_counters() == 0).all()
            want = np.full(4 * n_rows + n_max, launches, np.int32)
            if kind == 1:
                want[4 * n_rows + n_rows:] = 0             # the ready queue never released the surplus tasks
            np.testing.assert_array_equal(cg.exec_counts(), want)
