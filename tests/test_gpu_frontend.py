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
