"""The entry point that allocates nothing (isa_attention_static: scratch in a static device array inside the library)
against isa_attention on a caller-provided workspace, through the C ABI: same kernels, so the outputs must be identical
bit for bit (which is inside the benchmark spec's tolerance a fortiori).  Two calls in a row share the scratch array; the
second is a smaller problem, so whatever the first left behind must not leak into it."""
import ctypes as C

import pytest
import torch

import workloads as W
from util import problem_of

pytestmark = pytest.mark.gpu

BIG = W.CONFIGS["cfg1"].with_(name="static_big", H=6, src_grid=(4, 16, 33), ctx_grids=(((1, 10, 33), (2, 16, 33)),),
                              keep_ratio=0.5, full_frac=0.3, seed=301)
SMALL = W.CONFIGS["cfg1"].with_(name="static_small", H=3, src_grid=(2, 10, 33), ctx_grids=(((1, 9, 20),),),
                                keep_ratio=0.5, full_frac=0.3, seed=302)


def _reference(I, wl, q, k, v):
    pr = problem_of(wl)
    ws = I.new_workspace(pr)
    out = torch.full_like(q, float("nan"))
    I.isa_attention(pr, q, k, v, out, ws)
    torch.cuda.synchronize()
    return out


@pytest.mark.parametrize("variant", [dict(), dict(exact_frac=0.25, gamma=0.5), dict(D=64, block=64)],
                         ids=["plain", "exact_sets_residual", "portable_kernels"])
def test_static_scratch_matches_workspace_call_twice_in_a_row(variant):
    import paper_2605_04569_amd as I
    I.lib()
    cases = []
    for wl in (BIG.with_(**variant), SMALL.with_(**variant)):
        q, k, v = (t.cuda() for t in W.make_inputs(wl, "cpu"))
        cases.append((wl, q, k, v, _reference(I, wl, q, k, v)))
    outs = []
    for wl, q, k, v, _ in cases:                       # back to back on one stream, no synchronisation between them
        out = torch.full_like(q, float("nan"))
        I.isa_attention_static(problem_of(wl), q, k, v, out)
        outs.append(out)
    torch.cuda.synchronize()
    for (wl, q, k, v, ref), out in zip(cases, outs):
        n = wl.tokens(0)
        assert torch.isfinite(out[:, :, :n].float()).all(), wl.name
        assert torch.equal(out[:, :, :n], ref[:, :, :n]), wl.name
        if n < out.shape[2]:
            assert torch.isnan(out[:, :, n:]).all()


def test_static_scratch_call_replays_from_a_hip_graph():
    """What the entry point is for: it can be captured (no allocation, no workspace argument to keep alive).  The first
    call on the device is made before the capture (it looks the scratch array's address up); every replay reproduces the
    eager result bit for bit, with eager work of the same library between the replays."""
    import paper_2605_04569_amd as I
    I.lib()
    wl = SMALL.with_(gamma=0.25)
    q, k, v = (t.cuda() for t in W.make_inputs(wl, "cpu"))
    ref = _reference(I, wl, q, k, v)
    pr = problem_of(wl)
    out = torch.zeros_like(q)
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):
        I.isa_attention_static(pr, q, k, v, out)                    # warm-up on the capture stream
    torch.cuda.current_stream().wait_stream(side)
    torch.cuda.synchronize()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph):
        I.isa_attention_static(pr, q, k, v, out)
    n = wl.tokens(0)
    for rep in range(3):
        out.zero_()
        graph.replay()
        torch.cuda.synchronize()
        assert torch.equal(out[:, :, :n], ref[:, :, :n]), rep
        big = BIG
        qb, kb, vb = (t.cuda() for t in W.make_inputs(big, "cpu"))
        I.isa_attention_static(problem_of(big), qb, kb, vb, torch.empty_like(qb))    # another problem through the same scratch
        torch.cuda.synchronize()


def test_static_scratch_rejects_what_does_not_fit():
    """cfg2's forward-only workspace (0.7 GB) is beyond the array: a clear error, nothing launched."""
    import paper_2605_04569_amd as I
    pr = problem_of(W.CONFIGS["cfg2"])
    cp, keep = pr.c_struct()
    one = C.c_void_p(256)                              # never dereferenced: the size check comes before any launch
    assert I.lib().isa_attention_static(C.byref(cp), one, one, one, one, None) == -6
    assert I.lib().isa_attention_static(C.byref(cp), one, one, None, one, None) == -1
