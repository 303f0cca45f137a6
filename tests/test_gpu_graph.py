"""The single-tensor calls only launch kernels on the caller's stream (no
allocation, no host-to-device copy, no synchronisation), so they can be
recorded into a HIP graph and replayed.  Every replay is checked against an
eager call on the same input and one against the oracle; between replays the
program does eager work of its own and synchronises.
"""
import numpy as np
import pytest

from oracle import pwlq_ref as R
from paper_2002_00104_amd import synth
from parity import assert_quantize_matches, assert_search_matches

pytestmark = pytest.mark.gpu


@pytest.mark.parametrize("fast", [False, True])
@pytest.mark.parametrize("shape,mode,bits,n", [((64, 576), synth.PER_CHANNEL, 4, 100),
                                               ((40, 700), synth.PER_TENSOR, 3, 300)])
def test_search_and_quantize_replay_from_a_graph(shape, mode, bits, n, fast):
    import torch
    from paper_2002_00104_amd import pwlq as P

    rng = np.random.default_rng(5)
    first = rng.laplace(0, 0.05, size=shape).astype(np.float32)
    wd = torch.from_numpy(first).cuda()          # the graph's input buffer
    # warm-up outside the capture, on a side stream as torch asks
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):
        for _ in range(2):
            o = P.search(wd, bits, n, mode, fast=fast)
            P.quantize(wd, bits, o["p_star"], o["m"], mode)
    torch.cuda.current_stream().wait_stream(side)
    torch.cuda.synchronize()

    g = torch.cuda.CUDAGraph()
    with torch.cuda.graph(g):
        out = P.search(wd, bits, n, mode, fast=fast)
        q = P.quantize(wd, bits, out["p_star"], out["m"], mode)
    torch.cuda.synchronize()

    for rep in range(4):
        w = (rng.standard_normal(shape) * np.exp(rng.normal(-3, 1))).astype(np.float32)
        wd.copy_(torch.from_numpy(w))            # eager work between the replays
        for v in out.values():
            v.zero_()
        torch.cuda.synchronize()
        g.replay()
        torch.cuda.synchronize()
        got = {k: v.clone() for k, v in out.items()}
        gq = tuple(t.clone() for t in q)
        eager = P.search(wd, bits, n, mode, fast=fast)
        eq = P.quantize(wd, bits, eager["p_star"], eager["m"], mode)
        torch.cuda.synchronize()
        for k in ("k_star", "p_star", "m", "mse"):
            assert torch.equal(got[k], eager[k]), f"replay {rep}: {k} differs from the eager call"
        for a, b, name in zip(gq, eq, ("codes", "flags", "w_hat")):
            assert torch.equal(a, b), f"replay {rep}: {name} differs from the eager call"
        if rep == 3:
            r = R.search(w, bits, n, mode, want_curve=True)
            assert_search_matches({k: v.cpu().numpy() for k, v in got.items()}, r, "graph replay")
            ps, ms = got["p_star"].cpu().numpy(), got["m"].cpu().numpy()
            assert_quantize_matches(tuple(t.cpu().numpy() for t in gq),
                                    R.quantize(w, bits, ps, ms, mode), "graph replay")


def test_list_calls_replay_from_a_graph():
    """A list call writes its table through kernel arguments, so it can be recorded too."""
    import torch
    from paper_2002_00104_amd import pwlq as P

    rng = np.random.default_rng(6)
    shapes = [(8, 100), (3, 9000), (20, 33)]
    tensors = [torch.from_numpy(rng.standard_normal(s).astype(np.float32)).cuda() for s in shapes]
    tl = P.TensorList(tensors, synth.PER_CHANNEL)
    ws = torch.empty(P.search_list_workspace_bytes(tl, 4, 50), dtype=torch.uint8, device="cuda")
    wq = torch.empty(max(256, P.quantize_list_workspace_bytes(tl, 4)), dtype=torch.uint8, device="cuda")
    out = P.alloc_search_outputs(tl.n_groups, "cuda")
    qout = P.alloc_quantize_outputs(tl.n_elements, "cuda")
    P.search_list(tl, 4, 50, workspace=ws, out=out)
    P.quantize_list(tl, 4, out["p_star"], out["m"], workspace=wq, out=qout)
    torch.cuda.synchronize()
    g = torch.cuda.CUDAGraph()
    with torch.cuda.graph(g):
        P.search_list(tl, 4, 50, workspace=ws, out=out)
        P.quantize_list(tl, 4, out["p_star"], out["m"], workspace=wq, out=qout)
    torch.cuda.synchronize()
    for rep in range(3):
        for t, s in zip(tensors, shapes):        # eager work between the replays
            t.copy_(torch.from_numpy((rng.standard_normal(s) * 0.07).astype(np.float32)))
        ws.zero_()                               # the table in the workspace head is rewritten by the graph
        torch.cuda.synchronize()
        g.replay()
        torch.cuda.synchronize()
        got = {k: v.clone() for k, v in out.items()}
        gq = tuple(t.clone() for t in qout)
        eager = P.search_list(tl, 4, 50, workspace=ws, out=P.alloc_search_outputs(tl.n_groups, "cuda"))
        eq = P.quantize_list(tl, 4, eager["p_star"], eager["m"], workspace=wq,
                             out=P.alloc_quantize_outputs(tl.n_elements, "cuda"))
        torch.cuda.synchronize()
        for k in ("k_star", "p_star", "m", "mse"):
            assert torch.equal(got[k], eager[k]), f"replay {rep}: {k}"
        for a, b in zip(gq, eq):
            assert torch.equal(a, b), f"replay {rep}: quantizer output"
    go = 0
    for t in tensors:
        r = R.search(t.cpu().numpy(), 4, 50, synth.PER_CHANNEL, want_curve=True)
        C = t.shape[0]
        assert_search_matches({k: v[go:go + C].cpu().numpy() for k, v in got.items()}, r, "list graph replay")
        go += C
