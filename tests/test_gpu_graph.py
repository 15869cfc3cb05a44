"""The per-step calls allocate nothing and never synchronize, so a step can be captured into a HIP graph: a captured
forward + backward step is replayed several times, with eager work in between, and every replay must give the bits of
the eager step on the same inputs."""
import sys

import pytest

from paper_2505_14742_amd import synth

pytestmark = pytest.mark.gpu


def _layer(ec_idx):
    from tests.gpu_harness import Layer, bf16_dev
    ec = synth.EDGE_CASES[ec_idx]
    X, dY, W, O, A, B = synth.edge_case_inputs(ec, ec_idx)
    return Layer(W, O, A, B, 0.5, ec.t), bf16_dev(X), bf16_dev(dY), ec


@pytest.mark.parametrize("one_call_backward", [False, True])
def test_captured_step_replays_bit_exact(one_call_backward):
    import torch
    from paper_2505_14742_amd import binding as q
    from tests.gpu_harness import DEV
    idx = [i for i, e in enumerate(synth.EDGE_CASES) if e.name == "adjacent"][0]
    L, Xd, Gd, ec = _layer(idx)
    print("graph capture of one step, edge case %s, one-call backward %s" % (ec.name, one_call_backward), flush=True)
    sys.stdout.flush()
    r = L.r
    dA = torch.zeros((L.c_in, r), dtype=torch.float32, device=DEV)
    dB = torch.zeros((r, L.c_out), dtype=torch.float32, device=DEV)
    bws = torch.empty(q.bwd_step_workspace_bytes(ec.t, L.c_in, L.c_out, r), dtype=torch.int8, device=DEV)

    second = q.SideStream() if one_call_backward else None   # the caller's second stream: fork / join become graph nodes

    def step():
        L.fwd_step(Xd, 0.2)
        if one_call_backward:
            q.linear_bwd_step(Gd, Xd, L.Wq_packed, L.delta_w, L.c_in, L.c_out, L.A, L.B, r, L.lora_scale, L.dX, dA, dB,
                              bws, side=second)
        else:
            L.linear_bwd_dx(Gd)

    state = [L.s_O, L.colscale]
    s0 = [x.clone() for x in state]
    # eager reference: two steps from the initial state (the scaling factors carry over from step to step)
    step()
    torch.cuda.synchronize()
    ref1 = [L.Y.clone(), L.dX.clone(), L.Xq.clone(), L.s_O.clone(), dA.clone(), dB.clone()]
    step()
    torch.cuda.synchronize()
    ref2 = [L.Y.clone(), L.dX.clone(), L.Xq.clone(), L.s_O.clone(), dA.clone(), dB.clone()]
    # capture one step (a warm-up step on the capture stream first, as the framework asks), then replay it twice from
    # the initial state with unrelated eager work in between
    for x, x0 in zip(state, s0):
        x.copy_(x0)
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):
        step()
    torch.cuda.current_stream().wait_stream(side)
    torch.cuda.synchronize()
    for x, x0 in zip(state, s0):
        x.copy_(x0)
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph):
        step()
    torch.cuda.synchronize()
    for x, x0 in zip(state, s0):
        x.copy_(x0)
    for ref in (ref1, ref2):
        L.Y.fill_(float("nan"))
        L.dX.fill_(float("nan"))
        junk = torch.randn(1 << 20, device=DEV).sum()        # eager work between the replays
        graph.replay()
        torch.cuda.synchronize()
        got = [L.Y, L.dX, L.Xq, L.s_O, dA, dB]
        names = ["Y", "dX", "Xq", "s_O", "dA", "dB"]
        for n, a, b in zip(names, got, ref):
            if not one_call_backward and n in ("dA", "dB"):
                continue
            assert torch.equal(a, b), "replay differs from the eager step in " + n
        assert torch.isfinite(junk)
