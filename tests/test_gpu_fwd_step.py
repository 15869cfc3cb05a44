"""The one-call forward step must reproduce the three separate calls bit for bit (outputs and state)."""
import sys

import numpy as np
import pytest

from paper_2505_14742_amd import synth

pytestmark = pytest.mark.gpu

_FIELDS = ["s_O", "colscale", "what_int", "delta_what", "cmax", "Xq", "delta_x", "xq_O", "Y"]


def _compare(W, O, A, B, scale, batches, gamma, tag):
    import torch
    from tests.gpu_harness import Layer, bf16_dev
    print(tag, flush=True)
    sys.stdout.flush()
    t = batches[0].shape[0]
    L1, L2 = Layer(W, O, A, B, scale, t), Layer(W, O, A, B, scale, t)
    for step, X in enumerate(batches):
        Xd = bf16_dev(X)
        L1.scale_update(Xd, gamma)
        L1.quant_act(Xd)
        L1.linear_fwd(Xd)
        L2.fwd_step(Xd, gamma)
        torch.cuda.synchronize()
        for f in _FIELDS:
            if not L1.n and f in ("s_O", "what_int", "delta_what", "cmax", "xq_O"):
                continue
            a, b = getattr(L1, f), getattr(L2, f)
            if f == "cmax" or f == "s_O":
                a, b = a[:max(L1.n, 1)], b[:max(L1.n, 1)]
            assert torch.equal(a, b), "%s step %d: %s differs" % (tag, step, f)


_EDGE = [i for i, e in enumerate(synth.EDGE_CASES)]


@pytest.mark.parametrize("idx", _EDGE, ids=[synth.EDGE_CASES[i].name for i in _EDGE])
def test_fwd_step_edge_cases(idx):
    ec = synth.EDGE_CASES[idx]
    X, dY, W, O, A, B = synth.edge_case_inputs(ec, idx)
    has = ec.lora_rank > 0
    X2 = X[::-1].copy()                                      # a second, different batch
    _compare(W, O, A if has else None, B if has else None, 0.5, [X, X2, X], 0.2, "edge " + ec.name)


@pytest.mark.parametrize("cfg,name", [(1, "single"), (2, "qkv"), (2, "o_proj"), (3, "down"), (4, "q"), (5, "q"), (6, "down")])
def test_fwd_step_workloads(cfg, name):
    p = synth.projection(cfg, name)
    A, B = synth.lora(p)
    if p.lora_rank == 0:
        A = B = None
    _compare(synth.weight(p), synth.outlier_indices(p), A, B, p.lora_scale,
             [synth.activations(p, s) for s in range(2)], p.gamma, "cfg%d %s" % (cfg, name))


@pytest.mark.parametrize("case", ["edge_adjacent", "edge_ragged_rows", "cfg2_o_proj", "cfg3_down", "cfg1_single"])
def test_fwd_step_when_the_grid_wide_wait_gives_up(case):
    """The one-launch form bounds its wait for the other workgroups' column maxima.  With the bound forced to zero
    from the host, every workgroup but the last to arrive gives up and recomputes the maxima from X itself: the
    kernels still finish normally and every result must still be the bits of the three separate calls."""
    from paper_2505_14742_amd import binding as q
    if case.startswith("edge_"):
        idx = [i for i, e in enumerate(synth.EDGE_CASES) if e.name == case[5:]][0]
        ec = synth.EDGE_CASES[idx]
        X, dY, W, O, A, B = synth.edge_case_inputs(ec, idx)
        args = (W, O, A, B, 0.5, [X, X[::-1].copy()], 0.2)
    else:
        cfg, name = int(case[3]), case[5:]
        p = synth.projection(cfg, name)
        A, B = synth.lora(p)
        if p.lora_rank == 0:
            A = B = None
        args = (synth.weight(p), synth.outlier_indices(p), A, B, p.lora_scale,
                [synth.activations(p, s) for s in range(2)], p.gamma)
    prev = q.debug_grid_wait_ticks(0)
    try:
        assert q.debug_grid_wait_ticks(-1) == 0
        _compare(*args, "give-up path " + case)
    finally:
        q.debug_grid_wait_ticks(prev)
    assert q.debug_grid_wait_ticks(-1) == prev
