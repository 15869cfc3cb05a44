"""GPU parity of the full-precision input gradient on the outlier channels against the CPU oracle."""
import sys

import numpy as np
import pytest

from paper_2505_14742_amd import synth

pytestmark = pytest.mark.gpu


def _say(msg):
    print(msg, flush=True)
    sys.stdout.flush()


def _run(X, dY, W, O, A, B, scale, tag):
    import torch
    from oracle import api as orc
    from paper_2505_14742_amd import binding as q
    from tests.gpu_harness import DEV, Layer, assert_close_fp32, bf16_dev, host
    t, c_out = dY.shape
    c_in = W.shape[0]
    r = 0 if A is None else A.shape[1]
    _say("%s: t=%d c_in=%d c_out=%d n=%d r=%d" % (tag, t, c_in, c_out, O.size, r))
    L = Layer(W, O, A, B, scale, t)
    Gd = bf16_dev(dY)
    L.linear_bwd_dx(Gd)
    before = L.dX.clone()
    ws = torch.empty(q.bwd_dx_outlier_workspace_bytes(t, c_out), dtype=torch.int8, device=DEV)
    q.bwd_dx_outlier_exact(Gd, c_in, L.O, L.W_O, L.A, L.B, r, scale, L.dX, ws)
    W_O, _ = orc.outlier_rows(W, O)
    exact, _ = orc.bwd_dx_outlier_cols(dY, O, W_O, lora_A=A, lora_B=B, lora_scale=scale)
    got = host(L.dX)
    if O.size:
        err = assert_close_fp32(got[:, O], exact, tag + " dX[:, O]")
        # the call did replace something: the quantized columns are much farther from the true gradient on O
        old = host(before)[:, O]
        assert np.linalg.norm(got[:, O] - exact) < 0.1 * np.linalg.norm(old - exact), tag + " not closer to dX*"
    else:
        err = 0.0
    keep = np.ones(c_in, bool)
    keep[O] = False
    assert np.array_equal(got[:, keep], host(before)[:, keep]), tag + " other columns were touched"
    _say("%s ok: err %.2e" % (tag, err))


_EDGE = [i for i, e in enumerate(synth.EDGE_CASES) if e.t <= 2051 and e.c_out <= 4096]


@pytest.mark.parametrize("idx", _EDGE, ids=[synth.EDGE_CASES[i].name for i in _EDGE])
def test_outlier_grad_edge_cases(idx):
    ec = synth.EDGE_CASES[idx]
    X, dY, W, O, A, B = synth.edge_case_inputs(ec, idx)
    has = ec.lora_rank > 0
    _run(X, dY, W, O, A if has else None, B if has else None, 0.5, "edge " + ec.name)


@pytest.mark.parametrize("cfg,name", [(2, "qkv"), (3, "down"), (4, "q"), (5, "q")])
def test_outlier_grad_workloads(cfg, name):
    p = synth.projection(cfg, name)
    A, B = synth.lora(p)
    _run(None, synth.out_grad(p, 0), synth.weight(p), synth.outlier_indices(p), A, B, p.lora_scale,
         "cfg%d %s" % (cfg, name))
