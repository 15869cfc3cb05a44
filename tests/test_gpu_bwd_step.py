"""The one-call backward step (quaff_linear_bwd_step) against the two calls it stands for and against the oracle."""
import sys

import numpy as np
import pytest

from paper_2505_14742_amd import synth

pytestmark = pytest.mark.gpu


def _run(W, O, A, B, scale, X, dY, tag):
    import torch
    from oracle import api as orc
    from paper_2505_14742_amd import binding as q
    from tests.gpu_harness import DEV, Layer, assert_close_fp32, bf16_dev, host
    print(tag, flush=True)
    sys.stdout.flush()
    t = X.shape[0]
    L = Layer(W, O, A, B, scale, t)
    Xd, Gd = bf16_dev(X), bf16_dev(dY)
    r = L.r
    # the two separate calls
    L.linear_bwd_dx(Gd)
    dX_two = L.dX.clone()
    ws2 = torch.empty(q.lora_bwd_workspace_bytes(t, L.c_in, L.c_out, r), dtype=torch.int8, device=DEV)
    dA_two = torch.empty((L.c_in, r), dtype=torch.float32, device=DEV)
    dB_two = torch.empty((r, L.c_out), dtype=torch.float32, device=DEV)
    q.lora_bwd_weights(Xd, Gd, L.A, L.B, r, scale, dA_two, dB_two, ws2)
    dA_o, dB_o = orc.lora_grads(X, dY, A, B, scale)
    # the one call, on a scribbled workspace and NaN-filled outputs: everything on the caller's stream, then with the
    # weight gradients on a second stream of the caller's (used twice in a row: the events are reusable)
    side = q.SideStream()
    for how, sd in (("one stream", None), ("side stream", side), ("side stream again", side)):
        ws = torch.full((q.bwd_step_workspace_bytes(t, L.c_in, L.c_out, r),), 0x5A, dtype=torch.int8, device=DEV)
        dX = torch.full((t, L.c_in), float("nan"), dtype=torch.float32, device=DEV)
        dA = torch.full((L.c_in, r), float("nan"), dtype=torch.float32, device=DEV)
        dB = torch.full((r, L.c_out), float("nan"), dtype=torch.float32, device=DEV)
        q.linear_bwd_step(Gd, Xd, L.Wq_packed, L.delta_w, L.c_in, L.c_out, L.A, L.B, r, scale, dX, dA, dB, ws, side=sd)
        # no synchronize here: what follows on the caller's stream must already be ordered after the side stream's work
        dX_c, dA_c, dB_c = dX.clone(), dA.clone(), dB.clone()
        torch.cuda.synchronize()
        tg = "%s (%s)" % (tag, how)
        # dX and dB take the same kernels on the same inputs: same bits.  dA uses the down-projection dY B^T that the
        # dX launch produced, whose fp32 partial sums may be added in another order than the stand-alone one's.
        assert torch.equal(dX_c, dX_two), tg + ": dX differs from quaff_linear_bwd_dx"
        assert torch.equal(dB_c, dB_two), tg + ": dB differs from quaff_lora_bwd_weights"
        assert_close_fp32(host(dA_c), dA_o, tg + " dA vs oracle")
        assert_close_fp32(host(dB_c), dB_o, tg + " dB vs oracle")
        tol = 2e-5 * max(1.0, float(dA_two.abs().max()))
        assert float((dA_c - dA_two).abs().max()) <= tol, tg + ": dA differs from quaff_lora_bwd_weights beyond rounding"


_EDGE = [i for i, e in enumerate(synth.EDGE_CASES) if e.lora_rank > 0]


@pytest.mark.parametrize("idx", _EDGE, ids=[synth.EDGE_CASES[i].name for i in _EDGE])
def test_bwd_step_edge_cases(idx):
    ec = synth.EDGE_CASES[idx]
    X, dY, W, O, A, B = synth.edge_case_inputs(ec, idx)
    _run(W, O, A, B, 0.5, X, dY, "edge " + ec.name)


@pytest.mark.parametrize("cfg,name", [(2, "qkv"), (2, "o_proj"), (3, "down"), (4, "q")])
def test_bwd_step_workloads(cfg, name):
    p = synth.projection(cfg, name)
    A, B = synth.lora(p)
    _run(synth.weight(p), synth.outlier_indices(p), A, B, p.lora_scale, synth.activations(p, 0), synth.out_grad(p, 0),
         "cfg%d %s" % (cfg, name))


def test_bwd_step_argument_errors():
    import torch
    from paper_2505_14742_amd import binding as q
    from tests.gpu_harness import DEV, Layer, bf16_dev
    ec = synth.EDGE_CASES[0]
    X, dY, W, O, A, B = synth.edge_case_inputs(ec, 0)
    L = Layer(W, O, A, B, 1.0, ec.t)
    Xd, Gd = bf16_dev(X), bf16_dev(dY)
    r = L.r
    ws = torch.empty(q.bwd_step_workspace_bytes(ec.t, L.c_in, L.c_out, r), dtype=torch.int8, device=DEV)
    dX = torch.empty((ec.t, L.c_in), dtype=torch.float32, device=DEV)
    dA = torch.empty((L.c_in, r), dtype=torch.float32, device=DEV)
    dB = torch.empty((r, L.c_out), dtype=torch.float32, device=DEV)
    q.linear_bwd_step(Gd, Xd, L.Wq_packed, L.delta_w, L.c_in, L.c_out, L.A, L.B, r, 1.0, dX, dA, dB, ws)
    with pytest.raises(q.QuaffError, match="WORKSPACE"):
        q.linear_bwd_step(Gd, Xd, L.Wq_packed, L.delta_w, L.c_in, L.c_out, L.A, L.B, r, 1.0, dX, dA, dB, ws[:4096])
    with pytest.raises(q.QuaffError, match="SHAPE"):
        q.linear_bwd_step(Gd, Xd, L.Wq_packed, L.delta_w, L.c_in, L.c_out, L.A, L.B, 0, 1.0, dX, dA, dB, ws)
    with pytest.raises(q.QuaffError, match="NULL"):
        q.linear_bwd_step(Gd, Xd, L.Wq_packed, L.delta_w, L.c_in, L.c_out, L.A, L.B, r, 1.0, dX, None, dB, ws)
    assert q.bwd_step_workspace_bytes(ec.t, L.c_in, L.c_out, 0) == 0
