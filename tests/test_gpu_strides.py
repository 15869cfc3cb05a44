"""Leading dimensions larger than the row length (views into wider buffers) give the same bits as dense buffers,
and nothing outside the views is written."""
import numpy as np
import pytest

from paper_2505_14742_amd import synth

pytestmark = pytest.mark.gpu


def _wide(t_, pad, fill):
    """A [rows x cols] view with leading dimension cols + pad inside a buffer filled with `fill`."""
    import torch
    rows, cols = t_.shape
    big = torch.full((rows, cols + pad), fill, dtype=t_.dtype, device=t_.device)
    big[:, :cols] = t_
    return big, big[:, :cols]


@pytest.mark.parametrize("idx", [1, 4, 6])   # adjacent outliers r=16; n=65 r=32; ragged rows
def test_padded_leading_dimensions(idx):
    import torch
    from paper_2505_14742_amd import binding as q
    from tests.gpu_harness import DEV, Layer, bf16_dev
    ec = synth.EDGE_CASES[idx]
    X, dY, W, O, A, B = synth.edge_case_inputs(ec, idx)
    print("strided", ec.name, flush=True)
    Ld, Ls = Layer(W, O, A, B, 0.5, ec.t), Layer(W, O, A, B, 0.5, ec.t)
    Xd, Gd = bf16_dev(X), bf16_dev(dY)
    Xbig, Xv = _wide(Xd, 64, 0x7F7F)          # padding holds huge bf16 values: must never be read as data
    Gbig, Gv = _wide(Gd, 24, 0x7F7F)
    for step in range(2):
        # dense reference
        Ld.scale_update(Xd, 0.2); Ld.quant_act(Xd); Ld.linear_fwd(Xd); Ld.linear_bwd_dx(Gd)
        # views with padded leading dimensions, outputs into padded buffers too
        Ybig, Yv = _wide(torch.zeros_like(Ld.Y), 40, -7.0)
        dXbig, dXv = _wide(torch.zeros_like(Ld.dX), 8, -7.0)
        Ls.Y, Ls.dX = Yv, dXv
        if step == 0:
            Ls.scale_update(Xv, 0.2); Ls.quant_act(Xv); Ls.linear_fwd(Xv)
        else:
            Ls.fwd_step(Xv, 0.2)
        Ls.linear_bwd_dx(Gv)
        torch.cuda.synchronize()
        for f in ("s_O", "what_int", "Xq", "delta_x", "xq_O"):
            assert torch.equal(getattr(Ld, f), getattr(Ls, f)), "%s step %d: %s" % (ec.name, step, f)
        assert torch.equal(Ld.Y, Yv) and torch.equal(Ld.dX, dXv), "%s step %d: outputs" % (ec.name, step)
        assert torch.all(Ybig[:, Ld.c_out:] == -7.0) and torch.all(dXbig[:, Ld.c_in:] == -7.0), "padding written"
    # LoRA weight gradients and the exact outlier columns on the same views
    r = Ld.r
    ws = torch.empty(q.lora_bwd_workspace_bytes(ec.t, Ld.c_in, Ld.c_out, r), dtype=torch.int8, device=DEV)
    outs = []
    for xin, gin in ((Xd, Gd), (Xv, Gv)):
        dA = torch.empty((Ld.c_in, r), dtype=torch.float32, device=DEV)
        dB = torch.empty((r, Ld.c_out), dtype=torch.float32, device=DEV)
        q.lora_bwd_weights(xin, gin, Ld.A, Ld.B, r, 0.5, dA, dB, ws)
        outs.append((dA, dB))
    assert torch.equal(outs[0][0], outs[1][0]) and torch.equal(outs[0][1], outs[1][1]), "lora grads on views"
    ws2 = torch.empty(q.bwd_dx_outlier_workspace_bytes(ec.t, Ld.c_out), dtype=torch.int8, device=DEV)
    q.bwd_dx_outlier_exact(Gd, Ld.c_in, Ld.O, Ld.W_O, Ld.A, Ld.B, r, 0.5, Ld.dX, ws2)
    q.bwd_dx_outlier_exact(Gv, Ld.c_in, Ld.O, Ld.W_O, Ld.A, Ld.B, r, 0.5, dXv, ws2)
    assert torch.equal(Ld.dX, dXv) and torch.all(dXbig[:, Ld.c_in:] == -7.0), "exact outlier columns on views"
