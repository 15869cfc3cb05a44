"""Long inputs at rank 16 take the persistent LoRA down-projection, which also yields the abs-max of the outlier
columns (Eq. 8) in the one-call forward step.  Every slice length it is instantiated for is compared with the oracle
(scaling factors, codes and accumulators bit for bit, Y within the fp32 tolerance), and the one-call forward step with
the three separate calls bit for bit (the separate scale update uses the stand-alone abs-max kernel)."""
import sys

import numpy as np
import pytest

from paper_2505_14742_amd import synth

pytestmark = pytest.mark.gpu

# (t, c_in, outliers): 32-column steps per wavefront slice 8, 10, 12, 14 (the shorter ones are edge cases of the
# shared list); c_out stays small so that the oracle takes seconds
_CASES = [
    (4096 + 7, 8192, [0, 5, 4095, 4096, 8191]),
    (4096 + 16, 9216, [3, 4, 4607, 4608, 9000, 9215]),
    (4096 + 1, 11008, [0, 5503, 5504, 5505, 11007]),
    (4096 + 33, 13824, list(range(6900, 6924)) + [0, 13823]),
]


@pytest.mark.parametrize("t,c_in,outliers", _CASES, ids=["c%d" % c[1] for c in _CASES])
def test_long_inputs(t, c_in, outliers):
    import torch
    from tests.gpu_harness import Layer, OracleLayer, bf16_dev, check_prepare, check_step
    ec = synth.EdgeCase("long_rows_c%d" % c_in, t, c_in, 64, outliers, 16, zero_rows=[5])
    print("long input t=%d c_in=%d n=%d" % (t, c_in, len(outliers)), flush=True)
    sys.stdout.flush()
    X, dY, W, O, A, B = synth.edge_case_inputs(ec, 70 + len(outliers))
    L, R = Layer(W, O, A, B, 1.0, t), OracleLayer(W, O, A, B, 1.0)
    check_prepare(L, R)
    X2 = X[::-1].copy()
    for step, Xs in enumerate((X, X2)):
        check_step(L, R, Xs, dY, 0.2, tag="long c=%d step %d" % (c_in, step))
    # the one-call forward (abs-max inside the down-projection) against the state the separate calls left
    L2 = Layer(W, O, A, B, 1.0, t)
    for Xs in (X, X2):
        L2.fwd_step(bf16_dev(Xs), 0.2)
    torch.cuda.synchronize()
    for f in ("s_O", "colscale", "what_int", "delta_what", "Xq", "delta_x", "xq_O", "Y"):
        assert torch.equal(getattr(L, f), getattr(L2, f)), f
    n = len(outliers)
    assert torch.equal(L.cmax[:n], L2.cmax[:n])


# long gradients (at least 1024 groups of 8 rows) with rows of 5136 .. 14336 columns: the backward quantizer +
# down-projection reads dY once with L fetched per row group; both slice lengths it is instantiated for, ragged rows
@pytest.mark.parametrize("t,c_out", [(8192 + 13, 9216), (8192 + 1, 13824), (8192 + 8, 5136)],
                         ids=["c_out9216", "c_out13824", "c_out5136"])
def test_long_gradients(t, c_out):
    from tests.gpu_harness import Layer, OracleLayer, check_prepare, check_step
    ec = synth.EdgeCase("long_grad_c%d" % c_out, t, 64, c_out, [3, 60], 16, zero_rows=[7, t - 1])
    print("long gradient t=%d c_out=%d" % (t, c_out), flush=True)
    sys.stdout.flush()
    X, dY, W, O, A, B = synth.edge_case_inputs(ec, 77)
    L, R = Layer(W, O, A, B, 1.0, t), OracleLayer(W, O, A, B, 1.0)
    check_prepare(L, R)
    check_step(L, R, X, dY, 0.2, tag="long gradient c_out=%d" % c_out)
