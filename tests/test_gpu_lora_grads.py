"""GPU parity of the LoRA weight gradients (dA, dB) against the CPU oracle, through the C ABI."""
import sys

import numpy as np
import pytest

from paper_2505_14742_amd import synth

pytestmark = pytest.mark.gpu


def _say(msg):
    print(msg, flush=True)
    sys.stdout.flush()


def _run(X, dY, A, B, scale, tag):
    import torch
    from oracle import api as orc
    from paper_2505_14742_amd import binding as q
    from tests.gpu_harness import DEV, assert_close_fp32, bf16_dev, host
    t, c_in = X.shape
    c_out, r = dY.shape[1], A.shape[1]
    _say("%s: t=%d c_in=%d c_out=%d r=%d" % (tag, t, c_in, c_out, r))
    Xd, Gd, Ad, Bd = bf16_dev(X), bf16_dev(dY), bf16_dev(A), bf16_dev(B)
    ws = torch.empty(q.lora_bwd_workspace_bytes(t, c_in, c_out, r), dtype=torch.int8, device=DEV)
    dA = torch.full((c_in, r), float("nan"), dtype=torch.float32, device=DEV)
    dB = torch.full((r, c_out), float("nan"), dtype=torch.float32, device=DEV)
    q.lora_bwd_weights(Xd, Gd, Ad, Bd, r, scale, dA, dB, ws)
    dA_o, dB_o = orc.lora_grads(X, dY, A, B, scale)
    ea = assert_close_fp32(host(dA), dA_o, tag + " dA")
    eb = assert_close_fp32(host(dB), dB_o, tag + " dB")
    # reproducible: a second call on a scribbled workspace gives the same bits
    ws.fill_(0x5A)
    dA2, dB2 = torch.empty_like(dA), torch.empty_like(dB)
    q.lora_bwd_weights(Xd, Gd, Ad, Bd, r, scale, dA2, dB2, ws)
    assert torch.equal(dA, dA2) and torch.equal(dB, dB2), tag + " not reproducible"
    # a third call on the workspace the second one left, with the scale doubled: a power of two scales every
    # intermediate exactly, so the results must be exactly twice the first ones (partial results or ticket counts
    # left over from the call before would show here)
    dA3, dB3 = torch.empty_like(dA), torch.empty_like(dB)
    q.lora_bwd_weights(Xd, Gd, Ad, Bd, r, 2.0 * scale, dA3, dB3, ws)
    assert torch.equal(dA3, 2.0 * dA) and torch.equal(dB3, 2.0 * dB), tag + " stale workspace contents used"
    _say("%s ok: dA err %.2e dB err %.2e" % (tag, ea, eb))


_EDGE = [i for i, e in enumerate(synth.EDGE_CASES) if e.lora_rank > 0]


@pytest.mark.parametrize("idx", _EDGE, ids=[synth.EDGE_CASES[i].name for i in _EDGE])
def test_lora_grads_edge_cases(idx):
    ec = synth.EDGE_CASES[idx]
    X, dY, W, O, A, B = synth.edge_case_inputs(ec, idx)
    _run(X, dY, A, B, 0.5, "edge " + ec.name)


@pytest.mark.parametrize("cfg,name", [(2, "qkv"), (2, "o_proj"), (3, "down"), (4, "gate"), (4, "down")])
def test_lora_grads_workloads(cfg, name):
    p = synth.projection(cfg, name)
    A, B = synth.lora(p)
    _run(synth.activations(p, 0), synth.out_grad(p, 0), A, B, p.lora_scale, "cfg%d %s" % (cfg, name))


def test_lora_grads_argument_errors():
    import torch
    from paper_2505_14742_amd import binding as q
    from tests.gpu_harness import DEV
    t, c_in, c_out, r = 64, 128, 96, 16
    z = lambda *s: torch.zeros(s, dtype=torch.int16, device=DEV)
    X, G, A, B = z(t, c_in), z(t, c_out), z(c_in, r), z(r, c_out)
    dA = torch.zeros((c_in, r), dtype=torch.float32, device=DEV)
    dB = torch.zeros((r, c_out), dtype=torch.float32, device=DEV)
    ws = torch.empty(q.lora_bwd_workspace_bytes(t, c_in, c_out, r), dtype=torch.int8, device=DEV)
    q.lora_bwd_weights(X, G, A, B, r, 1.0, dA, dB, ws)
    with pytest.raises(q.QuaffError, match="WORKSPACE"):
        q.lora_bwd_weights(X, G, A, B, r, 1.0, dA, dB, ws[:1024])
    with pytest.raises(q.QuaffError, match="SHAPE"):
        q.lora_bwd_weights(X, G, A, B, 24, 1.0, dA, dB, ws)
    with pytest.raises(q.QuaffError, match="SHAPE"):
        q.lora_bwd_weights(X, G, A, B, 0, 1.0, dA, dB, ws)
    with pytest.raises(q.QuaffError, match="NULL"):
        q.lora_bwd_weights(X, G, A, B, r, 1.0, None, dB, ws)
