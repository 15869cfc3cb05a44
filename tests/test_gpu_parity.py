"""GPU parity: the HIP path (through the C ABI) against the CPU oracle, element by element."""
import sys
import time

import numpy as np
import pytest

from paper_2505_14742_amd import synth

pytestmark = pytest.mark.gpu


def _say(msg):
    print(msg, flush=True)
    sys.stdout.flush()


@pytest.mark.parametrize("idx", range(len(synth.EDGE_CASES)), ids=[e.name for e in synth.EDGE_CASES])
def test_edge_cases(idx):
    from tests.gpu_harness import Layer, OracleLayer, check_prepare, check_step
    ec = synth.EDGE_CASES[idx]
    _say("edge case %s t=%d c_in=%d c_out=%d n=%d r=%d" % (ec.name, ec.t, ec.c_in, ec.c_out, len(ec.outliers),
                                                           ec.lora_rank))
    X, dY, W, O, A, B = synth.edge_case_inputs(ec, idx)
    L = Layer(W, O, A if ec.lora_rank else None, B if ec.lora_rank else None, 1.0, ec.t)
    R = OracleLayer(W, O, A if ec.lora_rank else None, B if ec.lora_rank else None, 1.0)
    check_prepare(L, R)
    for step in range(2):
        check_step(L, R, X, dY, 0.2, tag="%s step %d" % (ec.name, step))


def test_config1_all_steps_full_compare():
    from tests.gpu_harness import Layer, OracleLayer, check_prepare, check_step
    p = synth.projection(1, "single")
    W, O = synth.weight(p), synth.outlier_indices(p)
    L, R = Layer(W, O, None, None, 0.0, p.t), OracleLayer(W, O, None, None, 0.0)
    check_prepare(L, R)
    for step in range(p.steps):
        _say("config 1 step %d" % step)
        check_step(L, R, synth.activations(p, step), None, p.gamma, backward=False, tag="cfg1 step %d" % step)


def _run_projection(p, steps, prepare_check=True, all_rows=True):
    """all_rows: every element of Y, dX and the accumulators is compared; otherwise the products are compared on a
    deterministic row subset (the long-sequence workload: a full oracle step takes minutes there)."""
    from tests.gpu_harness import Layer, OracleLayer, check_prepare, check_step, sample_rows
    t0 = time.time()
    W, O = synth.weight(p), synth.outlier_indices(p)
    A, B = synth.lora(p)
    L, R = Layer(W, O, A, B, p.lora_scale, p.t), OracleLayer(W, O, A, B, p.lora_scale)
    if prepare_check:
        check_prepare(L, R)
    rows = None if all_rows else sample_rows(p.t, every=13)
    for step in steps:
        X = synth.activations(p, step)
        dY = synth.out_grad(p, step) if p.backward else None
        res = check_step(L, R, X, dY, p.gamma, rows=rows, backward=p.backward,
                         tag="cfg%d %s step %d" % (p.config, p.name, step))
        _say("cfg%d %-8s step %d ok  fwd_err %.2e bwd_err %.2e  (%.1fs)" % (
            p.config, p.name, step, res["fwd_err"], res.get("bwd_err", 0.0), time.time() - t0))


@pytest.mark.parametrize("name", ["qkv", "o_proj"])
def test_config2_phi3_attention(name):
    _run_projection(synth.projection(2, name), range(3))


@pytest.mark.parametrize("name", ["gate_up", "down"])
def test_config3_phi3_mlp(name):
    """Ten consecutive steps end to end, every element compared (the 50-step chain of the scale update alone is in
    test_gpu_behaviour.py)."""
    _run_projection(synth.projection(3, name), range(10))


@pytest.mark.parametrize("name", ["q", "o", "gate", "down"])
def test_config4_llama7b_layer(name):
    _run_projection(synth.projection(4, name), range(2))


@pytest.mark.parametrize("name", ["q", "gate", "down"])
def test_config5_long_sequence(name):
    _run_projection(synth.projection(5, name), range(1), prepare_check=(name == "q"), all_rows=False)


@pytest.mark.parametrize("name", ["o_proj", "down"])
def test_paper_outlier_budget_workload(name):
    """4 % / 10 % of the input channels as outliers: the wide second product runs as its own launch."""
    _run_projection(synth.projection(6, name), range(2))
