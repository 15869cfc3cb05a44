"""bf16-output variants of the forward and dX products: the fp32 result rounded to nearest even."""
import numpy as np
import pytest

from paper_2505_14742_amd import synth

pytestmark = pytest.mark.gpu


def _check(got_bits, ref_f32, what):
    """got (uint16 bf16 bits) against the oracle's value: within half a bf16 step of it (2^-9 relative) plus the
    1e-3 rms allowance of the fp32 comparison, and the correctly rounded bf16 value almost everywhere."""
    got = synth.bf16_to_f32(got_bits.astype(np.uint16).ravel()).reshape(got_bits.shape).astype(np.float64)
    ref = np.asarray(ref_f32, np.float64)
    rms = np.sqrt(np.mean(ref * ref))
    lim = (2.0 ** -8) * np.abs(ref) + 1e-3 * rms
    worst = np.max(np.abs(got - ref) - lim)
    assert worst <= 0, "%s: tolerance exceeded by %g" % (what, worst)
    want = synth.f32_to_bf16(np.ascontiguousarray(ref_f32, np.float32).ravel()).reshape(ref_f32.shape)
    frac = float(np.mean((got_bits.astype(np.int32) & 0xFFFF) == want.astype(np.int32)))
    assert frac > 0.995, "%s: only %.4f of the values are the correctly rounded ones" % (what, frac)
    return frac


@pytest.mark.parametrize("case", ["edge1", "edge8", "cfg2_o", "cfg2_qkv"])
def test_bf16_outputs(case):
    import torch
    from paper_2505_14742_amd import binding as q
    from tests.gpu_harness import DEV, Layer, bf16_dev, host
    if case.startswith("edge"):
        idx = int(case[4:])
        ec = synth.EDGE_CASES[idx]
        X, dY, W, O, A, B = synth.edge_case_inputs(ec, idx)
        scale, t = 0.5, ec.t
    else:
        p = synth.projection(2, "o_proj" if case.endswith("_o") else "qkv")
        W, O = synth.weight(p), synth.outlier_indices(p)
        A, B = synth.lora(p)
        X, dY, scale, t = synth.activations(p, 0), synth.out_grad(p, 0), p.lora_scale, p.t
    print("bf16 out", case, flush=True)
    L = Layer(W, O, A, B, scale, t)
    Xd, Gd = bf16_dev(X), bf16_dev(dY)
    L.scale_update(Xd, 0.2); L.quant_act(Xd); L.linear_fwd(Xd); L.linear_bwd_dx(Gd)
    Y16 = torch.full((t, L.c_out), 0x7FC0, dtype=torch.int16, device=DEV)
    dX16 = torch.full((t, L.c_in), 0x7FC0, dtype=torch.int16, device=DEV)

    def fwd16():
        q.linear_fwd(L.Xq, L.delta_x, L.xq_O if L.n else None, L.Wq_packed, L.delta_w, L.c_in, L.c_out,
                     L.what_int if L.n else None, L.delta_what if L.n else None, L.n, Xd if L.r else None, L.A, L.B,
                     L.r, scale, Y16, L.ws, bf16_out=True)

    def bwd16():
        q.linear_bwd_dx(Gd, L.Wq_packed, L.delta_w, L.c_in, L.c_out, L.A, L.B, L.r, scale, dX16, L.ws, bf16_out=True)

    if L.c_in % 64 or L.c_out % 64:
        # the bf16-output launches exist for contractions that are multiples of 64: anything else is refused with
        # QUAFF_ERR_SHAPE before anything is enqueued, and the output stays untouched
        if L.c_in % 64:
            with pytest.raises(q.QuaffError, match="SHAPE"):
                fwd16()
        if L.c_out % 64:
            with pytest.raises(q.QuaffError, match="SHAPE"):
                bwd16()
        torch.cuda.synchronize()
        if L.c_in % 64:
            assert int((Y16 != 0x7FC0).sum()) == 0
        if L.c_out % 64:
            assert int((dX16 != 0x7FC0).sum()) == 0
        return
    fwd16()
    bwd16()
    torch.cuda.synchronize()
    # against the library's own fp32 result (itself checked against the oracle elsewhere): bit-exact rounding
    want_y = synth.f32_to_bf16(host(L.Y).ravel()).reshape(t, L.c_out).astype(np.int32)
    want_dx = synth.f32_to_bf16(host(L.dX).ravel()).reshape(t, L.c_in).astype(np.int32)
    assert np.array_equal(host(Y16).astype(np.int32) & 0xFFFF, want_y), "Y is not RNE(fp32 Y)"
    assert np.array_equal(host(dX16).astype(np.int32) & 0xFFFF, want_dx), "dX is not RNE(fp32 dX)"
    # and against the oracle directly, both outputs, every row
    from oracle import api as orc
    Wq, dw = orc.weight_quantize(W)
    O32 = O.astype(np.int32)
    W_O, wmax = orc.outlier_rows(W, O32)
    s, cs, what, dwh, _ = orc.scale_update(X, O32, W_O, wmax, 0.2, np.ones(O32.size, np.float32),
                                           np.ones(W.shape[0], np.float32))
    Xq, dx, xo = orc.quant_act(X, cs, O32)
    has_lora = L.r > 0
    Y_o = orc.linear_fwd(Xq, dx, xo, Wq, dw, what, dwh, X, A if has_lora else None, B if has_lora else None, scale)[0]
    _check(host(Y16), Y_o, case + " Y")
    dX_o = orc.linear_bwd_dx(dY, Wq, dw, A if has_lora else None, B if has_lora else None, scale)[0]
    _check(host(dX16), dX_o, case + " dX")
