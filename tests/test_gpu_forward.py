"""The compensated layer at inference (integer MFMA kernel) against oracle.compensated_forward.

Both sides read the same inputs: W codes and scales, L_A, L_B (fp32) and the smoothing diagonal from the
oracle's calibration of the layer.  The activation codes are bit-exact on both sides (checked), the
integer sums are exact, so what differs is fp32 rounding of the scales (about 1e-7) and the rank-r
branch: about 2^-16 relative per product in the split mode, about 2^-9 per factor in the plain bf16 mode
(three rounded factors, random signs over r terms).  Bars, relative Frobenius over the output:
1e-6 without compensation, 2e-5 split, 4e-3 plain.
"""
import numpy as np
import pytest
import torch

import aser_synth as synth
import paper_2411_07762_amd as aser
from oracle import aser_oracle as orc

from gpu_util import DEV, new_ctx, to_dev_x
from test_gpu_parity import say

pytestmark = pytest.mark.gpu


def forward_case(label, spec, sample, packed, act_bits=8, pad=0):
    W = synth.make_weight(spec)
    x_np = synth.make_activations(spec)
    X = synth.activations_as_f32(spec, x_np)
    ref = orc.calibrate_layer(W, X, spec.bits, spec.f, spec.r)
    md = ref.smooth.mdiag
    L_A32, L_B32 = ref.rec.L_A.astype(np.float32), ref.rec.L_B.astype(np.float32)
    ctx = new_ctx()
    ctx.ensure_workspace(aser.aser_forward_workspace_bytes(sample, spec.n, spec.m, spec.r))
    Xd = to_dev_x(spec, x_np[:sample])
    mdd = torch.from_numpy(md).to(DEV)
    xq = torch.empty((sample, spec.n), dtype=torch.int8, device=DEV)
    xs = torch.empty(sample, dtype=torch.float32, device=DEV)
    ctx.check(aser.aser_quantize_act_rtn(ctx, Xd, mdd, act_bits, xq, xs))
    q_ref, s_ref = orc.quantize_act_rtn(X[:sample], md, act_bits)
    torch.cuda.synchronize()
    assert np.array_equal(xq.cpu().numpy(), q_ref) and np.array_equal(xs.cpu().numpy(), s_ref)
    if packed:
        wq = torch.from_numpy(orc.pack_int4(ref.quant.codes)).to(DEV)
        layout = aser.ASER_CODES_INT4_PACKED
    else:
        wq = torch.from_numpy(ref.quant.codes).to(DEV)
        layout = aser.ASER_CODES_INT8
    wsd = torch.from_numpy(ref.quant.scales).to(DEV)
    LAd, LBd = torch.from_numpy(L_A32).to(DEV), torch.from_numpy(L_B32).to(DEV)
    for comp, split, bar in ((False, False, 1e-6), (True, True, 2e-5), (True, False, 4e-3)):
        want = orc.compensated_forward(X[:sample], md, ref.quant.codes, ref.quant.scales, L_A32 if comp else None,
                                       L_B32 if comp else None, act_bits)
        Ybuf = torch.full((sample, spec.m + pad), float("nan"), dtype=torch.float32, device=DEV)
        Y = Ybuf[:, :spec.m]
        ctx.check(aser.aser_compensated_forward(ctx, xq, xs, wq, layout, wsd, LAd if comp else None, LBd if comp else None,
                                                spec.r if comp else 0, split, Y))
        torch.cuda.synchronize()
        got = Y.cpu().numpy().astype(np.float64)
        rel = np.linalg.norm(got - want) / np.linalg.norm(want)
        say("%s: compensated=%s split=%s  ||Y - Y_oracle|| / ||Y_oracle|| = %.2e (bar %.0e)" % (label, comp, split, rel, bar))
        assert np.isfinite(got).all() and rel <= bar
        if split:
            got_split = got
        if pad:
            assert torch.isnan(Ybuf[:, spec.m:]).all()
    # the output error of the kernel's result is the layer-output error of Sec. 5.3's figure
    e_ref, _ = orc.layer_output_error(W, X[:sample], md, ref.quant.codes, ref.quant.scales, L_A32, L_B32, act_bits)
    Yexact = X[:sample].astype(np.float64) @ W.astype(np.float64).T
    e_kernel = np.linalg.norm(Yexact - got_split)
    e_plain = np.linalg.norm(Yexact - got)                     # got: the plain bf16 run, the last of the loop
    say("%s: output error of the kernel's result %.6g (factors rounded to bf16: %.6g), oracle %.6g" %
        (label, e_kernel, e_plain, e_ref))
    assert abs(e_kernel - e_ref) <= 1e-3 * e_ref + 2e-5 * np.linalg.norm(Yexact)


CASES = [
    ("c0_int8", synth.CONFIGS["c0"], 300, False, 8, 0),
    ("c0_int4", synth.CONFIGS["c0"], 1024, True, 8, 4),
    ("ragged_tokens_outputs", synth.mini("fw1", 333, 320, 1500, r=24, f=6), 777, True, 8, 0),
    ("r_not_multiple_of_32_a6", synth.mini("fw2", 600, 96, 700, r=40, f=4), 129, True, 6, 0),
    ("w8_tall", synth.mini("fw3", 700, 160, 900, x_dtype="f32", r=16, f=5, bits=8), 513, False, 8, 0),
    ("c1_shape_small", synth.CONFIGS["c1"].with_(m=768, n=1024, tokens=4096, r=64, f=16), 2048, True, 8, 0),
    # the 256 x 256 tiles with LDS-direct loads: a last step of 32 channels with packed int4 and with int8 codes, fewer
    # steps than the ring has stages, ragged tokens and outputs, a padded output
    ("w4_half_step_at_the_end", synth.mini("fw4", 300, 352, 1400, r=24, f=5), 600, True, 8, 4),
    ("w4_one_and_a_half_steps", synth.mini("fw5", 260, 96, 900, r=8, f=2), 700, True, 8, 0),
    ("w8_half_a_step", synth.mini("fw6", 257, 32, 600, x_dtype="f32", r=8, f=1, bits=8), 257, False, 8, 0),
    ("w8_two_steps_split_tiles", synth.mini("fw7", 513, 128, 1200, r=16, f=3, bits=8), 1025, False, 8, 0),
]


@pytest.mark.parametrize("name,spec,sample,packed,act_bits,pad", CASES, ids=[c[0] for c in CASES])
def test_compensated_forward(name, spec, sample, packed, act_bits, pad):
    say("forward case %s m=%d n=%d tokens=%d r=%d" % (name, spec.m, spec.n, sample, spec.r))
    forward_case(name, spec, sample, packed, act_bits, pad)


def test_mfma_rate_probe_runs():
    """The measurement aid: a loop of nothing but MFMA instructions must land between a tenth of the nominal peak and
    the nominal peak (2.5 PFLOP/s bf16, 5.0 POP/s int8); with the operand traffic of a tile around the instructions
    it cannot be faster than without (5 % for the clock's wander between launches)."""
    ctx = new_ctx()
    ctx.ensure_workspace((33 << 20) + 4 * 256 * 1024 + 256)
    for kind, peak in ((0, 2500.0), (1, 5000.0)):
        alone = {}
        for wgs in (1, 4):
            st, rate = aser.aser_mfma_rate_probe(ctx, kind, wgs, 2000)
            ctx.check(st)
            say("MFMA-only loop kind %d, %d workgroup(s) per compute unit: %.0f T op/s" % (kind, wgs, rate))
            assert 0.1 * peak < rate <= 1.001 * peak
            alone[wgs] = rate
        st, rate = aser.aser_mfma_rate_probe(ctx, kind + 2, 1, 2000)
        ctx.check(st)
        say("MFMA loop with operand traffic, kind %d: %.0f T op/s" % (kind + 2, rate))
        assert 0.1 * peak < rate <= 1.05 * alone[1]
