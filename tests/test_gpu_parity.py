"""Parity of the HIP path against the CPU oracle, stage by stage and end to end, through the C ABI.

Bars: int4/int8 codes, scales and outlier indices bit-exact; the whitened layer-output error
||(T - L_A L_B) S||_F, recomputed in fp64 from the GPU's L_A and L_B, within 1e-4 relative of
the oracle's; the product L_A L_B within 1e-3 relative Frobenius when the oracle's
sigma_r / sigma_{r+1} exceeds 1.05.  Tolerances of the fp32 intermediates are derived in the
design notes (Gram: fp32 accumulation over N tokens; fp32 inputs: bf16 hi/lo split, 2^-16 per product).
"""
import os
import sys
import time

import numpy as np
import pytest
import torch

import aser_synth as synth
import paper_2411_07762_amd as aser
from oracle import aser_oracle as orc

from gpu_util import DEV, lower, new_ctx, padded, run_gram, to_dev_x, unpack_int4

pytestmark = pytest.mark.gpu


_PROGRESS = os.path.join(os.path.dirname(os.path.dirname(os.path.abspath(__file__))), "gpurun_out", "test_progress.log")


def say(msg):
    """Names the case before each GPU step: on stdout (shown on failure or with -s) and, because pytest
    holds stdout back, appended to a progress file that a watcher of a long run can see grow."""
    print(msg, flush=True)
    try:
        os.makedirs(os.path.dirname(_PROGRESS), exist_ok=True)
        with open(_PROGRESS, "a") as fh:
            fh.write("%s %s\n" % (time.strftime("%H:%M:%S"), msg))
    except OSError:
        pass


def oracle_layer(spec, W, x_np, r=None, f=None):
    X = synth.activations_as_f32(spec, x_np)
    return orc.calibrate_layer(W, X, spec.bits, spec.f if f is None else f, spec.r if r is None else r)


GRAM_CASES = [
    ("c0", synth.CONFIGS["c0"], 1, 0),
    ("ragged_bf16", synth.mini("g1", 8, 200, 777), 1, 0),
    ("ragged_bf16_chunks_pad", synth.mini("g2", 8, 520, 2000), 3, 8),
    ("odd_n_bf16", synth.mini("g3", 8, 77, 300), 2, 3),
    ("f32_ragged", synth.mini("g4", 8, 300, 1111, x_dtype="f32"), 2, 4),
    ("multi_tile_bf16", synth.mini("g5", 8, 1300, 4500), 1, 0),
    ("persistent_schedule_bf16", synth.mini("g7", 8, 2100, 8300), 1, 0),
    ("persistent_schedule_f32", synth.mini("g8", 8, 2100, 4200, x_dtype="f32"), 1, 4),
    # the LDS-direct kernel (aligned bf16): channel count not a multiple of the tile, token counts not a multiple of the step
    ("lds_direct_ragged_bf16", synth.mini("g9", 8, 2104, 8227), 1, 0),
    ("lds_direct_ragged_chunks_pad_bf16", synth.mini("g10", 8, 2312, 17001), 2, 8),
]


@pytest.mark.parametrize("name,spec,chunks,pad", GRAM_CASES, ids=[c[0] for c in GRAM_CASES])
def test_gram_accumulate(name, spec, chunks, pad):
    say("gram case %s n=%d N=%d dtype=%s chunks=%d pad=%d" % (name, spec.n, spec.tokens, spec.x_dtype, chunks, pad))
    x_np = synth.make_activations(spec)
    G_ref, abs_ref, cnt = orc.gram(synth.activations_as_f32(spec, x_np))
    ctx = new_ctx()
    G, abs_sum, count = run_gram(ctx, spec, x_np, chunks, pad)
    G = G.cpu().numpy().astype(np.float64)
    d = np.sqrt(np.diag(G_ref))
    tol = (2e-5 if spec.x_dtype == "bf16" else 4e-5) * np.outer(d, d)
    bad = np.abs(lower(G) - lower(G_ref)) > lower(tol)
    assert not bad.any(), "max rel err %g" % (np.abs(lower(G) - lower(G_ref)) / np.outer(d, d)).max()
    assert int(count.item()) == cnt
    assert np.allclose(abs_sum.cpu().numpy(), abs_ref, rtol=1e-13, atol=0)


def test_gram_empty_chunk_and_stats_optional():
    spec = synth.mini("g6", 8, 64, 128)
    x = to_dev_x(spec, synth.make_activations(spec))
    ctx = new_ctx()
    G = torch.zeros((64, 64), dtype=torch.float32, device=DEV)
    ctx.check(aser.aser_gram_accumulate(ctx, x, G, rows=0, n=64, ldx=64))
    torch.cuda.synchronize()
    assert float(G.abs().max()) == 0.0
    count = torch.zeros(1, dtype=torch.int64, device=DEV)
    ctx.check(aser.aser_gram_accumulate(ctx, x, G, None, count))
    torch.cuda.synchronize()
    assert int(count.item()) == 128 and float(G.abs().max()) > 0


SMOOTH_CASES = [
    ("c0", synth.CONFIGS["c0"]),
    ("ragged", synth.mini("s1", 50, 333, 500, f=7)),
    ("wide", synth.mini("s2", 96, 2500, 640, f=32, n_outliers=16)),
    ("no_smoothing", synth.mini("s3", 40, 128, 256, f=0)),
    ("all_channels", synth.mini("s4", 16, 24, 64, f=24)),
]


@pytest.mark.parametrize("name,spec", SMOOTH_CASES, ids=[c[0] for c in SMOOTH_CASES])
def test_smooth_outliers(name, spec):
    say("smooth case %s m=%d n=%d f=%d" % (name, spec.m, spec.n, spec.f))
    W = synth.make_weight(spec)
    x_np = synth.make_activations(spec)
    G_ref, abs_ref, cnt = orc.gram(synth.activations_as_f32(spec, x_np))
    ref = orc.smooth_outliers(W, abs_ref, cnt, spec.f)
    ctx = new_ctx()
    ctx.ensure_workspace(aser.aser_workspace_bytes(spec.m, spec.n, 0))
    Wd = padded(torch.from_numpy(W).to(DEV), 4)
    abs_sum = torch.from_numpy(abs_ref).to(DEV)
    count = torch.tensor([cnt], dtype=torch.int64, device=DEV)
    idx = torch.full((max(spec.f, 1),), -1, dtype=torch.int32, device=DEV)
    mdiag = torch.empty(spec.n, dtype=torch.float32, device=DEV)
    W_o = torch.empty((spec.m, max(spec.f, 1)), dtype=torch.float32, device=DEV)
    score = torch.empty(spec.n, dtype=torch.float64, device=DEV)
    ctx.check(aser.aser_smooth_outliers(ctx, Wd, abs_sum, count, spec.f, idx, mdiag, W_o, score))
    torch.cuda.synchronize()
    assert np.allclose(score.cpu().numpy(), ref.score, rtol=1e-12, atol=0)
    if spec.f:
        assert ref.margin > 1e-9
        assert idx.cpu().numpy()[:spec.f].tolist() == ref.idx.tolist()
        assert np.allclose(W_o.cpu().numpy()[:, :spec.f], ref.W_o, rtol=1e-6, atol=0)
    md = mdiag.cpu().numpy()
    ulp = np.abs(md.view(np.int32).astype(np.int64) - ref.mdiag.view(np.int32).astype(np.int64))
    assert ulp.max() <= 1, "mdiag differs by %d ulp" % ulp.max()


def test_smooth_tie_break_lower_index():
    # identical channels 5 and 9 (same |x| sum, same |w| sum): the lower index must win the last slot
    n, m = 16, 8
    W = np.ones((m, n), dtype=np.float32)
    abs_sum = np.linspace(1.0, 2.0, n)
    abs_sum[5] = abs_sum[9] = 7.0
    abs_sum[2] = 9.0
    ref = orc.smooth_outliers(W, abs_sum, 10, 2)
    assert ref.idx.tolist() == [2, 5]
    ctx = new_ctx()
    ctx.ensure_workspace(aser.aser_workspace_bytes(m, n, 0))
    idx = torch.zeros(2, dtype=torch.int32, device=DEV)
    mdiag = torch.empty(n, dtype=torch.float32, device=DEV)
    ctx.check(aser.aser_smooth_outliers(ctx, torch.from_numpy(W).to(DEV), torch.from_numpy(abs_sum).to(DEV),
                                        torch.tensor([10], dtype=torch.int64, device=DEV), 2, idx, mdiag))
    torch.cuda.synchronize()
    assert idx.cpu().numpy().tolist() == [2, 5]
    assert np.array_equal(mdiag.cpu().numpy(), ref.mdiag)


def test_smooth_without_usable_scores_is_reported_not_faulted():
    """No tokens accumulated (count = 0), and a NaN in the statistics: the selection finds fewer than f
    channels with a finite score.  idx gets -1 there, every kernel that consumes idx skips such entries,
    and the next synchronising call returns ASER_ERR_INVALID_ARG instead of numbers."""
    spec = synth.mini("sg", 24, 96, 64, f=5)
    W = torch.from_numpy(synth.make_weight(spec)).to(DEV)
    n, m, f = spec.n, spec.m, spec.f
    for case in ("count_zero", "nan_statistics"):
        say("smooth guard case %s" % case)
        ctx = new_ctx()
        ctx.ensure_workspace(aser.aser_workspace_bytes(m, n, 4))
        abs_sum = torch.zeros(n, dtype=torch.float64, device=DEV)
        count = torch.zeros(1, dtype=torch.int64, device=DEV)
        if case == "nan_statistics":
            abs_sum += float("nan")
            abs_sum[:3] = torch.tensor([5.0, 9.0, 7.0], dtype=torch.float64)   # only three usable channels for f = 5
            count += 10
        idx = torch.full((f,), 77, dtype=torch.int32, device=DEV)
        mdiag = torch.empty(n, dtype=torch.float32, device=DEV)
        W_o = torch.empty((m, f), dtype=torch.float32, device=DEV)
        ctx.check(aser.aser_smooth_outliers(ctx, W, abs_sum, count, f, idx, mdiag, W_o))
        codes = torch.empty((m, n), dtype=torch.int8, device=DEV)
        scales = torch.empty(m, dtype=torch.float32, device=DEV)
        T = torch.empty((m, n), dtype=torch.float32, device=DEV)
        ctx.check(aser.aser_quantize_rtn(ctx, W, idx, mdiag, f, 4, aser.ASER_CODES_INT8, codes, scales, T))
        torch.cuda.synchronize()
        got = idx.cpu().numpy().tolist()
        if case == "count_zero":
            assert got == [-1] * f
        else:
            assert sorted(got[:3]) == [0, 1, 2] and got[3:] == [-1, -1]
            assert np.isfinite(mdiag.cpu().numpy()).all()
        G = torch.eye(n, dtype=torch.float32, device=DEV)
        S = torch.empty_like(G)
        st, info = aser.aser_whiten(ctx, G, None, 0.0, S)          # the next synchronising call carries the report
        assert st == aser.ASER_ERR_INVALID_ARG and "smooth_outliers" in ctx.last_error()
        st, info = aser.aser_whiten(ctx, G, None, 0.0, S)          # reported once
        assert st == aser.ASER_OK and info == 0


RTN_CASES = [
    ("c0_int4_packed", synth.CONFIGS["c0"], 4, True),
    ("c0_int8", synth.CONFIGS["c0"], 8, False),
    ("ragged_int4", synth.mini("q1", 37, 331, 400, f=5), 4, False),
    ("even_packed", synth.mini("q2", 65, 1030, 300, f=9), 4, True),
    ("wide_int8", synth.mini("q3", 20, 9000, 64, f=32, n_outliers=8), 8, False),
    ("very_wide_int4", synth.mini("q4", 6, 28672, 32, f=64, n_outliers=8), 4, True),
    ("no_outliers", synth.mini("q5", 33, 256, 128, f=0), 4, True),
    ("mid_width_int4", synth.mini("q6", 12, 6000, 64, f=16, n_outliers=8), 4, True),
    ("width_11008_int4", synth.mini("q7", 10, 11008, 48, f=32, n_outliers=8), 4, True),      # 768 threads per row
    ("width_13000_int8", synth.mini("q8", 7, 13000, 40, f=16, n_outliers=8), 8, False),      # 1024 threads, two groups each
    ("width_20000_int4", synth.mini("q9", 5, 20000, 40, f=24, n_outliers=8), 4, True),       # 1024 threads, three groups each
    ("width_30000_int8", synth.mini("q10", 4, 30000, 40, f=24, n_outliers=8), 8, False),     # 1024 threads, four groups each
]


@pytest.mark.parametrize("name,spec,bits,packed", RTN_CASES, ids=[c[0] for c in RTN_CASES])
def test_quantize_rtn(name, spec, bits, packed):
    say("rtn case %s m=%d n=%d bits=%d packed=%s f=%d" % (name, spec.m, spec.n, bits, packed, spec.f))
    W = synth.make_weight(spec)
    if spec.m > 3:
        W[3, :] = 0.0                                            # an all-zero output row: scale 1, codes 0
    x_np = synth.make_activations(spec)
    _, abs_ref, cnt = orc.gram(synth.activations_as_f32(spec, x_np))
    sm = orc.smooth_outliers(W, abs_ref, cnt, spec.f)
    ref = orc.quantize_rtn(W, sm.idx, sm.mdiag, bits)
    ctx = new_ctx()
    Wd = padded(torch.from_numpy(W).to(DEV), 0 if packed else 4)
    idx = torch.from_numpy(sm.idx if spec.f else np.zeros(1, np.int32)).to(DEV)
    mdiag = torch.from_numpy(sm.mdiag).to(DEV)
    codes = torch.zeros((spec.m, spec.n // 2 if packed else spec.n), dtype=torch.uint8 if packed else torch.int8, device=DEV)
    scales = torch.empty(spec.m, dtype=torch.float32, device=DEV)
    T = torch.empty((spec.m, spec.n), dtype=torch.float32, device=DEV)
    layout = aser.ASER_CODES_INT4_PACKED if packed else aser.ASER_CODES_INT8
    ctx.check(aser.aser_quantize_rtn(ctx, Wd, idx, mdiag, spec.f, bits, layout, codes, scales, T))
    torch.cuda.synchronize()
    got = codes.cpu().numpy()
    if packed:
        assert np.array_equal(got, orc.pack_int4(ref.codes))
        got = unpack_int4(got)
    assert np.array_equal(got, ref.codes)
    assert np.array_equal(scales.cpu().numpy(), ref.scales)
    Tg = T.cpu().numpy().astype(np.float64)
    assert np.all(np.abs(Tg - ref.T) <= 2.0 ** -23 * np.abs(ref.T) + 1e-30)
    if spec.m > 3:
        assert ref.scales[3] == 1.0 and not got[3].any()


BASE_QUANTIZER_CASES = [
    ("ragged", synth.mini("bq1", 37, 333, 64, f=6, n_outliers=4), 0),
    ("padded_rows", synth.mini("bq2", 130, 1032, 64, f=16, n_outliers=8), 4),
    ("unaligned_rows", synth.mini("bq3", 21, 2050, 48, f=9, n_outliers=4), 3),
    ("several_column_chunks", synth.mini("bq4", 19, 5000, 40, f=40, n_outliers=8), 0),
    ("no_outliers", synth.mini("bq5", 16, 256, 40, f=0, n_outliers=0), 0),
]


def groupwise_quantizer(W_s, bits=4, group=64):
    """A stand-in for the caller's own weight quantizer (not part of the library or of the oracle): asymmetric
    round-to-nearest with a scale and a zero point per group of `group` input channels, in fp32.  Zero stays zero."""
    W_s = np.asarray(W_s, dtype=np.float32)
    out = np.empty_like(W_s)
    levels = np.float32(2 ** bits - 1)
    for g0 in range(0, W_s.shape[1], group):
        blk = W_s[:, g0:g0 + group]
        lo = np.minimum(blk.min(axis=1), np.float32(0))
        hi = np.maximum(blk.max(axis=1), np.float32(0))
        scale = ((hi - lo) / levels).astype(np.float32)
        scale[scale == 0] = np.float32(1)
        zero = np.rint(-lo / scale)
        q = np.clip(np.rint(blk / scale[:, None]) + zero[:, None], 0, levels)
        out[:, g0:g0 + group] = ((q - zero[:, None]) * scale[:, None]).astype(np.float32)
    return out


@pytest.mark.parametrize("name,spec,pad", BASE_QUANTIZER_CASES, ids=[c[0] for c in BASE_QUANTIZER_CASES])
def test_passes_around_another_weight_quantizer(name, spec, pad):
    """aser_smoothed_weight bit-exact, aser_quant_target within the one rounding of its fused multiply-add."""
    say("base quantizer case %s m=%d n=%d f=%d pad=%d" % (name, spec.m, spec.n, spec.f, pad))
    W = synth.make_weight(spec)
    x_np = synth.make_activations(spec)
    _, abs_ref, cnt = orc.gram(synth.activations_as_f32(spec, x_np))
    sm = orc.smooth_outliers(W, abs_ref, cnt, spec.f)
    ctx = new_ctx()
    Wd = padded(torch.from_numpy(W).to(DEV), pad)
    idx = torch.from_numpy(sm.idx).to(DEV) if spec.f else None
    mdiag = torch.from_numpy(sm.mdiag).to(DEV)
    Ws = padded(torch.full((spec.m, spec.n), 7.0, dtype=torch.float32, device=DEV), pad)
    ctx.check(aser.aser_smoothed_weight(ctx, Wd, idx, spec.f, Ws))
    torch.cuda.synchronize()
    ws_np = Ws.cpu().numpy()
    assert np.array_equal(ws_np, orc.smoothed_weight(W, sm.idx))
    Wq_np = groupwise_quantizer(ws_np)
    ref_T = orc.target_from_dequantized(W, sm.mdiag, Wq_np)
    Wq = padded(torch.from_numpy(Wq_np).to(DEV), pad)
    T = padded(torch.empty((spec.m, spec.n), dtype=torch.float32, device=DEV), pad)
    ctx.check(aser.aser_quant_target(ctx, Wd, mdiag, Wq, T))
    torch.cuda.synchronize()
    Tg = T.cpu().numpy().astype(np.float64)
    assert np.all(np.abs(Tg - ref_T) <= 2.0 ** -23 * np.abs(ref_T) + 1e-37)
    if spec.f:
        rest = np.setdiff1d(np.arange(spec.n), sm.idx)
        assert np.array_equal(Tg[:, sm.idx], sm.W_o.astype(np.float32))   # exact products of two fp32 values, rounded once
        assert np.abs(Tg[:, rest]).max() < np.abs(W).max()                # only rounding error off the outlier columns
    # in place (T is W_q's own memory) and without a smoothing diagonal
    ctx.check(aser.aser_quant_target(ctx, Wd, mdiag, Wq, Wq))
    ctx.check(aser.aser_quant_target(ctx, Wd, None, Ws, T))
    torch.cuda.synchronize()
    assert np.array_equal(Wq.cpu().numpy().astype(np.float64), Tg)
    assert np.array_equal(T.cpu().numpy(), (W.astype(np.float64) - ws_np).astype(np.float32))


def test_layer_with_another_weight_quantizer():
    """Sec. 4.1's closing remark end to end: a group-wise asymmetric quantizer takes RTN's place between
    aser_smoothed_weight and aser_quant_target; the factors meet the same bars against the oracle run on the same W_q."""
    from types import SimpleNamespace
    spec = synth.CONFIGS["c1"].with_(m=640, n=1024, tokens=4096, r=32, f=16, n_outliers=8)
    say("layer with a group-wise quantizer m=%d n=%d r=%d f=%d" % (spec.m, spec.n, spec.r, spec.f))
    W = synth.make_weight(spec)
    x_np = synth.make_activations(spec)
    ref_rtn = oracle_layer(spec, W, x_np)
    ctx = new_ctx()
    buf = aser.LayerBuffers(spec.m, spec.n, spec.r, spec.f, spec.bits, False)
    ctx.ensure_workspace(aser.aser_workspace_bytes(spec.m, spec.n, spec.r))
    Wd = torch.from_numpy(W).to(DEV)
    ctx.check(aser.aser_gram_accumulate(ctx, to_dev_x(spec, x_np), buf.G, buf.abs_sum, buf.count))
    ctx.check(aser.aser_smooth_outliers(ctx, Wd, buf.abs_sum, buf.count, spec.f, buf.idx, buf.mdiag))
    Ws = torch.empty_like(Wd)
    ctx.check(aser.aser_smoothed_weight(ctx, Wd, buf.idx, spec.f, Ws))
    torch.cuda.synchronize()
    assert buf.idx.cpu().numpy()[:spec.f].tolist() == ref_rtn.smooth.idx.tolist()
    Wq_np = groupwise_quantizer(Ws.cpu().numpy())                     # the caller's quantizer
    Wq = torch.from_numpy(Wq_np).to(DEV)
    ctx.check(aser.aser_quant_target(ctx, Wd, buf.mdiag, Wq, buf.T))
    st, info = aser.aser_whiten(ctx, buf.G, buf.mdiag, 0.0, buf.S)
    ctx.check(st)
    assert info == 0
    st, err, _ = aser.aser_error_reconstruct(ctx, buf.T, buf.S, spec.r, buf.L_A, buf.L_B, buf.sigma, idx=buf.idx, f=spec.f)
    ctx.check(st)
    T_ref = orc.target_from_dequantized(W, ref_rtn.smooth.mdiag, Wq_np)
    ref = SimpleNamespace(quant=SimpleNamespace(T=T_ref), S=ref_rtn.S, rec=orc.error_reconstruct(T_ref, ref_rtn.S, spec.r))
    rec = check_reconstruction(spec, ref, buf.L_A.cpu().numpy(), buf.L_B.cpu().numpy(), buf.sigma.cpu().numpy(), err,
                               "group-wise quantizer")
    say("whitened error: group-wise %.5g (uncompensated %.5g), per-channel RTN %.5g (uncompensated %.5g)" %
        (rec.err, rec.err0, ref_rtn.rec.err, ref_rtn.rec.err0))
    assert rec.err < ref_rtn.rec.err                                  # finer scales leave less to compensate


ACT_CASES = [("bf16", synth.mini("a1", 8, 333, 70, f=5)), ("f32", synth.mini("a2", 8, 520, 33, x_dtype="f32", f=3)),
             ("wide_bf16", synth.mini("a3", 8, 4096, 16, f=8)), ("wave_ragged_bf16", synth.mini("a4", 8, 1000, 37, f=6)),
             ("wave_f32", synth.mini("a5", 8, 2048, 9, x_dtype="f32", f=4)), ("very_wide_bf16", synth.mini("a6", 8, 14336, 5, f=8)),
             ("width_11008_bf16", synth.mini("a7", 8, 11008, 7, f=8)), ("width_9000_f32", synth.mini("a8", 8, 9000, 6, x_dtype="f32", f=5)),
             ("width_6000_bf16", synth.mini("a9", 8, 6000, 9, f=6)), ("width_7000_f32", synth.mini("a12", 8, 7000, 5, x_dtype="f32", f=6)), ("width_20000_bf16", synth.mini("a10", 8, 20000, 5, f=8)),
             ("width_32768_f32", synth.mini("a11", 8, 32768, 3, x_dtype="f32", f=4))]


@pytest.mark.parametrize("name,spec", ACT_CASES, ids=[c[0] for c in ACT_CASES])
def test_quantize_act_rtn(name, spec):
    say("act rtn case %s n=%d tokens=%d" % (name, spec.n, spec.tokens))
    W = synth.make_weight(spec)
    x_np = synth.make_activations(spec)
    X = synth.activations_as_f32(spec, x_np)
    X[1, :] = 0.0
    if spec.x_dtype == "bf16":
        x_np = synth.f32_to_bf16_bits(X)
    else:
        x_np = X
    _, abs_ref, cnt = orc.gram(X)
    sm = orc.smooth_outliers(W, abs_ref, cnt, spec.f)
    ref_codes, ref_scales = orc.quantize_act_rtn(X, sm.mdiag, 8)
    ctx = new_ctx()
    xd = to_dev_x(spec, x_np)
    codes = torch.zeros((spec.tokens, spec.n), dtype=torch.int8, device=DEV)
    scales = torch.empty(spec.tokens, dtype=torch.float32, device=DEV)
    ctx.check(aser.aser_quantize_act_rtn(ctx, xd, torch.from_numpy(sm.mdiag).to(DEV), 8, codes, scales))
    torch.cuda.synchronize()
    assert np.array_equal(codes.cpu().numpy(), ref_codes)
    assert np.array_equal(scales.cpu().numpy(), ref_scales)
    assert ref_scales[1] == 1.0


# The wavefront-per-token kernel walks 2 to 4 tokens per wavefront once there are 8192 tokens or more (the
# shape of every activation stream of the bench): token counts that leave the last wavefront with fewer
# tokens than the others, a channel count below 4096 (lanes without channels), both input types.
ACT_MANY_TOKENS = [("bf16_8195x4096", 8195, 4096, "bf16"), ("bf16_16387x4096", 16387, 4096, "bf16"),
                   ("bf16_12290x2064", 12290, 2064, "bf16"), ("f32_8197x4096", 8197, 4096, "f32"),
                   ("f32_16386x1008", 16386, 1008, "f32")]


@pytest.mark.parametrize("name,tokens,n,dt", ACT_MANY_TOKENS, ids=[c[0] for c in ACT_MANY_TOKENS])
def test_quantize_act_rtn_many_tokens_per_wavefront(name, tokens, n, dt):
    say("act rtn case %s" % name)
    spec = synth.mini("am_" + name, 8, n, tokens, x_dtype=dt, f=32, n_outliers=16, seed_id=930)
    W = synth.make_weight(spec)
    x_np = synth.make_activations(spec)
    X = synth.activations_as_f32(spec, x_np).copy()
    X[5, :] = 0.0                                                # an all-zero token: scale 1
    X[tokens - 1, :] *= np.float32(3.0)                          # the last token, alone in its wavefront's tail
    x_np = synth.f32_to_bf16_bits(X) if dt == "bf16" else X
    X = synth.activations_as_f32(spec, x_np)
    _, abs_ref, cnt = orc.gram(X)
    sm = orc.smooth_outliers(W, abs_ref, cnt, spec.f)
    assert (sm.mdiag != 1.0).sum() >= spec.f - 1
    ctx = new_ctx()
    xd = to_dev_x(spec, x_np)
    for bits in (8, 6):
        ref_codes, ref_scales = orc.quantize_act_rtn(X, sm.mdiag, bits)
        codes = torch.zeros((tokens, n), dtype=torch.int8, device=DEV)
        scales = torch.empty(tokens, dtype=torch.float32, device=DEV)
        ctx.check(aser.aser_quantize_act_rtn(ctx, xd, torch.from_numpy(sm.mdiag).to(DEV), bits, codes, scales))
        torch.cuda.synchronize()
        assert np.array_equal(scales.cpu().numpy(), ref_scales)
        got = codes.cpu().numpy()
        bad = np.argwhere(got != ref_codes)
        assert bad.size == 0, "first mismatch at token %d channel %d" % (bad[0][0], bad[0][1])
        assert ref_scales[5] == 1.0


WHITEN_CASES = [
    ("c0", synth.CONFIGS["c0"], True),
    ("ragged", synth.mini("w1", 16, 333, 1200, f=6), True),
    ("multi_panel", synth.mini("w2", 16, 700, 2800, f=8), True),
    ("no_smoothing_ill_conditioned", synth.mini("w3", 16, 300, 900, f=0), False),
]


@pytest.mark.parametrize("name,spec,smooth", WHITEN_CASES, ids=[c[0] for c in WHITEN_CASES])
def test_whiten(name, spec, smooth):
    say("whiten case %s n=%d" % (name, spec.n))
    W = synth.make_weight(spec)
    x_np = synth.make_activations(spec)
    G_ref, abs_ref, cnt = orc.gram(synth.activations_as_f32(spec, x_np))
    sm = orc.smooth_outliers(W, abs_ref, cnt, spec.f)
    S_ref = orc.whiten(G_ref, sm.mdiag)
    ctx = new_ctx()
    ctx.ensure_workspace(aser.aser_workspace_bytes(spec.m, spec.n, 0))
    # only the lower triangle of G is defined by the ABI: poison the rest
    G32 = np.tril(G_ref).astype(np.float32) + np.triu(np.full_like(G_ref, 1e30, dtype=np.float32), 1)
    Gd = padded(torch.from_numpy(G32).to(DEV), 4)
    S = torch.empty_like(Gd)
    st, info = aser.aser_whiten(ctx, Gd, torch.from_numpy(sm.mdiag).to(DEV), 0.0, S)
    ctx.check(st)
    assert info == 0
    Sg = S.cpu().numpy().astype(np.float64)
    assert np.array_equal(Sg, np.tril(Sg)) and np.all(np.diag(Sg) > 0)
    Gp = S_ref @ S_ref.T
    assert np.linalg.norm(Sg @ Sg.T - Gp) / np.linalg.norm(Gp) < 2e-5
    assert np.linalg.norm(Sg - S_ref) / np.linalg.norm(S_ref) < 5e-4
    # in place, with damping
    st, info = aser.aser_whiten(ctx, Gd, torch.from_numpy(sm.mdiag).to(DEV), 0.01, Gd)
    ctx.check(st)
    Sd = orc.whiten(G_ref, sm.mdiag, damp=0.01)
    Sg = Gd.cpu().numpy().astype(np.float64)
    assert np.linalg.norm(Sg - Sd) / np.linalg.norm(Sd) < 5e-4


def test_whiten_reports_non_spd():
    n = 200
    rng = np.random.default_rng(5)
    X = rng.standard_normal((400, n)).astype(np.float32)
    X[:, 150] = 0.0                                              # a dead channel: zero pivot at index 151
    G = (X.astype(np.float64).T @ X.astype(np.float64)).astype(np.float32)
    ctx = new_ctx()
    ctx.ensure_workspace(aser.aser_workspace_bytes(8, n, 0))
    Gd = torch.from_numpy(G).to(DEV)
    S = torch.empty_like(Gd)
    st, info = aser.aser_whiten(ctx, Gd, None, 0.0, S)
    assert st == aser.ASER_ERR_NOT_SPD and info == 151
    st, info = aser.aser_whiten(ctx, Gd, None, 0.01, S)            # damping repairs it
    assert st == aser.ASER_OK and info == 0
    # without a host `info` the call does not synchronise; the pivot is reported by the next
    # aser_error_reconstruct on the context, and only once
    ctx.ensure_workspace(aser.aser_workspace_bytes(64, n, 4))
    st, info = aser.aser_whiten(ctx, Gd, None, 0.0, S, want_info=False)
    assert st == aser.ASER_OK and info is None
    T = torch.from_numpy(rng.standard_normal((64, n)).astype(np.float32)).to(DEV)
    Sok = torch.eye(n, dtype=torch.float32, device=DEV)
    L_A = torch.empty((64, 4), dtype=torch.float32, device=DEV)
    L_B = torch.empty((4, n), dtype=torch.float32, device=DEV)
    sigma = torch.empty(4, dtype=torch.float32, device=DEV)
    st, _, _ = aser.aser_error_reconstruct(ctx, T, Sok, 4, L_A, L_B, sigma)
    assert st == aser.ASER_ERR_NOT_SPD and "151" in ctx.last_error()
    st, err, _ = aser.aser_error_reconstruct(ctx, T, Sok, 4, L_A, L_B, sigma)
    assert st == aser.ASER_OK and np.isfinite(err)


def check_reconstruction(spec, ref, L_A, L_B, sigma, err_gpu, label):
    """The parity bars on L_A, L_B, evaluated against the oracle's fp64 T and S."""
    r = L_A.shape[1]
    rec = ref.rec if ref.rec.L_A.shape[1] == r else orc.error_reconstruct(ref.quant.T, ref.S, r)
    e = orc.whitened_error(ref.quant.T, ref.S, L_A, L_B)
    rel = abs(e - rec.err) / rec.err
    say("%s: r=%d gap=%.4f oracle err=%.6g gpu(recomputed)=%.6g rel=%.2e gpu scalar rel=%.2e" %
        (label, r, rec.gap, rec.err, e, rel, abs(err_gpu - rec.err) / rec.err))
    assert rel <= 1e-4
    assert abs(err_gpu - rec.err) / rec.err <= 1e-4
    # singular values: those of the planted outlier directions are isolated and must agree closely; the rest
    # sit in a near-continuous bulk where a Ritz value is a weighted mean of its neighbours
    k_iso = min(r, spec.n_outliers)
    assert np.allclose(sigma[:k_iso], rec.sigma[:k_iso], rtol=1e-3)
    assert np.allclose(sigma[:min(r, spec.f)], rec.sigma[:min(r, spec.f)], rtol=5e-3)
    assert np.all(np.diff(sigma) <= 1e-6 * sigma[0])
    if rec.gap > 1.05:
        P = L_A.astype(np.float64) @ L_B.astype(np.float64)
        Pr = rec.L_A @ rec.L_B
        relP = np.linalg.norm(P - Pr) / np.linalg.norm(Pr)
        say("%s: product rel Frobenius %.2e" % (label, relP))
        assert relP <= 1e-3
    return rec


REC_CASES = [
    ("c0", synth.CONFIGS["c0"], None),
    ("c0_r_eq_f", synth.CONFIGS["c0"], 4),
    ("ragged", synth.mini("r1", 150, 333, 1200, r=24, f=6), None),
    ("ragged_r_eq_f", synth.mini("r1", 150, 333, 1200, r=24, f=6), 6),
    ("wide", synth.mini("r2", 96, 700, 2800, r=16, f=8), None),
    ("tall_silu", synth.mini("r3", 600, 260, 1024, r=32, f=8, x_dist="silu_prod", out=(40.0, 40.0)), None),
]


@pytest.mark.parametrize("name,spec,r", REC_CASES, ids=[c[0] for c in REC_CASES])
def test_error_reconstruct_from_oracle_inputs(name, spec, r):
    """Stage 4b/4c alone: T and S come from the oracle (rounded to fp32)."""
    r = spec.r if r is None else r
    say("reconstruct case %s m=%d n=%d r=%d" % (name, spec.m, spec.n, r))
    W = synth.make_weight(spec)
    x_np = synth.make_activations(spec)
    ref = oracle_layer(spec, W, x_np, r=r)
    ctx = new_ctx()
    ctx.ensure_workspace(aser.aser_workspace_bytes(spec.m, spec.n, r))
    T = padded(torch.from_numpy(ref.quant.T.astype(np.float32)).to(DEV), 4)
    S = torch.from_numpy(ref.S.astype(np.float32)).to(DEV)
    L_A = torch.empty((spec.m, r), dtype=torch.float32, device=DEV)
    L_B = torch.empty((r, spec.n), dtype=torch.float32, device=DEV)
    sigma = torch.empty(r, dtype=torch.float32, device=DEV)
    # these layers are small enough for the dense solver (the default); a given iteration count asks for the
    # subspace iteration instead, here with the outlier columns of the oracle's selection leading its start block
    st, err, nit = aser.aser_error_reconstruct(ctx, T, S, r, L_A, L_B, sigma)
    ctx.check(st)
    assert nit == 0
    check_reconstruction(spec, ref, L_A.cpu().numpy(), L_B.cpu().numpy(), sigma.cpu().numpy(), err, name + " dense")
    idx = torch.from_numpy(ref.smooth.idx).to(DEV)
    st, err, nit = aser.aser_error_reconstruct(ctx, T, S, r, L_A, L_B, sigma, aser.aser_svd_opts(block=0, max_iter=12, seed=0),
                                               idx=idx, f=len(ref.smooth.idx))
    ctx.check(st)
    assert nit == 12
    check_reconstruction(spec, ref, L_A.cpu().numpy(), L_B.cpu().numpy(), sigma.cpu().numpy(), err, name + " iterative")


E2E_CASES = [
    ("c0", synth.CONFIGS["c0"], True),
    ("c0_int8_no_smoothing", synth.CONFIGS["c0"].with_(bits=8, f=0), False),
    ("ragged", synth.mini("e1", 130, 333, 1500, r=24, f=6), False),
    ("c1_shape_small", synth.CONFIGS["c1"].with_(m=512, n=768, tokens=3072, r=32, f=16), True),
    ("c2_shape_small", synth.CONFIGS["c2"].with_(m=384, n=1032, tokens=4096, r=32, f=16, n_outliers=8), True),
    # r = 128 fills the widest subspace block: no oversampling columns, the longer default iteration
    ("c4_shape_small", synth.CONFIGS["c4"].with_(m=1024, n=3584, tokens=8192), True),
    # W8 with smoothed outliers: the unquantized columns of T dwarf the int8 rounding error
    # (sigma_1 / sigma_b in the thousands); needs the graded start block (outlier columns first)
    ("w8_outliers", synth.mini("fz1", 613, 404, 1038, n_outliers=6, r=20, f=25, bits=8, seed_id=701), False),
    ("w8_outliers_silu_f32", synth.mini("fz8", 181, 548, 1501, x_dtype="f32", x_dist="silu_prod", n_outliers=6, r=40, f=23,
                                        bits=8, seed_id=708), False),
    ("w8_few_outliers", synth.mini("fz21", 145, 410, 1105, n_outliers=3, r=31, f=3, bits=8, seed_id=721), False),
    # ranks beyond the widest subspace block (128) take the dense solver whatever the size of the layer
    ("rank_160_dense_solver", synth.mini("rk1", 700, 1536, 4096, n_outliers=8, r=160, f=16, seed_id=731), True),
    ("rank_192_dense_solver_tall", synth.mini("rk2", 2304, 2048, 6144, x_dist="silu_prod", n_outliers=8, r=192, f=32,
                                              seed_id=732, out=(40.0, 40.0)), True),
    # the subspace block is nearly as wide as the matrix (b = 64 of n = 74): the end of the spectrum is in it
    ("block_as_wide_as_matrix", synth.mini("fz7", 322, 74, 333, x_dtype="f32", x_dist="silu_prod", n_outliers=6, r=23, f=6,
                                           bits=4, seed_id=707), True),
]


def run_e2e(name, spec, packed, x_np=None, ref=None, precision=None):
    W = synth.make_weight(spec)
    if x_np is None:
        x_np = synth.make_activations(spec)
    if ref is None:
        ref = oracle_layer(spec, W, x_np)
    ctx = new_ctx()
    if precision is not None:
        ctx.set_precision(precision)
    buf = aser.LayerBuffers(spec.m, spec.n, spec.r, spec.f, spec.bits, packed)
    aser.calibrate_layer(ctx, torch.from_numpy(W).to(DEV), to_dev_x(spec, x_np), buf)
    torch.cuda.synchronize()
    check_layer(name, spec, packed, buf, ref)
    return buf, ref


def check_layer(name, spec, packed, buf, ref):
    """Every bar of a calibrated layer in `buf` against the oracle's `ref`."""
    if spec.f:
        assert buf.idx.cpu().numpy()[:spec.f].tolist() == ref.smooth.idx.tolist()
        planted, _ = synth.outlier_channels(spec)
        assert set(planted.tolist()) <= set(ref.smooth.idx.tolist())
    codes = buf.codes.cpu().numpy()
    if packed:
        codes = unpack_int4(codes)
    assert np.array_equal(codes, ref.quant.codes)
    assert np.array_equal(buf.scales.cpu().numpy(), ref.quant.scales)
    check_reconstruction(spec, ref, buf.L_A.cpu().numpy(), buf.L_B.cpu().numpy(), buf.sigma.cpu().numpy(), buf.err, name)


@pytest.mark.parametrize("name,spec,packed", E2E_CASES, ids=[c[0] for c in E2E_CASES])
def test_end_to_end_layer(name, spec, packed):
    say("e2e case %s m=%d n=%d N=%d r=%d f=%d" % (name, spec.m, spec.n, spec.tokens, spec.r, spec.f))
    run_e2e(name, spec, packed)


def test_layers_in_flight():
    """aser_calibrate_layers: layers of different shapes, bit widths and solvers on three contexts (three streams),
    two of them sharing one input's finished statistics, one with empty statistics in the middle.  Every layer
    meets the bars against the oracle; the layer without tokens is reported in its own descriptor and disturbs
    no other; aser_error_reconstruct_enqueue / aser_finish refuse what their protocol forbids."""
    # ragged, c1 / c2 shapes, a c4-shaped layer that takes the subspace iteration (the others are small enough for
    # the dense solver), W8 with outliers, tiny block
    picks = [E2E_CASES[i] for i in (2, 3, 4, 5, 6, 11)]
    assert picks[3][0] == "c4_shape_small"
    pool = [torch.cuda.Stream(device=0) for _ in range(12)]
    st, picked = aser.aser_pick_concurrent_streams([s.cuda_stream for s in pool], 3)
    assert st == aser.ASER_OK and len(set(picked)) == len(picked) == 3           # four hardware queues per process
    streams = [pool[i] for i in picked]
    ctxs = [aser.Context(0, stream=s.cuda_stream) for s in streams]
    layers = []
    for i, (name, spec, packed) in enumerate(picks):
        W = synth.make_weight(spec)
        x_np = synth.make_activations(spec)
        # every other layer leaves G, T and S to the context's workspace
        buf = aser.LayerBuffers(spec.m, spec.n, spec.r, spec.f, spec.bits, packed, intermediates=(i % 2 == 0))
        layers.append(dict(name=name, spec=spec, packed=packed, W=torch.from_numpy(W).to(DEV), X=to_dev_x(spec, x_np), buf=buf,
                           ref=oracle_layer(spec, W, x_np)))
    # a second layer on the first one's input (another weight, same shape): its statistics are accumulated before the call
    name, spec, packed = picks[0]
    spec2 = spec.with_(name=spec.name + "_b", layer_id=spec.layer_id + 1)      # another weight, the same input stream
    W2 = synth.make_weight(spec2)
    assert not np.array_equal(W2, synth.make_weight(spec))
    x_np = synth.make_activations(spec)
    shared = aser.LayerBuffers(spec.m, spec.n, spec.r, spec.f, spec.bits, packed)
    c0 = new_ctx()
    c0.check(aser.aser_gram_accumulate(c0, layers[0]["X"], shared.G, shared.abs_sum, shared.count))
    layers.append(dict(name=name + "_shared_input", spec=spec2, packed=packed, W=torch.from_numpy(W2).to(DEV), X=None, buf=shared,
                       ref=oracle_layer(spec2, W2, x_np)))
    # a layer without tokens: statistics all zero
    empty = aser.LayerBuffers(spec.m, spec.n, spec.r, spec.f, spec.bits, packed)
    layers.insert(2, dict(name="no_tokens", spec=spec, packed=packed, W=layers[0]["W"], X=None, buf=empty, ref=None))
    torch.cuda.synchronize()
    descs = [aser.layer_desc(L["W"], L["buf"], X=L["X"], clear_stats=L["X"] is not None) for L in layers]
    need = max(aser.aser_layer_workspace_bytes(d) for d in descs)
    assert need > max(aser.aser_workspace_bytes(L["spec"].m, L["spec"].n, L["spec"].r) for L in layers)
    for c in ctxs:
        c.ensure_workspace(need)
    for L in layers:
        if L["X"] is not None and L["buf"].G is not None:
            L["buf"].G.fill_(7.0)                                   # clear_stats has to remove this
    torch.cuda.synchronize()
    say("layers in flight: %s on %d contexts" % ([L["name"] for L in layers], len(ctxs)))
    st = aser.aser_calibrate_layers(ctxs, descs)
    torch.cuda.synchronize()
    assert st == aser.ASER_ERR_INVALID_ARG                          # the first failing layer's status
    for L, d in zip(layers, descs):
        if L["ref"] is None:
            assert d.status == aser.ASER_ERR_INVALID_ARG
            continue
        assert d.status == aser.ASER_OK, (L["name"], d.status)
        L["buf"].err = d.err
        check_layer(L["name"], L["spec"], L["packed"], L["buf"], L["ref"])
    # the protocol of the two halves
    L = layers[0]
    b, ctx = L["buf"], ctxs[0]
    st = aser.aser_error_reconstruct_enqueue(ctx, b.T, b.S, b.r, b.L_A, b.L_B, b.sigma, idx=b.idx, f=b.f)
    assert st == aser.ASER_OK
    assert aser.aser_error_reconstruct_enqueue(ctx, b.T, b.S, b.r, b.L_A, b.L_B, b.sigma, idx=b.idx, f=b.f) == aser.ASER_ERR_INVALID_ARG
    assert aser.aser_set_workspace(ctx, None, 0) == aser.ASER_ERR_INVALID_ARG
    st, err, _ = aser.aser_finish(ctx)
    assert st == aser.ASER_OK and abs(err - descs[0].err) <= 1e-5 * err
    assert aser.aser_finish(ctx)[0] == aser.ASER_ERR_INVALID_ARG


def test_layers_that_share_an_input_in_one_call():
    """Three layers on one input stream (the q, k, v of an attention block: different weights and output widths),
    then two on another (gate, up), all in ONE aser_calibrate_layers call on three contexts: the first layer of
    each group accumulates the statistics, the others name it in stats_from and wait for its Gram update only.
    Every layer meets the bars; the shared Gram matrix is accumulated once."""
    groups = [(synth.mini("sh_q", 320, 512, 3000, r=24, f=8, seed_id=741), [(96, 742), (128, 743)]),
              (synth.mini("sh_gate", 700, 384, 2500, x_dist="silu_prod", r=20, f=6, seed_id=751, out=(40.0, 40.0)), [(700, 752)])]
    pool = [torch.cuda.Stream(device=0) for _ in range(12)]
    st, picked = aser.aser_pick_concurrent_streams([s.cuda_stream for s in pool], 3)
    assert st == aser.ASER_OK and len(picked) == 3
    ctxs = [aser.Context(0, stream=pool[i].cuda_stream) for i in picked]
    layers, descs = [], []
    for owner_spec, others in groups:
        x_np = synth.make_activations(owner_spec)
        X = to_dev_x(owner_spec, x_np)
        owner_index = len(layers)
        for k, spec in enumerate([owner_spec] + [owner_spec.with_(name="%s_%d" % (owner_spec.name, lid), m=m, layer_id=lid)
                                                for m, lid in others]):
            W = synth.make_weight(spec)
            buf = aser.LayerBuffers(spec.m, spec.n, spec.r, spec.f, spec.bits, True, intermediates=(k == 0))
            if k == 0:
                buf.G.fill_(3.0)                                    # clear_stats has to remove this
            Wd = torch.from_numpy(W).to(DEV)
            layers.append(dict(spec=spec, buf=buf, W=Wd, X=X, ref=oracle_layer(spec, W, x_np)))
            descs.append(aser.layer_desc(Wd, buf, X=X if k == 0 else None, clear_stats=(k == 0),
                                         stats_from=None if k == 0 else owner_index))
    need = max(aser.aser_layer_workspace_bytes(d) for d in descs)
    for c in ctxs:
        c.ensure_workspace(need)
    torch.cuda.synchronize()
    say("layers that share an input: %s" % [L["spec"].name for L in layers])
    assert aser.aser_calibrate_layers(ctxs, descs) == aser.ASER_OK
    torch.cuda.synchronize()
    for L, d in zip(layers, descs):
        assert d.status == aser.ASER_OK, (L["spec"].name, d.status)
        L["buf"].err = d.err
        check_layer(L["spec"].name, L["spec"], True, L["buf"], L["ref"])
    assert int(layers[0]["buf"].count.item()) == groups[0][0].tokens   # accumulated once, not once per layer
    # an owner that leaves its statistics to the workspace cannot be shared
    spec = groups[0][0]
    lone = aser.LayerBuffers(spec.m, spec.n, spec.r, spec.f, spec.bits, True, intermediates=False)
    other = aser.LayerBuffers(spec.m, spec.n, spec.r, spec.f, spec.bits, True, intermediates=False)
    bad = [aser.layer_desc(layers[0]["W"], lone, X=layers[0]["X"]), aser.layer_desc(layers[0]["W"], other, stats_from=0)]
    assert aser.aser_calibrate_layers(ctxs, bad) == aser.ASER_ERR_INVALID_ARG
    assert [d.status for d in bad] == [aser.ASER_ERR_INVALID_ARG, aser.ASER_ERR_INVALID_ARG]
    for c in ctxs:
        c.close()


def test_layer_chain_under_graph_capture():
    """The five stages of a layer captured into a HIP graph on the context's stream (aser_error_reconstruct_enqueue:
    nothing in the chain waits for the device, every clearing pass is a fill kernel) and replayed three times, with
    eager calibrations of another layer and synchronisations between the replays: every replay gives the codes,
    scales and outlier set of the eager run bit for bit, factors that meet the bars against the oracle, and the
    whitened error in the status block that the graph's copy node brings to the host."""
    name, spec, packed = E2E_CASES[5]                               # c4-shaped: the subspace iteration
    other = E2E_CASES[3][1]
    W = synth.make_weight(spec)
    x_np = synth.make_activations(spec)
    ref = oracle_layer(spec, W, x_np)
    Wd, Xd = torch.from_numpy(W).to(DEV), to_dev_x(spec, x_np)
    Wo, Xo = torch.from_numpy(synth.make_weight(other)).to(DEV), to_dev_x(other, synth.make_activations(other))
    s = torch.cuda.Stream(device=0)
    ctx = aser.Context(0, stream=s.cuda_stream)
    buf = aser.LayerBuffers(spec.m, spec.n, spec.r, spec.f, spec.bits, packed)
    ctx.ensure_workspace(aser.aser_workspace_bytes(spec.m, spec.n, spec.r))
    layout = aser.ASER_CODES_INT4_PACKED if packed else aser.ASER_CODES_INT8

    def enqueue():
        buf.reset_statistics()
        ctx.check(aser.aser_gram_accumulate(ctx, Xd, buf.G, buf.abs_sum, buf.count))
        ctx.check(aser.aser_smooth_outliers(ctx, Wd, buf.abs_sum, buf.count, buf.f, buf.idx, buf.mdiag))
        ctx.check(aser.aser_quantize_rtn(ctx, Wd, buf.idx, buf.mdiag, buf.f, buf.bits, layout, buf.codes, buf.scales, buf.T))
        st, _ = aser.aser_whiten(ctx, buf.G, buf.mdiag, 0.0, buf.S, want_info=False)
        ctx.check(st)
        ctx.check(aser.aser_error_reconstruct_enqueue(ctx, buf.T, buf.S, buf.r, buf.L_A, buf.L_B, buf.sigma, idx=buf.idx, f=buf.f))

    with torch.cuda.stream(s):
        enqueue()                                                   # eager once: function attributes, pinned status block
        st, err_eager, _ = aser.aser_finish(ctx)
        ctx.check(st)
    torch.cuda.synchronize()
    buf.err = err_eager
    check_layer(name + " eager", spec, packed, buf, ref)
    eager = [t.clone() for t in (buf.codes, buf.scales, buf.idx)]
    g = torch.cuda.CUDAGraph()
    with torch.cuda.graph(g, stream=s):
        enqueue()
    st, _, _ = aser.aser_finish(ctx)                                # nothing ran: this only ends the pending state of the capture
    ctx.check(st)
    ctx2 = new_ctx()
    buf2 = aser.LayerBuffers(other.m, other.n, other.r, other.f, other.bits, True)
    for rep in range(3):
        for t in (buf.codes, buf.scales, buf.idx, buf.L_A, buf.L_B, buf.sigma):
            t.zero_()
        aser.calibrate_layer(ctx2, Wo, Xo, buf2)                    # eager work of the program between the replays
        torch.cuda.synchronize()
        say("graph replay %d of layer %s" % (rep, name))
        g.replay()
        torch.cuda.synchronize()
        for t, e in zip((buf.codes, buf.scales, buf.idx), eager):
            assert torch.equal(t, e)
        # this replay's squared whitened error: the double at byte 16 of the status block, which is the last 256
        # bytes of the bound workspace
        off = (-ctx._ws.data_ptr()) % 256 + ctx._ws_bytes - 256
        buf.err = float(ctx._ws[off + 16:off + 24].view(torch.float64).item()) ** 0.5
        assert abs(buf.err - err_eager) <= 1e-4 * err_eager
        check_layer(name + " replay %d" % rep, spec, packed, buf, ref)


# Layers that a randomized sweep found beyond the bars while every fp32 product was three bf16 products
# (2^-16): int8 weights with smoothed outlier columns, a few hundred channels at most and a rank near
# half the width, so that the error left after compensation is a few 1e-5 of ||T S||_F.  Small problems
# now take six products per fp32 product (2^-24) in the Gram matrix of fp32 activations, the whitening
# and the reconstruction; each of these layers must meet every bar.
def _w8(tag, m, n, N, r, f, xd, dist, seed_id):
    return (tag, synth.mini(tag, m, n, N, x_dtype=xd, x_dist=dist, n_outliers=min(6, max(f, 1)), r=r, f=f, bits=8,
                            seed_id=seed_id))


W8_SMALL_LAYERS = [
    _w8("w8s_225x164", 225, 164, 624, 44, 9, "bf16", "gauss", 715),
    _w8("w8s_510x72", 510, 72, 265, 23, 13, "bf16", "gauss", 717),
    _w8("w8s_110x194", 110, 194, 533, 45, 34, "f32", "gauss", 724),
    _w8("w8s_151x82", 151, 82, 237, 44, 16, "f32", "gauss", 730),
    _w8("w8s_525x92", 525, 92, 192, 37, 16, "f32", "silu_prod", 733),
    _w8("w8s_288x74", 288, 74, 251, 46, 16, "bf16", "gauss", 739),
    _w8("w8s_563x122", 563, 122, 267, 31, 27, "f32", "silu_prod", 743),
    _w8("w8s_134x80", 134, 80, 190, 32, 9, "bf16", "silu_prod", 706),
    _w8("w8s_58x480", 58, 480, 1689, 32, 12, "bf16", "silu_prod", 732),
]


@pytest.mark.parametrize("name,spec", W8_SMALL_LAYERS, ids=[c[0] for c in W8_SMALL_LAYERS])
def test_small_int8_layers_with_tiny_residuals(name, spec):
    say("e2e case %s m=%d n=%d N=%d r=%d f=%d" % (name, spec.m, spec.n, spec.tokens, spec.r, spec.f))
    run_e2e(name, spec, False)


@pytest.mark.parametrize("precision", [aser.ASER_PRECISION_FAST, aser.ASER_PRECISION_EXACT], ids=["three_products", "six_products"])
def test_both_product_forms_meet_the_bars(precision):
    """The same mid-size layers through the three-product and the six-product form of the fp32 contractions
    (the automatic choice would take only one of them at each size)."""
    for name, spec, packed in (("c1_shape_small", synth.CONFIGS["c1"].with_(m=512, n=768, tokens=3072, r=32, f=16), True),
                               ("c4_shape_small", synth.CONFIGS["c4"].with_(m=1024, n=3584, tokens=8192), True),
                               ("f32_activations", synth.mini("pf1", 300, 1300, 4200, x_dtype="f32", r=24, f=8), False)):
        say("e2e case %s precision mode %d" % (name, precision))
        run_e2e(name + "_p%d" % precision, spec, packed, precision=precision)


def test_headline_layer_full_size():
    """The 4096 x 4096 layer with 32768 calibration tokens (the configuration the bench times),
    every output against the oracle: this is the only case where the persistent Gram schedule,
    32 Cholesky panels and the 128-wide subspace iteration all run at their real shapes."""
    spec = synth.CONFIGS["c1"]
    say("e2e case c1 full size m=%d n=%d N=%d r=%d f=%d" % (spec.m, spec.n, spec.tokens, spec.r, spec.f))
    _, ref = run_e2e("c1_full", spec, True)
    # the same layer twice through aser_calibrate_layers, two in flight, G / T / S in the contexts' workspaces (the
    # configuration the bench line's `value` times): the same bars against the same oracle results
    say("c1 full size, two layers in flight")
    pool = [torch.cuda.Stream(device=0) for _ in range(8)]
    st, picked = aser.aser_pick_concurrent_streams([s.cuda_stream for s in pool], 2)
    assert st == aser.ASER_OK and len(picked) == 2
    ctxs = [aser.Context(0, stream=pool[i].cuda_stream) for i in picked]
    W = torch.from_numpy(synth.make_weight(spec)).to(DEV)
    X = to_dev_x(spec, synth.make_activations(spec))
    bufs = [aser.LayerBuffers(spec.m, spec.n, spec.r, spec.f, spec.bits, True, intermediates=False) for _ in range(2)]
    descs = [aser.layer_desc(W, b, X=X) for b in bufs]
    for c in ctxs:
        c.ensure_workspace(aser.aser_layer_workspace_bytes(descs[0]))
    torch.cuda.synchronize()
    assert aser.aser_calibrate_layers(ctxs, descs) == aser.ASER_OK
    torch.cuda.synchronize()
    for k, (b, d) in enumerate(zip(bufs, descs)):
        assert d.status == aser.ASER_OK and d.n_iter == 9
        b.err = d.err
        check_layer("c1_full_in_flight_%d" % k, spec, True, b, ref)
    # sixteen contexts and twenty layers, as the bench line's headline runs them (there on streams that the
    # runtime really runs side by side; here on whatever queues sixteen streams get): contexts are reused for the
    # last four layers.  Integer outputs of every layer equal the verified ones; the first layer and one that ran
    # on a reused context meet every bar, the others' errors agree with theirs.
    say("c1 full size, twenty layers on sixteen contexts")
    for c in ctxs:
        c.close()
    pool = [torch.cuda.Stream(device=0) for _ in range(16)]
    ctxs = [aser.Context(0, stream=s.cuda_stream) for s in pool]
    many = [aser.LayerBuffers(spec.m, spec.n, spec.r, spec.f, spec.bits, True, intermediates=False) for _ in range(20)]
    descs = [aser.layer_desc(W, b, X=X) for b in many]
    for c in ctxs:
        c.ensure_workspace(aser.aser_layer_workspace_bytes(descs[0]))
    torch.cuda.synchronize()
    assert aser.aser_calibrate_layers(ctxs, descs) == aser.ASER_OK
    torch.cuda.synchronize()
    codes0, idx0 = bufs[0].codes.cpu(), bufs[0].idx.cpu()
    for k, (b, d) in enumerate(zip(many, descs)):
        assert d.status == aser.ASER_OK and d.n_iter == 9
        assert torch.equal(b.codes.cpu(), codes0) and torch.equal(b.idx.cpu(), idx0)
        assert torch.equal(b.scales, bufs[0].scales)
        assert abs(d.err - ref.rec.err) <= 1e-4 * ref.rec.err
        b.err = d.err
    check_layer("c1_full_sixteen_contexts_first", spec, True, many[0], ref)
    check_layer("c1_full_sixteen_contexts_reused", spec, True, many[18], ref)
    for c in ctxs:
        c.close()


def test_headline_layer_full_size_rank_at_the_spectral_gap():
    """The same layer with r = 16, the number of planted outlier channels: their columns of T stand far
    above everything else (sigma_16 / sigma_17 = 6.7; the other 16 of the f = 32 extracted channels are
    ordinary ones, so r = f = 32 sits in the bulk with a gap of 1.001), the product L_A L_B is determined
    and the 1e-3 bar on it runs at full size (Sec. 4.1 definitions of L_A, L_B)."""
    spec = synth.CONFIGS["c1"].with_(r=16)
    say("e2e case c1 full size with r = 16")
    _, ref = run_e2e("c1_full_r16", spec, True)
    assert ref.rec.gap > 1.05


def test_headline_layer_full_size_rank_beyond_the_subspace_block():
    """The same layer with r = 200: ranks above 128 (the rule of Eq. 9 can ask for them) go to the dense
    fp64 solver at any size, here with 4096 eigenvalues and stored reflectors."""
    spec = synth.CONFIGS["c1"].with_(r=200)
    say("e2e case c1 full size with r = 200 (dense solver)")
    assert aser.aser_svd_plan(spec.m, spec.n, spec.r) == (aser.ASER_OK, 0, 0)
    run_e2e("c1_full_r200", spec, True)


@pytest.mark.parametrize("cfg", ["c2", "c3.q", "c3.k", "c3.v", "c3.o", "c3.gate", "c3.up", "c3.down", "c4", "qkv"])
def test_large_layers_full_size(cfg):
    """Full-size layers whose oracle SVD takes minutes: the 4096 x 11008 layer with 65536 tokens of
    heavy-tailed activations, the seven layers of the Llama-3-8B-shaped block with 131072 tokens per
    input stream, and the 8192 x 28672 layer with 262144 tokens and r = 128 (15 GB of activations, a
    3.3 GB Gram matrix, no oversampling columns in the subspace block).  Nothing is sampled:
      * statistics, outlier set, smoothing diagonal, RTN codes, scales and T: every entry against the oracle;
      * Gram matrix: G V against X^T (X V) in fp64 for random sign vectors V (every entry of the lower
        triangle enters), plus exact entries on a set of channel pairs;
      * whitening factor: strictly upper triangle zero everywhere, S (S^T V) against M^-1 X^T (X M^-1 V)
        (Eq. 5 with the smoothed activations of Algorithm 1), both sides from fp64 host arithmetic on X;
      * factors: the whitened error of Eq. 8 recomputed in fp64 from L_A, L_B with T and S as the oracle
        defines them from this layer's statistics (T from the oracle's RTN; S enters only through
        S S^T = G', checked above), against the optimum from LAPACK's symmetric eigen-solver."""
    spec = synth.CONFIGS[cfg]
    say("%s full size m=%d n=%d N=%d r=%d f=%d" % (cfg, spec.m, spec.n, spec.tokens, spec.r, spec.f))
    rng = np.random.default_rng(7)
    W = synth.make_weight(spec)
    x_np = synth.make_activations(spec, workers=12)
    say("%s: inputs drawn" % cfg)
    ctx = new_ctx()
    buf = aser.LayerBuffers(spec.m, spec.n, spec.r, spec.f, spec.bits, True)
    aser.calibrate_layer(ctx, torch.from_numpy(W).to(DEV), to_dev_x(spec, x_np), buf)
    torch.cuda.synchronize()
    say("%s: device path done, err=%.6g" % (cfg, buf.err))
    n, m = spec.n, spec.m

    # one fp64 pass over X on the host: |x| sums, X^T (X V) and X^T (X M^-1 V) for random sign vectors
    nv = 3
    V = rng.choice([-1.0, 1.0], size=(n, nv))
    abs_ref = np.zeros(n)
    for a in range(0, spec.tokens, 8192):
        abs_ref += np.abs(synth.bf16_to_f32(x_np[a:a + 8192])).sum(axis=0, dtype=np.float64)
    assert np.allclose(buf.abs_sum.cpu().numpy(), abs_ref, rtol=1e-12, atol=0)
    sm = orc.smooth_outliers(W, abs_ref, spec.tokens, spec.f)
    assert buf.idx.cpu().numpy()[:spec.f].tolist() == sm.idx.tolist()
    assert np.array_equal(buf.mdiag.cpu().numpy(), sm.mdiag)
    minv = 1.0 / sm.mdiag.astype(np.float64)
    V2 = np.concatenate([V, minv[:, None] * V], axis=1)
    XtXV = np.zeros((n, 2 * nv))
    gdiag = np.zeros(n)
    for a in range(0, spec.tokens, 4096):
        xc = synth.bf16_to_f32(x_np[a:a + 4096]).astype(np.float64)
        XtXV += xc.T @ (xc @ V2)
        gdiag += np.einsum("ij,ij->j", xc, xc)
    del xc
    say("%s: host pass over X done" % cfg)

    # Gram matrix: every entry of the lower triangle through G V
    G = buf.G.cpu().numpy()
    GV = np.zeros((n, nv))
    for a in range(0, n, 2048):
        blk = np.tril(G[a:a + 2048].astype(np.float64), k=a)          # rows a.., columns <= row
        GV[a:a + 2048] += blk @ V
        blk[:, a:a + 2048] -= np.diag(np.diag(blk[:, a:a + 2048]))    # strictly lower part, transposed contribution
        GV += blk.T @ V[a:a + 2048]
    d = np.sqrt(gdiag)
    # entry errors are bounded by 2e-5 sqrt(G_ii G_jj) and have random signs: their sum over a row of n
    # entries against sign vectors stays within a fifth of that bound times sqrt(sum_j G_jj)
    tol = 4e-6 * d[:, None] * np.sqrt((gdiag[:, None] * V * V).sum(axis=0))[None, :]
    worst = float((np.abs(GV - XtXV[:, :nv]) / tol).max())
    say("%s: G V against X^T (X V): worst entry at %.2f of its tolerance" % (cfg, worst))
    assert worst <= 1.0
    assert np.allclose(np.diag(G), gdiag, rtol=2e-5)
    # exact entries on channel pairs across tiles, the last tile and planted outliers
    planted, _ = synth.outlier_channels(spec)
    cols = np.unique(np.concatenate([rng.integers(0, n, 20), [0, 255, 256, n - 1, n - 256], planted[:4]]))
    Xs = synth.bf16_to_f32(x_np[:, cols])
    G_ref, _, _ = orc.gram(Xs)
    Gs = np.where(cols[:, None] >= cols[None, :], G[np.ix_(cols, cols)], G[np.ix_(cols, cols)].T)
    dc = np.sqrt(np.diag(G_ref))
    assert np.all(np.abs(Gs - G_ref) <= 2e-5 * np.outer(dc, dc))
    del Xs, G

    # RTN: every row
    ref_q = orc.quantize_rtn(W, sm.idx, sm.mdiag, spec.bits)
    assert np.array_equal(unpack_int4(buf.codes.cpu().numpy()), ref_q.codes)
    assert np.array_equal(buf.scales.cpu().numpy(), ref_q.scales)
    assert np.all(np.abs(buf.T.cpu().numpy() - ref_q.T) <= 2.0 ** -23 * np.abs(ref_q.T) + 1e-30)
    T = ref_q.T                                                   # the oracle's target, fp64
    say("%s: RTN compared on every row" % cfg)

    # whitening factor: lower triangular everywhere, and S S^T V = G' V with G' = M^-1 X^T X M^-1 from the host pass
    assert int(torch.count_nonzero(torch.triu(buf.S, 1)).item()) == 0
    S = buf.S.cpu().numpy().astype(np.float64)
    assert np.all(np.diag(S) > 0)
    GpV = minv[:, None] * XtXV[:, nv:]
    SSV = S @ (S.T @ V)
    gp = gdiag * minv * minv
    tol = 6e-6 * np.sqrt(gp)[:, None] * np.sqrt((gp[:, None] * V * V).sum(axis=0))[None, :]
    worst = float((np.abs(SSV - GpV) / tol).max())
    say("%s: S S^T V against G' V: worst entry at %.2f of its tolerance" % (cfg, worst))
    assert worst <= 1.0

    # Eq. 8: the whitened error of the returned factors (oracle T, S as checked above), against the
    # reported scalar and against the optimum; sigma and the residual split the energy of T S
    L_A = buf.L_A.cpu().numpy()
    L_B = buf.L_B.cpu().numpy()
    sigma = buf.sigma.cpu().numpy().astype(np.float64)
    e = orc.whitened_error(T, S, L_A, L_B)
    say("%s: whitened error recomputed %.6g reported %.6g rel %.2e" % (cfg, e, buf.err, abs(e - buf.err) / e))
    assert abs(e - buf.err) / e <= 1e-4
    A = T @ S
    e0 = float(np.linalg.norm(A))
    assert e < e0
    lam = np.maximum(np.linalg.eigvalsh(A @ A.T if m <= n else A.T @ A)[::-1], 0.0)
    e_opt = float(np.sqrt(np.sum(lam[spec.r:])))
    say("%s: optimal whitened error %.6g, device %.6g, rel %.2e; sigma_r/sigma_r+1 = %.4f" %
        (cfg, e_opt, e, (e - e_opt) / e_opt, np.sqrt(lam[spec.r - 1] / lam[spec.r])))
    assert 0.0 <= (e - e_opt) / e_opt + 1e-9 and (e - e_opt) / e_opt <= 1e-4
    assert np.allclose(sigma[:spec.f], np.sqrt(lam[:spec.f]), rtol=1e-3)
    del A
    assert abs(e * e + float(np.sum(sigma ** 2)) - e0 * e0) <= 1e-4 * e0 * e0
    assert np.all(np.diff(sigma) <= 1e-6 * sigma[0])


def test_quantizers_with_denormal_scales():
    """Rows whose absmax / qmax is a denormal or tiny fp32 number: the reciprocal of such a scale is not
    finite, so the kernels must take true divisions there; codes and scales stay bit-exact."""
    spec = synth.mini("qd", 12, 512, 64, f=4)
    W = synth.make_weight(spec)
    W[2, :] *= np.float32(1e-37)                                 # scale ~ 1e-39 (int4) / 5e-41 (int8): denormal
    W[5, :] *= np.float32(1e-30)                                 # tiny but normal
    x_np = synth.make_activations(spec)
    _, abs_ref, cnt = orc.gram(synth.activations_as_f32(spec, x_np))
    sm = orc.smooth_outliers(W, abs_ref, cnt, spec.f)
    idx = torch.from_numpy(sm.idx).to(DEV)
    mdiag = torch.from_numpy(sm.mdiag).to(DEV)
    for bits, packed in ((4, True), (8, False)):
        ref = orc.quantize_rtn(W, sm.idx, sm.mdiag, bits)
        ctx = new_ctx()
        codes = torch.zeros((spec.m, spec.n // 2 if packed else spec.n), dtype=torch.uint8 if packed else torch.int8, device=DEV)
        scales = torch.empty(spec.m, dtype=torch.float32, device=DEV)
        T = torch.empty((spec.m, spec.n), dtype=torch.float32, device=DEV)
        layout = aser.ASER_CODES_INT4_PACKED if packed else aser.ASER_CODES_INT8
        ctx.check(aser.aser_quantize_rtn(ctx, torch.from_numpy(W).to(DEV), idx, mdiag, spec.f, bits, layout, codes, scales, T))
        torch.cuda.synchronize()
        got = codes.cpu().numpy()
        assert np.array_equal(unpack_int4(got) if packed else got, ref.codes)
        assert np.array_equal(scales.cpu().numpy(), ref.scales)
    X = synth.activations_as_f32(spec, x_np).copy()
    X[3, :] *= np.float32(1e-37)
    X[9, :] = 0.0
    X[9, 5] = np.float32(1e-41)                                  # a single denormal entry: scale 7.8e-44
    ref_codes, ref_scales = orc.quantize_act_rtn(X, sm.mdiag, 8)
    ctx = new_ctx()
    codes = torch.empty((X.shape[0], spec.n), dtype=torch.int8, device=DEV)
    scales = torch.empty(X.shape[0], dtype=torch.float32, device=DEV)
    ctx.check(aser.aser_quantize_act_rtn(ctx, torch.from_numpy(X).to(DEV), mdiag, 8, codes, scales))
    torch.cuda.synchronize()
    assert np.array_equal(codes.cpu().numpy(), ref_codes)
    assert np.array_equal(scales.cpu().numpy(), ref_scales)


def test_ill_conditioned_block_is_reported():
    """W8 with smoothed outlier columns: the unquantized outlier part of T is thousands of times larger
    than the int8 rounding error (sigma_1 / sigma_b = 4400 here).  With a purely random start block every
    column mixes both, which is more than the fp32-class products and the Cholesky-QR orthogonalisation
    resolve: without the outlier set (f = 0) the call must say so (ASER_ERR_NO_CONVERGE) instead of returning
    numbers; all kernels run to completion.  With the outlier set the same layer passes the parity bars
    (test_end_to_end_layer[w8_few_outliers])."""
    spec = synth.mini("fz21", 145, 410, 1105, x_dtype="bf16", x_dist="gauss", n_outliers=3, r=31, f=3, bits=8, seed_id=721)
    W = torch.from_numpy(synth.make_weight(spec)).to(DEV)
    X = to_dev_x(spec, synth.make_activations(spec))
    ctx = new_ctx()
    ctx.set_precision(aser.ASER_PRECISION_FAST)
    buf = aser.LayerBuffers(spec.m, spec.n, spec.r, spec.f, spec.bits, False)
    ctx.ensure_workspace(aser.aser_workspace_bytes(spec.m, spec.n, spec.r))
    ctx.check(aser.aser_gram_accumulate(ctx, X, buf.G, buf.abs_sum, buf.count))
    ctx.check(aser.aser_smooth_outliers(ctx, W, buf.abs_sum, buf.count, buf.f, buf.idx, buf.mdiag))
    ctx.check(aser.aser_quantize_rtn(ctx, W, buf.idx, buf.mdiag, buf.f, buf.bits, aser.ASER_CODES_INT8, buf.codes, buf.scales, buf.T))
    st, info = aser.aser_whiten(ctx, buf.G, buf.mdiag, 0.0, buf.S)
    assert st == aser.ASER_OK and info == 0
    st, _, _ = aser.aser_error_reconstruct(ctx, buf.T, buf.S, buf.r, buf.L_A, buf.L_B, buf.sigma)
    assert st == aser.ASER_ERR_NO_CONVERGE
    st, err, _ = aser.aser_error_reconstruct(ctx, buf.T, buf.S, buf.r, buf.L_A, buf.L_B, buf.sigma, idx=buf.idx, f=spec.f)
    assert st == aser.ASER_OK and np.isfinite(err)


def test_deterministic_integer_outputs():
    spec = synth.mini("d1", 130, 520, 1500, r=16, f=8)
    W = torch.from_numpy(synth.make_weight(spec)).to(DEV)
    X = to_dev_x(spec, synth.make_activations(spec))
    outs = []
    for _ in range(2):
        ctx = new_ctx()
        buf = aser.LayerBuffers(spec.m, spec.n, spec.r, spec.f, spec.bits, True)
        aser.calibrate_layer(ctx, W, X, buf)
        torch.cuda.synchronize()
        outs.append((buf.idx.cpu().numpy().copy(), buf.codes.cpu().numpy().copy(), buf.scales.cpu().numpy().copy()))
    for a, b in zip(outs[0], outs[1]):
        assert np.array_equal(a, b)


def test_c0_against_stored_oracle_results():
    """The HIP path on layer c0 against tests/golden/c0_oracle.json (written from the oracle alone):
    indices, factors, scales and codes exactly, singular values and the whitened error (Eq. 8) to 1e-4."""
    import hashlib
    import json
    import os
    with open(os.path.join(os.path.dirname(os.path.abspath(__file__)), "golden", "c0_oracle.json")) as fh:
        gold = json.load(fh)
    spec = synth.CONFIGS["c0"]
    say("golden c0")
    W = synth.make_weight(spec)
    x_np = synth.make_activations(spec)
    ctx = new_ctx()
    buf = aser.LayerBuffers(spec.m, spec.n, spec.r, spec.f, spec.bits, False)
    Xd = to_dev_x(spec, x_np)
    aser.calibrate_layer(ctx, torch.from_numpy(W).to(DEV), Xd, buf)
    torch.cuda.synchronize()
    idx = buf.idx.cpu().numpy()[:spec.f].tolist()
    assert idx == gold["idx"]
    md = buf.mdiag.cpu().numpy()
    assert [float(md[i]) for i in idx] == gold["mdiag_on_idx"]
    assert [float(s) for s in buf.scales.cpu().numpy()[:8]] == gold["rtn_scales_first8"]
    codes = np.ascontiguousarray(buf.codes.cpu().numpy(), dtype=np.int8)
    assert hashlib.sha256(codes.tobytes()).hexdigest() == gold["rtn_codes_sha256"]
    sig = buf.sigma.cpu().numpy()[:spec.r].astype(np.float64)
    assert np.allclose(sig, gold["sigma_first"][:spec.r], rtol=1e-4)
    assert abs(buf.err - gold["whitened_error"]) <= 1e-4 * gold["whitened_error"]
    act_codes = torch.empty((spec.tokens, spec.n), dtype=torch.int8, device=DEV)
    act_scales = torch.empty(spec.tokens, dtype=torch.float32, device=DEV)
    ctx.check(aser.aser_quantize_act_rtn(ctx, Xd, buf.mdiag, 8, act_codes, act_scales))
    torch.cuda.synchronize()
    assert [float(s) for s in act_scales.cpu().numpy()[:8]] == gold["act_scales_first8"]
    assert hashlib.sha256(np.ascontiguousarray(act_codes.cpu().numpy()).tobytes()).hexdigest() == gold["act_codes_sha256"]
