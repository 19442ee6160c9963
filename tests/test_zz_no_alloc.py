"""The allocation-free variant of the smoothing stage against the workspace-based entry point, through
the C ABI: same outlier set, smoothing diagonal, W_o and scores, on two calls in a row that share the
static scratch (the second on a smaller layer, so stale contents of the first lie behind its data)."""
import numpy as np
import pytest
import torch

import aser_synth as synth
import paper_2411_07762_amd as aser

pytestmark = pytest.mark.gpu
DEV = "cuda:0"


def _inputs(spec):
    W = synth.make_weight(spec)
    X = synth.activations_as_f32(spec, synth.make_activations(spec))
    abs_sum = np.abs(X.astype(np.float64)).sum(axis=0)            # input of the stage, not part of the method
    return (torch.from_numpy(W).to(DEV), torch.from_numpy(abs_sum).to(DEV),
            torch.tensor([spec.tokens], dtype=torch.int64, device=DEV))


def _run(fn, ctx, spec, W, abs_sum, count):
    idx = torch.full((spec.f,), -7, dtype=torch.int32, device=DEV)
    mdiag = torch.full((spec.n,), -1.0, dtype=torch.float32, device=DEV)
    W_o = torch.full((spec.m, spec.f), -1.0, dtype=torch.float32, device=DEV)
    score = torch.full((spec.n,), -1.0, dtype=torch.float64, device=DEV)
    ctx.check(fn(ctx, W, abs_sum, count, spec.f, idx, mdiag, W_o, score))
    torch.cuda.synchronize()
    return [t.cpu().numpy() for t in (idx, mdiag, W_o, score)]


def test_noalloc_smoothing_matches_the_workspace_entry_point():
    big = synth.mini("na1", 96, 2500, 640, f=32, n_outliers=16, seed_id=941)
    small = synth.mini("na2", 40, 333, 300, f=7, seed_id=942)
    ref_ctx = aser.Context(0)
    ref_ctx.ensure_workspace(aser.aser_workspace_bytes(big.m, big.n, 0))
    ctx = aser.Context(0)                                          # never gets a workspace
    for spec in (big, small):
        print("no-alloc smoothing case m=%d n=%d f=%d" % (spec.m, spec.n, spec.f), flush=True)
        W, abs_sum, count = _inputs(spec)
        want = _run(aser.aser_smooth_outliers, ref_ctx, spec, W, abs_sum, count)
        got = _run(aser.aser_smooth_outliers_noalloc, ctx, spec, W, abs_sum, count)
        for name, a, b in zip(("idx", "mdiag", "W_o", "score"), want, got):
            assert np.array_equal(a, b), name
        assert want[0].min() >= 0
    # without a score buffer the scores go to the static array as well
    W, abs_sum, count = _inputs(small)
    idx = torch.zeros(small.f, dtype=torch.int32, device=DEV)
    mdiag = torch.empty(small.n, dtype=torch.float32, device=DEV)
    ctx.check(aser.aser_smooth_outliers_noalloc(ctx, W, abs_sum, count, small.f, idx, mdiag))
    torch.cuda.synchronize()
    assert np.array_equal(idx.cpu().numpy(), want[0]) and np.array_equal(mdiag.cpu().numpy(), want[1])
    # sizes beyond the static array are refused before anything is launched
    st = aser.aser_smooth_outliers_noalloc(ctx, W, abs_sum, count, 4, idx, mdiag, m=8, n=40000, ldw=40000)
    assert st == aser.ASER_ERR_SHAPE
