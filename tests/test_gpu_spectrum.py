"""Full singular spectrum of T S on the device against the oracle's SVD, and what is derived from it:
the rank from the threshold alpha (Eq. 9), the effective rank (Eq. 3-4) and the profiles of the largest
singular values of the weight error and of the whitened error (Sec. 3.2).

Tolerance of a singular value: the device forms T S with products of about 2^-16 relative error per
term with random signs, so ||d(T S)||_2 is about 1e-5 ||T S||_F * 2 / sqrt(min(m, n)), and Weyl's
inequality bounds every |d sigma_i| by that; an isolated large singular value moves by u^T d(T S) v, a
few 1e-6 of itself; everything behind the product is fp64.  Written below as
|d sigma_i| <= 4e-5 ||sigma||_2 / sqrt(k) + 4e-6 sigma_i (measured: at most a third of it).
"""
import numpy as np
import pytest
import torch

import aser_synth as synth
import paper_2411_07762_amd as aser
from oracle import aser_oracle as orc

from gpu_util import DEV, new_ctx
from test_gpu_parity import say

pytestmark = pytest.mark.gpu

PAPER_ALPHAS = (0.1, 0.075, 0.05, 0.03, 0.015)          # the thresholds of the paper's rank table (Sec. 5.3)


def device_spectrum(ctx, T32, S32):
    m, n = T32.shape
    ctx.ensure_workspace(aser.aser_spectrum_workspace_bytes(m, n, S32 is not None))
    Td = torch.from_numpy(T32).to(DEV)
    Sd = torch.from_numpy(S32).to(DEV) if S32 is not None else None
    sig = torch.full((min(m, n),), -1.0, dtype=torch.float64, device=DEV)
    ctx.check(aser.aser_singular_values(ctx, Td, Sd, sig))
    torch.cuda.synchronize()
    return sig


def check_spectrum(label, sig_dev, ref):
    got = sig_dev.cpu().numpy()
    k = ref.shape[0]
    tol = 4e-5 * np.linalg.norm(ref) / np.sqrt(k) + 4e-6 * ref
    ratio = np.abs(got - ref) / tol
    worst = float(ratio.max())
    say("%s: k=%d worst singular value (index %d) at %.3f of its tolerance; sum rel %.2e" %
        (label, k, int(ratio.argmax()), worst, abs(got.sum() - ref.sum()) / ref.sum()))
    assert np.all(np.diff(got) <= 0) and got.min() >= 0
    assert worst <= 1.0
    return got


def check_rank_rule(ctx, label, sig_dev, ref):
    """Eq. 9 against oracle.rank_from_alpha: at the paper's thresholds and at thresholds placed half way
    between two consecutive cumulative shares of the oracle's spectrum (the widest margin a decision at
    that rank can have); the rank must agree whenever the oracle's margin exceeds 2e-5 of the sum."""
    share = np.cumsum(ref) / np.sum(ref)
    targets = sorted({1, 2, 5, 16, 17, 40, 64, 100, min(128, len(ref) - 2)} & set(range(1, len(ref) - 1)))
    alphas = list(PAPER_ALPHAS) + [0.5 * (share[r - 1] + share[r]) for r in targets] + [0.5, 0.9]
    agreed = 0
    for alpha in alphas:
        want = orc.rank_from_alpha(ref, alpha)
        margin = min(abs(alpha - share[want - 1]), abs(share[min(want, len(ref) - 1)] - alpha))
        st, r, (total, lo, hi) = aser.aser_select_rank(ctx, sig_dev, alpha)
        ctx.check(st)
        say("%s: alpha=%.6f rank oracle %d device %d (shares %.6f < alpha <= %.6f, oracle margin %.2e)" %
            (label, alpha, want, r, lo, hi, margin))
        assert abs(total - ref.sum()) <= 2e-5 * ref.sum()
        if want > 1 or share[0] < alpha:
            assert lo < alpha <= hi
        if margin > 2e-5:
            assert r == want
            agreed += 1
        else:
            assert abs(r - want) <= 1
    assert agreed >= len(alphas) - 2


def layer_targets(spec):
    W = synth.make_weight(spec)
    X = synth.activations_as_f32(spec, synth.make_activations(spec))
    G, abs_sum, cnt = orc.gram(X)
    sm = orc.smooth_outliers(W, abs_sum, cnt, spec.f)
    qz = orc.quantize_rtn(W, sm.idx, sm.mdiag, spec.bits)
    S = orc.whiten(G, sm.mdiag)
    return qz.T.astype(np.float32), S.astype(np.float32)


CASES = [
    ("c0", synth.CONFIGS["c0"]),
    ("wide_ragged", synth.mini("sp1", 150, 333, 1200, r=24, f=6)),
    ("tall_ragged", synth.mini("sp2", 601, 260, 1024, r=32, f=8, x_dist="silu_prod", out=(40.0, 40.0))),
    ("tiny", synth.mini("sp3", 3, 40, 128, r=2, f=2)),
    ("c1_shape_small", synth.CONFIGS["c1"].with_(m=768, n=1024, tokens=4096, r=32, f=16)),
]


@pytest.mark.parametrize("name,spec", CASES, ids=[c[0] for c in CASES])
def test_singular_values_rank_rule_and_effective_rank(name, spec):
    say("spectrum case %s m=%d n=%d" % (name, spec.m, spec.n))
    T32, S32 = layer_targets(spec)
    ctx = new_ctx()
    for label, Sx in ((name + " T S", S32), (name + " T", None)):
        ref = orc.singular_values(T32, Sx)
        sig_dev = device_spectrum(ctx, T32, Sx)
        got = check_spectrum(label, sig_dev, ref)
        if len(ref) > 4:
            check_rank_rule(ctx, label, sig_dev, ref)
        for eps in (1e-12, 0.0):
            st, er = aser.aser_effective_rank(ctx, sig_dev, eps)
            ctx.check(st)
            want = orc.effective_rank(ref, eps) if eps or ref.min() > 0 else orc.effective_rank(ref[ref > 0], 0.0)
            say("%s: effective rank device %.6f oracle %.6f" % (label, er, want))
            assert abs(er - want) <= 1e-4 * want
        prof = orc.normalized_profile(ref, 128)
        assert np.allclose(got[:len(prof)] / got[0], prof, rtol=0, atol=2e-5)


def test_headline_layer_spectrum_full_size():
    """The 4096 x 4096 layer of the bench: all 4096 singular values of T S, the rank the paper's
    thresholds select, the effective rank of the weight error against that of the whitened error."""
    spec = synth.CONFIGS["c1"]
    say("spectrum c1 full size")
    T32, S32 = layer_targets(spec)
    ctx = new_ctx()
    ref = orc.singular_values(T32, S32)
    sig_dev = device_spectrum(ctx, T32, S32)
    check_spectrum("c1 T S", sig_dev, ref)
    check_rank_rule(ctx, "c1 T S", sig_dev, ref)
    st, er = aser.aser_effective_rank(ctx, sig_dev)
    ctx.check(st)
    assert abs(er - orc.effective_rank(ref)) <= 1e-4 * er
    ref_w = orc.singular_values(T32, None)
    sig_w = device_spectrum(ctx, T32, None)
    check_spectrum("c1 T", sig_w, ref_w)
    st, er_w = aser.aser_effective_rank(ctx, sig_w)
    ctx.check(st)
    say("c1: effective rank of T %.1f, of T S %.1f" % (er_w, er))
    assert abs(er_w - orc.effective_rank(ref_w)) <= 1e-4 * er_w


def test_spectrum_of_known_matrices():
    """Matrices whose singular values are known in closed form: a diagonal matrix, an orthogonal
    projector of rank 3 (three ones, the rest zero), and a rank-one matrix."""
    ctx = new_ctx()
    dvals = np.array([9.0, -7.5, 4.0, 2.5, 1.0, 0.5, 0.25, 0.0], dtype=np.float32)
    sig = device_spectrum(ctx, np.diag(dvals), None).cpu().numpy()
    assert np.allclose(sig, np.sort(np.abs(dvals))[::-1], rtol=1e-7, atol=1e-7)
    rng = np.random.default_rng(3)
    Q, _ = np.linalg.qr(rng.standard_normal((40, 3)))
    sig = device_spectrum(ctx, (Q @ Q.T).astype(np.float32), None).cpu().numpy()
    assert np.allclose(sig[:3], 1.0, atol=1e-6) and np.all(sig[3:] < 1e-6)
    u, v = rng.standard_normal(50), rng.standard_normal(20)
    sig = device_spectrum(ctx, np.outer(u, v).astype(np.float32), None).cpu().numpy()
    assert abs(sig[0] - np.linalg.norm(u) * np.linalg.norm(v)) < 1e-5 * sig[0] and np.all(sig[1:] < 1e-5 * sig[0])
    st, er = aser.aser_effective_rank(ctx, torch.from_numpy(np.full(7, 2.5)).to(DEV), 0.0)
    assert st == aser.ASER_OK and abs(er - 7.0) < 1e-12
