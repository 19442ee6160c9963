"""Pins for the CPU oracle: what the paper and linear algebra fix, independent of the oracle.

Each test is chosen so that a plausible mistake in oracle/aser_oracle.py (a dropped term, a
transposed factor, a wrong rounding mode, a wrong axis) makes it fail.
"""
import numpy as np
import pytest
import scipy.linalg as sla
import scipy.optimize as sopt

import aser_synth as synth
from oracle import aser_oracle as orc


def _small_layer(seed=0, m=24, n=16, N=80, f=3, r=4, bits=4):
    rng = np.random.default_rng(seed)
    W = (rng.standard_normal((m, n)) * 0.02).astype(np.float32)
    X = rng.standard_normal((N, n)).astype(np.float32)
    X[:, [1, 7]] *= 25.0
    return W, X, bits, f, r


# ---------------------------------------------------------------- Gram (Eq. 5)
def test_gram_matches_triple_loop_and_invariants():
    rng = np.random.default_rng(1)
    X = rng.standard_normal((13, 5)).astype(np.float32)
    G, abs_sum, cnt = orc.gram(X, chunk=4)
    ref = np.zeros((5, 5))
    for t in range(13):
        for i in range(5):
            for j in range(5):
                ref[i, j] += float(X[t, i]) * float(X[t, j])
    assert np.allclose(G, ref, rtol=1e-14, atol=1e-14)
    assert np.array_equal(G, G.T)
    assert np.allclose(np.diag(G), (X.astype(np.float64) ** 2).sum(0))
    assert np.allclose(abs_sum, [sum(abs(float(X[t, i])) for t in range(13)) for i in range(5)])
    assert cnt == 13
    G2, a2, _ = orc.gram(X[::-1], chunk=7)          # token order / chunking do not matter
    assert np.allclose(G, G2, rtol=1e-13) and np.allclose(abs_sum, a2, rtol=1e-13)


# ---------------------------------------------------------------- smoothing (Eq. 10, Eq. 11)
def test_smoothing_hand_example_and_tie_break():
    # 2 output rows, 5 channels.  |W| column means: [1, 2, 0.5, 2, 1];  X-bar: [4, 1, 8, 1, 0.5]
    W = np.array([[1, -2, 0.5, 2, 1], [-1, 2, -0.5, -2, 1]], dtype=np.float32)
    abs_sum = np.array([8, 2, 16, 2, 1], dtype=np.float64)          # over 2 tokens
    sm = orc.smooth_outliers(W, abs_sum, 2, 3)
    assert np.allclose(sm.xbar, [4, 1, 8, 1, 0.5]) and np.allclose(sm.wbar, [1, 2, 0.5, 2, 1])
    assert np.allclose(sm.score, [4, 2, 4, 2, 0.5])
    # scores 4,4 tie -> channel 0 before 2; then 2,2 tie -> channel 1 (lower index) wins over 3
    assert sm.idx.tolist() == [0, 2, 1]
    # X-bar over I_f = {4, 8, 1}: min is 1 -> m = [4, 1, 8, 1, 1]
    assert sm.mdiag.tolist() == [4.0, 1.0, 8.0, 1.0, 1.0]
    assert np.allclose(sm.W_o, W[:, [0, 2, 1]].astype(np.float64) * np.array([4.0, 8.0, 1.0]))
    sm0 = orc.smooth_outliers(W, abs_sum, 2, 0)                      # w/o A.S. branch of Alg. 1
    assert sm0.idx.size == 0 and np.all(sm0.mdiag == 1.0)


def test_smoothing_invariants_and_exact_refactoring():
    W, X, bits, f, r = _small_layer(3)
    G, abs_sum, cnt = orc.gram(X)
    sm = orc.smooth_outliers(W, abs_sum, cnt, f)
    m = sm.mdiag.astype(np.float64)
    assert np.isclose(m[sm.idx].min(), 1.0) and np.all(m >= 1.0)
    off = np.setdiff1d(np.arange(W.shape[1]), sm.idx)
    assert np.all(m[off] == 1.0)
    assert {1, 7} <= set(sm.idx.tolist())                         # planted channels are found
    # Eq. 10: W X = (W M)(M^-1 X) exactly (up to fp64 rounding)
    Wd, Xd = W.astype(np.float64), X.astype(np.float64)
    lhs = Wd @ Xd.T
    rhs = (Wd * m[None, :]) @ (Xd / m[None, :]).T
    assert np.allclose(lhs, rhs, rtol=1e-12, atol=1e-12)
    # scores are means of absolute values, not absolute values of means
    assert np.allclose(sm.xbar, np.abs(Xd).mean(0)) and np.allclose(sm.wbar, np.abs(Wd).mean(0))


def test_c0_planted_channels_selected():
    spec = synth.CONFIGS["c0"]
    W = synth.make_weight(spec)
    X = synth.make_activations(spec)
    G, abs_sum, cnt = orc.gram(X)
    sm = orc.smooth_outliers(W, abs_sum, cnt, spec.f)
    assert {3, 77, 190} <= set(sm.idx.tolist())
    assert sm.margin > 1e-9


# ---------------------------------------------------------------- RTN (Sec. 3, Eq. 12)
def test_rtn_hand_example_half_to_even_and_packing():
    # row max 7/8 -> scale exactly 1/8; quotients 7, -3.5, 1.5, 2.5, 0.5, -0.5 pin half-to-even
    W = (np.array([[7, -3.5, 1.5, 2.5, 0.5, -0.5], [0, 0, 0, 0, 0, 0], [1, -7, 3.4, -3.6, 6.5, 5.5]])
         / 8.0).astype(np.float32)
    idx = np.zeros(0, dtype=np.int32)
    q = orc.quantize_rtn(W, idx, np.ones(6, np.float32), 4)
    assert q.codes.tolist() == [[7, -4, 2, 2, 0, 0], [0] * 6, [1, -7, 3, -4, 6, 6]]
    assert q.scales.tolist() == [0.125, 1.0, 0.125]
    assert np.allclose(q.T[0], np.array([0, 0.5, -0.5, 0.5, 0.5, -0.5]) / 8.0)
    packed = orc.pack_int4(q.codes)
    # low nibble = even column, two's complement: (7, -4) -> 0xC7 ; (2, 2) -> 0x22 ; (0,0) -> 0
    assert packed[0].tolist() == [0xC7, 0x22, 0x00]
    assert packed[2].tolist() == [0x91, 0xC3, 0x66]
    q8 = orc.quantize_rtn((np.array([[127, -63.5, 0.5, 1.5]]) / 64.0).astype(np.float32), idx,
                          np.ones(4, np.float32), 8)
    assert q8.codes.tolist() == [[127, -64, 0, 2]] and q8.scales.tolist() == [1.0 / 64.0]


def test_rtn_outlier_columns_and_eq12_split():
    W, X, bits, f, r = _small_layer(5, m=40, n=32)
    G, abs_sum, cnt = orc.gram(X)
    sm = orc.smooth_outliers(W, abs_sum, cnt, f)
    q = orc.quantize_rtn(W, sm.idx, sm.mdiag, bits)
    qmax = 7
    assert np.all(q.codes[:, sm.idx] == 0)                               # W_o is not quantized
    assert np.abs(q.codes).max() == qmax and np.all(np.abs(q.codes).max(axis=1) == qmax)
    off = np.setdiff1d(np.arange(W.shape[1]), sm.idx)
    assert np.all(np.abs(q.T[:, off]) <= q.scales[:, None].astype(np.float64) * 0.5 * (1 + 1e-6))
    # scale comes from W_s (outlier columns excluded), not from W or W M
    Ws = W.copy(); Ws[:, sm.idx] = 0
    assert np.array_equal(q.scales, (np.abs(Ws).max(1) / np.float32(7)).astype(np.float32))
    # Eq. 12: W M = Q(W_s) + (E_q + W_o)
    WM = W.astype(np.float64) * sm.mdiag.astype(np.float64)[None, :]
    assert np.allclose(orc.dequantize(q.codes, q.scales) + q.T, WM, rtol=0, atol=1e-15)
    assert np.allclose(q.T[:, sm.idx], sm.W_o, rtol=0, atol=1e-15)
    # f = 0 reduces to E = W - Q(W)
    q0 = orc.quantize_rtn(W, np.zeros(0, np.int32), np.ones(W.shape[1], np.float32), bits)
    assert np.allclose(q0.T, W.astype(np.float64) - orc.dequantize(q0.codes, q0.scales), atol=1e-15)


def test_act_rtn_hand_example():
    X = np.array([[127, -254, 1.0, 3.0], [0, 0, 0, 0]], dtype=np.float32)
    mdiag = np.array([1, 2, 1, 2], dtype=np.float32)               # X' = [127, -127, 1, 1.5]
    codes, scales = orc.quantize_act_rtn(X, mdiag, 8)
    assert codes.tolist() == [[127, -127, 1, 2], [0, 0, 0, 0]]
    assert scales.tolist() == [1.0, 1.0]


def test_act_rtn_ties_round_half_to_even():
    """Quotients exactly half way between two codes go to the even one: 0.5 -> 0, 2.5 -> 2, -3.5 -> -4,
    -0.5 -> 0, 6.5 -> 6 (half away from zero would give 1, 3, -4, -1, 7; truncation 0, 2, -3, 0, 6).
    Token 1 has a scale that is not 1 (absmax 63.5 at 6 bits: scale 63.5 / 31 is inexact, so its ties
    are made with scale 2: absmax 62), token 2 reaches its ties through the division by M."""
    X = np.array([[127.0, 0.5, 2.5, -3.5, -0.5, 6.5],
                  [62.0, 1.0, 5.0, -7.0, -1.0, 13.0],
                  [254.0, 1.0, 5.0, -7.0, 3.0, 39.0]], dtype=np.float32)
    codes, scales = orc.quantize_act_rtn(X[:1], np.ones(6, np.float32), 8)
    assert scales.tolist() == [1.0] and codes.tolist() == [[127, 0, 2, -4, 0, 6]]
    codes, scales = orc.quantize_act_rtn(X[1:2], np.ones(6, np.float32), 6)       # qmax 31, scale 2
    assert scales.tolist() == [2.0] and codes.tolist() == [[31, 0, 2, -4, 0, 6]]
    mdiag = np.array([2, 2, 2, 2, 2, 6], dtype=np.float32)                        # X' = [127, .5, 2.5, -3.5, 1.5, 6.5]
    codes, scales = orc.quantize_act_rtn(X[2:], mdiag, 8)
    assert scales.tolist() == [1.0] and codes.tolist() == [[127, 0, 2, -4, 2, 6]]


# ---------------------------------------------------------------- whitening (Eq. 5)
def test_whitening_identity_and_uniqueness():
    W, X, bits, f, r = _small_layer(7)
    G, abs_sum, cnt = orc.gram(X)
    sm = orc.smooth_outliers(W, abs_sum, cnt, f)
    S = orc.whiten(G, sm.mdiag)
    assert np.allclose(S, np.tril(S)) and np.all(np.diag(S) > 0)
    Xp = X.astype(np.float64) / sm.mdiag.astype(np.float64)[None, :]      # rows are (M^-1 x)^T
    Z = sla.solve_triangular(S, Xp.T, lower=True)                          # S^-1 M^-1 X
    assert np.allclose(Z @ Z.T, np.eye(S.shape[0]), atol=1e-9)
    assert np.allclose(S @ S.T, Xp.T @ Xp, rtol=1e-12)
    Sd = orc.whiten(G, None, damp=0.5)
    assert np.allclose(Sd @ Sd.T, G + 0.5 * np.mean(np.diag(G)) * np.eye(G.shape[0]), rtol=1e-12)


# ---------------------------------------------------------------- whitened SVD (Eq. 6 - Eq. 8)
def _layer_pieces(seed, **kw):
    W, X, bits, f, r = _small_layer(seed, **kw)
    res = orc.calibrate_layer(W, X, bits, f, r)
    return W, X, res, r


def test_eq8_identity_three_ways():
    W, X, res, r = _layer_pieces(11)
    T, S, rec, m = res.quant.T, res.S, res.rec, res.smooth.mdiag.astype(np.float64)
    P = rec.L_A @ rec.L_B
    Xp = X.astype(np.float64) / m[None, :]
    e_explicit = np.linalg.norm((T - P) @ Xp.T)                    # ||(T - L_A L_B) M^-1 X||_F
    U, s, Vt = np.linalg.svd(T @ S, full_matrices=False)
    e_whitened = np.linalg.norm(T @ S - (U[:, :r] * s[:r]) @ Vt[:r])
    e_tail = np.sqrt((s[r:] ** 2).sum())
    assert np.isclose(e_explicit, e_whitened, rtol=1e-9)
    assert np.isclose(e_whitened, e_tail, rtol=1e-9)
    assert np.isclose(rec.err, e_tail, rtol=1e-12)
    assert np.isclose(orc.whitened_error(T, S, rec.L_A, rec.L_B), e_explicit, rtol=1e-9)
    # single truncated value: L_i = sigma_i (Eq. 8)
    i = 2
    Ei = s[i] * np.outer(U[:, i], Vt[i]) @ np.linalg.inv(S)
    assert np.isclose(np.linalg.norm(Ei @ Xp.T), s[i], rtol=1e-8)
    # the uncompensated loss ||T M^-1 X|| equals err0
    assert np.isclose(np.linalg.norm(T @ Xp.T), rec.err0, rtol=1e-9)


def test_factor_definitions():
    W, X, res, r = _layer_pieces(12)
    T, S, rec = res.quant.T, res.S, res.rec
    U, s, Vt = np.linalg.svd(T @ S, full_matrices=False)
    assert np.allclose(rec.sigma, s)
    assert rec.L_A.shape == (T.shape[0], r) and rec.L_B.shape == (r, T.shape[1])
    # L_A = U_r Sigma_r: columns orthogonal with norms sigma_i ; L_B S = V_r^T: orthonormal rows
    assert np.allclose(rec.L_A.T @ rec.L_A, np.diag(s[:r] ** 2), atol=1e-9 * s[0] ** 2)
    LBS = rec.L_B @ S
    assert np.allclose(LBS @ LBS.T, np.eye(r), atol=1e-9)
    assert np.allclose(rec.L_A @ LBS, (U[:, :r] * s[:r]) @ Vt[:r], atol=1e-9 * s[0])


def test_closed_form_without_S_and_sqrt_invariance():
    W, X, res, r = _layer_pieces(13)
    T, S, rec = res.quant.T, res.S, res.rec
    P = rec.L_A @ rec.L_B
    Gp = S @ S.T
    lam, vec = np.linalg.eigh(T @ Gp @ T.T)
    Ur = vec[:, ::-1][:, :r]
    assert np.allclose(np.sqrt(lam[::-1][:r]), rec.sigma[:r], rtol=1e-9)
    assert np.allclose(Ur @ Ur.T @ T, P, atol=1e-9 * np.abs(P).max())
    # any square root of G' gives the same sigma and the same product
    w, V = np.linalg.eigh(Gp)
    S_sym = (V * np.sqrt(w)) @ V.T
    rng = np.random.default_rng(0)
    Qr, _ = np.linalg.qr(rng.standard_normal(S.shape))
    for S2 in (S_sym, S @ Qr):
        A2 = T @ S2
        U2, s2, Vt2 = np.linalg.svd(A2, full_matrices=False)
        P2 = (U2[:, :r] * s2[:r]) @ Vt2[:r] @ np.linalg.inv(S2)
        assert np.allclose(s2, rec.sigma, rtol=1e-9)
        assert np.allclose(P2, P, atol=1e-8 * np.abs(P).max())


def test_identity_gram_reduces_to_plain_svd():
    rng = np.random.default_rng(21)
    T = rng.standard_normal((9, 6))
    rec = orc.error_reconstruct(T, np.eye(6), 2)
    U, s, Vt = np.linalg.svd(T, full_matrices=False)
    assert np.allclose(rec.L_A @ rec.L_B, (U[:, :2] * s[:2]) @ Vt[:2], atol=1e-12)
    assert np.isclose(rec.gap, s[1] / s[2])


def test_monotone_in_r_and_zero_at_full_rank():
    W, X, res, _ = _layer_pieces(14, m=12, n=10, N=60, f=2)
    T, S = res.quant.T, res.S
    errs = []
    for r in range(1, 11):
        rec = orc.error_reconstruct(T, S, r)
        errs.append(orc.whitened_error(T, S, rec.L_A, rec.L_B))
        assert np.isclose(errs[-1], rec.err, rtol=1e-7, atol=1e-9 * rec.err0)
    assert all(a >= b - 1e-12 for a, b in zip(errs, errs[1:]))
    assert errs[-1] <= 1e-9 * res.rec.err0
    assert errs[0] < res.rec.err0


@pytest.mark.parametrize("m,n,r,seed", [(3, 3, 1, 0), (4, 5, 2, 1), (5, 4, 1, 2), (4, 4, 3, 3)])
def test_eckart_young_brute_force(m, n, r, seed):
    """No rank-r matrix found by a free search beats the oracle's whitened loss."""
    rng = np.random.default_rng(100 + seed)
    T = rng.standard_normal((m, n))
    Xs = rng.standard_normal((3 * n, n)) * rng.uniform(0.2, 5.0, size=n)[None, :]
    S = orc.whiten(Xs.T @ Xs)
    rec = orc.error_reconstruct(T, S, r)
    best_oracle = orc.whitened_error(T, S, rec.L_A, rec.L_B)

    def loss(p):
        A = p[:m * r].reshape(m, r)
        B = p[m * r:].reshape(r, n)
        R = (T - A @ B) @ S
        g = -2.0 * R @ S.T
        return (R ** 2).sum(), np.concatenate([(g @ B.T).ravel(), (A.T @ g).ravel()])

    best = np.inf
    for k in range(24):
        p0 = rng.standard_normal(m * r + r * n) * (0.1 if k % 2 else 1.0)
        out = sopt.minimize(loss, p0, jac=True, method="L-BFGS-B", options={"maxiter": 2000, "ftol": 1e-15, "gtol": 1e-12})
        best = min(best, np.sqrt(out.fun))
    assert best >= best_oracle * (1 - 1e-7)          # nothing beats it
    assert best <= best_oracle * (1 + 1e-4)          # and the search does reach it
    # a plain (unwhitened) truncated SVD of T is a rank-r candidate too, and is not better
    U, s, Vt = np.linalg.svd(T, full_matrices=False)
    P_plain = (U[:, :r] * s[:r]) @ Vt[:r]
    assert np.linalg.norm((T - P_plain) @ S) >= best_oracle * (1 - 1e-12)


def test_planted_mistakes_are_caught():
    """The pins above are sensitive: typical slips change the pinned quantities."""
    W, X, res, r = _layer_pieces(15)
    T, S, rec, m = res.quant.T, res.S, res.rec, res.smooth.mdiag.astype(np.float64)
    Xp = X.astype(np.float64) / m[None, :]
    good = np.linalg.norm((T - rec.L_A @ rec.L_B) @ Xp.T)
    # upper instead of lower factor in the product T S
    U, s, Vt = np.linalg.svd(T @ S.T, full_matrices=False)
    P_bad = (U[:, :r] * s[:r]) @ Vt[:r] @ np.linalg.inv(S.T)
    assert np.linalg.norm((T - P_bad) @ Xp.T) > good * (1 + 1e-6)
    # whitening with G instead of M^-1 G M^-1
    S_bad = np.linalg.cholesky(res.G)
    rb = orc.error_reconstruct(T, S_bad, r)
    assert np.linalg.norm((T - rb.L_A @ rb.L_B) @ Xp.T) > good * (1 + 1e-6)
    # dropping W_o from the target
    T_bad = T.copy(); T_bad[:, res.smooth.idx] = 0
    rb = orc.error_reconstruct(T_bad, S, r)
    assert np.linalg.norm((T - rb.L_A @ rb.L_B) @ Xp.T) > good * (1 + 1e-6)


def test_rank_from_alpha_hand_example():
    sig = np.array([5.0, 3.0, 1.0, 1.0])          # cumulative ratios 0.5, 0.8, 0.9, 1.0
    assert orc.rank_from_alpha(sig, 0.85) == 2
    assert orc.rank_from_alpha(sig, 0.8) == 1     # strict inequality (Eq. 9)
    assert orc.rank_from_alpha(sig, 0.1) == 1     # clamped to at least one
    assert orc.rank_from_alpha(sig, 0.95) == 3


def test_rank_from_alpha_follows_the_cumulative_ratio_by_brute_force():
    rng = np.random.default_rng(11)
    for _ in range(20):
        sig = np.sort(rng.gamma(0.7, size=rng.integers(3, 40)))[::-1]
        alpha = float(rng.uniform(0.05, 0.999))
        want = 0
        for r in range(1, len(sig) + 1):                 # Eq. 9 read literally: the largest r whose ratio stays below alpha
            if sum(sig[:r]) / sum(sig) < alpha:
                want = r
        assert orc.rank_from_alpha(sig, alpha) == max(1, want)


# ---------------------------------------------------------------- spectrum and effective rank (Eq. 3, Eq. 4)
def test_singular_values_against_the_gram_eigenvalues_and_eq6():
    W, X, bits, f, r = _small_layer(21, m=18, n=12, N=60)
    res = orc.calibrate_layer(W, X, bits, f, r)
    sig = orc.singular_values(res.quant.T, res.S)
    assert sig.shape == (12,) and np.all(np.diff(sig) <= 0)
    # sigma_i^2 are the eigenvalues of (T S)(T S)^T = T G' T^T: no S, no SVD on this side
    minv = 1.0 / res.smooth.mdiag.astype(np.float64)
    Gp = res.G * minv[:, None] * minv[None, :]
    lam = np.sort(np.linalg.eigvalsh(res.quant.T @ Gp @ res.quant.T.T))[::-1][:12]
    assert np.allclose(sig ** 2, lam, rtol=1e-9, atol=1e-12 * lam[0])
    assert np.allclose(sig, res.rec.sigma, rtol=1e-12)
    # without S: the spectrum of the weight error alone; a diagonal matrix returns its entries
    assert np.allclose(orc.singular_values(np.diag([3.0, -5.0, 1.0])), [5.0, 3.0, 1.0])
    assert np.isclose(np.linalg.norm(res.quant.T), np.sqrt((orc.singular_values(res.quant.T) ** 2).sum()))


def test_effective_rank_closed_forms():
    # k equal singular values: entropy ln k, effective rank k; rank one: 1
    assert orc.effective_rank(np.full(7, 2.5), eps=0.0) == pytest.approx(7.0, rel=1e-12)
    assert orc.effective_rank(np.array([4.0]), eps=0.0) == pytest.approx(1.0, rel=1e-12)
    assert orc.effective_rank(np.array([4.0, 0.0, 0.0])) == pytest.approx(1.0, abs=1e-9)     # eps keeps ln finite
    # two values 3 : 1 -> p = (3/4, 1/4), entropy 2 ln 2 - (3/4) ln 3, exp of it = 4 / 3^(3/4)
    assert orc.effective_rank(np.array([3.0, 1.0]), eps=0.0) == pytest.approx(4.0 / 3.0 ** 0.75, rel=1e-12)
    sig = np.array([9.0, 4.0, 2.0, 1.0, 0.5])
    assert orc.effective_rank(sig) == pytest.approx(orc.effective_rank(17.0 * sig[::-1]), rel=1e-10)   # scale, order
    assert 1.0 < orc.effective_rank(sig) < 5.0
    # the printed definition adds eps to every p_k (no renormalisation): with a large eps it shows
    p = sig / sig.sum() + 0.01
    assert orc.effective_rank(sig, eps=0.01) == pytest.approx(float(np.exp(-(p * np.log(p)).sum())), rel=1e-12)
    # whitening concentrates the spectrum of a layer with outlier channels (Sec. 3.2: E_q X is more low-rank than E_q)
    W, X, bits, f, r = _small_layer(22, m=40, n=32, N=200, f=0)
    res = orc.calibrate_layer(W, X, bits, 0, 4)
    assert orc.effective_rank(orc.singular_values(res.quant.T, res.S)) < orc.effective_rank(orc.singular_values(res.quant.T))
    prof = orc.normalized_profile(orc.singular_values(res.quant.T, res.S), 8)
    assert prof[0] == 1.0 and prof.shape == (8,) and np.all(np.diff(prof) <= 0)


def test_overhead_ratio_reproduces_the_papers_rank_table():
    """tests/golden/paper_rank_overhead.txt holds the rows the paper prints (Sec. 5.3, rank selection
    table: alpha, mean rank, extra FLOPs for d = 4096); the extra FLOPs are 2 r / d."""
    import os
    path = os.path.join(os.path.dirname(os.path.abspath(__file__)), "golden", "paper_rank_overhead.txt")
    rows = [ln.split() for ln in open(path) if ln.strip() and not ln.startswith("#")]
    assert len(rows) == 5
    for alpha, rbar, pct in rows:
        assert round(100.0 * orc.overhead_flops_ratio(float(rbar), 4096), 2) == float(pct), (alpha, rbar, pct)
    s, d, r = 2048, 4096, 64
    assert orc.overhead_flops_ratio(r, d) == pytest.approx((s * d * d + 2 * s * r * d) / (s * d * d) - 1.0)


# ---------------------------------------------------------------- compensated layer (end of Sec. 4.2, Sec. 5.3)
def test_compensated_forward_by_loops_and_error_identities():
    W, X, bits, f, r = _small_layer(23, m=10, n=8, N=30, f=2, r=3)
    res = orc.calibrate_layer(W, X, bits, f, r)
    md = res.smooth.mdiag
    q, s = orc.quantize_act_rtn(X[:5], md, 8)
    Y = orc.compensated_forward(X[:5], md, res.quant.codes, res.quant.scales, res.rec.L_A, res.rec.L_B, 8)
    ref = np.zeros((5, 10))
    for t in range(5):
        for o in range(10):
            acc = 0.0
            for i in range(8):
                w = float(res.quant.codes[o, i]) * float(res.quant.scales[o])
                for k in range(3):
                    w += res.rec.L_A[o, k] * res.rec.L_B[k, i]
                acc += float(q[t, i]) * float(s[t]) * w
            ref[t, o] = acc
    assert np.allclose(Y, ref, rtol=1e-12, atol=1e-14)
    # without activation quantization, over the calibration set itself, the output error is the whitened
    # error of Eq. 8 (X'^T X' = S S^T), and without compensation it is ||T S||_F
    e, ynorm = orc.layer_output_error(W, X, md, res.quant.codes, res.quant.scales, res.rec.L_A, res.rec.L_B, None)
    assert e == pytest.approx(res.rec.err, rel=1e-9)
    assert ynorm == pytest.approx(np.linalg.norm(X.astype(np.float64) @ W.astype(np.float64).T), rel=1e-12)
    e0, _ = orc.layer_output_error(W, X, md, res.quant.codes, res.quant.scales, None, None, None)
    assert e0 == pytest.approx(res.rec.err0, rel=1e-9) and e < e0
    # with activation quantization the error moves by at most ||dX W~^T||_F, dX the rounding of X' (|dX| <= s_t / 2)
    e8, _ = orc.layer_output_error(W, X, md, res.quant.codes, res.quant.scales, res.rec.L_A, res.rec.L_B, 8)
    q, s = orc.quantize_act_rtn(X, md, 8)
    Wt = orc.compensated_weight(res.quant.codes, res.quant.scales, res.rec.L_A, res.rec.L_B)
    bound = np.sqrt((X.shape[1] * (s.astype(np.float64) / 2) ** 2).sum()) * np.linalg.norm(Wt, 2)
    assert abs(e8 - e) <= bound and e8 != e
    e4, _ = orc.layer_output_error(W, X, md, res.quant.codes, res.quant.scales, res.rec.L_A, res.rec.L_B, 4)
    assert e4 > e8                                             # coarser activations, larger error
    # the smoothing diagonal belongs to the forward pass: dropping it changes the output
    Yw = orc.compensated_forward(X[:5], np.ones_like(md), res.quant.codes, res.quant.scales, res.rec.L_A, res.rec.L_B, None)
    Yr = orc.compensated_forward(X[:5], md, res.quant.codes, res.quant.scales, res.rec.L_A, res.rec.L_B, None)
    assert np.linalg.norm(Yw - Yr) > 1e-3 * np.linalg.norm(Yr)


# ---------------------------------------------------------------- generators
# ---------------------------------------------------------------- another weight quantizer in place of RTN (Sec. 4.1, closing remark)
def test_target_of_another_quantizer_hand_example():
    W = np.array([[1.0, 2.0, -4.0], [3.0, 4.0, 0.5]], dtype=np.float32)
    mdiag = np.array([1.0, 2.0, 1.0], dtype=np.float32)
    Wq = np.array([[0.5, 0.0, -4.0], [3.0, 0.0, 1.0]])
    assert np.array_equal(orc.target_from_dequantized(W, mdiag, Wq), [[0.5, 4.0, 0.0], [0.0, 8.0, -0.5]])
    assert np.array_equal(orc.smoothed_weight(W, np.array([1], dtype=np.int32)), [[1.0, 0.0, -4.0], [3.0, 0.0, 0.5]])


def test_target_of_another_quantizer_keeps_the_layer_exact_and_reduces_to_known_cases():
    W, X, bits, f, r = _small_layer(seed=21)
    _, abs_sum, cnt = orc.gram(X)
    sm = orc.smooth_outliers(W, abs_sum, cnt, f)
    rng = np.random.default_rng(22)
    md = sm.mdiag.astype(np.float64)
    Xs = X.astype(np.float64) / md[None, :]                       # tokens x n: rows of (M^-1 X)^T
    # whatever the quantizer returned, W_q + T applied to the smoothed input gives back the layer
    Wq = rng.standard_normal(W.shape)
    T = orc.target_from_dequantized(W, sm.mdiag, Wq)
    assert np.allclose(Xs @ (Wq + T).T, X.astype(np.float64) @ W.astype(np.float64).T, rtol=1e-12, atol=1e-12)
    # a quantizer without error leaves the outlier columns W_o and nothing else
    W_s = orc.smoothed_weight(W, sm.idx)
    T0 = orc.target_from_dequantized(W, sm.mdiag, W_s)
    rest = np.setdiff1d(np.arange(W.shape[1]), sm.idx)
    assert not T0[:, rest].any()
    assert np.array_equal(T0[:, sm.idx], sm.W_o)
    assert not W_s[:, sm.idx].any() and np.array_equal(W_s[:, rest], W[:, rest])
    # with RTN's own result it is the target of the RTN stage
    q = orc.quantize_rtn(W, sm.idx, sm.mdiag, bits)
    assert np.array_equal(orc.target_from_dequantized(W, sm.mdiag, orc.dequantize(q.codes, q.scales)), q.T)
    # a planted mistake (M applied to W_q as well) breaks the exactness
    Tbad = (W.astype(np.float64) - Wq) * md[None, :]
    assert not np.allclose(Xs @ (Wq + Tbad).T, X.astype(np.float64) @ W.astype(np.float64).T, rtol=1e-6)


def test_synth_is_chunk_addressable_and_bf16_exact():
    spec = synth.mini("t", 8, 32, 3 * synth.CHUNK + 100)
    full = synth.make_activations(spec)
    part = synth.make_activations(spec, synth.CHUNK - 5, 2 * synth.CHUNK + 9)
    assert np.array_equal(full[synth.CHUNK - 5:2 * synth.CHUNK + 9], part)
    f = synth.bf16_to_f32(full)
    assert np.array_equal(synth.f32_to_bf16_bits(f), full)                 # round trip is exact
    x = np.array([1.0, 1.00390625, 1.01171875, -3.0e-39], dtype=np.float32)  # ties go to even
    assert synth.f32_to_bf16_bits(x)[:3].tolist() == [0x3F80, 0x3F80, 0x3F82]


# ---------------------------------------------------------------- stored oracle results (tests/golden)
def test_golden_c0_fixture_is_what_the_oracle_computes():
    """tests/golden/c0_oracle.json was written by tests/golden/make_golden.py from the oracle alone; the
    oracle must still reproduce it (integers and hashes exactly, floats to 1e-9: LAPACK builds differ in
    the last bits).  A deliberate change of the oracle regenerates the fixture in the same commit."""
    import importlib.util
    import json
    import os
    here = os.path.join(os.path.dirname(os.path.abspath(__file__)), "golden")
    spec = importlib.util.spec_from_file_location("make_golden", os.path.join(here, "make_golden.py"))
    mod = importlib.util.module_from_spec(spec)
    spec.loader.exec_module(mod)
    now = mod.compute()
    with open(os.path.join(here, "c0_oracle.json")) as fh:
        stored = json.load(fh)
    assert set(now) == set(stored)
    for key, val in stored.items():
        if isinstance(val, float):
            assert now[key] == pytest.approx(val, rel=1e-9), key
        elif isinstance(val, list) and val and isinstance(val[0], float):
            assert now[key] == pytest.approx(val, rel=1e-9), key
        else:
            assert now[key] == val, key
    # the planted channels of c0 are in the stored outlier set, largest first
    assert set(stored["idx"][:3]) == {3, 77, 190}
