"""CPU oracle for ASER's per-layer calibration path (arXiv 2411.07762).

TEST INFRASTRUCTURE ONLY.  This file is the plain, slow, fp64 NumPy/SciPy statement of what
the calibration path computes.  It shares no code with the HIP library and must never be
imported by it: only tests/, __graft_entry__.smoke() and bench.py's cpu_baseline leg call it.

Orientation.  The paper writes a layer as W X with X of shape (in x tokens) and the Gram
matrix as X X^T.  Here activations are stored tokens x in (N x n, row-major), so the same
n x n matrix is G = X^T X.  W is m x n (out x in) as in the paper.

Where the method has a plain definition (Gram matrix, Cholesky factor, truncated SVD, the
factors L_A and L_B) the oracle is that definition in fp64 with LAPACK doing the
factorisations.  Where it is a heuristic or an encoding (outlier selection, the smoothing
diagonal, the RTN quantizer) the oracle takes the steps in the paper's order.

Readings of points the paper leaves open (each is also listed in the design notes):
  * Q(.) is symmetric per-output-channel round-to-nearest: qmax = 2^(bits-1) - 1,
    scale = rowmax|W_s| / qmax evaluated in IEEE fp32, code = rint_half_even(w / scale) with
    an IEEE fp32 division, an all-zero row gets scale 1.  (Sec. 3, Sec. 5.1 "per-channel".)
  * "absolute mean" of a channel is the mean of absolute values (over tokens for X-bar, over
    output rows for W-bar), Sec. 4.2.
  * I_f is the set of the f largest scores X-bar * W-bar, ties resolved towards the lower
    index, reported in descending score order.  (Sec. 4.2 gives only the count f.)
  * The target that is whitened is T = W M - deq(Q(W_s)) = E_q + W_o (Eq. 12 and the
    sentence after it); the corresponding line of Algorithm 1 is read the same way.
  * The scale of Q(W_s) comes from W_s, i.e. from W with the I_f columns set to zero.
  * S is the lower Cholesky factor of (M^-1 X)(M^-1 X)^T = M^-1 G M^-1 (Algorithm 1).
  * No damping unless asked for; damp adds damp * mean(diag G') to the diagonal of G'.

  * Eq. 9 is read with a strict "<" and r >= 1; eps of Eq. 4 is 1e-12 (not given in the paper).
  * The compensated layer reads the same per-token quantized activations in both branches
    (W_q X_q + L_A L_B X_q), which is what the error ||W X - W~ X_q||_F of Sec. 5.3 measures.

Pins (tests/test_oracle_pins.py): Eckart-Young brute force on tiny matrices, the Eq. 8
identity with an explicit X, monotone error in r, zero error at full rank, invariance to the
square root of G, the S-free closed form U_r U_r^T T, the G = I reduction to a plain SVD,
exactness of W X = (W M)(M^-1 X), RTN invariants, and hand-computed RTN / smoothing examples;
effective rank in closed form (equal values, rank one, a two-value entropy), the full spectrum
against the eigenvalues of the Gram matrix, the overhead ratios of the paper's rank table, the
compensated output by element-wise loops, and the output error without activation quantization
against the whitened error of Eq. 8 on the calibration set itself; the target of another weight
quantizer through the exactness of W X = (W_q + T)(M^-1 X) for an arbitrary W_q, a lossless quantizer
(T = W_o alone), a hand example, and the RTN case.
Parity unpinned (the paper prints no worked example): which rounding/clipping convention
Q(.) uses and the tie-break of the outlier selection follow the readings above.
"""
from __future__ import annotations

from dataclasses import dataclass
from typing import Optional

import numpy as np
import scipy.linalg as sla


# ------------------------------------------------------------------ stage 1: Gram (Eq. 5)
def gram(X: np.ndarray, chunk: int = 8192):
    """G = X^T X (the paper's X X^T), column sums of |X| and the token count, all in fp64.

    X: N x n array of exactly representable values (fp32, or bf16 widened to fp32).
    The chunk loop only bounds the fp64 temporary; the result does not depend on it beyond
    fp64 summation order.
    """
    N, n = X.shape
    G = np.zeros((n, n), dtype=np.float64)
    abs_sum = np.zeros(n, dtype=np.float64)
    for s in range(0, N, chunk):
        xc = np.asarray(X[s:s + chunk], dtype=np.float64)
        G += xc.T @ xc
        abs_sum += np.abs(xc).sum(axis=0)
    return G, abs_sum, N


# ------------------------------------------------------------------ stage 2: smoothing (Sec. 4.2)
@dataclass
class Smoothing:
    idx: np.ndarray        # (f,) int32, descending score, ties -> lower index
    mdiag: np.ndarray      # (n,) fp32 diagonal of M (Eq. 11)
    score: np.ndarray      # (n,) fp64  X-bar * W-bar
    xbar: np.ndarray       # (n,) fp64
    wbar: np.ndarray       # (n,) fp64
    W_o: np.ndarray        # (m, f) fp64: the I_f columns of W M
    margin: float          # (s_(f) - s_(f+1)) / s_(f): how far the selection is from a tie


def smooth_outliers(W: np.ndarray, abs_sum: np.ndarray, count: int, f: int) -> Smoothing:
    """Outlier index set I_f and the smoothing diagonal m (Eq. 10, Eq. 11)."""
    m_rows, n = W.shape
    if not 0 <= f <= n:
        raise ValueError("f out of range")
    xbar = np.asarray(abs_sum, dtype=np.float64) / float(count)
    wbar = np.abs(np.asarray(W, dtype=np.float64)).sum(axis=0) / float(m_rows)
    score = xbar * wbar
    order = np.argsort(-score, kind="stable")           # descending, ties -> lower index
    idx = order[:f].astype(np.int32)
    mvec = np.ones(n, dtype=np.float64)
    if f > 0:
        xmin = xbar[idx].min()
        mvec[idx] = xbar[idx] / xmin
    mdiag = mvec.astype(np.float32)
    W_o = np.asarray(W, dtype=np.float64)[:, idx] * mdiag[idx].astype(np.float64)[None, :]
    if 0 < f < n:
        sf, sf1 = score[order[f - 1]], score[order[f]]
        margin = float((sf - sf1) / sf) if sf > 0 else 0.0
    else:
        margin = float("inf")
    return Smoothing(idx, mdiag, score, xbar, wbar, W_o, margin)


# ------------------------------------------------------------------ stage 3: RTN + target (Eq. 12)
@dataclass
class Quantized:
    codes: np.ndarray      # (m, n) int8 in [-qmax, qmax]
    scales: np.ndarray     # (m,) fp32
    T: np.ndarray          # (m, n) fp64:  W M - codes * scales  = E_q + W_o


def quantize_rtn(W: np.ndarray, idx: np.ndarray, mdiag: np.ndarray, bits: int) -> Quantized:
    """Per-output-channel symmetric RTN of W_s and the target T = E_q + W_o.

    The scale and the codes are evaluated in IEEE fp32, the precision the quantizer runs in
    on any device, so that the integer decisions are reproducible bit for bit.
    """
    if bits not in (4, 8):
        raise ValueError("bits must be 4 or 8")
    W = np.asarray(W, dtype=np.float32)
    qmax = np.float32(2 ** (bits - 1) - 1)
    W_s = W.copy()
    W_s[:, idx] = np.float32(0.0)                        # outlier columns are not quantized
    amax = np.abs(W_s).max(axis=1)                       # exact
    scales = (amax / qmax).astype(np.float32)            # IEEE fp32 division
    scales[amax == 0] = np.float32(1.0)
    q = np.rint(W_s / scales[:, None])                   # fp32 division, round half to even
    q = np.clip(q, -qmax, qmax)
    codes = q.astype(np.int8)
    WM = W.astype(np.float64) * np.asarray(mdiag, dtype=np.float32).astype(np.float64)[None, :]
    T = WM - codes.astype(np.float64) * scales.astype(np.float64)[:, None]
    return Quantized(codes, scales, T)


# ------------------------------------------------------------------ stage 3 with another weight quantizer (Sec. 4.1, closing remark)
def smoothed_weight(W: np.ndarray, idx: np.ndarray) -> np.ndarray:
    """W_s, the matrix Algorithm 1 hands to the weight quantizer: W M with the I_f columns taken out.
    M differs from 1 only on those columns, so this is W with the I_f columns set to zero."""
    W_s = np.array(W, dtype=np.float32)
    W_s[:, np.asarray(idx, dtype=np.int64)] = np.float32(0.0)
    return W_s


def target_from_dequantized(W: np.ndarray, mdiag: np.ndarray, Wq: np.ndarray) -> np.ndarray:
    """T = W M - W_q for the dequantized result W_q of ANY weight-only quantizer run on W_s (the method
    "is orthogonal to" the choice of that quantizer).  W X = (W_q + T)(M^-1 X) holds whatever W_q is;
    where W_q keeps the I_f columns at zero, T = E_q + W_o as in Eq. 12."""
    WM = np.asarray(W, dtype=np.float32).astype(np.float64) * np.asarray(mdiag, dtype=np.float32).astype(np.float64)[None, :]
    return WM - np.asarray(Wq, dtype=np.float64)


def pack_int4(codes: np.ndarray) -> np.ndarray:
    """Two's-complement nibbles, even column in the low nibble; n must be even."""
    c = np.asarray(codes, dtype=np.int8)
    if c.shape[1] % 2:
        raise ValueError("packing needs an even number of columns")
    lo = c[:, 0::2].astype(np.uint8) & np.uint8(0x0F)
    hi = c[:, 1::2].astype(np.uint8) & np.uint8(0x0F)
    return (lo | (hi << np.uint8(4))).astype(np.uint8)


def dequantize(codes: np.ndarray, scales: np.ndarray) -> np.ndarray:
    return codes.astype(np.float64) * np.asarray(scales, dtype=np.float64)[:, None]


# ------------------------------------------------------------------ stage 4a: whitening (Eq. 5, Alg. 1)
def whiten(G: np.ndarray, mdiag: Optional[np.ndarray] = None, damp: float = 0.0) -> np.ndarray:
    """Lower Cholesky factor S of G' = M^-1 G M^-1, so that S^-1 G' S^-T = I."""
    Gp = np.array(G, dtype=np.float64)
    if mdiag is not None:
        inv = 1.0 / np.asarray(mdiag, dtype=np.float32).astype(np.float64)
        Gp = Gp * inv[:, None] * inv[None, :]
    if damp:
        Gp = Gp + damp * float(np.mean(np.diag(Gp))) * np.eye(Gp.shape[0])
    return np.linalg.cholesky(Gp)


# ------------------------------------------------------------------ stage 4b/c: whitened SVD (Eq. 6)
@dataclass
class Reconstruction:
    L_A: np.ndarray        # (m, r)  U_r Sigma_r
    L_B: np.ndarray        # (r, n)  V_r^T S^-1
    sigma: np.ndarray      # all min(m, n) singular values of T S, descending
    err: float             # ||(T - L_A L_B) S||_F = sqrt(sum_{i>r} sigma_i^2)   (Eq. 8)
    err0: float            # ||T S||_F (no compensation)
    gap: float             # sigma_r / sigma_{r+1}


def error_reconstruct(T: np.ndarray, S: np.ndarray, r: int) -> Reconstruction:
    """Rank-r truncation of the SVD of T S and the LoRA-style factors (Eq. 6, Sec. 4.1)."""
    m, n = T.shape
    k = min(m, n)
    if not 0 < r <= k:
        raise ValueError("r out of range")
    A = np.asarray(T, dtype=np.float64) @ S
    U, sig, Vt = np.linalg.svd(A, full_matrices=False)
    L_A = U[:, :r] * sig[:r][None, :]
    # L_B = V_r^T S^-1  <=>  L_B S = V_r^T  <=>  S^T L_B^T = V_r
    L_B = sla.solve_triangular(S, Vt[:r].T, lower=True, trans="T").T
    tail = sig[r:]
    gap = float(sig[r - 1] / sig[r]) if r < k and sig[r] > 0 else float("inf")
    return Reconstruction(L_A, L_B, sig, float(np.sqrt((tail ** 2).sum())),
                          float(np.sqrt((sig ** 2).sum())), gap)


def whitened_error(T: np.ndarray, S: np.ndarray, L_A: np.ndarray, L_B: np.ndarray) -> float:
    """||(T - L_A L_B) S||_F in fp64: the layer-output error of Eq. 2 after whitening."""
    R = np.asarray(T, dtype=np.float64) - np.asarray(L_A, dtype=np.float64) @ np.asarray(L_B, dtype=np.float64)
    return float(np.linalg.norm(R @ S))


# ------------------------------------------------------------------ rank from alpha (Eq. 9)
def rank_from_alpha(sigma: np.ndarray, alpha: float) -> int:
    """Largest r with sum_{i<=r} sigma_i / sum_i sigma_i < alpha (at least 1)."""
    c = np.cumsum(sigma) / np.sum(sigma)
    return max(1, int(np.searchsorted(c, alpha, side="left")))


# ------------------------------------------------------------------ per-token activation RTN (Sec. 5.1)
def quantize_act_rtn(X: np.ndarray, mdiag: np.ndarray, bits: int = 8):
    """Per-token symmetric RTN of the smoothed activations X' = X M^-1, in IEEE fp32."""
    qmax = np.float32(2 ** (bits - 1) - 1)
    Xp = (np.asarray(X, dtype=np.float32) / np.asarray(mdiag, dtype=np.float32)[None, :]).astype(np.float32)
    amax = np.abs(Xp).max(axis=1)
    scales = (amax / qmax).astype(np.float32)
    scales[amax == 0] = np.float32(1.0)
    q = np.clip(np.rint(Xp / scales[:, None]), -qmax, qmax)
    return q.astype(np.int8), scales


# ------------------------------------------------------------------ full spectrum, rank threshold, effective rank
def singular_values(T: np.ndarray, S: Optional[np.ndarray] = None) -> np.ndarray:
    """All min(m, n) singular values of T S (of T itself when S is None), descending (Eq. 6).

    With S the whitening factor this is the spectrum that Eq. 9 sums and that Sec. 3.2 plots for
    E_q X (E_q S and E_q X share their singular values because S S^T = X X^T); with S = None it is
    the spectrum of the weight error E_q alone.
    """
    A = np.asarray(T, dtype=np.float64)
    if S is not None:
        A = A @ np.asarray(S, dtype=np.float64)
    return np.linalg.svd(A, compute_uv=False)


def effective_rank(sigma: np.ndarray, eps: float = 1e-12) -> float:
    """exp(-sum_k p_k ln p_k) with p_k = sigma_k / sum_i sigma_i + eps (Eq. 3, Eq. 4).

    The paper does not give eps; 1e-12 only keeps ln p_k finite for zero singular values.
    """
    sg = np.asarray(sigma, dtype=np.float64)
    p = sg / sg.sum() + eps
    return float(np.exp(-(p * np.log(p)).sum()))


def normalized_profile(sigma: np.ndarray, k: int = 128) -> np.ndarray:
    """The k largest singular values divided by the largest one (the curves of Sec. 3.2's first figure;
    the paper says "normalized for comparison" without naming the divisor)."""
    sg = np.sort(np.asarray(sigma, dtype=np.float64))[::-1][:k]
    return sg / sg[0]


def overhead_flops_ratio(r: float, d: int) -> float:
    """Extra inference FLOPs of the L_A, L_B branch relative to the layer itself: (s d^2 + 2 s r d) / (s d^2) - 1
    = 2 r / d (overhead analysis of Sec. 5.3; s cancels)."""
    return 2.0 * float(r) / float(d)


# ------------------------------------------------------------------ compensated layer and its output error
def compensated_weight(codes: np.ndarray, scales: np.ndarray, L_A: Optional[np.ndarray],
                       L_B: Optional[np.ndarray]) -> np.ndarray:
    """W~ = deq(Q(W_s)) + L_A L_B, the weight the compensated layer applies to the smoothed input
    M^-1 X (end of Sec. 4.2: inference is W_q X + L_A L_B X).  L_A = None: the RTN baseline W_q."""
    Wt = dequantize(codes, scales)
    if L_A is not None:
        Wt = Wt + np.asarray(L_A, dtype=np.float64) @ np.asarray(L_B, dtype=np.float64)
    return Wt


def compensated_forward(X: np.ndarray, mdiag: np.ndarray, codes: np.ndarray, scales: np.ndarray,
                        L_A: Optional[np.ndarray], L_B: Optional[np.ndarray], act_bits: Optional[int]):
    """Output of the quantized, compensated layer for the tokens in X (tokens x n), as tokens x m:
    Y~ = X'_q W~^T with X' = X M^-1 and X'_q its per-token RTN image dequantized (Sec. 5.1; the remaining
    error that Sec. 5.3's figure plots is ||W X - W~ X_q||_F).  act_bits = None: X'_q = X' (weights only).
    Both branches read the same quantized activations."""
    md = np.asarray(mdiag, dtype=np.float32)
    if act_bits is None:
        Xq = np.asarray(X, dtype=np.float64) / md.astype(np.float64)[None, :]
    else:
        q, s = quantize_act_rtn(X, md, act_bits)
        Xq = q.astype(np.float64) * s.astype(np.float64)[:, None]
    return Xq @ compensated_weight(codes, scales, L_A, L_B).T


def layer_output_error(W: np.ndarray, X: np.ndarray, mdiag: np.ndarray, codes: np.ndarray, scales: np.ndarray,
                       L_A: Optional[np.ndarray], L_B: Optional[np.ndarray], act_bits: Optional[int]):
    """||X W^T - X'_q W~^T||_F over the tokens in X and the norm of the exact output ||X W^T||_F
    (the paper's ||W X - W~ X_q||_F in tokens x channels orientation; caption of Sec. 5.3's error figure)."""
    Y = np.asarray(X, dtype=np.float64) @ np.asarray(W, dtype=np.float64).T
    Yq = compensated_forward(X, mdiag, codes, scales, L_A, L_B, act_bits)
    return float(np.linalg.norm(Y - Yq)), float(np.linalg.norm(Y))


# ------------------------------------------------------------------ the whole layer (Algorithm 1, loop body)
@dataclass
class LayerResult:
    G: np.ndarray
    abs_sum: np.ndarray
    count: int
    smooth: Smoothing
    quant: Quantized
    S: np.ndarray
    rec: Reconstruction


def calibrate_layer(W: np.ndarray, X: np.ndarray, bits: int, f: int, r: int,
                    damp: float = 0.0, timings: Optional[dict] = None) -> LayerResult:
    """One pass of Algorithm 1's loop body for a single layer."""
    import time
    t = [time.perf_counter()]

    def lap(key):
        t.append(time.perf_counter())
        if timings is not None:
            timings[key] = timings.get(key, 0.0) + (t[-1] - t[-2])

    G, abs_sum, count = gram(X); lap("gram")
    sm = smooth_outliers(W, abs_sum, count, f); lap("smooth")
    qz = quantize_rtn(W, sm.idx, sm.mdiag, bits); lap("rtn")
    S = whiten(G, sm.mdiag, damp); lap("whiten")
    rec = error_reconstruct(qz.T, S, r); lap("reconstruct")
    return LayerResult(G, abs_sum, count, sm, qz, S, rec)
