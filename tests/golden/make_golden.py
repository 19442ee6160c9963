"""Writes tests/golden/c0_oracle.json: what the CPU oracle computes on the seeded layer c0.

The paper prints no worked numeric example of the per-layer computation (no small matrix with its
S, sigma or L_A / L_B), so no fixture here holds a value of the paper's.  This file stores the
oracle's own results on one seeded layer instead, as a tripwire: a change to the oracle's arithmetic,
to the input generators or to a library routine the oracle calls shows up as a diff of the fixture.
It calls nothing but oracle/ and the input generators; the HIP path is never involved.

    python tests/golden/make_golden.py          (from the repository root)

Stored per stage of Algorithm 1's loop body: the outlier set I_f and its smoothing factors (Eq. 11),
the RTN scales and a checksum of the codes (Eq. 12), diagonal entries of S (Eq. 5), the leading
singular values of T S and the whitened error (Eq. 6, Eq. 8), and the per-token A8 scales (Sec. 5.1).
"""
import hashlib
import json
import os
import sys

import numpy as np

ROOT = os.path.dirname(os.path.dirname(os.path.dirname(os.path.abspath(__file__))))
sys.path.insert(0, ROOT)

import aser_synth as synth                      # noqa: E402
from oracle import aser_oracle as orc           # noqa: E402


def compute():
    spec = synth.CONFIGS["c0"]
    W = synth.make_weight(spec)
    X = synth.activations_as_f32(spec, synth.make_activations(spec))
    res = orc.calibrate_layer(W, X, spec.bits, spec.f, spec.r)
    codes8, act_scales = orc.quantize_act_rtn(X, res.smooth.mdiag, 8)
    return {
        "config": "c0",
        "shape": {"m": spec.m, "n": spec.n, "tokens": spec.tokens, "bits": spec.bits, "r": spec.r, "f": spec.f},
        "gram_trace": float(np.trace(res.G)),
        "gram_frobenius": float(np.linalg.norm(res.G)),
        "idx": [int(i) for i in res.smooth.idx],
        "mdiag_on_idx": [float(res.smooth.mdiag[i]) for i in res.smooth.idx],
        "selection_margin": float(res.smooth.margin),
        "rtn_scales_first8": [float(s) for s in res.quant.scales[:8]],
        "rtn_codes_sha256": hashlib.sha256(np.ascontiguousarray(res.quant.codes, dtype=np.int8).tobytes()).hexdigest(),
        "T_frobenius": float(np.linalg.norm(res.quant.T)),
        "S_diag_first8": [float(res.S[i, i]) for i in range(8)],
        "S_frobenius": float(np.linalg.norm(res.S)),
        "sigma_first": [float(s) for s in res.rec.sigma[:spec.r + 1]],
        "whitened_error": float(res.rec.err),
        "whitened_error_uncompensated": float(res.rec.err0),
        "gap_sigma_r_over_next": float(res.rec.gap),
        "L_A_frobenius": float(np.linalg.norm(res.rec.L_A)),
        "L_A_L_B_frobenius": float(np.linalg.norm(res.rec.L_A @ res.rec.L_B)),
        "act_scales_first8": [float(s) for s in act_scales[:8]],
        "act_codes_sha256": hashlib.sha256(np.ascontiguousarray(codes8, dtype=np.int8).tobytes()).hexdigest(),
    }


if __name__ == "__main__":
    out = os.path.join(os.path.dirname(os.path.abspath(__file__)), "c0_oracle.json")
    with open(out, "w") as fh:
        json.dump(compute(), fh, indent=1)
        fh.write("\n")
    print("wrote", out)
