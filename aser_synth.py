"""Seeded synthetic layers for the ASER calibration path.

This module only draws random inputs (weights W, calibration activations X) with the
shapes and value distributions of the Llama-class workloads the method is evaluated on
(Sec. 5.1: 128 samples x 2048 tokens of calibration data, per-channel W4, r = 64, f = 32;
Sec. 3.2: fewer than 1 % of the channels are large-magnitude outliers).  It holds none of
the method's arithmetic: no Gram, no statistics, no quantizer, no factorisation.  Both the
HIP path and the CPU oracle receive the *same bytes* produced here.

Activations are chunk-addressable: rows [c*CHUNK, (c+1)*CHUNK) depend only on
(seed, layer id, stream id, c), so any token range can be regenerated independently.

bf16 is carried as uint16 bit patterns (NumPy has no bf16); `bf16_to_f32` widens exactly.
"""
from __future__ import annotations

from dataclasses import dataclass, replace
from typing import Dict, Tuple

import numpy as np

SEED = 20241107
CHUNK = 4096  # tokens per independently seeded chunk


# --------------------------------------------------------------------------- dtype helpers
def f32_to_bf16_bits(x: np.ndarray) -> np.ndarray:
    """Round fp32 to bf16 (round-to-nearest-even), returned as uint16 bit patterns."""
    u = np.ascontiguousarray(x, dtype=np.float32).view(np.uint32)
    rounded = u + np.uint32(0x7FFF) + ((u >> np.uint32(16)) & np.uint32(1))
    return (rounded >> np.uint32(16)).astype(np.uint16)


def bf16_to_f32(bits: np.ndarray) -> np.ndarray:
    """Widen bf16 bit patterns (uint16) to fp32 exactly."""
    return (np.ascontiguousarray(bits, dtype=np.uint16).astype(np.uint32) << np.uint32(16)).view(np.float32)


# --------------------------------------------------------------------------- specs
@dataclass(frozen=True)
class LayerSpec:
    """One synthetic linear layer y = W x with its calibration stream."""
    name: str
    m: int                 # output features (rows of W)
    n: int                 # input features (columns of W, channels of X)
    tokens: int            # calibration tokens N
    x_dtype: str           # "bf16" | "f32"
    x_dist: str            # "gauss" | "silu_prod"
    w_std: float           # std of the Gaussian bulk of W
    w_heavy: bool          # replace 0.1 % of W by Student-t(3) * 0.1
    n_outliers: int        # planted outlier channels in X
    out_lo: float          # outlier factor ~ U(out_lo, out_hi) (lo == hi: constant)
    out_hi: float
    bits: int              # weight bits
    r: int                 # rank
    f: int                 # outlier channels extracted
    layer_id: int          # seeds W
    stream_id: int         # seeds X (layers sharing an input share this)
    fixed_outliers: Tuple[int, ...] = ()   # if set, planted channels are these

    def with_(self, **kw) -> "LayerSpec":
        return replace(self, **kw)


def _gauss_layer(name, m, n, tokens, lid, sid, r=64, f=32) -> LayerSpec:
    return LayerSpec(name, m, n, tokens, "bf16", "gauss", 0.02, True, 16, 20.0, 60.0, 4, r, f, lid, sid)


CONFIGS: Dict[str, LayerSpec] = {
    # c0: tiny all-fp32 layer, planted channels {3, 77, 190} x 30
    "c0": LayerSpec("c0", 256, 256, 1024, "f32", "gauss", 0.02, False, 3, 30.0, 30.0, 4, 16, 4, 0, 0,
                    fixed_outliers=(3, 77, 190)),
    # c1: Llama-7B attention projection, the headline 4096 x 4096 layer
    "c1": _gauss_layer("c1", 4096, 4096, 32768, 100, 100),
    # c2: MLP down projection, heavy-tailed post-SiLU-like input
    "c2": LayerSpec("c2", 4096, 11008, 65536, "bf16", "silu_prod", 0.02, True, 24, 40.0, 40.0, 4, 64, 32, 200, 200),
    # c4: large-model down projection
    "c4": LayerSpec("c4", 8192, 28672, 262144, "bf16", "silu_prod", 0.015, False, 64, 40.0, 40.0, 4, 128, 64, 400, 400),
}

# c3: a Llama-3-8B-shaped block; q,k,v share the attention input, gate/up share the MLP input
_C3_TOKENS = 131072
for _i, (_nm, _m, _n, _sid) in enumerate([
        ("q", 4096, 4096, 300), ("k", 1024, 4096, 300), ("v", 1024, 4096, 300),
        ("o", 4096, 4096, 301), ("gate", 14336, 4096, 302), ("up", 14336, 4096, 302),
        ("down", 4096, 14336, 303)]):
    CONFIGS["c3." + _nm] = _gauss_layer("c3." + _nm, _m, _n, _C3_TOKENS, 310 + _i, _sid)
C3_LAYERS = tuple(k for k in CONFIGS if k.startswith("c3."))
# qkv: the block's three attention projections fused into one linear layer (the "qkv_proj" of the paper's
# singular-value figure): 4096 + 1024 + 1024 output rows on the attention input
CONFIGS["qkv"] = _gauss_layer("qkv", 6144, 4096, _C3_TOKENS, 320, 300)


def mini(name: str, m: int, n: int, tokens: int, *, x_dtype="bf16", x_dist="gauss", n_outliers=3,
         r=8, f=4, bits=4, seed_id=900, heavy=True, out=(20.0, 60.0)) -> LayerSpec:
    """A small layer with the statistics of c1/c2 for parity tests at odd shapes."""
    return LayerSpec(name, m, n, tokens, x_dtype, x_dist, 0.02, heavy, n_outliers, out[0], out[1],
                     bits, r, f, seed_id, seed_id)


# --------------------------------------------------------------------------- generators
def outlier_channels(spec: LayerSpec) -> Tuple[np.ndarray, np.ndarray]:
    """Planted outlier channel indices (sorted) and their multiplicative factors."""
    if spec.n_outliers == 0:
        return np.zeros(0, np.int64), np.zeros(0, np.float32)
    rng = np.random.default_rng([SEED, 2, spec.stream_id])
    if spec.fixed_outliers:
        idx = np.array(spec.fixed_outliers, dtype=np.int64)
    else:
        idx = np.sort(rng.choice(spec.n, size=spec.n_outliers, replace=False)).astype(np.int64)
    if spec.out_lo == spec.out_hi:
        fac = np.full(len(idx), spec.out_lo, dtype=np.float32)
    else:
        fac = rng.uniform(spec.out_lo, spec.out_hi, size=len(idx)).astype(np.float32)
    return idx, fac


def make_weight(spec: LayerSpec) -> np.ndarray:
    """W (m x n, fp32, row-major): Gaussian bulk, optionally 0.1 % heavy-tailed entries."""
    rng = np.random.default_rng([SEED, 1, spec.layer_id])
    w = rng.standard_normal((spec.m, spec.n), dtype=np.float32)
    w *= np.float32(spec.w_std)
    if spec.w_heavy:
        k = max(1, int(round(0.001 * spec.m * spec.n)))
        pos = rng.choice(spec.m * spec.n, size=k, replace=False)
        w.reshape(-1)[pos] = (rng.standard_t(3.0, size=k) * 0.1).astype(np.float32)
    return w


def _x_chunk_f32(spec: LayerSpec, c: int, rows: int) -> np.ndarray:
    rng = np.random.default_rng([SEED, 3, spec.stream_id, c])
    if spec.x_dist == "gauss":
        x = rng.standard_normal((rows, spec.n), dtype=np.float32)
    elif spec.x_dist == "silu_prod":
        a = rng.standard_normal((rows, spec.n), dtype=np.float32)
        b = rng.standard_normal((rows, spec.n), dtype=np.float32)
        x = a * (b / (np.float32(1.0) + np.exp(-b)))
    else:
        raise ValueError(spec.x_dist)
    idx, fac = outlier_channels(spec)
    if len(idx):
        x[:, idx] *= fac[None, :]
    return x


def make_activations(spec: LayerSpec, start: int = 0, stop: int | None = None, workers: int = 1) -> np.ndarray:
    """Rows [start, stop) of X (tokens x n, row-major).

    Returns uint16 bf16 bit patterns when spec.x_dtype == "bf16", else fp32.
    A chunk is always generated whole, so a row's values never depend on the range asked for,
    nor on `workers` (threads that draw different chunks at the same time).
    """
    stop = spec.tokens if stop is None else stop
    if not (0 <= start <= stop <= spec.tokens):
        raise ValueError("token range out of bounds")
    out = np.empty((stop - start, spec.n), dtype=np.uint16 if spec.x_dtype == "bf16" else np.float32)

    def fill(c):
        lo, hi = c * CHUNK, min((c + 1) * CHUNK, spec.tokens)
        x = _x_chunk_f32(spec, c, hi - lo)
        a, b = max(lo, start), min(hi, stop)
        part = x[a - lo:b - lo]
        out[a - start:b - start] = f32_to_bf16_bits(part) if spec.x_dtype == "bf16" else part

    chunks = range(start // CHUNK, (stop + CHUNK - 1) // CHUNK) if stop > start else range(0)
    if workers > 1 and len(chunks) > 1:
        from concurrent.futures import ThreadPoolExecutor
        with ThreadPoolExecutor(workers) as pool:
            list(pool.map(fill, chunks))
    else:
        for c in chunks:
            fill(c)
    return out


def activations_as_f32(spec: LayerSpec, x: np.ndarray) -> np.ndarray:
    """The exact values of X as fp32 (widening bf16 bit patterns when needed)."""
    return bf16_to_f32(x) if spec.x_dtype == "bf16" else np.asarray(x, dtype=np.float32)
