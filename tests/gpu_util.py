"""Helpers shared by the GPU parity tests: upload seeded inputs, call the C ABI through the
Python binding, and fetch results as NumPy arrays."""
import numpy as np
import torch

import aser_synth as synth
import paper_2411_07762_amd as aser

DEV = "cuda:0"


def to_dev_x(spec, x_np):
    """Uploads activations; bf16 bit patterns become a torch.bfloat16 tensor with the same bytes."""
    if spec.x_dtype == "bf16":
        return torch.from_numpy(x_np.view(np.int16)).to(DEV).view(torch.bfloat16)
    return torch.from_numpy(x_np).to(DEV)


def padded(t, pad):
    """A view with leading dimension cols + pad (rows stay contiguous in memory otherwise)."""
    if pad == 0:
        return t
    buf = torch.zeros((t.shape[0], t.shape[1] + pad), dtype=t.dtype, device=t.device)
    buf[:, :t.shape[1]] = t
    return buf[:, :t.shape[1]]


def new_ctx():
    return aser.Context(0)


def run_gram(ctx, spec, x_np, chunks=1, pad=0):
    n = spec.n
    G = torch.zeros((n, n), dtype=torch.float32, device=DEV)
    abs_sum = torch.zeros(n, dtype=torch.float64, device=DEV)
    count = torch.zeros(1, dtype=torch.int64, device=DEV)
    N = x_np.shape[0]
    bounds = np.linspace(0, N, chunks + 1).astype(int)
    for a, b in zip(bounds[:-1], bounds[1:]):
        xd = padded(to_dev_x(spec, x_np[a:b]), pad)
        ctx.check(aser.aser_gram_accumulate(ctx, xd, G, abs_sum, count))
    torch.cuda.synchronize()
    return G, abs_sum, count


def lower(a):
    return np.tril(np.asarray(a))


def unpack_int4(packed):
    p = np.asarray(packed, dtype=np.uint8)
    lo = (p & 0x0F).astype(np.int8)
    hi = (p >> 4).astype(np.int8)
    lo = np.where(lo > 7, lo - 16, lo).astype(np.int8)
    hi = np.where(hi > 7, hi - 16, hi).astype(np.int8)
    out = np.empty((p.shape[0], p.shape[1] * 2), dtype=np.int8)
    out[:, 0::2] = lo
    out[:, 1::2] = hi
    return out
