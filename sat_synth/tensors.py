"""Seeded dense inputs: features, weights, noise, labels, predictor parameters.

All draws come from numpy PCG64 streams spawned from one SeedSequence, one
sub-stream per artefact, so that changing one artefact's size never shifts
another's values. Large normal tensors are filled in fixed-size row chunks,
each chunk from its own spawned stream, so the result does not depend on how
many threads do the filling.
"""
from concurrent.futures import ThreadPoolExecutor
import os

import numpy as np

_ARTEFACTS = ("graph", "features", "weights", "noise", "labels", "predictor",
              "history", "misc")
_CHUNK_ELEMS = 1 << 22


def substreams(seed):
    """dict artefact-name -> SeedSequence, spawned from SeedSequence(seed)."""
    kids = np.random.SeedSequence(seed).spawn(len(_ARTEFACTS))
    return dict(zip(_ARTEFACTS, kids))


def _rng(ss):
    return np.random.Generator(np.random.PCG64(ss))


def normal_f32(ss, rows, cols, std=1.0, mean=0.0, out=None, ld=None):
    """[rows, cols] fp32 N(mean, std^2), written into out[:, :cols] if given.

    out may have a leading dimension ld >= cols (padding columns untouched).
    """
    ld = cols if ld is None else ld
    if out is None:
        out = np.zeros((rows, ld), dtype=np.float32)
    assert out.shape == (rows, ld) and out.dtype == np.float32
    if rows == 0 or cols == 0:
        return out
    rows_per = max(1, _CHUNK_ELEMS // cols)
    n_chunks = (rows + rows_per - 1) // rows_per
    kids = ss.spawn(n_chunks)

    def fill(c):
        r0 = c * rows_per
        r1 = min(rows, r0 + rows_per)
        g = _rng(kids[c])
        blk = g.standard_normal((r1 - r0, cols), dtype=np.float32)
        if std != 1.0:
            blk *= np.float32(std)
        if mean != 0.0:
            blk += np.float32(mean)
        out[r0:r1, :cols] = blk

    workers = min(n_chunks, max(1, min(16, os.cpu_count() or 1)))
    if workers == 1:
        for c in range(n_chunks):
            fill(c)
    else:
        with ThreadPoolExecutor(workers) as ex:
            list(ex.map(fill, range(n_chunks)))
    return out


def glorot_uniform_f32(ss, d_in, d_out):
    """[d_in, d_out] fp32, U(-a, a) with a = sqrt(6 / (d_in + d_out))."""
    a = np.sqrt(6.0 / (d_in + d_out))
    return _rng(ss).uniform(-a, a, size=(d_in, d_out)).astype(np.float32)


def labels_i32(ss, n, n_classes):
    return _rng(ss).integers(0, n_classes, size=n, dtype=np.int32)


def predictor_params_f32(ss, d, d_s, scale_g=0.5):
    """Random parameters of one embedding predictor (one hidden layer's).

    Wx [4*d_s, d], Wh [4*d_s, d_s], b [4*d_s] (gate blocks stacked i, f, g, o)
    drawn U(+-1/sqrt(d_s)); Wg [d_s, d] Glorot-uniform scaled by scale_g.
    """
    g = _rng(ss)
    k = 1.0 / np.sqrt(d_s)
    Wx = g.uniform(-k, k, size=(4 * d_s, d)).astype(np.float32)
    Wh = g.uniform(-k, k, size=(4 * d_s, d_s)).astype(np.float32)
    b = g.uniform(-k, k, size=(4 * d_s,)).astype(np.float32)
    a = scale_g * np.sqrt(6.0 / (d_s + d))
    Wg = g.uniform(-a, a, size=(d_s, d)).astype(np.float32)
    return dict(Wx=Wx, Wh=Wh, b=b, Wg=Wg)


def gat_heads(dims, hidden_heads=4):
    """Heads per layer of the attention backbone for feature widths `dims`: `hidden_heads`
    (four unless stated) on hidden layers whose width allows it (a multiple of four
    elements per head), one head on the last layer (the usual classifier) and otherwise."""
    L = len(dims) - 1
    return [hidden_heads if l < L - 1 and dims[l + 1] % (4 * hidden_heads) == 0 else 1 for l in range(L)]


def attention_vectors_f32(ss, heads, d_head):
    """(a_dst, a_src), each [heads, d_head] ~ N(0, 1 / d_head): scores of unit-scale
    rows then have unit scale, so the attention is neither flat nor one-hot."""
    r = _rng(ss)
    std = 1.0 / np.sqrt(d_head)
    return (r.normal(0.0, std, size=(heads, d_head)).astype(np.float32),
            r.normal(0.0, std, size=(heads, d_head)).astype(np.float32))


def history_standin_f32(ss, rows, cols, tau, noise_std, ld=None):
    """tau history slots [rows, ld] for sizes where nobody can afford the
    true full-graph embeddings: a shared base max(0, N(0,1)) (the shape of a
    ReLU layer's output: non-negative, about half zeros) plus independent
    N(0, noise_std^2) staleness noise per slot. Oldest slot first."""
    kids = ss.spawn(tau + 1)
    base = normal_f32(kids[0], rows, cols, ld=ld)
    np.maximum(base, 0.0, out=base)
    slots = []
    for s in range(tau):
        t = normal_f32(kids[1 + s], rows, cols, std=noise_std, ld=ld)
        t += base
        slots.append(t)
    return slots


def drifting_history_f32(ss, rows, cols, epochs, drift=0.3, spread=0.03, noise=0.01):
    """`epochs` matrices [rows, cols] (fp32, oldest first) that move at a steady pace:
    row r of epoch t is base[r] + t * (v + w[r]) + noise, with a velocity v shared by all rows
    (std `drift` per column), a small row-specific part w (std `spread`) and observation noise.
    A stand-in for hidden embeddings that keep evolving from epoch to epoch: the newest
    cached matrix is then a stale estimate of the next one, by about |v| per entry."""
    rng = _rng(ss)
    base = np.maximum(rng.standard_normal((rows, cols)), 0)
    vel = drift * rng.standard_normal(cols)[None, :] + spread * rng.standard_normal((rows, cols))
    return [(base + t * vel + noise * rng.standard_normal((rows, cols))).astype(np.float32)
            for t in range(epochs)]


def bf16_bits_from_f32(a):
    """Round fp32 values to bfloat16 (nearest, ties to even); returns the 16-bit
    patterns as uint16. A storage-format conversion only."""
    u = np.ascontiguousarray(a, dtype=np.float32).view(np.uint32)
    rounded = u + (np.uint32(0x7FFF) + ((u >> np.uint32(16)) & np.uint32(1)))
    return (rounded >> np.uint32(16)).astype(np.uint16)


def f32_from_bf16_bits(b):
    """Exact fp32 value of every bfloat16 bit pattern in b (uint16)."""
    return (np.ascontiguousarray(b, dtype=np.uint16).astype(np.uint32) << np.uint32(16)).view(np.float32)


# ---- generators that fill device memory directly (inputs too large to draw on the host)

def device_normal(rows, cols, ld, seed, device, bf16, std=1.0):
    """[rows, ld] N(0, std^2) in the first `cols` columns (zeros in the padding), drawn
    on `device` by torch's generator seeded with `seed`, 2^20 rows at a time.
    Returns a torch tensor (float32 or bfloat16)."""
    import torch
    gen = torch.Generator(device=device)
    gen.manual_seed(int(seed))
    out = torch.zeros((rows, ld), dtype=torch.bfloat16 if bf16 else torch.float32, device=device)
    step = 1 << 20
    for r0 in range(0, rows, step):
        r1 = min(rows, r0 + step)
        blk = torch.randn((r1 - r0, cols), generator=gen, device=device, dtype=torch.float32)
        if std != 1.0:
            blk *= std
        out[r0:r1, :cols] = blk.to(out.dtype)
    return out


def device_history_standin(rows, cols, ld, tau, noise_std, seed, device, bf16):
    """tau slots [rows, ld] of the stand-in of history_standin_f32 (shared base
    max(0, N(0,1)) plus N(0, noise_std^2) per slot), drawn on the device. Oldest first."""
    import torch
    gen = torch.Generator(device=device)
    gen.manual_seed(int(seed))
    dt = torch.bfloat16 if bf16 else torch.float32
    slots = [torch.zeros((rows, ld), dtype=dt, device=device) for _ in range(tau)]
    step = 1 << 20
    for r0 in range(0, rows, step):
        r1 = min(rows, r0 + step)
        base = torch.randn((r1 - r0, cols), generator=gen, device=device, dtype=torch.float32)
        base.clamp_(min=0.0)
        for s in range(tau):
            noise = torch.randn((r1 - r0, cols), generator=gen, device=device, dtype=torch.float32)
            slots[s][r0:r1, :cols] = (base + noise_std * noise).to(dt)
    return slots
