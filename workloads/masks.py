"""Seeded synthetic pruning masks with the structure of the paper's schemes.

The paper produces masks with trained pruning algorithms (magnitude, ADMM, ...),
which need datasets; these generators draw masks of the same *structure*
(section 3, Fig. 1 (e)-(g)) from a seed instead.  They only generate inputs:
validation, packing and execution of the masks live elsewhere.

Mask convention: uint8, same shape as the weights, 1 = weight kept.
"""
from __future__ import annotations

from fractions import Fraction

import numpy as np

from . import prng


def _keep_counts(sizes: np.ndarray, rate: Fraction) -> np.ndarray:
    """Exact-rate dithering: block b keeps floor(cum[b+1]/r) - floor(cum[b]/r)
    positions, cum = running number of positions, so the layer keeps
    floor(total/r) positions overall."""
    num, den = rate.numerator, rate.denominator
    cum = np.concatenate([[0], np.cumsum(sizes.astype(np.int64))])
    q = (cum * den) // num
    return (q[1:] - q[:-1]).astype(np.int64)


def block_punched_mask(F, C, KH, KW, Bf, Bc, rate, seed, stream=0):
    """Block-punched mask for W[F][C][KH][KW]: blocks of Bf filters x Bc channels
    (x all taps); inside a block, pruning rate `rate` (e.g. 2, 2.5, Fraction(4))
    of the (channel, kh, kw) positions are punched, the same ones in every
    filter of the block.  Edge blocks may be partial."""
    rate = Fraction(rate).limit_denominator(1000)
    G = -(-F // Bf)
    NB = -(-C // Bc)
    T = KH * KW
    Pmax = Bc * T
    # channels present in each channel block (the last one may be partial)
    nch = np.minimum(C, (np.arange(NB) + 1) * Bc) - np.arange(NB) * Bc
    sizes = np.tile(nch * T, G).astype(np.int64)            # block b = g*NB + cb
    keep = _keep_counts(sizes, rate)
    # one random key per (block, position); the `keep[b]` smallest keys survive
    keys = prng.u64(seed, stream, G * NB * Pmax).reshape(G * NB, Pmax)
    exists = np.arange(Pmax)[None, :] < sizes[:, None]
    keys = np.where(exists, keys >> np.uint64(1), np.uint64(0xFFFFFFFFFFFFFFFF))
    rank = np.argsort(np.argsort(keys, axis=1, kind="stable"), axis=1, kind="stable")
    kept = (rank < keep[:, None]) & exists                   # [G*NB][Pmax]
    # position p inside a block = (c_local, kh, kw) row-major
    per_group = kept.reshape(G, NB * Bc, KH, KW)[:, :C]      # [G][C][KH][KW]
    mask = np.repeat(per_group, Bf, axis=0)[:F].astype(np.uint8)
    return np.ascontiguousarray(mask)


def fc_block_mask(OUT, IN, Br, Bcol, rate, seed, stream=0):
    """Block-based mask for W[OUT][IN]: blocks of Br rows x Bcol columns; whole
    columns are pruned inside each block (rate as above)."""
    return block_punched_mask(OUT, IN, 1, 1, Br, Bcol, rate, seed, stream).reshape(OUT, IN)


def pattern_library(n_pat, seed, stream=0):
    """n_pat distinct 3x3 patterns with 4 kept taps each, the centre always kept.
    Returns uint8 [n_pat][9] of 0/1 in tap order kh*3+kw."""
    others = [0, 1, 2, 3, 5, 6, 7, 8]
    combos = [(a, b, c) for i, a in enumerate(others) for j, b in enumerate(others)
              for c in others[j + 1:] if j > i]
    keys = prng.u64(seed, (stream << 32) + 0x7A77, len(combos))
    chosen = sorted(np.argsort(keys, kind="stable")[:n_pat].tolist())
    lib = np.zeros((n_pat, 9), dtype=np.uint8)
    for p, ci in enumerate(chosen):
        lib[p, 4] = 1
        lib[p, list(combos[ci])] = 1
    return lib


def pattern_mask(F, C, library, dead_fraction, seed, stream=0):
    """Pattern + connectivity mask for W[F][C][3][3]: every kernel gets a library
    pattern (uniform iid), then round_half_up(dead_fraction*F*C) whole kernels,
    chosen uniformly over all (f, c), are removed.  Returns (mask, pat_id) with
    pat_id uint8 [F][C], 255 for a removed kernel."""
    n_pat = library.shape[0]
    ids = (prng.u64(seed, (stream << 32) + 1, F * C) % np.uint64(n_pat)).astype(np.uint8)
    n_dead = int(np.floor(dead_fraction * F * C + 0.5))
    keys = prng.u64(seed, (stream << 32) + 2, F * C)
    dead = np.argsort(keys, kind="stable")[:n_dead]
    ids[dead] = 255
    mask = np.zeros((F * C, 9), dtype=np.uint8)
    alive = ids != 255
    mask[alive] = library[ids[alive]]
    return mask.reshape(F, C, 3, 3), ids.reshape(F, C)
