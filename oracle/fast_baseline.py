"""A faster CPU implementation of the same pass, for the benchmark's CPU baseline only.
TEST / BENCHMARK INFRASTRUCTURE ONLY.

The oracle (`shifter_oracle.py`) sorts every weight because that is the plain definition;
timing it alone would make any GPU figure look good.  This module reaches the same result
the way a careful CPU program would - selection instead of a full sort (numpy's
introselect `partition` on the magnitude keys, then the ties by index), vectorised
masking, `any` reductions and fancy-index gathers - so that the benchmark can quote a
baseline that is not a strawman.  It is not the oracle of record: `tests/` checks it
against the oracle bit for bit, and nothing but the benchmark's CPU leg and that test
imports it.  It shares no code with the HIP library.

Steps as in the oracle: Sec. II-A / III-C (magnitude ranking, mask), Sec. III-D Module 2
(zero filters), Module 3 / Algorithm 1 on channel groups, Module 4 / Algorithm 2.
"""
from __future__ import annotations

import numpy as np


def prune_and_compact_fast(w, v, tensors, vecs, groups, n_prune: int):
    """One variant.  Returns (w_sparse, mask, new_width, compacted weights, compacted
    vectors) with the oracle's layouts."""
    w = np.asarray(w, dtype=np.float32)
    bits = w.view(np.uint32)
    pr = [t for t in tensors if t.prunable]
    keys = np.concatenate([bits[t.offset:t.offset + t.out_ch * t.in_ch * t.kh * t.kw] for t in pr]) \
        if pr else np.zeros(0, np.uint32)
    keys = keys & np.uint32(0x7FFFFFFF)
    n = keys.size
    if (keys > 0x7F800000).any():
        raise ValueError("NaN among prunable weights")
    removed = np.zeros(n, dtype=bool)
    if n_prune > 0:
        kth = np.partition(keys, n_prune - 1)[n_prune - 1]      # the P-th smallest key
        removed = keys < kth
        need = n_prune - int(removed.sum())
        removed[np.flatnonzero(keys == kth)[:need]] = True       # ties by ascending index
    mask = (~removed).astype(np.uint8)
    w_sparse = w.copy()
    g = 0
    for t in pr:
        m = t.out_ch * t.in_ch * t.kh * t.kw
        seg = w_sparse[t.offset:t.offset + m]
        seg[removed[g:g + m]] = 0.0
        g += m
    sb = w_sparse.view(np.uint32)
    alive = [np.array([bool(gr.pinned)] * gr.width) for gr in groups]
    for t in tensors:
        nz = (sb[t.offset:t.offset + t.out_ch * t.in_ch * t.kh * t.kw] & np.uint32(0x7FFFFFFF)) != 0
        alive[t.out_group] |= nz.reshape(t.out_ch, -1).any(axis=1)
    keep = [np.flatnonzero(a) for a in alive]
    new_width = np.array([k.size for k in keep], dtype=np.uint32)
    out_w = []
    for t in tensors:
        x = w_sparse[t.offset:t.offset + t.out_ch * t.in_ch * t.kh * t.kw]
        x = x.reshape(t.out_ch, t.in_ch // t.in_mult, t.in_mult * t.kh * t.kw)
        out_w.append(x[keep[t.out_group]][:, keep[t.in_group]].reshape(-1))
    out_v = [np.asarray(v[d.offset:d.offset + d.length])[keep[d.group]] for d in vecs]
    cat = lambda xs: np.concatenate(xs) if xs else np.zeros(0, np.float32)
    return w_sparse, mask, new_width, cat(out_w), cat(out_v)
