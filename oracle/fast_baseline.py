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


def prune_and_compact_fast_mt(w, v, tensors, vecs, groups, n_prune: int, threads: int,
                              slab: int = 1 << 22):
    """The same variant on `threads` host threads (numpy's loops run outside the interpreter
    lock).  The selection is by counting: a histogram of the keys' upper 16 bits over slabs of
    the prunable weights, the bucket that holds the P-th smallest key, then a partition of that
    bucket's keys alone; masks, the zero-filter scan and the gathers go tensor by tensor.
    Same results and layouts as ``prune_and_compact_fast``."""
    from concurrent.futures import ThreadPoolExecutor
    w = np.asarray(w, dtype=np.float32)
    bits = w.view(np.uint32)
    numel = lambda t: t.out_ch * t.in_ch * t.kh * t.kw
    slabs = []                       # (global index of the first weight, arena offset, length)
    g = 0
    for t in tensors:
        if not t.prunable:
            continue
        m = numel(t)
        for a in range(0, m, slab):
            slabs.append((g + a, t.offset + a, min(slab, m - a)))
        g += m
    n = g
    absmask = np.uint32(0x7FFFFFFF)
    w_sparse = w.copy()
    mask = np.ones(n, dtype=np.uint8)
    with ThreadPoolExecutor(max_workers=max(1, threads)) as pool:
        if n_prune > 0:
            def hist(s):
                k = bits[s[1]:s[1] + s[2]] & absmask
                if k.size and int(k.max()) > 0x7F800000:
                    raise ValueError("NaN among prunable weights")
                return np.bincount(k >> np.uint32(15), minlength=1 << 16)
            total = np.zeros(1 << 16, dtype=np.int64)
            for h in pool.map(hist, slabs):
                total += h
            cum = np.cumsum(total)
            b = int(np.searchsorted(cum, n_prune, side="left"))     # first bucket with cum >= P
            r = n_prune - (int(cum[b - 1]) if b else 0)              # rank inside the bucket

            def cands(s):
                k = bits[s[1]:s[1] + s[2]] & absmask
                idx = np.flatnonzero((k >> np.uint32(15)) == b)
                return k[idx], idx.astype(np.int64) + s[0]
            parts = list(pool.map(cands, slabs))
            ck = np.concatenate([p[0] for p in parts])
            cg = np.concatenate([p[1] for p in parts])               # ascending global index
            t_key = np.partition(ck, r - 1)[r - 1]
            need = r - int((ck < t_key).sum())
            g_cut = int(cg[np.flatnonzero(ck == t_key)[need - 1]])   # ties go by ascending index

            def apply(s):
                k = bits[s[1]:s[1] + s[2]] & absmask
                rem = k < t_key
                if s[0] <= g_cut:
                    tie = np.flatnonzero(k == t_key)
                    rem[tie[tie + s[0] <= g_cut]] = True
                w_sparse[s[1]:s[1] + s[2]][rem] = 0.0
                mask[s[0]:s[0] + s[2]][rem] = 0
            list(pool.map(apply, slabs))
        else:
            for s in slabs:
                if s[2] and int((bits[s[1]:s[1] + s[2]] & absmask).max()) > 0x7F800000:
                    raise ValueError("NaN among prunable weights")
        sb = w_sparse.view(np.uint32)

        def scan(t):
            nz = (sb[t.offset:t.offset + numel(t)] & absmask) != 0
            return nz.reshape(t.out_ch, -1).any(axis=1)
        alive = [np.array([bool(gr.pinned)] * gr.width) for gr in groups]
        for t, a in zip(tensors, pool.map(scan, tensors)):
            alive[t.out_group] |= a
        keep = [np.flatnonzero(a) for a in alive]
        new_width = np.array([k.size for k in keep], dtype=np.uint32)

        def gather(t):
            x = w_sparse[t.offset:t.offset + numel(t)]
            x = x.reshape(t.out_ch, t.in_ch // t.in_mult, t.in_mult * t.kh * t.kw)
            return x[keep[t.out_group]][:, keep[t.in_group]].reshape(-1)
        out_w = list(pool.map(gather, tensors))
    out_v = [np.asarray(v[d.offset:d.offset + d.length])[keep[d.group]] for d in vecs]
    cat = lambda xs: np.concatenate(xs) if xs else np.zeros(0, np.float32)
    return w_sparse, mask, new_width, cat(out_w), cat(out_v)
