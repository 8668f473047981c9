"""CPU oracle for the prune-and-compact pass.  TEST INFRASTRUCTURE ONLY.

Plain, slow, single-threaded numpy written from the paper's definitions.  It shares
no code with the HIP library and must never be imported by the product path: only
the tests, the smoke check and the benchmark's CPU-baseline leg call it.

The method is exact, so each function is the plain definition written out:

* ``select_pruned``      - unstructured magnitude ranking (Sec. II-A "weights with
  the lowest magnitude are masked", Sec. III-C): a *full stable sort* of |w| over all
  prunable weights; the first P of the sorted order are removed.  A stable sort
  breaks ties by ascending global index, so the selection is unique.
* ``apply_mask``         - sparse model of Sec. III-C: same shapes, zeros in place.
* ``dead_channel_scan``  - Module 2 (Sparsity Analyser): kernels that are entirely
  zero, and channels in which every kernel is zero.
* ``propagate_groups``   - Module 3 / Algorithm 1 (Prune Planner), stated on channel
  groups so that residual adds are covered: a channel of a group is prunable when
  every filter writing it is entirely zero.
* ``compact``            - Module 4 / Algorithm 2 (Model Pruner): new smaller layers
  holding the surviving out-channels, their per-channel vectors, and the surviving
  in-channels.
* ``kernel_scan`` / ``propagate_groups_fixpoint`` - an extension beyond Algorithm 1's
  single pass, on Module 2's kernel-level zero index: a channel also goes when every
  non-zero kernel writing it reads a removed channel, or when no surviving filter reads
  it through a non-zero kernel; repeated until nothing changes (the largest set of
  channels that is consistent with both rules).

Every function is pinned by tests that do not go through it (brute-force rank
counting, closed forms, hand-enumerated toy networks, Algorithm 1 on a chain, forward
equivalence of the compacted network); none is "parity unpinned".

Inputs are the descriptor objects of the synthetic-network module (attributes only:
offset, out_ch, in_ch, kh, kw, in_mult, out_group, in_group, prunable / offset,
length, group / width, pinned) and numpy arenas.
"""
from __future__ import annotations

from dataclasses import dataclass
from typing import List, Sequence, Tuple

import numpy as np

FLAG_JOINT = 0            # residual-add groups pruned jointly
FLAG_FREEZE_RESIDUAL = 1  # Sec. IV-B.2: skip / downsample connections left untouched
FLAG_FIXPOINT = 2         # liveness fixpoint on the kernel-level zero index (extension)


def _numel(t) -> int:
    return t.out_ch * t.in_ch * t.kh * t.kw


def prunable_ranges(tensors) -> List[Tuple[int, int, int]]:
    """Global index space: prunable tensors in descriptor order, each row-major.

    Returns (tensor index, first global index, element count) triples."""
    out, g = [], 0
    for ti, t in enumerate(tensors):
        if t.prunable:
            out.append((ti, g, _numel(t)))
            g += _numel(t)
    return out


def gather_prunable(w: np.ndarray, tensors) -> np.ndarray:
    parts = [w[t.offset:t.offset + _numel(t)] for t in tensors if t.prunable]
    if not parts:
        return np.zeros(0, dtype=np.float32)
    return np.concatenate(parts)


@dataclass
class Selection:
    n_prune: int
    pruned: np.ndarray      # global indices of the removed weights (sorted order)
    thr_value: float        # |w| of the P-th pair of the sorted order (0.0 if P == 0)
    thr_index: int          # its global index (-1 if P == 0)


def select_pruned(w: np.ndarray, tensors, n_prune: Sequence[int]) -> List[Selection]:
    """Sort all (|w_g|, g) pairs ascending; the first P are removed.

    One sort serves every P of a portfolio (the weights are the same dense arena)."""
    a = np.abs(gather_prunable(w, tensors))
    if np.isnan(a).any():
        raise ValueError("NaN among prunable weights: magnitude order undefined")
    order = np.argsort(a, kind="stable")
    out = []
    for p in n_prune:
        p = int(p)
        if not 0 <= p <= a.size:
            raise ValueError("prune count outside [0, N]")
        pruned = order[:p]
        if p == 0:
            out.append(Selection(0, pruned, 0.0, -1))
        else:
            last = int(order[p - 1])
            out.append(Selection(p, pruned, float(a[last]), last))
    return out


def apply_mask(w: np.ndarray, tensors, sel: Selection) -> Tuple[np.ndarray, np.ndarray]:
    """mask[g] = 0 for removed weights, else 1; removed weights become +0.0."""
    n = sum(_numel(t) for t in tensors if t.prunable)
    mask = np.ones(n, dtype=np.uint8)
    mask[sel.pruned] = 0
    w_sparse = w.copy()
    for ti, g0, cnt in prunable_ranges(tensors):
        t = tensors[ti]
        seg = w_sparse[t.offset:t.offset + cnt]
        seg[mask[g0:g0 + cnt] == 0] = np.float32(0.0)
    return w_sparse, mask


def dead_channel_scan(w_sparse: np.ndarray, tensors):
    """Per tensor: which output filters and which input features hold a non-zero.

    A kernel is the kh x kw slice of one (filter, input feature) pair; a filter is
    alive if any of its kernels holds a non-zero, an input feature likewise over all
    filters.  -0.0 compares equal to zero."""
    out_alive, in_alive = [], []
    for t in tensors:
        x = w_sparse[t.offset:t.offset + _numel(t)].reshape(t.out_ch, t.in_ch,
                                                             t.kh * t.kw)
        kernel_nz = (x != 0).any(axis=2)            # [O, I] zero-kernel index
        out_alive.append(kernel_nz.any(axis=1).astype(np.uint8))
        in_alive.append(kernel_nz.any(axis=0).astype(np.uint8))
    return out_alive, in_alive


@dataclass
class Plan:
    alive: List[np.ndarray]      # per group, uint8[width]
    index_map: List[np.ndarray]  # per group, int32[width]: new index or -1
    keep: List[np.ndarray]       # per group, uint32[new_width]: old indices ascending
    new_width: np.ndarray        # uint32[n_groups]


def propagate_groups(tensors, groups, out_alive, flags: int = FLAG_JOINT) -> Plan:
    """Single-pass prune plan.

    A channel c of group G survives iff G is pinned or some tensor whose filters write
    G has a non-zero filter c.  On a chain this is Algorithm 1: C_out(L_n) are the
    zero filters of L_n and C_in(L_n) are the zero filters of L_{n-1}; the first layer
    reads the pinned input group, so its C_in is empty.  With FLAG_FREEZE_RESIDUAL a
    group written by more than one tensor is left whole."""
    alive, index_map, keep = [], [], []
    for gi, g in enumerate(groups):
        producers = [ti for ti, t in enumerate(tensors) if t.out_group == gi]
        a = np.zeros(g.width, dtype=np.uint8)
        frozen = g.pinned or ((flags & FLAG_FREEZE_RESIDUAL) and len(producers) > 1)
        if frozen:
            a[:] = 1
        for ti in producers:
            a |= out_alive[ti]
        k = np.flatnonzero(a).astype(np.uint32)
        m = np.full(g.width, -1, dtype=np.int32)
        m[k] = np.arange(k.size, dtype=np.int32)
        alive.append(a)
        keep.append(k)
        index_map.append(m)
    new_width = np.array([k.size for k in keep], dtype=np.uint32)
    return Plan(alive, index_map, keep, new_width)


def kernel_scan(w_sparse: np.ndarray, tensors) -> List[np.ndarray]:
    """Module 2's kernel-level index: nz[t][o, i] = 1 iff the kh x kw kernel of filter o
    and input feature i of tensor t holds a non-zero (-0.0 counts as zero)."""
    out = []
    for t in tensors:
        x = w_sparse[t.offset:t.offset + _numel(t)].reshape(t.out_ch, t.in_ch,
                                                             t.kh * t.kw)
        out.append((x != 0).any(axis=2).astype(np.uint8))
    return out


def propagate_groups_fixpoint(tensors, groups, kernel_nz, flags: int = FLAG_FIXPOINT) -> Plan:
    """Prune plan with liveness propagated to a fixpoint.

    Start from every channel alive.  A channel c of a group that is neither pinned nor
    frozen stays alive only if
      * it is produced: some tensor writing the group has, in filter c, a non-zero kernel
        whose input feature belongs to an alive channel of that tensor's in-group, and
      * it is read: some tensor reading the group has a non-zero kernel on one of the
        input features of c in a filter whose out-channel is alive.
    Channels failing either rule are removed and the rules are applied again until no
    channel changes.  Removal only ever makes more channels fail, so the result is the
    largest rule-consistent set whatever the order of removal."""
    n_g = len(groups)
    producers = [[ti for ti, t in enumerate(tensors) if t.out_group == gi] for gi in range(n_g)]
    consumers = [[ti for ti, t in enumerate(tensors) if t.in_group == gi] for gi in range(n_g)]
    frozen = [bool(g.pinned) or bool((flags & FLAG_FREEZE_RESIDUAL) and len(producers[gi]) > 1)
              for gi, g in enumerate(groups)]
    alive = [np.ones(g.width, dtype=bool) for g in groups]
    changed = True
    while changed:
        changed = False
        new_alive = []
        for gi, g in enumerate(groups):
            if frozen[gi]:
                new_alive.append(alive[gi])
                continue
            produced = np.zeros(g.width, dtype=bool)
            for ti in producers[gi]:
                t = tensors[ti]
                feat_alive = np.repeat(alive[t.in_group], t.in_mult)        # per input feature
                produced |= (kernel_nz[ti].astype(bool) & feat_alive[None, :]).any(axis=1)
            read = np.zeros(g.width, dtype=bool)
            for ti in consumers[gi]:
                t = tensors[ti]
                feat_read = (kernel_nz[ti].astype(bool) & alive[t.out_group][:, None]).any(axis=0)
                read |= feat_read.reshape(g.width, t.in_mult).any(axis=1)
            a = alive[gi] & produced & read
            changed = changed or not np.array_equal(a, alive[gi])
            new_alive.append(a)
        alive = new_alive
    alive_u8, index_map, keep = [], [], []
    for gi, g in enumerate(groups):
        a = alive[gi].astype(np.uint8)
        k = np.flatnonzero(a).astype(np.uint32)
        m = np.full(g.width, -1, dtype=np.int32)
        m[k] = np.arange(k.size, dtype=np.int32)
        alive_u8.append(a)
        keep.append(k)
        index_map.append(m)
    new_width = np.array([k.size for k in keep], dtype=np.uint32)
    return Plan(alive_u8, index_map, keep, new_width)


@dataclass
class Compacted:
    w: np.ndarray                 # compacted weight arena (dense, descriptor order)
    v: np.ndarray                 # compacted vector arena
    tensor_shapes: List[Tuple[int, int, int, int, int]]  # (offset, O', I', kh, kw)
    vec_shapes: List[Tuple[int, int]]                    # (offset, len')


def compact(w_sparse: np.ndarray, vecs_arena: np.ndarray, tensors, vecs, plan: Plan
            ) -> Compacted:
    """Rebuild every layer without its prunable channels (Algorithm 2).

    W'[o', i', :, :] = W[keep_out[o'], col(i'), :, :] where, for a tensor reading m
    input features per channel, col(i') = keep_in[i' // m] * m + i' % m.  Every vector
    attached to a group keeps the entries of that group's surviving channels."""
    w_parts, shapes, off = [], [], 0
    for t in tensors:
        ko = plan.keep[t.out_group].astype(np.int64)
        ki = plan.keep[t.in_group].astype(np.int64)
        m = t.in_mult
        cols = (ki[:, None] * m + np.arange(m, dtype=np.int64)[None, :]).reshape(-1)
        x = w_sparse[t.offset:t.offset + _numel(t)].reshape(t.out_ch, t.in_ch, t.kh,
                                                             t.kw)
        y = x[ko][:, cols]
        shapes.append((off, int(ko.size), int(cols.size), t.kh, t.kw))
        w_parts.append(y.reshape(-1))
        off += y.size
    v_parts, vshapes, voff = [], [], 0
    for vd in vecs:
        k = plan.keep[vd.group].astype(np.int64)
        y = vecs_arena[vd.offset:vd.offset + vd.length][k]
        vshapes.append((voff, int(k.size)))
        v_parts.append(y)
        voff += y.size
    w_out = np.concatenate(w_parts) if w_parts else np.zeros(0, np.float32)
    v_out = np.concatenate(v_parts) if v_parts else np.zeros(0, np.float32)
    return Compacted(w_out.astype(np.float32, copy=False),
                     v_out.astype(np.float32, copy=False), shapes, vshapes)


@dataclass
class VariantResult:
    sel: Selection
    w_sparse: np.ndarray
    mask: np.ndarray
    out_alive: List[np.ndarray]
    in_alive: List[np.ndarray]
    plan: Plan
    compacted: Compacted


def prune_and_compact(w, v, tensors, vecs, groups, n_prune: Sequence[int],
                      flags: int = FLAG_JOINT) -> List[VariantResult]:
    """The whole pass for every prune count of a portfolio (one sort, then per
    variant: mask, scan, plan, rebuild)."""
    res = []
    for sel in select_pruned(w, tensors, n_prune):
        w_sparse, mask = apply_mask(w, tensors, sel)
        out_alive, in_alive = dead_channel_scan(w_sparse, tensors)
        if flags & FLAG_FIXPOINT:
            plan = propagate_groups_fixpoint(tensors, groups, kernel_scan(w_sparse, tensors),
                                             flags)
        else:
            plan = propagate_groups(tensors, groups, out_alive, flags)
        res.append(VariantResult(sel, w_sparse, mask, out_alive, in_alive, plan,
                                 compact(w_sparse, v, tensors, vecs, plan)))
    return res
