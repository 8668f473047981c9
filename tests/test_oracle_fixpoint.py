"""Pins for the oracle's liveness fixpoint (kernel_scan, propagate_groups_fixpoint): none
of them goes through the function under test for its expected values.

The plan extends Algorithm 1's single pass on Module 2's kernel-level zero index
(Sec. III-D): a channel also goes when every non-zero kernel writing it reads a removed
channel, or when no surviving filter reads it through a non-zero kernel.  The expected
values here come from a hand-worked chain, from an exhaustive search over all channel
subsets of tiny networks (the result must be the union of every rule-consistent subset),
and from the forward pass of the rebuilt network."""
import itertools
import os
import sys

import numpy as np
import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
sys.path.insert(0, ROOT)
sys.path.insert(0, os.path.dirname(os.path.abspath(__file__)))
from oracle import shifter_oracle as O  # noqa: E402
from paper_2309_06973_amd import synth  # noqa: E402

import forward_ref  # noqa: E402


class T:
    def __init__(self, offset, o, i, kh, kw, og, ig, prunable=1, in_mult=1):
        self.offset, self.out_ch, self.in_ch, self.kh, self.kw = offset, o, i, kh, kw
        self.out_group, self.in_group, self.prunable, self.in_mult = og, ig, prunable, in_mult


class G:
    def __init__(self, width, pinned=0):
        self.width, self.pinned = width, pinned


def dense_net(mats, groups, wiring, in_mults=None, k=1):
    """Tensors from explicit [O, I] 0/1 kernel patterns (k x k kernels whose first weight
    carries the pattern).  wiring[t] = (in_group, out_group)."""
    tensors, parts, off = [], [], 0
    for ti, m in enumerate(mats):
        m = np.asarray(m, dtype=np.float32)
        o, i = m.shape
        x = np.zeros((o, i, k * k), dtype=np.float32)
        x[:, :, (ti * 5) % (k * k)] = m * (1.0 + ti)        # a different tap per tensor
        ig, og = wiring[ti]
        tensors.append(T(off, o, i, k, k, og, ig, 1, (in_mults or {}).get(ti, 1)))
        parts.append(x.reshape(-1))
        off += x.size
    return tensors, groups, np.concatenate(parts)


# ----------------------------------------------------------------------------- kernel scan
def test_kernel_scan_against_loops():
    rng = np.random.Generator(np.random.Philox(11))
    tensors, w, off = [], [], 0
    for (o, i, kh, kw) in [(4, 3, 3, 3), (5, 4, 1, 1), (2, 5, 2, 3)]:
        x = rng.standard_normal(o * i * kh * kw).astype(np.float32)
        x[rng.random(x.size) < 0.7] = 0.0
        x[::11] = -0.0
        tensors.append(T(off, o, i, kh, kw, 1, 0))
        w.append(x)
        off += x.size
    w = np.concatenate(w)
    nz = O.kernel_scan(w, tensors)
    for t, got in zip(tensors, nz):
        khw = t.kh * t.kw
        for o in range(t.out_ch):
            for i in range(t.in_ch):
                base = t.offset + (o * t.in_ch + i) * khw
                want = any(w[base + j] != 0 for j in range(khw))
                assert bool(got[o, i]) == want
    # the channel-level scan is the row / column OR of the kernel-level index
    oa, ia = O.dead_channel_scan(w, tensors)
    for ti in range(len(tensors)):
        assert np.array_equal(oa[ti], nz[ti].any(axis=1).astype(np.uint8))
        assert np.array_equal(ia[ti], nz[ti].any(axis=0).astype(np.uint8))


# ----------------------------------------------------------------------------- hand-worked chain
def cascade_chain():
    """input(2, pinned) -L0-> g1(3) -L1-> g2(3) -L2-> g3(2) -L3-> logits(2, pinned).

    Single pass: only g1 channel 0 goes (L0's filter 0 is all-zero).
    Worked by hand for the fixpoint:
      round 1  g2 ch 1: L1's filter 1 reads only g1 ch 0, which is gone    -> not produced
               g2 ch 2: no filter of L2 has a non-zero kernel on it         -> not read
      round 2  g1 ch 2: its only reader was L1's filter 2 (g2 ch 2, gone)   -> not read
      left: g1 = {1}, g2 = {0}, g3 = {0, 1}."""
    L0 = [[0, 0], [1, 1], [1, 0]]              # g1 x input
    L1 = [[0, 1, 0], [1, 0, 0], [0, 0, 1]]     # g2 x g1
    L2 = [[1, 1, 0], [1, 0, 0]]                # g3 x g2
    L3 = [[1, 0], [0, 1]]                      # logits x g3
    groups = [G(2, 1), G(3), G(3), G(2), G(2, 1)]
    wiring = [(0, 1), (1, 2), (2, 3), (3, 4)]
    return dense_net([L0, L1, L2, L3], groups, wiring, k=3)


def test_fixpoint_hand_worked_cascade():
    tensors, groups, w = cascade_chain()
    oa, _ = O.dead_channel_scan(w, tensors)
    single = O.propagate_groups(tensors, groups, oa)
    assert [k.tolist() for k in single.keep] == [[0, 1], [1, 2], [0, 1, 2], [0, 1], [0, 1]]
    plan = O.propagate_groups_fixpoint(tensors, groups, O.kernel_scan(w, tensors))
    assert [k.tolist() for k in plan.keep] == [[0, 1], [1], [0], [0, 1], [0, 1]]
    assert plan.new_width.tolist() == [2, 1, 1, 2, 2]
    for gi in range(len(groups)):
        m, k = plan.index_map[gi], plan.keep[gi]
        assert np.array_equal(m[k], np.arange(k.size)) and (m >= 0).sum() == k.size
        assert np.array_equal(plan.alive[gi], (m >= 0).astype(np.uint8))


# ----------------------------------------------------------------------------- exhaustive search
def consistent(tensors, groups, nz, frozen, alive):
    """Pure-Python statement of the two rules for one candidate assignment."""
    for gi, g in enumerate(groups):
        for c in range(g.width):
            if frozen[gi]:
                if not alive[gi][c]:
                    return False
                continue
            if not alive[gi][c]:
                continue
            produced = False
            for ti, t in enumerate(tensors):
                if t.out_group != gi:
                    continue
                for i in range(t.in_ch):
                    if nz[ti][c][i] and alive[t.in_group][i // t.in_mult]:
                        produced = True
            read = False
            for ti, t in enumerate(tensors):
                if t.in_group != gi:
                    continue
                for o in range(t.out_ch):
                    for q in range(t.in_mult):
                        if nz[ti][o][c * t.in_mult + q] and alive[t.out_group][o]:
                            read = True
            if not (produced and read):
                return False
    return True


def union_of_consistent_subsets(tensors, groups, nz, flags):
    n_prod = [sum(1 for t in tensors if t.out_group == gi) for gi in range(len(groups))]
    frozen = [bool(g.pinned) or bool((flags & O.FLAG_FREEZE_RESIDUAL) and n_prod[gi] > 1)
              for gi, g in enumerate(groups)]
    free = [(gi, c) for gi, g in enumerate(groups) if not frozen[gi] for c in range(g.width)]
    assert len(free) <= 14
    union = [np.zeros(g.width, dtype=bool) for g in groups]
    for bits in itertools.product((False, True), repeat=len(free)):
        alive = [np.ones(g.width, dtype=bool) for g in groups]
        for (gi, c), b in zip(free, bits):
            alive[gi][c] = b
        if consistent(tensors, groups, nz, frozen, alive):
            for gi in range(len(groups)):
                union[gi] |= alive[gi]
    for gi in range(len(groups)):
        if frozen[gi]:
            union[gi][:] = True
    return union


def random_tiny_net(seed, residual):
    rng = np.random.Generator(np.random.Philox(1000 + seed))
    dens = 0.35 + 0.3 * rng.random()
    pat = lambda o, i: (rng.random((o, i)) < dens).astype(np.float32)
    if not residual:
        # chain with a flatten in front of the last layer (in_mult = 2)
        groups = [G(2, 1), G(4), G(4), G(3), G(2, 1)]
        wiring = [(0, 1), (1, 2), (2, 3), (3, 4)]
        mats = [pat(4, 2), pat(4, 4), pat(3, 4), pat(2, 6)]
        return dense_net(mats, groups, wiring, in_mults={3: 2}, k=1 + seed % 2)
    # stem -> stream(4); block: stream -> mid(3) -> stream (two producers of the stream)
    groups = [G(2, 1), G(4), G(3), G(2, 1)]
    wiring = [(0, 1), (1, 2), (2, 1), (1, 3)]
    mats = [pat(4, 2), pat(3, 4), pat(4, 3), pat(2, 4)]
    return dense_net(mats, groups, wiring, k=1)


@pytest.mark.parametrize("seed", range(8))
@pytest.mark.parametrize("residual", [False, True])
def test_fixpoint_is_union_of_all_consistent_subsets(seed, residual):
    tensors, groups, w = random_tiny_net(seed, residual)
    nz = O.kernel_scan(w, tensors)
    for flags in ((O.FLAG_FIXPOINT, O.FLAG_FIXPOINT | O.FLAG_FREEZE_RESIDUAL) if residual
                  else (O.FLAG_FIXPOINT,)):
        want = union_of_consistent_subsets(tensors, groups, [m.tolist() for m in nz], flags)
        plan = O.propagate_groups_fixpoint(tensors, groups, nz, flags)
        for gi in range(len(groups)):
            assert np.array_equal(plan.alive[gi].astype(bool), want[gi]), (seed, residual, gi)
        # never more than the single pass keeps
        oa, _ = O.dead_channel_scan(w, tensors)
        single = O.propagate_groups(tensors, groups, oa, flags & O.FLAG_FREEZE_RESIDUAL)
        for gi in range(len(groups)):
            assert not (plan.alive[gi] & ~single.alive[gi] & 1).any()


def test_exhaustive_search_sees_planted_mistakes(monkeypatch):
    """A forward-only or a backward-only propagation must disagree with the search."""
    tensors, groups, w = cascade_chain()
    nz = O.kernel_scan(w, tensors)
    want = union_of_consistent_subsets(tensors, groups, [m.tolist() for m in nz], O.FLAG_FIXPOINT)

    def one_sided(forward):
        alive = [np.ones(g.width, dtype=bool) for g in groups]
        for _ in range(8):
            for gi, g in enumerate(groups):
                if g.pinned:
                    continue
                ok = np.zeros(g.width, dtype=bool)
                for ti, t in enumerate(tensors):
                    if forward and t.out_group == gi:
                        ok |= (nz[ti].astype(bool) & alive[t.in_group][None, :]).any(axis=1)
                    if not forward and t.in_group == gi:
                        ok |= (nz[ti].astype(bool) & alive[t.out_group][:, None]).any(axis=0)
                alive[gi] &= ok
        return alive

    for forward in (True, False):
        got = one_sided(forward)
        assert any(not np.array_equal(got[gi], want[gi]) for gi in range(len(groups)))


# ----------------------------------------------------------------------------- whole pass
def equiv(spec, w, v, p, flags, dtype):
    r = O.prune_and_compact(w, v, spec.tensors, spec.vecs, spec.groups, [p], flags)[0]
    if (r.plan.new_width == 0).any():
        pytest.skip("layer collapse at this sparsity")
    err = forward_ref.forward_equivalence(
        spec, r.w_sparse, v, r.plan.alive, r.compacted.w, r.compacted.v,
        r.compacted.tensor_shapes, r.compacted.vec_shapes, seed=synth.SEED_BASE + 1000,
        batch=2, dtype=dtype)
    return r, err


@pytest.mark.parametrize("c,s", [(1, 0.9), (3, 0.8), (3, 0.93)])
def test_forward_equivalence_with_fixpoint(c, s):
    import torch
    spec, w, v = synth.generate_config(c)
    p = synth.prune_count(spec.n_prunable, s)
    r1, _ = equiv(spec, w, v, p, 0, torch.float64)
    r2, err = equiv(spec, w, v, p, O.FLAG_FIXPOINT, torch.float64)
    assert err <= 1e-12
    assert r2.compacted.w.size <= r1.compacted.w.size
    for gi in range(len(spec.groups)):
        assert not (r2.plan.alive[gi] & ~r1.plan.alive[gi] & 1).any()


def test_fixpoint_removes_more_on_a_planted_chain():
    """A chain in which one filter reads only a removed channel and one channel is read by
    nobody: the rebuilt network is smaller than the single pass's and computes the same."""
    import torch
    spec = synth.chain_spec([6, 5, 7], k=3)
    w, v = synth.generate_weights(spec, 5)
    t0, t1, t2 = spec.tensors[0], spec.tensors[1], spec.tensors[2]
    x0 = w[t0.offset:t0.offset + t0.numel].reshape(t0.out_ch, t0.in_ch, 9)
    x1 = w[t1.offset:t1.offset + t1.numel].reshape(t1.out_ch, t1.in_ch, 9)
    x2 = w[t2.offset:t2.offset + t2.numel].reshape(t2.out_ch, t2.in_ch, 9)
    x0[2] = 0                 # a1 channel 2: zero filter (single pass removes it)
    x1[3, :2] = 0
    x1[3, 3:] = 0             # a2 channel 3 reads only a1 channel 2 -> goes at the fixpoint
    x2[:, 1] = 0              # a2 channel 1 is read by nobody      -> goes at the fixpoint
    r1, e1 = equiv(spec, w, v, 0, 0, torch.float64)
    r2, e2 = equiv(spec, w, v, 0, O.FLAG_FIXPOINT, torch.float64)
    assert e1 <= 1e-12 and e2 <= 1e-12
    assert r1.plan.keep[t1.out_group].tolist() == [0, 1, 2, 3, 4]
    assert r2.plan.keep[t1.out_group].tolist() == [0, 2, 4]
    assert r2.plan.keep[t0.out_group].tolist() == [0, 1, 3, 4, 5]
