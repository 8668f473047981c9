"""Pins for the CPU oracle: every check here goes around the oracle's own code path
(brute-force rank counting, closed forms, hand-enumerated networks, Algorithm 1 and 2
of the paper on a chain, forward equivalence), so a dropped term, wrong index or
transposed operand in the oracle fails at least one of them."""
import os
import sys

import numpy as np
import pytest

sys.path.insert(0, os.path.join(os.path.dirname(__file__), ".."))

from oracle import shifter_oracle as O  # noqa: E402
from paper_2309_06973_amd import synth  # noqa: E402

import forward_ref  # noqa: E402


class T:  # minimal stand-alone descriptor (does not go through the synth builders)
    def __init__(self, offset, o, i, kh, kw, og, ig, prunable=1, in_mult=1):
        self.offset, self.out_ch, self.in_ch, self.kh, self.kw = offset, o, i, kh, kw
        self.out_group, self.in_group, self.prunable, self.in_mult = og, ig, prunable, in_mult


class V:
    def __init__(self, offset, length, group):
        self.offset, self.length, self.group = offset, length, group


class G:
    def __init__(self, width, pinned=0):
        self.width, self.pinned = width, pinned


def flat_model(n):
    """One prunable 'tensor' of n weights (n x 1 x 1 x 1)."""
    return [T(0, n, 1, 1, 1, 1, 0)]


# ----------------------------------------------------------------------------- selection
def brute_force_pruned(a, p):
    """Second definition: g is removed iff fewer than P pairs precede (|w_g|, g)."""
    n = len(a)
    out = []
    for g in range(n):
        rank = 0
        for h in range(n):
            if a[h] < a[g] or (a[h] == a[g] and h < g):
                rank += 1
        if rank < p:
            out.append(g)
    return out


@pytest.mark.parametrize("kind", synth.ADVERSARIAL_KINDS)
@pytest.mark.parametrize("n", [1, 7, 64, 257])
def test_selection_matches_rank_counting(kind, n):
    w = synth.adversarial_arena(kind, n, seed=n)
    a = [abs(float(x)) for x in w]
    ps = sorted({0, 1, n // 3, n // 2, n - 1, n})
    ps = [p for p in ps if 0 <= p <= n]
    sels = O.select_pruned(w, flat_model(n), ps)
    for p, sel in zip(ps, sels):
        assert sorted(sel.pruned.tolist()) == brute_force_pruned(a, p)
        assert sel.pruned.size == p


def test_selection_multi_tensor_global_index_and_nonprunable():
    # three tensors, middle one not prunable: its weights are never ranked or removed,
    # and the global index skips it.
    ts = [T(0, 2, 2, 1, 1, 1, 0), T(4, 2, 2, 1, 1, 2, 1, prunable=0), T(8, 1, 4, 1, 1, 3, 2)]
    w = np.array([5, -1, 3, 1, 0.1, 0.1, 0.1, 0.1, -1, 7, 1, 2], dtype=np.float32)
    sel = O.select_pruned(w, ts, [4])[0]
    # prunable magnitudes by global index: [5,1,3,1 | 1,7,1,2]; four smallest with ties by
    # index: g=1,3,4,6
    assert sorted(sel.pruned.tolist()) == [1, 3, 4, 6]
    assert (sel.thr_value, sel.thr_index) == (1.0, 6)
    ws, mask = O.apply_mask(w, ts, sel)
    assert mask.tolist() == [1, 0, 1, 0, 0, 1, 0, 1]
    assert ws.tolist() == [5, 0, 3, 0, np.float32(0.1), np.float32(0.1), np.float32(0.1),
                           np.float32(0.1), 0, 7, 0, 2]


def test_selection_closed_forms():
    n = 1000
    for p in (0, 1, 333, 999, 1000):
        sel = O.select_pruned(synth.adversarial_arena("ramp", n), flat_model(n), [p])[0]
        assert sorted(sel.pruned.tolist()) == list(range(p))          # ramp: first P
        sel = O.select_pruned(synth.adversarial_arena("ramp_desc_signed", n),
                              flat_model(n), [p])[0]
        assert sorted(sel.pruned.tolist()) == list(range(n - p, n))   # descending: last P
        sel = O.select_pruned(synth.adversarial_arena("all_equal", n), flat_model(n), [p])[0]
        assert sorted(sel.pruned.tolist()) == list(range(p))          # pure tie-break
        if p:
            assert sel.thr_index == p - 1 and sel.thr_value == 0.5
        sel = O.select_pruned(synth.adversarial_arena("all_zero", n), flat_model(n), [p])[0]
        assert sorted(sel.pruned.tolist()) == list(range(p))


def test_threshold_value_is_kth_order_statistic():
    spec, w, _ = synth.generate_config(1)
    n = spec.n_prunable
    a = np.abs(w)
    for s in (0.1, 0.5, 0.9, 0.99):
        p = synth.prune_count(n, s)
        sel = O.select_pruned(w, spec.tensors, [p])[0]
        assert sel.thr_value == float(np.partition(a, p - 1)[p - 1])
        # counting definition of the k-th smallest
        assert (a < sel.thr_value).sum() < p <= (a <= sel.thr_value).sum()


def test_selection_invariants_and_nesting():
    spec, w, _ = synth.generate_config(1)
    n = spec.n_prunable
    ps = [synth.prune_count(n, 1 - 0.8 ** k) for k in range(1, 12)]
    sels = O.select_pruned(w, spec.tensors, ps)
    a = np.abs(O.gather_prunable(w, spec.tensors))
    prev = None
    for p, sel in zip(ps, sels):
        _, mask = O.apply_mask(w, spec.tensors, sel)
        assert int(mask.sum()) == n - p                       # exact kept count
        assert a[mask == 0].max() <= a[mask == 1].min()       # cut respects magnitude
        if prev is not None:
            assert np.all(mask <= prev)                       # cumulative masks nest
        prev = mask


def test_kept_count_is_round_of_density():
    # a sparse model of compression ratio C keeps one of every C weights (s = 1 - 1/C)
    for n in (24112, 14715584, 1000003):
        for c in (2, 4, 16, 64, 256):
            p = synth.prune_count(n, 1.0 - 1.0 / c)
            assert n - p == int(np.floor(n / c + 0.5))
    assert synth.prune_count(10, 0.0) == 0 and synth.prune_count(10, 1.0) == 10


def test_nan_rejected():
    w = np.array([1, np.nan, 2], dtype=np.float32)
    with pytest.raises(ValueError):
        O.select_pruned(w, flat_model(3), [1])


# ----------------------------------------------------------------------------- mask
def test_mask_semantics_and_zero_bit_pattern():
    w = synth.adversarial_arena("inf_negzero", 4096)
    n = w.size
    for p in (0, 100, n // 2, n):
        sel = O.select_pruned(w, flat_model(n), [p])[0]
        ws, mask = O.apply_mask(w, flat_model(n), sel)
        assert mask.dtype == np.uint8 and int(mask.sum()) == n - p
        bits = ws.view(np.uint32)
        assert np.all(bits[mask == 0] == 0)                       # +0.0, never -0.0
        assert np.array_equal(bits[mask == 1], w.view(np.uint32)[mask == 1])  # untouched
        with np.errstate(invalid="ignore"):
            prod = w * mask                                       # inf * 0 = nan on removed
        fin = np.isfinite(w)
        assert np.array_equal(ws[fin], prod[fin] + np.float32(0.0))
        assert not np.shares_memory(ws, w)


# ----------------------------------------------------------------------------- scan
def loops_scan(x):
    o_n, i_n, kh, kw = x.shape
    out_alive = [0] * o_n
    in_alive = [0] * i_n
    for o in range(o_n):
        for i in range(i_n):
            for y in range(kh):
                for z in range(kw):
                    if x[o, i, y, z] != 0:
                        out_alive[o] = 1
                        in_alive[i] = 1
    return out_alive, in_alive


def test_scan_against_loops_and_enumerated():
    rng = np.random.Generator(np.random.Philox(5))
    shapes = [(5, 4, 3, 3), (3, 7, 1, 1), (4, 1, 2, 2), (1, 6, 3, 1)]
    ts, arena, off = [], [], 0
    for (o, i, kh, kw) in shapes:
        x = rng.standard_normal((o, i, kh, kw)).astype(np.float32)
        x[rng.random(x.shape) < 0.8] = 0
        x[rng.integers(0, o)] = 0            # a dead filter
        x[:, rng.integers(0, i)] = 0         # a dead input channel
        ts.append(T(off, o, i, kh, kw, 0, 0))
        arena.append(x.reshape(-1))
        off += x.size
    w = np.concatenate(arena)
    oa, ia = O.dead_channel_scan(w, ts)
    for t, a, b in zip(ts, oa, ia):
        x = w[t.offset:t.offset + t.out_ch * t.in_ch * t.kh * t.kw].reshape(
            t.out_ch, t.in_ch, t.kh, t.kw)
        eo, ei = loops_scan(x)
        assert a.tolist() == eo and b.tolist() == ei
    # enumerated: 3 filters x 2 input channels x (1x2) kernels
    w = np.array([0, 0, 0, 0,      # filter 0: all zero
                  0, 0, -0.0, 2,   # filter 1: only channel 1 (and a -0.0 that is zero)
                  0, 0, 0, 0], dtype=np.float32)
    oa, ia = O.dead_channel_scan(w, [T(0, 3, 2, 1, 2, 0, 0)])
    assert oa[0].tolist() == [0, 1, 0] and ia[0].tolist() == [0, 1]


# ----------------------------------------------------------------------------- plan
def algorithm1_on_chain(zero_filters_per_layer):
    """The paper's prune planner for a chain: layer n gets C_out = its own zero filters
    and C_in = the zero filters of layer n-1 (empty for n = 0)."""
    plans = []
    for n, c_zero in enumerate(zero_filters_per_layer):
        c_in = set(zero_filters_per_layer[n - 1]) if n > 0 else set()
        plans.append((c_in, set(c_zero)))
    return plans


def make_chain_sparse(widths, dead, seed=3):
    spec = synth.chain_spec(widths)
    w, v = synth.generate_weights(spec, seed)
    for li, filters in enumerate(dead):
        t = spec.tensors[li]
        x = w[t.offset:t.offset + t.numel].reshape(t.out_ch, -1)
        x[list(filters)] = 0
    return spec, w, v


def test_plan_equals_algorithm1_on_chain():
    widths = [6, 5, 7]
    dead = [{1, 4}, set(), {0, 2, 6}]
    spec, w, v = make_chain_sparse(widths, dead)
    oa, _ = O.dead_channel_scan(w, spec.tensors)
    plan = O.propagate_groups(spec.tensors, spec.groups, oa)
    expected = algorithm1_on_chain([sorted(d) for d in dead])
    for n in range(len(widths)):
        t = spec.tensors[n]
        c_in, c_out = expected[n]
        got_out = set(range(t.out_ch)) - set(plan.keep[t.out_group].tolist())
        got_in = set(range(t.in_ch)) - set(plan.keep[t.in_group].tolist())
        assert got_out == c_out and got_in == c_in
    # the classifier consumes the last conv group and keeps all its (pinned) outputs
    cls = spec.tensors[-1]
    assert set(range(cls.in_ch)) - set(plan.keep[cls.in_group].tolist()) == dead[-1]
    assert plan.new_width[cls.out_group] == cls.out_ch
    # map / keep consistency
    for gi, g in enumerate(spec.groups):
        k, m = plan.keep[gi], plan.index_map[gi]
        assert np.all(np.diff(k.astype(np.int64)) > 0)
        assert np.array_equal(m[k], np.arange(k.size))
        assert (m >= 0).sum() == k.size == plan.new_width[gi]


def test_plan_residual_group_is_joint_and_freeze_flag():
    spec = synth.residual_toy_spec(width=6, mid=5, n_blocks=2)
    w, v = synth.generate_weights(spec, 11)
    # tensors: 0 stem(->stream), 1 b1.conv1(->m1), 2 b1.conv2(->stream), 3 b2.conv1(->m2),
    #          4 b2.conv2(->stream), 5 classifier
    def kill(ti, filters):
        t = spec.tensors[ti]
        w[t.offset:t.offset + t.numel].reshape(t.out_ch, -1)[filters] = 0
    kill(0, [0, 1, 2])      # stem dead on 0,1,2
    kill(2, [1, 2, 3])      # block-1 conv2 dead on 1,2,3
    kill(4, [2, 3, 4])      # block-2 conv2 dead on 2,3,4   => only channel 2 dead in all
    kill(1, [0, 4])         # m1 dead on 0,4
    oa, _ = O.dead_channel_scan(w, spec.tensors)
    plan = O.propagate_groups(spec.tensors, spec.groups, oa)
    stream = spec.tensors[0].out_group
    m1 = spec.tensors[1].out_group
    m2 = spec.tensors[3].out_group
    assert plan.keep[stream].tolist() == [0, 1, 3, 4, 5]
    assert plan.keep[m1].tolist() == [1, 2, 3]
    assert plan.keep[m2].tolist() == [0, 1, 2, 3, 4]
    assert plan.keep[0].tolist() == [0, 1, 2]                     # pinned input
    assert plan.index_map[stream].tolist() == [0, 1, -1, 2, 3, 4]
    frozen = O.propagate_groups(spec.tensors, spec.groups, oa, O.FLAG_FREEZE_RESIDUAL)
    assert frozen.keep[stream].tolist() == [0, 1, 2, 3, 4, 5]     # multi-producer: whole
    assert frozen.keep[m1].tolist() == [1, 2, 3]                  # linear connection: pruned
    # invariants: every removed filter is all-zero; residual producers stay consistent
    for ti, t in enumerate(spec.tensors):
        removed = set(range(t.out_ch)) - set(plan.keep[t.out_group].tolist())
        assert all(oa[ti][c] == 0 for c in removed)
    comp = O.compact(w, v, spec.tensors, spec.vecs, plan)
    o_widths = {comp.tensor_shapes[ti][1] for ti in (0, 2, 4)}
    assert o_widths == {5}


# ----------------------------------------------------------------------------- rebuild
def test_compact_enumerated_values():
    # W[o,i,k] = 100*o + 10*i + k so every expected entry can be written down
    o_n, i_n, kk = 4, 3, 2
    x = np.array([[[100 * o + 10 * i + k for k in range(kk)] for i in range(i_n)]
                  for o in range(o_n)], dtype=np.float32)
    ts = [T(0, o_n, i_n, 1, kk, 1, 0)]
    groups = [G(i_n), G(o_n)]
    vec = np.array([7, 8, 9, 10], dtype=np.float32)
    plan = O.Plan(alive=None, index_map=None,
                  keep=[np.array([0, 2], np.uint32), np.array([1, 3], np.uint32)],
                  new_width=np.array([2, 2], np.uint32))
    c = O.compact(x.reshape(-1), vec, ts, [V(0, 4, 1)], plan)
    assert c.tensor_shapes == [(0, 2, 2, 1, 2)]
    assert c.w.tolist() == [100, 101, 120, 121, 300, 301, 320, 321]
    assert c.v.tolist() == [8, 10] and c.vec_shapes == [(0, 2)]
    # flatten -> linear: 2 input features per channel; channel 1 removed of 3
    lin = np.arange(2 * 6, dtype=np.float32)
    ts = [T(0, 2, 6, 1, 1, 1, 0, in_mult=2)]
    plan = O.Plan(None, None, [np.array([0, 2], np.uint32), np.array([0, 1], np.uint32)],
                  np.array([2, 2], np.uint32))
    c = O.compact(lin, np.zeros(0, np.float32), ts, [], plan)
    assert c.w.tolist() == [0, 1, 4, 5, 6, 7, 10, 11]
    assert c.tensor_shapes == [(0, 2, 4, 1, 1)]


def test_compact_size_closed_form_and_subtensor():
    spec, w, v = synth.generate_config(1)
    p = synth.prune_count(spec.n_prunable, 0.9)
    r = O.prune_and_compact(w, v, spec.tensors, spec.vecs, spec.groups, [p])[0]
    total = 0
    for t, (off, o2, i2, kh, kw) in zip(spec.tensors, r.compacted.tensor_shapes):
        assert off == total
        assert o2 == r.plan.new_width[t.out_group]
        assert i2 == r.plan.new_width[t.in_group] * t.in_mult
        total += o2 * i2 * kh * kw
    assert total == r.compacted.w.size
    # the designed-to-die filters (scaled by 1e-4) are all removed at s = 0.9
    removed_any = sum(g.width for g in spec.groups) - int(r.plan.new_width.sum())
    assert removed_any >= 0.2 * sum(g.width for g in spec.groups if not g.pinned)
    # invariants on the sparse model
    for ti, t in enumerate(spec.tensors):
        keep = r.plan.keep[t.out_group]
        if not spec.groups[t.out_group].pinned:                  # single-producer groups
            assert np.all(r.out_alive[ti][keep] == 1)
        dead = np.setdiff1d(np.arange(t.out_ch), keep)
        x = r.w_sparse[t.offset:t.offset + t.numel].reshape(t.out_ch, -1)
        assert not x[dead].any()


# ----------------------------------------------------------------------------- whole pass
def run_equiv(spec, w, v, p, flags=0, batch=4, hw=None, dtype=None):
    import torch
    r = O.prune_and_compact(w, v, spec.tensors, spec.vecs, spec.groups, [p], flags)[0]
    if (r.plan.new_width == 0).any():
        pytest.skip("layer collapse at this sparsity")
    return r, forward_ref.forward_equivalence(
        spec, r.w_sparse, v, r.plan.alive, r.compacted.w, r.compacted.v,
        r.compacted.tensor_shapes, r.compacted.vec_shapes, seed=synth.SEED_BASE + 1000,
        batch=batch, hw=hw, dtype=dtype or torch.float32)


@pytest.mark.parametrize("c,s", [(1, 0.9), (1, 0.5), (3, 0.8), (3, 0.95)])
def test_forward_equivalence_small_configs(c, s):
    import torch
    spec, w, v = synth.generate_config(c)
    p = synth.prune_count(spec.n_prunable, s)
    r, err32 = run_equiv(spec, w, v, p, batch=8)
    assert int(r.plan.new_width.sum()) < sum(g.width for g in spec.groups)  # something pruned
    assert err32 <= 1e-5
    _, err64 = run_equiv(spec, w, v, p, batch=2, dtype=torch.float64)
    assert err64 <= 1e-12


def test_forward_equivalence_residual_toy_and_freeze():
    import torch
    spec = synth.residual_toy_spec(width=8, mid=6, n_blocks=3)
    w, v = synth.generate_weights(spec, 21)
    for ti, dead in ((0, [1, 5]), (2, [1, 5, 6]), (4, [0, 1, 5]), (6, [1, 5, 7]), (1, [2]),
                     (3, [0, 3])):
        t = spec.tensors[ti]
        w[t.offset:t.offset + t.numel].reshape(t.out_ch, -1)[dead] = 0
    for flags in (0, O.FLAG_FREEZE_RESIDUAL):
        r, err = run_equiv(spec, w, v, 0, flags=flags, dtype=torch.float64)
        assert err <= 1e-12
    r = O.prune_and_compact(w, v, spec.tensors, spec.vecs, spec.groups, [0])[0]
    assert r.plan.keep[spec.tensors[0].out_group].tolist() == [0, 2, 3, 4, 6, 7]


def test_forward_equivalence_vgg16_and_resnet50_shapes():
    import torch
    spec, w, v = synth.generate_config(2)
    p = synth.prune_count(spec.n_prunable, 1 - 0.8 ** 10)
    r, err = run_equiv(spec, w, v, p, batch=2)
    assert err <= 1e-5
    assert r.compacted.w.size < 0.8 * spec.n_prunable
    spec, w, v = synth.generate_config(4)
    p = synth.prune_count(spec.n_prunable, 1 - 0.8 ** 12)
    r, err = run_equiv(spec, w, v, p, batch=1, hw=64)
    assert err <= 1e-5


# ----------------------------------------------------------------------------- the pins bite
def test_planted_mistakes_are_caught(monkeypatch):
    """Plant plausible mistakes in the oracle (on the CPU) and check a pin fails."""
    import torch
    spec = synth.residual_toy_spec(width=8, mid=6, n_blocks=2)
    w, v = synth.generate_weights(spec, 33)
    for ti, dead in ((0, [1, 5]), (2, [1, 5]), (4, [1, 5, 2]), (1, [2, 4])):
        t = spec.tensors[ti]
        w[t.offset:t.offset + t.numel].reshape(t.out_ch, -1)[dead] = 0

    stream, m1 = spec.tensors[0].out_group, spec.tensors[1].out_group

    def equiv_err():
        r = O.prune_and_compact(w, v, spec.tensors, spec.vecs, spec.groups, [0])[0]
        if (r.plan.keep[stream].tolist() != [0, 2, 3, 4, 6, 7]
                or r.plan.keep[m1].tolist() != [0, 1, 3, 5]):
            return float("inf")               # enumerated plan pin fails
        try:
            return forward_ref.forward_equivalence(
                spec, r.w_sparse, v, r.plan.alive, r.compacted.w, r.compacted.v,
                r.compacted.tensor_shapes, r.compacted.vec_shapes, seed=5, batch=2,
                dtype=torch.float64)
        except (RuntimeError, ValueError, AssertionError):
            return float("inf")

    assert equiv_err() <= 1e-12
    real_scan = O.dead_channel_scan

    def swapped_scan(ws, ts):                 # transposed operand: in/out roles swapped
        oa, ia = real_scan(ws, ts)
        return [np.resize(x, t.out_ch) for x, t in zip(ia, ts)], oa
    monkeypatch.setattr(O, "dead_channel_scan", swapped_scan)
    assert equiv_err() > 1e-6
    monkeypatch.setattr(O, "dead_channel_scan", real_scan)

    real_plan = O.propagate_groups

    def and_plan(ts, gs, oa, flags=0):        # wrong rule: any dead producer kills channel
        pl = real_plan(ts, gs, oa, flags)
        for gi, g in enumerate(gs):
            prods = [ti for ti, t in enumerate(ts) if t.out_group == gi]
            if not g.pinned and prods:
                a = np.ones(g.width, np.uint8)
                for ti in prods:
                    a &= oa[ti]
                pl.alive[gi] = a
                pl.keep[gi] = np.flatnonzero(a).astype(np.uint32)
        return pl
    monkeypatch.setattr(O, "propagate_groups", and_plan)
    assert equiv_err() > 1e-6
    monkeypatch.setattr(O, "propagate_groups", real_plan)
    assert equiv_err() <= 1e-12

    # unstable tie-break (descending index among equals) fails the rank-counting pin
    w_eq = synth.adversarial_arena("all_equal", 257)
    a = np.abs(w_eq)
    wrong = np.lexsort((-np.arange(a.size), a))[:100]
    assert sorted(wrong.tolist()) != brute_force_pruned([float(x) for x in a], 100)


# ----------------------------------------------------------------------------- the faster CPU baseline
def test_fast_baseline_equals_the_oracle():
    """The benchmark's faster CPU program (selection instead of a sort) gives the oracle's
    results bit for bit: configs, a residual net, ties, special values, edge counts."""
    from oracle import fast_baseline as FB
    cases = []
    for c, s_ in ((1, 0.9), (1, 0.5), (3, 0.8), (3, 0.97)):
        spec, w, v = synth.generate_config(c)
        cases.append((spec, w, v, synth.prune_count(spec.n_prunable, s_)))
    spec = synth.residual_toy_spec(width=8, mid=6, n_blocks=3)
    w, v = synth.generate_weights(spec, 21)
    cases += [(spec, w, v, p) for p in (0, 1, spec.n_prunable // 2, spec.n_prunable - 1,
                                        spec.n_prunable)]
    spec = synth.chain_spec([9, 11, 6], k=3, in_ch=2, n_cls=5)
    _, v = synth.generate_weights(spec, 1)
    for kind in synth.ADVERSARIAL_KINDS:
        if kind == "nan":
            continue
        w = synth.adversarial_arena(kind, spec.w_elems, seed=3)
        cases += [(spec, w, v, p) for p in (spec.n_prunable // 3, 2 * spec.n_prunable // 3)]
    for spec, w, v, p in cases:
        ref = O.prune_and_compact(w, v, spec.tensors, spec.vecs, spec.groups, [p])[0]
        ws, mask, nw, cw, cv = FB.prune_and_compact_fast(w, v, spec.tensors, spec.vecs,
                                                         spec.groups, p)
        assert np.array_equal(ws.view(np.uint32), ref.w_sparse.view(np.uint32))
        assert np.array_equal(mask, ref.mask)
        assert np.array_equal(nw, ref.plan.new_width)
        assert np.array_equal(cw.view(np.uint32), ref.compacted.w.view(np.uint32))
        assert np.array_equal(cv.view(np.uint32), ref.compacted.v.view(np.uint32))
        # the threaded form of the same program, with slabs small enough to split tensors
        ws, mask, nw, cw, cv = FB.prune_and_compact_fast_mt(w, v, spec.tensors, spec.vecs,
                                                            spec.groups, p, threads=3, slab=1000)
        assert np.array_equal(ws.view(np.uint32), ref.w_sparse.view(np.uint32))
        assert np.array_equal(mask, ref.mask)
        assert np.array_equal(nw, ref.plan.new_width)
        assert np.array_equal(cw.view(np.uint32), ref.compacted.w.view(np.uint32))
        assert np.array_equal(cv.view(np.uint32), ref.compacted.v.view(np.uint32))
