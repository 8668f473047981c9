"""Full-size parity at the stress shape (wide VGG-19 x4, 322 M weights), in the launch
configurations the benchmark times.  The oracle's full sort would take minutes here, so
the threshold is checked through the counting definition of the P-th smallest
(|w|, index) pair, which holds at any size; everything downstream of the threshold (mask,
sparse weights, alive flags, plan, rebuilt tensors) is the oracle's, element by element."""
import zlib

import numpy as np
import pytest
import torch

from oracle import deflate_oracle as DO
from oracle import fold_oracle as FO
from oracle import shifter_oracle as O
from paper_2309_06973_amd import shifter as S
from paper_2309_06973_amd import synth
from paper_2309_06973_amd.pipeline import Codec, Pipeline
from test_gpu_fold import bias_bound

pytestmark = pytest.mark.gpu


def bits(a):
    return np.ascontiguousarray(a).view(np.uint32)


def check_record_by_counting(rec, a, p):
    """(t, g) is the P-th smallest pair iff #{|w| < t} < P <= #{|w| <= t} and g is the
    (P - #{|w| < t})-th index, ascending, among the weights equal to t."""
    t = np.uint32(rec.t_key).view(np.float32)
    n_less = int((a < t).sum())
    eq = np.flatnonzero(a == t)
    assert n_less < p <= n_less + eq.size
    assert rec.n_less == n_less and rec.n_equal == eq.size
    assert rec.g_cut == int(eq[p - n_less - 1])
    assert rec.cut == ((int(rec.t_key) << 32) | int(rec.g_cut)) + 1
    return t, int(rec.g_cut)


def selection_from_threshold(a, t, g_cut, p):
    removed = a < t
    removed[np.flatnonzero(a == t)[:p - int(removed.sum())]] = True   # ties by index
    sel = O.Selection(p, np.flatnonzero(removed), float(t), g_cut)
    assert sel.pruned.size == p
    return sel


@pytest.fixture(scope="module")
def c5():
    spec, w, v = synth.generate_config(5)
    return spec, w, v, np.abs(w)


def downstream(spec, w, v, sel):
    w_sparse, mask = O.apply_mask(w, spec.tensors, sel)
    out_alive, in_alive = O.dead_channel_scan(w_sparse, spec.tensors)
    plan = O.propagate_groups(spec.tensors, spec.groups, out_alive)
    comp = O.compact(w_sparse, v, spec.tensors, spec.vecs, plan)
    return w_sparse, mask, out_alive, in_alive, plan, comp


def test_c5_single_sweep_fused(c5):
    spec, w, v, a = c5
    n = spec.n_prunable
    p = synth.prune_count(n, 0.95)
    pl = Pipeline(spec, w, v)
    try:
        rec = pl.prune_fused(p)
        assert S.shifter_get_select_stats(pl.ctx)["path"] == 1     # the single pass decided
        pl.propagate_groups(0, sync=False)
        rc, ot, ov, ew, ev = pl.compact()
        torch.cuda.synchronize()
        t, g_cut = check_record_by_counting(rec, a, p)
        ws, mask, oa, ia, plan, comp = downstream(spec, w, v, selection_from_threshold(a, t, g_cut, p))
        assert np.array_equal(pl.d_mask[:n].cpu().numpy(), mask)
        assert np.array_equal(bits(pl.d_w_sparse.cpu().numpy()), bits(ws))
        assert np.array_equal(pl.d_out_alive.cpu().numpy(), np.concatenate(oa))
        assert np.array_equal(pl.d_in_alive.cpu().numpy(), np.concatenate(ia))
        assert np.array_equal(pl.d_new_width.cpu().numpy().view(np.uint32), plan.new_width)
        kp = pl.d_keep.cpu().numpy().view(np.uint32)
        for gi in range(len(spec.groups)):
            o = pl.model.group_off[gi]
            assert np.array_equal(kp[o:o + plan.keep[gi].size], plan.keep[gi])
        assert rc == S.SHIFTER_OK and ew == comp.w.size and ev == comp.v.size
        assert np.array_equal(bits(pl.d_w_out[:ew].cpu().numpy()), bits(comp.w))
        assert np.array_equal(bits(pl.d_vecs_out[:ev].cpu().numpy()), bits(comp.v))
        for d, (off, o2, i2, kh, kw) in zip(ot, comp.tensor_shapes):
            assert (d.offset, d.out_ch, d.in_ch, d.kh, d.kw) == (off, o2, i2, kh, kw)
        # the liveness fixpoint on the same sparse arena
        nz_ref = O.kernel_scan(ws, spec.tensors)
        plan_f = O.propagate_groups_fixpoint(spec.tensors, spec.groups, nz_ref)
        comp_f = O.compact(ws, v, spec.tensors, spec.vecs, plan_f)
        pl.kernel_scan()
        rc, nw, rounds = pl.propagate_groups_fixpoint(0)
        nz = pl.d_kernel_nz.cpu().numpy()
        for ti, t in enumerate(spec.tensors):
            o = pl.model.kernel_off[ti]
            assert np.array_equal(nz[o:o + t.out_ch * t.in_ch].reshape(t.out_ch, t.in_ch), nz_ref[ti])
        assert np.array_equal(np.array(nw, dtype=np.uint32), plan_f.new_width)
        kp = pl.d_keep.cpu().numpy().view(np.uint32)
        for gi in range(len(spec.groups)):
            o = pl.model.group_off[gi]
            assert np.array_equal(kp[o:o + plan_f.keep[gi].size], plan_f.keep[gi])
        rc, ot, ov, ew, ev = pl.compact()
        assert ew == comp_f.w.size and ev == comp_f.v.size and ew <= comp.w.size
        assert np.array_equal(bits(pl.d_w_out[:ew].cpu().numpy()), bits(comp_f.w))
        assert np.array_equal(bits(pl.d_vecs_out[:ev].cpu().numpy()), bits(comp_f.v))
        # Module 1's fold of the sparse arena, in place, against the fp64 oracle at the
        # bound of its four roundings (see the fold tests); zeros stay zeros
        fspec, folds = synth.fused_spec(spec)
        eps = float(np.float32(1e-5))
        ref_w, ref_b = FO.fold_bn(ws, v, spec.tensors, spec.vecs, folds, eps, fspec.v_elems)
        got_w, got_b = pl.fold_bn(folds, fspec.v_elems, eps, dst=pl.d_w_sparse)
        torch.cuda.synchronize()
        gw = got_w.cpu().numpy()
        u = 2.0 ** -24
        assert np.all(np.abs(gw - ref_w) <= 4 * u * np.abs(ref_w) + 2.0 ** -149)
        assert np.array_equal(gw == 0, ws == 0)
        gb = got_b.cpu().numpy()[:fspec.v_elems]
        assert np.all(np.abs(gb - ref_b) <= 4 * u * bias_bound(v, spec, folds, fspec.v_elems, eps)
                      + u * np.abs(ref_b) + 2.0 ** -149)
        # Phase 3 codec on the sparse arena (1.29 GB): the stream through zlib (an independent
        # inflater) and through the library's inflate gives the arena back; sampled chunks
        # equal the oracle encoder's segments (a segment depends on its chunk alone, apart
        # from the BFINAL bit of the last one)
        del ref_w, gw
        raw = ws.tobytes()
        cd = Codec(ctx=pl.ctx)
        d_raw = torch.from_numpy(ws).to(pl.dev)
        pkg = cd.deflate(d_raw)
        stream = pkg.stream.cpu().numpy().tobytes()
        seg_off = pkg.seg_off.cpu().numpy().tolist()
        assert seg_off[-1] == len(stream) and 5 < len(raw) / len(stream) < 40
        dz = zlib.decompressobj(-15)
        back, at = bytearray(), 0
        while at < len(stream):                                  # bounded pieces: memory
            back += dz.decompress(stream[at:at + (64 << 20)])
            at += 64 << 20
        assert dz.eof and dz.unused_data == b"" and bytes(back) == raw
        del back
        out = cd.inflate(pkg)
        assert torch.equal(out[:len(raw)].view(torch.int32), d_raw.view(torch.int32))
        n_chunks = len(seg_off) - 1
        rng = np.random.default_rng(3)
        for c in [0, 1, n_chunks - 2, n_chunks - 1] + rng.integers(0, n_chunks - 1, 12).tolist():
            ref_stream, ref_off, ref_side = DO.deflate_runs(raw[c * DO.CHUNK:(c + 2) * DO.CHUNK])
            side = pkg.sub_bits[c * 64:(c + 1) * 64].cpu().numpy().view(np.uint16).tolist()
            assert side == ref_side[:64]
            if c < n_chunks - 1:
                assert stream[seg_off[c]:seg_off[c + 1]] == ref_stream[:ref_off[1]]
            else:
                assert stream[seg_off[c]:] == ref_stream
    finally:
        pl.close()


def test_c5_portfolio_batched(c5):
    spec, w, v, a = c5
    n = spec.n_prunable
    ps = [synth.prune_count(n, s) for s in synth.config_sparsities(5)]
    pl = Pipeline(spec, w, v)
    try:
        pl.enable_batch(len(ps))
        recs, (rc, ots, ovs, ews, evs) = pl.portfolio(ps)
        torch.cuda.synchronize()
        assert S.shifter_get_select_stats(pl.ctx)["path"] == 1
        info = pl.model.info
        prev_kept = None
        for k, (rec, p) in enumerate(zip(recs, ps)):
            t, g_cut = check_record_by_counting(rec, a, p)
            mask_dev = pl.b_mask[k * pl.m_stride:k * pl.m_stride + n]
            assert int(mask_dev.sum(dtype=torch.int64)) == n - p        # exact kept count
            if k not in (0, 9):
                continue
            ws, mask, oa, ia, plan, comp = downstream(spec, w, v,
                                                      selection_from_threshold(a, t, g_cut, p))
            assert np.array_equal(mask_dev.cpu().numpy(), mask)
            wsd = pl.b_w_sparse[k * pl.w_stride:k * pl.w_stride + info.w_extent].cpu().numpy()
            assert np.array_equal(bits(wsd), bits(ws))
            so, si, ng = info.sum_out_ch, info.sum_in_ch, info.n_groups
            assert np.array_equal(pl.b_out_alive[k * so:(k + 1) * so].cpu().numpy(), np.concatenate(oa))
            assert np.array_equal(pl.b_in_alive[k * si:(k + 1) * si].cpu().numpy(), np.concatenate(ia))
            assert np.array_equal(pl.b_new_width[k * ng:(k + 1) * ng].cpu().numpy().view(np.uint32),
                                  plan.new_width)
            assert ews[k] == comp.w.size and evs[k] == comp.v.size
            wc = pl.b_w_out[k * pl.cap_w:k * pl.cap_w + ews[k]].cpu().numpy()
            assert np.array_equal(bits(wc), bits(comp.w))
            vc = pl.b_vecs_out[k * pl.cap_v:k * pl.cap_v + evs[k]].cpu().numpy()
            assert np.array_equal(bits(vc), bits(comp.v))
        # masks of a cumulative schedule nest
        m0 = pl.b_mask[0:n]
        m9 = pl.b_mask[9 * pl.m_stride:9 * pl.m_stride + n]
        assert bool((m9 <= m0).all())
    finally:
        pl.close()
