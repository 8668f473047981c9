"""The enqueue-only forms of the calls (no h_* output: kernels and nothing else on the
context's stream) recorded into a HIP graph: every replay must give what the same calls
give eagerly - on the weights the arena holds at the time of the replay, since a graph
records pointers and prune counts, not data - and the eager result is the oracle's."""
import numpy as np
import pytest
import torch

from oracle import fold_oracle as FO
from oracle import shifter_oracle as O
from paper_2309_06973_amd import shifter as S
from paper_2309_06973_amd import synth
from paper_2309_06973_amd.pipeline import Pipeline

pytestmark = pytest.mark.gpu


def enqueue_portfolio(pl, ps):
    """Steps 1-5 for all prune counts, enqueue only: the multi-pass radix select (needs no
    decision on the host), the batched mask pass, the planner, the rebuild."""
    k = len(ps)
    pl.global_threshold(ps, sync=False)
    S.shifter_apply_mask_batch(pl.ctx, pl.model, pl.d_w, pl.d_thr, k, pl.b_w_sparse, pl.w_stride,
                               pl.b_mask, pl.m_stride, pl.b_out_alive, pl.b_in_alive)
    S.shifter_propagate_groups_batch(pl.ctx, pl.model, pl.b_out_alive, k, 0, pl.b_group_alive,
                                     pl.b_index_map, pl.b_keep, pl.b_new_width, sync=False)
    S.shifter_compact_batch_masked(pl.ctx, pl.model, pl.d_w, pl.d_thr, pl.d_vecs, pl.b_keep,
                                   pl.b_new_width, k, pl.b_w_out, pl.cap_w, pl.b_vecs_out,
                                   pl.cap_v, sync=False)


def outputs(pl):
    return [pl.d_thr, pl.b_mask, pl.b_w_sparse, pl.b_out_alive, pl.b_in_alive, pl.b_keep,
            pl.b_new_width, pl.b_w_out, pl.b_vecs_out]


def scribble(pl):
    pl.d_thr.zero_()
    pl.b_mask.fill_(7)
    pl.b_w_sparse.fill_(float("nan"))
    pl.b_w_out.fill_(float("nan"))
    pl.b_vecs_out.fill_(float("nan"))
    pl.b_out_alive.fill_(7)
    pl.b_keep.fill_(-5)


def same(a, b):
    return all(torch.equal(x.view(torch.uint8), y.view(torch.uint8)) for x, y in zip(a, b))


@pytest.mark.parametrize("c", [1, 3])
def test_portfolio_step_replayed_from_a_graph(c):
    spec, w, v = synth.generate_config(c)
    n = spec.n_prunable
    ps = [synth.prune_count(n, s) for s in (0.5, 0.9)] if c == 1 else \
        [synth.prune_count(n, s) for s in synth.config_sparsities(c)][1::3]
    w2 = np.roll(w, 12345).copy()                       # other weights for the same network
    stream = torch.cuda.Stream()
    with torch.cuda.stream(stream):
        pl = Pipeline(spec, w, v)
        try:
            pl.enable_batch(len(ps))
            scribble(pl)
            enqueue_portfolio(pl, ps)                   # eager: binds the model, gives the reference
            stream.synchronize()
            eager = [x.clone() for x in outputs(pl)]
            # the eager result is the oracle's (the rebuilt variants, bit for bit)
            refs = O.prune_and_compact(w, v, spec.tensors, spec.vecs, spec.groups, ps)
            for k, ref in enumerate(refs):
                got = pl.b_w_out[k * pl.cap_w:k * pl.cap_w + ref.compacted.w.size].cpu().numpy()
                assert np.array_equal(got.view(np.uint32), ref.compacted.w.view(np.uint32))
            graph = torch.cuda.CUDAGraph()
            with torch.cuda.graph(graph, stream=stream):
                enqueue_portfolio(pl, ps)
            for _ in range(3):                          # replays, eager work between them
                scribble(pl)
                stream.synchronize()
                graph.replay()
                stream.synchronize()
                assert same(outputs(pl), eager)
                pl.single(ps[0])                        # an eager call on the same context
            # other weights in the same arena: the replay works on what is there now
            pl.d_w.copy_(torch.from_numpy(w2))
            scribble(pl)
            enqueue_portfolio(pl, ps)
            stream.synchronize()
            eager2 = [x.clone() for x in outputs(pl)]
            assert not same(eager2, eager)
            scribble(pl)
            graph.replay()
            stream.synchronize()
            assert same(outputs(pl), eager2)
        finally:
            pl.close()


def enqueue_fold_and_fixpoint(pl, folds, d_folded, d_bias):
    """Module 1's fold of the sparse arena, then the kernel index, the liveness fixpoint and
    the rebuild on it, none of them waiting or reading anything back."""
    pl.fold_bn(folds, d_bias.numel(), 1e-5, dst=d_folded, bias=d_bias)
    pl.kernel_scan()
    pl.propagate_groups_fixpoint(0, sync=False)
    pl.compact(sync=False)


@pytest.mark.parametrize("c", [1, 3])
def test_fold_and_fixpoint_replayed_from_a_graph(c):
    spec, w, v = synth.generate_config(c)
    p = synth.prune_count(spec.n_prunable, 0.9)
    fspec, folds = synth.fused_spec(spec)
    stream = torch.cuda.Stream()
    with torch.cuda.stream(stream):
        pl = Pipeline(spec, w, v)
        try:
            pl.single(p)
            d_folded = torch.empty_like(pl.d_w_sparse)
            d_bias = torch.zeros(max(fspec.v_elems, 4), dtype=torch.float32, device=pl.dev)
            outs = lambda: [d_folded, d_bias, pl.d_kernel_nz, pl.d_group_alive, pl.d_index_map, pl.d_keep,
                            pl.d_new_width, pl.d_w_out, pl.d_vecs_out]

            def scrub():
                for x in outs():
                    x.view(torch.uint8).fill_(0x5a)
                d_bias.zero_()

            # eager, with the calls that wait: the reference, itself checked against the oracle
            pl.kernel_scan()
            scrub()
            enqueue_fold_and_fixpoint(pl, folds, d_folded, d_bias)   # first call: uploads the layer table
            rc, nw, rounds = pl.propagate_groups_fixpoint(0)
            pl.compact(sync=True)
            stream.synchronize()
            eager = [x.clone() for x in outs()]
            ws = pl.d_w_sparse[:spec.w_elems].cpu().numpy()
            plan = O.propagate_groups_fixpoint(spec.tensors, spec.groups, O.kernel_scan(ws, spec.tensors))
            assert nw == [int(x) for x in plan.new_width]
            fw, _ = FO.fold_bn(ws, v, spec.tensors, spec.vecs, folds, 1e-5, fspec.v_elems)
            assert np.allclose(d_folded[:spec.w_elems].cpu().numpy(), fw[:spec.w_elems], rtol=4 * 2.0 ** -23, atol=0)
            # the enqueue-only form alone gives the same and reports the same rounds
            scrub()
            enqueue_fold_and_fixpoint(pl, folds, d_folded, d_bias)
            stream.synchronize()
            assert same(outs(), eager)
            assert S.shifter_fixpoint_status(pl.ctx, pl.model) == (rounds, True)
            graph = torch.cuda.CUDAGraph()
            with torch.cuda.graph(graph, stream=stream):
                enqueue_fold_and_fixpoint(pl, folds, d_folded, d_bias)
            for _ in range(3):
                scrub()
                stream.synchronize()
                graph.replay()
                stream.synchronize()
                assert same(outs(), eager)
                assert S.shifter_fixpoint_status(pl.ctx, pl.model) == (rounds, True)
                pl.propagate_groups_fixpoint(0)            # an eager call between the replays
            # a new layer list cannot be uploaded while the stream is capturing
            with pytest.raises(S.ShifterError):
                g2 = torch.cuda.CUDAGraph()
                with torch.cuda.graph(g2, stream=stream):
                    d_bias.zero_()
                    pl.fold_bn(folds[:-1], d_bias.numel(), 1e-5, dst=d_folded, bias=d_bias)
        finally:
            pl.close()
