"""The entry point that allocates nothing (shifter_global_threshold_static: the ranking of
one flat run of weights with its scratch in a static device array) against the existing
entry point it is a variant of (shifter_global_threshold's multi-pass select on a model of
one tensor) and against the oracle, on two calls in a row, the second with a smaller
input."""
import numpy as np
import pytest
import torch

from oracle import shifter_oracle as O
from paper_2309_06973_amd import shifter as S
from paper_2309_06973_amd import synth

pytestmark = pytest.mark.gpu

T, G = synth.TensorDesc, synth.GroupDesc


def flat_weights(n, seed, ties):
    rng = np.random.Generator(np.random.Philox(seed))
    w = rng.standard_normal(n).astype(np.float32)
    w *= np.exp(rng.standard_normal(n).astype(np.float32))
    if ties:
        # many equal magnitudes (both signs) and exact zeros: the index-ordered tie rank and
        # the per-tile counts it needs
        w = np.round(w * 8.0) / 8.0
        w[rng.random(n) < 0.2] = 0.0
    return w.astype(np.float32)


def records(d_thr, k):
    raw = d_thr[:k * S.THRESHOLD_BYTES].cpu().numpy().tobytes()
    return [S.Threshold.from_buffer_copy(raw, i * S.THRESHOLD_BYTES) for i in range(k)]


def fields(r):
    return (r.cut, r.t_key, r.g_cut, r.n_prune, r.n_less, r.n_equal)


def existing_entry_point(ctx, d_w, n, counts, dev):
    """shifter_global_threshold (multi-pass select) on a one-tensor model of n weights."""
    groups = [G(n, 1), G(1, 1)]
    tensors = [T(0, 1, n, 1, 1, 1, 1, 0, 1)]
    model = S.shifter_model_create(tensors, [], groups)
    d_thr = torch.zeros(len(counts) * S.THRESHOLD_BYTES, dtype=torch.uint8, device=dev)
    S.shifter_set_select_path(ctx, 1)
    try:
        recs = S.shifter_global_threshold(ctx, model, d_w, counts, d_thr, sync=True)
    finally:
        S.shifter_set_select_path(ctx, 0)
        S.shifter_model_destroy(model)
    return recs, tensors


def check_call(ctx, dev, n, seed, ties, counts):
    w = flat_weights(n, seed, ties)
    d_w = torch.from_numpy(w).to(dev)
    k = len(counts)
    d_thr = torch.full((k * S.THRESHOLD_BYTES,), 0xAB, dtype=torch.uint8, device=dev)
    print(f"static select: n={n} seed={seed} ties={ties} counts={counts}", flush=True)
    S.shifter_global_threshold_static(ctx, d_w, n, counts, d_thr)
    torch.cuda.synchronize()
    got = records(d_thr, k)
    ref, tensors = existing_entry_point(ctx, d_w, n, counts, dev)
    for a, b in zip(got, ref):
        assert fields(a) == fields(b)
    # and the oracle's selection (full stable sort, ties by index)
    a_abs = np.abs(w)
    for rec, sel in zip(got, O.select_pruned(w, tensors, counts)):
        assert rec.n_prune == sel.n_prune
        if sel.n_prune == 0:
            assert rec.cut == 0
            continue
        key = int(np.float32(sel.thr_value).view(np.uint32))
        assert (rec.t_key, rec.g_cut) == (key, sel.thr_index)
        assert rec.cut == ((key << 32) | sel.thr_index) + 1
        assert rec.n_less == int((a_abs < np.float32(sel.thr_value)).sum())
        assert rec.n_equal == int((a_abs == np.float32(sel.thr_value)).sum())


def test_static_select_two_calls_second_smaller():
    dev = torch.device("cuda", 0)
    torch.cuda.set_device(dev)
    ctx = S.shifter_create(0, torch.cuda.current_stream().cuda_stream)
    try:
        # several tiles and a ragged tail, heavy ties; then a smaller input whose tiles and
        # histograms must not see what the first call left in the array
        n1 = 37 * 4096 + 1234
        check_call(ctx, dev, n1, 11, True, [0, 1, n1 // 3, n1 // 2, n1 - 1, n1])
        n2 = 3 * 4096 + 5
        check_call(ctx, dev, n2, 12, True, [n2 // 2, 7])
        check_call(ctx, dev, 100, 13, False, [50])
        check_call(ctx, dev, n1, 14, False, [n1 // 5 * 4])
    finally:
        S.shifter_destroy(ctx)


def test_static_select_limits_and_errors():
    dev = torch.device("cuda", 0)
    torch.cuda.set_device(dev)
    ctx = S.shifter_create(0, torch.cuda.current_stream().cuda_stream)
    try:
        d_w = torch.zeros(4096, dtype=torch.float32, device=dev)
        d_thr = torch.zeros(S.SHIFTER_MAX_VARIANTS * S.THRESHOLD_BYTES, dtype=torch.uint8, device=dev)
        with pytest.raises(S.ShifterError) as e:      # beyond the array: rejected on the host
            S.shifter_global_threshold_static(ctx, d_w, S.SHIFTER_STATIC_MAX_WEIGHTS + 1, [1], d_thr)
        assert e.value.code == S.SHIFTER_ERR_CAPACITY
        with pytest.raises(S.ShifterError) as e:      # K * tiles beyond the per-tile counts
            S.shifter_global_threshold_static(ctx, d_w, S.SHIFTER_STATIC_MAX_WEIGHTS, [1] * 17, d_thr)
        assert e.value.code == S.SHIFTER_ERR_CAPACITY
        with pytest.raises(S.ShifterError) as e:
            S.shifter_global_threshold_static(ctx, d_w, 4096, [4097], d_thr)
        assert e.value.code == S.SHIFTER_ERR_INVALID_ARG
        # n = 0: only P = 0 is possible
        S.shifter_global_threshold_static(ctx, None, 0, [0], d_thr)
        torch.cuda.synchronize()
        assert records(d_thr, 1)[0].cut == 0
    finally:
        S.shifter_destroy(ctx)
