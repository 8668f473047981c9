"""Shape builders are pinned to the parameter counts the paper prints (Table II)."""
import os

import numpy as np
import pytest

from paper_2309_06973_amd import synth

GOLDEN = os.path.join(os.path.dirname(__file__), "golden", "table2_param_counts.txt")


def read_table2():
    out = {}
    for line in open(GOLDEN):
        if line.startswith("#") or not line.strip():
            continue
        name, params_m, size_mb = line.split()
        out[name] = (float(params_m), float(size_mb))
    return out


def test_param_counts_match_table2():
    t2 = read_table2()
    vgg = synth.vgg16_cifar()
    r50 = synth.resnet50_imagenet()
    assert round(vgg.n_param_total / 1e6, 2) == t2["vgg16_cifar"][0]
    assert round(r50.n_param_total / 1e6, 2) == t2["resnet50_imagenet"][0]
    # 4 bytes per parameter (fp32): size in MiB as printed
    assert abs(vgg.n_param_total * 4 / 2 ** 20 - t2["vgg16_cifar"][1]) < 0.1
    assert abs(r50.n_param_total * 4 / 2 ** 20 - t2["resnet50_imagenet"][1]) < 0.4


def test_prunable_counts_and_layer_counts():
    expect = {1: (24112, 4), 2: (14715584, 14), 3: (851504, 58), 4: (25502912, 54),
              5: (322329344, 17)}
    for c, (n, n_t) in expect.items():
        spec = synth.build_config(c)
        assert spec.n_prunable == n and len(spec.tensors) == n_t
        assert spec.w_elems == n
        for t in spec.tensors:
            assert spec.groups[t.out_group].width == t.out_ch
            assert spec.groups[t.in_group].width * t.in_mult == t.in_ch
        for v in spec.vecs:
            assert spec.groups[v.group].width == v.length


def test_residual_groups_have_joint_producers():
    spec = synth.resnet56_cifar()
    producers = {}
    for t in spec.tensors:
        producers.setdefault(t.out_group, []).append(t)
    counts = sorted(len(v) for v in producers.values())
    # stage streams: stem + 9 conv2 / projection + 9 conv2 (x2); everything else single
    assert counts[-3:] == [10, 10, 10]
    spec = synth.resnet50_imagenet()
    producers = {}
    for t in spec.tensors:
        producers.setdefault(t.out_group, []).append(t)
    assert sorted(len(v) for v in producers.values())[-4:] == [4, 4, 5, 7]


def test_generation_is_seeded_and_heavy_tailed():
    spec, w, v = synth.generate_config(1)
    _, w2, v2 = synth.generate_config(1)
    assert np.array_equal(w, w2) and np.array_equal(v, v2)
    assert w.dtype == np.float32 and np.isfinite(w).all() and np.isfinite(v).all()
    t = spec.tensors[2]
    x = np.abs(w[t.offset:t.offset + t.numel]).reshape(t.out_ch, -1).mean(axis=1)
    assert x.max() / x.min() > 1e3       # killed filters sit decades below the bulk


def test_sparsity_schedule():
    assert synth.config_sparsities(1) == [0.9]
    s = synth.config_sparsities(4)
    assert len(s) == 20 and abs(s[-1] - 0.98847) < 1e-5
    assert len(synth.config_sparsities(2)) == 10 and len(synth.config_sparsities(3)) == 15


def test_random_nets_are_valid_and_deterministic():
    """The random descriptions pass the library's own validation (host only), are the same
    on every call, hold no NaN, and leave their gaps to a sentinel."""
    from paper_2309_06973_amd import shifter as S
    shapes = set()
    for seed in range(40):
        spec = synth.random_spec(seed)
        again = synth.random_spec(seed)
        assert spec.tensors == again.tensors and spec.vecs == again.vecs and spec.groups == again.groups
        m = S.shifter_model_create(spec.tensors, spec.vecs, spec.groups)
        assert m.info.n_prunable == spec.n_prunable > 0
        S.shifter_model_destroy(m)
        w, v = synth.random_weights(spec, seed)
        w2, _ = synth.random_weights(spec, seed)
        assert np.array_equal(w.view(np.uint32), w2.view(np.uint32))
        assert not np.isnan(w).any() and w.size >= spec.w_elems
        covered = np.zeros(w.size, dtype=bool)
        for t in spec.tensors:
            covered[t.offset:t.offset + t.numel] = True
            shapes.add((t.kh, t.kw, t.in_mult > 1, bool(t.prunable)))
        assert np.all(w[~covered] == np.float32(12345.0))
    assert len(shapes) >= 12                       # the shapes really vary
    producers = {}
    for seed in range(40):
        for t in synth.random_spec(seed).tensors:
            producers[(seed, t.out_group)] = producers.get((seed, t.out_group), 0) + 1
    assert max(producers.values()) >= 2            # residual-style groups occur
