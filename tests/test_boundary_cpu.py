"""Host-side checks of the C ABI that need no GPU: the library loads, exports every
symbol the header declares, validates descriptors, and reports sizes and layout."""
import ctypes as C
import os
import re

import pytest

from paper_2309_06973_amd import shifter as S
from paper_2309_06973_amd import synth

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
HEADER = os.path.join(ROOT, "include", "shifter.h")


@pytest.fixture(scope="module")
def lib():
    if not os.path.exists(S._LIB_PATH):
        from paper_2309_06973_amd import build
        build.build_library(verbose=False)
    return S.load_library()


def declared_symbols():
    text = open(HEADER).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(shifter_[a-z0-9_]+)\s*\(", text)))


def test_library_exports_every_declared_symbol(lib):
    names = declared_symbols()
    assert {"shifter_global_threshold", "shifter_apply_mask", "shifter_dead_channel_scan",
            "shifter_propagate_groups", "shifter_compact"} <= set(names)
    for n in names:
        assert hasattr(lib, n), n
    assert set(names) == set(S.EXPORTS)


def test_struct_sizes_match_header_layout():
    assert C.sizeof(S.TensorDesc) == 40 and C.sizeof(S.VecDesc) == 16
    assert C.sizeof(S.GroupDesc) == 8 and C.sizeof(S.Threshold) == 48
    assert C.sizeof(S.ModelInfo) == 80


def test_codec_layout_and_fold_descriptor(lib):
    # sizes of the codec's buffers are plain host arithmetic
    chunk = S.SHIFTER_CODEC_CHUNK
    for n, chunks in ((0, 1), (1, 1), (chunk - 1, 1), (chunk, 1), (chunk + 1, 2), (10 * chunk, 10),
                      (1289317376, 39347)):
        n_chunks, work, bound = S.shifter_codec_layout(n)
        assert n_chunks == chunks
        assert bound == n + 5 * chunks                       # every segment one stored block
        assert work >= chunks * (chunk + 8) + 4 * chunks and work % 8 == 0
    assert S.SHIFTER_CODEC_CHUNK // S.SHIFTER_CODEC_SUB == 64
    assert C.sizeof(S.FoldDesc) == 32


def test_model_info_and_layout(lib):
    spec = synth.build_config(3)
    m = S.shifter_model_create(spec.tensors, spec.vecs, spec.groups)
    assert m.info.n_prunable == spec.n_prunable == m.info.w_elems == m.info.w_extent
    assert m.info.v_elems == spec.v_elems
    assert m.info.sum_out_ch == sum(t.out_ch for t in spec.tensors)
    assert m.info.sum_in_ch == sum(t.in_ch for t in spec.tensors)
    assert m.info.sum_group_width == sum(g.width for g in spec.groups)
    off = 0
    for t, o in zip(spec.tensors, m.out_flag_off):
        assert o == off
        off += t.out_ch
    off = 0
    for g, o in zip(spec.groups, m.group_off):
        assert o == off
        off += g.width
    S.shifter_model_destroy(m)


def _bad(spec, mutate, match):
    import copy
    s = copy.deepcopy(spec)
    mutate(s)
    with pytest.raises(S.ShifterError) as e:
        S.shifter_model_create(s.tensors, s.vecs, s.groups)
    assert e.value.code == S.SHIFTER_ERR_BAD_MODEL
    assert match in str(e.value)


def test_model_validation_errors(lib):
    spec = synth.build_config(1)
    _bad(spec, lambda s: setattr(s.tensors[1], "out_group", 99), "group index")
    _bad(spec, lambda s: setattr(s.tensors[1], "out_ch", 31), "out_ch differs")
    _bad(spec, lambda s: setattr(s.tensors[1], "in_ch", 15), "in_ch differs")
    _bad(spec, lambda s: setattr(s.tensors[1], "kh", 0), "zero-sized")
    _bad(spec, lambda s: setattr(s.tensors[1], "offset", 10), "overlap")
    _bad(spec, lambda s: setattr(s.vecs[0], "length", 3), "vector length")
    _bad(spec, lambda s: setattr(s.vecs[1], "offset", 1), "vectors overlap")
    _bad(spec, lambda s: setattr(s.groups[1], "width", 0), "width 0")
    with pytest.raises(S.ShifterError) as e:
        S.shifter_model_create([], [], spec.groups)
    assert e.value.code == S.SHIFTER_ERR_INVALID_ARG


def test_model_size_limits(lib):
    """The global index is 32 bits wide: N stops short of 2^32 - 1; arena offsets stop at
    2^62 so that offset + size cannot wrap."""
    T, G = synth.TensorDesc, synth.GroupDesc
    groups = [G(1 << 15, 1), G(1 << 16, 0), G(1 << 15, 1)]
    half = 1 << 31                                  # 2^15 x 2^16 weights per tensor
    one = [T(0, 1 << 16, 1 << 15, 1, 1, 1, 1, 0, 1)]
    m = S.shifter_model_create(one, [], groups)
    assert m.info.n_prunable == half
    S.shifter_model_destroy(m)
    two = one + [T(half, 1 << 15, 1 << 16, 1, 1, 1, 2, 1, 1)]
    with pytest.raises(S.ShifterError) as e:
        S.shifter_model_create(two, [], groups)
    assert e.value.code == S.SHIFTER_ERR_BAD_MODEL and "2^32 - 1" in str(e.value)
    two[1].prunable = 0                             # not ranked: only the arena grows
    m = S.shifter_model_create(two, [], groups)
    assert m.info.n_prunable == half and m.info.w_elems == 2 * half
    S.shifter_model_destroy(m)
    far = [T(1 << 62, 1 << 16, 1 << 15, 1, 1, 1, 1, 0, 1)]
    with pytest.raises(S.ShifterError) as e:
        S.shifter_model_create(far, [], groups)
    assert e.value.code == S.SHIFTER_ERR_BAD_MODEL and "2^62" in str(e.value)


def test_no_device_is_an_error_not_a_fallback(lib):
    import torch
    if torch.cuda.is_available():
        pytest.skip("a GPU is visible")
    with pytest.raises(S.ShifterError) as e:
        S.shifter_create(0, 0)
    assert e.value.code == S.SHIFTER_ERR_NO_DEVICE
    from paper_2309_06973_amd.pipeline import Pipeline
    spec, w, v = synth.generate_config(1)
    with pytest.raises(RuntimeError):
        Pipeline(spec, w, v)


def test_product_path_does_not_import_the_oracle():
    pkg = os.path.join(ROOT, "paper_2309_06973_amd")
    for dirpath, _, files in os.walk(pkg):
        for f in files:
            if f.endswith((".py", ".hip", ".h", ".cpp")):
                text = open(os.path.join(dirpath, f)).read()
                assert "oracle" not in text.lower() or f == "synth.py", f
