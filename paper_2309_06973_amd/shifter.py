"""ctypes binding of libshifter.so: the same names as the C ABI (include/shifter.h),
argument marshalling only.  Device buffers are torch tensors on a ROCm device; every
step of the pass runs in the library's HIP kernels.  There is no CPU fallback: if the
library is missing or no GPU is visible, calls raise."""
from __future__ import annotations

import ctypes as C
import os
from typing import List, Optional, Sequence

_LIB_PATH = os.path.join(os.path.dirname(os.path.abspath(__file__)), "libshifter.so")

SHIFTER_OK = 0
SHIFTER_ERR_INVALID_ARG = 1
SHIFTER_ERR_BAD_MODEL = 2
SHIFTER_ERR_NONFINITE = 3
SHIFTER_ERR_CAPACITY = 4
SHIFTER_ERR_NO_DEVICE = 5
SHIFTER_ERR_HIP = 6
SHIFTER_ERR_OOM = 7
SHIFTER_ERR_INTERNAL = 8
SHIFTER_WARN_COLLAPSE = 100
SHIFTER_GROUPS_JOINT = 0
SHIFTER_PAPER_FREEZE_RESIDUAL = 1
SHIFTER_GROUPS_FIXPOINT = 2
SHIFTER_MAX_VARIANTS = 64


class TensorDesc(C.Structure):
    _fields_ = [("offset", C.c_uint64), ("out_ch", C.c_uint32), ("in_ch", C.c_uint32),
                ("kh", C.c_uint32), ("kw", C.c_uint32), ("in_mult", C.c_uint32),
                ("out_group", C.c_int32), ("in_group", C.c_int32),
                ("prunable", C.c_uint32)]


class VecDesc(C.Structure):
    _fields_ = [("offset", C.c_uint64), ("len", C.c_uint32), ("group", C.c_int32)]


class GroupDesc(C.Structure):
    _fields_ = [("width", C.c_uint32), ("pinned", C.c_uint32)]


class Threshold(C.Structure):
    _fields_ = [("cut", C.c_uint64), ("t_key", C.c_uint32), ("reserved", C.c_uint32),
                ("g_cut", C.c_uint64), ("n_prune", C.c_uint64), ("n_less", C.c_uint64),
                ("n_equal", C.c_uint64)]


class ModelInfo(C.Structure):
    _fields_ = [("n_prunable", C.c_uint64), ("w_extent", C.c_uint64),
                ("v_extent", C.c_uint64), ("w_elems", C.c_uint64), ("v_elems", C.c_uint64),
                ("sum_out_ch", C.c_uint64), ("sum_in_ch", C.c_uint64),
                ("sum_group_width", C.c_uint64), ("n_tensors", C.c_uint32),
                ("n_vecs", C.c_uint32), ("n_groups", C.c_uint32), ("reserved", C.c_uint32)]


THRESHOLD_BYTES = C.sizeof(Threshold)


class PortfolioArgs(C.Structure):
    _fields_ = [("d_w", C.c_void_p), ("d_vecs", C.c_void_p), ("h_n_prune", C.POINTER(C.c_uint64)),
                ("K", C.c_uint32), ("flags", C.c_uint32), ("d_thr", C.c_void_p),
                ("d_w_sparse", C.c_void_p), ("w_stride", C.c_uint64), ("d_mask", C.c_void_p),
                ("mask_stride", C.c_uint64), ("d_out_alive", C.c_void_p),
                ("d_in_alive", C.c_void_p), ("d_group_alive", C.c_void_p),
                ("d_index_map", C.c_void_p), ("d_keep", C.c_void_p), ("d_new_width", C.c_void_p),
                ("d_w_out", C.c_void_p), ("cap_w", C.c_uint64), ("d_vecs_out", C.c_void_p),
                ("cap_v", C.c_uint64)]


class FoldDesc(C.Structure):
    _fields_ = [("tensor", C.c_uint32), ("gamma", C.c_int32), ("beta", C.c_int32),
                ("mean", C.c_int32), ("var", C.c_int32), ("bias", C.c_int32),
                ("out_offset", C.c_uint64)]


EXPORTS = {
    "shifter_create": [C.POINTER(C.c_void_p), C.c_int, C.c_void_p],
    "shifter_destroy": [C.c_void_p],
    "shifter_last_error": [C.c_void_p],
    "shifter_model_create": [C.POINTER(TensorDesc), C.c_uint32, C.POINTER(VecDesc),
                             C.c_uint32, C.POINTER(GroupDesc), C.c_uint32,
                             C.POINTER(C.c_void_p)],
    "shifter_model_destroy": [C.c_void_p],
    "shifter_model_get_info": [C.c_void_p, C.POINTER(ModelInfo)],
    "shifter_model_get_layout": [C.c_void_p, C.POINTER(C.c_uint64), C.POINTER(C.c_uint64),
                                 C.POINTER(C.c_uint64)],
    "shifter_global_threshold": [C.c_void_p, C.c_void_p, C.c_void_p,
                                 C.POINTER(C.c_uint64), C.c_uint32, C.c_void_p,
                                 C.POINTER(Threshold)],
    "shifter_global_threshold_static": [C.c_void_p, C.c_void_p, C.c_uint64,
                                        C.POINTER(C.c_uint64), C.c_uint32, C.c_void_p],
    "shifter_portfolio_begin": [C.c_void_p, C.c_void_p, C.POINTER(PortfolioArgs)],
    "shifter_portfolio_end": [C.c_void_p, C.POINTER(Threshold), C.POINTER(TensorDesc),
                              C.POINTER(VecDesc), C.POINTER(C.c_uint64), C.POINTER(C.c_uint64)],
    "shifter_global_threshold_begin": [C.c_void_p, C.c_void_p, C.c_void_p,
                                       C.POINTER(C.c_uint64), C.c_uint32, C.c_void_p],
    "shifter_global_threshold_end": [C.c_void_p, C.POINTER(Threshold), C.POINTER(C.c_int)],
    "shifter_set_select_path": [C.c_void_p, C.c_int],
    "shifter_set_margin_sigmas": [C.c_void_p, C.c_double],
    "shifter_get_select_stats": [C.c_void_p, C.POINTER(C.c_uint64)],
    "shifter_prune_fused": [C.c_void_p, C.c_void_p, C.c_void_p, C.c_uint64, C.c_void_p,
                            C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p,
                            C.POINTER(Threshold)],
    "shifter_fold_bn": [C.c_void_p, C.c_void_p, C.POINTER(FoldDesc), C.c_uint32, C.c_float,
                        C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p, C.c_uint64],
    "shifter_codec_layout": [C.c_uint64, C.POINTER(C.c_uint64), C.POINTER(C.c_uint64),
                             C.POINTER(C.c_uint64)],
    "shifter_deflate": [C.c_void_p, C.c_void_p, C.c_uint64, C.c_void_p, C.c_uint64, C.c_void_p,
                        C.c_uint64, C.c_void_p, C.c_void_p, C.c_void_p, C.POINTER(C.c_uint64)],
    "shifter_inflate": [C.c_void_p, C.c_void_p, C.c_uint64, C.c_void_p, C.c_void_p, C.c_void_p,
                        C.c_uint64, C.c_void_p, C.c_int],
    "shifter_codec_status": [C.c_void_p, C.POINTER(C.c_uint64), C.POINTER(C.c_uint32)],
    "shifter_apply_mask": [C.c_void_p] * 8,
    "shifter_dead_channel_scan": [C.c_void_p] * 5,
    "shifter_propagate_groups": [C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p, C.c_uint32,
                                 C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p,
                                 C.POINTER(C.c_uint32)],
    "shifter_compact": [C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p,
                        C.c_void_p, C.c_void_p, C.c_uint64, C.c_void_p, C.c_uint64,
                        C.POINTER(TensorDesc), C.POINTER(VecDesc), C.POINTER(C.c_uint64),
                        C.POINTER(C.c_uint64)],
    "shifter_apply_mask_batch": [C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p, C.c_uint32,
                                 C.c_void_p, C.c_uint64, C.c_void_p, C.c_uint64, C.c_void_p,
                                 C.c_void_p],
    "shifter_propagate_groups_batch": [C.c_void_p, C.c_void_p, C.c_void_p, C.c_uint32,
                                       C.c_uint32, C.c_void_p, C.c_void_p, C.c_void_p,
                                       C.c_void_p, C.POINTER(C.c_uint32)],
    "shifter_compact_batch": [C.c_void_p, C.c_void_p, C.c_void_p, C.c_uint64, C.c_void_p,
                              C.c_void_p, C.c_void_p, C.c_uint32, C.c_void_p, C.c_uint64,
                              C.c_void_p, C.c_uint64, C.POINTER(TensorDesc),
                              C.POINTER(VecDesc), C.POINTER(C.c_uint64),
                              C.POINTER(C.c_uint64)],
    "shifter_compact_batch_masked": [C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p,
                                     C.c_void_p, C.c_void_p, C.c_uint32, C.c_void_p, C.c_uint64,
                                     C.c_void_p, C.c_uint64, C.POINTER(TensorDesc),
                                     C.POINTER(VecDesc), C.POINTER(C.c_uint64),
                                     C.POINTER(C.c_uint64)],
    "shifter_model_get_kernel_layout": [C.c_void_p, C.POINTER(C.c_uint64), C.POINTER(C.c_uint64)],
    "shifter_kernel_scan": [C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p],
    "shifter_propagate_groups_fixpoint": [C.c_void_p, C.c_void_p, C.c_void_p, C.c_uint32,
                                          C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p,
                                          C.POINTER(C.c_uint32), C.POINTER(C.c_uint32)],
    "shifter_set_select_grid": [C.c_void_p, C.c_uint32],
    "shifter_set_fused_min_bytes": [C.c_void_p, C.c_uint64],
    "shifter_fixpoint_status": [C.c_void_p, C.c_void_p, C.POINTER(C.c_uint32), C.POINTER(C.c_uint32)],
    "shifter_prune_fused_result": [C.c_void_p, C.POINTER(Threshold), C.POINTER(C.c_int)],
    "shifter_prune_fused_batch": [C.c_void_p, C.c_void_p, C.c_void_p, C.POINTER(C.c_uint64),
                                  C.c_uint32, C.c_void_p, C.c_void_p, C.c_uint64, C.c_void_p,
                                  C.c_uint64, C.c_void_p, C.c_void_p, C.POINTER(Threshold)],
    "shifter_profile_enable": [C.c_void_p, C.c_int],
    "shifter_profile_read": [C.c_void_p, C.POINTER(C.c_char_p), C.POINTER(C.c_uint32),
                             C.POINTER(C.c_double), C.c_uint32, C.POINTER(C.c_uint32)],
    "shifter_copy_f32": [C.c_void_p, C.c_void_p, C.c_void_p, C.c_uint64],
}

_lib = None


class ShifterError(RuntimeError):
    def __init__(self, code: int, msg: str):
        super().__init__(f"shifter status {code}: {msg}")
        self.code = code


def load_library() -> C.CDLL:
    """Loads libshifter.so; raises if it has not been built (no fallback exists)."""
    global _lib
    if _lib is None:
        if not os.path.exists(_LIB_PATH):
            raise RuntimeError(
                f"{_LIB_PATH} is missing: build it with "
                "`python -m paper_2309_06973_amd.build` (hipcc, gfx950)")
        # The device pointers and streams handed to the library come from torch, so the
        # library must run on the HIP runtime torch has loaded: import torch first, then
        # libshifter's dependency on libamdhip64.so.7 resolves to that same runtime.
        import torch  # noqa: F401
        lib = C.CDLL(_LIB_PATH)
        for name, argtypes in EXPORTS.items():
            fn = getattr(lib, name)
            fn.argtypes = argtypes
            fn.restype = C.c_char_p if name == "shifter_last_error" else C.c_int
        _lib = lib
    return _lib


def _check(rc: int, ctx=None, allow=()):
    if rc != SHIFTER_OK and rc not in allow:
        msg = load_library().shifter_last_error(ctx)
        raise ShifterError(rc, msg.decode() if msg else "")
    return rc


def _ptr(t) -> Optional[int]:
    return None if t is None else t.data_ptr()


# --------------------------------------------------------------------------- objects
class Context:
    def __init__(self, handle):
        self.handle = handle


class Model:
    def __init__(self, handle, info: ModelInfo, out_flag_off, in_flag_off, group_off):
        self.handle = handle
        self.info = info
        self.out_flag_off: List[int] = out_flag_off
        self.in_flag_off: List[int] = in_flag_off
        self.group_off: List[int] = group_off


def shifter_create(device: int = 0, hip_stream: int = 0) -> Context:
    h = C.c_void_p()
    _check(load_library().shifter_create(C.byref(h), device, C.c_void_p(hip_stream or None)))
    return Context(h)


def shifter_destroy(ctx: Context) -> None:
    _check(load_library().shifter_destroy(ctx.handle))
    ctx.handle = None


def shifter_last_error(ctx: Optional[Context] = None) -> str:
    msg = load_library().shifter_last_error(ctx.handle if ctx else None)
    return msg.decode() if msg else ""


def shifter_model_create(tensors: Sequence, vecs: Sequence, groups: Sequence) -> Model:
    """tensors / vecs / groups: objects with the descriptor attributes (see synth)."""
    lib = load_library()
    ta = (TensorDesc * max(len(tensors), 1))()
    for i, t in enumerate(tensors):
        ta[i] = TensorDesc(t.offset, t.out_ch, t.in_ch, t.kh, t.kw, t.in_mult, t.out_group,
                           t.in_group, t.prunable)
    va = (VecDesc * max(len(vecs), 1))()
    for i, v in enumerate(vecs):
        va[i] = VecDesc(v.offset, getattr(v, "length", getattr(v, "len", 0)), v.group)
    ga = (GroupDesc * max(len(groups), 1))()
    for i, g in enumerate(groups):
        ga[i] = GroupDesc(g.width, g.pinned)
    h = C.c_void_p()
    _check(lib.shifter_model_create(ta, len(tensors), va, len(vecs), ga, len(groups),
                                    C.byref(h)))
    info = ModelInfo()
    _check(lib.shifter_model_get_info(h, C.byref(info)))
    o = (C.c_uint64 * info.n_tensors)()
    i_ = (C.c_uint64 * info.n_tensors)()
    g_ = (C.c_uint64 * info.n_groups)()
    _check(lib.shifter_model_get_layout(h, o, i_, g_))
    model = Model(h, info, list(o), list(i_), list(g_))
    ko = (C.c_uint64 * max(info.n_tensors, 1))()
    sk = C.c_uint64()
    _check(lib.shifter_model_get_kernel_layout(h, ko, C.byref(sk)))
    model.kernel_off = list(ko)[:info.n_tensors]
    model.sum_kernels = int(sk.value)
    return model


def shifter_model_destroy(model: Model) -> None:
    _check(load_library().shifter_model_destroy(model.handle))
    model.handle = None


def shifter_global_threshold(ctx: Context, model: Model, d_w, n_prune: Sequence[int],
                             d_thr, sync: bool = True) -> Optional[List[Threshold]]:
    """d_thr: uint8 device tensor of len(n_prune) * THRESHOLD_BYTES bytes."""
    k = len(n_prune)
    arr = (C.c_uint64 * max(k, 1))(*[int(p) for p in n_prune])
    h = (Threshold * max(k, 1))() if sync else None
    _check(load_library().shifter_global_threshold(ctx.handle, model.handle, _ptr(d_w), arr, k,
                                                   _ptr(d_thr), h), ctx.handle)
    return list(h)[:k] if sync else None


SHIFTER_STATIC_MAX_WEIGHTS = 1 << 28
SHIFTER_STATIC_MAX_TILE_COUNTS = 1 << 20


def shifter_global_threshold_static(ctx: Context, d_w, n: int, n_prune: Sequence[int],
                                    d_thr) -> None:
    """The ranking for one flat run of n weights, no model, no allocation, enqueue only.
    d_thr: uint8 device tensor of len(n_prune) * THRESHOLD_BYTES bytes."""
    k = len(n_prune)
    arr = (C.c_uint64 * max(k, 1))(*[int(p) for p in n_prune])
    _check(load_library().shifter_global_threshold_static(ctx.handle, _ptr(d_w), int(n), arr, k,
                                                          _ptr(d_thr)), ctx.handle)


def shifter_set_select_path(ctx: Context, path: int) -> None:
    _check(load_library().shifter_set_select_path(ctx.handle, path), ctx.handle)


def shifter_set_margin_sigmas(ctx: Context, sigmas: float) -> None:
    _check(load_library().shifter_set_margin_sigmas(ctx.handle, float(sigmas)), ctx.handle)


def shifter_get_select_stats(ctx: Context) -> dict:
    out = (C.c_uint64 * 8)()
    _check(load_library().shifter_get_select_stats(ctx.handle, out), ctx.handle)
    keys = ("path", "n_prune", "n_below", "n_inside", "sample", "lo_key", "hi_key", "status")
    return dict(zip(keys, [int(x) for x in out]))


def shifter_prune_fused(ctx: Context, model: Model, d_w, n_prune: int, d_thr, d_w_out, d_mask,
                        d_out_alive, d_in_alive, defer: bool = False) -> Optional[Threshold]:
    """defer: only enqueue; collect the outcome with shifter_prune_fused_result."""
    h = None if defer else Threshold()
    _check(load_library().shifter_prune_fused(ctx.handle, model.handle, _ptr(d_w), int(n_prune),
                                              _ptr(d_thr), _ptr(d_w_out), _ptr(d_mask),
                                              _ptr(d_out_alive), _ptr(d_in_alive),
                                              None if defer else C.byref(h)),
           ctx.handle)
    return h


def shifter_prune_fused_result(ctx: Context):
    """Returns (record, redone): redone means the outputs of the deferred
    shifter_prune_fused were recomputed and everything derived from them is stale."""
    h = Threshold()
    redone = C.c_int()
    _check(load_library().shifter_prune_fused_result(ctx.handle, C.byref(h), C.byref(redone)),
           ctx.handle)
    return h, bool(redone.value)


def shifter_apply_mask(ctx: Context, model: Model, d_w, d_thr, d_w_out, d_mask,
                       d_out_alive=None, d_in_alive=None, thr_index: int = 0) -> None:
    thr_ptr = d_thr.data_ptr() + thr_index * THRESHOLD_BYTES
    _check(load_library().shifter_apply_mask(ctx.handle, model.handle, _ptr(d_w), thr_ptr,
                                             _ptr(d_w_out), _ptr(d_mask), _ptr(d_out_alive),
                                             _ptr(d_in_alive)), ctx.handle)


def shifter_dead_channel_scan(ctx: Context, model: Model, d_w_sparse, d_out_alive,
                              d_in_alive) -> None:
    _check(load_library().shifter_dead_channel_scan(ctx.handle, model.handle, _ptr(d_w_sparse),
                                                    _ptr(d_out_alive), _ptr(d_in_alive)),
           ctx.handle)


def shifter_propagate_groups(ctx: Context, model: Model, d_out_alive, d_in_alive, flags: int,
                             d_group_alive, d_index_map, d_keep, d_new_width,
                             sync: bool = True):
    """Returns (status, new_width list) when sync, else (SHIFTER_OK, None)."""
    h = (C.c_uint32 * model.info.n_groups)() if sync else None
    rc = _check(load_library().shifter_propagate_groups(
        ctx.handle, model.handle, _ptr(d_out_alive), _ptr(d_in_alive), flags,
        _ptr(d_group_alive), _ptr(d_index_map), _ptr(d_keep), _ptr(d_new_width), h),
        ctx.handle, allow=(SHIFTER_WARN_COLLAPSE,))
    return rc, (list(h) if sync else None)


def shifter_prune_fused_batch(ctx: Context, model: Model, d_w, n_prune: Sequence[int], d_thr,
                              d_w_out, w_stride: int, d_mask, mask_stride: int, d_out_alive,
                              d_in_alive) -> List[Threshold]:
    k = len(n_prune)
    arr = (C.c_uint64 * max(k, 1))(*[int(p) for p in n_prune])
    h = (Threshold * max(k, 1))()
    _check(load_library().shifter_prune_fused_batch(
        ctx.handle, model.handle, _ptr(d_w), arr, k, _ptr(d_thr), _ptr(d_w_out), w_stride,
        _ptr(d_mask), mask_stride, _ptr(d_out_alive), _ptr(d_in_alive), h), ctx.handle)
    return list(h)[:k]


def shifter_fold_bn(ctx: Context, model: Model, folds, eps: float, d_w, d_vecs, d_w_out,
                    d_bias_out) -> None:
    """folds: objects with tensor, gamma, beta, mean, var, bias, out_offset (-1: absent).
    The capacity of the bias arena is the length of d_bias_out."""
    arr = (FoldDesc * max(len(folds), 1))()
    for i, f in enumerate(folds):
        arr[i] = FoldDesc(f.tensor, f.gamma, f.beta, f.mean, f.var, f.bias, f.out_offset)
    cap = d_bias_out.numel() if d_bias_out is not None else 0
    _check(load_library().shifter_fold_bn(ctx.handle, model.handle, arr, len(folds), eps,
                                          _ptr(d_w), _ptr(d_vecs), _ptr(d_w_out),
                                          _ptr(d_bias_out), cap), ctx.handle)


SHIFTER_CODEC_CHUNK = 32768
SHIFTER_CODEC_SUB = 512


def shifter_codec_layout(n_bytes: int):
    """(chunks, workspace bytes, largest possible stream) for n_bytes of input."""
    a, b, c = C.c_uint64(), C.c_uint64(), C.c_uint64()
    _check(load_library().shifter_codec_layout(n_bytes, C.byref(a), C.byref(b), C.byref(c)))
    return int(a.value), int(b.value), int(c.value)


def shifter_deflate(ctx: Context, d_in, n_bytes: int, d_work, d_stream, d_seg_off, d_sub_bits,
                    d_sub_marks, sync: bool = True) -> Optional[int]:
    """Capacities are the byte sizes of d_work and d_stream.  Returns the stream's size when
    sync (raises ShifterError with code SHIFTER_ERR_CAPACITY if it does not fit)."""
    total = C.c_uint64()
    nbytes = lambda t: t.numel() * t.element_size()
    _check(load_library().shifter_deflate(
        ctx.handle, _ptr(d_in), n_bytes, _ptr(d_work), nbytes(d_work), _ptr(d_stream),
        nbytes(d_stream), _ptr(d_seg_off), _ptr(d_sub_bits), _ptr(d_sub_marks),
        C.byref(total) if sync else None), ctx.handle)
    return int(total.value) if sync else None


def shifter_inflate(ctx: Context, d_stream, stream_bytes: int, d_seg_off, d_sub_bits, d_sub_marks,
                    n_bytes: int, d_out, sync: bool = True) -> None:
    _check(load_library().shifter_inflate(ctx.handle, _ptr(d_stream), stream_bytes,
                                          _ptr(d_seg_off), _ptr(d_sub_bits), _ptr(d_sub_marks),
                                          n_bytes, _ptr(d_out), 1 if sync else 0), ctx.handle)


def shifter_codec_status(ctx: Context):
    """(stream bytes, bad) of the context's last codec call, once its stream has been waited for."""
    total, bad = C.c_uint64(), C.c_uint32()
    _check(load_library().shifter_codec_status(ctx.handle, C.byref(total), C.byref(bad)), ctx.handle)
    return int(total.value), bool(bad.value)


def shifter_portfolio_begin(ctx: Context, model: Model, d_w, d_vecs, n_prune: Sequence[int],
                            flags: int, d_thr, d_w_sparse, w_stride: int, d_mask, mask_stride: int,
                            d_out_alive, d_in_alive, d_group_alive, d_index_map, d_keep,
                            d_new_width, d_w_out, cap_w: int, d_vecs_out, cap_v: int) -> None:
    """Enqueues a whole portfolio step; collect it with shifter_portfolio_end."""
    k = len(n_prune)
    arr = (C.c_uint64 * max(k, 1))(*[int(p) for p in n_prune])
    a = PortfolioArgs(_ptr(d_w), _ptr(d_vecs), arr, k, flags, _ptr(d_thr), _ptr(d_w_sparse),
                      w_stride, _ptr(d_mask), mask_stride, _ptr(d_out_alive), _ptr(d_in_alive),
                      _ptr(d_group_alive), _ptr(d_index_map), _ptr(d_keep), _ptr(d_new_width),
                      _ptr(d_w_out), cap_w, _ptr(d_vecs_out), cap_v)
    _check(load_library().shifter_portfolio_begin(ctx.handle, model.handle, C.byref(a)), ctx.handle)
    ctx._portfolio_k = k


def shifter_portfolio_end(ctx: Context, model: Model):
    """(records, (status, tensor descs, vec descs, elems_w, elems_v)) of the last
    shifter_portfolio_begin; the descriptor arrays are flat as in shifter_compact_batch."""
    k = ctx._portfolio_k
    n_t, n_v = model.info.n_tensors, model.info.n_vecs
    h = (Threshold * k)()
    ot = (TensorDesc * (n_t * k))()
    ov = (VecDesc * max(n_v * k, 1))()
    ew = (C.c_uint64 * k)()
    ev = (C.c_uint64 * k)()
    rc = _check(load_library().shifter_portfolio_end(ctx.handle, h, ot, ov, ew, ev), ctx.handle,
                allow=(SHIFTER_WARN_COLLAPSE,))
    return list(h), (rc, ot, ov, ew, ev)


def shifter_global_threshold_begin(ctx: Context, model: Model, d_w, n_prune, d_thr) -> None:
    k = len(n_prune)
    arr = (C.c_uint64 * k)(*[int(p) for p in n_prune])
    _check(load_library().shifter_global_threshold_begin(ctx.handle, model.handle, _ptr(d_w), arr,
                                                         k, _ptr(d_thr)), ctx.handle)
    ctx._rank_k = k


def shifter_global_threshold_end(ctx: Context):
    """(records, redone) of the last shifter_global_threshold_begin."""
    k = ctx._rank_k
    h = (Threshold * k)()
    redone = C.c_int()
    _check(load_library().shifter_global_threshold_end(ctx.handle, h, C.byref(redone)), ctx.handle)
    return list(h), bool(redone.value)


def shifter_kernel_scan(ctx: Context, model: Model, d_w_sparse, d_kernel_nz) -> None:
    _check(load_library().shifter_kernel_scan(ctx.handle, model.handle, _ptr(d_w_sparse),
                                              _ptr(d_kernel_nz)), ctx.handle)


def shifter_propagate_groups_fixpoint(ctx: Context, model: Model, d_kernel_nz, flags: int,
                                      d_group_alive, d_index_map, d_keep, d_new_width,
                                      sync: bool = True):
    """Returns (status, new_width list, rounds); with sync=False nothing is waited for and
    nothing read back (see shifter_fixpoint_status)."""
    if not sync:
        _check(load_library().shifter_propagate_groups_fixpoint(
            ctx.handle, model.handle, _ptr(d_kernel_nz), flags, _ptr(d_group_alive),
            _ptr(d_index_map), _ptr(d_keep), _ptr(d_new_width), None, None), ctx.handle)
        return SHIFTER_OK, None, None
    h = (C.c_uint32 * model.info.n_groups)()
    rounds = C.c_uint32()
    rc = _check(load_library().shifter_propagate_groups_fixpoint(
        ctx.handle, model.handle, _ptr(d_kernel_nz), flags, _ptr(d_group_alive),
        _ptr(d_index_map), _ptr(d_keep), _ptr(d_new_width), h, C.byref(rounds)),
        ctx.handle, allow=(SHIFTER_WARN_COLLAPSE,))
    return rc, list(h), int(rounds.value)


def shifter_set_select_grid(ctx: Context, blocks: int) -> None:
    _check(load_library().shifter_set_select_grid(ctx.handle, blocks), ctx.handle)


def shifter_set_fused_min_bytes(ctx: Context, n_bytes: int) -> None:
    _check(load_library().shifter_set_fused_min_bytes(ctx.handle, n_bytes), ctx.handle)


def shifter_fixpoint_status(ctx: Context, model: Model):
    """(rounds, settled) of the last fixpoint call, once its stream has been waited for."""
    rounds, settled = C.c_uint32(), C.c_uint32()
    _check(load_library().shifter_fixpoint_status(ctx.handle, model.handle, C.byref(rounds),
                                                  C.byref(settled)), ctx.handle)
    return int(rounds.value), bool(settled.value)


def shifter_compact(ctx: Context, model: Model, d_w_sparse, d_vecs, d_keep, d_new_width,
                    d_w_out, d_vecs_out, sync: bool = True):
    """Capacities are the lengths of d_w_out / d_vecs_out.  When sync, returns
    (status, tensor descs, vec descs, elems_w, elems_v)."""
    cap_w = d_w_out.numel()
    cap_v = d_vecs_out.numel() if d_vecs_out is not None else 0
    if not sync:
        _check(load_library().shifter_compact(
            ctx.handle, model.handle, _ptr(d_w_sparse), _ptr(d_vecs), _ptr(d_keep),
            _ptr(d_new_width), _ptr(d_w_out), cap_w, _ptr(d_vecs_out), cap_v, None, None,
            None, None), ctx.handle)
        return SHIFTER_OK, None, None, None, None
    ot = (TensorDesc * model.info.n_tensors)()
    ov = (VecDesc * max(model.info.n_vecs, 1))()
    ew, ev = C.c_uint64(), C.c_uint64()
    rc = load_library().shifter_compact(
        ctx.handle, model.handle, _ptr(d_w_sparse), _ptr(d_vecs), _ptr(d_keep),
        _ptr(d_new_width), _ptr(d_w_out), cap_w, _ptr(d_vecs_out), cap_v, ot, ov,
        C.byref(ew), C.byref(ev))
    if rc == SHIFTER_ERR_CAPACITY:
        raise ShifterError(rc, f"{shifter_last_error(ctx)} (needs {ew.value} weight floats, "
                               f"{ev.value} vector floats)")
    _check(rc, ctx.handle, allow=(SHIFTER_WARN_COLLAPSE,))
    return rc, list(ot), list(ov)[:model.info.n_vecs], ew.value, ev.value


def shifter_apply_mask_batch(ctx: Context, model: Model, d_w, d_thr, k: int, d_w_out,
                             w_stride: int, d_mask, mask_stride: int, d_out_alive,
                             d_in_alive=None) -> None:
    _check(load_library().shifter_apply_mask_batch(
        ctx.handle, model.handle, _ptr(d_w), _ptr(d_thr), k, _ptr(d_w_out), w_stride,
        _ptr(d_mask), mask_stride, _ptr(d_out_alive), _ptr(d_in_alive)), ctx.handle)


def shifter_propagate_groups_batch(ctx: Context, model: Model, d_out_alive, k: int, flags: int,
                                   d_group_alive, d_index_map, d_keep, d_new_width,
                                   sync: bool = True):
    h = (C.c_uint32 * (model.info.n_groups * k))() if sync else None
    rc = _check(load_library().shifter_propagate_groups_batch(
        ctx.handle, model.handle, _ptr(d_out_alive), k, flags, _ptr(d_group_alive),
        _ptr(d_index_map), _ptr(d_keep), _ptr(d_new_width), h), ctx.handle,
        allow=(SHIFTER_WARN_COLLAPSE,))
    return rc, (list(h) if sync else None)


def shifter_compact_batch(ctx: Context, model: Model, d_w_sparse, w_stride: int, d_vecs, d_keep,
                          d_new_width, k: int, d_w_out, cap_w: int, d_vecs_out, cap_v: int,
                          sync: bool = True):
    """When sync: (status, tensor descs, vec descs, elems_w, elems_v) as flat ctypes arrays
    (variant k's tensor i at [k * n_tensors + i], vector i at [k * n_vecs + i])."""
    if not sync:
        _check(load_library().shifter_compact_batch(
            ctx.handle, model.handle, _ptr(d_w_sparse), w_stride, _ptr(d_vecs), _ptr(d_keep),
            _ptr(d_new_width), k, _ptr(d_w_out), cap_w, _ptr(d_vecs_out), cap_v, None, None,
            None, None), ctx.handle)
        return SHIFTER_OK, None, None, None, None
    n_t, n_v = model.info.n_tensors, model.info.n_vecs
    ot = (TensorDesc * (n_t * k))()
    ov = (VecDesc * max(n_v * k, 1))()
    ew = (C.c_uint64 * k)()
    ev = (C.c_uint64 * k)()
    rc = _check(load_library().shifter_compact_batch(
        ctx.handle, model.handle, _ptr(d_w_sparse), w_stride, _ptr(d_vecs), _ptr(d_keep),
        _ptr(d_new_width), k, _ptr(d_w_out), cap_w, _ptr(d_vecs_out), cap_v, ot, ov, ew, ev),
        ctx.handle, allow=(SHIFTER_WARN_COLLAPSE,))
    return rc, ot, ov, ew, ev


def shifter_compact_batch_masked(ctx: Context, model: Model, d_w, d_thr, d_vecs, d_keep,
                                 d_new_width, k: int, d_w_out, cap_w: int, d_vecs_out, cap_v: int,
                                 sync: bool = True):
    """shifter_compact_batch with the dense arena and the K threshold records as its source;
    same return value."""
    fn = load_library().shifter_compact_batch_masked
    if not sync:
        _check(fn(ctx.handle, model.handle, _ptr(d_w), _ptr(d_thr), _ptr(d_vecs), _ptr(d_keep),
                  _ptr(d_new_width), k, _ptr(d_w_out), cap_w, _ptr(d_vecs_out), cap_v, None,
                  None, None, None), ctx.handle)
        return SHIFTER_OK, None, None, None, None
    n_t, n_v = model.info.n_tensors, model.info.n_vecs
    ot = (TensorDesc * (n_t * k))()
    ov = (VecDesc * max(n_v * k, 1))()
    ew = (C.c_uint64 * k)()
    ev = (C.c_uint64 * k)()
    rc = _check(fn(ctx.handle, model.handle, _ptr(d_w), _ptr(d_thr), _ptr(d_vecs), _ptr(d_keep),
                   _ptr(d_new_width), k, _ptr(d_w_out), cap_w, _ptr(d_vecs_out), cap_v, ot, ov,
                   ew, ev), ctx.handle, allow=(SHIFTER_WARN_COLLAPSE,))
    return rc, ot, ov, ew, ev


def shifter_profile_enable(ctx: Context, on: bool) -> None:
    _check(load_library().shifter_profile_enable(ctx.handle, 1 if on else 0), ctx.handle)


def shifter_profile_read(ctx: Context):
    """Returns {kernel name: (launch count, total ms)} since the last read."""
    cap = 32
    names = (C.c_char_p * cap)()
    counts = (C.c_uint32 * cap)()
    ms = (C.c_double * cap)()
    n = C.c_uint32()
    _check(load_library().shifter_profile_read(ctx.handle, names, counts, ms, cap, C.byref(n)),
           ctx.handle)
    return {names[i].decode(): (counts[i], ms[i]) for i in range(n.value)}


def shifter_copy_f32(ctx: Context, d_src, d_dst, n: int) -> None:
    _check(load_library().shifter_copy_f32(ctx.handle, _ptr(d_src), _ptr(d_dst), n), ctx.handle)
