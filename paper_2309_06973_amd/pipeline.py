"""Device-side buffers for one network and the five calls of the pass in order.

Buffer management and argument marshalling only: every step runs in libshifter's HIP
kernels on the current torch stream.  Raises if no ROCm device is visible."""
from __future__ import annotations

from typing import List, Optional, Sequence

import numpy as np
import torch

from . import shifter as S


class Pipeline:
    def __init__(self, spec, w, v, device: int = 0,
                 max_variants: int = S.SHIFTER_MAX_VARIANTS):
        """w, v: the fp32 weight and vector arenas, numpy arrays (copied to the device) or
        float32 tensors already on it (used as they are)."""
        if not torch.cuda.is_available():
            raise RuntimeError("no ROCm device visible: the prune-and-compact pass has no "
                               "CPU path")
        self.spec = spec
        self.dev = torch.device("cuda", device)
        torch.cuda.set_device(self.dev)
        self.ctx = S.shifter_create(device, torch.cuda.current_stream().cuda_stream)
        self.model = S.shifter_model_create(spec.tensors, spec.vecs, spec.groups)
        info = self.model.info
        u8 = dict(dtype=torch.uint8, device=self.dev)
        self.d_w = w if isinstance(w, torch.Tensor) else torch.from_numpy(w).to(self.dev)
        self.d_vecs = v if isinstance(v, torch.Tensor) else torch.from_numpy(v).to(self.dev)
        for a, need in ((self.d_w, info.w_extent), (self.d_vecs, info.v_extent)):
            assert a.dtype == torch.float32 and a.device == self.dev and a.is_contiguous()
            assert a.numel() >= need
        self.d_w_sparse = torch.empty_like(self.d_w)
        self.d_mask = torch.empty(max(info.n_prunable, 4), **u8)
        self.d_out_alive = torch.empty(info.sum_out_ch, **u8)
        self.d_in_alive = torch.empty(info.sum_in_ch, **u8)
        self.d_group_alive = torch.empty(info.sum_group_width, **u8)
        self.d_index_map = torch.empty(info.sum_group_width, dtype=torch.int32, device=self.dev)
        self.d_keep = torch.empty(info.sum_group_width, dtype=torch.int32, device=self.dev)
        self.d_new_width = torch.empty(info.n_groups, dtype=torch.int32, device=self.dev)
        self.d_w_out = torch.empty(max(info.w_elems, 4), dtype=torch.float32, device=self.dev)
        self.d_vecs_out = torch.empty(max(info.v_elems, 4), dtype=torch.float32,
                                      device=self.dev)
        self.d_thr = torch.zeros(max_variants * S.THRESHOLD_BYTES, **u8)
        self.n_thr = 0

    def close(self):
        if self.model is not None:
            S.shifter_model_destroy(self.model)
            S.shifter_destroy(self.ctx)
            self.model = None

    # ---- the five steps -----------------------------------------------------------
    def global_threshold(self, n_prune: Sequence[int], sync: bool = True):
        self.n_thr = len(n_prune)
        return S.shifter_global_threshold(self.ctx, self.model, self.d_w, n_prune,
                                          self.d_thr, sync)

    def prune_fused(self, n_prune: int, defer: bool = False):
        """Steps 1-3 for one prune count in a single read of the arena.  defer: do not wait
        for the outcome (see prune_result)."""
        self.n_thr = 1
        return S.shifter_prune_fused(self.ctx, self.model, self.d_w, n_prune, self.d_thr,
                                     self.d_w_sparse, self.d_mask, self.d_out_alive,
                                     self.d_in_alive, defer)

    def prune_result(self):
        """(record, redone) of a deferred prune_fused; redone: repeat the later steps."""
        return S.shifter_prune_fused_result(self.ctx)

    def single(self, n_prune: int, flags: int = 0):
        """All five steps for one prune count with one wait: the plan and the rebuild are
        enqueued behind the fused pass before its outcome is known and repeated in the
        rare case that the pass has to be redone.  Returns (record, compact's tuple)."""
        self.prune_fused(n_prune, defer=True)
        self.propagate_groups(flags, sync=False)
        out = self.compact(sync=True)
        rec, redone = self.prune_result()
        if redone:
            self.propagate_groups(flags, sync=False)
            out = self.compact(sync=True)
        return rec, out

    def apply_mask(self, k: int = 0, fused_scan: bool = True, in_place: bool = False):
        dst = self.d_w if in_place else self.d_w_sparse
        S.shifter_apply_mask(self.ctx, self.model, self.d_w, self.d_thr, dst, self.d_mask,
                             self.d_out_alive if fused_scan else None,
                             self.d_in_alive if fused_scan else None, thr_index=k)

    def dead_channel_scan(self, src=None):
        S.shifter_dead_channel_scan(self.ctx, self.model,
                                    self.d_w_sparse if src is None else src,
                                    self.d_out_alive, self.d_in_alive)

    def propagate_groups(self, flags: int = 0, sync: bool = True):
        return S.shifter_propagate_groups(self.ctx, self.model, self.d_out_alive,
                                          self.d_in_alive, flags, self.d_group_alive,
                                          self.d_index_map, self.d_keep, self.d_new_width,
                                          sync)

    def fold_bn(self, folds, n_bias: int, eps: float, src=None, dst=None, bias=None):
        """Conv + BatchNorm fold of an arena (default: the sparse one) into ``dst`` (default:
        a new arena).  Returns (folded weight arena, bias arena of n_bias floats)."""
        src = self.d_w_sparse if src is None else src
        dst = torch.empty_like(src) if dst is None else dst
        d_bias = (torch.zeros(max(n_bias, 4), dtype=torch.float32, device=self.dev)
                  if bias is None else bias)
        S.shifter_fold_bn(self.ctx, self.model, folds, eps, src, self.d_vecs, dst, d_bias)
        return dst, d_bias

    def kernel_scan(self, src=None):
        """Kernel-level zero index of the sparse arena (input of the liveness fixpoint)."""
        if getattr(self, "d_kernel_nz", None) is None:
            self.d_kernel_nz = torch.empty(max(self.model.sum_kernels, 16), dtype=torch.uint8,
                                           device=self.dev)
        S.shifter_kernel_scan(self.ctx, self.model, self.d_w_sparse if src is None else src,
                              self.d_kernel_nz)

    def propagate_groups_fixpoint(self, flags: int = 0, sync: bool = True):
        return S.shifter_propagate_groups_fixpoint(self.ctx, self.model, self.d_kernel_nz, flags,
                                                   self.d_group_alive, self.d_index_map,
                                                   self.d_keep, self.d_new_width, sync)

    def compact(self, sync: bool = True, src=None):
        return S.shifter_compact(self.ctx, self.model,
                                 self.d_w_sparse if src is None else src, self.d_vecs,
                                 self.d_keep, self.d_new_width, self.d_w_out,
                                 self.d_vecs_out, sync)

    # ---- a whole portfolio per call -------------------------------------------------
    def enable_batch(self, k: int):
        """Allocates the K-variant output buffers (strides rounded to 64 elements)."""
        info = self.model.info
        r64 = lambda x: (int(x) + 63) // 64 * 64
        self.bk = k
        self.w_stride = r64(info.w_extent)
        self.m_stride = r64(max(info.n_prunable, 4))
        self.cap_w = r64(max(info.w_elems, 4))
        self.cap_v = r64(max(info.v_elems, 4))
        u8 = dict(dtype=torch.uint8, device=self.dev)
        i32 = dict(dtype=torch.int32, device=self.dev)
        f32 = dict(dtype=torch.float32, device=self.dev)
        self.b_w_sparse = torch.empty(k * self.w_stride, **f32)
        self.b_mask = torch.empty(k * self.m_stride, **u8)
        self.b_out_alive = torch.empty(k * info.sum_out_ch, **u8)
        self.b_in_alive = torch.empty(k * info.sum_in_ch, **u8)
        self.b_group_alive = torch.empty(k * info.sum_group_width, **u8)
        self.b_index_map = torch.empty(k * info.sum_group_width, **i32)
        self.b_keep = torch.empty(k * info.sum_group_width, **i32)
        self.b_new_width = torch.empty(k * info.n_groups, **i32)
        self.b_w_out = torch.empty(k * self.cap_w, **f32)
        self.b_vecs_out = torch.empty(k * self.cap_v, **f32)

    def portfolio(self, n_prune: Sequence[int], flags: int = 0, with_in_alive: bool = True,
                  sync: bool = True, from_sparse: bool = False, sparse_arenas: bool = True,
                  fused: Optional[bool] = None):
        """All five steps for every prune count.  fused: ranking, masks and flags in one read
        of the arena (else one ranking call, then the batched mask pass); by default for
        arenas larger than the last-level cache, where the second read costs a trip to
        memory (measured: 7 % faster on a 1.3 GB arena, 5 % slower on a 100 MB one).  The rebuild reads
        the dense arena and masks on the way unless from_sparse asks for the K sparse
        arenas as its source (same result).  sparse_arenas=False skips writing the K sparse
        arenas (masks, flags, plans and rebuilt variants only).
        Returns (threshold records, compact_batch's tuple)."""
        assert sparse_arenas or not from_sparse
        k = len(n_prune)
        assert k == self.bk
        self.n_thr = k
        recs = None
        if fused is None:
            fused = self.model.info.w_extent * 4 > (192 << 20)
        def later_steps():
            S.shifter_propagate_groups_batch(self.ctx, self.model, self.b_out_alive, k, flags,
                                             self.b_group_alive, self.b_index_map, self.b_keep,
                                             self.b_new_width, sync=False)
            if from_sparse:
                return S.shifter_compact_batch(self.ctx, self.model, self.b_w_sparse,
                                               self.w_stride, self.d_vecs, self.b_keep,
                                               self.b_new_width, k, self.b_w_out, self.cap_w,
                                               self.b_vecs_out, self.cap_v, sync=sync)
            return S.shifter_compact_batch_masked(self.ctx, self.model, self.d_w, self.d_thr,
                                                  self.d_vecs, self.b_keep, self.b_new_width, k,
                                                  self.b_w_out, self.cap_w, self.b_vecs_out,
                                                  self.cap_v, sync=sync)

        if fused:
            recs = S.shifter_prune_fused_batch(
                self.ctx, self.model, self.d_w, n_prune, self.d_thr,
                self.b_w_sparse if sparse_arenas else None, self.w_stride, self.b_mask,
                self.m_stride, self.b_out_alive, self.b_in_alive if with_in_alive else None)
            out = later_steps()
        else:
            # the ranking is enqueued and everything else behind it: one wait for the whole
            # step; in the rare case that the single pass could not decide, the later steps
            # are repeated on the exact records
            S.shifter_global_threshold_begin(self.ctx, self.model, self.d_w, n_prune, self.d_thr)
            while True:
                S.shifter_apply_mask_batch(self.ctx, self.model, self.d_w, self.d_thr, k,
                                           self.b_w_sparse if sparse_arenas else None,
                                           self.w_stride, self.b_mask, self.m_stride,
                                           self.b_out_alive,
                                           self.b_in_alive if with_in_alive else None)
                out = later_steps()
                if recs is not None:
                    break
                recs, redone = S.shifter_global_threshold_end(self.ctx)
                if not redone:
                    break
        return recs, out

    def step(self, n_prune: Sequence[int], flags: int = 0, with_in_alive: bool = True,
             sparse_arenas: bool = True):
        """All five steps for every prune count behind one pair of calls (the library
        chooses the fusion; one wait).  Works on the batch buffers (enable_batch) for
        several counts and on the single-variant buffers for one.  Returns (threshold
        records, compact_batch's tuple)."""
        k = len(n_prune)
        self.n_thr = k
        if k == 1 and getattr(self, "bk", 0) != 1:
            bufs = (self.d_w_sparse if sparse_arenas else None, 0, self.d_mask, 0,
                    self.d_out_alive, self.d_in_alive if with_in_alive else None,
                    self.d_group_alive, self.d_index_map, self.d_keep, self.d_new_width,
                    self.d_w_out, self.d_w_out.numel(), self.d_vecs_out, self.d_vecs_out.numel())
        else:
            assert k == self.bk
            bufs = (self.b_w_sparse if sparse_arenas else None, self.w_stride, self.b_mask,
                    self.m_stride, self.b_out_alive, self.b_in_alive if with_in_alive else None,
                    self.b_group_alive, self.b_index_map, self.b_keep, self.b_new_width,
                    self.b_w_out, self.cap_w, self.b_vecs_out, self.cap_v)
        S.shifter_portfolio_begin(self.ctx, self.model, self.d_w, self.d_vecs, n_prune, flags,
                                  self.d_thr, *bufs)
        return S.shifter_portfolio_end(self.ctx, self.model)

    def variant(self, k: int = 0, flags: int = 0, fused_scan: bool = True,
                sync: bool = True):
        """Steps 2-5 for threshold record k.  Returns compact()'s tuple."""
        self.apply_mask(k, fused_scan)
        if not fused_scan:
            self.dead_channel_scan()
        self.propagate_groups(flags, sync=False)
        return self.compact(sync)


def deflate_portfolio(pl: "Pipeline", elems_w: Sequence[int], elems_v: Sequence[int], codec=None):
    """Module 7 (Sec. III-E) on the rebuilt variants of the last portfolio() call: the
    variants ordered by size (smallest first, as the paper's switcher walks them) and each
    deflated (weights and per-channel vectors as one buffer).  elems_w / elems_v: the sizes
    portfolio() returned.  Returns [(variant index, Package)]."""
    codec = codec or Codec(device=pl.dev.index or 0, ctx=pl.ctx)
    order = sorted(range(len(elems_w)), key=lambda k: (int(elems_w[k]) + int(elems_v[k]), k))
    out = []
    for k in order:
        nw, nv = int(elems_w[k]), int(elems_v[k])
        buf = torch.cat((pl.b_w_out[k * pl.cap_w:k * pl.cap_w + nw],
                         pl.b_vecs_out[k * pl.cap_v:k * pl.cap_v + nv]))
        out.append((k, codec.deflate(buf)))
    return out


class Package:
    """One deflated buffer: the DEFLATE stream, and the side information and marks for
    inflating it in parallel."""
    def __init__(self, stream, seg_off, sub_bits, n_bytes: int, sub_marks):
        self.stream, self.seg_off, self.sub_bits, self.n_bytes = stream, seg_off, sub_bits, n_bytes
        self.sub_marks = sub_marks

    @property
    def stream_bytes(self) -> int:
        return self.stream.numel()


class Codec:
    """Buffers for deflating and inflating device tensors (marshalling only)."""
    def __init__(self, device: int = 0, ctx=None):
        if not torch.cuda.is_available():
            raise RuntimeError("no ROCm device visible: the codec has no CPU path")
        self.dev = torch.device("cuda", device)
        torch.cuda.set_device(self.dev)
        self.own = ctx is None
        self.ctx = ctx or S.shifter_create(device, torch.cuda.current_stream().cuda_stream)
        self.work = None

    def close(self):
        if self.own and self.ctx is not None:
            S.shifter_destroy(self.ctx)
        self.ctx = None

    def deflate(self, t, stream=None, sync: bool = True) -> Package:
        """Deflates the bytes of the contiguous device tensor ``t``.  ``stream``: a uint8
        buffer to write into (default: one of the largest possible size); the package's
        stream is the used part of it."""
        n_bytes = t.numel() * t.element_size()
        n_chunks, work_bytes, bound = S.shifter_codec_layout(n_bytes)
        if self.work is None or self.work.numel() < work_bytes:
            self.work = torch.empty(work_bytes, dtype=torch.uint8, device=self.dev)
        if stream is None:
            stream = torch.empty(bound, dtype=torch.uint8, device=self.dev)
        seg_off = torch.empty(n_chunks + 1, dtype=torch.int64, device=self.dev)
        sub_bits = torch.empty(n_chunks * (S.SHIFTER_CODEC_CHUNK // S.SHIFTER_CODEC_SUB),
                               dtype=torch.int16, device=self.dev)
        sub_marks = torch.empty(sub_bits.numel(), dtype=torch.int64, device=self.dev)
        total = S.shifter_deflate(self.ctx, t if n_bytes else None, n_bytes, self.work, stream,
                                  seg_off, sub_bits, sub_marks, sync)
        return Package(stream[:total] if sync else stream, seg_off, sub_bits, n_bytes, sub_marks)

    def inflate(self, p: Package, out=None, sync: bool = True, stream_bytes=None):
        """``stream_bytes``: the stream's size when the package's stream tensor is a larger
        buffer (a package made without waiting)."""
        if out is None:
            out = torch.empty(max(p.n_bytes, 16), dtype=torch.uint8, device=self.dev)
        S.shifter_inflate(self.ctx, p.stream, p.stream_bytes if stream_bytes is None else stream_bytes,
                          p.seg_off, p.sub_bits, p.sub_marks, p.n_bytes, out, sync)
        return out
