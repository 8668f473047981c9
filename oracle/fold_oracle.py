"""CPU oracle for the conv + BatchNorm fold.  TEST INFRASTRUCTURE ONLY.

Plain numpy in fp64, written from the definition; it shares no code with the HIP library
and must never be imported by the product path: only the tests, the smoke check and the
benchmark's CPU-baseline leg call it.

Module 1 of Sec. III-D (Model Pre-Processor) merges every convolution with the
BatchNorm layer that follows it, so that only convolutions (and their biases) remain for
the later modules.  The paper names the step and leaves the arithmetic to the cited
inference-time fusion, which is the textbook identity: in inference mode BatchNorm maps
channel o of its input to

    y_o = gamma_o * (x_o - mean_o) / sqrt(var_o + eps) + beta_o,

and x_o = conv(input, w[o]) + b_o is linear in w[o] and b_o, so with
s_o = gamma_o / sqrt(var_o + eps)

    w'[o, i, y, x] = w[o, i, y, x] * s_o        b'_o = beta_o + (b_o - mean_o) * s_o

(b_o = 0 for a convolution without a bias).  A layer with no BatchNorm keeps its weights
and its bias.  A filter that is entirely zero stays entirely zero, so the zero structure
that Modules 2 and 3 analyse is the same before and after the fold (unless gamma_o = 0,
which zeroes a whole filter).

``fold_bn`` is pinned by tests that do not go through it: the forward pass of the folded
network equals that of the unfolded one (BatchNorm evaluated by the library routine and
by its defining formula), closed forms (unit statistics, pure scale, pure shift), and a
single-channel case worked by hand; it is not "parity unpinned".

Inputs: descriptor objects with attributes (offset, out_ch, in_ch, kh, kw) for tensors,
(offset, length) for vectors and (tensor, gamma, beta, mean, var, bias, out_offset) for
the layers to fold; numpy arenas.
"""
from __future__ import annotations

from typing import Sequence, Tuple

import numpy as np


def fold_bn(w: np.ndarray, v: np.ndarray, tensors: Sequence, vecs: Sequence,
            folds: Sequence, eps: float, n_bias: int) -> Tuple[np.ndarray, np.ndarray]:
    """Module 1 (Sec. III-D).  Returns (folded weight arena, bias arena) in fp64.

    ``w``/``v`` are the weight and vector arenas of the unfused network, ``folds`` lists
    the layers with a BatchNorm and/or a bias; tensors not listed are copied unchanged.
    ``n_bias`` is the size of the bias arena (elements no layer writes stay 0)."""
    w_out = np.asarray(w, dtype=np.float64).copy()
    v64 = np.asarray(v, dtype=np.float64)
    bias = np.zeros(n_bias, dtype=np.float64)

    def vec(i):
        d = vecs[i]
        return v64[d.offset:d.offset + d.length]

    for f in folds:
        t = tensors[f.tensor]
        n = t.out_ch
        row = t.in_ch * t.kh * t.kw
        b = vec(f.bias) if f.bias >= 0 else np.zeros(n)
        if f.gamma >= 0:
            s = vec(f.gamma) / np.sqrt(vec(f.var) + np.float64(eps))
            b_new = vec(f.beta) + (b - vec(f.mean)) * s
            block = w_out[t.offset:t.offset + n * row].reshape(n, row)
            block *= s[:, None]
        else:
            b_new = b
        bias[f.out_offset:f.out_offset + n] = b_new
    return w_out, bias
