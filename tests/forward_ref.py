"""Forward pass of a synthetic network (test infrastructure, PyTorch CPU ops).

Used only to check forward equivalence: the compacted network must reproduce the
masked sparse network in which every removed channel outputs zero (Algorithm 2 of the
paper drops the bias of a pruned channel, i.e. defines that channel's output as 0).
"""
import numpy as np
import torch
import torch.nn.functional as F

BN_EPS = 1e-5


def forward(spec, tensor_arrays, vec_arrays, x, dtype=torch.float32):
    """tensor_arrays[i]: 4-D numpy OIHW; vec_arrays[i]: 1-D numpy; x: NCHW numpy."""
    act = {"x": torch.from_numpy(np.asarray(x)).to(dtype)}
    W = [torch.from_numpy(np.ascontiguousarray(a)).to(dtype) for a in tensor_arrays]
    V = [torch.from_numpy(np.ascontiguousarray(a)).to(dtype) for a in vec_arrays]
    for op in spec.ops:
        kind = op[0]
        if kind == "conv":
            _, t, stride, pad, src, dst = op
            act[dst] = F.conv2d(act[src], W[t], None, stride=stride, padding=pad)
        elif kind == "bn":
            _, (g, b, m, var), a = op
            y = act[a]
            sh = (1, -1, 1, 1)
            y = (y - V[m].view(sh)) / torch.sqrt(V[var].view(sh) + BN_EPS)
            act[a] = y * V[g].view(sh) + V[b].view(sh)
        elif kind == "bias":
            act[op[2]] = act[op[2]] + V[op[1]].view(1, -1, 1, 1)
        elif kind == "relu":
            act[op[1]] = torch.relu(act[op[1]])
        elif kind == "maxpool":
            _, k, s, p, a = op
            act[a] = F.max_pool2d(act[a], k, s, p)
        elif kind == "add":
            _, a, b, dst = op
            act[dst] = act[a] + act[b]
        elif kind == "gap":
            act[op[1]] = act[op[1]].mean(dim=(2, 3))
        elif kind == "linear":
            _, t, bvec, src, dst = op
            w2 = W[t].reshape(W[t].shape[0], -1)
            act[dst] = F.linear(act[src], w2, V[bvec] if bvec is not None else None)
        else:
            raise ValueError(kind)
    return act["logits"].double().numpy()


def split_dense(spec, w, v):
    ta = [w[t.offset:t.offset + t.numel].reshape(t.out_ch, t.in_ch, t.kh, t.kw)
          for t in spec.tensors]
    va = [v[d.offset:d.offset + d.length] for d in spec.vecs]
    return ta, va


def split_compacted(spec, w_c, v_c, tensor_shapes, vec_shapes):
    ta = [w_c[off:off + o * i * kh * kw].reshape(o, i, kh, kw)
          for (off, o, i, kh, kw) in tensor_shapes]
    va = [v_c[off:off + n] for (off, n) in vec_shapes]
    return ta, va


def neutralised_vecs(spec, v, group_alive):
    """Vector arena of the sparse reference: removed channels emit exactly zero.

    For a BatchNorm attached to a group, gamma = beta = mean = 0 on the group's dead
    channels (the variance is kept, so the output is 0 * x / sqrt(var + eps) + 0)."""
    v2 = v.copy()
    var_ids = {op[1][3] for op in spec.ops if op[0] == "bn"}
    for vi, d in enumerate(spec.vecs):
        if vi in var_ids:
            continue
        dead = group_alive[d.group] == 0
        v2[d.offset:d.offset + d.length][dead] = 0.0
    return v2


def forward_equivalence(spec, w_sparse, v, group_alive, comp_w, comp_v, tensor_shapes,
                        vec_shapes, seed, batch, hw=None, dtype=torch.float32):
    """Returns max |y_compact - y_sparse_neutralised| / max |y_sparse_neutralised|."""
    hw = hw or spec.input_hw
    rng = np.random.Generator(np.random.Philox(seed))
    x = rng.standard_normal((batch, spec.groups[0].width, hw, hw), dtype=np.float32)
    ta, va = split_dense(spec, w_sparse, neutralised_vecs(spec, v, group_alive))
    y_ref = forward(spec, ta, va, x, dtype)
    tc, vc = split_compacted(spec, comp_w, comp_v, tensor_shapes, vec_shapes)
    y = forward(spec, tc, vc, x, dtype)
    denom = np.abs(y_ref).max()
    assert np.isfinite(y_ref).all() and denom > 0
    return float(np.abs(y - y_ref).max() / denom)
