"""Operator value definitions, one textbook formula each, in float64.

Every function takes and returns numpy float64 (or int64) arrays.  Rounding to
the storage type of the output tensor is applied by the caller after each
operator, because the unfused graph materialises every operator output.
"""
from __future__ import annotations

import numpy as np
from scipy.special import erf

INT_MAX = 2 ** 31 - 1


def round_to(x: np.ndarray, dtype: str) -> np.ndarray:
    """Round float64 values to the storage type and return them as float64 again."""
    if dtype == "f32":
        return x.astype(np.float32).astype(np.float64)
    if dtype == "bf16":
        u = np.ascontiguousarray(x, dtype=np.float32).view(np.uint32)
        r = ((u + np.uint32(0x7FFF) + ((u >> np.uint32(16)) & np.uint32(1))) >> np.uint32(16)) << np.uint32(16)
        return r.astype(np.uint32).view(np.float32).astype(np.float64)
    if dtype in ("i64", "i32"):
        return x.astype(np.int64)
    raise ValueError(dtype)


def matmul(a, b, transB):
    return np.matmul(a, np.swapaxes(b, -1, -2) if transB else b)


def conv2d_nhwc(x, w, stride, pad):
    """out[n,oh,ow,o] = sum_{kh,kw,c} x[n, oh*s+kh-p, ow*s+kw-p, c] * w[o,kh,kw,c], zero padding."""
    n, h, wd, c = x.shape
    o, kh, kw, ci = w.shape
    assert c == ci
    oh = (h + 2 * pad - kh) // stride + 1
    ow = (wd + 2 * pad - kw) // stride + 1
    xp = np.zeros((n, h + 2 * pad, wd + 2 * pad, c), dtype=np.float64)
    xp[:, pad:pad + h, pad:pad + wd, :] = x
    out = np.zeros((n, oh, ow, o), dtype=np.float64)
    for i in range(kh):
        for j in range(kw):
            patch = xp[:, i:i + (oh - 1) * stride + 1:stride, j:j + (ow - 1) * stride + 1:stride, :]
            out += np.tensordot(patch, w[:, i, j, :], axes=([3], [1]))
    return out


def maxpool_nhwc(x, k, stride, pad):
    n, h, wd, c = x.shape
    oh = (h + 2 * pad - k) // stride + 1
    ow = (wd + 2 * pad - k) // stride + 1
    xp = np.full((n, h + 2 * pad, wd + 2 * pad, c), -np.inf)
    xp[:, pad:pad + h, pad:pad + wd, :] = x
    out = np.full((n, oh, ow, c), -np.inf)
    for i in range(k):
        for j in range(k):
            out = np.maximum(out, xp[:, i:i + (oh - 1) * stride + 1:stride, j:j + (ow - 1) * stride + 1:stride, :])
    return out


def avgpool_nhwc(x, k, stride, pad):
    """AveragePool (Table 2), channels last: the mean over the window positions that lie inside the input
    (padding positions are not counted)."""
    n, h, wd, c = x.shape
    oh = (h + 2 * pad - k) // stride + 1
    ow = (wd + 2 * pad - k) // stride + 1
    out = np.zeros((n, oh, ow, c))
    for i in range(oh):
        r0, r1 = max(i * stride - pad, 0), min(i * stride - pad + k, h)
        for j in range(ow):
            c0, c1 = max(j * stride - pad, 0), min(j * stride - pad + k, wd)
            out[:, i, j, :] = x[:, r0:r1, c0:c1, :].sum(axis=(1, 2)) / ((r1 - r0) * (c1 - c0))
    return out


def gelu(x):
    return 0.5 * x * (1.0 + erf(x / np.sqrt(2.0)))


def sigmoid(x):
    return 1.0 / (1.0 + np.exp(-x))


def softmax(x, causal):
    """Over the last axis; with ``causal`` row i of the last two axes sees columns j <= i + (Lk - Lq)."""
    if causal:
        lq, lk = x.shape[-2], x.shape[-1]
        i = np.arange(lq)[:, None]
        j = np.arange(lk)[None, :]
        x = np.where(j <= i + (lk - lq), x, -np.inf)
    m = x.max(axis=-1, keepdims=True)
    e = np.exp(x - m)
    return e / e.sum(axis=-1, keepdims=True)


def layernorm(x, gamma, beta, eps):
    mu = x.mean(axis=-1, keepdims=True)
    var = ((x - mu) ** 2).mean(axis=-1, keepdims=True)      # biased variance
    return (x - mu) / np.sqrt(var + eps) * gamma + beta


def maxunpool(x, idx, out_shape):
    """MaxUnpool (Table 2; the partial inverse of MaxPool): a tensor of zeros of shape ``out_shape`` in which
    element ``idx[i]`` (a position in the flattened result, as a pooling operator reports where it found each
    maximum) holds ``x[i]``.  Positions outside the result are ignored; the positions are expected to be distinct
    (windows that do not overlap), with repeats the highest ``i`` stays."""
    out_shape = tuple(int(v) for v in np.asarray(out_shape).reshape(-1))
    y = np.zeros(int(np.prod(out_shape)), dtype=np.float64)
    flat_x = np.asarray(x, np.float64).reshape(-1)
    flat_i = np.asarray(idx, np.int64).reshape(-1)
    for i in range(flat_x.size):
        if 0 <= flat_i[i] < y.size:
            y[flat_i[i]] = flat_x[i]
    return y.reshape(out_shape)


def groupnorm(x, gamma, beta, groups, eps):
    """GroupNormalization (Table 2), channels last: x [N, ..., C]; the C channels form ``groups`` groups of consecutive
    channels; per sample and group, mean and biased variance over the group's channels at every position; then the
    per-channel scale and shift."""
    n, c = x.shape[0], x.shape[-1]
    assert c % groups == 0
    xs = x.reshape(n, -1, groups, c // groups)
    mu = xs.mean(axis=(1, 3), keepdims=True)
    var = ((xs - mu) ** 2).mean(axis=(1, 3), keepdims=True)
    return ((xs - mu) / np.sqrt(var + eps)).reshape(x.shape) * gamma + beta


def slice_(x, starts, ends, axes):
    idx = [slice(None)] * x.ndim
    for s, e, a in zip(starts, ends, axes):
        idx[a] = slice(int(s), None if e >= INT_MAX else int(e))
    return x[tuple(idx)]


def nms(scores, boxes, max_out, iou):
    """Non-maximum suppression (Table 2 lists NMS with the execution-determined operators: how many boxes
    survive is known only once it has run).  Boxes are visited by decreasing score, equal scores by increasing
    index; a box is kept unless it overlaps an already kept box by more than ``iou`` (intersection over union),
    and at most ``max_out`` boxes are kept (0: no limit).  The overlap test decides an integer result, so it is
    taken in the operands' own precision, fp32, each operation rounded on its own:
    intersection > iou * ((area_a + area_b) - intersection).  Returns the kept indices in visiting order."""
    f = np.float32
    s = np.asarray(scores, dtype=f).reshape(-1)
    b = np.asarray(boxes, dtype=f).reshape(-1, 4)
    order = np.argsort(-s, kind="stable")
    thr = f(iou)
    area = (b[:, 2] - b[:, 0]) * (b[:, 3] - b[:, 1])              # float32 arrays: every operation rounds to fp32
    kept = []
    for i in order:
        k = b[kept]                                               # the boxes kept so far
        iw = np.maximum(f(0), np.minimum(b[i, 2], k[:, 2]) - np.maximum(b[i, 0], k[:, 0]))
        ih = np.maximum(f(0), np.minimum(b[i, 3], k[:, 3]) - np.maximum(b[i, 1], k[:, 1]))
        inter = iw * ih
        union = (area[i] + area[kept]) - inter
        if not (inter > thr * union).any():
            kept.append(int(i))
            if max_out > 0 and len(kept) == max_out:
                break
    return np.asarray(kept, dtype=np.int64)


def nonzero(x):
    """Coordinates of the non-zero elements, one column per element in row-major order: [rank, count]."""
    x = np.asarray(x)
    cols = [idx for idx in np.ndindex(*x.shape) if x[idx] != 0]
    return np.asarray(cols, dtype=np.int64).reshape(len(cols), x.ndim).T


def resize_nearest(x, sizes):
    """Nearest neighbour over every axis: out[i0, i1, ..] = x[floor(i0 * D0 / S0), floor(i1 * D1 / S1), ..]."""
    x = np.asarray(x)
    out = x
    for ax, (d, s_) in enumerate(zip(x.shape, [int(v) for v in sizes])):
        idx = [(i * d) // s_ for i in range(s_)]
        out = np.take(out, idx, axis=ax)
    return out


def topk(x, k):
    """TopK (Table 2; the operator of Fig. 3(c)): the k largest entries of every row (last axis),
    largest first, and their positions; of equal entries the one at the lower position comes first
    (neither the paper nor ONNX fixes that order)."""
    x = np.asarray(x)
    order = np.argsort(-x, axis=-1, kind="stable")[..., :k]
    return np.take_along_axis(x, order, axis=-1), order.astype(np.int64)
