"""Oracle: layer-graph evaluation (test infrastructure).

Every layer is its textbook definition evaluated in fp64, with one rounding to
the storage type at the layer's output (the path stores every activation in
that type).  Convolution is cross-correlation with zero padding; the fp64
contraction is delegated to torch's CPU conv2d / matmul (a library primitive
used as one step; it is pinned against `direct_conv` below and closed forms in
the tests).  The paper is silent on all of this (models run inside an inference
engine, Sec. III-A step 4).
"""
from __future__ import annotations

import numpy as np
import torch
import torch.nn.functional as F

from .rounding import round_storage

ACT_NONE, ACT_RELU, ACT_SILU = 0, 1, 2
RES_NONE, RES_BEFORE_ACT, RES_AFTER_ACT = 0, 1, 2


def activation(x: np.ndarray, act: int) -> np.ndarray:
    if act == ACT_NONE:
        return x
    if act == ACT_RELU:
        return np.maximum(x, 0.0)
    if act == ACT_SILU:
        return x / (1.0 + np.exp(-x))
    raise ValueError(act)


def direct_conv(x: np.ndarray, w: np.ndarray, stride: int, pad: int) -> np.ndarray:
    """Brute-force definition, plain loops, fp64.  x [N][H][W][C], w [K][R][S][C] -> [N][Ho][Wo][K].

    y[n,p,q,k] = sum_{r,s,c} x[n, p*stride + r - pad, q*stride + s - pad, c] * w[k,r,s,c]
    with out-of-range x taken as 0.  Only for tiny tensors.
    """
    n, h, wd, c = x.shape
    k, r, s, _ = w.shape
    ho = (h + 2 * pad - r) // stride + 1
    wo = (wd + 2 * pad - s) // stride + 1
    y = np.zeros((n, ho, wo, k), np.float64)
    for ni in range(n):
        for p in range(ho):
            for q in range(wo):
                for ki in range(k):
                    acc = 0.0
                    for ri in range(r):
                        for si in range(s):
                            yy, xx = p * stride + ri - pad, q * stride + si - pad
                            if 0 <= yy < h and 0 <= xx < wd:
                                for ci in range(c):
                                    acc += float(x[ni, yy, xx, ci]) * float(w[ki, ri, si, ci])
                    y[ni, p, q, ki] = acc
    return y


def conv2d(x: np.ndarray, w: np.ndarray, stride: int, pad: int) -> np.ndarray:
    """Same definition as `direct_conv`, contraction done by torch in fp64."""
    xt = torch.from_numpy(np.ascontiguousarray(x, dtype=np.float64)).permute(0, 3, 1, 2)
    wt = torch.from_numpy(np.ascontiguousarray(w, dtype=np.float64)).permute(0, 3, 1, 2)
    y = F.conv2d(xt, wt, None, stride=stride, padding=pad)
    return y.permute(0, 2, 3, 1).contiguous().numpy()


def conv_layer_at(x: np.ndarray, L, dtype: str, positions, res: np.ndarray = None) -> np.ndarray:
    """One conv layer (definition of `direct_conv`, then bias, residual, activation and the storage rounding of
    `run_model`) evaluated only at the listed output positions (n, p, q).  x [N][H][W][C] holds the layer's input;
    res, if the layer has a residual input, the tensor it adds.  Returns [len(positions)][K].  Lets a full-size
    tensor be checked on samples without evaluating all of it."""
    n, h, wd, c = x.shape
    k, r, s, _ = L.weight.shape
    w64 = L.weight.astype(np.float64)
    out = np.zeros((len(positions), k), np.float64)
    for j, (ni, p, q) in enumerate(positions):
        acc = np.zeros(k, np.float64)
        for ri in range(r):
            for si in range(s):
                yy, xx = p * L.stride + ri - L.pad, q * L.stride + si - L.pad
                if 0 <= yy < h and 0 <= xx < wd:
                    acc += w64[:, ri, si, :] @ x[ni, yy, xx, :].astype(np.float64)
        y = acc + L.bias.astype(np.float64)
        if L.res_mode == RES_BEFORE_ACT:
            y = activation(y + res[ni, p, q].astype(np.float64), L.act)
        elif L.res_mode == RES_AFTER_ACT:
            y = activation(y, L.act) + res[ni, p, q].astype(np.float64)
        else:
            y = activation(y, L.act)
        out[j] = y
    return round_storage(out, dtype)


def maxpool(x: np.ndarray, k: int, stride: int, pad: int) -> np.ndarray:
    """Window maximum; padding counts as -inf."""
    n, h, w, c = x.shape
    ho = (h + 2 * pad - k) // stride + 1
    wo = (w + 2 * pad - k) // stride + 1
    xp = np.full((n, h + 2 * pad, w + 2 * pad, c), -np.inf, np.float64)
    xp[:, pad:pad + h, pad:pad + w] = x
    y = np.full((n, ho, wo, c), -np.inf, np.float64)
    for r in range(k):
        for s in range(k):
            y = np.maximum(y, xp[:, r:r + stride * ho:stride, s:s + stride * wo:stride])
    return y


def run_model(spec, x0: np.ndarray, keep_all: bool = False):
    """Evaluate the layer graph.  x0: fp32 [N][H][W][3] of storage-type values.

    Returns the list of all tensors (index = tensor id; entries not needed later
    are dropped to None unless keep_all) - fp32 arrays of storage-type values,
    except `fc` outputs which stay fp32 logits.
    """
    dt = spec.dtype
    last_use = {}
    for i, L in enumerate(spec.layers):
        for t in L.inputs:
            last_use[t] = i
    for t in spec.outputs:
        last_use[t] = len(spec.layers)
    ts = [np.asarray(x0, np.float32)]
    for i, L in enumerate(spec.layers):
        a = ts[L.inputs[0]].astype(np.float64)
        if L.op == "conv":
            y = conv2d(a, L.weight, L.stride, L.pad) + L.bias.astype(np.float64)
            if L.res_mode == RES_BEFORE_ACT:
                y = activation(y + ts[L.inputs[1]].astype(np.float64), L.act)
            elif L.res_mode == RES_AFTER_ACT:
                y = activation(y, L.act) + ts[L.inputs[1]].astype(np.float64)
            else:
                y = activation(y, L.act)
            y = round_storage(y, dt)
        elif L.op == "maxpool":
            y = round_storage(maxpool(a, L.kh, L.stride, L.pad), dt)
        elif L.op == "upsample2x":
            y = np.repeat(np.repeat(ts[L.inputs[0]], 2, axis=1), 2, axis=2)      # out[y][x] = in[y//2][x//2]
        elif L.op == "concat":
            y = np.concatenate([ts[t] for t in L.inputs], axis=3)
        elif L.op == "add":
            y = round_storage(activation(a + ts[L.inputs[1]].astype(np.float64), L.act), dt)
        elif L.op == "gap":
            y = round_storage(a.mean(axis=(1, 2), keepdims=True), dt)
        elif L.op == "fc":
            n = a.shape[0]
            wmat = L.weight.reshape(L.cout, -1).astype(np.float64)
            y = (a.reshape(n, -1) @ wmat.T + L.bias.astype(np.float64)).astype(np.float32).reshape(n, 1, 1, L.cout)
        else:
            raise ValueError(L.op)
        ts.append(y)
        if not keep_all:
            for t in L.inputs:
                if last_use.get(t, -1) == i:
                    ts[t] = None
    return ts


def argmax_labels(logits: np.ndarray) -> np.ndarray:
    """Index of the largest fp32 logit per row; lowest index on ties."""
    return np.argmax(logits.reshape(logits.shape[0], -1), axis=1).astype(np.int32)
