"""Test-side helpers: a float64 forward pass, layer linearisation, a second DeepPoly in NumPy.

Nothing here is used by the HIP library or by the oracle.
"""
from __future__ import annotations

import numpy as np
import torch
import torch.nn.functional as F

import workloads as wl


def _avgpool(v, L):
    """Average pooling with zero padding and the divisor always kh*kw (padding of any size below the window)."""
    ph, pw = (L["pad"], L["pad"]) if np.isscalar(L["pad"]) else L["pad"]
    return F.avg_pool2d(F.pad(v, (pw, pw, ph, ph)), L["kernel"], stride=L["stride"], padding=0)


def forward(net: wl.Net, X: np.ndarray):
    """Concrete float64 forward pass.  X: [batch, n_in] (CHW-flattened).  Returns {layer id: [batch, n]}."""
    X = torch.as_tensor(np.asarray(X, dtype=np.float64))
    B = X.shape[0]
    vals = {0: X.reshape(B, *net.input_shape)}
    for i, L in enumerate(net.layers, start=1):
        t = L["type"]
        if t == "dense":
            v = vals[L["src"]].reshape(B, -1) @ torch.as_tensor(L["W"].astype(np.float64)).T
            v = v + torch.as_tensor(L["b"].astype(np.float64))
            v = v.reshape(B, -1, 1, 1)
        elif t == "conv":
            v = F.conv2d(vals[L["src"]], torch.as_tensor(L["W"].astype(np.float64)),
                         torch.as_tensor(L["b"].astype(np.float64)), stride=L["stride"], padding=L["pad"])
        elif t == "avgpool":
            v = _avgpool(vals[L["src"]], L)
        elif t == "relu":
            v = torch.clamp(vals[L["src"]], min=0.0)
        elif t == "add":
            v = vals[L["a"]] + vals[L["b"]]
        else:
            raise ValueError(t)
        vals[i] = v
    return {k: v.reshape(B, -1).numpy() for k, v in vals.items()}


def affine_matrix(net: wl.Net, lid: int):
    """(A, b) with layer_lid(x_src) = A x_src + b for a dense or conv layer, by pushing basis vectors."""
    L = net.layers[lid - 1]
    src = L["src"]
    shp = net.shape_of(src)
    n = int(np.prod(shp))
    eye = torch.eye(n, dtype=torch.float64).reshape(n, *shp)
    zero = torch.zeros(1, *shp, dtype=torch.float64)
    if L["type"] == "dense":
        return L["W"].astype(np.float64), L["b"].astype(np.float64)
    if L["type"] == "avgpool":
        cols = _avgpool(eye, L)
        return cols.reshape(n, -1).T.numpy().copy(), np.zeros(cols[0].numel())
    W = torch.as_tensor(L["W"].astype(np.float64))
    bvec = F.conv2d(zero, W, torch.as_tensor(L["b"].astype(np.float64)), stride=L["stride"], padding=L["pad"])
    cols = F.conv2d(eye, W, None, stride=L["stride"], padding=L["pad"])
    return cols.reshape(n, -1).T.numpy().copy(), bvec.reshape(-1).numpy().copy()


def sample_box(lo, hi, n, rng, corners=True):
    lo = np.asarray(lo, np.float64)
    hi = np.asarray(hi, np.float64)
    X = lo + (hi - lo) * rng.random((n, lo.size))
    if corners:
        m = n // 2
        pick = rng.random((m, lo.size)) < 0.5
        X[:m] = np.where(pick, lo, hi)
    return X


def ball_box(center, eps, clip_lo=0.0, clip_hi=1.0):
    c = np.asarray(center, np.float32).astype(np.float64)
    e = float(np.float32(eps))
    return np.maximum(c - e, clip_lo), np.minimum(c + e, clip_hi)


# ---- a second, independent DeepPoly: round-to-nearest float64, matrix form -----------------------
def _np_backsub(net, mats, bounds, relax, start, c0, upper, candidates):
    """start: {layer: matrix [rows, n_layer]}, c0: [rows].  Returns the best candidate per row."""
    expr = dict(start)
    c = np.array(c0, dtype=np.float64)
    best = np.full(c.shape[0], np.inf if upper else -np.inf)
    while True:
        k = max(expr)
        if len(expr) == 1 and k in bounds and (k == 0 or candidates == 0):
            l, u = bounds[k]
            Mp, Mn = np.maximum(expr[k], 0), np.minimum(expr[k], 0)
            v = (Mp @ u + Mn @ l + c) if upper else (Mp @ l + Mn @ u + c)
            best = np.minimum(best, v) if upper else np.maximum(best, v)
        if k == 0:
            return best
        M = expr.pop(k)
        L = net.layers[k - 1]
        if L["type"] in ("dense", "conv", "avgpool"):
            A, b = mats[k]
            expr[L["src"]] = expr.get(L["src"], 0) + M @ A
            c = c + M @ b
        elif L["type"] == "add":
            expr[L["a"]] = expr.get(L["a"], 0) + M
            expr[L["b"]] = expr.get(L["b"], 0) + M
        else:
            g, d, lam = relax[k]
            Mp, Mn = np.maximum(M, 0), np.minimum(M, 0)
            if upper:
                expr[L["src"]] = expr.get(L["src"], 0) + Mp * g + Mn * lam
                c = c + Mp @ d
            else:
                expr[L["src"]] = expr.get(L["src"], 0) + Mp * lam + Mn * g
                c = c + Mn @ d


def np_deeppoly(net: wl.Net, lo0, hi0, lambda_policy=0, candidates=0, extra_rows=None, lam_override=None):
    """All-neurons-at-once DeepPoly with plain float64 matrices (no outward rounding).

    Returns {layer id: (l, u)} for the input, ReLU inputs, ReLU layers and the last layer.
    extra_rows: optional matrix over the last layer; its lower bounds are returned under key "extra".
    lam_override: optional {ReLU layer id: array of 0/1}: the slope of the lower line to take for the neurons that
    are unstable here (the choice switches at u = -l, where two analyses that differ in the last bits can disagree)."""
    nL = len(net.layers)
    mats = {i: affine_matrix(net, i) for i, L in enumerate(net.layers, start=1) if L["type"] in ("dense", "conv", "avgpool")}
    feeds_relu = {L["src"] for L in net.layers if L["type"] == "relu"}
    bounds = {0: (np.asarray(lo0, np.float64), np.asarray(hi0, np.float64))}
    relax = {}

    def first_step(i, R):
        L = net.layers[i - 1]
        if L["type"] in ("dense", "conv", "avgpool"):
            A, b = mats[i]
            return {L["src"]: R @ A}, R @ b
        s = {}
        s[L["a"]] = s.get(L["a"], 0) + R
        s[L["b"]] = s.get(L["b"], 0) + R
        return s, np.zeros(R.shape[0])

    for i, L in enumerate(net.layers, start=1):
        if L["type"] == "relu":
            l, u = bounds[L["src"]]
            uns = (l < 0) & (u > 0)
            den = np.where(uns, u - l, 1.0)
            g = np.where(l >= 0, 1.0, np.where(u <= 0, 0.0, u / den))
            d = np.where(uns, -l * u / den, 0.0)
            lam_u = {0: (u > -l).astype(np.float64), 1: np.zeros_like(l), 2: np.ones_like(l)}[lambda_policy]
            if lam_override is not None and i in lam_override:
                lam_u = np.asarray(lam_override[i], np.float64)
            lam = np.where(l >= 0, 1.0, np.where(u <= 0, 0.0, lam_u))
            relax[i] = (g, d, lam)
            bounds[i] = (np.maximum(l, 0), np.maximum(u, 0))
        elif i in feeds_relu or i == nL:
            s, c0 = first_step(i, np.eye(net.n_neurons(i)))
            up = _np_backsub(net, mats, bounds, relax, s, c0, True, candidates)
            lw = _np_backsub(net, mats, bounds, relax, s, c0, False, candidates)
            bounds[i] = (lw, up)
    if extra_rows is not None:
        s, c0 = first_step(nL, np.asarray(extra_rows, np.float64))
        bounds["extra"] = _np_backsub(net, mats, bounds, relax, s, c0, False, candidates)
    return bounds


def np_deeppoly_early(net: wl.Net, lo0, hi0):
    """The early-termination procedure (Sections 3.2 and 4.2) written a second time, in matrix form with
    round-to-nearest float64: interval image of every layer first, only the neurons of a ReLU's input layer
    whose interval strictly contains 0 are back-substituted, upper and lower expression side by side, and a
    neuron's rows are removed from the matrices as soon as a candidate shows l >= 0 or u <= 0.

    Returns (bounds, term, ival): {layer: (l, u)}, {layer: int array}, {layer: (l, u)}."""
    nL = len(net.layers)
    mats = {i: affine_matrix(net, i) for i, L in enumerate(net.layers, start=1) if L["type"] in ("dense", "conv", "avgpool")}
    feeds_relu = {L["src"] for L in net.layers if L["type"] == "relu"}
    bounds = {0: (np.asarray(lo0, np.float64), np.asarray(hi0, np.float64))}
    ival, relax, term = {}, {}, {}

    def known(q):
        return bounds[q] if q in bounds else ival[q]

    def substitute(expr, c, k, upper):
        M = expr.pop(k)
        L = net.layers[k - 1]
        if L["type"] in ("dense", "conv", "avgpool"):
            A, b = mats[k]
            expr[L["src"]] = expr.get(L["src"], 0) + M @ A
            c = c + M @ b
        elif L["type"] == "add":
            expr[L["a"]] = expr.get(L["a"], 0) + M
            expr[L["b"]] = expr.get(L["b"], 0) + M
        else:
            g, d, lam = relax[k]
            Mp, Mn = np.maximum(M, 0), np.minimum(M, 0)
            if upper:
                expr[L["src"]] = expr.get(L["src"], 0) + Mp * g + Mn * lam
                c = c + Mp @ d
            else:
                expr[L["src"]] = expr.get(L["src"], 0) + Mp * lam + Mn * g
                c = c + Mn @ d
        return c

    for i, L in enumerate(net.layers, start=1):
        t = L["type"]
        if t == "relu":
            l, u = bounds[L["src"]]
            uns = (l < 0) & (u > 0)
            den = np.where(uns, u - l, 1.0)
            g = np.where(l >= 0, 1.0, np.where(u <= 0, 0.0, u / den))
            d = np.where(uns, -l * u / den, 0.0)
            lam = np.where(l >= 0, 1.0, np.where(u <= 0, 0.0, (u > -l).astype(np.float64)))
            relax[i] = (g, d, lam)
            bounds[i] = (np.maximum(l, 0), np.maximum(u, 0))
            continue
        if t == "add":
            (la, ua), (lb, ub) = known(L["a"]), known(L["b"])
            ival[i] = (la + lb, ua + ub)
        else:
            A, b = mats[i]
            pl, pu = known(L["src"])
            Ap, An = np.maximum(A, 0), np.minimum(A, 0)
            ival[i] = (Ap @ pl + An @ pu + b, Ap @ pu + An @ pl + b)
        if not (i in feeds_relu or i == nL):
            continue
        may_stop = i in feeds_relu and i != nL
        lo, hi = ival[i][0].copy(), ival[i][1].copy()
        n = lo.size
        tm = np.zeros(n, np.int64)
        idx = np.arange(n)
        if may_stop:
            act = (lo < 0) & (hi > 0)
            tm[~act] = i
            idx = idx[act]
        R = np.eye(n)[idx]
        eu, el = {i: R.copy()}, {i: R.copy()}
        cu, cl = np.zeros(idx.size), np.zeros(idx.size)
        cu = substitute(eu, cu, i, True)
        cl = substitute(el, cl, i, False)
        while idx.size:
            k = max(eu)
            if len(eu) == 1 and k in bounds:
                l, u = bounds[k]
                hi[idx] = np.minimum(hi[idx], np.maximum(eu[k], 0) @ u + np.minimum(eu[k], 0) @ l + cu)
                lo[idx] = np.maximum(lo[idx], np.maximum(el[k], 0) @ l + np.minimum(el[k], 0) @ u + cl)
                if k > 0 and may_stop:
                    done = (lo[idx] >= 0) | (hi[idx] <= 0)
                    tm[idx[done]] = k
                    keep = ~done
                    idx, cu, cl = idx[keep], cu[keep], cl[keep]
                    eu = {q: M[keep] for q, M in eu.items()}
                    el = {q: M[keep] for q, M in el.items()}
            if k == 0:
                break
            cu = substitute(eu, cu, k, True)
            cl = substitute(el, cl, k, False)
        bounds[i] = (lo, hi)
        term[i] = tm
    return bounds, term, ival


# ---- float32 inference in a chosen summation order ------------------------------------------------------
def _sum_f32(terms: np.ndarray, order: str, rng) -> np.ndarray:
    """Row-wise float32 sum of terms [rows, n] taken in the given order (every partial sum is rounded to float32)."""
    t = np.ascontiguousarray(terms, dtype=np.float32)
    n = t.shape[1]
    if order == "forward":
        idx = np.arange(n)
    elif order == "reverse":
        idx = np.arange(n)[::-1]
    elif order == "random":
        idx = rng.permutation(n)
    elif order in ("ascending", "descending"):       # by magnitude, per row
        key = np.abs(t) if order == "ascending" else -np.abs(t)
        t = np.take_along_axis(t, np.argsort(key, axis=1, kind="stable"), axis=1)
        idx = np.arange(n)
    elif order == "pairwise":                        # balanced tree
        cur = t
        while cur.shape[1] > 1:
            if cur.shape[1] % 2:
                cur = np.concatenate([cur, np.zeros((cur.shape[0], 1), np.float32)], axis=1)
            cur = (cur[:, 0::2] + cur[:, 1::2]).astype(np.float32)
        return cur[:, 0]
    else:
        raise ValueError(order)
    t = t[:, idx]
    acc = np.zeros(t.shape[0], np.float32)
    for k in range(n):                               # strictly sequential float32 accumulation
        acc = (acc + t[:, k]).astype(np.float32)
    return acc


def forward_float32(net: wl.Net, x: np.ndarray, order: str, rng) -> dict:
    """One float32 inference of the network at the float32 point x: every affine neuron is the float32 sum, in
    the given order, of its float32 products and its bias; an average is the float32 sum of its window, divided by
    the window size or multiplied by its rounded reciprocal; a residual sum is one float32 addition; ReLU is exact.
    Returns {layer id: float32 [n]} (CHW order).  Test-side code: the order models what an inference engine may do."""
    vals = {0: np.asarray(x, np.float32).reshape(-1)}
    for i, L in enumerate(net.layers, start=1):
        t = L["type"]
        if t == "avgpool":                           # float32 sum of the window in the given order, then one scaling
            A, _ = affine_matrix(net, i)
            k = L["kernel"]
            K = np.float32(k * k if np.isscalar(k) else k[0] * k[1])
            terms = np.where(A != 0, vals[L["src"]][None, :], np.float32(0)).astype(np.float32)
            s_ = _sum_f32(terms, order, rng)
            vals[i] = (s_ / K).astype(np.float32) if rng.random() < 0.5 else (s_ * (np.float32(1) / K)).astype(np.float32)
        elif t in ("dense", "conv"):
            A, b = affine_matrix(net, i)             # exact float32 values held in float64
            A32, b32 = A.astype(np.float32), b.astype(np.float32)
            assert np.array_equal(A32.astype(np.float64), A) and np.array_equal(b32.astype(np.float64), b)
            prod = (A32 * vals[L["src"]][None, :]).astype(np.float32)      # rounded products
            terms = np.concatenate([prod, b32[:, None]], axis=1)
            if t == "conv":                          # taps that fall into the padding are not terms of the sum
                terms = np.where(np.concatenate([A32 != 0, np.ones((A32.shape[0], 1), bool)], axis=1), terms, np.float32(0))
            vals[i] = _sum_f32(terms, order, rng)
        elif t == "relu":
            vals[i] = np.maximum(vals[L["src"]], np.float32(0))
        elif t == "add":
            vals[i] = (vals[L["a"]] + vals[L["b"]]).astype(np.float32)
        else:
            raise ValueError(t)
    return vals


FLOAT32_ORDERS = ("forward", "reverse", "random", "ascending", "descending", "pairwise")
