"""numpy front end of the CPU oracle (``laplex_oracle.c``).

TEST INFRASTRUCTURE ONLY.  Imported by ``tests/``, by the smoke check and by
the benchmark's CPU-baseline leg; never by the product package, and it imports
nothing of the product.  Inputs may be fp32 or fp64; they are widened to fp64
before anything is computed (App. "Numerical accuracy": the reference is the
fp64 evaluation of the same fp32 inputs).

Conventions: ``a`` (length k) are output anchors, ``b`` (length n) input
anchors, ``x`` is (n, batch), ``g`` is (k, batch), both batch-minor.
"""
from __future__ import annotations

import ctypes
import os
import subprocess

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "laplex_oracle.c")
_LIB = os.path.join(_HERE, "liblaplex_oracle.so")
_lib = None

_D = ctypes.POINTER(ctypes.c_double)
_I = ctypes.c_int64


def build(force: bool = False) -> str:
    """Compile the C oracle with gcc (fp64, OpenMP, no fast-math)."""
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        subprocess.check_call(
            ["gcc", "-O2", "-fopenmp", "-fPIC", "-shared", "-std=c11", "-Wall",
             "-o", _LIB, _SRC, "-lm"])
    return _LIB


def _load():
    global _lib
    if _lib is None:
        build()
        _lib = ctypes.CDLL(_LIB)
    return _lib


def _f64(v, ndim):
    v = np.ascontiguousarray(np.asarray(v), dtype=np.float64)
    if ndim == 2 and v.ndim == 1:
        v = v.reshape(-1, 1)
    assert v.ndim == ndim
    return v


def _p(v):
    return None if v is None else v.ctypes.data_as(_D)


# --------------------------------------------------------------------------
# Route A: the definition.
# --------------------------------------------------------------------------

def apply_brute(a, b, x):
    """y = L(a,b) x and the tolerance denominator sum_j L_ij |x_j|."""
    a, b, x = _f64(a, 1), _f64(b, 1), _f64(x, 2)
    k, n, batch = a.size, b.size, x.shape[1]
    assert x.shape[0] == n
    y = np.zeros((k, batch)); tol = np.zeros((k, batch))
    _load().oracle_apply_brute(_p(a), _I(k), _p(b), _I(n), _p(x), _I(batch), _I(batch),
                               _p(y), _p(tol), _I(batch))
    return y, tol


def apply_backward_brute(a, b, x, g):
    """(gx, ga, gb) and their tolerance denominators (tgx, tga, tgb)."""
    a, b, x, g = _f64(a, 1), _f64(b, 1), _f64(x, 2), _f64(g, 2)
    k, n, batch = a.size, b.size, x.shape[1]
    assert x.shape[0] == n and g.shape == (k, batch)
    gx = np.zeros((n, batch)); tgx = np.zeros((n, batch))
    ga = np.zeros(k); tga = np.zeros(k); gb = np.zeros(n); tgb = np.zeros(n)
    _load().oracle_apply_backward_brute(
        _p(a), _I(k), _p(b), _I(n), _p(x), _I(batch), _p(g), _I(batch), _I(batch),
        _p(gx), _p(tgx), _I(batch), _p(ga), _p(tga), _p(gb), _p(tgb))
    return (gx, ga, gb), (tgx, tga, tgb)


def gram_brute(a, x):
    a, x = _f64(a, 1), _f64(x, 2)
    n, batch = a.size, x.shape[1]
    assert x.shape[0] == n
    y = np.zeros((n, batch)); tol = np.zeros((n, batch))
    _load().oracle_gram_brute(_p(a), _I(n), _p(x), _I(batch), _I(batch), _p(y), _p(tol), _I(batch))
    return y, tol


def gram_backward_brute(a, x, g):
    a, x, g = _f64(a, 1), _f64(x, 2), _f64(g, 2)
    n, batch = a.size, x.shape[1]
    assert x.shape == g.shape == (n, batch)
    gx = np.zeros((n, batch)); tgx = np.zeros((n, batch)); ga = np.zeros(n); tga = np.zeros(n)
    _load().oracle_gram_backward_brute(_p(a), _I(n), _p(x), _I(batch), _p(g), _I(batch), _I(batch),
                                       _p(gx), _p(tgx), _I(batch), _p(ga), _p(tga))
    return (gx, ga), (tgx, tga)


# --------------------------------------------------------------------------
# The merged order (stable sort of a followed by b; equal anchors keep the
# order "outputs by index, then inputs by index").
# --------------------------------------------------------------------------

def merged_permutation(a, b=None):
    """ids of the stable ascending sort of concat(a, b) (or of a alone).
    numpy compares -0.0 == +0.0, so signed zeros tie, as intended."""
    m = np.asarray(a, dtype=np.float32) if b is None else np.concatenate(
        [np.asarray(a, dtype=np.float32), np.asarray(b, dtype=np.float32)])
    return np.argsort(m, kind="stable").astype(np.uint32)


# --------------------------------------------------------------------------
# Route B: Theorem "Dual reduction via the b-axis".
# --------------------------------------------------------------------------

def _dual(src, val, q, use_abs=False, want=(True, True, True)):
    """sort src (stable), carry val, evaluate the three sums at the queries."""
    src, val, q = _f64(src, 1), _f64(val, 2), _f64(q, 1)
    order = np.argsort(src, kind="stable")
    s = np.ascontiguousarray(src[order]); v = np.ascontiguousarray(val[order])
    batch = v.shape[1]
    outs = [np.zeros((q.size, batch)) if w else None for w in want]
    rc = _load().oracle_dual_sums(_p(s), _I(s.size), _p(v), _I(batch), _I(batch),
                                  _p(q), _I(q.size), ctypes.c_int(1 if use_abs else 0),
                                  _p(outs[0]), _p(outs[1]), _p(outs[2]), _I(batch))
    if rc != 0:
        raise MemoryError("oracle_dual_sums")
    return outs


def apply_scan(a, b, x, with_tol=True):
    """y = L(a,b) x through the dual theorem; also the tolerance denominator."""
    li, _, rs = _dual(b, x, a, want=(True, False, True))
    y = li + rs
    if not with_tol:
        return y, None
    li, _, rs = _dual(b, x, a, use_abs=True, want=(True, False, True))
    return y, li + rs


def apply_backward_scan(a, b, x, g):
    """(gx, ga, gb), (tgx, tga, tgb) through the dual theorem, used twice:
    inputs sorted / outputs queried for ga, outputs sorted / inputs queried
    (the transposed operator L(b,a)) for gx and gb.  Strict sums drop ties."""
    x64, g64 = _f64(x, 2), _f64(g, 2)
    _, ls, rs = _dual(b, x64, a, want=(False, True, True))
    ga = np.sum(g64 * (rs - ls), axis=1)
    li, _, rs_abs = _dual(b, x64, a, use_abs=True, want=(True, False, True))
    tga = np.sum(np.abs(g64) * (li + rs_abs), axis=1)
    li, ls, rs = _dual(a, g64, b)
    gx = li + rs
    gb = np.sum(x64 * (rs - ls), axis=1)
    li, _, rs = _dual(a, g64, b, use_abs=True, want=(True, False, True))
    tgx = li + rs
    tgb = np.sum(np.abs(x64) * tgx, axis=1)
    return (gx, ga, gb), (tgx, tga, tgb)


def gram_scan(a, x, with_tol=True):
    li, _, rs = _dual(a, x, a, want=(True, False, True))
    y = li + rs
    if not with_tol:
        return y, None
    li, _, rs = _dual(a, x, a, use_abs=True, want=(True, False, True))
    return y, li + rs


def gram_backward_scan(a, x, g):
    x64, g64 = _f64(x, 2), _f64(g, 2)
    lig, lsg, rsg = _dual(a, g64, a)
    _, lsx, rsx = _dual(a, x64, a, want=(False, True, True))
    gx = lig + rsg
    ga = np.sum(g64 * (rsx - lsx) + x64 * (rsg - lsg), axis=1)
    li, _, rs = _dual(a, g64, a, use_abs=True, want=(True, False, True))
    tgx = li + rs
    li, _, rs = _dual(a, x64, a, use_abs=True, want=(True, False, True))
    tga = np.sum(np.abs(g64) * (li + rs) + np.abs(x64) * tgx, axis=1)
    return (gx, ga), (tgx, tga)


# --------------------------------------------------------------------------
# Route C: the definition inside a window, on sampled outputs (batch 1).
# --------------------------------------------------------------------------

def apply_window(a_sample, b, x, window=64.0):
    """For each sampled output anchor: sum over inputs within ``window`` of it.
    What is dropped is below exp(-window) * sum|x| (2e-28 * sum|x| at 64)."""
    q, b, x = _f64(a_sample, 1), _f64(b, 1), _f64(x, 2)
    order = np.argsort(b, kind="stable")
    bs = np.ascontiguousarray(b[order]); xs = np.ascontiguousarray(x[order, :1])
    y = np.zeros(q.size); tol = np.zeros(q.size)
    _load().oracle_apply_window(_p(bs), _I(bs.size), _p(xs), _I(1), _p(q), _I(q.size),
                                ctypes.c_double(window), _p(y), _p(tol))
    return y, tol


# --------------------------------------------------------------------------
# Phased kernel (Sec. 3, "Phased Laplace kernels"):
#   P_ij = exp(-|a_i - b_j|) * cos(phi_i - psi_j),
# phi on the output anchors, psi on the input anchors.
# --------------------------------------------------------------------------

def _phased_dense(a, phi, b, psi):
    a, phi, b, psi = _f64(a, 1), _f64(phi, 1), _f64(b, 1), _f64(psi, 1)
    assert a.size == phi.size and b.size == psi.size
    diff = a[:, None] - b[None, :]
    L = np.exp(-np.abs(diff))
    ang = phi[:, None] - psi[None, :]
    return L, np.cos(ang), np.sin(ang), np.sign(diff)


def phased_apply_brute(a, phi, b, psi, x):
    """The definition, as a dense k x n matrix: y = P x, and the tolerance
    denominator sum_j L_ij |x_j| (|cos| <= 1)."""
    L, C, _, _ = _phased_dense(a, phi, b, psi)
    x = _f64(x, 2)
    return (L * C) @ x, L @ np.abs(x)


def phased_backward_brute(a, phi, b, psi, x, g):
    """Gradients of sum(g * (P x)) by differentiating the definition entry by
    entry (sgn(0) = 0 at ties): (gx, ga, gb, gphi, gpsi) and their tolerance
    denominators."""
    L, C, S, sgn = _phased_dense(a, phi, b, psi)
    x, g = _f64(x, 2), _f64(g, 2)
    M = g @ x.T                      # M_ij = sum_t g_it x_jt
    Mabs = np.abs(g) @ np.abs(x).T
    gx = (L * C).T @ g
    ga = np.sum(-sgn * L * C * M, axis=1)
    gb = np.sum(sgn * L * C * M, axis=0)
    gphi = np.sum(-L * S * M, axis=1)
    gpsi = np.sum(L * S * M, axis=0)
    tgx = L.T @ np.abs(g)
    trow = np.sum(L * Mabs, axis=1); tcol = np.sum(L * Mabs, axis=0)
    return (gx, ga, gb, gphi, gpsi), (tgx, trow, tcol, trow, tcol)


def phased_apply_scan(a, phi, b, psi, x):
    """The same through the angle-sum identity
    cos(phi - psi) = cos phi cos psi + sin phi sin psi: two non-phased products
    of the dual-theorem route with modulated inputs (for sizes where the dense
    matrix is too large)."""
    phi, psi, x = _f64(phi, 1), _f64(psi, 1), _f64(x, 2)
    yc, _ = apply_scan(a, b, x * np.cos(psi)[:, None], with_tol=False)
    ys, _ = apply_scan(a, b, x * np.sin(psi)[:, None], with_tol=False)
    _, tol = apply_scan(a, b, np.abs(x))
    return np.cos(phi)[:, None] * yc + np.sin(phi)[:, None] * ys, tol


def phased_backward_scan(a, phi, b, psi, x, g):
    """Gradients through the same identity: one non-phased forward and backward
    on the doubled batch [x cos psi | x sin psi], [g cos phi | g sin phi]."""
    phi, psi, x, g = _f64(phi, 1), _f64(psi, 1), _f64(x, 2), _f64(g, 2)
    B = x.shape[1]
    cf, sf, cp, sp = np.cos(phi)[:, None], np.sin(phi)[:, None], np.cos(psi)[:, None], np.sin(psi)[:, None]
    x2 = np.hstack([x * cp, x * sp]); g2 = np.hstack([g * cf, g * sf])
    (gx2, ga, gb), _ = apply_backward_scan(a, b, x2, g2)
    y2, _ = apply_scan(a, b, x2, with_tol=False)
    gx = cp * gx2[:, :B] + sp * gx2[:, B:]
    gphi = np.sum(g * (cf * y2[:, B:] - sf * y2[:, :B]), axis=1)
    gpsi = np.sum(x * (cp * gx2[:, B:] - sp * gx2[:, :B]), axis=1)
    _, (tgx, tga, tgb) = apply_backward_scan(a, b, x, g)
    return (gx, ga, gb, gphi, gpsi), (tgx, tga, tgb, tga, tgb)


# --------------------------------------------------------------------------
# Temperature (App. A "Expressivity"): L_t = [exp(-|a_i - b_j| / t)], with the
# inverse temperature tau = 1/t of the experiments: L_tau = exp(-tau |a_i - b_j|).
# --------------------------------------------------------------------------

def tau_apply_dense(a, b, tau, x):
    """The definition with the temperature inside the exponent (fp64 throughout)."""
    a, b, x = _f64(a, 1), _f64(b, 1), _f64(x, 2)
    L = np.exp(-float(tau) * np.abs(a[:, None] - b[None, :]))
    return L @ x, L @ np.abs(x)


def scaled_anchors(v, tau, fp32=True):
    """tau * v: rounded to fp32 (one multiplication, as the library forms its
    keys: the sorted order and the ties are those of the rounded products) or exact."""
    if fp32:
        return (np.float32(tau) * np.asarray(v, dtype=np.float32)).astype(np.float32)
    return float(tau) * _f64(v, 1)


def tau_apply(a, b, tau, x, fp32=True, brute=True):
    f = apply_brute if brute else apply_scan
    return f(scaled_anchors(a, tau, fp32), scaled_anchors(b, tau, fp32), x)


def tau_backward(a, b, tau, x, g, fp32=True, brute=True):
    """(gx, ga, gb, gtau) of sum(g * L_tau x) by the chain rule through the scaled
    anchors: ga = tau ga', gb = tau gb', gtau = sum a ga' + sum b gb'."""
    f = apply_backward_brute if brute else apply_backward_scan
    (gx, gas, gbs), (tgx, tga, tgb) = f(scaled_anchors(a, tau, fp32), scaled_anchors(b, tau, fp32), x, g)
    a64, b64 = _f64(a, 1), _f64(b, 1)
    gtau = float(np.dot(a64, gas) + np.dot(b64, gbs))
    ttau = float(np.dot(np.abs(a64), tga) + np.dot(np.abs(b64), tgb))
    t = float(tau)
    return (gx, t * gas, t * gbs, gtau), (tgx, t * tga, t * tgb, ttau)


def tau_gram_backward(a, tau, x, g, fp32=True, brute=True):
    f = gram_backward_brute if brute else gram_backward_scan
    (gx, gas), (tgx, tga) = f(scaled_anchors(a, tau, fp32), x, g)
    a64 = _f64(a, 1)
    t = float(tau)
    return (gx, t * gas, float(np.dot(a64, gas))), (tgx, t * tga, float(np.dot(np.abs(a64), tga)))


# --------------------------------------------------------------------------
# Weighted Gram matrix (Sec. 3 "Computation of Gram matrix"; App. "Fast weighted
# Gram matrix"):  M = A diag(d) A^T  with  A = L(a, b)  (k x n),  d in R^n:
#     M_ij = sum_t d_t exp(-|a_i - b_t|) exp(-|a_j - b_t|).
# In this repository's letters the Gram matrix is k x k (a: its k anchors) and
# b, d are the n middle anchors and their weights.
# --------------------------------------------------------------------------

def wgram_dense(a, b, d):
    """The definition, O(k^2 n): (M, T) with T the same sum over |d_t|."""
    a, b, d = _f64(a, 1), _f64(b, 1), _f64(d, 1)
    A = np.exp(-np.abs(a[:, None] - b[None, :]))
    return (A * d[None, :]) @ A.T, (A * np.abs(d)[None, :]) @ A.T


def _wgram_from_buckets(a, b, d):
    """Theorem "Exact Gram decomposition" with interval statistics.  Sorted anchors
    s_1 <= ... <= s_k cut the line into k + 1 intervals P_r = [s_{r-1}, s_r)
    (s_0 = -inf, s_{k+1} = +inf).  Per interval: u_r = sum e^{2(b_t - s_r)} d_t
    (relative to its right end), w_r = sum d_t, and the right-hand statistic taken
    relative to the interval's LEFT end, v_r = sum e^{-2(b_t - s_{r-1})} d_t: the
    theorem's e^{2(s_r - b_t)} has a positive exponent and overflows on wide
    intervals, and its index range r = 1..k leaves out the last interval.  Then
    U_j = sum_{r <= j} e^{-2(s_j - s_r)} u_r,  V_i = sum_{r > i} e^{-2(s_{r-1} - s_i)} v_r,
    W_i = sum_{r <= i} w_r,  and for i >= j
        M_ij = e^{s_j - s_i} (U_j + (W_i - W_j) + V_i)."""
    k = a.size
    order = np.argsort(a, kind="stable")
    s = a[order]
    bucket = np.searchsorted(s, b, side="right")          # number of anchors <= b_t: interval index r - 1, in 0..k
    left = np.concatenate([[-np.inf], s])                 # left end of interval r - 1
    right = np.concatenate([s, [np.inf]])
    with np.errstate(invalid="ignore"):
        eu = np.where(bucket < k, np.exp(2.0 * (b - right[bucket])), 0.0)     # the last interval has no right end
        ev = np.where(bucket > 0, np.exp(-2.0 * (b - left[bucket])), 0.0)     # the first none on the left
    u = np.bincount(bucket, weights=eu * d, minlength=k + 1)
    v = np.bincount(bucket, weights=ev * d, minlength=k + 1)
    w = np.bincount(bucket, weights=d, minlength=k + 1)
    U = np.zeros(k); V = np.zeros(k)
    for j in range(k):                                    # U_j = u_j + e^{-2(s_j - s_{j-1})} U_{j-1}
        U[j] = u[j] + (np.exp(-2.0 * (s[j] - s[j - 1])) * U[j - 1] if j else 0.0)
    for i in range(k - 1, -1, -1):                        # V_i = v_{i+1} + e^{-2(s_{i+1} - s_i)} V_{i+1}
        V[i] = v[i + 1] + (np.exp(-2.0 * (s[i + 1] - s[i])) * V[i + 1] if i + 1 < k else 0.0)
    W = np.cumsum(w[:k])
    hi = np.maximum(np.arange(k)[:, None], np.arange(k)[None, :])
    lo = np.minimum(np.arange(k)[:, None], np.arange(k)[None, :])
    Ms = np.exp(s[lo] - s[hi]) * (U[lo] + (W[hi] - W[lo]) + V[hi])
    M = np.empty_like(Ms)
    M[np.ix_(order, order)] = Ms
    return M


def wgram_scan(a, b, d):
    """(M, T) through the exact Gram decomposition, O(k^2 + n log k)."""
    a, b, d = _f64(a, 1), _f64(b, 1), _f64(d, 1)
    return _wgram_from_buckets(a, b, d), _wgram_from_buckets(a, b, np.abs(d))


# --------------------------------------------------------------------------
# LAPLEX^(r): a weighted sum of r Laplace-kernel operators with independent anchor
# pairs (Sec. 7 "Learned anchor geometry in neural heads"):  y = sum_q w_q L(a_q, b_q) x.
# a is (r, k), b is (r, n), w is (r,).
# --------------------------------------------------------------------------

def mix_apply(a, b, w, x, brute=True):
    """(y, T): the sum written out, one operator at a time; T sums |w_q| L_q |x|."""
    a, b, w = np.asarray(a), np.asarray(b), _f64(w, 1)
    f = apply_brute if brute else apply_scan
    y = tol = 0.0
    for q in range(w.size):
        yq, tq = f(a[q], b[q], x)
        y = y + w[q] * yq
        tol = tol + abs(w[q]) * tq
    return y, tol


def mix_backward(a, b, w, x, g, brute=True):
    """Gradients of sum(g * y): (gx, ga (r, k), gb (r, n), gw (r,)) and their tolerance
    denominators.  y is linear in every w_q L_q x, so gx = sum_q w_q L_q^T g, the anchor
    gradients of operator q are w_q times those of L_q alone, and gw_q = <g, L_q x>."""
    a, b, w = np.asarray(a), np.asarray(b), _f64(w, 1)
    g64 = _f64(g, 2)
    fb = apply_backward_brute if brute else apply_backward_scan
    ff = apply_brute if brute else apply_scan
    gx = tgx = 0.0
    ga, gb, tga, tgb, gw, tgw = [], [], [], [], [], []
    for q in range(w.size):
        (gxq, gaq, gbq), (tgxq, tgaq, tgbq) = fb(a[q], b[q], x, g)
        yq, tq = ff(a[q], b[q], x)
        gx = gx + w[q] * gxq; tgx = tgx + abs(w[q]) * tgxq
        ga.append(w[q] * gaq); gb.append(w[q] * gbq)
        tga.append(abs(w[q]) * tgaq); tgb.append(abs(w[q]) * tgbq)
        gw.append(float(np.sum(g64 * yq))); tgw.append(float(np.sum(np.abs(g64) * tq)))
    return ((gx, np.stack(ga), np.stack(gb), np.array(gw)),
            (tgx, np.stack(tga), np.stack(tgb), np.array(tgw)))
