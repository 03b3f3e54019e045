"""Seeded synthetic inputs for the LAPLEX workloads.

This module holds no arithmetic of the method itself: it only draws the
anchors, data vectors and upstream gradients that the tests, the benchmark and
the CPU oracle's callers feed to both sides, so that both see bit-identical
fp32 inputs.  It imports neither the HIP binding nor the oracle.

Generator: counter based.  Element ``i`` of stream ``seed`` is
``splitmix64_finalise(seed + (i + 1) * GOLDEN)``; the top 53 bits become a
uniform in [0, 1) in fp64.  Uniforms are scaled in fp64 and rounded to fp32
last, so "U(0, 2^24) in fp32" keeps its fractional part wherever fp32 has one.
Normals use Box-Muller in fp64 on counters ``2i`` and ``2i + 1``.

Workload shapes follow the paper's benchmarks: square n = k sweeps with small
batch (Sec. "Primitive GPU scaling", App. "Matvec benchmark"), one short axis
of 1024 against a long axis up to 2^20 (App. "Asymmetric shapes"), batch up to
256 (App. "Batch scaling"), the flattened 3x1024x1024 image dimension of the
density experiment, and the n ~ 2^29..2^30 end of the runtime curve (Fig. 1).
"""
from __future__ import annotations

import os

import numpy as np

_GOLDEN = np.uint64(0x9E3779B97F4A7C15)
_M1 = np.uint64(0xBF58476D1CE4E5B9)
_M2 = np.uint64(0x94D049BB133111EB)
_BASE_SEED = 260524584 * 16
_CHUNK = 1 << 20

STREAM_A, STREAM_B, STREAM_X, STREAM_G = 0, 1, 2, 3


def stream_seed(config: int, stream: int) -> int:
    """Seed of one input stream (0=a, 1=b, 2=x, 3=g) of workload ``config``."""
    return _BASE_SEED + 4 * int(config) + int(stream)


def _bits(seed: int, start: int, count: int) -> np.ndarray:
    with np.errstate(over="ignore"):
        idx = np.arange(start + 1, start + 1 + count, dtype=np.uint64)
        z = np.uint64(seed & 0xFFFFFFFFFFFFFFFF) + idx * _GOLDEN
        z = (z ^ (z >> np.uint64(30))) * _M1
        z = (z ^ (z >> np.uint64(27))) * _M2
        z = z ^ (z >> np.uint64(31))
    return z


def unit_uniform(seed: int, start: int, count: int) -> np.ndarray:
    """fp64 uniforms in [0, 1) for counters start .. start+count-1."""
    return (_bits(seed, start, count) >> np.uint64(11)).astype(np.float64) * (1.0 / (1 << 53))


def _chunks(count: int, fill) -> np.ndarray:
    """fill(start, c) -> fp32 chunk; chunks are independent (counter based), so
    large arrays are filled by a few threads (numpy releases the GIL)."""
    out = np.empty(count, dtype=np.float32)
    starts = range(0, count, _CHUNK)

    def one(s):
        c = min(_CHUNK, count - s)
        out[s:s + c] = fill(s, c)

    if count <= 4 * _CHUNK:
        for s in starts:
            one(s)
    else:
        from concurrent.futures import ThreadPoolExecutor
        with ThreadPoolExecutor(max_workers=min(16, os.cpu_count() or 1)) as pool:
            list(pool.map(one, starts))
    return out


def uniform(seed: int, count: int, lo: float, hi: float) -> np.ndarray:
    """fp32 array of ``count`` draws from U(lo, hi), scaled in fp64, rounded last."""
    return _chunks(count, lambda s, c: (lo + (hi - lo) * unit_uniform(seed, s, c)).astype(np.float32))


def normal(seed: int, count: int, sigma: float = 1.0) -> np.ndarray:
    """fp32 array of ``count`` draws from N(0, sigma^2) (Box-Muller in fp64)."""
    def fill(s, c):
        u = unit_uniform(seed, 2 * s, 2 * c)
        u1 = 1.0 - u[0::2]            # (0, 1]: log is finite
        u2 = u[1::2]
        return (sigma * (np.sqrt(-2.0 * np.log(u1)) * np.cos(2.0 * np.pi * u2))).astype(np.float32)
    return _chunks(count, fill)


def quarter_grid(v: np.ndarray) -> np.ndarray:
    """Round to the 1/4 grid (tie-heavy workload): many equal anchors result."""
    return (np.round(v.astype(np.float64) * 4.0) / 4.0).astype(np.float32)


# ---------------------------------------------------------------------------
# The five workloads.  ``scale`` shrinks n and k (never the anchor density:
# the anchor range shrinks with them) so that parity tests can run the same
# recipe at sizes the oracle finishes in seconds.
# ---------------------------------------------------------------------------

def _shrunk(v: int, scale: int) -> int:
    return max(1, v // scale)


def square_small(scale: int = 1):
    """n = k = 4096, batch 1, a, b ~ U(0, 64), x ~ N(0, 1): forward only."""
    n = k = _shrunk(4096, scale)
    hi = 64.0 / scale
    return dict(
        name="square_n4096", config=0, k=k, n=n, batch=1,
        a=uniform(stream_seed(0, STREAM_A), k, 0.0, hi),
        b=uniform(stream_seed(0, STREAM_B), n, 0.0, hi),
        x=normal(stream_seed(0, STREAM_X), n).reshape(n, 1),
    )


def projection_layer(scale: int = 1, batch: int = 256):
    """n = 2^20 inputs, k = 1024 outputs, batch 256, anchors U(0, 2^14);
    x and the upstream gradient g ~ N(0, 1), batch-minor."""
    n = _shrunk(1 << 20, scale)
    k = _shrunk(1024, scale)
    hi = float(1 << 14) / scale
    return dict(
        name="projection_n2^20_k1024_b256", config=1, k=k, n=n, batch=batch,
        a=uniform(stream_seed(1, STREAM_A), k, 0.0, hi),
        b=uniform(stream_seed(1, STREAM_B), n, 0.0, hi),
        x=normal(stream_seed(1, STREAM_X), n * batch).reshape(n, batch),
        g=normal(stream_seed(1, STREAM_G), k * batch).reshape(k, batch),
    )


def projection_layer_phased(scale: int = 1, batch: int = 256):
    """The projection layer with phases on both anchor sets, phi (outputs) and
    psi (inputs) ~ U(-pi, pi) (streams of their own, config slot 7)."""
    w = projection_layer(scale=scale, batch=batch)
    w["name"] = "projection_phased_n2^20_k1024_b256"
    w["phi"] = uniform(stream_seed(7, STREAM_A), w["k"], -np.pi, np.pi)
    w["psi"] = uniform(stream_seed(7, STREAM_B), w["n"], -np.pi, np.pi)
    return w


def weighted_gram(scale: int = 1, k: int = 1024):
    """Weighted Gram matrix with k = 1024 anchors (the result is k x k) and n = 2^20 middle
    anchors, the large end of the paper's sweep of the inner dimension (App. "Weighted Gram
    matrix": output dimension fixed at 1024, inner dimension 2^10 .. 2^20).  Anchors as in the
    projection layer, U(0, 2^14); weights d = 1/2 + |N(0, 1)|, positive like the variances of
    the density model (config slot 8)."""
    n = _shrunk(1 << 20, scale)
    k = _shrunk(k, scale)
    hi = float(1 << 14) / scale
    return dict(
        name="weighted_gram_k1024_n2^20", config=8, k=k, n=n, batch=1,
        a=uniform(stream_seed(8, STREAM_A), k, 0.0, hi),
        b=uniform(stream_seed(8, STREAM_B), n, 0.0, hi),
        d=(np.abs(normal(stream_seed(8, STREAM_X), n)) + np.float32(0.5)).astype(np.float32),
    )


def mix_head(scale: int = 1, r: int = 16, batch: int = 256):
    """LAPLEX^(r) classification head (Sec. 7): r = 16 operators of shape classes x features =
    1000 x 2048, batch 256; anchors U(0, 48) (about 64 anchors per unit, as in the other workloads),
    mixing weights, x and the upstream gradient ~ N(0, 1) (config slot 9)."""
    k = _shrunk(1000, scale); n = _shrunk(2048, scale)
    hi = 48.0 / scale
    return dict(
        name="mix_head_r16_k1000_n2048_b256", config=9, r=r, k=k, n=n, batch=batch,
        a=uniform(stream_seed(9, STREAM_A), r * k, 0.0, hi).reshape(r, k),
        b=uniform(stream_seed(9, STREAM_B), r * n, 0.0, hi).reshape(r, n),
        w=normal(stream_seed(9, STREAM_G) + 1, r),
        x=normal(stream_seed(9, STREAM_X), n * batch).reshape(n, batch),
        g=normal(stream_seed(9, STREAM_G), k * batch).reshape(k, batch),
    )


def paper_square(exp: int = 20, batch: int = 8):
    """The shape of the paper's runtime figure (App. "GPU runtime"): square apply n = k = 2^exp at
    batch 8; anchors ~ U(0, n / 32) (64 merged anchors per unit, as in the other workloads),
    x, g ~ N(0, 1) (config slot 10, one set of streams per size)."""
    n = k = 1 << exp
    return dict(
        name=f"paper_square_n2^{exp}_b{batch}", config=10, k=k, n=n, batch=batch,
        a=uniform(stream_seed(10, STREAM_A) + exp, k, 0.0, n / 32.0),
        b=uniform(stream_seed(10, STREAM_B) + exp, n, 0.0, n / 32.0),
        x=normal(stream_seed(10, STREAM_X) + exp, n * batch).reshape(n, batch),
        g=normal(stream_seed(10, STREAM_G) + exp, k * batch).reshape(k, batch),
    )


def tie_heavy(scale: int = 1):
    """n = k = 2^24, batch 1, anchors U(0, 2^18) rounded to a 1/4 grid."""
    n = k = _shrunk(1 << 24, scale)
    hi = float(1 << 18) / scale
    return dict(
        name="tie_heavy_n2^24", config=2, k=k, n=n, batch=1,
        a=quarter_grid(uniform(stream_seed(2, STREAM_A), k, 0.0, hi)),
        b=quarter_grid(uniform(stream_seed(2, STREAM_B), n, 0.0, hi)),
        x=normal(stream_seed(2, STREAM_X), n).reshape(n, 1),
        g=normal(stream_seed(2, STREAM_G), k).reshape(k, 1),
    )


def gram_images(scale: int = 1, batch: int = 64):
    """Gram form on n = 3 * 2^20 anchors a ~ N(0, (2^16)^2), batch 64."""
    n = _shrunk(3 << 20, scale)
    sigma = float(1 << 16) / scale
    return dict(
        name="gram_n3x2^20_b64", config=3, n=n, batch=batch,
        a=normal(stream_seed(3, STREAM_A), n, sigma),
        x=normal(stream_seed(3, STREAM_X), n * batch).reshape(n, batch),
        g=normal(stream_seed(3, STREAM_G), n * batch).reshape(n, batch),
    )


def billion_square(scale: int = 1):
    """n = k = 2^30, batch 1, a, b ~ U(0, 2^24)."""
    n = k = _shrunk(1 << 30, scale)
    hi = float(1 << 24) / scale
    return dict(
        name="billion_n2^30", config=4, k=k, n=n, batch=1,
        a=uniform(stream_seed(4, STREAM_A), k, 0.0, hi),
        b=uniform(stream_seed(4, STREAM_B), n, 0.0, hi),
        x=normal(stream_seed(4, STREAM_X), n).reshape(n, 1),
        g=normal(stream_seed(4, STREAM_G), k).reshape(k, 1),
    )


def clustered_anchors(k: int, n: int, batch: int, seed: int = 77):
    """Irregular anchors a, b ~ N(0, 1) (the paper's irregular-anchor benchmark
    recipe): every anchor lies within a few units, so no decay ever reaches
    zero and every carry travels the whole sequence."""
    return dict(
        name="clustered", k=k, n=n, batch=batch,
        a=normal(seed * 8 + 0, k), b=normal(seed * 8 + 1, n),
        x=normal(seed * 8 + 2, n * batch).reshape(n, batch),
        g=normal(seed * 8 + 3, k * batch).reshape(k, batch),
    )
