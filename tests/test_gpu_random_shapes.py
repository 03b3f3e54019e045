"""Seeded random shapes through every entry point: the bodies of the parity tests (same oracle, same bars),
called on shapes, batches and anchor kinds drawn from a fixed seed instead of the hand-picked lists, so that
tile, lane and workgroup boundaries fall in places nobody chose.  (One such draw -- 1072 Gram anchors on nine
values with three middle anchors -- found a rounding flaw in the weighted Gram matrix that the lists had missed.)
"""
import numpy as np
import pytest

import test_gpu_parity as T

pytestmark = pytest.mark.gpu


def body(f):
    while hasattr(f, "__wrapped__"):
        f = f.__wrapped__
    return f


def draw_shape(r, lo, hi, max_work):
    """(k, n, batch) with k + n ~ 2^U(lo, hi); one draw in three has few outputs; batch shrinks to bound the oracle's work."""
    total = int(2 ** r.uniform(lo, hi))
    k = int(r.integers(1, max(2, total)))
    if r.integers(3) == 0:
        k = int(r.integers(1, 2000))
    n = max(1, total - k)
    batch = int(r.choice([1, 2, 3, 4, 8, 17, 64, 100, 128, 256]))
    while k * n * batch > max_work and batch > 1:
        batch = max(1, batch // 2)
    return k, n, batch


@pytest.mark.parametrize("seed", range(40))
def test_apply_and_gram_random_shapes(oracle, seed):
    r = np.random.default_rng(9100 + seed)
    for lo, hi in ((1, 13.3), (13.0, 16.0)):          # the two-launch path for small problems; the large path
        k, n, batch = draw_shape(r, lo, hi, 3e8)
        kind = (T.KINDS + ["extreme"])[r.integers(len(T.KINDS) + 1)]
        body(T.test_apply_forward_backward)(oracle, kind, k, n, batch)
        body(T.test_gram_forward_backward)(oracle, kind, min(k, 9000), batch)


@pytest.mark.parametrize("seed", range(40))
def test_widened_entry_points_random_shapes(oracle, seed):
    r = np.random.default_rng(9200 + seed)
    kinds = T.KINDS
    k, n, batch = draw_shape(r, 6, 15.5, 2e8)
    body(T.test_phased_forward_backward)(oracle, kinds[r.integers(len(kinds))], k, n, batch)
    k, n, batch = draw_shape(r, 6, 15.5, 2e8)
    body(T.test_temperature_forward_backward)(oracle, float(r.choice([0.37, 1.0, 2.5, 5.0])), kinds[r.integers(len(kinds))], k, n, batch)
    k, n, batch = draw_shape(r, 6, 14.2, 5e7)
    body(T.test_mix_forward_backward)(oracle, kinds[r.integers(len(kinds))], int(r.integers(1, 6)), k, n, batch)
    k, n = int(r.integers(1, 1500)), int(2 ** r.uniform(0, 17.5))
    kind, weights = kinds[r.integers(len(kinds))], str(r.choice(["signed", "positive"]))
    body(T.test_weighted_gram_matrix)(oracle, weights, kind, k, n)
    body(T.test_weighted_gram_matrix_fp64)(oracle, weights, kind, k, n)
