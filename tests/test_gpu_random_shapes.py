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


def padded(v, ld):
    """(rows, cols) values in a buffer with leading dimension ld, NaN in the padding."""
    buf = T.torch.full((v.shape[0], ld), float("nan"), device="cuda")
    view = buf[:, : v.shape[1]]
    view.copy_(T.dev(v))
    return buf, view


@pytest.mark.parametrize("seed", range(60))
def test_flags_strides_and_subsets_random(oracle, seed):
    """Sorted-anchor flags (merge path / one flag alone), leading dimensions, gradient subsets, saved scans, a fresh or a
    reused plan in the backward, and the plan reused for another batch size."""
    B, torch = T.B, T.torch
    r = np.random.default_rng(9300 + seed)
    kind = T.KINDS[r.integers(len(T.KINDS))]
    total = int(2 ** r.uniform(2, 16.2))
    k = int(r.integers(1, max(2, total))); n = max(1, total - k)
    if r.integers(4) == 0:
        k = int(r.integers(1, 50)); n = max(1, total - k)
    batch = int(r.choice([1, 2, 3, 4, 5, 8, 12, 16, 33, 64, 128, 256, 260]))
    while k * n * batch > 2e8 and batch > 1:
        batch = max(1, batch // 2)
    a, b = T.anchors(kind, r, k, n)
    flags = 0
    if r.integers(3) == 0:
        a.sort(); b.sort(); flags |= B.LAPLEX_A_SORTED | B.LAPLEX_B_SORTED
    elif r.integers(3) == 0:
        a.sort(); flags |= B.LAPLEX_A_SORTED
    if r.integers(2):
        flags |= B.LAPLEX_SAVE_SCANS
    ldx, ldy = batch + int(r.choice([0, 0, 1, 3, 4, 8])), batch + int(r.choice([0, 0, 1, 4]))
    ldg, ldgx = batch + int(r.choice([0, 0, 2, 4])), batch + int(r.choice([0, 0, 4, 5]))
    x = r.normal(size=(n, batch)).astype(np.float32); g = r.normal(size=(k, batch)).astype(np.float32)
    small = k * n * batch <= 4e7
    ws = T.workspace(k, n, batch)
    da, db = T.dev(a), T.dev(b)
    _, dx = padded(x, ldx); _, dg = padded(g, ldg)
    ybuf = torch.full((k, ldy), float("nan"), device="cuda"); y = ybuf[:, :batch]
    B.laplex_apply(da, db, dx, y, ws, flags)
    torch.cuda.synchronize()
    ref, tol = (oracle.apply_brute if small else oracle.apply_scan)(a, b, x)
    T.assert_close("y", y.cpu().numpy(), ref, tol)
    assert ldy == batch or bool(torch.isnan(ybuf[:, batch:]).all())
    assert np.array_equal(T.gpu_perm(ws, k + n), oracle.merged_permutation(a, b))
    want = [bool(r.integers(4)) for _ in range(3)]
    if not any(want):
        want[0] = True
    gxbuf = torch.full((n, ldgx), float("nan"), device="cuda") if want[0] else None
    gx = gxbuf[:, :batch] if want[0] else None
    ga = torch.full((k,), float("nan"), device="cuda") if want[1] else None
    gb = torch.full((n,), float("nan"), device="cuda") if want[2] else None
    bflags = flags | (B.LAPLEX_REUSE_PLAN if r.integers(2) else 0)
    if not bflags & B.LAPLEX_REUSE_PLAN:
        bflags &= ~B.LAPLEX_SAVE_SCANS          # a fresh plan has no saved scans
    B.laplex_apply_backward(da, db, dx, dg, gx, ga, gb, ws, bflags)
    torch.cuda.synchronize()
    (rgx, rga, rgb), (tgx, tga, tgb) = (oracle.apply_backward_brute if small else oracle.apply_backward_scan)(a, b, x, g)
    if want[0]:
        T.assert_close("gx", gx.cpu().numpy(), rgx, tgx)
        assert ldgx == batch or bool(torch.isnan(gxbuf[:, batch:]).all())
    if want[1]:
        T.assert_close("ga", ga.cpu().numpy(), rga, tga)
    if want[2]:
        T.assert_close("gb", gb.cpu().numpy(), rgb, tgb)
    b2 = int(r.choice([1, 4, 7, 64]))
    while k * n * b2 > 1e8 and b2 > 1:
        b2 = max(1, b2 // 2)
    if B.laplex_workspace_bytes(k, n, b2) <= ws.numel():      # the same plan, another batch size
        x2 = r.normal(size=(n, b2)).astype(np.float32)
        y2 = torch.full((k, b2), float("nan"), device="cuda")
        B.laplex_apply(da, db, T.dev(x2), y2, ws, (flags & ~B.LAPLEX_SAVE_SCANS) | B.LAPLEX_REUSE_PLAN)
        torch.cuda.synchronize()
        ref2, tol2 = (oracle.apply_brute if k * n * b2 <= 4e7 else oracle.apply_scan)(a, b, x2)
        T.assert_close("y, plan reused at another batch size", y2.cpu().numpy(), ref2, tol2)


@pytest.mark.parametrize("seed", range(30))
def test_batch_one_routes_random(oracle, seed):
    """Batch 1 on the routes through partition passes (switched on for every size beyond the small path while the test
    runs): random shapes from 2^13 to 2^18.5 merged positions, sorted-anchor flags, leading dimensions, gradient subsets,
    saved scans or a re-scan, a fresh or a reused plan; the square form on the same routes."""
    B, torch = T.B, T.torch
    r = np.random.default_rng(9400 + seed)
    kind = T.KINDS[r.integers(len(T.KINDS))]
    total = int(2 ** r.uniform(13.05, 18.5))
    k = int(r.integers(1, total)); n = max(1, total - k)
    if r.integers(4) == 0:
        k = int(r.integers(1, 50)); n = total - k
    a, b = T.anchors(kind, r, k, n)
    flags = 0
    if r.integers(3) == 0:
        a.sort(); b.sort(); flags |= B.LAPLEX_A_SORTED | B.LAPLEX_B_SORTED
    if r.integers(2):
        flags |= B.LAPLEX_SAVE_SCANS
    ldx, ldy, ldg, ldgx = (1 + int(r.choice([0, 0, 1, 3])) for _ in range(4))
    x = r.normal(size=(n, 1)).astype(np.float32); g = r.normal(size=(k, 1)).astype(np.float32)
    small = k * n <= 4e7
    B.laplex_diag_set_route_min(0)
    try:
        ws = T.workspace(k, n, 1)
        da, db = T.dev(a), T.dev(b)
        _, dx = padded(x, ldx); _, dg = padded(g, ldg)
        ybuf = torch.full((k, ldy), float("nan"), device="cuda"); y = ybuf[:, :1]
        B.laplex_apply(da, db, dx, y, ws, flags)
        torch.cuda.synchronize()
        ref, tol = (oracle.apply_brute if small else oracle.apply_scan)(a, b, x)
        T.assert_close("y", y.cpu().numpy(), ref, tol)
        assert ldy == 1 or bool(torch.isnan(ybuf[:, 1:]).all())
        assert np.array_equal(T.gpu_perm(ws, k + n), oracle.merged_permutation(a, b))
        want = [bool(r.integers(4)) for _ in range(3)]
        if not any(want):
            want[0] = True
        gxbuf = torch.full((n, ldgx), float("nan"), device="cuda") if want[0] else None
        gx = gxbuf[:, :1] if want[0] else None
        ga = torch.full((k,), float("nan"), device="cuda") if want[1] else None
        gb = torch.full((n,), float("nan"), device="cuda") if want[2] else None
        bflags = flags | (B.LAPLEX_REUSE_PLAN if r.integers(2) else 0)
        if not bflags & B.LAPLEX_REUSE_PLAN:
            bflags &= ~B.LAPLEX_SAVE_SCANS          # a fresh plan has no saved scans
        B.laplex_apply_backward(da, db, dx, dg, gx, ga, gb, ws, bflags)
        torch.cuda.synchronize()
        (rgx, rga, rgb), (tgx, tga, tgb) = (oracle.apply_backward_brute if small else oracle.apply_backward_scan)(a, b, x, g)
        if want[0]:
            T.assert_close("gx", gx.cpu().numpy(), rgx, tgx)
            assert ldgx == 1 or bool(torch.isnan(gxbuf[:, 1:]).all())
        if want[1]:
            T.assert_close("ga", ga.cpu().numpy(), rga, tga)
        if want[2]:
            T.assert_close("gb", gb.cpu().numpy(), rgb, tgb)
        # the square form on the anchors of the larger side
        m = min(max(k, n), 120000)
        if m > 8192:
            body(T.test_routes_gram_form)(oracle, None, kind, m)
    finally:
        B.laplex_diag_set_route_min(1 << 22)


@pytest.mark.parametrize("seed", range(24))
def test_phased_wide_batches_random(oracle, seed):
    """The phased kernel with the modulation inside the wide kernels: batches of 68 to 256 columns, shapes from 2^13.1 to
    2^15.3 merged positions, outputs spread out or bunched (blocks with many outputs take the other downsweeps and the
    block-wise split and merge), gradient subsets, and leading dimensions that do or do not allow 16-byte rows."""
    B, torch = T.B, T.torch
    r = np.random.default_rng(9500 + seed)
    batch = 4 * int(r.integers(17, 65))
    total = int(2 ** r.uniform(13.1, 15.3))
    k = int(r.integers(1, total // 2)); n = total - k
    if r.integers(3) == 0:
        k = int(r.integers(1, 40)); n = total - k
    kind = str(r.choice(["uniform", "ties", "clustered_outputs", "clustered"]))
    a, b = T.clustered_outputs(r, k, n) if kind == "clustered_outputs" else T.anchors(kind, r, k, n)
    sorted_flags = 0
    if r.integers(3) == 0:          # both anchor sets ascending: the merge path
        a = np.sort(a); b = np.sort(b); sorted_flags = B.LAPLEX_A_SORTED | B.LAPLEX_B_SORTED
    phi = r.uniform(-7, 7, k).astype(np.float32); psi = r.uniform(-7, 7, n).astype(np.float32)
    x = r.normal(size=(n, batch)).astype(np.float32); g = r.normal(size=(k, batch)).astype(np.float32)
    ref, tol = oracle.phased_apply_scan(a, phi, b, psi, x)
    refs, tols = oracle.phased_backward_scan(a, phi, b, psi, x, g)
    ldx = batch + int(r.choice([0, 0, 4, 8, 1])); ldgx = batch + int(r.choice([0, 0, 4, 3]))
    ws = T.phased_workspace(k, n, batch)
    da, dphi, db, dpsi = T.dev(a), T.dev(phi), T.dev(b), T.dev(psi)
    _, dx = padded(x, ldx); dg = T.dev(g)
    y = torch.full((k, batch), float("nan"), device="cuda")
    save = bool(r.integers(2))
    B.laplex_phased_apply(da, dphi, db, dpsi, dx, y, ws, sorted_flags | (B.LAPLEX_SAVE_SCANS if save else 0))
    torch.cuda.synchronize()
    T.assert_close("y", y.cpu().numpy(), ref, tol)
    want = [bool(r.integers(3)) for _ in range(5)]
    if not any(want):
        want[0] = True
    gxbuf = torch.full((n, ldgx), float("nan"), device="cuda") if want[0] else None
    outs = [gxbuf[:, :batch] if want[0] else None] + [torch.full((m,), float("nan"), device="cuda") if w else None
                                                      for m, w in zip((k, n, k, n), want[1:])]
    bflags = sorted_flags | ((B.LAPLEX_SAVE_SCANS | B.LAPLEX_REUSE_PLAN) if save and r.integers(2) else 0)
    B.laplex_phased_apply_backward(da, dphi, db, dpsi, dx, dg, *outs, ws, bflags)
    torch.cuda.synchronize()
    for name, got, rv, tv, w in zip(("gx", "ga", "gb", "gphi", "gpsi"), outs, refs, tols, want):
        if w:
            T.assert_close(name, got.cpu().numpy(), rv, tv)
    assert not want[0] or ldgx == batch or bool(torch.isnan(gxbuf[:, batch:]).all())
