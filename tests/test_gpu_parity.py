"""Parity of the HIP path (through the C-ABI library) with the CPU oracle, on the
same seeded fp32 inputs.

Bars: permutation ids bit-exact; floating point
    |gpu - ref| <= 1e-5 * T + 1e-7,
T the same sum over absolute values of the summands (per output), the bound the
task states for y and, in the same form, for every gradient.
"""
import numpy as np
import pytest

from paper_2605_24584_amd import binding as B
from paper_2605_24584_amd import synth

torch = pytest.importorskip("torch")
pytestmark = pytest.mark.gpu

RTOL, ATOL = 1e-5, 1e-7


def dev(v):
    return torch.from_numpy(np.ascontiguousarray(v)).cuda()


def workspace(k, n, batch):
    return torch.empty(B.laplex_workspace_bytes(k, n, batch), dtype=torch.uint8, device="cuda")


def assert_close(name, got, ref, tol):
    got = np.asarray(got, dtype=np.float64).reshape(ref.shape)
    assert np.all(np.isfinite(got)), f"{name}: non-finite values"
    ratio = np.abs(got - ref) / (RTOL * tol + ATOL)
    worst = float(ratio.max()) if ratio.size else 0.0
    assert worst <= 1.0, f"{name}: worst |err|/(1e-5 T + 1e-7) = {worst:.3g} at {np.unravel_index(ratio.argmax(), ratio.shape)}"
    return worst


def gpu_apply(a, b, x, flags=0, ws=None, ldx=None, ldy=None):
    k, n, batch = a.size, b.size, x.shape[1]
    ws = workspace(k, n, batch) if ws is None else ws
    da, db = dev(a), dev(b)
    if ldx is None:
        dx = dev(x)
    else:
        dx = torch.zeros(n, ldx, device="cuda")[:, :batch]
        dx.copy_(dev(x))
    ybuf = torch.full((k, batch if ldy is None else ldy), float("nan"), device="cuda")
    y = ybuf[:, :batch]
    B.laplex_apply(da, db, dx, y, ws, flags)
    torch.cuda.synchronize()
    return y.cpu().numpy(), ws


def gpu_backward(a, b, x, g, flags=0, ws=None, want=(True, True, True)):
    k, n, batch = a.size, b.size, x.shape[1]
    ws = workspace(k, n, batch) if ws is None else ws
    gx = torch.full((n, batch), float("nan"), device="cuda") if want[0] else None
    ga = torch.full((k,), float("nan"), device="cuda") if want[1] else None
    gb = torch.full((n,), float("nan"), device="cuda") if want[2] else None
    B.laplex_apply_backward(dev(a), dev(b), dev(x), dev(g), gx, ga, gb, ws, flags)
    torch.cuda.synchronize()
    return tuple(None if t is None else t.cpu().numpy() for t in (gx, ga, gb))


def gpu_plan_status(ws, count):
    out = torch.full((1,), -1, dtype=torch.int32, device="cuda")
    B.laplex_get_plan_status(ws, count, out)
    torch.cuda.synchronize()
    return int(out.item())


def gpu_perm(ws, count):
    out = torch.empty(count, dtype=torch.int32, device="cuda")
    B.laplex_get_perm(ws, count, out)
    torch.cuda.synchronize()
    return out.cpu().numpy().view(np.uint32)


def anchors(kind, r, k, n):
    if kind == "uniform":
        span = max(1.0, (k + n) / 128.0)
        a, b = r.uniform(0, span, k), r.uniform(0, span, n)
    elif kind == "ties":
        span = max(1.0, (k + n) / 64.0)
        a, b = np.round(r.uniform(0, span, k) * 4) / 4, np.round(r.uniform(0, span, n) * 4) / 4
    elif kind == "all_equal":
        a, b = np.full(k, -2.5), np.full(n, -2.5)
    elif kind == "huge_gaps":
        a, b = r.integers(0, 9, k) * 300.0, r.integers(0, 9, n) * 300.0 + r.integers(0, 2, n) * 0.5
    elif kind == "clustered":
        a, b = r.normal(size=k), r.normal(size=n)
    elif kind == "signed":
        a, b = r.normal(size=k) * 40, -r.uniform(0, 30, n)
        a[: k // 7] = 0.0; b[: n // 5] = -0.0
    elif kind == "narrow":          # all in [1, 2): the top key byte is the same for every anchor
        a, b = 1.0 + r.uniform(0, 1, k), 1.0 + r.uniform(0, 1, n)
    elif kind == "small_ints":      # few mantissa bits: the two low key bytes are zero for every anchor
        a, b = r.integers(0, 8, k).astype(np.float64), r.integers(0, 8, n).astype(np.float64)
    elif kind == "extreme":         # denormals to 3e38, both signs, exact zeros of both signs (the random-shape tests use it)
        def draw(m):
            lo, hi = [(-45, -30), (-45, 38), (30, 38.5), (-3, 3), (-45, 2)][r.integers(5)]
            with np.errstate(over="ignore", under="ignore"):
                v = (10.0 ** r.uniform(lo, hi, m)) * r.choice([-1.0, 1.0], m)
                v[r.integers(0, m, max(1, m // 10))] = 0.0
                v[r.integers(0, m, max(1, m // 10))] = -0.0
                v = v.astype(np.float32)
            v[~np.isfinite(v)] = np.float32(3.0e38)
            return v
        a, b = draw(k), draw(n)
    else:
        raise KeyError(kind)
    return a.astype(np.float32), b.astype(np.float32)


# "all_equal", "narrow" and "small_ints" have key bytes that are constant over all anchors: sort passes are skipped
KINDS = ["uniform", "ties", "all_equal", "huge_gaps", "clustered", "signed", "narrow", "small_ints"]
# (k, n, batch): single elements, ragged tails, several tiles of both lane geometries, two slabs
SHAPES = [(1, 1, 1), (5, 1, 2), (1, 6, 1), (37, 53, 3), (100, 9000, 1), (9000, 100, 5),
          (3000, 21000, 1), (2500, 4000, 8), (513, 9000, 64), (300, 2100, 256), (70, 1500, 260),
          (50, 1700, 67),
          # very few outputs / very few inputs: tile lists drive the heavy kernels
          (3, 70000, 1), (70000, 3, 1), (2, 40000, 8), (5, 30000, 64),
          # wide batches with few outputs / few inputs: blocks with a handful of result (injected) rows
          (20, 6000, 256), (6000, 20, 256), (3, 2000, 512)]


# ------------------------------------------------------------------ the sort

@pytest.mark.parametrize("kind", KINDS)
# the last four: one size for each tile size of the sort passes (2048, 4096 and 8192 pairs), with ragged last tiles, and one
# beyond 2^22 merged positions, where the histogram keeps its counters once per LDS bank
@pytest.mark.parametrize("k,n", [(1, 1), (3, 0), (0, 5), (100, 157), (9000, 8000), (20000, 70001),
                                 (130000, 132001), (300001, 400122), (1500000, 1000003), (2300001, 2100003)])
def test_permutation_bit_exact(oracle, kind, k, n):
    if k == 0 or n == 0:
        pytest.skip("apply with an empty side builds no plan")
    r = np.random.default_rng(k * 7 + n)
    a, b = anchors(kind, r, k, n)
    x = r.normal(size=(n, 1)).astype(np.float32)
    _, ws = gpu_apply(a, b, x)
    assert np.array_equal(gpu_perm(ws, k + n), oracle.merged_permutation(a, b))
    assert gpu_plan_status(ws, k + n) == 0       # no tile of the sort gave up waiting for its predecessors


@pytest.mark.parametrize("off_a,off_b", [(1, 0), (2, 3), (3, 1), (0, 2)])
@pytest.mark.parametrize("k,n", [(1, 2), (2, 1), (3, 7), (4100, 4100), (9001, 20003), (2100001, 2100002)])
def test_anchor_arrays_off_a_16_byte_boundary(oracle, off_a, off_b, k, n):
    """The histogram reads the anchors 16 bytes at a time between a scalar head and a scalar tail."""
    r = np.random.default_rng(k * 5 + n + off_a * 16 + off_b)
    a, b = anchors("ties", r, k, n)
    x = r.normal(size=(n, 1)).astype(np.float32)
    da = torch.zeros(k + 8, device="cuda")[off_a:off_a + k]; da.copy_(dev(a))
    db = torch.zeros(n + 8, device="cuda")[off_b:off_b + n]; db.copy_(dev(b))
    assert da.data_ptr() % 16 == 4 * off_a and db.data_ptr() % 16 == 4 * off_b
    ws = workspace(k, n, 1)
    y = torch.full((k, 1), float("nan"), device="cuda")
    B.laplex_apply(da, db, dev(x), y, ws, 0)
    torch.cuda.synchronize()
    assert np.array_equal(gpu_perm(ws, k + n), oracle.merged_permutation(a, b))
    ref, tol = oracle.apply_scan(a, b, x)
    assert_close("y", y.cpu().numpy(), ref, tol)


@pytest.mark.parametrize("kind", ["uniform", "ties", "all_equal", "signed"])
@pytest.mark.parametrize("k,n", [(1, 1), (100, 157), (5000, 3), (3, 5000), (20000, 70001)])
def test_merge_path_when_both_sorted(oracle, kind, k, n):
    r = np.random.default_rng(k + 3 * n)
    a, b = anchors(kind, r, k, n)
    a.sort(); b.sort()
    x = r.normal(size=(n, 2)).astype(np.float32)
    y, ws = gpu_apply(a, b, x, flags=B.LAPLEX_A_SORTED | B.LAPLEX_B_SORTED)
    assert np.array_equal(gpu_perm(ws, k + n), oracle.merged_permutation(a, b))
    ref, tol = oracle.apply_scan(a, b, x)
    assert_close("y", y, ref, tol)


# ------------------------------------------------------------------ forward and backward

@pytest.mark.parametrize("kind", KINDS)
@pytest.mark.parametrize("k,n,batch", SHAPES)
def test_apply_forward_backward(oracle, kind, k, n, batch):
    r = np.random.default_rng(1000 + k + n + batch)
    a, b = anchors(kind, r, k, n)
    x = r.normal(size=(n, batch)).astype(np.float32)
    g = r.normal(size=(k, batch)).astype(np.float32)
    small = k * n * batch <= 4e7
    ref, tol = (oracle.apply_brute if small else oracle.apply_scan)(a, b, x)
    y, ws = gpu_apply(a, b, x, flags=B.LAPLEX_SAVE_SCANS)
    assert_close("y", y, ref, tol)
    (rgx, rga, rgb), (tgx, tga, tgb) = (oracle.apply_backward_brute if small else oracle.apply_backward_scan)(a, b, x, g)
    # with the forward's saved scans and the plan kept ...
    gx, ga, gb = gpu_backward(a, b, x, g, flags=B.LAPLEX_SAVE_SCANS | B.LAPLEX_REUSE_PLAN, ws=ws)
    assert_close("gx", gx, rgx, tgx); assert_close("ga", ga, rga, tga); assert_close("gb", gb, rgb, tgb)
    # ... and standing alone (sorts and re-scans x itself): the same bits
    gx2, ga2, gb2 = gpu_backward(a, b, x, g)
    assert np.array_equal(gx, gx2) and np.array_equal(ga, ga2) and np.array_equal(gb, gb2)


def test_backward_subsets_and_plain_path(oracle):
    r = np.random.default_rng(5)
    a, b = anchors("ties", r, 700, 3000)
    x = r.normal(size=(3000, 4)).astype(np.float32); g = r.normal(size=(700, 4)).astype(np.float32)
    (rgx, rga, rgb), (tgx, tga, tgb) = oracle.apply_backward_scan(a, b, x, g)
    gx, _, _ = gpu_backward(a, b, x, g, want=(True, False, False))
    assert_close("gx", gx, rgx, tgx)
    _, ga, _ = gpu_backward(a, b, x, g, want=(False, True, False))
    assert_close("ga", ga, rga, tga)
    _, _, gb = gpu_backward(a, b, x, g, want=(False, False, True))
    assert_close("gb", gb, rgb, tgb)


def test_plan_reuse_across_batches(oracle):
    r = np.random.default_rng(6)
    a, b = anchors("uniform", r, 800, 5000)
    x1 = r.normal(size=(5000, 8)).astype(np.float32); x2 = r.normal(size=(5000, 8)).astype(np.float32)
    y1, ws = gpu_apply(a, b, x1)
    y2, _ = gpu_apply(a, b, x2, flags=B.LAPLEX_REUSE_PLAN, ws=ws)
    y2_fresh, _ = gpu_apply(a, b, x2)
    assert np.array_equal(y2, y2_fresh)
    ref, tol = oracle.apply_scan(a, b, x2)
    assert_close("y", y2, ref, tol)


@pytest.mark.parametrize("batch,ldx,ldy", [(4, 5, 7), (8, 12, 8), (1, 3, 2), (64, 65, 64),
                                           # wide batches: padded rows with 4-column lanes, and with 1-column lanes
                                           (256, 260, 264), (256, 257, 256), (300, 304, 300)])
def test_leading_dimensions_and_scalar_lanes(oracle, batch, ldx, ldy):
    r = np.random.default_rng(7)
    a, b = anchors("uniform", r, 300, 2500)
    x = r.normal(size=(2500, batch)).astype(np.float32)
    y, _ = gpu_apply(a, b, x, ldx=ldx, ldy=ldy)
    ref, tol = oracle.apply_scan(a, b, x)
    assert_close("y", y, ref, tol)


def test_wide_batch_padded_rows_backward(oracle):
    """Backward with padded rows of x, gy and gx in the wide geometry (few outputs: the few-row kernels)."""
    r = np.random.default_rng(17)
    k, n, batch = 24, 7000, 256
    a, b = anchors("ties", r, k, n)
    x = r.normal(size=(n, batch)).astype(np.float32); g = r.normal(size=(k, batch)).astype(np.float32)
    ws = workspace(k, n, batch)
    dx = torch.zeros(n, batch + 8, device="cuda")[:, :batch]; dx.copy_(dev(x))
    dg = torch.zeros(k, batch + 4, device="cuda")[:, :batch]; dg.copy_(dev(g))
    gxbuf = torch.full((n, batch + 12), float("nan"), device="cuda"); gx = gxbuf[:, :batch]
    ga = torch.full((k,), float("nan"), device="cuda"); gb = torch.full((n,), float("nan"), device="cuda")
    B.laplex_apply_backward(dev(a), dev(b), dx, dg, gx, ga, gb, ws, 0)
    torch.cuda.synchronize()
    assert bool(torch.isnan(gxbuf[:, batch:]).all()), "the padding of gx was written"
    (rgx, rga, rgb), (tgx, tga, tgb) = oracle.apply_backward_scan(a, b, x, g)
    assert_close("gx", gx.cpu().numpy(), rgx, tgx)
    assert_close("ga", ga.cpu().numpy(), rga, tga)
    assert_close("gb", gb.cpu().numpy(), rgb, tgb)


def test_results_are_deterministic():
    r = np.random.default_rng(8)
    a, b = anchors("clustered", r, 5000, 40000)
    x = r.normal(size=(40000, 4)).astype(np.float32); g = r.normal(size=(5000, 4)).astype(np.float32)
    y1, _ = gpu_apply(a, b, x); y2, _ = gpu_apply(a, b, x)
    assert np.array_equal(y1, y2)
    o1 = gpu_backward(a, b, x, g); o2 = gpu_backward(a, b, x, g)
    assert all(np.array_equal(u, v) for u, v in zip(o1, o2))


def test_countsketch_limit_exact_in_fp32():
    """Anchors on well separated labels: decays are exactly 1 inside a label and
    exactly 0 across labels, so the apply is an exact bucket sum."""
    r = np.random.default_rng(9)
    k, n = 50, 4000
    labels = (300.0 * np.arange(k)).astype(np.float32)
    h = r.integers(0, k, n)
    x = r.integers(-8, 9, size=(n, 2)).astype(np.float32)      # sums exact in fp32
    y, _ = gpu_apply(labels, labels[h], x)
    want = np.zeros((k, 2)); np.add.at(want, h, x.astype(np.float64))
    assert np.array_equal(y.astype(np.float64), want)


# ------------------------------------------------------------------ empty sides

def test_empty_sides():
    a = np.array([1.0, 2.0, 3.0], dtype=np.float32)
    e = np.zeros(0, dtype=np.float32)
    y, _ = gpu_apply(a, e, np.zeros((0, 2), dtype=np.float32))
    assert y.shape == (3, 2) and not y.any()
    g = np.ones((3, 2), dtype=np.float32)
    gx, ga, gb = gpu_backward(a, e, np.zeros((0, 2), dtype=np.float32), g)
    assert ga.shape == (3,) and not ga.any() and gx.size == 0 and gb.size == 0
    gx, ga, gb = gpu_backward(e, a, np.ones((3, 2), dtype=np.float32), np.zeros((0, 2), dtype=np.float32))
    assert not gx.any() and not gb.any() and ga.size == 0


# ------------------------------------------------------------------ Gram form

def gpu_gram(a, x, flags=0, ws=None):
    n, batch = a.size, x.shape[1]
    ws = workspace(0, n, batch) if ws is None else ws
    y = torch.full((n, batch), float("nan"), device="cuda")
    B.laplex_gram(dev(a), dev(x), y, ws, flags)
    torch.cuda.synchronize()
    return y.cpu().numpy(), ws


def gpu_gram_backward(a, x, g, flags=0, ws=None, want=(True, True)):
    n, batch = a.size, x.shape[1]
    ws = workspace(0, n, batch) if ws is None else ws
    gx = torch.full((n, batch), float("nan"), device="cuda") if want[0] else None
    ga = torch.full((n,), float("nan"), device="cuda") if want[1] else None
    B.laplex_gram_backward(dev(a), dev(x), dev(g), gx, ga, ws, flags)
    torch.cuda.synchronize()
    return tuple(None if t is None else t.cpu().numpy() for t in (gx, ga))


@pytest.mark.parametrize("kind", KINDS)
@pytest.mark.parametrize("n,batch", [(1, 1), (2, 3), (777, 1), (6000, 4), (20000, 64), (3000, 67)])
def test_gram_forward_backward(oracle, kind, n, batch):
    r = np.random.default_rng(2000 + n + batch)
    a, _ = anchors(kind, r, n, 1)
    x = r.normal(size=(n, batch)).astype(np.float32); g = r.normal(size=(n, batch)).astype(np.float32)
    small = n * n * batch <= 4e7
    ref, tol = (oracle.gram_brute if small else oracle.gram_scan)(a, x)
    y, ws = gpu_gram(a, x, flags=B.LAPLEX_SAVE_SCANS)
    assert_close("y", y, ref, tol)
    assert np.array_equal(gpu_perm(ws, n), oracle.merged_permutation(a))
    (rgx, rga), (tgx, tga) = (oracle.gram_backward_brute if small else oracle.gram_backward_scan)(a, x, g)
    gx, ga = gpu_gram_backward(a, x, g, flags=B.LAPLEX_SAVE_SCANS | B.LAPLEX_REUSE_PLAN, ws=ws)
    assert_close("gx", gx, rgx, tgx); assert_close("ga", ga, rga, tga)
    gx2, ga2 = gpu_gram_backward(a, x, g)
    assert np.array_equal(gx, gx2) and np.array_equal(ga, ga2)
    _, ga3 = gpu_gram_backward(a, x, g, want=(False, True))
    assert np.array_equal(ga, ga3)


def test_gram_sorted_anchor_flag(oracle):
    r = np.random.default_rng(11)
    a = np.sort(r.uniform(0, 50, 5000)).astype(np.float32)
    x = r.normal(size=(5000, 4)).astype(np.float32)
    y, ws = gpu_gram(a, x, flags=B.LAPLEX_A_SORTED)
    assert np.array_equal(gpu_perm(ws, 5000), np.arange(5000, dtype=np.uint32))
    ref, tol = oracle.gram_scan(a, x)
    assert_close("y", y, ref, tol)


def test_gram_tridiagonal_inverse_recovers_x():
    """Property that holds at any size: for distinct anchors K^-1 is tridiagonal
    (Ornstein-Uhlenbeck precision), so applying it in fp64 to the GPU's y gives x back."""
    r = np.random.default_rng(12)
    n, batch = 200000, 4
    a_sorted = np.cumsum(r.uniform(0.02, 0.5, n)).astype(np.float32)
    assert np.all(np.diff(a_sorted) > 0)
    p = r.permutation(n)
    a = a_sorted[p]
    x = r.normal(size=(n, batch)).astype(np.float32)
    y, _ = gpu_gram(a, x)
    inv = np.empty(n, dtype=np.int64); inv[p] = np.arange(n)
    ys = y[inv].astype(np.float64); xs = x[inv].astype(np.float64)
    a64 = a_sorted.astype(np.float64)
    rho = np.exp(-np.diff(a64)); r2 = rho ** 2 / (1 - rho ** 2); off = -rho / (1 - rho ** 2)
    diag = np.ones(n); diag[:-1] += r2; diag[1:] += r2
    back = diag[:, None] * ys; back[:-1] += off[:, None] * ys[1:]; back[1:] += off[:, None] * ys[:-1]
    # row tolerance: sum_j |Kinv_ij| * (1e-5 * T_j + 1e-7) with T_j <= sum_j K_ij |x_j| ~ a few dozen
    tol_y = RTOL * 60.0 + ATOL
    bound = (diag + np.r_[np.abs(off), 0] + np.r_[0, np.abs(off)]) * tol_y
    assert np.all(np.abs(back - xs) <= bound[:, None])


# ------------------------------------------------------------------ the five workloads

def test_workload_square_4096_every_output(oracle):
    w = synth.square_small()
    ref, tol = oracle.apply_brute(w["a"], w["b"], w["x"])
    y, ws = gpu_apply(w["a"], w["b"], w["x"])
    worst = assert_close("y", y, ref, tol)
    assert np.array_equal(gpu_perm(ws, 8192), oracle.merged_permutation(w["a"], w["b"]))
    rel_inf = np.abs(y - ref).max() / np.abs(ref).max()
    print(f"square 4096: worst tolerance ratio {worst:.3g}, rel linf {rel_inf:.3g}")
    assert rel_inf < 5e-6


@pytest.mark.parametrize("scale", [16, 64])
def test_workload_projection_scaled(oracle, scale):
    w = synth.projection_layer(scale=scale)
    a, b, x, g = w["a"], w["b"], w["x"], w["g"]
    ref, tol = oracle.apply_scan(a, b, x)
    y, ws = gpu_apply(a, b, x, flags=B.LAPLEX_SAVE_SCANS)
    assert_close("y", y, ref, tol)
    (rgx, rga, rgb), (tgx, tga, tgb) = oracle.apply_backward_scan(a, b, x, g)
    gx, ga, gb = gpu_backward(a, b, x, g, flags=B.LAPLEX_SAVE_SCANS | B.LAPLEX_REUSE_PLAN, ws=ws)
    assert_close("gx", gx, rgx, tgx); assert_close("ga", ga, rga, tga); assert_close("gb", gb, rgb, tgb)


def test_workload_tie_heavy_scaled(oracle):
    w = synth.tie_heavy(scale=64)            # n = k = 2^18 on a 1/4 grid of 2^14 points
    a, b, x, g = w["a"], w["b"], w["x"], w["g"]
    y, ws = gpu_apply(a, b, x, flags=B.LAPLEX_SAVE_SCANS)
    assert np.array_equal(gpu_perm(ws, a.size + b.size), oracle.merged_permutation(a, b))
    ref, tol = oracle.apply_scan(a, b, x)
    assert_close("y", y, ref, tol)
    (rgx, rga, rgb), (tgx, tga, tgb) = oracle.apply_backward_scan(a, b, x, g)
    gx, ga, gb = gpu_backward(a, b, x, g, flags=B.LAPLEX_SAVE_SCANS | B.LAPLEX_REUSE_PLAN, ws=ws)
    assert_close("gx", gx, rgx, tgx); assert_close("ga", ga, rga, tga); assert_close("gb", gb, rgb, tgb)


def test_workload_gram_images_scaled(oracle):
    w = synth.gram_images(scale=32)          # n = 98304, batch 64
    a, x, g = w["a"], w["x"], w["g"]
    ref, tol = oracle.gram_scan(a, x)
    y, ws = gpu_gram(a, x, flags=B.LAPLEX_SAVE_SCANS)
    assert_close("y", y, ref, tol)
    (rgx, rga), (tgx, tga) = oracle.gram_backward_scan(a, x, g)
    gx, ga = gpu_gram_backward(a, x, g, flags=B.LAPLEX_SAVE_SCANS | B.LAPLEX_REUSE_PLAN, ws=ws)
    assert_close("gx", gx, rgx, tgx); assert_close("ga", ga, rga, tga)


def test_workload_billion_scaled(oracle):
    w = synth.billion_square(scale=1024)     # n = k = 2^20, anchors U(0, 2^14)
    a, b, x, g = w["a"], w["b"], w["x"], w["g"]
    ref, tol = oracle.apply_scan(a, b, x)
    y, ws = gpu_apply(a, b, x, flags=B.LAPLEX_SAVE_SCANS)
    assert_close("y", y, ref, tol)
    assert np.array_equal(gpu_perm(ws, a.size + b.size), oracle.merged_permutation(a, b))
    (rgx, rga, rgb), (tgx, tga, tgb) = oracle.apply_backward_scan(a, b, x, g)
    gx, ga, gb = gpu_backward(a, b, x, g, flags=B.LAPLEX_SAVE_SCANS | B.LAPLEX_REUSE_PLAN, ws=ws)
    assert_close("gx", gx, rgx, tgx); assert_close("ga", ga, rga, tga); assert_close("gb", gb, rgb, tgb)


# ------------------------------------------------------------------ stream capture

@pytest.mark.parametrize("n", [20000, 2000])          # the large path, and the two-launch path for small problems
def test_hip_graph_replays_match_eager(n):
    """The calls only enqueue kernels (no allocation, no synchronisation, no memset), so a
    forward + backward pair can be captured in a HIP graph.  Every replay, with fresh inputs
    copied into the captured buffers and eager work in between, must give the eager bits."""
    r = np.random.default_rng(21)
    k, batch = 300, 16
    a, b = anchors("uniform", r, k, n)
    da, db = dev(a), dev(b)
    dx = torch.empty(n, batch, device="cuda"); dg = torch.empty(k, batch, device="cuda")
    y = torch.empty(k, batch, device="cuda"); gx = torch.empty(n, batch, device="cuda")
    ga = torch.empty(k, device="cuda"); gb = torch.empty(n, device="cuda")
    ws = workspace(k, n, batch)

    def run():
        B.laplex_apply(da, db, dx, y, ws, B.LAPLEX_SAVE_SCANS)
        B.laplex_apply_backward(da, db, dx, dg, gx, ga, gb, ws, B.LAPLEX_SAVE_SCANS | B.LAPLEX_REUSE_PLAN)

    dx.normal_(); dg.normal_()
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):
        run()                                   # warm-up outside the capture
    torch.cuda.current_stream().wait_stream(side)
    torch.cuda.synchronize()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph, stream=side):
        run()
    for rep in range(4):
        xs = torch.from_numpy(r.normal(size=(n, batch)).astype(np.float32)).cuda()
        gs = torch.from_numpy(r.normal(size=(k, batch)).astype(np.float32)).cuda()
        dx.copy_(xs); dg.copy_(gs)
        run(); torch.cuda.synchronize()
        want = [t.clone() for t in (y, gx, ga, gb)]
        for t in (y, gx, ga, gb):
            t.fill_(float("nan"))
        graph.replay(); torch.cuda.synchronize()
        for name, got, ref in zip(("y", "gx", "ga", "gb"), (y, gx, ga, gb), want):
            assert torch.equal(got, ref), f"replay {rep}: {name} differs from the eager result"


def _replay_check(run, inputs, outputs, fresh, reps=4):
    """capture `run` in a HIP graph; every replay on fresh inputs must give the eager bits"""
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):
        run()                                   # warm-up outside the capture
    torch.cuda.current_stream().wait_stream(side)
    torch.cuda.synchronize()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph, stream=side):
        run()
    for rep in range(reps):
        for t, f in zip(inputs, fresh()):
            t.copy_(f)
        run(); torch.cuda.synchronize()
        want = [t.clone() for t in outputs]
        for t in outputs:
            t.fill_(float("nan"))
        graph.replay(); torch.cuda.synchronize()
        for i, (got, ref) in enumerate(zip(outputs, want)):
            assert torch.equal(got, ref), f"replay {rep}: output {i} differs from the eager result"


def test_hip_graph_replays_batch_one_routes(routed):
    """The routes through partition passes under capture: cursors are cleared by a kernel, the reservations are atomics
    whose order changes nothing in the results."""
    r = np.random.default_rng(22)
    k, n = 21000, 47000
    a, b = anchors("ties", r, k, n)
    da, db = dev(a), dev(b)
    dx = torch.empty(n, 1, device="cuda"); dg = torch.empty(k, 1, device="cuda")
    y = torch.empty(k, 1, device="cuda"); gx = torch.empty(n, 1, device="cuda")
    ga = torch.empty(k, device="cuda"); gb = torch.empty(n, device="cuda")
    ws = workspace(k, n, 1)

    def run():
        B.laplex_apply(da, db, dx, y, ws, B.LAPLEX_SAVE_SCANS)
        B.laplex_apply_backward(da, db, dx, dg, gx, ga, gb, ws, B.LAPLEX_SAVE_SCANS | B.LAPLEX_REUSE_PLAN)

    dx.normal_(); dg.normal_()
    fresh = lambda: (torch.from_numpy(r.normal(size=(n, 1)).astype(np.float32)).cuda(),
                     torch.from_numpy(r.normal(size=(k, 1)).astype(np.float32)).cuda())
    _replay_check(run, (dx, dg), (y, gx, ga, gb), fresh)


def test_hip_graph_replays_phased_wide_batch():
    r = np.random.default_rng(23)
    k, n, batch = 900, 26000, 128
    a, b = clustered_outputs(r, k, n)
    da, db = dev(a), dev(b)
    dphi = dev(r.uniform(-3, 3, k).astype(np.float32)); dpsi = dev(r.uniform(-3, 3, n).astype(np.float32))
    dx = torch.empty(n, batch, device="cuda"); dg = torch.empty(k, batch, device="cuda")
    y = torch.empty(k, batch, device="cuda"); gx = torch.empty(n, batch, device="cuda")
    ga = torch.empty(k, device="cuda"); gb = torch.empty(n, device="cuda")
    gphi = torch.empty(k, device="cuda"); gpsi = torch.empty(n, device="cuda")
    ws = phased_workspace(k, n, batch)

    def run():
        B.laplex_phased_apply(da, dphi, db, dpsi, dx, y, ws, B.LAPLEX_SAVE_SCANS)
        B.laplex_phased_apply_backward(da, dphi, db, dpsi, dx, dg, gx, ga, gb, gphi, gpsi, ws,
                                       B.LAPLEX_SAVE_SCANS | B.LAPLEX_REUSE_PLAN)

    dx.normal_(); dg.normal_()
    fresh = lambda: (torch.from_numpy(r.normal(size=(n, batch)).astype(np.float32)).cuda(),
                     torch.from_numpy(r.normal(size=(k, batch)).astype(np.float32)).cuda())
    _replay_check(run, (dx, dg), (y, gx, ga, gb, gphi, gpsi), fresh, reps=3)


def test_hip_graph_replays_mix_on_the_large_path():
    """Under capture the operators of a sum stay on the captured stream; the arithmetic (a sum of gx per lane, then the
    lanes' sums) is the one of the eager call on the lanes' streams, so every replay gives the eager bits."""
    r = np.random.default_rng(24)
    ops, k, n, batch = 6, 400, 8400, 8
    ab = [anchors("ties", r, k, n) for _ in range(ops)]
    da = dev(np.stack([u for u, _ in ab])); db = dev(np.stack([v for _, v in ab]))
    dw = dev(r.normal(size=ops).astype(np.float32))
    dx = torch.empty(n, batch, device="cuda"); dg = torch.empty(k, batch, device="cuda")
    y = torch.empty(k, batch, device="cuda"); gx = torch.empty(n, batch, device="cuda")
    ga = torch.empty(ops, k, device="cuda"); gb = torch.empty(ops, n, device="cuda"); gw = torch.empty(ops, device="cuda")
    ws = torch.empty(B.laplex_mix_workspace_bytes(ops, k, n, batch), dtype=torch.uint8, device="cuda")

    def run():
        B.laplex_mix_apply(da, db, dw, dx, y, ws, B.LAPLEX_SAVE_SCANS)
        B.laplex_mix_apply_backward(da, db, dw, dx, dg, gx, ga, gb, gw, ws, B.LAPLEX_SAVE_SCANS | B.LAPLEX_REUSE_PLAN)

    dx.normal_(); dg.normal_()
    fresh = lambda: (torch.from_numpy(r.normal(size=(n, batch)).astype(np.float32)).cuda(),
                     torch.from_numpy(r.normal(size=(k, batch)).astype(np.float32)).cuda())
    _replay_check(run, (dx, dg), (y, gx, ga, gb, gw), fresh, reps=3)


# ------------------------------------------------------------------ non-finite anchors

@pytest.mark.parametrize("sorted_flags", [0, B.LAPLEX_A_SORTED | B.LAPLEX_B_SORTED])
def test_non_finite_anchors_do_not_fault(oracle, sorted_flags):
    """NaN and infinite anchors are unsupported: values are unspecified, but the calls must run
    to completion without touching memory out of bounds, and the library must work afterwards."""
    r = np.random.default_rng(31)
    k, n, batch = 700, 9000, 4
    a, b = anchors("uniform", r, k, n)
    a[::50] = np.nan; a[7] = np.inf; a[9] = -np.inf
    b[::333] = np.nan; b[5] = np.inf; b[11] = -np.inf
    x = r.normal(size=(n, batch)).astype(np.float32); g = r.normal(size=(k, batch)).astype(np.float32)
    y, ws = gpu_apply(a, b, x, flags=sorted_flags | B.LAPLEX_SAVE_SCANS)
    gpu_backward(a, b, x, g, flags=B.LAPLEX_SAVE_SCANS | B.LAPLEX_REUSE_PLAN, ws=ws)
    gpu_gram(a, np.ascontiguousarray(x[:k]))
    perm = gpu_perm(ws, k + n)
    if sorted_flags == 0:                      # the radix sort still yields a permutation of all ids
        assert np.array_equal(np.sort(perm), np.arange(k + n, dtype=np.uint32))
    # and a clean problem right after is still exact
    a2, b2 = anchors("uniform", r, k, n)
    y2, _ = gpu_apply(a2, b2, x, ws=ws)
    ref, tol = oracle.apply_scan(a2, b2, x)
    assert_close("y", y2, ref, tol)


# ------------------------------------------------------------------ phased kernel

def phased_workspace(k, n, batch):
    return torch.empty(B.laplex_phased_workspace_bytes(k, n, batch), dtype=torch.uint8, device="cuda")


def gpu_phased(a, phi, b, psi, x, g, flags_fwd=B.LAPLEX_SAVE_SCANS, flags_bwd=B.LAPLEX_SAVE_SCANS | B.LAPLEX_REUSE_PLAN,
               want=(True, True, True, True, True), ws=None, forward=True):
    k, n, batch = a.size, b.size, x.shape[1]
    ws = phased_workspace(k, n, batch) if ws is None else ws
    da, dphi, db, dpsi, dx, dg = dev(a), dev(phi), dev(b), dev(psi), dev(x), dev(g)
    y = torch.full((k, batch), float("nan"), device="cuda")
    if forward:
        B.laplex_phased_apply(da, dphi, db, dpsi, dx, y, ws, flags_fwd)
    outs = [torch.full(s, float("nan"), device="cuda") if w else None
            for s, w in zip(((n, batch), (k,), (n,), (k,), (n,)), want)]
    B.laplex_phased_apply_backward(da, dphi, db, dpsi, dx, dg, *outs, ws, flags_bwd)
    torch.cuda.synchronize()
    return y.cpu().numpy(), tuple(None if t is None else t.cpu().numpy() for t in outs), ws


@pytest.mark.parametrize("kind", ["uniform", "ties"])
@pytest.mark.parametrize("k,n,batch", [(5, 1, 2), (37, 53, 3), (2500, 4000, 8), (300, 2100, 64), (24, 7000, 128),
                                       (700, 900, 130)])
def test_phased_forward_backward(oracle, kind, k, n, batch):
    r = np.random.default_rng(5000 + k + n + batch)
    a, b = anchors(kind, r, k, n)
    phi = r.uniform(-7, 7, k).astype(np.float32); psi = r.uniform(-7, 7, n).astype(np.float32)
    x = r.normal(size=(n, batch)).astype(np.float32); g = r.normal(size=(k, batch)).astype(np.float32)
    small = k * n <= 4e6
    ref, tol = (oracle.phased_apply_brute if small else oracle.phased_apply_scan)(a, phi, b, psi, x)
    want, tols = (oracle.phased_backward_brute if small else oracle.phased_backward_scan)(a, phi, b, psi, x, g)
    y, grads, ws = gpu_phased(a, phi, b, psi, x, g)
    assert_close("y", y, ref, tol)
    for name, got, rv, tv in zip(("gx", "ga", "gb", "gphi", "gpsi"), grads, want, tols):
        assert_close(name, got, rv, tv)
    # standing alone (sorts, modulates and, for gphi, multiplies itself): the same bits
    _, alone, _ = gpu_phased(a, phi, b, psi, x, g, flags_bwd=0, forward=False)
    for name, u, v in zip(("gx", "ga", "gb", "gphi", "gpsi"), grads, alone):
        assert np.array_equal(u, v), name


def test_phased_subsets_and_empty_sides(oracle):
    r = np.random.default_rng(77)
    k, n, batch = 40, 300, 5
    a, b = anchors("uniform", r, k, n)
    phi = r.uniform(-3, 3, k).astype(np.float32); psi = r.uniform(-3, 3, n).astype(np.float32)
    x = r.normal(size=(n, batch)).astype(np.float32); g = r.normal(size=(k, batch)).astype(np.float32)
    want, tols = oracle.phased_backward_brute(a, phi, b, psi, x, g)
    names = ("gx", "ga", "gb", "gphi", "gpsi")
    for pick in ((True, False, False, False, False), (False, False, False, True, False),
                 (False, True, False, False, True), (False, False, True, False, False)):
        _, grads, _ = gpu_phased(a, phi, b, psi, x, g, flags_bwd=0, want=pick, forward=False)
        for name, got, rv, tv, w in zip(names, grads, want, tols, pick):
            if w:
                assert_close(name, got, rv, tv)
    # gx alone needs no x
    ws = phased_workspace(k, n, batch)
    gx = torch.full((n, batch), float("nan"), device="cuda")
    B.laplex_phased_apply_backward(dev(a), dev(phi), dev(b), dev(psi), None, dev(g), gx, None, None, None, None, ws, 0)
    torch.cuda.synchronize()
    assert_close("gx", gx.cpu().numpy(), want[0], tols[0])
    # no inputs: y = 0 and every gradient 0
    e = np.zeros(0, dtype=np.float32)
    y, grads, _ = gpu_phased(a, phi, e, e, np.zeros((0, batch), dtype=np.float32), g, flags_fwd=0, flags_bwd=0)
    assert np.all(y == 0) and all(np.all(t == 0) for t in grads)


def clustered_outputs(r, k, n):
    """Inputs spread out, outputs bunched into a few narrow clusters: some 64-row blocks of the merged order hold many
    outputs (the downsweeps with a scan inside the block own them), most hold none or a handful."""
    span = (k + n) / 128.0
    b = r.uniform(0, span, n)
    centres = r.uniform(0, span, 6)
    a = centres[r.integers(0, 6, k)] + r.normal(size=k) * 0.02
    a[: k // 3] = r.uniform(0, span, k // 3)
    return a.astype(np.float32), b.astype(np.float32)


@pytest.mark.parametrize("kind", ["uniform", "ties", "clustered_outputs"])
@pytest.mark.parametrize("k,n,batch", [(3000, 20000, 128), (1500, 30000, 192), (40, 30000, 256), (6000, 9000, 68)])
def test_phased_backward_merges_in_the_downsweep(oracle, kind, k, n, batch):
    """Wide batches on the large path: the streaming downsweep of the backward forms gx, gpsi and gb from both halves in
    registers; blocks with many outputs go through the doubled result matrix and are merged afterwards."""
    r = np.random.default_rng(6100 + k + n + batch)
    a, b = clustered_outputs(r, k, n) if kind == "clustered_outputs" else anchors(kind, r, k, n)
    phi = r.uniform(-7, 7, k).astype(np.float32); psi = r.uniform(-7, 7, n).astype(np.float32)
    x = r.normal(size=(n, batch)).astype(np.float32); g = r.normal(size=(k, batch)).astype(np.float32)
    ref, tol = oracle.phased_apply_scan(a, phi, b, psi, x)
    want, tols = oracle.phased_backward_scan(a, phi, b, psi, x, g)
    y, grads, ws = gpu_phased(a, phi, b, psi, x, g)
    assert_close("y", y, ref, tol)
    names = ("gx", "ga", "gb", "gphi", "gpsi")
    for name, got, rv, tv in zip(names, grads, want, tols):
        assert_close(name, got, rv, tv)
    _, alone, _ = gpu_phased(a, phi, b, psi, x, g, flags_bwd=0, forward=False)
    for name, u, v in zip(names, grads, alone):
        assert np.array_equal(u, v), name
    # subsets of the gradients (gx needs no x; gpsi alone; gb alone)
    for pick in ((True, False, False, False, False), (False, False, False, False, True), (False, False, True, False, False),
                 (True, False, True, False, False)):
        _, part, _ = gpu_phased(a, phi, b, psi, x, g, flags_bwd=0, want=pick, forward=False)
        for name, got, rv, tv, w in zip(names, part, want, tols, pick):
            if w:
                assert_close(name, got, rv, tv)
    # rows that do not allow 16-byte accesses take the route through the doubled result matrix: same results within the bar
    da, dphi, db, dpsi, dg = dev(a), dev(phi), dev(b), dev(psi), dev(g)
    xp = torch.zeros(n, batch + 1, device="cuda"); xp[:, :batch] = dev(x)
    outs = [torch.full(s_, float("nan"), device="cuda") for s_ in ((n, batch), (k,), (n,), (k,), (n,))]
    B.laplex_phased_apply_backward(da, dphi, db, dpsi, xp, dg, *outs, ws, 0)
    torch.cuda.synchronize()
    for name, got, rv, tv in zip(names, outs, want, tols):
        assert_close(name, got.cpu().numpy(), rv, tv)
    # ... also when it continues a forward that was given rows it could read directly (the doubled copy of x that the
    # forward left holds the rows of some blocks only: the backward finds that out and completes it), and the other way round
    y2 = torch.full((k, batch), float("nan"), device="cuda")
    xv = xp[:, :batch]              # the same rows, 4 * (batch + 1) bytes apart
    for fwd_x, bwd_x in ((dev(x), xv), (xv, dev(x))):
        B.laplex_phased_apply(da, dphi, db, dpsi, fwd_x, y2, ws, B.LAPLEX_SAVE_SCANS)
        outs = [torch.full(s_, float("nan"), device="cuda") for s_ in ((n, batch), (k,), (n,), (k,), (n,))]
        B.laplex_phased_apply_backward(da, dphi, db, dpsi, bwd_x, dg, *outs, ws, B.LAPLEX_SAVE_SCANS | B.LAPLEX_REUSE_PLAN)
        torch.cuda.synchronize()
        assert_close("y", y2.cpu().numpy(), ref, tol)
        for name, got, rv, tv in zip(names, outs, want, tols):
            assert_close(name, got.cpu().numpy(), rv, tv)


def test_phased_backward_invalid_plan_poisons():
    r = np.random.default_rng(6200)
    k, n, batch = 2000, 24000, 128
    a, b = clustered_outputs(r, k, n)
    phi = r.uniform(-7, 7, k).astype(np.float32); psi = r.uniform(-7, 7, n).astype(np.float32)
    x = r.normal(size=(n, batch)).astype(np.float32); g = r.normal(size=(k, batch)).astype(np.float32)
    y, grads, ws = gpu_phased(a, phi, b, psi, x, g)
    assert all(np.isfinite(t).all() for t in grads)
    B.laplex_diag_set_plan_status(ws, k + n, 1)
    # (the forward runs again on the marked plan: ga and gphi are formed from what it saves)
    y, grads, _ = gpu_phased(a, phi, b, psi, x, g, ws=ws, flags_fwd=B.LAPLEX_SAVE_SCANS | B.LAPLEX_REUSE_PLAN)
    assert np.isnan(y).all()
    for name, t in zip(("gx", "ga", "gb", "gphi", "gpsi"), grads):
        assert np.isnan(t).all(), f"{name}: a value computed from an invalid plan is not NaN"


# ------------------------------------------------------------------ temperature

@pytest.mark.parametrize("tau", [0.37, 1.0, 5.0])
@pytest.mark.parametrize("kind", ["uniform", "ties", "signed"])
@pytest.mark.parametrize("k,n,batch", [(5, 1, 2), (37, 53, 3), (3000, 21000, 1), (2500, 4000, 8), (300, 2100, 256),
                                       (20, 6000, 256)])
def test_temperature_forward_backward(oracle, tau, kind, k, n, batch):
    """exp(-tau |a_i - b_j|): values, the permutation of the scaled anchors, all four gradients."""
    r = np.random.default_rng(int(tau * 100) + k + n + batch)
    a, b = anchors(kind, r, k, n)
    x = r.normal(size=(n, batch)).astype(np.float32); g = r.normal(size=(k, batch)).astype(np.float32)
    brute = k * n * batch <= 4e7
    ref, tol = oracle.tau_apply(a, b, tau, x, brute=brute)
    (rgx, rga, rgb, rgt), (tgx, tga, tgb, tgt) = oracle.tau_backward(a, b, tau, x, g, brute=brute)
    ws = workspace(k, n, batch)
    da, db, dx, dg = dev(a), dev(b), dev(x), dev(g)
    y = torch.full((k, batch), float("nan"), device="cuda")
    gx = torch.full((n, batch), float("nan"), device="cuda")
    ga = torch.full((k,), float("nan"), device="cuda"); gb = torch.full((n,), float("nan"), device="cuda")
    gt = torch.full((1,), float("nan"), device="cuda")
    B.laplex_apply_tau(da, db, tau, dx, y, ws, B.LAPLEX_SAVE_SCANS)
    B.laplex_apply_backward_tau(da, db, tau, dx, dg, gx, ga, gb, gt, ws, B.LAPLEX_SAVE_SCANS | B.LAPLEX_REUSE_PLAN)
    torch.cuda.synchronize()
    assert np.array_equal(gpu_perm(ws, k + n),
                          oracle.merged_permutation(oracle.scaled_anchors(a, tau), oracle.scaled_anchors(b, tau)))
    assert_close("y", y.cpu().numpy(), ref, tol)
    assert_close("gx", gx.cpu().numpy(), rgx, tgx)
    assert_close("ga", ga.cpu().numpy(), rga, tga)
    assert_close("gb", gb.cpu().numpy(), rgb, tgb)
    assert_close("gtau", gt.cpu().numpy(), np.array([rgt]), np.array([tgt]))
    if tau == 1.0:                                          # the bits of the plain calls
        y1, ws1 = gpu_apply(a, b, x, flags=B.LAPLEX_SAVE_SCANS)
        g1 = gpu_backward(a, b, x, g, flags=B.LAPLEX_SAVE_SCANS | B.LAPLEX_REUSE_PLAN, ws=ws1)
        for u, v in zip((y, gx, ga, gb), (y1,) + g1):
            assert np.array_equal(u.cpu().numpy(), v)


@pytest.mark.parametrize("top,tau", [(2.0 ** 14, 5.0), (2.0 ** 14, 0.37), (2.0 ** 14, 1.0 / 3.0), (64.0, 5.0), (64.0, 0.37)])
@pytest.mark.parametrize("k,n,batch", [(400, 30000, 4), (2000, 9000, 1)])
def test_temperature_against_the_definition(oracle, top, tau, k, n, batch):
    """laplex_apply_tau against exp(-tau |a_i - b_j|) itself (App. A), fp64, nothing rounded on the way in.
    The library scales the anchors in fp32: each product tau*a is off by at most 2^-24 of itself, so every
    exponent is off by at most delta = 2^-24 tau (|a_i| + |b_j|) <= 2^-23 tau `top`, every term by a factor of at
    most e^delta, and the bound becomes (e^delta - 1) T + 1e-5 e^delta T + 1e-7: the input-rounding term and
    the bar of every other parity test."""
    r = np.random.default_rng(int(top) + int(100 * tau) + k)
    a = r.uniform(0, top, k).astype(np.float32); b = r.uniform(0, top, n).astype(np.float32)
    b[: n // 8] = a[r.integers(0, k, n // 8)] + r.uniform(-0.5, 0.5, n // 8).astype(np.float32)   # near neighbours
    x = r.normal(size=(n, batch)).astype(np.float32)
    ref, tol = oracle.tau_apply_dense(a, b, tau, x)
    ws = workspace(k, n, batch)
    y = torch.full((k, batch), float("nan"), device="cuda")
    B.laplex_apply_tau(dev(a), dev(b), tau, dev(x), y, ws, 0)
    torch.cuda.synchronize()
    got = y.cpu().numpy().astype(np.float64)
    delta = 2.0 ** -23 * tau * top
    bound = np.expm1(delta) * tol + RTOL * np.exp(delta) * tol + ATOL
    worst = float((np.abs(got - ref) / bound).max())
    assert np.all(np.isfinite(got)) and worst <= 1.0, f"{worst:.3g}x the bound (delta = {delta:.3g})"


@pytest.mark.parametrize("tau", [0.25, 3.0])
def test_temperature_merge_path_and_gram(oracle, tau):
    r = np.random.default_rng(901)
    k, n, batch = 700, 9000, 4
    a, b = anchors("ties", r, k, n)
    a.sort(); b.sort()
    x = r.normal(size=(n, batch)).astype(np.float32)
    ws = workspace(k, n, batch)
    y = torch.full((k, batch), float("nan"), device="cuda")
    B.laplex_apply_tau(dev(a), dev(b), tau, dev(x), y, ws, B.LAPLEX_A_SORTED | B.LAPLEX_B_SORTED)
    torch.cuda.synchronize()
    assert np.array_equal(gpu_perm(ws, k + n),
                          oracle.merged_permutation(oracle.scaled_anchors(a, tau), oracle.scaled_anchors(b, tau)))
    ref, tol = oracle.tau_apply(a, b, tau, x, brute=False)
    assert_close("y", y.cpu().numpy(), ref, tol)
    # Gram form with its temperature gradient
    m = 5000
    ag = (r.normal(size=m) * 30).astype(np.float32); ag[::9] = ag[3]
    xg = r.normal(size=(m, batch)).astype(np.float32); gg = r.normal(size=(m, batch)).astype(np.float32)
    wsg = workspace(0, m, batch)
    yg = torch.full((m, batch), float("nan"), device="cuda"); gxg = torch.full((m, batch), float("nan"), device="cuda")
    gag = torch.full((m,), float("nan"), device="cuda"); gt = torch.full((1,), float("nan"), device="cuda")
    B.laplex_gram_tau(dev(ag), tau, dev(xg), yg, wsg, B.LAPLEX_SAVE_SCANS)
    B.laplex_gram_backward_tau(dev(ag), tau, dev(xg), dev(gg), gxg, gag, gt, wsg, B.LAPLEX_SAVE_SCANS | B.LAPLEX_REUSE_PLAN)
    torch.cuda.synchronize()
    sa = oracle.scaled_anchors(ag, tau)
    refy, toly = oracle.gram_scan(sa, xg)
    (rgx, rga, rgt), (tgx, tga, tgt) = oracle.tau_gram_backward(ag, tau, xg, gg, brute=False)
    assert_close("gram y", yg.cpu().numpy(), refy, toly)
    assert_close("gram gx", gxg.cpu().numpy(), rgx, tgx)
    assert_close("gram ga", gag.cpu().numpy(), rga, tga)
    assert_close("gram gtau", gt.cpu().numpy(), np.array([rgt]), np.array([tgt]))


# ------------------------------------------------------------------ weighted Gram matrix

def gpu_wgram(a, b, d, flags=0, ws=None, ldm=None):
    k, n = a.size, b.size
    ws = torch.empty(B.laplex_wgram_workspace_bytes(k, n), dtype=torch.uint8, device="cuda") if ws is None else ws
    mbuf = torch.full((k, k if ldm is None else ldm), float("nan"), device="cuda")
    m = mbuf[:, :k]
    B.laplex_wgram(dev(a), dev(b), dev(d), m, ws, flags)
    torch.cuda.synchronize()
    return m.cpu().numpy(), ws


WGRAM_SHAPES = [(1, 1), (2, 3), (5, 1), (1, 700), (37, 53), (100, 9000), (9000 // 8, 100), (1024, 40000), (333, 70001),
                (700, 700), (3, 150000),
                # runs of equal Gram anchors longer than a lane's 16 positions, with hardly any middle anchor between:
                # entries far from every middle anchor are tiny and take the difference of two prefix sums exactly
                (1072, 3), (4500, 40)]


@pytest.mark.parametrize("weights", ["signed", "positive"])
@pytest.mark.parametrize("kind", ["uniform", "ties", "all_equal", "huge_gaps", "clustered", "signed"])
@pytest.mark.parametrize("k,n", WGRAM_SHAPES)
def test_weighted_gram_matrix(oracle, weights, kind, k, n):
    """M = A diag(d) A^T: every entry against the oracle, |err| <= 1e-5 T + 1e-7 with
    T_ij = sum_t |d_t| A_it A_jt; the plan is that of the doubled anchors."""
    r = np.random.default_rng(11 * k + n + len(kind))
    a, b = anchors(kind, r, k, n)
    d = r.normal(size=n).astype(np.float32)
    if weights == "positive":
        d = np.abs(d) + np.float32(0.5)
    ref, tol = (oracle.wgram_dense if k * k * n <= 3e8 else oracle.wgram_scan)(a, b, d)
    m, ws = gpu_wgram(a, b, d)
    assert_close("M", m, ref, tol)
    assert np.array_equal(m, m.T), "the two triangles must hold the same bits"
    two = np.float32(2)
    assert np.array_equal(gpu_perm(ws, k + n), oracle.merged_permutation(two * a, two * b))


def test_weighted_gram_options(oracle):
    r = np.random.default_rng(404)
    k, n = 300, 20000
    a, b = anchors("ties", r, k, n)
    d = r.normal(size=n).astype(np.float32)
    ref, tol = oracle.wgram_scan(a, b, d)
    m, ws = gpu_wgram(a, b, d, ldm=k + 5)                          # padded rows: scalar stores
    assert_close("M (padded)", m, ref, tol)
    d2 = r.normal(size=n).astype(np.float32)                       # new weights on the kept plan
    ref2, tol2 = oracle.wgram_scan(a, b, d2)
    m2, _ = gpu_wgram(a, b, d2, flags=B.LAPLEX_REUSE_PLAN, ws=ws)
    assert_close("M (plan reused)", m2, ref2, tol2)
    sa, sb_order = np.sort(a), np.argsort(b, kind="stable")        # both sorted: the merge path
    m3, _ = gpu_wgram(sa, b[sb_order], d[sb_order], flags=B.LAPLEX_A_SORTED | B.LAPLEX_B_SORTED)
    ref3, tol3 = oracle.wgram_scan(sa, b[sb_order], d[sb_order])
    assert_close("M (merge path)", m3, ref3, tol3)
    e = np.zeros(0, dtype=np.float32)                              # nothing to sum over
    m4, _ = gpu_wgram(a, e, e)
    assert np.all(m4 == 0)


# ------------------------------------------------------------------ LAPLEX^(r): weighted sums of operators

def gpu_mix(a, b, w, x, g, flags_fwd, flags_bwd, want=(True, True, True, True), forward=True):
    r, k = a.shape; n = b.shape[1]; batch = x.shape[1]
    ws = torch.empty(B.laplex_mix_workspace_bytes(r, k, n, batch), dtype=torch.uint8, device="cuda")
    da, db, dw, dx, dg = dev(a), dev(b), dev(w), dev(x), dev(g)
    y = torch.full((k, batch), float("nan"), device="cuda")
    if forward:
        B.laplex_mix_apply(da, db, dw, dx, y, ws, flags_fwd)
    outs = [torch.full(s, float("nan"), device="cuda") if wnt else None
            for s, wnt in zip(((n, batch), (r, k), (r, n), (r,)), want)]
    B.laplex_mix_apply_backward(da, db, dw, dx, dg, *outs, ws, flags_bwd)
    torch.cuda.synchronize()
    return y.cpu().numpy(), tuple(None if t is None else t.cpu().numpy() for t in outs)


@pytest.mark.parametrize("kind", ["uniform", "ties"])
@pytest.mark.parametrize("r,k,n,batch", [(1, 5, 1, 2), (3, 37, 53, 3), (4, 10, 512, 64), (16, 100, 768, 128),
                                         (2, 1000, 2048, 256), (5, 300, 2100, 1),
                                         # more than 8192 merged positions: the large path, up to four operators side by
                                         # side on streams of the library's own (the last case: two rounds of them)
                                         (2, 500, 9000, 4), (3, 40, 8200, 64), (6, 300, 8300, 16)])
def test_mix_forward_backward(oracle, kind, r, k, n, batch):
    """y = sum_q w_q L(a_q, b_q) x and the gradients (gx, ga, gb, gw), the classification-head shapes
    (classes x features) among them."""
    q = np.random.default_rng(9000 + r + k + n + batch)
    ab = [anchors(kind, q, k, n) for _ in range(r)]
    a = np.stack([u for u, _ in ab]); b = np.stack([v for _, v in ab])
    w = q.normal(size=r).astype(np.float32)
    x = q.normal(size=(n, batch)).astype(np.float32); g = q.normal(size=(k, batch)).astype(np.float32)
    brute = r * k * n * batch <= 6e7
    ref, tol = oracle.mix_apply(a, b, w, x, brute=brute)
    want, tols = oracle.mix_backward(a, b, w, x, g, brute=brute)
    y, grads = gpu_mix(a, b, w, x, g, B.LAPLEX_SAVE_SCANS, B.LAPLEX_SAVE_SCANS | B.LAPLEX_REUSE_PLAN)
    assert_close("y", y, ref, tol)
    for name, got, rv, tv in zip(("gx", "ga", "gb", "gw"), grads, want, tols):
        assert_close(name, got, rv, tv)
    # the backward standing alone (sorts and recomputes the products itself): the same bits
    _, alone = gpu_mix(a, b, w, x, g, 0, 0, forward=False)
    for name, u, v in zip(("gx", "ga", "gb", "gw"), grads, alone):
        assert np.array_equal(u, v), name


def test_mix_subsets_and_empty(oracle):
    q = np.random.default_rng(9100)
    r, k, n, batch = 3, 20, 150, 6
    ab = [anchors("uniform", q, k, n) for _ in range(r)]
    a = np.stack([u for u, _ in ab]); b = np.stack([v for _, v in ab])
    w = q.normal(size=r).astype(np.float32)
    x = q.normal(size=(n, batch)).astype(np.float32); g = q.normal(size=(k, batch)).astype(np.float32)
    want, tols = oracle.mix_backward(a, b, w, x, g)
    names = ("gx", "ga", "gb", "gw")
    for pick in ((True, False, False, False), (False, False, False, True), (False, True, True, False)):
        _, grads = gpu_mix(a, b, w, x, g, 0, 0, want=pick, forward=False)
        for name, got, rv, tv, wnt in zip(names, grads, want, tols, pick):
            if wnt:
                assert_close(name, got, rv, tv)
    # no operators: y = 0 and gx = 0
    e = np.zeros((0, k), dtype=np.float32)
    y, grads = gpu_mix(e, np.zeros((0, n), dtype=np.float32), np.zeros(0, dtype=np.float32), x, g, 0, 0,
                       want=(True, False, False, False))
    assert np.all(y == 0) and np.all(grads[0] == 0)


@pytest.mark.parametrize("weights", ["signed", "positive"])
@pytest.mark.parametrize("kind", ["uniform", "ties", "all_equal", "huge_gaps", "clustered"])
@pytest.mark.parametrize("k,n", [(1, 1), (5, 1), (37, 53), (100, 9000), (1024, 40000), (333, 70001), (3, 150000), (1072, 3), (4500, 40)])
def test_weighted_gram_matrix_fp64(oracle, weights, kind, k, n):
    """The fp64 instantiation: fp32 anchors, fp64 weights and arithmetic.  Tolerance 1e-12 T + 1e-300:
    an entry sums a few thousand non-negligible terms, each a product of at most a few hundred fp64 decays
    (16 per thread, 8 scan levels, the tiles of the spine) with one exp each."""
    r = np.random.default_rng(13 * k + n + len(kind))
    a, b = anchors(kind, r, k, n)
    d = r.normal(size=n)
    if weights == "positive":
        d = np.abs(d) + 0.5
    ref, tol = (oracle.wgram_dense if k * k * n <= 3e8 else oracle.wgram_scan)(a, b, d)
    ws = torch.empty(B.laplex_wgram_f64_workspace_bytes(k, n), dtype=torch.uint8, device="cuda")
    m = torch.full((k, k), float("nan"), dtype=torch.float64, device="cuda")
    B.laplex_wgram_f64(dev(a), dev(b), dev(d), m, ws, 0)
    torch.cuda.synchronize()
    got = m.cpu().numpy()
    assert np.all(np.isfinite(got))
    ratio = np.abs(got - ref) / (1e-12 * tol + 1e-300)
    assert ratio.max() <= 1.0, f"worst |err| / (1e-12 T) = {ratio.max():.3g}"
    assert np.array_equal(got, got.T)


# ------------------------------------------------------------------ the paper's accuracy experiments

@pytest.mark.parametrize("grid", ["irregular", "uniform"])
def test_accuracy_levels_of_the_paper(oracle, grid, capsys):
    """App. "Numerical accuracy" and "Numerical accuracy on a uniform-grid (Toeplitz) problem": square
    kernel, batch 8, n = 2^10 .. 2^14, fp32 inputs widened to fp64 for the dense reference.  The paper
    reports, for its own fp32 path, relative l_inf errors below 5e-7 and relative l_2 errors around
    1.5e-7 (4.2e-7 l_inf on the uniform grid a_i = b_i = i / n at n = 2^14).  A sanity band (this path:
    1.7e-7 .. 5.7e-7 l_inf, the largest on the uniform grid at n = 2^14, where every output is a
    sum of 16384 terms of like size and random sign: 5.7e-7 of the largest output is 2e-8 of the sum of
    their magnitudes); the acceptance bar of this repository is the per-output tolerance above."""
    r = np.random.default_rng(1234)
    for e in range(10, 15):
        n = 1 << e
        if grid == "uniform":
            a = b = (np.arange(n) / n).astype(np.float32)
        else:
            a = r.uniform(0, n / 32.0, n).astype(np.float32); b = r.uniform(0, n / 32.0, n).astype(np.float32)
        x = r.normal(size=(n, 8)).astype(np.float32)
        y, _ = gpu_apply(a, b, x)
        ref = np.exp(-np.abs(a.astype(np.float64)[:, None] - b.astype(np.float64)[None, :])) @ x.astype(np.float64)
        linf = np.abs(y - ref).max() / np.abs(ref).max()
        l2 = np.linalg.norm(y - ref) / np.linalg.norm(ref)
        with capsys.disabled():
            print(f"[accuracy {grid} n=2^{e}] rel l_inf = {linf:.3g}, rel l_2 = {l2:.3g}", flush=True)
        assert linf < 1.5e-6 and l2 < 1e-6


@pytest.mark.parametrize("gap", [1.0 / 4096, 3.1e-4, 1.3e-3])
@pytest.mark.parametrize("k,n,batch", [(4096, 4096, 1), (1000, 3000, 8), (3000, 5000, 64), (20000, 20000, 1)])
def test_regular_grid_equal_decays(oracle, gap, k, n, batch):
    """Anchors on a regular grid: every neighbour decay is the same number with the same rounding error, so
    a decay over m rows formed as a product is off by m times that error, systematically; all weights
    stay large (the whole grid spans a few units), so every output feels it.  Both paths take decays over
    more than a handful of rows from anchor differences instead."""
    r = np.random.default_rng(k + n + batch)
    a = (np.arange(k) * (gap * n / k)).astype(np.float32)
    b = (np.arange(n) * gap).astype(np.float32)
    x = r.normal(size=(n, batch)).astype(np.float32); g = r.normal(size=(k, batch)).astype(np.float32)
    brute = k * n * batch <= 4e7
    ref, tol = (oracle.apply_brute if brute else oracle.apply_scan)(a, b, x)
    (rgx, rga, rgb), (tgx, tga, tgb) = (oracle.apply_backward_brute if brute else oracle.apply_backward_scan)(a, b, x, g)
    y, ws = gpu_apply(a, b, x, flags=B.LAPLEX_SAVE_SCANS)
    gx, ga, gb = gpu_backward(a, b, x, g, flags=B.LAPLEX_SAVE_SCANS | B.LAPLEX_REUSE_PLAN, ws=ws)
    assert_close("y", y, ref, tol)
    assert_close("gx", gx, rgx, tgx); assert_close("ga", ga, rga, tga); assert_close("gb", gb, rgb, tgb)


# ------------------------------------------------------------------ diagnostics

def test_diag_move_rows_copies_the_named_rows():
    r = np.random.default_rng(77)
    rows, cols = 5000, 256
    src = torch.from_numpy(r.normal(size=(rows, cols)).astype(np.float32)).cuda()
    ids = torch.from_numpy(r.permutation(rows)[:3001].astype(np.int32)).cuda()       # a ragged number of rows, each once
    dst = torch.zeros(rows, cols, device="cuda")
    B.laplex_diag_move_rows(src, dst, ids)
    B.laplex_diag_move_rows(src, None, ids)                                          # read only: must just run
    torch.cuda.synchronize()
    want = torch.zeros(rows, cols, device="cuda")
    want[ids.long()] = src[ids.long()]
    assert torch.equal(dst, want)


# ------------------------------------------------------------------ an invalid plan is never silent

@pytest.mark.parametrize("k,n,batch", [(3000, 21000, 1), (40, 70000, 256), (2500, 9000, 8), (5000, 6000, 64)])
def test_invalid_plan_poisons_every_output(k, n, batch):
    """The radix sort's bounded wait can, in principle, give up; the plan is then marked invalid.  The mark is
    planted here through the test hook (no kernel is made to wait): every output of every call that computes
    from such a plan must be NaN, and a call that rebuilds the plan must be clean again."""
    r = np.random.default_rng(k + n + batch)
    a, b = anchors("uniform", r, k, n)
    x = r.normal(size=(n, batch)).astype(np.float32); g = r.normal(size=(k, batch)).astype(np.float32)
    da, db, dx, dg = dev(a), dev(b), dev(x), dev(g)
    ws = workspace(k, n, batch)
    y = torch.zeros(k, batch, device="cuda")
    B.laplex_apply(da, db, dx, y, ws, B.LAPLEX_SAVE_SCANS)
    torch.cuda.synchronize()
    good = y.clone()
    assert gpu_plan_status(ws, k + n) == 0 and bool(torch.isfinite(y).all())
    B.laplex_diag_set_plan_status(ws, k + n, 1)
    assert gpu_plan_status(ws, k + n) == 1
    y.zero_()
    gx = torch.zeros(n, batch, device="cuda"); ga = torch.zeros(k, device="cuda"); gb = torch.zeros(n, device="cuda")
    B.laplex_apply(da, db, dx, y, ws, B.LAPLEX_SAVE_SCANS | B.LAPLEX_REUSE_PLAN)
    B.laplex_apply_backward(da, db, dx, dg, gx, ga, gb, ws, B.LAPLEX_SAVE_SCANS | B.LAPLEX_REUSE_PLAN)
    torch.cuda.synchronize()
    for name, t in (("y", y), ("gx", gx), ("ga", ga), ("gb", gb)):
        assert bool(torch.isnan(t).all()), f"{name}: a value computed from an invalid plan is not NaN"
    # without saved scans (the backward scans x itself) and for the Gram form on the same workspace size
    B.laplex_apply_backward(da, db, dx, dg, gx, ga, gb, ws, B.LAPLEX_REUSE_PLAN)
    torch.cuda.synchronize()
    assert bool(torch.isnan(ga).all()) and bool(torch.isnan(gx).all()) and bool(torch.isnan(gb).all())
    # a call that builds the plan again clears the mark
    B.laplex_apply(da, db, dx, y, ws, B.LAPLEX_SAVE_SCANS)
    torch.cuda.synchronize()
    assert gpu_plan_status(ws, k + n) == 0 and torch.equal(y, good)


def test_invalid_plan_poisons_gram_and_weighted_gram():
    r = np.random.default_rng(77)
    n, batch = 20000, 4
    a, _ = anchors("uniform", r, n, 1)
    x = r.normal(size=(n, batch)).astype(np.float32); g = r.normal(size=(n, batch)).astype(np.float32)
    da, dx, dg = dev(a), dev(x), dev(g)
    ws = workspace(0, n, batch)
    y = torch.zeros(n, batch, device="cuda"); gx = torch.zeros(n, batch, device="cuda"); ga = torch.zeros(n, device="cuda")
    B.laplex_gram(da, dx, y, ws, B.LAPLEX_SAVE_SCANS)
    B.laplex_diag_set_plan_status(ws, n, 1)
    B.laplex_gram(da, dx, y, ws, B.LAPLEX_SAVE_SCANS | B.LAPLEX_REUSE_PLAN)
    B.laplex_gram_backward(da, dx, dg, gx, ga, ws, B.LAPLEX_SAVE_SCANS | B.LAPLEX_REUSE_PLAN)
    torch.cuda.synchronize()
    assert bool(torch.isnan(y).all()) and bool(torch.isnan(gx).all()) and bool(torch.isnan(ga).all())
    k, n = 300, 12000
    a, b = anchors("uniform", r, k, n)
    d = r.normal(size=n).astype(np.float32)
    wsg = torch.empty(B.laplex_wgram_workspace_bytes(k, n), dtype=torch.uint8, device="cuda")
    m = torch.zeros(k, k, device="cuda")
    B.laplex_wgram(dev(a), dev(b), dev(d), m, wsg, 0)
    torch.cuda.synchronize()
    assert bool(torch.isfinite(m).all())
    B.laplex_diag_set_plan_status(wsg, k + n, 1)
    B.laplex_wgram(dev(a), dev(b), dev(d), m, wsg, B.LAPLEX_REUSE_PLAN)
    torch.cuda.synchronize()
    assert bool(torch.isnan(m).all())


# ------------------------------------------------------------------ batch 1: the routes without random accesses

@pytest.fixture
def routed():
    """Batch-1 problems of any size (beyond the small path) take the partition routes while the test runs."""
    B.laplex_diag_set_route_min(0)
    yield
    B.laplex_diag_set_route_min(1 << 22)


def _apply_both_ways(a, b, x, g, save, want=(True, True, True), merge=False):
    """forward + backward at batch 1, on the current route; returns (y, gx, ga, gb) as numpy arrays (None where not wanted)"""
    k, n = a.size, b.size
    ws = workspace(k, n, 1)
    da, db, dx, dg = dev(a), dev(b), dev(x), dev(g)
    y = torch.full((k, 1), float("nan"), device="cuda")
    gx = torch.full((n, 1), float("nan"), device="cuda") if want[0] else None
    ga = torch.full((k,), float("nan"), device="cuda") if want[1] else None
    gb = torch.full((n,), float("nan"), device="cuda") if want[2] else None
    f = (B.LAPLEX_A_SORTED | B.LAPLEX_B_SORTED) if merge else 0
    if save:
        B.laplex_apply(da, db, dx, y, ws, f | B.LAPLEX_SAVE_SCANS)
        B.laplex_apply_backward(da, db, dx, dg, gx, ga, gb, ws, f | B.LAPLEX_SAVE_SCANS | B.LAPLEX_REUSE_PLAN)
    else:
        B.laplex_apply(da, db, dx, y, ws, f)
        B.laplex_apply_backward(da, db, dx, dg, gx, ga, gb, ws, f)        # stands alone: builds its own plan, scans x itself
    torch.cuda.synchronize()
    assert gpu_plan_status(ws, k + n) == 0
    perm = gpu_perm(ws, k + n)
    return [None if t is None else t.cpu().numpy() for t in (y, gx, ga, gb)], perm


ROUTE_SHAPES = [(100, 9000), (9000, 100), (1, 20000), (20000, 1), (3000, 21000), (50000, 70000), (8192, 8192 * 3),
                (300000, 500000), (2200000, 2400000)]


@pytest.mark.parametrize("kind", ["uniform", "ties", "all_equal", "clustered", "ascending"])
@pytest.mark.parametrize("k,n", ROUTE_SHAPES)
def test_routes_without_random_access(oracle, routed, kind, k, n):
    """At batch 1 x and gy reach sorted order, and y, the saved scans, gx and gb the caller's order, through partition
    passes when there are many rows, with scan kernels that work on plain arrays in sorted order in between.  One and
    two partition levels, ragged windows, a single output or input, sources that arrive in order: the permutation equals
    the other route's bit for bit, every value sits within the bar of the oracle, and the two routes agree to rounding."""
    if kind != "uniform" and k + n > 1000000:
        pytest.skip("the largest shape runs once")
    r = np.random.default_rng(k * 7 + n)
    if kind == "ascending":
        a = np.sort(r.uniform(0, (k + n) / 64.0, k)).astype(np.float32); b = np.sort(r.uniform(0, (k + n) / 64.0, n)).astype(np.float32)
    else:
        a, b = anchors(kind, r, k, n)
    x = r.normal(size=(n, 1)).astype(np.float32); g = r.normal(size=(k, 1)).astype(np.float32)
    brute = k * n <= 4e7
    ref, tol = (oracle.apply_brute if brute else oracle.apply_scan)(a, b, x)
    refs, tols = (oracle.apply_backward_brute if brute else oracle.apply_backward_scan)(a, b, x, g)
    refs, tols = (ref,) + tuple(refs), (tol,) + tuple(tols)
    for save in (True, False):
        got, perm = _apply_both_ways(a, b, x, g, save)
        B.laplex_diag_set_route_min(1 << 40)
        other, perm0 = _apply_both_ways(a, b, x, g, save)
        B.laplex_diag_set_route_min(0)
        assert np.array_equal(perm, perm0)
        for name, u, v, rf, tl in zip(("y", "gx", "ga", "gb"), got, other, refs, tols):
            assert_close(name, u, rf, tl)
            tl = np.asarray(tl).reshape(u.shape)
            assert np.all(np.abs(u.astype(np.float64) - v) <= 2e-6 * tl + 1e-7), f"{name}: the routes disagree (save={save})"


@pytest.mark.parametrize("want", [(True, False, False), (False, True, False), (False, False, True), (True, False, True), (False, True, True)])
def test_routes_gradient_subsets_and_merge_path(oracle, routed, want):
    r = np.random.default_rng(sum(want) * 11 + want[0])
    k, n = 30000, 41000
    a = np.sort(r.uniform(0, 900, k)).astype(np.float32); b = np.sort(r.uniform(0, 900, n)).astype(np.float32)
    b[::7] = a[r.integers(0, k, b[::7].size)]; b.sort()                   # exact ties between the two sets
    x = r.normal(size=(n, 1)).astype(np.float32); g = r.normal(size=(k, 1)).astype(np.float32)
    (rgx, rga, rgb), (tgx, tga, tgb) = oracle.apply_backward_scan(a, b, x, g)
    for save in (True, False):
        for merge in (False, True):
            got, _ = _apply_both_ways(a, b, x, g, save, want=want, merge=merge)
            if want[0]: assert_close("gx", got[1], rgx, tgx)
            if want[1]: assert_close("ga", got[2], rga, tga)
            if want[2]: assert_close("gb", got[3], rgb, tgb)


@pytest.mark.parametrize("kind", ["uniform", "ties", "clustered"])
@pytest.mark.parametrize("n", [8193, 20000, 70001, 300000])
def test_routes_gram_form(oracle, routed, kind, n):
    """The square form at batch 1 on the same routes: every row is injected and read; ga = gy Z^x + x Z^g is completed
    from the saved scans in the caller's order."""
    r = np.random.default_rng(9100 + n)
    a, _ = anchors(kind, r, n, 1)
    x = r.normal(size=(n, 1)).astype(np.float32); g = r.normal(size=(n, 1)).astype(np.float32)
    small = n * n <= 4e7
    ref, tol = (oracle.gram_brute if small else oracle.gram_scan)(a, x)
    (rgx, rga), (tgx, tga) = (oracle.gram_backward_brute if small else oracle.gram_backward_scan)(a, x, g)
    y, ws = gpu_gram(a, x, flags=B.LAPLEX_SAVE_SCANS)
    assert_close("y", y, ref, tol)
    assert np.array_equal(gpu_perm(ws, n), oracle.merged_permutation(a))
    gx, ga = gpu_gram_backward(a, x, g, flags=B.LAPLEX_SAVE_SCANS | B.LAPLEX_REUSE_PLAN, ws=ws)
    assert_close("gx", gx, rgx, tgx); assert_close("ga", ga, rga, tga)
    gx2, ga2 = gpu_gram_backward(a, x, g)                       # standing alone: scans x itself
    assert np.array_equal(gx, gx2) and np.array_equal(ga, ga2)
    _, ga3 = gpu_gram_backward(a, x, g, want=(False, True))
    assert np.array_equal(ga, ga3)
    gx4, _ = gpu_gram_backward(a, x, g, want=(True, False))
    assert np.array_equal(gx, gx4)
    # the other route: the same within rounding
    B.laplex_diag_set_route_min(1 << 40)
    y0, ws0 = gpu_gram(a, x, flags=B.LAPLEX_SAVE_SCANS)
    gx0, ga0 = gpu_gram_backward(a, x, g, flags=B.LAPLEX_SAVE_SCANS | B.LAPLEX_REUSE_PLAN, ws=ws0)
    B.laplex_diag_set_route_min(0)
    for name, u, v, tl in (("y", y, y0, tol), ("gx", gx, gx0, tgx), ("ga", ga, ga0, tga)):
        tl = np.asarray(tl).reshape(u.shape)
        assert np.all(np.abs(u.astype(np.float64) - v) <= 2e-6 * tl + 1e-7), f"{name}: the routes disagree"
    # an invalid plan poisons every result of this route too
    B.laplex_diag_set_plan_status(ws, n, 1)
    y5, _ = gpu_gram(a, x, flags=B.LAPLEX_SAVE_SCANS | B.LAPLEX_REUSE_PLAN, ws=ws)
    gx5, ga5 = gpu_gram_backward(a, x, g, flags=B.LAPLEX_SAVE_SCANS | B.LAPLEX_REUSE_PLAN, ws=ws)
    assert np.isnan(y5).all() and np.isnan(gx5).all() and np.isnan(ga5).all()


def test_routes_invalid_plan_poisons(routed):
    r = np.random.default_rng(5)
    k, n = 20000, 30000
    a, b = anchors("uniform", r, k, n)
    x = r.normal(size=(n, 1)).astype(np.float32); g = r.normal(size=(k, 1)).astype(np.float32)
    da, db, dx, dg = dev(a), dev(b), dev(x), dev(g)
    ws = workspace(k, n, 1)
    y = torch.zeros(k, 1, device="cuda"); gx = torch.zeros(n, 1, device="cuda"); ga = torch.zeros(k, device="cuda"); gb = torch.zeros(n, device="cuda")
    B.laplex_apply(da, db, dx, y, ws, B.LAPLEX_SAVE_SCANS)
    B.laplex_diag_set_plan_status(ws, k + n, 1)
    B.laplex_apply(da, db, dx, y, ws, B.LAPLEX_SAVE_SCANS | B.LAPLEX_REUSE_PLAN)
    B.laplex_apply_backward(da, db, dx, dg, gx, ga, gb, ws, B.LAPLEX_SAVE_SCANS | B.LAPLEX_REUSE_PLAN)
    torch.cuda.synchronize()
    for name, t in (("y", y), ("gx", gx), ("ga", ga), ("gb", gb)):
        assert bool(torch.isnan(t).all()), name
