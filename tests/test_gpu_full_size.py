"""Parity at the full sizes of the five workloads, in the launch configuration the
benchmark times.  Where the oracle cannot produce every output in seconds, it
produces sampled ones (brute force restricted to a window of 64 around the
sampled anchors: what is dropped is below exp(-64) * sum|x|), and the
permutation is checked through properties that pin it uniquely: it is a
permutation, keys ascend along it, and equal keys keep ascending ids.

The 2^30 workload needs ~76 GiB of HBM and 16 GiB of host arrays and takes about
half a minute on the GPU machine; LAPLEX_SMALL_BILLION=1 shrinks it to n = k = 2^27.
"""
import os
import sys
import time

import numpy as np
import pytest

from paper_2605_24584_amd import binding as B
from paper_2605_24584_amd import synth

torch = pytest.importorskip("torch")
pytestmark = pytest.mark.gpu

RTOL, ATOL = 1e-5, 1e-7


def log(msg):
    print(f"[full-size {time.strftime('%H:%M:%S')}] {msg}", file=sys.stderr, flush=True)


def dev(v):
    return torch.from_numpy(np.ascontiguousarray(v)).cuda()


def worst_ratio(got, ref, tol):
    got = np.asarray(got, dtype=np.float64).reshape(ref.shape)
    assert np.all(np.isfinite(got))
    return float((np.abs(got - ref) / (RTOL * tol + ATOL)).max())


def check_permutation_properties(perm_i32, merged_dev):
    """perm: int32 device tensor holding u32 ids; merged_dev: fp32 anchors a ++ b."""
    N = merged_dev.numel()
    ids = perm_i32.to(torch.int64) & 0xFFFFFFFF
    assert int(ids.min()) == 0 and int(ids.max()) == N - 1
    seen = torch.zeros(N, dtype=torch.bool, device="cuda")
    seen[ids] = True
    assert bool(seen.all()), "not a permutation"
    del seen
    m = merged_dev[ids]
    step_ok = (m[1:] > m[:-1]) | ((m[1:] == m[:-1]) & (ids[1:] > ids[:-1]))
    assert bool(step_ok.all()), "keys do not ascend, or equal keys lost their order"


def window_samples(a, b, centers, core=4.0, halo=64.0):
    """For each centre c: outputs with a in [c, c+core), inputs with b in the halo
    around that range, and the converse (inputs in the core, outputs in the halo)."""
    out = []
    for c in centers:
        a_core = np.nonzero((a >= c) & (a < c + core))[0]
        b_halo = np.nonzero((b >= c - halo) & (b < c + core + halo))[0]
        b_core = np.nonzero((b >= c) & (b < c + core))[0]
        a_halo = np.nonzero((a >= c - halo) & (a < c + core + halo))[0]
        out.append((a_core, b_halo, b_core, a_halo))
    return out


def check_windows(oracle, a, b, x, g, y, gx, ga, gb, centers, core=4.0):
    worst = {"y": 0.0, "gx": 0.0, "ga": 0.0, "gb": 0.0}
    checked = 0
    for a_core, b_halo, b_core, a_halo in window_samples(a, b, centers, core=core):
        if a_core.size and b_halo.size:
            ref, tol = oracle.apply_brute(a[a_core], b[b_halo], x[b_halo])
            worst["y"] = max(worst["y"], worst_ratio(y[a_core], ref, tol))
            if ga is not None:
                (_, rga, _), (_, tga, _) = oracle.apply_backward_brute(a[a_core], b[b_halo], x[b_halo], g[a_core])
                worst["ga"] = max(worst["ga"], worst_ratio(ga[a_core], rga, tga))
            checked += a_core.size
        if gx is not None and b_core.size and a_halo.size:
            (rgx, _, rgb), (tgx, _, tgb) = oracle.apply_backward_brute(a[a_halo], b[b_core], x[b_core], g[a_halo])
            worst["gx"] = max(worst["gx"], worst_ratio(gx[b_core], rgx, tgx))
            worst["gb"] = max(worst["gb"], worst_ratio(gb[b_core], rgb, tgb))
            checked += b_core.size
    return worst, checked


# ------------------------------------------------------------------ projection layer, the benchmark's workload

def test_projection_full_size_every_element(oracle):
    w = synth.projection_layer()
    a, b, x, g = w["a"], w["b"], w["x"], w["g"]
    k, n, batch = a.size, b.size, x.shape[1]
    ws = torch.empty(B.laplex_workspace_bytes(k, n, batch), dtype=torch.uint8, device="cuda")
    da, db, dx, dg = dev(a), dev(b), dev(x), dev(g)
    y = torch.empty(k, batch, device="cuda"); gx = torch.empty(n, batch, device="cuda")
    ga = torch.empty(k, device="cuda"); gb = torch.empty(n, device="cuda")
    B.laplex_apply(da, db, dx, y, ws, B.LAPLEX_SAVE_SCANS)
    B.laplex_apply_backward(da, db, dx, dg, gx, ga, gb, ws, B.LAPLEX_SAVE_SCANS | B.LAPLEX_REUSE_PLAN)
    perm = torch.empty(k + n, dtype=torch.int32, device="cuda")
    B.laplex_get_perm(ws, k + n, perm)
    status = torch.full((1,), -1, dtype=torch.int32, device="cuda")
    B.laplex_get_plan_status(ws, k + n, status)
    assert int(status.item()) == 0, "a tile of the radix sort gave up waiting for its predecessors"
    torch.cuda.synchronize()
    assert np.array_equal(perm.cpu().numpy().view(np.uint32), oracle.merged_permutation(a, b))
    y, gx, ga, gb = y.cpu().numpy(), gx.cpu().numpy(), ga.cpu().numpy(), gb.cpu().numpy()
    # every element of y, gx, ga and gb (all 256 batch columns) through the dual-theorem route
    ref, tol = oracle.apply_scan(a, b, x)
    (rgx, rga, rgb), (tgx, tga, tgb) = oracle.apply_backward_scan(a, b, x, g)
    r = {"y": worst_ratio(y, ref, tol), "gx": worst_ratio(gx, rgx, tgx),
         "ga": worst_ratio(ga, rga, tga), "gb": worst_ratio(gb, rgb, tgb)}
    # ... and the definition itself on windows of rows
    centers = [0.0, 1017.25, 4100.5, 8191.0, 12000.75, 16384.0 - 256.0]
    worst, checked = check_windows(oracle, a, b, x, g, y, gx, ga, gb, centers, core=256.0)
    log(f"projection full: worst ratios over every element {r}; windows (definition) {worst} over {checked} rows")
    assert max(r.values()) <= 1.0 and max(worst.values()) <= 1.0 and checked > 1000


# ------------------------------------------------------------------ tie-heavy square apply, n = k = 2^24

def test_tie_heavy_full_size(oracle):
    w = synth.tie_heavy()
    a, b, x, g = w["a"], w["b"], w["x"], w["g"]
    k, n = a.size, b.size
    ws = torch.empty(B.laplex_workspace_bytes(k, n, 1), dtype=torch.uint8, device="cuda")
    da, db, dx, dg = dev(a), dev(b), dev(x), dev(g)
    y = torch.empty(k, 1, device="cuda"); gx = torch.empty(n, 1, device="cuda")
    ga = torch.empty(k, device="cuda"); gb = torch.empty(n, device="cuda")
    B.laplex_apply(da, db, dx, y, ws, B.LAPLEX_SAVE_SCANS)
    B.laplex_apply_backward(da, db, dx, dg, gx, ga, gb, ws, B.LAPLEX_SAVE_SCANS | B.LAPLEX_REUSE_PLAN)
    perm = torch.empty(k + n, dtype=torch.int32, device="cuda")
    B.laplex_get_perm(ws, k + n, perm)
    status = torch.full((1,), -1, dtype=torch.int32, device="cuda")
    B.laplex_get_plan_status(ws, k + n, status)
    assert int(status.item()) == 0, "a tile of the radix sort gave up waiting for its predecessors"
    torch.cuda.synchronize()
    assert np.array_equal(perm.cpu().numpy().view(np.uint32), oracle.merged_permutation(a, b))   # bit-exact
    ref, tol = oracle.apply_scan(a, b, x)
    r_y = worst_ratio(y.cpu().numpy(), ref, tol)
    (rgx, rga, rgb), (tgx, tga, tgb) = oracle.apply_backward_scan(a, b, x, g)
    r = (r_y, worst_ratio(gx.cpu().numpy(), rgx, tgx), worst_ratio(ga.cpu().numpy(), rga, tga),
         worst_ratio(gb.cpu().numpy(), rgb, tgb))
    log(f"tie-heavy 2^24: worst ratios y, gx, ga, gb = {r}")
    assert max(r) <= 1.0


# ------------------------------------------------------------------ Gram form on n = 3 * 2^20, batch 64

def test_gram_images_full_size(oracle):
    w = synth.gram_images()
    a, x, g = w["a"], w["x"], w["g"]
    n, batch = a.size, x.shape[1]
    ws = torch.empty(B.laplex_workspace_bytes(0, n, batch), dtype=torch.uint8, device="cuda")
    da, dx, dg = dev(a), dev(x), dev(g)
    y = torch.empty(n, batch, device="cuda"); gx = torch.empty(n, batch, device="cuda"); ga = torch.empty(n, device="cuda")
    B.laplex_gram(da, dx, y, ws, B.LAPLEX_SAVE_SCANS)
    B.laplex_gram_backward(da, dx, dg, gx, ga, ws, B.LAPLEX_SAVE_SCANS | B.LAPLEX_REUSE_PLAN)
    perm = torch.empty(n, dtype=torch.int32, device="cuda")
    B.laplex_get_perm(ws, n, perm)
    status = torch.full((1,), -1, dtype=torch.int32, device="cuda")
    B.laplex_get_plan_status(ws, n, status)
    assert int(status.item()) == 0, "a tile of the radix sort gave up waiting for its predecessors"
    torch.cuda.synchronize()
    assert np.array_equal(perm.cpu().numpy().view(np.uint32), oracle.merged_permutation(a))
    ref, tol = oracle.gram_scan(a, x)    # every row, all 64 columns
    r_y = worst_ratio(y.cpu().numpy(), ref, tol)
    del ref, tol
    refg, tolg = oracle.gram_scan(a, g)
    r_gx = worst_ratio(gx.cpu().numpy(), refg, tolg)
    del refg, tolg
    (_, rga), (_, tga) = oracle.gram_backward_scan(a, x, g)      # ga sums over all 64 columns
    r_ga = worst_ratio(ga.cpu().numpy(), rga, tga)
    dup = n - np.unique(a).size
    log(f"gram 3*2^20 x 64: worst ratios y, gx, ga = {(r_y, r_gx, r_ga)}; {dup} duplicated anchors")
    assert max(r_y, r_gx, r_ga) <= 1.0


# ------------------------------------------------------------------ billion-scale square apply

def test_billion_scale(oracle):
    full = os.environ.get("LAPLEX_SMALL_BILLION") != "1"
    scale = 1 if full else 8
    log(f"billion workload at n = k = 2^{30 - (0 if full else 3)}: generating inputs")
    w = synth.billion_square(scale=scale)
    a, b, x, g = w["a"], w["b"], w["x"], w["g"]
    k, n = a.size, b.size
    ws_bytes = B.laplex_workspace_bytes(k, n, 1)
    log(f"workspace {ws_bytes / 2**30:.1f} GiB; uploading")
    ws = torch.empty(ws_bytes, dtype=torch.uint8, device="cuda")
    da, db, dx, dg = dev(a), dev(b), dev(x), dev(g)
    y = torch.empty(k, 1, device="cuda"); gx = torch.empty(n, 1, device="cuda")
    ga = torch.empty(k, device="cuda"); gb = torch.empty(n, device="cuda")
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    B.laplex_apply(da, db, dx, y, ws, B.LAPLEX_SAVE_SCANS)
    torch.cuda.synchronize()
    t1 = time.perf_counter()
    B.laplex_apply_backward(da, db, dx, dg, gx, ga, gb, ws, B.LAPLEX_SAVE_SCANS | B.LAPLEX_REUSE_PLAN)
    torch.cuda.synchronize()
    t2 = time.perf_counter()
    peak = torch.cuda.max_memory_allocated()
    log(f"forward {1e3 * (t1 - t0):.1f} ms (sort included), backward {1e3 * (t2 - t1):.1f} ms, "
        f"device footprint {peak / 2**30:.1f} GiB")
    perm = torch.empty(k + n, dtype=torch.int32, device="cuda")
    B.laplex_get_perm(ws, k + n, perm)
    status = torch.full((1,), -1, dtype=torch.int32, device="cuda")
    B.laplex_get_plan_status(ws, k + n, status)
    assert int(status.item()) == 0, "a tile of the radix sort gave up waiting for its predecessors"
    torch.cuda.synchronize()
    del ws
    check_permutation_properties(perm, torch.cat([da, db]))
    log("permutation properties hold")
    N = k + n
    # sorted copies of (b, x) and (a, g) for the windowed route, gathered on the device along the verified permutation
    # (the oracle sorts for itself; inputs that arrive sorted only make its sort quick)
    def sorted_side(lo, hi, anchors_dev, values_dev):
        out_a, out_v = [], []
        step = 1 << 27
        for c0 in range(0, N, step):
            p = perm[c0:c0 + step].to(torch.int64) & 0xFFFFFFFF
            sel = p[(p >= lo) & (p < hi)] - lo
            out_a.append(anchors_dev[sel].cpu()); out_v.append(values_dev.view(-1)[sel].cpu())
        return torch.cat(out_a).numpy(), torch.cat(out_v).numpy()
    bs, xs = sorted_side(k, N, db, dx)
    as_, gs = sorted_side(0, k, da, dg)
    y, gx, ga, gb = y.cpu().numpy(), gx.cpu().numpy(), ga.cpu().numpy(), gb.cpu().numpy()

    # (1) rows on both sides of the boundaries of the launch geometry, taken from the plan itself: at batch 1 a scan
    # block is 8192 rows, a chunk of the two-level spine 4096 blocks = 2^25 rows (a chunk carry matters only within
    # ~100 units of anchor distance of a chunk boundary), a sort tile 8192 pairs.  Every chunk boundary, and block
    # boundaries spread over the sequence, 192 rows on either side, against the definition over a halo of >= 64 units.
    block, chunk, core, halo = 8192, 1 << 25, 192, 12288
    bounds = [m * chunk for m in range(1, (N + chunk - 1) // chunk)]
    rb = np.random.default_rng(30)
    bounds += [int(m) * block for m in rb.integers(1, N // block, 24)] + [block, N - block, core, N - core]
    worst = {"y": 0.0, "gx": 0.0, "ga": 0.0, "gb": 0.0}
    checked = 0
    for j0 in bounds:
        lo, hi = max(0, j0 - core - halo), min(N, j0 + core + halo)
        ids = (perm[lo:hi].cpu().numpy().view(np.uint32)).astype(np.int64)
        pos = np.arange(lo, hi)
        in_core = (pos >= j0 - core) & (pos < j0 + core)
        is_out = ids < k
        anchor = np.where(is_out, a[np.minimum(ids, k - 1)], b[np.maximum(ids - k, 0)]).astype(np.float64)
        c_lo, c_hi = anchor[in_core].min(), anchor[in_core].max()
        # the halo reaches 64 units beyond the core on both sides, or the end of the sequence
        assert lo == 0 or anchor[0] <= c_lo - 64.0, "halo too short on the left"
        assert hi == N or anchor[-1] >= c_hi + 64.0, "halo too short on the right"
        a_core, b_halo = ids[in_core & is_out], ids[~is_out] - k
        b_core, a_halo = ids[in_core & ~is_out] - k, ids[is_out]
        ref, tol = oracle.apply_brute(a[a_core], b[b_halo], x[b_halo])
        worst["y"] = max(worst["y"], worst_ratio(y[a_core], ref, tol))
        (_, rga, _), (_, tga, _) = oracle.apply_backward_brute(a[a_core], b[b_halo], x[b_halo], g[a_core])
        worst["ga"] = max(worst["ga"], worst_ratio(ga[a_core], rga, tga))
        (rgx, _, rgb), (tgx, _, tgb) = oracle.apply_backward_brute(a[a_halo], b[b_core], x[b_core], g[a_halo])
        worst["gx"] = max(worst["gx"], worst_ratio(gx[b_core], rgx, tgx))
        worst["gb"] = max(worst["gb"], worst_ratio(gb[b_core], rgb, tgb))
        checked += a_core.size + b_core.size
    log(f"billion workload: {len(bounds)} chunk / block boundaries from the plan: ratios {worst} over {checked} rows")
    assert max(worst.values()) <= 1.0 and checked >= 2 * core * len(bounds) - 4 * core
    del perm

    # (2) windows at fixed anchor values: both ends, the dense-fraction region, where fp32 spacing is 0.5 / 1.0 (many exact ties)
    hi_a = float(1 << 24) / scale
    centers = [0.0, 3.5, hi_a / 1024, hi_a / 16 + 0.25, hi_a / 4, hi_a / 2 + 1.0, 0.75 * hi_a, hi_a - 70.0, hi_a - 4.0]
    worst, checked = check_windows(oracle, a, b, x, g, y, gx, ga, gb, centers)
    log(f"billion workload: window ratios {worst} over {checked} rows")
    assert max(worst.values()) <= 1.0 and checked > 2000

    # (3) 2^20 seeded random outputs and 2^20 random inputs through the windowed definition (|a - b| <= 64; what is
    # dropped is below exp(-64) sum|x|)
    rs = np.random.default_rng(31)
    pick = np.sort(rs.choice(k, 1 << 20, replace=False))
    log("windowed definition on 2^20 random outputs")
    ref, tol = oracle.apply_window(a[pick], bs, xs)
    r_y = worst_ratio(y[pick, 0], ref, tol)
    del bs, xs
    pick = np.sort(rs.choice(n, 1 << 20, replace=False))
    log("windowed definition on 2^20 random inputs (gx through the transposed operator)")
    ref, tol = oracle.apply_window(b[pick], as_, gs)
    r_gx = worst_ratio(gx[pick, 0], ref, tol)
    log(f"billion workload: random samples: y ratio {r_y:.3g}, gx ratio {r_gx:.3g}")
    assert r_y <= 1.0 and r_gx <= 1.0


def test_two_level_spine_every_output(oracle):
    """Batch 1 with more than 2^25 merged positions: the tile summaries no longer fit one chunk of the spine, so its
    upper level runs (at the benchmark's size it always does; here on a size where the oracle's scan route can produce
    EVERY output: n = k = 2^25, the billion workload's recipe with the same density and ties).  Always run."""
    w = synth.billion_square(scale=32)
    a, b, x, g = w["a"], w["b"], w["x"], w["g"]
    k, n = a.size, b.size
    assert k + n > (1 << 25)
    ws = torch.empty(B.laplex_workspace_bytes(k, n, 1), dtype=torch.uint8, device="cuda")
    da, db, dx, dg = dev(a), dev(b), dev(x), dev(g)
    y = torch.empty(k, 1, device="cuda"); gx = torch.empty(n, 1, device="cuda")
    ga = torch.empty(k, device="cuda"); gb = torch.empty(n, device="cuda")
    B.laplex_apply(da, db, dx, y, ws, B.LAPLEX_SAVE_SCANS)
    B.laplex_apply_backward(da, db, dx, dg, gx, ga, gb, ws, B.LAPLEX_SAVE_SCANS | B.LAPLEX_REUSE_PLAN)
    perm = torch.empty(k + n, dtype=torch.int32, device="cuda")
    B.laplex_get_perm(ws, k + n, perm)
    torch.cuda.synchronize()
    log("two-level spine, n = k = 2^25: permutation")
    assert np.array_equal(perm.cpu().numpy().view(np.uint32), oracle.merged_permutation(a, b))   # bit-exact
    del ws, perm
    log("forward through the scan route")
    ref, tol = oracle.apply_scan(a, b, x)
    r_y = worst_ratio(y.cpu().numpy(), ref, tol)
    log(f"y ratio {r_y:.3g}; backward through the scan route")
    (rgx, rga, rgb), (tgx, tga, tgb) = oracle.apply_backward_scan(a, b, x, g)
    r = (r_y, worst_ratio(gx.cpu().numpy(), rgx, tgx), worst_ratio(ga.cpu().numpy(), rga, tga),
         worst_ratio(gb.cpu().numpy(), rgb, tgb))
    log(f"two-level spine, n = k = 2^25, every output: worst ratios y, gx, ga, gb = {r}")
    assert max(r) <= 1.0


def test_two_level_spine_dense_anchors_every_output(oracle):
    """The same size with all anchors inside 24 units (and many exact ties): no decay is ever small, so every
    carry, the chunks' included, reaches every output.  Forward, every output against the scan route."""
    k = n = 1 << 25
    a = synth.uniform(synth.stream_seed(21, synth.STREAM_A), k, 0.0, 24.0)
    b = synth.uniform(synth.stream_seed(21, synth.STREAM_B), n, 0.0, 24.0)
    x = synth.normal(synth.stream_seed(21, synth.STREAM_X), n).reshape(n, 1)
    ws = torch.empty(B.laplex_workspace_bytes(k, n, 1), dtype=torch.uint8, device="cuda")
    y = torch.empty(k, 1, device="cuda")
    B.laplex_apply(dev(a), dev(b), dev(x), y, ws, 0)
    torch.cuda.synchronize()
    del ws
    log("dense anchors, n = k = 2^25: forward through the scan route")
    ref, tol = oracle.apply_scan(a, b, x)
    r_y = worst_ratio(y.cpu().numpy(), ref, tol)
    log(f"dense anchors, n = k = 2^25: y ratio {r_y:.3g}")
    assert r_y <= 1.0


def test_weighted_gram_full_size(oracle):
    """k = 1024 Gram anchors, n = 2^20 middle anchors, positive weights: every entry of the
    1024 x 1024 matrix against the oracle's decomposition route, and a sample of 24 rows against
    the definition itself."""
    w = synth.weighted_gram()
    a, b, d = w["a"], w["b"], w["d"]
    k, n = a.size, b.size
    ws = torch.empty(B.laplex_wgram_workspace_bytes(k, n), dtype=torch.uint8, device="cuda")
    m = torch.full((k, k), float("nan"), device="cuda")
    log(f"weighted Gram: k={k} n={n}, workspace {ws.numel() / 2**20:.0f} MiB")
    B.laplex_wgram(dev(a), dev(b), dev(d), m, ws, 0)
    torch.cuda.synchronize()
    got = m.cpu().numpy()
    ref, tol = oracle.wgram_scan(a, b, d)
    worst = worst_ratio(got, ref, tol)
    log(f"weighted Gram: worst |err| / (1e-5 T + 1e-7) = {worst:.3g} over {k * k} entries")
    assert worst <= 1.0
    # sampled rows against the definition, restricted to the middle anchors within 64 of the row's
    # anchor (what is dropped is below exp(-64) * sum|d|)
    a64, b64, d64 = a.astype(np.float64), b.astype(np.float64), d.astype(np.float64)
    for i in np.random.default_rng(8).choice(k, 24, replace=False):
        near = np.abs(b64 - a64[i]) <= 64.0
        col = d64[near] * np.exp(-np.abs(a64[i] - b64[near]))
        A = np.exp(-np.abs(a64[:, None] - b64[near][None, :]))
        assert worst_ratio(got[i], A @ col, A @ np.abs(col)) <= 1.0


# ------------------------------------------------------------------ the widened entry points at their benchmark sizes

def test_phased_projection_full_size_sampled(oracle):
    """The phased kernel on the projection layer's shape (n = 2^20, k = 1024, batch 256, phases ~ U(-pi, pi)):
    every output of 16 sampled batch columns through the angle-sum route of the oracle, and all five gradients
    on windows of rows against the definition differentiated entry by entry."""
    w = synth.projection_layer_phased()
    a, b, x, g, phi, psi = w["a"], w["b"], w["x"], w["g"], w["phi"], w["psi"]
    k, n, batch = a.size, b.size, x.shape[1]
    ws = torch.empty(B.laplex_phased_workspace_bytes(k, n, batch), dtype=torch.uint8, device="cuda")
    log(f"phased projection: workspace {ws.numel() / 2**30:.2f} GiB")
    da, db, dphi, dpsi, dx, dg = dev(a), dev(b), dev(phi), dev(psi), dev(x), dev(g)
    y = torch.empty(k, batch, device="cuda"); gx = torch.empty(n, batch, device="cuda")
    ga = torch.empty(k, device="cuda"); gb = torch.empty(n, device="cuda")
    gphi = torch.empty(k, device="cuda"); gpsi = torch.empty(n, device="cuda")
    B.laplex_phased_apply(da, dphi, db, dpsi, dx, y, ws, B.LAPLEX_SAVE_SCANS)
    B.laplex_phased_apply_backward(da, dphi, db, dpsi, dx, dg, gx, ga, gb, gphi, gpsi, ws,
                                   B.LAPLEX_SAVE_SCANS | B.LAPLEX_REUSE_PLAN)
    torch.cuda.synchronize()
    y, gx, ga, gb, gphi, gpsi = (t.cpu().numpy() for t in (y, gx, ga, gb, gphi, gpsi))
    del ws
    cols = np.arange(0, batch, 16)
    ref, tol = oracle.phased_apply_scan(a, phi, b, psi, x[:, cols])
    r_y = worst_ratio(y[:, cols], ref, tol)
    worst = {"y": 0.0, "gx": 0.0, "ga": 0.0, "gb": 0.0, "gphi": 0.0, "gpsi": 0.0}
    checked = 0
    centers = [0.0, 1017.25, 4100.5, 8191.0, 12000.75, 16384.0 - 256.0]
    for a_core, b_halo, b_core, a_halo in window_samples(a, b, centers, core=256.0):
        if a_core.size and b_halo.size:       # outputs in the core see every input that matters
            ry, ty = oracle.phased_apply_brute(a[a_core], phi[a_core], b[b_halo], psi[b_halo], x[b_halo])
            worst["y"] = max(worst["y"], worst_ratio(y[a_core], ry, ty))
            (_, rga, _, rgphi, _), (_, tga, _, tgphi, _) = oracle.phased_backward_brute(
                a[a_core], phi[a_core], b[b_halo], psi[b_halo], x[b_halo], g[a_core])
            worst["ga"] = max(worst["ga"], worst_ratio(ga[a_core], rga, tga))
            worst["gphi"] = max(worst["gphi"], worst_ratio(gphi[a_core], rgphi, tgphi))
            checked += a_core.size
        if b_core.size and a_halo.size:       # inputs in the core see every output that matters
            (rgx, _, rgb, _, rgpsi), (tgx, _, tgb, _, tgpsi) = oracle.phased_backward_brute(
                a[a_halo], phi[a_halo], b[b_core], psi[b_core], x[b_core], g[a_halo])
            worst["gx"] = max(worst["gx"], worst_ratio(gx[b_core], rgx, tgx))
            worst["gb"] = max(worst["gb"], worst_ratio(gb[b_core], rgb, tgb))
            worst["gpsi"] = max(worst["gpsi"], worst_ratio(gpsi[b_core], rgpsi, tgpsi))
            checked += b_core.size
    log(f"phased projection: y ratio {r_y:.3g} (16 columns, all outputs); windows {worst} over {checked} rows")
    assert r_y <= 1.0 and max(worst.values()) <= 1.0 and checked > 1000


def test_mix_head_full_size(oracle):
    """LAPLEX^(16) head of 1000 x 2048 at batch 256 (all operators in each launch): every output and every
    gradient against the sum written out operator by operator with the dense definition."""
    w = synth.mix_head()
    a, b, wq, x, g = w["a"], w["b"], w["w"], w["x"], w["g"]
    r, k, n, batch = w["r"], w["k"], w["n"], w["batch"]
    ws = torch.empty(B.laplex_mix_workspace_bytes(r, k, n, batch), dtype=torch.uint8, device="cuda")
    da, db, dw, dx, dg = dev(a), dev(b), dev(wq), dev(x), dev(g)
    y = torch.empty(k, batch, device="cuda"); gx = torch.empty(n, batch, device="cuda")
    ga = torch.empty(r, k, device="cuda"); gb = torch.empty(r, n, device="cuda"); gw = torch.empty(r, device="cuda")
    B.laplex_mix_apply(da, db, dw, dx, y, ws, B.LAPLEX_SAVE_SCANS)
    B.laplex_mix_apply_backward(da, db, dw, dx, dg, gx, ga, gb, gw, ws, B.LAPLEX_SAVE_SCANS | B.LAPLEX_REUSE_PLAN)
    torch.cuda.synchronize()
    ref, tol = oracle.mix_apply(a, b, wq, x)
    (rgx, rga, rgb, rgw), (tgx, tga, tgb, tgw) = oracle.mix_backward(a, b, wq, x, g)
    ratios = {"y": worst_ratio(y.cpu().numpy(), ref, tol), "gx": worst_ratio(gx.cpu().numpy(), rgx, tgx),
              "ga": worst_ratio(ga.cpu().numpy(), rga, tga), "gb": worst_ratio(gb.cpu().numpy(), rgb, tgb),
              "gw": worst_ratio(gw.cpu().numpy(), rgw, tgw)}
    log(f"mix head r={r} k={k} n={n} batch={batch}: worst ratios {ratios}")
    assert max(ratios.values()) <= 1.0


def test_temperature_projection_full_size_sampled(oracle):
    """The temperature-scaled kernel exp(-tau |a_i - b_j|) on the projection layer's shape, tau = 0.37: every output
    of 16 sampled batch columns, gradients on windows (in the scaled anchors tau a, tau b, where the kernel is the
    plain one), and gtau against its chain-rule identity with the anchor gradients."""
    tau = 0.37
    w = synth.projection_layer()
    a, b, x, g = w["a"], w["b"], w["x"], w["g"]
    k, n, batch = a.size, b.size, x.shape[1]
    ws = torch.empty(B.laplex_workspace_bytes(k, n, batch), dtype=torch.uint8, device="cuda")
    da, db, dx, dg = dev(a), dev(b), dev(x), dev(g)
    y = torch.empty(k, batch, device="cuda"); gx = torch.empty(n, batch, device="cuda")
    ga = torch.empty(k, device="cuda"); gb = torch.empty(n, device="cuda"); gtau = torch.empty(1, device="cuda")
    B.laplex_apply_tau(da, db, tau, dx, y, ws, B.LAPLEX_SAVE_SCANS)
    B.laplex_apply_backward_tau(da, db, tau, dx, dg, gx, ga, gb, gtau, ws, B.LAPLEX_SAVE_SCANS | B.LAPLEX_REUSE_PLAN)
    torch.cuda.synchronize()
    y, gx, ga, gb, gtau = y.cpu().numpy(), gx.cpu().numpy(), ga.cpu().numpy(), gb.cpu().numpy(), float(gtau.item())
    sa, sb = oracle.scaled_anchors(a, tau), oracle.scaled_anchors(b, tau)
    cols = np.arange(0, batch, 16)
    ref, tol = oracle.apply_scan(sa, sb, x[:, cols])
    r_y = worst_ratio(y[:, cols], ref, tol)
    # windows in the scaled anchors; the anchor gradients of the scaled problem are ga / tau, gb / tau
    centers = [tau * c for c in (0.0, 1017.25, 4100.5, 8191.0, 12000.75, 16384.0 - 700.0)]
    worst, checked = check_windows(oracle, sa, sb, x, g, y, gx, ga / tau, gb / tau, centers, core=tau * 256.0)
    # gtau = sum_i a_i ga'_i + sum_j b_j gb'_j with the scaled problem's gradients ga' = ga / tau
    a64, b64 = a.astype(np.float64), b.astype(np.float64)
    want = (np.dot(a64, ga.astype(np.float64)) + np.dot(b64, gb.astype(np.float64))) / tau
    scale = (np.dot(np.abs(a64), np.abs(ga)) + np.dot(np.abs(b64), np.abs(gb))) / tau
    log(f"temperature {tau}: y ratio {r_y:.3g}; windows {worst} over {checked} rows; gtau {gtau:.6g} vs {want:.6g}")
    assert r_y <= 1.0 and max(worst.values()) <= 1.0 and checked > 1000
    assert abs(gtau - want) <= 1e-5 * scale + 1e-7
