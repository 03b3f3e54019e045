#!/usr/bin/env python3
"""Benchmark of the LAPLEX hot path on one MI355X.

One step = one pass of the whole path over one batch of synthetic input:
    laplex_apply          (key build, radix sort, decay, forward + backward scan, scatter)
    laplex_apply_backward (gx, ga, gb; plan and saved scans of the forward reused)
Default workload: the billion-scale square apply (n = k = 2^30, batch 1, fp32), the largest
configuration that fits one GPU; inputs are resident in HBM before the timed region.

Prints ONE JSON line: throughput in (n + k) * batch elements per second, the roofline of the
step's dominant kernel family (found by timing every family for one step, then timed with HIP
events on its own stream during the timed steps), the device footprint, and the CPU oracle
timed beside it on a bounded sub-problem of the same recipe.  The projection layer
(n = 2^20, k = 1024, batch 256) and the Gram form (n = 3 * 2^20, batch 64) ride along as
extra objects of the same line, each with its own roofline.
"""
import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0


def parse():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=50)
    ap.add_argument("--warmup", type=int, default=10)
    ap.add_argument("--scale", type=int, default=1, help="shrink n and k by this factor (debug only)")
    ap.add_argument("--batch", type=int, default=256)
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--cpu-sample-columns", type=int, default=256)
    ap.add_argument("--steps-extra", type=int, default=20, help="timed steps of the extra workloads")
    ap.add_argument("--workload", default="billion",
                    choices=["billion", "projection", "gram", "tie_heavy", "square", "phased", "wgram", "wgram64", "mix", "square_b8"],
                    help="billion is the benchmark (with projection and gram as extra objects); projection, gram and "
                         "tie_heavy alone print the same kind of line for that workload; the others time one "
                         "forward+backward step (for profiles; no roofline object, no CPU baseline)")
    ap.add_argument("--no-extra", action="store_true", help="billion only: skip the projection and Gram objects")
    ap.add_argument("--paper-sweep", action="store_true",
                    help="instead of the benchmark: the paper's runtime sweep (App. 'GPU runtime'): square apply "
                         "n = k = 2^10 .. 2^20 at batch 8, forward and forward + backward, one JSON line per size")
    ap.add_argument("--calibrate-copy", action="store_true",
                    help="instead of the benchmark: time a plain device copy of 1 GiB (counter calibration)")
    return ap.parse_args()


def sparse_bwd_bytes(a, b, batch, block_rows, blocks_per_tile=8, few=4):
    """Algorithmic bytes of one launch of the dominant kernel, the streaming backward
    downsweep (one wavefront per block of `block_rows` sorted rows).  It visits the
    blocks that hold at most `few` output anchors (blocks with more go to the generic
    downsweep).  Per visited input row: sorted id, two decays' worth of metadata and
    the sorted anchor (12 B), the x row read and the gx row written (4 B per batch
    column each), gb written (4 B).  Per tile of `blocks_per_tile` blocks: the four
    carry rows of the tile (forward/backward, inclusive/strict: 16 B per batch
    column); per visited block of a tile that holds output anchors: the four rows of
    the state the block starts from inside its tile (16 B per batch column) and, per
    output anchor in the block, its gy row (4 B per batch column).
    Returns (bytes, visited rows, visited blocks, all blocks)."""
    import numpy as np
    k = a.size
    order = np.argsort(np.concatenate([a, b]), kind="stable")
    N = order.size
    blocks = (N + block_rows - 1) // block_rows
    outputs = np.bincount(np.nonzero(order < k)[0] // block_rows, minlength=blocks)
    rows_per_block = np.full(blocks, block_rows, dtype=np.int64)
    rows_per_block[-1] = N - (blocks - 1) * block_rows
    visited = outputs <= few
    rows = int((rows_per_block - outputs)[visited].sum())
    tiles = (blocks + blocks_per_tile - 1) // blocks_per_tile
    pad = tiles * blocks_per_tile - blocks
    tile_outputs = np.concatenate([outputs, np.zeros(pad, dtype=outputs.dtype)]).reshape(tiles, blocks_per_tile).sum(axis=1)
    tile_visited = np.concatenate([visited, np.zeros(pad, dtype=bool)]).reshape(tiles, blocks_per_tile).any(axis=1)
    in_output_tile = np.repeat(tile_outputs > 0, blocks_per_tile)[:blocks]
    total = (rows * (12 + 8 * batch + 4)
             + int(tile_visited.sum()) * 16 * batch
             + int((visited & in_output_tile).sum()) * 16 * batch
             + int(outputs[visited].sum()) * 4 * batch)
    return total, rows, int(visited.sum()), int(blocks)


def other_workload(args, torch, np, B, synth):
    """One forward + backward step of a workload other than the benchmark's, timed the same way."""
    dev = lambda v: torch.from_numpy(np.ascontiguousarray(v)).cuda()
    if args.workload == "gram":
        w = synth.gram_images(scale=args.scale)
        a, x, g = w["a"], w["x"], w["g"]
        n, batch = a.size, x.shape[1]
        k = 0
        ws = torch.empty(B.laplex_workspace_bytes(0, n, batch), dtype=torch.uint8, device="cuda")
        da, dx, dg = dev(a), dev(x), dev(g)
        y = torch.empty(n, batch, device="cuda"); gx = torch.empty(n, batch, device="cuda"); ga = torch.empty(n, device="cuda")

        def step():
            B.laplex_gram(da, dx, y, ws, B.LAPLEX_SAVE_SCANS)
            B.laplex_gram_backward(da, dx, dg, gx, ga, ws, B.LAPLEX_SAVE_SCANS | B.LAPLEX_REUSE_PLAN)
        elements = n * batch
    elif args.workload == "wgram":
        w = synth.weighted_gram(scale=args.scale)
        a, b, d = w["a"], w["b"], w["d"]
        k, n, batch = a.size, b.size, 1
        ws = torch.empty(B.laplex_wgram_workspace_bytes(k, n), dtype=torch.uint8, device="cuda")
        da, db, dd = dev(a), dev(b), dev(d)
        m = torch.empty(k, k, device="cuda")

        def step():
            B.laplex_wgram(da, db, dd, m, ws, 0)
        elements = n + k
    elif args.workload == "wgram64":
        w = synth.weighted_gram(scale=args.scale)
        a, b, d = w["a"], w["b"], w["d"].astype(np.float64)
        k, n, batch = a.size, b.size, 1
        ws = torch.empty(B.laplex_wgram_f64_workspace_bytes(k, n), dtype=torch.uint8, device="cuda")
        da, db, dd = dev(a), dev(b), dev(d)
        m = torch.empty(k, k, dtype=torch.float64, device="cuda")

        def step():
            B.laplex_wgram_f64(da, db, dd, m, ws, 0)
        elements = n + k
    elif args.workload == "mix":
        w = synth.mix_head(scale=args.scale)
        a, b, x, g = w["a"], w["b"], w["x"], w["g"]
        r, k, n, batch = w["r"], w["k"], w["n"], w["batch"]
        ws = torch.empty(B.laplex_mix_workspace_bytes(r, k, n, batch), dtype=torch.uint8, device="cuda")
        da, db, dw, dx, dg = dev(a), dev(b), dev(w["w"]), dev(x), dev(g)
        y = torch.empty(k, batch, device="cuda"); gx = torch.empty(n, batch, device="cuda")
        ga = torch.empty(r, k, device="cuda"); gb = torch.empty(r, n, device="cuda"); gw = torch.empty(r, device="cuda")

        def step():
            B.laplex_mix_apply(da, db, dw, dx, y, ws, B.LAPLEX_SAVE_SCANS)
            B.laplex_mix_apply_backward(da, db, dw, dx, dg, gx, ga, gb, gw, ws, B.LAPLEX_SAVE_SCANS | B.LAPLEX_REUSE_PLAN)
        elements = r * (n + k) * batch
    elif args.workload == "phased":
        w = synth.projection_layer_phased(scale=args.scale, batch=args.batch)
        a, b, x, g = w["a"], w["b"], w["x"], w["g"]
        k, n, batch = a.size, b.size, x.shape[1]
        ws = torch.empty(B.laplex_phased_workspace_bytes(k, n, batch), dtype=torch.uint8, device="cuda")
        da, db, dphi, dpsi, dx, dg = dev(a), dev(b), dev(w["phi"]), dev(w["psi"]), dev(x), dev(g)
        y = torch.empty(k, batch, device="cuda"); gx = torch.empty(n, batch, device="cuda")
        ga = torch.empty(k, device="cuda"); gb = torch.empty(n, device="cuda")
        gphi = torch.empty(k, device="cuda"); gpsi = torch.empty(n, device="cuda")

        def step():
            B.laplex_phased_apply(da, dphi, db, dpsi, dx, y, ws, B.LAPLEX_SAVE_SCANS)
            B.laplex_phased_apply_backward(da, dphi, db, dpsi, dx, dg, gx, ga, gb, gphi, gpsi, ws,
                                           B.LAPLEX_SAVE_SCANS | B.LAPLEX_REUSE_PLAN)
        elements = (n + k) * batch
    else:
        make = {"square": synth.square_small, "tie_heavy": synth.tie_heavy, "billion": synth.billion_square,
                "square_b8": lambda scale: synth.paper_square(20)}[args.workload]
        w = make(scale=args.scale)
        a, b, x = w["a"], w["b"], w["x"]
        g = w.get("g", np.ones((a.size, 1), dtype=np.float32))
        k, n, batch = a.size, b.size, x.shape[1]
        ws = torch.empty(B.laplex_workspace_bytes(k, n, batch), dtype=torch.uint8, device="cuda")
        da, db, dx, dg = dev(a), dev(b), dev(x), dev(g)
        y = torch.empty(k, batch, device="cuda"); gx = torch.empty(n, batch, device="cuda")
        ga = torch.empty(k, device="cuda"); gb = torch.empty(n, device="cuda")

        def step():
            B.laplex_apply(da, db, dx, y, ws, B.LAPLEX_SAVE_SCANS)
            B.laplex_apply_backward(da, db, dx, dg, gx, ga, gb, ws, B.LAPLEX_SAVE_SCANS | B.LAPLEX_REUSE_PLAN)
        elements = (n + k) * batch
    for _ in range(args.warmup):
        step()
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(args.steps):
        step()
    torch.cuda.synchronize()
    ms = (time.perf_counter() - t0) * 1e3 / args.steps
    # an invalid plan (a sort tile that gave up its wait) turns every result into NaN: none may be here
    results = locals()
    for name in ("y", "gx", "ga", "gb", "gw", "gphi", "gpsi", "m"):
        t = results.get(name)
        if t is not None:
            assert bool(torch.isfinite(t.reshape(-1)[:65536]).all()), f"{name} holds non-finite values (invalid plan?)"
    print(json.dumps({
        "metric": "LAPLEX fwd+bwd (n+k)*batch elements/s", "value": elements / (ms * 1e-3), "unit": "elements/s",
        "n_gpus": 1, "steps": args.steps, "warmup": args.warmup, "ms_per_step": round(ms, 4),
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "f64" if args.workload == "wgram64" else "f32", "data": "synthetic",
        "config": {"workload": w["name"] + ("_fp64" if args.workload == "wgram64" else "") + ("" if args.scale == 1 else "/scaled"), "k": k, "n": n, "batch": batch,
                   "pass": ("weighted Gram matrix (k x k), sort inside every step" if args.workload.startswith("wgram")
                            else "forward+backward, sort inside every step"), "workspace_bytes": ws.numel(),
                   "device_bytes_peak": torch.cuda.max_memory_allocated()},
    }), flush=True)


def paper_sweep(args, torch, np, B, synth):
    """The paper's runtime experiments on synthetic inputs of the same shapes.
    Square apply n = k = 2^10 .. 2^20, batch 8 (the sizes of the paper's runtime figure; inputs:
    synth.paper_square).  Timing as in the paper's protocol: warm-ups, then the best of 3 x 30 calls, sort inside every call."""
    dev = lambda v: torch.from_numpy(np.ascontiguousarray(v)).cuda()
    for e in range(10, 21):
        w = synth.paper_square(e)
        a, b, x, g = w["a"], w["b"], w["x"], w["g"]
        k, n, batch = w["k"], w["n"], w["batch"]
        ws = torch.empty(B.laplex_workspace_bytes(k, n, batch), dtype=torch.uint8, device="cuda")
        da, db, dx, dg = dev(a), dev(b), dev(x), dev(g)
        y = torch.empty(k, batch, device="cuda"); gx = torch.empty(n, batch, device="cuda")
        ga = torch.empty(k, device="cuda"); gb = torch.empty(n, device="cuda")

        def fwd():
            B.laplex_apply(da, db, dx, y, ws, 0)

        def both():
            B.laplex_apply(da, db, dx, y, ws, B.LAPLEX_SAVE_SCANS)
            B.laplex_apply_backward(da, db, dx, dg, gx, ga, gb, ws, B.LAPLEX_SAVE_SCANS | B.LAPLEX_REUSE_PLAN)

        out = {"n": n, "k": k, "batch": batch}
        for name, fn in (("forward_ms", fwd), ("forward_backward_ms", both)):
            for _ in range(10):
                fn()
            best = float("inf")
            for _ in range(3):
                torch.cuda.synchronize()
                t0 = time.perf_counter()
                for _ in range(30):
                    fn()
                torch.cuda.synchronize()
                best = min(best, (time.perf_counter() - t0) * 1e3 / 30)
            out[name] = round(best, 4)
        out["elements_per_s_fwd_bwd"] = (n + k) * batch / (out["forward_backward_ms"] * 1e-3)
        print(json.dumps(out), flush=True)

    def timed(fn):
        for _ in range(10):
            fn()
        best = float("inf")
        for _ in range(3):
            torch.cuda.synchronize()
            t0 = time.perf_counter()
            for _ in range(30):
                fn()
            torch.cuda.synchronize()
            best = min(best, (time.perf_counter() - t0) * 1e3 / 30)
        return round(best, 4)

    def forward_ms(a, b, x):
        k, n, batch = a.size, b.size, x.shape[1]
        ws = torch.empty(B.laplex_workspace_bytes(k, n, batch), dtype=torch.uint8, device="cuda")
        da, db, dx = dev(a), dev(b), dev(x)
        y = torch.empty(k, batch, device="cuda")
        return timed(lambda: B.laplex_apply(da, db, dx, y, ws, 0))

    # App. "Asymmetric kernels: fixed short axis": one axis 1024, the other 2^10 .. 2^20, batch 8
    for e in range(10, 21, 2):
        n = 1 << e
        a = synth.uniform(synth.stream_seed(11, synth.STREAM_A) + e, 1024, 0.0, n / 64.0)
        b = synth.uniform(synth.stream_seed(11, synth.STREAM_B) + e, n, 0.0, n / 64.0)
        x = synth.normal(synth.stream_seed(11, synth.STREAM_X) + e, n * 8).reshape(n, 8)
        print(json.dumps({"experiment": "asymmetric, short axis 1024 (outputs)", "n": n, "k": 1024, "batch": 8,
                          "forward_ms": forward_ms(a, b, x)}), flush=True)
    # App. "Batch-size scaling": n = k = 2^14, batch 1 .. 256
    n = k = 1 << 14
    a = synth.uniform(synth.stream_seed(12, synth.STREAM_A), k, 0.0, n / 32.0)
    b = synth.uniform(synth.stream_seed(12, synth.STREAM_B), n, 0.0, n / 32.0)
    for batch in (1, 2, 4, 8, 16, 32, 64, 128, 256):
        x = synth.normal(synth.stream_seed(12, synth.STREAM_X) + batch, n * batch).reshape(n, batch)
        print(json.dumps({"experiment": "batch scaling", "n": n, "k": k, "batch": batch,
                          "forward_ms": forward_ms(a, b, x)}), flush=True)
    # Sec. 6 / App. "Random Fourier Features": a single product on irregular anchors a, b ~ N(0, 1), n = k = 2^16, batch 1
    n = k = 1 << 16
    a = synth.normal(synth.stream_seed(13, synth.STREAM_A), k)
    b = synth.normal(synth.stream_seed(13, synth.STREAM_B), n)
    x = synth.normal(synth.stream_seed(13, synth.STREAM_X), n).reshape(n, 1)
    print(json.dumps({"experiment": "irregular anchors N(0,1), single product", "n": n, "k": k, "batch": 1,
                      "forward_ms": forward_ms(a, b, x)}), flush=True)
    # App. "Weighted Gram matrix": A diag(d) A^T with output dimension 1024, inner dimension 2^10 .. 2^20
    for e in range(10, 21, 2):
        n, k = 1 << e, 1024
        a = synth.uniform(synth.stream_seed(14, synth.STREAM_A) + e, k, 0.0, n / 64.0)
        b = synth.uniform(synth.stream_seed(14, synth.STREAM_B) + e, n, 0.0, n / 64.0)
        d = (np.abs(synth.normal(synth.stream_seed(14, synth.STREAM_X) + e, n)) + np.float32(0.5)).astype(np.float32)
        ws = torch.empty(B.laplex_wgram_workspace_bytes(k, n), dtype=torch.uint8, device="cuda")
        da, db, dd = dev(a), dev(b), dev(d)
        m = torch.empty(k, k, device="cuda")
        print(json.dumps({"experiment": "weighted Gram matrix, output dimension 1024", "n": n, "k": k,
                          "wgram_ms": timed(lambda: B.laplex_wgram(da, db, dd, m, ws, 0))}), flush=True)



KERNEL_OF = {
    "scan_down_sparse.bwd": "k_scan_down_sparse_wide<true> (backward downsweep: reads x, writes gx and gb)",
    "scan_reduce.fwd": "forward reduce (reads the injected rows of x once for both directions)",
    "scan_reduce.bwd": "backward reduce (reads the injected rows of gy once for both directions)",
    "scan_down.fwd": "k_scan_down, forward problem (reads x, writes y and the saved scans)",
    "scan_down.bwd": "k_scan_down, backward problem (reads gy, x and the saved scans, writes gx and the anchor gradient)",
    "radix_scatter": "k_onesweep_pass (one radix pass: reads the pairs once, writes them once)",
    "permute_part.fwd": "k_part (partition levels: x into sorted order, y and the saved scans home)",
    "permute_part.bwd": "k_part (partition levels: gy into sorted order, gx and gb home)",
    "permute_part.rank": "k_part (partition levels of the inverse permutation)",
}


def family_bytes(fam, spec, np, B):
    """Algorithmic bytes of ALL launches of a kernel family in one step (what the method itself must move:
    4 B per float or id; per merged position the plan's id and decay, per injected / result row its batch
    columns), and a note saying what was counted."""
    k, n, batch, gram = spec["k"], spec["n"], spec["batch"], spec["gram"]
    N = n if gram else k + n
    inj = {"fwd": n, "bwd": n if gram else k}
    res = {"fwd": n if gram else k, "bwd": n}
    if fam == "radix_scatter":
        return 4 * N + 8 * N + 3 * 16 * N, "4 passes: the first reads the anchors (4 B) and writes pairs (8 B), the others 8 B + 8 B a pair"
    if fam == "sort_hist":
        return 4 * N, "the anchors read once"
    if fam == "decay":
        if batch == 1 and N >= (1 << 22):
            return 9 * N, "sorted anchors read (the sort's last pass wrote them), decays written, every eighth anchor pair once more"
        return 8 * N, "sorted anchors read (the sort's last pass wrote them), decays written"
    base, _, tag = fam.partition(".")
    # batch 1 from 2^22 merged positions on: values travel between the caller's order and the sorted order as records
    # (destination, value[, value]) through partition levels, and the scans work on plain arrays in sorted order
    routed = batch == 1 and N >= (1 << 22)
    if routed and base == "permute_part":
        if tag == "rank":
            return 12 * N + 16 * N, "level 1: ids read, (id, position) pairs written; level 2: pairs read and written"
        m_in, m_out = inj.get(tag, 0), res.get(tag, 0)
        return 32 * m_in + 24 * m_out, ("the injected values: rank and value read, pairs written, pairs read and written (two levels); "
                                        "the results: level 2 only (12 B records read and written; level 1 is the downsweep's)")
    if routed and base == "permute_final":
        if tag == "rank":
            return 8 * N + 4 * N, "pairs read, rank written"
        m_in, m_out = inj.get(tag, 0), res.get(tag, 0)
        return 8 * m_in + 4 * N + 12 * m_out + 8 * m_out, "pairs read, the sorted-order array written whole; result records read, both outputs written"
    if tag not in inj:
        return None, None
    if routed and base == "scan_reduce":
        return 8 * N, "decay and injected value per sorted row"
    if routed and base == "scan_down":
        extra = 4 * N if tag == "bwd" else 0
        return 12 * N + extra + 12 * res[tag], ("decay, injected value and id per sorted row" + (", the weight of the row reduction" if extra else "")
                                                + ", one 12-byte record per result row written")
    narrow = batch <= 8
    if base == "scan_reduce":
        if batch >= 253 and batch % 4 == 0:
            return 16 * N + 4 * batch * inj[tag] + 16 * batch * ((N + 511) // 512), "id, two decays and the anchor per row, the injected rows, one summary per tile of 512 rows"
        total = 8 * N + 4 * batch * inj[tag] + (4 * batch * N if narrow else 0)
        return total, "id and decay per row, the injected rows gathered" + (", the same rows written in sorted order" if narrow else "")
    if base == "scan_down":
        total = 8 * N + 4 * batch * (N if narrow else inj[tag]) + 4 * batch * res[tag]
        note = "id and decay per row, the injected rows" + (" (from the sorted-order stage)" if narrow else "") + ", the result rows written"
        if tag == "fwd":
            total += 4 * batch * res[tag]; note += ", the saved strict scans written"
        else:
            total += 4 * batch * (N if narrow else res[tag]) + 4 * res[tag]
            note += ", the weights of the row reduction read, the anchor gradient written"
            if gram:
                total += 4 * batch * res[tag]; note += ", the saved strict scans read"
        return total, note
    if fam == "scan_down_sparse.bwd" and not gram and batch >= 253 and batch % 4 == 0:
        rows = B.laplex_scan_tile_rows(batch, True)
        total, visited, blocks, all_blocks = sparse_bwd_bytes(spec["a"], spec["b"], batch, rows)
        return total, f"{visited} input rows in {blocks} of {all_blocks} blocks: 12 B of plan, the x row read, the gx row and gb written, carries per tile"
    return None, None


def make_spec(name, args, torch, np, B, synth):
    """Inputs on the device, outputs, workspace and the step function of one of the roofline workloads."""
    dev = lambda v: torch.from_numpy(np.ascontiguousarray(v)).cuda()
    scale = args.scale
    torch.cuda.reset_peak_memory_stats()       # device_bytes_peak is this workload's own
    if name == "gram":
        w = synth.gram_images(scale=scale)
        a, x, g = w["a"], w["x"], w["g"]
        n, batch, k = a.size, x.shape[1], 0
        ws = torch.empty(B.laplex_workspace_bytes(0, n, batch), dtype=torch.uint8, device="cuda")
        da, dx, dg = dev(a), dev(x), dev(g)
        y = torch.empty(n, batch, device="cuda"); gx = torch.empty(n, batch, device="cuda"); ga = torch.empty(n, device="cuda")

        def step():
            B.laplex_gram(da, dx, y, ws, B.LAPLEX_SAVE_SCANS)
            B.laplex_gram_backward(da, dx, dg, gx, ga, ws, B.LAPLEX_SAVE_SCANS | B.LAPLEX_REUSE_PLAN)
        spec = dict(a=a, b=None, x=x, g=g, k=0, n=n, batch=batch, gram=True, anchors="N(0, (2^16)^2)",
                    compulsory=4 * n * 2 + 4 * batch * 5 * n,       # a, ga; x twice, gy, y, gx
                    passname="Gram form: forward + backward (gx, ga)")
    else:
        make = {"billion": synth.billion_square, "tie_heavy": synth.tie_heavy}.get(name)
        w = synth.projection_layer(scale=scale, batch=args.batch) if make is None else make(scale=scale)
        a, b, x, g = w["a"], w["b"], w["x"], w["g"]
        k, n, batch = a.size, b.size, x.shape[1]
        ws = torch.empty(B.laplex_workspace_bytes(k, n, batch), dtype=torch.uint8, device="cuda")
        da, db, dx, dg = dev(a), dev(b), dev(x), dev(g)
        y = torch.empty(k, batch, device="cuda"); gx = torch.empty(n, batch, device="cuda")
        ga = torch.empty(k, device="cuda"); gb = torch.empty(n, device="cuda")

        def step():
            B.laplex_apply(da, db, dx, y, ws, B.LAPLEX_SAVE_SCANS)
            B.laplex_apply_backward(da, db, dx, dg, gx, ga, gb, ws, B.LAPLEX_SAVE_SCANS | B.LAPLEX_REUSE_PLAN)
        spec = dict(a=a, b=b, x=x, g=g, k=k, n=n, batch=batch, gram=False,
                    anchors={"billion": "U(0,2^24)", "tie_heavy": "U(0,2^18) on a 1/4 grid"}.get(name, "U(0,2^14)"),
                    compulsory=4 * (n + k) * 2 + 4 * batch * (3 * n + 2 * k),   # anchors, gradients; x twice, gx, gy, y
                    passname="forward+backward (gx, ga, gb)")
    spec.update(name=w["name"] if scale == 1 and (name != "projection" or args.batch == 256) else w["name"] + "/scaled",
                step=step, ws=ws, outputs=(y, gx, ga), keep=(da, dx, dg))
    return spec


def measure(spec, steps, warmup, torch, np, B):
    """Warm up, find the step's dominant kernel family (every family timed for one step), then time exactly
    `steps` steps with one HIP event pair per launch of that family on the stream it is launched on."""
    step, k, n, batch = spec["step"], spec["k"], spec["n"], spec["batch"]
    for _ in range(max(warmup, 1)):
        step()
    torch.cuda.synchronize()
    B.laplex_profile_begin("*")
    step()
    torch.cuda.synchronize()
    B.laplex_profile_end()
    families = B.laplex_profile_families()
    dominant = max(families, key=lambda f: families[f][0])
    torch.cuda.synchronize()

    B.laplex_profile_begin(dominant)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(steps):
        step()
    torch.cuda.synchronize()
    t1 = time.perf_counter()
    dom_ms, dom_launches = B.laplex_profile_end()

    N = n if spec["gram"] else n + k
    status = torch.full((1,), -1, dtype=torch.int32, device="cuda")
    B.laplex_get_plan_status(spec["ws"], N, status)
    assert int(status.item()) == 0, "the plan is marked invalid: a tile of the radix sort gave up its wait"
    for t in spec["outputs"]:
        assert bool(torch.isfinite(t.view(-1)[:4096]).all())

    ms_per_step = (t1 - t0) * 1e3 / steps
    elements = N * batch
    per_step_launches = dom_launches / steps
    fam_bytes, note = family_bytes(dominant, spec, np, B)
    dom_ms_per_step = dom_ms / steps
    roofline = {"bound": "hbm", "kernel": KERNEL_OF.get(dominant, dominant), "family": dominant,
                "achieved": None, "peak": HBM_PEAK_GBS, "unit": "GB/s", "frac": None, "traffic": None,
                "avg_kernel_ms": round(dom_ms / max(dom_launches, 1), 5), "launches": dom_launches,
                "launches_per_step": per_step_launches, "family_ms_per_step": round(dom_ms_per_step, 5),
                "algorithmic_bytes_per_step": fam_bytes,
                "algorithmic_bytes_per_launch": (fam_bytes / per_step_launches) if fam_bytes and per_step_launches else None,
                "counted": note}
    if fam_bytes:
        achieved = fam_bytes / (dom_ms_per_step * 1e-3) / 1e9
        roofline.update(achieved=round(achieved, 1), frac=round(achieved / HBM_PEAK_GBS, 4))
    traffic_file = os.path.join(ROOT, "profiles", f"traffic_{dominant.replace('.', '_')}_{spec['name'].split('/')[0].replace('^', 'p')}.json")
    if os.path.exists(traffic_file) and "/scaled" not in spec["name"]:
        with open(traffic_file) as fh:
            rec = json.load(fh)
            # per launch, like avg_kernel_ms (a family with several launches per step: the step's bytes over its launches)
            if "hbm_bytes_per_step" in rec:
                roofline["traffic"] = rec["hbm_bytes_per_step"] / max(per_step_launches, 1)
                roofline["traffic_per_step"] = rec["hbm_bytes_per_step"]
            else:
                roofline["traffic"] = rec.get("hbm_bytes_per_launch")
        roofline["traffic_source"] = "rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE, " + os.path.relpath(traffic_file, ROOT)
    out = {
        "ms_per_step": round(ms_per_step, 4), "value": elements / (ms_per_step * 1e-3),
        "config": {"workload": spec["name"], "k": k, "n": n, "batch": batch, "anchors": spec["anchors"],
                   "pass": spec["passname"], "sort": "radix sort inside every step",
                   "workspace_bytes": spec["ws"].numel(), "device_bytes_peak": torch.cuda.max_memory_allocated()},
        "roofline": roofline,
        "families_ms_one_step": {f: round(v[0], 4) for f, v in sorted(families.items(), key=lambda kv: -kv[1][0])[:16]},
        # compulsory HBM bytes of one step over the step time
        "end_to_end_hbm_frac": round(spec["compulsory"] / (ms_per_step * 1e-3) / 1e9 / HBM_PEAK_GBS, 4),
    }
    return out, dominant


def projection_ceilings(spec, roofline, torch, B):
    """Measured ceilings beside the nominal peak: a kernel that only moves the rows of x (and gx) in the order of the plan."""
    k, n, batch = spec["k"], spec["n"], spec["batch"]
    _, gx, _ = spec["outputs"]
    _, dx, _ = spec["keep"]
    perm = torch.empty(k + n, dtype=torch.int32, device="cuda")
    B.laplex_get_perm(spec["ws"], k + n, perm)
    rows_of_x = (perm[(perm >= k)] - k).contiguous()
    ceil = {}
    for name, dst, moved in (("copy_rows_GBps", gx, 2), ("read_rows_GBps", None, 1)):
        for _ in range(3):
            B.laplex_diag_move_rows(dx, dst, rows_of_x)
        torch.cuda.synchronize()
        c0 = time.perf_counter()
        for _ in range(10):
            B.laplex_diag_move_rows(dx, dst, rows_of_x)
        torch.cuda.synchronize()
        ceil[name] = round(moved * 4 * n * batch / ((time.perf_counter() - c0) / 10) / 1e9, 1)
    roofline["measured_ceiling"] = dict(ceil, note="laplex_diag_move_rows on x (and gx) in the plan's row order")


def cpu_baseline(name, spec, args, np, synth):
    """The CPU oracle (fp64 sort + dual-theorem scans, forward + backward without the tolerance denominators: the
    same results the timed GPU step produces) on a bounded sample of the same workload."""
    from oracle import laplex_oracle as oracle
    oracle.build()
    if name == "gram":
        return None
    if name in ("billion", "tie_heavy"):
        # the same recipe (same anchor density and ties) at n = k = 2^23
        make = synth.billion_square if name == "billion" else synth.tie_heavy
        shrink = max(1, spec["n"] >> 23)
        w = make(scale=args.scale * shrink)
        a, b, xs, gs = w["a"], w["b"], w["x"], w["g"]
        sample = f"the same recipe at n = k = {a.size} (batch 1), every output"
    else:
        a, b = spec["a"], spec["b"]
        cols = min(args.cpu_sample_columns, spec["batch"])
        xs = np.ascontiguousarray(spec["x"][:, :cols]); gs = np.ascontiguousarray(spec["g"][:, :cols])
        sample = f"all n and k, first {cols} of {spec['batch']} batch columns"
    cols = xs.shape[1]
    c0 = time.perf_counter()
    oracle.apply_scan(a, b, xs, with_tol=False)
    x64 = xs.astype(np.float64); g64 = gs.astype(np.float64)
    _, ls, rs = oracle._dual(b, x64, a, want=(False, True, True))
    (g64 * (rs - ls)).sum(axis=1)
    li, ls, rs = oracle._dual(a, g64, b)
    (li + rs); (x64 * (rs - ls)).sum(axis=1)
    c1 = time.perf_counter()
    threads = min(os.cpu_count() or 1, int(os.environ.get("OMP_NUM_THREADS", os.cpu_count() or 1)))
    return {"value": (a.size + b.size) * cols / (c1 - c0), "unit": "elements/s",
            # the oracle's scans run one thread per batch column; its sorts and searches use every thread
            "cores": threads, "kind": "oracle",
            "sample": "fp64 stable sort + dual-theorem scans, forward + backward; " + sample, "seconds": round(c1 - c0, 3)}


def main():
    args = parse()
    if args.gpus != 1 or int(os.environ.get("WORLD_SIZE", "1")) != 1:
        print("bench.py: this build runs on one GPU only; multi-GPU runs are not part of it "
              "(the path would shard by batch columns: anchors and plan replicated, one all-reduce of ga and gb).", file=sys.stderr)
        sys.exit(2)

    import numpy as np
    import torch
    from paper_2605_24584_amd import binding as B
    from paper_2605_24584_amd import synth

    assert torch.cuda.is_available(), "bench.py needs the GPU"
    torch.cuda.set_device(0)
    B.lib()   # fails loudly if the HIP library is not built

    if args.calibrate_copy:
        src = torch.empty(1 << 28, device="cuda").normal_()
        dst = torch.empty_like(src)
        for _ in range(3):
            dst.copy_(src)
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for _ in range(20):
            dst.copy_(src)
        torch.cuda.synchronize()
        dt = (time.perf_counter() - t0) / 20
        print(json.dumps({"copy_bytes_read": 4 << 28, "copy_bytes_written": 4 << 28, "ms": dt * 1e3,
                          "GBps_read_plus_write": 2 * (4 << 28) / dt / 1e9}), flush=True)
        return

    if args.paper_sweep:
        paper_sweep(args, torch, np, B, synth)
        return

    if args.workload not in ("billion", "projection", "gram", "tie_heavy"):
        other_workload(args, torch, np, B, synth)
        return

    spec = make_spec(args.workload, args, torch, np, B, synth)
    res, dominant = measure(spec, args.steps, args.warmup, torch, np, B)
    if args.workload == "projection":
        projection_ceilings(spec, res["roofline"], torch, B)
    out = {
        "metric": "LAPLEX fwd+bwd (n+k)*batch elements/s", "value": res["value"], "unit": "elements/s",
        "n_gpus": 1, "steps": args.steps, "warmup": args.warmup, "ms_per_step": res["ms_per_step"],
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "f32", "data": "synthetic",
        "config": res["config"], "roofline": res["roofline"],
        "families_ms_one_step": res["families_ms_one_step"], "end_to_end_hbm_frac": res["end_to_end_hbm_frac"],
        # the paper's own numbers for neighbouring shapes, with their hardware (context, not a baseline for this workload)
        "paper_context": {
            "hardware": "NVIDIA H100, fp32 (App. 'Kernel-algebra benchmarks', 'GPU runtime')",
            "square_n=k=2^29_forward_ms": 704.0,
            "asymmetric_one_axis_1024_forward_ms_at_long_axis_2^20": 7.0,
            "square_n=k=2^20_batch8_forward_backward_ms": 71.0,
            "note": "other hardware and other sizes; vs_baseline stays null",
        },
    }
    if not args.no_cpu_baseline:
        base = cpu_baseline(args.workload, spec, args, np, synth)
        if base:
            out["cpu_baseline"] = base
    if args.workload == "billion" and not args.no_extra:
        # the other two single-GPU workloads with a roofline of their own, after the benchmark's memory is released
        del spec
        torch.cuda.empty_cache()
        extra = {}
        for name in ("projection", "gram"):
            sp = make_spec(name, args, torch, np, B, synth)
            r, _ = measure(sp, args.steps_extra, 5, torch, np, B)
            if name == "projection":
                projection_ceilings(sp, r["roofline"], torch, B)
            r["steps"] = args.steps_extra
            extra[sp["name"]] = r
            del sp
            torch.cuda.empty_cache()
        out["extra_workloads"] = extra
    print(json.dumps(out), flush=True)


if __name__ == "__main__":
    main()
