#!/usr/bin/env python3
"""Benchmark of the SCD local solver on one MI355X (arXiv 1803.06333, Section 3.1 / 4.1).

A step is one whole epoch of the hot path -- every coordinate updated once (inner products with the
shared vector, scalar step, write-back into the shared vector), the accept check of the adaptive
safeguard included -- on the click-log-shaped logistic-regression workload (45 840 617 x 1 000 000,
39 one-hot fields, seeded synthetic stand-in for the public click logs the paper uses), with all
inputs resident in HBM before the timed region.

Config 4 (the default) is timed in two ways:
  groups  exact sweeps over the 39 one-hot fields (columns of a field share no row): the headline;
  async   the permutation-ordered asynchronous epoch with atomic write-back, which needs no
          structure: reported beside it under "async_general_path".
Prints ONE JSON line: coordinate updates per second, the roofline of the dominant kernel, and a CPU
baseline (the fp64 oracle timed on the host cores on a bounded sample of the same workload).
"""
import argparse
import ctypes as C
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)


def avg(xs):
    return float(sum(xs) / len(xs)) if xs else 0.0


def timed_epochs(g, torch, steps, warmup, seed0):
    """W untimed epochs, K timed ones, then a few more to read the per-kernel device times."""
    for e in range(warmup):
        g.epoch(seed0 + e)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for e in range(steps):
        g.epoch(seed0 + 1000 + e)
    torch.cuda.synchronize()
    elapsed = time.perf_counter() - t0
    per = {"large_ms": [], "small_ms": [], "perm_ms": [], "scd_ms": [], "copy_ms": [], "epoch_ms": []}
    rejected = 0
    for e in range(min(5, max(1, steps))):        # outside the timed region: reading them synchronises
        g.epoch(seed0 + 2000 + e)
        st = g.epoch_stats()
        for k in per:
            per[k].append(st[k])
        rejected += st["rejected"]
    return elapsed, {k: avg(v) for k, v in per.items()}, g.epoch_stats(), rejected


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=20)
    ap.add_argument("--warmup", type=int, default=2)
    ap.add_argument("--config", type=int, default=4,
                    help="benchmark configuration 1..5 (default: 4; 5 = streamed from pinned host memory)")
    ap.add_argument("--mode", choices=["auto", "async", "groups", "tiles"], default="auto",
                    help="groups: exact sweeps over the one-hot fields (config 4); tiles: exact tile sweeps (dense "
                         "ridge, config 2); async: permutation-ordered asynchronous epoch with atomic write-back "
                         "(any data); auto: groups for config 4 with the async path measured beside it, tiles for "
                         "config 2, async otherwise")
    ap.add_argument("--scale", type=float, default=1.0, help="shrink the row count (debugging only)")
    ap.add_argument("--budget-gib", type=float, default=16.0, help="config 5: device budget for the matrix")
    ap.add_argument("--chunk-gib", type=float, default=4.0, help="config 5: chunk size")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-gap", action="store_true", help="skip the time-to-gap leg")
    ap.add_argument("--gap-target", type=float, default=1e-3)
    ap.add_argument("--gap-max-epochs", type=int, default=1500)
    ap.add_argument("--gap-max-seconds", type=float, default=40.0)
    ap.add_argument("--inflight", type=int, default=0, help="async: override the cap on nonzeros in flight")
    ap.add_argument("--damping", type=float, default=0.0, help="initial step scaling (0 = library default 1)")
    ap.add_argument("--calibrate", action="store_true",
                    help="also run one elementwise pass over 1 GiB (read 1 GiB, write 1 GiB) so that a counter "
                         "run can scale FETCH_SIZE / WRITE_SIZE against known traffic")
    args = ap.parse_args()
    if args.gpus != 1 or int(os.environ.get("WORLD_SIZE", "1")) != 1:
        print("bench.py: this build runs the one-GPU local solver only; --gpus must be 1", file=sys.stderr)
        sys.exit(2)

    import numpy as np
    import torch
    import datagen
    import paper_1803_06333_amd as snap

    if not torch.cuda.is_available():
        print("bench.py: no GPU visible", file=sys.stderr)
        sys.exit(1)
    dev = "cuda:0"
    snap.load_library()           # fails loudly when the HIP library is not built
    mode = args.mode
    if mode == "auto":
        mode = {4: "groups", 2: "tiles"}.get(args.config, "async")
    if (mode == "groups" and args.config != 4) or (mode == "tiles" and args.config != 2):
        print("bench.py: --mode groups needs the one-hot config 4, --mode tiles the dense config 2", file=sys.stderr)
        sys.exit(2)

    t0 = time.time()
    p = datagen.config(args.config, device=dev, scale=args.scale)
    torch.cuda.synchronize()
    gen_s = time.time() - t0
    dense = p.layout.startswith("dense")
    m = p.d if p.layout != "csr" else p.n
    nnz = p.nnz

    kw = {}
    if args.config == 5:
        # the matrix lives in pinned host memory and is streamed in chunks (Section 3.2)
        t1 = time.time()
        for name in ("ptr", "idx", "val", "y"):
            src = getattr(p, name)
            dst = torch.empty(src.shape, dtype=src.dtype, pin_memory=True)
            dst.copy_(src)
            setattr(p, name, dst)
            del src
        torch.cuda.synchronize()
        torch.cuda.empty_cache()
        kw = {"device_budget_bytes": int(args.budget_gib * 2 ** 30), "chunk_bytes": int(args.chunk_gib * 2 ** 30)}
        gen_s += time.time() - t1
    if mode == "groups":
        kw["group_bounds"] = p.meta["field_starts"] + [p.d]
    elif not dense and p.layout == "csc":
        kw["auto_groups"] = False                 # async: the structure-free epoch, no search for groups
    if dense:
        kw["dense_tiles"] = mode == "tiles"
    t0 = time.time()
    # group sweeps: every fourth row pass carries its pair of events, a different one each epoch (timing
    # all of them holds the chain of dependent kernels up by 3 %); the other engines time every kernel
    g = snap.Solver.from_problem(p, profile=2 if mode == "groups" else True, max_inflight_nnz=args.inflight,
                                 damping=args.damping, **kw)
    torch.cuda.synchronize()
    create_s = time.time() - t0

    elapsed, kms, st, rejected = timed_epochs(g, torch, args.steps, args.warmup, 1000)
    ms_per_step = 1e3 * elapsed / args.steps
    updates_per_s = m * args.steps / elapsed

    # algorithmic bytes: 16 B per nonzero (index, value, read and write of v) sparse, 12 B per
    # element dense, plus 24 B per coordinate (order entry, offsets, model read+write, norm)
    per_elem = 12 if dense else 16
    alg_epoch = per_elem * nnz + 24 * m
    if mode == "groups":
        # one row pass retires the write-back of one field (n nonzeros) and the inner products of the
        # next field's hot columns: counted as n nonzeros x 16 B (also its real traffic: two row-map
        # words, read and write of v per row)
        passes = max(1, st["n_items"])
        dom, dom_ms, dom_bytes = "k_group_rows", kms["large_ms"] / passes, 16 * p.n
    elif mode == "tiles":
        # one pass reads the columns of two tiles (write-back of one, inner products of the next) and
        # reads v, y and writes v once: 2 x 4 B per element per epoch plus 12 B per row per pass
        passes = max(1, st["n_items"])
        dom, dom_ms, dom_bytes = "k_tile_pass", kms["large_ms"] / passes, (8 * nnz + 12 * p.n * passes) / passes
    elif args.config == 5:
        dom, dom_ms, dom_bytes = "scd kernels of all chunks", kms["scd_ms"], alg_epoch
    elif kms["large_ms"] >= kms["small_ms"]:
        dom, dom_ms, dom_bytes = "k_scd_large", kms["large_ms"], per_elem * st["nnz_large"] + 24 * st["n_large"]
    else:
        dom, dom_ms, dom_bytes = "k_scd_small", kms["small_ms"], per_elem * st["nnz_small"] + 24 * st["n_small"]
    achieved = dom_bytes / (dom_ms * 1e-3) / 1e9 if dom_ms > 0 else 0.0
    traffic = None
    tf = os.path.join(ROOT, "profiles", "traffic_config%d.json" % args.config)
    if os.path.exists(tf) and args.scale == 1.0:
        try:
            traffic = json.load(open(tf)).get(dom)
        except Exception:
            traffic = None
    roofline = {"bound": "hbm", "kernel": dom, "achieved": round(achieved, 2), "peak": 8000.0, "unit": "GB/s",
                "frac": round(achieved / 8000.0, 5), "traffic": traffic,
                "kernel_ms": round(dom_ms, 4), "algorithmic_bytes_per_launch": int(dom_bytes),
                "epoch_algorithmic_GBps": round(alg_epoch / (ms_per_step * 1e-3) / 1e9, 2),
                "epoch_frac_of_peak": round(alg_epoch / (ms_per_step * 1e-3) / 8e12, 5)}

    out = {
        "metric": "coordinate updates/s (one SCD epoch: inner products with v, step, write-back for every "
                  "coordinate)",
        "value": updates_per_s, "unit": "coordinate updates/s", "n_gpus": 1, "steps": args.steps,
        "warmup": args.warmup, "ms_per_step": ms_per_step, "higher_is_better": True, "scaling": "weak",
        "vs_baseline": None, "dtype": "f32", "data": "synthetic",
        "config": {"workload": "config%d:%s" % (args.config, p.name), "mode": mode, "n_rows": p.n, "n_cols": p.d,
                   "nnz": nnz, "loss": p.loss, "lambda": p.lam, "layout": p.layout, "scale": args.scale},
        "roofline": roofline,
        "epochs_per_s": args.steps / elapsed, "nnz_per_s": nnz * args.steps / elapsed,
        "kernel_ms": {k: round(v, 4) for k, v in kms.items()},
        "damping": st["damping"], "rejected_epochs_in_sample": rejected,
        "generate_s": round(gen_s, 2), "create_s": round(create_s, 2),
    }
    if mode == "tiles":
        out["tiles"] = {"n_tiles": st["n_chunks"], "row_passes_per_epoch": st["n_items"]}
    elif mode == "groups":
        out["groups"] = {"n_groups": st["n_chunks"], "row_passes_per_epoch": st["n_items"],
                         "hot_coordinates": st["n_large"], "hot_nnz": st["nnz_large"],
                         "cold_coordinates": st["n_small"], "cold_nnz": st["nnz_small"]}
    else:
        out["inflight_nnz"] = st["inflight_nnz"]
        out["n_small"], out["n_large"] = st["n_small"], st["n_large"]
    if args.config == 5:
        tc, tk, tw = kms["copy_ms"], kms["scd_ms"], kms["epoch_ms"]
        out["streaming"] = {"n_chunks": st["n_chunks"], "copy_ms_per_epoch": round(tc, 2),
                            "kernel_ms_per_epoch": round(tk, 2), "wall_ms_per_epoch": round(tw, 2),
                            "copy_ms_per_chunk": round(tc / st["n_chunks"], 2),
                            "kernel_ms_per_chunk": round(tk / st["n_chunks"], 2),
                            "overlap_fraction": round((tc + tk - tw) / max(min(tc, tk), 1e-9), 4),
                            "bytes_copied_per_epoch": g.stream_bytes(),
                            "host_to_device_GBps": round(g.stream_bytes() / (tc * 1e-3) / 1e9, 2) if tc > 0 else None,
                            "paper_context_ms_per_chunk": {"copy_pcie_gen3": 318, "copy_nvlink2": 55, "train": 90}}

    # ---- time to duality gap (fresh solver state) ------------------------------------------------
    def time_to_gap(solver, ms_epoch):
        """Fresh (zero) model, then snap_solve in slices of 5 epochs (one gap evaluation each) until the target."""
        solver.set_model(np.zeros(solver.n_coords, dtype=np.float32))
        torch.cuda.synchronize()
        t_start = time.perf_counter()
        reached, ep, gap, trace = False, 0, float("nan"), []
        while ep < args.gap_max_epochs and time.perf_counter() - t_start < args.gap_max_seconds:
            done, gap = solver.solve(5000 + ep, 5, args.gap_target, check_every=5)
            ep += done
            trace.append([ep, round(time.perf_counter() - t_start, 4), gap])
            if gap <= args.gap_target:
                reached = True
                break
        wall = time.perf_counter() - t_start
        return {"target": args.gap_target, "reached": reached, "epochs": ep,
                "seconds_with_gap_evaluations": round(wall, 4),
                "epochs_times_ms_per_step_seconds": round(ep * ms_epoch * 1e-3, 4), "final_gap": gap,
                "final_objective": solver.objective(), "trace": trace[-6:]}

    if not args.no_gap and args.config != 5:
        out["time_to_gap"] = time_to_gap(g, ms_per_step)
    g.close()

    # ---- the structure-free asynchronous path on the same data (config 4, auto) --------------------
    if args.mode == "auto" and args.config == 4:
        ga = snap.Solver.from_problem(p, profile=True, max_inflight_nnz=args.inflight, damping=args.damping,
                                      auto_groups=False)
        steps_a = max(3, min(args.steps, 8))
        el, kma, sta, rej = timed_epochs(ga, torch, steps_a, 1, 9000)
        big = kma["large_ms"] >= kma["small_ms"]
        kb = (16 * sta["nnz_large"] + 24 * sta["n_large"]) if big else (16 * sta["nnz_small"] + 24 * sta["n_small"])
        kt = kma["large_ms"] if big else kma["small_ms"]
        out["async_general_path"] = {
            "value": m * steps_a / el, "unit": "coordinate updates/s", "steps": steps_a,
            "ms_per_step": 1e3 * el / steps_a, "epoch_algorithmic_GBps": round(alg_epoch / (el / steps_a) / 1e9, 2),
            "kernel_ms": {k: round(v, 4) for k, v in kma.items()}, "inflight_nnz": sta["inflight_nnz"],
            "rejected_epochs_in_sample": rej,
            "roofline": {"bound": "hbm", "kernel": "k_scd_large" if big else "k_scd_small",
                         "achieved": round(kb / (kt * 1e-3) / 1e9, 2), "peak": 8000.0, "unit": "GB/s",
                         "frac": round(kb / (kt * 1e-3) / 8e12, 5), "kernel_ms": round(kt, 4),
                         "algorithmic_bytes_per_launch": int(kb)}}
        if not args.no_gap:
            out["async_general_path"]["time_to_gap"] = time_to_gap(ga, 1e3 * el / steps_a)
        ga.close()

    # ---- CPU baseline: the oracle, one thread, on a bounded sample of the same epoch --------------
    if not args.no_cpu_baseline:
        import oracle
        A = oracle.Matrix.from_problem(p)
        yh = p.y.cpu().numpy()
        o = oracle.Solver(A, yh, p.loss, p.lam)
        perm = oracle.permutation(7000, o.m)
        # visit the first coordinates of one epoch order until about 15 s of CPU time are spent
        L = oracle.lib()
        done, t_cpu, batch, nnz_done = 0, 0.0, max(1, o.m // 200), 0
        while done < o.m and t_cpu < 15.0:
            mc = min(batch, o.m - done)
            sl = np.ascontiguousarray(perm[done:done + mc])
            ts = time.perf_counter()
            args_t = (oracle._p(sl), C.c_int64(0), C.c_int64(mc), oracle._p(o.x), oracle._p(o.v))
            lam_t = (C.c_double(o.lam), C.c_double(0.0))
            if o.form == "dual":
                L.oracle_epoch_dual_hinge(C.c_int64(A.n), oracle._p(A.ptr), oracle._p(A.idx), oracle._p(A.val),
                                          oracle._p(o.y), lam_t[0], *args_t)
            elif A.layout == "csc":
                L.oracle_epoch_primal_sparse(C.c_int(o.loss), C.c_int64(A.n), oracle._p(A.ptr), oracle._p(A.idx),
                                             oracle._p(A.val), oracle._p(o.y), *lam_t, *args_t)
            else:
                L.oracle_epoch_primal_dense(C.c_int(o.loss), C.c_int64(A.n), oracle._p(A.val), oracle._p(o.y), *lam_t,
                                            *args_t)
            t_cpu += time.perf_counter() - ts
            if A.ptr is not None:
                nnz_done += int((A.ptr[sl.astype(np.int64) + 1] - A.ptr[sl.astype(np.int64)]).sum())
            else:
                nnz_done += mc * A.n
            done += mc
        out["cpu_baseline"] = {"value": done / t_cpu, "unit": "coordinate updates/s", "cores": 1, "kind": "oracle",
                               "sample": "first %d of %d coordinates of one epoch order (%d nonzeros, %.1f s), "
                                         "sequential fp64 oracle" % (done, o.m, nnz_done, t_cpu),
                               "nnz_per_s": nnz_done / t_cpu, "host_cores_available": os.cpu_count()}
    if args.calibrate:
        a = torch.zeros(1 << 28, dtype=torch.float32, device=dev)
        b = torch.empty_like(a)
        torch.cuda.synchronize()
        torch.add(a, 1.0, out=b)
        torch.cuda.synchronize()
    print(json.dumps(out))


if __name__ == "__main__":
    main()
