#!/usr/bin/env python3
"""Benchmark of the SCD local solver on one MI355X (arXiv 1803.06333, Section 3.1 / 4.1).

A step is one whole epoch of the hot path -- every coordinate updated once (inner products with the
shared vector, scalar step, write-back into the shared vector) -- with all inputs resident in HBM
before the timed region (config 5: in pinned host memory, which is the point of that config).

The headline is config 4, the click-log-shaped logistic-regression workload (45 840 617 x 1 000 000,
39 one-hot fields, seeded synthetic stand-in for the public click logs the paper uses), timed in two
ways:
  groups  exact sweeps over the 39 one-hot fields (columns of a field share no row): `value`.
          This engine needs neither the coordinate permutation (the order inside a field does not
          change the result) nor the accept check of the adaptive safeguard (nothing is asynchronous),
          and the timed epoch contains neither;
  async   the permutation-ordered asynchronous epoch with atomic write-back, which needs no
          structure: reported beside it under "async_general_path", permutation and accept check
          included.
After the headline the other four configurations are run with fewer steps and reported under
"other_configs".  Prints ONE JSON line.

Bytes.  `roofline.achieved` counts, per launch of the dominant kernel, the bytes of the storage format
that kernel reads and writes (for a row pass of the group sweeps: two row-map entries, one read and one
write of the shared vector, one label bit per row; values only when they are not all 1).  The survey's
format-independent figure of 16 bytes per nonzero is given beside it, labelled as such, and so is the
compulsory traffic (the matrix in the format used, read once per epoch).
"""
import argparse
import ctypes as C
import gc
import json
import os
import sys
import time
import traceback

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)
PEAK_GBPS = 8000.0


def avg(xs):
    return float(sum(xs) / len(xs)) if xs else 0.0


def host_info():
    model, mem_gib = "unknown", None
    try:
        for line in open("/proc/cpuinfo"):
            if line.startswith("model name"):
                model = line.split(":", 1)[1].strip()
                break
        for line in open("/proc/meminfo"):
            if line.startswith("MemTotal"):
                mem_gib = round(int(line.split()[1]) / 2 ** 20, 1)
                break
    except OSError:
        pass
    try:
        usable = len(os.sched_getaffinity(0))
    except AttributeError:
        usable = os.cpu_count()
    return {"cpu_model": model, "logical_cpus": os.cpu_count(), "cpus_usable": usable, "ram_GiB": mem_gib,
            "omp_num_threads": os.environ.get("OMP_NUM_THREADS")}


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


def stored_traffic(cfg, kernel, scale):
    """HBM bytes per launch from rocprofv3 counter runs of this command, as committed under profiles/:
    a stored figure of an earlier run (the file names the commit), not a measurement of this run."""
    tf = os.path.join(ROOT, "profiles", "traffic_config%d.json" % cfg)
    if not os.path.exists(tf) or scale != 1.0:
        return None, None
    try:
        d = json.load(open(tf))
    except Exception:
        return None, None
    src = "profiles/traffic_config%d.json: rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE of an earlier run of this " \
          "command (%s); not measured by this run" % (cfg, d.get("_measured_at", "commit not recorded"))
    return d.get(kernel), src


def roofline_of(cfg, mode, p, nnz, m, dense, st, kms, ms_per_step, scale):
    """Roofline of the dominant kernel and the per-epoch bandwidth figures."""
    n = p.n
    survey_epoch = (12 if dense else 16) * nnz + 24 * m          # the survey's format-independent count
    extra = {}
    if mode == "groups":
        # a row pass between two fields: map entry of the previous and of the current field, v in, v out,
        # one label bit (logistic), the two value arrays only when the values are not all 1
        unit = bool(st["unit_values"])
        lab = 0.125 if p.loss == "logistic" else 4.0
        passes = max(1, st["n_items"])
        G = st["n_chunks"]
        # bytes per map entry, averaged over the groups (groups of at most 255 columns are read as bytes); a pass
        # reads the maps of two groups that the epoch's random order puts next to each other
        mb = (st["row_map_bytes"] * (G - st["byte_map_groups"]) + st["byte_map_groups"]) / max(1, G)
        per_row = 2 * mb + 8 + lab + (0 if unit else 8)
        dom, dom_ms, dom_bytes = "k_group_rows", kms["large_ms"] / passes, per_row * n
        if cfg == 5:
            # streamed row maps: the kernels of a visit (decoding of the map, row pass, step kernel) are
            # timed together, from the moment the visit's map has arrived; the epoch is bound by the host link
            dom, dom_ms = "row passes + step kernels of all %d visits" % G, kms["scd_ms"]
            dom_bytes = n * (2 * G * mb + 4 * (2 * G + 1) + G * lab) + 24 * m
        # whole epoch in this format: every map is read twice (as current, then as previous field), v is read
        # by G + 1 passes and written by G, labels by the G passes that take sums
        fmt_epoch = n * (2 * G * mb + 4 * (2 * G + 1) + G * lab + (0 if unit else 8 * G)) + 24 * m
        compulsory = n * (G * mb + lab + (0 if unit else 4 * G))
        extra["bytes_per_row_of_a_pass"] = {"row_map_prev": round(mb, 4), "row_map_cur": round(mb, 4), "v_read": 4, "v_write": 4,
                                            "label": lab, "values": 0 if unit else 8}
    elif mode == "tiles":
        # one pass reads the columns of two tiles (write-back of one, inner products of the next) and
        # reads v, y and writes v once: 2 x 4 B per element per epoch plus 12 B per row per pass
        passes = max(1, st["n_items"])
        dom, dom_ms, dom_bytes = "k_tile_pass", kms["large_ms"] / passes, (8 * nnz + 12 * n * passes) / passes
        fmt_epoch = 8 * nnz + 12 * n * passes + 24 * m
        compulsory = 4 * nnz
    else:
        fmt_epoch = survey_epoch                                    # index, value, v in, v out per nonzero
        compulsory = (4 if dense else 8) * nnz
        if cfg == 5:
            dom, dom_ms, dom_bytes = "scd kernels of all chunks", kms["scd_ms"], fmt_epoch
        elif kms["large_ms"] >= kms["small_ms"]:
            dom, dom_ms = "k_scd_large", kms["large_ms"]
            dom_bytes = (12 if dense else 16) * st["nnz_large"] + 24 * st["n_large"]
        else:
            dom, dom_ms = "k_scd_small", kms["small_ms"]
            dom_bytes = 16 * st["nnz_small"] + 24 * st["n_small"]
    achieved = dom_bytes / (dom_ms * 1e-3) / 1e9 if dom_ms > 0 else 0.0
    traffic, traffic_src = stored_traffic(cfg, dom, scale)
    t = ms_per_step * 1e-3
    r = {"bound": "hbm", "kernel": dom, "achieved": round(achieved, 2), "peak": PEAK_GBPS, "unit": "GB/s",
         "frac": round(achieved / PEAK_GBPS, 5), "traffic": traffic, "traffic_source": traffic_src,
         "kernel_ms": round(dom_ms, 4), "algorithmic_bytes_per_launch": int(dom_bytes),
         "epoch": {"format_bytes": int(fmt_epoch), "format_GBps": round(fmt_epoch / t / 1e9, 2),
                   "format_frac_of_peak": round(fmt_epoch / t / 1e9 / PEAK_GBPS, 5),
                   "compulsory_bytes": int(compulsory), "compulsory_GBps": round(compulsory / t / 1e9, 2),
                   "survey_16B_per_nnz_bytes": int(survey_epoch),
                   "survey_16B_per_nnz_GBps": round(survey_epoch / t / 1e9, 2),
                   "note": "format_*: bytes of the storage format the epoch's kernels read and write; compulsory_*: "
                           "the matrix in that format once; survey_*: 16 B per nonzero (12 B per element dense) "
                           "whatever the format, for comparison only"}}
    r.update(extra)
    if mode == "groups" and cfg == 5:
        r["note"] = "the epoch is bound by the host link (see streaming.host_to_device_GBps), not by HBM: the kernels " \
                    "(the decoding of the prefix-coded maps included) take two fifths of the epoch and run behind the " \
                    "copies; achieved / frac are those of the kernels alone"
    if mode not in ("groups", "tiles") and cfg != 5:
        r["note"] = "bound in practice by the memory side's atomic unit (about 21 G scattered fp32 atomics/s on " \
                    "this part), not by bandwidth; the fraction of the HBM peak is what the metric asks for"
    return r


def time_to_gap(solver, np, torch, ms_epoch, target, max_epochs, max_seconds, zero_start=True):
    """Fresh model, then snap_solve in slices of 5 epochs (one gap evaluation each) until the target."""
    if zero_start:
        solver.set_model(np.zeros(solver.n_coords, dtype=np.float32))
    torch.cuda.synchronize()
    t_start = time.perf_counter()
    reached, ep, gap, trace = False, 0, float("nan"), []
    while ep < max_epochs and time.perf_counter() - t_start < max_seconds:
        done, gap = solver.solve(5000 + ep, 5, target, check_every=5)
        ep += done
        trace.append([ep, round(time.perf_counter() - t_start, 4), gap])
        if gap <= target:
            reached = True
            break
    wall = time.perf_counter() - t_start
    return {"target": target, "reached": reached, "epochs": ep,
            "seconds_with_gap_evaluations": round(wall, 4),
            "epochs_times_ms_per_step_seconds": round(ep * ms_epoch * 1e-3, 4), "final_gap": gap,
            "final_objective": solver.objective(), "trace": trace[-6:]}


def make_problem(cfg, args, torch, datagen, dev):
    t0 = time.time()
    # config 5 is pattern-only data (no value array: every stored value is 1), which halves what has to sit
    # in pinned host memory; the boxes here allow about 64 GiB of it
    p = datagen.config(cfg, device=dev, scale=args.scale, **({"pattern_only": True} if cfg == 5 else {}))
    torch.cuda.synchronize()
    kw = {}
    if cfg == 5:
        # the matrix lives in pinned host memory and is streamed in chunks (Section 3.2)
        for name in ("ptr", "idx", "y"):
            src = getattr(p, name)
            dst = torch.empty(src.shape, dtype=src.dtype, pin_memory=True)
            dst.copy_(src)
            setattr(p, name, dst)
            del src
        torch.cuda.synchronize()
        torch.cuda.empty_cache()
        kw = {"device_budget_bytes": int(args.budget_gib * 2 ** 30), "chunk_bytes": int(args.chunk_gib * 2 ** 30)}
    return p, kw, time.time() - t0


def run_config(cfg, mode, steps, warmup, args, mods, want_gap=True, keep_problem=False):
    """One configuration: generate, create, time K epochs, roofline, (time to gap).  Returns the result
    dictionary and, on request, the problem and its constructor arguments for further legs."""
    np, torch, datagen, snap = mods
    dev = "cuda:0"
    p, kw, gen_s = make_problem(cfg, args, torch, datagen, dev)
    dense = p.layout.startswith("dense")
    m = p.d if p.layout != "csr" else p.n
    nnz = p.nnz
    if mode in ("groups", "stream_groups"):
        kw["group_bounds"] = p.meta["field_starts"] + [p.d]
    elif not dense and p.layout == "csc":
        kw["auto_groups"] = False                 # async: the structure-free epoch, no search for groups
    if dense:
        kw["dense_tiles"] = mode == "tiles"
    t0 = time.time()
    # group sweeps: every fourth row pass carries its pair of events, a different one each epoch (timing
    # all of them holds the chain of dependent kernels up by 3 %); the other engines time every kernel
    try:
        g = snap.Solver.from_problem(p, profile=2 if mode == "groups" else True, max_inflight_nnz=args.inflight,
                                     damping=args.damping, **kw)
    except snap.SnapError as e:
        if mode != "stream_groups" or e.code != -2:
            raise
        mode = "async"                            # a library without group sweeps on streamed data
        kw.pop("group_bounds")
        g = snap.Solver.from_problem(p, profile=True, max_inflight_nnz=args.inflight, damping=args.damping, **kw)
    torch.cuda.synchronize()
    create_s = time.time() - t0

    first_epochs_ms = None
    if cfg == 3:
        # from alpha = 0 every row moves and the few features that almost every row holds take a million
        # same-address atomics each: the first epochs are a regime of their own and are shown separately
        first_epochs_ms = []
        for e in range(6):
            torch.cuda.synchronize()
            t1 = time.perf_counter()
            g.epoch(400 + e)
            torch.cuda.synchronize()
            first_epochs_ms.append(round(1e3 * (time.perf_counter() - t1), 3))
    elapsed, kms, st, rejected = timed_epochs(g, torch, steps, warmup, 1000)
    ms_per_step = 1e3 * elapsed / steps
    engine = "groups" if mode == "stream_groups" else mode
    out = {
        "value": m * steps / elapsed, "unit": "coordinate updates/s", "steps": steps, "warmup": warmup,
        "ms_per_step": ms_per_step,
        "config": {"workload": "config%d:%s" % (cfg, p.name), "mode": mode, "n_rows": p.n, "n_cols": p.d,
                   "nnz": nnz, "loss": p.loss, "lambda": p.lam, "layout": p.layout, "scale": args.scale},
        "roofline": roofline_of(cfg, engine, p, nnz, m, dense, st, kms, ms_per_step, args.scale),
        "epochs_per_s": steps / elapsed, "nnz_per_s": nnz * steps / elapsed,
        "kernel_ms": {k: round(v, 4) for k, v in kms.items()},
        "damping": st["damping"], "rejected_epochs_in_sample": rejected,
        "generate_s": round(gen_s, 2), "create_s": round(create_s, 2),
    }
    if first_epochs_ms is not None:
        out["first_epochs_from_zero_ms"] = first_epochs_ms
    if mode == "tiles":
        out["tiles"] = {"n_tiles": st["n_chunks"], "row_passes_per_epoch": st["n_items"]}
    elif engine == "groups":
        out["groups"] = {"n_groups": st["n_chunks"], "row_passes_per_epoch": st["n_items"],
                         "hot_coordinates": st["n_large"], "hot_nnz": st["nnz_large"],
                         "cold_coordinates": st["n_small"], "cold_nnz": st["nnz_small"],
                         "row_map_bytes": st["row_map_bytes"], "byte_map_groups": st["byte_map_groups"],
                         "unit_values": bool(st["unit_values"])}
        out["epoch_contents"] = "row passes and step kernels of all fields; no permutation (the order inside a field " \
                                "does not change the result) and no accept check (nothing is asynchronous)"
    else:
        out["inflight_nnz"] = st["inflight_nnz"]
        out["n_small"], out["n_large"] = st["n_small"], st["n_large"]
        out["epoch_contents"] = "key generation and sort, both epoch kernels, the accept check (state copy, objective)"
    if cfg == 5:
        tc, tk, tw = kms["copy_ms"], kms["scd_ms"], kms["epoch_ms"]
        nch = max(1, st["n_chunks"])
        out["streaming"] = {"n_chunks": st["n_chunks"], "copy_ms_per_epoch": round(tc, 2),
                            "kernel_ms_per_epoch": round(tk, 2), "wall_ms_per_epoch": round(tw, 2),
                            "copy_ms_per_chunk": round(tc / nch, 2),
                            "kernel_ms_per_chunk": round(tk / nch, 2),
                            "overlap_fraction": round((tc + tk - tw) / max(min(tc, tk), 1e-9), 4),
                            "bytes_copied_per_epoch": g.stream_bytes(),
                            "host_to_device_GBps": round(g.stream_bytes() / (tc * 1e-3) / 1e9, 2) if tc > 0 else None,
                            "paper_context_ms_per_chunk": {"copy_pcie_gen3": 318, "copy_nvlink2": 55, "train": 90}}
        out["objective_after_%d_epochs" % (warmup + steps + min(5, max(1, steps)))] = g.objective()
    if want_gap and cfg != 5:
        out["time_to_gap"] = time_to_gap(g, np, torch, ms_per_step, args.gap_target, args.gap_max_epochs,
                                         args.gap_max_seconds)
    g.close()
    if keep_problem:
        return out, p, kw
    del p
    torch.cuda.empty_cache()
    if cfg == 5:
        gc.collect()
        torch._C._host_emptyCache()               # give the pinned host memory back
    return out, None, None


def cpu_baseline(p, np):
    """(a) the sequential fp64 oracle on the first coordinates of one epoch order (one thread: sequential
    coordinate descent is one dependent chain) for about ten seconds; (b) the oracle's objective and duality
    gap (its sparse products run over all host cores) once each at the zero model."""
    import oracle
    A = oracle.Matrix.from_problem(p)
    yh = p.y.cpu().numpy()
    o = oracle.Solver(A, yh, p.loss, p.lam)
    perm = oracle.permutation(7000, o.m)
    L = oracle.lib()
    done, t_cpu, batch, nnz_done = 0, 0.0, max(1, o.m // 200), 0
    while done < o.m and t_cpu < 10.0:
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
    info = host_info()
    out = {"value": done / t_cpu, "unit": "coordinate updates/s", "cores": 1, "kind": "oracle",
           "sample": "first %d of %d coordinates of one epoch order (%d nonzeros, %.1f s), sequential fp64 oracle"
                     % (done, o.m, nnz_done, t_cpu),
           "nnz_per_s": nnz_done / t_cpu, "host": info}
    # (b) objective and gap by the oracle, all cores
    ts = time.perf_counter()
    P = o.primal()
    t_obj = time.perf_counter() - ts
    ts = time.perf_counter()
    G = o.gap()
    t_gap = time.perf_counter() - ts
    out["evaluations_all_cores"] = {"threads": info["omp_num_threads"] or info["cpus_usable"],
                                    "objective_s": round(t_obj, 3), "duality_gap_s": round(t_gap, 3),
                                    "objective": P, "gap": G,
                                    "what": "oracle objective (one pass over v) and duality gap (u = grad f(v), X^T u: one "
                                            "inner product per coordinate, OpenMP over the coordinates) at the state "
                                            "the sample left"}
    return out


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=20)
    ap.add_argument("--warmup", type=int, default=2)
    ap.add_argument("--config", type=int, default=0,
                    help="benchmark configuration 1..5 alone; default: config 4 as the headline, then the other four "
                         "with fewer steps under \"other_configs\"")
    ap.add_argument("--mode", choices=["auto", "async", "groups", "tiles", "stream_groups"], default="auto",
                    help="groups: exact sweeps over the one-hot fields (config 4); tiles: exact tile sweeps (dense "
                         "ridge, config 2); stream_groups: group sweeps over streamed row maps (config 5); async: "
                         "permutation-ordered asynchronous epoch with atomic write-back (any data); auto: groups for "
                         "config 4 with the async path measured beside it, tiles for config 2, stream_groups for "
                         "config 5, async otherwise")
    ap.add_argument("--scale", type=float, default=1.0, help="shrink the row count (debugging only)")
    ap.add_argument("--budget-gib", type=float, default=16.0, help="config 5: device budget for the matrix")
    ap.add_argument("--chunk-gib", type=float, default=4.0, help="config 5: chunk size")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-gap", action="store_true", help="skip the time-to-gap legs")
    ap.add_argument("--no-others", action="store_true", help="headline only: skip configs 1, 2, 3 and 5")
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
    snap.load_library()           # fails loudly when the HIP library is not built
    mods = (np, torch, datagen, snap)
    cfg = args.config or 4
    default_mode = {4: "groups", 2: "tiles", 5: "stream_groups"}

    def mode_of(c):
        return default_mode.get(c, "async") if args.mode == "auto" else args.mode
    mode = mode_of(cfg)
    ok = {"groups": (4,), "tiles": (2,), "stream_groups": (5,)}
    if mode in ok and cfg not in ok[mode]:
        print("bench.py: --mode groups needs config 4, tiles config 2, stream_groups config 5", file=sys.stderr)
        sys.exit(2)

    res, p, kw = run_config(cfg, mode, args.steps, args.warmup, args, mods, want_gap=not args.no_gap, keep_problem=True)
    out = {
        "metric": "coordinate updates/s (one SCD epoch: inner products with v, step, write-back for every "
                  "coordinate)",
        "value": res.pop("value"), "unit": res.pop("unit"), "n_gpus": 1, "steps": res.pop("steps"),
        "warmup": res.pop("warmup"), "ms_per_step": res.pop("ms_per_step"), "higher_is_better": True,
        "scaling": "weak", "vs_baseline": None, "dtype": "f32", "data": "synthetic",
    }
    out.update(res)

    # ---- what bare streaming kernels reach on this device, beside the dominant kernel's figure ---------
    if mode == "groups" and out["roofline"].get("achieved"):
        n_rows = p.n
        bare = {}
        for kind, name, per_row in ((0, "read_only", 4), (1, "copy", 8), (2, "row_pass_mix", 12)):
            us = snap.stream_probe(kind, n_rows, 40)
            bare[name + "_GBps"] = round(per_row * n_rows / (us * 1e-6) / 1e9, 1)
        bare["achieved_over_row_pass_mix"] = round(out["roofline"]["achieved"] / bare["row_pass_mix_GBps"], 3)
        bare["note"] = "bare kernels over as many rows (snap_stream_probe): a read of 4 B per row, a copy (4 in, 4 out), and " \
                       "the row pass's mix with two-byte maps (4 + 2 + 2 in, 4 out) that does nothing else; best launch shape each"
        out["roofline"]["bare_kernels"] = bare

    # ---- the accept check on top of the group sweeps: what it costs (config 4, auto) ------------------
    if args.mode == "auto" and cfg == 4:
        gc_ = snap.Solver.from_problem(p, adaptive=True, **kw)
        for e in range(3):
            gc_.epoch(100 + e)
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for e in range(args.steps):
            gc_.epoch(200 + e)
        torch.cuda.synchronize()
        ms_chk = 1e3 * (time.perf_counter() - t0) / args.steps
        gn = snap.Solver.from_problem(p, **kw)       # the same loop without events or check, as the reference
        for e in range(3):
            gn.epoch(100 + e)
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for e in range(args.steps):
            gn.epoch(200 + e)
        torch.cuda.synchronize()
        ms_plain = 1e3 * (time.perf_counter() - t0) / args.steps
        out["groups_with_accept_check"] = {
            "ms_per_step": round(ms_chk, 4), "ms_per_step_without": round(ms_plain, 4),
            "overhead_fraction": round(ms_chk / ms_plain - 1.0, 4),
            "what": "every epoch followed by the objective (loss summed by the epoch's last row pass, one small "
                    "reduction, one host synchronisation) and the accept / discard decision; the state before the "
                    "epoch is kept by writing into a second array, not by a copy"}
        gc_.close()
        gn.close()

    # ---- the structure-free asynchronous path on the same data (config 4, auto) --------------------
    if args.mode == "auto" and cfg == 4:
        ga = snap.Solver.from_problem(p, profile=True, max_inflight_nnz=args.inflight, damping=args.damping,
                                      auto_groups=False)
        steps_a = max(3, min(args.steps, 8))
        el, kma, sta, rej = timed_epochs(ga, torch, steps_a, 1, 9000)
        m = p.d
        ra = roofline_of(4, "async", p, p.nnz, m, False, sta, kma, 1e3 * el / steps_a, args.scale)
        out["async_general_path"] = {
            "value": m * steps_a / el, "unit": "coordinate updates/s", "steps": steps_a,
            "ms_per_step": 1e3 * el / steps_a,
            "epoch_contents": "key generation and sort, both epoch kernels, the accept check (state copy, objective)",
            "kernel_ms": {k: round(v, 4) for k, v in kma.items()}, "inflight_nnz": sta["inflight_nnz"],
            "rejected_epochs_in_sample": rej, "roofline": ra}
        if not args.no_gap:
            out["async_general_path"]["time_to_gap"] = time_to_gap(ga, np, torch, 1e3 * el / steps_a, args.gap_target,
                                                                   args.gap_max_epochs, args.gap_max_seconds)
        ga.close()

    # ---- CPU baseline: the oracle on the host cores, on a bounded sample of the same workload --------
    if not args.no_cpu_baseline:
        out["cpu_baseline"] = cpu_baseline(p, np)
    del p
    torch.cuda.empty_cache()

    # ---- the other configurations, fewer steps ------------------------------------------------------
    if args.config == 0 and not args.no_others:
        others = {}
        for c in (1, 2, 3, 5):
            k = 3 if c == 5 else max(3, min(args.steps, 10))
            w = 1 if c == 5 else max(1, min(args.warmup, 2))
            gc.collect()
            torch.cuda.empty_cache()
            free_b, total_b = torch.cuda.mem_get_info()
            print("bench.py: config %d next, device memory free %.1f of %.1f GiB" % (c, free_b / 2 ** 30, total_b / 2 ** 30),
                  file=sys.stderr, flush=True)
            try:
                r, _, _ = run_config(c, mode_of(c), k, w, args, mods, want_gap=not args.no_gap)
                others["config%d" % c] = r
            except Exception as e:                      # one config failing must not lose the headline
                traceback.print_exc()
                others["config%d" % c] = {"error": "%s: %s" % (type(e).__name__, str(e).splitlines()[0])}
        out["other_configs"] = others
    if args.calibrate:
        a = torch.zeros(1 << 28, dtype=torch.float32, device="cuda:0")
        b = torch.empty_like(a)
        torch.cuda.synchronize()
        torch.add(a, 1.0, out=b)
        torch.cuda.synchronize()
    print(json.dumps(out))


if __name__ == "__main__":
    main()
