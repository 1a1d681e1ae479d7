#!/usr/bin/env python3
"""Benchmark of the DMT tower hot path on one MI355X.

One step = one pass of the whole path over one synthetic batch:
    dmt_tower_lookup_fwd  ->  dmt_tower_module_fwd  ->  dmt_tower_lookup_bwd_update
on the "Mid" tables and lookups (64 fp16 tables x 1M rows x D=128, 8 towers of
8, batch 8192, Poisson(20) bags, Zipf 1.05 ids; dot-product Tower Module to 256
on bf16 MFMA), with the "Backward" configuration's sorted / segment-reduced
gradient and in-place rowwise Adagrad.  Inputs are resident in HBM before the
timed region.  Prints ONE JSON line; the same line carries, as `other_workloads`,
the Imbalanced step and the Large forward timed the same way.

The bytes that cross the L2 <-> fabric boundary per kernel are counted in this
run: before this process touches the GPU it runs itself twice per workload under
`rocprofv3 --pmc` (FETCH_SIZE, then WRITE_SIZE), a few steps plus a copy kernel of
known size that calibrates the counters.

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--batches N] [--no-cpu]
                    [--no-traffic] [--no-others] [--workload NAME]
"""
from __future__ import annotations

import argparse
import json
import os
import shutil
import signal
import subprocess
import sys
import tempfile
import time

import numpy as np

HBM_PEAK_GBS = 8000.0
MFMA_PEAK_TFLOPS_16BIT = 2500.0
RTILE = 128          # sorted records per reduce tile in the backward kernel (for byte accounting)
ROOT = os.path.dirname(os.path.abspath(__file__))
OTHERS = ("imbalanced", "large")


def parse():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=60)
    ap.add_argument("--warmup", type=int, default=10)
    ap.add_argument("--batches", type=int, default=8, help="pool of pre-generated id batches")
    ap.add_argument("--no-cpu", action="store_true", help="skip the CPU-oracle baseline leg")
    ap.add_argument("--workload", default="backward")
    ap.add_argument("--no-tm-bwd", action="store_true",
                    help="skip the separate timing of the Tower Module backward")
    ap.add_argument("--no-tp", action="store_true",
                    help="skip the separate timing of the Tower Partitioner")
    ap.add_argument("--no-traffic", action="store_true",
                    help="do not count L2 <-> fabric bytes under rocprofv3 (the committed summary "
                         "under profiles/ is quoted instead, and named as the source)")
    ap.add_argument("--no-others", action="store_true",
                    help="time only the named workload, not Imbalanced and Large beside it")
    ap.add_argument("--calibrate", action="store_true",
                    help="also run dmt_calibration_copy on 1 GiB three times (for rocprofv3 --pmc runs)")
    ap.add_argument("--traffic-out", default=None, metavar="DIR",
                    help="also write the counted bytes per kernel as bench_<workload>_hbm_traffic.txt "
                         "and .json into DIR (the form kept under profiles/)")
    ap.add_argument("--chunk-sweep", action="store_true",
                    help="instead of the step: lookup -> Tower Module run over the batch in 1, 2, 4 ... "
                         "chunks (each chunk a batch of its own), to see whether a pooled block that "
                         "stays in the caches between the two calls pays for the smaller launches")
    ap.add_argument("--gather-rates", action="store_true",
                    help="instead of the step: the rate of plain random row reads on this machine "
                         "(dmt_calibration_gather) from tables that fit the L2, the Infinity Cache, "
                         "or neither")
    ap.add_argument("--traffic-child", action="store_true", help=argparse.SUPPRESS)
    return ap.parse_args()


def log(*a):
    print(*a, file=sys.stderr, flush=True)


def batch_accounting(torch, w, idx, off):
    """Per-batch counts the algorithmic byte figures need, from the device tensors
    (torch sort / unique on the ids: bookkeeping of the benchmark, not part of the path).
    Returns per-table nnz and distinct rows, runs that span reduce tiles, partial slots."""
    F, B = w.num_tables, w.batch
    nnz = idx.numel()
    bounds = off[::B]
    nnz_f = (bounds[1:] - bounds[:-1])
    tab = torch.repeat_interleave(torch.arange(F, device=idx.device), nnz_f)
    key, _ = torch.sort((tab << 32) | idx.to(torch.int64))
    head = torch.ones(nnz, dtype=torch.bool, device=idx.device)
    head[1:] = key[1:] != key[:-1]
    U_f = torch.bincount((key[head] >> 32), minlength=F)
    edges = torch.arange(RTILE, nnz, RTILE, device=idx.device)
    crossing = key[edges] == key[edges - 1]
    seg_id = torch.cumsum(head.to(torch.int64), 0) - 1
    span = int(torch.unique(seg_id[edges[crossing]]).numel())
    return dict(nnz=nnz, nnz_f=nnz_f.cpu().numpy().astype(np.float64),
                U_f=U_f.cpu().numpy().astype(np.float64), U=int(head.sum().item()), span=span,
                partial_slots=int(crossing.sum().item()) + span)


# --------------------------------------------------------------------------------------------
# L2 <-> fabric bytes per kernel, counted under rocprofv3 in child runs of this same file
# --------------------------------------------------------------------------------------------

# kernel (as the profiler names it) -> the family dmt_kernel_name() reports
FAMILIES = (("lookup_fwd_kernel", "lookup_fwd"), ("bwd_reduce_update", "bwd_reduce_update"),
            ("bwd_fixup_update", "bwd_fixup_update"), ("bwd_build_keys", "bwd_build_keys"),
            ("radix_hist", "radix_hist"), ("radix_scan", "radix_scan"), ("radix_scatter", "radix_scatter"),
            ("tm_gemm", "tm_gemm"), ("tm_pack_w", "tm_pack_w"), ("tm_dots", "tm_dots"),
            ("dmt_copy_kernel", "copy"))
KERNEL_REGEX = "lookup_fwd|bwd_|radix_|tm_|dmt_copy"
CHILD_STEPS = 3
COPY_BYTES = 1 << 30


def traffic_child(args):
    """What runs under rocprofv3: CHILD_STEPS steps of the workload, then three copies of 1 GiB by
    dmt_copy_kernel (whose traffic is known exactly)."""
    import torch
    ctx = setup(args, args.workload, nb=2)
    for i in range(CHILD_STEPS):
        ctx["step"](i)
    dmt = ctx["dmt"]
    a = torch.empty(COPY_BYTES, dtype=torch.uint8, device="cuda")
    c = torch.ones(COPY_BYTES, dtype=torch.uint8, device="cuda")
    for _ in range(3):
        dmt.dmt_calibration_copy(a, c)
    torch.cuda.synchronize()
    return 0


def read_counter_db(path):
    """{family: [sum of the counter over the family's dispatches, dispatches]} from a rocprofv3
    results database."""
    import sqlite3
    con = sqlite3.connect(path)
    cur = con.execute("select * from counters_collection limit 1")
    cols = [d[0] for d in cur.description]
    ni = cols.index("kernel_name") if "kernel_name" in cols else cols.index("name")
    vi = cols.index("value")
    out = {}
    for r in con.execute("select * from counters_collection"):
        for pat, fam in FAMILIES:
            if pat in r[ni]:
                e = out.setdefault(fam, [0.0, 0])
                e[0] += float(r[vi])
                e[1] += 1
                break
    con.close()
    return out


def write_traffic_summary(outdir, name, cmds, scale, fam, per, source):
    """The text and JSON summaries of one workload's counter runs, in the form profiles/ keeps."""
    os.makedirs(outdir, exist_ok=True)
    base = os.path.join(outdir, "bench_%s_hbm_traffic" % name)
    with open(base + ".txt", "w") as f:
        f.write("L2 <-> memory-fabric bytes per kernel family on the %s workload, MI355X\n" % name)
        f.write("written by: python3 bench.py --traffic-out DIR, which ran (from /tmp, TMPDIR=/tmp):\n")
        for c in cmds:
            f.write("  " + c + "\n")
        f.write("(each child run: %d steps of the path, then dmt_copy_kernel on 1 GiB three times)\n" % CHILD_STEPS)
        f.write("calibration: the copy reads and writes 1048576 KiB; FETCH_SIZE scale %.4f, WRITE_SIZE scale %.4f\n"
                % (scale["FETCH_SIZE"], scale["WRITE_SIZE"]))
        f.write("the counters sit between L2 and the fabric: an Infinity-Cache hit counts like an HBM access\n\n")
        f.write("%-20s %10s %15s %15s %12s %12s %12s\n" % ("kernel family", "dispatches", "FETCH_raw_avg",
                                                          "WRITE_raw_avg", "read_MB/step", "write_MB/step", "MB/step"))
        for k in sorted(fam):
            v = fam[k]
            if "FETCH_SIZE" not in v or "WRITE_SIZE" not in v:
                continue
            fa = v["FETCH_SIZE"][0] / v["FETCH_SIZE"][1]
            wa = v["WRITE_SIZE"][0] / v["WRITE_SIZE"][1]
            if k == "copy":
                f.write("%-20s %10d %15.1f %15.1f %12s %12s %12s\n" % (k, v["FETCH_SIZE"][1], fa, wa, "-", "-", "-"))
            else:
                e = per[k]
                f.write("%-20s %10d %15.1f %15.1f %12.1f %12.1f %12.1f\n" %
                        (k, v["FETCH_SIZE"][1], fa, wa, e["read_bytes"] / 1e6, e["write_bytes"] / 1e6,
                         e["bytes"] / 1e6))
    with open(base + ".json", "w") as f:
        json.dump(dict(workload=name, source="profiles/bench_%s_hbm_traffic.txt (%s)" % (name, source),
                       fetch_scale=round(scale["FETCH_SIZE"], 4), write_scale=round(scale["WRITE_SIZE"], 4),
                       per_step=per), f, indent=1)
        f.write("\n")


def collect_traffic(names, outdir=None):
    """FETCH_SIZE and WRITE_SIZE (KiB per dispatch, L2 <-> fabric, so Infinity-Cache hits count)
    of every kernel family of the named workloads, from two rocprofv3 --pmc runs each of this
    file with --traffic-child; scaled by what the same counter reads for dmt_copy_kernel on
    1 GiB.  Runs BEFORE this process initialises the GPU.  {workload: {...} or {"error": ...}}."""
    exe = shutil.which("rocprofv3") or "/opt/rocm/bin/rocprofv3"
    res = {}
    if not os.path.exists(exe):
        return {n: {"error": "rocprofv3 not found"} for n in names}
    for name in names:
        fam = {}
        scale = {}
        err = None
        cmds = []
        for counter in ("FETCH_SIZE", "WRITE_SIZE"):
            tmp = tempfile.mkdtemp(prefix="dmt_pmc_", dir="/tmp")
            # (counters only on this library's kernels: the profiler has crashed while counting
            # on the generators that draw the Large workload's ids)
            cmd = [exe, "--pmc", counter, "--kernel-include-regex", KERNEL_REGEX, "-d", tmp, "-o", "p",
                   "--", sys.executable,
                   os.path.join(ROOT, "bench.py"), "--traffic-child", "--workload", name]
            env = dict(os.environ, TMPDIR="/tmp")
            cmds.append(" ".join(cmd[:4] + ["'%s'" % cmd[4], "-d", "<tmp>"] + cmd[7:9] + ["--", "python3", "bench.py"] + cmd[12:]))
            t0 = time.time()
            try:
                # the profiler and the child under it form a process group of their own, so that a
                # time-out ends both and nothing outlives this function
                pr = subprocess.Popen(cmd, cwd="/tmp", env=env, stdout=subprocess.DEVNULL,
                                      stderr=subprocess.PIPE, start_new_session=True)
                try:
                    _, stderr = pr.communicate(timeout=240)
                except subprocess.TimeoutExpired:
                    os.killpg(pr.pid, signal.SIGKILL)
                    pr.communicate()
                    raise
                if pr.returncode != 0:
                    err = "%s run exited with %d: %s" % (counter, pr.returncode, stderr.decode()[-200:])
                else:
                    dbs = [os.path.join(d, f) for d, _, fs in os.walk(tmp) for f in fs
                           if f.endswith("_results.db")]
                    if not dbs:
                        err = "%s run left no results database" % counter
                    else:
                        got = read_counter_db(dbs[0])
                        if "copy" not in got or got["copy"][0] <= 0:
                            err = "%s run has no calibration kernel" % counter
                        else:
                            scale[counter] = (COPY_BYTES / 1024.0) / (got["copy"][0] / got["copy"][1])
                            for k, (tot, n) in got.items():
                                fam.setdefault(k, {})[counter] = (tot, n)
            except Exception as e:                       # a missing profiler must not cost the bench line
                err = "%s run failed: %r" % (counter, e)
            finally:
                shutil.rmtree(tmp, ignore_errors=True)
            log("[bench] rocprofv3 --pmc %s on %s: %.1fs%s" %
                (counter, name, time.time() - t0, "" if err is None else " (" + err + ")"))
            if err:
                break
        if err:
            res[name] = {"error": err}
            continue
        per = {}
        for k, v in fam.items():
            if k == "copy" or "FETCH_SIZE" not in v or "WRITE_SIZE" not in v:
                continue
            rd = v["FETCH_SIZE"][0] * scale["FETCH_SIZE"] * 1024.0 / CHILD_STEPS
            wr = v["WRITE_SIZE"][0] * scale["WRITE_SIZE"] * 1024.0 / CHILD_STEPS
            per[k] = dict(read_bytes=int(rd), write_bytes=int(wr), bytes=int(rd + wr),
                          launches_per_step=v["FETCH_SIZE"][1] // CHILD_STEPS)
        res[name] = dict(per_step=per,
                         source="rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE child runs of this command "
                                "(%d steps each), scaled by dmt_copy_kernel on 1 GiB (factors %.3f / %.3f)"
                                % (CHILD_STEPS, scale["FETCH_SIZE"], scale["WRITE_SIZE"]))
        if outdir:
            write_traffic_summary(outdir, name, cmds, scale, fam, per, res[name]["source"])
    return res


def committed_traffic(name):
    """The committed summary of an earlier counter run of this command, when this run counted
    nothing itself."""
    tfile = os.path.join(ROOT, "profiles", "bench_%s_hbm_traffic.json" % name)
    if not os.path.exists(tfile):
        return None
    tj = json.load(open(tfile))
    per = {k: dict(bytes=int(v["bytes"]), launches_per_step=int(v.get("launches_per_step", 1)))
           for k, v in tj.get("per_step", tj.get("per_launch", {})).items()}
    return dict(per_step=per, source="committed: " + tj.get("source", tfile))


# --------------------------------------------------------------------------------------------
# one workload: set-up, timed steps, byte accounting
# --------------------------------------------------------------------------------------------

DTYPE_TEXT = {
    "backward": "f16 tables, bf16 pooled values and Tower Module on MFMA, f32 accumulation, gradients and state",
    "mid": "f16 tables, bf16 pooled values and Tower Module on MFMA, f32 accumulation",
    "mid_dlrm": "f16 tables, bf16 pooled values and Tower Module on MFMA, f32 accumulation",
    "large": "bf16 tables, pooled values and Tower Module on MFMA, f32 accumulation",
    "large_lowrank": "bf16 tables, pooled values and Tower Module on MFMA, f32 accumulation",
    "imbalanced": "f16 tables, pooled values and Tower Module on MFMA, f32 accumulation, gradients and state",
    "tiny": "f32",
}
NAMES = {"backward": "backward (Mid tables and lookups: lookup fwd + dot-product TM fwd + sorted "
                     "segment-reduce bwd + rowwise Adagrad)",
         "mid": "mid (lookup fwd + dot-product TM fwd)",
         "mid_dlrm": "mid tables (lookup fwd + DLRM TM fwd: flat 1024 -> 128 next to a shared 128 -> 32 "
                     "per feature)",
         "large": "large (lookup fwd + 2 cross layers + projection TM fwd)",
         "large_lowrank": "large tables (lookup fwd + 2 low-rank (r = 512) cross layers + projection TM fwd)",
         "imbalanced": "imbalanced (lookup fwd + linear TM fwd + bwd + rowwise Adagrad)",
         "tiny": "tiny"}


def setup(args, wname, nb):
    """Tables, id batches, plan, Tower Module weights and buffers of a workload, all resident on
    the device; `step(i)` enqueues one pass of the hot path on batch i of the pool."""
    import torch
    import paper_2403_00877_amd as dmt
    import workloads as wl

    torch.cuda.set_device(0)
    w = wl.by_name(wname)
    F, B, T = w.num_tables, w.batch, w.num_towers
    tdt = {"f32": torch.float32, "f16": torch.float16, "bf16": torch.bfloat16}
    on_device = w.name in ("large", "large_lowrank", "imbalanced")   # id streams too large for numpy

    t0 = time.time()
    tables = wl.tables_device(w)
    states = [torch.zeros(r, dtype=torch.float32, device="cuda") for r in w.rows] if w.backward else None
    torch.cuda.synchronize()
    log("[bench] %s: tables on device: %.1f GB in %.1fs" %
        (w.name, sum(t.numel() * t.element_size() for t in tables) / 1e9, time.time() - t0))

    cache = {}
    batches = []
    t0 = time.time()
    base_w, widths_w, _ = wl.pooled_layout(w)
    for i in range(nb):
        host = None
        if on_device:
            d_idx, d_off = wl.lookup_batch_device(w, i)
        else:
            idx, off = wl.lookup_batch(w, i, cache)
            d_idx, d_off = torch.from_numpy(idx).cuda(), torch.from_numpy(off).cuda()
        grad = None
        if w.backward:
            if on_device:
                g = torch.Generator(device="cuda")
                g.manual_seed(1000 * w.seed + i)
                grad = torch.randn(base_w[-1], generator=g, device="cuda", dtype=torch.float32)
            else:
                hg = wl.grad_pooled(w, i)
                grad = torch.from_numpy(hg).cuda()
                if i == 0:
                    host = (idx, off, hg)
        batches.append(dict(idx=d_idx, off=d_off, grad=grad, host=host,
                            acct=None if args.traffic_child else batch_accounting(torch, w, d_idx, d_off)))
    log("[bench] %d batches generated in %.1fs" % (len(batches), time.time() - t0))
    max_nnz = max(b["idx"].numel() for b in batches)

    plan = dmt.dmt_plan_create(w.rows, w.dims, w.table_dtype, T, w.table_to_tower, B, max_nnz)
    dmt.dmt_plan_bind(plan, tables, states)
    base, widths, col = dmt.dmt_plan_layout(plan, B)

    def dev(a, dt):
        t = torch.from_numpy(wl.encode(a, dt))
        return (t.view(torch.int16).view(torch.bfloat16) if dt == "bf16" else t).cuda()

    tm_host = wl.tm_weights(w)
    tm_dev = [dict(kind=w.tm_kind, out_dim=w.tm_out[t], w_proj=dev(h["w_proj"], w.tm_dtype),
                   b_proj=dev(h["b_proj"], w.tm_dtype),
                   w_cross=[dev(a, w.tm_dtype) for a in h["w_cross"]],
                   b_cross=[dev(a, w.tm_dtype) for a in h["b_cross"]], feat_out=w.tm_feat_out)
              for t, h in enumerate(tm_host)]
    tm_params = dmt.make_tm_params(tm_dev)
    tm_ws = torch.empty(max(dmt.dmt_tm_workspace_bytes(plan, tm_params, B), 256), dtype=torch.uint8,
                        device="cuda")
    bwd_ws = None
    if w.backward:
        bwd_ws = torch.empty(max(dmt.dmt_bwd_workspace_bytes(plan, B, max_nnz), 256), dtype=torch.uint8,
                             device="cuda")
    pooled = torch.empty(base[-1], dtype=tdt[w.pooled_dtype], device="cuda")
    tm_out = torch.empty(B * sum(w.tm_out), dtype=tdt[w.tm_dtype], device="cuda")

    def step(i):
        b = batches[i % len(batches)]
        dmt.dmt_tower_lookup_fwd(plan, b["idx"], b["off"], B, pooled)
        dmt.dmt_tower_module_fwd(plan, tm_params, pooled, B, tm_out, tm_ws)
        if w.backward:
            dmt.dmt_tower_lookup_bwd_update(plan, b["idx"], b["off"], B, b["grad"], w.lr, w.eps, bwd_ws)

    return dict(torch=torch, dmt=dmt, wl=wl, w=w, tables=tables, states=states, batches=batches, plan=plan,
                widths=widths, tm_host=tm_host, tm_dev=tm_dev, tm_params=tm_params, tm_ws=tm_ws,
                bwd_ws=bwd_ws, pooled=pooled, tm_out=tm_out, step=step)


def run_workload(args, wname, traffic, primary):
    """Times `wname` and returns its result object: the whole bench line for the primary
    workload, the same fields without the side measurements for the others."""
    default = wname == "backward"
    nb = args.batches if default else min(args.batches, 2)
    ctx = setup(args, wname, nb)
    torch, dmt, wl, w = ctx["torch"], ctx["dmt"], ctx["wl"], ctx["w"]
    plan, batches, step = ctx["plan"], ctx["batches"], ctx["step"]
    tables, states, pooled, tm_out = ctx["tables"], ctx["states"], ctx["pooled"], ctx["tm_out"]
    tm_params, tm_ws, bwd_ws, widths = ctx["tm_params"], ctx["tm_ws"], ctx["bwd_ws"], ctx["widths"]
    F, B, T = w.num_tables, w.batch, w.num_towers
    eb = wl.ELT_BYTES[w.table_dtype]
    eo = wl.ELT_BYTES[w.pooled_dtype]
    a0 = batches[0]["acct"]
    log("[bench] %s: nnz %d, unique rows %d (%.0f%% duplicates)" %
        (w.name, a0["nnz"], a0["U"], 100 * (1 - a0["U"] / max(a0["nnz"], 1))))

    # ---- CPU oracle leg: baseline timing + a live parity check on the same inputs
    cpu = None
    if primary and default and not args.no_cpu:
        cpu = cpu_leg(dmt, wl, w, plan, tables, states, ctx["tm_host"], batches[0], pooled, tm_out, tm_params,
                      tm_ws, bwd_ws, widths)
        for s in states:                      # restart the optimizer state for the timed run
            s.zero_()

    # ---- timed region: exactly args.steps steps between two synchronisations; an event pair
    # around every step (on the stream the kernels are launched on) gives the spread
    for i in range(args.warmup):
        step(i)
    torch.cuda.synchronize()
    timed = ["lookup_fwd", "tm_gemm", "radix_scatter", "bwd_reduce_update"]
    name_to_id = {dmt.dmt_kernel_name(i): i for i in range(dmt.DMT_K_COUNT)}
    dmt.dmt_profile_enable(plan, sum(1 << name_to_id[n] for n in timed))
    ev = [(torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True))
          for _ in range(args.steps)]
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for i in range(args.steps):
        ev[i][0].record()
        step(args.warmup + i)
        ev[i][1].record()
    torch.cuda.synchronize()
    elapsed = time.perf_counter() - t0
    prof = dmt.dmt_profile_read(plan)
    ms_per_step = elapsed * 1e3 / args.steps
    # the spread is reported over at least 50 steps: when fewer were asked for, more steps follow
    # the timed region (they do not enter `value`), each with its own event pair
    extra = max(0, 50 - args.steps)
    ev += [(torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True))
           for _ in range(extra)]
    for i in range(args.steps, args.steps + extra):
        ev[i][0].record()
        step(args.warmup + i)
        ev[i][1].record()
    torch.cuda.synchronize()
    if extra:
        dmt.dmt_profile_read(plan)                  # (their kernel timings are dropped)
    per_step_ms = np.array([a.elapsed_time(b) for a, b in ev])
    assert dmt.dmt_last_device_error(plan) == -1

    # ---- per-kernel breakdown (outside the timed region, every family timed)
    dmt.dmt_profile_enable(plan, (1 << dmt.DMT_K_COUNT) - 1)
    for i in range(nb):
        step(args.warmup + args.steps + i)
    full = dmt.dmt_profile_read(plan)
    dmt.dmt_profile_enable(plan, 0)

    # ---- Tower Module backward, timed on its own after the step (it is not part of `value`)
    tm_bwd = None
    if primary and not args.no_tm_bwd:
        tm_bwd = time_tm_bwd(torch, dmt, wl, w, plan, tm_params, pooled, tm_out, tm_ws, B, args.steps)
        if w.backward:
            tm_bwd["whole_tower_step"] = time_whole_step(torch, dmt, wl, w, plan, tm_params, pooled, tm_out,
                                                         tm_ws, bwd_ws, batches, B, args.steps)

    # ---- Tower Partitioner on this batch's pooled embeddings (not part of `value`)
    tp_out = None
    if primary and not args.no_tp and len(set(w.dims)) == 1 and w.dims[0] % 8 == 0:
        dmt.dmt_tower_lookup_fwd(plan, batches[0]["idx"], batches[0]["off"], B, pooled)
        tp_out = time_tower_partitioner(torch, dmt, wl, w, plan, pooled, B, args.steps,
                                        with_oracle=default and not args.no_cpu)

    # ---- SPTT's explicit shuffle steps on a buffer the size of the pooled tensor (not part of `value`)
    sptt_out = None if (args.no_tp or not primary) else time_sptt_shuffles(torch, dmt, pooled, F, args.steps)

    if args.calibrate:
        a = torch.empty(1 << 30, dtype=torch.uint8, device="cuda")
        c = torch.ones(1 << 30, dtype=torch.uint8, device="cuda")
        for _ in range(3):
            dmt.dmt_calibration_copy(a, c)
        torch.cuda.synchronize()

    # ---- bytes per step, averaged over the batches the timed steps used.  Three figures per
    # gather / scatter kernel: LOGICAL (every lookup's row or gradient slice counted, whether a
    # cache served it or not), COMPULSORY (each distinct row and each gradient slice once) and
    # MEASURED (the L2 <-> fabric counters).
    used = [batches[(args.warmup + i) % nb]["acct"] for i in range(args.steps)]
    mean = lambda k: np.mean([u[k] for u in used], axis=0)
    nnz, U, span, pslots = float(mean("nnz")), float(mean("U")), float(mean("span")), float(mean("partial_slots"))
    nnz_f, U_f = mean("nnz_f"), mean("U_f")
    Df = np.array(w.dims, dtype=np.float64)
    Dmax = float(Df.max())
    logical = {
        # per lookup: row + id; per bag: offset + pooled store
        "lookup_fwd": float((nnz_f * (Df * eb + 4) + B * (8 + Df * eo)).sum()),
        # per lookup: sorted record + gradient slice; per row finished in-tile: row read + write and
        # state read + write; partial sums of rows that span tiles
        "bwd_reduce_update": float((nnz_f * (8 + Df * 4) + U_f * (2 * Df * eb + 8)).sum()
                                   - span * (2 * Dmax * eb + 8) + pslots * Dmax * 4),
        # one radix pass: records read and written
        "radix_scatter": nnz * 16,
    }
    compulsory = {
        # each distinct row once; ids, offsets and the pooled store as they are
        "lookup_fwd": float((U_f * Df * eb + nnz_f * 4 + B * (8 + Df * eo)).sum()),
        # each bag's gradient slice once, every sorted record once, each distinct row read and
        # written once with its state
        "bwd_reduce_update": float((B * Df * 4 + nnz_f * 8 + U_f * (2 * Df * eb + 8)).sum()),
        "radix_scatter": nnz * 16,
    }
    kin = w.tm_in_dims()
    tw = w.tower_widths()
    nl = w.tm_cross_layers if w.tm_kind == wl.TM_CROSS_LINEAR else 0
    tm_fwd_flops = tm_flops(wl, w, B)[0]
    tm_bytes = sum(B * (d * eo * (1 + 3 * nl) + o * eo) + (o * k + nl * d * d) * eo
                   for o, k, d in zip(w.tm_out, kin, tw))
    kernels = {}
    for name, (ms, n) in sorted(full.items()):
        kernels[name] = dict(ms_per_launch=round(ms / n, 4), launches_per_step=n // nb,
                             ms_per_step=round(ms / nb, 4))
    if traffic is None or "per_step" not in traffic:
        if traffic is not None:
            log("[bench] no traffic counted for %s: %s" % (wname, traffic.get("error")))
        traffic = committed_traffic(wname)
    measured = traffic["per_step"] if traffic else {}

    def describe(name):
        """Roofline entry of one kernel family from the timed region (all its launches of a step
        taken together).  For the kernels bound by memory `achieved` and `frac` are the MEASURED
        rate when the counters are there (never the logical one: a cache-served byte is no HBM
        byte), else the compulsory rate."""
        ms, n = prof[name]
        per_step = ms / args.steps
        launches = n // args.steps
        sec = per_step * 1e-3
        mt = measured.get(name, {}).get("bytes")
        if name in logical:
            mult = launches if name == "radix_scatter" else 1      # its byte figures are per pass
            lg, cp = logical[name] * mult / sec / 1e9, compulsory[name] * mult / sec / 1e9
            mg = mt / sec / 1e9 if mt else None
            ach = mg if mg is not None else cp
            return dict(kernel=name, bound="hbm", achieved=round(ach, 1), peak=HBM_PEAK_GBS, unit="GB/s",
                        frac=round(ach / HBM_PEAK_GBS, 4),
                        achieved_is="measured L2<->fabric bytes / time" if mg is not None
                        else "compulsory bytes / time (no counters in this run)",
                        traffic=int(mt) if mt else None,
                        logical_GBs=round(lg, 1), compulsory_GBs=round(cp, 1),
                        measured_GBs=round(mg, 1) if mg is not None else None,
                        traffic_over_compulsory=round(mt / (compulsory[name] * mult), 3) if mt else None,
                        ms_per_launch=round(per_step / launches, 4), launches_per_step=launches,
                        logical_bytes=int(logical[name] * mult), compulsory_bytes=int(compulsory[name] * mult))
        tf = tm_fwd_flops / sec / 1e12
        g = tm_bytes / sec / 1e9
        mg = mt / sec / 1e9 if mt else None
        # the Tower Module's contraction is bound by whichever roof its FLOP per byte puts lower
        if tm_fwd_flops / tm_bytes < MFMA_PEAK_TFLOPS_16BIT * 1e12 / (HBM_PEAK_GBS * 1e9):
            ach = mg if mg is not None else g
            return dict(kernel=name, bound="hbm", achieved=round(ach, 1), peak=HBM_PEAK_GBS, unit="GB/s",
                        frac=round(ach / HBM_PEAK_GBS, 4),
                        achieved_is="measured L2<->fabric bytes / time" if mg is not None
                        else "algorithmic bytes / time (no counters in this run)",
                        traffic=int(mt) if mt else None, algorithmic_GBs=round(g, 1),
                        measured_GBs=round(mg, 1) if mg is not None else None,
                        traffic_over_algorithmic=round(mt / tm_bytes, 3) if mt else None,
                        ms_per_launch=round(per_step / launches, 4), launches_per_step=launches,
                        algorithmic_bytes=int(tm_bytes), algorithmic_flops=int(tm_fwd_flops),
                        achieved_TFLOPs=round(tf, 2))
        return dict(kernel=name, bound="mfma", achieved=round(tf, 2), peak=MFMA_PEAK_TFLOPS_16BIT,
                    unit="TFLOP/s", frac=round(tf / MFMA_PEAK_TFLOPS_16BIT, 4),
                    traffic=int(mt) if mt else None,
                    ms_per_launch=round(per_step / launches, 4), launches_per_step=launches,
                    algorithmic_flops=int(tm_fwd_flops), algorithmic_GBs=round(g, 1))

    dom = max(prof.items(), key=lambda kv: kv[1][0])[0]
    roofline = describe(dom)
    if traffic:
        roofline["traffic_source"] = traffic["source"]
    others = {n: describe(n) for n in timed if n in prof and n != dom}

    out = {
        "metric": "tower lookup+TM samples/sec; achieved HBM GB/s and % of peak (fwd, bwd)",
        "value": round(B / (ms_per_step * 1e-3), 1),
        "unit": "samples/s",
        "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": round(ms_per_step, 4),
        "ms_per_step_median": round(float(np.median(per_step_ms)), 4),
        "ms_per_step_p10": round(float(np.percentile(per_step_ms, 10)), 4),
        "ms_per_step_p90": round(float(np.percentile(per_step_ms, 90)), 4),
        "ms_per_step_samples": int(len(per_step_ms)),
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": DTYPE_TEXT[w.name], "data": "synthetic",
        "config": {"workload": NAMES[w.name], "tables": F, "rows": [min(w.rows), max(w.rows)],
                   "dims": sorted(set(w.dims)), "table_dtype": w.table_dtype, "towers": T, "batch": B,
                   "mean_nnz": int(nnz), "mean_unique_rows": int(U),
                   "duplicate_fraction": round(1 - U / max(nnz, 1.0), 3), "id_batches": nb},
        "roofline": roofline,
        "other_kernels": others,
        "kernel_breakdown": kernels,
    }
    if primary:
        out.update({
            "cpu_baseline": cpu["baseline"] if cpu else None,
            "parity_vs_oracle_on_sample": cpu["parity"] if cpu else None,
            "tm_backward": tm_bwd,
            "tower_partitioner": tp_out,
            "sptt_shuffle_steps": sptt_out,
        })
    else:
        for k in ("metric", "n_gpus", "higher_is_better", "scaling", "vs_baseline", "data"):
            out.pop(k)
    return out


def chunk_sweep(args):
    """Lookup -> Tower Module over the whole batch as k chunks of B / k samples, k = 1, 2, 4 ...:
    the existing entry points called on batch slices (a chunk's pooled block is B / k rows of
    every tower, written by the lookup and read back by the Tower Module right after).  One JSON
    line; the time is per WHOLE batch, so k = 1 is the ordinary forward."""
    import torch
    import paper_2403_00877_amd as dmt
    import workloads as wl
    name = args.workload
    w0 = wl.by_name(name)
    tdt = {"f32": torch.float32, "f16": torch.float16, "bf16": torch.bfloat16}
    tables = wl.tables_device(w0)

    def dev(a, dt):
        t = torch.from_numpy(wl.encode(a, dt))
        return (t.view(torch.int16).view(torch.bfloat16) if dt == "bf16" else t).cuda()

    tm_dev = [dict(kind=w0.tm_kind, out_dim=w0.tm_out[t], w_proj=dev(h["w_proj"], w0.tm_dtype),
                   b_proj=dev(h["b_proj"], w0.tm_dtype), w_cross=[dev(a, w0.tm_dtype) for a in h["w_cross"]],
                   b_cross=[dev(a, w0.tm_dtype) for a in h["b_cross"]], feat_out=w0.tm_feat_out)
              for t, h in enumerate(wl.tm_weights(w0))]
    on_device = w0.name in ("large", "large_lowrank", "imbalanced")
    rows = []
    k = 1
    while k <= 64 and w0.batch // k >= 256:
        w = wl.by_name(name)
        w.batch = B = w0.batch // k
        chunks = []
        for i in range(k):                      # k different chunks, ids drawn per chunk
            if on_device:
                d_idx, d_off = wl.lookup_batch_device(w, i)
            else:
                idx, off = wl.lookup_batch(w, i)
                d_idx, d_off = torch.from_numpy(idx).cuda(), torch.from_numpy(off).cuda()
            chunks.append((d_idx, d_off))
        max_nnz = max(c[0].numel() for c in chunks)
        plan = dmt.dmt_plan_create(w.rows, w.dims, w.table_dtype, w.num_towers, w.table_to_tower, B, max_nnz)
        dmt.dmt_plan_bind(plan, tables, None)
        base, _, _ = dmt.dmt_plan_layout(plan, B)
        tm_params = dmt.make_tm_params(tm_dev)
        tm_ws = torch.empty(max(dmt.dmt_tm_workspace_bytes(plan, tm_params, B), 256), dtype=torch.uint8,
                            device="cuda")
        pooled = [torch.empty(base[-1], dtype=tdt[w.pooled_dtype], device="cuda") for _ in range(min(k, 2))]
        tm_out = torch.empty(B * sum(w.tm_out), dtype=tdt[w.tm_dtype], device="cuda")

        def whole():
            for i, (d_idx, d_off) in enumerate(chunks):
                p = pooled[i % len(pooled)]
                dmt.dmt_tower_lookup_fwd(plan, d_idx, d_off, B, p)
                dmt.dmt_tower_module_fwd(plan, tm_params, p, B, tm_out, tm_ws)

        for _ in range(3):
            whole()
        torch.cuda.synchronize()
        n = max(5, min(args.steps, 20))
        t0 = time.perf_counter()
        for _ in range(n):
            whole()
        torch.cuda.synchronize()
        ms = (time.perf_counter() - t0) * 1e3 / n
        dmt.dmt_profile_enable(plan, (1 << dmt.DMT_K_COUNT) - 1)
        for _ in range(5):
            whole()
        prof = dmt.dmt_profile_read(plan)
        dmt.dmt_profile_enable(plan, 0)
        rows.append(dict(chunks=k, samples_per_chunk=B,
                         pooled_MB_per_chunk=round(pooled[0].numel() * pooled[0].element_size() / 1e6, 1),
                         ms_per_whole_batch=round(ms, 4),
                         kernel_ms_per_whole_batch={kk: round(v[0] / 5, 4) for kk, v in prof.items()}))
        log("[bench] %s in %d chunks: %.3f ms per whole batch" % (name, k, ms))
        del plan
        k *= 2
    print(json.dumps({"chunk_sweep": {"workload": name, "what": "lookup_fwd -> tower_module_fwd per chunk, "
                                      "ms per whole batch", "rows": rows}}), flush=True)
    return 0


def gather_rates(args):
    """What rows at random addresses reach on this machine, with a kernel that does nothing else:
    uniform random ids, 64-, 256- and 512-byte rows, tables of 2 MiB (inside one XCD's L2), 64 MiB
    (inside the Infinity Cache), 1 GiB and 16 GiB.  One JSON line."""
    import torch
    import paper_2403_00877_amd as dmt
    n = 1 << 25
    out = torch.empty(dmt.binding.DMT_CALIBRATION_GATHER_BLOCKS * 256 * 16, dtype=torch.uint8, device="cuda")
    rows_out = []
    for table_bytes in (2 << 20, 64 << 20, 1 << 30, 16 << 30):
        table = torch.zeros(table_bytes, dtype=torch.uint8, device="cuda")
        for row_bytes in (64, 256, 512):
            g = torch.Generator(device="cuda")
            g.manual_seed(table_bytes // row_bytes)
            ids = torch.randint(0, table_bytes // row_bytes, (n,), generator=g, device="cuda", dtype=torch.int32)
            for _ in range(3):
                dmt.dmt_calibration_gather(table, row_bytes, ids, out)
            a, b = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            reps = 10
            a.record()
            for _ in range(reps):
                dmt.dmt_calibration_gather(table, row_bytes, ids, out)
            b.record()
            torch.cuda.synchronize()
            ms = a.elapsed_time(b) / reps
            rows_out.append(dict(table_MiB=table_bytes >> 20, row_bytes=row_bytes, rows_gathered=n,
                                 ms=round(ms, 4), row_GBs=round(n * row_bytes / ms / 1e6, 1),
                                 rows_per_us=round(n / ms / 1e3, 1)))
            log("[bench] gather: table %6d MiB, %3d-byte rows: %.3f ms, %.0f GB/s" %
                (table_bytes >> 20, row_bytes, ms, n * row_bytes / ms / 1e6))
        del table
    print(json.dumps({"gather_rates": {"what": "dmt_calibration_gather, uniform random ids, 2^25 rows per launch",
                                       "rows": rows_out}}), flush=True)
    return 0


def main():
    args = parse()
    if args.gpus != 1:
        print("bench.py: this build runs on ONE GPU only (no collectives, no sharding); "
              "--gpus %d is not supported" % args.gpus, file=sys.stderr)
        return 2
    if args.traffic_child:
        return traffic_child(args)
    if args.chunk_sweep:
        return chunk_sweep(args)
    if args.gather_rates:
        return gather_rates(args)
    with_others = args.workload == "backward" and not args.no_others
    names = [args.workload] + (list(OTHERS) if with_others else [])
    # the counter runs come first: children of a process that has not touched the GPU yet
    traffic = {} if args.no_traffic else collect_traffic(names, args.traffic_out)
    out = run_workload(args, args.workload, traffic.get(args.workload), primary=True)
    if with_others:
        import gc
        import torch
        out["other_workloads"] = {}
        for n in OTHERS:
            gc.collect()
            torch.cuda.empty_cache()
            try:                                   # the default line must not hang on a side workload
                out["other_workloads"][n] = run_workload(args, n, traffic.get(n), primary=False)
            except Exception as e:
                log("[bench] %s failed: %r" % (n, e))
                out["other_workloads"][n] = {"error": repr(e)}
    print(json.dumps(out), flush=True)
    return 0


def time_sptt_shuffles(torch, dmt, pooled, F, steps, G=8, L=4):
    """Steps c and e of Sec. 3.1.1 in their explicit form, on a buffer of the pooled tensor's size
    read as [features][G ranks][block] resp. [features][peers][block]: pure data movement, timed by
    events on the launch stream against the HBM peak (bytes read + bytes written)."""
    nbytes = pooled.numel() * pooled.element_size()
    if nbytes % (F * G * 16) != 0:
        return None
    block = nbytes // (F * G)
    src = pooled.view(torch.uint8)
    dst = torch.empty_like(src)
    out = dict(features=F, ranks=G, per_host=L, block_bytes=block, bytes_moved=2 * nbytes)
    for name, call in (("peer_permute", lambda: dmt.dmt_sptt_peer_permute(src, dst, F, G, L, block)),
                       ("shuffle", lambda: dmt.dmt_sptt_shuffle(src, dst, F, G, block))):
        for _ in range(3):
            call()
        a, b = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        a.record()
        for _ in range(steps):
            call()
        b.record()
        torch.cuda.synchronize()
        ms = a.elapsed_time(b) / steps
        g = 2 * nbytes / (ms * 1e-3) / 1e9
        out[name] = dict(ms=round(ms, 4), bound="hbm", achieved=round(g, 1), peak=HBM_PEAK_GBS, unit="GB/s",
                         frac=round(g / HBM_PEAK_GBS, 4))
    return out


def time_tower_partitioner(torch, dmt, wl, w, plan, pooled, B, steps, with_oracle):
    """The Tower Partitioner (Sec. 3.3) on the pooled embeddings of one batch: the interaction
    matrix on the device (timed per launch by HIP events), then the embedding by Adam and the
    constrained K-means on the host, with as many towers as the workload has."""
    F, N, T = w.num_tables, w.dims[0], w.num_towers
    eo = wl.ELT_BYTES[w.pooled_dtype]
    ws = torch.empty(max(16, dmt.dmt_tp_workspace_bytes(plan, B)), dtype=torch.uint8, device="cuda")
    I = torch.empty(F, F, dtype=torch.float32, device="cuda")
    for _ in range(3):
        dmt.dmt_tp_interaction(plan, pooled, B, I, ws)
    torch.cuda.synchronize()
    name_to_id = {dmt.dmt_kernel_name(i): i for i in range(dmt.DMT_K_COUNT)}
    dmt.dmt_profile_enable(plan, (1 << name_to_id["tp_gram"]) | (1 << name_to_id["tp_finish"]))
    t0 = time.perf_counter()
    for _ in range(steps):
        dmt.dmt_tp_interaction(plan, pooled, B, I, ws)
    torch.cuda.synchronize()
    ms = (time.perf_counter() - t0) * 1e3 / steps
    prof = dmt.dmt_profile_read(plan)
    dmt.dmt_profile_enable(plan, 0)
    gram_ms = prof["tp_gram"][0] / prof["tp_gram"][1]
    fin_ms = prof["tp_finish"][0] / prof["tp_finish"][1]
    nbytes = B * F * N * eo                       # every pooled embedding read once
    flops = 2.0 * B * F * F * N
    I_host = I.cpu().numpy()
    x0, start = wl.tp_start(w.seed, F, 2, T)
    t0 = time.perf_counter()
    x, stress = dmt.dmt_tp_embed(I_host, "coherent", 2, 2000, 0.02, x0)
    embed_ms = (time.perf_counter() - t0) * 1e3
    t0 = time.perf_counter()
    labels, _, it = dmt.dmt_tp_kmeans(x, T, 1.0, x[start])
    kmeans_ms = (time.perf_counter() - t0) * 1e3
    sizes = np.bincount(labels, minlength=T)
    out = dict(features=F, dim=N, towers=T, batch=B,
               interaction_ms=round(ms, 4), samples_per_s=round(B / (ms * 1e-3), 1),
               tp_gram=dict(ms_per_launch=round(gram_ms, 4), bound="hbm", algorithmic_bytes=int(nbytes),
                            achieved=round(nbytes / (gram_ms * 1e-3) / 1e9, 1), peak=HBM_PEAK_GBS,
                            unit="GB/s", frac=round(nbytes / (gram_ms * 1e-3) / 1e9 / HBM_PEAK_GBS, 4),
                            tflops=round(flops / (gram_ms * 1e-3) / 1e12, 2)),
               tp_finish_ms=round(fin_ms, 4),
               host=dict(embed_ms=round(embed_ms, 2), adam_steps=2000, stress=round(stress, 4),
                         kmeans_ms=round(kmeans_ms, 2), kmeans_assignment_steps=it,
                         tower_sizes=[int(sizes.min()), int(sizes.max())]))
    if with_oracle:
        from oracle import tp as otp
        nb = min(B, 512)                          # a bounded sample of the batch for the CPU oracle
        R = np.zeros((nb, F, N))
        base, widths, col = wl.pooled_layout(w)
        host = pooled.float().cpu().numpy()
        for f in range(F):
            t = w.table_to_tower[f]
            R[:, f, :] = host[base[t]:base[t + 1]].reshape(B, widths[t])[:nb, col[f]:col[f] + N]
        t0 = time.perf_counter()
        I_ref = otp.tp_interaction(R)
        dt = time.perf_counter() - t0
        out["cpu_oracle"] = dict(samples_per_s=round(nb / dt, 1), sample="first %d samples of the batch" % nb,
                                 kind="oracle")
    return out


def tm_grad_buffers(torch, wl, w):
    """Float32 device buffers for every parameter gradient of the workload's Tower Modules."""
    kin, tw = w.tm_in_dims(), w.tower_widths()
    f32 = lambda *shape: torch.empty(shape, dtype=torch.float32, device="cuda")
    out = []
    for o, k, d, fs in zip(w.tm_out, kin, tw, w.tower_tables()):
        if w.tm_kind == wl.TM_DLRM:
            po = o - len(fs) * w.tm_feat_out
            out.append(dict(dw_proj=f32(po, d), db_proj=f32(po), dw_cross=[f32(w.tm_feat_out, d // len(fs))],
                            db_cross=[f32(w.tm_feat_out)]))
        elif w.tm_kind == wl.TM_CROSS_LOWRANK_LINEAR:
            r = w.tm_feat_out
            out.append(dict(dw_proj=f32(o, k), db_proj=f32(o),
                            dw_cross=[f32(*sh) for _ in range(w.tm_cross_layers) for sh in ((r, d), (d, r))],
                            db_cross=[f32(d) for _ in range(w.tm_cross_layers)]))
        else:
            nl = w.tm_cross_layers if w.tm_kind == wl.TM_CROSS_LINEAR else 0
            out.append(dict(dw_proj=f32(o, k), db_proj=f32(o), dw_cross=[f32(d, d) for _ in range(nl)],
                            db_cross=[f32(d) for _ in range(nl)]))
    return out


def tm_flops(wl, w, B):
    """(forward, backward with recomputation, backward on kept activations) FLOPs of the Tower
    Modules' contractions: a projection counts once forward and twice backward (data and weight
    gradient); a full-rank cross layer d^2 forward, 2 d^2 backward plus d^2 recomputed; a low-rank
    one 2 d r forward (t and u), 4 d r backward plus t recomputed always and u unless kept."""
    kin, tw = w.tm_in_dims(), w.tower_widths()
    fwd = bwd = kept = 0.0
    for o, k, d, fs in zip(w.tm_out, kin, tw, w.tower_tables()):
        proj, cf, cb, ck = o * k, 0, 0, 0
        if w.tm_kind == wl.TM_DLRM:
            proj = (o - len(fs) * w.tm_feat_out) * d + w.tm_feat_out * d
        elif w.tm_kind == wl.TM_CROSS_LINEAR:
            cf, cb, ck = d * d, 3 * d * d, 2 * d * d
        elif w.tm_kind == wl.TM_CROSS_LOWRANK_LINEAR:
            dr = d * w.tm_feat_out
            cf, cb, ck = 2 * dr, 6 * dr, 5 * dr
        fwd += 2.0 * B * (proj + w.tm_cross_layers * cf)
        bwd += 2.0 * B * (2 * proj + w.tm_cross_layers * cb)
        kept += 2.0 * B * (2 * proj + w.tm_cross_layers * ck)
    return fwd, bwd, kept


def time_tm_bwd(torch, dmt, wl, w, plan, tm_params, pooled, tm_out, tm_ws, B, steps):
    """dmt_tower_module_bwd on the step's pooled / tm_out tensors and a N(0,1) output gradient:
    ms per call, its kernels' shares, and the MFMA rate over the contractions' FLOPs (each
    projection twice: data and weight gradient; each cross layer three times: recomputed
    forward, data and weight gradient)."""
    tw = w.tower_widths()
    grads = tm_grad_buffers(torch, wl, w)
    arr = dmt.make_tm_grads(grads)
    ws = torch.empty(dmt.dmt_tm_bwd_workspace_bytes(plan, tm_params, B), dtype=torch.uint8, device="cuda")
    g = torch.Generator(device="cuda")
    g.manual_seed(7 + w.seed)
    dy = torch.randn(B * sum(w.tm_out), generator=g, device="cuda", dtype=torch.float32)
    dx = torch.empty(B * sum(tw), dtype=torch.float32, device="cuda")
    run = lambda: dmt.dmt_tower_module_bwd(plan, tm_params, pooled, tm_out, B, dy, dx, arr, ws)
    for _ in range(3):
        run()
    torch.cuda.synchronize()
    n = max(3, min(steps, 20))
    t0 = time.perf_counter()
    for _ in range(n):
        run()
    torch.cuda.synchronize()
    ms = (time.perf_counter() - t0) * 1e3 / n
    dmt.dmt_profile_enable(plan, (1 << dmt.DMT_K_COUNT) - 1)
    for _ in range(n):
        run()
    prof = dmt.dmt_profile_read(plan)
    dmt.dmt_profile_enable(plan, 0)
    _, flops, flops_kept = tm_flops(wl, w, B)
    gemm_ms = prof.get("tm_bwd_gemm", (0.0, 0))[0] / n
    out = dict(ms_per_call=round(ms, 4), workspace_GB=round(ws.numel() / 1e9, 3),
               kernels={k: dict(ms_per_call=round(v[0] / n, 4), launches_per_call=v[1] // n)
                        for k, v in sorted(prof.items())},
               algorithmic_flops=int(flops),
               gemm_TFLOPs=round(flops / (gemm_ms * 1e-3) / 1e12, 1) if gemm_ms > 0 else None,
               mfma_peak_TFLOPs=MFMA_PEAK_TFLOPS_16BIT)
    # with the cross layers' activations kept by a training forward instead of recomputed
    kept_bytes = dmt.dmt_tm_kept_bytes(plan, tm_params, B, w.tm_dtype)
    if kept_bytes:
        kept = torch.empty(kept_bytes, dtype=torch.uint8, device="cuda")
        fwd = lambda: dmt.dmt_tower_module_fwd_keep(plan, tm_params, pooled, B, tm_out, kept, tm_ws)
        bwd = lambda: dmt.dmt_tower_module_bwd(plan, tm_params, pooled, tm_out, B, dy, dx, arr, ws, kept=kept)
        res = {}
        for name, fn in (("fwd_keep", fwd), ("bwd", bwd)):
            for _ in range(2):
                fn()
            torch.cuda.synchronize()
            t0 = time.perf_counter()
            for _ in range(n):
                fn()
            torch.cuda.synchronize()
            res[name] = (time.perf_counter() - t0) * 1e3 / n
        out["with_kept_activations"] = dict(kept_GB=round(kept_bytes / 1e9, 3),
                                            fwd_keep_ms_per_call=round(res["fwd_keep"], 4),
                                            bwd_ms_per_call=round(res["bwd"], 4),
                                            bwd_flops=int(flops_kept))
    return out


def time_whole_step(torch, dmt, wl, w, plan, tm_params, pooled, tm_out, tm_ws, bwd_ws, batches, B, steps):
    """One GPU's whole tower step with the real gradient chain: lookup -> Tower Module (training
    forward) -> Tower Module backward on a fixed N(0,1) gradient of the module outputs -> sorted
    segment-reduce + rowwise Adagrad fed by the module's dL/d(pooled).  Timed after everything
    else; not part of `value`."""
    tw = w.tower_widths()
    grads = tm_grad_buffers(torch, wl, w)
    arr = dmt.make_tm_grads(grads)
    ws = torch.empty(dmt.dmt_tm_bwd_workspace_bytes(plan, tm_params, B), dtype=torch.uint8, device="cuda")
    kept_bytes = dmt.dmt_tm_kept_bytes(plan, tm_params, B, w.tm_dtype)
    kept = torch.empty(kept_bytes, dtype=torch.uint8, device="cuda") if kept_bytes else None
    g = torch.Generator(device="cuda")
    g.manual_seed(11 + w.seed)
    dy = torch.randn(B * sum(w.tm_out), generator=g, device="cuda", dtype=torch.float32)
    dx = torch.empty(B * sum(tw), dtype=torch.float32, device="cuda")

    def step(i):
        b = batches[i % len(batches)]
        dmt.dmt_tower_lookup_fwd(plan, b["idx"], b["off"], B, pooled)
        dmt.dmt_tower_module_fwd_keep(plan, tm_params, pooled, B, tm_out, kept, tm_ws)
        dmt.dmt_tower_module_bwd(plan, tm_params, pooled, tm_out, B, dy, dx, arr, ws, kept=kept)
        dmt.dmt_tower_lookup_bwd_update(plan, b["idx"], b["off"], B, dx, w.lr, w.eps, bwd_ws)

    for i in range(3):
        step(i)
    torch.cuda.synchronize()
    n = max(3, min(steps, 40))
    t0 = time.perf_counter()
    for i in range(n):
        step(3 + i)
    torch.cuda.synchronize()
    ms = (time.perf_counter() - t0) * 1e3 / n
    assert dmt.dmt_last_device_error(plan) == -1
    out = dict(ms_per_step=round(ms, 4), samples_per_s=round(B / (ms * 1e-3), 1), steps=n)
    # the same steps as HIP graphs, one captured per id batch of the pool and replayed in turn
    # (the calls only enqueue kernels, so they capture as they are)
    side = torch.cuda.Stream()
    graphs = []
    for i in range(len(batches)):
        g = torch.cuda.CUDAGraph()
        with torch.cuda.graph(g, stream=side):
            step(i)
        graphs.append(g)
    for i in range(3):
        graphs[i % len(graphs)].replay()
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for i in range(n):
        graphs[(3 + i) % len(graphs)].replay()
    torch.cuda.synchronize()
    gms = (time.perf_counter() - t0) * 1e3 / n
    assert dmt.dmt_last_device_error(plan) == -1
    out["hip_graph_ms_per_step"] = round(gms, 4)
    return out


def cpu_leg(dmt, wl, w, plan, tables, states, tm_host, b0, pooled, tm_out, tm_params, tm_ws, bwd_ws,
            widths):
    """Time the CPU oracle on a bounded sample of the workload (batch 0 of the id
    pool, all towers: one step's worth of lookups) and check the GPU step on the
    same inputs against it."""
    import torch
    import oracle

    def assert_close(got, ref, rtol, what):
        # |got - ref| <= rtol*|ref| + rtol*rms(ref), the tolerance the parity tests use
        rms = float(np.sqrt(np.mean(ref * ref)))
        bad = np.abs(got - ref) > rtol * np.abs(ref) + rtol * rms
        if bad.any():
            raise AssertionError("%s: %d of %d outside tolerance" % (what, int(bad.sum()), ref.size))

    B = w.batch
    n_tow = w.num_towers
    tabs = [f for f in range(w.num_tables) if w.table_to_tower[f] < n_tow]
    nt = len(tabs)
    assert tabs == list(range(nt)), "sample towers must own the leading tables"
    idx, off, grad = b0["host"]
    s_off = off[:nt * B + 1]
    s_idx = idx[:s_off[-1]]
    s_dims = w.dims[:nt]
    s_t2t = w.table_to_tower[:nt]
    s_grad = grad[:B * sum(widths[:n_tow])]
    host_tables = [t.cpu().numpy() for t in tables[:nt]]            # fp16 arrays
    host_states = [np.zeros(w.rows[f], dtype=np.float32) for f in range(nt)]
    enc = lambda a: wl.encode(a, w.tm_dtype)
    dec = [dict(w=wl.decode(enc(h["w_proj"]), w.tm_dtype), b=wl.decode(enc(h["b_proj"]), w.tm_dtype))
           for h in tm_host[:n_tow]]
    oracle.lib()
    threads = oracle.threads()

    t0 = time.perf_counter()
    o_pooled = oracle.lookup_towered(host_tables, w.table_dtype, s_dims, s_t2t, s_idx, s_off, B)
    o_x = [wl.decode(oracle.round_to(p, w.pooled_dtype), w.pooled_dtype) for p in o_pooled]
    t1 = time.perf_counter()
    o_y = [oracle.tm_dot_linear(x, len(w.tower_tables()[t]), dec[t]["w"], dec[t]["b"])
           for t, x in enumerate(o_x)]
    t2 = time.perf_counter()
    o_b = oracle.bwd_update(host_tables, w.table_dtype, host_states, s_dims, s_t2t, s_idx, s_off, B,
                            s_grad, w.lr, w.eps)
    t3 = time.perf_counter()
    t_cpu = t3 - t0
    frac = nt / w.num_tables
    log("[bench] oracle on %d/%d tables, %d threads: lookup %.2fs, TM %.2fs, bwd %.2fs" %
        (nt, w.num_tables, threads, t1 - t0, t2 - t1, t3 - t2))
    # the same oracle on ONE thread, on the first tower only (its share of the step)
    nt1 = len(w.tower_tables()[0])
    oracle.set_threads(1)
    t4 = time.perf_counter()
    o1 = oracle.lookup_towered(host_tables[:nt1], w.table_dtype, s_dims[:nt1], s_t2t[:nt1],
                               s_idx[:s_off[nt1 * B]], s_off[:nt1 * B + 1], B)
    x1 = wl.decode(oracle.round_to(o1[0], w.pooled_dtype), w.pooled_dtype)
    oracle.tm_dot_linear(x1, nt1, dec[0]["w"], dec[0]["b"])
    oracle.bwd_update(host_tables[:nt1], w.table_dtype, [np.zeros(w.rows[f], dtype=np.float32) for f in range(nt1)],
                      s_dims[:nt1], s_t2t[:nt1], s_idx[:s_off[nt1 * B]], s_off[:nt1 * B + 1], B,
                      s_grad[:B * widths[0]], w.lr, w.eps)
    t_one = time.perf_counter() - t4
    oracle.set_threads(threads)
    frac1 = nt1 / w.num_tables
    log("[bench] oracle on %d/%d tables, 1 thread: %.2fs" % (nt1, w.num_tables, t_one))

    # the same step on the GPU, from the same starting tables
    dmt.dmt_tower_lookup_fwd(plan, b0["idx"], b0["off"], B, pooled)
    dmt.dmt_tower_module_fwd(plan, tm_params, pooled, B, tm_out, tm_ws)
    torch.cuda.synchronize()
    parity = {}
    try:
        pos = 0
        ypos = 0
        for t in range(n_tow):
            g = pooled[pos:pos + B * widths[t]].to(torch.float64).cpu().numpy().reshape(B, widths[t])
            assert_close(g, o_x[t], 2e-2, "pooled tower %d" % t)
            pos += B * widths[t]
            gy = tm_out[ypos:ypos + B * w.tm_out[t]].to(torch.float64).cpu().numpy().reshape(B, -1)
            assert_close(gy, wl.decode(oracle.round_to(o_y[t], w.tm_dtype), w.tm_dtype), 2e-2,
                         "TM tower %d" % t)
            ypos += B * w.tm_out[t]
        parity["lookup_fwd"] = parity["tm_fwd"] = "ok"
        dmt.dmt_tower_lookup_bwd_update(plan, b0["idx"], b0["off"], B, b0["grad"], w.lr, w.eps, bwd_ws)
        torch.cuda.synchronize()
        for f in range(nt):
            m = o_b["key_table"] == f
            rows = torch.from_numpy(o_b["key_row"][m]).cuda()
            got = tables[f][rows].to(torch.float64).cpu().numpy()
            want = wl.decode(oracle.round_to(o_b["new_rows"][m][:, :w.dims[f]], w.table_dtype), w.table_dtype)
            assert_close(got, want, 2e-2, "updated rows of table %d" % f)
            gs = states[f][rows].to(torch.float64).cpu().numpy()
            assert_close(gs, o_b["new_state"][m], 1e-5, "state of table %d" % f)
        parity["bwd_update"] = "ok"
    except AssertionError as e:            # report, do not hide
        parity["error"] = str(e)[:300]
        log("[bench] PARITY FAILURE: %s" % e)
    return dict(
        baseline=dict(value=round(B / (t_cpu / frac), 1), unit="samples/s", cores=threads,
                      kind="oracle",
                      sample="batch 0 of the id pool, all %d tables and %d samples (one step): lookup+TM+"
                             "bwd took %.2f s; value = batch / time" % (nt, B, t_cpu),
                      seconds=round(t_cpu, 3),
                      single_thread=dict(value=round(B / (t_one / frac1), 1), unit="samples/s", cores=1,
                                         sample="the first tower's %d tables, all %d samples: %.2f s; value = "
                                                "batch / (time x %d towers)" % (nt1, B, t_one, w.num_towers),
                                         seconds=round(t_one, 3))),
        parity=parity)


if __name__ == "__main__":
    sys.exit(main())
