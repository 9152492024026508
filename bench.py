"""Benchmark of the hot path on one MI355X.

A step = one classical RK4 step (4 x [ghost fill -> stencils -> right-hand side -> stage update])
of the 24-field system on the ~1e5-block adaptive tree ("C5"), inputs resident in HBM.
Prints ONE JSON line: block-point right-hand-side updates per second (fp64, per variable), the
HBM roofline of the dominant kernel (its launch time measured live with events on the launch stream;
the counter traffic comes from the committed profile of exactly this build, or is null), and the CPU
oracle timed on this machine's host cores on a bounded sample of the same workload.

The 24-field system is a throughput workload: with the prescribed step dt = h/4 its second-derivative
term is far beyond the explicit stability limit, so the state grows by about ten orders of magnitude
per step and would overflow after a few steps.  Every timed step therefore starts from the initial state
again (restored between the steps, outside the per-step event pairs); parity with the oracle is checked
on the first evaluation (cpu_baseline.parity_on_sample) and in the tests.
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
# Algorithmic HBM bytes per block-point and variable of one RK stage launch (fused kernel, zipped in,
# zipped out; ghost reads are re-reads of neighbours' owned data and count as cache traffic):
#   first  stage: read u, write acc, write stage                   = 24 B
#   middle stages: read stage, read u, read+write acc, write stage = 40 B   (twice)
#   last   stage: read stage, read acc, read+write u               = 32 B
STAGE_BYTES = (24.0, 40.0, 40.0, 32.0)


# fp64 vector peak of the device (256 compute units x 4 SIMDs x 16 lanes x 2 flop x 2.4 GHz): prices the arithmetic
FP64_VECTOR_PEAK_TFLOPS = 78.6


def csrc_digest():
    """SHA-256 over the kernel and host sources of the library (names and contents, sorted): identifies the
    build that a committed counter summary was taken from."""
    import hashlib
    d = os.path.join(ROOT, "paper_2007_12792_amd", "csrc")
    h = hashlib.sha256()
    for name in sorted(os.listdir(d)):
        h.update(name.encode())
        h.update(open(os.path.join(d, name), "rb").read())
    return h.hexdigest()


def committed_counters(config, nb):
    """What the committed rocprofv3 counter summary says about the dominant kernel on this workload: bytes per
    launch between the L2 caches and the memory fabric (FETCH_SIZE and WRITE_SIZE passes, scaled by the same
    counters on a device copy of known size) and fp64 operations per launch (SQ_INSTS_VALU_* passes).  The counters
    cannot be read inside this process, so the record is only used when it was taken from exactly these sources
    (csrc_sha256) on exactly this tree; otherwise None, and the bench line says traffic: null."""
    path = os.path.join(ROOT, "profiles", "hbm_traffic.json")
    try:
        rec = json.load(open(path)).get(config)
    except (OSError, ValueError):
        return None
    if not rec or rec.get("n_blocks") != nb or rec.get("csrc_sha256") != csrc_digest():
        return None
    return rec


def other_kernels(args, cfg, kind, dev):
    """ms per call and algorithmic GB/s of the kernels that the headline step does not use."""
    import numpy as np
    import torch

    import paper_2007_12792_amd as octfd
    import synthdata as sd

    t = octfd.Tree.build(**sd.tree_params(args.config, args.seed))
    nb, Vi, Vo = t.n, octfd.nvar_in(kind), octfd.nvar_out(kind)
    u = sd.make_fields(args.config, t.leaves, args.seed, device=dev)
    pad = torch.empty((Vi, nb, 14, 14, 14), dtype=torch.float64, device=dev)
    rp = torch.zeros((Vo, nb, 14, 14, 14), dtype=torch.float64, device=dev)
    out = torch.empty((Vo, nb, 8, 8, 8), dtype=torch.float64, device=dev)
    t.upload()
    stream = torch.cuda.current_stream()

    def timed(f):
        f()
        torch.cuda.synchronize()
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record(stream)
        for _ in range(args.steps):
            f()
        e1.record(stream)
        torch.cuda.synchronize()
        return e0.elapsed_time(e1) / args.steps

    pts = nb * 512
    res = {}

    def row(name, ms, bytes_per_call, what):
        res[name] = {"ms": ms, "algorithmic_GBs": bytes_per_call / ms / 1e6, "bytes": what}

    row("unzip", timed(lambda: t.unzip(u, pad)), 50.9 * pts * Vi, "8 B read + 42.9 B written per block-point and variable")
    row("unzip_centred", timed(lambda: t.unzip_centred(u, pad)), 50.9 * pts * Vi, "as unzip")
    t.unzip(u, pad)
    row("rhs_eval", timed(lambda: t.rhs_eval(kind, pad, rp, sigma=sd.KO_SIGMA)), (42.9 * Vi + 8.0 * Vo) * pts,
        "42.9 B read per input variable + 8 B written per output variable")
    row("zip", timed(lambda: t.zip(rp, out)), 16.0 * pts * Vo, "8 B read + 8 B written")
    row("rhs_eval_zipped", timed(lambda: t.rhs_eval_zipped(kind, u, out, sigma=sd.KO_SIGMA)), (8.0 * Vi + 8.0 * Vo) * pts,
        "8 B read per input variable + 8 B written per output variable")
    if Vi == Vo:
        ws = torch.empty(t.rk_centred_workspace_bytes(kind) // 8, dtype=torch.float64, device=dev)
        uc = u.clone()
        dt = sd.time_step(cfg["lmax"])
        row("rk_step_centred", timed(lambda: t.rk_step_centred(kind, uc, dt, ws, sigma=sd.KO_SIGMA)), 4 * 34.0 * pts * Vi,
            "whole RK4 step with the centred ghost rule; 34 B per block-point, variable and stage as for rk_step")
        del ws, uc
    if cfg["style"] == "orbit":
        t2 = octfd.Tree.build(**sd.tree_params(args.config, args.seed, phase=0.013))
        plan = octfd.Transfer(t, t2)
        u2 = torch.empty((Vi, t2.n, 8, 8, 8), dtype=torch.float64, device=dev)
        row("regrid_transfer", timed(lambda: plan.apply(u, u2)), 16.0 * t2.n * 512 * Vi, "8 B read + 8 B written")
        res["regrid_transfer"]["blocks_copied_interpolated_injected"] = np.bincount(plan.table[:, 0], minlength=3).tolist()
    print(json.dumps({"workload": args.config, "n_blocks": nb, "n_vars_in": Vi, "n_vars_out": Vo, "calls_timed": args.steps,
                      "kernels": res}), flush=True)


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=10)
    ap.add_argument("--warmup", type=int, default=3)
    ap.add_argument("--config", default="C5", help="workload name from synthdata.CONFIGS (default: the headline one)")
    ap.add_argument("--seed", type=int, default=1)
    ap.add_argument("--region", choices=("auto", "rk", "rhs"), default="auto",
                    help="timed step: one RK4 step (rk) or one fused right-hand-side evaluation (rhs); auto = what the workload names")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--cpu-sample-blocks", type=int, default=0, help="0 = every block of the tree")
    ap.add_argument("--other-kernels", action="store_true",
                    help="instead of the benchmark, time every other kernel of the library once on the workload (the "
                         "literal unzip / rhs_eval / zip calls, the centred ghost rule, the fused right-hand side, the "
                         "regrid transfer) and print one JSON line; this is what the summaries under profiles/ are made with")
    ap.add_argument("--csrc-digest", action="store_true", help="print the digest of the library sources (the key of profiles/hbm_traffic.json) and exit")
    ap.add_argument("--calibrate-copy", type=float, default=0.0, metavar="GB",
                    help="instead of the benchmark, run 5 plain device copies of this many GB (a kernel of known "
                         "HBM traffic, used to scale the rocprofv3 FETCH_SIZE / WRITE_SIZE counters)")
    args = ap.parse_args()
    if args.gpus != 1:
        sys.exit("bench.py: this build runs on exactly one GPU (no sharding, no collectives); use --gpus 1")
    if args.csrc_digest:
        print(csrc_digest())
        return

    import numpy as np
    import torch

    import paper_2007_12792_amd as octfd
    import synthdata as sd

    if not torch.cuda.is_available():
        sys.exit("bench.py: no GPU visible; the hot path has no CPU fallback")
    dev = torch.device("cuda:0")
    if args.calibrate_copy > 0:
        n = int(args.calibrate_copy * 1e9) // 8
        src = torch.ones(n, dtype=torch.float64, device=dev)
        dst = torch.empty_like(src)
        for _ in range(5):
            dst.copy_(src)
        torch.cuda.synchronize()
        print(json.dumps({"calibration": "device copy", "bytes_read_per_copy": n * 8, "bytes_written_per_copy": n * 8, "copies": 5}))
        return
    cfg = sd.CONFIGS[args.config]
    kind = octfd.KINDS[cfg["kind"]]
    if args.other_kernels:
        other_kernels(args, cfg, kind, dev)
        return
    # the step: one RK4 step, or, for the workloads whose timed region is a single evaluation (and for kinds
    # that cannot be stepped), one fused right-hand-side evaluation
    single_rhs = args.region == "rhs" or (args.region == "auto" and (args.config in ("C1", "C2", "C4")
                                                                     or octfd.nvar_in(kind) != octfd.nvar_out(kind)))
    if not single_rhs and octfd.nvar_in(kind) != octfd.nvar_out(kind):
        sys.exit("bench.py: --region rk needs a workload whose kind can be stepped")
    p = sd.tree_params(args.config, args.seed)
    t0 = time.time()
    tree = octfd.Tree.build(**p)
    t_build = time.time() - t0
    leaves = tree.leaves
    nb, V = tree.n, octfd.nvar_out(kind)
    u = sd.make_fields(args.config, leaves, args.seed, device=dev)
    u0 = u.clone()
    dt, sg = sd.time_step(cfg["lmax"]), (0.0 if cfg["kind"] == "DERIVS" else sd.KO_SIGMA)
    tree.upload()
    stream = torch.cuda.current_stream()
    if single_rhs:
        kout = torch.empty((V, nb, 8, 8, 8), dtype=torch.float64, device=dev)
        step = lambda: tree.rhs_eval_zipped(kind, u, kout, sigma=sg, stream=stream)
        launches_per_step, stage_bytes = 1, (16.0,) if octfd.nvar_in(kind) == V else (8.0 * octfd.nvar_in(kind) / V + 8.0,)
    else:
        ws = torch.empty(tree.rk_workspace_bytes(kind) // 8, dtype=torch.float64, device=dev)
        step = lambda: tree.rk_step(kind, u, dt, ws, sigma=sg, stream=stream)
        launches_per_step, stage_bytes = 4, STAGE_BYTES

    for _ in range(args.warmup):
        u.copy_(u0)
        step()
    # Every timed step starts from the same initial state: an RK4 step overwrites its input, and the 24-field
    # system grows by ten orders of magnitude per step, so that without this the later steps would run on
    # inf/NaN (which the device happens to process a few per cent faster).  Putting the input in place is not
    # part of the step: each step is timed by its own pair of events, recorded on the stream of the launches,
    # and the step time is the mean of these K intervals.
    restore = not single_rhs
    ev = [(torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)) for _ in range(args.steps)]
    u.copy_(u0)
    torch.cuda.synchronize()
    w0 = time.perf_counter()
    for i in range(args.steps):
        if restore and i:
            u.copy_(u0)
        ev[i][0].record(stream)
        step()
        ev[i][1].record(stream)
    torch.cuda.synchronize()
    wall = time.perf_counter() - w0
    per_step_ms = [a.elapsed_time(b) for a, b in ev]
    total_ms = float(sum(per_step_ms))
    ms_per_step = total_ms / args.steps
    updates_per_step = nb * 512 * V * launches_per_step
    value = updates_per_step / (ms_per_step * 1e-3)

    # what a plain device copy reaches on this GPU: the practical ceiling under the published HBM peak
    n_copy = 1 << 28                                   # 2 GiB read + 2 GiB written per copy
    src = torch.empty(n_copy, dtype=torch.float64, device=dev).fill_(1.0)
    dst = torch.empty_like(src)
    dst.copy_(src)
    c0, c1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    c0.record(stream)
    for _ in range(5):
        dst.copy_(src)
    c1.record(stream)
    torch.cuda.synchronize()
    copy_gbs = 5 * 2 * n_copy * 8 / (c0.elapsed_time(c1) * 1e-3) / 1e9
    del src, dst

    # dominant kernel = the fused right-hand-side/stage kernel, launched 4 times per step, each time behind the small
    # kernel that fills the virtual blocks of its input; nothing else runs in the timed region, and the pair is
    # priced as one launch: average duration = region / (4 * steps)
    launch_ms = total_ms / (launches_per_step * args.steps)
    bytes_per_launch = sum(stage_bytes) / len(stage_bytes) * nb * 512 * V
    achieved = bytes_per_launch / (launch_ms * 1e-3) / 1e9
    rec = None if single_rhs else committed_counters(args.config, nb)
    # roofline time of one launch: the larger of the algorithmic bytes at the HBM peak and the fp64 operations the
    # counters saw at the vector peak (no counter record for this build: the bytes alone, which dominate)
    hbm_ms = bytes_per_launch / (HBM_PEAK_GBS * 1e9) * 1e3
    valu_ms = None if not rec or not rec.get("fp64_flop_per_launch") else rec["fp64_flop_per_launch"] / (FP64_VECTOR_PEAK_TFLOPS * 1e12) * 1e3
    roofline_ms = max(hbm_ms, valu_ms or 0.0)
    out = {
        "metric": "block-point RHS updates/sec (fp64, per var) + achieved HBM GB/s, 1 GPU",
        "value": value, "unit": "updates/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": ms_per_step, "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "f64", "data": "synthetic",
        "config": {"workload": "%s: %s %s, 2:1-balanced octree levels %d-%d, %d blocks of 8^3 (pad 3), %d fields, KO sigma %.1f, seed %d"
                   % (args.config, cfg["kind"], "fused right-hand-side evaluation" if single_rhs else "RK4 step", cfg["lmin"], cfg["lmax"],
                      nb, V, sg, args.seed),
                   "n_blocks": nb, "n_vars": V, "rhs_evals_per_step": launches_per_step,
                   "zipped_state_GB": nb * 512 * V * 8 / 1e9, "tree_build_s": t_build,
                   "ms_per_step_all": per_step_ms, "ms_per_step_median": float(np.median(per_step_ms)),
                   "ms_per_step_min": float(min(per_step_ms)), "state_restored_before_each_step": restore,
                   "wall_s_timed_region": wall},
        # one launch = one right-hand-side evaluation: the fill of the virtual blocks (k_virtual, 6 % of the time on
        # the headline workload) and the fused kernel that does everything else; launch_ms covers both
        "roofline": {"bound": "hbm", "kernel": "k_virtual + %s<%s, zipped in, %s> (%d per step)"
                               % ("k_rhs_pair" if cfg["kind"] == "SYN24" else "k_rhs", cfg["kind"],
                                  "plain output" if single_rhs else "RK-stage epilogue", launches_per_step),
                     "achieved": achieved, "peak": HBM_PEAK_GBS, "unit": "GB/s", "frac": achieved / HBM_PEAK_GBS,
                     "launch_ms": launch_ms, "algorithmic_bytes_per_launch": bytes_per_launch,
                     # bytes between the L2 caches and the memory fabric per launch (HBM plus whatever the memory-side
                     # cache serves), from the committed counter summary of exactly this build; null otherwise
                     "traffic": rec["bytes_per_launch"] if rec else None,
                     "traffic_source": "committed profile (rocprofv3 FETCH_SIZE / WRITE_SIZE, L2 <-> fabric)" if rec else None,
                     "hbm_ms": hbm_ms, "valu_ms": valu_ms, "roofline_time_ms": roofline_ms,
                     "roofline_time_frac": roofline_ms / launch_ms,
                     # the same launch time against three byte counts: what the method must move at the very
                     # least (8 B in + 8 B out per update), what this pipeline moves by construction
                     # (= achieved), and what the counters saw (= traffic)
                     "compulsory_GBs": (8.0 * octfd.nvar_in(kind) + 8.0 * V) * nb * 512 / (launch_ms * 1e-3) / 1e9,
                     "device_copy_GBs": copy_gbs},
    }
    tr = out["roofline"]["traffic"]
    out["roofline"]["measured_GBs"] = None if tr is None else tr / (launch_ms * 1e-3) / 1e9

    if not args.no_cpu_baseline:
        import oracle
        to = oracle.Tree.build(**p)
        assert (to.leaves == leaves).all()
        ns = min(args.cpu_sample_blocks, nb) if args.cpu_sample_blocks > 0 else nb
        start = (nb - ns) // 2
        blocks = np.arange(start, start + ns)
        uh = u0.cpu().numpy()
        threads = len(os.sched_getaffinity(0))
        omp = os.environ.get("OMP_NUM_THREADS")
        if omp:
            threads = min(threads, int(omp))
        c0 = time.perf_counter()
        ref = to.F(kind, uh, sigma=sg, blocks=blocks)
        cpu_s = time.perf_counter() - c0
        # also use the sample as a live parity check of the kernel just timed: every value of every sampled block
        k1 = torch.empty((V, nb, 8, 8, 8), dtype=torch.float64, device=dev)
        tree.rhs_eval_zipped(kind, u0, k1, sigma=sg)
        ok = True
        for v in range(V):                               # one field at a time, to bound the temporaries
            got, want = k1[v, start:start + ns].cpu().numpy(), ref[v]
            ok = ok and bool((np.abs(got - want) <= 1e-12 * np.abs(want) + 1e-13).all())
        # the same oracle on one thread, on the middle 1/16 of that sample
        import ctypes
        gomp = ctypes.CDLL("libgomp.so.1")
        n1 = max(1, ns // 16)
        b1 = blocks[(ns - n1) // 2:(ns - n1) // 2 + n1]
        gomp.omp_set_num_threads(1)
        s0 = time.perf_counter()
        to.F(kind, uh, sigma=sg, blocks=b1)
        one_s = time.perf_counter() - s0
        gomp.omp_set_num_threads(threads)
        out["cpu_baseline"] = {"value": ns * 512 * V / cpu_s, "unit": "updates/s", "cores": threads, "kind": "oracle",
                               "single_thread_value": n1 * 512 * V / one_s, "single_thread_sample_blocks": int(n1),
                               "sample": "one right-hand-side evaluation (unzip->rhs->zip) of %d contiguous Morton-order blocks "
                                         "(%d..%d of %d) of the same tree and fields, %.1f s" % (ns, start, start + ns - 1, nb, cpu_s),
                               "parity_on_sample": ok}
    print(json.dumps(out), flush=True)
    if "cpu_baseline" in out and not out["cpu_baseline"]["parity_on_sample"]:
        sys.exit("bench.py: the kernel just timed disagrees with the oracle on the sampled blocks")


if __name__ == "__main__":
    main()
