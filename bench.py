"""Benchmark of the whole F3M hot path on one MI355X.

A step is one pass of the whole path over one batch of synthetic input that is
already resident in HBM: f3m_plan (enclosing cube, keys, sort, box tables,
interaction lists, kernel tables) followed by f3m_kmvm (P2M, M2L, L2P per depth,
near-field P2P, permutations).  Prints ONE JSON line on stdout.

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--config 5|3|4|2] [--n N] [--rows R] [--no-cpu]

The default workload is configuration 5 of the benchmark list: n = 1e9 points,
D = 3, iid Uniform[0,1]^3, Gaussian lengthscale 1.0, b ~ N(0,1), 4 nodes per
dimension, far ratio 2.

With --xy the step is the two-set product v = K(X, Y) b (f3m_plan_xy + f3m_kmvm) on the
stand-in for the paper's two-set experiment (Sec. 5 "KMVM experiments": uniformly
distributed X, normally distributed Y): X ~ Uniform[0,1]^3, Y ~ N(0, I_3), --n points in
EACH set (default 5e8, the largest size the paper runs in 3-D), same kernel and nodes.
"""
import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

PEAK_VALU_F32_TFLOPS = 157.3     # published fp32 vector peak: 256 CU x 128 lanes-equivalents (packed) x 2.4 GHz x 2 flop
UNPACKED_F32_TFLOPS = 78.6       # 256 CU x 64 lanes x 2.4 GHz x 2 flop: what plain (unpacked) FMAs can reach; this build
                                 # generates no packed fp32 instructions
PEAK_HBM_GBS = 8000.0


def log(*a):
    print(*a, file=sys.stderr, flush=True)


def cpu_baseline(cfg, n_sample):
    """The CPU oracle (fp64 F3M, as it stands) on a bounded sample of the same workload."""
    import oracle
    from paper_2202_01085_amd import inputs
    gen = {"uniform": inputs.points_uniform, "normal": inputs.points_normal, "mixture": inputs.points_mixture}[cfg["dist"]]
    X = gen(n_sample, cfg["D"], 1000 + cfg["k"]).numpy()
    b = inputs.rhs_normal(n_sample, 2000 + cfg["k"]).numpy()
    t0 = time.time()
    T = oracle.Tree(X, theta=cfg["theta"], zeta=128)
    t_tree = time.time() - t0
    T.apply(b, cfg["lengthscale"], cfg["p"])
    dt = time.time() - t0
    leaf = n_sample / max(T.nboxes(T.L), 1)
    return {"value": n_sample / dt, "unit": "points/s", "cores": oracle.num_threads(), "kind": "oracle",
            "sample": "oracle F3M (tree %.1f s + product, fp64, dense node-to-node matrices) on n=%d points of the same "
                      "distribution: depth %d, %.0f points per leaf box, %.1f s in all"
                      % (t_tree, n_sample, T.L, leaf, dt)}


def cpu_baseline_xy(cfg, n_sample):
    """The two-set CPU oracle on a bounded sample of the same two distributions."""
    import oracle
    from paper_2202_01085_amd import inputs
    X = inputs.points_uniform(n_sample, 3, 1101).numpy()
    Y = inputs.points_normal(n_sample, 3, 1102).numpy()
    b = inputs.rhs_normal(n_sample, 1103).numpy()
    t0 = time.time()
    T = oracle.Tree2(X, Y, theta=cfg["theta"], zeta=128)
    T.apply(b, cfg["lengthscale"], cfg["p"])
    dt = time.time() - t0
    return {"value": 2 * n_sample / dt, "unit": "points/s", "cores": oracle.num_threads(), "kind": "oracle",
            "sample": "two-set oracle F3M (trees + product, fp64) on %d + %d points of the same distributions, "
                      "depth %d, %.1f s" % (n_sample, n_sample, T.L, dt)}


def source_digest():
    """sha256 over the HIP sources of the library: stored with the counter figures under profiles/ so that a figure
    measured on other kernels is never reported as this build's"""
    import hashlib
    h = hashlib.sha256()
    csrc = os.path.join(ROOT, "paper_2202_01085_amd", "csrc")
    for name in sorted(os.listdir(csrc)):
        with open(os.path.join(csrc, name), "rb") as f:
            h.update(name.encode() + b"\0" + f.read())
    return h.hexdigest()


def load_counters(tag):
    """profiles/counters_<tag>.json: HBM bytes per launch (rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE, scaled by a copy
    of known size) and issue counters of the near-field kernel, with the digest of the sources they were measured
    on.  Returns (bytes per stage, issue counters, note)."""
    path = os.path.join(ROOT, "profiles", "counters_%s.json" % tag)
    if not os.path.exists(path):
        return {}, None, "no counter summary for this workload under profiles/"
    with open(path) as f:
        cj = json.load(f)
    if cj.get("source_digest") != source_digest():
        return {}, None, ("profiles/counters_%s.json was measured on other kernel sources (digest differs): traffic and "
                          "issue counters withheld until it is measured again" % tag)
    return cj.get("bytes_per_launch", {}), cj.get("issue_counters"), "profiles/counters_%s.json" % tag


def median(v):
    v = sorted(v)
    m = len(v) // 2
    return v[m] if len(v) % 2 else 0.5 * (v[m - 1] + v[m])


def bench_direct(args):
    """direct_kmvm (the exact product, Sec. 2) on configuration-1-shaped inputs of --direct points."""
    import torch
    from paper_2202_01085_amd import f3m, inputs
    n = int(args.direct)
    X, b, cfg = inputs.make_config(1, n=n, device="cuda:0")
    y = torch.empty_like(b)
    for _ in range(max(args.warmup, 1)):
        f3m.direct_kmvm(X, b, cfg["lengthscale"], y=y)
    torch.cuda.synchronize()
    times = []
    for _ in range(args.steps):
        t0 = time.perf_counter()
        f3m.direct_kmvm(X, b, cfg["lengthscale"], y=y)
        torch.cuda.synchronize()
        times.append((time.perf_counter() - t0) * 1e3)
    ms = sum(times) / len(times)
    pairs = float(n) * n
    ach = 11.0 * pairs / (ms * 1e-3) / 1e12
    out = {"metric": "direct_kmvm throughput (exact product)", "value": n / (ms * 1e-3), "unit": "points/s", "n_gpus": 1,
           "steps": args.steps, "warmup": args.warmup, "ms_per_step": ms, "ms_per_step_median": median(times),
           "ms_per_step_min": min(times), "ms_per_step_max": max(times), "higher_is_better": True, "scaling": "weak",
           "vs_baseline": None, "dtype": "f32", "data": "synthetic",
           "config": {"workload": "direct_kmvm: n=%d D=3 uniform, Gaussian lengthscale 1, b~N(0,1), all n^2 pairs" % n},
           "roofline": {"kernel": "direct_kmvm", "bound": "alu", "achieved": ach, "peak": PEAK_VALU_F32_TFLOPS,
                        "unit": "TFLOP/s", "frac": ach / PEAK_VALU_F32_TFLOPS, "traffic": None, "launch_ms": ms,
                        "pairs_per_s": pairs / (ms * 1e-3),
                        "valu_slot_frac": 3.0 * pairs / (ms * 1e-3) / (256 * 64 * 2.4e9)},
           "cpu_baseline": None}
    print(json.dumps(out), flush=True)


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=5)
    ap.add_argument("--warmup", type=int, default=1)
    ap.add_argument("--config", type=int, default=None, choices=[2, 3, 4, 5],
                    help="configuration of the benchmark list (default 5: n = 1e9 uniform 3-D points, the headline)")
    ap.add_argument("--n", type=float, default=None, help="points: a reduced or enlarged n of the configuration's recipe "
                                                           "(with --xy: points per set, default 5e8)")
    ap.add_argument("--xy", action="store_true", help="two point sets: X uniform (targets), Y normal (sources)")
    ap.add_argument("--rows", type=int, default=10000, help="sampled rows for the error against the exact product")
    ap.add_argument("--cpu-sample", type=int, default=None, help="points of the CPU oracle sample")
    ap.add_argument("--no-cpu", action="store_true", help="skip the CPU oracle baseline")
    ap.add_argument("--eta-smooth", type=float, default=0.0,
                    help="smooth-field limit of Sec. 4.3 (0 = off, the headline configuration; the paper uses 0.5)")
    ap.add_argument("--adaptive-far", action="store_true", help="adaptive far-field node rule of Sec. 4.3")
    ap.add_argument("--overlap", action="store_true",
                    help="f3m_options.overlap: the near field on the plan's second stream beside the far field")
    ap.add_argument("--cg", type=int, default=0,
                    help="after the timed steps, also time this many conjugate-gradient iterations of f3m_cg_solve "
                         "(kernel ridge regression, Sec. 5) on the last plan; reported under \"cg\", not part of `value`")
    ap.add_argument("--cg-lambda", type=float, default=1.0, help="ridge parameter of --cg")
    ap.add_argument("--copy-calibration", action="store_true",
                    help="first copy 1 GiB device-to-device with a plain kernel: the reference that the "
                         "FETCH_SIZE / WRITE_SIZE counter readings of a rocprofv3 --pmc run are scaled by")
    ap.add_argument("--direct", type=float, default=0,
                    help="time direct_kmvm (the exact O(n^2) product) on this many points instead of the F3M path")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build runs on one GPU only (the kernels are one GPU's share of the path; nothing "
              "here uses a second device); run with --gpus 1", file=sys.stderr)
        sys.exit(2)
    if args.direct:
        return bench_direct(args)

    import torch
    from paper_2202_01085_amd import f3m, inputs

    if args.config is not None:
        k = args.config
        n = int(args.n if args.n is not None else inputs.CONFIGS[k]["n"])
    else:
        n = int(args.n if args.n is not None else (5e8 if args.xy else 1e9))
        k = 5 if n >= 500_000_000 else 3
    cfg = dict(inputs.CONFIGS[k], k=k)
    dev = "cuda:0"
    torch.cuda.set_device(0)
    Y = None
    if args.xy:
        log("generating %d uniform targets and %d normal sources on the device ..." % (n, n))
        X = inputs.points_uniform(n, 3, 1101, device=dev)
        Y = inputs.points_normal(n, 3, 1102, device=dev)
        b = inputs.rhs_normal(n, 1103, device=dev)
    else:
        log("generating n=%d %s points on the device ..." % (n, cfg["dist"]))
        X, b, _ = inputs.make_config(k, n=n, device=dev)
    y = torch.empty_like(b)
    torch.cuda.synchronize()
    if args.copy_calibration:
        src = torch.ones(1 << 28, dtype=torch.float32, device=dev)      # 1 GiB read + 1 GiB written
        dst = torch.empty_like(src)
        dst.copy_(src)
        torch.cuda.synchronize()
        del src, dst

    def step():
        plan = f3m.Plan(X, cfg["lengthscale"], cfg["p"], cfg["theta"], eta_smooth=args.eta_smooth,
                        adaptive_far=args.adaptive_far, Y=Y, overlap=args.overlap)
        plan.kmvm(b, y)
        return plan

    plan = None
    for _ in range(args.warmup):
        if plan is not None:
            plan.close()
        plan = step()
    torch.cuda.synchronize()
    depth_known = None
    if plan is not None:
        depth_known = plan.info().depth     # (the first f3m_plan_info of a plan counts point pairs on the device: not
        plan.close()                        # something to call between the timed steps)
        plan = None

    # K steps between two synchronisations.  Closing the previous step's plan (its memory is needed at n = 1e9) waits
    # for the device, so the host clock read after it marks the end of that step: per-step durations come for free.
    stage_runs, level_runs, marks = [], [], []
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(args.steps):
        if plan is not None:
            stage_runs.append(plan.stage_times())        # HIP events of the finished step (read before the plan goes)
            if depth_known is not None:
                level_runs.append({l: plan.level_times(l) for l in range(1, depth_known + 1)})
            plan.close()
            marks.append(time.perf_counter())
        plan = step()
    torch.cuda.synchronize()
    t_end = time.perf_counter()
    wall = t_end - t0
    ms_per_step = wall * 1e3 / args.steps
    marks = [t0] + marks + [t_end]
    step_ms = [(marks[i + 1] - marks[i]) * 1e3 for i in range(args.steps)]

    # per-kernel durations from the HIP events the library records on the launch stream: median over the steps
    inf = plan.info()
    L = inf.depth
    stage_runs.append(plan.stage_times())
    if depth_known not in (None, L):
        level_runs = []
    level_runs.append({l: plan.level_times(l) for l in range(1, L + 1)})
    st = {key: median([run[key] for run in stage_runs]) for key in stage_runs[0]}
    level_ms = {l: tuple(median([run[l][j] for run in level_runs]) for j in range(3)) for l in range(1, L + 1)}
    far_L = int(inf.far_pairs[L])
    r = inf.nodes_per_box
    m2l_ms = level_ms[L][1] if L >= 1 else 0.0
    D = cfg["D"]
    pairs = int(inf.near_point_pairs)
    nb_L = int(inf.nboxes[L])
    tag = ("xy_n%d" % n) if args.xy else "config%d_n%d" % (k, n)
    traffic, issue, counters_note = load_counters(tag)
    rates = None
    rates_path = os.path.join(ROOT, "profiles", "pipe_rates_mi355x.json")
    if os.path.exists(rates_path):
        with open(rates_path) as f:
            rates = json.load(f)
    rooflines = {}

    def hbm_stage(name, kernel, nbytes, ms):
        # algorithmic bytes: what the stage itself must move (stated per point / per box), not what the kernel moves
        if ms <= 0:
            return
        ach = nbytes / (ms * 1e-3) / 1e9
        rooflines[name] = {"kernel": kernel, "bound": "hbm", "achieved": ach, "peak": PEAK_HBM_GBS, "unit": "GB/s",
                           "frac": ach / PEAK_HBM_GBS, "traffic": traffic.get(name), "launch_ms": ms,
                           "algorithmic_bytes": nbytes}

    ns = n                                                  # sources (= targets for one set)
    key_bits = D * int(inf.quant_depth)
    passes = (key_bits + 7) // 8
    if not args.xy:
        hbm_stage("bbox_keys", "bbox_kernel + keys_kernel: 4D B/pt read twice, 4 B/pt written", (8.0 * D + 4) * n, st["bbox_keys"])
        hbm_stage("sort", "rs_hist_kernel + %d passes of rs_scatter_kernel over %d-bit keys: 4 + %d x 16 B/pt"
                  % (passes, key_bits, passes), (4.0 + 16.0 * passes) * n, st["sort"])
        hbm_stage("gather_x", "gather of the points into box order: 4 + 8D B/pt", (4.0 + 8.0 * D) * n, st["gather"])
        hbm_stage("permute_in", "right-hand side into box order: 12 B/pt", 12.0 * ns, st["permute_in"])
        hbm_stage("permute_out", "result back to the caller's order: 12 B/pt", 12.0 * n, st["permute_out"])
        if L >= 1 and level_ms[L][0] > 0:
            hbm_stage("p2m_leaf", "P2M at depth %d: 4(D+1) B/pt + 4r B/box" % L, 4.0 * (D + 1) * ns + 4.0 * r * nb_L,
                      level_ms[L][0])
        if L >= 1 and level_ms[L][2] > 0:
            hbm_stage("l2p_leaf", "L2P at depth %d: (4D+8) B/pt + 4r B/box" % L, (4.0 * D + 8) * n + 4.0 * r * nb_L,
                      level_ms[L][2])
    if far_L > 0 and m2l_ms > 0:
        # algorithmic: 2 r^2 flop per far pair (the dense node-to-node product).  For D = 3 with 4 nodes per
        # dimension the kernel applies the Kronecker factors per candidate / line / plane of the 6x6x6 grid around
        # the parent, and shares the line and plane sums between the eight children: 936 factor applications of 256
        # multiply-adds per parent (117 per target box) instead of 189 x 4096 per target, on the vector ALU.
        # Every other shape applies D one-dimensional factors per far pair: 2 D r p flop.
        # `achieved` counts the multiply-adds it executes; `algorithmic_tflops` the dense equivalent.
        t = m2l_ms * 1e-3
        if D == 3 and cfg["p"] == 4 and cfg["theta"] == 2.0 and not args.xy:
            executed = 2.0 * 117 * 256 * nb_L
            kernel = "m2l_stencil_shared_kernel"
        else:
            executed = 2.0 * D * r * cfg["p"] * far_L
            kernel = "m2l_kron_small_kernel" if r // cfg["p"] <= 32 else \
                "m2l_kron_grouped_kernel (shares partial sums between far partners, so it executes fewer than the " \
                "2 D r p flop per far pair counted here)"
        ach = executed / t / 1e12
        rooflines["m2l"] = {"kernel": "%s, leaf depth %d, %d far pairs, %d target boxes" % (kernel, L, far_L, nb_L),
                            "bound": "alu", "achieved": ach, "peak": PEAK_VALU_F32_TFLOPS, "unit": "TFLOP/s",
                            "frac": ach / PEAK_VALU_F32_TFLOPS, "traffic": traffic.get("m2l"), "launch_ms": m2l_ms,
                            "frac_of_unpacked_fp32_peak": ach / UNPACKED_F32_TFLOPS,
                            "algorithmic_tflops": 2.0 * r * r * far_L / t / 1e12,
                            "far_pairs_per_s": far_L / t,
                            "peak_note": "peak = the published fp32 vector figure (packed FP32); plain FMAs, the only kind "
                                         "this build generates, reach 78.6 TFLOP/s on 256 CUs x 64 lanes at 2.4 GHz"}
    if pairs > 0 and st["p2p"] > 0:
        # algorithmic: D sub, D mul/fma, exp2, fma = 3D+2 flop per point pair.  The kernel computes the
        # D-term part as a Gram matrix on the matrix cores, so per pair the vector ALU is left with one
        # v_exp_f32 (2 issue slots per lane: measured half rate) and one FMA: 3 slots per pair is the floor
        # of this instruction mix, reported as valu_slot_frac.
        t = st["p2p"] * 1e-3
        flops = (3.0 * D + 2.0) * pairs
        ach = flops / t / 1e12
        lane_slots_per_s = 256 * 64 * 2.4e9
        rooflines["p2p"] = {"kernel": "near field: p2p_gram3_pair_kernel (first runs of up to 64 targets of two sibling boxes "
                                      "per wavefront) + p2p_gram3_kernel (the other runs) + p2p_small_kernel (last runs of "
                                      "<= 10 targets), %d point pairs" % pairs if D == 3 and not args.xy else
                                      "near field, %d point pairs" % pairs, "bound": "alu", "achieved": ach,
                            "peak": PEAK_VALU_F32_TFLOPS, "unit": "TFLOP/s", "frac": ach / PEAK_VALU_F32_TFLOPS,
                            "traffic": traffic.get("p2p"), "launch_ms": st["p2p"],
                            "pairs_per_s": pairs / t,
                            "valu_slot_frac": 3.0 * pairs / t / lane_slots_per_s,
                            "frac_of_unpacked_fp32_peak": ach / UNPACKED_F32_TFLOPS,
                            "issue_counters": issue,
                            "frac_of_measured_exp2_fma_rate": (pairs / t / rates["exp2_fma_pairs_per_s"]) if rates else None,
                            "measured_rate_note": "profiles/pipe_rates_mi355x.json: one v_exp_f32 + one v_fma_f32 per lane "
                                                  "issue at 1.37e13 pairs/s on this device; no near-field kernel that "
                                                  "evaluates one exponential per pair can pass that",
                            "achieved_note": "flop-equivalent: (3D+2) flop per point pair / launch time; the D-term part of "
                                             "every pair runs on the matrix cores (fp16-split operands, fp32 accumulate), so "
                                             "this is not a count of executed VALU flops",
                            "peak_note": "peak = the published fp32 vector figure, which needs packed FP32; this build "
                                         "generates none, so plain FMAs top out at 78.6 TFLOP/s. The (3D+2)-flop count can "
                                         "exceed that because the D-term part of every pair runs on the matrix cores; "
                                         "valu_slot_frac (3 issue slots per pair: one half-rate exp2 + one FMA, over all "
                                         "lane slots) is the utilisation figure to read"}
    # the dominant kernel of the step is the one reported as `roofline`
    roof = None
    if rooflines:
        roof = max(rooflines.values(), key=lambda v: v["launch_ms"])

    # error against the exact product on sampled rows (fp64 row kernel, pinned to the oracle in the tests)
    rows = inputs.sample_rows(n, args.rows, 3000 + k)
    t1 = time.perf_counter()
    if args.xy:
        y64 = f3m.direct_kmvm_xy_rows_f64(X, Y, b, cfg["lengthscale"], rows)
    else:
        y64 = f3m.direct_kmvm_rows_f64(X, b, cfg["lengthscale"], rows)
    torch.cuda.synchronize()
    t_rows = time.perf_counter() - t1
    yr = y[rows.to(dev)].double()
    rel_err = (torch.linalg.norm(yr - y64) / torch.linalg.norm(y64)).item()
    log("exact rows: %d rows in %.1f s, rel err %.3e" % (rows.numel(), t_rows, rel_err))

    out = {
        "metric": "full KMVM throughput (plan + product), F3M",
        "value": (2 * n if args.xy else n) / (ms_per_step * 1e-3),
        "unit": "points/s",
        "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": ms_per_step,
        "ms_per_step_median": median(step_ms), "ms_per_step_min": min(step_ms), "ms_per_step_max": max(step_ms),
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "f32", "data": "synthetic",
        "config": {"workload": ("two sets: %d uniform targets x %d normal sources, D=3, Gaussian lengthscale %g, b~N(0,1), "
                                "%d nodes/dim, far ratio %g (value counts the points of both sets)"
                                % (n, n, cfg["lengthscale"], cfg["p"], cfg["theta"])) if args.xy else
                               "config %d: n=%d D=%d %s, Gaussian lengthscale %g, b~N(0,1), %d nodes/dim, far ratio %g"
                               % (k, n, cfg["D"], cfg["dist"], cfg["lengthscale"], cfg["p"], cfg["theta"]),
                   "depth": L, "leaf_max": 128, "boxes_leaf": nb_L, "near_pairs_leaf": int(inf.near_pairs[L]),
                   "far_pairs_leaf": far_L, "device_bytes": int(inf.device_bytes),
                   "eta_smooth": args.eta_smooth, "adaptive_far": bool(args.adaptive_far),
                   "smooth_depth": int(inf.smooth_depth),
                   "arithmetic": "fp32 throughout; the near-field exponents -|x-y|^2/(2 gamma^2) come from one fp16 MFMA on "
                                 "operands split in two fp16 halves (3 cross terms, about 22 significant bits) with fp32 "
                                 "accumulation, exp2 and the sums in fp32; cells in fp32, box centres and local "
                                 "coordinates in fp64"},
        "wall_s_per_kmvm_with_plan": ms_per_step * 1e-3,
        "rel_err_vs_exact": rel_err, "rel_err_rows": int(rows.numel()),
        "stage_ms": st,
        "stage_ms_note": "median over the timed steps of the HIP-event durations the library records on its launch stream",
        "level_ms": {str(l): {"p2m": v[0], "m2l": v[1], "l2p": v[2]} for l, v in level_ms.items()},
        "roofline": roof,
        "rooflines_all": rooflines,
        "counters": counters_note,
        "paper_context": ("paper: 74.9+-28.5 s mean over its data sets at n=5e8, D=3 on one V100-32GB (the uniform-and-normal "
                          "pair is one of them, run up to n=5e8)") if args.xy else
                         "paper: 125.9 s (r=64) and 174.0+-76.6 s (mean over data sets) for n=1e9, D=3 on one V100-32GB",
    }
    if args.cg > 0 and not args.xy:
        # the paper's synthetic ridge-regression right-hand side: b = k(X, D) alpha + eps, D = the first 1000 points,
        # alpha ~ N(0, I), eps ~ N(0, 0.1^2)
        alpha = inputs.rhs_normal(1000, 4000 + k, device=dev)
        bk = f3m.direct_kmvm_xy(X, X[:1000].contiguous(), alpha, cfg["lengthscale"])
        bk += 0.1 * inputs.rhs_normal(n, 5000 + k, device=dev)
        torch.cuda.synchronize()
        t1 = time.perf_counter()
        _, iters, hist = plan.cg_solve(bk, args.cg_lambda, tol=0.0, max_iter=args.cg, x=y)
        torch.cuda.synchronize()
        t_cg = time.perf_counter() - t1
        out["cg"] = {"iterations": iters, "ms_per_iteration": t_cg * 1e3 / max(iters, 1), "lambda": args.cg_lambda,
                     "kmvm_ms": plan.stage_times()["kmvm_total"],
                     "relative_residuals": [float(v) for v in hist],
                     "note": "one f3m_kmvm + three fused vector passes + one 40-byte copy per iteration; fp32 products "
                             "stall the residual near 5e-7 x condition number (no preconditioner here)"}
        del bk
    plan.close()
    del X, Y, y
    if not args.no_cpu:
        # sample sizes of about 30 s of oracle work on 16 cores; 2e6 uniform points divide to depth 5 with 61 points
        # per leaf box, the leaf occupancy of the 1e9-point workload at depth 8
        sample = args.cpu_sample or {5: 2_000_000, 3: 2_000_000, 2: 300_000, 4: 1_500}[k]
        out["cpu_baseline"] = cpu_baseline_xy(cfg, sample // 2) if args.xy else cpu_baseline(cfg, sample)
    else:
        out["cpu_baseline"] = None
    print(json.dumps(out), flush=True)


if __name__ == "__main__":
    main()
