"""Benchmark of the NGDB training hot path on one MI355X.

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--config 1] [--streams S]

One step = plan one batch (host) + one ngdb_train_step (forward over the
operator-level frontiers, scoring against 1 positive and K negatives per query,
loss, backward, segmented scatter-add, Adam) on synthetic data of the
FB15k-237-shaped workload (15k entities, d=400, hidden 800, 512 queries of 14
structures, K=128).  Parameters, optimiser state and the negatives are
resident in HBM before the timed region; 8 pre-generated batches are cycled.
Prints ONE JSON line.
"""
import argparse
import json
import os
import sys
import time

import numpy as np

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

import workloads as wl  # noqa: E402

HBM_PEAK_GBS = 8000.0     # MI355X HBM3E, published
N_BATCHES = 8


def cpu_baseline(cfg, kg, sample):
    """The oracle as it stands, one full step (loss, gradients, Adam) on `sample` queries,
    single process with BLAS held to one thread."""
    from oracle import model as om
    try:
        from threadpoolctl import threadpool_limits
    except Exception:                      # pragma: no cover
        threadpool_limits = None
    qb = wl.make_batch(kg, sample, cfg.mix, cfg.seed + 100)
    negs = wl.make_negatives(cfg.N, sample, cfg.K, cfg.seed + 200)
    P = om.to_f64(wl.make_params(cfg.N, cfg.R, cfg.d, cfg.h, cfg.seed + 3))
    st = om.new_state(P)
    hp = dict(lr=cfg.lr, beta1=cfg.beta1, beta2=cfg.beta2, eps=cfg.eps, gamma=cfg.gamma)

    def run():
        t0 = time.perf_counter()
        om.train_step(qb, negs, P, st, 1, hp)
        return time.perf_counter() - t0

    if threadpool_limits is not None:
        with threadpool_limits(limits=1):
            dt = run()
    else:
        dt = run()
    return {"value": sample / dt, "unit": "queries/s", "cores": 1, "kind": "oracle",
            "sample": "%d queries of the same workload with all %d negatives, one full step "
                      "(per-query fp64 numpy forward, loss, backward, Adam), %.1f s" % (sample, cfg.K, dt)}


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=200)
    ap.add_argument("--warmup", type=int, default=20)
    ap.add_argument("--config", type=int, default=1)
    ap.add_argument("--streams", type=int, default=0, help="0 = the workload's default")
    ap.add_argument("--cpu-sample", type=int, default=-1, help="queries timed on the CPU oracle (0 = skip)")
    ap.add_argument("--all-classes", action="store_true", help="time every kernel class (perturbs the step time)")
    ap.add_argument("--calibrate-copy", type=int, default=0, metavar="MiB",
                    help="also run the library's plain copy kernel on this many MiB, 5 times (reference "
                         "for scaling rocprofv3 traffic counters)")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build runs on one GPU; --gpus %d is not supported (no sharding, no collectives)"
              % args.gpus, file=sys.stderr)
        sys.exit(2)

    cfg = wl.get_config(args.config)
    kg = wl.make_kg(cfg.N, cfg.R, cfg.T, cfg.alpha, cfg.seed)
    batches = [wl.make_batch(kg, cfg.B, cfg.mix, cfg.seed + 10 + i) for i in range(N_BATCHES)]
    negs_np = [wl.make_negatives(cfg.N, cfg.B, cfg.K, cfg.seed + 50 + i) for i in range(N_BATCHES)]
    params = wl.make_params(cfg.N, cfg.R, cfg.d, cfg.h, cfg.seed + 3)

    # CPU oracle first, before this process touches the GPU
    sample = args.cpu_sample if args.cpu_sample >= 0 else min(cfg.B, 512 if cfg.K <= 128 else 64)
    cpu = cpu_baseline(cfg, kg, sample) if sample > 0 else None

    import torch
    from paper_2602_21597_amd import Engine
    streams = args.streams or cfg.streams
    eng = Engine(cfg.N, cfg.R, cfg.d, cfg.h, cfg.gamma, lr=cfg.lr, beta1=cfg.beta1, beta2=cfg.beta2, eps=cfg.eps,
                 num_streams=streams)
    eng.bind_numpy(params)
    negs = [torch.from_numpy(n).cuda() for n in negs_np]
    stream = torch.cuda.current_stream()

    def step(i):
        plan = eng.plan(batches[i % N_BATCHES])
        eng.train_step(plan, negs[i % N_BATCHES], stream)
        plan.free()        # the library recycles the plan's buffers once the step has finished

    for i in range(args.warmup):
        step(i)
    torch.cuda.synchronize()

    timed = ("score", "table_E") if not args.all_classes else \
        ("index", "sem", "gemm_fwd", "inter", "score", "gemm_bwd", "wgrad", "table_E", "table_R", "adam")
    eng.set_timing(timed)
    eng.get_timing(reset=True)
    touched = 0
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for i in range(args.steps):
        step(args.warmup + i)
    torch.cuda.synchronize()
    dt = time.perf_counter() - t0
    timing = eng.get_timing(reset=True)
    eng.set_timing(())

    # device-only time of the same steps with plans prebuilt (context figure)
    plans = [eng.plan(b) for b in batches]
    torch.cuda.synchronize()
    t1 = time.perf_counter()
    for i in range(args.steps):
        eng.train_step(plans[i % N_BATCHES], negs[i % N_BATCHES], stream)
    torch.cuda.synchronize()
    dt_dev = time.perf_counter() - t1
    touched = eng.n_touched_entities()
    pexp = plans[(args.steps - 1) % N_BATCHES].export()

    copy_gbs = None
    if args.calibrate_copy:
        from paper_2602_21597_amd import binding
        src = torch.empty(args.calibrate_copy << 20, dtype=torch.uint8, device="cuda")
        dst = torch.empty_like(src)
        binding.debug_copy(dst, src)
        torch.cuda.synchronize()
        tc = time.perf_counter()
        for _ in range(5):
            nb = binding.debug_copy(dst, src)
        torch.cuda.synchronize()
        copy_gbs = 2 * nb * 5 / (time.perf_counter() - tc) / 1e9

    # roofline of the dominant HBM kernels (algorithmic bytes / measured kernel time)
    row = 4 * cfg.d
    pairs = cfg.B * (cfg.K + 1)
    score_bytes = pairs * (row + 4 + 12) + pexp["n_roots"] * 2 * row
    n_contrib = pexp["n_anchor"] + cfg.B + cfg.B * cfg.K
    table_bytes = touched * 6 * row + n_contrib * 12 + pexp["n_anchor"] * row
    kern = {}
    for name, nbytes in (("score", score_bytes), ("table_E", table_bytes)):
        ms, n = timing[name]
        if n:
            avg = ms / n
            kern[name] = {"avg_us": 1e3 * avg, "bytes": nbytes, "GBs": nbytes / (avg * 1e-3) / 1e9}
    dom = max(kern, key=lambda k: kern[k]["avg_us"])
    roofline = {"bound": "hbm", "kernel": dom, "achieved": kern[dom]["GBs"], "peak": HBM_PEAK_GBS, "unit": "GB/s",
                "frac": kern[dom]["GBs"] / HBM_PEAK_GBS, "traffic": None,
                "avg_us": kern[dom]["avg_us"], "algorithmic_bytes": kern[dom]["bytes"],
                "other": {k: v for k, v in kern.items() if k != dom}}

    out = {
        "metric": "training queries/sec (fwd+bwd+Adam) at d=400, K=128 negatives; % of HBM peak",
        "value": cfg.B * args.steps / dt,
        "unit": "queries/s",
        "n_gpus": 1,
        "steps": args.steps,
        "warmup": args.warmup,
        "ms_per_step": 1e3 * dt / args.steps,
        "higher_is_better": True,
        "scaling": "weak",
        "vs_baseline": None,
        "dtype": "f32",
        "data": "synthetic",
        "config": {"workload": "configs[%d] %s: N=%d R=%d d=%d h=%d B=%d K=%d, 14-structure mix, gamma=%g"
                   % (cfg.index, cfg.name, cfg.N, cfg.R, cfg.d, cfg.h, cfg.B, cfg.K, cfg.gamma),
                   "streams": streams, "step": "ngdb_plan (host) + ngdb_train_step",
                   "touched_entity_rows": touched},
        "device_only": {"queries_per_s": cfg.B * args.steps / dt_dev, "ms_per_step": 1e3 * dt_dev / args.steps,
                        "note": "same steps with plans prebuilt"},
        "roofline": roofline,
        "cpu_baseline": cpu,
    }
    if copy_gbs is not None:
        out["copy_kernel_GBs"] = copy_gbs
    if args.all_classes:
        out["kernel_classes_ms_per_step"] = {k: v[0] / args.steps for k, v in timing.items()}
    print(json.dumps(out))


if __name__ == "__main__":
    main()
