"""Benchmark of the NGDB training hot path on one MI355X.

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--config 1] [--streams S]
    python bench.py --rank 1024 --config 4 --steps 3 --warmup 1      (all-entity ranking pass)

One step = plan one batch (host, overlapped with the previous step) + one ngdb_train_step (forward over the
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

from concurrent.futures import ThreadPoolExecutor

import numpy as np

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

import workloads as wl  # noqa: E402

HBM_PEAK_GBS = 8000.0     # MI355X HBM3E, published
MFMA_F32_PEAK_TF = 157.3  # dense fp32 matrix, published
MFMA_BF16_PEAK_TF = 2500.0
N_BATCHES = 8
CLASSES = ("index", "sem", "gemm_fwd", "inter", "score", "gemm_bwd", "wgrad", "table_E", "table_R", "adam")
# HBM bytes per launch of a workload's dominant kernel from the rocprofv3 --pmc runs summarised
# under profiles/ (FETCH_SIZE + WRITE_SIZE, scaled by the copy kernel): {(config, kernel): bytes}
MEASURED_TRAFFIC = {
    (1, "gemm"): 19.7e6,        # mean over the 17 contraction launches of a step (weight gradients: 90 MB)
    (3, "table_E"): 26.4e9,     # of which 9.75 GB written; 6.7 GB are re-reads of branch rows served by the caches
    (4, "sem"): 14.2e9,         # projection 16.2 GB + its gradient 12.1 GB per step, two launches
    ("box", 1, "gemm"): 18.3e6,     # mean over the 9 contraction launches of a step
    ("box", 3, "table_E"): 32.6e9,  # the winning branches' offset rows are re-read beside their centre rows
}


def cpu_baseline(cfg, kg, sample, sem_bits, box_alpha=None, score_bf16=False):
    """The oracle as it stands, full steps (loss, gradients, Adam) on batches of `sample` queries
    until about 10 s of CPU time have passed (at most 16 steps), single process with BLAS held
    to one thread."""
    from oracle import box as ob
    from oracle import model as om
    try:
        from threadpoolctl import threadpool_limits
    except Exception:                      # pragma: no cover
        threadpool_limits = None
    box = box_alpha is not None
    P = om.to_f64(wl.make_box_params(cfg.N, cfg.R, cfg.d, cfg.h, cfg.seed + 3) if box else
                  wl.make_params(cfg.N, cfg.R, cfg.d, cfg.h, cfg.seed + 3, d_sem=cfg.d_sem))
    st = om.new_state(P)
    hp = dict(lr=cfg.lr, beta1=cfg.beta1, beta2=cfg.beta2, eps=cfg.eps, gamma=cfg.gamma, alpha=box_alpha)

    def run():
        total, steps = 0.0, 0
        while total < 10.0 and steps < 16:
            qb = wl.make_batch(kg, sample, cfg.mix, cfg.seed + 100 + steps)
            negs = wl.make_negatives(cfg.N, sample, cfg.K, cfg.seed + 200 + steps)
            t0 = time.perf_counter()
            if box:
                ob.train_step(qb, negs, P, st, steps + 1, hp)
            else:
                om.train_step(qb, negs, P, st, steps + 1, hp, sem_bits, score_bf16=score_bf16)
            total += time.perf_counter() - t0
            steps += 1
        return total, steps

    if threadpool_limits is not None:
        with threadpool_limits(limits=1):
            dt, steps = run()
    else:
        dt, steps = run()
    return {"value": sample * steps / dt, "unit": "queries/s", "cores": 1, "kind": "oracle",
            "sample": "%d steps of %d queries of the same workload with all %d negatives (per-query fp64 numpy "
                      "forward, loss, backward, Adam), %.1f s" % (steps, sample, cfg.K, dt)}


def say(msg):
    """Progress on stderr (the JSON line on stdout stays alone)."""
    print("[bench] " + msg, file=sys.stderr, flush=True)


def kernel_models(cfg, pexp, touched, box=False, score_bf16=False):
    """Algorithmic work of one step per kernel class: what the method itself has to move or
    multiply, whatever the kernels do.  Returns {class: (bound, amount, peak, unit)} with
    amounts in bytes (hbm) or flops (mfma)."""
    row = 4 * cfg.d
    pairs = cfg.B * (cfg.K + 1)
    n_contrib = pexp["n_anchor"] + cfg.B + cfg.B * cfg.K
    mlp_rows = pexp["n_proj"] + pexp["n_int_rows"] + pexp["n_neg"]
    sem = cfg.d_sem > 0
    # every pair: one entity row, its index, 12 bytes of (score, dL/ds, winning branch); every branch
    # embedding read once and its gradient written once
    score_bytes = pairs * (row + 4 + 12) + pexp["n_roots"] * 2 * row
    # every touched row: p, m, v read and written; every contribution: 12 bytes of record; anchor
    # gradient rows read; with text features also the fused row read and the bf16 gradient written
    table_bytes = touched * 6 * row + n_contrib * 12 + pexp["n_anchor"] * row
    if sem:
        table_bytes += touched * (row + 2 * cfg.d)
    if score_bf16:   # candidate rows at 2 bytes per coordinate; the copy's row written with every touched row
        score_bytes -= pairs * (row // 2)
        table_bytes += touched * (row // 2)
    if box:   # boxes at the roots are two rows wide; two MLPs over the inputs of the intersections, none elsewhere
        score_bytes += pexp["n_roots"] * 2 * row
        mlp_rows = 2 * pexp["n_int_rows"]
    mlp_flops = 4 * cfg.d * cfg.h * mlp_rows       # two layers, 2 flops per multiply-add
    models = {
        "score": ("hbm", score_bytes, HBM_PEAK_GBS, "GB/s"),
        "table_E": ("hbm", table_bytes, HBM_PEAK_GBS, "GB/s"),
        "gemm_fwd": ("mfma", mlp_flops, MFMA_F32_PEAK_TF, "TFLOP/s"),
        "gemm_bwd": ("mfma", mlp_flops, MFMA_F32_PEAK_TF, "TFLOP/s"),
        "wgrad": ("mfma", mlp_flops, MFMA_F32_PEAK_TF, "TFLOP/s"),
    }
    if sem:   # projection of the touched rows and its weight gradient, 2 flops per multiply-add each
        models["sem"] = ("mfma", 4 * touched * cfg.d * cfg.d_sem, MFMA_BF16_PEAK_TF, "TFLOP/s")
    return models


VALU_PEAK_TOPS = 39.3     # 256 CUs x 4 SIMDs x 16 lanes x 2.4 GHz, one fp32 op per lane and clock
                          # (packed forms are switched off in this build)


def rank_bench(args, cfg, kg, params, sem_bits, box=False):
    """All-entity ranking pass (ngdb_score without candidates): Q queries against every entity,
    top-10 by L1 distance.  One step = one pass.  Prints ONE JSON line."""
    from oracle import box as ob
    from oracle import model as om
    from oracle import rank as orank
    Q, k = args.rank, 10
    qb = wl.make_batch(kg, Q, cfg.mix, cfg.seed + 7)
    cpu = None
    sample = args.cpu_sample if args.cpu_sample >= 0 else (2 if cfg.N <= 100000 else 0)
    if sample > 0:
        say("CPU oracle ranking of %d queries" % sample)
        M = ob.BoxModel(params, cfg.gamma, args.box_alpha) if box else om.Model(params, cfg.gamma, sem_bits)
        t0 = time.perf_counter()
        for q in range(sample):
            orank.topk_all(qb, q, M, k, ob.distances_all if box else orank.distances_all)
        dtc = time.perf_counter() - t0
        cpu = {"value": sample / dtc, "unit": "queries/s", "cores": os.cpu_count(), "kind": "oracle",
               "sample": "%d queries against all %d entities (fp64 numpy, BLAS threads as configured), %.1f s"
                         % (sample, cfg.N, dtc)}
        del M
    import torch
    from paper_2602_21597_amd import Engine
    eng = Engine(cfg.N, cfg.R, cfg.d, cfg.h, cfg.gamma, d_sem=cfg.d_sem, family=1 if box else 0,
                 box_alpha=args.box_alpha)
    eng.bind_numpy(params, sem_bits=sem_bits)
    plan = eng.plan(qb)
    rows = plan.export()["n_roots"]
    if args.answers > 0:      # evaluation: filtered ranks of A listed answers per query (the positive first)
        rng = np.random.default_rng(cfg.seed + 9)
        ans = rng.integers(0, cfg.N, (Q, args.answers)).astype(np.int32)
        ans[:, 0] = qb.pos
        ans_off = torch.arange(0, Q * args.answers + 1, args.answers, dtype=torch.int32, device="cuda")
        ans_dev = torch.from_numpy(ans.reshape(-1)).cuda()
        run = lambda: eng.rank_answers(plan, ans_off, ans_dev)
    else:
        run = lambda: eng.rank_all(plan, k)
    for _ in range(args.warmup):
        run()
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(args.steps):
        run()
    torch.cuda.synchronize()
    dt = (time.perf_counter() - t0) / args.steps
    eng.set_timing(("score",))
    eng.get_timing(reset=True)
    for _ in range(args.steps):
        run()
    ms, n = eng.get_timing(reset=True)["score"]
    # subtract and |.|-accumulate per coordinate, branch row and entity (box distance: subtract,
    # scale, subtract the shrunk offset, maximum, accumulate)
    ops = (5.0 if box else 2.0) * rows * cfg.N * cfg.d
    ach = ops / (ms / n * 1e-3) / 1e12
    what = "top-%d" % k if args.answers <= 0 else "filtered ranks of %d answers per query, MRR, Hit@k" % args.answers
    out = {"metric": "all-entity ranking queries/sec (forward + L1 distance to every entity + %s)" % what,
           "value": Q / dt, "unit": "queries/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
           "ms_per_step": 1e3 * dt, "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
           "dtype": "f32", "data": "synthetic",
           "config": {"workload": "configs[%d] %s ranking pass: %d queries (%d branch rows) x N=%d entities, d=%d%s, top-%d"
                      % (cfg.index, cfg.name + (" (box family, alpha=%g)" % args.box_alpha if box else ""), Q, rows,
                         cfg.N, cfg.d, " d_sem=%d" % cfg.d_sem if cfg.d_sem else "", k), "evaluation": what},
           "roofline": {"bound": "alu", "kernel": "rank (distance tiles + %s%s)" % (
                            "top-k merge" if args.answers <= 0 else "closer-entity counts",
                            " + projection of every entity chunk" if cfg.d_sem else ""),
                        "achieved": ach, "peak": VALU_PEAK_TOPS, "unit": "Tlane-op/s", "frac": ach / VALU_PEAK_TOPS,
                        "traffic": None, "avg_us": 1e3 * ms / n,
                        "algorithmic_work_per_launch": ops},
           "cpu_baseline": cpu}
    print(json.dumps(out))


def calibrate_hbm(args):
    """What this machine delivers for the access patterns of the step's memory-bound kernels, without
    their arithmetic (ngdb_debug_stream): plain copy / read / write of 4 GiB, the scoring kernel's
    gather (B*(K+1) random rows of d floats out of an N-row table) and the table kernel's update
    (the rows of three N-row tables that a step touches, in ascending order).  Shapes of --config.
    Prints ONE JSON line; every figure is bytes moved / HIP-event time of 5 launches."""
    import torch
    from paper_2602_21597_amd import binding as nb
    cfg = wl.get_config(args.config)
    rng = np.random.default_rng(7)
    dev = torch.device("cuda:0")
    big = 1 << 32
    src = torch.empty(big, dtype=torch.uint8, device=dev)
    dst = torch.empty(big, dtype=torch.uint8, device=dev)
    src.zero_(); dst.zero_()
    sink = torch.zeros(4, dtype=torch.float32, device=dev)
    table = torch.zeros((3, cfg.N, cfg.d), dtype=torch.float32, device=dev)
    n_pairs = cfg.B * (cfg.K + 1)
    gather_rows = torch.from_numpy(rng.integers(0, cfg.N, n_pairs, dtype=np.int32)).to(dev)
    touched = np.unique(np.concatenate([gather_rows.cpu().numpy(), rng.integers(0, cfg.N, 2 * cfg.B, dtype=np.int32)]))
    upd_rows = torch.from_numpy(touched.astype(np.int32)).to(dev)
    row = 4 * cfg.d
    cases = [
        ("copy", lambda: nb.debug_stream(nb.STREAM_COPY, dst, src), 2 * big),
        ("read", lambda: nb.debug_stream(nb.STREAM_READ, sink, src), big),
        ("write", lambda: nb.debug_stream(nb.STREAM_WRITE, dst), big),
        ("gather_rows", lambda: nb.debug_stream(nb.STREAM_GATHER, sink, table[0], gather_rows, cfg.d), n_pairs * row),
        ("update_rows", lambda: nb.debug_stream(nb.STREAM_UPDATE, table, None, upd_rows, cfg.d,
                                                nbytes=table.numel() * 4), len(touched) * 6 * row),
        ("copy_nontemporal", lambda: nb.debug_stream(nb.STREAM_COPY_NT, dst, src), 2 * big),
        ("update_rows_nontemporal", lambda: nb.debug_stream(nb.STREAM_UPDATE_NT, table, None, upd_rows, cfg.d,
                                                            nbytes=table.numel() * 4), len(touched) * 6 * row),
    ]
    out = {"calibration": "HBM access patterns at the shapes of configs[%d] %s: N=%d d=%d, %d gathered rows, %d updated rows"
                          % (cfg.index, cfg.name, cfg.N, cfg.d, n_pairs, len(touched)), "peak_GBs": HBM_PEAK_GBS}
    for name, fn, nbytes in cases:
        fn()
        torch.cuda.synchronize()
        a, b = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        a.record()
        for _ in range(5):
            fn()
        b.record()
        torch.cuda.synchronize()
        gbs = 5 * nbytes / (a.elapsed_time(b) * 1e-3) / 1e9
        out[name] = {"GBs": gbs, "frac_of_peak": gbs / HBM_PEAK_GBS, "bytes_per_launch": nbytes,
                     "ms_per_launch": a.elapsed_time(b) / 5}
        say("%s: %.0f GB/s" % (name, gbs))
    print(json.dumps(out))


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=200)
    ap.add_argument("--warmup", type=int, default=20)
    ap.add_argument("--config", type=int, default=1)
    ap.add_argument("--streams", type=int, default=0, help="0 = the workload's default")
    ap.add_argument("--cpu-sample", type=int, default=-1, help="queries timed on the CPU oracle (0 = skip)")
    ap.add_argument("--schedule", choices=("level", "max_fill"), default="level",
                    help="order of execution of the operators (max_fill: the ready-set loop of Alg. 1)")
    ap.add_argument("--family", choices=("vec", "box"), default="vec",
                    help="operator family: the vector model of the headline workload, or box embeddings (Q2B "
                         "operators) on the 9 negation-free structures of the same workload")
    ap.add_argument("--score-bf16", action="store_true",
                    help="candidate rows from a bf16 copy of the entity table (optional mode, not the headline)")
    ap.add_argument("--box-alpha", type=float, default=0.02, help="weight of the inside distance (box family)")
    ap.add_argument("--bmax", type=int, default=0, help="largest batch of one Max-Fillness step, 0 = unbounded")
    ap.add_argument("--sampler", type=int, default=0, metavar="THREADS",
                    help="draw every batch (queries and negatives) inside the run with the library's online sampler "
                         "on this many threads, instead of cycling pre-generated batches")
    ap.add_argument("--rank", type=int, default=0, metavar="Q",
                    help="time the all-entity ranking pass of Q queries instead of the training step")
    ap.add_argument("--answers", type=int, default=0, metavar="A",
                    help="with --rank: filtered ranks of A listed answers per query instead of the top-10")
    ap.add_argument("--calibrate-copy", type=int, default=0, metavar="MiB",
                    help="also run the library's plain copy kernel on this many MiB, 5 times (reference "
                         "for scaling rocprofv3 traffic counters)")
    ap.add_argument("--calibrate-hbm", action="store_true",
                    help="instead of the step: plain copy / read / write and the row gather and row update "
                         "patterns of the scoring and table kernels at the shapes of --config (no arithmetic)")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build runs on one GPU; --gpus %d is not supported (no sharding, no collectives)"
              % args.gpus, file=sys.stderr)
        sys.exit(2)
    if args.calibrate_hbm:
        return calibrate_hbm(args)

    cfg = wl.get_config(args.config)
    box = args.family == "box"
    if box:
        if cfg.d_sem:
            print("bench.py: the box family has no text features", file=sys.stderr)
            sys.exit(2)
        import dataclasses
        cfg = dataclasses.replace(cfg, mix={n: 1.0 / len(wl.EPFO9) for n in wl.EPFO9})
    say("generating the graph (N=%d, T=%d)" % (cfg.N, cfg.T))
    kg = wl.make_kg(cfg.N, cfg.R, cfg.T, cfg.alpha, cfg.seed)
    if args.rank:
        params = (wl.make_box_params(cfg.N, cfg.R, cfg.d, cfg.h, cfg.seed + 3) if box else
                  wl.make_params(cfg.N, cfg.R, cfg.d, cfg.h, cfg.seed + 3, d_sem=cfg.d_sem))
        sem_bits = wl.make_sem_features(cfg.N, cfg.d_sem, cfg.seed + 5) if cfg.d_sem else None
        return rank_bench(args, cfg, kg, params, sem_bits, box)
    say("generating %d batches of %d queries, negatives, parameters" % (N_BATCHES, cfg.B))
    batches = [wl.make_batch(kg, cfg.B, cfg.mix, cfg.seed + 10 + i) for i in range(N_BATCHES)]
    negs_np = [wl.make_negatives(cfg.N, cfg.B, cfg.K, cfg.seed + 50 + i) for i in range(N_BATCHES)]
    params = (wl.make_box_params(cfg.N, cfg.R, cfg.d, cfg.h, cfg.seed + 3) if box else
              wl.make_params(cfg.N, cfg.R, cfg.d, cfg.h, cfg.seed + 3, d_sem=cfg.d_sem))
    sem_bits = wl.make_sem_features(cfg.N, cfg.d_sem, cfg.seed + 5) if cfg.d_sem else None

    # CPU oracle first, before this process touches the GPU
    default_sample = 512 if cfg.K <= 128 else (8 if cfg.d_sem else 64)
    sample = args.cpu_sample if args.cpu_sample >= 0 else min(cfg.B, default_sample)
    say("CPU oracle on %d queries" % sample)
    cpu = cpu_baseline(cfg, kg, sample, sem_bits, args.box_alpha if box else None, args.score_bf16) if sample > 0 else None
    say("uploading parameters")

    import torch
    from paper_2602_21597_amd import Engine
    streams = args.streams or cfg.streams
    eng = Engine(cfg.N, cfg.R, cfg.d, cfg.h, cfg.gamma, lr=cfg.lr, beta1=cfg.beta1, beta2=cfg.beta2, eps=cfg.eps,
                 num_streams=streams, d_sem=cfg.d_sem, schedule={"level": 0, "max_fill": 1}[args.schedule],
                 b_max=args.bmax, family=1 if box else 0, box_alpha=args.box_alpha, score_bf16=args.score_bf16)
    eng.bind_numpy(params, sem_bits=sem_bits)
    del params, sem_bits
    negs = [torch.from_numpy(n).cuda() for n in negs_np]
    stream = torch.cuda.current_stream()

    # Producer/consumer (Sec. 4.3): batch t+1 is planned on a second host thread while step t
    # is enqueued and runs; every batch of the run is planned inside the run.
    planner = ThreadPoolExecutor(1)
    sampler = None
    if args.sampler:
        from paper_2602_21597_amd import Sampler
        names = sorted(cfg.mix)
        sampler = Sampler(cfg.N, cfg.R, kg.head, kg.rel, kg.tail, names, [cfg.mix[n] for n in names], cfg.seed,
                          args.sampler)
        neg_host = [torch.empty((cfg.B, cfg.K), dtype=torch.int32).pin_memory() for _ in range(2)]
        neg_dev = [torch.empty((cfg.B, cfg.K), dtype=torch.int32, device="cuda") for _ in range(2)]
        copied = [torch.cuda.Event() for _ in range(2)]     # upload of a pinned buffer has finished
        for ev in copied:
            ev.record(stream)

    def produce(i):
        """Producer side of one step: with the sampler, a fresh batch and its negatives; the plan."""
        if sampler is None:
            return eng.plan(batches[i % N_BATCHES]), None
        c_batch, neg_view = sampler.next_raw(cfg.B, cfg.K)
        copied[i % 2].synchronize()            # the upload two steps ago has left this buffer
        neg_host[i % 2].numpy()[:] = neg_view
        return eng.plan(c_batch), i % 2

    def run_steps(first, count):
        nxt = planner.submit(produce, first) if count > 0 else None
        for i in range(first, first + count):
            plan, slot = nxt.result()
            if slot is None:
                neg = negs[i % N_BATCHES]
            else:                      # negatives of this batch: pinned host -> device on the compute stream
                neg_dev[slot].copy_(neg_host[slot], non_blocking=True)
                copied[slot].record(stream)
                neg = neg_dev[slot]
            if i + 1 < first + count:
                nxt = planner.submit(produce, i + 1)
            eng.train_step(plan, neg, stream)
            plan.free()        # the library recycles the plan's buffers once the step has finished

    say("warm-up")
    run_steps(0, args.warmup)
    torch.cuda.synchronize()
    say("timing %d steps" % args.steps)

    # the timed region: K whole steps (planning included), nothing else on the device
    t0 = time.perf_counter()
    run_steps(args.warmup, args.steps)
    torch.cuda.synchronize()
    dt = time.perf_counter() - t0

    # device-only time of the same steps with plans prebuilt (context figure)
    plans = [eng.plan(b) for b in batches]
    torch.cuda.synchronize()
    t1 = time.perf_counter()
    for i in range(args.steps):
        eng.train_step(plans[i % N_BATCHES], negs[i % N_BATCHES], stream)
    torch.cuda.synchronize()
    dt_dev = time.perf_counter() - t1

    say("kernel classes")
    # the same steps once more with every kernel class bracketed by HIP events on its own stream
    eng.set_timing(CLASSES)
    eng.get_timing(reset=True)
    for i in range(args.steps):
        eng.train_step(plans[i % N_BATCHES], negs[i % N_BATCHES], stream)
    timing = eng.get_timing(reset=True)
    eng.set_timing(())
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

    # roofline per kernel class: algorithmic work of one step / measured time of the class per step.
    # The three contraction classes are launches of one kernel and are reported together as "gemm".
    models = kernel_models(cfg, pexp, touched, box, args.score_bf16)
    kern = {}
    for name, (bound, amount, peak, unit) in models.items():
        ms, n = timing[name]
        if n:
            kern[name] = {"bound": bound, "ms_per_step": ms / args.steps, "launches_per_step": n / args.steps,
                          "avg_us": 1e3 * ms / n, "work_per_step": amount, "unit": unit, "peak": peak}
    gemm = [kern.pop(k) for k in ("gemm_fwd", "gemm_bwd", "wgrad") if k in kern]
    if gemm:
        tot_ms = sum(g["ms_per_step"] for g in gemm)
        n_l = sum(g["launches_per_step"] for g in gemm)
        kern["gemm"] = {"bound": "mfma", "ms_per_step": tot_ms, "launches_per_step": n_l,
                        "avg_us": 1e3 * tot_ms / n_l, "work_per_step": sum(g["work_per_step"] for g in gemm),
                        "unit": "TFLOP/s", "peak": MFMA_F32_PEAK_TF}
    for k in kern.values():
        scale = 1e9 if k["bound"] == "hbm" else 1e12
        k["achieved"] = k["work_per_step"] / (k["ms_per_step"] * 1e-3) / scale
        k["frac"] = k["achieved"] / k["peak"]
    dom = max(kern, key=lambda k: kern[k]["ms_per_step"])
    kd = kern[dom]
    traffic = None if args.score_bf16 else MEASURED_TRAFFIC.get(("box", cfg.index, dom) if box else (cfg.index, dom))
    roofline = {"bound": kd["bound"], "kernel": dom, "achieved": kd["achieved"], "peak": kd["peak"],
                "unit": kd["unit"], "frac": kd["frac"], "traffic": traffic,
                "avg_us": kd["avg_us"], "launches_per_step": kd["launches_per_step"],
                "algorithmic_work_per_launch": kd["work_per_step"] / kd["launches_per_step"],
                "other": {k: {f: v[f] for f in ("bound", "achieved", "peak", "unit", "frac", "avg_us",
                                                "launches_per_step", "ms_per_step")}
                          for k, v in kern.items() if k != dom}}
    if dom == "gemm":
        # fp32 contractions, priced against the fp32 matrix peak; the split route (six bf16 MFMAs per
        # fp32 product block) has a ceiling of its own, the bf16 peak over six
        roofline["peak_basis"] = ("fp32 MFMA peak; the bf16-split route's own ceiling is %.0f TFLOP/s (bf16 peak / 6)"
                                  % (MFMA_BF16_PEAK_TF / 6.0))

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
        "config": {"workload": "configs[%d] %s: N=%d R=%d d=%d h=%d B=%d K=%d%s, %s, gamma=%g"
                   % (cfg.index, cfg.name, cfg.N, cfg.R, cfg.d, cfg.h, cfg.B, cfg.K,
                      " d_sem=%d (bf16 text features)" % cfg.d_sem if cfg.d_sem else "",
                      "box family (alpha=%g) on the 9 negation-free structures" % args.box_alpha if box
                      else "14-structure mix" + (", candidate rows from a bf16 copy of E" if args.score_bf16 else ""),
                      cfg.gamma),
                   "contractions": "fp32 results; operands split exactly into three bf16 pieces, six partial products on "
                                   "the bf16 MFMA with fp32 accumulation (fp32 MFMA for the small weight-gradient tiles)",
                   "streams": streams,
                   "schedule": args.schedule if args.schedule == "level" else "max_fill, B_max=%s" % (args.bmax or "inf"),
                   "steps_per_batch": pexp["n_levels"], "peak_live_outputs": pexp["peak_live"],
                   "operator_outputs": pexp["n_slots"],
                   "step": ("ngdb_sampler_next + " if args.sampler else "") +
                           "ngdb_plan of batch t+1 on a second host thread while ngdb_train_step of batch t is enqueued",
                   "batches": "online sampler, %d threads" % args.sampler if args.sampler else
                              "%d pre-generated batches cycled" % N_BATCHES,
                   "touched_entity_rows": touched},
        "device_only": {"queries_per_s": cfg.B * args.steps / dt_dev, "ms_per_step": 1e3 * dt_dev / args.steps,
                        "note": "same steps with plans prebuilt"},
        "roofline": roofline,
        "cpu_baseline": cpu,
        "kernel_classes_ms_per_step": {k: v[0] / args.steps for k, v in timing.items()},
    }
    if copy_gbs is not None:
        out["copy_kernel_GBs"] = copy_gbs
    print(json.dumps(out))


if __name__ == "__main__":
    main()
