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

def _cpu_worker(job, barrier=None, out=None):
    """One worker process of the CPU baseline: full oracle steps (loss, gradients, Adam) on its share
    of every batch, BLAS held to one thread; inputs are built first, the steps start together."""
    cfg, kg, sem_bits, box_alpha, score_bf16, share, n_steps, worker = job
    from oracle import box as ob
    from oracle import model as om
    try:
        from threadpoolctl import threadpool_limits
        limit = threadpool_limits(limits=1)
    except Exception:                      # pragma: no cover
        limit = None
    box = box_alpha is not None
    P = om.to_f64(wl.make_box_params(cfg.N, cfg.R, cfg.d, cfg.h, cfg.seed + 3) if box else
                  wl.make_params(cfg.N, cfg.R, cfg.d, cfg.h, cfg.seed + 3, d_sem=cfg.d_sem))
    st = om.new_state(P)
    hp = dict(lr=cfg.lr, beta1=cfg.beta1, beta2=cfg.beta2, eps=cfg.eps, gamma=cfg.gamma, alpha=box_alpha)
    batches = [(wl.make_batch(kg, share, cfg.mix, cfg.seed + 100 + 977 * worker + k),
                wl.make_negatives(cfg.N, share, cfg.K, cfg.seed + 200 + 977 * worker + k)) for k in range(n_steps)]
    if barrier is not None:
        barrier.wait()
    t0 = time.time()
    for k, (qb, negs) in enumerate(batches):
        if box:
            ob.train_step(qb, negs, P, st, k + 1, hp)
        else:
            om.train_step(qb, negs, P, st, k + 1, hp, sem_bits, score_bf16=score_bf16)
    t1 = time.time()
    del limit
    if out is not None:
        out.put((share * n_steps, t0, t1))
    return share * n_steps, t0, t1


def cpu_baseline(cfg, kg, sample, sem_bits, box_alpha=None, score_bf16=False, cores=None):
    """The oracle as it stands on the host's cores: `sample` queries per step are split over one
    worker process per core (forked before this process touches the GPU); every worker runs full
    oracle steps (per-query fp64 numpy forward, loss, backward, Adam) on its share.  The figure is
    all queries done / wall time from the common start of the steps to the end of the last worker."""
    import multiprocessing as mp
    cores = cores or host_cores()
    cores = max(1, min(cores, sample))
    share = max(1, sample // cores)
    # a few queries on one core size the run: about 10 s of wall time, at most 8 steps
    probe = min(share, 4)
    _, t0, t1 = _cpu_worker((cfg, kg, sem_bits, box_alpha, score_bf16, probe, 1, 0))
    n_steps = int(max(1, min(8, 10.0 / max((t1 - t0) / probe * share, 1e-9))))
    ctx = mp.get_context("fork")
    barrier, out = ctx.Barrier(cores), ctx.Queue()
    procs = [ctx.Process(target=_cpu_worker, args=((cfg, kg, sem_bits, box_alpha, score_bf16, share, n_steps, w),
                                                   barrier, out)) for w in range(cores)]
    for pr in procs:
        pr.start()
    done = [out.get() for _ in procs]
    for pr in procs:
        pr.join()
    wall = max(t for _, _, t in done) - min(t for _, t, _ in done)
    queries = sum(q for q, _, _ in done)
    return {"value": queries / wall, "unit": "queries/s", "cores": cores, "kind": "oracle",
            "sample": "%d steps of %d queries of the same workload with all %d negatives, split over %d worker "
                      "processes (one per core, %d queries each per step; per-query fp64 numpy forward, loss, backward, "
                      "Adam), %.1f s wall, %.1f s of CPU time" % (n_steps, share * cores, cfg.K, cores, share, wall,
                                                                  sum(b - a for _, a, b in done))}


def host_cores():
    """Cores this process may use: the scheduler's affinity mask, capped by the thread count the
    environment configures for numerical libraries (the share of the machine that goes with one GPU)."""
    try:
        n = len(os.sched_getaffinity(0))
    except Exception:                      # pragma: no cover
        n = os.cpu_count() or 1
    cap = os.environ.get("OMP_NUM_THREADS", "")
    if cap.isdigit() and int(cap) > 0:
        n = min(n, int(cap))
    return max(1, n)


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


PROFILE_NAMES = {1: "fb15k237", 2: "nell", 3: "wikikg2", 4: "text_features"}


def profile_figures(cfg, box):
    """Per kernel class, what the tracked rocprofv3 summaries under profiles/ hold for this workload:
    {class: {"avg_us": .., "launches_per_step": .., "traffic": bytes per launch (FETCH_SIZE + WRITE_SIZE,
    scaled by the copy kernel)}}, from the lines `class <name> launches_per_step <n> avg_us <t>` of
    train_step_<workload>_kernel_stats.txt and `traffic <name> <bytes>` of ..._hbm_traffic.txt."""
    name = ("box_" if box else "") + PROFILE_NAMES.get(cfg.index, "")
    out, files = {}, []
    for kind in ("kernel_stats", "hbm_traffic"):
        path = os.path.join(ROOT, "profiles", "train_step_%s_%s.txt" % (name, kind))
        if not os.path.exists(path):
            continue
        files.append(os.path.relpath(path, ROOT))
        for line in open(path):
            w = line.split()
            try:
                if len(w) == 6 and w[0] == "class" and w[2] == "launches_per_step" and w[4] == "avg_us":
                    out.setdefault(w[1], {}).update(launches_per_step=float(w[3]), avg_us=float(w[5]))
                elif len(w) == 3 and w[0] == "traffic":
                    out.setdefault(w[1], {})["traffic"] = float(w[2])
            except ValueError:
                pass
    return out, files


def measure_workload(cfg, args, kg, steps, warmup, box=False, streams=None):
    """Runs the training step of one workload: K timed steps with planning inside the timed region,
    the same steps with plans prebuilt, and once more with every kernel class bracketed by HIP
    events.  Returns (figures for the JSON line, kernel classes with their rooflines)."""
    import torch
    from paper_2602_21597_amd import Engine
    say("generating %d batches of %d queries, negatives, parameters" % (N_BATCHES, cfg.B))
    batches = [wl.make_batch(kg, cfg.B, cfg.mix, cfg.seed + 10 + i) for i in range(N_BATCHES)]
    negs_np = [wl.make_negatives(cfg.N, cfg.B, cfg.K, cfg.seed + 50 + i) for i in range(N_BATCHES)]
    params = (wl.make_box_params(cfg.N, cfg.R, cfg.d, cfg.h, cfg.seed + 3) if box else
              wl.make_params(cfg.N, cfg.R, cfg.d, cfg.h, cfg.seed + 3, d_sem=cfg.d_sem))
    sem_bits = wl.make_sem_features(cfg.N, cfg.d_sem, cfg.seed + 5) if cfg.d_sem else None
    say("uploading parameters")
    streams = streams or args.streams or cfg.streams
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
    run_steps(0, warmup)
    torch.cuda.synchronize()
    say("timing %d steps" % steps)

    # the timed region: K whole steps (planning included), nothing else on the device
    t0 = time.perf_counter()
    run_steps(warmup, steps)
    torch.cuda.synchronize()
    dt = time.perf_counter() - t0

    # device-only time of the same steps with plans prebuilt (context figure)
    plans = [eng.plan(b) for b in batches]
    torch.cuda.synchronize()
    t1 = time.perf_counter()
    for i in range(steps):
        eng.train_step(plans[i % N_BATCHES], negs[i % N_BATCHES], stream)
    torch.cuda.synchronize()
    dt_dev = time.perf_counter() - t1

    say("kernel classes")
    # the same steps once more with every kernel class bracketed by HIP events on its own stream
    eng.set_timing(CLASSES)
    eng.get_timing(reset=True)
    for i in range(steps):
        eng.train_step(plans[i % N_BATCHES], negs[i % N_BATCHES], stream)
    timing = eng.get_timing(reset=True)
    routes = eng.last_routes
    eng.set_timing(())
    touched = eng.n_touched_entities()
    pexp = plans[(steps - 1) % N_BATCHES].export()

    # roofline per kernel class: algorithmic work of one step / measured time of the class per step.
    # Contractions are reported by the matrix instructions their launches ran on: the fp32 ones
    # against the fp32 matrix peak; the ones on split operands execute six bf16 products per fp32
    # product and are priced with those executed flops against the bf16 matrix peak (their
    # algorithmic rate is a sixth of that).
    models = kernel_models(cfg, pexp, touched, box, args.score_bf16)
    kern = {}
    for name, (bound, amount, peak, unit) in models.items():
        ms, n = timing[name]
        if n and bound == "hbm" or (n and name == "sem"):
            kern[name] = {"bound": bound, "ms_per_step": ms / steps, "launches_per_step": n / steps,
                          "avg_us": 1e3 * ms / n, "work_per_step": amount, "unit": unit, "peak": peak}
    for route, peak, factor in (("fp32", MFMA_F32_PEAK_TF, 1.0), ("bf16_split", MFMA_BF16_PEAK_TF, 6.0)):
        ms = sum(routes[c][route][0] for c in ("gemm_fwd", "gemm_bwd", "wgrad"))
        n = sum(routes[c][route][1] for c in ("gemm_fwd", "gemm_bwd", "wgrad"))
        flop = sum(routes[c][route][2] for c in ("gemm_fwd", "gemm_bwd", "wgrad"))
        if n:
            kern["gemm_" + route] = {"bound": "mfma", "ms_per_step": ms / steps, "launches_per_step": n / steps,
                                     "avg_us": 1e3 * ms / n, "work_per_step": factor * flop / steps, "unit": "TFLOP/s",
                                     "peak": peak, "algorithmic_TFLOPs": flop / (ms * 1e-3) / 1e12,
                                     "executed_per_algorithmic_flop": factor}
    prof, prof_files = profile_figures(cfg, box)
    for name, k in kern.items():
        scale = 1e9 if k["bound"] == "hbm" else 1e12
        k["achieved"] = k["work_per_step"] / (k["ms_per_step"] * 1e-3) / scale
        k["frac"] = k["achieved"] / k["peak"]
        k["algorithmic_work_per_launch"] = k["work_per_step"] / k["launches_per_step"]
        pf = prof.get(name, {})
        k["traffic"] = pf.get("traffic")
        if "avg_us" in pf:      # the same class in the tracked rocprofv3 summary (kernel durations, no event brackets)
            per_step_us = pf["avg_us"] * pf["launches_per_step"]
            k["profile"] = {"avg_us": pf["avg_us"], "launches_per_step": pf["launches_per_step"],
                            "frac": k["work_per_step"] / (per_step_us * 1e-6) / scale / k["peak"]}
    res = {
        "queries_per_s": cfg.B * steps / dt, "ms_per_step": 1e3 * dt / steps,
        "device_only": {"queries_per_s": cfg.B * steps / dt_dev, "ms_per_step": 1e3 * dt_dev / steps,
                        "note": "same steps with plans prebuilt"},
        "workload": "configs[%d] %s: N=%d R=%d d=%d h=%d B=%d K=%d%s, %s, gamma=%g"
                    % (cfg.index, cfg.name, cfg.N, cfg.R, cfg.d, cfg.h, cfg.B, cfg.K,
                       " d_sem=%d (bf16 text features)" % cfg.d_sem if cfg.d_sem else "",
                       "box family (alpha=%g) on the 9 negation-free structures" % args.box_alpha if box
                       else "14-structure mix" + (", candidate rows from a bf16 copy of E" if args.score_bf16 else ""),
                       cfg.gamma),
        "streams": streams, "touched_entity_rows": touched, "steps_per_batch": pexp["n_levels"],
        "peak_live_outputs": pexp["peak_live"], "operator_outputs": pexp["n_slots"],
        "kernel_classes_ms_per_step": {k: v[0] / steps for k, v in timing.items()},
        "profile_files": prof_files,
        # activation memory of a forward-only pass (ngdb_score, ngdb_rank_answers) over this batch: one row
        # per operator output and MLP row, against outputs reclaimed once their consumer has run (eager
        # reference counting, Sec. 4.3) with the per-type MLP buffers holding one step at a time
        "forward_only_activation_bytes": {
            "one_row_per_output": 4 * (pexp["n_slots"] * cfg.d + (pexp["n_proj"] + pexp["n_int_rows"] + pexp["n_neg"])
                                       * (cfg.d + cfg.h) + pexp["n_int_rows"] * cfg.d),
            "reclaimed": 4 * (pexp["n_f_rows"] * cfg.d + int(pexp["f_step_rows"].sum()) * (cfg.d + cfg.h)
                              + int(pexp["f_step_rows"][1]) * cfg.d)},
    }
    for p_ in plans:
        p_.free()
    del eng, negs, plans
    torch.cuda.empty_cache()
    return res, kern


ROOFLINE_FIELDS = ("bound", "achieved", "peak", "unit", "frac", "traffic", "avg_us", "launches_per_step",
                   "ms_per_step", "algorithmic_work_per_launch", "algorithmic_TFLOPs",
                   "executed_per_algorithmic_flop", "profile")


def roofline_of(kern):
    """The class with the largest time per step as the line's roofline object, the others beside it."""
    dom = max(kern, key=lambda k: kern[k]["ms_per_step"])
    pick = lambda v: {f: v[f] for f in ROOFLINE_FIELDS if f in v}
    out = dict(pick(kern[dom]), kernel=dom)
    out["other"] = {k: pick(v) for k, v in kern.items() if k != dom}
    return out


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=200)
    ap.add_argument("--warmup", type=int, default=20)
    ap.add_argument("--config", type=int, default=1)
    ap.add_argument("--streams", type=int, default=0, help="0 = the workload's default")
    ap.add_argument("--cpu-sample", type=int, default=-1, help="queries per step timed on the CPU oracle (0 = skip)")
    ap.add_argument("--others", default="", metavar="LIST",
                    help="workloads measured beside the headline one and reported under other_workloads "
                         "(comma separated config numbers; default: 2,3 beside config 1, none otherwise; 'none')")
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

    # CPU oracle first, on all host cores, before this process touches the GPU
    default_sample = 512 if cfg.K <= 128 else (16 if cfg.d_sem else 64)
    sample = args.cpu_sample if args.cpu_sample >= 0 else min(cfg.B, default_sample)
    cpu = None
    if sample > 0:
        say("CPU oracle on %d queries per step, %d cores" % (sample, host_cores()))
        sem_bits = wl.make_sem_features(cfg.N, cfg.d_sem, cfg.seed + 5) if cfg.d_sem else None
        cpu = cpu_baseline(cfg, kg, sample, sem_bits, args.box_alpha if box else None, args.score_bf16)
        del sem_bits

    res, kern = measure_workload(cfg, args, kg, args.steps, args.warmup, box)
    del kg

    others = args.others or ("2,3" if args.config == 1 and not box and not args.sampler and not args.score_bf16 else "none")
    other_workloads = {}
    for idx in ([] if others == "none" else [int(x) for x in others.split(",")]):
        ocfg = wl.get_config(idx)
        say("other workload: configs[%d] %s; generating the graph (N=%d, T=%d)" % (idx, ocfg.name, ocfg.N, ocfg.T))
        okg = wl.make_kg(ocfg.N, ocfg.R, ocfg.T, ocfg.alpha, ocfg.seed)
        o_steps = args.steps if ocfg.K <= 128 else max(5, min(args.steps, 20))
        ores, okern = measure_workload(ocfg, args, okg, o_steps, min(args.warmup, 5), False, streams=ocfg.streams)
        del okg
        pick = lambda v: {f: v[f] for f in ROOFLINE_FIELDS if f in v}
        other_workloads["configs[%d]" % idx] = {
            "workload": ores["workload"], "queries_per_s": ores["queries_per_s"], "ms_per_step": ores["ms_per_step"],
            "steps": o_steps, "device_only": ores["device_only"], "streams": ores["streams"],
            "touched_entity_rows": ores["touched_entity_rows"],
            "forward_only_activation_bytes": ores["forward_only_activation_bytes"],
            "kernels": {k: pick(v) for k, v in okern.items()}, "profile_files": ores["profile_files"]}

    copy_gbs = None
    if args.calibrate_copy:
        import torch
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

    out = {
        "metric": "training queries/sec (fwd+bwd+Adam) at d=400, K=128 negatives; % of HBM peak",
        "value": res["queries_per_s"],
        "unit": "queries/s",
        "n_gpus": 1,
        "steps": args.steps,
        "warmup": args.warmup,
        "ms_per_step": res["ms_per_step"],
        "higher_is_better": True,
        "scaling": "weak",
        "vs_baseline": None,
        "dtype": "f32",
        "data": "synthetic",
        "config": {"workload": res["workload"],
                   "contractions": "fp32 results; operands split exactly into three bf16 pieces, six partial products on "
                                   "the bf16 MFMA with fp32 accumulation (fp32 MFMA for small weight-gradient tiles)",
                   "streams": res["streams"],
                   "schedule": args.schedule if args.schedule == "level" else "max_fill, B_max=%s" % (args.bmax or "inf"),
                   "steps_per_batch": res["steps_per_batch"], "peak_live_outputs": res["peak_live_outputs"],
                   "operator_outputs": res["operator_outputs"],
                   "step": ("ngdb_sampler_next + " if args.sampler else "") +
                           "ngdb_plan of batch t+1 on a second host thread while ngdb_train_step of batch t is enqueued",
                   "batches": "online sampler, %d threads" % args.sampler if args.sampler else
                              "%d pre-generated batches cycled" % N_BATCHES,
                   "touched_entity_rows": res["touched_entity_rows"],
                   "forward_only_activation_bytes": res["forward_only_activation_bytes"]},
        "device_only": res["device_only"],
        "roofline": roofline_of(kern),
        "roofline_note": "achieved = algorithmic work of the class per step / HIP-event time of its launches on their own "
                         "stream (contractions on split operands: executed bf16 flops, six per fp32 product, against the "
                         "bf16 matrix peak); traffic and profile.* come from the rocprofv3 summaries named in profile_files",
        "profile_files": res["profile_files"],
        "cpu_baseline": cpu,
        "kernel_classes_ms_per_step": res["kernel_classes_ms_per_step"],
        "other_workloads": other_workloads,
    }
    if copy_gbs is not None:
        out["copy_kernel_GBs"] = copy_gbs
    print(json.dumps(out))


if __name__ == "__main__":
    main()
