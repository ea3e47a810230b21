#!/usr/bin/env python3
"""Benchmark of the vAttention decode step (libvatt) on one MI355X.

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--config 2|3|4|5] [--no-cpu]

A step is one vatt_decode call: the whole hot path (score pass, per-head selection / base sample /
statistics / budget / final sample, gather and merge) for one layer and one batch of synthetic input that
is already resident in HBM.  Calls cycle through `--buffers` distinct copies of the KV cache so that no
call finds its K/V in the 256 MB last-level cache.  Prints ONE JSON line.  The default run times config 2
(the headline: B = 1, 32K tokens), and adds two sub-objects: `batched` (config 3, B = 16, where the path is
bound by HBM bandwidth rather than by latency) and `adaptive_budget` (config 2 with a 32-token base sample,
where the budget rule sets the sample sizes).
--config 5 is the ragged paged decode loop (B=32, one appended token per sequence and step): it reports the step
latency distribution and the budgets of the last step instead of the roofline of the score kernel.
"""
import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

HBM_PEAK_GBPS = 8000.0   # MI355X HBM3E, published

# HBM bytes per score-kernel launch from two rocprofv3 --pmc runs of `bench.py --only score` (FETCH_SIZE, then
# WRITE_SIZE, KiB per dispatch), each scaled by what the same counter reads for `bench.py --only copy`, a
# 256 MiB device copy: FETCH_SIZE reads 131084.4 KiB for its 262144 KiB (factor 1.99981), WRITE_SIZE 262144
# (factor 1).  Score kernel at config 2: FETCH_SIZE 32827.5, WRITE_SIZE 4608.0; at config 3: 524827.5 and
# 73728.0.  The summaries are kept under profiles/.  Only the configurations that were measured have a figure.
SCORE_KERNEL_TRAFFIC_BYTES = {"config2": int((32827.5 * 262144.0 / 131084.4 + 4608.0) * 1024),
                              "config3": int((524827.5 * 262144.0 / 131084.4 + 73728.0) * 1024)}
# score_chunk_kernel, same two counters and scaling (config 2 with 4 query tokens)
SCORE_CHUNK_TRAFFIC_BYTES = {("config2", 4): int((32928.6 * 262144.0 / 131084.4 + 18432.7) * 1024)}
# HBM bytes of all kernels of one vatt_decode step, same two counters, scaled by what they read for a 256 MiB
# device copy (FETCH_SIZE x 1.99974, WRITE_SIZE x 1.0): profiles/decode_config{2,3,4}_kernel_stats.md
STEP_TRAFFIC_BYTES = {"config2": 91222118, "config3": 1537473331, "config4": 1421102828}
# rocprofv3 --kernel-trace --stats averages (us) of the kernels of one step, `python3 bench.py --no-cpu` under the
# profiler (profiles/decode_config2_kernel_stats.md, profiles/decode_config3_kernel_stats.md)
PROFILE_KERNEL_US = {
    "config2": {"score_kernel": 13.61, "head_kernel (selection with the gather fused in)": 23.49, "gather_merge_kernel": 4.29},
    "config3": {"score_kernel": 181.11, "head_kernel": 31.20, "gather_kernel": 41.14, "gather_merge_kernel": 4.47},
    "config4": {"score_kernel": 177.42, "head_kernel": 44.03, "gather_kernel": 30.33, "gather_merge_kernel": 4.40},
}
LLAMA8B_LAYERS = 32


def plan_params(wl):
    p = wl.params
    return dict(batch=wl.batch, n_q_heads=wl.n_q_heads, n_kv_heads=wl.n_kv_heads, head_dim=wl.head_dim,
                n_max=wl.n_max, kv_layout=0, page_size=0, num_blocks=0, sink=int(p["sink"]), window=int(p["window"]),
                topk_abs=int(p["topk_abs"]), topk_frac=float(p["topk_frac"]), base_abs=int(p["base_abs"]),
                base_frac=float(p["base_frac"]), epsilon=float(p["epsilon"]), delta=float(p["delta"]),
                target=int(p["target"]), sm_scale=float(p["sm_scale"]), budget_cap_frac=float(p["budget_cap_frac"]))


def time_calls(fn, n_calls, torch):
    """Average milliseconds per call of fn(i), bracketed by events on the current stream."""
    start = torch.cuda.Event(enable_timing=True)
    stop = torch.cuda.Event(enable_timing=True)
    torch.cuda.synchronize()
    start.record()
    for i in range(n_calls):
        fn(i)
    stop.record()
    torch.cuda.synchronize()
    return start.elapsed_time(stop) / n_calls


def cpu_baseline(wl, budget_s=12.0):
    """The oracle as it stands, one thread, on whole heads of the same workload until ~budget_s have passed."""
    import numpy as np
    from oracle import vatt_oracle as vo
    try:
        from threadpoolctl import threadpool_limits
        limiter = threadpool_limits(limits=1)
    except Exception:
        limiter = None
    g = wl.n_q_heads // wl.n_kv_heads
    q_all = wl.q_f32()
    t0 = time.perf_counter()
    done = 0
    total_heads = wl.batch * wl.n_q_heads
    while True:
        b, h = divmod(done % total_heads, wl.n_q_heads)
        n = int(wl.seq_lens[b])
        vo.decode_head(q_all[b, h].astype(np.float64), wl.k_f32(b, h // g, n).astype(np.float64),
                       wl.v_f32(b, h // g, n).astype(np.float64), seed=int(wl.seeds[b]), head=h, params=wl.params)
        done += 1
        el = time.perf_counter() - t0
        if el >= budget_s:
            break
    if limiter is not None:
        limiter.unregister() if hasattr(limiter, "unregister") else None
    us_per_layer = el / done * total_heads * 1e6
    return dict(value=us_per_layer, unit="us/layer", cores=1, kind="oracle",
                sample="%d (sequence, head) units of the same workload in %.1f s, scaled to the %d units of one layer"
                       % (done, el, total_heads))


def _cpu_worker(job):
    """One worker of the all-core oracle timing: whole heads of the workload, round robin, for budget_s."""
    config, rank, world, budget_s = job
    import numpy as np
    import workloads
    from oracle import vatt_oracle as vo
    wl = {2: workloads.config2, 3: workloads.config3, 4: workloads.config4}[config]()
    g = wl.n_q_heads // wl.n_kv_heads
    q_all = wl.q_f32()
    total = wl.batch * wl.n_q_heads
    t0 = time.perf_counter()
    done, unit = 0, rank
    while True:
        b, h = divmod(unit % total, wl.n_q_heads)
        n = int(wl.seq_lens[b])
        vo.decode_head(q_all[b, h].astype(np.float64), wl.k_f32(b, h // g, n).astype(np.float64),
                       wl.v_f32(b, h // g, n).astype(np.float64), seed=int(wl.seeds[b]), head=h, params=wl.params)
        done += 1
        unit += world
        el = time.perf_counter() - t0
        if el >= budget_s:
            return done, el


def cpu_baseline_all_cores(config, budget_s=8.0):
    """The same oracle in one process per host core the job may use (fresh processes that never touch the GPU),
    each on whole heads for about budget_s; the aggregate rate scaled to one layer."""
    import multiprocessing as mp
    import workloads
    cores = max(1, min(os.cpu_count() or 1, int(os.environ.get("OMP_NUM_THREADS", "16"))))
    if config != 2:
        cores = min(cores, 4)       # (every worker generates the workload for itself: bound the host memory)
    keep = {k: os.environ.get(k) for k in ("OMP_NUM_THREADS", "OPENBLAS_NUM_THREADS", "MKL_NUM_THREADS")}
    try:
        for k in keep:
            os.environ[k] = "1"
        with mp.get_context("spawn").Pool(cores) as pool:
            res = pool.map(_cpu_worker, [(config, r, cores, budget_s) for r in range(cores)])
    finally:
        for k, v in keep.items():
            if v is None:
                os.environ.pop(k, None)
            else:
                os.environ[k] = v
    wl_heads = {2: 32, 3: 512, 4: 128}[config]
    rate = sum(d / el for d, el in res)          # heads per second over all workers
    return dict(value=wl_heads / rate * 1e6, unit="us/layer", cores=cores,
                sample="%d (sequence, head) units in %d processes of about %.0f s each" % (sum(d for d, _ in res), cores, budget_s))


def measure_adaptive(args, torch, np, workloads, DecodeSession):
    """Config 2's tensors with a base sample of 32 tokens per head and epsilon = 0.02: the budget rule of
    Algorithm 2, not the lower cap, then sets the size of the final sample on most heads (final samples of a
    few hundred to a few thousand tokens, several batches of draws, more gathered V rows)."""
    wl = workloads.config2()
    pp = plan_params(wl)
    pp.update(base_abs=32, base_frac=0.0, epsilon=0.02)
    sess = DecodeSession(pp)
    sess.upload(wl.q_bits, wl.k_bits, wl.v_bits, wl.seq_lens, wl.seeds)
    nbuf = 16
    ks = [sess.k] + [sess.k.clone() for _ in range(nbuf - 1)]
    vs = [sess.v] + [sess.v.clone() for _ in range(nbuf - 1)]

    def step(i):
        sess.decode(k=ks[i % nbuf], v=vs[i % nbuf])

    for i in range(args.warmup):
        step(i)
    ms = time_calls(step, args.steps, torch)
    res = sess.results_host()
    counts = res["counts"].reshape(-1, 8).astype(np.int64)
    b_star = res["b_star"].reshape(-1)
    b_dyn = counts[:, 4]
    out = {"workload": wl.name + " with base_abs = 32, epsilon = 0.02", "us_per_layer": ms * 1e3,
           "heads_above_base": int((b_dyn > counts[:, 3]).sum()), "heads": int(b_dyn.size),
           "budget_b": {"min": int(b_dyn.min()), "p50": float(np.percentile(b_dyn, 50)),
                        "p90": float(np.percentile(b_dyn, 90)), "max": int(b_dyn.max())},
           "b_star": {"p50": float(np.percentile(b_star, 50)), "p90": float(np.percentile(b_star, 90)),
                      "max": float(b_star.max())}}
    sess.close()
    del ks, vs, sess
    torch.cuda.empty_cache()
    return out


def decode_loop(args, torch, np, workloads, DecodeSession):
    """Config 5: ragged paged decode loop.  A step appends one token per sequence and runs vatt_decode."""
    from paper_2510_05688_amd.session import _bf16_from_bits
    steps, warm = args.steps, args.warmup
    wl = workloads.config5(steps=steps + warm + 1)
    k_pages, v_pages, table = workloads.configs.to_paged(wl, page=16, seed=3)
    pp = plan_params(wl)
    pp.update(kv_layout=1, page_size=16, num_blocks=int(k_pages.shape[0]))
    sess = DecodeSession(pp)
    if args.score_order != "plan":
        from paper_2510_05688_amd import binding as vb_
        vb_.vatt_plan_set_option(sess.plan, vb_.VATT_OPT_SCORE_ORDER,
                                 dict(tile=0, kvhead=1, blocks=2)[args.score_order])
    sess.upload(wl.q_bits, k_pages, v_pages, wl.seq_lens, wl.seeds, block_table=table)
    new_tokens = [workloads.configs.append_tokens(5, s_, wl.batch, wl.n_kv_heads, wl.head_dim) for s_ in range(steps + warm)]
    new_dev = [(_bf16_from_bits(kn, sess.device), _bf16_from_bits(vn, sess.device)) for kn, vn in new_tokens]
    seeds_dev = [torch.from_numpy((wl.seeds + np.uint64(7919 * s_)).view(np.int64)).to(sess.device)
                 for s_ in range(steps + warm)]

    def step(i):
        sess.append_device(*new_dev[i])
        sess.seq_seeds = seeds_dev[i]
        sess.decode()

    for i in range(warm):
        step(i)
    events = [torch.cuda.Event(enable_timing=True) for _ in range(steps + 1)]
    torch.cuda.synchronize()
    events[0].record()
    for i in range(steps):
        step(warm + i)
        events[i + 1].record()
    torch.cuda.synchronize()
    per_step = np.array([events[i].elapsed_time(events[i + 1]) for i in range(steps)]) * 1e3
    ms_step = events[0].elapsed_time(events[steps]) / steps
    res = sess.results_host()
    counts = res["counts"].reshape(-1, 8).astype(np.int64)
    b_star = res["b_star"].reshape(-1)
    seq_n = sess.seq_lens.cpu().numpy().astype(np.int64)
    n_f = counts[:, 0] + counts[:, 1] + counts[:, 2]
    dens = (n_f + counts[:, 4]) / np.repeat(seq_n, wl.n_q_heads)
    pct = lambda a, q: float(np.percentile(a, q))
    # this build's dense attention on the final state of the same paged cache (the cache is 2.2 GB, far beyond the
    # last-level cache, so one copy does), and the sparse step on that state without the append
    for i in range(5):
        sess.dense()
    ms_dense = time_calls(lambda i: sess.dense(), min(steps, 100), torch)
    ms_final = time_calls(lambda i: sess.decode(), min(steps, 100), torch)
    out = {
        "metric": "vattention_decode_us_per_layer", "value": ms_step * 1e3, "unit": "us", "n_gpus": 1,
        "steps": steps, "warmup": warm, "ms_per_step": ms_step, "higher_is_better": False, "scaling": "weak",
        "vs_baseline": None, "dtype": "bf16", "data": "synthetic",
        "config": {"workload": wl.name, "accumulate": "fp32", "batch": wl.batch, "n_q_heads": wl.n_q_heads, "n_kv_heads": wl.n_kv_heads,
                   "head_dim": wl.head_dim, "n_start": "U[1024, 32768] per sequence", "page_size": 16,
                   "epsilon": float(wl.params["epsilon"]), "delta": float(wl.params["delta"]),
                   "step": "vatt_append_kv + vatt_decode"},
        "step_latency_us": {"p10": pct(per_step, 10), "p50": pct(per_step, 50), "p90": pct(per_step, 90),
                            "max": float(per_step.max())},
        "sum_of_lengths_at_end": int(seq_n.sum()),
        "dense_decode_us_per_layer": ms_dense * 1e3, "vatt_decode_us_on_final_state": ms_final * 1e3,
        "speedup_vs_dense": ms_dense / ms_final,
        "budget_last_step": {"b_min": int(counts[:, 4].min()), "b_p50": pct(counts[:, 4], 50),
                             "b_p90": pct(counts[:, 4], 90), "b_max": int(counts[:, 4].max()),
                             "heads_above_base": int((counts[:, 4] > counts[:, 3]).sum()),
                             "b_star_p50": pct(b_star, 50), "b_star_p90": pct(b_star, 90),
                             "b_star_max": float(b_star.max()), "density_mean": float(dens.mean())},
    }
    print(json.dumps(out))


def host_kv_bench(args, torch, np, workloads, DecodeSession):
    """The setting of the paper's efficiency experiment: K and V in pinned host memory, only the random cache of
    base-sample rows (and the caller's top-k sets) on the GPU.  Times vatt_decode_given_topk_cached,
    vatt_decode_given_topk, vatt_decode and vatt_dense_decode with every K / V row read over the host link, and
    reports the bytes each moves over it.  The top-k sets are the exact ones of the workload (they stand in for an
    approximate top-k method's)."""
    from paper_2510_05688_amd import binding as vb
    wl = {2: workloads.config2, 3: workloads.config3, 4: workloads.config4}[args.config]()
    if args.batch > 0 and args.config == 3:
        wl = workloads.config3(batch=args.batch)
    sess = DecodeSession(plan_params(wl))
    sess.upload(wl.q_bits, wl.k_bits, wl.v_bits, wl.seq_lens, wl.seeds)
    B, Hq, Hkv, d, n = wl.batch, wl.n_q_heads, wl.n_kv_heads, wl.head_dim, wl.n_max
    sess.decode()
    seg2, seg3 = vb.vatt_plan_index_segment(sess.plan, 2), vb.vatt_plan_index_segment(sess.plan, 3)
    topk_idx = sess.out_idx[:, :, seg2:seg3].contiguous()
    topk_cnt = sess.out_counts[:, :, 2].contiguous()
    sess.make_random_cache(np.arange(1, B + 1, dtype=np.uint64) * np.uint64(0x9E3779B97F4A7C15))
    legs = {"given_topk_cached": lambda i: sess.decode_given_topk_cached(topk_idx, topk_cnt),
            "given_topk": lambda i: sess.decode_given_topk(topk_idx, topk_cnt),
            "exact_scoring": lambda i: sess.decode(),
            "dense": lambda i: sess.dense()}
    steps = max(5, min(args.steps, 50))
    on_device = {}
    for name, fn in legs.items():
        for i in range(3):
            fn(i)
        on_device[name] = time_calls(fn, steps, torch) * 1e3
    sess.move_kv_to_host()
    out = {"metric": "vattention_decode_us_per_layer_kv_on_host", "unit": "us", "n_gpus": 1, "steps": steps,
           "higher_is_better": False, "dtype": "bf16", "data": "synthetic",
           "config": {"workload": wl.name, "kv_cache": "pinned host memory, read by the kernels over the host link",
                      "on_gpu": "q, top-k lists, random cache of base-sample rows, workspace, outputs"}}
    row = 2 * d
    for name, fn in legs.items():
        for i in range(2):
            fn(i)
        us = time_calls(fn, steps, torch) * 1e3
        counts = sess.results_host()["counts"].reshape(-1, 8).astype(np.int64)
        n_f = int((counts[:, 0] + counts[:, 1] + counts[:, 2]).sum())
        b0, b = int(counts[:, 3].sum()), int(counts[:, 4].sum())
        flags = counts[:, 7]
        cached_heads = int(((flags & 64) != 0).sum())
        if name == "dense":
            link = 2 * int(np.asarray(wl.seq_lens).sum()) * Hkv * row
        elif name == "exact_scoring":
            link = int(np.asarray(wl.seq_lens).sum()) * Hkv * row + (n_f + b) * row
        elif name == "given_topk":
            # K and V rows of I_f and of the final sample; of the base sample its K rows (its scores), and its V
            # rows too when the numerator is verified
            link = (n_f + b) * 2 * row + b0 * row * (2 if int(wl.params.get("target", 0)) != 0 else 1)
        else:
            link = (n_f + b) * 2 * row                # the base sample's rows come from the cache on the GPU
        out[name] = {"us_per_layer": us, "kv_on_device_us_per_layer": on_device[name], "host_link_bytes": link,
                     "host_link_GBps": link / (us * 1e-6) / 1e9}
        if name == "given_topk_cached":
            out[name]["heads_with_base_sample_from_cache"] = cached_heads
            out[name]["heads"] = int(counts.shape[0])
    out["value"] = out["given_topk_cached"]["us_per_layer"]
    out["ms_per_step"] = out["value"] * 1e-3
    out["speedup_vs_dense"] = {k: out["dense"]["us_per_layer"] / out[k]["us_per_layer"]
                               for k in ("given_topk_cached", "given_topk", "exact_scoring")}
    out["bytes_ratio_vs_dense"] = {k: out["dense"]["host_link_bytes"] / out[k]["host_link_bytes"]
                                   for k in ("given_topk_cached", "given_topk", "exact_scoring")}
    print(json.dumps(out))


def chunk_bench(args, torch, np, workloads, DecodeSession):
    """A multi-query step: the q_len newest tokens of every sequence are queries in one vatt_decode call.

    Compared with q_len single-token calls on the same cache (what a caller without the multi-query plan
    would issue for those tokens, K scanned once per token) and with this build's dense attention of the
    same queries.
    """
    Q = args.q_len
    wl = {2: workloads.config2, 3: workloads.config3, 4: workloads.config4}[args.config]()
    q_bits = workloads.chunk_queries(wl, Q, seed=1)
    sess = DecodeSession(plan_params(wl), q_len=Q)
    sess.upload(q_bits, wl.k_bits, wl.v_bits, wl.seq_lens, wl.seeds)
    single = DecodeSession(plan_params(wl))
    single.upload(wl.q_bits, wl.k_bits, wl.v_bits, wl.seq_lens, wl.seeds)
    B, Hq, Hkv, d, n = wl.batch, wl.n_q_heads, wl.n_kv_heads, wl.head_dim, wl.n_max
    kv_bytes = 2 * B * Hkv * n * d * 2
    nbuf = args.buffers if args.buffers > 0 else max(2, min(32, int(60e9 // kv_bytes)))
    ks = [sess.k] + [sess.k.clone() for _ in range(nbuf - 1)]
    vs = [sess.v] + [sess.v.clone() for _ in range(nbuf - 1)]

    def step(i):
        sess.decode(k=ks[i % nbuf], v=vs[i % nbuf])

    def score_only(i):
        sess.score(k=ks[i % nbuf])

    def dense(i):
        sess.dense(k=ks[i % nbuf], v=vs[i % nbuf])

    def singles(i):
        for _ in range(Q):
            single.decode(k=ks[i % nbuf], v=vs[i % nbuf])

    if args.given_topk:
        # the exact top-k sets of the scored path stand in for an approximate top-k method's output
        from paper_2510_05688_amd import binding as vb
        seg2, seg3 = vb.vatt_plan_index_segment(sess.plan, 2), vb.vatt_plan_index_segment(sess.plan, 3)
        sess.decode()
        topk_idx = sess.out_idx[:, :, seg2:seg3].contiguous()
        topk_cnt = sess.out_counts[:, :, 2].contiguous()
        single.decode()
        s_idx = single.out_idx[:, :, seg2:seg3].contiguous()
        s_cnt = single.out_counts[:, :, 2].contiguous()

        def step(i):  # noqa: F811
            sess.decode_given_topk(topk_idx, topk_cnt, k=ks[i % nbuf], v=vs[i % nbuf])

        def singles(i):  # noqa: F811
            for _ in range(Q):
                single.decode_given_topk(s_idx, s_cnt, k=ks[i % nbuf], v=vs[i % nbuf])

    if args.only:
        fn = dict(decode=step, score=score_only, dense=dense)[args.only]
        for i in range(args.warmup):
            fn(i)
        print(json.dumps({"only": args.only, "q_len": Q, "ms_per_call": time_calls(fn, args.steps, torch),
                          "steps": args.steps}))
        return
    timed = {}
    for name, fn in (("step", step), ("score", score_only), ("dense", dense), ("singles", singles)):
        for i in range(args.warmup):
            fn(i)
        timed[name] = time_calls(fn, args.steps, torch)
    res = sess.results_host()
    counts = res["counts"].reshape(-1, 8).astype(np.int64)
    n_f = counts[:, 0] + counts[:, 1] + counts[:, 2]
    b_dyn = counts[:, 4]
    seq_n = np.asarray(wl.seq_lens, dtype=np.int64)
    k_scan = int(Hkv * d * 2 * seq_n.sum())                       # read once for all Q query tokens
    score_w = int(Q * Hq * 4 * seq_n.sum())
    submax_w = int(Q * Hq * 4 * ((seq_n + 63) // 64 * 8).sum())
    v_rows = int(((n_f + b_dyn) * d * 2).sum())
    select_r = 2 * submax_w + int(((counts[:, 2] + 2 * counts[:, 3] + b_dyn) * 32).sum())
    gather_r = int(((n_f + b_dyn) * 8).sum())
    path_bytes = k_scan + score_w + submax_w + select_r + gather_r + v_rows
    if args.given_topk:
        path_bytes = int(((n_f + counts[:, 3] + b_dyn) * d * 2).sum()) + v_rows + int(((n_f + counts[:, 3] + b_dyn) * 12).sum())
    score_kernel_bytes = k_scan + score_w + submax_w + B * Q * Hq * d * 2
    score_flops = 2.0 * Q * Hq * d * float(seq_n.sum())
    us = timed["step"] * 1e3
    out = {
        "metric": "vattention_chunk_us_per_layer" + ("_given_topk" if args.given_topk else ""), "value": us, "unit": "us", "n_gpus": 1, "steps": args.steps,
        "warmup": args.warmup, "ms_per_step": timed["step"], "higher_is_better": False, "scaling": "weak",
        "vs_baseline": None, "dtype": "bf16", "data": "synthetic",
        "config": {"workload": wl.name + "_q%d" % Q, "accumulate": "fp32", "batch": B, "q_len": Q, "n_q_heads": Hq,
                   "n_kv_heads": Hkv, "head_dim": d, "n": n, "sink": int(wl.params["sink"]),
                   "window": int(wl.params["window"]), "topk_frac": float(wl.params["topk_frac"]),
                   "base_frac": float(wl.params["base_frac"]), "epsilon": float(wl.params["epsilon"]),
                   "delta": float(wl.params["delta"]), "target": "denominator", "kv_buffers_cycled": nbuf},
        "us_per_query_token": us / Q,
        "path_hbm_gbps": path_bytes / (timed["step"] * 1e-3) / 1e9,
        "path_bytes": path_bytes,
        "q_len_single_token_calls_us": timed["singles"] * 1e3,
        "speedup_vs_single_token_calls": timed["singles"] / timed["step"],
        "dense_same_queries_us": timed["dense"] * 1e3,
        "speedup_vs_dense": timed["dense"] / timed["step"],
        "token_density": float(((n_f + b_dyn) / np.maximum(counts[:, 6], 1)).mean()),
        "budget_b": {"min": int(b_dyn.min()), "mean": float(b_dyn.mean()), "max": int(b_dyn.max())},
        "roofline": {
            "kernel": "score_chunk_kernel (K scan shared by all query tokens and group heads, MFMA)",
            "bound": "hbm",
            "achieved": score_kernel_bytes / (timed["score"] * 1e-3) / 1e9,
            "peak": HBM_PEAK_GBPS, "unit": "GB/s",
            "frac": score_kernel_bytes / (timed["score"] * 1e-3) / 1e9 / HBM_PEAK_GBPS,
            "traffic": SCORE_CHUNK_TRAFFIC_BYTES.get(("config%d" % args.config, Q)),
            "bytes_per_launch": score_kernel_bytes,
            "us_per_launch": timed["score"] * 1e3,
            "mfma_tflops": score_flops / (timed["score"] * 1e-3) / 1e12,
        },
    }
    print(json.dumps(out))


def measure_config(config, args, torch, np, workloads, DecodeSession, headline):
    """Times vatt_decode, vatt_score, vatt_dense_decode and the read-only kernel on one configuration and
    returns the result object (the headline line for `headline`, else a sub-object with fewer steps)."""
    steps = args.steps if headline else max(20, min(args.steps, 60))
    warmup = args.warmup if headline else max(5, min(args.warmup, 10))
    wl = {2: workloads.config2, 3: workloads.config3, 4: workloads.config4}[config]()
    if args.batch > 0 and config == 3:
        wl = workloads.config3(batch=args.batch)   # tuning aid: config 3's sequences at another batch size
    sess = DecodeSession(plan_params(wl))
    if args.budget_multiple != 1:
        from paper_2510_05688_amd import binding as vb_
        vb_.vatt_plan_set_option(sess.plan, vb_.VATT_OPT_BUDGET_MULTIPLE, args.budget_multiple)
    if args.score_order != "plan":
        from paper_2510_05688_amd import binding as vb_
        vb_.vatt_plan_set_option(sess.plan, vb_.VATT_OPT_SCORE_ORDER,
                                 dict(tile=0, kvhead=1, blocks=2)[args.score_order])
    if args.nested:
        from paper_2510_05688_amd import binding as vb_
        vb_.vatt_plan_set_option(sess.plan, vb_.VATT_OPT_NESTED_SAMPLES, 1)
    if args.ascending:
        from paper_2510_05688_amd import binding as vb_
        vb_.vatt_plan_set_option(sess.plan, vb_.VATT_OPT_ASCENDING_SAMPLES, 1)
    if args.given_fused >= 0:
        from paper_2510_05688_amd import binding as vb_
        vb_.vatt_plan_set_option(sess.plan, vb_.VATT_OPT_GIVEN_FUSED, args.given_fused)
    for opt, val in (("VATT_OPT_GIVEN_SPLITS", args.given_splits), ("VATT_OPT_SPARSE_SPLITS", args.sparse_splits)):
        if val > 0:
            from paper_2510_05688_amd import binding as vb_
            vb_.vatt_plan_set_option(sess.plan, getattr(vb_, opt), val)
    if args.fused_gather >= 0:
        from paper_2510_05688_amd import binding as vb_
        vb_.vatt_plan_set_option(sess.plan, vb_.VATT_OPT_FUSED_GATHER, args.fused_gather)
    sess.upload(wl.q_bits, wl.k_bits, wl.v_bits, wl.seq_lens, wl.seeds)
    B, Hq, Hkv, d, n = wl.batch, wl.n_q_heads, wl.n_kv_heads, wl.head_dim, wl.n_max
    kv_bytes = 2 * B * Hkv * n * d * 2
    nbuf = args.buffers if args.buffers > 0 else max(2, min(32, int(80e9 // kv_bytes)))
    ks = [sess.k] + [sess.k.clone() for _ in range(nbuf - 1)]
    vs = [sess.v] + [sess.v.clone() for _ in range(nbuf - 1)]

    def step(i):
        sess.decode(k=ks[i % nbuf], v=vs[i % nbuf])

    if args.given_topk:
        from paper_2510_05688_amd import binding as vb
        sess.decode()
        seg2, seg3 = vb.vatt_plan_index_segment(sess.plan, 2), vb.vatt_plan_index_segment(sess.plan, 3)
        topk_idx = sess.out_idx[:, :, seg2:seg3].contiguous()
        topk_cnt = sess.out_counts[:, :, 2].contiguous()

        def step(i):  # noqa: F811
            sess.decode_given_topk(topk_idx, topk_cnt, k=ks[i % nbuf], v=vs[i % nbuf])

        if args.cached:
            # base samples from the random cache of base-sample rows (one cache serves every KV copy: the
            # copies are identical)
            sess.make_random_cache(np.arange(1, B + 1, dtype=np.uint64) * np.uint64(0x9E3779B97F4A7C15))

            def step(i):  # noqa: F811
                sess.decode_given_topk_cached(topk_idx, topk_cnt, k=ks[i % nbuf], v=vs[i % nbuf])

    def score_only(i):
        sess.score(k=ks[i % nbuf])

    def dense(i):
        sess.dense(k=ks[i % nbuf], v=vs[i % nbuf])

    if args.graph_steps > 0:
        # the same launches captured in HIP graphs of `graph_steps` consecutive steps each (one graph per group
        # of KV buffers, since a graph fixes its pointers) and replayed
        per = args.graph_steps
        n_graphs = max(1, nbuf // per)
        side = torch.cuda.Stream()
        graphs = []
        for j in range(n_graphs):
            side.wait_stream(torch.cuda.current_stream())
            g = torch.cuda.CUDAGraph()
            with torch.cuda.stream(side):
                with torch.cuda.graph(g, stream=side):
                    for u in range(per):
                        step(j * per + u)
            torch.cuda.current_stream().wait_stream(side)
            graphs.append(g)
        for i in range(warmup):
            step(i)
        ms_plain = time_calls(step, steps, torch)
        for i in range(max(2, warmup // per)):
            graphs[i % n_graphs].replay()
        ms_graph = time_calls(lambda i: graphs[i % n_graphs].replay(), max(4, steps // per), torch) / per
        print(json.dumps({"only": "graph", "steps_per_graph": per, "plain_us_per_step": ms_plain * 1e3,
                          "graph_us_per_step": ms_graph * 1e3, "steps": steps}))
        return None
    if args.only:
        if args.only == "copy":
            # plain device copy of known size: calibrates the HBM byte counters of the profiler
            src = torch.empty(256 << 20, dtype=torch.uint8, device="cuda").random_(0, 255)
            dsts = [torch.empty_like(src) for _ in range(4)]
        from paper_2510_05688_amd import binding as vb3
        sink0 = torch.zeros(4096, dtype=torch.uint8, device="cuda")
        read0 = lambda i: vb3.vatt_stream_read(ks[i % nbuf], int(ks[0].numel() * ks[0].element_size()), sink0,
                                               torch.cuda.current_stream().cuda_stream)
        fn = dict(decode=step, score=score_only, dense=dense, read=read0,
                  copy=lambda i: dsts[i % 4].copy_(src) if args.only == "copy" else None)[args.only]
        for i in range(warmup):
            fn(i)
        ms = time_calls(fn, steps, torch)
        print(json.dumps({"only": args.only, "ms_per_call": ms, "steps": steps}))
        return None

    for i in range(warmup):
        step(i)
    torch.cuda.synchronize()
    t_wall = time.perf_counter()
    ms_step = time_calls(step, steps, torch)
    t_wall = time.perf_counter() - t_wall
    res = sess.results_host()
    counts = res["counts"].reshape(-1, 8).astype(np.int64)
    # spread of single calls: a second pass with an event after every call (the events cost a little, so the
    # headline figure above comes from the undisturbed loop)
    n_spread = min(steps, 200)
    marks = [torch.cuda.Event(enable_timing=True) for _ in range(n_spread + 1)]
    torch.cuda.synchronize()
    marks[0].record()
    for i in range(n_spread):
        step(i)
        marks[i + 1].record()
    torch.cuda.synchronize()
    per_call = np.array([marks[i].elapsed_time(marks[i + 1]) for i in range(n_spread)]) * 1e3

    for i in range(warmup):
        score_only(i)
    ms_score = time_calls(score_only, steps, torch)
    for i in range(warmup):
        dense(i)
    ms_dense = time_calls(dense, steps, torch)
    # what a kernel that only reads takes for the bytes of the K scan, on the same cycled buffers
    from paper_2510_05688_amd import binding as vb2
    sink = torch.zeros(4096, dtype=torch.uint8, device="cuda")
    k_bytes_all = int(ks[0].numel() * ks[0].element_size())

    def read_only(i):
        vb2.vatt_stream_read(ks[i % nbuf], k_bytes_all, sink, torch.cuda.current_stream().cuda_stream)

    for i in range(warmup):
        read_only(i)
    ms_read = time_calls(read_only, steps, torch)

    # what a kernel that only reads rows takes for the V rows this step gathers (the listed tokens of every
    # head, in list order), on the same cycled buffers: the practical floor of the gather
    seg_ = res["seg"]
    row_list = []
    for bh in range(counts.shape[0]):
        b_, h_ = divmod(bh, Hq)
        base_row = (b_ * Hkv + h_ // (Hq // Hkv)) * n
        ix = res["idx"].reshape(-1, res["idx"].shape[-1])[bh]
        toks = np.concatenate([ix[seg_[s_]:seg_[s_] + int(counts[bh, c_])] for s_, c_ in ((0, 0), (1, 1), (2, 2), (4, 4))])
        row_list.append(base_row + toks.astype(np.int64))
    row_list = np.concatenate(row_list)
    rows_dev = torch.from_numpy(row_list.astype(np.int32)).to("cuda")
    n_rows_total = B * Hkv * n

    def rows_only(i):
        vb2.vatt_row_read(vs[i % nbuf], n_rows_total, rows_dev, int(row_list.size), sink,
                          torch.cuda.current_stream().cuda_stream)

    ms_rows = None
    if d == 128 and n_rows_total < 2 ** 31:
        for i in range(warmup):
            rows_only(i)
        ms_rows = time_calls(rows_only, steps, torch)

    # the same step with the top-k set supplied by the caller (here: the exact one found above, standing in for
    # an approximate top-k method): no K scan, only the attended rows are read
    given = None
    if not args.given_topk and not args.ascending and args.q_len == 1 and not args.no_extra:
        from paper_2510_05688_amd import binding as vb3
        seg2, seg3 = vb3.vatt_plan_index_segment(sess.plan, 2), vb3.vatt_plan_index_segment(sess.plan, 3)
        g_idx = sess.out_idx[:, :, seg2:seg3].contiguous()
        g_cnt = sess.out_counts[:, :, 2].contiguous()

        def given_step(i):
            sess.decode_given_topk(g_idx, g_cnt, k=ks[i % nbuf], v=vs[i % nbuf])

        for i in range(warmup):
            given_step(i)
        ms_given = time_calls(given_step, steps, torch)
        gc = sess.out_counts.cpu().numpy().reshape(-1, 8).astype(np.int64)
        g_rows = int((((gc[:, 0] + gc[:, 1] + gc[:, 2]) * 2 + gc[:, 3] + 2 * gc[:, 4]) * d * 2).sum())   # K and V rows read
        given = {"entry_point": "vatt_decode_given_topk (top-k sets supplied by the caller: the exact ones of this workload)",
                 "us_per_layer": ms_given * 1e3, "speedup_vs_dense": ms_dense / ms_given,
                 "kv_row_bytes": g_rows, "achieved_gbps": g_rows / (ms_given * 1e-3) / 1e9,
                 "frac_of_hbm_peak": g_rows / (ms_given * 1e-3) / 1e9 / HBM_PEAK_GBPS}

    # algorithmic bytes of one layer, from the returned counts
    n_f = counts[:, 0] + counts[:, 1] + counts[:, 2]
    b_dyn = counts[:, 4]
    seq_n = np.asarray(wl.seq_lens, dtype=np.int64)
    k_scan = int(Hkv * d * 2 * seq_n.sum())
    score_w = int(Hq * 4 * seq_n.sum())                        # fp32 scores, written once
    submax_w = int(Hq * 4 * ((seq_n + 63) // 64 * 8).sum())     # largest score of every 8 keys
    v_rows = int(((n_f + b_dyn) * d * 2).sum())
    if int(wl.params["target"]) != 0:
        v_rows += int(((n_f + counts[:, 3]) * d * 2).sum())
    # the selection reads the 8-key maxima (twice) and a few thousand scores per head; the gather reads one
    # score and one index per gathered row
    select_r = 2 * submax_w + int(((counts[:, 2] + 2 * counts[:, 3] + b_dyn) * 32).sum())
    gather_r = int(((n_f + b_dyn) * 8).sum())
    path_bytes = k_scan + score_w + submax_w + select_r + gather_r + v_rows
    if args.given_topk:
        # K rows of I_f, I_bs and I_dyn (no scan), V rows of I_f and I_dyn, the sparse scores and index lists
        k_rows = int(((n_f + (0 if args.nested else counts[:, 3]) + b_dyn) * d * 2).sum())
        path_bytes = k_rows + v_rows + int(((n_f + counts[:, 3] + b_dyn) * 12).sum())
    score_kernel_bytes = k_scan + score_w + submax_w + B * Hq * d * 2
    dense_bytes = 2 * k_scan

    us_layer = ms_step * 1e3
    out = {
        "metric": "vattention_decode_us_per_layer" + ("_given_topk" if args.given_topk else "")
                  + ("_cached_base" if args.given_topk and args.cached else "")
                  + ("_nested_samples" if args.nested else "") + ("_ascending_samples" if args.ascending else "")
                  + ("_budget_multiple_%d" % args.budget_multiple if args.budget_multiple != 1 else ""),
        "value": us_layer,
        "unit": "us",
        "n_gpus": 1,
        "steps": steps,
        "warmup": warmup,
        "ms_per_step": ms_step,
        "higher_is_better": False,
        "scaling": "weak",
        "vs_baseline": None,
        "dtype": "bf16",
        "data": "synthetic",
        "config": {"workload": wl.name, "accumulate": "fp32", "batch": B, "n_q_heads": Hq, "n_kv_heads": Hkv, "head_dim": d, "n": n,
                   "sink": int(wl.params["sink"]), "window": int(wl.params["window"]),
                   "topk_frac": float(wl.params["topk_frac"]), "base_frac": float(wl.params["base_frac"]),
                   "epsilon": float(wl.params["epsilon"]), "delta": float(wl.params["delta"]),
                   "target": "denominator", "kv_buffers_cycled": nbuf},
        "tokens_per_s_attention_only": B / (us_layer * 1e-6 * LLAMA8B_LAYERS),
        "path_hbm_gbps": path_bytes / (ms_step * 1e-3) / 1e9,
        "path_bytes": path_bytes,
        "path_frac_of_hbm_peak": path_bytes / (ms_step * 1e-3) / 1e9 / HBM_PEAK_GBPS,
        "dense_decode_us_per_layer": ms_dense * 1e3,
        "dense_hbm_gbps": dense_bytes / (ms_dense * 1e-3) / 1e9,
        "speedup_vs_dense": ms_dense / ms_step,
        "given_topk": given,
        "token_density": float(((n_f + b_dyn) / np.repeat(seq_n, Hq)).mean()),
        "budget_b": {"min": int(b_dyn.min()), "mean": float(b_dyn.mean()), "max": int(b_dyn.max()),
                     "base_b0_mean": float(counts[:, 3].mean())},
        "wall_s_timed_region": t_wall,
        "step_latency_us": {"p10": float(np.percentile(per_call, 10)), "p50": float(np.percentile(per_call, 50)),
                            "p90": float(np.percentile(per_call, 90)), "calls": int(n_spread),
                            "note": "one event per call; the events add two to three microseconds per call"},
        # The roofline of the target's quantity: the whole score-plus-gather path (every kernel of one step),
        # algorithmic bytes from the returned counts over the step time; `kernels` splits it.  The score kernel
        # is timed live (vatt_score launches back to back on the same cycled buffers); the rest of the step is
        # the difference; `profile_us` are the rocprofv3 averages kept under profiles/ for the same command.
        "roofline": {
            "scope": "one vatt_decode step: score kernel, selection (with the gather fused in at small batch), gather, merge",
            "bound": "hbm",
            "achieved": path_bytes / (ms_step * 1e-3) / 1e9,
            "peak": HBM_PEAK_GBPS,
            "unit": "GB/s",
            "frac": path_bytes / (ms_step * 1e-3) / 1e9 / HBM_PEAK_GBPS,
            "traffic": STEP_TRAFFIC_BYTES.get("config%d" % config),
            "bytes_per_step": path_bytes,
            "us_per_step": us_layer,
            "kernels": [
                {"name": "score_kernel (K scan, q.K for the GQA group; the dominant kernel)",
                 "us": ms_score * 1e3, "us_source": "HIP events on the launch stream, vatt_score back to back",
                 "bytes": score_kernel_bytes,
                 "achieved": score_kernel_bytes / (ms_score * 1e-3) / 1e9,
                 "frac": score_kernel_bytes / (ms_score * 1e-3) / 1e9 / HBM_PEAK_GBPS,
                 "traffic": SCORE_KERNEL_TRAFFIC_BYTES.get("config%d" % config),
                 # a kernel that only reads the K cache (vatt_stream_read), same buffers: the practical floor
                 "read_only_same_k_us": ms_read * 1e3,
                 "read_only_gbps": k_bytes_all / (ms_read * 1e-3) / 1e9},
                {"name": "selection, gather and merge kernels (the rest of the step)",
                 "us": (ms_step - ms_score) * 1e3, "us_source": "step time minus the score kernel's",
                 "bytes": path_bytes - score_kernel_bytes,
                 "achieved": (path_bytes - score_kernel_bytes) / max((ms_step - ms_score) * 1e-3, 1e-9) / 1e9,
                 "frac": (path_bytes - score_kernel_bytes) / max((ms_step - ms_score) * 1e-3, 1e-9) / 1e9 / HBM_PEAK_GBPS,
                 # a kernel that only reads the V rows this step gathers (vatt_row_read), same buffers: the floor of
                 # the gather part alone
                 "read_only_gathered_rows_us": None if ms_rows is None else ms_rows * 1e3,
                 "read_only_gathered_rows_gbps": None if ms_rows is None else row_list.size * d * 2 / (ms_rows * 1e-3) / 1e9,
                 "gathered_rows": int(row_list.size)},
            ],
            "profile_us": PROFILE_KERNEL_US.get("config%d" % config),
        },
    }
    # the kernels after the score pass one by one: durations are the rocprofv3 kernel-trace averages recorded under
    # profiles/ (the profiler cannot run inside this timed loop), bytes are each kernel's share of the path's
    # algorithmic bytes
    prof = PROFILE_KERNEL_US.get("config%d" % config)
    if prof and not args.given_topk:
        fused = "gather_kernel" not in prof
        sel_bytes = select_r + (v_rows + gather_r if fused else 0)
        n_heads = int(counts.shape[0])
        # partial sums per head that the merge adds: 8 workgroups of the fused kernel, else the plan's gather splits
        # (enough for 16 workgroups per CU of a 256-CU chip, at most 16)
        n_part = 8 if fused else min(16, max(1, -(-16 * 256 // n_heads)))
        shares = [("head_kernel", sel_bytes)] + ([] if fused else [("gather_kernel", v_rows + gather_r)]) + \
                 [("gather_merge_kernel", n_heads * n_part * (d + 4) * 4 + n_heads * d * 4)]
        for key, nbytes in shares:
            name = next(k for k in prof if k.startswith(key))
            out["roofline"]["kernels"].append(
                {"name": name, "us": prof[name], "us_source": "rocprofv3 --kernel-trace --stats average, profiles/decode_config%d_kernel_stats.md" % config,
                 "bytes": int(nbytes), "achieved": nbytes / (prof[name] * 1e-6) / 1e9,
                 "frac": nbytes / (prof[name] * 1e-6) / 1e9 / HBM_PEAK_GBPS})
    sess.close()
    del ks, vs, sess
    torch.cuda.empty_cache()
    return out




def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=200)
    ap.add_argument("--warmup", type=int, default=20)
    ap.add_argument("--config", type=int, default=2, choices=[2, 3, 4, 5])
    ap.add_argument("--buffers", type=int, default=0, help="distinct KV copies to cycle through (0 = auto)")
    ap.add_argument("--no-cpu", action="store_true", help="skip the cpu_baseline leg")
    ap.add_argument("--no-extra", action="store_true",
                    help="skip the extra legs of the default run: batched (config 3), adaptive budget, caller-supplied top-k")
    ap.add_argument("--given-topk", action="store_true",
                    help="time vatt_decode_given_topk (top-k set supplied by the caller: here the exact top-k that "
                         "vatt_decode found, standing in for an approximate top-k method) instead of vatt_decode")
    ap.add_argument("--cached", action="store_true",
                    help="with --given-topk: base samples come from the random cache of base-sample rows "
                         "(vatt_decode_given_topk_cached)")
    ap.add_argument("--ascending", action="store_true",
                    help="sample lists in ascending token order (VATT_OPT_ASCENDING_SAMPLES)")
    ap.add_argument("--fused-gather", type=int, default=-1,
                    help="workgroups per head of the selection kernel that also gathers (0: separate selection and "
                         "gather kernels; default: the plan's own choice, 8 at config 2 and 0 at the batched configs)")
    ap.add_argument("--batch", type=int, default=0, help="tuning aid: with --config 3, another batch size than 16")
    ap.add_argument("--given-fused", type=int, default=-1, help="tuning aid: VATT_OPT_GIVEN_FUSED (0: separate kernels)")
    ap.add_argument("--given-splits", type=int, default=0, help="tuning aid: workgroups per head of given_gather_kernel")
    ap.add_argument("--sparse-splits", type=int, default=0, help="tuning aid: workgroups per head of sparse_score_kernel")
    ap.add_argument("--nested", action="store_true",
                    help="nested samples (an option beyond the paper): the final sample keeps the base sample")
    ap.add_argument("--budget-multiple", type=int, default=1,
                    help="round every budget up to a multiple of this (an option beyond the paper; 1 = the paper's rule)")
    ap.add_argument("--score-order", default="plan", choices=["plan", "tile", "kvhead", "blocks"],
                    help="launch order of the score pass (VATT_OPT_SCORE_ORDER): the plan's choice, tile-major, "
                         "KV-head-major, or tile-major in blocks of 256 KiB; results are identical")
    ap.add_argument("--q-len", type=int, default=1,
                    help="query tokens per sequence and call (configs 2-4); above 1 times a multi-query step")
    ap.add_argument("--graph-steps", type=int, default=0,
                    help="time plain launches against replays of HIP graphs that hold this many steps each")
    ap.add_argument("--host-kv", action="store_true",
                    help="K and V in pinned host memory (the paper's efficiency experiment): times the caller-supplied-"
                         "top-k step with the base sample from the random cache, the same without it, vatt_decode and "
                         "dense decode, all reading the cache over the host link")
    ap.add_argument("--only", default="", help="profiling aid: run only 'decode', 'score', 'dense', 'read' (a kernel that only reads the K cache) or 'copy' (a 256 MiB device copy) in the timed loop")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py measures one GPU: this build has no multi-GPU path (the step shards by sequence and "
              "KV head without communication). Run with --gpus 1.", file=sys.stderr)
        sys.exit(2)

    import numpy as np
    import torch
    import workloads
    from paper_2510_05688_amd.session import DecodeSession

    if not torch.cuda.is_available():
        print("bench.py needs a GPU (no CPU path exists for the product)", file=sys.stderr)
        sys.exit(2)

    if args.config == 5:
        decode_loop(args, torch, np, workloads, DecodeSession)
        return
    if args.host_kv:
        host_kv_bench(args, torch, np, workloads, DecodeSession)
        return
    if args.q_len > 1:
        chunk_bench(args, torch, np, workloads, DecodeSession)
        return
    out = measure_config(args.config, args, torch, np, workloads, DecodeSession, headline=True)
    if args.only or out is None:
        return
    if (args.config == 2 and not args.given_topk and not args.nested and not args.ascending
            and args.budget_multiple == 1 and not args.no_extra):
        # the same step where the budget rule, not the lower cap, sets the sample size on most heads
        out["adaptive_budget"] = measure_adaptive(args, torch, np, workloads, DecodeSession)
        # the batched configuration (config 3, B = 16), where the path is bound by HBM rather than by latency
        b3 = measure_config(3, args, torch, np, workloads, DecodeSession, headline=False)
        out["batched"] = {k: b3[k] for k in ("config", "value", "unit", "ms_per_step", "steps", "tokens_per_s_attention_only",
                                              "path_bytes", "dense_decode_us_per_layer", "speedup_vs_dense", "given_topk",
                                              "token_density", "budget_b", "roofline")}
    if not args.no_cpu:
        wl = {2: workloads.config2, 3: workloads.config3, 4: workloads.config4}[args.config]()
        out["cpu_baseline"] = cpu_baseline(wl)
        out["cpu_baseline"]["all_cores"] = cpu_baseline_all_cores(args.config)
    print(json.dumps(out))


if __name__ == "__main__":
    main()
