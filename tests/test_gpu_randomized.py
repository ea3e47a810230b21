"""GPU parity on seeded random configurations: shapes, lengths, layouts and every parameter of Algorithm 1
drawn at random, small enough for the oracle to check every head."""
import numpy as np
import pytest
import torch

import workloads
from workloads.configs import default_params
from parity import ChunkView, check_all, say
from util import plan_params

pytestmark = pytest.mark.gpu

# The committed runs use the seeds below; VATT_TEST_SEED=k shifts all of them (a way to try other draws by hand).
import os  # noqa: E402
SEED_SHIFT = int(os.environ.get("VATT_TEST_SEED", "0"))


def _draw_case(rng):
    d = int(rng.choice([64, 128]))
    g = int(rng.choice([1, 2, 4, 8]))
    hkv = int(rng.choice([1, 2]))
    page = int(rng.choice([8, 16, 16, 64, 256]))
    n_max = max(int(rng.choice([48, 130, 517, 1000, 2048, 3100, 4500])) // page * page, page)
    batch = int(rng.integers(1, 4))
    lens = [int(rng.integers(1, n_max + 1)) for _ in range(batch)]
    lens[0] = n_max
    if (n_max // page + batch) % 4 == 0:
        hkv = 8        # (no draw of its own: the other cases stay as they were) 8 KV heads: heads placed by KV head
    over = dict(
        sink=int(rng.choice([0, 1, 4, 16, 100])), window=int(rng.choice([0, 1, 8, 24, 200])),
        epsilon=float(rng.choice([0.3, 0.1, 0.05, 0.02, 0.008])), delta=float(rng.choice([0.3, 0.1, 0.05, 0.01])),
        target=int(rng.choice([0, 0, 0, 1, 2])), budget_cap_frac=float(rng.choice([1.0, 1.0, 0.5, 0.1])),
    )
    if rng.random() < 0.5:
        over.update(topk_abs=int(rng.choice([1, 7, 64, 300])), topk_frac=0.0)
    else:
        over.update(topk_frac=float(rng.choice([0.0, 0.01, 0.025, 0.1, 0.5])))
    if rng.random() < 0.5:
        over.update(base_abs=int(rng.choice([1, 2, 9, 64, 500])), base_frac=0.0)
    else:
        over.update(base_frac=float(rng.choice([0.0, 0.01, 0.025, 0.2, 0.6])))
    # library options (each changes how, not what, except nested samples and the budget bound, which the oracle follows)
    opts = dict(small_batches=bool(rng.random() < 0.2), general_topk=bool(rng.random() < 0.2),
                wide=bool(rng.random() < 0.2), nested=bool(rng.random() < 0.25),
                hoeffding=bool(over["target"] == 0 and rng.random() < 0.25))
    return dict(d=d, g=g, hkv=hkv, n_max=n_max, batch=batch, lens=lens, over=over, opts=opts, page=page,
                paged=bool(rng.random() < 0.4), q_len=int(rng.choice([1, 1, 1, 2, 3])),
                v_mean=float(rng.choice([0.0, 1.0])), flat=bool(rng.random() < 0.5))


def _budget_multiple(c):
    """The budget rounding of a case, derived from what was drawn (so that adding it left the cases as they were)."""
    return (1, 1, 16, 64, 7)[(c["n_max"] + c["batch"]) % 5]


@pytest.mark.timeout(900)
def test_random_configurations_match_the_oracle():
    from paper_2510_05688_amd.session import DecodeSession
    from paper_2510_05688_amd import binding as vb
    rng = np.random.default_rng(20251005 + SEED_SHIFT)
    n_cases, heads_checked = 80, 0
    for case in range(n_cases):
        c = _draw_case(rng)
        p = default_params(c["d"], **c["over"])
        wl = workloads.make_workload("random%d" % case, batch=c["batch"], n_q_heads=c["hkv"] * c["g"],
                                     n_kv_heads=c["hkv"], head_dim=c["d"], n_max=c["n_max"], seq_lens=c["lens"],
                                     seed=1000 + case, params=p, v_mean=c["v_mean"], all_flat=c["flat"],
                                     plant_frac=0.004)
        q_len = c["q_len"]
        if q_len > 1:
            wl.seq_lens = np.maximum(wl.seq_lens, q_len).astype(np.int32)   # a chunk never exceeds its sequence
        say("random case %d: d=%d G=%d Hkv=%d n_max=%d lens=%s paged=%s/%d q_len=%d %s %s" % (
            case, c["d"], c["g"], c["hkv"], c["n_max"], [int(x) for x in wl.seq_lens], c["paged"], c["page"], q_len, c["over"],
            {k: v for k, v in c["opts"].items() if v}))
        q_bits = workloads.chunk_queries(wl, q_len, seed=case) if q_len > 1 else wl.q_bits
        if c["paged"]:
            k_pages, v_pages, table = workloads.to_paged(wl, page=c["page"], seed=case)
            sess = DecodeSession(plan_params(wl, paged=True, page=c["page"], num_blocks=k_pages.shape[0]), q_len=q_len)
            sess.upload(q_bits, k_pages, v_pages, wl.seq_lens, wl.seeds, block_table=table)
        else:
            sess = DecodeSession(plan_params(wl), q_len=q_len)
            sess.upload(q_bits, wl.k_bits, wl.v_bits, wl.seq_lens, wl.seeds)
        o = c["opts"]
        vb.vatt_plan_set_option(sess.plan, vb.VATT_OPT_SAMPLER_SMALL_BATCHES, int(o["small_batches"]))
        vb.vatt_plan_set_option(sess.plan, vb.VATT_OPT_TOPK_GENERAL_PATH, int(o["general_topk"]))
        vb.vatt_plan_set_option(sess.plan, vb.VATT_OPT_HEAD_THREADS, 1024 if o["wide"] else 512)
        vb.vatt_plan_set_option(sess.plan, vb.VATT_OPT_NESTED_SAMPLES, int(o["nested"]))
        # (which of the two Hoeffding forms: derived from what was drawn, so that adding it left the cases as they were)
        range_form = o["hoeffding"] and (c["n_max"] + c["hkv"]) % 2 == 1
        if o["hoeffding"]:
            vb.vatt_plan_set_option(sess.plan, vb.VATT_OPT_BUDGET_BOUND,
                                    vb.VATT_BOUND_HOEFFDING_RANGE if range_form else vb.VATT_BOUND_HOEFFDING)
        multiple = _budget_multiple(c)
        vb.vatt_plan_set_option(sess.plan, vb.VATT_OPT_BUDGET_MULTIPLE, multiple)
        if q_len == 1:
            vb.vatt_plan_set_option(sess.plan, vb.VATT_OPT_SCORE_ORDER, (c["n_max"] // 7 + c["hkv"]) % 3)
        oracle_params = dict(wl.params, nested=o["nested"], budget_multiple=multiple,
                             bound=("hoeffding_range" if range_form else "hoeffding") if o["hoeffding"] else "clt")
        sess.decode()
        res = sess.results_host()
        view = ChunkView(wl, q_bits, q_len) if q_len > 1 else wl
        reps = check_all(view, res, params=oracle_params, gpu_scores=sess.scores_host(), label="random%d" % case)
        heads_checked += len(reps)
        sess.close()
    say("random configurations: %d cases, %d heads checked" % (n_cases, heads_checked))


@pytest.mark.timeout(900)
def test_random_configurations_with_caller_supplied_topk():
    from parity import check_head_given
    from oracle import vatt_oracle as vo
    from paper_2510_05688_amd.session import DecodeSession
    from paper_2510_05688_amd import binding as vb
    rng = np.random.default_rng(7102510 + SEED_SHIFT)
    n_cases, heads_checked = 40, 0
    for case in range(n_cases):
        c = _draw_case(rng)
        p = default_params(c["d"], **c["over"])
        wl = workloads.make_workload("random_given%d" % case, batch=c["batch"], n_q_heads=c["hkv"] * c["g"],
                                     n_kv_heads=c["hkv"], head_dim=c["d"], n_max=c["n_max"], seq_lens=c["lens"],
                                     seed=5000 + case, params=p, v_mean=c["v_mean"], all_flat=c["flat"],
                                     plant_frac=0.004)
        q_len = c["q_len"]
        if q_len > 1:
            wl.seq_lens = np.maximum(wl.seq_lens, q_len).astype(np.int32)
        nested = c["opts"]["nested"]
        say("random given case %d: d=%d G=%d Hkv=%d n_max=%d lens=%s paged=%s q_len=%d nested=%s %s" % (
            case, c["d"], c["g"], c["hkv"], c["n_max"], [int(x) for x in wl.seq_lens], c["paged"], q_len, nested,
            c["over"]))
        q_bits = workloads.chunk_queries(wl, q_len, seed=case) if q_len > 1 else wl.q_bits
        if c["paged"]:
            k_pages, v_pages, table = workloads.to_paged(wl, page=c["page"], seed=case)
            sess = DecodeSession(plan_params(wl, paged=True, page=c["page"], num_blocks=k_pages.shape[0]), q_len=q_len)
            sess.upload(q_bits, k_pages, v_pages, wl.seq_lens, wl.seeds, block_table=table)
        else:
            sess = DecodeSession(plan_params(wl), q_len=q_len)
            sess.upload(q_bits, wl.k_bits, wl.v_bits, wl.seq_lens, wl.seeds)
        vb.vatt_plan_set_option(sess.plan, vb.VATT_OPT_NESTED_SAMPLES, int(nested))
        multiple = _budget_multiple(c)
        vb.vatt_plan_set_option(sess.plan, vb.VATT_OPT_BUDGET_MULTIPLE, multiple)
        view = ChunkView(wl, q_bits, q_len) if q_len > 1 else wl
        k_max = vb.vatt_plan_index_segment(sess.plan, 3) - vb.vatt_plan_index_segment(sess.plan, 2)
        rows, Hq, g = view.batch, wl.n_q_heads, c["g"]
        idx = rng.integers(-5, c["n_max"] + 5, size=(rows, Hq, max(k_max, 1))).astype(np.int32)   # junk beyond cnt
        cnt = np.zeros((rows, Hq), dtype=np.int32)
        supplied = {}
        for v in range(rows):
            n = int(view.seq_lens[v])
            for h in range(Hq):
                s = vo.scores(view.q_f32()[v, h].astype(np.float64), view.k_f32(v, h // g, n).astype(np.float64),
                              p["sm_scale"]) + rng.normal(0.0, 0.5, size=n)
                k = vo.topk_count(n, int(p["sink"]), int(p["window"]), int(p.get("topk_abs", 0)),
                                  float(p.get("topk_frac", 0.0)))
                top = vo.deterministic_set(s, int(p["sink"]), int(p["window"]), k)[2]
                # an approximate method's list: shuffled, with a few repeats and strays, cut to the capacity
                extra = rng.integers(-3, n + 3, size=int(rng.integers(0, 4)))
                lst = rng.permutation(np.concatenate([top, top[:2], extra]))[:k_max].astype(np.int32)
                supplied[(v, h)] = lst
                idx[v, h, :len(lst)] = lst
                cnt[v, h] = len(lst)
        # a third of the single-token cases take their base samples from a random cache of base-sample rows
        # (derived from what was drawn, so that adding it left the cases as they were); its slot count varies
        # from far too few for any head to use it to plenty
        use_cache = q_len == 1 and (c["n_max"] + c["hkv"] + c["batch"]) % 3 == 0
        caches = None
        if use_cache:
            cache_seeds = np.arange(c["batch"], dtype=np.uint64) * np.uint64(0x1F123BB5) + np.uint64(99 + case)
            sess.make_random_cache(cache_seeds, slots=(None, 8, 64, 512)[(c["n_max"] + case) % 4])
            caches = {(b, kvh): vo.random_cache_fill(int(wl.seq_lens[b]), sess.cache_slots, int(cache_seeds[b]), kvh)
                      for b in range(c["batch"]) for kvh in range(c["hkv"])}
            sess.decode_given_topk_cached(torch.from_numpy(idx).to(sess.device), torch.from_numpy(cnt).to(sess.device))
        else:
            sess.decode_given_topk(torch.from_numpy(idx).to(sess.device), torch.from_numpy(cnt).to(sess.device))
        res = sess.results_host()
        params = dict(wl.params, nested=nested, budget_multiple=multiple)
        from_cache = 0
        for v in range(rows):
            for h in range(Hq):
                r = check_head_given(view, res, v, h, supplied[(v, h)], params=params, label="random given %d" % case,
                                     cache_tokens=caches[(v, h // g)] if use_cache else None)
                from_cache += r["from_cache"]
                heads_checked += 1
        if use_cache:
            say("    random cache of %d slots: %d of %d heads took their base sample from it" % (
                sess.cache_slots, from_cache, rows * Hq))
        sess.close()
    say("random configurations with supplied top-k: %d cases, %d heads checked" % (n_cases, heads_checked))


@pytest.mark.timeout(900)
def test_random_medium_configurations_match_the_oracle():
    # rows of 8K to 80K tokens (both workgroup sizes of the selection kernel by the plan's own choice, resident
    # and streamed 8-key maxima, samples of several batches), a few heads each, every head checked
    from paper_2510_05688_amd.session import DecodeSession
    rng = np.random.default_rng(31337 + SEED_SHIFT)
    heads_checked = 0
    for case in range(14):
        n_max = int(rng.choice([8192, 16384, 32768, 40000, 65536, 80000])) // 16 * 16
        d = int(rng.choice([64, 128]))
        g = int(rng.choice([1, 4]))
        batch = int(rng.integers(1, 3))
        lens = [n_max] + [int(rng.integers(n_max // 3, n_max + 1)) for _ in range(batch - 1)]
        over = dict(epsilon=float(rng.choice([0.05, 0.02, 0.01, 0.004])), delta=float(rng.choice([0.2, 0.05])),
                    topk_frac=float(rng.choice([0.005, 0.025, 0.1])), base_frac=float(rng.choice([0.01, 0.025, 0.1])),
                    sink=int(rng.choice([0, 128])), window=int(rng.choice([128, 512])))
        paged = bool(rng.random() < 0.4)
        p = default_params(d, **over)
        wl = workloads.make_workload("medium%d" % case, batch=batch, n_q_heads=g, n_kv_heads=1, head_dim=d,
                                     n_max=n_max, seq_lens=lens, seed=9000 + case, params=p,
                                     all_flat=bool(rng.random() < 0.5), cluster=int(rng.choice([1, 64])))
        say("medium case %d: d=%d G=%d n_max=%d lens=%s paged=%s %s" % (case, d, g, n_max, lens, paged, over))
        if paged:
            k_pages, v_pages, table = workloads.to_paged(wl, page=16, seed=case)
            sess = DecodeSession(plan_params(wl, paged=True, page=16, num_blocks=k_pages.shape[0]))
            sess.upload(wl.q_bits, k_pages, v_pages, wl.seq_lens, wl.seeds, block_table=table)
        else:
            sess = DecodeSession(plan_params(wl))
            sess.upload(wl.q_bits, wl.k_bits, wl.v_bits, wl.seq_lens, wl.seeds)
        sess.decode()
        res = sess.results_host()
        heads_checked += len(check_all(wl, res, gpu_scores=sess.scores_host(), label="medium%d" % case))
        sess.close()
    say("medium random configurations: %d heads checked" % heads_checked)
