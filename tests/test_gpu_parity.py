"""GPU parity: libvatt (through its C ABI) against the CPU oracle on the same seeded inputs."""
import numpy as np
import pytest
import torch

import workloads
from workloads.configs import default_params, append_tokens
from oracle import vatt_oracle as vo
from parity import (alternatives_used, check_all, check_head, check_head_given, gpu_segments, head_inputs, say,
                    score_tolerance)
from util import plan_params

pytestmark = pytest.mark.gpu


def _session(wl, **over):
    from paper_2510_05688_amd.session import DecodeSession
    sess = DecodeSession(plan_params(wl, **over))
    sess.upload(wl.q_bits, wl.k_bits, wl.v_bits, wl.seq_lens, wl.seeds)
    return sess


def _paged_session(wl, page=16, seed=0):
    from paper_2510_05688_amd.session import DecodeSession
    k_pages, v_pages, table = workloads.to_paged(wl, page=page, seed=seed)
    sess = DecodeSession(plan_params(wl, paged=True, page=page, num_blocks=k_pages.shape[0]))
    sess.upload(wl.q_bits, k_pages, v_pages, wl.seq_lens, wl.seeds, block_table=table)
    return sess


def _run(sess):
    sess.decode()
    return sess.results_host()


# ------------------------------------------------------------------ scores ---
@pytest.mark.parametrize("d,hq,hkv,n,lens", [
    (128, 8, 2, 3000, [3000, 2963]),        # G = 4, ragged tail, several tiles
    (128, 4, 4, 777, [777, 1]),             # G = 1, one-token sequence
    (128, 16, 2, 1500, [1500, 1029]),       # G = 8
    (64, 4, 2, 2100, [2100, 517]),          # d = 64, G = 2
    (64, 8, 1, 600, [600, 256]),            # d = 64, G = 8
])
def test_score_pass(d, hq, hkv, n, lens):
    say("score pass d=%d Hq=%d Hkv=%d n=%d" % (d, hq, hkv, n))
    wl = workloads.small_gqa(seed=11, batch=2, n_q_heads=hq, n_kv_heads=hkv, head_dim=d, n=n, seq_lens=lens)
    for paged in (False, True):
        sess = _paged_session(wl, page=16 if n % 16 == 0 else 8) if (paged and n % 8 == 0) else _session(wl)
        sess.score()
        torch.cuda.synchronize()
        gs = sess.scores_host()
        for b in range(2):
            for h in range(hq):
                q, K, V, nn = head_inputs(wl, b, h)
                s = vo.scores(q, K, wl.params["sm_scale"])
                err = np.abs(gs[b, h, :nn] - s)
                assert np.all(err <= score_tolerance(q, K, wl.params["sm_scale"])), (b, h, err.max())
        sess.close()


# ------------------------------------------------------ whole step, small ----
SMALL_CASES = {
    "default": dict(),
    "target_N": dict(target=1, epsilon=0.2),
    "target_SDPA": dict(target=2, epsilon=0.3),
    "no_sink_no_window": dict(sink=0, window=0),
    "no_topk": dict(topk_frac=0.0),
    "no_base_rate": dict(base_frac=0.0),
    "abs_counts": dict(topk_abs=40, base_abs=64),
    "tight_eps": dict(epsilon=0.01, delta=0.01),
    "capped": dict(epsilon=0.005, budget_cap_frac=0.3),
    "window_covers_all": dict(sink=2000, window=2000),
    "topk_covers_all": dict(topk_abs=100000),
}


@pytest.mark.parametrize("name", list(SMALL_CASES))
def test_decode_small(name):
    over = SMALL_CASES[name]
    say("decode small case %s" % name)
    wl = workloads.small_gqa(seed=7, **over)
    sess = _session(wl)
    res = _run(sess)
    check_all(wl, res, gpu_scores=sess.scores_host(), label="small/" + name)
    sess.close()


def test_decode_small_mean_shifted_values_all_targets():
    # V ~ N(1, 1): the numerator has a mean component, so the N and SDPA budgets are not clamped
    for target, eps in ((0, 0.05), (1, 0.1), (2, 0.25)):
        say("decode small mean-shifted target %d" % target)
        p = default_params(128, sink=16, window=24, target=target, epsilon=eps, delta=0.1, base_abs=64, base_frac=0.0)
        wl = workloads.make_workload("shifted", batch=2, n_q_heads=8, n_kv_heads=2, head_dim=128, n_max=4096,
                                     seq_lens=[4096, 3333], seed=13, params=p, v_mean=1.0, all_flat=True)
        sess = _session(wl)
        res = _run(sess)
        reps = check_all(wl, res, label="shifted/target%d" % target)
        assert sum(r["b"] > r["b0"] for r in reps) >= len(reps) // 2, "budgets should come from the formula"
        sess.close()


def test_tiny_sequences():
    say("decode tiny sequences")
    p = default_params(64, sink=4, window=4, topk_abs=3, topk_frac=0.0, base_abs=2, base_frac=0.0)
    wl = workloads.make_workload("tiny", batch=6, n_q_heads=2, n_kv_heads=2, head_dim=64, n_max=64,
                                 seq_lens=[1, 2, 7, 9, 12, 64], seed=3, params=p, all_flat=True)
    sess = _session(wl)
    res = _run(sess)
    check_all(wl, res, label="tiny")
    sess.close()


def test_d64_group8():
    say("decode d=64 G=8")
    wl = workloads.small_gqa(seed=21, batch=1, n_q_heads=8, n_kv_heads=1, head_dim=64, n=5000, seq_lens=[4999])
    sess = _session(wl)
    res = _run(sess)
    check_all(wl, res, gpu_scores=sess.scores_host(), label="d64g8")
    sess.close()


def test_config1_tiny_single_head():
    say("config 1")
    wl = workloads.config1()
    sess = _session(wl)
    res = _run(sess)
    reps = check_all(wl, res, gpu_scores=sess.scores_host(), label="config1")
    assert reps[0]["b"] == 32 and reps[0]["n_s"] == 1024 - 4 - 32 - 32
    assert alternatives_used(reps) == (0, 0)      # sets and budget bit-exact, no tie or boundary alternative
    sess.close()


# ------------------------------------------------------- layout, determinism --
def test_paged_equals_contiguous_bit_for_bit():
    say("paged vs contiguous")
    wl = workloads.small_gqa(seed=5, batch=3, n=4096, seq_lens=[4096, 3001, 130])
    a = _session(wl)
    ra = _run(a)
    b = _paged_session(wl, page=16, seed=9)
    rb = _run(b)
    for key in ("O", "lse", "counts", "b_star", "stats"):
        assert np.array_equal(ra[key], rb[key]), key
    for bb in range(3):
        for h in range(wl.n_q_heads):
            ga, gb = gpu_segments(ra, bb, h), gpu_segments(rb, bb, h)
            for key in ("I_t", "I_bs", "I_dyn"):
                assert np.array_equal(ga[key], gb[key]), (bb, h, key)
    check_all(wl, rb, label="paged")
    a.close()
    b.close()


def test_same_seed_same_bits_and_other_seed_other_sample():
    say("determinism")
    wl = workloads.small_gqa(seed=6, batch=2, n=6000)
    sess = _session(wl)
    r1 = _run(sess)
    r2 = _run(sess)
    for key in ("O", "lse", "idx", "counts", "b_star", "stats"):
        assert np.array_equal(r1[key], r2[key]), key
    sess.set_seeds(wl.seeds + np.uint64(1000))
    r3 = _run(sess)
    g1, g3 = gpu_segments(r1, 0, 0), gpu_segments(r3, 0, 0)
    assert np.array_equal(g1["I_t"], g3["I_t"])
    assert not np.array_equal(g1["I_bs"], g3["I_bs"]) and not np.array_equal(g1["I_dyn"], g3["I_dyn"])
    sess.close()


def _same_results(wl, x, y, output_by_norm=False):
    """Two runs that may sum in a different order: identical integers, floats equal to rounding.
    output_by_norm: the output rows were summed in another order (signed terms): compared per head by norm."""
    assert np.array_equal(x["counts"][..., :7], y["counts"][..., :7])
    for key in ("lse", "b_star", "stats") if output_by_norm else ("O", "lse", "b_star", "stats"):
        assert np.allclose(x[key], y[key], rtol=2e-6, atol=1e-30), key
    if output_by_norm:
        err = np.linalg.norm(x["O"].astype(np.float64) - y["O"], axis=-1)
        assert np.all(err <= 2e-6 * np.linalg.norm(x["O"].astype(np.float64), axis=-1) + 1e-30), err.max()
    for b in range(wl.batch):
        for h in range(wl.n_q_heads):
            gx, gy = gpu_segments(x, b, h), gpu_segments(y, b, h)
            for key in ("I_t", "I_bs", "I_dyn"):
                assert np.array_equal(gx[key], gy[key]), (b, h, key)


def test_sampler_in_small_batches_gives_identical_results():
    say("sampler in batches of 256 draws")
    from paper_2510_05688_amd import binding as vb
    wl = workloads.small_gqa(seed=8, batch=2, n=9000, epsilon=0.02)
    sess = _session(wl)
    fast = _run(sess)
    vb.vatt_plan_set_option(sess.plan, vb.VATT_OPT_SAMPLER_SMALL_BATCHES, 1)
    small = _run(sess)
    # flag bit 3: the final sample needed more than one batch of draws
    assert np.any(small["counts"][..., 7] & 8 == 8)
    _same_results(wl, fast, small)
    check_all(wl, small, label="small-batches")
    sess.close()


def test_topk_general_path_gives_identical_results():
    say("top-k by the general path (histogram over the whole row)")
    from paper_2510_05688_amd import binding as vb
    for wl in (workloads.small_gqa(seed=31, batch=2, n=9000), workloads.small_gqa(seed=32, batch=1, n=20000, topk_frac=0.05)):
        sess = _session(wl)
        fast = _run(sess)
        vb.vatt_plan_set_option(sess.plan, vb.VATT_OPT_TOPK_GENERAL_PATH, 1)
        general = _run(sess)
        assert np.all(general["counts"][..., 7] & 32 == 32) and np.all(fast["counts"][..., 7] & 32 == 0)
        _same_results(wl, fast, general)
        check_all(wl, general, label="topk-general")
        sess.close()


def test_large_topk_sets_leave_the_shortcut():
    say("top-k sets too large for the shortcut: more members than whole sub-tiles, more candidates than the list holds")
    # k = 4000 of 20000: fewer whole 8-key sub-tiles (2495) than members -> general path from the start
    wl = workloads.small_gqa(seed=34, batch=1, n_q_heads=4, n_kv_heads=2, n=20000, topk_frac=0.2)
    sess = _session(wl)
    res = _run(sess)
    assert np.all(res["counts"][..., 7] & 32 == 32)
    check_all(wl, res, label="k > sub-tiles")
    sess.close()
    # k = 3900 of 39000: the bound leaves more than 4096 candidates -> general path after the candidate pass
    wl = workloads.small_gqa(seed=35, batch=1, n_q_heads=4, n_kv_heads=2, n=39000, topk_frac=0.1)
    sess = _session(wl)
    res = _run(sess)
    assert np.all(res["counts"][..., 7] & 32 == 32)
    check_all(wl, res, label="candidates > list")
    sess.close()


def test_topk_with_runs_of_equal_scores():
    say("many equal scores around the top-k threshold")
    # keys repeated in blocks: scores come in runs of equal values, so ties at the threshold go by token order
    wl = workloads.small_gqa(seed=33, batch=1, n_q_heads=4, n_kv_heads=1, n=6000)
    wl.k_bits[:, :, 40:5960] = np.repeat(wl.k_bits[:, :, 40:5960:740], 740, axis=2)
    for general in (0, 1):
        from paper_2510_05688_amd import binding as vb
        sess = _session(wl)
        vb.vatt_plan_set_option(sess.plan, vb.VATT_OPT_TOPK_GENERAL_PATH, general)
        res = _run(sess)
        check_all(wl, res, label="equal-scores general=%d" % general)
        sess.close()


def test_samples_taken_as_complements():
    say("complement regime (c > n_s / 2) for the final sample, then for both samples")
    # a tiny epsilon asks for every residual token; the cap leaves 70 % of them: 30 % are drawn to be left out
    wl = workloads.small_gqa(seed=21, batch=2, n=5000, epsilon=1e-4, budget_cap_frac=0.7)
    sess = _session(wl)
    res = _run(sess)
    capped = res["counts"][..., 7] & 2 == 2          # the flat heads; spiky heads need few samples even so
    assert capped.sum() >= wl.batch * wl.n_q_heads // 2
    assert np.all(res["counts"][..., 4][capped] ==
                  np.ceil(np.float64(np.float32(0.7)) * res["counts"][..., 5][capped].astype(np.float64)))
    check_all(wl, res, label="complement-final")
    sess.close()
    wl = workloads.small_gqa(seed=22, batch=1, n=6000, base_frac=0.8)
    sess = _session(wl)
    res = _run(sess)
    assert np.all(res["counts"][..., 7] & 3 == 3)
    check_all(wl, res, label="complement-both")
    sess.close()


def test_repeated_proposals_inside_a_batch():
    say("short middle region: many repeated tokens inside one batch of draws")
    # 1024 draws over about 4100 tokens propose about 250 tokens more than once, many of them in the same
    # bitmap word: the earliest draw of each must win
    wl = workloads.small_gqa(seed=23, batch=3, n=4200, seq_lens=[4200, 4150, 4137], base_frac=0.2, epsilon=0.01)
    sess = _session(wl)
    res = _run(sess)
    check_all(wl, res, label="repeats")
    sess.close()


def test_draw_cap_completes_samples_in_index_order():
    say("draw cap")
    from paper_2510_05688_amd import binding as vb
    wl = workloads.small_gqa(seed=24, batch=2, n=3000)
    sess = _session(wl)
    vb.vatt_plan_set_option(sess.plan, vb.VATT_OPT_SAMPLER_DRAW_CAP, 40)
    res = _run(sess)
    assert np.all(res["counts"][..., 7] & 16 == 16)
    params = dict(wl.params, draw_cap=40)
    check_all(wl, res, params=params, label="draw-cap")
    # and in the complement regime
    wl2 = workloads.small_gqa(seed=25, batch=1, n=2500, base_frac=0.9)
    sess2 = _session(wl2)
    vb.vatt_plan_set_option(sess2.plan, vb.VATT_OPT_SAMPLER_DRAW_CAP, 100)
    res2 = _run(sess2)
    assert np.all(res2["counts"][..., 7] & 16 == 16)
    check_all(wl2, res2, params=dict(wl2.params, draw_cap=100), label="draw-cap-complement")
    sess.close()
    sess2.close()


def test_append_to_a_contiguous_cache_then_decode():
    say("vatt_append_kv on a contiguous cache")
    from workloads.configs import append_tokens
    wl = workloads.small_gqa(seed=52, batch=3, n=2000, seq_lens=[1990, 1500, 7])
    sess = _session(wl)
    for step in range(3):
        k_new, v_new = append_tokens(52, step, wl.batch, wl.n_kv_heads, wl.head_dim)
        sess.append(k_new, v_new)
        for b in range(wl.batch):          # mirror the append in the host copy the oracle reads
            n = int(wl.seq_lens[b])
            wl.k_bits[b, :, n] = k_new[b]
            wl.v_bits[b, :, n] = v_new[b]
        wl.seq_lens = wl.seq_lens + 1
    assert np.array_equal(sess.seq_lens.cpu().numpy(), wl.seq_lens)
    res = _run(sess)
    check_all(wl, res, label="append-contiguous")
    sess.close()


@pytest.mark.parametrize("path", ["scored", "scored_sdpa_target", "given_topk", "given_topk_cached", "multi_query"])
def test_decode_inside_a_hip_graph(path):
    say("%s step captured in a HIP graph and replayed" % path)
    import torch
    over = dict(target=2, epsilon=0.3) if path == "scored_sdpa_target" else dict()
    wl = workloads.small_gqa(seed=51, batch=2, n=6000, **over)
    if path == "multi_query":
        from paper_2510_05688_amd.session import DecodeSession
        sess = DecodeSession(plan_params(wl), q_len=3)
        sess.upload(workloads.chunk_queries(wl, 3, seed=2), wl.k_bits, wl.v_bits, wl.seq_lens, wl.seeds)
    else:
        sess = _session(wl)
    call = sess.decode
    if path == "given_topk":
        first = _run(sess)
        seg = first["seg"]
        topk_idx = sess.out_idx[:, :, seg[2]:seg[3]].contiguous()
        topk_cnt = sess.out_counts[:, :, 2].contiguous()
        call = lambda: sess.decode_given_topk(topk_idx, topk_cnt)  # noqa: E731
    if path == "given_topk_cached":
        first = _run(sess)
        seg = first["seg"]
        topk_idx = sess.out_idx[:, :, seg[2]:seg[3]].contiguous()
        topk_cnt = sess.out_counts[:, :, 2].contiguous()
        sess.make_random_cache(np.array([11, 12], dtype=np.uint64))
        call = lambda: sess.decode_given_topk_cached(topk_idx, topk_cnt)  # noqa: E731
    call()
    eager = sess.results_host()
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.stream(side):
        with torch.cuda.graph(graph, stream=side):
            call()
    torch.cuda.current_stream().wait_stream(side)
    for _ in range(3):
        sess.out_o.zero_()
        sess.out_idx.zero_()
        sess.dense()                      # other work of the program between the replays
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        again = sess.results_host()
        for key in ("O", "lse", "counts", "b_star", "stats"):
            assert np.array_equal(eager[key], again[key]), key
        for b in range(eager["counts"].shape[0]):
            for h in range(wl.n_q_heads):
                ge, ga = gpu_segments(eager, b, h), gpu_segments(again, b, h)
                for key in ("I_s", "I_l", "I_t", "I_bs", "I_dyn"):
                    assert np.array_equal(ge[key], ga[key]), (b, h, key)
    sess.close()


# ---------------------------------------------------- dense, and check (a) ----
def test_dense_decode_matches_eq1():
    say("dense decode")
    for wl in (workloads.small_gqa(seed=9, batch=2, n=5000, seq_lens=[5000, 1234]),
               workloads.small_gqa(seed=10, batch=1, n_q_heads=8, n_kv_heads=1, head_dim=64, n=900, seq_lens=[900])):
        for paged in (False, True):
            sess = _paged_session(wl, page=8) if paged and wl.n_max % 8 == 0 else _session(wl)
            sess.dense()
            torch.cuda.synchronize()
            O, L = sess.dense_o.cpu().numpy(), sess.dense_lse.cpu().numpy()
            for b in range(wl.batch):
                for h in range(wl.n_q_heads):
                    q, K, V, n = head_inputs(wl, b, h)
                    ro, rl = vo.dense_sdpa(q, K, V, wl.params["sm_scale"])
                    assert np.linalg.norm(O[b, h] - ro) / np.linalg.norm(ro) <= 2e-3, (b, h)
                    assert abs(L[b, h] - rl) <= 2e-3
            sess.close()


def test_budget_covering_the_residual_equals_dense():
    say("check (a) on the GPU")
    wl = workloads.small_gqa(seed=12, batch=2, n=4000, base_abs=10 ** 6)
    sess = _session(wl)
    res = _run(sess)
    sess.dense()
    torch.cuda.synchronize()
    dense_o = sess.dense_o.cpu().numpy()
    for b in range(2):
        for h in range(wl.n_q_heads):
            g = gpu_segments(res, b, h)
            assert g["b"] == g["n_s"] == g["b0"]
            q, K, V, n = head_inputs(wl, b, h)
            ro, rl = vo.dense_sdpa(q, K, V, wl.params["sm_scale"])
            assert np.linalg.norm(res["O"][b, h] - ro) / np.linalg.norm(ro) <= 2e-3
            assert np.linalg.norm(res["O"][b, h] - dense_o[b, h]) / np.linalg.norm(ro) <= 2e-3
    check_all(wl, res, label="full-budget")
    sess.close()


# ----------------------------------------------------------- error handling ---
def test_launch_argument_errors_are_caught_on_the_host():
    say("argument errors")
    from paper_2510_05688_amd import binding as vb
    wl = workloads.small_gqa(seed=2, batch=1, n=512, seq_lens=[512])
    sess = _session(wl)
    small = torch.empty(256, dtype=torch.uint8, device="cuda")
    with pytest.raises(vb.VattError) as e:
        vb.vatt_score(sess.plan, sess.q, sess.k, None, sess.seq_lens, small)
    assert e.value.status == vb.VATT_E_WORKSPACE_TOO_SMALL
    with pytest.raises(vb.VattError) as e:
        vb.vatt_score(sess.plan, sess.q, sess.k, None, sess.seq_lens, sess.workspace[128:])
    assert e.value.status in (vb.VATT_E_INVALID_ARG, vb.VATT_E_WORKSPACE_TOO_SMALL)
    with pytest.raises(vb.VattError) as e:
        vb.vatt_decode(sess.plan, sess.q, sess.k, None, None, sess.seq_lens, sess.seq_seeds, sess.workspace,
                       sess.out_o, None, sess.out_idx, sess.out_counts, None, None)
    assert e.value.status == vb.VATT_E_INVALID_ARG
    # optional outputs may be NULL
    vb.vatt_decode(sess.plan, sess.q, sess.k, sess.v, None, sess.seq_lens, sess.seq_seeds, sess.workspace,
                   sess.out_o, None, sess.out_idx, sess.out_counts, None, None)
    torch.cuda.synchronize()
    sess.close()


def test_hoeffding_type_budget():
    say("conservative (Hoeffding-type) denominator budget")
    from paper_2510_05688_amd import binding as vb
    # epsilon small enough that budgets rise above the base sample on most heads
    wl = workloads.small_gqa(seed=41, batch=2, n=9000, epsilon=0.03, delta=0.2)
    sess = _session(wl)
    clt = _run(sess)
    vb.vatt_plan_set_option(sess.plan, vb.VATT_OPT_BUDGET_BOUND, vb.VATT_BOUND_HOEFFDING)
    hoe = _run(sess)
    params = dict(wl.params, bound="hoeffding")
    reps = check_all(wl, hoe, params=params, label="hoeffding")
    assert any(r["b"] > r["b0"] for r in reps)
    # same base sample, same statistics: b* grows by the constant 2 ln(2/delta) / z^2 (2.80 at delta = 0.2)
    ratio = hoe["b_star"] / clt["b_star"]
    assert np.all(np.abs(ratio - 2.8037) < 2e-3), (ratio.min(), ratio.max())
    assert np.all(hoe["counts"][..., 4] >= clt["counts"][..., 4])
    vb.vatt_plan_set_option(sess.plan, vb.VATT_OPT_BUDGET_BOUND, vb.VATT_BOUND_CLT)
    back = _run(sess)
    assert np.array_equal(back["counts"], clt["counts"]) and np.array_equal(back["b_star"], clt["b_star"])
    sess.close()


@pytest.mark.parametrize("fused", [0, 8])
def test_range_based_hoeffding_budget(fused):
    say("range-based Hoeffding budget (fused gather: %d)" % fused)
    from paper_2510_05688_amd import binding as vb
    # flat heads get budgets of several hundred (between the base sample and the residual size); spiky heads,
    # whose weight sits in the top-k set, have a tiny range and stay at the base sample
    wl = workloads.small_gqa(seed=42, batch=2, n=6000, epsilon=0.1, delta=0.1)
    sess = _session(wl)
    vb.vatt_plan_set_option(sess.plan, vb.VATT_OPT_FUSED_GATHER, fused)
    clt = _run(sess)
    vb.vatt_plan_set_option(sess.plan, vb.VATT_OPT_BUDGET_BOUND, vb.VATT_BOUND_HOEFFDING_RANGE)
    rng_ = _run(sess)
    reps = check_all(wl, rng_, params=dict(wl.params, bound="hoeffding_range"), label="hoeffding range")
    assert any(r["b0"] < r["b"] < r["oracle"]["n_s"] for r in reps)
    assert np.all(rng_["b_star"] >= clt["b_star"])
    assert np.array_equal(rng_["stats"], clt["stats"])      # same base sample, same statistics
    # the general top-k path finds the same range
    vb.vatt_plan_set_option(sess.plan, vb.VATT_OPT_TOPK_GENERAL_PATH, 1)
    gen = _run(sess)
    # (D_f is summed in another order there: b* agrees to rounding, the budgets exactly)
    assert np.allclose(gen["b_star"], rng_["b_star"], rtol=1e-6, atol=0) and np.array_equal(gen["counts"][..., :7], rng_["counts"][..., :7])
    vb.vatt_plan_set_option(sess.plan, vb.VATT_OPT_TOPK_GENERAL_PATH, 0)
    # a supplied top-k set bounds nothing: refused
    seg = rng_["seg"]
    with pytest.raises(vb.VattError) as e:
        sess.decode_given_topk(sess.out_idx[:, :, seg[2]:seg[3]].contiguous(), sess.out_counts[:, :, 2].contiguous())
    assert e.value.status == vb.VATT_E_UNSUPPORTED_SHAPE
    vb.vatt_plan_set_option(sess.plan, vb.VATT_OPT_BUDGET_BOUND, vb.VATT_BOUND_CLT)
    back = _run(sess)
    assert np.array_equal(back["counts"], clt["counts"]) and np.array_equal(back["b_star"], clt["b_star"])
    sess.close()


@pytest.mark.parametrize("name,over", [
    ("default", dict()),                                       # budgets at the base sample: nothing more is drawn
    ("tight_eps", dict(epsilon=0.01, delta=0.01)),             # budgets well above the base sample
    ("complement", dict(base_frac=0.2, epsilon=0.004)),        # the added tokens are taken as a complement
    ("target_sdpa", dict(target=2, epsilon=0.3)),
])
def test_nested_samples(name, over):
    say("nested samples: %s" % name)
    from paper_2510_05688_amd import binding as vb
    wl = workloads.small_gqa(seed=43, batch=2, n=6000, **over)
    sess = _session(wl)
    vb.vatt_plan_set_option(sess.plan, vb.VATT_OPT_NESTED_SAMPLES, 1)
    res = _run(sess)
    reps = check_all(wl, res, params=dict(wl.params, nested=True), label="nested " + name)
    seg = res["seg"]
    for b in range(wl.batch):
        for h in range(wl.n_q_heads):
            b0, bb = int(res["counts"][b, h, 3]), int(res["counts"][b, h, 4])
            # the final sample's list starts with the base sample, in the base sample's own order
            assert np.array_equal(res["idx"][b, h, seg[4]:seg[4] + b0], res["idx"][b, h, seg[3]:seg[3] + b0])
            assert bb >= b0
    if name != "default":
        assert any(r["b"] > r["b0"] for r in reps)
    if name == "complement":
        assert any(r["flags"] & 2 for r in reps)
    sess.close()


@pytest.mark.parametrize("name,over,q", [
    ("d_target_64", dict(epsilon=0.02, delta=0.1), 64),          # budgets above the base sample, rounded to 64
    ("d_target_16", dict(epsilon=0.02, delta=0.1), 16),
    ("at_base_7", dict(), 7),                                    # budgets at the base sample: b0 rounded up
    ("capped_64", dict(epsilon=0.004, budget_cap_frac=0.3), 64), # the rounding stops at the explicit cap
    ("near_all_64", dict(base_frac=0.2, epsilon=0.002), 64),     # ... and at the residual count
    ("target_sdpa_16", dict(target=2, epsilon=0.3), 16),
])
def test_budget_rounded_up_to_a_multiple(name, over, q):
    say("budget rounded up to a multiple of %d: %s" % (q, name))
    from paper_2510_05688_amd import binding as vb
    wl = workloads.small_gqa(seed=47, batch=2, n=6000, seq_lens=[6000, 3301], **over)
    sess = _session(wl)
    plain = _run(sess)
    vb.vatt_plan_set_option(sess.plan, vb.VATT_OPT_BUDGET_MULTIPLE, q)
    res = _run(sess)
    params = dict(wl.params, budget_multiple=q)
    reps = check_all(wl, res, params=params, label="multiple " + name)
    b_plain, b_round = plain["counts"][..., 4].astype(np.int64), res["counts"][..., 4].astype(np.int64)
    n_s, b0 = res["counts"][..., 5].astype(np.int64), res["counts"][..., 3].astype(np.int64)
    cap = np.ceil(np.float64(np.float32(wl.params["budget_cap_frac"])) * n_s).astype(np.int64)
    top = np.minimum(n_s, np.maximum(b0, cap))
    assert np.array_equal(b_round, np.minimum(top, (b_plain + q - 1) // q * q))
    assert np.array_equal(res["b_star"], plain["b_star"])           # b* itself is not touched
    assert np.any(b_round > b_plain)
    if name == "capped_64":
        assert np.any((b_round == top) & (b_round % q != 0))
    # the same option on the path with a caller-supplied top-k set
    if name == "d_target_64":
        seg = res["seg"]
        topk_idx = sess.out_idx[:, :, seg[2]:seg[3]].contiguous()
        topk_cnt = sess.out_counts[:, :, 2].contiguous()
        sess.decode_given_topk(topk_idx, topk_cnt)
        given = sess.results_host()
        bg = given["counts"][..., 4].astype(np.int64)
        assert np.all((bg % q == 0) | (bg == top)) and np.array_equal(given["counts"][..., 2], res["counts"][..., 2])
    vb.vatt_plan_set_option(sess.plan, vb.VATT_OPT_BUDGET_MULTIPLE, 1)
    back = _run(sess)
    assert np.array_equal(back["counts"], plain["counts"])
    sess.close()


@pytest.mark.parametrize("hq,hkv,paged", [(16, 8, False), (8, 8, True), (8, 2, False), (4, 1, True)])
def test_score_launch_orders_give_identical_results(hq, hkv, paged):
    say("score pass launched in each of its three orders: Hq=%d Hkv=%d paged=%s" % (hq, hkv, paged))
    from paper_2510_05688_amd import binding as vb
    wl = workloads.small_gqa(seed=71, batch=3, n_q_heads=hq, n_kv_heads=hkv, n=4096, seq_lens=[4096, 1500, 33],
                             epsilon=0.03)
    sess = _paged_session(wl) if paged else _session(wl)
    runs = []
    for order in (0, 1, 2):
        vb.vatt_plan_set_option(sess.plan, vb.VATT_OPT_SCORE_ORDER, order)
        sess.out_o.zero_()
        sess.out_idx.zero_()
        sess.workspace.zero_()
        runs.append(_run(sess))
        check_all(wl, runs[-1], gpu_scores=sess.scores_host(), label="order %d" % order)
    for other in runs[1:]:
        for key in ("O", "lse", "counts", "b_star", "stats"):
            assert np.array_equal(runs[0][key], other[key]), key
        for b in range(wl.batch):
            for h in range(hq):
                g0, g1 = gpu_segments(runs[0], b, h), gpu_segments(other, b, h)
                for key in ("I_s", "I_l", "I_t", "I_bs", "I_dyn"):
                    assert np.array_equal(g0[key], g1[key]), (b, h, key)
    sess.close()


def test_selection_kernel_with_1024_threads_gives_identical_results():
    say("selection kernel with 1024 threads (the variant for rows longer than 32768 tokens)")
    from paper_2510_05688_amd import binding as vb
    cases = (workloads.small_gqa(seed=71, batch=2, n=9000, epsilon=0.02),
             workloads.small_gqa(seed=72, batch=2, n=700, seq_lens=[700, 33], base_frac=0.3),
             workloads.small_gqa(seed=73, batch=1, n=20000, base_frac=0.3, epsilon=0.004),     # several big batches
             workloads.small_gqa(seed=74, batch=1, n=6000, target=2, epsilon=0.3))
    for wl in cases:
        sess = _session(wl)
        narrow = _run(sess)
        vb.vatt_plan_set_option(sess.plan, vb.VATT_OPT_HEAD_THREADS, 1024)
        wide = _run(sess)
        _same_results(wl, narrow, wide, output_by_norm=True)   # (narrow may run with the gather fused in)
        check_all(wl, wide, label="1024-threads")
        vb.vatt_plan_set_option(sess.plan, vb.VATT_OPT_TOPK_GENERAL_PATH, 1)
        _same_results(wl, narrow, _run(sess), output_by_norm=True)
        with pytest.raises(vb.VattError):
            vb.vatt_plan_set_option(sess.plan, vb.VATT_OPT_HEAD_THREADS, 768)
        sess.close()


@pytest.mark.parametrize("case", ["d128", "d64_paged", "long_lists", "tiny", "complement"])
def test_fused_gather_matches_the_separate_kernels(case):
    # Small batches run selection and gather as one kernel with several workgroups per head; the same step with
    # the kernels apart (option 0) and with every legal number of workgroups per head must give identical index
    # sets, budgets and statistics, outputs equal to rounding, and match the oracle.
    say("fused gather: " + case)
    from paper_2510_05688_amd import binding as vb
    wl = {
        "d128": lambda: workloads.small_gqa(seed=81, batch=2, n=5000, seq_lens=[5000, 1333], epsilon=0.03),
        "d64_paged": lambda: workloads.small_gqa(seed=82, batch=3, n_q_heads=8, n_kv_heads=1, head_dim=64, n=4096,
                                                 seq_lens=[4096, 700, 31]),
        # top-k and final sample longer than one round of rows per workgroup
        "long_lists": lambda: workloads.small_gqa(seed=83, batch=1, n=20000, topk_frac=0.2, base_frac=0.05,
                                                  epsilon=0.01),
        "tiny": lambda: workloads.small_gqa(seed=84, batch=4, n=64, seq_lens=[64, 41, 3, 1], sink=2, window=3),
        "complement": lambda: workloads.small_gqa(seed=85, batch=1, n=3000, base_frac=0.7, epsilon=0.002),
    }[case]()
    sess = _paged_session(wl) if case == "d64_paged" else _session(wl)
    vb.vatt_plan_set_option(sess.plan, vb.VATT_OPT_FUSED_GATHER, 0)
    apart = _run(sess)
    check_all(wl, apart, label="kernels apart / " + case)
    tried = 0
    for splits in (1, 2, 4, 8, 16):
        try:
            vb.vatt_plan_set_option(sess.plan, vb.VATT_OPT_FUSED_GATHER, splits)
        except vb.VattError as e:       # the kernel's LDS does not hold a workgroup's share of the lists
            assert e.status == vb.VATT_E_UNSUPPORTED_SHAPE and splits < 4
            continue
        tried += 1
        sess.out_o.fill_(float("nan"))
        sess.out_idx.fill_(-3)
        sess.out_counts.fill_(-3)
        fused = _run(sess)
        _same_results(wl, apart, fused, output_by_norm=True)
        check_all(wl, fused, label="fused, %d workgroups per head / %s" % (splits, case))
    assert tried >= 3
    # the sampler's first batches made by the selection kernel itself instead of workgroups of the score launch
    vb.vatt_plan_set_option(sess.plan, vb.VATT_OPT_SCORE_PREWORK, 0)
    own = _run(sess)
    for key in ("O", "lse", "b_star", "stats", "idx", "counts"):
        assert np.array_equal(own[key], fused[key]), key
    with pytest.raises(vb.VattError):
        vb.vatt_plan_set_option(sess.plan, vb.VATT_OPT_FUSED_GATHER, 3)
    sess.close()


@pytest.mark.parametrize("target", [0, 2])
def test_sample_lists_in_ascending_order(target):
    say("samples written in ascending token order, target %d" % target)
    from paper_2510_05688_amd import binding as vb
    wl = workloads.small_gqa(seed=91, batch=2, n=6000, seq_lens=[6000, 911], epsilon=0.02 if target == 0 else 0.3,
                             target=target)
    sess = _session(wl)
    vb.vatt_plan_set_option(sess.plan, vb.VATT_OPT_FUSED_GATHER, 0)
    plain = _run(sess)
    vb.vatt_plan_set_option(sess.plan, vb.VATT_OPT_ASCENDING_SAMPLES, 1)
    asc = _run(sess)
    seg = asc["seg"]
    assert np.array_equal(plain["counts"][..., :7], asc["counts"][..., :7])
    some_unsorted = False
    for b in range(wl.batch):
        for h in range(wl.n_q_heads):
            c = asc["counts"][b, h]
            for s_, cnt in ((3, c[3]), (4, c[4])):
                a, p_ = asc["idx"][b, h, seg[s_]:seg[s_] + cnt], plain["idx"][b, h, seg[s_]:seg[s_] + cnt]
                assert np.all(np.diff(a) > 0) and np.array_equal(a, np.sort(p_))
                some_unsorted |= bool(np.any(np.diff(p_) < 0))
    assert some_unsorted      # (the default order is the sampler's acceptance order)
    _same_results(wl, plain, asc, output_by_norm=True)
    check_all(wl, asc, label="ascending samples, target %d" % target)
    sess.close()


def test_lengths_outside_the_cache_are_clamped():
    # seq_lens outside [1, n_max] are clamped by every kernel alike: 0 becomes one token, too large becomes n_max
    wl = workloads.small_gqa(seed=81, batch=3, n=2048, seq_lens=[2048, 1, 2048])
    sess = _session(wl)
    sess.seq_lens = torch.tensor([0, -7, 5000], dtype=torch.int32, device=sess.device)
    res = _run(sess)
    assert [int(res["counts"][b, 0, 6]) for b in range(3)] == [1, 1, 2048]
    assert np.all(np.isfinite(res["O"])) and np.all(np.isfinite(res["lse"]))
    wl.seq_lens = np.array([1, 1, 2048], dtype=np.int32)   # what the kernels made of them
    check_all(wl, res, label="clamped lengths")
    sess.dense()
    torch.cuda.synchronize()
    assert np.all(np.isfinite(sess.dense_o.cpu().numpy()))
    sess.close()


def test_block_table_entries_out_of_range_are_clamped():
    # a corrupted block table must not make any kernel leave the cache: entries are clamped into [0, num_blocks),
    # the sequence they belong to gets a meaningless result, the other sequences are untouched
    wl = workloads.small_gqa(seed=83, batch=2, n=2048, seq_lens=[2048, 1777])
    good = _paged_session(wl)
    ref = _run(good)
    bad = _paged_session(wl)
    table = bad.block_table.clone()
    table[0, 3] = -12345
    table[0, 40] = 2 ** 30
    bad.block_table = table
    res = _run(bad)
    bad.dense()
    torch.cuda.synchronize()
    assert np.array_equal(res["counts"][1], ref["counts"][1])
    assert np.array_equal(res["O"][1], ref["O"][1])
    for h in range(wl.n_q_heads):   # (the used parts of the index lists: the rest of the buffer is not written)
        gx, gy = gpu_segments(res, 1, h), gpu_segments(ref, 1, h)
        for key in ("I_s", "I_l", "I_t", "I_bs", "I_dyn"):
            assert np.array_equal(gx[key], gy[key]), (h, key)
    assert np.all(np.isfinite(res["O"][0]))
    good.close()
    bad.close()


@pytest.mark.parametrize("n_max", [1, 2, 7, 33])
def test_tiny_caches(n_max):
    # capacities far below one tile, one bitmap word, one batch of draws
    say("tiny cache n_max=%d" % n_max)
    p = default_params(128, sink=1, window=2, topk_abs=2, topk_frac=0.0, base_abs=2, base_frac=0.0, epsilon=0.02)
    wl = workloads.make_workload("tiny_cache", batch=2, n_q_heads=4, n_kv_heads=1, head_dim=128, n_max=n_max,
                                 seq_lens=[n_max, max(1, n_max // 2)], seed=4, params=p, all_flat=True)
    sess = _session(wl)
    res = _run(sess)
    check_all(wl, res, gpu_scores=sess.scores_host(), label="tiny cache %d" % n_max)
    sess.dense()
    torch.cuda.synchronize()
    assert np.all(np.isfinite(sess.dense_o.cpu().numpy()))
    sess.close()


@pytest.mark.timeout(300)
def test_largest_supported_capacity():
    # the selection kernel's LDS bitmaps bound the capacity: 170752 tokens is the last one a plan accepts, one
    # more is refused on the host; a full row and a ragged one at that capacity against the oracle, every head,
    # on a contiguous and on a paged cache, and with the top-k sets handed back in
    from paper_2510_05688_amd import binding as vb
    from paper_2510_05688_amd.session import DecodeSession
    n_max = 170752
    say("largest capacity n_max=%d" % n_max)
    p = default_params(128, sink=128, window=512, topk_frac=0.01)
    wl = workloads.make_workload("cap_max", batch=2, n_q_heads=4, n_kv_heads=1, head_dim=128, n_max=n_max,
                                 seq_lens=[n_max, n_max - 4097], seed=170, params=p)
    with pytest.raises(vb.VattError) as e:
        DecodeSession(plan_params(wl, n_max=n_max + 1))
    assert e.value.status == vb.VATT_E_UNSUPPORTED_SHAPE
    sess = _session(wl)
    res = _run(sess)
    reps = check_all(wl, res, gpu_scores=sess.scores_host(), label="cap_max")
    assert len(reps) == 8 and alternatives_used(reps) == (0, 0)
    seg2, seg3 = vb.vatt_plan_index_segment(sess.plan, 2), vb.vatt_plan_index_segment(sess.plan, 3)
    topk_idx = sess.out_idx[:, :, seg2:seg3].contiguous()
    topk_cnt = sess.out_counts[:, :, 2].contiguous()
    sess.decode_given_topk(topk_idx, topk_cnt)
    res_g = sess.results_host()
    for b in range(2):
        for h in range(4):
            supplied = res["idx"][b, h][res["seg"][2]:res["seg"][2] + int(res["counts"][b, h, 2])]
            check_head_given(wl, res_g, b, h, supplied, label="cap_max")
    sess.close()
    sess = _paged_session(wl, page=16, seed=5)
    res_p = _run(sess)
    _same_results(wl, res, res_p)
    sess.close()


@pytest.mark.timeout(300)
def test_plans_of_different_capacities_in_any_order():
    # the dynamic-LDS limit is a property of a kernel, not of a plan: a long-context plan must keep working
    # after a plan with a smaller capacity has been made (both use the 1024-thread selection kernel here)
    say("plans of different capacities used in any order")
    from paper_2510_05688_amd.session import DecodeSession
    p = default_params(128, sink=128, window=128)
    big = workloads.make_workload("cap_big", batch=1, n_q_heads=2, n_kv_heads=1, head_dim=128, n_max=120000,
                                  seq_lens=[120000], seed=91, params=p)
    small = workloads.make_workload("cap_small", batch=1, n_q_heads=2, n_kv_heads=1, head_dim=128, n_max=70000,
                                    seq_lens=[70000], seed=92, params=p)
    s_big = DecodeSession(plan_params(big))
    s_big.upload(big.q_bits, big.k_bits, big.v_bits, big.seq_lens, big.seeds)
    s_small = DecodeSession(plan_params(small))          # made after the big one
    s_small.upload(small.q_bits, small.k_bits, small.v_bits, small.seq_lens, small.seeds)
    check_all(big, _run(s_big), label="big plan after a smaller one was made")
    check_all(small, _run(s_small), label="small plan")
    seg = s_big.seg
    s_big.decode_given_topk(s_big.out_idx[:, :, seg[2]:seg[3]].contiguous(), s_big.out_counts[:, :, 2].contiguous())
    torch.cuda.synchronize()
    assert np.all(np.isfinite(s_big.out_o.cpu().numpy()))
    s_big.close()
    s_small.close()


@pytest.mark.timeout(300)
def test_many_short_sequences():
    # a large batch of short sequences: grid dimensions grow with the batch, every head is still checked
    say("1200 short sequences")
    p = default_params(64, sink=4, window=8, topk_abs=6, topk_frac=0.0, base_abs=8, base_frac=0.0, epsilon=0.1)
    rng = np.random.default_rng(5)
    lens = [int(x) for x in rng.integers(1, 257, size=1200)]
    wl = workloads.make_workload("many_short", batch=1200, n_q_heads=2, n_kv_heads=1, head_dim=64, n_max=256,
                                 seq_lens=lens, seed=6, params=p, all_flat=True)
    for paged in (False, True):
        sess = _paged_session(wl) if paged else _session(wl)
        res = _run(sess)
        check_all(wl, res, label="many short sequences, paged=%s" % paged)
        sess.close()


def test_seeds_use_all_64_bits():
    # the sampler's Philox key is (low word, high word) of the 64-bit seed: seeds that differ only in the high word,
    # or have the top bit set, must reach the kernels intact
    say("64-bit seeds")
    wl = workloads.small_gqa(seed=85, batch=4, n=3000, seq_lens=[3000, 3000, 2500, 2500])
    wl.seeds = np.array([0xFFFFFFFFFFFFFFFF, 1 << 63, (7 << 32) | 5, 5], dtype=np.uint64)
    sess = _session(wl)
    res = _run(sess)
    check_all(wl, res, label="64-bit seeds")
    a, b = gpu_segments(res, 2, 0), gpu_segments(res, 3, 0)   # same low word, different high word
    assert not np.array_equal(a["I_bs"], b["I_bs"])
    sess.close()
