"""GPU parity of vatt_decode_given_topk (top-k set supplied by the caller) against the oracle."""
import numpy as np
import pytest
import torch

import workloads
from oracle import vatt_oracle as vo
from parity import check_head_given, gpu_segments, head_inputs, say
from util import plan_params

pytestmark = pytest.mark.gpu


def _session(wl, paged=False):
    from paper_2510_05688_amd.session import DecodeSession
    if paged:
        k_pages, v_pages, table = workloads.to_paged(wl, page=16, seed=11)
        sess = DecodeSession(plan_params(wl, paged=True, page=16, num_blocks=k_pages.shape[0]))
        sess.upload(wl.q_bits, k_pages, v_pages, wl.seq_lens, wl.seeds, block_table=table)
    else:
        sess = DecodeSession(plan_params(wl))
        sess.upload(wl.q_bits, wl.k_bits, wl.v_bits, wl.seq_lens, wl.seeds)
    return sess


def _k_max(sess):
    from paper_2510_05688_amd import binding as vb
    return vb.vatt_plan_index_segment(sess.plan, 3) - vb.vatt_plan_index_segment(sess.plan, 2)


def _oracle_topk(wl, b, h, noise=0.0, rng=None):
    """Top-k of the oracle's scores (optionally of a noisy copy, as an approximate top-k method would give)."""
    q, K, V, n = head_inputs(wl, b, h)
    p = wl.params
    s = vo.scores(q, K, p["sm_scale"])
    if noise > 0.0:
        s = s + rng.normal(0.0, noise, size=s.shape)
    k = vo.topk_count(n, int(p["sink"]), int(p["window"]), int(p.get("topk_abs", 0)), float(p.get("topk_frac", 0.0)))
    return vo.deterministic_set(s, int(p["sink"]), int(p["window"]), k)[2]


def _run_given(sess, wl, supplied):
    """supplied: dict (b, h) -> int array.  Returns results_host()."""
    k_max = _k_max(sess)
    idx = np.full((wl.batch, wl.n_q_heads, max(k_max, 1)), -7, dtype=np.int32)
    cnt = np.zeros((wl.batch, wl.n_q_heads), dtype=np.int32)
    for (b, h), arr in supplied.items():
        arr = np.asarray(arr, dtype=np.int32)[:k_max]
        idx[b, h, :len(arr)] = arr
        cnt[b, h] = len(arr)
    d_idx = torch.from_numpy(idx).to(sess.device)
    d_cnt = torch.from_numpy(cnt).to(sess.device)
    from paper_2510_05688_amd import binding as vb
    # both forms of the second half of the step: the second selection phase with the gather fused in (the plan's
    # choice for few heads) and the two as kernels of their own: same index sets, budgets and statistics, outputs
    # equal up to the order of summation
    sess.decode_given_topk(d_idx, d_cnt)
    a = sess.results_host()
    vb.vatt_plan_set_option(sess.plan, vb.VATT_OPT_GIVEN_FUSED, 0)
    sess.out_o.zero_()
    sess.decode_given_topk(d_idx, d_cnt)
    b = sess.results_host()
    for key in ("counts", "b_star", "stats"):
        assert np.array_equal(a[key], b[key], equal_nan=True), "fused and separate kernels differ in " + key
    seg = a["seg"]
    for v in range(a["counts"].shape[0]):
        for h in range(a["counts"].shape[1]):
            c = a["counts"][v, h]
            for s_, cn in ((0, c[0]), (1, c[1]), (2, c[2]), (3, c[3]), (4, c[4])):
                assert np.array_equal(a["idx"][v, h, seg[s_]:seg[s_] + cn], b["idx"][v, h, seg[s_]:seg[s_] + cn])
    num = np.linalg.norm((a["O"] - b["O"]).reshape(-1, a["O"].shape[-1]), axis=1)
    den = np.linalg.norm(b["O"].reshape(-1, b["O"].shape[-1]), axis=1)
    assert np.all(num <= 3e-6 * np.maximum(den, 1e-30)), "fused and separate outputs differ: %g" % float((num / np.maximum(den, 1e-30)).max())
    assert np.allclose(a["lse"], b["lse"], rtol=0, atol=2e-5)
    return a if int(np.sum(wl.seq_lens)) % 2 else b   # either one goes on to the oracle check


@pytest.mark.parametrize("paged", [False, True])
def test_exact_topk_supplied_matches_oracle_and_the_scored_path(paged):
    say("given top-k = the oracle's exact top-k (paged=%s)" % paged)
    wl = workloads.small_gqa(seed=41, batch=2, n=3008, seq_lens=[3008, 2963])
    sess = _session(wl, paged)
    supplied = {(b, h): _oracle_topk(wl, b, h) for b in range(wl.batch) for h in range(wl.n_q_heads)}
    res = _run_given(sess, wl, supplied)
    for (b, h), arr in supplied.items():
        check_head_given(wl, res, b, h, arr, label="exact")
    # the same sets and samples as the path that scores every key (where its top-k had no near-tie swap)
    sess.decode()
    scored = sess.results_host()
    same = 0
    for b in range(wl.batch):
        for h in range(wl.n_q_heads):
            g1, g2 = gpu_segments(res, b, h), gpu_segments(scored, b, h)
            if np.array_equal(g1["I_t"], g2["I_t"]):
                same += 1
                assert np.array_equal(g1["I_bs"], g2["I_bs"])
                if g1["b"] == g2["b"]:
                    assert np.array_equal(g1["I_dyn"], g2["I_dyn"])
                assert np.linalg.norm(res["O"][b, h] - scored["O"][b, h]) <= 1e-4 * np.linalg.norm(scored["O"][b, h]) + 1e-6
    assert same >= wl.batch * wl.n_q_heads - 2
    sess.close()


def test_approximate_and_dirty_topk_sets():
    say("given top-k from noisy scores, with repeats, strays, short and empty lists")
    wl = workloads.small_gqa(seed=42, batch=2, n=5000, seq_lens=[5000, 2777], epsilon=0.03)
    sess = _session(wl)
    rng = np.random.default_rng(7)
    supplied = {}
    for b in range(wl.batch):
        n = int(wl.seq_lens[b])
        for h in range(wl.n_q_heads):
            approx = _oracle_topk(wl, b, h, noise=0.5, rng=rng)
            kind = (b * wl.n_q_heads + h) % 4
            if kind == 0:
                arr = rng.permutation(approx)                                  # any order
            elif kind == 1:
                arr = np.concatenate([approx[: len(approx) // 2], approx[:10], [0, 3, n - 1, n + 50, -4]])  # repeats, strays
                arr = rng.permutation(arr)
            elif kind == 2:
                arr = approx[:5]                                               # a short list
            else:
                arr = np.empty(0, dtype=np.int64)                              # nothing: sink, window and samples only
            supplied[(b, h)] = arr
    res = _run_given(sess, wl, supplied)
    reps = [check_head_given(wl, res, b, h, arr, label="approx") for (b, h), arr in supplied.items()]
    say("  budgets b in [%d, %d], |I_t| in [%d, %d], max O rel L2 %.2e" % (
        min(r["b"] for r in reps), max(r["b"] for r in reps), min(r["k"] for r in reps), max(r["k"] for r in reps),
        max(r["o_rel"] for r in reps)))
    sess.close()


def test_given_topk_when_a_residual_score_exceeds_every_listed_one():
    say("supplied set misses the heaviest keys: the final sample may hold scores above the shift")
    # spiky heads with planted heavy keys, and a supplied set of arbitrary tokens that misses them: sampled
    # tokens can then outweigh everything in I_f by e^20 and more; the gather rescales as it goes
    wl = workloads.small_gqa(seed=43, batch=1, n=4000, epsilon=0.02)
    sess = _session(wl)
    supplied = {(0, h): np.arange(200 + h, 3800, 37) for h in range(wl.n_q_heads)}
    res = _run_given(sess, wl, supplied)
    for (b, h), arr in supplied.items():
        check_head_given(wl, res, b, h, arr, label="missed-heavy")
    sess.close()


@pytest.mark.timeout(300)
def test_given_topk_config2_sampled_heads():
    say("config 2, given top-k from noisy scores, 8 heads checked")
    wl = workloads.config2()
    sess = _session(wl)
    rng = np.random.default_rng(3)
    heads = [0, 1, 6, 13, 16, 22, 27, 31]
    supplied = {(0, h): (_oracle_topk(wl, 0, h, noise=0.3, rng=rng) if h in heads else np.empty(0, np.int64))
                for h in range(wl.n_q_heads)}
    res = _run_given(sess, wl, supplied)
    for h in heads:
        check_head_given(wl, res, 0, h, supplied[(0, h)], label="config2")
    sess.close()


@pytest.mark.timeout(300)
def test_given_topk_config4_size_sampled_heads():
    say("config 4 shape (n = 131072, B = 1), given top-k from noisy scores, 5 heads checked")
    wl = workloads.config4(batch=1)
    sess = _session(wl)
    rng = np.random.default_rng(5)
    heads = [0, 3, 14, 21, 31]
    supplied = {(0, h): (_oracle_topk(wl, 0, h, noise=0.3, rng=rng) if h in heads else np.empty(0, np.int64))
                for h in range(wl.n_q_heads)}
    res = _run_given(sess, wl, supplied)
    for h in heads:
        check_head_given(wl, res, 0, h, supplied[(0, h)], label="config4")
    sess.close()


@pytest.mark.parametrize("d,hq,hkv", [(64, 8, 1), (64, 4, 4), (128, 16, 2)])
def test_given_topk_other_head_shapes(d, hq, hkv):
    say("given top-k, d=%d, %d/%d heads" % (d, hq, hkv))
    wl = workloads.small_gqa(seed=45, batch=2, n_q_heads=hq, n_kv_heads=hkv, head_dim=d, n=2100, seq_lens=[2100, 517])
    sess = _session(wl)
    rng = np.random.default_rng(5)
    supplied = {(b, h): _oracle_topk(wl, b, h, noise=0.2, rng=rng) for b in range(wl.batch) for h in range(hq)}
    res = _run_given(sess, wl, supplied)
    for (b, h), arr in supplied.items():
        check_head_given(wl, res, b, h, arr, label="shapes")
    sess.close()


def test_given_topk_with_nested_samples():
    say("given top-k with nested samples")
    from paper_2510_05688_amd import binding as vb
    for over in (dict(), dict(epsilon=0.01, delta=0.01)):
        wl = workloads.small_gqa(seed=47, batch=2, n=3008, seq_lens=[3008, 2963], **over)
        sess = _session(wl)
        vb.vatt_plan_set_option(sess.plan, vb.VATT_OPT_NESTED_SAMPLES, 1)
        supplied = {(b, h): _oracle_topk(wl, b, h) for b in range(wl.batch) for h in range(wl.n_q_heads)}
        res = _run_given(sess, wl, supplied)
        params = dict(wl.params, nested=True)
        reps = [check_head_given(wl, res, b, h, supplied[(b, h)], params=params, label="nested")
                for b in range(wl.batch) for h in range(wl.n_q_heads)]
        if over:
            assert any(r["b"] > r["b0"] for r in reps)
        sess.close()


@pytest.mark.parametrize("target,eps", [(1, 0.2), (2, 0.3)])
def test_given_topk_numerator_and_sdpa_targets(target, eps):
    # values with a mean component, so that the numerator budgets stay below the residual size
    say("given top-k, target %d" % target)
    from workloads.configs import default_params
    p = default_params(128, sink=16, window=24, target=target, epsilon=eps)
    wl = workloads.make_workload("given_mean_v", batch=2, n_q_heads=8, n_kv_heads=2, head_dim=128, n_max=4096,
                                 seq_lens=[4096, 3333], seed=53, params=p, v_mean=1.0, all_flat=True)
    for paged in (False, True):
        sess = _session(wl, paged=paged)
        supplied = {(b, h): _oracle_topk(wl, b, h) for b in range(wl.batch) for h in range(wl.n_q_heads)}
        res = _run_given(sess, wl, supplied)
        reps = [check_head_given(wl, res, b, h, supplied[(b, h)], label="given target %d" % target)
                for b in range(wl.batch) for h in range(wl.n_q_heads)]
        assert any(r["b0"] < r["b"] < r["oracle"]["n_s"] for r in reps)
        sess.close()


def test_given_topk_counts_out_of_range_are_clamped():
    # topk_cnt below 0 means an empty list, above the capacity means the whole row of topk_idx
    say("given top-k with out-of-range counts")
    wl = workloads.small_gqa(seed=49, batch=1, n=2000, seq_lens=[2000])
    sess = _session(wl)
    k_max = _k_max(sess)
    rng = np.random.default_rng(2)
    idx = rng.integers(-50, 2100, size=(1, wl.n_q_heads, k_max)).astype(np.int32)
    cnt = np.zeros((1, wl.n_q_heads), dtype=np.int32)
    cnt[0, ::2] = -9
    cnt[0, 1::2] = 10 ** 6
    sess.decode_given_topk(torch.from_numpy(idx).to(sess.device), torch.from_numpy(cnt).to(sess.device))
    res = sess.results_host()
    for h in range(wl.n_q_heads):
        supplied = np.empty(0, dtype=np.int64) if h % 2 == 0 else idx[0, h].astype(np.int64)
        check_head_given(wl, res, 0, h, supplied, label="clamped counts")
    sess.close()
