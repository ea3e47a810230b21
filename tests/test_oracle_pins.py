"""Pins for the CPU oracle: each part is checked against something other than itself.

Published known-answer vectors (Philox), textbook quantiles, library dense
attention (Eq. 1), brute-force enumeration on tiny inputs, textbook
simple-random-sampling moments, and hand-computed budgets on constructed
populations (Corollaries for N and D, Theorem 4.3).
"""
import itertools
import math
import os
import statistics

import numpy as np
import pytest
import scipy.special
import torch

from oracle import vatt_oracle as vo

GOLDEN = os.path.join(os.path.dirname(__file__), "golden")


def _params(**over):
    p = dict(sink=2, window=3, topk_abs=4, topk_frac=0.0, base_abs=4, base_frac=0.0,
             epsilon=0.05, delta=0.05, target=vo.TARGET_D, sm_scale=1.0, budget_cap_frac=1.0)
    p.update(over)
    return p


def _rand_head(rng, n, d, scale=1.0):
    q = rng.standard_normal(d)
    K = rng.standard_normal((n, d)) * scale
    V = rng.standard_normal((n, d))
    return q, K, V


# ---------------------------------------------------------------- Philox ----
def test_philox_known_answers():
    rows = [l.split() for l in open(os.path.join(GOLDEN, "philox4x32_10_kat.txt")) if l[0] != "#"]
    assert len(rows) == 3
    for r in rows:
        vals = [int(x, 16) for x in r]
        out = vo.philox4x32_10([np.array([v], dtype=np.uint64) for v in vals[:4]], vals[4:6])
        assert [int(o[0]) for o in out] == vals[6:10]


def test_philox_is_a_bijection_on_a_small_slice():
    # distinct counters under one key never collide (counter-mode bijection)
    blk = np.arange(4096, dtype=np.uint64)
    out = vo.philox4x32_10((blk, blk * 0, blk * 0, blk * 0), (123, 456))
    packed = (out[0].astype(np.uint64) << np.uint64(32)) | out[1].astype(np.uint64)
    packed2 = (out[2].astype(np.uint64) << np.uint64(32)) | out[3].astype(np.uint64)
    assert len(set(zip(packed.tolist(), packed2.tolist()))) == 4096


def test_draw_words_counter_layout():
    seed = (0xDEADBEEF << 32) | 0x12345678
    words = vo.draw_words(0, 23, seed, head=5, stream=1)
    assert words.dtype == np.uint32 and words.shape == (23,)
    for j in (0, 1, 3, 4, 7, 22):
        blk = vo.philox4x32_10(
            [np.array([c], dtype=np.uint64) for c in (j // 4, 1, 5, 0)], (0x12345678, 0xDEADBEEF))
        assert int(words[j]) == int(blk[j % 4][0])
    # any window of the sequence is the same sequence
    assert np.array_equal(vo.draw_words(5, 19, seed, 5, 1), words[5:19])
    assert vo.draw_words(7, 7, seed, 5, 1).shape == (0,)
    # stream, head and seed each change the words
    assert not np.array_equal(words, vo.draw_words(0, 23, seed, 5, 0))
    assert not np.array_equal(words, vo.draw_words(0, 23, seed, 6, 1))
    assert not np.array_equal(words, vo.draw_words(0, 23, seed + 1, 5, 1))
    assert not np.array_equal(words, vo.draw_words(0, 23, seed + (1 << 32), 5, 1))


def test_draw_words_look_uniform():
    u = vo.draw_words(0, 1 << 16, 99, 3, 0).astype(np.float64) / 2.0 ** 32
    assert abs(u.mean() - 0.5) < 4 * math.sqrt(1 / 12 / 65536)
    hist, _ = np.histogram(u, bins=64, range=(0, 1))
    chi2 = ((hist - 1024.0) ** 2 / 1024.0).sum()
    assert chi2 < 130.0  # chi2(63) 99.999 % point is ~ 121


def test_bounded_draw_is_exactly_uniform_by_enumeration():
    # all 2^12 words of a 12-bit generator: every value keeps exactly floor(4096 / L) words
    for L in (1, 2, 3, 7, 10, 100, 1000, 4095, 4096):
        ok, val = vo.bounded_draw(np.arange(4096), L, bits=12)
        assert val.min() >= 0 and val.max() < L
        kept = np.bincount(val[ok], minlength=L)
        assert np.all(kept == 4096 // L)
        assert int((~ok).sum()) == 4096 % L
    # 32-bit words: the value is floor(u L / 2^32), rejection is rare
    rng = np.random.default_rng(0)
    u = rng.integers(0, 1 << 32, size=1000, dtype=np.uint64)
    ok, val = vo.bounded_draw(u, 32512)
    assert [int(v) for v in val] == [(int(x) * 32512) >> 32 for x in u]
    assert ok.all()  # 2^32 mod 32512 words out of 2^32 are rejected


# ------------------------------------------------------- normal quantile ----
def test_normal_quantile_textbook_values():
    for line in open(os.path.join(GOLDEN, "normal_quantiles.txt")):
        if line.startswith("#"):
            continue
        p, z = map(float, line.split())
        assert abs(vo.normal_quantile(p) - z) < 1e-6


def test_normal_quantile_against_libraries():
    for p in [1e-6, 0.01, 0.2, 0.5, 0.8, 0.9, 0.95, 0.975, 0.9875, 0.999]:
        z = vo.normal_quantile(p)
        assert abs(z - scipy.special.ndtri(p)) < 1e-9 * max(1.0, abs(z))
        assert abs(z - statistics.NormalDist().inv_cdf(p)) < 1e-7 * max(1.0, abs(z))
    # the upper-tail form stays accurate where 1 - t is no longer representable
    for t in [0.3, 0.025, 0.0125, 1e-4, 1e-9, 1e-15]:
        z = vo.upper_tail_quantile(t)
        assert abs(z + scipy.special.ndtri(t)) < 1e-11 * max(1.0, abs(z))
    assert vo.normal_quantile(0.3) == pytest.approx(-vo.normal_quantile(0.7), abs=1e-12)


# ------------------------------------------------------ dense attention -----
def test_dense_sdpa_matches_library_softmax_attention():
    rng = np.random.default_rng(0)
    q, K, V = _rand_head(rng, 257, 16)
    scale = 0.25
    O, lse = vo.dense_sdpa(q, K, V, scale)
    a = scipy.special.softmax(scale * (K @ q))
    assert np.allclose(O, a @ V, rtol=1e-12, atol=1e-14)
    assert lse == pytest.approx(scipy.special.logsumexp(scale * (K @ q)), rel=1e-13)
    tO = torch.nn.functional.scaled_dot_product_attention(
        torch.from_numpy(q)[None, None, None, :], torch.from_numpy(K)[None, None],
        torch.from_numpy(V)[None, None], scale=scale)
    assert np.allclose(O, tO.numpy().reshape(-1), rtol=1e-10, atol=1e-13)


def test_scores_operand_order_and_scale():
    # asymmetric shapes: a transposed operand or a dropped scale cannot pass
    K = np.array([[1.0, 2.0, 3.0], [0.0, -1.0, 0.5]])
    q = np.array([2.0, 0.5, -1.0])
    assert np.allclose(vo.scores(q, K, 0.5), [0.5 * (2 + 1 - 3), 0.5 * (0 - 0.5 - 0.5)])


# --------------------------------------------------- deterministic set ------
def test_deterministic_set_vs_sort_and_bruteforce():
    rng = np.random.default_rng(1)
    for n, sink, window, k in [(64, 4, 8, 5), (50, 0, 0, 7), (40, 3, 0, 0), (33, 5, 6, 100), (10, 8, 8, 3), (6, 0, 9, 2)]:
        s = rng.standard_normal(n)
        I_s, I_l, I_t, R = vo.deterministic_set(s, sink, window, k)
        ns_ = min(sink, n)
        nl_ = min(window, n - ns_)
        assert I_s.tolist() == list(range(ns_))
        assert I_l.tolist() == list(range(n - nl_, n))
        mid = list(range(ns_, n - nl_))
        kk = min(k, len(mid))
        brute = sorted(sorted(mid, key=lambda i: (-s[i], i))[:kk])
        assert I_t.tolist() == brute
        if kk:
            arg = np.argsort(-s[ns_:n - nl_], kind="stable")[:kk] + ns_
            assert sorted(arg.tolist()) == brute
        assert sorted(I_s.tolist() + I_l.tolist() + I_t.tolist() + R.tolist()) == list(range(n))
        if len(R) and kk:
            assert s[R].max() <= s[I_t].min()


def test_topk_ties_go_to_lower_index():
    s = np.array([9.0, 1.0, 5.0, 5.0, 5.0, 0.0, 5.0, 9.0])
    _, _, I_t, R = vo.deterministic_set(s, 1, 1, 2)
    assert I_t.tolist() == [2, 3]
    assert R.tolist() == [1, 4, 5, 6]


def test_topk_and_base_counts():
    assert vo.topk_count(32768, 128, 128, 0, 0.025) == 819
    assert vo.topk_count(131072, 128, 512, 0, 0.01) == 1310
    assert vo.topk_count(1024, 4, 32, 32, 0.5) == 32
    assert vo.base_count(31693, 0, 0.025) == 792
    assert vo.base_count(100, 0, 0.0) == 2      # f_b = 0 still leaves two tokens for a variance
    assert vo.base_count(1, 0, 0.5) == 1
    assert vo.base_count(10, 64, 0.0) == 10


# ------------------------------------------------------------- sampler ------
def _sample(residual, c, seed, head=0, stream=0, lo=None, L=None, cap=None):
    residual = np.asarray(residual)
    lo = int(residual.min()) if lo is None else lo
    L = int(residual.max()) - lo + 1 if L is None else L
    return vo.uniform_sample(residual, c, mid_lo=lo, mid_len=L, seed=seed, head=head, stream=stream, draw_cap=cap)


def test_uniform_sample_worked_example_from_the_published_vector():
    # Philox4x32-10 of the all-zero counter under the all-zero key is 6627e8d5 e169c58d bc57ac4c 9b00dbd8
    # (first row of the known-answer file).  With a middle region of 10 tokens starting at token 5 the first
    # four draws of (seed 0, head 0, stream 0) propose floor(u * 10 / 2^32) = 3, 8, 7, 6 -> tokens 8, 13, 12, 11.
    assert [(w * 10) >> 32 for w in (0x6627E8D5, 0xE169C58D, 0xBC57AC4C, 0x9B00DBD8)] == [3, 8, 7, 6]
    residual = np.arange(5, 15)
    assert _sample(residual, 1, 0, lo=5, L=10).tolist() == [8]
    assert _sample(residual, 3, 0, lo=5, L=10).tolist() == [8, 12, 13]
    assert _sample(residual, 4, 0, lo=5, L=10).tolist() == [8, 11, 12, 13]
    # token 13 in the top-k set (not residual): its draw is skipped
    no13 = np.setdiff1d(residual, [13])
    assert _sample(no13, 3, 0, lo=5, L=10).tolist() == [8, 11, 12]
    # more than half of the residual: the first n_s - c accepted tokens are the ones left out
    assert _sample(residual, 9, 0, lo=5, L=10).tolist() == np.setdiff1d(residual, [8]).tolist()
    assert _sample(residual, 7, 0, lo=5, L=10).tolist() == np.setdiff1d(residual, [8, 13, 12]).tolist()
    assert _sample(residual, 10, 0, lo=5, L=10).tolist() == residual.tolist()
    assert _sample(residual, 0, 0, lo=5, L=10).tolist() == []


def test_decode_head_draws_over_the_middle_region_worked_example():
    # The same published vector, now through decode_head: 20 tokens, sink 5, window 5 -> the middle region is
    # tokens 5 .. 14 (10 tokens), so with seed 0 and head 0 the base sample's draws propose tokens 8, 13, 12, 11
    # whatever the scores are.  (Drawing over a longer or shifted range, e.g. including the window, would
    # propose other tokens: floor(0x6627e8d5 * 15 / 2^32) = 5.)
    rng = np.random.default_rng(3)
    q, K, V = rng.standard_normal(8), rng.standard_normal((20, 8)), rng.standard_normal((20, 8))
    params = dict(sm_scale=0.3, sink=5, window=5, topk_abs=0, topk_frac=0.0, base_abs=3, base_frac=0.0,
                  epsilon=0.9, delta=0.9, target=vo.TARGET_D, budget_cap_frac=1.0)
    r = vo.decode_head(q, K, V, seed=0, head=0, params=params)
    assert r["n_s"] == 10 and r["I_bs"].tolist() == [8, 12, 13]
    # token 13 made the largest score of the middle region and k = 1: it is in I_t, its draw is skipped
    K2 = K.copy()
    K2[13] = 50.0 * q / np.linalg.norm(q)
    r = vo.decode_head(q, K2, V, seed=0, head=0, params=dict(params, topk_abs=1))
    assert r["I_t"].tolist() == [13] and r["n_s"] == 9 and r["I_bs"].tolist() == [8, 11, 12]
    # nested samples: the base sample is kept and the extension comes from the second draw sequence (stream 1),
    # skipping the base sample; the first sequence would continue with token 11
    ok, val = vo.bounded_draw(vo.draw_words(0, 64, 0, 0, 1), 10)
    second = [5 + int(v) for a, v in zip(ok, val) if a and 5 + int(v) not in (8, 12, 13)]
    r = vo.decode_head(q, K, V, seed=0, head=0, params=dict(params, nested=True), forced_b=4)
    assert r["I_bs"].tolist() == [8, 12, 13] and r["I_dyn"].tolist() == sorted([8, 12, 13, second[0]])
    assert second[0] != 11


def test_uniform_sample_invariants():
    residual = np.setdiff1d(np.arange(10, 480), np.arange(50, 400, 7))
    n_s = len(residual)
    prev = np.empty(0, dtype=np.int64)
    for c in [0, 1, 2, 17, 100, n_s // 2]:
        smp = _sample(residual, c, 42, head=2, lo=10, L=470)
        assert smp.shape[0] == c
        assert np.all(np.diff(smp) > 0)                  # ascending, no duplicates
        assert np.all(np.isin(smp, residual))            # only residual tokens
        assert np.all(np.isin(prev, smp))                # first-c-accepted: sample(c) lies in sample(c+1)
        prev = smp
    prev = residual
    for c in [n_s, n_s - 1, n_s - 30, n_s // 2 + 1]:     # complement regime shrinks the same way
        smp = _sample(residual, c, 42, head=2, lo=10, L=470)
        assert smp.shape[0] == c and np.all(np.diff(smp) > 0) and np.all(np.isin(smp, residual))
        assert np.all(np.isin(smp, prev))
        prev = smp
    assert np.array_equal(_sample(residual, 60, 42, head=2, lo=10, L=470), _sample(residual, 60, 42, head=2, lo=10, L=470))
    assert not np.array_equal(_sample(residual, 60, 42, head=2, lo=10, L=470), _sample(residual, 60, 42, head=2, stream=1, lo=10, L=470))


def test_default_draw_cap_does_not_disturb_uniformity_of_a_sparse_residual():
    # two residual tokens in a middle region of 1000 (everything else is in the top-k set): a draw hits one of
    # them with probability 1/500, so a sample needs about 500 draws and sometimes several thousand.  The draw
    # limit must be far beyond that, or the fall-back (lowest index first) would favour token 300: with a limit
    # of 1000 draws it would be chosen in 57 % of the seeds.
    residual = np.array([300, 700])
    first = sum(int(vo.uniform_sample(residual, 1, mid_lo=100, mid_len=1000, seed=s, head=0, stream=0)[0] == 300)
                for s in range(1500))
    assert abs(first / 1500.0 - 0.5) < 4.0 * math.sqrt(0.25 / 1500.0)
    assert vo.default_draw_cap(1000) >= 64 * 1000


def test_uniform_sample_draw_cap_completes_in_index_order():
    residual = np.arange(5, 15)
    # cap of two draws: tokens 8 and 13 are accepted, the rest of a sample of 4 is filled from the low end
    assert _sample(residual, 4, 0, lo=5, L=10, cap=2).tolist() == [5, 6, 8, 13]
    assert _sample(residual, 4, 0, lo=5, L=10, cap=0).tolist() == [5, 6, 7, 8]
    # complement regime: tokens left out are 8 (drawn) and then 5, 6 (filled)
    assert _sample(residual, 7, 0, lo=5, L=10, cap=1).tolist() == [7, 9, 10, 11, 12, 13, 14]


@pytest.mark.parametrize("c", [2, 3])
def test_uniform_sample_is_uniform_over_subsets(c):
    # n_s = 5 inside a middle region of 7 tokens; c = 2 (direct) and c = 3 (complement): each of the 10
    # subsets should appear with probability 1/10
    residual = np.array([2, 3, 5, 6, 7])
    counts = {}
    trials = 20000
    for seed in range(trials):
        smp = tuple(_sample(residual, c, seed, stream=1, lo=2, L=7).tolist())
        counts[smp] = counts.get(smp, 0) + 1
    assert len(counts) == 10
    chi2 = sum((v - trials / 10) ** 2 / (trials / 10) for v in counts.values())
    assert chi2 < 33.7  # chi2(9) 99.99 % point


@pytest.mark.parametrize("c", [16, 40])
def test_uniform_sample_inclusion_frequency(c):
    residual = np.setdiff1d(np.arange(8, 76), [20, 21, 40, 63])   # 64 residual tokens in a region of 68
    trials = 6000
    hits = np.zeros(80)
    for seed in range(trials):
        hits[_sample(residual, c, 1000 + seed, head=4, lo=8, L=68)] += 1
    p = c / len(residual)
    z = (hits[residual] - trials * p) / math.sqrt(trials * p * (1 - p))
    assert np.abs(z).max() < 4.5
    assert hits[:8].sum() == 0 and hits[76:].sum() == 0 and hits[[20, 21, 40, 63]].sum() == 0


# ------------------------------------------------- estimator, brute force ---
def test_estimator_mean_over_all_subsets_is_exact():
    rng = np.random.default_rng(3)
    n, d = 20, 3
    q, K, V = _rand_head(rng, n, d)
    s = vo.scores(q, K, 0.7)
    m = s.max()
    I_s, I_l, I_t, R = vo.deterministic_set(s, 2, 3, 4)
    I_f = np.concatenate([I_s, I_l, I_t])
    n_s = len(R)
    assert n_s == 11
    w = np.exp(s - m)
    D_true = w.sum()
    N_true = w @ V
    for b in (1, 3, 5, n_s):
        Ds, Ns = [], []
        for combo in itertools.combinations(R.tolist(), b):
            N, D = vo.estimate(s, V, m, I_f, np.array(combo), n_s)
            Ds.append(D)
            Ns.append(N)
        assert np.mean(Ds) == pytest.approx(D_true, rel=1e-12)
        assert np.allclose(np.mean(Ns, axis=0), N_true, rtol=1e-11, atol=1e-13)
        # textbook variance of the expansion estimator under sampling without replacement
        S2 = w[R].var(ddof=1)
        assert np.var(Ds) == pytest.approx(n_s ** 2 * (1 - b / n_s) * S2 / b, rel=1e-9, abs=1e-18)


def test_estimate_with_empty_sample_is_softmax_over_I_f():
    rng = np.random.default_rng(4)
    q, K, V = _rand_head(rng, 30, 4)
    s = vo.scores(q, K, 1.0)
    I_f = np.array([0, 1, 7, 28, 29])
    N, D = vo.estimate(s, V, s.max(), I_f, np.empty(0, np.int64), 25)
    a = scipy.special.softmax(s[I_f])
    assert np.allclose(N / D, a @ V[I_f], rtol=1e-12)


# ------------------------------------------------- whole step, check (a) ----
@pytest.mark.parametrize("target", [vo.TARGET_D, vo.TARGET_N, vo.TARGET_SDPA])
def test_full_budget_equals_dense(target):
    rng = np.random.default_rng(5)
    n, d = 300, 8
    q, K, V = _rand_head(rng, n, d)
    V = V + 1.0
    # a base sample that already covers the residual forces b = n_s
    r = vo.decode_head(q, K, V, seed=11, head=0,
                       params=_params(sink=5, window=9, topk_abs=20, base_abs=10 ** 6, target=target, sm_scale=0.4))
    O, lse = vo.dense_sdpa(q, K, V, 0.4)
    assert r["b"] == r["n_s"] == n - 34
    assert np.allclose(r["O"], O, rtol=1e-12, atol=1e-14)
    assert r["lse"] == pytest.approx(lse, rel=1e-13)
    # a tiny epsilon reaches the same through the budget formula
    r2 = vo.decode_head(q, K, V, seed=11, head=0,
                        params=_params(sink=5, window=9, topk_abs=20, base_abs=8, epsilon=1e-7, target=target, sm_scale=0.4))
    assert r2["b"] == r2["n_s"]
    assert np.allclose(r2["O"], O, rtol=1e-12, atol=1e-14)


def test_no_residual_is_exact_softmax():
    rng = np.random.default_rng(6)
    q, K, V = _rand_head(rng, 12, 4)
    for p in (_params(sink=8, window=8), _params(sink=2, window=3, topk_abs=50)):
        r = vo.decode_head(q, K, V, seed=1, head=0, params=p)
        O, lse = vo.dense_sdpa(q, K, V, 1.0)
        assert r["n_s"] == 0 and r["b"] == 0
        assert np.allclose(r["O"], O, rtol=1e-13)
        assert r["lse"] == pytest.approx(lse, rel=1e-14)


def test_output_is_importance_weighted_softmax_of_eq3():
    # Eq. 3 written out: weights exp(s_i)/p_i over S = [I_f, I_dyn], p = [1, b/n_s]
    rng = np.random.default_rng(7)
    q, K, V = _rand_head(rng, 200, 6)
    r = vo.decode_head(q, K, V, seed=3, head=1, params=_params(sink=4, window=6, topk_abs=10, base_abs=12, sm_scale=0.5))
    s = 0.5 * (K @ q)
    I_f = np.concatenate([r["I_s"], r["I_l"], r["I_t"]])
    S = np.concatenate([I_f, r["I_dyn"]])
    p = np.concatenate([np.ones(len(I_f)), np.full(r["b"], r["b"] / r["n_s"])])
    a = np.exp(s[S]) / p
    a = a / a.sum()
    assert np.allclose(r["O"], a @ V[S], rtol=1e-11)
    assert r["lse"] == pytest.approx(math.log((np.exp(s[S]) / p).sum()), rel=1e-12)
    assert len(np.intersect1d(I_f, r["I_dyn"])) == 0
    assert len(np.intersect1d(I_f, r["I_bs"])) == 0


# ------------------------------------------------------ budget formulas -----
def _scalar_head(s_values, v_values=None):
    """A head whose scores are exactly s_values: d = 1, q = [1], K[i] = [s_i]."""
    s_values = np.asarray(s_values, dtype=np.float64)
    K = s_values[:, None]
    V = np.ones_like(K) if v_values is None else np.asarray(v_values, np.float64)[:, None]
    return np.array([1.0]), K, V


def test_constant_residual_needs_no_samples():
    s = np.concatenate([[3.0, 2.0], np.full(40, -1.0), [0.5, 0.7]])
    q, K, V = _scalar_head(s)
    r = vo.decode_head(q, K, V, seed=0, head=0, params=_params(sink=2, window=2, topk_abs=0, base_abs=6))
    assert r["stats"]["sigma2"] == pytest.approx(0.0, abs=1e-30)
    assert r["b_star"] == pytest.approx(0.0, abs=1e-20)
    assert r["b"] == r["b0"] == 6
    # and the estimate is then exact whatever the sample
    O, _ = vo.dense_sdpa(q, K, V, 1.0)
    assert np.allclose(r["O"], O, rtol=1e-13)


def test_two_valued_residual_budget_by_hand_target_D():
    # residual: a tokens with weight alpha, c tokens with weight beta; base sample = whole residual,
    # so sigma is the population value and D_hat = D exactly.
    a, c = 30, 70
    sa, sb = math.log(0.5), math.log(0.1)          # weights relative to the max score 0
    s = np.concatenate([[0.0], np.full(a, sa), np.full(c, sb), [math.log(0.25)]])
    q, K, V = _scalar_head(s)
    eps, dlt = 0.05, 0.1
    r = vo.decode_head(q, K, V, seed=9, head=0,
                       params=_params(sink=1, window=1, topk_abs=0, base_abs=1000, epsilon=eps, delta=dlt))
    n_s = a + c
    mean = (a * 0.5 + c * 0.1) / n_s
    S2 = (a * (0.5 - mean) ** 2 + c * (0.1 - mean) ** 2) / (n_s - 1)
    D = 1.0 + 0.25 + a * 0.5 + c * 0.1
    # the interface carries delta as a 32-bit float: 0.1 is stored as 0.100000001490116
    z = scipy.special.ndtri(1.0 - np.float64(np.float32(dlt)) / 2.0)
    assert z == pytest.approx(1.6448536269514722, rel=1e-8)  # Phi^{-1}(0.95)
    hand = (z * n_s * math.sqrt(S2) / (np.float64(np.float32(eps)) * D)) ** 2
    assert r["n_s"] == n_s and r["b0"] == n_s
    assert r["stats"]["sigma2"] == pytest.approx(S2, rel=1e-12)
    assert r["stats"]["D_hat"] == pytest.approx(D, rel=1e-12)
    assert r["b_star"] == pytest.approx(hand, rel=1e-9)
    assert r["b"] == n_s  # lower cap by the base sample


def test_two_valued_residual_budget_by_hand_target_N_and_SDPA():
    a, c = 25, 55
    s = np.concatenate([[0.0], np.full(a, math.log(0.5)), np.full(c, math.log(0.2)), [math.log(0.25)]])
    v = np.concatenate([[2.0], np.full(a, 1.0), np.full(c, 3.0), [-1.0]])
    q, K, V = _scalar_head(s, v)
    eps, dlt = 0.1, 0.2
    n_s = a + c
    # r_i = w_i v_i: 0.5 and 0.6
    rm = (a * 0.5 + c * 0.6) / n_s
    tr = (a * (0.5 - rm) ** 2 + c * (0.6 - rm) ** 2) / (n_s - 1)
    N = 1.0 * 2.0 + 0.25 * -1.0 + a * 0.5 + c * 0.6
    wm = (a * 0.5 + c * 0.2) / n_s
    S2 = (a * (0.5 - wm) ** 2 + c * (0.2 - wm) ** 2) / (n_s - 1)
    D = 1.0 + 0.25 + a * 0.5 + c * 0.2
    e = float(np.float64(np.float32(eps)))
    dl = float(np.float64(np.float32(dlt)))
    rN = vo.decode_head(q, K, V, seed=9, head=0,
                        params=_params(sink=1, window=1, topk_abs=0, base_abs=1000, epsilon=eps, delta=dlt, target=vo.TARGET_N))
    z = scipy.special.ndtri(1 - dl / 2)
    assert rN["stats"]["tr_sigma"] == pytest.approx(tr, rel=1e-12)
    assert rN["stats"]["N_hat_sq"] == pytest.approx(N * N, rel=1e-12)
    assert rN["b_star"] == pytest.approx((z * n_s * math.sqrt(tr) / (e * abs(N))) ** 2, rel=1e-9)
    rS = vo.decode_head(q, K, V, seed=9, head=0,
                        params=_params(sink=1, window=1, topk_abs=0, base_abs=1000, epsilon=eps, delta=dlt, target=vo.TARGET_SDPA))
    rho_D = n_s * math.sqrt(S2) / D
    rho_N = n_s * math.sqrt(tr) / abs(N)
    z4 = scipy.special.ndtri(1 - dl / 4)
    assert rS["b_star"] == pytest.approx((2 * z4 * (rho_D + rho_N) / e) ** 2, rel=1e-9)

    # Theorem 4.3: b_SDPA is min over (eps', delta') of max(b_D(eps'/2, delta'), b_N((eps-eps')/2, delta-delta')).
    # The closed form is that expression at delta' = delta/2 minimised over eps'; a grid search of the
    # theorem's expression at delta' = delta/2 must agree, and no grid point with another delta' is
    # required to be worse -- only the closed form must be a feasible value (>= the global minimum).
    def bD(e_, d_):
        return (scipy.special.ndtri(1 - d_ / 2) * rho_D / e_) ** 2

    def bN(e_, d_):
        return (scipy.special.ndtri(1 - d_ / 2) * rho_N / e_) ** 2

    grid_e = np.linspace(1e-4, e - 1e-4, 20001)
    at_half = min(max(bD(x / 2, dl / 2), bN((e - x) / 2, dl / 2)) for x in grid_e)
    assert rS["b_star"] == pytest.approx(at_half, rel=1e-4)
    glob = min(max(bD(x / 2, y), bN((e - x) / 2, dl - y))
               for x in np.linspace(1e-3, e - 1e-3, 400) for y in np.linspace(1e-3, dl - 1e-3, 100))
    assert rS["b_star"] >= glob * (1 - 1e-9)


def test_budget_scales_as_the_formula_says():
    # b* ~ (z/eps)^2: halving eps quadruples b*, and delta enters only through the quantile
    rng = np.random.default_rng(8)
    q, K, V = _rand_head(rng, 400, 8, scale=0.5)
    base = _params(sink=4, window=4, topk_abs=10, base_abs=50, epsilon=0.1, delta=0.1, sm_scale=0.35)
    r1 = vo.decode_head(q, K, V, seed=2, head=0, params=base)
    r2 = vo.decode_head(q, K, V, seed=2, head=0, params=dict(base, epsilon=0.05))
    r3 = vo.decode_head(q, K, V, seed=2, head=0, params=dict(base, delta=0.02))
    e1, e2 = np.float64(np.float32(0.1)), np.float64(np.float32(0.05))
    assert r2["b_star"] / r1["b_star"] == pytest.approx((e1 / e2) ** 2, rel=1e-12)
    zq = lambda d_: scipy.special.ndtri(1 - np.float64(np.float32(d_)) / 2)
    assert r3["b_star"] / r1["b_star"] == pytest.approx((zq(0.02) / zq(0.1)) ** 2, rel=1e-9)
    # the statistics are those of the base sample, recomputed here from their definitions
    s = 0.35 * (K @ q)
    w = np.exp(s - s.max())
    I_f = np.concatenate([r1["I_s"], r1["I_l"], r1["I_t"]])
    assert r1["stats"]["sigma2"] == pytest.approx(np.var(w[r1["I_bs"]], ddof=1), rel=1e-12)
    assert r1["stats"]["D_hat"] == pytest.approx(w[I_f].sum() + r1["n_s"] * w[r1["I_bs"]].mean(), rel=1e-12)
    rN = vo.decode_head(q, K, V, seed=2, head=0, params=dict(base, target=vo.TARGET_N))
    rr = w[rN["I_bs"], None] * V[rN["I_bs"]]
    assert rN["stats"]["tr_sigma"] == pytest.approx(np.trace(np.cov(rr.T, ddof=1)), rel=1e-11)
    Nh = w[I_f] @ V[I_f] + rN["n_s"] * rr.mean(axis=0)
    assert rN["stats"]["N_hat_sq"] == pytest.approx(Nh @ Nh, rel=1e-11)


def test_shift_invariance():
    # appending a constant coordinate to K and q adds the same constant to every score:
    # selections, budget and output must not move
    rng = np.random.default_rng(9)
    q, K, V = _rand_head(rng, 300, 8, scale=0.6)
    p = _params(sink=4, window=8, topk_abs=12, base_abs=30, epsilon=0.02, sm_scale=0.5)
    r1 = vo.decode_head(q, K, V, seed=5, head=2, params=p)
    q2 = np.concatenate([q, [2.0]])
    K2 = np.concatenate([K, np.full((300, 1), 7.0)], axis=1)
    r2 = vo.decode_head(q2, K2, V, seed=5, head=2, params=p)
    for key in ("I_t", "I_bs", "I_dyn"):
        assert np.array_equal(r1[key], r2[key])
    assert r1["b"] == r2["b"] and r1["b_star"] == pytest.approx(r2["b_star"], rel=1e-9)
    assert np.allclose(r1["O"], r2["O"], rtol=1e-10)
    assert r2["lse"] - r1["lse"] == pytest.approx(0.5 * 14.0, rel=1e-10)


def test_clamp_budget_cases():
    assert vo.clamp_budget(0.0, 32, 1000, 1.0) == 32          # lower cap
    assert vo.clamp_budget(100.2, 32, 1000, 1.0) == 101        # ceil
    assert vo.clamp_budget(100.0, 32, 1000, 1.0) == 100        # exact integer stays
    assert vo.clamp_budget(5000.0, 32, 1000, 1.0) == 1000      # cannot exceed the residual
    assert vo.clamp_budget(float("inf"), 32, 1000, 1.0) == 1000
    assert vo.clamp_budget(float("nan"), 32, 1000, 1.0) == 1000
    assert vo.clamp_budget(800.0, 32, 1000, 0.5) == 500        # explicit cap
    assert vo.clamp_budget(800.0, 600, 1000, 0.5) == 600       # lower cap wins over the explicit cap
    assert vo.clamp_budget(3.0, 2, 2, 1.0) == 2


def test_clamp_budget_rounds_up_to_a_multiple_when_asked():
    # an option beyond the paper: b goes up to the next multiple of 64, never beyond what the plain rule can reach
    assert vo.clamp_budget(100.2, 32, 1000, 1.0, 64) == 128
    assert vo.clamp_budget(128.0, 32, 1000, 1.0, 64) == 128       # a multiple stays
    assert vo.clamp_budget(128.5, 32, 1000, 1.0, 64) == 192
    assert vo.clamp_budget(0.0, 32, 1000, 1.0, 64) == 64          # the lower cap first, then the rounding
    assert vo.clamp_budget(990.0, 32, 1000, 1.0, 64) == 1000      # 1024 would exceed the residual
    assert vo.clamp_budget(800.0, 32, 1000, 0.5, 64) == 500       # ... or the explicit cap
    assert vo.clamp_budget(200.0, 32, 1000, 0.5, 64) == 256
    assert vo.clamp_budget(3.0, 600, 1000, 0.5, 64) == 600        # lower cap above the explicit cap: nothing above it
    assert vo.clamp_budget(100.2, 32, 1000, 1.0, 1) == 101
    for b_star in (0.0, 17.3, 64.0, 65.0, 400.0, 5000.0):         # never fewer samples than the paper's rule
        for q in (2, 16, 64, 100):
            plain, rounded = vo.clamp_budget(b_star, 8, 777, 1.0), vo.clamp_budget(b_star, 8, 777, 1.0, q)
            assert plain <= rounded <= 777 and (rounded % q == 0 or rounded == 777) and rounded - plain < q
    # the legal budgets near an integer b* follow the same rounding
    assert vo.budget_alternatives(128.000001, 10, 1000, 1.0, multiple=64) == [192, 128]
    assert vo.budget_alternatives(100.5, 10, 1000, 1.0, multiple=64) == [128]
    # through Algorithm 1: the final sample has the rounded size and the estimate stays exact over all samples
    rng = np.random.default_rng(5)
    q, K, V = _rand_head(rng, 400, 8)
    p = _params(sink=4, window=4, topk_abs=8, base_abs=20, sm_scale=0.4, epsilon=0.2, delta=0.2)
    plain = vo.decode_head(q, K, V, seed=3, head=1, params=p)
    rounded = vo.decode_head(q, K, V, seed=3, head=1, params=dict(p, budget_multiple=64))
    assert plain["b_star"] == rounded["b_star"] and np.array_equal(plain["I_bs"], rounded["I_bs"])
    assert plain["b"] % 64 != 0 and rounded["b"] == (plain["b"] + 63) // 64 * 64 == len(rounded["I_dyn"])


def test_alternatives_enumerate_near_ties():
    s = np.array([5.0, 4.0, 3.0, 3.0 + 1e-7, 2.0, 1.0, 0.0])
    alts = vo.topk_alternatives(s, 0, 0, 3, rel_tol=1e-5)
    assert [a.tolist() for a in alts] == [[0, 1, 3], [0, 1, 2]]
    assert len(vo.topk_alternatives(s, 0, 0, 2, rel_tol=1e-5)) == 1
    # the tolerance is relative: at scores near 300 a gap of 1e-3 is a tie (3e-6 relative), a gap of 1e-2 is not
    big = np.array([500.0, 300.0, 300.0 + 1e-3, 300.0 - 1e-2, 10.0])
    assert [a.tolist() for a in vo.topk_alternatives(big, 0, 0, 2, rel_tol=1e-5)] == [[0, 2], [0, 1]]
    assert vo.budget_alternatives(100.000001, 10, 1000, 1.0) == [101, 100]
    assert vo.budget_alternatives(100.5, 10, 1000, 1.0) == [101]
    # the window around b* is 1e-6 relative: 100.001 (1e-5 above an integer) has one legal budget only,
    # 99.99999995 (5e-10 below one) has the next integer as well
    assert vo.budget_alternatives(100.001, 10, 1000, 1.0) == [101]
    assert vo.budget_alternatives(99.99999995, 10, 1000, 1.0) == [100, 101]
    r = vo.decode_head(*_scalar_head(s), seed=1, head=0,
                       params=_params(sink=0, window=0, topk_abs=3, base_abs=2), forced_topk=alts[1])
    assert r["I_t"].tolist() == [0, 1, 2] and 3 not in r["I_t"] and r["n_s"] == 4


def test_decode_batch_maps_gqa_heads():
    # the batch driver against Algorithm 1 called by hand on hand-sliced inputs, for every (sequence, head):
    # query head h reads KV head h // 4, draws with its own index h and the seed of its sequence, and sees
    # seq_lens[b] tokens
    rng = np.random.default_rng(10)
    B, Hq, Hkv, n, d = 2, 8, 2, 200, 8
    q = rng.standard_normal((B, Hq, d))
    K = rng.standard_normal((B, Hkv, n, d))
    V = rng.standard_normal((B, Hkv, n, d))
    lens = np.array([200, 140])
    seeds = np.array([7, 8], dtype=np.uint64)
    p = _params(sink=2, window=2, topk_abs=4, base_abs=16, sm_scale=0.3, epsilon=0.5, delta=0.5)
    out = vo.decode(q, K, V, lens, seeds, p)
    assert set(out) == {(b, h) for b in range(B) for h in range(Hq)}
    for b in range(B):
        for h in range(Hq):
            kv = [0, 0, 0, 0, 1, 1, 1, 1][h]
            one = vo.decode_head(q[b, h], K[b, kv, :lens[b]], V[b, kv, :lens[b]], seed=int(seeds[b]), head=h, params=p)
            assert out[(b, h)]["n"] == lens[b]
            for key in ("I_t", "I_bs", "I_dyn"):
                assert np.array_equal(out[(b, h)][key], one[key]), (b, h, key)
            assert np.allclose(out[(b, h)]["O"], one["O"], rtol=0, atol=0)
    assert any(out[(b, h)]["b"] < out[(b, h)]["n_s"] for b in range(B) for h in range(Hq))   # real samples
    # the draws do depend on the head index and on the sequence's seed
    other_head = vo.decode_head(q[1, 3], K[1, 0, :140], V[1, 0, :140], seed=8, head=0, params=p)
    other_seed = vo.decode_head(q[1, 3], K[1, 0, :140], V[1, 0, :140], seed=7, head=3, params=p)
    assert not np.array_equal(out[(1, 3)]["I_bs"], other_head["I_bs"])
    assert not np.array_equal(out[(1, 3)]["I_bs"], other_seed["I_bs"])


# ------------------------------------------------- multi-query step (chunk) ----
def test_draw_words_places_the_query_in_the_last_counter_word():
    # the published vector with four different counter words fixes which argument lands in which word:
    # counter (243f6a88, 85a308d3, 13198a2e, 03707344), key (a4093822, 299f31d0)
    rows = [l.split() for l in open(os.path.join(GOLDEN, "philox4x32_10_kat.txt")) if l[0] != "#"]
    vals = [int(x, 16) for x in rows[2]]
    seed = (vals[5] << 32) | vals[4]
    words = vo.draw_words(4 * vals[0], 4 * vals[0] + 4, seed, head=vals[2], stream=vals[1], query=vals[3])
    assert [int(w) for w in words] == vals[6:10]
    # query 0 is the single-token sequence
    assert np.array_equal(vo.draw_words(0, 64, 77, 3, 1), vo.draw_words(0, 64, 77, 3, 1, query=0))
    assert not np.array_equal(vo.draw_words(0, 64, 77, 3, 1), vo.draw_words(0, 64, 77, 3, 1, query=1))


def test_chunk_lengths_are_causal():
    # query t of Q sits at position n - Q + t and sees positions 0 .. n - Q + t
    assert [vo.chunk_length(100, 4, t) for t in range(4)] == [97, 98, 99, 100]
    assert vo.chunk_length(100, 1, 0) == 100
    assert vo.chunk_length(2, 4, 0) == 0


def test_chunk_with_full_budget_is_causal_dense_attention():
    # b0 = n_s makes every query exact; the library's causal attention over the chunk is the reference.
    # (is_causal aligns the mask to the top left, so the explicit lower-right mask is built here.)
    rng = np.random.default_rng(31)
    B, Q, Hq, Hkv, d, n = 2, 3, 4, 2, 8, 40
    q = rng.standard_normal((B, Q, Hq, d))
    K = rng.standard_normal((B, Hkv, n, d))
    V = rng.standard_normal((B, Hkv, n, d))
    lens = np.array([40, 29])
    p = _params(sink=2, window=3, topk_abs=4, base_abs=1000, sm_scale=0.3)
    res = vo.decode_chunk(q, K, V, lens, np.array([5, 6]), p)
    for b in range(B):
        nb = int(lens[b])
        mask = torch.zeros(Q, nb, dtype=torch.bool)
        for t in range(Q):
            mask[t, : nb - Q + 1 + t] = True
        for h in range(Hq):
            ref = torch.nn.functional.scaled_dot_product_attention(
                torch.from_numpy(q[b, :, h])[None], torch.from_numpy(K[b, h // 2, :nb])[None],
                torch.from_numpy(V[b, h // 2, :nb])[None], attn_mask=mask[None], scale=0.3)[0].numpy()
            for t in range(Q):
                r = res[(b, t, h)]
                assert r["n"] == nb - Q + 1 + t and r["b"] == r["n_s"]
                np.testing.assert_allclose(r["O"], ref[t], rtol=1e-12, atol=1e-13)


def test_chunk_of_one_query_is_the_single_token_step():
    rng = np.random.default_rng(32)
    q = rng.standard_normal((1, 1, 2, 8))
    K = rng.standard_normal((1, 1, 300, 8))
    V = rng.standard_normal((1, 1, 300, 8))
    p = _params(sink=4, window=4, topk_abs=10, base_abs=20, sm_scale=0.35)
    a = vo.decode_chunk(q, K, V, np.array([300]), np.array([9]), p)
    b = vo.decode(q[:, 0], K, V, np.array([300]), np.array([9]), p)
    for h in range(2):
        assert np.array_equal(a[(0, 0, h)]["I_dyn"], b[(0, h)]["I_dyn"])
        assert np.array_equal(a[(0, 0, h)]["O"], b[(0, h)]["O"])


def test_chunk_queries_draw_independent_samples_from_their_own_residual():
    rng = np.random.default_rng(33)
    Q, n = 4, 400
    q = rng.standard_normal((1, Q, 1, 8))
    K = rng.standard_normal((1, 1, n, 8))
    V = rng.standard_normal((1, 1, n, 8))
    p = _params(sink=4, window=6, topk_abs=12, base_abs=40, sm_scale=0.35)
    res = vo.decode_chunk(q, K, V, np.array([n]), np.array([1234]), p)
    samples = []
    for t in range(Q):
        r = res[(0, t, 0)]
        nt = n - Q + 1 + t
        assert r["n"] == nt
        assert np.array_equal(r["I_l"], np.arange(nt - 6, nt))          # the window ends at the query itself
        taken = set(r["I_t"].tolist())
        assert all(4 <= i < nt - 6 and i not in taken for i in r["I_dyn"].tolist())
        assert len(set(r["I_dyn"].tolist())) == r["b"]
        samples.append(set(r["I_dyn"].tolist()))
    # different query tokens use different draw sequences
    assert samples[0] != samples[1] and samples[1] != samples[2]


def test_chunk_driver_passes_prefix_query_position_head_and_seed():
    # every (sequence, query token, head) of the chunk driver against Algorithm 1 called by hand on the causal
    # prefix, with the query's position as the last counter word
    rng = np.random.default_rng(34)
    B, Q, Hq, Hkv, n, d = 2, 3, 4, 2, 300, 8
    q = rng.standard_normal((B, Q, Hq, d))
    K = rng.standard_normal((B, Hkv, n, d))
    V = rng.standard_normal((B, Hkv, n, d))
    lens, seeds = np.array([300, 170]), np.array([21, 22], dtype=np.uint64)
    p = _params(sink=3, window=5, topk_abs=8, base_abs=24, sm_scale=0.35, epsilon=0.5, delta=0.5)
    res = vo.decode_chunk(q, K, V, lens, seeds, p)
    assert set(res) == {(b, t, h) for b in range(B) for t in range(Q) for h in range(Hq)}
    for (b, t, h), r in res.items():
        nt = int(lens[b]) - (Q - 1 - t)
        kv = [0, 0, 1, 1][h]
        one = vo.decode_head(q[b, t, h], K[b, kv, :nt], V[b, kv, :nt], seed=int(seeds[b]), head=h, params=p, query=t)
        for key in ("I_t", "I_bs", "I_dyn"):
            assert np.array_equal(r[key], one[key]), (b, t, h, key)
        assert np.array_equal(r["O"], one["O"])
        if t > 0:   # the position does change the draws
            zero = vo.decode_head(q[b, t, h], K[b, kv, :nt], V[b, kv, :nt], seed=int(seeds[b]), head=h, params=p)
            assert not np.array_equal(r["I_bs"], zero["I_bs"])


# ------------------------------------------------ Hoeffding-type budget ----
def test_hoeffding_budget_reproduces_the_ratio_the_paper_reports():
    rows = [l.split() for l in open(os.path.join(GOLDEN, "hoeffding_vs_clt_ratio.txt")) if l[0] != "#"]
    eps, delta, ratio = (float(x) for x in rows[0])
    st = dict(D_f=3.0, w_bar=0.01, sigma2=0.0004, D_hat=3.0 + 5000 * 0.01, tr_sigma=0.0, N_hat_sq=0.0)
    clt = vo.budget_raw(st, 5000, eps, delta, vo.TARGET_D)
    hoe = vo.budget_raw(st, 5000, eps, delta, vo.TARGET_D, bound="hoeffding")
    assert abs(hoe / clt - ratio) < 0.05          # the paper prints one decimal
    # the ratio does not depend on the data, only on delta
    st2 = dict(st, sigma2=0.09, D_hat=77.0)
    assert abs(vo.budget_raw(st2, 900, eps, delta, vo.TARGET_D, bound="hoeffding")
               / vo.budget_raw(st2, 900, eps, delta, vo.TARGET_D) - hoe / clt) < 1e-12


def test_hoeffding_factor_inverts_the_subgaussian_tail_and_dominates_the_normal_quantile():
    import scipy.stats
    for delta in (0.01, 0.05, 0.1, 0.2, 0.5):
        f = vo.hoeffding_factor(delta)
        # a normal variable exceeds f standard deviations (two-sided) with probability below delta: the
        # library's exact tail sits under the bound the factor comes from
        assert 2.0 * scipy.stats.norm.sf(f) < delta
        assert f > vo.upper_tail_quantile(delta / 2.0)
    with pytest.raises(ValueError):
        vo.budget_raw(dict(D_f=1.0, w_bar=0.1, sigma2=0.1, D_hat=2.0, tr_sigma=1.0, N_hat_sq=1.0), 10, 0.1, 0.1,
                      vo.TARGET_N, bound="hoeffding")


def test_hoeffding_budget_meets_the_guarantee_on_a_bounded_population():
    # residual weights uniform on [0, 1]: with the true sigma and D in the formula, a sample of ceil(b*)
    # tokens (without replacement) estimates D within eps in clearly more than a 1 - delta fraction of draws
    rng = np.random.default_rng(8)
    n_s, eps, delta = 4000, 0.02, 0.2
    w = rng.random(n_s)
    D_f = 50.0
    D = D_f + w.sum()
    st = dict(D_f=D_f, w_bar=float(w.mean()), sigma2=float(w.var(ddof=1)), D_hat=D, tr_sigma=0.0, N_hat_sq=0.0)
    b = int(math.ceil(vo.budget_raw(st, n_s, eps, delta, vo.TARGET_D, bound="hoeffding")))
    assert 2 <= b < n_s
    hits = 0
    trials = 2000
    for _ in range(trials):
        pick = rng.choice(n_s, size=b, replace=False)
        hits += abs(D_f + n_s / b * w[pick].sum() - D) <= eps * D
    assert hits / trials >= 1 - delta / 2


def test_range_based_hoeffding_budget_by_hand_and_against_the_inequality():
    # by hand: n_s = 1000, R = 0.2, D = 50, eps = 0.1, delta = 0.05:
    #   t = eps D / n_s = 0.005; b* = R^2 ln(2 / delta) / (2 t^2) = 0.04 * 3.688879454 / 0.00005 = 2951.1035...
    st = dict(D_f=10.0, w_bar=0.04, sigma2=123.0, D_hat=50.0, tr_sigma=0.0, N_hat_sq=0.0)
    b = vo.budget_raw(st, 1000, 0.1, 0.05, vo.TARGET_D, bound="hoeffding_range", w_range=0.2)
    assert b == pytest.approx(0.04 * math.log(40.0) / 0.00005, rel=1e-6)     # (eps, delta pass through fp32)
    # the variance plays no part, the range enters squared, D and eps inversely squared
    assert vo.budget_raw(dict(st, sigma2=0.0), 1000, 0.1, 0.05, vo.TARGET_D, bound="hoeffding_range", w_range=0.2) == b
    assert vo.budget_raw(st, 1000, 0.1, 0.05, vo.TARGET_D, bound="hoeffding_range", w_range=0.4) == pytest.approx(4 * b)
    assert vo.budget_raw(dict(st, D_hat=100.0), 1000, 0.1, 0.05, vo.TARGET_D, bound="hoeffding_range",
                         w_range=0.2) == pytest.approx(b / 4)
    assert vo.budget_raw(st, 2000, 0.1, 0.05, vo.TARGET_D, bound="hoeffding_range", w_range=0.2) == pytest.approx(4 * b)
    # inverting the inequality: with b = b* samples the bound 2 exp(-2 b t^2 / R^2) is exactly delta
    t = 0.1 * 50.0 / 1000
    assert 2.0 * math.exp(-2.0 * b * t * t / 0.04) == pytest.approx(0.05, rel=1e-6)
    # it is the conservative one: never below the CLT budget for weights inside the range (sigma <= R / 2)
    for sigma in (0.01, 0.05, 0.1):
        clt = vo.budget_raw(dict(st, sigma2=sigma ** 2), 1000, 0.1, 0.05, vo.TARGET_D)
        assert b > clt
    with pytest.raises(ValueError):
        vo.budget_raw(st, 1000, 0.1, 0.05, vo.TARGET_N, bound="hoeffding_range", w_range=0.2)
    with pytest.raises(ValueError):
        vo.budget_raw(st, 1000, 0.1, 0.05, vo.TARGET_D, bound="hoeffding_range")


def test_residual_weight_range_bounds_every_residual_weight():
    rng = np.random.default_rng(12)
    for trial in range(20):
        n = int(rng.integers(80, 400))
        s = rng.normal(0.0, 2.0, size=n)
        sink, window, k = int(rng.integers(0, 8)), int(rng.integers(0, 8)), int(rng.integers(0, 30))
        I_s, I_l, I_t, residual = vo.deterministic_set(s, sink, window, k)
        m = float(s.max())
        R = vo.residual_weight_range(s, m, I_t)
        w = np.exp(s[residual] - m)
        assert np.all(w <= R * (1 + 1e-15)) and np.all(w >= 0.0) and R <= 1.0
        if len(I_t):
            # tight: it is the weight of the weakest member of the top-k set, which the best residual token approaches
            assert R == pytest.approx(math.exp(s[I_t].min() - m))
        else:
            assert R == 1.0
    with pytest.raises(ValueError):
        vo.residual_weight_range(s, m, I_t, supplied=True)


def test_range_based_hoeffding_budget_holds_on_the_worst_population_for_its_range():
    # weights that are 0 or R, half each: the largest variance an interval of length R allows.  With R / t = 20
    # (t = eps D / n_s) the budget is (ln(2 / delta) / 2) * 400 = 599 of 3000 tokens, and a sample of that size
    # misses by more than eps D in well under delta of the draws (the inequality is not tight), while a quarter
    # of it misses far more often than delta: the budget has the right order of magnitude, from above.
    rng = np.random.default_rng(13)
    n_s, eps, delta, R = 3000, 0.05, 0.1, 0.05
    w = np.zeros(n_s)
    w[rng.choice(n_s, n_s // 2, replace=False)] = R
    D_f = 75.0
    D = D_f + w.sum()
    assert D == pytest.approx(150.0)
    st = dict(D_f=D_f, w_bar=float(w.mean()), sigma2=float(w.var(ddof=1)), D_hat=D, tr_sigma=0.0, N_hat_sq=0.0)
    b = int(math.ceil(vo.budget_raw(st, n_s, eps, delta, vo.TARGET_D, bound="hoeffding_range", w_range=R)))
    assert b == 600          # 599.15 with eps, delta taken through fp32

    def miss_rate(size, trials=3000):
        miss = 0
        for _ in range(trials):
            pick = rng.choice(n_s, size=size, replace=False)
            miss += abs(D_f + n_s / size * w[pick].sum() - D) > eps * D
        return miss / trials
    assert miss_rate(b) <= delta / 2
    assert miss_rate(b // 8) > delta


def test_decode_head_with_the_range_based_budget():
    rng = np.random.default_rng(14)
    n, d = 600, 8
    q = rng.standard_normal(d)
    K = rng.standard_normal((n, d)) * 0.5
    V = rng.standard_normal((n, d))
    p = dict(sink=4, window=8, topk_abs=20, topk_frac=0.0, base_abs=16, base_frac=0.0, epsilon=0.5, delta=0.1,
             target=vo.TARGET_D, sm_scale=1.0, budget_cap_frac=1.0, bound="hoeffding_range")
    r = vo.decode_head(q, K, V, seed=5, head=0, params=p)
    s = r["scores"]
    R = math.exp(s[r["I_t"]].min() - r["m"])
    want = 0.5 * math.log(2.0 / float(np.float32(0.1))) * (r["n_s"] * R / (float(np.float32(0.5)) * r["stats"]["D_hat"])) ** 2
    assert r["b_star"] == pytest.approx(want, rel=1e-12)
    assert r["b0"] < r["b"] < r["n_s"] and r["b"] == math.ceil(want)
    # same samples as the CLT run up to the budget: only the size of the final sample changes
    c = vo.decode_head(q, K, V, seed=5, head=0, params=dict(p, bound="clt"))
    assert np.array_equal(c["I_bs"], r["I_bs"]) and c["b_star"] < r["b_star"]
    with pytest.raises(ValueError):
        vo.decode_head(q, K, V, seed=5, head=0, params=p, forced_topk=r["I_t"])


def test_planted_mistakes_list_follows_the_oracle():
    # tests/plant_mistakes_in_oracle.py (run by hand) replaces pieces of the oracle's text by mistakes; every
    # piece it names has to occur in the oracle as it stands, or the check silently shrinks
    import plant_mistakes_in_oracle as pm
    assert pm.stale_patterns() == []
    assert len(pm.M) >= 95
