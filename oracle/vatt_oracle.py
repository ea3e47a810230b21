"""CPU oracle for the vAttention decode step.  TEST INFRASTRUCTURE ONLY.

A plain, slow, fp64 NumPy implementation of what one decode step computes for
one (sequence, query head): Algorithm 1 (vAttention) with Algorithm 2
(budget_X) inlined, in the paper's order and notation.  It exists to check the
HIP library; nothing in the product path may import it, and it imports
nothing from the product.  Only tests, the smoke check and the benchmark's
cpu_baseline leg call it.

Notation (Section 4.1): K, V in R^{n x d}, q in R^{1 x d};
s_i = sm_scale * <K[i], q>, w_i = exp(s_i - m) with m = max_i s_i (the shift
cancels in every ratio below), r_i = w_i V[i].  I_s, I_l, I_t are the sink,
local-window and top-k index sets, I_f their (disjoint) union, n_s the number
of residual tokens, I_bs the base sample and I_dyn the final sample, b its
size.

Pinned by tests/test_oracle_*.py against: the published Philox4x32-10
known-answer vectors, textbook normal quantiles, dense attention from library
routines (Eq. 1), brute-force enumeration of all samples on tiny inputs,
textbook simple-random-sampling variance, closed-form budgets on constructed
populations, and the (epsilon, delta) coverage of Definition 4.1.
One function is "parity unpinned": hoeffding_factor (the paper prints no formula for its Hoeffding-based
budget, only a ratio; the ratio is pinned, the form is a reading fitted to it).  Every other function is pinned,
including the range-based Hoeffding budget (bound = "hoeffding_range"), which is the textbook inequality.

Readings of the paper taken where it is silent (each also listed in the design
notes): softmax scale is an explicit factor sm_scale; sink / window are absolute
token counts; top-k is taken over the tokens outside sink and window, so the
three sets are disjoint and n_f is the sum of their sizes; sampling is without
replacement, by sequential uniform draws from the middle region that skip
top-k members and repeats (the paper only says "uniform sample"; the cost is
proportional to the sample, not to the context); the base sample holds floor(f_b * n_s) tokens (at least 2) and
sample variances divide by (b0 - 1); D and ||N|| in the budget formulas are
the full quantities D_f + residual estimate; the budget is ceil(b*), lower
capped by the base sample size and upper capped by n_s; I_dyn is a fresh draw
independent of I_bs; in a step with several query tokens every (query token,
head) is an independent instance on the causal prefix of that token; the
Hoeffding-type budget is the sub-Gaussian form that reproduces the sample ratio
the paper reports (hoeffding_factor: the formula is a reading, pinned by that
ratio and by the tail inequality it comes from); the random cache the paper
says the base sample can come from is a reservoir sample in random slot order
(random_cache_append).  Two options go beyond the paper and are off unless
asked for: nested samples (the final sample extends the base sample) and a
budget rounded up to a multiple (clamp_budget).
"""
from __future__ import annotations

import math
from itertools import combinations
from typing import Dict, List, Optional, Sequence

import numpy as np

TARGET_D = 0
TARGET_N = 1
TARGET_SDPA = 2

_M0 = 0xD2511F53
_M1 = 0xCD9E8D57
_W0 = 0x9E3779B9
_W1 = 0xBB67AE85
_MASK32 = 0xFFFFFFFF


# --------------------------------------------------------------------------
# Philox4x32-10 (Salmon, Moraes, Dror, Shaw: "Parallel random numbers: as easy
# as 1, 2, 3", SC'11).  Counter-based: output = bijection_key(counter).
# --------------------------------------------------------------------------
def philox4x32_10(ctr: Sequence, key: Sequence[int]) -> List[np.ndarray]:
    """Ten Philox-4x32 rounds.

    ctr: four uint32 arrays (or ints) of one shape; key: two Python ints.
    Each round multiplies words 0 and 2 by fixed odd constants, keeps the low
    halves and mixes the high halves with words 1, 3 and the round key; the
    key is advanced by the Weyl constants between rounds.
    """
    c0, c1, c2, c3 = (np.asarray(c, dtype=np.uint64) & np.uint64(_MASK32) for c in ctr)
    k0 = int(key[0]) & _MASK32
    k1 = int(key[1]) & _MASK32
    mask = np.uint64(_MASK32)
    sh = np.uint64(32)
    for _ in range(10):
        p0 = np.uint64(_M0) * c0
        p1 = np.uint64(_M1) * c2
        hi0, lo0 = p0 >> sh, p0 & mask
        hi1, lo1 = p1 >> sh, p1 & mask
        c0, c1, c2, c3 = hi1 ^ c1 ^ np.uint64(k0), lo1, hi0 ^ c3 ^ np.uint64(k1), lo0
        k0 = (k0 + _W0) & _MASK32
        k1 = (k1 + _W1) & _MASK32
    return [c.astype(np.uint32) for c in (c0, c1, c2, c3)]


def draw_words(j_lo: int, j_hi: int, seed: int, head: int, stream: int, query: int = 0) -> np.ndarray:
    """Words u_j, j in [j_lo, j_hi), of the sampler's draw sequence.

    Draw j reads word (j mod 4) of Philox4x32-10 applied to the counter
    (j div 4, stream, head, query) under the key (low 32 bits of seed, high 32
    bits of seed).  `head` is the query-head index, `stream` separates the base
    sample (0) from the final sample (1), `query` is the position of the query
    token inside a multi-query step (0 for single-token decoding).
    """
    b_lo, b_hi = j_lo // 4, (j_hi + 3) // 4
    nblk = max(b_hi - b_lo, 0)
    blk = np.arange(b_lo, b_lo + nblk, dtype=np.uint64)
    out = philox4x32_10(
        (blk, np.full(nblk, stream, np.uint64), np.full(nblk, head, np.uint64), np.full(nblk, query, np.uint64)),
        (int(seed) & _MASK32, (int(seed) >> 32) & _MASK32),
    )
    return np.stack(out, axis=1).reshape(-1)[j_lo - 4 * b_lo: j_hi - 4 * b_lo]


def bounded_draw(u, L: int, bits: int = 32):
    """Map uniform `bits`-bit words to [0, L) without bias (multiply-and-reject).

    With x = u * L, the value is the high part x >> bits; the word is rejected
    when the low part x mod 2^bits is below 2^bits mod L.  Every value of
    [0, L) then keeps exactly floor(2^bits / L) words, so an accepted value
    is exactly uniform.  Returns (accepted, value), arrays like u.
    """
    u = np.asarray(u, dtype=np.uint64)
    x = u * np.uint64(L)
    low = x & np.uint64((1 << bits) - 1)
    thr = (1 << bits) % int(L)
    return low >= np.uint64(thr), (x >> np.uint64(bits)).astype(np.int64)


def default_draw_cap(L: int) -> int:
    """Draws after which the sampler stops drawing and completes the sample in index order.

    With at least half of the residual still free, a draw is accepted with
    probability >= 1 / (2 L); 64 L draws then fail to deliver one token with
    probability about e^-32.  The cap only exists so that the procedure is finite.
    """
    return 64 * int(L) + 4096


def uniform_sample(residual: np.ndarray, c: int, *, mid_lo: int, mid_len: int, seed: int, head: int,
                   stream: int, draw_cap: Optional[int] = None, query: int = 0) -> np.ndarray:
    """uniform-sample of Algorithms 1 and 2: c residual tokens, uniformly, without replacement.

    Sequential draws: draw j proposes the token mid_lo + bounded_draw(u_j,
    mid_len) of the middle region (the tokens outside sink and window); it is
    accepted when the word is not rejected by bounded_draw, the token is a
    residual token (not in the top-k set) and it has not been accepted before.
    Drawing uniformly from the tokens not yet chosen, one at a time, is simple
    random sampling without replacement.

    c <= n_s / 2: the sample is the first c accepted tokens.
    c >  n_s / 2: the first n_s - c accepted tokens are left out and the
                  sample is the rest of the residual (the complement of a
                  uniform subset is a uniform subset), so that the number of
                  draws stays proportional to min(c, n_s - c).
    If `draw_cap` draws (default_draw_cap) do not suffice, the missing tokens
    are the lowest-index residual tokens not yet accepted.
    Returned in ascending index order.
    """
    residual = np.asarray(residual, dtype=np.int64)
    n_s = int(residual.shape[0])
    c = int(c)
    if c <= 0:
        return np.empty(0, dtype=np.int64)
    if c >= n_s:
        return residual.copy()
    invert = 2 * c > n_s
    want = n_s - c if invert else c
    cap = default_draw_cap(mid_len) if draw_cap is None else int(draw_cap)
    is_res = set(residual.tolist())
    chosen: List[int] = []
    chosen_set = set()
    j = 0
    while len(chosen) < want and j < cap:
        j_hi = min(j + 4096, cap)
        ok, val = bounded_draw(draw_words(j, j_hi, seed, head, stream, query), mid_len)
        for a, v in zip(ok.tolist(), val.tolist()):
            if not a:
                continue
            t = mid_lo + v
            if t in is_res and t not in chosen_set:
                chosen.append(t)
                chosen_set.add(t)
                if len(chosen) == want:
                    break
        j = j_hi
    if len(chosen) < want:
        rest = [t for t in residual.tolist() if t not in chosen_set]
        chosen.extend(rest[: want - len(chosen)])
    chosen_arr = np.asarray(chosen, dtype=np.int64)
    if invert:
        return np.setdiff1d(residual, chosen_arr)
    return np.sort(chosen_arr)


# --------------------------------------------------------------------------
# Normal quantile
# --------------------------------------------------------------------------
def upper_tail_quantile(t: float) -> float:
    """z with 1 - Phi(z) = t for the standard normal, by bisection on erfc(z / sqrt 2) / 2 = t.

    Working with the upper tail keeps Phi^{-1}(1 - delta/2) accurate for small delta,
    where 1 - delta/2 itself would lose digits.
    """
    if not (0.0 < t < 1.0):
        raise ValueError("t must be in (0, 1)")
    lo, hi = -40.0, 40.0
    for _ in range(200):
        mid = 0.5 * (lo + hi)
        if 0.5 * math.erfc(mid / math.sqrt(2.0)) > t:
            lo = mid
        else:
            hi = mid
    return 0.5 * (lo + hi)


def normal_quantile(p: float) -> float:
    """Phi^{-1}(p) for the standard normal."""
    if not (0.0 < p < 1.0):
        raise ValueError("p must be in (0, 1)")
    return -upper_tail_quantile(p) if p < 0.5 else upper_tail_quantile(1.0 - p)


# --------------------------------------------------------------------------
# Attention pieces
# --------------------------------------------------------------------------
def scores(q: np.ndarray, K: np.ndarray, sm_scale: float) -> np.ndarray:
    """s_i = sm_scale * <K[i], q> for all i (the exponent of Eq. 1), fp64."""
    return np.float64(sm_scale) * (np.asarray(K, np.float64) @ np.asarray(q, np.float64))


def dense_sdpa(q: np.ndarray, K: np.ndarray, V: np.ndarray, sm_scale: float):
    """Eq. 1: full softmax attention of one query over all n tokens.  Returns (O, lse)."""
    s = scores(q, K, sm_scale)
    m = s.max()
    w = np.exp(s - m)
    D = w.sum()
    N = w @ np.asarray(V, np.float64)
    return N / D, m + math.log(D)


def deterministic_set(s: np.ndarray, sink: int, window: int, k: int):
    """The deterministic index sets of Algorithm 1 (sink, local window, top-k) with oracle top-k.

    I_s = first `sink` tokens, I_l = last `window` tokens (not overlapping
    I_s), I_t = the k largest scores among the tokens in between (ties go to
    the lower index).  Returns (I_s, I_l, I_t ascending, residual ascending).
    """
    n = s.shape[0]
    ns_ = min(int(sink), n)
    nl_ = min(int(window), n - ns_)
    I_s = np.arange(0, ns_, dtype=np.int64)
    I_l = np.arange(n - nl_, n, dtype=np.int64)
    mid = np.arange(ns_, n - nl_, dtype=np.int64)
    kk = min(max(int(k), 0), mid.shape[0])
    if kk > 0:
        order = np.lexsort((mid, -s[mid]))  # descending score, ties by lower index
        I_t = np.sort(mid[order[:kk]])
    else:
        I_t = np.empty(0, dtype=np.int64)
    member = np.zeros(n, dtype=bool)
    member[I_t] = True
    residual = mid[~member[mid]]
    return I_s, I_l, I_t, residual


def topk_count(n: int, sink: int, window: int, topk_abs: int, topk_frac: float) -> int:
    """k = topk_abs if positive else floor(f_t * n)  (Algorithm 1's f_t n, rounded down)."""
    if topk_abs > 0:
        return int(topk_abs)
    return int(math.floor(np.float64(np.float32(topk_frac)) * n))


def base_count(n_s: int, base_abs: int, base_frac: float) -> int:
    """b0' = min(max(b0, 2), n_s) with b0 = base_abs if positive else floor(f_b * n_s)."""
    b0 = int(base_abs) if base_abs > 0 else int(math.floor(np.float64(np.float32(base_frac)) * n_s))
    return min(max(b0, 2), int(n_s))


def sample_stats(s: np.ndarray, V: Optional[np.ndarray], m: float, I_f: np.ndarray,
                 I_bs: np.ndarray, n_s: int, need_num: bool) -> Dict[str, float]:
    """get-stats / compute-stats of Algorithm 2.

    D_f, N_f are exact sums over I_f.  From the base sample: mean and unbiased
    variance of w (sigma^2), mean vector of r and the trace of its unbiased
    covariance estimate (Tr Sigma).  D_hat = D_f + n_s * mean(w),
    N_hat = N_f + n_s * mean(r).
    """
    w_f = np.exp(s[I_f] - m)
    D_f = float(w_f.sum())
    b0 = int(I_bs.shape[0])
    w_b = np.exp(s[I_bs] - m)
    w_bar = float(w_b.mean()) if b0 > 0 else 0.0
    sigma2 = float(((w_b - w_bar) ** 2).sum() / (b0 - 1)) if b0 > 1 else 0.0
    out = dict(D_f=D_f, w_bar=w_bar, sigma2=sigma2, D_hat=D_f + n_s * w_bar,
               tr_sigma=0.0, N_hat_sq=0.0)
    if need_num:
        V64 = np.asarray(V, np.float64)
        N_f = w_f @ V64[I_f]
        r_b = w_b[:, None] * V64[I_bs]
        r_bar = r_b.mean(axis=0) if b0 > 0 else np.zeros(V64.shape[1])
        tr = float(((r_b - r_bar[None, :]) ** 2).sum() / (b0 - 1)) if b0 > 1 else 0.0
        N_hat = N_f + n_s * r_bar
        out.update(tr_sigma=tr, N_hat_sq=float(N_hat @ N_hat))
    return out


def hoeffding_factor(delta: float) -> float:
    """What takes the place of the normal quantile in the conservative (Hoeffding-type) denominator budget.

    The appendix on the tightness of the bounds compares the CLT budget with a budget from Hoeffding's
    inequality and prints no formula, only that it asks for 2.8 times the samples at delta = 0.2.  The
    sub-Gaussian form of the inequality, P(|mean - mu| >= t) <= 2 exp(-b t^2 / (2 sigma^2)), gives
    b >= 2 ln(2 / delta) (n_s sigma / (eps D))^2: the CLT budget with Phi^{-1}(1 - delta/2)^2 replaced by
    2 ln(2 / delta), a ratio of 2.80 at delta = 0.2.  That reading is taken; this returns sqrt(2 ln(2 / delta)).

    Parity unpinned beyond that ratio: the form is fitted to the one printed number.  It uses the sample
    variance where Hoeffding's inequality proper uses the range of the weights, so it has no distribution-free
    finite-sample guarantee (the range-based form would ask for far more than 2.8 times the CLT budget).
    """
    return math.sqrt(2.0 * math.log(2.0 / float(delta)))


def residual_weight_range(s: np.ndarray, m: float, I_t: np.ndarray, supplied: bool = False) -> float:
    """An interval length that holds every residual weight w_i = exp(s_i - m), known without looking at them.

    Every residual token scores at most the smallest score of the exact top-k set, so its weight lies in
    [0, exp(min_{I_t} s - m)].  Without a top-k set (k = 0) only w <= 1 is known.  A top-k set supplied by the
    caller bounds nothing (a residual token may outscore it), so the range is undefined there.
    """
    if supplied:
        raise ValueError("a caller-supplied top-k set does not bound the residual weights")
    if len(I_t) == 0:
        return 1.0
    return float(math.exp(float(np.min(s[I_t])) - m))


def budget_raw(stats: Dict[str, float], n_s: int, epsilon: float, delta: float, target: int,
               bound: str = "clt", w_range: Optional[float] = None) -> float:
    """b* of Algorithm 2.

    Denominator (Corollary for D):  b* = (Phi^{-1}(1 - delta/2) * n_s * sigma / (eps * D))^2.
    Numerator   (Corollary for N):  same with sqrt(Tr Sigma) and ||N||_2.
    SDPA (Theorem 4.3): the minimisation over (eps', delta') is taken at
    delta' = delta/2, where max(b_D(eps'/2), b_N((eps - eps')/2)) is smallest
    when the two are equal: eps' = eps * rho_D / (rho_D + rho_N), giving
    b* = (2 * Phi^{-1}(1 - delta/4) * (rho_D + rho_N) / eps)^2.  That choice is
    a feasible point of the theorem's minimum, so its guarantee applies.

    bound = "hoeffding_range" (denominator target): Hoeffding's inequality proper, which also holds for
    sampling without replacement: for weights in an interval of length R, P(|mean - mu| >= t) <=
    2 exp(-2 b t^2 / R^2); the estimate n_s * mean misses the residual mass by at most eps * D when
    t = eps * D / n_s, so b* = (ln(2 / delta) / 2) * (n_s * R / (eps * D))^2 with D the full estimate D_hat.
    It needs no variance and holds for every distribution of the weights; w_range = R.
    """
    eps = float(np.float64(np.float32(epsilon)))
    dlt = float(np.float64(np.float32(delta)))
    if bound == "hoeffding_range":
        if target != TARGET_D:
            raise ValueError("the Hoeffding budget is defined for the denominator target only")
        if w_range is None:
            raise ValueError("the range of the residual weights is needed")
        return 0.5 * math.log(2.0 / dlt) * (n_s * float(w_range) / (eps * stats["D_hat"])) ** 2
    rho_D = n_s * math.sqrt(stats["sigma2"]) / stats["D_hat"]
    if bound == "hoeffding":
        if target != TARGET_D:
            raise ValueError("the Hoeffding-type budget is defined for the denominator target only")
        return (hoeffding_factor(dlt) * rho_D / eps) ** 2
    if bound != "clt":
        raise ValueError("unknown bound")
    if target == TARGET_D:
        return (upper_tail_quantile(dlt / 2.0) * rho_D / eps) ** 2
    nn = math.sqrt(stats["N_hat_sq"])
    num = n_s * math.sqrt(stats["tr_sigma"])
    rho_N = (num / nn) if nn > 0.0 else (math.inf if num > 0.0 else 0.0)
    if target == TARGET_N:
        return (upper_tail_quantile(dlt / 2.0) * rho_N / eps) ** 2
    if target == TARGET_SDPA:
        return (2.0 * upper_tail_quantile(dlt / 4.0) * (rho_D + rho_N) / eps) ** 2
    raise ValueError("unknown target")


def clamp_budget(b_star: float, b0: int, n_s: int, cap_frac: float, multiple: int = 1) -> int:
    """b = min(n_s, max(b0', min(ceil(b*), ceil(cap_frac * n_s)))).

    The budget is lower capped by the base sample size (as the paper does in
    its experiments) and cannot exceed the residual count when sampling
    without replacement.  cap_frac = 1 leaves it uncapped.

    multiple > 1 (an option beyond the paper, for hardware that reads rows in
    groups): b is then rounded up to the next multiple of `multiple`, but not
    beyond min(n_s, max(b0', ceil(cap_frac * n_s))), the largest value the rule
    above can give.  Rounding up only adds samples, so the guarantee stands.
    """
    cap = int(math.ceil(np.float64(np.float32(cap_frac)) * n_s))
    if not math.isfinite(b_star) or b_star >= n_s:
        want = n_s
    else:
        want = int(math.ceil(b_star))
    b = int(min(n_s, max(b0, min(want, cap))))
    q = int(multiple)
    if q > 1:
        top = int(min(n_s, max(b0, cap)))
        b = min(top, (b + q - 1) // q * q)
    return b


def estimate(s: np.ndarray, V: np.ndarray, m: float, I_f: np.ndarray, I_dyn: np.ndarray, n_s: int):
    """N and D of Section 4.1 for given index sets: exact over I_f plus (n_s/b) * sampled sums.

    Returns (N_hat, D_hat) in the e^{-m}-shifted scale.  With b = 0 the sampled
    part is absent (Eq. 2).
    """
    V64 = np.asarray(V, np.float64)
    w_f = np.exp(s[I_f] - m)
    D = float(w_f.sum())
    N = w_f @ V64[I_f]
    b = int(I_dyn.shape[0])
    if b > 0:
        w_d = np.exp(s[I_dyn] - m)
        scale = n_s / b
        D = D + scale * float(w_d.sum())
        N = N + scale * (w_d @ V64[I_dyn])
    return N, D


def decode_head(q: np.ndarray, K: np.ndarray, V: np.ndarray, *, seed: int, head: int,
                params: Dict[str, float], s: Optional[np.ndarray] = None,
                forced_topk: Optional[np.ndarray] = None,
                forced_b: Optional[int] = None, query: int = 0,
                cache_tokens: Optional[Sequence[int]] = None) -> Dict[str, object]:
    """Algorithm 1 for one (sequence, query head).

    cache_tokens: the random cache of the head's (sequence, KV head) in slot order; the base sample is then
    taken from it (base_sample_from_cache) when it holds enough residual tokens.

    q: [d], K, V: [n, d] (values already rounded to the storage precision).
    `s` may carry precomputed scores of the same inputs.  forced_topk /
    forced_b replace the top-k set / the budget by a caller-chosen legal
    alternative (see topk_alternatives, budget_alternatives) and recompute
    everything downstream; they are never taken from another implementation's
    output.
    """
    n = K.shape[0]
    sm_scale = float(params["sm_scale"])
    target = int(params.get("target", TARGET_D))
    if s is None:
        s = scores(q, K, sm_scale)
    m = float(s.max())
    k = topk_count(n, int(params["sink"]), int(params["window"]),
                   int(params.get("topk_abs", 0)), float(params.get("topk_frac", 0.0)))
    I_s, I_l, I_t, residual = deterministic_set(s, int(params["sink"]), int(params["window"]), k)
    if forced_topk is not None:
        I_t = np.sort(np.asarray(forced_topk, dtype=np.int64))
        mid = np.arange(I_s.shape[0], n - I_l.shape[0], dtype=np.int64)
        member = np.zeros(n, dtype=bool)
        member[I_t] = True
        residual = mid[~member[mid]]
    I_f = np.concatenate([I_s, I_l, I_t])
    n_s = int(residual.shape[0])
    res: Dict[str, object] = dict(n=n, m=m, I_s=I_s, I_l=I_l, I_t=I_t, n_s=n_s, scores=s)
    if n_s == 0:
        N, D = estimate(s, V, m, I_f, np.empty(0, np.int64), 0)
        res.update(I_bs=np.empty(0, np.int64), I_dyn=np.empty(0, np.int64), b0=0, b=0,
                   b_star=0.0, stats=dict(D_f=D, w_bar=0.0, sigma2=0.0, D_hat=D, tr_sigma=0.0, N_hat_sq=0.0),
                   O=N / D, lse=m + math.log(D), D_out=D, N_out=N)
        return res
    b0 = base_count(n_s, int(params.get("base_abs", 0)), float(params.get("base_frac", 0.0)))
    mid_lo, mid_len = int(I_s.shape[0]), n - int(I_s.shape[0]) - int(I_l.shape[0])
    draw_cap = params.get("draw_cap")
    I_bs = base_sample_from_cache(cache_tokens, residual, b0) if cache_tokens is not None else None
    base_from_cache = I_bs is not None
    if I_bs is None:
        I_bs = uniform_sample(residual, b0, mid_lo=mid_lo, mid_len=mid_len, seed=seed, head=head, stream=0,
                              draw_cap=draw_cap, query=query)
    st = sample_stats(s, V, m, I_f, I_bs, n_s, need_num=(target != TARGET_D))
    bound = str(params.get("bound", "clt"))
    b_star = budget_raw(st, n_s, float(params["epsilon"]), float(params["delta"]), target, bound=bound,
                        w_range=residual_weight_range(s, m, I_t, forced_topk is not None) if bound == "hoeffding_range" else None)
    b = clamp_budget(b_star, b0, n_s, float(params.get("budget_cap_frac", 1.0)),
                     int(params.get("budget_multiple", 1)))
    if forced_b is not None:
        b = int(forced_b)
    if params.get("nested"):
        # Nested samples (not the paper's Algorithm 1, which draws I_dyn afresh): the base sample is kept and
        # b - b0 further tokens are drawn, with the second draw sequence, from the residual tokens outside it.
        # A uniform b0-subset plus a uniform (b - b0)-subset of the rest is a uniform b-subset for fixed b;
        # b itself was computed from the base sample, which is where a (small) bias can enter.
        rest = np.setdiff1d(residual, I_bs, assume_unique=True)
        extra = uniform_sample(rest, b - b0, mid_lo=mid_lo, mid_len=mid_len, seed=seed, head=head, stream=1,
                               draw_cap=draw_cap, query=query)
        I_dyn = np.sort(np.concatenate([I_bs, extra]))
    else:
        I_dyn = uniform_sample(residual, b, mid_lo=mid_lo, mid_len=mid_len, seed=seed, head=head, stream=1,
                               draw_cap=draw_cap, query=query)
    N, D = estimate(s, V, m, I_f, I_dyn, n_s)
    res.update(I_bs=I_bs, I_dyn=I_dyn, b0=b0, b=b, b_star=b_star, stats=st, base_from_cache=base_from_cache,
               O=N / D, lse=m + math.log(D), D_out=D, N_out=N)
    return res


# --------------------------------------------------------------------------
# Random cache of base-sample tokens.  The paper's implementation note after Theorem 4.3 says that the base
# sample can be served from a small random cache that is populated and updated during generation; it gives
# no procedure.  Reading taken here: per (sequence, KV head) a cache of C slots holds a uniform random C-subset
# of the tokens seen so far, in uniformly random slot order, maintained by reservoir sampling as tokens
# arrive; the base sample of a query head is then the first b0 cached tokens, in slot order, that are
# residual tokens of that head (not in I_s, I_l, I_t).  A uniform random subset in random order, filtered by
# a condition that does not depend on the order, yields a uniform b0-subset of the residual.  When the
# cache holds fewer than b0 residual tokens the base sample is drawn by the sampler as without a cache.
# --------------------------------------------------------------------------
CACHE_STREAM = 2


def cache_words(t_lo: int, t_hi: int, seed: int, kv_head: int) -> np.ndarray:
    """Rows t_lo .. t_hi-1: the four words of Philox4x32-10(counter = (t, CACHE_STREAM, kv_head, 0), key = halves of seed)."""
    t = np.arange(int(t_lo), int(t_hi), dtype=np.uint64) & np.uint64(_MASK32)
    w = philox4x32_10((t, np.full(t.size, CACHE_STREAM, np.uint64), np.full(t.size, kv_head, np.uint64),
                       np.full(t.size, 0, np.uint64)),
                      (int(seed) & _MASK32, (int(seed) >> 32) & _MASK32))
    return np.stack([np.asarray(x, dtype=np.uint64) for x in w], axis=1)


def cache_draw(words4, R: int) -> int:
    """Uniform integer in [0, R) from the four words of one token's arrival.

    Each word is mapped by the unbiased multiply-and-reject rule; the first accepted one counts, and the
    fourth is taken whether accepted or not (probability below (R / 2^32)^3 per draw).
    """
    ok, val = bounded_draw(np.asarray(words4, dtype=np.uint64), int(R))
    for a, v in zip(ok, val):
        if bool(a):
            return int(v)
    return int(val[-1])


def random_cache_append(slots: List[int], C: int, t: int, seed: int, kv_head: int, words4=None) -> None:
    """Token t (the t-th token of the sequence, counted from 0) arrives; `slots` is the cache in slot order.

    While the cache is not full, t is inserted at a uniformly random place of the t + 1 entries (the entry
    that was there moves to the end): the entries stay in uniformly random order.  Once it is full, t
    replaces slot r when r, uniform in [0, t], falls below C (reservoir sampling: every C-subset of the
    t + 1 tokens is then equally likely, and the slot order stays exchangeable).
    """
    if words4 is None:
        words4 = cache_words(t, t + 1, seed, kv_head)[0]
    c = len(slots)
    if c < C:
        j = cache_draw(words4, c + 1)
        if j == c:
            slots.append(int(t))
        else:
            slots.append(slots[j])
            slots[j] = int(t)
    else:
        r = cache_draw(words4, t + 1)
        if r < C:
            slots[r] = int(t)


def random_cache_fill(n: int, C: int, seed: int, kv_head: int) -> List[int]:
    """The cache after tokens 0 .. n-1 have arrived one by one."""
    slots: List[int] = []
    words = cache_words(0, n, seed, kv_head)
    for t in range(int(n)):
        random_cache_append(slots, C, t, seed, kv_head, words[t])
    return slots


def base_sample_from_cache(cache_tokens: Sequence[int], residual: np.ndarray, b0: int) -> Optional[np.ndarray]:
    """First b0 cached tokens, in slot order, that are residual tokens; None when the cache has fewer."""
    is_res = set(int(x) for x in residual)
    got = [int(t) for t in cache_tokens if int(t) in is_res][:int(b0)]
    if len(got) < int(b0):
        return None
    return np.sort(np.asarray(got, dtype=np.int64))


# --------------------------------------------------------------------------
# Legal alternatives where floating point decides an integer
# --------------------------------------------------------------------------
def topk_alternatives(s: np.ndarray, sink: int, window: int, k: int, rel_tol: float = 1e-5,
                      limit: int = 256) -> List[np.ndarray]:
    """All top-k sets that differ from the oracle's only by swaps among near-tied scores.

    A score is "near-tied" with the k-th largest score tau when
    |s_i - tau| <= rel_tol * max(|s_i|, |tau|).  Tokens clearly above tau are in
    every legal set, tokens clearly below in none; the near-tied ones may be
    chosen in any combination that fills the set to k.  The oracle's own
    choice comes first.  Raises if there are more than `limit` combinations.
    """
    n = s.shape[0]
    I_s, I_l, I_t, _ = deterministic_set(s, sink, window, k)
    if I_t.shape[0] == 0:
        return [I_t]
    mid = np.arange(I_s.shape[0], n - I_l.shape[0], dtype=np.int64)
    if I_t.shape[0] == mid.shape[0]:
        return [I_t]
    tau = s[I_t].min()
    near = np.abs(s[mid] - tau) <= rel_tol * np.maximum(np.abs(s[mid]), abs(tau))
    amb = mid[near]
    sel = np.zeros(n, dtype=bool)
    sel[I_t] = True
    sure = I_t[~np.isin(I_t, amb)]
    need = I_t.shape[0] - sure.shape[0]
    # tokens above tau but outside the tolerance band are "sure"; ambiguous ones not selected lie below
    if math.comb(amb.shape[0], need) > limit:
        raise RuntimeError("too many near-tied top-k alternatives")
    alts = [I_t]
    for combo in combinations(amb.tolist(), need):
        cand = np.sort(np.concatenate([sure, np.asarray(combo, dtype=np.int64)]))
        if not np.array_equal(cand, I_t):
            alts.append(cand)
    return alts


def budget_alternatives(b_star: float, b0: int, n_s: int, cap_frac: float, rel_tol: float = 1e-6,
                        multiple: int = 1) -> List[int]:
    """Budgets a correct fp32-statistics implementation may reach: the clamped ceil(b') of every b' within
    rel_tol (relative) of b*, the oracle's own budget first.  The window is 1e-6: b* is a ratio of sums of
    some hundreds of fp32 weights whose individual relative errors (about 1e-6 from the fp32 score and the
    fp32 exponential) are independent, so the sums agree with the fp64 ones to well under 1e-6; a budget is
    bit-exact unless b* lies that close to an integer."""
    own = clamp_budget(b_star, b0, n_s, cap_frac, multiple)
    if not math.isfinite(b_star):
        return [own]
    lo = clamp_budget(b_star * (1.0 - rel_tol), b0, n_s, cap_frac)
    hi = clamp_budget(b_star * (1.0 + rel_tol), b0, n_s, cap_frac)
    out = [own]
    for v in range(min(lo, hi), max(lo, hi) + 1):        # every ceil(b') in the range, then the same rounding
        w = clamp_budget(float(v), b0, n_s, cap_frac, multiple)
        if w not in out:
            out.append(w)
    return out


# --------------------------------------------------------------------------
# Whole-batch driver
# --------------------------------------------------------------------------
def decode(q: np.ndarray, K: np.ndarray, V: np.ndarray, seq_lens: np.ndarray, seeds: np.ndarray,
           params: Dict[str, float], heads: Optional[Sequence] = None) -> Dict[tuple, Dict[str, object]]:
    """One decode step for a batch: q [B, Hq, d], K, V [B, Hkv, n_max, d] (fp32/fp64 values).

    Query head h reads KV head h // (Hq / Hkv).  Returns {(b, h): decode_head result}.
    `heads` restricts the (b, h) pairs computed.
    """
    B, Hq, _ = q.shape
    Hkv = K.shape[1]
    g = Hq // Hkv
    out = {}
    pairs = heads if heads is not None else [(b, h) for b in range(B) for h in range(Hq)]
    for (b, h) in pairs:
        n = int(seq_lens[b])
        out[(b, h)] = decode_head(q[b, h], K[b, h // g, :n], V[b, h // g, :n],
                                  seed=int(seeds[b]), head=h, params=params)
    return out


def chunk_length(n: int, q_len: int, t: int) -> int:
    """Tokens visible to query t of a step that processes the q_len newest tokens of an n-token sequence.

    The queries are the tokens at positions n - q_len .. n - 1, in this order; attention is causal, so query t
    (at position n - q_len + t) sees the tokens up to and including itself.
    """
    return max(int(n) - (int(q_len) - 1 - int(t)), 0)


def decode_chunk(q: np.ndarray, K: np.ndarray, V: np.ndarray, seq_lens: np.ndarray, seeds: np.ndarray,
                 params: Dict[str, float], items: Optional[Sequence] = None) -> Dict[tuple, Dict[str, object]]:
    """A step with several query tokens per sequence (the question tokens of the evaluation set-up, where the
    context is processed densely and question and generation sparsely): q [B, Q, Hq, d]; K, V [B, Hkv, n_max, d]
    already hold the Q newest tokens; seq_lens counts them.

    Every (query token, query head) is one instance of Algorithm 1 over the tokens that query may see
    (chunk_length), with its own top-k set, samples and budget; the draw sequences of different query tokens
    differ in the last counter word.  Returns {(b, t, h): decode_head result}; `items` restricts the triples.
    """
    B, Q, Hq, _ = q.shape
    Hkv = K.shape[1]
    g = Hq // Hkv
    out = {}
    todo = items if items is not None else [(b, t, h) for b in range(B) for t in range(Q) for h in range(Hq)]
    for (b, t, h) in todo:
        n = chunk_length(int(seq_lens[b]), Q, t)
        out[(b, t, h)] = decode_head(q[b, t, h], K[b, h // g, :n], V[b, h // g, :n],
                                     seed=int(seeds[b]), head=h, params=params, query=t)
    return out
