"""Plants one mistake at a time in a temporary copy of the oracle and runs the CPU pins against the copy.

    python tests/plant_mistakes_in_oracle.py [name-fragment]

Every entry of M replaces one piece of oracle/vatt_oracle.py by a plausible mistake (a dropped term, a wrong
sign or index, swapped arguments, a wrong constant).  The copy, with tests/ and workloads/, goes to a temporary
directory, and tests/test_oracle_pins.py and tests/test_oracle_statistics.py run there: a mistake is caught when
they fail.  Prints one line per mistake and exits with status 1 if one is not caught (entries in EQUIVALENT
change nothing that can be observed and are expected to pass); an entry whose text no longer occurs in the
oracle stops the run (tests/test_oracle_pins.py checks the list against the oracle on every CPU run).  CPU only; about five minutes on eight cores.
Not collected by pytest (it would multiply the suite's run time); run by hand after changing the oracle or
its pins.
"""
import os, shutil, subprocess, sys, tempfile
from concurrent.futures import ThreadPoolExecutor
ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
# min(n_s, .) around operands that are each at most n_s already
EQUIVALENT = {"clamp no upper"}
SRC = open(os.path.join(ROOT, "oracle/vatt_oracle.py")).read()
M = [
 ("philox swap mult", "p0 = np.uint64(_M0) * c0\n        p1 = np.uint64(_M1) * c2", "p0 = np.uint64(_M1) * c0\n        p1 = np.uint64(_M0) * c2"),
 ("philox 9 rounds", "for _ in range(10):", "for _ in range(9):"),
 ("philox key order", "hi1 ^ c1 ^ np.uint64(k0), lo1, hi0 ^ c3 ^ np.uint64(k1), lo0", "hi1 ^ c1 ^ np.uint64(k1), lo1, hi0 ^ c3 ^ np.uint64(k0), lo0"),
 ("philox weyl", "k1 = (k1 + _W1) & _MASK32", "k1 = (k1 + _W0) & _MASK32"),
 ("counter order head/stream", "(blk, np.full(nblk, stream, np.uint64), np.full(nblk, head, np.uint64), np.full(nblk, query, np.uint64))", "(blk, np.full(nblk, head, np.uint64), np.full(nblk, stream, np.uint64), np.full(nblk, query, np.uint64))"),
 ("query word dropped", "np.full(nblk, query, np.uint64)),", "np.full(nblk, 0, np.uint64)),"),
 ("seed halves swapped", "(int(seed) & _MASK32, (int(seed) >> 32) & _MASK32)", "((int(seed) >> 32) & _MASK32, int(seed) & _MASK32)"),
 ("reject test dropped", "return low >= np.uint64(thr), (x >> np.uint64(bits)).astype(np.int64)", "return low >= np.uint64(0), (x >> np.uint64(bits)).astype(np.int64)"),
 ("modulo mapping", "(x >> np.uint64(bits)).astype(np.int64)", "(u % np.uint64(L)).astype(np.int64)"),
 ("sample with repeats", "if t in is_res and t not in chosen_set:", "if t in is_res:"),
 ("sample ignores top-k", "if t in is_res and t not in chosen_set:", "if t not in chosen_set:"),
 ("complement off by one", "want = n_s - c if invert else c", "want = n_s - c + 1 if invert else c"),
 ("complement not inverted", "    if invert:\n        return np.setdiff1d(residual, chosen_arr)", "    if False:\n        return np.setdiff1d(residual, chosen_arr)"),
 ("mid_lo dropped", "t = mid_lo + v", "t = v"),
 ("quantile wrong tail", "if 0.5 * math.erfc(mid / math.sqrt(2.0)) > t:", "if 0.5 * math.erfc(mid / 2.0) > t:"),
 ("scores transposed scale", "return np.float64(sm_scale) * (np.asarray(K, np.float64) @ np.asarray(q, np.float64))", "return (np.asarray(K, np.float64) @ np.asarray(q, np.float64))"),
 ("dense no shift sign", "w = np.exp(s - m)\n    D = w.sum()", "w = np.exp(m - s)\n    D = w.sum()"),
 ("topk smallest", "order = np.lexsort((mid, -s[mid]))", "order = np.lexsort((mid, s[mid]))"),
 ("topk ties high index", "order = np.lexsort((mid, -s[mid]))", "order = np.lexsort((-mid, -s[mid]))"),
 ("window overlaps", "I_l = np.arange(n - nl_, n, dtype=np.int64)", "I_l = np.arange(n - nl_ - 1, n - 1, dtype=np.int64)"),
 ("topk over whole row", "mid = np.arange(ns_, n - nl_, dtype=np.int64)\n    kk", "mid = np.arange(0, n, dtype=np.int64)\n    kk"),
 ("base count min 1", "return min(max(b0, 2), int(n_s))", "return min(max(b0, 1), int(n_s))"),
 ("base frac of n ceil", "int(math.floor(np.float64(np.float32(base_frac)) * n_s))", "int(math.ceil(np.float64(np.float32(base_frac)) * n_s))"),
 ("variance biased", "sigma2 = float(((w_b - w_bar) ** 2).sum() / (b0 - 1)) if b0 > 1 else 0.0", "sigma2 = float(((w_b - w_bar) ** 2).sum() / b0) if b0 > 1 else 0.0"),
 ("D_hat without D_f", "D_hat=D_f + n_s * w_bar,", "D_hat=n_s * w_bar,"),
 ("D_hat scaled by b0", "D_hat=D_f + n_s * w_bar,", "D_hat=D_f + b0 * w_bar,"),
 ("trace biased", "tr = float(((r_b - r_bar[None, :]) ** 2).sum() / (b0 - 1)) if b0 > 1 else 0.0", "tr = float(((r_b - r_bar[None, :]) ** 2).sum() / b0) if b0 > 1 else 0.0"),
 ("trace not centred", "tr = float(((r_b - r_bar[None, :]) ** 2).sum() / (b0 - 1))", "tr = float(((r_b) ** 2).sum() / (b0 - 1))"),
 ("N_hat without N_f", "N_hat = N_f + n_s * r_bar", "N_hat = n_s * r_bar"),
 ("rho_D variance not sqrt", 'rho_D = n_s * math.sqrt(stats["sigma2"]) / stats["D_hat"]', 'rho_D = n_s * stats["sigma2"] / stats["D_hat"]'),
 ("rho_D no n_s", 'rho_D = n_s * math.sqrt(stats["sigma2"]) / stats["D_hat"]', 'rho_D = math.sqrt(stats["sigma2"]) / stats["D_hat"]'),
 ("budget D one-sided", "if target == TARGET_D:\n        return (upper_tail_quantile(dlt / 2.0) * rho_D / eps) ** 2", "if target == TARGET_D:\n        return (upper_tail_quantile(dlt) * rho_D / eps) ** 2"),
 ("budget not squared", "if target == TARGET_D:\n        return (upper_tail_quantile(dlt / 2.0) * rho_D / eps) ** 2", "if target == TARGET_D:\n        return (upper_tail_quantile(dlt / 2.0) * rho_D / eps)"),
 ("budget N uses rho_D", "return (upper_tail_quantile(dlt / 2.0) * rho_N / eps) ** 2", "return (upper_tail_quantile(dlt / 2.0) * rho_D / eps) ** 2"),
 ("rho_N norm squared", 'nn = math.sqrt(stats["N_hat_sq"])', 'nn = stats["N_hat_sq"]'),
 ("sdpa factor 2 dropped", "return (2.0 * upper_tail_quantile(dlt / 4.0) * (rho_D + rho_N) / eps) ** 2", "return (upper_tail_quantile(dlt / 4.0) * (rho_D + rho_N) / eps) ** 2"),
 ("sdpa delta/2", "return (2.0 * upper_tail_quantile(dlt / 4.0) * (rho_D + rho_N) / eps) ** 2", "return (2.0 * upper_tail_quantile(dlt / 2.0) * (rho_D + rho_N) / eps) ** 2"),
 ("sdpa max instead of sum", "(rho_D + rho_N) / eps) ** 2", "max(rho_D, rho_N) / eps) ** 2"),
 ("hoeffding ln(1/delta)", "return math.sqrt(2.0 * math.log(2.0 / float(delta)))", "return math.sqrt(2.0 * math.log(1.0 / float(delta)))"),
 ("clamp floor", "want = int(math.ceil(b_star))", "want = int(math.floor(b_star))"),
 ("clamp no lower cap", "b = int(min(n_s, max(b0, min(want, cap))))", "b = int(min(n_s, min(want, cap)))"),
 ("clamp no upper", "b = int(min(n_s, max(b0, min(want, cap))))", "b = int(max(b0, min(want, cap)))"),
 ("multiple rounds down", "b = min(top, (b + q - 1) // q * q)", "b = min(top, b // q * q)"),
 ("multiple beyond the residual", "b = min(top, (b + q - 1) // q * q)", "b = (b + q - 1) // q * q"),
 ("multiple ignores the lower cap", "top = int(min(n_s, max(b0, cap)))", "top = int(min(n_s, cap))"),
 ("estimate scale b/n_s", "scale = n_s / b\n", "scale = b / n_s\n"),
 ("estimate scale missing in N", "N = N + scale * (w_d @ V64[I_dyn])", "N = N + (w_d @ V64[I_dyn])"),
 ("estimate scale missing in D", "D = D + scale * float(w_d.sum())", "D = D + float(w_d.sum())"),
 ("final sample same stream", "I_dyn = uniform_sample(residual, b, mid_lo=mid_lo, mid_len=mid_len, seed=seed, head=head, stream=1,", "I_dyn = uniform_sample(residual, b, mid_lo=mid_lo, mid_len=mid_len, seed=seed, head=head, stream=0,"),
 ("final sample size b0", "I_dyn = uniform_sample(residual, b, mid_lo", "I_dyn = uniform_sample(residual, b0, mid_lo"),
 ("lse without m", "               O=N / D, lse=m + math.log(D), D_out=D, N_out=N)\n    return res\n\n\n# ---", "               O=N / D, lse=math.log(D), D_out=D, N_out=N)\n    return res\n\n\n# ---"),
 ("I_f misses window", "I_f = np.concatenate([I_s, I_l, I_t])", "I_f = np.concatenate([I_s, I_t])"),
 ("mid_len includes window", "mid_lo, mid_len = int(I_s.shape[0]), n - int(I_s.shape[0]) - int(I_l.shape[0])", "mid_lo, mid_len = int(I_s.shape[0]), n - int(I_s.shape[0])"),
 ("topk count ceil", "return int(math.floor(np.float64(np.float32(topk_frac)) * n))", "return int(math.ceil(np.float64(np.float32(topk_frac)) * n))"),
 ("chunk length off by one", "return max(int(n) - (int(q_len) - 1 - int(t)), 0)", "return max(int(n) - (int(q_len) - int(t)), 0)"),
 ("chunk reversed", "return max(int(n) - (int(q_len) - 1 - int(t)), 0)", "return max(int(n) - int(t), 0)"),
 ("decode gqa map", "out[(b, h)] = decode_head(q[b, h], K[b, h // g, :n], V[b, h // g, :n],", "out[(b, h)] = decode_head(q[b, h], K[b, h % Hkv, :n], V[b, h % Hkv, :n],"),
 ("decode head index dropped", "seed=int(seeds[b]), head=h, params=params)\n    return out", "seed=int(seeds[b]), head=0, params=params)\n    return out"),
 ("decode seed of seq 0", "seed=int(seeds[b]), head=h, params=params)\n    return out", "seed=int(seeds[0]), head=h, params=params)\n    return out"),
 ("decode ignores seq_lens", "n = int(seq_lens[b])\n        out[(b, h)]", "n = K.shape[2]\n        out[(b, h)]"),
 ("chunk query dropped", "seed=int(seeds[b]), head=h, params=params, query=t)", "seed=int(seeds[b]), head=h, params=params, query=0)"),
 ("chunk gqa map", "out[(b, t, h)] = decode_head(q[b, t, h], K[b, h // g, :n], V[b, h // g, :n],", "out[(b, t, h)] = decode_head(q[b, t, h], K[b, h % Hkv, :n], V[b, h % Hkv, :n],"),
 ("chunk not causal", "n = chunk_length(int(seq_lens[b]), Q, t)", "n = int(seq_lens[b])"),
 ("nested from whole residual", "rest = np.setdiff1d(residual, I_bs, assume_unique=True)", "rest = residual"),
 ("nested stream 0", "extra = uniform_sample(rest, b - b0, mid_lo=mid_lo, mid_len=mid_len, seed=seed, head=head, stream=1,", "extra = uniform_sample(rest, b - b0, mid_lo=mid_lo, mid_len=mid_len, seed=seed, head=head, stream=0,"),
 ("nested size b", "extra = uniform_sample(rest, b - b0, mid_lo", "extra = uniform_sample(rest, b, mid_lo"),
 ("cache replace range t", "r = cache_draw(words4, t + 1)", "r = cache_draw(words4, t)"),
 ("cache replace always", "        if r < C:\n            slots[r] = int(t)", "        slots[r % C] = int(t)"),
 ("cache fills in arrival order", "j = cache_draw(words4, c + 1)", "j = c"),
 ("cache fill swaps wrong range", "j = cache_draw(words4, c + 1)", "j = cache_draw(words4, max(c, 1))"),
 ("cache kv head dropped", "np.full(t.size, kv_head, np.uint64)", "np.full(t.size, 0, np.uint64)"),
 ("cache seed low half only", "                      (int(seed) & _MASK32, (int(seed) >> 32) & _MASK32))\n    return np.stack([np.asarray(x", "                      (int(seed) & _MASK32, 0))\n    return np.stack([np.asarray(x"),
 ("cache token counter dropped", "t = np.arange(int(t_lo), int(t_hi), dtype=np.uint64) & np.uint64(_MASK32)\n    w = philox", "t = np.arange(int(t_lo), int(t_hi), dtype=np.uint64) * np.uint64(0)\n    w = philox"),
 ("base from cache not filtered", "got = [int(t) for t in cache_tokens if int(t) in is_res][:int(b0)]", "got = [int(t) for t in cache_tokens][:int(b0)]"),
 ("base from cache lowest tokens", "got = [int(t) for t in cache_tokens if int(t) in is_res][:int(b0)]", "got = sorted(int(t) for t in cache_tokens if int(t) in is_res)[:int(b0)]"),
 ("base from cache short sample", "    if len(got) < int(b0):\n        return None", "    if len(got) < 1:\n        return None"),
 ("cache never used", "I_bs = base_sample_from_cache(cache_tokens, residual, b0) if cache_tokens is not None else None", "I_bs = None"),
 ("range bound without the half", "return 0.5 * math.log(2.0 / dlt) * (n_s * float(w_range)", "return math.log(2.0 / dlt) * (n_s * float(w_range)"),
 ("range bound ln(1/delta)", "return 0.5 * math.log(2.0 / dlt) * (n_s * float(w_range)", "return 0.5 * math.log(1.0 / dlt) * (n_s * float(w_range)"),
 ("range bound not squared", "* (n_s * float(w_range) / (eps * stats[\"D_hat\"])) ** 2", "* (n_s * float(w_range) / (eps * stats[\"D_hat\"]))"),
 ("range bound over D_f", "* (n_s * float(w_range) / (eps * stats[\"D_hat\"])) ** 2", "* (n_s * float(w_range) / (eps * stats[\"D_f\"])) ** 2"),
 ("range from the largest top-k score", "return float(math.exp(float(np.min(s[I_t])) - m))", "return float(math.exp(float(np.max(s[I_t])) - m))"),
 ("range without the shift", "return float(math.exp(float(np.min(s[I_t])) - m))", "return float(math.exp(float(np.min(s[I_t]))))"),
 ("range for a supplied set", "    if supplied:\n        raise ValueError(\"a caller-supplied top-k set does not bound the residual weights\")", "    if False:\n        raise ValueError(\"a caller-supplied top-k set does not bound the residual weights\")"),
 ("base sample stream 1", "I_bs = uniform_sample(residual, b0, mid_lo=mid_lo, mid_len=mid_len, seed=seed, head=head, stream=0,", "I_bs = uniform_sample(residual, b0, mid_lo=mid_lo, mid_len=mid_len, seed=seed, head=head, stream=1,"),
 ("stats over I_dyn scale", "st = sample_stats(s, V, m, I_f, I_bs, n_s, need_num=(target != TARGET_D))", "st = sample_stats(s, V, m, I_f, I_bs, n_s - 1, need_num=(target != TARGET_D))"),
 ("m over I_f only", "    m = float(s.max())\n    k = topk_count", "    m = float(s[:1].max())\n    k = topk_count"),
 ("n_s counts top-k", "n_s = int(residual.shape[0])\n    res: Dict", "n_s = int(residual.shape[0]) + int(I_t.shape[0])\n    res: Dict"),
 ("cap frac ignored", "cap = int(math.ceil(np.float64(np.float32(cap_frac)) * n_s))", "cap = n_s"),
 ("budget alt only own", "for v in range(min(lo, hi), max(lo, hi) + 1):        # every ceil(b')", "for v in range(0):        # every ceil(b')"),
 ("budget alt window 1e-4", "rel_tol: float = 1e-6,\n                        multiple: int = 1) -> List[int]:", "rel_tol: float = 1e-4,\n                        multiple: int = 1) -> List[int]:"),
 ("topk alt tolerance abs", "near = np.abs(s[mid] - tau) <= rel_tol * np.maximum(np.abs(s[mid]), abs(tau))", "near = np.abs(s[mid] - tau) <= rel_tol"),
 ("dense lse base", "return N / D, m + math.log(D)", "return N / D, math.log(D)"),
 ("draw cap tiny", "return 64 * int(L) + 4096", "return int(L)"),
 ("eps not squared in N", "if target == TARGET_N:\n        return (upper_tail_quantile(dlt / 2.0) * rho_N / eps) ** 2", "if target == TARGET_N:\n        return (upper_tail_quantile(dlt / 2.0) * rho_N) ** 2 / eps"),
]

def run(i):
    name, old, new = M[i]
    if old is None:
        return name, "skipped"
    if SRC.count(old) < 1:
        raise SystemExit("pattern of mistake %r no longer occurs in the oracle: update the list" % name)
    d = tempfile.mkdtemp(prefix="oracle_mistake_%02d_" % i)
    for sub in ("oracle", "tests", "workloads"):
        shutil.copytree(os.path.join(ROOT, sub), os.path.join(d, sub), ignore=shutil.ignore_patterns("__pycache__", "test_gpu_*"))
    open(os.path.join(d, "oracle/vatt_oracle.py"), "w").write(SRC.replace(old, new, 1))
    env = dict(os.environ, PYTHONDONTWRITEBYTECODE="1", OMP_NUM_THREADS="1")
    r = subprocess.run([sys.executable, "-m", "pytest", "tests/test_oracle_pins.py", "tests/test_oracle_statistics.py", "-x", "-q", "-m", "not gpu", "-p", "no:cacheprovider",
                        # that test compares this list with the oracle's text, which the planted mistake has just changed
                        "--deselect", "tests/test_oracle_pins.py::test_planted_mistakes_list_follows_the_oracle"],
                       cwd=d, env=env, capture_output=True, text=True)
    tail = [l for l in r.stdout.splitlines() if l.startswith("FAILED") or "passed" in l or "failed" in l]
    shutil.rmtree(d, ignore_errors=True)
    return name, ("caught: " + (tail[0][:150] if tail else "?")) if r.returncode != 0 else "NOT CAUGHT " + (tail[-1] if tail else "")


def stale_patterns():
    """Names of the entries whose text no longer occurs in the oracle (the list has to follow the oracle)."""
    return [name for name, old, _ in M if old is not None and SRC.count(old) < 1]


def main():
    sel = [i for i in range(len(M)) if len(sys.argv) < 2 or sys.argv[1] in M[i][0]]
    missed = 0
    with ThreadPoolExecutor(max(1, min(6, (os.cpu_count() or 2) - 2))) as ex:
        for name, res in ex.map(run, sel):
            if res.startswith("NOT CAUGHT") and name in EQUIVALENT:
                res = "passes, as expected of an equivalent change"
            elif not res.startswith("caught"):
                missed += 1
            print("%-32s %s" % (name, res), flush=True)
    print("%d mistakes planted, %d not caught" % (len(sel), missed))
    sys.exit(1 if missed else 0)


if __name__ == "__main__":
    main()
