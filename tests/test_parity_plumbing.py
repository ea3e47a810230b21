"""The parity harness itself, on the CPU: the checks that fan out over worker processes must see the same
tensors and reach the same verdicts as the in-process ones.  The "library results" here are made from the
oracle's own outputs (this tests the harness, not the library)."""
import numpy as np
import pytest

import workloads
from oracle import vatt_oracle as vo
from parity import alternatives_used, check_all, check_all_parallel, release_shared, share_workload


def _results_from_oracle(wl, cap=4096):
    B, Hq, d = wl.batch, wl.n_q_heads, wl.head_dim
    p = wl.params
    seg = [0, int(p["sink"]), int(p["sink"]) + int(p["window"]), 0, 0]
    seg[3] = seg[2] + 64
    seg[4] = seg[3] + 64
    res = dict(O=np.zeros((B, Hq, d), np.float32), lse=np.zeros((B, Hq), np.float32),
               idx=np.zeros((B, Hq, cap), np.int32), counts=np.zeros((B, Hq, 8), np.int32),
               b_star=np.zeros((B, Hq)), stats=np.zeros((B, Hq, 4), np.float32), seg=seg)
    q = wl.q_f32().astype(np.float64)
    g = Hq // wl.n_kv_heads
    for b in range(B):
        n = int(wl.seq_lens[b])
        for h in range(Hq):
            r = vo.decode_head(q[b, h], wl.k_f32(b, h // g, n).astype(np.float64),
                               wl.v_f32(b, h // g, n).astype(np.float64), seed=int(wl.seeds[b]), head=h, params=p)
            for s, key in enumerate(("I_s", "I_l", "I_t", "I_bs", "I_dyn")):
                res["idx"][b, h, seg[s]:seg[s] + len(r[key])] = r[key]
            res["counts"][b, h] = [len(r["I_s"]), len(r["I_l"]), len(r["I_t"]), len(r["I_bs"]), r["b"], r["n_s"], n, 0]
            res["b_star"][b, h] = r["b_star"]
            st = r["stats"]
            res["stats"][b, h] = [st["D_hat"], st["sigma2"], st["tr_sigma"], st["N_hat_sq"]]
            res["O"][b, h], res["lse"][b, h] = r["O"], r["lse"]
    return res


def test_parallel_check_agrees_with_the_in_process_check_and_sees_later_writes():
    wl0 = workloads.small_gqa(seed=3, batch=2, n_q_heads=4, n_kv_heads=2, head_dim=64, n=700,
                              topk_frac=0.03, base_abs=24)
    wl, shared = share_workload(wl0)
    try:
        assert np.array_equal(wl.k_bits, wl0.k_bits) and np.array_equal(wl.q_bits, wl0.q_bits)
        res = _results_from_oracle(wl)
        a = check_all(wl, res, label="in-process")
        b = check_all_parallel(wl, res, shared, label="workers", workers=2)
        assert len(a) == len(b) == 8 and alternatives_used(b) == (0, 0)
        assert sorted(r["b"] for r in a) == sorted(r["b"] for r in b)
        # a result that is wrong in one head fails in the workers too
        bad = dict(res, O=res["O"].copy())
        bad["O"][1, 2] *= 1.01
        with pytest.raises(AssertionError):
            check_all_parallel(wl, bad, shared, label="workers", workers=2)
        # a token written through the shared workload (an append) reaches workers started afterwards
        wl.k_bits[0, :, 5] = wl.k_bits[0, :, 6]
        with pytest.raises(AssertionError):
            check_all_parallel(wl, res, shared, label="workers", workers=2)
        res2 = _results_from_oracle(wl)
        check_all_parallel(wl, res2, shared, label="workers after a write", workers=2)
    finally:
        release_shared(shared)
