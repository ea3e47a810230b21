"""vatt_decode_static (the entry point that allocates nothing: its scratch memory is an array inside the
library) against vatt_decode, through the C ABI: two calls in a row, the second with a smaller input, each
compared with the existing entry point on the same inputs (the kernels are the same, so every output must be
identical bit for bit) and with the oracle."""
import numpy as np
import pytest
import torch

import workloads
from parity import alternatives_used, check_all, say
from util import plan_params

pytestmark = pytest.mark.gpu


def _both(wl):
    from paper_2510_05688_amd import binding as vb
    from paper_2510_05688_amd.session import DecodeSession
    sess = DecodeSession(plan_params(wl))
    sess.upload(wl.q_bits, wl.k_bits, wl.v_bits, wl.seq_lens, wl.seeds)
    assert vb.vatt_plan_workspace_bytes(sess.plan) <= vb.vatt_static_scratch_bytes()
    sess.decode()
    ref = sess.results_host()
    # poison the outputs, then the call without a workspace
    for t in (sess.out_o, sess.out_lse, sess.out_stats, sess.out_budget_raw):
        t.fill_(float("nan"))
    sess.out_idx.fill_(-7)
    sess.out_counts.fill_(-7)
    before = torch.cuda.memory_allocated()
    vb.vatt_decode_static(sess.plan, sess.q, sess.k, sess.v, sess.block_table, sess.seq_lens, sess.seq_seeds,
                          sess.out_o, sess.out_lse, sess.out_idx, sess.out_counts, sess.out_budget_raw,
                          sess.out_stats, torch.cuda.current_stream().cuda_stream)
    got = sess.results_host()
    assert torch.cuda.memory_allocated() == before
    sess.close()
    return ref, got


def _same(ref, got, wl):
    seg = ref["seg"]
    assert np.array_equal(ref["counts"], got["counts"])
    for b in range(wl.batch):
        for h in range(wl.n_q_heads):
            c = ref["counts"][b, h]
            for s, cnt in ((0, c[0]), (1, c[1]), (2, c[2]), (3, c[3]), (4, c[4])):
                assert np.array_equal(ref["idx"][b, h, seg[s]:seg[s] + cnt], got["idx"][b, h, seg[s]:seg[s] + cnt])
    for key in ("O", "lse", "b_star", "stats"):
        assert np.array_equal(ref[key], got[key]), key


def test_decode_static_matches_decode_on_two_calls_the_second_smaller():
    from paper_2510_05688_amd import binding as vb
    say("vatt_decode_static: 4096-token batch of 2, then a 1500-token single sequence")
    big = workloads.small_gqa(seed=11, batch=2, n=4096, seq_lens=[4096, 3333])
    ref, got = _both(big)
    _same(ref, got, big)
    reps = check_all(big, got, label="static scratch, first call")
    small = workloads.small_gqa(seed=12, batch=1, n=1500, seq_lens=[1500], n_q_heads=4, n_kv_heads=1)
    ref2, got2 = _both(small)
    _same(ref2, got2, small)
    reps += check_all(small, got2, label="static scratch, second (smaller) call")
    assert alternatives_used(reps) == (0, 0)
    # a plan that needs more than the array holds is refused before anything is launched
    wl = workloads.small_gqa(seed=13, batch=1, n=2048, seq_lens=[2048])
    from paper_2510_05688_amd.session import DecodeSession
    sess = DecodeSession(plan_params(wl, batch=16, n_max=32768))
    assert vb.vatt_plan_workspace_bytes(sess.plan) > vb.vatt_static_scratch_bytes()
    with pytest.raises(vb.VattError) as e:
        vb.vatt_decode_static(sess.plan, sess.out_o, sess.out_o, sess.out_o, None, sess.out_o, sess.out_o,
                              sess.out_o, sess.out_lse, sess.out_idx, sess.out_counts, sess.out_budget_raw,
                              sess.out_stats, torch.cuda.current_stream().cuda_stream)
    assert e.value.status == vb.VATT_E_WORKSPACE_TOO_SMALL
    sess.close()
