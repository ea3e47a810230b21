"""KV cache in pinned host memory (the setting of the paper's efficiency experiment): the same kernels read the
rows they need over the host link.  Results must equal those with the cache in device memory bit for bit (same
data, same launches), and the oracle's on the checked heads; appends must land in the host copy."""
import numpy as np
import pytest
import torch

import workloads
from parity import check_all, check_head_given, say
from test_gpu_random_cache import CACHE_SEEDS, _oracle_caches, _oracle_topk, _run_cached, _session
from util import plan_params

pytestmark = pytest.mark.gpu

KEYS = ("O", "lse", "counts", "b_star", "stats")


def _same(a, b, what):
    for key in KEYS:
        assert np.array_equal(a[key], b[key], equal_nan=True), "%s: %s differs" % (what, key)
    # the index lists, in the order written, up to their counts (the buffer is not cleared beyond them)
    seg, cnt = a["seg"], a["counts"]
    for bq in range(cnt.shape[0]):
        for h in range(cnt.shape[1]):
            for s_, c in zip(seg, cnt[bq, h, :5]):
                assert np.array_equal(a["idx"][bq, h, s_:s_ + c], b["idx"][bq, h, s_:s_ + c]), \
                    "%s: list at %d of (%d, %d) differs" % (what, s_, bq, h)


def test_pointer_translation_accepts_pinned_memory_only():
    from paper_2510_05688_amd import binding as vb
    pinned = torch.empty(4096, dtype=torch.uint8, pin_memory=True)
    addr = vb.vatt_host_kv_device_pointer(pinned)
    assert addr != 0
    inner = vb.vatt_host_kv_device_pointer(int(pinned.data_ptr()) + 1024)   # anywhere inside the allocation
    assert inner == addr + 1024
    plain = np.zeros(4096, dtype=np.uint8)
    with pytest.raises(vb.VattError) as e:
        vb.vatt_host_kv_device_pointer(int(plain.ctypes.data))
    assert e.value.status == vb.VATT_E_INVALID_ARG
    device = torch.empty(4096, dtype=torch.uint8, device="cuda")
    with pytest.raises(vb.VattError) as e:
        vb.vatt_host_kv_device_pointer(device)
    assert e.value.status == vb.VATT_E_INVALID_ARG
    # the runtime is left without a pending error
    torch.cuda.synchronize()


@pytest.mark.parametrize("paged", [False, True])
def test_given_topk_with_the_cache_on_the_host(paged):
    say("caller-supplied top-k, K and V in pinned host memory (paged=%s)" % paged)
    wl = workloads.small_gqa(seed=71, batch=2, n=3008, seq_lens=[3008, 2963], epsilon=0.02)
    sess = _session(wl, paged=paged)          # random cache filled from the device copy
    caches = _oracle_caches(wl, sess.cache_slots)
    g = wl.n_q_heads // wl.n_kv_heads
    supplied = {(b, h): _oracle_topk(wl, b, h) for b in range(wl.batch) for h in range(wl.n_q_heads)}
    on_device_cached = _run_cached(sess, wl, supplied)
    on_device_plain = _run_cached(sess, wl, supplied, cached=False)
    sess.dense()
    torch.cuda.synchronize()
    dense_device = sess.dense_o.cpu().numpy().copy()

    sess.move_kv_to_host()
    assert isinstance(sess.k, int) and isinstance(sess.v, int)
    res = _run_cached(sess, wl, supplied)
    _same(res, on_device_cached, "base sample from the random cache")
    reps = [check_head_given(wl, res, b, h, supplied[(b, h)], label="host kv", cache_tokens=caches[(b, h // g)])
            for b in range(wl.batch) for h in range(wl.n_q_heads)]
    assert all(r["from_cache"] for r in reps)
    _same(_run_cached(sess, wl, supplied, cached=False), on_device_plain, "base sample drawn")
    sess.dense()
    torch.cuda.synchronize()
    assert np.array_equal(sess.dense_o.cpu().numpy(), dense_device)
    # a random cache filled from the host copy is the same cache
    kept = sess.rcache.clone()
    sess.rcache.zero_()
    from paper_2510_05688_amd import binding as vb
    vb.vatt_random_cache_fill(sess.plan, sess.k, sess.v, sess.block_table, sess.seq_lens, sess.cache_seeds, sess.rcache)
    torch.cuda.synchronize()
    tok, cnt = sess.random_cache_host()
    for (b, kvh), want in caches.items():
        assert tok[b, kvh, :len(want)].tolist() == want
    _same(_run_cached(sess, wl, supplied), on_device_cached, "cache filled from the host copy")
    del kept
    sess.close()


def test_exact_scoring_with_the_cache_on_the_host():
    # vatt_decode itself (K scanned over the host link): the same results as from device memory, and the oracle's
    say("vatt_decode, K and V in pinned host memory")
    wl = workloads.small_gqa(seed=72, batch=2, n=2500, seq_lens=[2500, 777])
    from paper_2510_05688_amd.session import DecodeSession
    sess = DecodeSession(plan_params(wl))
    sess.upload(wl.q_bits, wl.k_bits, wl.v_bits, wl.seq_lens, wl.seeds)
    sess.decode()
    on_device = sess.results_host()
    on_device = {k: (v.copy() if isinstance(v, np.ndarray) else v) for k, v in on_device.items()}
    sess.move_kv_to_host()
    sess.decode()
    res = sess.results_host()
    _same(res, on_device, "vatt_decode")
    check_all(wl, res, label="host kv, exact scoring")
    sess.close()


@pytest.mark.parametrize("paged", [False, True])
def test_appends_reach_the_host_copy(paged):
    say("appends into a cache in pinned host memory (paged=%s)" % paged)
    from paper_2510_05688_amd.session import _bf16_from_bits
    wl = workloads.small_gqa(seed=73, batch=2, n=1024, seq_lens=[1000, 17])
    sess = _session(wl, paged=paged, slots=64)
    sess.move_kv_to_host()
    lens = np.asarray(wl.seq_lens).copy()
    k_ref = sess.k_host.clone()
    v_ref = sess.v_host.clone()
    page = 16
    for t in range(20):
        kn, vn = workloads.configs.append_tokens(73, t, wl.batch, wl.n_kv_heads, wl.head_dim)
        kd, vd = _bf16_from_bits(kn, sess.device), _bf16_from_bits(vn, sess.device)
        if t % 2:
            sess.append_device_cached(kd, vd)
        else:
            sess.append_device(kd, vd)
        for b in range(wl.batch):
            pos = int(lens[b])
            for kvh in range(wl.n_kv_heads):
                if paged:
                    blk = int(sess.block_table[b, pos // page])
                    k_ref[blk, kvh, pos % page] = kd[b, kvh].cpu()
                    v_ref[blk, kvh, pos % page] = vd[b, kvh].cpu()
                else:
                    k_ref[b, kvh, pos] = kd[b, kvh].cpu()
                    v_ref[b, kvh, pos] = vd[b, kvh].cpu()
        lens += 1
    torch.cuda.synchronize()
    assert sess.seq_lens.cpu().numpy().tolist() == lens.tolist()
    assert torch.equal(sess.k_host.view(torch.int16), k_ref.view(torch.int16))
    assert torch.equal(sess.v_host.view(torch.int16), v_ref.view(torch.int16))
    sess.close()
