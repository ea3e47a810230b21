"""Seeded generators for the synthetic decode workloads.

The workloads stand in for the paper's 32K-context evaluation settings
(Table 1 and Table 2: Llama-3.1-8B-class attention, 32 query heads, 8 KV
heads, head_dim 128; sink = local window = 128 tokens, top-k fraction and base
sampling rate 0.025, epsilon = delta = 0.05).  The benchmark data and model
weights are not available, so keys, values and queries are Gaussian with two
kinds of KV head:

* "spiky" heads: K ~ N(0, 1) with a small number of planted heavy keys aligned
  with the mean query of the GQA group (attention mass concentrated on a few
  tokens, the regime where top-k selection carries the result);
* "flat" heads: K ~ N(0, 0.25) (variance 0.25, i.e. std 0.5; a long tail of
  comparable scores, the regime where uniform sampling carries the result).

In N(a, b) the second argument is a variance throughout.  Every tensor is
rounded to bf16 exactly once, here; consumers get the uint16 bit patterns.
Nothing in this module computes a score, a selection or a sample.
"""
from __future__ import annotations

import dataclasses
from typing import Dict, Optional

import numpy as np

from .bf16 import f32_to_bf16_bits, bf16_bits_to_f32

TARGET_D = 0
TARGET_N = 1
TARGET_SDPA = 2


@dataclasses.dataclass
class Workload:
    """One decode step's inputs.

    q_bits:   uint16 [B, Hq, d]          bf16 queries
    k_bits:   uint16 [B, Hkv, n_max, d]  bf16 keys, contiguous layout
    v_bits:   uint16 [B, Hkv, n_max, d]  bf16 values, contiguous layout
    seq_lens: int32  [B]                 valid tokens per sequence (<= n_max)
    seeds:    uint64 [B]                 per-sequence sampler seed for this call
    params:   method parameters (sink, window, topk_abs, topk_frac, base_abs,
              base_frac, epsilon, delta, target, sm_scale, budget_cap_frac)
    """

    name: str
    q_bits: np.ndarray
    k_bits: np.ndarray
    v_bits: np.ndarray
    seq_lens: np.ndarray
    seeds: np.ndarray
    params: Dict[str, float]
    spiky_heads: Optional[np.ndarray] = None  # bool [Hkv]

    @property
    def batch(self) -> int:
        return int(self.q_bits.shape[0])

    @property
    def n_q_heads(self) -> int:
        return int(self.q_bits.shape[1])

    @property
    def n_kv_heads(self) -> int:
        return int(self.k_bits.shape[1])

    @property
    def head_dim(self) -> int:
        return int(self.q_bits.shape[2])

    @property
    def n_max(self) -> int:
        return int(self.k_bits.shape[2])

    def q_f32(self) -> np.ndarray:
        return bf16_bits_to_f32(self.q_bits)

    def k_f32(self, b: int, kvh: int, n: Optional[int] = None) -> np.ndarray:
        n = int(self.seq_lens[b]) if n is None else n
        return bf16_bits_to_f32(self.k_bits[b, kvh, :n])

    def v_f32(self, b: int, kvh: int, n: Optional[int] = None) -> np.ndarray:
        n = int(self.seq_lens[b]) if n is None else n
        return bf16_bits_to_f32(self.v_bits[b, kvh, :n])


def default_params(head_dim: int, **over) -> Dict[str, float]:
    p = dict(
        sink=128,
        window=128,
        topk_abs=0,
        topk_frac=0.025,
        base_abs=0,
        base_frac=0.025,
        epsilon=0.05,
        delta=0.05,
        target=TARGET_D,
        sm_scale=float(np.float32(1.0 / np.sqrt(np.float64(head_dim)))),
        budget_cap_frac=1.0,
    )
    p.update(over)
    return p


def make_workload(
    name: str,
    *,
    batch: int,
    n_q_heads: int,
    n_kv_heads: int,
    head_dim: int,
    n_max: int,
    seq_lens,
    seed: int,
    params: Dict[str, float],
    spiky_every: int = 2,
    flat_var: float = 0.25,
    plant_frac: float = 0.001,
    plant_scale: float = 3.0,
    plant_noise_var: float = 0.1,
    cluster: int = 1,
    v_mean: float = 0.0,
    all_flat: bool = False,
    all_spiky: bool = False,
) -> Workload:
    """General recipe behind the named configs.

    KV head j is spiky when j % spiky_every == 0 (even heads by default), else
    flat.  A spiky head gets floor(plant_frac * n) planted keys (rounded up to
    whole clusters of `cluster` consecutive tokens, at least one cluster when
    plant_frac > 0), each set to plant_scale * sqrt(d) * qbar / ||qbar|| plus
    N(0, plant_noise_var) noise, qbar being the mean query of the head's GQA
    group.  V ~ N(v_mean, 1).  q ~ N(0, 1).  Sequence b uses seed + b for its
    sampler seed.
    """
    assert n_q_heads % n_kv_heads == 0
    g = n_q_heads // n_kv_heads
    rng = np.random.default_rng(seed)
    seq_lens = np.asarray(seq_lens, dtype=np.int32).reshape(batch)
    assert seq_lens.max() <= n_max
    q = rng.standard_normal((batch, n_q_heads, head_dim), dtype=np.float32)
    k_bits = np.empty((batch, n_kv_heads, n_max, head_dim), dtype=np.uint16)
    v_bits = np.empty((batch, n_kv_heads, n_max, head_dim), dtype=np.uint16)
    spiky = np.zeros(n_kv_heads, dtype=bool)
    for j in range(n_kv_heads):
        spiky[j] = (j % spiky_every == 0)
    if all_flat:
        spiky[:] = False
    if all_spiky:
        spiky[:] = True
    for b in range(batch):
        n = int(seq_lens[b])
        for j in range(n_kv_heads):
            kk = rng.standard_normal((n_max, head_dim), dtype=np.float32)
            if spiky[j]:
                n_plant = int(np.floor(plant_frac * n))
                if plant_frac > 0.0 and n > cluster:
                    n_clusters = max(1, int(round(n_plant / cluster)))
                    qbar = q[b, j * g:(j + 1) * g].mean(axis=0)
                    direction = qbar / np.linalg.norm(qbar)
                    starts = rng.choice(max(1, (n - cluster) // cluster), size=n_clusters,
                                        replace=False) * cluster
                    for s0 in np.sort(starts):
                        noise = rng.standard_normal((cluster, head_dim), dtype=np.float32)
                        kk[s0:s0 + cluster] = (
                            np.float32(plant_scale * np.sqrt(head_dim)) * direction[None, :]
                            + np.float32(np.sqrt(plant_noise_var)) * noise
                        )
            else:
                kk *= np.float32(np.sqrt(flat_var))
            k_bits[b, j] = f32_to_bf16_bits(kk)
            vv = rng.standard_normal((n_max, head_dim), dtype=np.float32)
            if v_mean != 0.0:
                vv += np.float32(v_mean)
            v_bits[b, j] = f32_to_bf16_bits(vv)
    seeds = (np.uint64(seed) + np.arange(batch, dtype=np.uint64)).astype(np.uint64)
    return Workload(
        name=name,
        q_bits=f32_to_bf16_bits(q),
        k_bits=k_bits,
        v_bits=v_bits,
        seq_lens=seq_lens,
        seeds=seeds,
        params=dict(params),
        spiky_heads=spiky,
    )


def config1(seed: int = 0) -> Workload:
    """Tiny single head: B=1, 1 query head, 1 KV head, d=64, n=1024.

    q, K, V ~ N(0, 1); 8 planted heavy keys 3*sqrt(64)*q/||q|| + N(0, 0.1) at
    random positions; sink 4, window 32, top-k 32, base sample 32,
    epsilon = delta = 0.05.  Generated in fp32 and rounded to bf16 once.
    """
    p = default_params(64, sink=4, window=32, topk_abs=32, topk_frac=0.0,
                       base_abs=32, base_frac=0.0, epsilon=0.05, delta=0.05)
    return make_workload("config1_tiny", batch=1, n_q_heads=1, n_kv_heads=1, head_dim=64,
                         n_max=1024, seq_lens=[1024], seed=seed, params=p,
                         spiky_every=1, plant_frac=8.0 / 1024.0)


def config2(seed: int = 1, n: int = 32768, batch: int = 1) -> Workload:
    """Llama-3.1-8B-shaped decode layer: 32 query / 8 KV heads, d=128, n=32768.

    Even KV heads spiky (0.1 % planted keys at scale 3), odd KV heads flat
    (K ~ N(0, 0.25)); V ~ N(0, 1); sink = window = 128, k = floor(0.025 n),
    base sample floor(0.025 n_s), epsilon = delta = 0.05.
    """
    p = default_params(128)
    return make_workload("config2_llama8b_32k" if batch == 1 else "config3_llama8b_32k_b%d" % batch,
                         batch=batch, n_q_heads=32, n_kv_heads=8, head_dim=128,
                         n_max=n, seq_lens=[n] * batch, seed=seed, params=p)


def config3(seed: int = 1, batch: int = 16, n: int = 32768) -> Workload:
    """Batched throughput: config 2's head shapes at batch 16, per-sequence seeds."""
    return config2(seed=seed, n=n, batch=batch)


def config4(seed: int = 4, batch: int = 4, n: int = 131072) -> Workload:
    """Long context: B=4, 32/8 heads, d=128, n=131072, contiguous.

    Heavy tokens planted in 64-token clusters at 0.05 % density (whole clusters,
    at least one per spiky head); sink 128, window 512, k = floor(0.01 n).
    """
    p = default_params(128, sink=128, window=512, topk_frac=0.01)
    return make_workload("config4_long_128k", batch=batch, n_q_heads=32, n_kv_heads=8,
                         head_dim=128, n_max=n, seq_lens=[n] * batch, seed=seed, params=p,
                         plant_frac=0.0005, cluster=64)


def config5(seed: int = 5, batch: int = 32, n_lo: int = 1024, n_hi: int = 32768,
            steps: int = 256, page: int = 16) -> Workload:
    """Ragged decode loop start state: B=32, lengths ~ U[n_lo, n_hi] from the seed.

    The cache has room for `steps` appended tokens (capacity rounded up to a
    whole page).  epsilon = delta = 0.1.  The caller pages it with to_paged()
    and appends one N(0, 1) token per sequence per step (append_tokens()).
    """
    rng = np.random.default_rng(seed + 1000)
    lens = rng.integers(n_lo, n_hi + 1, size=batch).astype(np.int32)
    n_max = int(-(-(n_hi + steps) // page) * page)
    p = default_params(128, epsilon=0.1, delta=0.1)
    return make_workload("config5_ragged_paged", batch=batch, n_q_heads=32, n_kv_heads=8,
                         head_dim=128, n_max=n_max, seq_lens=lens, seed=seed, params=p)


def small_gqa(seed: int = 7, batch: int = 2, n_q_heads: int = 8, n_kv_heads: int = 2,
              head_dim: int = 128, n: int = 3000, seq_lens=None, **over) -> Workload:
    """Small GQA case for element-by-element parity: several tiles and a ragged tail."""
    if seq_lens is None:
        seq_lens = [n - 37 * b for b in range(batch)]
    kw = dict(sink=16, window=24)
    kw.update(over)
    p = default_params(head_dim, **kw)
    return make_workload("small_gqa", batch=batch, n_q_heads=n_q_heads, n_kv_heads=n_kv_heads,
                         head_dim=head_dim, n_max=n, seq_lens=seq_lens, seed=seed, params=p,
                         plant_frac=0.004)


def append_tokens(seed: int, step: int, batch: int, n_kv_heads: int, head_dim: int):
    """New K/V token for every sequence at a decode step: N(0, 1), bf16 bits [B, Hkv, d] each."""
    rng = np.random.default_rng([seed, step])
    k_new = rng.standard_normal((batch, n_kv_heads, head_dim), dtype=np.float32)
    v_new = rng.standard_normal((batch, n_kv_heads, head_dim), dtype=np.float32)
    return f32_to_bf16_bits(k_new), f32_to_bf16_bits(v_new)


def chunk_queries(wl: Workload, q_len: int, seed: int = 0, spread: float = 0.5) -> np.ndarray:
    """Queries of a multi-query step over wl's cache: bf16 bits [B, q_len, Hq, d].

    The newest query token (the last of the chunk) is wl's own query; the older ones are that query plus
    N(0, spread^2) noise, so that neighbouring query tokens look at related keys (the planted keys of a spiky
    head stay heavy for all of them) without being copies of each other.
    """
    rng = np.random.default_rng([seed, 4242, q_len])
    base = wl.q_f32()  # [B, Hq, d]
    B, Hq, d = base.shape
    q = np.repeat(base[:, None], q_len, axis=1).astype(np.float32)
    noise = rng.standard_normal((B, q_len, Hq, d), dtype=np.float32) * np.float32(spread)
    noise[:, q_len - 1] = 0.0
    return f32_to_bf16_bits(q + noise)


def to_paged(wl: Workload, page: int = 16, seed: int = 0):
    """Re-lay a contiguous cache into shuffled pages.

    Returns (k_pages, v_pages, block_table): pages are uint16
    [num_blocks, Hkv, page, d]; block_table is int32 [B, n_max / page] and maps
    logical page p of sequence b to a physical block.  Physical blocks are a
    random permutation, so neighbouring logical pages are not neighbours in
    memory.
    """
    B, Hkv, n_max, d = wl.k_bits.shape
    assert n_max % page == 0
    ppb = n_max // page
    rng = np.random.default_rng(seed + 77)
    perm = rng.permutation(B * ppb).astype(np.int32)
    block_table = perm.reshape(B, ppb)
    k_pages = np.empty((B * ppb, Hkv, page, d), dtype=np.uint16)
    v_pages = np.empty((B * ppb, Hkv, page, d), dtype=np.uint16)
    kb = wl.k_bits.reshape(B, Hkv, ppb, page, d).transpose(0, 2, 1, 3, 4)  # [B, ppb, Hkv, page, d]
    vb = wl.v_bits.reshape(B, Hkv, ppb, page, d).transpose(0, 2, 1, 3, 4)
    k_pages[block_table.reshape(-1)] = kb.reshape(B * ppb, Hkv, page, d)
    v_pages[block_table.reshape(-1)] = vb.reshape(B * ppb, Hkv, page, d)
    return k_pages, v_pages, block_table
