"""Device buffers for one plan: allocation and upload only (PyTorch as the memory allocator).

No arithmetic of the method happens here; every call goes straight to the C ABI.
"""
from __future__ import annotations

from typing import Dict, Optional

import numpy as np
import torch

from . import binding as vb


def _bf16_from_bits(bits: np.ndarray, device) -> torch.Tensor:
    t = torch.from_numpy(np.ascontiguousarray(bits).view(np.int16))
    return t.to(device).view(torch.bfloat16)


class DecodeSession:
    """Owns a plan, its workspace and output buffers on one GPU."""

    def __init__(self, params: Dict, device: int = 0, q_len: int = 1):
        """q_len > 1: a plan for multi-query steps; q is then [B, q_len, Hq, d] and every output has one row per
        (sequence, query token) pair, b * q_len + t, where the single-token shapes have one per sequence."""
        if not torch.cuda.is_available():
            raise RuntimeError("DecodeSession needs a GPU; there is no CPU path")
        self.device = torch.device("cuda", device)
        torch.cuda.set_device(self.device)
        self.params = dict(params)
        self.q_len = int(q_len)
        self.plan = (vb.vatt_plan_create(self.params, device) if self.q_len == 1
                     else vb.vatt_plan_create_chunk(self.params, self.q_len, device))
        p = self.params
        self.Hq, self.Hkv, self.d = p["n_q_heads"], p["n_kv_heads"], p["head_dim"]
        self.B = p["batch"] * self.q_len  # rows of every per-query buffer
        self.n_max = p["n_max"]
        self.paged = p.get("kv_layout", 0) == vb.VATT_LAYOUT_PAGED
        self.idx_cap = vb.vatt_plan_index_capacity(self.plan)
        self.seg = [vb.vatt_plan_index_segment(self.plan, s) for s in range(5)]
        self.ws_bytes = vb.vatt_plan_workspace_bytes(self.plan)
        dev = self.device
        self.workspace = torch.empty(self.ws_bytes, dtype=torch.uint8, device=dev)
        assert self.workspace.data_ptr() % 256 == 0
        self.out_o = torch.empty(self.B, self.Hq, self.d, dtype=torch.float32, device=dev)
        self.out_lse = torch.empty(self.B, self.Hq, dtype=torch.float32, device=dev)
        self.out_idx = torch.empty(self.B, self.Hq, self.idx_cap, dtype=torch.int32, device=dev)
        self.out_counts = torch.empty(self.B, self.Hq, 8, dtype=torch.int32, device=dev)
        self.out_budget_raw = torch.empty(self.B, self.Hq, dtype=torch.float64, device=dev)
        self.out_stats = torch.empty(self.B, self.Hq, 4, dtype=torch.float32, device=dev)
        self.dense_o = torch.empty(self.B, self.Hq, self.d, dtype=torch.float32, device=dev)
        self.dense_lse = torch.empty(self.B, self.Hq, dtype=torch.float32, device=dev)
        self.block_table: Optional[torch.Tensor] = None
        self.q = self.k = self.v = self.seq_lens = self.seq_seeds = None

    def close(self):
        if self.plan:
            vb.vatt_plan_destroy(self.plan)
            self.plan = None

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass

    # ---- uploads -----------------------------------------------------------
    def upload(self, q_bits, k_bits, v_bits, seq_lens, seeds, block_table=None):
        dev = self.device
        self.q = _bf16_from_bits(q_bits, dev)
        self.k = _bf16_from_bits(k_bits, dev)
        self.v = _bf16_from_bits(v_bits, dev)
        self.seq_lens = torch.from_numpy(np.ascontiguousarray(seq_lens, dtype=np.int32)).to(dev)
        self.seq_seeds = torch.from_numpy(np.ascontiguousarray(seeds, dtype=np.uint64).view(np.int64)).to(dev)
        self.block_table = None
        if block_table is not None:
            self.block_table = torch.from_numpy(np.ascontiguousarray(block_table, dtype=np.int32)).to(dev)
        return self

    def move_kv_to_host(self):
        """Moves the uploaded K and V to pinned host memory; self.k / self.v become the addresses the kernels
        read them at (vatt_host_kv_device_pointer), and the pinned tensors stay alive in self.k_host / v_host."""
        torch.cuda.synchronize(self.device)
        self.k_host = torch.empty(self.k.shape, dtype=self.k.dtype, pin_memory=True).copy_(self.k)
        self.v_host = torch.empty(self.v.shape, dtype=self.v.dtype, pin_memory=True).copy_(self.v)
        self.k = vb.vatt_host_kv_device_pointer(self.k_host)
        self.v = vb.vatt_host_kv_device_pointer(self.v_host)
        return self

    def set_seeds(self, seeds):
        self.seq_seeds = torch.from_numpy(np.ascontiguousarray(seeds, dtype=np.uint64).view(np.int64)).to(self.device)

    def _stream(self):
        return torch.cuda.current_stream(self.device).cuda_stream

    # ---- calls ---------------------------------------------------------------
    def decode(self, q=None, k=None, v=None):
        vb.vatt_decode(self.plan, self.q if q is None else q, self.k if k is None else k,
                       self.v if v is None else v, self.block_table, self.seq_lens, self.seq_seeds,
                       self.workspace, self.out_o, self.out_lse, self.out_idx, self.out_counts,
                       self.out_budget_raw, self.out_stats, self._stream())

    def decode_given_topk(self, topk_idx, topk_cnt, k=None, v=None):
        """vatt_decode_given_topk with int32 device tensors topk_idx [B, Hq, k_max], topk_cnt [B, Hq]."""
        vb.vatt_decode_given_topk(self.plan, self.q, self.k if k is None else k, self.v if v is None else v,
                                  self.block_table, self.seq_lens, self.seq_seeds, topk_idx, topk_cnt,
                                  self.workspace, self.out_o, self.out_lse, self.out_idx, self.out_counts,
                                  self.out_budget_raw, self.out_stats, self._stream())

    # ---- random cache of base-sample rows ------------------------------------
    def make_random_cache(self, cache_seeds, slots: Optional[int] = None):
        """Allocates the cache buffer and fills it from the sequences as uploaded (vatt_random_cache_fill)."""
        if slots is not None:
            vb.vatt_plan_set_option(self.plan, vb.VATT_OPT_CACHE_SLOTS, int(slots))
        self.cache_slots = vb.vatt_random_cache_slots(self.plan)
        self.cache_seeds = torch.from_numpy(np.ascontiguousarray(cache_seeds, dtype=np.uint64).view(np.int64)).to(self.device)
        self.rcache = torch.empty(vb.vatt_random_cache_bytes(self.plan), dtype=torch.uint8, device=self.device)
        assert self.rcache.data_ptr() % 256 == 0
        vb.vatt_random_cache_fill(self.plan, self.k, self.v, self.block_table, self.seq_lens, self.cache_seeds,
                                  self.rcache, self._stream())

    def random_cache_host(self):
        """(tokens int32 [B, Hkv, slots] with -1 in unused slots, counts int32 [B, Hkv]) of the cache."""
        B = self.params["batch"]
        tok = torch.empty(B, self.Hkv, self.cache_slots, dtype=torch.int32, device=self.device)
        cnt = torch.empty(B, self.Hkv, dtype=torch.int32, device=self.device)
        vb.vatt_random_cache_read(self.plan, self.rcache, tok, cnt, self._stream())
        torch.cuda.synchronize(self.device)
        return tok.cpu().numpy(), cnt.cpu().numpy()

    def append_device_cached(self, k_new, v_new):
        vb.vatt_append_kv_cached(self.plan, k_new, v_new, self.k, self.v, self.block_table, self.seq_lens,
                                 self.cache_seeds, self.rcache, self._stream())

    def decode_given_topk_cached(self, topk_idx, topk_cnt, k=None, v=None):
        vb.vatt_decode_given_topk_cached(self.plan, self.q, self.k if k is None else k,
                                         self.v if v is None else v, self.block_table, self.seq_lens,
                                         self.seq_seeds, topk_idx, topk_cnt, self.rcache, self.workspace,
                                         self.out_o, self.out_lse, self.out_idx, self.out_counts,
                                         self.out_budget_raw, self.out_stats, self._stream())

    def dense(self, q=None, k=None, v=None):
        vb.vatt_dense_decode(self.plan, self.q if q is None else q, self.k if k is None else k,
                             self.v if v is None else v, self.block_table, self.seq_lens, self.workspace,
                             self.dense_o, self.dense_lse, self._stream())

    def score(self, q=None, k=None):
        vb.vatt_score(self.plan, self.q if q is None else q, self.k if k is None else k, self.block_table,
                      self.seq_lens, self.workspace, self._stream())

    def append(self, k_new_bits, v_new_bits):
        kn = _bf16_from_bits(k_new_bits, self.device)
        vn = _bf16_from_bits(v_new_bits, self.device)
        self.append_device(kn, vn)

    def append_device(self, k_new, v_new):
        """Append one token per sequence from tensors that are already on the device (bf16 [B, Hkv, d])."""
        vb.vatt_append_kv(self.plan, k_new, v_new, self.k, self.v, self.block_table, self.seq_lens, self._stream())

    # ---- read-back -----------------------------------------------------------
    def scores_host(self) -> np.ndarray:
        """float32 [B, Hq, n_max] view of the score region of the workspace (copied to host)."""
        off = vb.vatt_plan_workspace_offset(self.plan, vb.VATT_WS_SCORES)
        stride = vb.vatt_plan_score_stride(self.plan)
        nbytes = self.B * self.Hq * stride * 4
        t = self.workspace[off:off + nbytes].view(torch.float32).view(self.B, self.Hq, stride)
        return t[:, :, :self.n_max].cpu().numpy()

    def results_host(self) -> Dict[str, np.ndarray]:
        torch.cuda.synchronize(self.device)
        return dict(
            O=self.out_o.cpu().numpy(), lse=self.out_lse.cpu().numpy(), idx=self.out_idx.cpu().numpy(),
            counts=self.out_counts.cpu().numpy(), b_star=self.out_budget_raw.cpu().numpy(),
            stats=self.out_stats.cpu().numpy(), seg=list(self.seg),
        )
