"""Shared helpers for the library tests: workload -> vatt_params fields."""
import numpy as np


def plan_params(wl, paged=False, page=16, num_blocks=0, n_max=None, **over):
    p = dict(
        batch=wl.batch, n_q_heads=wl.n_q_heads, n_kv_heads=wl.n_kv_heads, head_dim=wl.head_dim,
        n_max=wl.n_max if n_max is None else n_max,
        kv_layout=1 if paged else 0, page_size=page if paged else 0, num_blocks=num_blocks if paged else 0,
        sink=int(wl.params["sink"]), window=int(wl.params["window"]),
        topk_abs=int(wl.params.get("topk_abs", 0)), topk_frac=float(wl.params.get("topk_frac", 0.0)),
        base_abs=int(wl.params.get("base_abs", 0)), base_frac=float(wl.params.get("base_frac", 0.0)),
        epsilon=float(wl.params["epsilon"]), delta=float(wl.params["delta"]),
        target=int(wl.params.get("target", 0)), sm_scale=float(wl.params["sm_scale"]),
        budget_cap_frac=float(wl.params.get("budget_cap_frac", 1.0)),
    )
    p.update(over)
    return p
