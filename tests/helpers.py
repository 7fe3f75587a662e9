"""Glue shared by the tests: workload -> oracle config, buffer comparison."""
import numpy as np

from oracle import innerq_oracle as orc
from paper_2602_23200_amd import workloads as wl


def oracle_config(w: wl.Workload, kind=orc.KIND_INNER, capacity=None, sym_denominator=0, **over) -> orc.Config:
    cap = capacity if capacity is not None else -(-(w.n_tokens + 2 * w.group) // w.group) * w.group
    cfg = orc.Config(batch=w.batch, n_q_heads=w.n_q_heads, n_kv_heads=w.n_kv_heads,
                     head_dim=w.head_dim, bits=w.bits, group=w.group, w_sink=w.w_sink,
                     w_recent=w.w_recent, k_mode=w.k_mode, v_mode=w.v_mode,
                     sym_denominator=sym_denominator, kind=kind, capacity_tokens=cap)
    for k, v in over.items():
        setattr(cfg, k, v)
    return cfg


CACHE_FIELDS = ("k_codes", "k_scales", "k_zeros", "v_codes", "v_scales", "v_zeros",
                "k_sink", "v_sink", "k_recent", "v_recent")


def bits_view(a: np.ndarray) -> np.ndarray:
    """Reinterpret fp16 as uint16 so that -0.0 / +0.0 and NaN payloads compare by bits."""
    return a.view(np.uint16) if a.dtype == np.float16 else a
