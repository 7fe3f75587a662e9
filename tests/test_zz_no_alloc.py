"""innerq_decode_attention_static (split-K partials in the library's static device array, for callers
that cannot allocate) against innerq_decode_attention on the same caches, through the raw C ABI.

Both calls run the same kernels with the same launch plan, so the outputs must be bit-identical; the
oracle bar (2e-3) is checked as well.  Two calls in a row share the one array: the second uses a
smaller cache, so stale partials of the first call would show.
"""
import ctypes as C

import numpy as np
import pytest

from oracle import innerq_oracle as orc
from paper_2602_23200_amd import workloads as wl
from tests.helpers import gpu_config, max_rel_err, oracle_config

pytestmark = pytest.mark.gpu
TOL = 2e-3


def _case(torch, iq, w):
    """Prefilled cache + query on the device, and the oracle's output for it."""
    o = oracle_config(w)
    K, V = wl.kv_full(w)
    q = wl.query(w)
    g = iq.allocate_cache(gpu_config(o))
    iq.innerq_quantize_append(g, torch.from_numpy(K).cuda(), torch.from_numpy(V).cuda())
    want = orc.decode_attention(o, orc.cache_init_prefill(o, K, V), q)
    return g, torch.from_numpy(q).cuda(), want


def test_static_workspace_entry_matches_the_workspace_entry_on_two_calls_in_a_row():
    import torch
    from paper_2602_23200_amd import binding as iq
    assert torch.cuda.is_available(), "needs the MI355X"
    L = iq.lib()
    stream = torch.cuda.current_stream().cuda_stream or None
    big = wl.Workload(name="big", batch=2, n_q_heads=8, n_kv_heads=2, head_dim=128, n_tokens=3000, bits=2,
                      group=32, w_sink=4, w_recent=48, seed=41, key_dist="student_t")
    little = big.with_(name="little", batch=1, n_q_heads=4, n_kv_heads=1, n_tokens=389, seed=42)
    for w in (big, little):                                  # second call: smaller input, same array
        g, qd, want = _case(torch, iq, w)
        ws = iq.allocate_workspace(g.cfg)
        ref = torch.empty(qd.shape, dtype=torch.float32, device="cuda")
        got = torch.full(qd.shape, float("nan"), dtype=torch.float32, device="cuda")
        st = L.innerq_decode_attention(C.byref(g.cfg), C.byref(g.c), qd.data_ptr(), None, ref.data_ptr(), 1,
                                       ws.data_ptr(), ws.numel(), stream)
        assert st == iq.OK
        st = L.innerq_decode_attention_static(C.byref(g.cfg), C.byref(g.c), qd.data_ptr(), None, got.data_ptr(), 1,
                                              stream)
        assert st == iq.OK, iq.status_string(st)
        torch.cuda.synchronize()
        assert torch.equal(got, ref), f"{w.name}: static-workspace output differs from the workspace call"
        assert max_rel_err(got.cpu().numpy(), want) <= TOL, w.name
