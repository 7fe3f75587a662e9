"""Pins for the oracle's cache state machine (windows, eviction, partition).

Checked against: the partition written out as a closed form of N, verbatim
copies of the input rows in the fp16 windows, the eviction cadence the paper
states (one key token per step, G value tokens every G steps; the reverse for
outer-dimension grouping), and independence of the result from how the tokens
were chunked (bulk initialisation at the end of prefill vs one token at a time).
"""
import numpy as np
import pytest

from oracle import innerq_oracle as orc
from paper_2602_23200_amd import workloads as wl
from tests.helpers import CACHE_FIELDS, bits_view, oracle_config


def small_workload(**kw):
    base = dict(name="t", batch=2, n_q_heads=4, n_kv_heads=2, head_dim=64, n_tokens=200,
                bits=2, group=32, w_sink=4, w_recent=16, seed=9)
    base.update(kw)
    return wl.Workload(**base)


def closed_form(N, ws, wr, G):
    n_s = min(N, ws)
    n_qK = max(0, N - ws - wr)
    n_qV = (n_qK // G) * G
    return n_s, n_qK, n_qV, N - n_s - n_qK, N - n_s - n_qV


@pytest.mark.parametrize("kind", [orc.KIND_INNER, orc.KIND_OUTER, orc.KIND_FP16])
def test_partition_closed_form_sweep(kind):
    w = small_workload()
    cfg = oracle_config(w, kind=kind)
    for N in range(0, 400):
        n_s, n_qK, n_qV, n_rK, n_rV = closed_form(N, w.w_sink, w.w_recent, w.group)
        pk, pv = orc.partition(cfg, "k", N), orc.partition(cfg, "v", N)
        if kind == orc.KIND_INNER:
            assert pk == (n_s, n_qK, n_rK) and pv == (n_s, n_qV, n_rV)
        elif kind == orc.KIND_OUTER:
            assert pk == (n_s, n_qV, n_rV) and pv == (n_s, n_qK, n_rK)
        else:
            assert pk == pv == (n_s, n_qK, n_rK)
        # the token-grouped tensor keeps between w_recent and w_recent+G-1 recent tokens
        if N >= w.w_sink + w.w_recent:
            assert w.w_recent <= n_rV <= w.w_recent + w.group - 1 and n_rK == w.w_recent


def test_baseline_config_counts():
    """Derived counts of the five benchmark configurations."""
    want = {"tiny": (476, 448, 60), "llama2_7b_4k": (3964, 3936, 156),
            "llama3_8b_32k": (32636, 32608, 156), "mistral_7b_8k": (8060, 8000, 188),
            "llama3_8b_128k_32L": (130940, 130912, 156)}
    for name, (n_qK, n_qV, n_rV) in want.items():
        w = wl.WORKLOADS[name]
        cfg = oracle_config(w)
        assert orc.partition(cfg, "k", w.n_tokens)[1] == n_qK
        assert orc.partition(cfg, "v", w.n_tokens)[1:] == (n_qV, n_rV)


@pytest.mark.parametrize("kind", [orc.KIND_INNER, orc.KIND_OUTER, orc.KIND_FP16])
@pytest.mark.parametrize("N", [3, 4, 19, 20, 21, 51, 52, 53, 84, 200])
def test_windows_are_verbatim_and_eviction_cadence(kind, N):
    w = small_workload(n_tokens=N)
    cfg = oracle_config(w, kind=kind, capacity=256)
    K, V = wl.kv_full(w)
    cache = orc.cache_new(cfg)
    evicted = {"k": [], "v": []}
    for t in range(N):
        before = {x: orc.partition(cfg, x, cache.n_tokens)[1] for x in "kv"}
        orc.append_token(cfg, cache, K[:, :, t], V[:, :, t])
        for x in "kv":
            evicted[x].append(orc.partition(cfg, x, cache.n_tokens)[1] - before[x])
    assert cache.n_tokens == N
    for x, X in (("k", K), ("v", V)):
        n_s, n_q, n_r = orc.partition(cfg, x, N)
        sink = getattr(cache, x + "_sink")
        ring = getattr(cache, x + "_recent")
        assert np.array_equal(bits_view(sink[:, :, :n_s]), bits_view(X[:, :, :n_s]))
        for t in range(n_s + n_q, N):
            assert np.array_equal(bits_view(ring[:, :, t % ring.shape[2]]), bits_view(X[:, :, t]))
        # cadence: per-token form evicts 0/1 token per step, token-grouped form 0 or G
        ev = set(evicted[x])
        if cfg.form(x) == orc.FORM_PER_CHANNEL:
            assert ev <= {0, w.group}
        else:
            assert ev <= {0, 1}
            steady = evicted[x][w.w_sink + w.w_recent:]
            assert all(e == 1 for e in steady)


@pytest.mark.parametrize("kind", [orc.KIND_INNER, orc.KIND_OUTER, orc.KIND_FP16])
@pytest.mark.parametrize("bits,mode", [(2, orc.HYBRID), (4, orc.SYM), (4, orc.ASYM), (3, orc.HYBRID)])
def test_chunking_independence_bulk_vs_token_by_token(kind, bits, mode):
    w = small_workload(n_tokens=157, bits=bits, k_mode=mode, v_mode=mode)
    cfg = oracle_config(w, kind=kind, capacity=192)
    K, V = wl.kv_full(w)
    for N in (2, 20, 21, 85, 157):
        bulk = orc.cache_init_prefill(cfg, K[:, :, :N], V[:, :, :N])
        step = orc.cache_new(cfg)
        orc.quantize_append(cfg, step, K[:, :, :N], V[:, :, :N])
        # prefill of 60 then decode appends
        mixed = orc.cache_init_prefill(cfg, K[:, :, :min(N, 60)], V[:, :, :min(N, 60)])
        orc.quantize_append(cfg, mixed, K[:, :, min(N, 60):N], V[:, :, min(N, 60):N])
        for other in (step, mixed):
            assert other.n_tokens == bulk.n_tokens == N
            for f in CACHE_FIELDS:
                a, b = getattr(bulk, f), getattr(other, f)
                if a is None:
                    assert b is None
                    continue
                if f.endswith("recent"):
                    # stale ring slots differ (they held tokens evicted since); compare live slots
                    x = f[0]
                    n_s, n_q, _ = orc.partition(cfg, x, N)
                    live = [t % a.shape[2] for t in range(n_s + n_q, N)]
                    a, b = a[:, :, live], b[:, :, live]
                assert np.array_equal(bits_view(a), bits_view(b)), f


def test_quantised_store_holds_the_middle_tokens():
    """Dequantising the store gives back tokens [ws, ws+n_q) to within half a step."""
    w = small_workload(n_tokens=150, bits=4, k_mode=orc.ASYM, v_mode=orc.ASYM)
    cfg = oracle_config(w, capacity=192)
    K, V = wl.kv_full(w)
    cache = orc.cache_init_prefill(cfg, K, V)
    for x, X in (("k", K), ("v", V)):
        n_s, n_q, n_r = orc.partition(cfg, x, 150)
        eff = orc.effective_tensor(cfg, cache, x, 1, 0)
        assert np.array_equal(eff[:n_s], X[1, 0, :n_s].astype(np.float64))
        assert np.array_equal(eff[n_s + n_q:], X[1, 0, n_s + n_q:].astype(np.float64))
        mid = X[1, 0, n_s:n_s + n_q].astype(np.float64)
        rng = (mid.max() - mid.min())
        assert np.abs(eff[n_s:n_s + n_q] - mid).max() <= rng / 15 / 2 * 1.01
        # and it is the right tokens, not a permutation of them
        assert np.abs(eff[n_s:n_s + n_q] - mid).max() < 0.3 * np.abs(mid - np.roll(mid, 1, axis=0)).mean()


def test_key_inv_norm_applied_at_append_equals_prescaled_input():
    w = small_workload(n_tokens=90, key_dist="student_t")
    cfg = oracle_config(w, capacity=128)
    K, V = wl.kv_full(w)
    norm, inv = orc.calibrate_key_norm(K, per_head=True)
    a = orc.cache_init_prefill(cfg, K, V, k_inv_norm=inv)
    b = orc.cache_init_prefill(cfg, orc.apply_channel_scale(K, inv), V)
    c = orc.cache_new(cfg)
    orc.quantize_append(cfg, c, K, V, k_inv_norm=inv)
    for f in ("k_codes", "k_scales", "k_zeros", "k_sink", "v_codes"):
        assert np.array_equal(bits_view(getattr(a, f)), bits_view(getattr(b, f)))
        assert np.array_equal(bits_view(getattr(a, f)), bits_view(getattr(c, f)))
