"""Pins for the oracle's decode attention.

Checked against: a pure-Python triple loop over the stored fields on a tiny
cache (brute force; it decodes every element from the packed bytes on its
own), the textbook softmax attention of a library routine when nothing is
quantised, closed-form special cases, and convergence to the unquantised
result.
"""
import math

import numpy as np
import pytest
import torch

from oracle import innerq_oracle as orc
from paper_2602_23200_amd import workloads as wl
from tests.helpers import oracle_config


def tiny(**kw):
    base = dict(name="t", batch=2, n_q_heads=4, n_kv_heads=2, head_dim=32, n_tokens=75,
                bits=2, group=16, w_sink=3, w_recent=8, seed=21, key_dist="student_t")
    base.update(kw)
    return wl.Workload(**base)


def brute_force_attention(cfg, cache, q16):
    """Loops only: decode each stored element from its bits, then softmax attention."""
    B, Hq, d = q16.shape
    G, ws, wr = cfg.group, cfg.w_sink, cfg.w_recent
    r = Hq // cfg.n_kv_heads
    N = cache.n_tokens
    out = np.zeros((B, Hq, d))

    def field_of(row_bytes, i, n, bits):
        """Field i of a packed run of n fields, read bit by bit from its bytes."""
        per = 8 // bits
        if bits != 3:
            return (int(row_bytes[i // per]) >> (bits * (i % per))) & ((1 << bits) - 1)
        lo = (int(row_bytes[i // 4]) >> (2 * (i % 4))) & 3          # plane of 2-bit low parts: n/4 bytes
        hi = (int(row_bytes[n // 4 + i // 8]) >> (i % 8)) & 1       # then the plane of high bits
        return lo + 4 * hi

    def fp(x):
        return float(x)

    def element(which, b, hk, t, c):
        form = cfg.form(which)
        n_mid = max(0, N - ws - wr)
        if form == orc.FORM_PER_CHANNEL:
            n_mid -= n_mid % G
        if t < ws:
            return fp(getattr(cache, which + "_sink")[b, hk, t, c])
        if t >= ws + n_mid:
            ring = getattr(cache, which + "_recent")
            return fp(ring[b, hk, t % ring.shape[2], c])
        row = t - ws
        codes = getattr(cache, which + "_codes")
        if form == orc.FORM_FP16:
            return fp(codes[b, hk, row, c])
        S = getattr(cache, which + "_scales")
        Z = getattr(cache, which + "_zeros")
        bits = cfg.v_bits if (which == "v" and cfg.v_bits) else cfg.bits
        if form == orc.FORM_PER_TOKEN:
            field = field_of(codes[b, hk, row], c, d, bits)
            s, z = S[b, hk, row, c // G], Z[b, hk, row, c // G]
        else:
            field = field_of(codes[b, hk, row // G, c], row % G, G, bits)
            s, z = S[b, hk, row // G, c], Z[b, hk, row // G, c]
        asym = bool(np.signbit(s))
        code = field if asym else field - (1 << (bits - 1))
        return abs(fp(s)) * code + (fp(z) if asym else 0.0)

    for b in range(B):
        for hq in range(Hq):
            hk = hq // r
            s = [sum(fp(q16[b, hq, c]) * element("k", b, hk, t, c) for c in range(d)) / math.sqrt(d)
                 for t in range(N)]
            m = max(s)
            e = [math.exp(x - m) for x in s]
            tot = sum(e)
            for c in range(d):
                out[b, hq, c] = sum(e[t] / tot * element("v", b, hk, t, c) for t in range(N))
    return out


@pytest.mark.parametrize("kind", [orc.KIND_INNER, orc.KIND_OUTER, orc.KIND_FP16])
@pytest.mark.parametrize("bits,mode", [(2, orc.HYBRID), (4, orc.ASYM), (4, orc.SYM), (3, orc.HYBRID), (3, orc.SYM),
                                       ((3, 2), orc.HYBRID), ((2, 4), orc.SYM)])
def test_attention_matches_brute_force_over_stored_bits(kind, bits, mode):
    v_bits = 0
    if isinstance(bits, tuple):
        bits, v_bits = bits
    w = tiny(bits=bits, k_mode=mode, v_mode=mode)
    cfg = oracle_config(w, kind=kind, capacity=96, v_bits=v_bits)
    K, V = wl.kv_full(w)
    cache = orc.cache_new(cfg)
    orc.quantize_append(cfg, cache, K, V)
    q = wl.query(w)
    got = orc.decode_attention(cfg, cache, q)
    want = brute_force_attention(cfg, cache, q)
    assert np.abs(got - want).max() <= 1e-12 * max(1.0, np.abs(want).max())


def test_nothing_quantised_equals_library_sdpa():
    """N <= w_sink + w_recent: every token is fp16, so the result is textbook attention."""
    w = tiny(n_tokens=11)
    for kind in (orc.KIND_INNER, orc.KIND_OUTER, orc.KIND_FP16):
        cfg = oracle_config(w, kind=kind, capacity=32)
        K, V = wl.kv_full(w)
        cache = orc.cache_init_prefill(cfg, K, V)
        q = wl.query(w)
        got = orc.decode_attention(cfg, cache, q)
        r = w.n_q_heads // w.n_kv_heads
        Kt = torch.from_numpy(K.astype(np.float64)).repeat_interleave(r, dim=1)
        Vt = torch.from_numpy(V.astype(np.float64)).repeat_interleave(r, dim=1)
        qt = torch.from_numpy(q.astype(np.float64))[:, :, None, :]
        want = torch.nn.functional.scaled_dot_product_attention(qt, Kt, Vt)[:, :, 0].numpy()
        assert np.abs(got - want).max() < 1e-12


def test_fp16_kind_equals_library_sdpa_at_any_length():
    w = tiny(n_tokens=75)
    cfg = oracle_config(w, kind=orc.KIND_FP16, capacity=96)
    K, V = wl.kv_full(w)
    cache = orc.cache_new(cfg)
    orc.quantize_append(cfg, cache, K, V)
    q = wl.query(w)
    got = orc.decode_attention(cfg, cache, q)
    r = w.n_q_heads // w.n_kv_heads
    Kt = torch.from_numpy(K.astype(np.float64)).repeat_interleave(r, dim=1)
    Vt = torch.from_numpy(V.astype(np.float64)).repeat_interleave(r, dim=1)
    qt = torch.from_numpy(q.astype(np.float64))[:, :, None, :]
    want = torch.nn.functional.scaled_dot_product_attention(qt, Kt, Vt)[:, :, 0].numpy()
    assert np.abs(got - want).max() < 1e-12


def test_identical_keys_give_the_mean_of_values():
    w = tiny(n_tokens=60)
    cfg = oracle_config(w, capacity=64)
    K, V = wl.kv_full(w)
    K[:] = K[:, :, :1]                      # every token has the same key
    cache = orc.cache_init_prefill(cfg, K, V)
    got = orc.decode_attention(cfg, cache, wl.query(w))
    r = w.n_q_heads // w.n_kv_heads
    for b in range(w.batch):
        for hk in range(w.n_kv_heads):
            # quantisation of identical rows is identical for per-token groups, so the
            # scores are still equal wherever the key is quantised the same way ...
            Ve = orc.effective_tensor(cfg, cache, "v", b, hk)
            Ke = orc.effective_tensor(cfg, cache, "k", b, hk)
            n_s, n_q, _ = orc.partition(cfg, "k", 60)
            assert np.all(Ke[n_s:n_s + n_q] == Ke[n_s])
    # ... and with a zero query the scores are all equal exactly: output = mean of effective V
    q0 = np.zeros_like(wl.query(w))
    got = orc.decode_attention(cfg, cache, q0)
    for b in range(w.batch):
        for hq in range(w.n_q_heads):
            Ve = orc.effective_tensor(cfg, cache, "v", b, hq // r)
            assert np.abs(got[b, hq] - Ve.mean(0)).max() < 1e-13


def test_one_dominant_key_selects_its_value_row():
    """A query aligned with one fp16 (recent) key of huge norm -> output is that token's value."""
    w = tiny(n_tokens=70, key_dist="normal")
    cfg = oracle_config(w, capacity=96)
    K, V = wl.kv_full(w)
    q = wl.query(w)
    t_star = 68                                            # inside the recent window
    K[:, :, t_star] = 0
    K[:, :, t_star, 0] = 200.0
    q[:] = 0
    q[:, :, 0] = 50.0
    cache = orc.cache_init_prefill(cfg, K, V)
    got = orc.decode_attention(cfg, cache, q)
    r = w.n_q_heads // w.n_kv_heads
    for hq in range(w.n_q_heads):
        assert np.abs(got[:, hq] - V[:, hq // r, t_star].astype(np.float64)).max() < 1e-9


def test_more_bits_converge_to_unquantised_attention():
    """Error against the fp16 cache shrinks with the bit width (2 -> 3 -> 4 -> 8 bits)."""
    w = tiny(n_tokens=75, group=16)
    K, V = wl.kv_full(w)
    q = wl.query(w)
    ref_cfg = oracle_config(w, kind=orc.KIND_FP16, capacity=96)
    ref = orc.decode_attention(ref_cfg, orc.cache_init_prefill(ref_cfg, K, V), q)
    errs = []
    for bits in (2, 3, 4, 8):
        cfg = oracle_config(w.with_(bits=bits), capacity=96)
        out = orc.decode_attention(cfg, orc.cache_init_prefill(cfg, K, V), q)
        errs.append(np.abs(out - ref).max())
    assert errs[0] > errs[1] > errs[2] > errs[3]
    assert errs[3] < 2e-2 * np.abs(ref).max()


def test_folded_and_unfolded_key_norm_agree():
    """Caller-folded (q*n, K/n given) and library-applied (k_inv_norm, q_scale) are the same bits."""
    w = tiny(n_tokens=75)
    cfg = oracle_config(w, capacity=96)
    K, V = wl.kv_full(w)
    q = wl.query(w)
    norm, inv = orc.calibrate_key_norm(K, per_head=True)
    unfolded = orc.decode_attention(cfg, orc.cache_init_prefill(cfg, K, V, k_inv_norm=inv), q, q_scale=norm)
    Kf, qf = orc.apply_channel_scale(K, inv), orc.apply_channel_scale(q, norm)
    folded = orc.decode_attention(cfg, orc.cache_init_prefill(cfg, Kf, V), qf)
    assert np.array_equal(folded, unfolded)
    # and on an fp16 cache normalisation changes the result only by fp16 rounding of K/n, q*n
    cfg16 = oracle_config(w, kind=orc.KIND_FP16, capacity=96)
    plain = orc.decode_attention(cfg16, orc.cache_init_prefill(cfg16, K, V), q)
    normed = orc.decode_attention(cfg16, orc.cache_init_prefill(cfg16, Kf, V), qf)
    assert np.abs(plain - normed).max() < 2e-2 * np.abs(plain).max()


def test_heads_subset_matches_full():
    w = tiny()
    cfg = oracle_config(w, capacity=96)
    K, V = wl.kv_full(w)
    cache = orc.cache_init_prefill(cfg, K, V)
    q = wl.query(w)
    full = orc.decode_attention(cfg, cache, q)
    part = orc.decode_attention(cfg, cache, q, heads=[(1, 0)])
    assert np.array_equal(part[1, 0:2], full[1, 0:2]) and np.isnan(part[0]).all()
