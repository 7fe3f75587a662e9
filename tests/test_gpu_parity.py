"""GPU parity: the HIP path (through the C ABI) against the CPU oracle on the same seeded inputs.

Integer / byte / flag results (packed codes, fp16 scale and zero-point bits, window
contents) must be bit-exact; attention outputs must be within 2e-3 of the oracle,
measured as max|got - want| / max|want| per (batch, head) row.
"""
import numpy as np
import pytest

from oracle import innerq_oracle as orc
from paper_2602_23200_amd import workloads as wl
from tests.helpers import (assert_cache_equal, midpoint_scale_and_values, gpu_buffer_as_numpy, gpu_config, max_rel_err,
                           oracle_config)

pytestmark = pytest.mark.gpu
TOL = 2e-3


@pytest.fixture(scope="module")
def env():
    import torch
    from paper_2602_23200_amd import binding as iq
    assert torch.cuda.is_available(), "these tests need the MI355X"
    iq.lib()
    return torch, iq


def small(**kw):
    base = dict(name="s", batch=2, n_q_heads=8, n_kv_heads=2, head_dim=128, n_tokens=700,
                bits=2, group=32, w_sink=4, w_recent=48, seed=31, key_dist="student_t")
    base.update(kw)
    return wl.Workload(**base)


def to_dev(torch, a):
    return torch.from_numpy(np.ascontiguousarray(a)).cuda()


KINDS = [orc.KIND_INNER, orc.KIND_OUTER, orc.KIND_FP16]
QUANT_CASES = [(2, 32, orc.HYBRID), (2, 64, orc.HYBRID), (4, 32, orc.HYBRID), (4, 64, orc.ASYM),
               (2, 32, orc.SYM), (4, 32, orc.SYM), (3, 32, orc.HYBRID), (3, 64, orc.HYBRID), (3, 32, orc.SYM)]


@pytest.mark.parametrize("kind", KINDS)
@pytest.mark.parametrize("bits,group,mode", QUANT_CASES)
def test_bulk_append_bit_exact(env, kind, bits, group, mode):
    torch, iq = env
    if kind == orc.KIND_FP16 and (bits, group, mode) != QUANT_CASES[0]:
        pytest.skip("fp16 cache does not depend on the quantiser settings")
    w = small(bits=bits, group=group, k_mode=mode, v_mode=mode)
    o = oracle_config(w, kind=kind)
    K, V = wl.kv_full(w)
    want = orc.cache_init_prefill(o, K, V)
    g = iq.allocate_cache(gpu_config(o))
    iq.innerq_quantize_append(g, to_dev(torch, K), to_dev(torch, V))
    torch.cuda.synchronize()
    assert_cache_equal(g, want, o, what=f"kind{kind} b{bits} G{group} m{mode}")
    if mode == orc.HYBRID and kind != orc.KIND_FP16:
        M = np.signbit(gpu_buffer_as_numpy(g, o, "v_scales"))
        assert M.any() and not M.all()          # both branches of the hybrid rule were exercised


@pytest.mark.parametrize("sym_den", [0, 1])
def test_symmetric_denominator_readings_bit_exact(env, sym_den):
    torch, iq = env
    w = small(k_mode=orc.SYM, v_mode=orc.HYBRID, n_tokens=300)
    o = oracle_config(w, sym_denominator=sym_den)
    K, V = wl.kv_full(w)
    want = orc.cache_init_prefill(o, K, V)
    g = iq.allocate_cache(gpu_config(o))
    iq.innerq_quantize_append(g, to_dev(torch, K), to_dev(torch, V))
    torch.cuda.synchronize()
    assert_cache_equal(g, want, o)


@pytest.mark.parametrize("kind", KINDS)
def test_incremental_appends_bit_exact_and_chunking_independent(env, kind):
    """Prefill chunk, then single-token decode steps across several evictions and value spills,
    then a ragged multi-token chunk: every stage equals the oracle's token-by-token cache."""
    torch, iq = env
    w = small(n_tokens=420, group=32, w_recent=40)
    o = oracle_config(w, kind=kind)
    K, V = wl.kv_full(w)
    Kd, Vd = to_dev(torch, K), to_dev(torch, V)
    want = orc.cache_new(o)
    g = iq.allocate_cache(gpu_config(o))
    pos = 0
    for step in [3, 1, 1, 60, 1] + [1] * 150 + [37, 1, 1, 100, 1, 1]:
        if pos + step > w.n_tokens:
            break
        orc.quantize_append(o, want, K[:, :, pos:pos + step], V[:, :, pos:pos + step])
        iq.innerq_quantize_append(g, Kd[:, :, pos:pos + step].contiguous(), Vd[:, :, pos:pos + step].contiguous())
        pos += step
        if step != 1 or pos % 16 == 0:
            torch.cuda.synchronize()
            assert_cache_equal(g, want, o, what=f"after {pos} tokens")
    torch.cuda.synchronize()
    assert_cache_equal(g, want, o, what="final")
    bulk = iq.allocate_cache(gpu_config(o))
    iq.innerq_quantize_append(bulk, Kd[:, :, :pos].contiguous(), Vd[:, :, :pos].contiguous())
    torch.cuda.synchronize()
    assert_cache_equal(bulk, want, o, what="bulk")


@pytest.mark.parametrize("per_head", [False, True])
def test_calibrate_key_norm_exact(env, per_head):
    torch, iq = env
    w = small(n_tokens=2500, batch=3, n_kv_heads=4, n_q_heads=8)
    o = oracle_config(w)
    K, _ = wl.kv_full(w)
    K[:, 1, :, 17] = 0                                   # a dead channel -> norm 1
    want_n, want_i = orc.calibrate_key_norm(K, per_head)
    n, i = iq.innerq_calibrate_key_norm(gpu_config(o), to_dev(torch, K), per_head)
    torch.cuda.synchronize()
    assert np.array_equal(n.cpu().numpy(), want_n)
    assert np.array_equal(i.cpu().numpy(), want_i)


def run_attention(torch, iq, o, K, V, q, k_inv_norm=None, q_scale=None, fp16_out=False):
    g = iq.allocate_cache(gpu_config(o))
    inv = None if k_inv_norm is None else to_dev(torch, k_inv_norm)
    iq.innerq_quantize_append(g, to_dev(torch, K), to_dev(torch, V), k_inv_norm=inv)
    ws = iq.allocate_workspace(g.cfg)
    out = torch.empty(q.shape, dtype=torch.float16, device="cuda") if fp16_out else None
    qs = None if q_scale is None else to_dev(torch, q_scale)
    out = iq.innerq_decode_attention(g, to_dev(torch, q), ws, out=out, q_scale=qs)
    torch.cuda.synchronize()
    return g, out.float().cpu().numpy()


@pytest.mark.parametrize("kind", KINDS)
@pytest.mark.parametrize("bits,group,mode", QUANT_CASES)
def test_attention_small_all_variants(env, kind, bits, group, mode):
    torch, iq = env
    if kind == orc.KIND_FP16 and (bits, group, mode) != QUANT_CASES[0]:
        pytest.skip("fp16 cache does not depend on the quantiser settings")
    w = small(bits=bits, group=group, k_mode=mode, v_mode=mode, n_tokens=1237)
    o = oracle_config(w, kind=kind)
    K, V = wl.kv_full(w)
    q = wl.query(w)
    want = orc.decode_attention(o, orc.cache_init_prefill(o, K, V), q)
    _, got = run_attention(torch, iq, o, K, V, q)
    assert max_rel_err(got, want) <= TOL


@pytest.mark.parametrize("bits,mode", [(2, orc.SYM), (2, orc.HYBRID), (3, orc.HYBRID), (4, orc.SYM), (4, orc.HYBRID)])
def test_attention_keys_near_the_top_of_fp16(env, bits, mode):
    """Forty tokens spread over sink, quantised region and recent window carry keys up to 6e4 in
    magnitude, so that 2^(b-1) times the scale of a symmetric group lies beyond fp16: the
    zero-point term of the scores has to stay finite, and the softmax has to follow scores
    thousands of units apart."""
    torch, iq = env
    w = small(bits=bits, k_mode=mode, v_mode=mode, n_tokens=900)
    o = oracle_config(w)
    K, V = wl.kv_full(w)
    K = K.astype(np.float32)
    big = np.random.default_rng(5).choice(w.n_tokens, 40, replace=False)
    big[:3] = [1, 400, w.n_tokens - 2]
    K[:, :, big] *= 8192.0
    K = np.clip(K, -6.0e4, 6.0e4).astype(np.float16)
    q = wl.query(w)
    want = orc.decode_attention(o, orc.cache_init_prefill(o, K, V), q)
    assert np.isfinite(want).all()
    _, got = run_attention(torch, iq, o, K, V, q)
    assert np.isfinite(got).all()
    assert max_rel_err(got, want) <= TOL


@pytest.mark.parametrize("kind", [orc.KIND_INNER, orc.KIND_OUTER])
@pytest.mark.parametrize("log2_q", [-13, -6, 6])
@pytest.mark.parametrize("bits,mode", [(2, orc.SYM), (2, orc.HYBRID), (3, orc.HYBRID), (4, orc.HYBRID)])
def test_attention_query_magnitudes(env, bits, mode, log2_q, kind):
    """Queries scaled by 2^-13 (mostly fp16 denormals), 2^-6 and 2^6, keys scaled the other way so
    that the scores keep their size: the fused kernels' query tables carry a power of two per
    head (the outer-grouped one a second one per tile for the scales folded in), so their accuracy
    must not depend on the magnitude of q or of the keys."""
    torch, iq = env
    w = small(bits=bits, k_mode=mode, v_mode=mode, n_tokens=900)
    o = oracle_config(w, kind=kind)
    K, V = wl.kv_full(w)
    K = np.clip(K.astype(np.float32) * 2.0 ** (-log2_q - 1), -6.0e4, 6.0e4).astype(np.float16)
    q = (wl.query(w).astype(np.float32) * 2.0 ** log2_q).astype(np.float16)
    want = orc.decode_attention(o, orc.cache_init_prefill(o, K, V), q)
    _, got = run_attention(torch, iq, o, K, V, q)
    assert max_rel_err(got, want) <= TOL


@pytest.mark.parametrize("kind", [orc.KIND_INNER, orc.KIND_OUTER])
@pytest.mark.parametrize("order", ["rising", "falling"])
@pytest.mark.parametrize("bits,mode", [(2, orc.SYM), (2, orc.HYBRID), (4, orc.HYBRID)])
def test_attention_value_magnitudes_change_along_the_context(env, bits, mode, order, kind):
    """Values whose magnitude changes by 2^10 from one third of the context to the next, in both
    directions: the outer-grouped kernel folds the tokens' value scales into the softmax weights under
    a running power of two that has to follow the largest scale seen so far (and must not lose the
    small tokens while they are all there is); the other kernels must not care."""
    torch, iq = env
    w = small(bits=bits, k_mode=mode, v_mode=mode, n_tokens=1100)
    o = oracle_config(w, kind=kind)
    K, V = wl.kv_full(w)
    third = w.n_tokens // 3
    steps = [-10, 0, 10] if order == "rising" else [10, 0, -10]
    V = V.astype(np.float32)
    for i, e in enumerate(steps):
        V[:, :, i * third:(i + 1) * third if i < 2 else w.n_tokens] *= 2.0 ** e
    V = np.clip(V, -6.0e4, 6.0e4).astype(np.float16)
    q = wl.query(w)
    want = orc.decode_attention(o, orc.cache_init_prefill(o, K, V), q)
    _, got = run_attention(torch, iq, o, K, V, q)
    assert np.isfinite(got).all()
    assert max_rel_err(got, want) <= TOL
    # the small third on its own (a cache that never sees a large scale)
    n_small = third if order == "rising" else w.n_tokens - 2 * third
    sl = slice(0, third) if order == "rising" else slice(2 * third, w.n_tokens)
    w2 = small(bits=bits, k_mode=mode, v_mode=mode, n_tokens=n_small)
    o2 = oracle_config(w2, kind=kind)
    K2, V2 = np.ascontiguousarray(K[:, :, sl]), np.ascontiguousarray(V[:, :, sl])
    want2 = orc.decode_attention(o2, orc.cache_init_prefill(o2, K2, V2), q)
    _, got2 = run_attention(torch, iq, o2, K2, V2, q)
    assert max_rel_err(got2, want2) <= TOL


@pytest.mark.parametrize("n_tokens", [1, 2, 4, 5, 51, 52, 53, 83, 84, 85, 116, 117, 180])
@pytest.mark.parametrize("kind", [orc.KIND_INNER, orc.KIND_OUTER])
def test_attention_edge_lengths(env, kind, n_tokens):
    """Below, at and just above every boundary: sink only, windows only, first evicted key,
    first value spill (w_sink 4, w_recent 48, G 32)."""
    torch, iq = env
    w = small(n_tokens=n_tokens)
    o = oracle_config(w, kind=kind, capacity=256)
    K, V = wl.kv_full(w)
    q = wl.query(w)
    want = orc.decode_attention(o, orc.cache_init_prefill(o, K, V), q)
    _, got = run_attention(torch, iq, o, K, V, q)
    assert max_rel_err(got, want) <= TOL


@pytest.mark.parametrize("kind", [orc.KIND_INNER, orc.KIND_OUTER])
@pytest.mark.parametrize("heads", [(4, 4), (2, 1), (16, 2), (12, 4)])
def test_attention_head_ratios(env, heads, kind):
    torch, iq = env
    hq, hk = heads
    w = small(n_q_heads=hq, n_kv_heads=hk, n_tokens=600)
    o = oracle_config(w, kind=kind)
    K, V = wl.kv_full(w)
    q = wl.query(w)
    want = orc.decode_attention(o, orc.cache_init_prefill(o, K, V), q)
    _, got = run_attention(torch, iq, o, K, V, q)
    assert max_rel_err(got, want) <= TOL


def test_attention_no_sink_window(env):
    torch, iq = env
    w = small(w_sink=0, n_tokens=500)
    o = oracle_config(w)
    K, V = wl.kv_full(w)
    q = wl.query(w)
    want = orc.decode_attention(o, orc.cache_init_prefill(o, K, V), q)
    _, got = run_attention(torch, iq, o, K, V, q)
    assert max_rel_err(got, want) <= TOL


def test_attention_after_decode_steps_and_fp16_output(env):
    """Attention right after single-token appends (ring wrapped several times), fp16 output."""
    torch, iq = env
    w = small(n_tokens=400, w_recent=40)
    o = oracle_config(w)
    K, V = wl.kv_full(w)
    q = wl.query(w)
    want_cache = orc.cache_new(o)
    orc.quantize_append(o, want_cache, K, V)
    want = orc.decode_attention(o, want_cache, q)
    g = iq.allocate_cache(gpu_config(o))
    Kd, Vd = to_dev(torch, K), to_dev(torch, V)
    iq.innerq_quantize_append(g, Kd[:, :, :250].contiguous(), Vd[:, :, :250].contiguous())
    for t in range(250, 400):
        iq.innerq_quantize_append(g, Kd[:, :, t:t + 1].contiguous(), Vd[:, :, t:t + 1].contiguous())
    ws = iq.allocate_workspace(g.cfg)
    out32 = iq.innerq_decode_attention(g, to_dev(torch, q), ws)
    out16 = torch.empty(q.shape, dtype=torch.float16, device="cuda")
    iq.innerq_decode_attention(g, to_dev(torch, q), ws, out=out16)
    torch.cuda.synchronize()
    assert max_rel_err(out32.cpu().numpy(), want) <= TOL
    assert max_rel_err(out16.float().cpu().numpy(), want) <= TOL + 2.0 ** -10


def test_key_norm_unfolded_path_matches_oracle_and_folded(env):
    torch, iq = env
    w = small(n_tokens=900)
    o = oracle_config(w)
    K, V = wl.kv_full(w)
    q = wl.query(w)
    norm, inv = orc.calibrate_key_norm(K, per_head=True)
    want_cache = orc.cache_init_prefill(o, K, V, k_inv_norm=inv)
    want = orc.decode_attention(o, want_cache, q, q_scale=norm)
    g, got = run_attention(torch, iq, o, K, V, q, k_inv_norm=inv, q_scale=norm)
    assert_cache_equal(g, want_cache, o)
    assert max_rel_err(got, want) <= TOL
    Kf, qf = orc.apply_channel_scale(K, inv), orc.apply_channel_scale(q, norm)
    g2, got2 = run_attention(torch, iq, o, Kf, V, qf)
    assert_cache_equal(g2, want_cache, o)
    assert np.array_equal(got, got2)


@pytest.mark.parametrize("kind", KINDS)
def test_key_norm_keeps_the_fp32_rounding_of_the_product(env, kind):
    """Keys and queries chosen so that rounding the exact product K x inv_norm (q x norm) once gives
    a different fp16 value than rounding it to fp32 first: windows, codes and scales must still be
    the oracle's, bit for bit."""
    torch, iq = env
    w = small(n_tokens=4 + 16 * 32 + 32, batch=1, n_kv_heads=2, n_q_heads=4)
    o = oracle_config(w, kind=kind)
    ks = [midpoint_scale_and_values(w.head_dim, w.n_tokens, seed=h, lo_exp=-1, hi_exp=3) for h in range(w.n_kv_heads)]
    inv = np.stack([k[0] for k in ks])
    K = np.stack([k[1] for k in ks])[None]
    V = wl.kv_full(w)[1]
    r = w.n_q_heads // w.n_kv_heads
    # the query factor need not be the reciprocal of the key factor for this check
    qs = [midpoint_scale_and_values(w.head_dim, r, seed=50 + h, lo_exp=-6, hi_exp=-3) for h in range(w.n_kv_heads)]
    norm = np.stack([x[0] for x in qs])
    q = np.concatenate([x[1] for x in qs])[None]
    want_cache = orc.cache_init_prefill(o, K, V, k_inv_norm=inv)
    want = orc.decode_attention(o, want_cache, q, q_scale=norm)
    g, got = run_attention(torch, iq, o, K, V, q, k_inv_norm=inv, q_scale=norm)
    assert_cache_equal(g, want_cache, o)
    assert max_rel_err(got, want) <= TOL


@pytest.mark.parametrize("name", ["tiny", "llama2_7b_4k"])
def test_attention_baseline_configs_full(env, name):
    torch, iq = env
    w = wl.WORKLOADS[name]
    o = oracle_config(w)
    K, V = wl.kv_full(w)
    q = wl.query(w)
    want_cache = orc.cache_init_prefill(o, K, V)
    want = orc.decode_attention(o, want_cache, q)
    g, got = run_attention(torch, iq, o, K, V, q)
    assert_cache_equal(g, want_cache, o)
    assert max_rel_err(got, want) <= TOL


@pytest.mark.parametrize("name,slabs", [("llama3_8b_32k", [(0, 0), (3, 5), (7, 7)]),
                                         ("mistral_7b_8k", [(0, 0), (17, 3), (31, 7)])])
def test_attention_baseline_configs_full_size_sampled(env, name, slabs):
    """Full-size cache on the GPU in the launch configuration the benchmark times; the oracle
    recomputes sampled (batch, kv-head) slabs on their own: packed bytes bit-exact, outputs in tolerance."""
    torch, iq = env
    w = wl.WORKLOADS[name]
    o = oracle_config(w)
    B, Hk, N, d = w.batch, w.n_kv_heads, w.n_tokens, w.head_dim
    Kd = torch.empty((B, Hk, N, d), dtype=torch.float16, device="cuda")
    Vd = torch.empty_like(Kd)
    keep = {}
    for b in range(B):
        for h in range(Hk):
            k, v = wl.kv_slab(w, b, h)
            Kd[b, h].copy_(torch.from_numpy(k))
            Vd[b, h].copy_(torch.from_numpy(v))
            if (b, h) in slabs:
                keep[(b, h)] = (k, v)
    q = wl.query(w)
    g = iq.allocate_cache(gpu_config(o))
    iq.innerq_quantize_append(g, Kd, Vd)
    ws = iq.allocate_workspace(g.cfg)
    got = iq.innerq_decode_attention(g, to_dev(torch, q), ws)
    torch.cuda.synchronize()
    got = got.cpu().numpy()
    assert np.isfinite(got).all()
    r = w.n_q_heads // w.n_kv_heads
    o1 = oracle_config(w.with_(batch=1, n_kv_heads=1, n_q_heads=r))
    for (b, h), (k, v) in keep.items():
        want_cache = orc.cache_init_prefill(o1, k[None, None], v[None, None])
        assert_cache_equal(g, want_cache, o1, bsel=slice(b, b + 1), hsel=slice(h, h + 1), what=f"slab {b},{h}")
        want = orc.decode_attention(o1, want_cache, q[b:b + 1, h * r:(h + 1) * r])
        assert max_rel_err(got[b:b + 1, h * r:(h + 1) * r], want) <= TOL


@pytest.mark.parametrize("layer", [0, 31])
def test_long_context_layer_full_size_sampled_with_folded_key_norm(env, layer):
    """One layer of the 128k-token configuration at full size, key normalisation folded the way the
    benchmark does it (factors calibrated over the prefill keys, keys divided on their way into the
    cache, the query multiplied).  The oracle recomputes two (batch, kv-head) slabs on their own."""
    torch, iq = env
    w = wl.WORKLOADS["llama3_8b_128k_32L"]
    o = oracle_config(w)
    B, Hk, N, d = w.batch, w.n_kv_heads, w.n_tokens, w.head_dim
    slabs = [(0, 0), (3, 7)]
    # the sampled slabs come from the host generator; the others are drawn on the device with the
    # same per-channel scales (the host generator needs minutes for a whole layer of this size)
    gen = torch.Generator(device="cuda")
    gen.manual_seed(1000 + layer)
    sigma = to_dev(torch, wl.key_channel_sigma(w, layer).astype(np.float32))       # [Hk, d]
    Kd = (torch.randn((B, Hk, N, d), device="cuda", generator=gen) * sigma[None, :, None, :]).half()
    Vd = torch.randn((B, Hk, N, d), device="cuda", generator=gen).half()
    keep = {}
    for (b, h) in slabs:
        k, v = wl.kv_slab(w, b, h, layer)
        Kd[b, h].copy_(torch.from_numpy(k))
        Vd[b, h].copy_(torch.from_numpy(v))
        keep[(b, h)] = (k, v)
    peak = Kd.abs().amax(dim=(0, 2)).cpu().numpy()[None, :, None, :]      # max |K| per head and channel
    norm, inv = orc.calibrate_key_norm(peak, per_head=False)
    cfg = gpu_config(o)
    got_norm, got_inv = iq.innerq_calibrate_key_norm(cfg, Kd, per_head=False)
    assert np.array_equal(got_norm.cpu().numpy(), norm)
    assert np.array_equal(got_inv.cpu().numpy(), inv)
    q = wl.query(w, layer)
    g = iq.allocate_cache(cfg)
    iq.innerq_quantize_append(g, Kd, Vd, k_inv_norm=to_dev(torch, inv))
    del Kd, Vd
    ws = iq.allocate_workspace(g.cfg)
    got = iq.innerq_decode_attention(g, to_dev(torch, q), ws, q_scale=to_dev(torch, norm))
    torch.cuda.synchronize()
    got = got.cpu().numpy()
    assert np.isfinite(got).all()
    r = w.n_q_heads // w.n_kv_heads
    o1 = oracle_config(w.with_(batch=1, n_kv_heads=1, n_q_heads=r))
    for (b, h), (k, v) in keep.items():
        want_cache = orc.cache_init_prefill(o1, k[None, None], v[None, None], k_inv_norm=inv[h:h + 1])
        assert_cache_equal(g, want_cache, o1, bsel=slice(b, b + 1), hsel=slice(h, h + 1),
                           what=f"layer {layer} slab {b},{h}")
        want = orc.decode_attention(o1, want_cache, q[b:b + 1, h * r:(h + 1) * r], q_scale=norm[h:h + 1])
        assert max_rel_err(got[b:b + 1, h * r:(h + 1) * r], want) <= TOL


@pytest.mark.parametrize("frac", [0.05, 0.6])
def test_crafted_flag_density_cache(env, frac):
    """The density sweep's crafted cache: flags of the HIP path equal the planned ones and the
    oracle's, group by group, and attention over it stays within tolerance."""
    torch, iq = env
    import bench
    w = small(n_tokens=4 + 48 + 12 * 32, bits=2, group=32, k_mode=orc.HYBRID, v_mode=orc.HYBRID)
    o = oracle_config(w)
    B, Hk, N, d, G = w.batch, w.n_kv_heads, w.n_tokens, w.head_dim, w.group
    gen = torch.Generator(device="cuda")
    gen.manual_seed(11)
    k, km = bench.crafted_groups(torch, gen, (B, Hk, N, d // G), G, w.bits, frac, return_mask=True)
    k = k.reshape(B, Hk, N, d).contiguous()
    n_grp = (N - w.w_sink) // G
    vg, vm = bench.crafted_groups(torch, gen, (B, Hk, n_grp, d), G, w.bits, frac, return_mask=True)
    v = torch.zeros((B, Hk, N, d), dtype=torch.float16, device="cuda")
    v[:, :, w.w_sink:w.w_sink + n_grp * G] = vg.permute(0, 1, 2, 4, 3).reshape(B, Hk, n_grp * G, d)
    g = iq.allocate_cache(gpu_config(o))
    iq.innerq_quantize_append(g, k, v)
    torch.cuda.synchronize()
    want = orc.cache_init_prefill(o, k.cpu().numpy(), v.cpu().numpy())
    assert_cache_equal(g, want, o, what=f"crafted {frac}")
    n_qk = N - w.w_sink - w.w_recent
    got_k = np.signbit(gpu_buffer_as_numpy(g, o, "k_scales"))[:, :, :n_qk]
    assert np.array_equal(got_k, km.cpu().numpy()[:, :, w.w_sink:w.w_sink + n_qk])
    n_qv = n_qk // G
    got_v = np.signbit(gpu_buffer_as_numpy(g, o, "v_scales"))[:, :, :n_qv]
    assert np.array_equal(got_v, vm.cpu().numpy()[:, :, :n_qv])
    q = wl.query(w)
    out = torch.empty((B, w.n_q_heads, d), dtype=torch.float32, device="cuda")
    iq.innerq_decode_attention(g, to_dev(torch, q), iq.allocate_workspace(gpu_config(o)), out=out)
    torch.cuda.synchronize()
    ref = orc.decode_attention(o, want, q, None)
    assert max_rel_err(out.cpu().numpy(), ref) <= TOL


@pytest.mark.parametrize("kind", [orc.KIND_INNER, orc.KIND_OUTER])
@pytest.mark.parametrize("k_bits,v_bits,group,k_mode,v_mode", [
    (3, 2, 32, orc.SYM, orc.HYBRID),      # the paper's Hybrid preset
    (3, 2, 32, orc.SYM, orc.SYM),         # Small
    (3, 3, 32, orc.SYM, orc.SYM),         # Base
    (3, 2, 64, orc.HYBRID, orc.HYBRID),
    (2, 4, 32, orc.HYBRID, orc.ASYM),     # a pair the fused kernel is not built for: generic path
])
def test_separate_key_and_value_widths(env, kind, k_bits, v_bits, group, k_mode, v_mode):
    """Caches whose keys and values have different code widths: stores bit-exact, attention within
    tolerance, after a bulk append followed by single-token appends (so that both quantiser
    paths and a value spill run at both widths)."""
    torch, iq = env
    w = small(bits=k_bits, group=group, k_mode=k_mode, v_mode=v_mode, n_tokens=900)
    o = oracle_config(w, kind=kind, v_bits=v_bits)
    K, V = wl.kv_full(w)
    n0 = 900 - 70
    want = orc.cache_init_prefill(o, K[:, :, :n0], V[:, :, :n0])
    orc.quantize_append(o, want, K[:, :, n0:], V[:, :, n0:])
    g = iq.allocate_cache(gpu_config(o))
    iq.innerq_quantize_append(g, to_dev(torch, K[:, :, :n0]), to_dev(torch, V[:, :, :n0]))
    for t in range(n0, 900):
        iq.innerq_quantize_append(g, to_dev(torch, K[:, :, t:t + 1]), to_dev(torch, V[:, :, t:t + 1]))
    torch.cuda.synchronize()
    assert_cache_equal(g, want, o, what=f"kind{kind} k{k_bits} v{v_bits} G{group}")
    q = wl.query(w)
    out = iq.innerq_decode_attention(g, to_dev(torch, q), iq.allocate_workspace(g.cfg))
    torch.cuda.synchronize()
    ref = orc.decode_attention(o, want, q)
    assert max_rel_err(out.cpu().numpy(), ref) <= TOL


@pytest.mark.parametrize("bits,v_bits,group,k_mode,v_mode", [
    (3, 0, 32, orc.HYBRID, orc.HYBRID), (4, 0, 32, orc.HYBRID, orc.HYBRID), (3, 2, 32, orc.SYM, orc.HYBRID),
    (3, 0, 64, orc.HYBRID, orc.HYBRID), (4, 0, 64, orc.ASYM, orc.SYM), (2, 0, 32, orc.SYM, orc.ASYM)])
def test_long_context_other_widths_with_key_norm(env, bits, v_bits, group, k_mode, v_mode):
    """32k tokens of the heavy-tailed workload at the widths, group sizes and modes the full-size
    layer tests do not reach, keys normalised on their way in: a quarter of a million groups per
    tensor must come out bit-exact (events of one in 10^4 show at this size, not at a few hundred
    tokens), and the long fused pass must stay within tolerance."""
    torch, iq = env
    w = wl.WORKLOADS["llama3_8b_32k"].with_(batch=1, n_kv_heads=2, n_q_heads=8, bits=bits, group=group,
                                             k_mode=k_mode, v_mode=v_mode, w_recent=128 if group == 64 else 32)
    o = oracle_config(w, v_bits=v_bits)
    K, V = wl.kv_full(w)
    q = wl.query(w)
    norm, inv = orc.calibrate_key_norm(K, per_head=True)
    want_cache = orc.cache_init_prefill(o, K, V, k_inv_norm=inv)
    want = orc.decode_attention(o, want_cache, q, q_scale=norm)
    g, got = run_attention(torch, iq, o, K, V, q, k_inv_norm=inv, q_scale=norm)
    assert_cache_equal(g, want_cache, o, what=f"k{bits} v{v_bits} G{group}")
    assert max_rel_err(got, want) <= TOL


@pytest.mark.parametrize("kind", KINDS)
def test_single_kv_head_long_context_uses_every_partial_slot(env, kind):
    """One (batch, kv-head) pair and 40k tokens: the launch wants more wavefronts than the split
    cap allows, so the number of partial results is set by the caps that size the workspace (the
    fused inner kernel's window-carrying wavefronts count against the split cap).  A guard band
    behind the workspace must stay untouched and the result must match the oracle."""
    torch, iq = env
    w = wl.WORKLOADS["llama3_8b_32k"].with_(batch=1, n_kv_heads=1, n_q_heads=4, n_tokens=40000)
    o = oracle_config(w, kind=kind)
    K, V = wl.kv_full(w)
    q = wl.query(w)
    want = orc.decode_attention(o, orc.cache_init_prefill(o, K, V), q)
    g = iq.allocate_cache(gpu_config(o))
    iq.innerq_quantize_append(g, to_dev(torch, K), to_dev(torch, V))
    need = iq.innerq_workspace_bytes(g.cfg)
    guard = 1 << 16
    buf = torch.full((need + guard,), 0x5A, dtype=torch.uint8, device="cuda")
    out = iq.innerq_decode_attention(g, to_dev(torch, q), buf[:need])
    torch.cuda.synchronize()
    assert bool((buf[need:] == 0x5A).all())
    assert max_rel_err(out.cpu().numpy(), want) <= TOL


def _random_case(i):
    r = np.random.default_rng(1000 + i)
    k_bits = int(r.choice([2, 3, 4]))
    v_bits = 2 if (k_bits == 3 and i % 2 == 0) else 0
    hk = int(r.choice([1, 2, 3]))
    ratio = int(r.choice([1, 2, 4, 5, 8]))
    group = int(r.choice([32, 64]))
    w_sink = int(r.choice([0, 1, 4, 7]))
    w_recent = int(r.choice([1, 16, 48, 130]))
    n_tokens = int(r.integers(1, 4200))
    modes = [orc.SYM, orc.ASYM, orc.HYBRID]
    return dict(batch=int(r.choice([1, 2])), n_q_heads=hk * ratio, n_kv_heads=hk, bits=k_bits, group=group,
                w_sink=w_sink, w_recent=w_recent, n_tokens=n_tokens, k_mode=modes[int(r.integers(3))],
                v_mode=modes[int(r.integers(3))], seed=500 + i), v_bits


@pytest.mark.parametrize("kind", [orc.KIND_INNER, orc.KIND_OUTER])
@pytest.mark.parametrize("i", range(24))
def test_random_configurations(env, i, kind):
    """Seeded random shapes, widths, modes, windows and lengths (ragged tiles, windows longer than
    the context, 1 to 8 query heads per kv head), for both groupings: cache bit-exact, attention
    within tolerance."""
    torch, iq = env
    kw, v_bits = _random_case(i)
    w = small(**kw)
    o = oracle_config(w, kind=kind, v_bits=v_bits)
    K, V = wl.kv_full(w)
    q = wl.query(w)
    want_cache = orc.cache_init_prefill(o, K, V)
    want = orc.decode_attention(o, want_cache, q)
    g, got = run_attention(torch, iq, o, K, V, q)
    assert_cache_equal(g, want_cache, o, what=str(kw))
    assert max_rel_err(got, want) <= TOL, (kw, v_bits)


# ---------------------------------------------------------------------------
# The second fused kernel for 2-bit caches (block-scaled fp8 x fp4 matrix instruction, off by
# default): same oracle, same tolerance.
# ---------------------------------------------------------------------------
@pytest.fixture
def f4_kernel(env):
    _, iq = env
    iq.innerq_select_inner_kernel(1)
    yield
    iq.innerq_select_inner_kernel(0)


@pytest.mark.parametrize("group,k_mode,v_mode", [(32, orc.HYBRID, orc.HYBRID), (64, orc.HYBRID, orc.HYBRID),
                                                  (32, orc.SYM, orc.SYM), (64, orc.SYM, orc.HYBRID),
                                                  (32, orc.ASYM, orc.SYM)])
@pytest.mark.parametrize("n_tokens", [181, 308, 1237, 2900])
def test_fp4_kernel_small(env, f4_kernel, group, k_mode, v_mode, n_tokens):
    """One tile, ragged tiles (the quantised range is no multiple of 128), several splits."""
    torch, iq = env
    w = small(bits=2, group=group, k_mode=k_mode, v_mode=v_mode, n_tokens=n_tokens)
    o = oracle_config(w)
    K, V = wl.kv_full(w)
    q = wl.query(w)
    want = orc.decode_attention(o, orc.cache_init_prefill(o, K, V), q)
    _, got = run_attention(torch, iq, o, K, V, q)
    assert max_rel_err(got, want) <= TOL


@pytest.mark.parametrize("heads", [(4, 4), (2, 1), (12, 4), (3, 1)])
def test_fp4_kernel_head_ratios_and_key_norm(env, f4_kernel, heads):
    """Fewer than four query heads per kv head (empty operand rows), and the query rescaled by the
    key norm inside the kernel."""
    torch, iq = env
    hq, hk = heads
    w = small(n_q_heads=hq, n_kv_heads=hk, n_tokens=900)
    o = oracle_config(w)
    K, V = wl.kv_full(w)
    q = wl.query(w)
    norm, inv = orc.calibrate_key_norm(K, per_head=True)
    want = orc.decode_attention(o, orc.cache_init_prefill(o, K, V, k_inv_norm=inv), q, q_scale=norm)
    _, got = run_attention(torch, iq, o, K, V, q, k_inv_norm=inv, q_scale=norm)
    assert max_rel_err(got, want) <= TOL


def test_fp4_kernel_extreme_queries(env, f4_kernel):
    """Queries whose heads differ in magnitude by many binades (the per-head power-of-two scaling of
    the fp8 operand), a zero head, and one dominant key (the reference level of the softmax rises)."""
    torch, iq = env
    w = small(n_tokens=1500)
    o = oracle_config(w)
    K, V = wl.kv_full(w)
    K = K.copy()
    K[:, :, 777] *= np.float16(6.0)
    q = wl.query(w).copy()
    q[:, 0] *= np.float16(2.0 ** -12)
    q[:, 1] *= np.float16(24.0)
    q[:, 2] = 0
    q[:, 3, :64] = 0
    want = orc.decode_attention(o, orc.cache_init_prefill(o, K, V), q)
    _, got = run_attention(torch, iq, o, K, V, q)
    assert max_rel_err(got, want) <= TOL


def test_fp4_kernel_full_size_sampled(env, f4_kernel):
    test_attention_baseline_configs_full_size_sampled(env, "llama3_8b_32k", [(0, 0), (7, 7)])
    test_attention_baseline_configs_full_size_sampled(env, "mistral_7b_8k", [(31, 7)])


# ---------------------------------------------------------------------------
# Quantisation one step ahead (innerq_quantize_ahead / innerq_decode_attention_next /
# innerq_append_deferred): every step equals the oracle's append followed by attention.
# ---------------------------------------------------------------------------
def _deferred_steps(torch, iq, o, K, V, Q, n_prompt, side_stream=None, fused=False):
    """Runs tokens n_prompt .. N-1 through the deferred calls; returns the cache and the outputs."""
    g = iq.allocate_cache(gpu_config(o))
    Kd, Vd = to_dev(torch, K), to_dev(torch, V)
    if n_prompt:
        iq.innerq_quantize_append(g, Kd[:, :, :n_prompt].contiguous(), Vd[:, :, :n_prompt].contiguous())
    iq.innerq_quantize_ahead(g)
    ws = iq.allocate_workspace(g.cfg)
    main = torch.cuda.current_stream()
    outs, keep = [], []
    done_prev = None
    for t in range(n_prompt, K.shape[2]):
        k_t, v_t = Kd[:, :, t:t + 1].contiguous(), Vd[:, :, t:t + 1].contiguous()
        q_t = to_dev(torch, Q[t - n_prompt])
        keep.append((k_t, v_t, q_t))                  # alive until the side stream has used them
        if fused:
            outs.append(iq.innerq_decode_step(g, k_t, v_t, q_t, ws))
        elif side_stream is None:
            outs.append(iq.innerq_decode_attention_next(g, k_t, v_t, q_t, ws))
            iq.innerq_append_deferred(g, k_t, v_t)
        else:
            ready = torch.cuda.Event()
            ready.record(main)
            if done_prev is not None:
                main.wait_event(done_prev)            # this step's attention needs the previous step's side work
            outs.append(iq.innerq_decode_attention_next(g, k_t, v_t, q_t, ws))
            side_stream.wait_event(ready)
            iq.innerq_append_deferred(g, k_t, v_t, stream=side_stream)
            done_prev = torch.cuda.Event()
            done_prev.record(side_stream)
    torch.cuda.synchronize()
    return g, [x.cpu().numpy() for x in outs]


@pytest.mark.parametrize("kind", KINDS)
@pytest.mark.parametrize("n_prompt,n_steps,group", [(0, 70, 32), (2, 100, 32), (50, 150, 32), (300, 140, 64)])
def test_deferred_append_steps_match_oracle(env, kind, n_prompt, n_steps, group):
    """From an empty or short cache through the sink window, the first eviction and several value
    spills (w_sink 4, w_recent 48): outputs of every step and the final cache."""
    torch, iq = env
    w = small(n_tokens=n_prompt + n_steps, group=group)
    o = oracle_config(w, kind=kind)
    K, V = wl.kv_full(w)
    rng = np.random.default_rng(5)
    Q = rng.standard_normal((n_steps, w.batch, w.n_q_heads, w.head_dim)).astype(np.float16)
    g, outs = _deferred_steps(torch, iq, o, K, V, Q, n_prompt)
    # the ordinary calls on a second cache, step by step: the deferred outputs are the same bits
    # (same kernels, same split plan; only the newest token's rows come from another address)
    want_cache = orc.cache_new(o)
    g_ref = iq.allocate_cache(gpu_config(o))
    ws_ref = iq.allocate_workspace(g_ref.cfg)
    Kd, Vd = to_dev(torch, K), to_dev(torch, V)
    if n_prompt:
        orc.quantize_append(o, want_cache, K[:, :, :n_prompt], V[:, :, :n_prompt])
        iq.innerq_quantize_append(g_ref, Kd[:, :, :n_prompt].contiguous(), Vd[:, :, :n_prompt].contiguous())
    for i, t in enumerate(range(n_prompt, n_prompt + n_steps)):
        orc.quantize_append(o, want_cache, K[:, :, t:t + 1], V[:, :, t:t + 1])
        iq.innerq_quantize_append(g_ref, Kd[:, :, t:t + 1].contiguous(), Vd[:, :, t:t + 1].contiguous())
        ref = iq.innerq_decode_attention(g_ref, to_dev(torch, Q[i]), ws_ref)
        torch.cuda.synchronize()
        assert np.array_equal(outs[i], ref.cpu().numpy()), f"step {i}"
        if kind == orc.KIND_INNER and (i % 7 == 0 or i >= n_steps - 3):
            want = orc.decode_attention(o, want_cache, Q[i])
            assert max_rel_err(outs[i], want) <= TOL, f"step {i}"
    assert_cache_equal(g, want_cache, o)
    # the ordinary calls still work on such a cache (the rows written ahead are simply rewritten)
    k1, v1 = K[:, :, -1:] * np.float16(0.5), V[:, :, -1:] * np.float16(2.0)
    iq.innerq_quantize_append(g, to_dev(torch, k1), to_dev(torch, v1))
    orc.quantize_append(o, want_cache, k1, v1)
    ws = iq.allocate_workspace(g.cfg)
    got = iq.innerq_decode_attention(g, to_dev(torch, Q[0]), ws)
    torch.cuda.synchronize()
    assert_cache_equal(g, want_cache, o)
    assert max_rel_err(got.cpu().numpy(), orc.decode_attention(o, want_cache, Q[0])) <= TOL


def test_deferred_append_on_a_side_stream(env):
    """The deferred append of step t runs on a second stream next to the attention of step t
    (and of step t + 1 up to the event): same outputs, same cache."""
    torch, iq = env
    n_prompt, n_steps = 2100, 200
    w = small(n_tokens=n_prompt + n_steps, batch=4, n_q_heads=16, n_kv_heads=4)
    o = oracle_config(w)
    K, V = wl.kv_full(w)
    rng = np.random.default_rng(6)
    Q = rng.standard_normal((n_steps, w.batch, w.n_q_heads, w.head_dim)).astype(np.float16)
    side = torch.cuda.Stream()
    g, outs = _deferred_steps(torch, iq, o, K, V, Q, n_prompt, side_stream=side)
    g2, outs2 = _deferred_steps(torch, iq, o, K, V, Q, n_prompt)
    for a_, b_ in zip(outs, outs2):
        assert np.array_equal(a_, b_)
    want_cache = orc.cache_init_prefill(o, K, V)
    assert_cache_equal(g, want_cache, o)
    want = orc.decode_attention(o, want_cache, Q[-1])
    assert max_rel_err(outs[-1], want) <= TOL


@pytest.mark.parametrize("kind", KINDS)
@pytest.mark.parametrize("n_prompt,n_steps,group", [(0, 120, 32), (300, 140, 64)])
def test_decode_step_two_launches(env, kind, n_prompt, n_steps, group):
    """innerq_decode_step (merge and append in one launch) against the separate deferred calls:
    same outputs bit for bit, same cache as the oracle."""
    torch, iq = env
    w = small(n_tokens=n_prompt + n_steps, group=group)
    o = oracle_config(w, kind=kind)
    K, V = wl.kv_full(w)
    rng = np.random.default_rng(7)
    Q = rng.standard_normal((n_steps, w.batch, w.n_q_heads, w.head_dim)).astype(np.float16)
    g, outs = _deferred_steps(torch, iq, o, K, V, Q, n_prompt, fused=True)
    _, outs2 = _deferred_steps(torch, iq, o, K, V, Q, n_prompt)
    for i, (a_, b_) in enumerate(zip(outs, outs2)):
        assert np.array_equal(a_, b_), f"step {i}"
    want_cache = orc.cache_init_prefill(o, K, V)
    assert g.n_tokens == n_prompt + n_steps
    assert_cache_equal(g, want_cache, o)
    if kind == orc.KIND_INNER:
        assert max_rel_err(outs[-1], orc.decode_attention(o, want_cache, Q[-1])) <= TOL


def test_decode_step_with_key_norm_and_fp16_output(env):
    """Keys normalised by the caller before they are handed over, query rescaled inside the kernel
    (q_scale), fp16 output: the oracle's append + attention with the same factors."""
    torch, iq = env
    n_prompt, n_steps = 400, 40
    w = small(n_tokens=n_prompt + n_steps)
    o = oracle_config(w)
    K, V = wl.kv_full(w)
    norm, inv = orc.calibrate_key_norm(K[:, :, :n_prompt], per_head=True)
    Kn = orc.apply_channel_scale(K, inv)
    rng = np.random.default_rng(8)
    Q = rng.standard_normal((n_steps, w.batch, w.n_q_heads, w.head_dim)).astype(np.float16)
    g = iq.allocate_cache(gpu_config(o))
    Kd, Vd = to_dev(torch, Kn), to_dev(torch, V)
    iq.innerq_quantize_append(g, Kd[:, :, :n_prompt].contiguous(), Vd[:, :, :n_prompt].contiguous())
    iq.innerq_quantize_ahead(g)
    ws = iq.allocate_workspace(g.cfg)
    scale = to_dev(torch, norm)
    want_cache = orc.cache_init_prefill(o, Kn[:, :, :n_prompt], V[:, :, :n_prompt])
    for i, t in enumerate(range(n_prompt, n_prompt + n_steps)):
        out16 = torch.empty((w.batch, w.n_q_heads, w.head_dim), dtype=torch.float16, device="cuda")
        iq.innerq_decode_step(g, Kd[:, :, t:t + 1].contiguous(), Vd[:, :, t:t + 1].contiguous(), to_dev(torch, Q[i]),
                              ws, out=out16, q_scale=scale)
        orc.quantize_append(o, want_cache, Kn[:, :, t:t + 1], V[:, :, t:t + 1])
        if i % 5 == 0 or i == n_steps - 1:
            torch.cuda.synchronize()
            want = orc.decode_attention(o, want_cache, Q[i], q_scale=norm)
            assert max_rel_err(out16.float().cpu().numpy(), want) <= TOL + 2.0 ** -10, f"step {i}"
    assert_cache_equal(g, want_cache, o)


def test_deferred_calls_on_a_full_cache(env):
    torch, iq = env
    w = small(n_tokens=96)
    o = oracle_config(w, capacity=96)
    K, V = wl.kv_full(w)
    g = iq.allocate_cache(gpu_config(o))
    iq.innerq_quantize_append(g, to_dev(torch, K), to_dev(torch, V))
    iq.innerq_quantize_ahead(g)                      # nothing left to write: accepted
    ws = iq.allocate_workspace(g.cfg)
    k1, v1, q = to_dev(torch, K[:, :, :1]), to_dev(torch, V[:, :, :1]), to_dev(torch, wl.query(w))
    with pytest.raises(iq.InnerQError):
        iq.innerq_decode_attention_next(g, k1, v1, q, ws)
    with pytest.raises(iq.InnerQError):
        iq.innerq_append_deferred(g, k1, v1)
    with pytest.raises(iq.InnerQError):
        iq.innerq_decode_step(g, k1, v1, q, ws)
    assert g.n_tokens == 96


def _decode_steps_full_size(torch, iq, w, o, Kd, Vd, keep, n_prompt, n_steps, check_at, layer=0, inv=None, norm=None):
    """Bulk prompt of n_prompt tokens (already on the device as Kd, Vd, which hold all n_prompt + n_steps
    tokens), innerq_quantize_ahead, then n_steps innerq_decode_step calls: the path the benchmark times.
    The oracle follows the sampled (batch, kv-head) slabs in `keep` token by token; outputs are compared at
    the steps in check_at, the cache of every sampled slab at the end."""
    B, Hk, d = w.batch, w.n_kv_heads, w.head_dim
    r = w.n_q_heads // w.n_kv_heads
    o1 = oracle_config(w.with_(batch=1, n_kv_heads=1, n_q_heads=r), capacity=o.capacity_tokens)
    g = iq.allocate_cache(gpu_config(o))
    inv_d = None if inv is None else to_dev(torch, inv)
    iq.innerq_quantize_append(g, Kd[:, :, :n_prompt].contiguous(), Vd[:, :, :n_prompt].contiguous(), k_inv_norm=inv_d)
    ws = iq.allocate_workspace(g.cfg)
    k1 = Kd[:, :, n_prompt:n_prompt + 1].contiguous()
    q0 = to_dev(torch, wl.query(w, layer, 0))
    with pytest.raises(iq.InnerQError):                 # the store has not been run ahead yet
        iq.innerq_decode_step(g, k1, k1, q0, ws)
    assert g.n_tokens == n_prompt
    iq.innerq_quantize_ahead(g)
    want = {}
    for (b, h), (k, v) in keep.items():
        want[(b, h)] = orc.cache_init_prefill(o1, k[None, None, :n_prompt], v[None, None, :n_prompt],
                                              k_inv_norm=None if inv is None else inv[h:h + 1])
    scale = None if norm is None else to_dev(torch, norm)
    # keys that arrive during decoding have the factors folded in already (the projection carries them)
    if inv is not None:
        Kd[:, :, n_prompt:] = (Kd[:, :, n_prompt:].float() * inv_d[None, :, None, :]).half()
    for i in range(n_steps):
        t = n_prompt + i
        q = wl.query(w, layer, i)
        out = iq.innerq_decode_step(g, Kd[:, :, t:t + 1].contiguous(), Vd[:, :, t:t + 1].contiguous(),
                                    to_dev(torch, q), ws, q_scale=scale)
        for (b, h), (k, v) in keep.items():
            kn = k[None, None, t:t + 1] if inv is None else orc.apply_channel_scale(k[None, None, t:t + 1], inv[h:h + 1])
            orc.quantize_append(o1, want[(b, h)], kn, v[None, None, t:t + 1])
        if i in check_at:
            torch.cuda.synchronize()
            got = out.cpu().numpy()
            assert np.isfinite(got).all()
            for (b, h) in keep:
                ref = orc.decode_attention(o1, want[(b, h)], q[b:b + 1, h * r:(h + 1) * r],
                                           q_scale=None if norm is None else norm[h:h + 1])
                assert max_rel_err(got[b:b + 1, h * r:(h + 1) * r], ref) <= TOL, f"step {i} slab {b},{h}"
    torch.cuda.synchronize()
    assert g.n_tokens == n_prompt + n_steps
    for (b, h) in keep:
        assert_cache_equal(g, want[(b, h)], o1, bsel=slice(b, b + 1), hsel=slice(h, h + 1), what=f"slab {b},{h}")


@pytest.mark.parametrize("name,slabs,n_steps", [("llama3_8b_32k", [(0, 0), (3, 5), (7, 7)], 72),
                                                 ("mistral_7b_8k", [(0, 0), (17, 3), (31, 7)], 132)])
def test_decode_step_full_size_sampled(env, name, slabs, n_steps):
    """The path the benchmark times, at the benchmark's size and launch shape: a whole prompt appended
    in bulk, the store run one step ahead, then single-token innerq_decode_step calls across two value
    spills.  Three (batch, kv-head) slabs are followed by the oracle: outputs within tolerance at the
    first step, after each spill and at the end; packed bytes, flags and windows bit-exact at the end."""
    torch, iq = env
    w = wl.WORKLOADS[name]
    B, Hk, N, d, G = w.batch, w.n_kv_heads, w.n_tokens, w.head_dim, w.group
    n_prompt = N - n_steps
    o = oracle_config(w)
    Kd = torch.empty((B, Hk, N, d), dtype=torch.float16, device="cuda")
    Vd = torch.empty_like(Kd)
    keep = {}
    for b in range(B):
        for h in range(Hk):
            k, v = wl.kv_slab(w, b, h)
            Kd[b, h].copy_(torch.from_numpy(k))
            Vd[b, h].copy_(torch.from_numpy(v))
            if (b, h) in slabs:
                keep[(b, h)] = (k, v)
    # steps at which a value group has just been spilled: the token count minus the windows is a multiple of G
    spills = [i for i in range(n_steps) if (n_prompt + i + 1 - w.w_sink - w.w_recent) % G == 0]
    assert len(spills) >= 2
    check_at = sorted({0, spills[0], spills[0] + 1, spills[1], n_steps - 1})
    _decode_steps_full_size(torch, iq, w, o, Kd, Vd, keep, n_prompt, n_steps, check_at)


def test_decode_step_long_context_layer_full_size_sampled(env):
    """One layer of the 128k-token configuration driven the way the benchmark drives it: key factors
    calibrated over the prompt and folded (prompt keys divided on their way in, later keys arrive
    divided, the query multiplied in the kernel), then innerq_decode_step calls across a value spill."""
    torch, iq = env
    w = wl.WORKLOADS["llama3_8b_128k_32L"]
    layer, n_steps = 7, 40
    B, Hk, N, d, G = w.batch, w.n_kv_heads, w.n_tokens, w.head_dim, w.group
    n_prompt = N - n_steps
    o = oracle_config(w)
    slabs = [(1, 2), (3, 7)]
    gen = torch.Generator(device="cuda")
    gen.manual_seed(2000 + layer)
    sigma = to_dev(torch, wl.key_channel_sigma(w, layer).astype(np.float32))
    Kd = (torch.randn((B, Hk, N, d), device="cuda", generator=gen) * sigma[None, :, None, :]).half()
    Vd = torch.randn((B, Hk, N, d), device="cuda", generator=gen).half()
    keep = {}
    for (b, h) in slabs:
        k, v = wl.kv_slab(w, b, h, layer)
        Kd[b, h].copy_(torch.from_numpy(k))
        Vd[b, h].copy_(torch.from_numpy(v))
        keep[(b, h)] = (k, v)
    peak = Kd[:, :, :n_prompt].abs().amax(dim=(0, 2)).cpu().numpy()[None, :, None, :]
    norm, inv = orc.calibrate_key_norm(peak, per_head=False)
    spills = [i for i in range(n_steps) if (n_prompt + i + 1 - w.w_sink - w.w_recent) % G == 0]
    assert spills
    check_at = sorted({0, spills[0], n_steps - 1})
    _decode_steps_full_size(torch, iq, w, o, Kd, Vd, keep, n_prompt, n_steps, check_at, layer=layer, inv=inv, norm=norm)


@pytest.mark.parametrize("frac", [0.0, 0.02, 0.5, 1.0])
@pytest.mark.parametrize("bits,group,k_mode", [(2, 32, orc.HYBRID), (2, 64, orc.SYM), (4, 32, orc.HYBRID), (3, 32, orc.SYM)])
def test_sparse_value_zero_points_equal_the_dense_read(env, frac, bits, group, k_mode):
    """sparse_zeros = 1 (a value zero-point is fetched only where its group is flagged asymmetric) must give
    the output of the dense read bit for bit, at every flag density from none to all, and stay within
    tolerance of the oracle (Section "Sparsity of M")."""
    torch, iq = env
    import bench
    from dataclasses import replace
    w = small(n_tokens=4 + 48 + 20 * group + 7, bits=bits, group=group, k_mode=k_mode, v_mode=orc.HYBRID)
    o = oracle_config(w)
    B, Hk, N, d, G = w.batch, w.n_kv_heads, w.n_tokens, w.head_dim, w.group
    gen = torch.Generator(device="cuda")
    gen.manual_seed(23)
    K, _ = wl.kv_full(w)
    n_grp = (N - w.w_sink) // G
    vg = bench.crafted_groups(torch, gen, (B, Hk, n_grp, d), G, min(bits, 4), frac)
    v = torch.randn((B, Hk, N, d), device="cuda", generator=gen).half()
    v[:, :, w.w_sink:w.w_sink + n_grp * G] = vg.permute(0, 1, 2, 4, 3).reshape(B, Hk, n_grp * G, d)
    g = iq.allocate_cache(gpu_config(o))
    iq.innerq_quantize_append(g, to_dev(torch, K), v.contiguous())
    torch.cuda.synchronize()
    flags = np.signbit(gpu_buffer_as_numpy(g, o, "v_scales"))[:, :, :(N - w.w_sink - w.w_recent) // G]
    if bits != 3:                                           # (the crafted grids are exact for 2 and 4 bits)
        assert abs(flags.mean() - frac) <= 0.05
    q = to_dev(torch, wl.query(w))
    ws = iq.allocate_workspace(g.cfg)
    dense = iq.innerq_decode_attention(g, q, ws)
    cfg_sparse = iq.make_config(o.batch, o.n_q_heads, o.n_kv_heads, o.head_dim, o.bits, o.group, o.w_sink, o.w_recent,
                                o.k_mode, o.v_mode, o.sym_denominator, o.kind, o.capacity_tokens, o.v_bits, 1)
    sparse = iq.innerq_decode_attention(replace(g, cfg=cfg_sparse), q, ws)
    torch.cuda.synchronize()
    assert torch.equal(dense, sparse)
    want = orc.decode_attention(o, orc.cache_init_prefill(o, K, v.cpu().numpy()), wl.query(w))
    assert max_rel_err(sparse.cpu().numpy(), want) <= TOL


@pytest.mark.parametrize("kind", KINDS)
@pytest.mark.parametrize("per_head,group,n_tokens", [(False, 32, 2500), (True, 64, 1300), (False, 32, 37)])
def test_prefill_in_one_call_equals_calibration_then_append(env, kind, per_head, group, n_tokens):
    """innerq_prefill (maxima of the keys in the launch that quantises the values, keys in a second
    launch) against innerq_calibrate_key_norm + innerq_quantize_append: factors and every cache byte
    identical, and both equal to the oracle's calibration and cache."""
    torch, iq = env
    w = small(n_tokens=n_tokens, batch=3, n_kv_heads=4, n_q_heads=8, group=group)
    o = oracle_config(w, kind=kind)
    K, V = wl.kv_full(w)
    K[:, 2, :, 5] = 0                                   # a dead channel -> factor 1
    Kd, Vd = to_dev(torch, K), to_dev(torch, V)
    g = iq.allocate_cache(gpu_config(o))
    norm, inv = iq.innerq_prefill(g, Kd, Vd, per_head=per_head)
    torch.cuda.synchronize()
    want_n, want_i = orc.calibrate_key_norm(K, per_head)
    assert np.array_equal(norm.cpu().numpy(), want_n) and np.array_equal(inv.cpu().numpy(), want_i)
    want = orc.cache_init_prefill(o, K, V, k_inv_norm=want_i)
    assert g.n_tokens == n_tokens
    assert_cache_equal(g, want, o, what="prefill in one call")
    g2 = iq.allocate_cache(gpu_config(o))
    n2, i2 = iq.innerq_calibrate_key_norm(g2.cfg, Kd, per_head)
    iq.innerq_quantize_append(g2, Kd, Vd, k_inv_norm=i2)
    torch.cuda.synchronize()
    assert torch.equal(n2, norm) and torch.equal(i2, inv)
    for name in g.buffers:
        if g.buffers[name] is not None:
            assert torch.equal(g.buffers[name], g2.buffers[name]), name
    with pytest.raises(iq.InnerQError):                 # only into an empty cache
        iq.innerq_prefill(g, Kd, Vd, per_head=per_head)


@pytest.mark.parametrize("group,lengths", [(32, [40, 700, 1900]), (64, [133, 5, 1210, 2047])])
def test_decode_step_with_per_sequence_lengths_on_the_device(env, group, lengths):
    """innerq_decode_step_ragged: sequences of different lengths in one batch, their token counts in device
    memory only.  Every sequence is filled on its own (a batch-1 view of its slice of the buffers), then
    70 steps run on the whole batch; the oracle follows each sequence separately: outputs in tolerance on
    sampled steps, counters advanced by the device, every sequence's cache bit-exact at the end."""
    torch, iq = env
    n_steps = 70
    B = len(lengths)
    w = small(batch=B, n_kv_heads=2, n_q_heads=8, group=group, n_tokens=max(lengths) + n_steps)
    o = oracle_config(w)
    o1 = oracle_config(w.with_(batch=1), capacity=o.capacity_tokens)
    K, V = wl.kv_full(w)
    g = iq.allocate_cache(gpu_config(o))
    want = []
    for b, n in enumerate(lengths):
        view = iq.sequence_view(g, b)
        iq.innerq_quantize_append(view, to_dev(torch, K[b:b + 1, :, :n]), to_dev(torch, V[b:b + 1, :, :n]))
        iq.innerq_quantize_ahead(view)
        want.append(orc.cache_init_prefill(o1, K[b:b + 1, :, :n], V[b:b + 1, :, :n]))
    n_dev = torch.tensor(lengths, dtype=torch.int32, device="cuda")
    ws = iq.allocate_workspace(g.cfg)
    rng = np.random.default_rng(5)
    for i in range(n_steps):
        # the new token of sequence b is its own next token
        k1 = np.stack([K[b, :, n + i:n + i + 1] for b, n in enumerate(lengths)])
        v1 = np.stack([V[b, :, n + i:n + i + 1] for b, n in enumerate(lengths)])
        q = rng.standard_normal((B, w.n_q_heads, w.head_dim)).astype(np.float16)
        out = iq.innerq_decode_step_ragged(g, n_dev, max(lengths) + n_steps, to_dev(torch, k1), to_dev(torch, v1),
                                           to_dev(torch, q), ws)
        for b in range(B):
            orc.quantize_append(o1, want[b], k1[b:b + 1], v1[b:b + 1])
        if i % 9 == 0 or i == n_steps - 1:
            torch.cuda.synchronize()
            got = out.cpu().numpy()
            assert n_dev.cpu().tolist() == [n + i + 1 for n in lengths]
            for b in range(B):
                ref = orc.decode_attention(o1, want[b], q[b:b + 1])
                assert max_rel_err(got[b:b + 1], ref) <= TOL, f"step {i} sequence {b}"
    torch.cuda.synchronize()
    for b in range(B):
        assert_cache_equal(g, want[b], o1, bsel=slice(b, b + 1), what=f"sequence {b}", per_sequence=True)


def test_ragged_decode_step_replayed_from_a_hip_graph(env):
    """One innerq_decode_step_ragged recorded in a HIP graph (two kernel nodes, no memset, no length on the
    host) and replayed for successive tokens, with eager work and synchronisations between the replays:
    every replay equals the eager call on a twin cache bit for bit, and the device counters advance."""
    torch, iq = env
    lengths, n_steps = [300, 77, 1500], 40
    B = len(lengths)
    w = small(batch=B, n_kv_heads=2, n_q_heads=8, n_tokens=max(lengths) + n_steps + 1)
    o = oracle_config(w)
    K, V = wl.kv_full(w)
    caches, counters = [], []
    for _ in range(2):                                       # twin caches: one driven by the graph, one eagerly
        g = iq.allocate_cache(gpu_config(o))
        for b, n in enumerate(lengths):
            view = iq.sequence_view(g, b)
            iq.innerq_quantize_append(view, to_dev(torch, K[b:b + 1, :, :n]), to_dev(torch, V[b:b + 1, :, :n]))
            iq.innerq_quantize_ahead(view)
        caches.append(g)
        counters.append(torch.tensor(lengths, dtype=torch.int32, device="cuda"))
    ws = [iq.allocate_workspace(caches[0].cfg) for _ in range(2)]
    k_in = torch.zeros((B, w.n_kv_heads, 1, w.head_dim), dtype=torch.float16, device="cuda")
    v_in, q_in = torch.zeros_like(k_in), torch.zeros((B, w.n_q_heads, w.head_dim), dtype=torch.float16, device="cuda")
    out_graph = torch.zeros((B, w.n_q_heads, w.head_dim), dtype=torch.float32, device="cuda")
    bound = max(lengths) + n_steps + 1
    rng = np.random.default_rng(9)

    def inputs(i):
        k1 = np.stack([K[b, :, n + i:n + i + 1] for b, n in enumerate(lengths)])
        v1 = np.stack([V[b, :, n + i:n + i + 1] for b, n in enumerate(lengths)])
        return to_dev(torch, k1), to_dev(torch, v1), to_dev(torch, rng.standard_normal(q_in.shape).astype(np.float16))

    # step 0 eagerly on both (also the first use of the kernels outside any capture)
    k1, v1, q = inputs(0)
    k_in.copy_(k1); v_in.copy_(v1); q_in.copy_(q)
    iq.innerq_decode_step_ragged(caches[0], counters[0], bound, k_in, v_in, q_in, ws[0], out=out_graph)
    ref = iq.innerq_decode_step_ragged(caches[1], counters[1], bound, k1, v1, q, ws[1])
    torch.cuda.synchronize()
    assert torch.equal(out_graph, ref)
    graph = torch.cuda.CUDAGraph()
    k1, v1, q = inputs(1)
    k_in.copy_(k1); v_in.copy_(v1); q_in.copy_(q)
    torch.cuda.synchronize()
    with torch.cuda.graph(graph):
        iq.innerq_decode_step_ragged(caches[0], counters[0], bound, k_in, v_in, q_in, ws[0], out=out_graph)
    for i in range(1, n_steps):
        k1, v1, q = inputs(i) if i > 1 else (k1, v1, q)
        k_in.copy_(k1); v_in.copy_(v1); q_in.copy_(q)
        graph.replay()
        ref = iq.innerq_decode_step_ragged(caches[1], counters[1], bound, k1, v1, q, ws[1])     # eager work in between
        torch.cuda.synchronize()
        assert torch.equal(out_graph, ref), f"replay {i}"
        assert counters[0].cpu().tolist() == [n + i + 1 for n in lengths] == counters[1].cpu().tolist()
    for name in caches[0].buffers:
        if caches[0].buffers[name] is not None:
            assert torch.equal(caches[0].buffers[name], caches[1].buffers[name]), name
