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


# ---------------------------------------------------------------------------
# GPU side (imported lazily so that CPU-only test modules never need torch.cuda)
# ---------------------------------------------------------------------------
def gpu_config(o: orc.Config):
    from paper_2602_23200_amd import binding as iq
    return iq.make_config(o.batch, o.n_q_heads, o.n_kv_heads, o.head_dim, o.bits, o.group, o.w_sink,
                          o.w_recent, o.k_mode, o.v_mode, o.sym_denominator, o.kind, o.capacity_tokens,
                          o.v_bits)


def gpu_buffer_as_numpy(gcache, o: orc.Config, name: str):
    """Download one device buffer shaped and typed like the oracle's buffer of that name."""
    buf = gcache.buffers[name]
    if buf is None:
        return None
    which = name[0]
    raw = buf.cpu().numpy()
    B, H, d = o.batch, o.n_kv_heads, o.head_dim
    if name.endswith("codes"):
        cs, ss = orc._store_shapes(o, which)
        return raw.view(np.float16).reshape(cs) if ss is None else raw.reshape(cs)
    if name.endswith("scales") or name.endswith("zeros"):
        _, ss = orc._store_shapes(o, which)
        return raw.view(np.float16).reshape(ss)
    if name.endswith("sink"):
        return raw.view(np.float16).reshape(B, H, o.w_sink, d)
    return raw.view(np.float16).reshape(B, H, o.ring_slots(which), d)


def assert_cache_equal(gcache, ocache, o: orc.Config, bsel=slice(None), hsel=slice(None), what="", per_sequence=False):
    """Bit-exact comparison of every live part of the GPU cache against the oracle cache.

    bsel / hsel select the (batch, kv-head) slab of the GPU buffers that the oracle cache
    (possibly built for a single slab) corresponds to.
    """
    N = ocache.n_tokens
    assert per_sequence or gcache.n_tokens == N            # (per_sequence: the counts live on the device)
    for x in "kv":
        n_s, n_q, n_r = orc.partition(o, x, N)
        form = o.form(x)
        rows = n_q // o.group if form == orc.FORM_PER_CHANNEL else n_q
        for part in ("codes", "scales", "zeros"):
            name = f"{x}_{part}"
            want = getattr(ocache, name)
            got = gpu_buffer_as_numpy(gcache, o if bsel == slice(None) else _full_cfg(gcache, o), name)
            if want is None:
                continue
            if got is None:
                # symmetric tensors keep no zero-points on the device; the oracle's are all +0
                assert part == "zeros" and not want.view(np.uint16).any()
                continue
            g = got[bsel, hsel][:, :, :rows]          # store rows run along axis 2 in every form
            w_ = want[:, :, :rows]
            assert np.array_equal(bits_view(np.ascontiguousarray(g)), bits_view(np.ascontiguousarray(w_))), \
                f"{what} {name} differs"
        sink_g = gpu_buffer_as_numpy(gcache, o if bsel == slice(None) else _full_cfg(gcache, o), f"{x}_sink")
        if sink_g is not None and n_s:
            assert np.array_equal(bits_view(np.ascontiguousarray(sink_g[bsel, hsel][:, :, :n_s])),
                                  bits_view(getattr(ocache, f"{x}_sink")[:, :, :n_s])), f"{what} {x}_sink"
        ring_g = gpu_buffer_as_numpy(gcache, o if bsel == slice(None) else _full_cfg(gcache, o), f"{x}_recent")
        ring_o = getattr(ocache, f"{x}_recent")
        live = [t % ring_o.shape[2] for t in range(n_s + n_q, N)]
        assert np.array_equal(bits_view(np.ascontiguousarray(ring_g[bsel, hsel][:, :, live])),
                              bits_view(np.ascontiguousarray(ring_o[:, :, live]))), f"{what} {x}_recent"


def _full_cfg(gcache, o: orc.Config) -> orc.Config:
    """Oracle-style config with the GPU cache's full batch / head counts (for reshaping)."""
    from dataclasses import replace
    c = gcache.cfg
    return replace(o, batch=c.batch, n_kv_heads=c.n_kv_heads, n_q_heads=c.n_q_heads)


def max_rel_err(got: np.ndarray, want: np.ndarray) -> float:
    """max_i |got - want| / max_i |want| per (batch, head) row, maximum over rows."""
    num = np.abs(got.astype(np.float64) - want).max(axis=-1)
    den = np.abs(want).max(axis=-1)
    return float((num / den).max())


def midpoint_scale_and_values(d: int, n: int, seed: int, lo_exp: int, hi_exp: int):
    """An fp32 factor per channel, scale [d] in [0.25, 1), and fp16 values [n, d] with magnitudes in
    [2^lo_exp, 2^hi_exp), such that EVERY product value x scale changes when it is rounded to fp32
    before it is rounded to fp16: the exact product lies just beside an fp16 midpoint and its fp32
    rounding lands on it.  Only the 10 mantissa bits of a value matter, and a given factor has
    such a mantissa with probability of about 1/16, so factors are drawn until one has."""
    rng = np.random.default_rng(seed)
    mant = (np.arange(1024, 2048, dtype=np.float32) / np.float32(1024)).astype(np.float16)   # [1, 2)
    scale = np.empty(d, dtype=np.float32)
    out = np.empty((n, d), dtype=np.float16)
    for c in range(d):
        while True:
            s = np.float32(rng.uniform(0.25, 1.0))
            twice = (mant.astype(np.float32) * s).astype(np.float16)
            once = (mant.astype(np.float64) * np.float64(s)).astype(np.float16)    # exact product, one rounding
            pick = mant[twice != once]
            if pick.size:
                break
        scale[c] = s
        v = pick[rng.integers(0, pick.size, n)].astype(np.float32)
        v *= np.exp2(rng.integers(lo_exp, hi_exp, n)).astype(np.float32) * rng.choice(np.float32([-1, 1]), n)
        out[:, c] = v.astype(np.float16)
    return scale, out
