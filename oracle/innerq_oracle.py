"""Plain CPU oracle for the InnerQ quantised-KV decode-attention path.

TEST INFRASTRUCTURE ONLY.  This file is the slow, obviously-correct statement
of what the method computes, written from the paper (InnerQ, arXiv 2602.23200)
and checked against the paper's equations, closed forms and brute force by the
CPU tests.  It shares no code with the HIP library and must never be imported
by it; only the tests, the smoke check and the benchmark's cpu_baseline leg may
call it.

Arithmetic: the quantiser runs in IEEE fp32 on fp16 inputs (numpy float32 ops,
one rounding per operation, no fused multiply-add), because the integer codes
and the sym/asym flag depend on it; attention runs in float64.

What each function follows
--------------------------
calibrate_key_norm   Section "Per-channel Normalization of K"
quantize_groups      Section "Asymmetric and Symmetric Quantization"
                     (Eq. asym_quant, Eq. asym_dequant, the symmetric scale),
                     Section "Hybrid Quantization" and Figure "hybrid"
dequantize_groups    Eq. hybrid_dequant
cache_init_prefill   Eq. kv_cache_init_quantized_window
append_token         Section "High-precision Window" (last paragraph) and the
                     eviction pattern stated in Section "Latency"
decode_attention     Eq. att:1, att:2, att:3 with Eq. kv_cached_quantized and
                     Figure "quantization_overall" (windows and quantised part
                     are concatenated before the softmax)

Parity pins: every function here is pinned by tests/test_oracle_*.py.  The one
thing that cannot be pinned is accuracy on real models (needs trained weights
and the evaluation datasets): "parity unpinned" for that, and nothing in this
file claims it.
"""
from __future__ import annotations

from dataclasses import dataclass, field
from typing import Optional, Tuple

import numpy as np

SYM, ASYM, HYBRID = 0, 1, 2                      # quantisation mode of a tensor
KIND_INNER, KIND_OUTER, KIND_FP16 = 0, 1, 2      # grouping of the whole cache
FORM_PER_TOKEN, FORM_PER_CHANNEL, FORM_FP16 = 0, 1, 2

f32 = np.float32
f16 = np.float16


# --------------------------------------------------------------------------
# configuration and derived counts
# --------------------------------------------------------------------------
@dataclass
class Config:
    batch: int
    n_q_heads: int
    n_kv_heads: int
    head_dim: int
    bits: int
    group: int
    w_sink: int
    w_recent: int
    k_mode: int = HYBRID
    v_mode: int = HYBRID
    sym_denominator: int = 0     # 0: 2^(b-1)-1 ; 1: 2^b-1 (the formula as printed)
    kind: int = KIND_INNER
    capacity_tokens: int = 0
    v_bits: int = 0              # width of the value codes; 0: same as bits (the key width)

    def bits_of(self, which: str) -> int:
        """Code width of tensor 'k' or 'v' (the paper's presets pair 3-bit keys with 2- or 3-bit
        values: Section "Experimental Setup")."""
        return self.v_bits if (which == "v" and self.v_bits) else self.bits

    def form(self, which: str) -> int:
        """Grouping form of tensor 'k' or 'v'.

        Inner-dimension grouping (Section "InnerQ"): K per-token group-wise,
        V per-channel group-wise.  Outer-dimension grouping is the reverse.
        """
        if self.kind == KIND_FP16:
            return FORM_FP16
        inner = FORM_PER_TOKEN if which == "k" else FORM_PER_CHANNEL
        outer = FORM_PER_CHANNEL if which == "k" else FORM_PER_TOKEN
        return inner if self.kind == KIND_INNER else outer

    def mode(self, which: str) -> int:
        return self.k_mode if which == "k" else self.v_mode

    def ring_slots(self, which: str) -> int:
        # the recent window holds w_recent tokens (up to w_recent + G - 1 for a tensor grouped
        # along tokens); the buffer has one spare slot (G spare slots) beyond that
        extra = self.group if self.form(which) == FORM_PER_CHANNEL else 1
        return self.w_recent + extra


def partition(cfg: Config, which: str, n_tokens: int) -> Tuple[int, int, int]:
    """(n_sink, n_quantised, n_recent) of one tensor when N tokens are cached.

    Eq. kv_cache_init_quantized_window gives sink / middle / recent; a tensor
    grouped along tokens can only quantise whole groups of G tokens (Section
    "Latency": G value tokens every G steps), the remainder stays in fp16.
    """
    n_s = min(n_tokens, cfg.w_sink)
    n_mid = max(0, n_tokens - cfg.w_sink - cfg.w_recent)
    if cfg.form(which) == FORM_PER_CHANNEL:
        n_mid = (n_mid // cfg.group) * cfg.group
    return n_s, n_mid, n_tokens - n_s - n_mid


# --------------------------------------------------------------------------
# per-channel key normalisation
# --------------------------------------------------------------------------
def calibrate_key_norm(K: np.ndarray, per_head: bool = False):
    """norm_c = sqrt(max |K[..., c]|), K fp16 [B, Hk, N, d] -> (norm, inv) fp32 [Hk, d].

    The paper's maximum runs over heads and tokens (per_head=False; batch is
    included so one weight fold serves every sequence).  per_head=True keeps
    one vector per kv head.  A channel that is identically zero gets norm 1.
    """
    a = np.abs(K.astype(f32))
    m = a.max(axis=(0, 2))                      # [Hk, d]
    if not per_head:
        m = np.broadcast_to(m.max(axis=0, keepdims=True), m.shape).copy()
    norm = np.sqrt(m, dtype=f32)
    norm[m == 0] = f32(1.0)
    inv = (f32(1.0) / norm).astype(f32)
    return norm, inv


def apply_channel_scale(x16: np.ndarray, scale: np.ndarray) -> np.ndarray:
    """fp16_rn(float(x) * scale_c): how K (x inv_norm) or q (x norm) is rescaled.

    x16 [B, H, ..., d] fp16, scale [Hs, d] fp32 where H is a multiple of Hs
    (query heads map onto kv heads contiguously).
    """
    H, Hs = x16.shape[1], scale.shape[0]
    s = np.repeat(scale, H // Hs, axis=0)                  # [H, d]
    shape = [1, H] + [1] * (x16.ndim - 3) + [x16.shape[-1]]
    return (x16.astype(f32) * s.reshape(shape).astype(f32)).astype(f16)


# --------------------------------------------------------------------------
# the group quantiser
# --------------------------------------------------------------------------
def _sym_den(bits: int, sym_denominator: int) -> int:
    return (1 << bits) - 1 if sym_denominator else (1 << (bits - 1)) - 1


def quantize_asym(g16: np.ndarray, bits: int):
    """Eq. asym_quant on groups g16 [..., G] (fp16).  Returns codes, S (fp16>=0), Z (fp16)."""
    g = g16.astype(f32)
    qmax = (1 << bits) - 1
    Z = g.min(axis=-1)                                       # an fp16 value
    S32 = (g.max(axis=-1) - Z) / f32(qmax)
    S = S32.astype(f16)                                      # stored precision
    Sf = S.astype(f32)[..., None]
    with np.errstate(divide="ignore", invalid="ignore"):
        c = np.rint((g - Z[..., None]) / Sf)
    c = np.clip(c, 0, qmax)
    c = np.where(Sf == 0, f32(0), c)
    return c.astype(np.int32), S, Z.astype(f16)


def quantize_sym(g16: np.ndarray, bits: int, sym_denominator: int = 0):
    """Symmetric mode: Z = 0, S = max|g| / den, signed b-bit codes."""
    g = g16.astype(f32)
    lo, hi = -(1 << (bits - 1)), (1 << (bits - 1)) - 1
    S32 = np.abs(g).max(axis=-1) / f32(_sym_den(bits, sym_denominator))
    S = S32.astype(f16)
    Sf = S.astype(f32)[..., None]
    with np.errstate(divide="ignore", invalid="ignore"):
        c = np.rint(g / Sf)
    c = np.clip(c, lo, hi)
    c = np.where(Sf == 0, f32(0), c)
    return c.astype(np.int32), S


def _l1_error_sequential(g: np.ndarray, recon: np.ndarray) -> np.ndarray:
    """sum_i |g_i - recon_i| in fp32, added one term at a time in index order."""
    e = np.zeros(g.shape[:-1], dtype=f32)
    for i in range(g.shape[-1]):
        e = e + np.abs(g[..., i] - recon[..., i])
    return e


def quantize_groups(g16: np.ndarray, bits: int, mode: int, sym_denominator: int = 0):
    """Quantise groups g16 [..., G] and return what is stored.

    Returns (u, scale, zero):
      u      uint8 [..., G]  stored field: the code itself for an asymmetric
                             group, code + 2^(b-1) for a symmetric one
      scale  fp16  [...]     +S_sym, or -S_asym (sign bit = the mask M)
      zero   fp16  [...]     Z for an asymmetric group, +0 otherwise
    Hybrid (Figure "hybrid"): quantise both ways, reconstruct both, compare the
    L1 errors, keep asymmetric only when its error is strictly smaller.
    """
    g = g16.astype(f32)
    half = 1 << (bits - 1)
    if mode in (SYM, HYBRID):
        cs, Ss = quantize_sym(g16, bits, sym_denominator)
    if mode in (ASYM, HYBRID):
        ca, Sa, Za = quantize_asym(g16, bits)
    if mode == SYM:
        M = np.zeros(g.shape[:-1], dtype=bool)
    elif mode == ASYM:
        M = np.ones(g.shape[:-1], dtype=bool)
    else:
        rec_s = Ss.astype(f32)[..., None] * cs.astype(f32)
        rec_a = Sa.astype(f32)[..., None] * ca.astype(f32) + Za.astype(f32)[..., None]
        M = _l1_error_sequential(g, rec_a) < _l1_error_sequential(g, rec_s)
    if mode == SYM:
        u = cs + half
        scale, zero = Ss, np.zeros_like(Ss)
    elif mode == ASYM:
        u, scale, zero = ca, -Sa, Za
    else:
        u = np.where(M[..., None], ca, cs + half)
        scale = np.where(M, -Sa, Ss).astype(f16)
        zero = np.where(M, Za, f16(0)).astype(f16)
    return u.astype(np.uint8), scale.astype(f16), zero.astype(f16)


def dequantize_groups(u: np.ndarray, scale: np.ndarray, zero: np.ndarray, bits: int) -> np.ndarray:
    """Eq. hybrid_dequant: x^ = S * code + M * Z, exact in float64."""
    M = np.signbit(scale)
    code = u.astype(np.float64) - np.where(M, 0, 1 << (bits - 1))[..., None]
    S = np.abs(scale.astype(np.float64))[..., None]
    return S * code + np.where(M, zero.astype(np.float64), 0.0)[..., None]


# --------------------------------------------------------------------------
# bit packing (this build's storage layout; the paper does not give one)
# --------------------------------------------------------------------------
def pack_fields(u: np.ndarray, bits: int) -> np.ndarray:
    """b-bit fields [..., n] -> bytes [..., n*b/8]; field i sits at bit b*i (little-endian).

    3-bit fields are stored as two planes, one after the other: the low two bits of every field
    packed as 2-bit fields (n/4 bytes), then the high bits packed as 1-bit fields (n/8 bytes).
    """
    if bits == 3:
        return np.concatenate([pack_fields(u & 3, 2), pack_fields(u >> 2, 1)], axis=-1)
    per = 8 // bits
    u = u.reshape(u.shape[:-1] + (u.shape[-1] // per, per)).astype(np.uint16)
    out = np.zeros(u.shape[:-1], dtype=np.uint16)
    for i in range(per):
        out |= u[..., i] << (bits * i)
    return out.astype(np.uint8)


def unpack_fields(p: np.ndarray, bits: int) -> np.ndarray:
    if bits == 3:
        n_lo = p.shape[-1] * 2 // 3
        return unpack_fields(p[..., :n_lo], 2) | (unpack_fields(p[..., n_lo:], 1) << 2)
    per = 8 // bits
    mask = (1 << bits) - 1
    cols = [(p >> (bits * i)) & mask for i in range(per)]
    return np.stack(cols, axis=-1).reshape(p.shape[:-1] + (p.shape[-1] * per,)).astype(np.uint8)


# --------------------------------------------------------------------------
# cache container
# --------------------------------------------------------------------------
@dataclass
class Cache:
    k_codes: np.ndarray
    k_scales: Optional[np.ndarray]
    k_zeros: Optional[np.ndarray]
    v_codes: np.ndarray
    v_scales: Optional[np.ndarray]
    v_zeros: Optional[np.ndarray]
    k_sink: np.ndarray
    v_sink: np.ndarray
    k_recent: np.ndarray
    v_recent: np.ndarray
    n_tokens: int = 0


def _store_shapes(cfg: Config, which: str):
    B, H, d, G, b, cap = cfg.batch, cfg.n_kv_heads, cfg.head_dim, cfg.group, cfg.bits_of(which), cfg.capacity_tokens
    form = cfg.form(which)
    if form == FORM_FP16:
        return (B, H, cap, d), None
    if form == FORM_PER_TOKEN:
        return (B, H, cap, d * b // 8), (B, H, cap, d // G)
    return (B, H, cap // G, d, G * b // 8), (B, H, cap // G, d)


def cache_new(cfg: Config) -> Cache:
    assert cfg.capacity_tokens % cfg.group == 0
    B, H, d = cfg.batch, cfg.n_kv_heads, cfg.head_dim
    bufs = {}
    for which in ("k", "v"):
        cs, ss = _store_shapes(cfg, which)
        bufs[which + "_codes"] = np.zeros(cs, dtype=f16 if ss is None else np.uint8)
        bufs[which + "_scales"] = None if ss is None else np.zeros(ss, dtype=f16)
        bufs[which + "_zeros"] = None if ss is None else np.zeros(ss, dtype=f16)
        bufs[which + "_sink"] = np.zeros((B, H, cfg.w_sink, d), dtype=f16)
        bufs[which + "_recent"] = np.zeros((B, H, cfg.ring_slots(which), d), dtype=f16)
    return Cache(**bufs)


def _quantise_into_store(cfg: Config, cache: Cache, which: str, x16: np.ndarray, first_row: int):
    """Quantise tokens x16 [B, Hk, T, d] into store rows first_row .. first_row+T."""
    codes = getattr(cache, which + "_codes")
    scales = getattr(cache, which + "_scales")
    zeros = getattr(cache, which + "_zeros")
    B, H, T, d = x16.shape
    G, b = cfg.group, cfg.bits_of(which)
    form, mode = cfg.form(which), cfg.mode(which)
    if T == 0:
        return
    if form == FORM_FP16:
        codes[:, :, first_row:first_row + T] = x16
    elif form == FORM_PER_TOKEN:
        # groups of G consecutive channels inside each token
        u, s, z = quantize_groups(x16.reshape(B, H, T, d // G, G), b, mode, cfg.sym_denominator)
        codes[:, :, first_row:first_row + T] = pack_fields(u.reshape(B, H, T, d), b)
        scales[:, :, first_row:first_row + T] = s
        zeros[:, :, first_row:first_row + T] = z
    else:
        # groups of G consecutive tokens inside each channel
        assert T % G == 0 and first_row % G == 0
        g = x16.reshape(B, H, T // G, G, d).transpose(0, 1, 2, 4, 3)      # [B,H,T/G,d,G]
        u, s, z = quantize_groups(g, b, mode, cfg.sym_denominator)
        r0 = first_row // G
        codes[:, :, r0:r0 + T // G] = pack_fields(u, b)
        scales[:, :, r0:r0 + T // G] = s
        zeros[:, :, r0:r0 + T // G] = z


def cache_init_prefill(cfg: Config, K16: np.ndarray, V16: np.ndarray,
                       k_inv_norm: Optional[np.ndarray] = None) -> Cache:
    """Eq. kv_cache_init_quantized_window on prefill tensors [B, Hk, N, d] (fp16)."""
    cache = cache_new(cfg)
    if k_inv_norm is not None:
        K16 = apply_channel_scale(K16, k_inv_norm)
    N = K16.shape[2]
    assert N <= cfg.capacity_tokens
    for which, X in (("k", K16), ("v", V16)):
        n_s, n_q, n_r = partition(cfg, which, N)
        getattr(cache, which + "_sink")[:, :, :n_s] = X[:, :, :n_s]
        _quantise_into_store(cfg, cache, which, X[:, :, n_s:n_s + n_q], 0)
        ring = getattr(cache, which + "_recent")
        for t in range(n_s + n_q, N):                       # ring slot = token index mod slots
            ring[:, :, t % ring.shape[2]] = X[:, :, t]
    cache.n_tokens = N
    return cache


def append_token(cfg: Config, cache: Cache, k16: np.ndarray, v16: np.ndarray):
    """One decode-time append of k16, v16 [B, Hk, d] (already normalised).

    The new token joins the fp16 windows; tokens that no longer fit the recent
    window are quantised and moved to the quantised store: one token at a time
    for a per-token grouped tensor, G tokens at once for a tensor grouped along
    tokens.
    """
    t = cache.n_tokens
    assert t < cfg.capacity_tokens
    for which, x in (("k", k16), ("v", v16)):
        sink = getattr(cache, which + "_sink")
        ring = getattr(cache, which + "_recent")
        slots = ring.shape[2]
        if t < cfg.w_sink:
            sink[:, :, t] = x
            continue
        _, n_q_before, _ = partition(cfg, which, t)
        _, n_q_after, _ = partition(cfg, which, t + 1)
        n_evict = n_q_after - n_q_before
        if n_evict:
            # gather the oldest recent tokens (absolute indices) before the
            # new token may reuse one of their slots
            first = cfg.w_sink + n_q_before
            old = np.stack([ring[:, :, (first + i) % slots] for i in range(n_evict)], axis=2)
            _quantise_into_store(cfg, cache, which, old, n_q_before)
        ring[:, :, t % slots] = x
    cache.n_tokens = t + 1


def quantize_append(cfg: Config, cache: Cache, k_new: np.ndarray, v_new: np.ndarray,
                    k_inv_norm: Optional[np.ndarray] = None):
    """Append T tokens [B, Hk, T, d] one after the other."""
    if k_inv_norm is not None:
        k_new = apply_channel_scale(k_new, k_inv_norm)
    for i in range(k_new.shape[2]):
        append_token(cfg, cache, k_new[:, :, i], v_new[:, :, i])


# --------------------------------------------------------------------------
# attention
# --------------------------------------------------------------------------
def effective_tensor(cfg: Config, cache: Cache, which: str, b: int, hk: int) -> np.ndarray:
    """All N cached rows of K or V of one (batch, kv-head) as the decoder sees them, float64 [N, d]."""
    N = cache.n_tokens
    d, G, bits = cfg.head_dim, cfg.group, cfg.bits_of(which)
    n_s, n_q, n_r = partition(cfg, which, N)
    out = np.empty((N, d), dtype=np.float64)
    out[:n_s] = getattr(cache, which + "_sink")[b, hk, :n_s]
    codes = getattr(cache, which + "_codes")[b, hk]
    form = cfg.form(which)
    if n_q:
        if form == FORM_FP16:
            out[n_s:n_s + n_q] = codes[:n_q]
        elif form == FORM_PER_TOKEN:
            u = unpack_fields(codes[:n_q], bits).reshape(n_q, d // G, G)
            s = getattr(cache, which + "_scales")[b, hk, :n_q]
            z = getattr(cache, which + "_zeros")[b, hk, :n_q]
            out[n_s:n_s + n_q] = dequantize_groups(u, s, z, bits).reshape(n_q, d)
        else:
            u = unpack_fields(codes[:n_q // G], bits)                      # [n_q/G, d, G]
            s = getattr(cache, which + "_scales")[b, hk, :n_q // G]
            z = getattr(cache, which + "_zeros")[b, hk, :n_q // G]
            x = dequantize_groups(u, s, z, bits)                           # [n_q/G, d, G]
            out[n_s:n_s + n_q] = x.transpose(0, 2, 1).reshape(n_q, d)
    ring = getattr(cache, which + "_recent")[b, hk]
    for t in range(n_s + n_q, N):
        out[t] = ring[t % ring.shape[0]]
    return out


def decode_attention(cfg: Config, cache: Cache, q16: np.ndarray,
                     q_scale: Optional[np.ndarray] = None,
                     heads: Optional[list] = None) -> np.ndarray:
    """softmax(q K^T / sqrt(d)) V over all cached tokens, float64 [B, Hq, d].

    q16 fp16 [B, Hq, d]; query head hq reads kv head hq // (Hq / Hk).  `heads`
    restricts the work to a list of (b, hk) pairs; other rows are left as NaN.
    """
    if q_scale is not None:
        q16 = apply_channel_scale(q16, q_scale)
    B, Hq, d = q16.shape
    r = Hq // cfg.n_kv_heads
    out = np.full((B, Hq, d), np.nan, dtype=np.float64)
    pairs = heads if heads is not None else [(b, h) for b in range(B) for h in range(cfg.n_kv_heads)]
    for b, hk in pairs:
        Ke = effective_tensor(cfg, cache, "k", b, hk)
        Ve = effective_tensor(cfg, cache, "v", b, hk)
        for hq in range(hk * r, (hk + 1) * r):
            s = (Ke @ q16[b, hq].astype(np.float64)) / np.sqrt(np.float64(d))
            p = np.exp(s - s.max())
            p /= p.sum()
            out[b, hq] = p @ Ve
    return out
