"""Pins for the oracle's group quantiser, flag encoding, packing and key norm.

None of these re-type the oracle's formulas: they check it against brute force
over all code levels, closed-form extremes, error bounds, constructed groups
whose answer is known in advance, and numbers printed in the paper
(tests/golden/effective_bits.txt, from Table "bits").
"""
import os

import numpy as np
import pytest

from oracle import innerq_oracle as orc

GOLDEN = os.path.join(os.path.dirname(__file__), "golden")


def random_groups(seed, n, G, kind):
    r = np.random.default_rng(seed)
    if kind == "normal":
        x = r.standard_normal((n, G))
    elif kind == "positive":
        x = r.uniform(0.5, 4.0, (n, G))
    elif kind == "outlier":
        x = r.standard_normal((n, G))
        x[np.arange(n), r.integers(0, G, n)] *= 20
    elif kind == "shifted":
        x = r.standard_normal((n, G)) * 0.3 + r.uniform(-3, 3, (n, 1))
    elif kind == "tiny":
        x = r.standard_normal((n, G)) * 1e-6
    return x.astype(np.float16)


KINDS = ["normal", "positive", "outlier", "shifted", "tiny"]


@pytest.mark.parametrize("bits", [2, 3, 4])
@pytest.mark.parametrize("kind", KINDS)
def test_asym_codes_are_nearest_level_brute_force(bits, kind):
    g = random_groups(1, 300, 32, kind)
    c, S, Z = orc.quantize_asym(g, bits)
    x = g.astype(np.float64)
    Sd, Zd = S.astype(np.float64)[:, None], Z.astype(np.float64)[:, None]
    levels = np.arange(1 << bits)
    err_all = np.abs(x[:, :, None] - (Sd[:, :, None] * levels + Zd[:, :, None]))   # [n,G,levels]
    best = err_all.min(axis=-1)
    mine = np.abs(x - (Sd * c + Zd))
    assert c.min() >= 0 and c.max() <= (1 << bits) - 1
    # the chosen level is a minimiser (fp32 quotient rounding may flip an exact tie only)
    assert np.all(mine <= best + 2.0 ** -20 * (np.abs(x) + np.abs(Zd) + Sd))
    # zero-point is the group minimum and the scale spans the range
    assert np.array_equal(Z, g.min(axis=1))
    rng = g.astype(np.float64).max(1) - g.astype(np.float64).min(1)
    assert np.allclose(S.astype(np.float64), rng / ((1 << bits) - 1), rtol=2.0 ** -10, atol=2.0 ** -24)
    nz = S >= 2.0 ** -14        # normal fp16 scale: rounding it cannot move max below the top level
    rows = np.arange(len(g))
    assert np.all(c[rows, g.argmin(1)] == 0)
    assert np.all(c[rows, g.argmax(1)][nz] == (1 << bits) - 1)


@pytest.mark.parametrize("bits", [2, 3, 4])
@pytest.mark.parametrize("den", [0, 1])
@pytest.mark.parametrize("kind", KINDS)
def test_sym_codes_are_nearest_level_brute_force(bits, den, kind):
    g = random_groups(2, 300, 32, kind)
    c, S = orc.quantize_sym(g, bits, den)
    x = g.astype(np.float64)
    Sd = S.astype(np.float64)[:, None]
    lo, hi = -(1 << (bits - 1)), (1 << (bits - 1)) - 1
    levels = np.arange(lo, hi + 1)
    best = np.abs(x[:, :, None] - Sd[:, :, None] * levels).min(axis=-1)
    mine = np.abs(x - Sd * c)
    assert c.min() >= lo and c.max() <= hi
    assert np.all(mine <= best + 2.0 ** -20 * (np.abs(x) + Sd))
    amax = np.abs(x).max(1)
    denom = (1 << bits) - 1 if den else (1 << (bits - 1)) - 1
    assert np.allclose(S.astype(np.float64), amax / denom, rtol=2.0 ** -10, atol=2.0 ** -24)
    if den == 0:
        # default reading: +-max|g| land on +-(2^(b-1)-1) and nothing is clipped
        rows = np.arange(len(g))
        j = np.abs(x).argmax(1)
        nz = S >= 2.0 ** -14
        assert np.all(np.abs(c[rows, j])[nz] == denom)
        assert np.all(c[nz] >= -denom)     # (a denormal fp16 scale may round far enough to reach -2^(b-1))


@pytest.mark.parametrize("bits", [2, 3, 4])
@pytest.mark.parametrize("mode", [orc.SYM, orc.ASYM, orc.HYBRID])
@pytest.mark.parametrize("kind", KINDS)
def test_round_trip_error_at_most_half_a_step(bits, mode, kind):
    g = random_groups(3, 400, 32, kind)
    u, s, z = orc.quantize_groups(g, bits, mode, 0)
    xh = orc.dequantize_groups(u, s, z, bits)
    S = np.abs(s.astype(np.float64))[:, None]
    err = np.abs(g.astype(np.float64) - xh)
    # The bound needs the stored scale to be a normal fp16 number (relative rounding 2^-11);
    # a denormal scale is rounded to a multiple of 2^-24 and may saturate the extreme element.
    ok = (S[:, 0] >= 2.0 ** -14) | (S[:, 0] == 0)
    assert np.all(err[ok] <= S[ok] / 2 * (1 + 2.0 ** -9))
    assert np.all(err[~ok] <= S[~ok] / 2 + 2.0 ** -24 * (1 << bits))


def test_round_trip_literal_denominator_holds_for_unclipped():
    g = random_groups(4, 400, 32, "normal")
    for bits in (2, 4):
        c, S = orc.quantize_sym(g, bits, 1)
        x = g.astype(np.float64)
        Sd = S.astype(np.float64)[:, None]
        q = x / Sd
        unclipped = (q >= -(1 << (bits - 1)) - 0.5) & (q <= (1 << (bits - 1)) - 0.5)
        err = np.abs(x - Sd * c)
        assert np.all(err[unclipped] <= Sd.repeat(32, 1)[unclipped] / 2 * (1 + 2.0 ** -9))
        assert (~unclipped).any()          # the literal formula does saturate some elements


@pytest.mark.parametrize("bits", [2, 3, 4])
def test_hybrid_flag_matches_float64_error_comparison(bits):
    near_tie = 0
    for kind in KINDS:
        g = random_groups(5, 500, 32, kind)
        u, s, z = orc.quantize_groups(g, bits, orc.HYBRID, 0)
        M = np.signbit(s)
        x = g.astype(np.float64)
        cs, Ss = orc.quantize_sym(g, bits, 0)
        ca, Sa, Za = orc.quantize_asym(g, bits)
        es = np.abs(x - Ss.astype(np.float64)[:, None] * cs).sum(1)
        ea = np.abs(x - (Sa.astype(np.float64)[:, None] * ca + Za.astype(np.float64)[:, None])).sum(1)
        close = np.abs(ea - es) <= 1e-5 * (ea + es)
        near_tie += int(close.sum())
        assert np.array_equal(M[~close], (ea < es)[~close])
        # the stored fields are those of the chosen mode
        half = 1 << (bits - 1)
        assert np.array_equal(u[M], ca[M].astype(np.uint8))
        assert np.array_equal(u[~M], (cs[~M] + half).astype(np.uint8))
        assert np.array_equal(np.abs(s[M]), Sa[M]) and np.array_equal(s[~M], Ss[~M])
    assert near_tie < 50


def test_hybrid_constructed_groups():
    G = 32
    # all-positive, evenly spaced: asymmetric uses every level, symmetric wastes the negative half
    pos = np.linspace(1.0, 4.0, G).astype(np.float16)[None]
    u, s, z = orc.quantize_groups(pos, 2, orc.HYBRID, 0)
    assert np.signbit(s[0]) and z[0] == pos.min()
    # values exactly on a symmetric grid: symmetric error is zero -> symmetric wins the tie or outright
    grid = (np.array([-1, 0, 1, 1] * 8, dtype=np.float16) * np.float16(0.75))[None]
    u, s, z = orc.quantize_groups(grid, 2, orc.HYBRID, 0)
    assert not np.signbit(s[0]) and s[0] == np.float16(0.75) and z[0] == 0
    assert np.array_equal(orc.dequantize_groups(u, s, z, 2)[0], grid[0].astype(np.float64))
    # all-zero group: both errors are zero, tie -> symmetric, scale +0
    zero = np.zeros((1, G), dtype=np.float16)
    u, s, z = orc.quantize_groups(zero, 2, orc.HYBRID, 0)
    assert not np.signbit(s[0]) and s[0] == 0 and np.all(orc.dequantize_groups(u, s, z, 2) == 0)
    # constant non-zero group at 4 bits: asymmetric reproduces it exactly with S = 0;
    # the flag must survive as the sign bit of a zero scale
    const = np.full((1, G), 0.3, dtype=np.float16)
    u, s, z = orc.quantize_groups(const, 4, orc.HYBRID, 0)
    assert np.signbit(s[0]) and s[0] == 0 and z[0] == const[0, 0]
    assert np.all(orc.dequantize_groups(u, s, z, 4) == const.astype(np.float64))
    # strict comparison: symmetric data symmetric about zero with equal errors stays symmetric
    pm = np.array([-1.0, 1.0] * 16, dtype=np.float16)[None]
    u, s, z = orc.quantize_groups(pm, 2, orc.HYBRID, 0)
    assert not np.signbit(s[0])


@pytest.mark.parametrize("mode", [orc.SYM, orc.ASYM, orc.HYBRID])
def test_flag_encoding_sign_bit_and_zero_point(mode):
    g = np.concatenate([random_groups(6, 200, 32, k) for k in KINDS])
    u, s, z = orc.quantize_groups(g, 2, mode, 0)
    M = np.signbit(s)
    if mode == orc.SYM:
        assert not M.any()
    if mode == orc.ASYM:
        assert M.all()
    assert np.all(z[~M].view(np.uint16) == 0)            # +0.0 exactly when symmetric
    assert np.array_equal(z[M], g.min(1)[M])
    if mode == orc.HYBRID:
        assert M.any() and (~M).any()


@pytest.mark.parametrize("bits", [2, 3, 4])
def test_pack_unpack_all_patterns(bits):
    if bits == 3:
        # plane layout: every combination of the 8 fields that share one high-bit byte
        r = np.random.default_rng(1)
        u = r.integers(0, 8, (4096, 8), dtype=np.uint8)
        packed = orc.pack_fields(u, 3)
        assert packed.shape == (4096, 3)
        assert np.array_equal(orc.unpack_fields(packed, 3), u)
        # the high-bit byte alone decides which fields are >= 4, the first two bytes the rest
        hi = np.unpackbits(packed[:, 2:3], axis=1, bitorder="little")
        assert np.array_equal(hi, (u >= 4).astype(np.uint8))
        u = r.integers(0, 8, (7, 5, 128), dtype=np.uint8)
        assert np.array_equal(orc.unpack_fields(orc.pack_fields(u, 3), 3), u)
        assert orc.pack_fields(u, 3).shape == (7, 5, 48)
        return
    per = 8 // bits
    # every byte value appears: enumerate all field combinations of one byte
    vals = np.arange(256, dtype=np.uint16)
    fields = np.stack([(vals >> (bits * i)) & ((1 << bits) - 1) for i in range(per)], -1).astype(np.uint8)
    packed = orc.pack_fields(fields, bits)
    assert np.array_equal(packed[:, 0], vals.astype(np.uint8))
    assert np.array_equal(orc.unpack_fields(packed, bits), fields)
    r = np.random.default_rng(0)
    u = r.integers(0, 1 << bits, (7, 5, 128), dtype=np.uint8)
    assert np.array_equal(orc.unpack_fields(orc.pack_fields(u, bits), bits), u)


def test_pack_golden_example():
    """Hand-written rows of tests/golden/pack_example.txt (layout: field i at bit b*i)."""
    rows = [l.split("|") for l in open(os.path.join(GOLDEN, "pack_example.txt")) if l[0] not in "#\n"]
    assert rows
    for bits, fields, hexbytes in rows:
        u = np.array([int(t) for t in fields.split()], dtype=np.uint8)
        want = np.array([int(t, 16) for t in hexbytes.split()], dtype=np.uint8)
        assert np.array_equal(orc.pack_fields(u[None], int(bits))[0], want)


def test_effective_bits_match_paper_table():
    """Bytes of the oracle's stores per quantised number vs Table "bits" (G = 32)."""
    want = {}
    for line in open(os.path.join(GOLDEN, "effective_bits.txt")):
        if line[0] in "#\n":
            continue
        name, val = line.split()
        want[name] = float(val)

    def bits_per_number(kind, which, bits, mode, v_bits=0):
        cfg = orc.Config(1, 4, 1, 128, bits, 32, 4, 32, mode, mode, 0, kind, 1024, v_bits)
        cs, ss = orc._store_shapes(cfg, which)
        n = 1024 * 128
        total = np.prod(cs) + 2 * np.prod(ss) * (1 if mode == orc.SYM else 2)
        return 8.0 * total / n

    # KIVI: outer-grouped 2-bit asymmetric keys and values
    kivi = 0.5 * (bits_per_number(orc.KIND_OUTER, "k", 2, orc.ASYM) + bits_per_number(orc.KIND_OUTER, "v", 2, orc.ASYM))
    assert kivi == want["KIVI"]
    # value-cache halves of the InnerQ presets (their key half is 3-bit symmetric = 3.5 bits)
    small_v = bits_per_number(orc.KIND_INNER, "v", 2, orc.SYM)
    hybrid_v = bits_per_number(orc.KIND_INNER, "v", 2, orc.HYBRID)
    assert 0.5 * (3.5 + small_v) == want["InnerQ_Small"]
    assert 0.5 * (3.5 + hybrid_v) == want["InnerQ_Hybrid"]
    # 4-bit symmetric: b + 16/G
    assert bits_per_number(orc.KIND_INNER, "k", 4, orc.SYM) == 4.5
    # Hybrid and Small presets as one configuration each: 3-bit symmetric keys, 2-bit values
    assert 0.5 * (bits_per_number(orc.KIND_INNER, "k", 3, orc.SYM, 2) +
                  bits_per_number(orc.KIND_INNER, "v", 3, orc.SYM, 2)) == want["InnerQ_Small"]
    assert 0.5 * (bits_per_number(orc.KIND_INNER, "k", 3, orc.SYM, 2) +
                  bits_per_number(orc.KIND_INNER, "v", 3, orc.HYBRID, 2)) == want["InnerQ_Hybrid"]
    # the presets' key half and the Base preset, from the 3-bit stores themselves
    assert bits_per_number(orc.KIND_INNER, "k", 3, orc.SYM) == 3.5
    assert 0.5 * (bits_per_number(orc.KIND_INNER, "k", 3, orc.SYM) +
                  bits_per_number(orc.KIND_INNER, "v", 3, orc.SYM)) == want["InnerQ_Base"]


def test_key_norm_definition_and_fold_identity():
    r = np.random.default_rng(7)
    K = (r.standard_normal((2, 3, 50, 16)) * r.uniform(0.2, 9, (1, 3, 1, 16))).astype(np.float16)
    K[..., 5] = 0                                           # a dead channel
    norm_h, inv_h = orc.calibrate_key_norm(K, per_head=True)
    norm_g, inv_g = orc.calibrate_key_norm(K, per_head=False)
    # brute force
    for h in range(3):
        for c in range(16):
            m = max(abs(float(K[b, h, j, c])) for b in range(2) for j in range(50))
            want = np.float32(np.sqrt(np.float32(m))) if m > 0 else np.float32(1)
            assert norm_h[h, c] == want
    assert np.array_equal(norm_g, np.broadcast_to(norm_h.max(0), norm_h.shape))
    assert norm_h[0, 5] == 1 and inv_h[0, 5] == 1
    assert np.array_equal(inv_h, (np.float32(1) / norm_h))
    # the fold is an identity in exact arithmetic: (q * n) . (k / n) == q . k
    q = r.standard_normal(16)
    k = K[0, 1, 3].astype(np.float64)
    n = norm_h[1].astype(np.float64)
    assert abs((q * n) @ (k / n) - q @ k) < 1e-12 * np.abs(q * k).sum()
    # with fp16 storage of both rescaled vectors the error is bounded by the two roundings
    q16 = q.astype(np.float16)[None, None]
    qn = orc.apply_channel_scale(np.repeat(q16, 3, 1), norm_h)[0, 1].astype(np.float64)
    kn = orc.apply_channel_scale(K, inv_h)[0, 1, 3].astype(np.float64)
    exact = q16[0, 0].astype(np.float64) @ k
    assert abs(qn @ kn - exact) <= 2.0 ** -9 * np.abs(q16[0, 0].astype(np.float64) * k).sum()
    # normalisation flattens the per-channel range: max|K/n| == sqrt(max|K|) == n
    Kn = orc.apply_channel_scale(K, inv_h).astype(np.float32)
    assert np.allclose(np.abs(Kn).max(axis=(0, 2)), np.where(norm_h == 1, np.abs(Kn).max(axis=(0, 2)), norm_h), rtol=2e-3)


@pytest.mark.parametrize("bits", [2, 3, 4])
def test_crafted_density_groups_decide_as_planned(bits):
    """The flag-density sweep of bench.py fills caches with groups whose hybrid decision is fixed
    by construction (exact asymmetric grid of positive values / exact symmetric grid).  The oracle
    must take exactly the planned decision for every group and reproduce every value exactly."""
    import torch

    import bench
    gen = torch.Generator(device="cpu")
    gen.manual_seed(5)
    x, planned = bench.crafted_groups(torch, gen, (6, 50), 32, bits, 0.3, device="cpu", return_mask=True)
    g = x.numpy()
    u, s, z = orc.quantize_groups(g, bits, orc.HYBRID, 0)
    assert np.array_equal(np.signbit(s), planned.numpy())
    assert 0.2 < planned.float().mean().item() < 0.4
    assert np.array_equal(orc.dequantize_groups(u, s, z, bits), g.astype(np.float64))


def test_channel_scale_rounds_the_fp32_product():
    """K x inv_norm (and q x norm) is an fp32 multiply followed by a conversion to fp16: the same
    two roundings torch's CPU kernels make for (x.float() * s).half().  Values whose exact
    product sits beside an fp16 midpoint tell this apart from a single rounding of the exact
    product; the oracle must side with the two-step result on every one of them."""
    import torch

    from tests.helpers import midpoint_scale_and_values
    scale, x = midpoint_scale_and_values(128, 64, seed=5, lo_exp=-3, hi_exp=4)
    got = orc.apply_channel_scale(x[None, None], scale[None])[0, 0]
    two_step = (torch.from_numpy(x).float() * torch.from_numpy(scale)[None, :]).half().numpy()
    one_step = (x.astype(np.float64) * scale.astype(np.float64)[None, :]).astype(np.float16)
    assert np.array_equal(got.view(np.uint16), two_step.view(np.uint16))
    assert (got != one_step).all()
