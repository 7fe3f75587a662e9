"""Arithmetic identities the HIP quantiser relies on, checked on the CPU with numpy (no GPU, no
library code: the kernel's instruction sequence is re-enacted with exact intermediate types)."""
import numpy as np
import pytest

f32, f64, ld = np.float32, np.float64, np.longdouble


def correction_step_quotient(num, S):
    """q0 = fl(num * r), rem = num - S * q0 (exact in a fused multiply-add), q = fl(q0 + rem * r)
    with r = fl(1 / S): the sequence the kernel uses instead of a division per element."""
    r = (f32(1) / S).astype(f32)
    q0 = (num * r).astype(f32)
    rem = num.astype(f64) - S.astype(f64) * q0.astype(f64)          # 24 x 24-bit product: exact in fp64
    assert np.array_equal(rem, rem.astype(f32).astype(f64))          # and the remainder fits fp32
    return (q0.astype(ld) + rem.astype(ld) * r.astype(ld)).astype(f32)   # one rounding to fp32


def fp16_values(rng, n, lo=0):
    return rng.integers(lo, 0x7C00, n, dtype=np.uint16).view(np.float16).astype(f32)


@pytest.mark.skipif(np.finfo(ld).nmant < 63, reason="needs an extended-precision long double")
@pytest.mark.parametrize("kind", ["asym_numerators", "sym_numerators", "group_like", "ties"])
def test_reciprocal_correction_step_equals_ieee_division(kind):
    """Code formula of Section "Quantization Scheme" (Eq. asym_quant): the quotient (x - Z) / S is
    an fp32 division.  The kernel's three-instruction replacement must give the identical fp32
    value for every numerator the quantiser can meet (differences of fp16 values, fp16 values)
    and every fp16 scale, including quotients that sit on or beside k + 0.5."""
    rng = np.random.default_rng({"asym_numerators": 1, "sym_numerators": 2, "group_like": 3, "ties": 4}[kind])
    n = 3_000_000
    S = fp16_values(rng, n, lo=1)                                    # every positive finite fp16, subnormals too
    if kind == "asym_numerators":
        num = (fp16_values(rng, n) - fp16_values(rng, n)).astype(f32)
    elif kind == "sym_numerators":
        num = fp16_values(rng, n) * rng.choice(f32([-1, 1]), n)
    elif kind == "group_like":
        lo = rng.standard_normal(n).astype(np.float16).astype(f32)
        hi = lo + np.abs(rng.standard_normal(n)).astype(np.float16).astype(f32)
        S = ((hi - lo) / f32(3)).astype(np.float16).astype(f32)
        S[S == 0] = f32(2.0 ** -24)
        x = (lo + (hi - lo) * rng.random(n).astype(f32)).astype(np.float16).astype(f32)
        num = (x - lo).astype(f32)
    else:
        k = rng.integers(-8, 8, n).astype(f32)
        S = fp16_values(rng, n, lo=0x0400) * f32(2.0 ** -4)             # keep (k + 0.5) S and its neighbours finite in fp16
        mid = ((k + f32(0.5)) * S).astype(f32)                        # exact: few bits times 11 bits
        step = np.spacing(np.abs(mid).astype(np.float16)).astype(f32)
        num = (mid + rng.integers(-2, 3, n).astype(f32) * step).astype(f32)
    with np.errstate(all="ignore"):
        want = (num / S).astype(f32)
        got = correction_step_quotient(num, S)
    ok = np.isfinite(want)
    assert ok.mean() > 0.9
    assert np.array_equal(want[ok], got[ok])
    if kind == "ties":
        frac = np.abs(want - np.trunc(want))
        assert (frac[ok] == 0.5).mean() > 0.1                        # the exact ties are really in the sample


def test_zero_scale_gives_code_zero_without_a_select():
    """A group whose scale is 0 gets r = 0 instead of 1 / 0: every quotient is then exactly 0."""
    num = f32([0.0, 1.5, -3.0, 65504.0])
    S, r = f32(0), f32(0)
    q0 = num * r
    rem = num - S * q0
    assert np.array_equal(q0 + rem * r, np.zeros(4, dtype=f32))
