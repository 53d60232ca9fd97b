"""The compressor kernels do not divide per value: they multiply by the token's reciprocal and take
the IEEE divide only when the product is near a rounding tie (csrc/compress.hip: quantize_value for
packs of 8, within 1e-3 of a tie with the correctly rounded reciprocal; quantize_token8 for packs
of 16, codes below 16, within 2^-15 of a tie with a reciprocal that may be an ulp off).  This checks
those rules themselves, in numpy float32 arithmetic (IEEE, like the
kernel's): for fp16 inputs of many magnitudes, and for inputs placed on and next to the ties, it
gives exactly the code of the plain definition clamp(rint(fl((x - min) / scale)), 0, qmax)
(PackKV Sec. III-B.2) -- the definition the oracle implements."""
import numpy as np


def _codes(x, mn, s, qmax):
    x, mn, s = x.astype(np.float32), mn.astype(np.float32), s.astype(np.float32)
    a = (x - mn).astype(np.float32)
    exact = np.rint((a / s).astype(np.float32))
    r = (np.float32(1.0) / s).astype(np.float32)
    q1 = (a * r).astype(np.float32)
    t = np.rint(q1)
    near_tie = np.abs(np.abs((q1 - t).astype(np.float32)) - np.float32(0.5)) < np.float32(1e-3)
    fast = np.where(near_tie, exact, t)
    return np.clip(exact, 0, qmax), np.clip(fast, 0, qmax), int(near_tie.sum())


def test_reciprocal_rule_gives_the_codes_of_the_divide():
    rng = np.random.default_rng(5)
    n = 2_000_000
    fallbacks = 0
    with np.errstate(over="ignore", invalid="ignore", divide="ignore"):
        for _ in range(3):
            mag = np.float32(2.0) ** rng.integers(-12, 12, n)
            mn = (rng.standard_normal(n).astype(np.float32) * mag).astype(np.float16)
            rel = rng.choice([0.1, 0.2, 0.05, 1 / 255, 1 / 33, 1.0, 0.5], n).astype(np.float32)
            span = np.abs(rng.standard_normal(n).astype(np.float32) * mag * 4).astype(np.float16).astype(np.float32)
            s = (rel * span).astype(np.float32).astype(np.float16)
            x = (mn.astype(np.float32) + rng.random(n).astype(np.float32) * span).astype(np.float16)
            qmax = np.rint(1 / rel)
            ok = (s.astype(np.float32) > 0) & np.isfinite(s.astype(np.float32)) & np.isfinite(x.astype(np.float32))
            exact, fast, k = _codes(x[ok], mn[ok], s[ok], qmax[ok])
            assert np.array_equal(exact, fast)
            fallbacks += k
            # inputs on and next to the ties k + 1/2 of their token's grid
            tie = rng.integers(0, 256, n).astype(np.float32) + np.float32(0.5)
            at = (mn.astype(np.float32) + tie * s.astype(np.float32)).astype(np.float32).astype(np.float16)
            for step in (0, 1, -1, 2, -2):
                xb = (at.view(np.uint16).astype(np.int32) + step).clip(0, 0xFBFF).astype(np.uint16).view(np.float16)
                okb = ok & np.isfinite(xb.astype(np.float32))
                exact, fast, k = _codes(xb[okb], mn[okb], s[okb], qmax[okb])
                assert np.array_equal(exact, fast)
                fallbacks += k
    assert fallbacks > 100_000, "the tie cases are meant to reach the divide"


def _codes16(x, mn, s, qmax, ulp_off):
    """The rule of packs of 16: q = fl(a * r), r = 1 / s up to an ulp, rounded to nearest even; near a
    tie, or where q could round above qmax, the divide with the clamp."""
    x, mn, s = x.astype(np.float32), mn.astype(np.float32), s.astype(np.float32)
    a = (x - mn).astype(np.float32)
    quotient = (a / s).astype(np.float32)
    exact = np.clip(np.rint(quotient), 0, qmax)
    r = (np.float32(1.0) / s).astype(np.float32)
    r = (r.view(np.int32) + ulp_off).view(np.float32)          # the hardware reciprocal: within one ulp
    q = (a * r).astype(np.float32)
    frac = (q - np.floor(q)).astype(np.float32)
    guard = np.float32(2.0 ** -15)
    near_tie = np.abs((frac - np.float32(0.5)).astype(np.float32)) < guard
    # a quotient that could round above qmax also takes the divide, which clamps; the fast path
    # rounds to nearest even and saturates at 0 and 255 only
    too_big = q >= (qmax.astype(np.float32) + np.float32(0.5) - guard).astype(np.float32)
    slow = near_tie | too_big
    fast = np.where(slow, np.clip(np.rint(np.minimum(quotient, qmax)), 0, 255), np.clip(np.rint(q), 0, 255))
    return exact, fast, int(near_tie.sum())


def test_rule_of_packs_of_16_gives_the_codes_of_the_divide():
    rng = np.random.default_rng(16)
    n = 2_000_000
    fallbacks = 0
    with np.errstate(over="ignore", invalid="ignore", divide="ignore"):
        for ulp_off in (0, 1, -1):
            mag = np.float32(2.0) ** rng.integers(-12, 12, n)
            mn = (rng.standard_normal(n).astype(np.float32) * mag).astype(np.float16)
            rel = rng.choice([0.1, 0.2, 1 / 15, 1 / 7, 0.3, 1.0, 0.5], n).astype(np.float32)
            span = np.abs(rng.standard_normal(n).astype(np.float32) * mag * 4).astype(np.float16).astype(np.float32)
            s = (rel * span).astype(np.float32).astype(np.float16)
            x = (mn.astype(np.float32) + rng.random(n).astype(np.float32) * span).astype(np.float16)
            qmax = np.rint(1 / rel)
            assert qmax.max() < 16
            ok = (s.astype(np.float32) > 0) & np.isfinite(s.astype(np.float32)) & np.isfinite(x.astype(np.float32))
            exact, fast, k = _codes16(x[ok], mn[ok], s[ok], qmax[ok], ulp_off)
            assert np.array_equal(exact, fast)
            fallbacks += k
            # inputs on and next to the ties k + 1/2 of their token's grid, also far above qmax
            tie = rng.integers(0, 80, n).astype(np.float32) + np.float32(0.5)
            at = (mn.astype(np.float32) + tie * s.astype(np.float32)).astype(np.float32).astype(np.float16)
            for step in (0, 1, -1, 2, -2):
                xb = (at.view(np.uint16).astype(np.int32) + step).clip(0, 0xFBFF).astype(np.uint16).view(np.float16)
                okb = ok & np.isfinite(xb.astype(np.float32))
                exact, fast, k = _codes16(xb[okb], mn[okb], s[okb], qmax[okb], ulp_off)
                assert np.array_equal(exact, fast)
                fallbacks += k
    assert fallbacks > 100_000, "the tie cases are meant to reach the divide"
