"""The identity the e4m3 ingest kernel relies on to avoid one division per element (CPU, float32 numpy).

Claim: with r = RN(1/s) and q0 = RN(x * r), encode(q0) == encode(RN(x / s)) unless q0 is within 4 ulp of a
rounding boundary of e4m3's normal range (float32 pattern: three mantissa bits, then 1000...0) or |x| is
under 2^-6 * s (plus one ulp), where the quotient may fall into e4m3's subnormal range; those cases take the
real division.  Checked on quotients placed within a few
ulp of every boundary, where the shortcut alone does go wrong.
"""
import numpy as np

from oracle import fp8


def test_reciprocal_shortcut_with_fallback_equals_division():
    rng = np.random.default_rng(0)
    pos = fp8.TABLE[1:127]
    mids = (pos[:-1] + pos[1:]) / 2
    n = 2_000_000
    s = np.exp2(rng.uniform(-12, 4, n)).astype(np.float32) * (1 + rng.random(n).astype(np.float32))
    x = (rng.choice(mids, n) * s.astype(np.float64)).astype(np.float32)
    x = (x.view(np.int32) + rng.integers(-6, 7, n).astype(np.int32)).view(np.float32)      # a few ulp around
    x *= rng.choice([-1, 1], n).astype(np.float32)
    exact = fp8.encode((x / s).astype(np.float32))
    q0 = (x * (np.float32(1) / s).astype(np.float32)).astype(np.float32)
    near = ((q0.view(np.uint32) << np.uint32(12)) + np.uint32(0x80004000)).astype(np.uint32) <= 0x8000
    subnormal = np.abs(x) < (s * np.float32(1 + 2.0 ** -23) * np.float32(2.0 ** -6)).astype(np.float32)
    shortcut = fp8.encode(q0)
    assert (shortcut != exact).sum() > 1000                       # the inputs are adversarial ...
    assert (np.where(near | subnormal, exact, shortcut) == exact).all()   # ... and the fallback catches every one
    # a near quotient with zero residual x - q0 * s is exact and needs no division either (the product of two
    # float32 values and its difference from x are exact in float64)
    residual = x.astype(np.float64) - q0.astype(np.float64) * s.astype(np.float64)
    divide = (near & (residual != 0)) | subnormal
    assert (np.where(divide, exact, shortcut) == exact).all()
    # ... which is what makes ties of short mantissas (bf16 inputs, power-of-two scales) cheap
    xb = (rng.integers(0x3F80, 0x4000, n).astype(np.uint32) << np.uint32(16)).view(np.float32)
    sb = np.float32(2.0 ** -7)
    qb = xb * np.float32(128)
    nearb = ((qb.view(np.uint32) << np.uint32(12)) + np.uint32(0x80004000)).astype(np.uint32) <= 0x8000
    assert nearb.mean() > 0.05 and not (nearb & ((xb.astype(np.float64) - qb.astype(np.float64) * float(sb)) != 0)).any()
    # ordinary data rarely needs the fallback
    y = rng.standard_normal(n).astype(np.float32)
    q = (y * np.float32(1 / 0.0078)).astype(np.float32)
    mag = q.view(np.uint32) & np.uint32(0x7FFFFFFF)
    frac = ((((mag & np.uint32(0xFFFFF)) - np.uint32(0x7FFFC)).astype(np.uint32) <= 8) |
            ((mag - np.uint32(1)).astype(np.uint32) < np.uint32(0x3C800000 - 1))).mean()
    assert frac < 1e-3
