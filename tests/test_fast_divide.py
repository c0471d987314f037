"""The bf16 merge + quantize kernel does not run the 11-instruction IEEE divide per weight.  One lane per (row, group)
forms the correctly rounded reciprocal of the scale,

    r0 = rcp(s)  (hardware estimate, within 1 ulp);  e = fma(-s, r0, 1);  r1 = fma(e, r0, r0);
    r  = whichever of r1 and its two neighbours has the smallest exact residual |fma(-s, r, 1)|         = RN(1 / s)

and every weight of the group then costs one multiply and two fused multiply-adds,

    x' = med3(x, -1024 s, 1024 s);   q = x' r;   t = fma(-s, q, x');   w = fma(t, r, q)                = RN(x / s)

(Markstein's division: with r correctly rounded, q lies within one unit of the quotient and one correction with the
exact remainder rounds it correctly).  The header's contract says "correctly rounded divide"; on the GPU the codes and
the mask are compared bit for bit with the oracle's IEEE division, and l4q_check_fast_divide runs the sequence against
the hardware's IEEE divide for all 2^23 significands of the scale.  This file checks the arithmetic claims themselves
on the CPU, with an exact emulation of the binary32 fused multiply-add: the reciprocal step for every estimate within
one unit of 1 / s, and the quotient on the neighbourhoods of every decision point of the quantizer (rounding ties
k + 1/2 and the grid ends of all code widths, a few ulps to either side), on scales with awkward significands, and on
random operands."""
import numpy as np
import pytest

F32, F64 = np.float32, np.float64


def fma32(a, b, c):
    """RN_binary32(a * b + c) for binary32 arrays, exactly: the product is exact in binary64, the sum is rounded to
    odd there (53 >= 2 * 24 + 2 bits), and one final rounding to binary32 follows."""
    a, b, c = (np.asarray(v, F32).astype(F64) for v in (a, b, c))
    p = a * b
    t = p + c
    bb = t - p
    err = (p - (t - bb)) + (c - bb)                      # exact error of the binary64 sum
    other = np.nextafter(t, np.where(err > 0, np.inf, -np.inf))
    odd = (t.view(np.int64) & 1) == 1
    t_odd = np.where((err == 0) | odd, t, other)
    return t_odd.astype(F32)


def test_fma_emulation_is_exact_where_binary64_double_rounding_is_not():
    # 1 + 2^-24 + 2^-60: a binary64 sum rounds to 1 + 2^-24 (a tie for binary32, resolved to 1); the exact value is
    # above the tie and must round to 1 + 2^-23
    a, b, c = F32(1.0 + 2.0 ** -12), F32(2.0 ** -12 + 2.0 ** -48 * 0), F32(1.0)
    x = fma32(F32(2.0 ** -30), F32(2.0 ** -30), F32(1.0 + 2.0 ** -23) - F32(2.0 ** -24) * 0)
    assert x == F32(1.0 + 2.0 ** -23)
    got = fma32(F32(2.0 ** -30), F32(2.0 ** -30), np.nextafter(F32(1.0), F32(2.0)))   # 1 + 2^-23 + 2^-60
    assert got == np.nextafter(F32(1.0), F32(2.0))
    # tie broken by a tiny product: (1 + 2^-24 is not binary32) use c = 1, a b = 2^-24 + 2^-50 -> above the tie
    a = F32(2.0 ** -12)
    b = F32(2.0 ** -12 + 2.0 ** -35)                     # a b = 2^-24 + 2^-47
    assert fma32(a, b, F32(1.0)) == np.nextafter(F32(1.0), F32(2.0))
    assert F32(F64(a) * F64(b) + 1.0) == np.nextafter(F32(1.0), F32(2.0))   # (binary64 happens to get this one right)
    rng = np.random.default_rng(0)
    u, v, w = (rng.standard_normal(200000).astype(F32) for _ in range(3))
    # against exact rational arithmetic on a sample
    from fractions import Fraction
    got = fma32(u[:300], v[:300], w[:300])
    for k in range(300):
        exact = Fraction(float(u[k])) * Fraction(float(v[k])) + Fraction(float(w[k]))
        lo = np.nextafter(got[k], F32(-np.inf))
        hi = np.nextafter(got[k], F32(np.inf))
        d = abs(Fraction(float(got[k])) - exact)
        assert d <= abs(Fraction(float(lo)) - exact) and d <= abs(Fraction(float(hi)) - exact)


def refined_reciprocal(s, r0):
    """The kernel's reciprocal step from an estimate r0."""
    s, r0 = np.asarray(s, F32), np.asarray(r0, F32)
    one = np.ones_like(s)
    e = fma32(-s, r0, one)
    r = fma32(e, r0, r0)
    e0 = np.abs(fma32(-s, r, one))
    rp = (r.view(np.uint32) + np.uint32(1)).view(F32)
    rm = (r.view(np.uint32) - np.uint32(1)).view(F32)
    ep, em = np.abs(fma32(-s, rp, one)), np.abs(fma32(-s, rm, one))
    r = np.where(ep < e0, rp, r)
    r = np.where(em < e0, rm, r)
    return r


def fast_quotient(x, s):
    """The kernel's per-weight sequence with r = RN(1 / s)."""
    x, s = np.asarray(x, F32), np.asarray(s, F32)
    r = (F32(1.0) / s).astype(F32)
    hi = (s * F32(1024.0)).astype(F32)
    xc = np.minimum(np.maximum(x, -hi), hi)
    q = (xc * r).astype(F32)
    t = fma32(-s, q, xc)
    return fma32(t, r, q)


def awkward_scales(rng, n):
    """Scales between 2^-40 and 2^20: random ones, and significands that stress a reciprocal (all ones, all zeros,
    one above / below a power of two, around sqrt 2 and 4/3)."""
    expo = rng.integers(-40, 21, n)
    sig = rng.integers(0, 1 << 23, n)
    special = np.array([0, 1, 2, 3, (1 << 23) - 1, (1 << 23) - 2, 0x3504F3, 0x3504F4, 0x2AAAAA, 0x2AAAAB, 0x555555,
                        0x400000, 0x3FFFFF, 0x400001, 0x7FFFFE, 0x100000, 0x600000])
    sig[: 40 * len(special)] = np.tile(special, 40)
    bits = ((expo + 127).astype(np.uint32) << np.uint32(23)) | sig.astype(np.uint32)
    return bits.view(F32)


def test_reciprocal_step_is_correctly_rounded_for_any_estimate_within_one_ulp():
    rng = np.random.default_rng(5)
    s = awkward_scales(rng, 600000)
    want = (F32(1.0) / s).astype(F32)
    true = 1.0 / s.astype(F64)
    lo = np.where(want.astype(F64) <= true, want, np.nextafter(want, F32(0.0)))       # the floats bracketing 1 / s
    hi = np.nextafter(lo, F32(np.inf))
    hi = np.where(lo.astype(F64) == true, lo, hi)
    estimates = [lo, hi, want]
    # where 1 / s is closer than one ulp to a third float, that one is a legal estimate too
    for cand in (np.nextafter(lo, F32(0.0)), np.nextafter(hi, F32(np.inf))):
        ok = np.abs(cand.astype(F64) - true) <= np.spacing(want).astype(F64)
        estimates.append(np.where(ok, cand, want))
    for r0 in estimates:
        got = refined_reciprocal(s, r0)
        assert np.array_equal(got.view(np.uint32), want.view(np.uint32)), int((got != want).sum())
    # the significand of all ones, where the Newton step alone stays on the wrong neighbour
    s1 = F32(np.uint32(0x3FFFFFFF).view(F32))
    stuck = fma32(fma32(-s1, F32(0.5), F32(1.0)), F32(0.5), F32(0.5))
    assert stuck == F32(0.5) and F32(1.0) / s1 != F32(0.5)
    assert refined_reciprocal(np.array([s1]), np.array([0.5], F32))[0] == F32(1.0) / s1


def test_quotient_equals_ieee_division_around_every_decision_point():
    rng = np.random.default_rng(7)
    s = awkward_scales(rng, 3000)
    ties = np.arange(-128, 128) + 0.5                                   # rounding ties of every code width up to 8
    ends = np.array([v for n in range(2, 9) for v in (-(1 << (n - 1)), (1 << (n - 1)) - 1)], dtype=F64)
    points = np.concatenate([ties, ends]).astype(F32)                    # all exactly representable
    x0 = (s[:, None] * points[None, :]).astype(F32)                      # quotient lands on / next to the point
    xs = [x0]
    up, dn = x0, x0
    for _ in range(5):                                                   # five ulps to either side
        up = np.nextafter(up, F32(np.inf))
        dn = np.nextafter(dn, F32(-np.inf))
        xs += [up, dn]
    x = np.stack(xs, axis=2)
    sb = np.broadcast_to(s[:, None, None], x.shape)
    want = (x / sb).astype(F32)
    got = fast_quotient(x.ravel(), sb.ravel()).reshape(x.shape)
    assert np.array_equal(got.view(np.uint32), want.view(np.uint32)), int((got != want).sum())
    # the sample does sit on decision points: many quotients are exactly a tie or a grid end
    assert (want == points[None, :, None]).sum() > 0.05 * want.size
    # without the correction step the product alone is wrong on a large part of it
    r = (F32(1.0) / sb).astype(F32)
    assert ((x * r).astype(F32) != want).mean() > 0.1


def test_quotient_equals_ieee_division_on_random_operands():
    rng = np.random.default_rng(11)
    s = awkward_scales(rng, 2000000)
    w = (rng.standard_normal(s.size) * rng.choice([1e-3, 0.3, 4.0, 60.0, 900.0], s.size)).astype(F32)
    x = (w * s).astype(F32)
    x[:1000] = 0.0
    x[1000:2000] = -0.0
    want = (x / s).astype(F32)
    got = fast_quotient(x, s)
    inside = np.abs(want) <= 1024                       # beyond that the numerator is clamped (next test)
    assert inside.mean() > 0.9
    nz = inside & (x != 0)
    assert np.array_equal(got[nz].view(np.uint32), want[nz].view(np.uint32))
    # a zero numerator gives a zero of either sign (-0 comes back as +0): code 0, in range, factor 0 all the same
    assert not got[x == 0].any()


def test_clamping_the_numerator_changes_no_decision():
    """|x| > 1024 s means |w| > 1024, beyond the ends of every grid (|Q_N| <= 128): code, mask and d(Wq)/d(scale)
    depend on the sign alone there, so dividing med3(x, -1024 s, 1024 s) instead of x decides the same."""
    rng = np.random.default_rng(13)
    s = awkward_scales(rng, 100000)
    x = (s * (rng.standard_normal(s.size) * 3000).astype(F32)).astype(F32)
    w, wc = (x / s).astype(F32), fast_quotient(x, s)
    for bits in (2, 4, 8):
        qn, qp = F32(-(1 << (bits - 1))), F32((1 << (bits - 1)) - 1)
        assert np.array_equal(np.rint(np.clip(w, qn, qp)), np.rint(np.clip(wc, qn, qp)))
        assert np.array_equal((w >= qn) & (w <= qp), (wc >= qn) & (wc <= qp))
    big = np.abs(w) > 1024
    assert big.sum() > 1000 and np.array_equal(w[~big], wc[~big]) and (np.abs(wc[big]) == 1024).all()
