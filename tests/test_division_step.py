"""The three-instruction division by a block-constant scale that the qkv epilogues of the FP8 GEMM use
(y = RN(1/d) once; q = RN(x y); r = x - d q, exact in one fma; result RN(q + r y)) must give the bits of the IEEE
division that the stand-alone quantiser performs (App. B.2: x / scale, clamp, cast).  Emulated here in numpy: an fp32
fma is (float64(a) * float64(b) + float64(c)) rounded once to fp32 -- the product of two fp32 numbers is exact in
fp64, and the sums below are of nearby magnitudes, so the fp64 sum is exact too -- over the numerators and divisors
the kernels see: bf16 values over a scale derived from a block maximum, including the half-way cases of E4M3."""
import numpy as np


def _fma32(a, b, c):
    return (a.astype(np.float64) * b.astype(np.float64) + c.astype(np.float64)).astype(np.float32)


def _step(x, d):
    y = (np.float32(1.0) / d).astype(np.float32)
    q = (x * y).astype(np.float32)
    r = _fma32(-q, d, x)
    return _fma32(r, y, q)


def _bf16(x):
    b = np.asarray(x, dtype=np.float32).view(np.uint32)
    b = (b + np.uint32(0x7FFF) + ((b >> np.uint32(16)) & np.uint32(1))) & np.uint32(0xFFFF0000)
    return b.view(np.float32)


def test_division_step_equals_ieee_division():
    rng = np.random.default_rng(5)
    n = 2_000_000
    amax = _bf16(np.exp(rng.uniform(-20, 20, n)).astype(np.float32))
    d = (np.maximum(amax, np.float32(1e-8)) / np.float32(448.0)).astype(np.float32)          # the block scale
    x = _bf16(amax * rng.uniform(-1, 1, n).astype(np.float32))                                 # |x| <= amax
    plain = (d.view(np.uint32) & np.uint32(0x7FFFFF)) == np.uint32(0x7FFFFF)                   # these take the division itself
    want = (x / d).astype(np.float32)
    got = _step(x, d)
    keep = ~plain
    assert np.array_equal(got[keep].view(np.uint32), want[keep].view(np.uint32))


def test_division_step_on_exact_ties_of_the_code_grid():
    """x / amax = m / 448 with m half-way between two E4M3 values: the quotient by the rounded scale must land on the
    same side as the IEEE division puts it."""
    mids = np.array([(2 * k + 1) * 2.0 ** (e - 4) for e in range(-6, 9) for k in range(8, 16)], dtype=np.float64)
    mids = mids[mids < 448]
    out = []
    for a in _bf16(np.array([1.0, 3.0, 0.4375, 7.0, 448.0, 1.75, 96.0, 0.109375, 5.5, 224.0], dtype=np.float32)):
        d = np.float32(max(a, np.float32(1e-8))) / np.float32(448.0)
        x = (mids * float(a) / 448.0).astype(np.float32)
        x = x[_bf16(x) == x]                                     # numerators that are bf16 values
        if x.size == 0:
            continue
        dd = np.full(x.shape, d, dtype=np.float32)
        out.append(np.array_equal(_step(x, dd).view(np.uint32), (x / dd).astype(np.float32).view(np.uint32)))
    assert out and all(out)
