"""Arithmetic facts the kernels rely on, checked on the CPU in fp64 (no GPU, no library call).

* The cell selection's sweeps (Alg. 3, first loop) multiply the bf16 "hi" parts of queries and centroids
  alone (8 significant bits: a hi part is within 2^-8 of its value) and widen every compared value by
  t = c |y| |c_j| with c = 2^-6 * 1.02 (2^-7 * 1.02 when the queries are their own hi parts), twice the bound of the
  inner product checked here.  The encoder's split product hi.hi + hi.lo + lo.hi is taken to be within 3 * 2^-16.
  The bounds must hold for any input, so they are checked on random vectors and on vectors built to align every
  rounding error.
* The neighbour products add the 16 partial sums of a row across 16 lanes while transposing them (register s of
  lane l holds row s ^ g(l)).  The map g must make every exchange step meet the same row in the partner lane.
"""
import numpy as np
import pytest


def bf16_rne(x):
    """Round fp32 values to bf16 (round to nearest, ties to even), returned as fp32."""
    u = np.asarray(x, dtype=np.float32).view(np.uint32).astype(np.uint64)
    r = ((u + 0x7FFF + ((u >> 16) & 1)) >> 16) << 16
    return r.astype(np.uint32).view(np.float32)


def product_error(a, b):
    ah, bh = bf16_rne(a).astype(np.float64), bf16_rne(b).astype(np.float64)
    a64, b64 = a.astype(np.float64), b.astype(np.float64)
    return abs(a64 @ b64 - ah @ bh), np.linalg.norm(a64) * np.linalg.norm(b64)


@pytest.mark.parametrize("D", [32, 96, 128])
def test_hi_only_product_stays_inside_its_band(D):
    rng = np.random.default_rng(D)
    worst = 0.0
    for trial in range(400):
        kind = trial % 4
        if kind == 0:  # real-valued, isotropic
            a, b = rng.normal(size=D), rng.normal(size=D)
        elif kind == 1:  # wide dynamic range
            a = rng.normal(size=D) * np.exp(rng.normal(scale=3.0, size=D))
            b = rng.normal(size=D) * np.exp(rng.normal(scale=3.0, size=D))
        elif kind == 2:  # every component just below a rounding boundary, errors aligned in sign
            e = rng.integers(-3, 4, size=D).astype(np.float64)
            a = (1.0 + 2.0 ** -8 - 2.0 ** -20) * 2.0 ** e
            b = (1.0 + 2.0 ** -8 - 2.0 ** -20) * 2.0 ** rng.integers(-3, 4, size=D)
        else:  # just above a boundary: both round up
            a = (1.0 + 2.0 ** -8 + 2.0 ** -20) * np.ones(D)
            b = (1.0 + 3 * 2.0 ** -8 + 2.0 ** -20) * np.ones(D)
        a, b = a.astype(np.float32), b.astype(np.float32)
        err, scale = product_error(a, b)
        assert err <= 2.0 ** -7 * 1.02 * scale, (trial, err / scale)
        worst = max(worst, err / scale)
    assert worst > 2.0 ** -8  # the adversarial vectors do come near the bound: the test is not vacuous


@pytest.mark.parametrize("D", [32, 128])
def test_hi_only_product_with_exact_rows_has_half_the_band(D):
    """Integer-valued descriptors (|v| <= 256 after the integer shift of the origin) are their own hi parts: only the
    centroids' rounding is left."""
    rng = np.random.default_rng(7 * D)
    for trial in range(300):
        a = rng.integers(-255, 256, size=D).astype(np.float32)
        assert (bf16_rne(a) == a).all()
        if trial % 2:
            b = (rng.normal(size=D) * 100).astype(np.float32)
        else:
            b = ((1.0 + 2.0 ** -8 - 2.0 ** -20) * 2.0 ** rng.integers(0, 8, size=D)).astype(np.float32)
        err, scale = product_error(a, b)
        assert err <= 2.0 ** -8 * 1.02 * scale, (trial, err / scale)


@pytest.mark.parametrize("D", [32, 128])
def test_split_product_stays_inside_its_band(D):
    rng = np.random.default_rng(11 * D)
    worst = 0.0
    for trial in range(400):
        if trial % 2:
            a, b = rng.normal(size=D), rng.normal(size=D) * np.exp(rng.normal(scale=3.0, size=D))
        else:  # hi and lo both just below their rounding boundaries
            a = (1.0 + 2.0 ** -8 - 2.0 ** -16 - 2.0 ** -22) * 2.0 ** rng.integers(-3, 4, size=D)
            b = (1.0 + 2.0 ** -8 - 2.0 ** -16 - 2.0 ** -22) * 2.0 ** rng.integers(-3, 4, size=D)
        a, b = a.astype(np.float32), b.astype(np.float32)
        ah, bh = bf16_rne(a), bf16_rne(b)
        al, bl = bf16_rne(a - ah), bf16_rne(b - bh)
        f = lambda x: x.astype(np.float64)
        got = f(ah) @ f(bh) + f(ah) @ f(bl) + f(al) @ f(bh)
        scale = np.linalg.norm(f(a)) * np.linalg.norm(f(b))
        err = abs(f(a) @ f(b) - got)
        assert err <= 3 * 2.0 ** -16 * 1.01 * scale, (trial, err / scale)
        worst = max(worst, err / scale)
    assert worst > 2.0 ** -18


def g(l):
    """Row offset of register 0 in lane l of a group of 16 (the kernel's map)."""
    return (l & 3) ^ (7 if l & 4 else 0) ^ (12 if l & 8 else 0)


def test_transposing_reduction_meets_the_same_row_at_every_step():
    """Steps of the 16-lane sum: neighbour (l ^ 1), other pair of the quad (l ^ 2), other quad of the half (mirror inside
    8 lanes: l ^ 7), other half (mirror inside 16: l ^ 15).  At step k a lane keeps its registers s = 0 mod 2^(k+1) and
    takes the partner's register s + 2^k: both must belong to the same row, and in the end every lane holds another row."""
    assert sorted(g(l) for l in range(16)) == list(range(16))
    for k, partner in enumerate((1, 2, 7, 15)):
        step = 1 << k
        for l in range(16):
            for s in range(0, 16, 2 * step):
                assert s ^ g(l) == (s + step) ^ g(l ^ partner), (k, l, s)


def test_transposing_reduction_adds_what_the_butterfly_adds():
    """The same additions in the same association as the plain 16-lane butterfly, so the fp32 sums are identical:
    simulated here in fp32 for random partial sums."""
    rng = np.random.default_rng(3)
    p = (rng.normal(size=(16, 16)) * np.exp(rng.normal(scale=4.0, size=(16, 16)))).astype(np.float32)  # [row][lane]
    # plain butterfly, row by row
    want = np.empty(16, np.float32)
    for r in range(16):
        v = p[r].copy()
        for partner in (1, 2, 7, 15):
            v = (v + v[[l ^ partner for l in range(16)]]).astype(np.float32)
        assert (v == v[0]).all()
        want[r] = v[0]
    # transposing form: reg[l][s] holds row s ^ g(l)
    reg = np.empty((16, 16), np.float32)
    for l in range(16):
        for s in range(16):
            reg[l][s] = p[s ^ g(l)][l]
    for k, partner in enumerate((1, 2, 7, 15)):
        step = 1 << k
        new = reg.copy()
        for l in range(16):
            for s in range(0, 16, 2 * step):
                new[l][s] = np.float32(reg[l][s] + reg[l ^ partner][s + step])
        reg = new
    for l in range(16):
        assert reg[l][0] == want[g(l)]
