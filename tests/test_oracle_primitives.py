"""Pins of the oracle's primitives: the random generator, the two quantizers,
data quantization and index sampling (no GPU)."""
import os

import numpy as np
import pytest

from oracle import ref

GOLDEN = os.path.join(os.path.dirname(__file__), "golden")


# ------------------------------------------------------------------ Philox

def _kat_rows():
    rows = []
    with open(os.path.join(GOLDEN, "philox4x32_10_kat.txt")) as f:
        for line in f:
            line = line.strip()
            if not line or line.startswith("#"):
                continue
            v = [int(t, 16) for t in line.split()]
            rows.append((v[0:4], v[4:6], v[6:10]))
    return rows


def test_philox_known_answers():
    """Published known-answer vectors of Philox4x32-10 (SC'11 paper's generator)."""
    rows = _kat_rows()
    assert len(rows) == 3
    for ctr, key, want in rows:
        got = ref.philox4x32_10(ctr, key)
        assert [int(x) for x in got] == want


def test_philox_is_a_bijection_on_small_counter_range():
    """Distinct counters give distinct blocks (the round function is a permutation)."""
    seen = set()
    for c0 in range(2000):
        out = tuple(int(x) for x in ref.philox4x32_10([c0, 0, 7, 2], [123, 456]))
        assert out not in seen
        seen.add(out)


def test_stream_word_layout():
    """word n of a purpose's stream = word n%4 of block n/4, counter (lo, hi, epoch, purpose)."""
    seed = 0x0123456789ABCDEF
    for n in [0, 1, 2, 3, 4, 5, 1023, (1 << 34) + 6]:
        blk = n >> 2
        out = ref.philox4x32_10([blk & 0xFFFFFFFF, blk >> 32, 9, ref.PURPOSE_GAMMA],
                                [seed & 0xFFFFFFFF, seed >> 32])
        assert ref.stream_word(seed, ref.PURPOSE_GAMMA, 9, n) == int(out[n & 3])


@pytest.mark.parametrize("b", [8, 16])
def test_zround_bits_layout(b):
    """16/b coordinates form a strip; a strip shares one block with the eight steps 8s..8s+7."""
    seed, epoch, d = 99, 3, 51
    cps = 16 // b
    U = (d + cps - 1) // cps
    for c in range(2):
        for j in [0, 1, cps - 1, cps, d - 2, d - 1]:
            for t in [0, 1, 2, 7, 8, 13, 2 ** 33 + 5]:
                out = ref.philox4x32_10([c * U + j // cps, (t >> 3) & 0xFFFFFFFF, epoch,
                                         ref.PURPOSE_ZROUND], [seed, 0])
                bits = 0
                for k, w in enumerate(out):
                    bits |= int(w) << (32 * k)
                pos = (t & 7) * 16 + (j % cps) * b
                want = (bits >> pos) & ((1 << b) - 1)
                assert ref.zround_bits(seed, epoch, t, d, b, c, j) == want


def test_random_bits_statistics():
    """Per-bit frequency and byte chi-square of the rounding stream."""
    d, b = 512, 8
    vals = np.array([ref.zround_bits(5, 0, t, d, b, 0, j) for t in range(40) for j in range(d)])
    n = vals.size
    for bit in range(8):
        ones = np.count_nonzero((vals >> bit) & 1)
        assert abs(ones - n / 2) < 5 * np.sqrt(n / 4)
    counts = np.bincount(vals, minlength=256)
    chi2 = np.sum((counts - n / 256) ** 2 / (n / 256))
    assert chi2 < 255 + 6 * np.sqrt(2 * 255)


# ------------------------------------------------------------- Q int -> int

@pytest.mark.parametrize("b", [8, 16])
def test_round_shift_exactly_unbiased(b):
    """Exhaustive over all 2^b draws: the mean of Q(u) is exactly u (in units of
    delta_m) and the variance is frac (1 - frac) <= 1/4 (proof of Lemma 1)."""
    rng = np.random.default_rng(0)
    M = 1 << b
    cases = [(0, 0), (3, 1), (-5, -1), (0, M - 1), (0, -(M - 1)), (10, 17 * M + 5), (-20, -3 * M - 77)]
    cases += [(int(rng.integers(-40, 40)), int(rng.integers(-20 * M, 20 * M))) for _ in range(6)]
    for z, v in cases:
        outs = np.array([ref.round_shift(z, v, r, b)[0] for r in range(M)], dtype=np.int64)
        assert outs.sum() * 1 == z * M + v  # sum over draws == 2^b * (z + v/2^b), exactly
        frac = (v % M) / M
        var = np.mean((outs - (z + v / M)) ** 2)
        assert abs(var - frac * (1 - frac)) < 1e-12
        assert var <= 0.25 + 1e-12
        assert set(outs.tolist()) <= {z + v // M, z + v // M + 1}


@pytest.mark.parametrize("b", [8, 16])
def test_round_shift_clamps_to_nearest_end(b):
    qmax, qmin = 2 ** (b - 1) - 1, -(2 ** (b - 1))
    M = 1 << b
    for r in [0, 1, M - 1]:
        assert ref.round_shift(qmax, 5 * M, r, b) == (qmax, True)
        assert ref.round_shift(qmin, -5 * M, r, b) == (qmin, True)
        assert ref.round_shift(0, 10 * M * M, r, b) == (qmax, True)
    # the domain is asymmetric: -2^(b-1) is representable, +2^(b-1) is not
    assert ref.round_shift(qmin + 1, -M, 0, b) == (qmin, False)
    assert ref.round_shift(qmax - 1, M, 0, b) == (qmax, False)
    assert ref.round_shift(qmax, M, 0, b) == (qmax, True)


def test_round_shift_zero_is_fixed():
    """z_{k,0} = Q(0) = 0 for every draw."""
    for r in range(256):
        assert ref.round_shift(0, 0, r, 8) == (0, False)


# ------------------------------------------------------------ Q real -> int

def test_quantize_real_rule():
    inv = 1.0 / 0.25
    # Q(0) = 0 for every rho
    for r in [0, 1, 2 ** 31, 2 ** 32 - 1]:
        assert ref.quantize_real(0.0, inv, r, -128, 127) == (0, False)
    # lattice points are fixed points
    for q in [-128, -3, 0, 5, 127]:
        for r in [0, 2 ** 32 - 1]:
            assert ref.quantize_real(q * 0.25, inv, r, -128, 127)[0] == q
    # x = 1.3 delta: up iff rho >= 0.7
    x = 1.3 * 0.25
    thr = int(np.ceil((1 - 0.3) * 2 ** 32))
    assert ref.quantize_real(x, inv, thr - 2, -128, 127)[0] == 1
    assert ref.quantize_real(x, inv, thr + 2, -128, 127)[0] == 2
    # negative side: -1.3 delta lies between -2 and -1; up (to -1) with probability 0.7
    thr = int(np.ceil((1 - 0.7) * 2 ** 32))
    assert ref.quantize_real(-x, inv, thr - 2, -128, 127)[0] == -2
    assert ref.quantize_real(-x, inv, thr + 2, -128, 127)[0] == -1
    # outside the domain: nearest end, whatever the draw
    for r in [0, 2 ** 32 - 1]:
        assert ref.quantize_real(1000.0, inv, r, -128, 127) == (127, True)
        assert ref.quantize_real(-1000.0, inv, r, -128, 127) == (-128, True)


def test_quantize_real_monotone_in_draw_and_unbiased():
    rng = np.random.default_rng(1)
    inv = 1.0 / 0.01
    for x in [0.0371, -0.0029, 0.5]:
        draws = rng.integers(0, 2 ** 32, size=20000, dtype=np.uint64)
        outs = np.array([ref.quantize_real(x, inv, int(r), -32768, 32767)[0] for r in draws])
        order = np.argsort(draws)
        assert np.all(np.diff(outs[order]) >= 0)
        frac = x * inv - np.floor(x * inv)
        sigma = np.sqrt(max(frac * (1 - frac), 1e-12) / draws.size)
        assert abs(outs.mean() * 0.01 - x) < 5 * sigma * 0.01 + 1e-9


def test_lemma1_bound_monte_carlo():
    """E (Q(w) - w*)^2 <= (w - w*)^2 + delta^2/4 for w* inside the domain (Lemma 1, d = 1)."""
    rng = np.random.default_rng(2)
    delta, b = 0.1, 4
    lo, hi = -8, 7
    for w, wstar in [(0.234, -0.31), (0.95, 0.7), (-1.3, -0.8), (0.05, 0.0)]:
        draws = rng.integers(0, 2 ** 32, size=20000, dtype=np.uint64)
        q = np.array([ref.quantize_real(w, 1 / delta, int(r), lo, hi)[0] for r in draws]) * delta
        lhs = np.mean((q - wstar) ** 2)
        assert lhs <= (w - wstar) ** 2 + delta ** 2 / 4 + 4 * delta ** 2 / np.sqrt(draws.size)


# --------------------------------------------------------- data quantization

@pytest.mark.parametrize("b", [8, 16])
def test_quantize_data(b):
    rng = np.random.default_rng(3)
    X = rng.standard_normal((37, 19)).astype(np.float32)
    qmax = 2 ** (b - 1) - 1
    delta_d = float(np.abs(X).max()) / qmax
    Xq = ref.quantize_data(X, delta_d, b)
    assert Xq.dtype == (np.int8 if b == 8 else np.int16)
    assert Xq.max() <= qmax and Xq.min() >= -qmax  # symmetric range
    assert np.max(np.abs(Xq.astype(np.float64) * delta_d - X)) <= delta_d / 2 * (1 + 1e-9)
    # ties go to even; large values clamp
    T = np.array([0.5, 1.5, 2.5, -0.5, -1.5, 1e9, -1e9], dtype=np.float32)
    got = ref.quantize_data(T, 1.0, b)
    assert got.tolist() == [0, 2, 2, 0, -2, qmax, -qmax]
    # agrees with numpy's rint on the same fp64 quotient
    want = np.clip(np.rint(X.astype(np.float64) / delta_d), -qmax, qmax)
    assert np.array_equal(Xq.astype(np.float64), want)


# ------------------------------------------------------------ index sampling

def test_sample_index_range_and_uniformity():
    N, B = 37, 3
    idx = np.array([ref.sample_index(11, 2, t, B, m, N) for t in range(4000) for m in range(B)])
    assert idx.min() >= 0 and idx.max() < N
    counts = np.bincount(idx, minlength=N)
    chi2 = np.sum((counts - idx.size / N) ** 2 / (idx.size / N))
    assert chi2 < (N - 1) + 6 * np.sqrt(2 * (N - 1))
    # slot (t, m) reads word t*B+m of the IDX stream
    r = ref.stream_word(11, ref.PURPOSE_IDX, 2, 5 * B + 1)
    assert ref.sample_index(11, 2, 5, B, 1, N) == (r * N) >> 32


# -------------------------------------------------- exp of the inner loop

def test_inner_exp_is_within_one_ulp_of_exp():
    """Against exp computed to 50 digits on sampled points (all magnitudes, subnormal results
    included), and against libm on a dense sample."""
    from decimal import Decimal, getcontext
    getcontext().prec = 50
    rng = np.random.default_rng(0)
    x = np.concatenate([rng.uniform(-745.0, 709.7, 1500), rng.uniform(-30, 30, 1500),
                        rng.normal(0, 1, 1000), rng.uniform(-1e-6, 1e-6, 200),
                        np.array([0.5, -0.5, np.log(2.0), -np.log(2.0) / 2, 1.0, -1.0, 100.0, -100.0])])
    e = ref.exp_inner(x)
    for xv, ev in zip(x, e):
        exact = Decimal(float(xv)).exp()
        assert abs(Decimal(float(ev)) - exact) <= Decimal(float(np.spacing(ev))), xv
    xs = np.concatenate([rng.uniform(-700, 700, 500_000), rng.uniform(-20, 20, 500_000)])
    es, ts = ref.exp_inner(xs), np.exp(xs)
    assert np.all(np.abs(es - ts) <= 2 * np.spacing(ts))


def test_inner_exp_special_values():
    x = np.array([0.0, -0.0, -np.inf, np.inf, -745.2, -800.0, 709.79, 1e6])
    assert np.array_equal(ref.exp_inner(x), np.array([1.0, 1.0, 0.0, np.inf, 0.0, 0.0, np.inf, np.inf]))
    assert np.isnan(ref.exp_inner(np.array([np.nan]))[0])
    assert np.isfinite(ref.exp_inner(np.array([709.78]))[0])
    tiny = ref.exp_inner(np.array([-745.0, -744.0, -710.0]))  # subnormal results
    assert np.all(tiny > 0) and np.all(tiny < 2.3e-308)
    grid = np.linspace(-5, 5, 200_001)  # monotone
    assert np.all(np.diff(ref.exp_inner(grid)) >= 0)
