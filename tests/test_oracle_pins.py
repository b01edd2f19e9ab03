"""Pins of the CPU oracle against what the paper and the mathematics fix.

None of these tests touches the HIP library.  Each one checks the oracle
against something other than its own formula: hand-worked fixtures
(tests/golden), closed forms, invariants, special cases that reduce to
S-SGD (eq. 1), exact rational arithmetic, or a table of expected outcomes
on tiny inputs.
"""
import os
from fractions import Fraction

import numpy as np
import pytest

GOLDEN = os.path.join(os.path.dirname(os.path.abspath(__file__)), "golden")
F32 = np.float32


def f32(x):
    return np.array(x, dtype=np.float32).reshape(-1)


# --------------------------------------------------------------------------
# fixtures worked by hand
# --------------------------------------------------------------------------
def _read_golden(name):
    rows = []
    with open(os.path.join(GOLDEN, name)) as fh:
        for line in fh:
            line = line.strip()
            if line and not line.startswith("#"):
                rows.append(line)
    return rows


def test_hand_unrolled_recurrence(oracle):
    """eq. 10 / eq. 11 / Alg. 1 unrolled by hand for n=1, N=2, k=2 (exact in fp32)."""
    rows = _read_golden("hand_unrolled_n1_N2_k2.txt")
    assert rows[0].startswith("setup")
    _, n, N, k, t, lrl, lrg, w0 = rows[0].split()
    n, N, k = int(n), int(N), int(k)
    sim = oracle.Simulation(f32([float(w0)] * n), N, k, float(t), float(lrl), float(lrg))
    steps = 0
    for row in rows[1:]:
        lhs, rhs = row.split("|")
        g = [float(x) for x in lhs.split()[1:]]
        mode, agg, W, Wloc, r0, r1, w_0, w_1 = rhs.split()
        comp, got_agg, words = sim.step([f32([g[0]]), f32([g[1]])])
        assert comp == (mode == "comp")
        assert got_agg[0] == F32(float(agg))
        assert sim.w_global[0] == F32(float(W))
        assert sim.w_local[0] == F32(float(Wloc))
        assert sim.residual[0][0] == F32(float(r0))
        assert sim.residual[1][0] == F32(float(r1))
        if comp:
            assert int(words[0][0]) == int(w_0) and int(words[1][0]) == int(w_1)
        else:
            assert words is None and int(w_0) == -1
        steps += 1
    assert steps == 4


def test_pack_layout_fixture(oracle):
    rows = _read_golden("pack_layout_n18.txt")
    codes = np.array([int(x) for x in rows[0].split()[1:]], np.uint8)
    words = np.array([int(x, 16) for x in rows[1].split()[1:]], np.uint32)
    got = oracle.pack(codes)
    assert got.tolist() == words.tolist()
    assert oracle.unpack(words, codes.size).tolist() == codes.tolist()


# --------------------------------------------------------------------------
# pack / unpack
# --------------------------------------------------------------------------
def test_pack_roundtrip_every_tail(oracle):
    rng = np.random.default_rng(7)
    for n in range(1, 71):
        code = rng.integers(0, 3, n).astype(np.uint8)
        w = oracle.pack(code)
        assert w.size == (n + 15) // 16
        # independent statement of the layout with Python integers
        expect = [0] * w.size
        for e, c in enumerate(code.tolist()):
            expect[e // 16] += c * 4 ** (e % 16)
        assert [int(x) for x in w] == expect
        assert oracle.unpack(w, n).tolist() == code.tolist()


def test_pack_overwrites_stale_words(oracle):
    # pad bits of the last word must be zero whatever the buffer held before
    import ctypes
    code = np.array([1, 2, 1], np.uint8)
    word = np.full(1, 0xFFFFFFFF, np.uint32)
    oracle.lib().oracle_pack(code.ctypes.data_as(ctypes.POINTER(ctypes.c_uint8)), 3,
                             word.ctypes.data_as(ctypes.POINTER(ctypes.c_uint32)))
    assert int(word[0]) == 1 + 2 * 4 + 1 * 16


# --------------------------------------------------------------------------
# quantiser: outcome table on tiny inputs, brute force
# --------------------------------------------------------------------------
# Sec. 3.4.1: a value beyond the threshold is sent as the threshold, the error
# stays behind; below it nothing is sent.  "Reaches the threshold" (Sec. 2.3)
# is read as |a| >= t.  For t = 0.5 the five offered values below have these
# outcomes (code, kept residual):
_T = 0.5
_A = np.array([-0.75, -0.5, 0.0, 0.5, 0.75], np.float32)
_CODE = np.array([2, 2, 0, 1, 1], np.uint8)
_KEEP = np.array([-0.25, 0.0, 0.0, 0.0, 0.25], np.float32)


@pytest.mark.parametrize("r0", [0.0, 0.125, -0.375])
def test_bruteforce_all_8_element_inputs(oracle, r0):
    """All 5^8 = 390625 eight-element inputs: codes, residuals and packed word."""
    idx = np.indices((5,) * 8).reshape(8, -1).T  # (390625, 8) digits
    a = _A[idx]
    r = np.full(a.shape, r0, np.float32)
    g = (a - r).astype(np.float32)  # exact: all values are multiples of 1/8
    assert np.array_equal((r + g).astype(np.float32), a)
    gf = np.ascontiguousarray(g.reshape(-1))
    rf = np.ascontiguousarray(r.reshape(-1))
    code = oracle.quantize(gf, rf, _T)
    assert np.array_equal(code.reshape(-1, 8), _CODE[idx])
    assert np.array_equal(rf.reshape(-1, 8), _KEEP[idx])
    # every 8-element row is packed on its own (one word per row)
    pow4 = (4 ** np.arange(8)).astype(np.int64)
    expect_words = (_CODE[idx].astype(np.int64) * pow4).sum(axis=1)
    # pack 16 elements per word: two rows share a word -> low half / high half
    words = oracle.pack(code)
    lo = (words.astype(np.int64) & 0xFFFF)
    hi = (words.astype(np.int64) >> 16)
    got = np.empty(expect_words.size + (expect_words.size % 2), np.int64)
    got[0::2] = lo
    got[1::2] = hi
    assert np.array_equal(got[: expect_words.size], expect_words)
    if expect_words.size % 2:
        assert got[-1] == 0  # padding of the ragged last word


def test_emitted_values_are_threshold_or_zero(oracle):
    for c, v in ((0, 0.0), (1, 0.3), (2, -0.3), (3, 0.0)):
        assert oracle.dequant(c, 0.3) == F32(v)


def test_special_values(oracle):
    """NaN is never sent and stays NaN; infinities are sent; denormals survive."""
    den = np.float32(1e-45)  # smallest positive denormal
    g = f32([np.nan, np.inf, -np.inf, den, -den, 0.0])
    r = np.zeros(6, np.float32)
    code = oracle.quantize(g, r, 0.5)
    assert code.tolist() == [0, 1, 2, 0, 0, 0]
    assert np.isnan(r[0]) and r[1] == np.inf and r[2] == -np.inf
    assert r[3] == den and r[4] == -den and r[3] != 0.0
    # two denormals add to a denormal (no flush to zero)
    g2 = f32([den])
    r2 = f32([den])
    oracle.quantize(g2, r2, 0.5)
    assert r2[0] == np.float32(3e-45) and r2[0] > den


# --------------------------------------------------------------------------
# invariants
# --------------------------------------------------------------------------
def test_conservation_exact_for_dyadic_inputs(oracle):
    """Nothing is lost: sum(g) + r_start == sum(sent) + r_end, exactly."""
    rng = np.random.default_rng(11)
    n, S, t = 4099, 40, 0.5
    r = (rng.integers(-400, 401, n) / 1024.0).astype(np.float32)
    r_start = r.astype(np.float64)
    sum_g = np.zeros(n, np.float64)
    sum_sent = np.zeros(n, np.float64)
    lut = np.array([0.0, t, -t, 0.0])
    for _ in range(S):
        g = (rng.integers(-2047, 2048, n) / 1024.0).astype(np.float32)
        r_before = r.copy()
        code = oracle.quantize(g, r, t)
        assert set(np.unique(code).tolist()) <= {0, 1, 2}
        # per step, exactly
        assert np.array_equal(g.astype(np.float64) + r_before, lut[code] + r.astype(np.float64))
        sum_g += g
        sum_sent += lut[code]
    assert np.array_equal(sum_g + r_start, sum_sent + r.astype(np.float64))
    assert (sum_sent != 0).mean() > 0.5  # the run really sent something


def test_conservation_general_inputs_one_rounding(oracle):
    """For arbitrary fp32 inputs the only error is the rounding of a = r + g."""
    rng = np.random.default_rng(12)
    n, t = 20000, 0.05
    r = rng.normal(0, 0.03, n).astype(np.float32)
    g = rng.laplace(0, 0.02, n).astype(np.float32)
    r0 = r.copy()
    code = oracle.quantize(g, r, t)
    t32 = float(np.float32(t))
    lut = np.array([0.0, t32, -t32, 0.0])
    a = (r0.astype(np.float64) + g.astype(np.float64))
    a32 = (r0 + g).astype(np.float32)
    resid = lut[code] + r.astype(np.float64) - a
    ulp = np.spacing(np.abs(a32)).astype(np.float64)
    assert np.all(np.abs(resid) <= ulp)
    # the decision is taken on the rounded fp32 sum
    assert np.array_equal(code == 1, a32 >= np.float32(t))
    assert np.array_equal(code == 2, a32 <= -np.float32(t))
    assert (code != 0).mean() > 0.05


def test_residual_stays_below_threshold(oracle):
    """Theorem 1's remark: what waits in the residual is bounded by the threshold."""
    rng = np.random.default_rng(13)
    n, t = 5000, 0.5
    r = np.zeros(n, np.float32)
    for _ in range(60):
        g = rng.uniform(-t, t, n).astype(np.float32)
        oracle.quantize(g, r, t)
        assert np.all(np.abs(r) < t)


def test_clipping_growth_closed_form(oracle):
    """Constant g > t: every step sends +t and the residual grows by g - t."""
    g = f32([0.75, -0.875])
    r = np.zeros(2, np.float32)
    for s in range(1, 33):
        code = oracle.quantize(g, r, 0.5)
        assert code.tolist() == [1, 2]
        assert r.tolist() == [s * 0.25, -s * 0.375]


@pytest.mark.parametrize("num,den", [(3, 16), (1, 4), (7, 64), (-5, 32), (-1, 2), (1, 2)])
def test_sigma_delta_closed_form(oracle, num, den):
    """Constant |g| <= t from r = 0 is a first-order error-diffusion accumulator:
    after S steps floor(S|g|/t) codes were sent and r = S g - sign * t * floor(S|g|/t)."""
    t = 0.5
    gval = num / den
    g = f32([gval])
    r = np.zeros(1, np.float32)
    sent = 0
    for S in range(1, 101):
        code = oracle.quantize(g, r, t)
        sent += int(code[0] != 0)
        if code[0]:
            assert code[0] == (1 if gval > 0 else 2)
        cnt = (Fraction(abs(num), den) * S) // Fraction(1, 2)
        assert sent == cnt
        expect_r = Fraction(num, den) * S - (1 if gval > 0 else -1) * Fraction(1, 2) * cnt
        assert Fraction(float(r[0])) == expect_r


def test_all_below_threshold(oracle):
    """While sum |g| < t nothing is sent: words 0, residual = running sum, W fixed."""
    rng = np.random.default_rng(14)
    n, N, k, S = 37, 3, 100, 9
    w0 = rng.normal(0, 1, n).astype(np.float32)
    sim = oracle.Simulation(w0, N, k, 0.5, 0.25, 0.25)
    run = [np.zeros(n, np.float32) for _ in range(N)]
    for s in range(S):
        grads = [(rng.integers(-50, 51, n) / 1024.0).astype(np.float32) for _ in range(N)]
        w_before = sim.w_global.copy()
        comp, agg, words = sim.step(grads)
        if s == 0:
            assert not comp
            continue
        assert comp
        for j in range(N):
            run[j] = (run[j] + grads[j]).astype(np.float32)
            assert np.array_equal(sim.residual[j], run[j])
            assert not words[j].any()
        assert not agg.any()
        assert np.array_equal(sim.w_global, w_before)
        expect_loc = (w_before.astype(np.float64) - 0.25 * grads[0].astype(np.float64))
        assert np.allclose(sim.w_local, expect_loc, rtol=0, atol=1e-7)


# --------------------------------------------------------------------------
# update rules
# --------------------------------------------------------------------------
def _round_f32(x: Fraction) -> np.float32:
    """Correctly rounded (nearest-even) fp32 of an exact rational."""
    c = np.float32(float(x))
    cands = {c, np.nextafter(c, np.float32(np.inf)), np.nextafter(c, np.float32(-np.inf))}
    best = None
    for v in cands:
        d = abs(Fraction(float(v)) - x)
        key = (d, int(np.float32(v).view(np.uint32)) & 1)  # tie -> even mantissa
        if best is None or key < best[0]:
            best = (key, v)
    return np.float32(best[1])


def test_update_is_one_rounding_of_the_exact_rule(oracle):
    """eq. 10 and eq. 11 evaluated in exact rational arithmetic, rounded once."""
    rng = np.random.default_rng(15)
    n, N = 64, 3
    W = rng.normal(0, 1, n).astype(np.float32)
    g = rng.normal(0, 1, n).astype(np.float32)
    agg = rng.normal(0, 2, n).astype(np.float32)
    lr_l, lr_g = np.float32(0.1), np.float32(0.3)
    scale = np.float32(lr_g / np.float32(N))
    W0 = W.copy()
    Wloc = np.zeros(n, np.float32)
    oracle.update(W, Wloc, g, agg, float(lr_l), float(lr_g), N)
    differs_from_two_roundings = 0
    for e in range(n):
        loc = _round_f32(Fraction(float(W0[e])) - Fraction(float(lr_l)) * Fraction(float(g[e])))
        glo = _round_f32(Fraction(float(W0[e])) - Fraction(float(scale)) * Fraction(float(agg[e])))
        assert Wloc[e] == loc and W[e] == glo
        two = np.float32(W0[e] - np.float32(lr_l * g[e]))
        differs_from_two_roundings += int(two != loc)
    assert differs_from_two_roundings > 0  # the test can tell fma from mul-then-add


def test_update_optional_halves(oracle):
    W = f32([1.0, 2.0])
    Wloc = f32([9.0, 9.0])
    g = f32([0.5, -0.5])
    agg = f32([1.0, 1.0])
    oracle.update(W, None, None, agg, 0.25, 0.5, 2)       # global only
    assert W.tolist() == [0.75, 1.75] and Wloc.tolist() == [9.0, 9.0]
    oracle.update(W, Wloc, g, None, 0.25, 0.5, 2)         # local only
    assert W.tolist() == [0.75, 1.75] and Wloc.tolist() == [0.625, 1.875]


def test_local_and_global_start_from_the_same_weight(oracle):
    """eq. 11 uses W_k, not W_{k+1}: the local rule must not see this step's aggregate."""
    W = f32([1.0])
    Wloc = f32([0.0])
    oracle.update(W, Wloc, f32([1.0]), f32([4.0]), 0.5, 0.5, 1)
    assert Wloc[0] == 0.5      # 1 - 0.5*1, not (1 - 0.5*4) - 0.5*1
    assert W[0] == -1.0


def test_reduces_to_ssgd_when_gradients_are_plus_minus_t(oracle):
    """g in {-t, 0, +t}: decoding returns g itself, so eq. 10 is eq. 1."""
    rng = np.random.default_rng(16)
    n, N, S, t, lr = 53, 4, 12, 0.5, 0.125
    w0 = (rng.integers(-4096, 4096, n) / 256.0).astype(np.float32)
    sim = oracle.Simulation(w0, N, 3, t, lr, lr)
    ref = w0.astype(np.float64)
    for s in range(S):
        grads = [(rng.integers(-1, 2, n) * t).astype(np.float32) for _ in range(N)]
        sim.step(grads)
        ref = ref - (lr / N) * np.sum([g.astype(np.float64) for g in grads], axis=0)  # eq. 1, exact
        assert np.array_equal(sim.w_global.astype(np.float64), ref)
        for j in range(N):
            assert not sim.residual[j].any()


def test_k1_is_ssgd_for_any_gradient(oracle):
    rng = np.random.default_rng(17)
    n, N, S, lr = 40, 5, 6, 0.1
    w0 = rng.normal(0, 1, n).astype(np.float32)
    sim = oracle.Simulation(w0, N, 1, 0.5, lr, lr)
    ref = w0.astype(np.float64)
    for s in range(S):
        grads = [rng.normal(0, 1, n).astype(np.float32) for _ in range(N)]
        comp, _, words = sim.step(grads)
        assert not comp and words is None
        ref = ref - (float(np.float32(lr)) / N) * np.sum([g.astype(np.float64) for g in grads], axis=0)
        assert np.allclose(sim.w_global, ref, rtol=0, atol=(s + 1) * 4e-7)
        for j in range(N):
            assert not sim.residual[j].any()


def test_single_worker_local_equals_global(oracle):
    """N = 1, equal rates, g in {-t,0,+t}: eq. 10 and eq. 11 are the same rule."""
    rng = np.random.default_rng(18)
    n, t = 29, 0.25
    w0 = rng.normal(0, 1, n).astype(np.float32)
    sim = oracle.Simulation(w0, 1, 4, t, 0.3, 0.3)
    for s in range(10):
        g = (rng.integers(-1, 2, n) * t).astype(np.float32)
        sim.step([g])
        assert np.array_equal(sim.w_local, sim.w_global)


def test_mode_switch_and_untouched_state_on_correction(oracle):
    """Alg. 1: compress iff count % k != 0 (count from 0); a correction iteration
    does no quantisation, so residuals and packed buffers keep their contents."""
    rng = np.random.default_rng(19)
    n, N, k = 50, 3, 4
    sim = oracle.Simulation(np.zeros(n, np.float32), N, k, 0.5, 0.1, 0.1)
    modes = []
    for s in range(9):
        grads = [rng.normal(0, 0.6, n).astype(np.float32) for _ in range(N)]
        r_before = [r.copy() for r in sim.residual]
        w_before = [w.copy() for w in sim.word]
        comp, agg, _ = sim.step(grads)
        modes.append(comp)
        if not comp:
            for j in range(N):
                assert np.array_equal(sim.residual[j], r_before[j])
                assert np.array_equal(sim.word[j], w_before[j])
            exact = np.sum([g.astype(np.float64) for g in grads], axis=0)
            assert np.allclose(agg, exact, rtol=0, atol=1e-6)
    assert modes == [False, True, True, True, False, True, True, True, False]


def test_linearity_closed_form(oracle):
    """Gradients are exogenous, so W_S = W_0 - scale * sum_s agg_s and
    Wloc_{s+1} = W_s - lr_local * g_0^s (checked in double)."""
    rng = np.random.default_rng(20)
    n, N, k, S, t = 300, 4, 4, 16, 0.5
    lr_l, lr_g = 0.4, 0.1
    w0 = rng.normal(0, 0.2, n).astype(np.float32)
    sim = oracle.Simulation(w0, N, k, t, lr_l, lr_g)
    acc = np.zeros(n, np.float64)
    scale = float(np.float32(np.float32(lr_g) / np.float32(N)))
    for s in range(S):
        grads = [rng.normal(0, 0.3, n).astype(np.float32) for _ in range(N)]
        w_prev = sim.w_global.astype(np.float64)
        comp, agg, words = sim.step(grads)
        if comp:
            # the aggregate is an integer multiple of t between -N and N
            m = agg.astype(np.float64) / t
            assert np.array_equal(m, np.round(m)) and np.all(np.abs(m) <= N)
            # ... and equals what the words say, counted independently
            cnt = np.zeros(n, np.int64)
            for j in range(N):
                c = oracle.unpack(words[j], n).astype(np.int64)
                cnt += (c == 1).astype(np.int64) - (c == 2).astype(np.int64)
            assert np.array_equal(m.astype(np.int64), cnt)
        acc += agg
        assert np.allclose(sim.w_local, w_prev - float(np.float32(lr_l)) * grads[0], rtol=0, atol=2e-7)
        assert np.allclose(sim.w_global, w0 - scale * acc, rtol=0, atol=(s + 1) * 1.5e-7)


# --------------------------------------------------------------------------
# decode-and-sum
# --------------------------------------------------------------------------
def test_decode_sum_counts_and_unused_code(oracle):
    n, N, t = 45, 6, 0.5
    rng = np.random.default_rng(21)
    codes = rng.integers(0, 4, (N, n)).astype(np.uint8)       # includes the unused code 3
    words = [oracle.pack(np.ascontiguousarray(codes[j])) for j in range(N)]
    agg = oracle.decode_sum(words, n, t)
    cnt = (codes == 1).sum(axis=0).astype(np.int64) - (codes == 2).sum(axis=0)
    assert np.array_equal(agg.astype(np.float64), cnt * t)    # exact: t is a power of two


def test_decode_sum_is_sequential_in_worker_order(oracle):
    """With t = 0.05 the fp32 sum depends on the order; the oracle must add
    worker 0 first.  Checked against exact arithmetic rounded after every add."""
    t = np.float32(0.05)
    patterns = [   # chosen so that worker order and the m*t shortcut both change the result
        [1, 1, 1, 2, 0, 2, 2, 0, 1, 2, 1, 0, 2, 2, 2, 0],
        [0, 0, 1, 2, 1, 2, 0, 0, 2, 2, 0, 0, 2, 1, 1, 0],
        [2, 1, 2, 2, 2, 0, 2, 0, 1, 1, 2, 0, 2, 0, 1, 1],
        [1, 1, 0, 1, 2, 2, 0, 1, 2, 0, 0, 0, 0, 2, 0, 0],
        [1, 1, 1, 1, 1, 1, 1, 1, 1, 1, 1, 1, 1, 1, 1, 1],
    ]
    N = 16
    n = len(patterns)
    codes = np.array(patterns, np.uint8).T.copy()   # (N, n)
    words = [oracle.pack(np.ascontiguousarray(codes[j])) for j in range(N)]
    agg = oracle.decode_sum(words, n, float(t))
    def chain(seq):
        s = Fraction(0)
        for c in seq:
            d = {0: Fraction(0), 1: Fraction(float(t)), 2: -Fraction(float(t))}[int(c)]
            s = Fraction(float(_round_f32(s + d)))
        return s

    shortcut_differs = reverse_differs = 0
    for e in range(n):
        s = chain(codes[:, e])
        assert Fraction(float(agg[e])) == s
        m = int((codes[:, e] == 1).sum()) - int((codes[:, e] == 2).sum())
        shortcut_differs += (Fraction(float(_round_f32(m * Fraction(float(t))))) != s)
        reverse_differs += (chain(codes[::-1, e]) != s)
    assert shortcut_differs >= 3 and reverse_differs >= 3  # the patterns can tell


def test_first_step_fire_rate_matches_laplace_tail(oracle):
    """Statistical pin of quantiser + generator recipe: Laplace(0, b=0.02) against
    t = 0.05 fires with probability exp(-t/b) = exp(-2.5) on the first step."""
    rng = np.random.default_rng(22)
    n = 400000
    g = rng.laplace(0, 0.02, n).astype(np.float32)
    r = np.zeros(n, np.float32)
    code = oracle.quantize(g, r, 0.05)
    p = (code != 0).mean()
    assert abs(p - np.exp(-2.5)) < 4 * np.sqrt(np.exp(-2.5) / n)
    assert abs((code == 1).mean() - (code == 2).mean()) < 0.003


# --------------------------------------------------------------------------
# Alg. 1 end to end: WARMUP, then FormalTraining
# --------------------------------------------------------------------------
@pytest.mark.parametrize("fixture", ["hand_unrolled_warmup_n1.txt", "hand_unrolled_warmup_n0.txt"])
def test_hand_unrolled_warmup_then_formal(oracle, fixture):
    """Alg. 1 through WARMUP into FormalTraining, worked by hand.  The n = 0 fixture starts the
    local buffer at a sentinel that differs from W0: the local update of pass 0 must start from
    the global weight (eq. 11), and the first formal local update from the pulled W_{n+1}."""
    rows = _read_golden(fixture)
    fields = rows[0].split()
    _, n, N, wn, k, t, lrl, lrg, w0 = fields[:9]
    loc0 = f32([float(fields[9])] * int(n)) if len(fields) > 9 else None
    sim = oracle.TrainerSimulation(f32([float(w0)] * int(n)), int(N), int(wn), int(k), float(t), float(lrl),
                                   float(lrg), w_local0=loc0)
    steps = 0
    for row in rows[1:]:
        lhs, rhs = row.split("|")
        g = [float(x) for x in lhs.split()[1:]]
        mode, agg, W, Wloc, r0, r1 = rhs.split()
        got_mode, got_agg, _ = sim.step([f32([g[0]]), f32([g[1]])])
        assert got_mode == int(mode)
        assert got_agg[0] == F32(float(agg))
        assert sim.w_global[0] == F32(float(W))
        assert sim.w_local[0] == F32(float(Wloc))
        assert sim.residual[0][0] == F32(float(r0)) and sim.residual[1][0] == F32(float(r1))
        steps += 1
    assert steps == len(rows) - 1 >= 3


@pytest.mark.parametrize("warmup_n", [0, 1, 2, 5])
def test_warmup_is_ssgd_and_hands_over_to_formal_training(oracle, warmup_n):
    """WARMUP runs for i = 0..n as plain S-SGD (eq. 1, exact on dyadic inputs); the local
    buffer receives W_n after pass n-1 and W_n - lr_local * g_n in pass n; pass n+1 is
    FormalTraining's first pass (count 0, a correction pass), pass n+2 is compressed."""
    rng = np.random.default_rng(30 + warmup_n)
    n, N, k, t, lr_l, lr_g = 41, 4, 3, 0.5, 0.25, 0.125
    w0 = (rng.integers(-2048, 2048, n) / 64.0).astype(np.float32)
    # the local buffer starts at a sentinel unrelated to W0: Alg. 1 never reads it before writing it
    sentinel = np.full(n, -1234.5, np.float32)
    sim = oracle.TrainerSimulation(w0, N, warmup_n, k, t, lr_l, lr_g, self_rank=2, w_local0=sentinel)
    ref = w0.astype(np.float64)
    modes = []
    for it in range(warmup_n + 1 + 2 * k):
        grads = [(rng.integers(-64, 65, n) / 64.0).astype(np.float32) for _ in range(N)]
        w_before = sim.w_global.copy()
        loc_before = sim.w_local.copy()
        mode, agg, words = sim.step(grads)
        modes.append(mode)
        if it <= warmup_n:
            ref = ref - (lr_g / N) * np.sum([g.astype(np.float64) for g in grads], axis=0)
            assert np.array_equal(sim.w_global.astype(np.float64), ref)          # eq. 1, exactly
            for j in range(N):
                assert not sim.residual[j].any()
            if it == warmup_n - 1:
                assert np.array_equal(sim.w_local, sim.w_global)                 # copy after the pull
            elif it == warmup_n:
                assert np.array_equal(sim.w_local.astype(np.float64),
                                      w_before.astype(np.float64) - lr_l * grads[2].astype(np.float64))
            else:
                assert np.array_equal(sim.w_local, sentinel)                     # untouched before n-1
                assert np.array_equal(sim.w_local, loc_before)
        else:
            # formal training: local weights from the pre-pass global weights, own 32-bit gradient
            assert np.array_equal(sim.w_local.astype(np.float64),
                                  w_before.astype(np.float64) - lr_l * grads[2].astype(np.float64))
    expect = [0] * (warmup_n + 1) + [2 if c % k == 0 else 1 for c in range(2 * k)]
    assert modes == expect


# --------------------------------------------------------------------------
# sparse form of a packed stream (this build's wire format; pinned to its definition only)
# --------------------------------------------------------------------------
def test_sparse_layout_fixture(oracle):
    rows = _read_golden("sparse_layout_n4200.txt")
    n = int(rows[0].split()[1])
    word = np.zeros(oracle.packed_words(n), np.uint32)
    segs = {}
    for row in rows[1:]:
        f = row.split()
        if f[0] == "word":
            word[int(f[1])] = int(f[2], 16)
        else:
            assert f[0] == "segment" and f[2] == "bitmap" and f[11] == "values"
            segs[int(f[1])] = ([int(x, 16) for x in f[3:11]], [int(x, 16) for x in f[12:]])
    sparse, seg_words = oracle.sparse_encode(word, n, fill=0xDEADBEEF)
    assert oracle.sparse_segments(n) == len(segs) == 2 and sparse.size == 2 * 264
    for s_i, (bitmap, values) in segs.items():
        seg = sparse[264 * s_i: 264 * (s_i + 1)]
        assert [int(x) for x in seg[:8]] == bitmap
        assert [int(x) for x in seg[8: 8 + len(values)]] == values
        assert (seg[8 + len(values):] == 0xDEADBEEF).all()          # slots after the values are left alone
        assert int(seg_words[s_i]) == 8 + len(values)
    assert np.array_equal(oracle.sparse_decode(sparse, n), word)


def test_sparse_roundtrip_every_tail_and_density(oracle):
    rng = np.random.default_rng(11)
    sizes = list(range(1, 71)) + [4095, 4096, 4097, 4111, 8191, 8192, 8193, 3 * 4096 + 5, 16 * 256 * 5 + 16]
    for n in sizes:
        nw = oracle.packed_words(n)
        for density in (0.0, 1.0, 0.02, 0.5):
            word = rng.integers(1, 1 << 32, nw, dtype=np.uint64).astype(np.uint32)
            word[rng.random(nw) >= density] = 0
            sparse, seg_words = oracle.sparse_encode(word, n, fill=0xA5A5A5A5)
            assert sparse.size == 264 * ((nw + 255) // 256)
            # the format stated independently, in Python integers
            for s_i in range((nw + 255) // 256):
                part = [int(x) for x in word[256 * s_i: 256 * (s_i + 1)]]
                nz = [(i, v) for i, v in enumerate(part) if v]
                seg = sparse[264 * s_i: 264 * (s_i + 1)]
                bits = sum(1 << i for i, _ in nz)
                assert [int(x) for x in seg[:8]] == [(bits >> (32 * m)) & 0xFFFFFFFF for m in range(8)]
                assert [int(x) for x in seg[8: 8 + len(nz)]] == [v for _, v in nz]
                assert (seg[8 + len(nz):] == 0xA5A5A5A5).all()
                assert int(seg_words[s_i]) == 8 + len(nz)
            if density == 0.0:
                assert int(seg_words.sum()) == 8 * seg_words.size                    # bitmaps only
            if density == 1.0:
                assert int(seg_words.sum()) == 8 * seg_words.size + nw               # every word travels
            assert np.array_equal(oracle.sparse_decode(sparse, n), word)


def test_sparse_decode_then_sum_is_the_dense_sum(oracle):
    """The method is untouched by the wire format: decode-and-sum of streams that went through
    the sparse form equals decode-and-sum of the packed streams, for real quantiser output."""
    rng = np.random.default_rng(12)
    n, N, t = 10000, 5, 0.5
    words = []
    for j in range(N):
        g = rng.normal(0, 0.25 * (j + 1), n).astype(np.float32)
        words.append(oracle.quantize_pack(g, np.zeros(n, np.float32), t))
    through = [oracle.sparse_decode(oracle.sparse_encode(w, n)[0], n) for w in words]
    assert all(np.array_equal(a, b) for a, b in zip(words, through))
    assert np.array_equal(oracle.decode_sum(through, n, t), oracle.decode_sum(words, n, t))
    wire = sum(int(oracle.sparse_encode(w, n)[1].sum()) for w in words)
    assert wire < N * oracle.packed_words(n) + 8 * N * oracle.sparse_segments(n) + 1


# --------------------------------------------------------------------------
# time-cost model (Sec. 2.1-2.3, Sec. 3.3)
# --------------------------------------------------------------------------
def _eq8_table(tau, phi, psi, delta, k, i):
    """T_s^bit as the paper prints it (eq. 8)."""
    phi_cd = delta + psi if i % k != 0 else phi
    if tau > phi_cd:
        return delta + psi
    if i % k != 0:
        return tau
    return tau + delta + psi - phi


def _eq9_table(tau, phi, psi, delta, k, i):
    """T_s^loc as the paper prints it (eq. 9)."""
    phi_cd = delta + psi if i % k != 0 else phi
    if tau > phi:
        return 0.0
    if tau > phi_cd:
        return phi - tau
    if i % k != 0:
        return phi - delta - psi
    return 0.0


def test_cost_model_against_the_printed_case_tables(oracle):
    """The oracle computes iteration times from eq. 2, 4, 5, 6, 7 and the savings as
    differences; the paper prints the savings as case tables (eq. 8, eq. 9).  On dyadic
    inputs both must agree exactly (eq. 9 under its tacit assumption delta + psi <= phi)."""
    rng = np.random.default_rng(40)
    checked9 = 0
    seen8, seen9 = set(), set()
    for _ in range(4000):
        tau, phi, psi, delta = (float(x) / 8 for x in rng.integers(0, 80, 4))
        k = int(rng.integers(1, 7))
        i = int(rng.integers(0, 20))
        m = oracle.cost_model(tau, phi, psi, delta, k, i)
        assert m["t_ssgd"] == tau + phi                       # eq. 2
        assert m["t_bit"] == tau + delta + psi                # eq. 5
        assert m["t_loc"] == max(tau, phi)                    # eq. 4
        assert m["phi_cd"] == (phi if i % k == 0 else delta + psi)   # eq. 6
        assert m["t_cd"] == max(tau, m["phi_cd"])             # eq. 7
        assert m["save_vs_bit"] == _eq8_table(tau, phi, psi, delta, k, i)
        seen8.add((tau > m["phi_cd"], i % k != 0))
        if delta + psi <= phi:
            assert m["save_vs_loc"] == _eq9_table(tau, phi, psi, delta, k, i)
            checked9 += 1
            seen9.add((tau > phi, tau > m["phi_cd"], i % k != 0))
    assert checked9 > 500 and len(seen8) == 4 and len(seen9) >= 5


def test_cost_model_average_when_communication_dominates(oracle):
    """Sec. 3.3: with tau below every communication time the mean CD-SGD iteration over a
    period of k is ((k-1)(delta+psi)+phi)/k; CD-SGD always beats the local-update mechanism
    there, and beats BIT-SGD on every compressed iteration."""
    tau, phi, psi, delta = 1.0, 16.0, 2.0, 0.5
    for k in (1, 2, 5, 20):
        ts = [oracle.cost_model(tau, phi, psi, delta, k, i) for i in range(k)]
        mean_cd = sum(t["t_cd"] for t in ts) / k
        assert mean_cd == ((k - 1) * (delta + psi) + phi) / k
        assert all(t["save_vs_loc"] >= 0 for t in ts)
        assert all(t["save_vs_bit"] > 0 for i, t in enumerate(ts) if i % k != 0)
