"""Pins for the oracle's quantizer against what the paper and arithmetic fix (CPU only).

Each test is chosen so that one plausible mistake in the oracle (wrong side of
the comparison, sign-magnitude instead of signed floor, a wrong binade spacing,
an encode slip, a biased threshold) fails it.
"""
import math
import os
from fractions import Fraction

import numpy as np
import pytest
import torch

import oracle
from oracle import E4M0, E4M1, E4M2, E4M3, E5M2, INT4, INT8, RTN, SR

KINDS = [INT8, INT4, E4M3, E5M2, E4M2, E4M1, E4M0]
# fraction bits, smallest normal exponent, torch dtype whose byte encoding the codes use
FKINDS = {E4M3: (3, -6, torch.float8_e4m3fn), E5M2: (2, -14, torch.float8_e5m2),
          E4M2: (2, -6, torch.float8_e4m3fn), E4M1: (1, -6, torch.float8_e4m3fn), E4M0: (0, -6, torch.float8_e4m3fn)}
SUBGRID_ZERO_BITS = {E4M2: 1, E4M1: 2, E4M0: 3}  # stored as E4M3 codes with these low fraction bits zero
ALL_R16 = np.arange(65536)
EPS = np.array([oracle.eps_from_r16(int(r)) for r in ALL_R16], dtype=np.float32)


def _golden(golden_dir):
    kv = {}
    with open(os.path.join(golden_dir, "worked_example_sec_2_2_1.txt")) as f:
        for line in f:
            if line.startswith("#") or not line.strip():
                continue
            k, v = line.split()
            kv[k] = float(v)
    return kv


# ---- Eq. 1 itself -----------------------------------------------------------------

def test_eq1_rtn_ties_toward_plus_infinity():
    # Def. 2: eps = 1/2, ties go up
    assert oracle.Q(0.5, 1.0, 0.5) == 1.0
    assert oracle.Q(-0.5, 1.0, 0.5) == 0.0
    assert oracle.Q(-1.5, 1.0, 0.5) == -1.0
    assert oracle.Q(2.49, 1.0, 0.5) == 2.0
    assert oracle.Q(0.3, 0.25, 0.5) == 0.25


def test_eq1_delta_zero_is_identity():
    for x in (0.0, -3.25, 1e-30, 7.7):
        assert oracle.Q(x, 0.0, 0.123) == x


def test_eq1_threshold_decides_direction():
    # frac(0.7) = 0.7: down iff 0.7 < eps
    assert oracle.Q(0.7, 1.0, 0.71) == 0.0
    assert oracle.Q(0.7, 1.0, 0.69) == 1.0
    assert oracle.Q(-0.3, 1.0, 0.71) == -1.0  # frac(-0.3) = 0.7 with the signed floor
    assert oracle.Q(-0.3, 1.0, 0.69) == 0.0
    assert oracle.Q(-1e-20, 1.0, 0.999) == 0.0  # never leaves the two neighbours


def test_worked_example_of_the_paper(golden_dir):
    g = _golden(golden_dir)
    x, terms = g["x"], int(g["terms"])
    # RTN: every 0.7 becomes 1
    assert sum(oracle.Q(x, g["delta"], 0.5) for _ in range(terms)) == g["rtn_sum"]
    # SR through the tensor quantizer (scale = Delta = 1): ten-fold sums over many seeds
    xs = np.full(terms, x, dtype=np.float32)
    sums = []
    for seed in range(4000):
        codes = oracle.quantize(xs, INT8, 1.0, seed, 0)
        assert set(np.unique(codes)) <= {0, 1}
        sums.append(int(codes.sum()))
    sums = np.array(sums)
    # expectation 7, binomial(10, 0.7) spread: s.e. of the mean = sqrt(2.1/4000) = 0.023
    assert abs(sums.mean() - g["sr_expected_sum"]) < 5 * math.sqrt(2.1 / 4000)
    assert abs(sums.var() - terms * 0.7 * 0.3) < 0.25
    assert {6, 7, 8} <= set(sums.tolist())
    # probability of rounding up over every possible threshold: 0.7 to within 2^-16
    ups = sum(oracle.quantize_one(x, 1.0, INT8, float(e)) for e in EPS)
    assert ups == 45875  # fl32(0.7) * 65536 = 45875.2
    assert abs(ups / 65536 - g["sr_prob_up"]) < 2.0**-16


# ---- exact-arithmetic brute force ---------------------------------------------------

def _exact_quantize(x: Fraction, scale: Fraction, kind: int, eps: Fraction) -> Fraction:
    """Eq. 1 in exact rationals on the format's grid; returns the value in grid units."""
    qmax = Fraction(oracle.qmax(kind))
    t = max(-qmax, min(qmax, x / scale))
    if kind in FKINDS:
        m, emin, _ = FKINDS[kind]
        e = emin
        if t != 0:
            e = 0
            a = abs(t)
            while Fraction(2) ** e > a:
                e -= 1
            while Fraction(2) ** (e + 1) <= a:
                e += 1
            e = max(e, emin)
        delta = Fraction(2) ** (e - m)
    else:
        delta = Fraction(1)
    y = t / delta
    fl = math.floor(y)
    return delta * (fl if y - fl < eps else fl + 1)


@pytest.mark.parametrize("kind", KINDS)
def test_brute_force_against_exact_rationals(kind):
    # inputs and scales for which every binary32 step of the oracle is exact
    rng = np.random.default_rng(kind)
    scale = 0.25
    span = oracle.qmax(kind) * scale * 1.1
    xs = (rng.integers(-2**20, 2**20, size=300) / 2**20 * span).astype(np.float32)
    xs = np.concatenate([xs, np.float32([0.0, scale, -scale, scale / 2, -scale / 2, 1e-3, -1e-3,
                                         2.0**-12, -2.0**-12, span, -span])])
    for x in xs:
        for r in (0, 1, 13107, 32767, 32768, 52428, 65534, 65535):
            eps = Fraction(2 * r + 1, 2**17)
            want = _exact_quantize(Fraction(float(x)), Fraction(scale), kind, eps)
            code = oracle.quantize_one(float(x), 1.0 / scale, kind, oracle.eps_from_r16(r))
            assert Fraction(oracle.decode(kind, code)) == want, (x, r)


@pytest.mark.parametrize("kind", KINDS)
def test_number_of_thresholds_rounding_up_is_closed_form(kind):
    # over all 2^16 thresholds exactly round-half-up(frac * 2^16) round up, so
    # P(up) = frac to within 2^-17: the bias is at most 2^-17 of a step, and centred
    for x in np.float32([0.7, -0.3, 0.1, 5.0 / 3.0, -2.9999, 0.5, 100.37, 2.0**-9 * 0.3,
                         -2.0**-16 * 0.77, 3.3e-6, 1.0, -4.0]):
        xf = Fraction(float(x))
        lo = _exact_quantize(xf, Fraction(1), kind, Fraction(1))   # eps = 1: always down
        hi = _exact_quantize(xf, Fraction(1), kind, Fraction(0))   # eps = 0: always up
        assert hi > lo
        qm = Fraction(oracle.qmax(kind))
        t = max(-qm, min(qm, xf))
        want_ups = math.floor((t - lo) / (hi - lo) * 65536 + Fraction(1, 2))
        vals = [Fraction(oracle.decode(kind, oracle.quantize_one(float(x), 1.0, kind, float(e))))
                for e in EPS]
        assert set(vals) <= {lo, hi}
        assert sum(1 for v in vals if v == hi) == want_ups, (kind, x)


# ---- properties that hold for every input --------------------------------------------

def _spacing(kind, t):
    if kind in FKINDS:
        m, emin, _ = FKINDS[kind]
        a = np.abs(t)
        e = np.floor(np.log2(np.where(a > 0, a, 1.0)))
        e = np.where(a > 0, np.maximum(e, emin), emin)
        return 2.0 ** (e - m)
    return np.ones_like(t)


@pytest.mark.parametrize("kind", KINDS)
@pytest.mark.parametrize("mode", [SR, RTN])
def test_two_neighbours_and_error_bounds(kind, mode):
    # Eq. 1: output is one of the two grid neighbours; proof of Lemma 1: |x - xhat| <= Delta
    # for SR and <= Delta/2 for RTN
    rng = np.random.default_rng(10 * kind + mode)
    x = rng.standard_normal(20000).astype(np.float32) * np.float32(3.0)
    scale = oracle.absmax_scale(x, kind)
    codes = oracle.quantize(x, kind, scale, 5, 0, mode)
    t = (x * np.float32(1.0 / np.float32(scale))).astype(np.float64)
    v = oracle.decode_array(kind, codes)
    d = _spacing(kind, t)
    err = np.abs(v - t)
    bound = d if mode == SR else d / 2
    assert np.all(err <= bound)
    lo = np.floor(t / d) * d
    assert np.all((v == lo) | (v == lo + d))
    if mode == SR:
        assert np.any(v == lo) and np.any(v == lo + d)


@pytest.mark.parametrize("kind", KINDS)
def test_grid_points_pass_through_for_every_threshold(kind):
    codes = [c for c in range(256) if math.isfinite(oracle.decode(kind, c))]
    if kind == INT8:
        codes = [c for c in codes if oracle.decode(kind, c) >= -127]
    if kind == INT4:
        codes = [c for c in codes if abs(oracle.decode(kind, c)) <= 7]
    if kind in SUBGRID_ZERO_BITS:
        low = (1 << SUBGRID_ZERO_BITS[kind]) - 1
        codes = [c for c in codes if (c & low) == 0 and abs(oracle.decode(kind, c)) <= oracle.qmax(kind)]
        assert len(codes) == {E4M2: 128, E4M1: 64, E4M0: 32}[kind]  # every such E4M3 code is finite and in range
    scale = 0.5  # exact arithmetic: value = grid * 0.5
    for c in codes:
        v = oracle.decode(kind, c)
        for r in (0, 1, 32768, 65535):
            got = oracle.quantize_one(v * scale, 1.0 / scale, kind, oracle.eps_from_r16(r))
            assert oracle.decode(kind, got) == v
            if v == 0:
                assert got == 0  # any zero is stored as +0
            else:
                assert got == c


@pytest.mark.parametrize("kind", KINDS)
def test_unbiased_with_bernoulli_variance(kind):
    # E[xhat | x] = x and Var = p (1 - p) Delta^2 (Bernoulli between the two neighbours);
    # Lemma 3 uses the weaker sigma^2 <= Delta^2
    rng = np.random.default_rng(100 + kind)
    n, seeds = 1024, 3000
    x = rng.standard_normal(n).astype(np.float32)
    scale = oracle.absmax_scale(x, kind)
    t = (x * np.float32(1.0 / np.float32(scale))).astype(np.float64)
    d = _spacing(kind, t)
    p = t / d - np.floor(t / d)
    acc = np.zeros(n)
    acc2 = np.zeros(n)
    for s in range(seeds):
        v = oracle.decode_array(kind, oracle.quantize(x, kind, scale, s, 17))
        acc += v
        acc2 += v * v
    mean = acc / seeds
    var = acc2 / seeds - mean**2
    want_var = p * (1 - p) * d * d
    assert np.all(var <= d * d)
    z = (mean - t) / np.sqrt(np.maximum(want_var, 1e-30) / seeds)
    assert np.all(np.abs(z[want_var > 1e-12]) < 5.5)
    assert abs(z[want_var > 1e-12].mean()) < 5 / math.sqrt(n)      # no common bias
    ratio = var.sum() / want_var.sum()
    assert abs(ratio - 1) < 0.02


def test_rtn_is_biased_where_sr_is_not():
    # the paper's motivation: most values within one step of zero
    x = np.full(4096, 0.3, dtype=np.float32)
    rt = oracle.decode_array(INT8, oracle.quantize(x, INT8, 1.0, 0, 0, RTN))
    sr = oracle.decode_array(INT8, oracle.quantize(x, INT8, 1.0, 0, 0, SR))
    assert rt.mean() == 0.0
    assert abs(sr.mean() - 0.3) < 5 * math.sqrt(0.21 / 4096)


# ---- the 8-bit float grids against torch's float8 dtypes -------------------------------

@pytest.mark.parametrize("kind", [E4M3, E5M2])
def test_decode_matches_torch_float8(kind):
    tdt = FKINDS[kind][2]
    ref = torch.arange(256, dtype=torch.int32).to(torch.uint8).view(tdt).to(torch.float64).numpy()
    got = np.array([oracle.decode(kind, c) for c in range(256)])
    assert np.array_equal(np.isnan(ref), np.isnan(got))
    ok = ~np.isnan(ref)
    assert np.array_equal(ref[ok], got[ok])


@pytest.mark.parametrize("kind", [E4M3, E5M2])
def test_rtn_matches_torch_float8_cast_away_from_ties(kind):
    # round-to-nearest differs from IEEE only at exact ties (up versus even)
    m, emin, tdt = FKINDS[kind]
    rng = np.random.default_rng(kind)
    qm = oracle.qmax(kind)
    mag = np.exp2(rng.uniform(emin - m - 3, math.log2(qm), size=40000))
    x = (mag * rng.choice([-1.0, 1.0], size=mag.size)).astype(np.float32)
    x = x[np.abs(x) <= qm * (1 - 2.0**-(m + 2))]       # stay below the saturating half-step
    d = _spacing(kind, x.astype(np.float64))
    frac = x / d - np.floor(x / d)
    x = x[frac != 0.5]
    ref = torch.from_numpy(x).to(tdt)
    codes = oracle.quantize(x, kind, 1.0, 0, 0, RTN)
    ref_vals = ref.to(torch.float64).numpy()
    got_vals = oracle.decode_array(kind, codes)
    assert np.array_equal(ref_vals, got_vals)
    nz = got_vals != 0
    assert np.array_equal(ref.view(torch.uint8).numpy()[nz], codes[nz])


@pytest.mark.parametrize("kind", [INT8, INT4])
def test_int_rtn_matches_numpy_rint_away_from_ties(kind):
    rng = np.random.default_rng(kind)
    qm = oracle.qmax(kind)
    t = rng.uniform(-qm, qm, size=20000).astype(np.float32)
    t = t[(t - np.floor(t)) != 0.5]
    codes = oracle.quantize(t, kind, 1.0, 0, 0, RTN)
    assert np.array_equal(codes.view(np.int8).astype(np.float64), np.rint(t.astype(np.float64)))


# ---- saturation, special values (rules of this build, not of the paper) ----------------

@pytest.mark.parametrize("kind", KINDS)
def test_saturation_and_specials(kind):
    qm = oracle.qmax(kind)
    for r in (0, 65535):
        e = oracle.eps_from_r16(r)
        assert oracle.decode(kind, oracle.quantize_one(1e30, 1.0, kind, e)) == qm
        assert oracle.decode(kind, oracle.quantize_one(-1e30, 1.0, kind, e)) == -qm
        assert oracle.decode(kind, oracle.quantize_one(math.inf, 1.0, kind, e)) == qm
        assert oracle.decode(kind, oracle.quantize_one(-math.inf, 1.0, kind, e)) == -qm
        assert oracle.quantize_one(-0.0, 1.0, kind, e) == 0
        nan_code = oracle.quantize_one(math.nan, 1.0, kind, e)
        assert nan_code == (0x7F if kind in FKINDS else 0)
    # a small negative that rounds up lands on +0
    assert oracle.quantize_one(-(2.0**-20), 1.0, kind, oracle.eps_from_r16(0)) == 0
    # int8 never emits -128, int4 never -8
    if kind in (INT8, INT4):
        x = np.float32([-1e9, -qm - 0.9, -qm - 0.01])
        codes = oracle.quantize(x, kind, 1.0, 3, 0).view(np.int8)
        assert np.all(codes == -int(qm))


def test_max_codes_are_the_published_ones():
    assert oracle.quantize_one(448.0, 1.0, E4M3, 0.5) == 0x7E
    assert oracle.quantize_one(57344.0, 1.0, E5M2, 0.5) == 0x7B
    assert oracle.quantize_one(2.0**-9, 1.0, E4M3, 0.5) == 0x01    # smallest subnormal
    assert oracle.quantize_one(2.0**-16, 1.0, E5M2, 0.5) == 0x01
    assert oracle.quantize_one(2.0**-6, 1.0, E4M3, 0.5) == 0x08    # smallest normal
    assert oracle.quantize_one(-1.0, 1.0, E4M3, 0.5) == 0xB8
    assert oracle.quantize_one(-1.0, 1.0, E5M2, 0.5) == 0xBC
    assert oracle.quantize_one(-127.0, 1.0, INT8, 0.5) == 0x81


def test_sub_grids_of_e4m3():
    # E4M2 / E4M1 / E4M0: same exponent range as E4M3, fewer fraction bits, stored as E4M3 codes
    assert oracle.quantize_one(448.0, 1.0, E4M2, 0.5) == 0x7E and oracle.qmax(E4M2) == 448.0
    assert oracle.quantize_one(1e9, 1.0, E4M1, 0.5) == 0x7C and oracle.qmax(E4M1) == 384.0
    assert oracle.quantize_one(1e9, 1.0, E4M0, 0.5) == 0x78 and oracle.qmax(E4M0) == 256.0
    assert oracle.quantize_one(2.0**-8, 1.0, E4M2, 0.5) == 0x02   # smallest subnormal: half the E4M3 resolution
    assert oracle.quantize_one(2.0**-7, 1.0, E4M1, 0.5) == 0x04
    assert oracle.quantize_one(2.0**-6, 1.0, E4M0, 0.5) == 0x08   # no subnormals but zero
    assert oracle.quantize_one(2.0**-7 * 0.99, 1.0, E4M0, 0.5) == 0x00 and oracle.quantize_one(2.0**-7, 1.0, E4M0, 0.5) == 0x08
    # 1.3 lies between 1.25 and 1.5 (E4M2), 1.0 and 1.5 (E4M1), 1.0 and 2.0 (E4M0)
    for kind, lo, hi in ((E4M2, 1.25, 1.5), (E4M1, 1.0, 1.5), (E4M0, 1.0, 2.0)):
        assert oracle.decode(kind, oracle.quantize_one(1.3, 1.0, kind, oracle.eps_from_r16(65535))) == lo
        assert oracle.decode(kind, oracle.quantize_one(1.3, 1.0, kind, oracle.eps_from_r16(0))) == hi
    rng = np.random.default_rng(0)
    x = (rng.standard_normal(50000) * 40).astype(np.float32)
    e4m3_values = torch.arange(256, dtype=torch.uint8).view(torch.float8_e4m3fn).float().numpy()
    for kind, zero_bits in SUBGRID_ZERO_BITS.items():
        codes = oracle.quantize(x, kind, 1.0, 3, 0)
        assert np.all(codes & ((1 << zero_bits) - 1) == 0)
        assert np.all(np.abs(e4m3_values[codes]) <= oracle.qmax(kind))
        assert np.array_equal(e4m3_values[codes].astype(np.float64), oracle.decode_array(kind, codes))


# ---- int4 storage ------------------------------------------------------------------------

def test_int4_packing_brute_force():
    assert list(oracle.pack_int4(np.array([1, -2], dtype=np.int8).view(np.uint8))) == [0xE1]
    assert list(oracle.pack_int4(np.array([-7, 7], dtype=np.int8).view(np.uint8))) == [0x79]
    pairs = np.array([(a, b) for a in range(-7, 8) for b in range(-7, 8)], dtype=np.int8)
    packed = oracle.pack_int4(pairs.reshape(-1).view(np.uint8))
    assert packed.size == 225
    for (a, b), byte in zip(pairs, packed):
        assert byte & 0xF == int(a) & 0xF and byte >> 4 == int(b) & 0xF
    assert np.array_equal(oracle.unpack_int4(packed).view(np.int8), pairs.reshape(-1))


# ---- scale, sources, stream positions ------------------------------------------------------

@pytest.mark.parametrize("kind", KINDS)
def test_absmax_scale(kind):
    rng = np.random.default_rng(0)
    x = rng.standard_normal(5000).astype(np.float32)
    want = np.float32(np.abs(x).max()) / np.float32(oracle.qmax(kind))
    assert oracle.absmax_scale(x, kind) == float(want)
    assert oracle.absmax_scale(np.zeros(16, dtype=np.float32), kind) == 1.0
    y = x.copy()
    y[3], y[4], y[5] = np.nan, np.inf, -np.inf
    y[6] = x[6]
    assert oracle.absmax_scale(y, kind) == float(np.float32(np.abs(np.delete(x, [3, 4, 5])).max())
                                                 / np.float32(oracle.qmax(kind)))
    # with this scale the largest element sits on +-Qmax (up to the rounding of x * 1/scale)
    codes = oracle.quantize(x, kind, float(want), 1, 0)
    assert abs(oracle.decode(kind, int(codes[np.argmax(np.abs(x))]))) >= oracle.qmax(kind) * 0.87


@pytest.mark.parametrize("kind", KINDS)
def test_absmax_scale_has_a_floor(kind):
    # max|x| / Qmax below 2^-100 would make 2^16 / scale overflow binary32: the step is floored
    # there, and Eq. 1 on that grid sends 2^-120 (2^-20 of a step; for the float grids 2^-11 of the
    # subnormal spacing at most) to zero for every one of the 65536 thresholds but never to Qmax
    x = np.full(64, 2.0 ** -120, dtype=np.float32)
    x[1::2] *= -1
    assert oracle.absmax_scale(x, kind) == 2.0 ** -100
    # just above the floor nothing changes
    y = np.full(8, 2.0 ** -80, dtype=np.float32)
    assert oracle.absmax_scale(y, kind) == float(np.float32(2.0 ** -80) / np.float32(oracle.qmax(kind)))
    for r16 in (0, 1, 65535):
        for v in (x[0], x[1]):
            code = oracle.quantize_one(float(v), 1.0 / 2.0 ** -100, kind, (r16 + 0.5) / 65536)
            got = oracle.decode(kind, code)
            # the two grid neighbours of 2^-20 of a step: zero and one spacing (the smallest
            # subnormal for the float grids), never anything near Qmax
            spacing = {INT8: 1.0, INT4: 1.0, oracle.E4M3: 2.0 ** -9, oracle.E5M2: 2.0 ** -16, oracle.E4M2: 2.0 ** -8,
                       oracle.E4M1: 2.0 ** -7, oracle.E4M0: 2.0 ** -6}[kind]
            assert got in (0.0, np.sign(v) * spacing), (kind, r16, v, got)
            if kind in (INT8, INT4):
                assert got == 0.0  # frac = 2^-20 (or 1 - 2^-20): below (above) every threshold


def test_bf16_source_is_widened_exactly():
    from paper_2511_00874_amd import synth
    x = synth.gaussian((257,), 0.02, 3)
    bits = synth.to_bf16_bits(x)
    wide = torch.from_numpy(bits.view(np.int16)).view(torch.bfloat16).to(torch.float32).numpy()
    s = oracle.absmax_scale(wide, INT8)
    assert oracle.absmax_scale(bits, INT8) == s
    assert np.array_equal(oracle.quantize(bits, INT8, s, 9, 4), oracle.quantize(wide, INT8, s, 9, 4))


def test_codes_depend_only_on_index_seed_and_offset():
    # fixed thresholds => fixed result (note under Alg. 1), whatever the order of evaluation
    x = np.random.default_rng(1).standard_normal(64 * 24).astype(np.float32)
    s = oracle.absmax_scale(x, INT8)
    whole = oracle.quantize(x, INT8, s, 77, 1000)
    for start in (0, 8, 512, 1016):
        part = oracle.quantize(x[start:start + 200], INT8, s, 77, 1000 + start // 8)
        assert np.array_equal(part, whole[start:start + 200])
    oracle.set_threads(1)
    one = oracle.quantize(x, INT8, s, 77, 1000)
    oracle.set_threads(os.cpu_count() or 1)
    assert np.array_equal(one, whole)
    assert not np.array_equal(whole, oracle.quantize(x, INT8, s, 78, 1000))
