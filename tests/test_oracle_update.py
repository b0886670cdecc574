"""Pins for the oracle's weight update of Eq. 10 (stochastic rounding onto the bfloat16 grid).
None of these call the GPU library."""
import numpy as np
import pytest
import torch

import oracle


def f32(bits):
    return np.array([bits], dtype=np.uint32).view(np.float32)[0]


def bf16_value(bits):
    return np.array([int(bits) << 16], dtype=np.uint32).view(np.float32)[0]


def test_bfloat16_values_pass_through_for_every_threshold():
    # frac = 0: Eq. 1 never moves a value already on the grid
    rng = np.random.default_rng(1)
    pats = np.concatenate([rng.integers(0, 0x7F80, 200), rng.integers(0x8001, 0xFF80, 200), [0x0001, 0x007F, 0x0080, 0x7F7F, 0xFF7F]])
    for p in pats:
        u = bf16_value(p)
        for r in (0, 1, 32767, 65535):
            assert oracle.sr_bf16_one(float(u), oracle.eps_from_r16(r)) == int(p)


@pytest.mark.parametrize("bits", [0x3F801234, 0x3F80FFFF, 0x3F800001, 0xBF801234, 0xC2FEDCBA, 0x00012345, 0x80700001,
                                  0x3FFFFFFF, 0x7F7F0001])
def test_count_of_thresholds_that_round_away_from_zero_is_the_dropped_bits(bits):
    # P(|result| is the larger neighbour) = low16 / 65536, for either sign; and the mean over all
    # thresholds is u exactly (unbiased)
    u = f32(bits)
    low = bits & 0xFFFF
    trunc = bits >> 16
    results = np.array([oracle.sr_bf16_one(float(u), oracle.eps_from_r16(r)) for r in range(65536)])
    if (bits & 0x7FFFFFFF) > 0x7F7F0000:  # beyond the largest finite bfloat16: saturates
        assert np.all(results == (0x7F7F | (trunc & 0x8000)))
        return
    away = int(np.sum(results == trunc + 1))
    assert away == low and int(np.sum(results == trunc)) == 65536 - low
    mean = (float(bf16_value(trunc)) * (65536 - low) + float(bf16_value(trunc + 1)) * low) / 65536.0
    assert mean == float(u)


def test_direction_follows_eq1_not_sign_magnitude():
    # Eq. 1 rounds down (toward -inf) iff frac < eps.  For u = -(1 + 2^-8) the floor is the
    # value further from zero, frac = 1/2: a small eps rounds up (toward zero), a large one down.
    u = -(1.0 + 2.0 ** -8)
    assert bf16_value(oracle.sr_bf16_one(u, 0.25)) == -1.0
    assert bf16_value(oracle.sr_bf16_one(u, 0.75)) == -(1.0 + 2.0 ** -7)
    assert bf16_value(oracle.sr_bf16_one(-u, 0.25)) == 1.0 + 2.0 ** -7
    assert bf16_value(oracle.sr_bf16_one(-u, 0.75)) == 1.0


def test_round_up_across_a_binade_and_specials():
    just_below_two = f32(0x3FFFFFFF)
    assert oracle.sr_bf16_one(float(just_below_two), oracle.eps_from_r16(0)) == 0x4000  # 2.0
    assert oracle.sr_bf16_one(float("nan"), 0.5) == 0x7FC0
    assert oracle.sr_bf16_one(float("inf"), 0.5) == 0x7F7F
    assert oracle.sr_bf16_one(float("-inf"), 0.5) == 0xFF7F
    assert oracle.sr_bf16_one(-0.0, 0.5) == 0
    assert oracle.sr_bf16_one(-1e-45, oracle.eps_from_r16(0)) == 0  # rounds up to zero: +0


def test_half_threshold_matches_torch_bfloat16_conversion_away_from_ties():
    # eps = 1/2 is round-to-nearest (ties toward +inf); torch converts with ties-to-even, so the
    # two agree wherever the dropped bits are not exactly half
    rng = np.random.default_rng(7)
    bits = rng.integers(0, 2 ** 32, 20000, dtype=np.uint64).astype(np.uint32)
    bits = bits[((bits >> 23) & 0xFF) != 0xFF]
    bits = bits[(bits & 0xFFFF) != 0x8000]
    bits = bits[(bits & 0x7FFFFFFF) < 0x7F7F8000]  # torch would round these to inf; the update saturates
    x = bits.view(np.float32)
    ref = torch.from_numpy(x.copy()).to(torch.bfloat16).view(torch.int16).numpy().view(np.uint16)
    got = np.array([oracle.sr_bf16_one(float(v), 0.5) for v in x], dtype=np.uint16)
    nz = x != 0  # any zero result is +0 here
    assert np.array_equal(got[nz] & 0x7FFF, ref[nz] & 0x7FFF)
    nonzero_result = (got & 0x7FFF) != 0
    assert np.array_equal(got[nz & nonzero_result], ref[nz & nonzero_result])


def test_update_arithmetic_and_stream_positions():
    # u = fl32(w - fl32(eta * g)); element i draws slice i of the stream that starts at
    # counter_offset blocks, like the quantizers
    rng = np.random.default_rng(3)
    n = 4099
    w = torch.from_numpy(rng.normal(0, 0.02, n).astype(np.float32)).to(torch.bfloat16)
    wb = w.view(torch.int16).numpy().view(np.uint16)
    g = rng.normal(0, 1e-2, n).astype(np.float32)
    eta = np.float32(0.37)
    out = oracle.update_bf16(wb, g, float(eta), seed=11, counter_offset=5)
    wf = w.to(torch.float32).numpy()
    u = (wf - (eta * g).astype(np.float32)).astype(np.float32)
    for i in list(range(16)) + [1000, n - 1]:
        eps = oracle.eps_from_r16(oracle.r16(11, 5, i))
        assert out[i] == oracle.sr_bf16_one(float(u[i]), eps)
    # the result is one of the two bfloat16 neighbours of u and unbiased on average
    val = (out.astype(np.uint32) << 16).view(np.float32)
    lo = ((u.view(np.uint32) >> 16) << 16).view(np.float32)
    spacing = np.abs(lo) * 2.0 ** -7 + 1e-45
    assert np.all(np.abs(val - u) <= spacing)
    err = (val.astype(np.float64) - u.astype(np.float64)) / spacing
    assert abs(err.mean()) < 4 * 0.5 / np.sqrt(n)
    # zero gradient: weights unchanged
    assert np.array_equal(oracle.update_bf16(wb, np.zeros(n, np.float32), 0.1, 1, 0), np.where(wb == 0x8000, 0, wb))


def test_mean_over_seeds_follows_the_gradient_where_nearest_rounding_stalls():
    # the situation Eq. 10 is meant for: a step far below half a bfloat16 spacing.  Nearest
    # rounding never moves the weight; stochastic rounding moves it by eta * g on average.
    w = np.full(20000, 0x3F80, dtype=np.uint16)  # 1.0, spacing 2^-7 below... above 1: 2^-7
    g = np.full(20000, 1.0, dtype=np.float32)
    eta = 2.0 ** -12
    rtn = oracle.update_bf16(w, g, eta, 0, 0, oracle.RTN)
    assert np.all(rtn == 0x3F80)
    sr = oracle.update_bf16(w, g, eta, 5, 0)
    val = (sr.astype(np.uint32) << 16).view(np.float32).astype(np.float64)
    moved = np.mean(1.0 - val)
    # below 1.0 the spacing is 2^-8: P(down) = eta / 2^-8 = 1/16
    assert abs(moved - eta) < 4 * np.sqrt((1 / 16) * (15 / 16) / 20000) * 2.0 ** -8
