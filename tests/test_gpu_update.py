"""Parity of sr_update_bf16 (Eq. 10 on the bfloat16 grid) with the oracle, through the C ABI:
bit patterns must be equal."""
import numpy as np
import pytest
import torch

import oracle
from gpu_util import DEV, say
from paper_2511_00874_amd import lib as L

pytestmark = pytest.mark.gpu


def bits_of(t):
    return t.cpu().view(torch.int16).numpy().view(np.uint16)


def run_both(w_bits, g, eta, seed, off, mode):
    w = torch.from_numpy(w_bits.view(np.int16).copy()).to(DEV).view(torch.bfloat16)
    gd = torch.from_numpy(g).to(DEV)
    L.sr_update_bf16(w, gd, eta, seed=seed, counter_offset=off, round_mode=mode)
    torch.cuda.synchronize()
    return bits_of(w), oracle.update_bf16(w_bits, g, eta, seed, off, mode)


@pytest.mark.parametrize("mode", [L.SR, L.RTN])
@pytest.mark.parametrize("n", [1, 5, 8, 511, 512, 513, 4099, (1 << 20) + 3])
def test_update_matches_oracle(n, mode):
    say("update", n, mode)
    rng = np.random.default_rng(n)
    w = torch.from_numpy(rng.normal(0, 0.02, n).astype(np.float32)).to(torch.bfloat16)
    wb = w.view(torch.int16).numpy().view(np.uint16).copy()
    g = rng.normal(0, 1e-2, n).astype(np.float32)
    got, ref = run_both(wb, g, 0.05, seed=0xABCDEF0123, off=(1 << 33) + 7, mode=mode)
    assert np.array_equal(got, ref)
    if mode == L.SR and n > 4000:
        assert np.any(got != wb)  # the step is far below a bfloat16 spacing for most: some move, most stay


@pytest.mark.parametrize("mode", [L.SR, L.RTN])
def test_every_bfloat16_pattern_with_zero_gradient(mode):
    # pass-through of the whole grid, NaN patterns to 0x7FC0, infinities to the largest finite, -0 to +0
    wb = np.arange(65536, dtype=np.uint16)
    got, ref = run_both(wb, np.zeros(65536, np.float32), 0.1, 3, 0, mode)
    assert np.array_equal(got, ref)
    finite = (wb & 0x7FFF) < 0x7F80
    assert np.array_equal(got[finite & (wb != 0x8000)], wb[finite & (wb != 0x8000)])


@pytest.mark.parametrize("mode", [L.SR, L.RTN])
def test_specials_subnormals_and_saturation(mode):
    say("update specials", mode)
    rng = np.random.default_rng(5)
    n = 8192
    # bfloat16 subnormals and tiny normals with gradients that keep u subnormal in binary32
    w_small = rng.integers(0, 0x0100, n // 4).astype(np.uint16) | (rng.integers(0, 2, n // 4).astype(np.uint16) << 15)
    g_small = (rng.normal(0, 1, n // 4) * 2.0 ** -130).astype(np.float32)
    # near the largest finite value, pushed outwards: must saturate, never reach infinity
    w_big = np.full(n // 4, 0x7F7F, np.uint16) ^ (rng.integers(0, 2, n // 4).astype(np.uint16) << 15)
    g_big = (-np.sign(np.where(w_big & 0x8000, -1.0, 1.0)) * rng.uniform(0, 1, n // 4) * 1e37).astype(np.float32)
    # binade crossings: just below a power of two
    w_edge = np.full(n // 4, 0x3FFF, np.uint16)
    g_edge = (-rng.uniform(0, 1, n // 4) * 2.0 ** -7).astype(np.float32)
    # non-finite gradients
    w_nf = rng.integers(0x3000, 0x4000, n // 4).astype(np.uint16)
    g_nf = rng.choice(np.array([np.nan, np.inf, -np.inf, 0.0, 1.0], np.float32), n // 4)
    wb = np.concatenate([w_small, w_big, w_edge, w_nf])
    g = np.concatenate([g_small, g_big, g_edge, g_nf])
    got, ref = run_both(wb, g, 1.0, seed=9, off=0, mode=mode)
    assert np.array_equal(got, ref)
    assert not np.any((got & 0x7FFF) == 0x7F80)


def test_update_at_the_size_of_a_large_weight_matrix():
    # 32000 x 768 (the largest matrix of the small decoder configuration)
    n = 32000 * 768
    say("update full", n)
    g = torch.Generator(device=DEV).manual_seed(1)
    w = (torch.randn(n, device=DEV, generator=g) * 0.02).to(torch.bfloat16)
    grad = torch.randn(n, device=DEV, generator=g) * 1e-3
    wb = bits_of(w).copy()
    L.sr_update_bf16(w, grad, 0.1, seed=77, counter_offset=123456789)
    torch.cuda.synchronize()
    ref = oracle.update_bf16(wb, grad.cpu().numpy(), 0.1, 77, 123456789)
    assert np.array_equal(bits_of(w), ref)


def test_update_past_2_to_32_elements():
    # element indices past 32 bits, with a ragged tail: slices around index 2^32 and at the end
    n = (1 << 32) + (1 << 16) + 3
    say("update", n)
    g = torch.Generator(device=DEV).manual_seed(5)
    w = torch.empty(n, dtype=torch.bfloat16, device=DEV)
    grad = torch.empty(n, dtype=torch.float32, device=DEV)
    for i in range(0, n, 1 << 30):
        w[i:i + (1 << 30)].normal_(std=0.02, generator=g)
        grad[i:i + (1 << 30)].normal_(std=1e-3, generator=g)
    slices = (((1 << 32) - (1 << 16), (1 << 32) + (1 << 16)), (n - 4099, n), (0, 1 << 12))
    before = [bits_of(w[lo:hi]).copy() for lo, hi in slices]
    seed, off = 3, (1 << 64) - 17  # the block counter wraps at 2^64 inside the tensor
    L.sr_update_bf16(w, grad, 0.25, seed=seed, counter_offset=off)
    torch.cuda.synchronize()
    for (lo, hi), wb in zip(slices, before):
        # a slice that starts at a multiple of 8 continues the stream at its own block
        lo8 = lo - lo % 8
        pad = lo - lo8
        wb8 = bits_of(w[lo8:lo]).copy() if pad else np.empty(0, dtype=np.uint16)  # (already updated: not compared)
        ref = oracle.update_bf16(np.concatenate([wb8, wb]), grad[lo8:hi].cpu().numpy(), 0.25, seed, (off + lo8 // 8) & (2**64 - 1))
        assert np.array_equal(bits_of(w[lo:hi]), ref[pad:]), lo
