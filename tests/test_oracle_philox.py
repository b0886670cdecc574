"""Pins for the oracle's random-bit source (CPU only)."""
import os

import numpy as np

import oracle


def _kat(golden_dir):
    rows = []
    with open(os.path.join(golden_dir, "philox4x32_10_kat.txt")) as f:
        for line in f:
            if line.startswith("#") or not line.strip():
                continue
            v = [int(t, 16) for t in line.split()]
            rows.append((v[0:4], v[4:6], v[6:10]))
    return rows


def test_philox_known_answers(golden_dir):
    rows = _kat(golden_dir)
    assert len(rows) == 3
    for ctr, key, want in rows:
        assert oracle.philox4x32_10(ctr, key) == want


def test_philox_is_a_bijection_on_small_counter_range():
    # a counter-mode generator maps distinct counters to distinct blocks
    outs = {tuple(oracle.philox4x32_10([c, 0, 0, 0], [7, 9])) for c in range(4096)}
    assert len(outs) == 4096


def test_r16_slices_follow_block_word_half_order():
    seed, off = 0x0123456789ABCDEF, 0xFFFFFFFFFFFFFFFE  # offset wraps mod 2^64 at i = 16
    for i in range(40):
        block = (off + i // 8) % 2**64
        w = oracle.philox4x32_10([block & 0xFFFFFFFF, block >> 32, 0, 0],
                                 [seed & 0xFFFFFFFF, seed >> 32])
        halves = []
        for word in w:
            halves += [word & 0xFFFF, word >> 16]
        assert oracle.r16(seed, off, i) == halves[i % 8]


def test_eps_is_centred_and_strictly_inside_unit_interval():
    assert oracle.eps_from_r16(0) == 2.0**-17
    assert oracle.eps_from_r16(65535) == 1.0 - 2.0**-17
    assert oracle.eps_from_r16(32768) == 0.5 + 2.0**-17
    e = np.array([oracle.eps_from_r16(r) for r in range(0, 65536, 257)])
    assert np.all(np.diff(e) > 0)


def test_r16_uniformity_chi_square():
    n = 1 << 16
    r = np.array([oracle.r16(42, 0, i) for i in range(n)], dtype=np.int64)
    for bits in (r >> 8, r & 0xFF):
        counts = np.bincount(bits, minlength=256)
        chi2 = float(((counts - n / 256) ** 2 / (n / 256)).sum())
        # 255 dof: mean 255, sd 22.6; 6 sd window
        assert 255 - 6 * 22.6 < chi2 < 255 + 6 * 22.6
    # neighbouring elements uncorrelated
    a = r[:-1] - 32767.5
    b = r[1:] - 32767.5
    corr = float((a * b).mean() / (a.std() * b.std()))
    assert abs(corr) < 5 / np.sqrt(n)


def test_streams_of_different_seed_or_offset_differ():
    base = [oracle.r16(1, 0, i) for i in range(256)]
    assert base != [oracle.r16(2, 0, i) for i in range(256)]
    assert base != [oracle.r16(1, 32, i) for i in range(256)]
    # offset is in blocks of 8 elements: shifting by one block shifts the stream by 8
    assert base[8:] == [oracle.r16(1, 1, i) for i in range(248)]
