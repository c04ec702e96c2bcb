"""Pins for oracle/rng.py: published Philox vectors, closed-form sampler
properties, distribution checks of the Gaussian test matrix."""
import os

import numpy as np
from scipy import stats

from oracle import rng


def test_philox_known_answers(golden_dir):
    rows = [l.split() for l in open(os.path.join(golden_dir, "philox4x32_10_kat.txt"))
            if l.strip() and not l.startswith("#")]
    assert len(rows) == 3
    for w in rows:
        v = [int(x, 16) for x in w]
        out = rng.philox4x32_10(v[0:4], v[4:6])
        assert [int(x) for x in out] == v[6:10]


def test_philox_stream_layout():
    # word w of a stream = lane w%4 of block w//4; slices agree with the whole
    a = rng.philox_words(12345678901234567, 2, 0, 64)
    b = rng.philox_words(12345678901234567, 2, 13, 20)
    assert np.array_equal(a[13:33], b)
    blk = rng.philox4x32_10([3, 0, 2, 0], [12345678901234567 & 0xFFFFFFFF, 12345678901234567 >> 32])
    assert np.array_equal(a[12:16], blk)
    # different streams / seeds differ
    assert not np.array_equal(a, rng.philox_words(12345678901234567, 1, 0, 64))
    assert not np.array_equal(a, rng.philox_words(12345678901234568, 2, 0, 64))


def test_philox_bits_uniform():
    w = rng.philox_words(99, 1, 0, 1 << 16)
    bits = ((w[:, None] >> np.arange(32, dtype=np.uint32)) & 1).mean(axis=0)
    assert np.all(np.abs(bits - 0.5) < 0.01)
    # chi-square of the top byte
    cnt = np.bincount(w >> 24, minlength=256)
    chi = ((cnt - 256.0) ** 2 / 256.0).sum()
    assert chi < stats.chi2.ppf(0.9999, 255)


def test_sample_count():
    assert rng.sample_count(256, 8, 8, 0.25) == 64
    assert rng.sample_count(8192, 64, 16, 1 / 16) == 512
    assert rng.sample_count(8192, 64, 16, 0.001) == 80      # never below k+p
    assert rng.sample_count(4096, 64, 16, 1.0) == 4096
    assert rng.sample_count(50, 64, 16, 1.0) == 50           # never above M


def test_sample_rows_closed_form():
    for M, Ms in [(256, 64), (8192, 512), (1000, 77), (97, 97)]:
        idx = rng.sample_rows(5, M, Ms)
        assert idx.shape == (Ms,)
        assert np.all(np.diff(idx) > 0)                      # distinct and ascending
        j = np.arange(Ms)
        assert np.all(idx >= (j * M) // Ms) and np.all(idx < ((j + 1) * M) // Ms)
    assert np.array_equal(rng.sample_rows(5, 97, 97), np.arange(97))   # rho = 1: identity


def test_sample_rows_uniform_within_strata():
    off = np.concatenate([rng.sample_rows(s, 16 * 4096, 4096) % 16 for s in range(8)])
    cnt = np.bincount(off, minlength=16)
    chi = ((cnt - cnt.mean()) ** 2 / cnt.mean()).sum()
    assert chi < stats.chi2.ppf(0.9999, 15)


def test_omega_is_standard_normal():
    om = rng.gaussian_omega(11, 4096, 80)
    assert om.shape == (4096, 80)
    z = om.ravel()
    assert abs(z.mean()) < 5.0 / np.sqrt(z.size)
    assert abs(z.var() - 1.0) < 0.01
    assert abs(stats.kurtosis(z)) < 0.05
    # bf16 rounding moves values by <= 2^-9 relative: KS against N(0,1) still passes
    assert stats.kstest(z, "norm").pvalue > 1e-3
    # columns are independent draws
    cc = np.corrcoef(om.T)
    assert np.abs(cc - np.eye(80)).max() < 0.1


def test_omega_values_are_bf16():
    om = rng.gaussian_omega(3, 64, 16)
    bits = om.astype(np.float32).view(np.uint32)
    assert np.all((bits & 0xFFFF) == 0)


def test_round_to_bf16_ties_even():
    # 1 + 2^-8 is midway between bf16 neighbours 1 and 1+2^-7 -> even (1.0)
    assert rng.round_to_bf16(np.array([1 + 2.0 ** -8]))[0] == 1.0
    assert rng.round_to_bf16(np.array([1 + 3 * 2.0 ** -8]))[0] == 1 + 2.0 ** -6
    x = np.random.default_rng(0).standard_normal(1000)
    import torch
    ref = torch.from_numpy(x).to(torch.bfloat16).double().numpy()
    assert np.array_equal(rng.round_to_bf16(x), ref)


def test_omega_entry_definition():
    # entry e uses words 2e, 2e+1; recompute one entry by hand with Python floats
    import math
    seed, N, r = 21, 8, 4
    om = rng.gaussian_omega(seed, N, r)
    e = 2 * r + 3
    w = rng.philox_words(seed, 2, 2 * e, 2)
    u1 = ((int(w[0]) >> 9) + 0.5) / 2 ** 23
    u2 = (int(w[1]) >> 8) / 2 ** 24
    z = math.sqrt(-2 * math.log(u1)) * math.cos(2 * math.pi * u2)
    assert abs(om[2, 3] - z) <= abs(z) * 2.0 ** -8


def test_sequence_granular_sample_closed_form():
    # whole sequences of `group` consecutive rows: group-aligned runs, distinct, ascending, one sequence per stratum
    # of sequences, the sequence indices being the (already pinned) row sampler's draw over M/group items
    for M, group, k, p, rho in ((4096, 64, 8, 8, 1.0 / 16), (8192, 512, 64, 16, 1.0 / 16), (1024, 16, 64, 16, 0.01),
                                (960, 32, 4, 4, 0.5), (256, 256, 8, 8, 0.1)):
        Ms = rng.sample_count(M, k, p, rho, group)
        G = M // group
        assert Ms % group == 0 and Ms <= M
        Gs = Ms // group
        assert Gs == min(G, max(-(-(k + p) // group), int(np.ceil(rho * G - 1e-12))))
        assert Ms >= min(M, k + p)
        idx = rng.sample_rows(123, M, Ms, group)
        assert idx.shape == (Ms,) and np.all(np.diff(idx) > 0) and idx.min() >= 0 and idx.max() < M
        runs = idx.reshape(Gs, group)
        assert np.all(runs[:, 0] % group == 0) and np.all(np.diff(runs, axis=1) == 1)
        g = runs[:, 0] // group
        j = np.arange(Gs)
        assert np.all(g >= (j * G) // Gs) and np.all(g < ((j + 1) * G) // Gs)
        assert np.array_equal(g, rng.sample_rows(123, G, Gs))
    # group = 1 is the row sampler itself
    assert rng.sample_count(8192, 64, 16, 1.0 / 16, 1) == rng.sample_count(8192, 64, 16, 1.0 / 16)
    assert np.array_equal(rng.sample_rows(9, 8192, 512, 1), rng.sample_rows(9, 8192, 512))
