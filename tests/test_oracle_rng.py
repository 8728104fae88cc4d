"""Pins for the oracle's noise source (CPU only).

What fixes each part:
  * Threefry-2x32-20 block function: bit-for-bit against rocRAND's host-callable engine, an
    independent implementation of the published generator (Salmon et al., SC'11).
  * stream addressing (seed, step, layer, which, member, block): rebuilt from the rocRAND engine.
  * u32 -> normal: invariants of the Box-Muller pair, N(0,1) moments and KS, and for rank 1 the
    product density K_0(|e|)/pi of the paper's mean-field appendix (generalised Gaussian with
    s = sqrt(2), i.e. unit variance).
  * byte -> bounded integer: exhaustive over the 256 bytes.
  * bfloat16 rounding: against torch's conversion.
"""
import numpy as np
import pytest
import scipy.integrate
import scipy.special
import scipy.stats

import oracle


def test_threefry_block_matches_rocrand(rocrand_pin):
    rng = np.random.default_rng(7)
    cases = [((0, 0), (0, 0)), ((0xFFFFFFFF, 0xFFFFFFFF), (0xFFFFFFFF, 0xFFFFFFFF)),
             ((0x80000000, 1), (0, 0x80000000)), ((1, 0), (0, 0)), ((0, 1), (0, 0)),
             ((0, 0), (1, 0)), ((0, 0), (0, 1))]
    for _ in range(3000):
        v = rng.integers(0, 2**32, size=4, dtype=np.uint64)
        cases.append(((int(v[0]), int(v[1])), (int(v[2]), int(v[3]))))
    for ctr, key in cases:
        got = oracle.threefry2x32_20(ctr, key)
        ref = rocrand_pin.block(ctr, key)
        assert (got == ref).all(), (ctr, key, got, ref)


def test_threefry_sequential_words_match_rocrand(rocrand_pin):
    # a long run of consecutive blocks, crossing the 2^32 carry of the first counter word
    key = (0x9E3779B9, 0x7F4A7C15)
    seed = (key[1] << 32) | key[0]
    start_block = 2**32 - 40
    ref = rocrand_pin.words(seed, 5, 2 * start_block, 160)
    got = []
    for b in range(80):
        blk = start_block + b
        c0, c1 = blk & 0xFFFFFFFF, 5 + (blk >> 32)
        got.extend(oracle.threefry2x32_20((c0, c1), key))
    assert (np.array(got, np.uint32) == ref).all()


@pytest.mark.parametrize("seed,step,layer,which,member", [
    (0, 0, 0, 0, 0), (0, 0, 0, 1, 0), (0xDEADBEEFCAFEF00D, 17, 96, 1, 8191),
    (1, 2**32 - 1, 2**31 - 1, 0, 2**32 - 1)])
def test_stream_addressing_rebuilt_from_rocrand(rocrand_pin, seed, step, layer, which, member):
    sk = rocrand_pin.block((step, layer | (which << 31)), (seed & 0xFFFFFFFF, seed >> 32))
    assert (oracle.stream_key(seed, step, layer, which) == sk).all()
    first = 37  # odd start: first word is the second half of a block
    got = oracle.raw_words(seed, step, layer, which, member, first, 64)
    ref = []
    for w in range(first, first + 64):
        ref.append(rocrand_pin.block((w >> 1, member), sk)[w & 1])
    assert (got == np.array(ref, np.uint32)).all()


def test_streams_are_distinct_and_chunking_is_irrelevant():
    base = oracle.raw_words(3, 1, 2, 0, 5, 0, 256)
    for args in [(4, 1, 2, 0, 5), (3, 2, 2, 0, 5), (3, 1, 3, 0, 5), (3, 1, 2, 1, 5), (3, 1, 2, 0, 6)]:
        other = oracle.raw_words(*args, 0, 256)
        assert (other != base).mean() > 0.95
    # random access: any window of the stream equals the same window of a longer read
    assert (oracle.raw_words(3, 1, 2, 0, 5, 100, 50) == base[100:150]).all()


def test_bit_balance_and_avalanche():
    w = oracle.raw_words(0, 0, 0, 0, 0, 0, 1 << 17)
    bits = ((w[:, None] >> np.arange(32, dtype=np.uint32)) & 1).astype(np.float64)
    assert np.abs(bits.mean(axis=0) - 0.5).max() < 0.01
    # neighbouring members / blocks differ in about half of their bits
    a = oracle.raw_words(0, 0, 0, 0, 1, 0, 4096)
    b = oracle.raw_words(0, 0, 0, 0, 2, 0, 4096)
    flips = np.unpackbits((a ^ b).view(np.uint8)).mean()
    assert abs(flips - 0.5) < 0.01
    flips = np.unpackbits((w[:-2] ^ w[2:]).view(np.uint8)).mean()
    assert abs(flips - 0.5) < 0.01


def test_box_muller_pair_invariants():
    n = 4096
    words = oracle.raw_words(11, 3, 5, 1, 77, 0, n).astype(np.float64)
    z = oracle.noise_normal(11, 3, 5, 1, 77, 0, n)
    u1 = (np.floor(words[0::2] / 512.0) + 0.5) / 2.0**23
    u2 = (np.floor(words[1::2] / 512.0) + 0.5) / 2.0**23
    # radius of pair p is fixed by word 2p, angle by word 2p+1 (even value = cosine branch)
    np.testing.assert_allclose(z[0::2] ** 2 + z[1::2] ** 2, -2.0 * np.log(u1), rtol=1e-12)
    ang = np.mod(np.arctan2(z[1::2], z[0::2]), 2 * np.pi)
    np.testing.assert_allclose(ang, 2 * np.pi * u2, atol=1e-9)
    # extreme words: all-ones radius word gives the smallest radius, zero word the largest (finite)
    assert np.isfinite(z).all() and np.abs(z).max() < np.sqrt(-2 * np.log(2.0**-24)) + 1e-12
    # random access agrees with the bulk read, including an odd start
    assert (oracle.noise_normal(11, 3, 5, 1, 77, 33, 10) == z[33:43]).all()


def test_normal_moments_and_ks():
    n = 1 << 21
    z = np.concatenate([oracle.noise_normal(0, 0, 0, w, m, 0, n // 8) for w in (0, 1) for m in range(4)])
    assert abs(z.mean()) < 4.0 / np.sqrt(n)
    assert abs(z.var() - 1.0) < 4.0 * np.sqrt(2.0 / n)
    assert abs(scipy.stats.kurtosis(z, fisher=False) - 3.0) < 4.0 * np.sqrt(24.0 / n)
    assert abs(scipy.stats.skew(z)) < 4.0 * np.sqrt(6.0 / n)
    assert scipy.stats.kstest(z, "norm").pvalue > 1e-3
    # cosine and sine branches separately, and their independence
    assert scipy.stats.kstest(z[0::2], "norm").pvalue > 1e-3
    assert scipy.stats.kstest(z[1::2], "norm").pvalue > 1e-3
    assert abs(np.corrcoef(z[0::2], z[1::2])[0, 1]) < 4.0 / np.sqrt(n / 2)


def test_rank1_entry_follows_bessel_k0_density():
    # Mean-field appendix: for r = 1 with Gaussian factors of unit variance, an entry e = a*b of E
    # has density K_0(|e|)/pi.  CDF by numerical integration; KS test on a_j * b_k samples.
    n = 200000
    a = oracle.noise_normal(5, 0, 0, 0, 0, 0, n)
    b = oracle.noise_normal(5, 0, 0, 1, 0, 0, n)
    e = a * b
    grid = np.concatenate([[0.0], np.geomspace(1e-6, 16.0, 500)])
    cdf_pos = np.zeros_like(grid)
    for g in range(1, grid.size):  # the log singularity at 0 is integrable; quad cell by cell
        cell, _ = scipy.integrate.quad(lambda t: scipy.special.k0(t) / np.pi, grid[g - 1], grid[g])
        cdf_pos[g] = cdf_pos[g - 1] + cell
    assert abs(cdf_pos[-1] - 0.5) < 1e-7

    def cdf(x):
        x = np.asarray(x)
        half = np.interp(np.abs(x), grid, cdf_pos)
        return np.where(x >= 0, 0.5 + half, 0.5 - half)

    assert scipy.stats.kstest(e, cdf).pvalue > 1e-3
    assert abs(e.var() - 1.0) < 0.03  # unit variance of vec(E) entries


@pytest.mark.parametrize("bound", [0, 1, 3, 8, 16, 127])
def test_int_map_exhaustive(bound):
    vals = np.array([oracle.int_from_byte(b, bound) for b in range(256)])
    assert vals.min() == -bound and vals.max() == bound
    assert vals.sum() == 0
    counts = {v: int((vals == v).sum()) for v in range(-bound, bound + 1)}
    for v in range(1, bound + 1):
        assert counts[v] == counts[-v] == 256 // (2 * bound + 1)
    assert counts[0] == 256 - 2 * bound * (256 // (2 * bound + 1))
    # monotone over the bytes that are not folded onto zero
    q = 256 // (2 * bound + 1)
    assert (np.diff(vals[: q * (2 * bound + 1)]) >= 0).all()


def test_int_noise_reads_bytes_little_end_first():
    words = oracle.raw_words(9, 1, 4, 0, 123, 0, 64)
    got = oracle.noise_int(9, 1, 4, 0, 123, 0, 256, 8)
    by = words.view(np.uint8) if np.little_endian else words.byteswap().view(np.uint8)
    ref = np.array([oracle.int_from_byte(int(b), 8) for b in by], np.int8)
    assert (got == ref).all()
    assert (oracle.noise_int(9, 1, 4, 0, 123, 13, 40, 8) == got[13:53]).all()
    assert abs(got.astype(np.float64).mean()) < 1.0


def test_bf16_rounding_matches_torch():
    import torch
    rng = np.random.default_rng(3)
    vals = np.concatenate([rng.standard_normal(20000) * 3, [0.0, -0.0, 1.0, 1.00390625, 1.01171875,
                           1.0 + 2.0**-8, 1.0 + 3 * 2.0**-8, -(1.0 + 2.0**-8), 6e-5, 3.3e38]])
    got = np.array([oracle.round_bf16(v) for v in vals])
    ref = torch.tensor(vals, dtype=torch.float64).to(torch.float32).to(torch.bfloat16).to(torch.float64).numpy()
    assert (got == ref).all()
    from paper_2511_16652_amd import inputs
    assert (inputs.round_to_bf16(vals.astype(np.float32)).astype(np.float64) == ref).all()


def test_noise_matrix_layout_and_rounding():
    d, r = 37, 4
    flat = oracle.noise_normal(2, 1, 3, 0, 9, 0, d * r)
    m32 = oracle.noise_matrix(2, 1, 3, 0, 9, d, r, oracle.NOISE_F32)
    mbf = oracle.noise_matrix(2, 1, 3, 0, 9, d, r, oracle.NOISE_BF16)
    assert (m32 == flat.astype(np.float32).astype(np.float64).reshape(d, r)).all()  # index d*r + l
    from paper_2511_16652_amd import inputs
    assert (mbf == inputs.round_to_bf16(flat.astype(np.float32)).reshape(d, r)).all()
