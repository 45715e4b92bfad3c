"""Pins for the oracle's subsampled variant of Alg. 2 ("Sparse Binarization": threshold from a
random subsample, noisy amount of sparsity).  CPU only."""
import math

import numpy as np
import pytest

from oracle import sbc_oracle as o


# ------------------------------------------------------------ generator ----

def unmix32(x):
    """Inverse of the mixing function, step by step in reverse: a xor-shift by s >= 11 of a
    32-bit word is undone by applying it often enough, an odd multiplier by its inverse mod 2^32."""
    def unshift(v, s):
        out = v
        for _ in range(32 // s + 1):
            out = v ^ (out >> s)
        return out
    x = unshift(x, 16)
    x = (x * pow(0x846CA68B, -1, 1 << 32)) & 0xFFFFFFFF
    x = unshift(x, 15)
    x = (x * pow(0x7FEB352D, -1, 1 << 32)) & 0xFFFFFFFF
    x = unshift(x, 16)
    return x


def test_mix32_is_a_bijection_with_known_structure():
    rng = np.random.default_rng(5)
    for x in [0, 1, 2, 0x80000000, 0xFFFFFFFF] + [int(v) for v in rng.integers(0, 1 << 32, 2000)]:
        y = o.mix32(x)
        assert 0 <= y < (1 << 32)
        assert unmix32(y) == x
    assert o.mix32(0) == 0                       # every step maps zero to zero
    # avalanche: flipping one input bit flips about half of the output bits
    flips = [bin(o.mix32(12345) ^ o.mix32(12345 ^ (1 << b))).count("1") for b in range(32)]
    assert 11 < sum(flips) / 32 < 21


@pytest.mark.parametrize("n", [16385, 20000, 65536, 1000003, 2359296])
def test_sample_positions_structure(n):
    pos = o.sample_positions(n, 3)
    assert pos.shape == (o.SAMPLE_MAX,) and pos.min() >= 0 and pos.max() < n
    assert len(set(pos.tolist())) == o.SAMPLE_MAX                  # no entry twice
    runs = pos.reshape(o.SAMPLE_RUNS, o.SAMPLE_RUN)
    assert np.all(runs[:, 0] % 64 == 0)                            # aligned slots
    assert np.all(np.diff(runs, axis=1) == 1)                      # 64 consecutive entries
    slots = n // 64
    for r in range(o.SAMPLE_RUNS):                                 # one run in each stratum
        s = int(runs[r, 0]) // 64
        assert math.floor(r * slots / 256) <= s < math.floor((r + 1) * slots / 256)
    assert np.array_equal(pos, o.sample_positions(n, 3))           # deterministic
    assert not np.array_equal(pos, o.sample_positions(n, 4)) or n < 16384 + 256 * 64


def test_sample_positions_spread_within_strata():
    # the offsets inside the strata use the whole stratum: over many tensors the mean relative
    # offset is 1/2 and both ends are reached
    n = 64 * 256 * 100
    rel = []
    for t in range(40):
        runs = o.sample_positions(n, t).reshape(256, 64)[:, 0] // 64
        rel.extend(((runs - np.arange(256) * 100) / 100.0).tolist())
    rel = np.asarray(rel)
    assert abs(rel.mean() - 0.495) < 0.01 and rel.min() == 0.0 and rel.max() == 0.99


def test_small_tensor_is_sampled_completely():
    for n in (1, 2, 63, 16384):
        assert np.array_equal(o.sample_positions(n, 7), np.arange(n))


# ------------------------------------------------------------ thresholds ----

def test_thresholds_brute_force():
    rng = np.random.default_rng(11)
    for n, p in ((20000, 0.01), (70001, 0.001), (16385, 0.3)):
        A = rng.standard_normal(n).astype(np.float32)
        pos = o.sample_positions(n, 2)
        r = max(1, int(math.floor(p * len(pos))))
        vals = sorted(float(A[j]) for j in pos)
        t_pos, t_neg = o.sampled_thresholds(A, p, 2)
        assert float(t_pos) == vals[-r] and float(t_neg) == -vals[r - 1]
        # exactly r - 1 sampled values are strictly beyond each threshold (no ties in this data)
        assert sum(v > float(t_pos) for v in vals) == r - 1
        assert sum(-v > float(t_neg) for v in vals) == r - 1


def test_complete_sample_equals_exact_selection_without_ties():
    # up to 16384 entries the sample is the tensor and r = k: with distinct values the variant
    # is Alg. 2 itself
    rng = np.random.default_rng(12)
    for n, p in ((1, 0.5), (2, 0.5), (100, 0.03), (5000, 0.01), (16384, 0.001)):
        A = rng.permutation(np.linspace(-3.0, 4.0, n)).astype(np.float32)
        exact = o.sparse_binary_compress(A, p)
        sampled = o.sparse_binary_compress_sampled(A, p, 0)
        assert exact[0] == sampled[0]
        assert np.array_equal(exact[1], sampled[1]) and np.array_equal(exact[2], sampled[2])
        assert exact[3:7] == sampled[3:7] and np.array_equal(exact[7], sampled[7])


def test_every_entry_beyond_the_threshold_is_kept():
    rng = np.random.default_rng(13)
    n, p = 300000, 0.002
    A = rng.standard_t(4, n).astype(np.float32)
    k, idx_pos, idx_neg, mu_pos, mu_neg, side, mu, kept = o.sparse_binary_compress_sampled(A, p, 5)
    t_pos, t_neg = o.sampled_thresholds(A, p, 5)
    want_pos = [j for j in range(n) if A[j] >= t_pos]
    want_neg = [j for j in range(n) if -A[j] >= t_neg]
    assert len(want_pos) <= o.sampled_cap(n, k) and len(want_neg) <= o.sampled_cap(n, k)
    assert sorted(idx_pos.tolist()) == want_pos and sorted(idx_neg.tolist()) == want_neg
    # each side's mean is over its own count
    assert mu_pos == pytest.approx(sum(float(A[j]) for j in want_pos) / len(want_pos), rel=1e-12)
    assert mu_neg == pytest.approx(sum(-float(A[j]) for j in want_neg) / len(want_neg), rel=1e-12)
    assert side == (1 if mu_pos >= mu_neg else -1)
    assert np.array_equal(kept, np.asarray(want_pos if side > 0 else want_neg))


def test_amount_of_sparsity_is_noisy_but_unbiased():
    # the tail mass beyond the r-th largest of m samples has mean r/(m+1) and relative
    # standard deviation about 1/sqrt(r)
    rng = np.random.default_rng(14)
    n, p = 1 << 20, 0.01
    k = o.num_kept(n, p)
    r = o.num_kept(o.SAMPLE_MAX, p)
    ratios = []
    for t in range(24):
        A = rng.standard_normal(n).astype(np.float32)
        _, idx_pos, idx_neg, *_ = o.sparse_binary_compress_sampled(A, p, t)
        ratios += [len(idx_pos) / k, len(idx_neg) / k]
    ratios = np.asarray(ratios)
    assert abs(ratios.mean() - 1.0) < 3.0 / math.sqrt(r * len(ratios))
    assert 0.4 / math.sqrt(r) < ratios.std() < 1.8 / math.sqrt(r)
    assert len(set(ratios.tolist())) > 40            # the count really varies


def test_cap_keeps_the_most_extreme_lowest_index_first():
    n, p = 1000, 0.01                                 # k = 10, cap = 84
    A = np.zeros(n, dtype=np.float32)
    A[100:300] = 2.0                                  # 200 entries tie at the top
    A[500:520] = -1.0
    A[520] = -3.0
    k, idx_pos, idx_neg, mu_pos, mu_neg, side, mu, kept = o.sparse_binary_compress_sampled(A, p, 0)
    assert k == 10 and o.sampled_cap(n, k) == 84
    assert idx_pos.tolist() == list(range(100, 184))  # ties go to the lowest index
    # negative side: the 10th smallest value is -1, so all 21 entries at or below it are kept
    assert sorted(idx_neg.tolist()) == list(range(500, 521))
    assert mu_pos == 2.0 and mu_neg == pytest.approx(23.0 / 21.0, rel=1e-15)
    assert side == 1 and mu == np.float32(2.0) and kept.tolist() == list(range(100, 184))
    assert o.sampled_cap(50, 30) == 50                # never more than the tensor holds


def test_side_is_decided_by_the_means_not_the_sums():
    n, p = 1000, 0.01                                 # k = 10
    A = np.zeros(n, dtype=np.float32)
    A[0:9] = 1.1
    A[9:39] = 1.0                                     # the 10th largest value has 30 copies: c+ = 39
    A[600:610] = -1.05                                # c- = 10
    k, idx_pos, idx_neg, mu_pos, mu_neg, side, mu, kept = o.sparse_binary_compress_sampled(A, p, 0)
    assert len(idx_pos) == 39 and len(idx_neg) == 10
    assert mu_pos * 39 > mu_neg * 10 and mu_pos < mu_neg
    assert side == -1 and mu == np.float32(-np.float32(mu_neg)) and kept.tolist() == list(range(600, 610))


def test_compress_tensor_sampled_round_trip():
    rng = np.random.default_rng(15)
    sizes = [40000, 300, 20000]
    dW = [rng.standard_normal(n).astype(np.float32) for n in sizes]
    R = [(0.5 * rng.standard_normal(n)).astype(np.float32) for n in sizes]
    p = 0.005
    res = o.compress_model(dW, R, p, sampled=True)
    msg = o.build_message(res)
    outs = [np.zeros(n, dtype=np.float32) for n in sizes]
    o.decode_accumulate(msg, sizes, 1.0, outs)
    for t, (r, out) in enumerate(zip(res, outs)):
        A = (R[t] + dW[t]).astype(np.float32)
        ref = o.sparse_binary_compress_sampled(A, p, t)
        assert np.array_equal(r.kept, ref[7]) and r.mu_signed == ref[6]
        assert np.array_equal(out, r.dense_update())
        assert np.array_equal(r.R_new + out, np.where(out != 0, (A - r.mu_signed).astype(np.float32) + r.mu_signed, A).astype(np.float32))
        assert o.golomb_decode(r.bits, r.bstar) == r.kept.tolist()
    # the tensor index enters the sample: the same data in another place of the list differs
    a = o.sparse_binary_compress_sampled((R[0] + dW[0]).astype(np.float32), p, 0)
    b = o.sparse_binary_compress_sampled((R[0] + dW[0]).astype(np.float32), p, 1)
    assert len(a[1]) != len(b[1]) or len(a[2]) != len(b[2])
