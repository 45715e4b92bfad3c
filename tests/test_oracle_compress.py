"""Pins for the oracle's Alg. 1 (client and server lines) and Alg. 2.  CPU only."""
from fractions import Fraction

import numpy as np
import pytest
import torch

from oracle import sbc_oracle as o
from paper_1805_08768_amd import synth


def brute_rank_topk(A, k):
    """Independent definition with no sort: rank_j = #{i: A_i > A_j} +
    #{i < j: A_i == A_j}; keep j iff rank_j < k."""
    n = len(A)
    kept = []
    for j in range(n):
        rank = 0
        for i in range(n):
            if A[i] > A[j] or (A[i] == A[j] and i < j):
                rank += 1
        if rank < k:
            kept.append(j)
    return kept


# ------------------------------------------------------------------ k ------

def test_num_kept():
    assert o.num_kept(2 ** 20, 0.01) == 10485
    assert o.num_kept(4194304, 0.001) == 4194
    assert o.num_kept(2359296, 0.001) == 2359
    assert o.num_kept(64, 0.001) == 1          # p*n < 1 still keeps one entry
    assert o.num_kept(15_000_000, 1e-4) == 1500
    assert o.num_kept(3, 0.9) == 2
    assert o.num_kept(1, 0.5) == 1
    with pytest.raises(ValueError):
        o.num_kept(0, 0.1)
    with pytest.raises(ValueError):
        o.num_kept(10, 0.0)


def test_resnet50_total_kept_matches_closed_form():
    ns = synth.numels(synth.resnet50_shapes())
    ks = [o.num_kept(n, 0.001) for n in ns]
    assert sum(ks) == 25595 and sum(1 for n in ns if 0.001 * n < 1) == 84


# -------------------------------------------------------------- top-k ------

def test_topk_brute_force_with_ties():
    rng = np.random.default_rng(1)
    palette = np.array([-1.5, 0.0, 0.25, 2.0], dtype=np.float32)
    for case in range(1500):
        n = int(rng.integers(1, 33))
        if case % 3 == 0:
            A = palette[rng.integers(0, 4, n)]
        elif case % 3 == 1:
            A = rng.standard_normal(n).astype(np.float32)
        else:
            A = np.round(rng.standard_normal(n) * 2).astype(np.float32)  # few distinct values, signed zeros
            A[rng.random(n) < 0.2] = -0.0
        k = int(rng.integers(1, n + 1))
        assert sorted(o.top_fraction(A, k).tolist()) == brute_rank_topk(A, k)
        assert sorted(o.top_fraction(-A, k).tolist()) == brute_rank_topk(-A, k)


def test_topk_rank_order_is_value_desc_index_asc():
    A = np.array([1, 3, 3, 2, 3, 0], dtype=np.float32)
    assert o.top_fraction(A, 4).tolist() == [1, 2, 4, 3]
    assert o.top_fraction(-A, 3).tolist() == [5, 0, 3]


def test_topk_k1_is_argmax_argmin_lowest_index():
    rng = np.random.default_rng(2)
    for _ in range(200):
        n = int(rng.integers(1, 500))
        A = rng.integers(-5, 6, n).astype(np.float32)
        assert o.top_fraction(A, 1)[0] == int(np.argmax(A))   # numpy returns the first maximum
        assert o.top_fraction(-A, 1)[0] == int(np.argmin(A))


def test_topk_value_multiset_matches_library_topk():
    rng = np.random.default_rng(3)
    for _ in range(20):
        n = int(rng.integers(100, 20000))
        k = int(rng.integers(1, n // 2))
        A = rng.standard_t(3, n).astype(np.float32)
        A[rng.integers(0, n, n // 50)] = A[rng.integers(0, n, n // 50)]
        got = np.sort(A[o.top_fraction(A, k)])
        assert np.array_equal(got, np.sort(np.partition(A, n - k)[n - k:]))
        want = torch.topk(torch.from_numpy(A), k).values.numpy()
        assert np.array_equal(got, np.sort(want))
        got_neg = np.sort(A[o.top_fraction(-A, k)])
        assert np.array_equal(got_neg, np.sort(np.partition(A, k - 1)[:k]))


def test_threshold_property():
    """count(A > tau) < k <= count(A >= tau), and kept ties have the lowest indices."""
    A = synth.palette_update(50000)
    k = o.num_kept(len(A), 0.01)
    idx = o.top_fraction(A, k)
    tau = A[idx].min()
    assert (A > tau).sum() < k <= (A >= tau).sum()
    ties_kept = np.sort(idx[A[idx] == tau])
    all_ties = np.flatnonzero(A == tau)
    assert np.array_equal(ties_kept, all_ties[: len(ties_kept)])


# ------------------------------------------------------- means and side ----

def test_means_exact_rational():
    rng = np.random.default_rng(4)
    for _ in range(300):
        n = int(rng.integers(2, 40))
        A = (rng.standard_normal(n) * 10 ** rng.uniform(-6, 3)).astype(np.float32)
        p = float(rng.uniform(0.05, 0.9))
        k, ip, ineg, mu_p, mu_n, side, mu_s, kept = o.sparse_binary_compress(A, p)
        ex_p = sum(Fraction(float(v)) for v in sorted(A, reverse=True)[:k]) / k
        ex_n = sum(Fraction(float(-v)) for v in sorted(A)[:k]) / k
        assert abs(Fraction(mu_p) - ex_p) <= abs(ex_p) * Fraction(1, 2 ** 50)
        assert abs(Fraction(mu_n) - ex_n) <= abs(ex_n) * Fraction(1, 2 ** 50)
        if ex_p != ex_n:
            assert side == (1 if ex_p > ex_n else -1)
        want = np.float32(float(ex_p)) if side == 1 else np.float32(-float(ex_n))
        assert mu_s == want
        assert len(kept) == k and np.all(np.diff(kept) > 0)


def test_special_cases():
    # all equal: mean is that value, mask is the first k indices, positive side on the tie of means
    A = np.full(100, 0.5, dtype=np.float32)
    k, _, _, mu_p, mu_n, side, mu_s, kept = o.sparse_binary_compress(A, 0.1)
    assert (k, side, float(mu_s)) == (10, 1, 0.5) and kept.tolist() == list(range(10))
    # all zero: side +, mu 0, first k
    k, _, _, _, _, side, mu_s, kept = o.sparse_binary_compress(np.zeros(64, np.float32), 0.05)
    assert (k, side, float(mu_s)) == (3, 1, 0.0) and kept.tolist() == [0, 1, 2]
    # signed zeros compare equal
    A = np.array([-0.0, 0.0, -0.0, 0.0], dtype=np.float32)
    assert o.sparse_binary_compress(A, 0.5)[7].tolist() == [0, 1]
    # one-hot
    A = np.zeros(50, np.float32); A[17] = 3.0
    k, _, _, _, _, side, mu_s, kept = o.sparse_binary_compress(A, 0.02)
    assert (k, side, float(mu_s), kept.tolist()) == (1, 1, 3.0, [17])
    # all negative: the negative side wins and the transmitted mean is negative
    A = -np.arange(1, 101, dtype=np.float32)
    k, _, _, mu_p, mu_n, side, mu_s, kept = o.sparse_binary_compress(A, 0.04)
    assert side == -1 and float(mu_s) == -98.5 and kept.tolist() == [96, 97, 98, 99]
    assert mu_p == -2.5  # top_p%(A) ranks by value whatever the sign
    # exactly symmetric: equal means -> positive side (Alg. 2 uses >=)
    A = (np.array([3, -3, 2, -2, 1, -1, 0, 0], dtype=np.float32) * 2.0 ** -10)
    k, _, _, mu_p, mu_n, side, mu_s, kept = o.sparse_binary_compress(A, 0.25)
    assert mu_p == mu_n and side == 1 and kept.tolist() == [0, 2]
    # non-finite input is a precondition violation
    with pytest.raises(ValueError):
        o.sparse_binary_compress(np.array([1.0, np.inf], dtype=np.float32), 0.5)


def test_sides_may_overlap_when_2k_exceeds_n():
    A = np.array([1, 2, 3], dtype=np.float32)
    k, ip, ineg, *_ = o.sparse_binary_compress(A, 0.9)
    assert k == 2 and sorted(ip.tolist()) == [1, 2] and sorted(ineg.tolist()) == [0, 1]


# --------------------------------------------------- residual, Eq. 2 -------

def test_residual_identity_one_round():
    dW = synth.gaussian_update(20000)
    R = synth.gaussian_update(20000, tensor=1)
    res = o.compress_tensor(dW, R, 0.01)
    assert np.array_equal(res.A, R + dW)                      # one fp32 add
    off = np.ones(res.n, bool); off[res.kept] = False
    assert np.array_equal(res.R_new[off], res.A[off])          # untouched off the kept set
    assert len(res.kept) == res.k == 200
    recon = res.dense_update().astype(np.float64) + res.R_new.astype(np.float64)
    ulp = np.spacing(np.abs(res.mu_signed))
    assert np.max(np.abs(recon - res.A)) <= ulp
    assert np.count_nonzero(res.dense_update()) == res.k


def test_residual_telescopes_over_ten_rounds():
    """Eq. 2: R_tau = sum_t (dW_t - dW*_t)."""
    n, p = 30000, 0.01
    R = np.zeros(n, np.float32)
    sum_dW = np.zeros(n, np.float64)
    sum_star = np.zeros(n, np.float64)
    for t in range(10):
        dW = synth.student_t_update(n, round_=t)
        res = o.compress_tensor(dW, R, p)
        sum_dW += dW
        sum_star += res.dense_update()
        R = res.R_new
    err = np.abs(sum_dW - sum_star - R)
    scale = np.maximum(np.abs(sum_dW), np.abs(R)).max()
    assert err.max() <= 10 * 2.0 ** -23 * scale


def test_kept_side_and_threshold_semantics():
    """Kept entries are exactly the k best of the chosen side; every kept value
    is at least as extreme as every dropped one."""
    for seed in range(5):
        dW = synth.small_model_update([5000], round_=seed)[0]
        res = o.compress_tensor(dW, np.zeros_like(dW), 0.01)
        kept_vals = res.A[res.kept] * res.side
        mask = np.zeros(res.n, bool); mask[res.kept] = True
        assert kept_vals.min() >= (res.A[~mask] * res.side).max()
        assert np.isclose(float(res.mu_signed) * res.side, kept_vals.astype(np.float64).mean(), rtol=1e-6)


# ------------------------------------------------- message, server side ----

def test_message_round_trip_and_accounting():
    sizes = [64, 1000, 4096, 33333]
    dWs = synth.small_model_update(sizes)
    Rs = [np.zeros_like(d) for d in dWs]
    results = o.compress_model(dWs, Rs, 0.01)
    msg = o.build_message(results)
    b, entries = o.parse_message(msg)
    assert b == 6 and len(entries) == 4
    total_words = 0
    for res, (mu, nnz, bit_len, words) in zip(results, entries):
        assert mu == res.mu_signed and nnz == res.k and bit_len == res.bit_len
        assert bit_len == int(((res.gaps >> b) + 1 + b).sum())
        assert np.array_equal(words, res.words)
        assert o.golomb_decode(o.unpack_bits(words, bit_len), b) == res.kept.tolist()
        total_words += len(words)
    assert len(msg) == 32 + 24 * 4 + 4 * total_words


def test_decode_accumulate_equals_dense_average():
    sizes = [300, 5000, 12345]
    clients = 4
    outs = [np.zeros(n, np.float32) for n in sizes]
    dense = [np.zeros(n, np.float64) for n in sizes]
    for c in range(clients):
        dWs = synth.small_model_update(sizes, client=c)
        results = o.compress_model(dWs, [np.zeros_like(d) for d in dWs], 0.02)
        o.decode_accumulate(o.build_message(results), sizes, 1.0 / clients, outs)
        for d, res in zip(dense, results):
            d += res.dense_update().astype(np.float64) / clients
    for out, d in zip(outs, dense):
        assert np.allclose(out, d, rtol=1e-6, atol=1e-12)
        assert np.count_nonzero(out) == np.count_nonzero(d)


def test_decode_one_message_scale_one_reproduces_dense_update():
    dW = synth.gaussian_update(10000)
    res = o.compress_tensor(dW, np.zeros_like(dW), 0.01)
    out = [np.zeros(10000, np.float32)]
    o.decode_accumulate(o.build_message([res]), [10000], 1.0, out)
    assert np.array_equal(out[0], res.dense_update())


def test_decode_rejects_corrupt_message():
    dW = synth.gaussian_update(1000)
    res = o.compress_tensor(dW, np.zeros_like(dW), 0.05)
    msg = o.build_message([res])
    with pytest.raises(ValueError):
        o.decode_accumulate(msg, [res.kept[-1]], 1.0, [np.zeros(int(res.kept[-1]), np.float32)])
    with pytest.raises(ValueError):
        o.parse_message(b"XXXX" + msg[4:])
