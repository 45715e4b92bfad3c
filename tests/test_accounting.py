"""The bit accounting against the factors the paper states, on masks made by the oracle."""
import numpy as np

from oracle import sbc_oracle as o
from paper_1805_08768_amd import accounting, synth


def test_factors_on_an_oracle_mask_at_p_001():
    n, p = 1 << 18, 0.01
    res = o.compress_model([synth.gaussian_update(n)], [np.zeros(n, np.float32)], p)
    acc = accounting.message_bits([n], [r.k for r in res], [r.bit_len for r in res])
    # binarization: 48 bits per kept entry become 16 (plus one mean per tensor): "approximately x3"
    assert abs(acc["gain_binarization"] - 3.0) < 0.01
    # Golomb positions: the b-bar_pos equation gives 8.108 bits at b* = 6 (16 / 8.108 = x1.97; the
    # paper prints 8.38 and x1.9, which is the same equation at b = 7)
    assert abs(acc["position_bits_per_kept_entry"] - o.mean_position_bits(p, o.golomb_bstar(p))) < 0.05
    assert 1.9 < acc["gain_golomb"] < 2.0
    # everything together: 32 n / (k * b-bar_pos + 32)
    want = 32.0 * n / (res[0].bit_len + 32.0)
    assert abs(acc["gain_total"] - want) < 1e-9 * want
    assert abs(acc["gain_sparsification"] - 32.0 / (p * 48.0)) < 0.05 * 32.0 / (p * 48.0)


def test_sizes_add_up():
    acc = accounting.message_bits([1000, 50], [10, 1], [90, 12])
    assert acc["dense_bits"] == 32 * 1050
    assert acc["sparse_fp32_values_bits"] == 11 * 48
    assert acc["sparse_binary_naive_positions_bits"] == 11 * 16 + 64
    assert acc["sparse_binary_golomb_bits"] == 102 + 64
