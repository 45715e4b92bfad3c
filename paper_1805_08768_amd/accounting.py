"""Message-size accounting for one round, from the sizes a compress call reports.

The paper's running example splits the gain of Sparse Binary Compression over a dense fp32
update into three factors (figure "Step-by-step explanation ...", Eq. 1, "Optimal Position
Encoding"): sparsification, binarization (no value bits; about x3 against 32 value bits plus 16
position bits) and Golomb position encoding (x1.9 at p = 0.01 against a naive distance encoding
with 16 fixed bits).  message_bits() evaluates the same breakdown on the masks a call actually
produced: per tensor it needs the number of kept entries and the Golomb stream length in bits.
Pure host arithmetic; nothing here touches the kernels.
"""
from __future__ import annotations

from typing import Dict, Sequence

NAIVE_POSITION_BITS = 16      # fixed-width distance encoding the paper compares against
VALUE_BITS = 32               # fp32 values of a sparse, non-binarized update
MEAN_BITS = 32                # the one fp32 mean per tensor of a sparse binary update


def message_bits(numel: Sequence[int], nnz: Sequence[int], golomb_bits: Sequence[int]) -> Dict[str, float]:
    """Sizes in bits of one round's update under the encodings the paper compares, for the same
    kept positions, and the factors between them."""
    n_total = float(sum(int(n) for n in numel))
    kept = float(sum(int(k) for k in nnz))
    tensors = len(numel)
    dense = VALUE_BITS * n_total
    sparse_values = kept * (VALUE_BITS + NAIVE_POSITION_BITS)            # top-k with fp32 values
    sparse_binary_naive = kept * NAIVE_POSITION_BITS + MEAN_BITS * tensors
    sparse_binary_golomb = float(sum(int(b) for b in golomb_bits)) + MEAN_BITS * tensors
    return {
        "dense_bits": dense,
        "sparse_fp32_values_bits": sparse_values,
        "sparse_binary_naive_positions_bits": sparse_binary_naive,
        "sparse_binary_golomb_bits": sparse_binary_golomb,
        "gain_sparsification": dense / sparse_values if sparse_values else float("inf"),
        "gain_binarization": sparse_values / sparse_binary_naive,
        "gain_golomb": sparse_binary_naive / sparse_binary_golomb,
        "gain_total": dense / sparse_binary_golomb,
        "position_bits_per_kept_entry": (sparse_binary_golomb - MEAN_BITS * tensors) / kept if kept else 0.0,
    }
