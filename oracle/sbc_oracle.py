"""CPU oracle for Sparse Binary Compression (arXiv 1805.08768).

TEST INFRASTRUCTURE ONLY.  This module is the slow, plain definition of what the
client-side SBC step and the server-side decode-and-average compute.  Only the
tests, the smoke check and the benchmark's CPU-baseline leg may import it; the
product path (the HIP library and its Python binding) never does, and this
module imports nothing from the product path.

Every function follows one passage of the paper, with NumPy fp32/fp64
element-wise operations, one library sort, and plain Python loops for
everything that is sequential in the paper (the Golomb coder and decoder work
on a list of single bits through a small bit writer and reader).  Nothing here
is blocked, fused or reordered.

Readings taken where the paper leaves a choice (each is repeated at the place
it is used):

* "fraction p" of a tensor with n entries keeps k = max(1, floor(p*n)) entries
  (fp64 product), never more than n.
* top_p% returns exactly k entries: the first k in (value descending, index
  ascending) order, so equal values are resolved towards the lowest index.
  Alg. 2's literal threshold mask (W >= min(val+)) would keep more than k when
  the k-th value is duplicated; it is not used.
* top_p%(dW) ranks by value whatever the sign (Alg. 2), not "positive entries
  only" as the prose suggests.
* mu+ >= mu- selects the positive side (Alg. 2 uses >=).
* The transmitted mean is one fp32 number per tensor carrying the sign of the
  chosen side.
* Positions are 0-based here; Alg. 3/4 are 1-based with I_0 = 0, so the encoded
  number d-1 is the count of skipped entries before a kept one.
* binary_b*(r) is written most significant bit first; stream bit i lives in
  32-bit word i // 32 at bit 31 - i % 32; padding bits are zero.
* b* = max(0, 1 + floor(log2(log(phi-1)/log(1-p)))).
* The subsampled variant mentioned in "Sparse Binarization" (threshold from a
  random subsample, noisy amount of sparsity) is read as: per tensor, a
  stratified sample of at most 16384 entries of A (256 runs of 64 consecutive
  entries, one run at a hashed place in each of 256 equal strata; the whole
  tensor if it has no more than 16384 entries); a side's threshold is the r-th
  most extreme sampled value, r = max(1, floor(p*m)) for m sampled entries;
  the side keeps every entry at or beyond its threshold, at most
  min(n, 2k + 64) of them (the most extreme ones, ties to the lowest index, if
  more qualify); each side's mean is over its own count.

Pins: every function below is pinned by tests/test_oracle_*.py (closed forms,
brute force on tiny inputs, exact rational arithmetic, invariants, special
cases, the paper's printed mean code length).  No function is "parity
unpinned".
"""
from __future__ import annotations

import math
import struct
from dataclasses import dataclass, field
from typing import List, Sequence

import numpy as np

PHI = (math.sqrt(5.0) + 1.0) / 2.0  # golden ratio, "Optimal Position Encoding"

MSG_MAGIC = 0x31434253  # the bytes 'S','B','C','1' read as a little-endian u32
MSG_VERSION = 1
MSG_HEADER_BYTES = 32
MSG_ENTRY_BYTES = 24


# --------------------------------------------------------------------------
# Scalars derived from the sparsity rate p
# --------------------------------------------------------------------------

def golomb_bstar(p: float) -> int:
    """b* of Alg. 3 (second step) / "Optimal Position Encoding":
    b* = 1 + floor(log2(log(phi - 1) / log(1 - p))), clamped below at 0."""
    if not (0.0 < p < 1.0):
        raise ValueError("p must lie in (0, 1)")
    b = 1 + math.floor(math.log2(math.log(PHI - 1.0) / math.log(1.0 - p)))
    return max(0, int(b))


def mean_position_bits(p: float, b: int) -> float:
    """Mean Golomb code length for geometric gaps, the displayed equation of
    "Optimal Position Encoding": b + 1 / (1 - (1-p)^(2^b))."""
    return b + 1.0 / (1.0 - (1.0 - p) ** (2 ** b))


def num_kept(n: int, p: float) -> int:
    """Entries kept per side of a tensor with n entries ("fraction p", Alg. 2
    first step).  Reading: k = max(1, floor(p*n)) with the product in fp64."""
    if n <= 0:
        raise ValueError("empty tensor")
    if not (0.0 < p < 1.0):
        raise ValueError("p must lie in (0, 1)")
    k = int(math.floor(p * float(n)))
    return max(1, min(n, k))


# --------------------------------------------------------------------------
# Alg. 1 client lines and Alg. 2, one tensor
# --------------------------------------------------------------------------

def accumulate(R: np.ndarray, dW: np.ndarray) -> np.ndarray:
    """Alg. 1, client: dW_i <- R_i + (SGD_n(W_i) - W_i).  One IEEE fp32 add."""
    assert R.dtype == np.float32 and dW.dtype == np.float32 and R.shape == dW.shape
    return (R + dW).astype(np.float32)


def top_fraction(A: np.ndarray, k: int) -> np.ndarray:
    """top_p%(A) of Alg. 2: indices of the k largest entries of the flat tensor
    A, in rank order.  Full sort on (value descending, index ascending)."""
    n = A.shape[0]
    j = np.arange(n, dtype=np.int64)
    # lexsort sorts by the LAST key first: primary -A ascending (= A descending),
    # secondary the index ascending.
    order = np.lexsort((j, -A.astype(np.float64)))
    return order[:k]


def side_mean(values: np.ndarray) -> float:
    """mean(val) of Alg. 2, second step, in fp64 with an exactly rounded sum."""
    return math.fsum(float(v) for v in values) / float(len(values))


@dataclass
class TensorResult:
    """Everything Alg. 1 (client lines), Alg. 2 and Alg. 3 produce for one tensor."""
    n: int
    k: int
    A: np.ndarray              # accumulated update, fp32
    idx_pos: np.ndarray        # top_p%(A), rank order
    idx_neg: np.ndarray        # top_p%(-A), rank order
    mu_pos: float              # fp64
    mu_neg: float              # fp64
    side: int                  # +1 or -1
    mu_signed: np.float32      # +fl32(mu+) or -fl32(mu-)
    kept: np.ndarray           # kept positions, ascending, int64
    R_new: np.ndarray          # residual after the round, fp32
    bstar: int
    gaps: np.ndarray           # d-1 of Alg. 3 for every kept position, int64
    bits: List[int] = field(repr=False, default_factory=list)  # the Golomb bit string
    words: np.ndarray = None   # the bit string packed MSB-first into uint32

    @property
    def bit_len(self) -> int:
        return len(self.bits)

    def dense_update(self) -> np.ndarray:
        """The sparse binary tensor dW* of Alg. 2, materialised."""
        out = np.zeros(self.n, dtype=np.float32)
        out[self.kept] = self.mu_signed
        return out


def sparse_binary_compress(A: np.ndarray, p: float):
    """Alg. 2 on the flat fp32 tensor A.  Returns
    (k, idx_pos, idx_neg, mu_pos, mu_neg, side, mu_signed, kept_ascending)."""
    assert A.dtype == np.float32 and A.ndim == 1
    if not np.all(np.isfinite(A)):
        raise ValueError("non-finite entry")
    k = num_kept(A.shape[0], p)
    idx_pos = top_fraction(A, k)                 # val+ = top_p%(dW)
    idx_neg = top_fraction(-A, k)                # val- = top_p%(-dW)
    mu_pos = side_mean(A[idx_pos])               # mu+ = mean(val+)
    mu_neg = side_mean(-A[idx_neg])              # mu- = mean(val-)
    if mu_pos >= mu_neg:
        side, mu_signed, kept = +1, np.float32(mu_pos), idx_pos
    else:
        side, mu_signed, kept = -1, np.float32(-np.float32(mu_neg)), idx_neg
    return k, idx_pos, idx_neg, mu_pos, mu_neg, side, np.float32(mu_signed), np.sort(kept)


def residual_update(A: np.ndarray, kept: np.ndarray, mu_signed: np.float32) -> np.ndarray:
    """Alg. 1, client: R_i <- dW_i - dW_i*  (Eq. 2), in fp32."""
    R_new = A.copy()
    R_new[kept] = (A[kept] - np.float32(mu_signed)).astype(np.float32)
    return R_new


# --------------------------------------------------------------------------
# Subsampled variant of Alg. 2 ("Sparse Binarization": the threshold comes from a
# random subsample, which makes the amount of sparsity noisy)
# --------------------------------------------------------------------------

SAMPLE_MAX = 16384   # entries sampled per tensor
SAMPLE_RUN = 64      # consecutive entries per run
SAMPLE_RUNS = SAMPLE_MAX // SAMPLE_RUN


def mix32(x: int) -> int:
    """Counter-based generator of the sample: a bijective 32-bit mixing function
    (xor-shift 16, multiply 0x7FEB352D, xor-shift 15, multiply 0x846CA68B,
    xor-shift 16).  Both implementations of the method use this function, so
    the random numbers the method draws are the same on both."""
    x &= 0xFFFFFFFF
    x ^= x >> 16
    x = (x * 0x7FEB352D) & 0xFFFFFFFF
    x ^= x >> 15
    x = (x * 0x846CA68B) & 0xFFFFFFFF
    x ^= x >> 16
    return x


def sample_positions(n: int, tensor_index: int) -> np.ndarray:
    """Positions of the subsample of tensor number tensor_index (its place in the
    model's tensor list) with n entries.  Up to SAMPLE_MAX entries: all of them.
    Otherwise the n // 64 aligned slots of 64 entries are cut into SAMPLE_RUNS
    equal strata (stratum r holds slots floor(r*slots/256) .. floor((r+1)*slots/256)-1)
    and stratum r contributes the slot at offset floor(h * size / 2^32) where
    h = mix32(r * 0x9E3779B9 + tensor_index * 0x85EBCA6B + 1 mod 2^32)."""
    if n <= SAMPLE_MAX:
        return np.arange(n, dtype=np.int64)
    slots = n // SAMPLE_RUN
    pos = []
    for r in range(SAMPLE_RUNS):
        h = mix32((r * 0x9E3779B9 + tensor_index * 0x85EBCA6B + 1) & 0xFFFFFFFF)
        lo = (r * slots) // SAMPLE_RUNS
        hi = ((r + 1) * slots) // SAMPLE_RUNS
        slot = lo + ((h * (hi - lo)) >> 32)
        pos.extend(range(slot * SAMPLE_RUN, (slot + 1) * SAMPLE_RUN))
    return np.asarray(pos, dtype=np.int64)


def sampled_thresholds(A: np.ndarray, p: float, tensor_index: int):
    """(t+, t-): the r-th largest sampled value of A and of -A, r = max(1, floor(p*m))
    for m sampled entries."""
    sample = A[sample_positions(A.shape[0], tensor_index)]
    r = num_kept(sample.shape[0], p)
    ascending = np.sort(sample.astype(np.float64))
    return np.float32(ascending[-r]), np.float32(-ascending[r - 1])


def sampled_cap(n: int, k: int) -> int:
    """Most entries a side may keep in the subsampled variant."""
    return min(n, 2 * k + 64)


def sparse_binary_compress_sampled(A: np.ndarray, p: float, tensor_index: int):
    """Alg. 2 with thresholds from the subsample.  Same return value as
    sparse_binary_compress; idx_pos / idx_neg hold c+ / c- entries in rank order."""
    assert A.dtype == np.float32 and A.ndim == 1
    if not np.all(np.isfinite(A)):
        raise ValueError("non-finite entry")
    n = A.shape[0]
    k = num_kept(n, p)
    cap = sampled_cap(n, k)
    t_pos, t_neg = sampled_thresholds(A, p, tensor_index)
    c_pos = min(cap, int(np.count_nonzero(A >= t_pos)))
    c_neg = min(cap, int(np.count_nonzero(-A >= t_neg)))
    idx_pos = top_fraction(A, c_pos)             # every entry >= t+, or the cap most extreme
    idx_neg = top_fraction(-A, c_neg)
    mu_pos = side_mean(A[idx_pos])
    mu_neg = side_mean(-A[idx_neg])
    if mu_pos >= mu_neg:
        side, mu_signed, kept = +1, np.float32(mu_pos), idx_pos
    else:
        side, mu_signed, kept = -1, np.float32(-np.float32(mu_neg)), idx_neg
    return k, idx_pos, idx_neg, mu_pos, mu_neg, side, np.float32(mu_signed), np.sort(kept)


# --------------------------------------------------------------------------
# Alg. 3 (encode) and Alg. 4 (decode), bit by bit
# --------------------------------------------------------------------------

def golomb_gaps(kept: Sequence[int]) -> np.ndarray:
    """d - 1 of Alg. 3 for each kept position (ascending, 0-based): the number
    of skipped entries since the previous kept one (I_0 = 0 in 1-based terms)."""
    gaps = []
    prev = -1
    for pos in kept:
        pos = int(pos)
        gaps.append(pos - prev - 1)
        prev = pos
    return np.asarray(gaps, dtype=np.int64)


class BitWriter:
    """A growing list of bits with the two shapes a Golomb code word is made of."""

    def __init__(self) -> None:
        self.bits: List[int] = []

    def unary(self, count: int) -> None:
        """`count` ones closed by a zero."""
        self.bits += [1] * count + [0]

    def field(self, value: int, width: int) -> None:
        """`value` as a `width`-bit number, most significant bit first."""
        self.bits += [(value >> (width - 1 - t)) & 1 for t in range(width)]


class BitReader:
    """Reads the same two shapes back from a list of bits whose length is the exact stream length."""

    def __init__(self, bits: Sequence[int]) -> None:
        self.bits = bits
        self.at = 0

    def exhausted(self) -> bool:
        return self.at >= len(self.bits)

    def unary(self) -> int:
        """Number of ones before the next zero; the zero is consumed.  None if the stream ends
        before a zero turns up (only ones were left: no further code word)."""
        run = 0
        while self.at + run < len(self.bits) and self.bits[self.at + run]:
            run += 1
        if self.at + run >= len(self.bits):
            self.at = len(self.bits)
            return None
        self.at += run + 1
        return run

    def field(self, width: int) -> int:
        if self.at + width > len(self.bits):
            raise IndexError("bit stream ends inside a %d-bit field" % width)
        value = 0
        for bit in self.bits[self.at:self.at + width]:
            value = 2 * value + int(bit)
        self.at += width
        return value


def golomb_encode(kept: Sequence[int], b: int) -> List[int]:
    """Alg. 3: every kept position is sent as the number of skipped entries since the previous
    kept one (d - 1), split by 2^b into a quotient in unary and a remainder in b bits."""
    out = BitWriter()
    for skipped in golomb_gaps(kept):
        quotient, remainder = divmod(int(skipped), 1 << b)
        out.unary(quotient)
        out.field(remainder, b)
    return out.bits


def golomb_decode(msg: Sequence[int], b: int) -> List[int]:
    """Alg. 4: code words are read until the stream (whose exact bit length is len(msg)) is used
    up; each gives the distance to the next kept position.  Returns 0-based positions."""
    src = BitReader(msg)
    positions: List[int] = []
    nxt = 0                                   # first position a code word with no skipped entries would name
    while not src.exhausted():
        quotient = src.unary()
        if quotient is None:
            break
        nxt += (quotient << b) + src.field(b)
        positions.append(nxt)
        nxt += 1
    return positions


def pack_bits(bits: Sequence[int]) -> np.ndarray:
    """Bit i of the stream -> word i // 32, bit 31 - i % 32; zero padding."""
    n_words = (len(bits) + 31) // 32
    words = [0] * n_words
    for i, bit in enumerate(bits):
        if bit:
            words[i // 32] |= 1 << (31 - (i % 32))
    return np.asarray(words, dtype=np.uint32)


def unpack_bits(words: np.ndarray, bit_len: int) -> List[int]:
    """Inverse of pack_bits for the first bit_len bits."""
    return [(int(words[i // 32]) >> (31 - (i % 32))) & 1 for i in range(bit_len)]


# --------------------------------------------------------------------------
# One tensor, one round; a model (list of tensors); the message container
# --------------------------------------------------------------------------

def compress_tensor(dW: np.ndarray, R: np.ndarray, p: float, sampled_index: int = None) -> TensorResult:
    """Client lines of Alg. 1 for one tensor: accumulate, Alg. 2, residual
    update, Alg. 3.  With sampled_index (the tensor's place in the model's list)
    the subsampled variant of Alg. 2 is used."""
    dW = np.ascontiguousarray(dW, dtype=np.float32).reshape(-1)
    R = np.ascontiguousarray(R, dtype=np.float32).reshape(-1)
    A = accumulate(R, dW)
    if sampled_index is None:
        k, idx_pos, idx_neg, mu_pos, mu_neg, side, mu_signed, kept = sparse_binary_compress(A, p)
    else:
        k, idx_pos, idx_neg, mu_pos, mu_neg, side, mu_signed, kept = sparse_binary_compress_sampled(A, p, sampled_index)
    R_new = residual_update(A, kept, mu_signed)
    b = golomb_bstar(p)
    bits = golomb_encode(kept, b)
    return TensorResult(
        n=A.shape[0], k=k, A=A, idx_pos=idx_pos, idx_neg=idx_neg, mu_pos=mu_pos,
        mu_neg=mu_neg, side=side, mu_signed=mu_signed, kept=kept.astype(np.int64),
        R_new=R_new, bstar=b, gaps=golomb_gaps(kept), bits=bits, words=pack_bits(bits))


def compress_model(dWs: Sequence[np.ndarray], Rs: Sequence[np.ndarray], p: float, sampled: bool = False) -> List[TensorResult]:
    """Per-tensor SBC over the list of weight tensors of a model (W in script-W)."""
    return [compress_tensor(dW, R, p, t if sampled else None) for t, (dW, R) in enumerate(zip(dWs, Rs))]


def build_message(results: Sequence[TensorResult]) -> bytes:
    """Serialise what a client uploads: per tensor one signed fp32 mean and the
    Golomb bit string ("Optimal Position Encoding": positions plus one mean per
    tensor; shapes and b* are known to both sides).

    Layout (little endian): header {u32 magic, u32 version, u32 n_tensors,
    u32 b*, u64 payload_words, u64 0}; then per tensor {f32 mu_signed, u32 nnz,
    u64 bit_len, u64 word_offset}; then the payload of u32 words, each tensor's
    stream starting on a word boundary, streams in tensor order without gaps."""
    T = len(results)
    b = results[0].bstar if T else 0
    table = b""
    payload = []
    word_offset = 0
    for res in results:
        table += struct.pack("<fIQQ", float(res.mu_signed), len(res.kept), res.bit_len, word_offset)
        payload.append(res.words)
        word_offset += len(res.words)
    header = struct.pack("<IIIIQQ", MSG_MAGIC, MSG_VERSION, T, b, word_offset, 0)
    body = np.concatenate(payload).astype("<u4").tobytes() if payload else b""
    return header + table + body


def parse_message(msg: bytes):
    """Inverse of build_message: returns (b*, [(mu_signed, nnz, bit_len, words)])."""
    magic, version, T, b, payload_words, _ = struct.unpack_from("<IIIIQQ", msg, 0)
    if magic != MSG_MAGIC or version != MSG_VERSION:
        raise ValueError("not an SBC message")
    base = MSG_HEADER_BYTES + MSG_ENTRY_BYTES * T
    words_all = np.frombuffer(msg, dtype="<u4", count=payload_words, offset=base)
    out = []
    for t in range(T):
        mu, nnz, bit_len, woff = struct.unpack_from("<fIQQ", msg, MSG_HEADER_BYTES + MSG_ENTRY_BYTES * t)
        n_words = (bit_len + 31) // 32
        out.append((np.float32(mu), nnz, bit_len, words_all[woff:woff + n_words]))
    return b, out


def decode_accumulate(msg: bytes, numels: Sequence[int], scale: float, outs: Sequence[np.ndarray]) -> None:
    """Server lines of Alg. 1 for one client message: decode (Alg. 4) and add
    scale * dW* into the dense accumulators (scale = 1/|I_t| gives the average).
    fp32: the addend fl32(scale * mu) is formed once, then added."""
    b, entries = parse_message(msg)
    assert len(entries) == len(numels) == len(outs)
    for (mu, nnz, bit_len, words), n, out in zip(entries, numels, outs):
        bits = unpack_bits(words, bit_len)
        positions = golomb_decode(bits, b)
        if len(positions) != nnz or (positions and positions[-1] >= n):
            raise ValueError("corrupt message")
        addend = np.float32(np.float32(scale) * np.float32(mu))
        for j in positions:
            out[j] = np.float32(out[j] + addend)
