"""Seeded synthetic weight updates shaped like the paper's CNN and RNN workloads.

This module only draws random numbers and lists tensor shapes; it holds none of
the method's arithmetic and is shared by the tests, the benchmark and the smoke
check.  It depends on NumPy alone (no GPU, no compiled extension).

The paper trains ResNet50 on ImageNet and a two-layer word LSTM on PTB
("Networks and Datasets"); neither the data sets nor trained weights are
available here, so weight updates are synthetic stand-ins with the same tensor
shapes and heavy-tailed value distributions.

Every array comes from numpy.random.Generator(PCG64(SeedSequence([BASE_SEED,
config, client, round, tensor]))) and is cast to fp32 on the host, so that
every consumer sees identical bits.
"""
from __future__ import annotations

from typing import List, Tuple

import numpy as np

BASE_SEED = 180508768


def rng_for(config: int, client: int = 0, round_: int = 0, tensor: int = 0) -> np.random.Generator:
    return np.random.Generator(np.random.PCG64(np.random.SeedSequence(
        [BASE_SEED, int(config), int(client), int(round_), int(tensor)])))


# ---------------------------------------------------------------- shapes ----

def resnet50_shapes() -> List[Tuple[str, Tuple[int, ...]]]:
    """Bottleneck ResNet-50: 7x7 stem, stages of 3-4-6-3 blocks with widths
    64/128/256/512 (1x1 -> 3x3 -> 1x1 expanding x4, 1x1 projection in the first
    block of each stage), scale and shift per batch-norm, 2048x1000 classifier
    with bias.  161 tensors, 25,557,032 parameters."""
    shapes: List[Tuple[str, Tuple[int, ...]]] = []

    def conv_bn(name, kh, kw, cin, cout):
        shapes.append((name + ".w", (kh, kw, cin, cout)))
        shapes.append((name + ".bn.gamma", (cout,)))
        shapes.append((name + ".bn.beta", (cout,)))

    conv_bn("stem", 7, 7, 3, 64)
    cin = 64
    for s, (width, blocks) in enumerate(zip((64, 128, 256, 512), (3, 4, 6, 3))):
        for blk in range(blocks):
            name = "stage%d.block%d" % (s + 1, blk)
            if blk == 0:
                conv_bn(name + ".proj", 1, 1, cin, 4 * width)
            conv_bn(name + ".conv1", 1, 1, cin, width)
            conv_bn(name + ".conv2", 3, 3, width, width)
            conv_bn(name + ".conv3", 1, 1, width, 4 * width)
            cin = 4 * width
    shapes.append(("fc.w", (2048, 1000)))
    shapes.append(("fc.b", (1000,)))
    return shapes


def lstm_lm_shapes(vocab: int = 10000, hidden: int = 1500) -> List[Tuple[str, Tuple[int, ...]]]:
    """Two-layer LSTM language model: embedding, per layer input and recurrent
    weights for the four gates plus a gate bias, soft-max weights and bias.
    9 tensors, 66,022,000 parameters at vocab 10000 / hidden 1500."""
    shapes = [("embedding", (vocab, hidden))]
    for layer in range(2):
        shapes.append(("lstm%d.w_ih" % layer, (4 * hidden, hidden)))
        shapes.append(("lstm%d.w_hh" % layer, (4 * hidden, hidden)))
        shapes.append(("lstm%d.b" % layer, (4 * hidden,)))
    shapes.append(("softmax.w", (hidden, vocab)))
    shapes.append(("softmax.b", (vocab,)))
    return shapes


def numels(shapes) -> List[int]:
    return [int(np.prod(s)) for _, s in shapes]


# ---------------------------------------------------------------- values ----

def gaussian_update(n: int, sigma: float = 1e-3, *, config: int = 1, client: int = 0,
                    round_: int = 0, tensor: int = 0) -> np.ndarray:
    """Config 1: dW ~ N(0, sigma^2), fp32."""
    g = rng_for(config, client, round_, tensor)
    return (g.standard_normal(n, dtype=np.float64) * sigma).astype(np.float32)


def student_t_update(n: int, scale: float = 1e-3, dup_frac: float = 0.01, *, config: int = 2,
                     client: int = 0, round_: int = 0, tensor: int = 0) -> np.ndarray:
    """Config 2: scale * Student-t(nu=3); then dup_frac of the positions are
    overwritten with the fp32 value found at another uniformly random position,
    so exact duplicates also occur in the tails."""
    g = rng_for(config, client, round_, tensor)
    x = (g.standard_t(3.0, n) * scale).astype(np.float32)
    m = int(dup_frac * n)
    if m > 0:
        dst = g.integers(0, n, size=m)
        src = g.integers(0, n, size=m)
        x[dst] = x[src]
    return x


def palette_update(n: int, *, config: int = 6, client: int = 0, round_: int = 0,
                   tensor: int = 0) -> np.ndarray:
    """Tie-stress companion of config 2: Student-t draws snapped to the 257
    values i * 2^-17, i = -128..128, so every threshold is tied many times and
    the lowest-index rule decides most of the mask."""
    g = rng_for(config, client, round_, tensor)
    x = g.standard_t(3.0, n) * 1e-3
    i = np.clip(np.rint(x * 2.0 ** 17), -128, 128)
    return (i * 2.0 ** -17).astype(np.float32)


def tensor_scale(config: int, tensor: int) -> float:
    """s_t = 10^U(-4, -2): a property of the tensor (layer), the same in every round and client."""
    return 10.0 ** rng_for(config, 0, 0, tensor).uniform(-4.0, -2.0)


def resnet50_update(*, client: int = 0, round_: int = 0, config: int = 3) -> List[np.ndarray]:
    """Config 3: Laplace(0, s_t) per tensor with s_t = 10^U(-4, -2)."""
    out = []
    for t, n in enumerate(numels(resnet50_shapes())):
        g = rng_for(config, client + 1, round_ + 1, t)
        out.append(g.laplace(0.0, tensor_scale(config, t), n).astype(np.float32))
    return out


def lstm_lm_update(*, client: int = 0, round_: int = 0, config: int = 4, sigma: float = 1e-3,
                   active_rows: float = 0.05, vocab: int = 10000, hidden: int = 1500) -> List[np.ndarray]:
    """Config 4: Gaussian entries (sigma); the embedding has only a fraction
    active_rows of its rows non-zero in a round (words seen in the batch)."""
    out = []
    for t, (name, shape) in enumerate(lstm_lm_shapes(vocab, hidden)):
        g = rng_for(config, client, round_, t)
        n = int(np.prod(shape))
        if name == "embedding":
            x = np.zeros(shape, dtype=np.float32)
            rows = g.choice(shape[0], size=max(1, int(active_rows * shape[0])), replace=False)
            x[rows] = (g.standard_normal((len(rows), shape[1])) * sigma).astype(np.float32)
            out.append(x.reshape(-1))
        else:
            out.append((g.standard_normal(n, dtype=np.float32) * np.float32(sigma)).astype(np.float32))
    return out


def flat_gaussian_chunks(n: int, sigma: float = 1e-3, chunk: int = 1 << 26, *, config: int = 5,
                         client: int = 0, round_: int = 0):
    """Config 5b: a flat N(0, sigma^2) update of n entries, yielded in chunks
    (offset, fp32 array) so that a 1.5e9-entry tensor never sits in host memory
    twice."""
    off = 0
    c = 0
    while off < n:
        m = min(chunk, n - off)
        g = rng_for(config, client, round_, c)
        yield off, (g.standard_normal(m, dtype=np.float32) * np.float32(sigma)).astype(np.float32)
        off += m
        c += 1


def small_model_update(sizes, *, config: int = 7, client: int = 0, round_: int = 0) -> List[np.ndarray]:
    """A few tensors of arbitrary sizes with Laplace values, for fast tests that
    still span several tiles and ragged tails."""
    out = []
    for t, n in enumerate(sizes):
        g = rng_for(config, client + 1, round_ + 1, t)
        out.append(g.laplace(0.0, tensor_scale(config, t), int(n)).astype(np.float32))
    return out
