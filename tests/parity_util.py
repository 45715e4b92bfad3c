"""Shared helper of the GPU parity tests: runs the HIP path through the C ABI binding and
the oracle on the same inputs and compares every output the parity contract names."""
from __future__ import annotations

import struct
from typing import List, Sequence

import numpy as np
import torch

from oracle import sbc_oracle as o
from paper_1805_08768_amd import binding as sbc

REL_TOL = 1e-5  # mu+, mu- and the residual at kept positions, against the fp64 oracle
FUSED_STEP = 0  # set by the test modules' fixtures: every DeviceRun then sets SBC_OPT_FUSED_STEP


def mask_to_positions(words: torch.Tensor, n: int) -> np.ndarray:
    w = words.numpy().view(np.uint32)
    bits = np.unpackbits(w.view(np.uint8), bitorder="little")[:n]
    return np.flatnonzero(bits).astype(np.int64)


class DeviceRun:
    """One sbc context plus device copies of a model's update and residual."""

    def __init__(self, sizes: Sequence[int], device: str = "cuda:0", slack: int = 0, sampled: bool = False,
                 compact: bool = False):
        self.sizes = [int(s) for s in sizes]
        self.device = device
        self.sampled = sampled
        dev_index = 0 if device == "cpu" else torch.device(device).index or 0
        self.ctx = (sbc.sbc_create_compact if compact else sbc.sbc_create)(dev_index, sum(self.sizes) + slack, len(self.sizes))
        if sampled:
            sbc.sbc_set_option(self.ctx, sbc.SBC_OPT_SAMPLED_THRESHOLD, 1)
        if FUSED_STEP:
            sbc.sbc_set_option(self.ctx, sbc.SBC_OPT_FUSED_STEP, 1)
        self.R = [torch.zeros(n, dtype=torch.float32, device=device) for n in self.sizes]

    def close(self):
        if self.ctx is not None:
            sbc.sbc_destroy(self.ctx)
            self.ctx = None

    def __enter__(self):
        return self

    def __exit__(self, *exc):
        self.close()

    def msg_bound(self, p: float) -> int:
        return (sbc.sbc_msg_bound_sampled if self.sampled else sbc.sbc_msg_bound)(self.sizes, p)

    def compress(self, dWs: Sequence[np.ndarray], p: float):
        d_dW = [torch.from_numpy(np.ascontiguousarray(x)).to(self.device) for x in dWs]
        bound = self.msg_bound(p)
        assert bound > 0
        msg = torch.full((bound + 64,), 0xAB, dtype=torch.uint8, device=self.device)
        nbytes = sbc.sbc_compress(self.ctx, d_dW, self.R, p, msg)
        return msg, nbytes


def check_round(run: DeviceRun, dWs: Sequence[np.ndarray], R_before: Sequence[np.ndarray], p: float,
                check_decode: bool = True) -> List[o.TensorResult]:
    """One round: HIP compress vs oracle compress.  Returns the oracle results."""
    results = o.compress_model(dWs, R_before, p, sampled=run.sampled)
    want_msg = o.build_message(results)
    msg, nbytes = run.compress(dWs, p)
    got_msg = bytes(msg[:nbytes].cpu().numpy().tobytes())
    T = len(results)

    # --- per-tensor table and statistics
    assert nbytes <= run.msg_bound(p)
    assert got_msg[:32] == want_msg[:32], "message header differs"
    for t, res in enumerate(results):
        mu_g, nnz_g, bl_g, wo_g = struct.unpack_from("<fIQQ", got_msg, 32 + 24 * t)
        mu_w, nnz_w, bl_w, wo_w = struct.unpack_from("<fIQQ", want_msg, 32 + 24 * t)
        mu_pos, mu_neg, side, nnz, bit_len = sbc.sbc_last_tensor_stats(run.ctx, t)
        assert side == res.side, "tensor %d: side %d, oracle %d (mu+ %r mu- %r)" % (t, side, res.side, res.mu_pos, res.mu_neg)
        assert abs(mu_pos - res.mu_pos) <= REL_TOL * abs(res.mu_pos), (t, mu_pos, res.mu_pos)
        assert abs(mu_neg - res.mu_neg) <= REL_TOL * abs(res.mu_neg), (t, mu_neg, res.mu_neg)
        assert nnz == nnz_g == len(res.kept), (t, nnz, nnz_g, len(res.kept))
        assert run.sampled or nnz == res.k
        # mask (bit exact)
        kept = mask_to_positions(sbc.sbc_last_mask(run.ctx, t, res.n), res.n)
        assert np.array_equal(kept, res.kept), "tensor %d: mask differs" % t
        assert (bl_g, wo_g) == (bl_w, wo_w) and bit_len == bl_w, (t, bl_g, bl_w, wo_g, wo_w)
        assert abs(mu_g - float(res.mu_signed)) <= REL_TOL * abs(float(res.mu_signed)), (t, mu_g, res.mu_signed)
        assert np.float32(mu_g) == res.mu_signed, \
            "tensor %d: transmitted mean differs in the last place (%r vs %r)" % (t, mu_g, res.mu_signed)
        # residual
        R_got = run.R[t].cpu().numpy()
        off = np.ones(res.n, dtype=bool)
        off[res.kept] = False
        assert np.array_equal(R_got[off], res.R_new[off]), "tensor %d: residual off the kept set" % t
        tol = REL_TOL * np.maximum(np.abs(res.A[res.kept]), abs(float(res.mu_signed)))
        assert np.all(np.abs(R_got[res.kept].astype(np.float64) - res.R_new[res.kept]) <= tol), \
            "tensor %d: residual at kept positions" % t
    # --- bitstream and whole message (bit exact)
    assert got_msg == want_msg, "message bytes differ"
    # the cleared-but-unused tail of the payload and the guard bytes behind the bound
    assert (msg[nbytes:].cpu().numpy() == 0xAB).all(), "wrote past the message"

    if check_decode:
        outs = [torch.zeros(n, dtype=torch.float32, device=run.device) for n in run.sizes]
        sbc.sbc_decompress_accumulate(run.ctx, msg, nbytes, p, 1.0, outs)
        for t, res in enumerate(results):
            assert np.array_equal(outs[t].cpu().numpy(), res.dense_update()), "tensor %d: decode" % t
        # accumulate a second time with another scale onto non-zero accumulators
        base = [np.full(n, 0.5, dtype=np.float32) for n in run.sizes]
        outs = [torch.from_numpy(b.copy()).to(run.device) for b in base]
        sbc.sbc_decompress_accumulate(run.ctx, msg, nbytes, p, 0.25, outs)
        o.decode_accumulate(want_msg, run.sizes, 0.25, base)
        for t in range(T):
            assert np.array_equal(outs[t].cpu().numpy(), base[t]), "tensor %d: scaled decode" % t
    return results
