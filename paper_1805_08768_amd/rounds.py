"""Synchronous rounds of Alg. 1 on one GPU with synthetic local training.

Alg. 1 alternates between clients (download the averaged update, train locally for n
iterations, add the residual, compress, keep the new residual, upload) and a server (gather
the messages of the participating clients I_t, average the sparse binary updates, broadcast).
Here every client is an object holding its residual R_i and an sbc context; "training" is a
callback that returns the client's dense weight update, so no model, data set or optimizer is
involved.  All of the method's arithmetic runs in the HIP library through the C ABI binding:
sbc_compress on the client side, sbc_decompress_accumulate on the server side; this module
only moves buffers and calls the callback.

Two ways of running the loop: with the weights and the callback's updates in host memory
(the form the tests compare with the oracle's loop), or with everything resident in device
memory (`on_device=True`): the callback writes each client's update into that client's device
buffer, the server's average is added to the device weights, and nothing crosses PCIe but the
16-byte result blocks.  Buffers are flat (one allocation per client and kind, every tensor a
view at a 256-byte aligned offset), so that clearing the server's accumulator and the weight
update are one elementwise launch each, not one per tensor.

The kept-position mask of a client's last upload (the input of momentum masking, supplement
"Momentum Masking") is available as Client.last_mask().
"""
from __future__ import annotations

from typing import Callable, List, Optional, Sequence

import numpy as np
import torch

from . import binding as sbc


class TensorViews(list):
    """The per-tensor views of a flat buffer; `flat` is the buffer itself (padding included)."""
    flat: torch.Tensor = None


def flat_buffer(sizes: Sequence[int], device: str):
    """One zeroed fp32 allocation holding a tensor of every size, each at a 256-byte aligned
    offset (the streaming kernel takes 16-byte loads only from 16-byte aligned chunks), and
    the per-tensor views (a TensorViews list)."""
    offsets, total = [], 0
    for n in sizes:
        offsets.append(total)
        total += (int(n) + 63) // 64 * 64
    flat = torch.zeros(max(total, 1), dtype=torch.float32, device=device)
    views = TensorViews(flat[o:o + int(n)] for o, n in zip(offsets, sizes))
    views.flat = flat
    return flat, views


class Client:
    """Client i of Alg. 1: weights W_i, residual R_i (initially zero), one message buffer."""

    def __init__(self, sizes: Sequence[int], p: float, device: str = "cuda:0"):
        self.sizes = [int(s) for s in sizes]
        self.p = float(p)
        self.device = device
        index = torch.device(device).index or 0
        self.ctx = sbc.sbc_create(index, sum(self.sizes), len(self.sizes))
        self.R_flat, self.R = flat_buffer(self.sizes, device)
        self.dW_flat, self.dW = flat_buffer(self.sizes, device)
        self._R_list = sbc.TensorList(self.R)
        self._dW_list = sbc.TensorList(self.dW)
        self.msg = torch.zeros(sbc.sbc_msg_bound(self.sizes, self.p), dtype=torch.uint8, device=device)
        self.nbytes = 0
        self.stream = torch.cuda.Stream(device=device)    # clients work in parallel (Alg. 1)

    def begin_upload(self, update: Optional[Sequence[np.ndarray]] = None):
        """dW_i <- R_i + update; dW*_i <- SBC(dW_i); R_i <- dW_i - dW*_i, enqueued on the client's
        stream without waiting.  update: host arrays, or None if the caller has written the
        update into self.dW (device memory) on the client's stream already."""
        if update is not None:
            with torch.cuda.stream(self.stream):
                for dst, src in zip(self.dW, update):
                    dst.copy_(torch.from_numpy(np.ascontiguousarray(src, dtype=np.float32)))
        sbc.sbc_compress_begin(self.ctx, self._dW_list, self._R_list, self.p, self.msg, self.stream)

    def end_upload(self):
        """Waits for begin_upload; returns (msg, nbytes).  The size is known as soon as the step's
        last kernel has reported it, which may be before the client's stream is idle: whatever the
        caller's current stream does next (the server's decoding) is ordered behind the client's."""
        self.nbytes = sbc.sbc_compress_end(self.ctx)
        torch.cuda.current_stream().wait_stream(self.stream)
        return self.msg, self.nbytes

    def upload(self, update: Sequence[np.ndarray]):
        self.begin_upload(update)
        return self.end_upload()

    def last_mask(self, tensor: int) -> torch.Tensor:
        """Bit mask (uint32 words, bit j of word j // 32) of the positions sent in the last upload."""
        return sbc.sbc_last_mask(self.ctx, tensor, self.sizes[tensor])

    def close(self):
        if self.ctx is not None:
            sbc.sbc_destroy(self.ctx)
            self.ctx = None


class Server:
    """Server of Alg. 1: decodes the gathered messages and averages them into a dense update."""

    def __init__(self, sizes: Sequence[int], p: float, device: str = "cuda:0"):
        self.sizes = [int(s) for s in sizes]
        self.p = float(p)
        index = torch.device(device).index or 0
        self.ctx = sbc.sbc_create(index, sum(self.sizes), len(self.sizes))
        # the messages of a round are decoded back to back; one status check at the end
        sbc.sbc_set_option(self.ctx, sbc.SBC_OPT_DEFER_DECODE_STATUS, 1)
        self.acc_flat, self.acc = flat_buffer(self.sizes, device)
        self._acc_list = sbc.TensorList(self.acc)

    def average(self, messages) -> List[torch.Tensor]:
        """dW <- 1/|I_t| * sum of the clients' sparse binary updates (messages in client order)."""
        self.acc_flat.zero_()
        scale = 1.0 / len(messages)
        for msg, nbytes in messages:
            sbc.sbc_decompress_accumulate(self.ctx, msg, nbytes, self.p, scale, self._acc_list)
        sbc.sbc_decode_status(self.ctx)
        return self.acc

    def close(self):
        if self.ctx is not None:
            sbc.sbc_destroy(self.ctx)
            self.ctx = None


def run_rounds(sizes: Sequence[int], p: float, n_clients: int, n_rounds: int,
               local_update: Callable, weights: Optional[List[np.ndarray]] = None,
               participants: Optional[Callable[[int], Sequence[int]]] = None,
               device: str = "cuda:0", on_device: bool = False,
               on_round_end: Optional[Callable[[int], None]] = None):
    """Runs n_rounds of Alg. 1; participants(round) lists I_t (default: every client).

    on_device=False: local_update(client, round, W) returns the dense update SGD_n(W) - W of that
    client as fp32 host arrays (W: the current global weights, host arrays).  Returns the final
    global weights (host arrays) and the bytes uploaded per round.

    on_device=True: local_update(client, round, W, out) writes that update into `out` (the
    client's device buffers, one fp32 tensor per model tensor; W: the global weights, device
    tensors; both are TensorViews, whose `flat` is the whole buffer in flat_buffer's layout) with
    torch operations on the current stream, which is the client's.  Returns the
    final global weights (device tensors) and the bytes uploaded per round.

    on_round_end(round), if given, is called after each round's weight update has been enqueued."""
    clients = [Client(sizes, p, device) for _ in range(n_clients)]
    server = Server(sizes, p, device)
    uploaded = []
    if on_device:
        W_flat, W = flat_buffer(sizes, device)
        if weights is not None:
            for w, src in zip(W, weights):
                w.copy_(torch.from_numpy(np.ascontiguousarray(src, dtype=np.float32)))
    else:
        W = [np.zeros(n, np.float32) for n in sizes] if weights is None else [w.astype(np.float32).copy() for w in weights]
    try:
        for rnd in range(n_rounds):
            chosen = list(range(n_clients)) if participants is None else list(participants(rnd))
            for i in chosen:                          # "for all clients in parallel"
                if on_device:
                    clients[i].stream.wait_stream(torch.cuda.current_stream())    # the weights of this round
                    with torch.cuda.stream(clients[i].stream):
                        local_update(i, rnd, W, clients[i].dW)
                    clients[i].begin_upload()
                else:
                    clients[i].begin_upload(local_update(i, rnd, W))
            messages = [clients[i].end_upload() for i in chosen]
            avg = server.average(messages)
            # W <- W + dW, the broadcast every client downloads
            if on_device:
                W_flat.add_(server.acc_flat)          # (the padding between the tensors stays zero)
            else:
                for w, a in zip(W, avg):
                    w += a.cpu().numpy()
            uploaded.append(sum(nb for _, nb in messages))
            if on_round_end is not None:
                on_round_end(rnd)
        if on_device:
            torch.cuda.current_stream().synchronize()
    finally:
        for c in clients:
            c.close()
        server.close()
    return W, uploaded
