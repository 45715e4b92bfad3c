"""Synchronous rounds of Alg. 1 on one GPU with synthetic local training.

Alg. 1 alternates between clients (download the averaged update, train locally for n
iterations, add the residual, compress, keep the new residual, upload) and a server (gather
the messages of the participating clients I_t, average the sparse binary updates, broadcast).
Here every client is an object holding its residual R_i and an sbc context; "training" is a
callback that returns the client's dense weight update, so no model, data set or optimizer is
involved.  All of the method's arithmetic runs in the HIP library through the C ABI binding:
sbc_compress on the client side, sbc_decompress_accumulate on the server side; this module
only moves buffers and calls the callback.

The kept-position mask of a client's last upload (the input of momentum masking, supplement
"Momentum Masking") is available as Client.last_mask().
"""
from __future__ import annotations

from typing import Callable, List, Optional, Sequence

import numpy as np
import torch

from . import binding as sbc


class Client:
    """Client i of Alg. 1: weights W_i, residual R_i (initially zero), one message buffer."""

    def __init__(self, sizes: Sequence[int], p: float, device: str = "cuda:0"):
        self.sizes = [int(s) for s in sizes]
        self.p = float(p)
        self.device = device
        index = torch.device(device).index or 0
        self.ctx = sbc.sbc_create(index, sum(self.sizes), len(self.sizes))
        self.R = [torch.zeros(n, dtype=torch.float32, device=device) for n in self.sizes]
        self.dW = [torch.zeros(n, dtype=torch.float32, device=device) for n in self.sizes]
        self._R_list = sbc.TensorList(self.R)
        self._dW_list = sbc.TensorList(self.dW)
        self.msg = torch.zeros(sbc.sbc_msg_bound(self.sizes, self.p), dtype=torch.uint8, device=device)
        self.nbytes = 0
        self.stream = torch.cuda.Stream(device=device)    # clients work in parallel (Alg. 1)

    def begin_upload(self, update: Sequence[np.ndarray]):
        """dW_i <- R_i + update; dW*_i <- SBC(dW_i); R_i <- dW_i - dW*_i, enqueued on the client's
        stream without waiting."""
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
        self.acc = [torch.zeros(n, dtype=torch.float32, device=device) for n in self.sizes]
        self._acc_list = sbc.TensorList(self.acc)

    def average(self, messages) -> List[torch.Tensor]:
        """dW <- 1/|I_t| * sum of the clients' sparse binary updates (messages in client order)."""
        for a in self.acc:
            a.zero_()
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
               local_update: Callable[[int, int, List[np.ndarray]], List[np.ndarray]],
               weights: Optional[List[np.ndarray]] = None,
               participants: Optional[Callable[[int], Sequence[int]]] = None,
               device: str = "cuda:0"):
    """Runs n_rounds of Alg. 1.  local_update(client, round, W) returns the dense update
    SGD_n(W) - W of that client as fp32 host arrays (W: the current global weights, host arrays);
    participants(round) lists I_t (default: every client).  Returns the final global weights
    (host arrays) and the bytes uploaded per round."""
    W = [np.zeros(n, np.float32) for n in sizes] if weights is None else [w.astype(np.float32).copy() for w in weights]
    clients = [Client(sizes, p, device) for _ in range(n_clients)]
    server = Server(sizes, p, device)
    uploaded = []
    try:
        for rnd in range(n_rounds):
            chosen = list(range(n_clients)) if participants is None else list(participants(rnd))
            for i in chosen:                          # "for all clients in parallel"
                clients[i].begin_upload(local_update(i, rnd, W))
            messages = [clients[i].end_upload() for i in chosen]
            avg = server.average(messages)
            for w, a in zip(W, avg):
                w += a.cpu().numpy()              # W <- W + dW, the broadcast every client downloads
            uploaded.append(sum(nb for _, nb in messages))
    finally:
        for c in clients:
            c.close()
        server.close()
    return W, uploaded
