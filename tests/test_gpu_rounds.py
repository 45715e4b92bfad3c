"""Alg. 1's round loop through the HIP library against the same loop through the oracle."""
import numpy as np
import pytest

from oracle import sbc_oracle as o
from paper_1805_08768_amd import rounds, synth

pytestmark = pytest.mark.gpu


def _toy_problem(sizes, n_clients, seed=9):
    """Every client pulls the weights towards its own target; n local gradient steps of size lr."""
    g = synth.rng_for(seed)
    common = [g.standard_normal(n).astype(np.float32) for n in sizes]
    targets = [[(c + np.float32(0.1) * g.standard_normal(len(c)).astype(np.float32)).astype(np.float32) for c in common]
               for _ in range(n_clients)]
    lr, n_local = np.float32(0.25), 3

    def local_update(client, rnd, W):
        out = []
        for w, t in zip(W, targets[client]):
            wi = w.copy()
            for _ in range(n_local):
                wi = (wi - lr * (wi - t)).astype(np.float32)
            out.append((wi - w).astype(np.float32))
        return out

    return targets, local_update


def _oracle_rounds(sizes, p, n_clients, n_rounds, local_update, participants):
    W = [np.zeros(n, np.float32) for n in sizes]
    R = [[np.zeros(n, np.float32) for n in sizes] for _ in range(n_clients)]
    uploaded = []
    for rnd in range(n_rounds):
        chosen = list(participants(rnd))
        acc = [np.zeros(n, np.float32) for n in sizes]
        total = 0
        for i in chosen:
            res = o.compress_model(local_update(i, rnd, W), R[i], p)
            R[i] = [x.R_new for x in res]
            msg = o.build_message(res)
            total += len(msg)
            o.decode_accumulate(msg, sizes, 1.0 / len(chosen), acc)
        for w, a in zip(W, acc):
            w += a
        uploaded.append(total)
    return W, uploaded


def test_rounds_match_the_oracle_loop_and_converge():
    sizes = [5000, 64, 20000, 8193]
    p, n_clients, n_rounds = 0.05, 4, 12
    targets, local_update = _toy_problem(sizes, n_clients)
    participants = lambda rnd: [i for i in range(n_clients) if i != rnd % n_clients]    # three of four
    W_gpu, up_gpu = rounds.run_rounds(sizes, p, n_clients, n_rounds, local_update, participants=participants)
    W_cpu, up_cpu = _oracle_rounds(sizes, p, n_clients, n_rounds, local_update, participants)
    assert up_gpu == up_cpu
    for a, b in zip(W_gpu, W_cpu):
        assert np.array_equal(a, b)
    # error feedback at work: the weights move towards the mean target although only 5 % of the
    # entries of each update are sent, all with the same magnitude
    mean_t = [np.mean([targets[i][t] for i in range(n_clients)], axis=0) for t in range(len(sizes))]
    d0 = sum(float(np.sum(m.astype(np.float64) ** 2)) for m in mean_t)
    d1 = sum(float(np.sum((w.astype(np.float64) - m) ** 2)) for w, m in zip(W_gpu, mean_t))
    assert d1 < d0


def test_rounds_with_everything_resident_on_the_device():
    """The same loop with the weights, the updates and the averaging in device memory gives the
    weights of the loop that goes through host memory, bit for bit (that one is compared with the
    oracle's loop above)."""
    import torch
    sizes = [5000, 64, 20000, 8193]
    p, n_clients, n_rounds = 0.05, 4, 6
    targets, local_update = _toy_problem(sizes, n_clients)
    participants = lambda rnd: [i for i in range(n_clients) if i != rnd % n_clients]
    W_host, up_host = rounds.run_rounds(sizes, p, n_clients, n_rounds, local_update, participants=participants)
    dev_targets = [[torch.from_numpy(t).cuda() for t in per_client] for per_client in targets]

    def local_update_dev(client, rnd, W, out):
        for w, t, dst in zip(W, dev_targets[client], out):
            wi = w.clone()
            for _ in range(3):
                wi = wi - 0.25 * (wi - t)            # fp32 throughout, as in the host callback
            torch.sub(wi, w, out=dst)

    W_dev, up_dev = rounds.run_rounds(sizes, p, n_clients, n_rounds, local_update_dev, participants=participants,
                                      on_device=True)
    assert up_dev == up_host
    for a, b in zip(W_dev, W_host):
        assert np.array_equal(a.cpu().numpy(), b)
