#!/usr/bin/env python3
"""Benchmark of the SBC hot path on one MI355X.

A step is one communication round of one client on the ResNet-50-shaped update (161 fp32
tensors, 25,557,032 entries, p = 0.001): sbc_compress (residual accumulation, exact top-k on
both sign sides, means, binarization, residual update, Golomb encoding) followed by
sbc_decompress_accumulate of the produced message into a dense accumulator (Golomb decoding
and the server's scaled accumulation).  Inputs are resident in HBM before the timed region.

Prints ONE JSON line.  `value` is entries per second over whole steps (wall clock between two
device synchronisations; the client call waits for its result, the client's next round is
enqueued into a second message buffer, then the server call on the round's message, whose
validation status is collected once for all steps before the clock stops); the median and the
minimum of the single steps' periods stand beside the mean.  `compress_ms` and `decode_ms` are
the latencies of the two calls when each is waited for, from a second loop.

`roofline` is for the dominant kernel, the residual-accumulation pass: 12 algorithmic bytes per
entry (read dW, read R, write R') times the entries of the update, divided by that kernel's
duration measured with HIP events on the launch stream.  Its headline figures (`frac`,
`achieved`, `kernel_avg_us`) are taken with the caches flushed before every call, so that no
part of the residual is still in the last-level cache from the round before; `timed_region`
holds the same kernel's duration on the launches inside the timed steps (back to back, partly
cache-warm).  `step_frac` is the same byte count over the whole compress call.  `traffic` is
read from the committed counter summary under profiles/, with its source beside it.
`cpu_baseline` is the CPU oracle timed on this machine's host cores: on one core, and with
the tensors dealt out over all cores the process may use.
"""
from __future__ import annotations

import argparse
import json
import multiprocessing
import os
import re
import statistics
import sys
import time

import numpy as np

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0          # MI355X HBM3E, published peak
BYTES_PER_ENTRY = 12           # read dW, read R, write R'
P = 0.001
PROFILE_EVERY = 6            # timed steps between two event-bracketed launches of the streaming kernel
COLD_LAUNCHES = 12           # calls with the caches flushed before each
CPU_ROUNDS = 3               # rounds of the whole update the CPU oracle is timed on, per leg

# HBM bytes per launch of the streaming kernel on the default workload come from two rocprofv3
# --pmc runs (FETCH_SIZE, then WRITE_SIZE, each scaled by what the same counter shows for the
# plain copy kernel of known size); the summary of those runs is read at run time.
TRAFFIC_SUMMARY = os.path.join("profiles", "bench_resnet50_hbm_counters.md")


def traffic_from_profile():
    """(bytes per launch, kernel name, source) from the committed counter summary, or (None, None, None)."""
    try:
        text = open(os.path.join(ROOT, TRAFFIC_SUMMARY)).read()
    except OSError:
        return None, None, None
    m = re.search(r"^HBM traffic per launch of (\S+) = (\d+) bytes", text, flags=re.M)
    if not m:
        return None, None, None
    return int(m.group(2)), m.group(1), TRAFFIC_SUMMARY


# ---------------------------------------------------------------------------------------------
# CPU baseline: the oracle as it stands, in child processes that never touch the GPU.  They are
# started before the parent's first GPU call and wait for their work until the GPU part is over.
# ---------------------------------------------------------------------------------------------
def _cpu_worker(conn):
    import numpy as np
    from oracle import sbc_oracle as oracle
    updates, sizes, p, scale = None, None, None, None
    while True:
        msg = conn.recv()
        if msg[0] == "data":                       # the worker's tensors of every round (untimed)
            _, updates, p, scale = msg
            sizes = [len(d) for d in updates[0]]
            conn.send(("ready", os.getpid()))
        elif msg[0] == "go":                       # Alg. 1 on those tensors: client rounds + server accumulation
            t0 = time.perf_counter()
            R = [np.zeros(n, np.float32) for n in sizes]
            accs = [np.zeros(n, np.float32) for n in sizes]
            nbytes = 0
            for dWs in updates:
                res = oracle.compress_model(dWs, R, p)
                R = [x.R_new for x in res]
                m = oracle.build_message(res)
                nbytes += len(m)
                oracle.decode_accumulate(m, sizes, scale, accs)
            conn.send(("done", time.perf_counter() - t0, nbytes))
        else:
            return


class CpuBaseline:
    """One child process per usable core, each with a share of the tensors (largest first, always
    to the least loaded: the tensors of a model are compressed independently, Alg. 2)."""

    def __init__(self):
        self.cores = sorted(os.sched_getaffinity(0))
        ctx = multiprocessing.get_context("spawn")
        self.workers = []
        for _ in self.cores:
            parent, child = ctx.Pipe()
            pr = ctx.Process(target=_cpu_worker, args=(child,), daemon=True)
            pr.start()
            child.close()
            self.workers.append((pr, parent))

    def _leg(self, n_workers, host_sets, sizes, p, scale):
        order = sorted(range(len(sizes)), key=lambda t: -sizes[t])
        load, share = [0] * n_workers, [[] for _ in range(n_workers)]
        for t in order:
            w = min(range(n_workers), key=lambda i: load[i])
            share[w].append(t)
            load[w] += sizes[t]
        used = [w for w in range(n_workers) if share[w]]
        for w in used:
            self.workers[w][1].send(("data", [[h[t] for t in share[w]] for h in host_sets], p, scale))
        for w in used:
            assert self.workers[w][1].recv()[0] == "ready"
        t0 = time.perf_counter()
        for w in used:
            self.workers[w][1].send(("go",))
        results = [self.workers[w][1].recv() for w in used]
        wall = time.perf_counter() - t0
        n_total = sum(sizes) * len(host_sets)
        return {"value": n_total / wall, "unit": "elements/s", "cores": len(used), "kind": "oracle",
                "seconds": round(wall, 2), "slowest_worker_seconds": round(max(r[1] for r in results), 2),
                "message_bytes_per_round": sum(r[2] for r in results) / len(host_sets)}

    def run(self, host_sets, sizes, p, scale):
        one = self._leg(1, host_sets, sizes, p, scale)
        every = self._leg(len(self.workers), host_sets, sizes, p, scale)
        sample = ("%d rounds (compress + build message + decode-accumulate, residual carried) of the same "
                  "%d-tensor update, %d entries per round; one core: %.1f s; %d processes, tensors dealt out "
                  "by size: %.1f s" % (len(host_sets), len(sizes), sum(sizes), one["seconds"], every["cores"],
                                       every["seconds"]))
        out = dict(every)
        out["sample"] = sample
        out["usable_cores"] = len(self.cores)
        out["legs"] = [one, every]
        return out

    def close(self):
        for pr, conn in self.workers:
            try:
                conn.send(("stop",))
            except OSError:
                pass
        for pr, conn in self.workers:
            pr.join(timeout=10)


def main() -> int:
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=50)
    ap.add_argument("--warmup", type=int, default=5)
    ap.add_argument("--no-cpu-baseline", action="store_true", help="skip timing the CPU oracle")
    ap.add_argument("--breakdown", action="store_true", help="also print per-kernel times to stderr")
    ap.add_argument("--no-carry-keys", action="store_true",
                    help="clear SBC_OPT_CARRY_FILTER_KEYS (every round estimates its filter keys from a sample "
                         "instead of starting from the previous round's)")
    ap.add_argument("--fused-step", action="store_true", help="set SBC_OPT_FUSED_STEP")
    ap.add_argument("--compact-context", action="store_true",
                    help="contexts from sbc_create_compact (candidate lists of a quarter of each tensor per side: about 5 "
                         "bytes of scratch per entry instead of 17)")
    ap.add_argument("--sampled-threshold", action="store_true",
                    help="set SBC_OPT_SAMPLED_THRESHOLD (the subsampled variant with a noisy amount of sparsity; "
                         "reported for reference, not the benchmark's mode)")
    ap.add_argument("--no-pipelined-extra", action="store_true",
                    help="skip the untimed three-client run (used under the profiler, where overlapping "
                         "launches would blur the per-kernel averages)")
    ap.add_argument("--clients-in-flight", type=int, default=1,
                    help="independent clients (own residual, context, stream, message) whose steps overlap; "
                         "step s belongs to client s mod C")
    ap.add_argument("--workload", default="resnet50", choices=["resnet50", "lstm", "gauss2p20", "student4m", "flat1p5e9"],
                    help="resnet50 (default) is the benchmark workload; the others are reported for reference")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build runs on one GPU; --gpus %d is not supported "
              "(nothing here shards over several GPUs)" % args.gpus, file=sys.stderr)
        return 2

    # the CPU baseline's processes start before this process touches the GPU
    cpu_pool = None
    if not args.no_cpu_baseline and args.workload == "resnet50":
        cpu_pool = CpuBaseline()

    import torch
    from paper_1805_08768_amd import accounting, binding as sbc, synth

    if not torch.cuda.is_available():
        print("bench.py: no GPU visible", file=sys.stderr)
        return 2
    dev = "cuda:0"
    global P
    n_sets = 3
    if args.workload == "resnet50":
        sizes = synth.numels(synth.resnet50_shapes())
        gen = lambda r: synth.resnet50_update(round_=r)
        name = ("ResNet-50-shaped update: 161 fp32 tensors, 25,557,032 entries, "
                "Laplace values with per-tensor scale 10^U(-4,-2), p=0.001, residual carried")
    elif args.workload == "lstm":
        sizes = synth.numels(synth.lstm_lm_shapes()); P = 1e-4
        gen = lambda r: synth.lstm_lm_update(round_=r)
        name = "2-layer LSTM LM-shaped update: 9 tensors, 66,022,000 entries, p=1e-4"
    elif args.workload == "gauss2p20":
        sizes = [1 << 20]; P = 0.01
        gen = lambda r: [synth.gaussian_update(1 << 20, round_=r)]
        name = "one tensor, 2^20 entries, N(0,1e-6), p=0.01"
    elif args.workload == "student4m":
        sizes = [4194304]
        gen = lambda r: [synth.student_t_update(4194304, round_=r)]
        name = "one tensor, 4,194,304 entries, Student-t(3), p=0.001"
    else:
        sizes = [1_500_000_000]; n_sets = 2
        gen = lambda r: [np.concatenate([c for _, c in synth.flat_gaussian_chunks(sizes[0], round_=r)])]
        name = "one flat tensor, 1.5e9 entries, N(0,1e-6), p=0.001"
    N = sum(sizes)
    T = len(sizes)

    # a few different updates resident in HBM, used round-robin; the residual carries over
    host_sets = [gen(r) for r in range(n_sets)]
    flat_sets = [torch.from_numpy(np.concatenate(h) if len(h) > 1 else h[0]).to(dev) for h in host_sets]
    C = max(1, args.clients_in_flight)

    def views(flat):
        out, off = [], 0
        for n in sizes:
            out.append(flat[off:off + n])
            off += n
        return out

    # pointer tables are marshalled once, as a training loop with persistent buffers would
    dW_sets = [sbc.TensorList(views(f)) for f in flat_sets]
    bound = (sbc.sbc_msg_bound_sampled if args.sampled_threshold else sbc.sbc_msg_bound)(sizes, P)
    scale = 1.0 / 32.0

    class Client:
        """One client of Alg. 1 with its server-side accumulator: residual, message buffer, context
        and stream of its own (the updates it compresses are shared, read-only)."""

        def __init__(self, index):
            self.R = sbc.TensorList(views(torch.zeros(N, dtype=torch.float32, device=dev)))
            self.out = sbc.TensorList(views(torch.zeros(N, dtype=torch.float32, device=dev)))
            # two message buffers, used in turn: a round's message is decoded while the next is written
            self.msgs = [sbc.MessageBuffer(torch.zeros(bound, dtype=torch.uint8, device=dev)) for _ in range(2)]
            self.msg = self.msgs[0]
            self.stream_obj = torch.cuda.current_stream() if index == 0 else torch.cuda.Stream()
            self.stream = self.stream_obj.cuda_stream     # raw handle, looked up once
            self.ctx = (sbc.sbc_create_compact if args.compact_context else sbc.sbc_create)(0, N, T)
            if args.no_carry_keys:
                sbc.sbc_set_option(self.ctx, sbc.SBC_OPT_CARRY_FILTER_KEYS, 0)
            if args.fused_step:
                sbc.sbc_set_option(self.ctx, sbc.SBC_OPT_FUSED_STEP, 1)
            if args.sampled_threshold:
                sbc.sbc_set_option(self.ctx, sbc.SBC_OPT_SAMPLED_THRESHOLD, 1)
            # the server calls only enqueue; their status is collected once, inside the timed region
            sbc.sbc_set_option(self.ctx, sbc.SBC_OPT_DEFER_DECODE_STATUS, 1)

    clients = [Client(i) for i in range(C)]
    ctx, R, out, msg, stream = clients[0].ctx, clients[0].R, clients[0].out, clients[0].msg, clients[0].stream

    def run_steps(clients, first, count, profile_every=0, routes=None, stamps=None):
        """Steps first .. first+count-1; step s is client s mod C's next round: the client call
        (begin ... end: the message size is needed on the host), then the server call on the
        produced message.  Every client has at most one step in flight.  With profile_every, every
        profile_every-th step of a client carries the events that time the streaming kernel."""
        C = len(clients)

        def begin(s):
            c = clients[s % C]
            if profile_every:
                sbc.sbc_profile_level(c.ctx, 1 if ((s - first) // C) % profile_every == 0 else 0)
            sbc.sbc_compress_begin(c.ctx, dW_sets[s % n_sets], c.R, P, c.msgs[(s // C) % 2], c.stream)

        total_bytes = 0
        for s in range(first, min(first + C, first + count)):
            begin(s)
        for s in range(first, first + count):
            c = clients[s % C]
            nbytes = sbc.sbc_compress_end(c.ctx)
            if stamps is not None:
                stamps.append(time.perf_counter())          # this step's message is complete
            total_bytes += nbytes
            if routes is not None:
                rt = sbc.sbc_last_route(c.ctx)
                routes[rt] = routes.get(rt, 0) + 1
            # the client's next round is enqueued first (it writes the other message buffer), then
            # the server call on this round's message: the GPU has work while the host comes back
            # from waiting for the next round's result
            if s + C < first + count:
                begin(s + C)
            sbc.sbc_decompress_accumulate(c.ctx, c.msgs[(s // C) % 2], nbytes, P, scale, c.out, c.stream)
        for c in clients:
            sbc.sbc_decode_status(c.ctx, c.stream)
        return total_bytes

    run_steps(clients, 0, max(args.warmup, C))
    torch.cuda.synchronize()

    # The streaming kernel's own duration is taken live, inside the timed region, from the
    # start/stop events of its dispatch on every PROFILE_EVERY-th step (events on a dispatch add a
    # few microseconds of idle time around it, so not every step carries them).
    routes = {}
    for c in clients:
        sbc.sbc_profile_enable(c.ctx, 0)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    stamps = []
    msg_bytes = run_steps(clients, args.warmup, args.steps, PROFILE_EVERY, routes, stamps)
    torch.cuda.synchronize()
    t1 = time.perf_counter()
    # single steps: the time from one step's finished message to the next one's
    periods_ms = [(b - a) * 1e3 for a, b in zip(stamps, stamps[1:])]
    prof = {}
    for c in clients:
        for kernel, ms, calls in sbc.sbc_profile_read(c.ctx):
            acc_ms, acc_calls = prof.get(kernel, (0.0, 0))
            prof[kernel] = (acc_ms + ms, acc_calls + calls)
    ms_per_step = (t1 - t0) * 1e3 / args.steps

    # untimed extra: latency of each call on its own (one client, every call waited for)
    sbc.sbc_set_option(ctx, sbc.SBC_OPT_DEFER_DECODE_STATUS, 0)
    sbc.sbc_profile_level(ctx, 0)
    compress_all, decode_all = [], []
    for i in range(args.steps):
        ta = time.perf_counter()
        nbytes = sbc.sbc_compress(ctx, dW_sets[i % n_sets], R, P, msg, stream)
        tb = time.perf_counter()
        sbc.sbc_decompress_accumulate(ctx, msg, nbytes, P, scale, out, stream)
        decode_all.append((time.perf_counter() - tb) * 1e3)
        compress_all.append((tb - ta) * 1e3)
    compress_ms = sum(compress_all) / args.steps
    decode_ms = sum(decode_all) / args.steps
    stream_kernel = sbc.sbc_profile_read(ctx)[1][0]       # the residual-accumulation kernel of this configuration
    k1_ms, k1_calls = prof[stream_kernel]
    if k1_calls == 0:
        print("bench.py: no timed launch of the streaming kernel", file=sys.stderr)
        return 1
    warm_us = k1_ms / k1_calls * 1e3

    # untimed extras: per-kernel breakdown, copy yardstick, paper-accounted compression ratio
    sbc.sbc_profile_enable(ctx, 2)
    for i in range(10):
        sbc.sbc_compress(ctx, dW_sets[i % n_sets], R, P, msg, stream)
    breakdown = {name: round(ms / max(1, calls) * 1e3, 2) for name, ms, calls in sbc.sbc_profile_read(ctx)}
    sbc.sbc_profile_enable(ctx, 0)
    # untimed extra: the kernels' durations with the caches flushed before every call (512 MiB,
    # twice the last-level cache, read in between; a write would leave the cache full of dirty
    # lines whose write-back the next kernel pays for), against the back-to-back figures above
    # where part of the residual may still be cached from the previous round
    cold = None
    if args.workload != "flat1p5e9":
        flush = torch.zeros(128 << 20, dtype=torch.int32, device=dev)
        sbc.sbc_profile_enable(ctx, 2)
        for i in range(COLD_LAUNCHES):
            flush.sum()
            torch.cuda.synchronize()
            sbc.sbc_compress(ctx, dW_sets[i % n_sets], R, P, msg, stream)
        cold_read = sbc.sbc_profile_read(ctx)
        cold_us = {kernel: round(ms / max(1, calls) * 1e3, 2) for kernel, ms, calls in cold_read}
        sbc.sbc_profile_enable(ctx, 0)
        cold_compress = []                                  # the call's latency, no events on its dispatches
        for i in range(COLD_LAUNCHES):
            flush.sum()
            torch.cuda.synchronize()
            ta = time.perf_counter()
            sbc.sbc_compress(ctx, dW_sets[i % n_sets], R, P, msg, stream)
            cold_compress.append((time.perf_counter() - ta) * 1e3)
        cold = {"kernel_us": cold_us, "launches": cold_read[1][2],
                "compress_ms_median": statistics.median(cold_compress), "compress_ms_min": min(cold_compress)}
        del flush
    # the headline kernel figure: caches flushed before the call where the call's footprint could
    # otherwise partly stay in the last-level cache; beyond it there is nothing to flush
    if cold is not None:
        k1_us, k1_launches, k1_how = cold["kernel_us"][stream_kernel], cold["launches"], "caches flushed before every call"
    else:
        # (no flush needed: the footprint is far beyond the last-level cache; the ten back-to-back calls
        # of the breakdown loop, which come after the first rounds' floods of candidates have settled)
        k1_us, k1_launches, k1_how = breakdown[stream_kernel], 10, "ten back-to-back calls after the timed steps (footprint far beyond the last-level cache)"
    achieved = BYTES_PER_ENTRY * N / (k1_us * 1e-6) / 1e9
    traffic, traffic_kernel, traffic_source = traffic_from_profile()
    if args.workload != "resnet50" or traffic_kernel is None or not stream_kernel.startswith(traffic_kernel):
        traffic, traffic_source = None, None
    ev0, ev1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    src, dst = flat_sets[0], (flat_sets[1] if n_sets > 1 else out.tensors[0])
    for _ in range(3):
        sbc.sbc_copy_baseline(dst, src)
    torch.cuda.synchronize()
    ev0.record()
    for _ in range(10):
        sbc.sbc_copy_baseline(dst, src)
    ev1.record()
    torch.cuda.synchronize()
    copy_gbs = 2 * 4 * N * 10 / (ev0.elapsed_time(ev1) * 1e-3) / 1e9
    stats = [sbc.sbc_last_tensor_stats(ctx, t) for t in range(T)]
    bits = sum(s[4] for s in stats)
    ratio = 32.0 * N / (bits + 32.0 * T)
    bit_accounting = accounting.message_bits(sizes, [s[3] for s in stats], [s[4] for s in stats])
    if args.breakdown:
        print("per-kernel us (event-bracketed):", breakdown, file=sys.stderr)

    # untimed extra: the server side of one round with 32 participating clients (Alg. 1, server:
    # decode every client's message and average): 32 decode calls back to back on messages of
    # this workload (the three resident updates compressed from a zero residual, used in turn), one
    # status check
    server32 = None
    if args.workload != "flat1p5e9":
        sbc.sbc_set_option(ctx, sbc.SBC_OPT_DEFER_DECODE_STATUS, 1)
        server_msgs = []
        for i in range(n_sets):
            buf = sbc.MessageBuffer(torch.zeros(bound, dtype=torch.uint8, device=dev))
            for r_t in R.tensors:
                r_t.zero_()
            server_msgs.append((buf, sbc.sbc_compress(ctx, dW_sets[i], R, P, buf, stream)))
        for rep_ in range(2):
            torch.cuda.synchronize()
            ts0 = time.perf_counter()
            for i in range(32):
                buf, nb = server_msgs[i % n_sets]
                sbc.sbc_decompress_accumulate(ctx, buf, nb, P, scale, out, stream)
            sbc.sbc_decode_status(ctx, stream)
            torch.cuda.synchronize()
            ts1 = time.perf_counter()
        server32 = {"clients": 32, "ms_total": (ts1 - ts0) * 1e3, "ms_per_message": (ts1 - ts0) * 1e3 / 32}
        sbc.sbc_set_option(ctx, sbc.SBC_OPT_DEFER_DECODE_STATUS, 0)

    # untimed extra: the same steps with three independent clients in flight, whose latency-bound
    # kernels and host round trips overlap one another's streaming pass
    pipelined = None
    if C == 1 and args.workload != "flat1p5e9" and not args.no_pipelined_extra:
        sbc.sbc_set_option(ctx, sbc.SBC_OPT_DEFER_DECODE_STATUS, 1)
        three = clients + [Client(1), Client(2)]
        run_steps(three, 0, 9)
        torch.cuda.synchronize()
        tp0 = time.perf_counter()
        run_steps(three, 9, args.steps)
        torch.cuda.synchronize()
        tp = (time.perf_counter() - tp0) / args.steps
        pipelined = {"clients_in_flight": 3, "ms_per_step": tp * 1e3, "elements_per_s": N / tp,
                     "streaming_bytes_frac_of_hbm_peak": BYTES_PER_ENTRY * N / tp / 1e9 / HBM_PEAK_GBS}
        for c in three[1:]:
            sbc.sbc_destroy(c.ctx)

    for c in clients:
        sbc.sbc_destroy(c.ctx)
    torch.cuda.synchronize()

    # untimed extra: Alg. 1's round loop with everything resident in device memory: four clients
    # (each: its update written into its buffer, sbc_compress), the server's four decodes into the
    # average, W <- W + dW; per round, with a device synchronisation after each
    round_loop = None
    if C == 1 and args.workload == "resnet50" and not args.no_pipelined_extra:
        from paper_1805_08768_amd import rounds as rounds_mod
        n_cl = 4
        ups = []
        for i in range(n_cl):
            flat, views = rounds_mod.flat_buffer(sizes, dev)
            for v, x in zip(views, gen(100 + i)):
                v.copy_(torch.from_numpy(x))
            ups.append(flat)

        def on_device_update(client, rnd, W, out_views):
            out_views.flat.copy_(ups[(client + rnd) % n_cl])

        stamps = []

        def stamp(rnd):
            torch.cuda.synchronize()
            stamps.append(time.perf_counter())

        rounds_mod.run_rounds(sizes, P, n_cl, 24, on_device_update, device=dev, on_device=True, on_round_end=stamp)
        per_round = sorted(b_ - a_ for a_, b_ in zip(stamps[3:-1], stamps[4:]))      # (the first rounds: warm-up)
        round_loop = {"clients": n_cl, "ms_per_round_median": per_round[len(per_round) // 2] * 1e3,
                      "ms_per_round_min": per_round[0] * 1e3, "rounds": len(per_round),
                      "what": "update copied into each client's buffer, 4 x sbc_compress, 4 x sbc_decompress_accumulate, W += average; all in device memory"}
        del ups
    torch.cuda.synchronize()

    # the GPU part is over: the waiting CPU processes get their work
    cpu = None
    if cpu_pool is not None:
        cpu = cpu_pool.run([gen(r) for r in range(CPU_ROUNDS)], sizes, P, scale)
        cpu_pool.close()

    def frac_of_peak(ms):
        return BYTES_PER_ENTRY * N / (ms * 1e-3) / 1e9 / HBM_PEAK_GBS

    line = {
        "metric": "SBC compress+encode throughput (elements/s, HBM GB/s, % of peak) per round",
        "value": N / (ms_per_step * 1e-3),
        "unit": "elements/s",
        "n_gpus": 1,
        "steps": args.steps,
        "warmup": args.warmup,
        "ms_per_step": ms_per_step,
        "ms_per_step_median": statistics.median(periods_ms) if periods_ms else ms_per_step,
        "ms_per_step_min": min(periods_ms) if periods_ms else ms_per_step,
        "higher_is_better": True,
        "scaling": "weak",
        "vs_baseline": None,
        "dtype": "f32",
        "data": "synthetic",
        "config": {"workload": name, "p": P, "tensors": T, "entries": N,
                   "step": "sbc_compress (begin/end) + sbc_decompress_accumulate (one client, one round); the "
                           "decode status is collected once for all steps (SBC_OPT_DEFER_DECODE_STATUS)",
                   "clients_in_flight": C,
                   "selection": "subsampled threshold (noisy count)" if args.sampled_threshold else "exact top-k"},
        "roofline": {"bound": "hbm", "achieved": achieved, "peak": HBM_PEAK_GBS, "unit": "GB/s",
                     "frac": achieved / HBM_PEAK_GBS,
                     "traffic": traffic, "traffic_source": traffic_source,
                     "kernel": stream_kernel, "kernel_avg_us": k1_us,
                     "kernel_launches_timed": k1_launches, "kernel_timed": k1_how,
                     "algorithmic_bytes_per_launch": BYTES_PER_ENTRY * N,
                     "timed_region": {"kernel_avg_us": warm_us, "kernel_launches_timed": k1_calls,
                                      "frac": BYTES_PER_ENTRY * N / (warm_us * 1e-6) / 1e9 / HBM_PEAK_GBS},
                     # the same bytes over the whole compress call (every kernel of it and the wait for its result)
                     "step_frac": frac_of_peak(compress_ms),
                     "step_frac_median": frac_of_peak(statistics.median(compress_all)),
                     "step_frac_best": frac_of_peak(min(compress_all)),
                     "step_frac_caches_flushed": frac_of_peak(cold["compress_ms_median"]) if cold else None},
        "cpu_baseline": cpu,
        "compress_ms": compress_ms,
        "compress_ms_median": statistics.median(compress_all),
        "compress_ms_min": min(compress_all),
        "decode_ms": decode_ms,
        "decode_ms_median": statistics.median(decode_all),
        "decode_ms_min": min(decode_all),
        "compress_elements_per_s": N / (compress_ms * 1e-3),
        "compress_algorithmic_GBs": BYTES_PER_ENTRY * N / (compress_ms * 1e-3) / 1e9,
        "compress_frac_of_hbm_peak": frac_of_peak(compress_ms),
        "kernel_us": breakdown,
        "cold_cache": cold,
        "pipelined": pipelined,
        "server_average_32": server32,
        "round_loop": round_loop,
        "copy_kernel_GBs": copy_gbs,
        "message_bytes": msg_bytes / args.steps,
        "routes": {"sampled": sum(v for k, v in routes.items() if not k & 1),
                   "carried_keys": sum(v for k, v in routes.items() if k & 1),
                   "histogram_fallback": sum(v for k, v in routes.items() if k & 2),
                   "grid_wide_selection": sum(v for k, v in routes.items() if k & 4)},
        "compression_ratio_paper_accounting": ratio,
        "bit_accounting": {k: round(v, 3) for k, v in bit_accounting.items() if k.startswith("gain_")
                           or k == "position_bits_per_kept_entry"},
    }
    print(json.dumps(line))
    return 0


if __name__ == "__main__":
    sys.exit(main())
