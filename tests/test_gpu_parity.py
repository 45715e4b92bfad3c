"""Parity of the HIP path (through the C ABI) with the CPU oracle on the same seeded inputs.

Bit exact: mask, gap list / bitstream, message bytes, side, nnz, bit length, decoded dense
update.  Within 1e-5 relative of the fp64 oracle: mu+, mu-, residual at kept positions."""
import numpy as np
import pytest
import torch

from oracle import sbc_oracle as o
from paper_1805_08768_amd import binding as sbc, synth
import parity_util
from parity_util import DeviceRun, check_round, mask_to_positions

pytestmark = pytest.mark.gpu

# tests that only run with the default setting of SBC_OPT_FUSED_STEP (the largest inputs, and calls
# that create their contexts themselves)
DEFAULT_ONLY = ("test_config5b", "test_compact_context", "test_config5a", "test_more_wide_tensors", "test_tensor_of_several_scan_tiles", "test_config2_companion", "test_tensor_of_many_chunks", "test_unaligned_views",
                "test_inspection_requires", "test_same_input_twice")


@pytest.fixture(autouse=True, params=[0, 1], ids=["plain", "fused"])
def fused_step(request):
    """Every test runs with the streaming kernel leaving all tensors to the selection kernel, and
    with the streaming kernel finishing the tensors it can by itself."""
    if request.param and request.node.name.startswith(DEFAULT_ONLY):
        pytest.skip("runs with the default setting only")
    parity_util.FUSED_STEP = request.param
    yield request.param
    parity_util.FUSED_STEP = 0


def main_route(ctx):
    """Which of the three candidate routes the latest call took (without the advisory bits)."""
    return sbc.sbc_last_route(ctx) & (sbc.SBC_ROUTE_CARRIED_KEYS | sbc.SBC_ROUTE_HISTOGRAM | sbc.SBC_ROUTE_WIDE)


def run_rounds(sizes, gen, p, rounds=1, check_decode=True):
    with DeviceRun(sizes) as run:
        R = [np.zeros(n, np.float32) for n in sizes]
        for r in range(rounds):
            print("round", r, "sizes", sizes[:4], "p", p, flush=True)
            res = check_round(run, gen(r), R, p, check_decode=check_decode)
            R = [x.R_new for x in res]
        return res


# ---------------------------------------------------------------- small, ragged ----

@pytest.mark.parametrize("p", [0.1, 0.01, 0.001])
def test_small_ragged_model(p):
    sizes = [64, 1000, 8192, 8193, 20000, 5, 1, 16384, 40001]
    run_rounds(sizes, lambda r: synth.small_model_update(sizes, round_=r), p, rounds=2)


def test_unaligned_views():
    """Tensors that are slices of one flat buffer at odd offsets (only 4-byte aligned)."""
    sizes = [8192 * 2 + 3, 777, 8192]
    p = 0.01
    dWs = synth.small_model_update(sizes, round_=3)
    results = o.compress_model(dWs, [np.zeros_like(d) for d in dWs], p)
    flat_dw = torch.zeros(sum(sizes) + 16, dtype=torch.float32, device="cuda:0")
    flat_r = torch.zeros(sum(sizes) + 16, dtype=torch.float32, device="cuda:0")
    views_dw, views_r, off = [], [], 1
    for d in dWs:
        views_dw.append(flat_dw[off:off + len(d)]); views_dw[-1].copy_(torch.from_numpy(d))
        views_r.append(flat_r[off:off + len(d)])
        off += len(d) + 1
    ctx = sbc.sbc_create(0, sum(sizes), len(sizes))
    try:
        msg = torch.zeros(sbc.sbc_msg_bound(sizes, p), dtype=torch.uint8, device="cuda:0")
        nbytes = sbc.sbc_compress(ctx, views_dw, views_r, p, msg)
        assert msg[:nbytes].cpu().numpy().tobytes() == o.build_message(results)
        for v, res in zip(views_r, results):
            assert np.allclose(v.cpu().numpy(), res.R_new, rtol=0, atol=1e-5 * abs(float(res.mu_signed)))
    finally:
        sbc.sbc_destroy(ctx)


# ------------------------------------------------------------- degenerate inputs ----

def test_degenerate_tensors():
    sym = (np.array([3, -3, 2, -2, 1, -1, 0, 0] * 100, dtype=np.float32) * 2.0 ** -10)
    szero = np.zeros(300, np.float32); szero[::2] = -0.0; szero[7] = 1e-30
    onehot = np.zeros(10000, np.float32); onehot[9999] = -2.0
    cases = [
        ("zeros", [np.zeros(5000, np.float32), np.zeros(64, np.float32)], 0.01),
        ("constant", [np.full(9000, -0.25, np.float32)], 0.05),
        ("all negative", [-np.abs(synth.gaussian_update(9000))], 0.01),
        ("symmetric, equal means", [sym], 0.25),
        ("signed zeros and a denormal-scale entry", [szero], 0.05),
        ("one hot at the end", [onehot], 0.001),
        ("keep everything but one", [synth.gaussian_update(50)], 0.99),
        ("single element", [np.array([-3.5], np.float32)], 0.5),
        ("denormals", [(synth.gaussian_update(4000) * 1e-36).astype(np.float32)], 0.01),
        ("huge values", [(synth.gaussian_update(4000) * 1e36).astype(np.float32)], 0.01),
    ]
    for name, dWs, p in cases:
        print("case", name, flush=True)
        sizes = [len(d) for d in dWs]
        run_rounds(sizes, lambda r: dWs, p, rounds=2)


def test_palette_ties_three_rounds():
    sizes = [300000, 777]
    run_rounds(sizes, lambda r: [synth.palette_update(n, round_=r, tensor=i) for i, n in enumerate(sizes)],
               0.01, rounds=3)


def test_long_unary_runs():
    """Kept entries clustered at the far end: the first gap needs a long run of ones."""
    n = 3_000_000
    x = np.zeros(n, np.float32)
    x[-40:] = np.linspace(1, 2, 40, dtype=np.float32)
    x[5] = -0.5
    run_rounds([n], lambda r: [x], 1e-5)      # k = 30, b* = 16


# ------------------------------------------- candidate search: both routes, all list sizes ----

def test_histogram_path_forced():
    """SBC_OPT_FORCE_EXACT_PATH sends every tensor through the histogram route; results must
    be the same as with the sampled filter."""
    sizes = [64, 1000, 8193, 40001, 300000, 5]
    for p in (0.1, 0.001):
        with DeviceRun(sizes) as run:
            sbc.sbc_set_option(run.ctx, sbc.SBC_OPT_FORCE_EXACT_PATH, 1)
            R = [np.zeros(n, np.float32) for n in sizes]
            for r in range(2):
                res = check_round(run, synth.small_model_update(sizes, round_=r), R, p)
                assert main_route(run.ctx) == sbc.SBC_ROUTE_HISTOGRAM
                R = [x.R_new for x in res]
    dWs = [synth.palette_update(200000), np.zeros(70000, np.float32)]
    with DeviceRun([200000, 70000]) as run:
        sbc.sbc_set_option(run.ctx, sbc.SBC_OPT_FORCE_EXACT_PATH, 1)
        check_round(run, dWs, [np.zeros_like(d) for d in dWs], 0.01)


def _mix32(x):
    x &= 0xFFFFFFFF
    x ^= x >> 16; x = (x * 0x7FEB352D) & 0xFFFFFFFF
    x ^= x >> 15; x = (x * 0x846CA68B) & 0xFFFFFFFF
    x ^= x >> 16
    return x


def sampled_positions(n, tensor):
    """Positions the threshold sampler reads for a tensor of more than 16384 entries: 256 runs of
    64 entries, one per stratum (mirrors k_sample_thresholds; the test below checks that the
    histogram route really ran, so a change of the layout shows)."""
    slots = n // 64
    pos = []
    for run in range(256):
        h = _mix32(run * 0x9E3779B9 + tensor * 0x85EBCA6B + 1)
        lo, hi = run * slots // 256, (run + 1) * slots // 256
        first = (lo + ((h * (hi - lo)) >> 32)) * 64
        pos.extend(range(first, first + 64))
    return np.array(pos)


def test_misleading_sample_falls_back_per_tensor():
    """Tensor 1 carries its few large entries exactly where the sampler looks, so the sampled
    threshold lands above the true k-th entry and the filter keeps too few candidates; the
    histogram route must redo that tensor only, and the message must still equal the oracle's."""
    sizes = [50000, 400000, 3000]
    dWs = synth.small_model_update(sizes, round_=4)
    x = (np.abs(dWs[1]) * 1e-3).astype(np.float32)           # small noise everywhere
    pos = sampled_positions(sizes[1], 1)
    x[pos[::200]] = 5.0                                      # 82 large entries, all of them sampled
    x[pos[1::200]] = -7.0
    dWs[1] = x
    with DeviceRun(sizes) as run:
        R = [np.zeros(n, np.float32) for n in sizes]
        res = check_round(run, dWs, R, 0.001)                # k = 400 for tensor 1
        assert main_route(run.ctx) == sbc.SBC_ROUTE_HISTOGRAM, "the sample was meant to mislead the filter"
        # after a fallback the next round samples again; the residual still holds the planted
        # entries, so it falls back again
        check_round(run, synth.small_model_update(sizes, round_=5), [r.R_new for r in res], 0.001)
        assert main_route(run.ctx) == sbc.SBC_ROUTE_HISTOGRAM
    with DeviceRun(sizes) as run:                            # ordinary data: the fast route alone
        check_round(run, synth.small_model_update(sizes, round_=5), [np.zeros(n, np.float32) for n in sizes], 0.001)
        assert main_route(run.ctx) == 0


def test_carried_filter_keys():
    """From the second round on the filter keys come from the previous round's exact thresholds.
    Results stay exact when the data scale drifts, jumps up (keys far too low: a flood of
    candidates, after which rounds sample until their samples say that carried keys would hold
    again) or collapses (keys far too high: the histogram route takes over)."""
    sizes = [300000, 64, 20000, 8193]
    routes = []
    with DeviceRun(sizes) as run:                            # (the option is set by default)
        R = [np.zeros(n, np.float32) for n in sizes]

        def one_round(r, sc, clear=False):
            nonlocal R
            if clear:                                        # the client starts over: residual cleared
                R = [np.zeros(n, np.float32) for n in sizes]
                for x in run.R:
                    x.zero_()
            dWs = [(d * np.float32(sc)).astype(np.float32) for d in synth.small_model_update(sizes, round_=r)]
            res = check_round(run, dWs, R, 0.001, check_decode=(r % 4 == 0))
            routes.append(main_route(run.ctx))
            R = [x.R_new for x in res]

        for r, sc in enumerate([1.0, 1.05, 0.9, 1.2, 40.0, 40.0]):
            one_round(r, sc)
        assert routes[0] == 0                                # first round samples
        assert routes[1] == sbc.SBC_ROUTE_CARRIED_KEYS and routes[2] == sbc.SBC_ROUTE_CARRIED_KEYS
        assert routes[4] & sbc.SBC_ROUTE_CARRIED_KEYS        # the jump: carried keys, a flood of candidates
        assert routes[5] == 0                                # ... which made round 5 sample again
        r = 6
        while not routes[-1] & sbc.SBC_ROUTE_CARRIED_KEYS:   # sampling goes on while the residual still grows fast
            assert r < 16
            one_round(r, 40.0)
            r += 1
        one_round(r, 0.01, clear=True)                       # the collapse forces the exact route
        assert routes[-1] & sbc.SBC_ROUTE_CARRIED_KEYS and routes[-1] & sbc.SBC_ROUTE_HISTOGRAM
        one_round(r + 1, 0.01)
        one_round(r + 2, 1.0)
    print("routes", routes)
    with DeviceRun(sizes) as run:                            # option cleared: every round samples
        sbc.sbc_set_option(run.ctx, sbc.SBC_OPT_CARRY_FILTER_KEYS, 0)
        R = [np.zeros(n, np.float32) for n in sizes]
        for r in range(3):
            res = check_round(run, synth.small_model_update(sizes, round_=r), R, 0.001, check_decode=False)
            assert main_route(run.ctx) == 0
            R = [x.R_new for x in res]


def test_candidate_lists_beyond_the_register_cache():
    """Mostly-constant data: the filter cannot separate ties, so the lists hold tens of thousands
    of candidates (streamed instead of cached) and ties decide the mask."""
    x = np.zeros(500000, np.float32); x[::7] = 1e-3; x[3::11] = -2e-3
    y = np.full(100000, 0.125, np.float32)
    run_rounds([500000, 100000], lambda r: [x, y], 0.01, rounds=2)


# ------------------------------------------------------------------- the configs ----

def test_config1_gaussian_2p20():
    n = 1 << 20
    res = run_rounds([n], lambda r: [synth.gaussian_update(n)], 0.01)
    assert res[0].k == 10485 and res[0].bstar == 6


def test_config2_student_t_ten_rounds_with_duplicates():
    n = 4_194_304
    with DeviceRun([n]) as run:
        R = [np.zeros(n, np.float32)]
        sum_dW = np.zeros(n, np.float64)
        sum_star = np.zeros(n, np.float64)
        for r in range(10):
            print("config 2 round", r, flush=True)
            dW = synth.student_t_update(n, round_=r)
            res = check_round(run, [dW], R, 0.001, check_decode=(r in (0, 9)))
            assert res[0].k == 4194
            sum_dW += dW
            sum_star += res[0].dense_update()
            R = [res[0].R_new]
        # Eq. 2 telescoped over the ten rounds, on the device's residual
        R_dev = run.R[0].cpu().numpy().astype(np.float64)
        scale = max(np.abs(sum_dW).max(), np.abs(R_dev).max())
        assert np.abs(sum_dW - sum_star - R_dev).max() <= 10 * 2.0 ** -23 * scale


def test_config2_companion_palette_full_size():
    n = 4_194_304
    run_rounds([n], lambda r: [synth.palette_update(n, round_=r)], 0.001, rounds=3, check_decode=False)


def test_config3_resnet50_two_rounds():
    sizes = synth.numels(synth.resnet50_shapes())
    res = run_rounds(sizes, lambda r: synth.resnet50_update(round_=r), 0.001, rounds=2)
    assert sum(x.k for x in res) == 25595


def test_config4_lstm_two_rounds():
    sizes = synth.numels(synth.lstm_lm_shapes())
    res = run_rounds(sizes, lambda r: synth.lstm_lm_update(round_=r), 1e-4, rounds=2)
    assert sum(x.k for x in res) == 6603 and res[0].bstar == 13


def test_config5a_server_average_of_32_clients():
    """Decode-and-average of 32 clients' messages for the ResNet-50-shaped model (Alg. 1, server
    lines).  All 32 messages are compressed on the GPU from independent seeds.  The oracle
    compresses 4 of them at full size (32 would take a quarter of an hour on the host) and
    those messages are compared byte for byte; every one of the 32 GPU messages then goes through
    the oracle's decoder, and the dense average must equal the GPU's exactly.  Positions that
    several clients send exist, so the accumulation really adds."""
    sizes = synth.numels(synth.resnet50_shapes())
    clients, oracle_checked, scale, p = 32, 4, 1.0 / 32, 0.001
    want = [np.zeros(n, np.float32) for n in sizes]
    hits = [np.zeros(n, np.uint8) for n in sizes]
    outs = [torch.zeros(n, dtype=torch.float32, device="cuda:0") for n in sizes]
    with DeviceRun(sizes) as run:
        for c in range(clients):
            print("client", c, flush=True)
            dWs = synth.resnet50_update(client=c + 1)
            for r in run.R:
                r.zero_()
            msg, nbytes = run.compress(dWs, p)
            got_msg = msg[:nbytes].cpu().numpy().tobytes()
            if c < oracle_checked:
                results = o.compress_model(dWs, [np.zeros_like(d) for d in dWs], p)
                assert got_msg == o.build_message(results)
            sbc.sbc_decompress_accumulate(run.ctx, msg, nbytes, p, scale, outs)
            o.decode_accumulate(got_msg, sizes, scale, want)
            one = [np.zeros(n, np.float32) for n in sizes]
            o.decode_accumulate(got_msg, sizes, 1.0, one)
            for t in range(len(sizes)):
                hits[t] += (one[t] != 0).astype(np.uint8)
    assert sum(int((h >= 2).sum()) for h in hits) > 0, "no position was sent by two clients"
    assert sum(int(h.sum()) for h in hits) == clients * 25595
    for t in range(len(sizes)):
        assert np.array_equal(outs[t].cpu().numpy(), want[t]), t


def test_config5b_flat_1p5e9_properties():
    """One flat tensor of 1.5e9 entries, p = 0.001 (k = 1.5e6, b* = 9).  A full sort on the host is
    out of reach, so the result is checked by what defines it, with no sort: exactly k kept
    entries, every kept entry at least as extreme as every dropped one with equal values resolved
    to the lowest indices, mu = mean of the kept values, residual identity, the closed-form bit
    length of the Golomb stream, the oracle's bit-serial decoder on the first codes, and the
    library's decoder on the whole stream."""
    n, p = 1_500_000_000, 0.001
    free, total = torch.cuda.mem_get_info()
    if free < 60 * 2 ** 30:
        pytest.skip("needs about 60 GiB of free device memory")
    k = o.num_kept(n, p)
    b = o.golomb_bstar(p)
    dW = torch.empty(n, dtype=torch.float32, device="cuda:0")
    host = np.empty(n, dtype=np.float32)
    for off, chunk in synth.flat_gaussian_chunks(n):
        host[off:off + len(chunk)] = chunk
        dW[off:off + len(chunk)].copy_(torch.from_numpy(chunk))
    print("generated", flush=True)
    R = torch.zeros(n, dtype=torch.float32, device="cuda:0")
    ctx = sbc.sbc_create_compact(0, n, 1)                    # 5 bytes of scratch per entry instead of 17
    try:
        bound = sbc.sbc_msg_bound([n], p)
        msg = torch.zeros(bound, dtype=torch.uint8, device="cuda:0")
        nbytes = sbc.sbc_compress(ctx, [dW], [R], p, msg)
        print("compressed", nbytes, flush=True)
        mu_pos, mu_neg, side, nnz, bit_len = sbc.sbc_last_tensor_stats(ctx, 0)
        assert nnz == k
        kept = mask_to_positions(sbc.sbc_last_mask(ctx, 0, n), n)
        assert len(kept) == k
        A = host                                              # zero residual: A = dW
        vals = A[kept].astype(np.float64) * side
        mask = np.zeros(n, dtype=bool); mask[kept] = True
        dropped_max = (A[~mask] * np.float32(side)).max()
        assert vals.min() >= dropped_max                      # kept entries are the k most extreme of the side
        if vals.min() == dropped_max:                         # ties at the threshold: lowest indices win
            tied = np.flatnonzero(A * np.float32(side) == np.float32(dropped_max))
            assert mask[tied[: int(mask[tied].sum())]].all()
        mu = mu_pos if side > 0 else mu_neg
        assert abs(mu - vals.mean()) <= 1e-5 * abs(vals.mean())
        other = np.partition(A * np.float32(-side), n - k)[n - k:].astype(np.float64).mean()
        assert abs((mu_neg if side > 0 else mu_pos) - other) <= 1e-5 * abs(other) and mu >= other
        header = msg[:56].cpu().numpy().tobytes()
        import struct
        mu_signed, nnz_m, bl_m, woff = struct.unpack_from("<fIQQ", header, 32)
        assert nnz_m == k and woff == 0 and np.float32(mu_signed) == np.float32(side * mu)
        # residual
        Rh = R.cpu().numpy()
        assert np.array_equal(Rh[~mask], A[~mask])
        assert np.allclose(Rh[kept], A[kept] - np.float32(mu_signed), rtol=0, atol=1e-5 * abs(mu))
        # code lengths in closed form
        gaps = np.diff(np.concatenate(([-1], kept))) - 1
        assert bl_m == bit_len == int(((gaps >> b) + 1 + b).sum())
        assert nbytes == 32 + 24 + 4 * ((bl_m + 31) // 32)
        # the oracle's decoder on the first 20000 codes
        first_bits = int(((gaps[:20000] >> b) + 1 + b).sum())
        words = msg[56:56 + 4 * ((first_bits + 31) // 32)].cpu().numpy().view("<u4")
        assert o.golomb_decode(o.unpack_bits(words, first_bits), b) == kept[:20000].tolist()
        # the library's decoder on the whole stream
        del dW
        out = torch.zeros(n, dtype=torch.float32, device="cuda:0")
        sbc.sbc_decompress_accumulate(ctx, msg, nbytes, p, 1.0, [out])
        nz = torch.nonzero(out).flatten().cpu().numpy()
        assert np.array_equal(nz, kept) and bool((out[torch.from_numpy(kept).cuda()] == mu_signed).all())
    finally:
        sbc.sbc_destroy(ctx)


# ------------------------------------------------------- determinism and errors ----

def test_same_input_twice_gives_identical_bytes():
    sizes = [1 << 18, 5000, 64]
    dWs = synth.small_model_update(sizes, round_=9)
    outs = []
    for _ in range(3):
        with DeviceRun(sizes) as run:
            msg, nbytes = run.compress(dWs, 0.01)
            outs.append((msg[:nbytes].cpu().numpy().tobytes(), [r.cpu().numpy().tobytes() for r in run.R]))
    assert outs[0] == outs[1] == outs[2]


@pytest.mark.parametrize("tiled_decode", [False, True])
def test_error_paths(tiled_decode):
    sizes = [5000, 64]
    dWs = synth.small_model_update(sizes)
    with DeviceRun(sizes) as run:
        if tiled_decode:       # tensor 0 goes through the grid-wide selection and the tile decoder
            sbc.sbc_set_option(run.ctx, sbc.SBC_OPT_WIDE_MIN_KEPT, 10)
        d_dW = [torch.from_numpy(x).cuda() for x in dWs]
        bound = sbc.sbc_msg_bound(sizes, 0.01)
        msg = torch.zeros(bound, dtype=torch.uint8, device="cuda:0")

        def code(fn):
            with pytest.raises(sbc.SbcError) as e:
                fn()
            return e.value.code

        assert code(lambda: sbc.sbc_compress(run.ctx, d_dW, run.R, 0.0, msg)) == sbc.SBC_EINVAL
        assert code(lambda: sbc.sbc_compress(run.ctx, d_dW, run.R, 1.0, msg)) == sbc.SBC_EINVAL
        assert code(lambda: sbc.sbc_compress(run.ctx, d_dW, run.R, 0.01, msg[: bound - 8])) == sbc.SBC_ECAPACITY
        assert code(lambda: sbc.sbc_compress(run.ctx, d_dW, run.R, 0.01, msg[1:])) == sbc.SBC_EINVAL   # misaligned
        assert code(lambda: sbc.sbc_compress(run.ctx, d_dW, d_dW, 0.01, msg)) == sbc.SBC_EINVAL        # aliasing
        big = [torch.zeros(6000, device="cuda:0"), torch.zeros(64, device="cuda:0")]
        assert code(lambda: sbc.sbc_compress(run.ctx, big, [torch.zeros_like(b) for b in big], 0.01,
                                             torch.zeros(10000, dtype=torch.uint8, device="cuda:0"))) == sbc.SBC_ECAPACITY
        three = d_dW + [d_dW[0].clone()]
        assert code(lambda: sbc.sbc_compress(run.ctx, three, [torch.zeros_like(b) for b in three], 0.01,
                                             msg)) == sbc.SBC_ECAPACITY
        # non-finite accumulated entry
        bad = [d_dW[0].clone(), d_dW[1].clone()]
        bad[0][123] = float("inf")
        assert code(lambda: sbc.sbc_compress(run.ctx, bad, [torch.zeros_like(b) for b in bad], 0.01, msg)) == sbc.SBC_ENONFINITE

        # a good message, then corrupted variants: never a write out of bounds, always an error
        for r in run.R:
            r.zero_()
        nbytes = sbc.sbc_compress(run.ctx, d_dW, run.R, 0.01, msg)
        good = msg[:nbytes].clone()

        def decode(m, nb=None, p=0.01, szs=sizes):
            guard = [torch.zeros(n + 64, dtype=torch.float32, device="cuda:0") for n in szs]
            outs = [g[32:32 + n] for g, n in zip(guard, szs)]
            try:
                sbc.sbc_decompress_accumulate(run.ctx, m, len(m) if nb is None else nb, p, 1.0, outs)
                rc = 0
            except sbc.SbcError as e:
                rc = e.code
            for g, n in zip(guard, szs):
                assert not g[:32].any() and not g[32 + n:].any(), "decode wrote out of bounds"
            return rc

        assert decode(good) == 0
        assert decode(good, nb=nbytes - 4) == sbc.SBC_ECORRUPT                  # truncated
        assert decode(good, p=0.001) == sbc.SBC_ECORRUPT                       # b* mismatch
        assert decode(good, szs=[5000]) == sbc.SBC_ECORRUPT                    # tensor count mismatch
        assert decode(good, szs=[100, 64]) == sbc.SBC_ECORRUPT                 # positions beyond numel
        m = good.clone(); m[0] = 0
        assert decode(m) == sbc.SBC_ECORRUPT                                   # magic
        m = good.clone(); m[32 + 4] += 1
        assert decode(m) == sbc.SBC_ECORRUPT                                   # nnz off by one
        m = good.clone(); m[32 + 8] += 5
        assert decode(m) == sbc.SBC_ECORRUPT                                   # bit_len too long
        m = good.clone(); m[32 + 24 * 2: 32 + 24 * 2 + 8] = 0xFF
        assert decode(m) == sbc.SBC_ECORRUPT                                   # unary run to the end


def test_inspection_requires_a_successful_compress():
    ctx = sbc.sbc_create(0, 1000, 1)
    try:
        with pytest.raises(sbc.SbcError):
            sbc.sbc_last_tensor_stats(ctx, 0)
        with pytest.raises(sbc.SbcError):
            sbc.sbc_last_mask(ctx, 0, 100)
    finally:
        sbc.sbc_destroy(ctx)


def test_alternating_buffer_sets():
    """A caller that cycles through more sets of update buffers than the library keeps tensor
    tables for (hits, misses and evictions of the table cache), one residual throughout."""
    sizes = [5000, 64, 20000, 8193]
    p = 0.01
    n_sets = 6
    host = [synth.small_model_update(sizes, round_=s) for s in range(n_sets)]
    order = [0, 1, 0, 1, 2, 3, 4, 5, 0, 5, 5, 1]
    with DeviceRun(sizes) as run:
        dev = [[torch.from_numpy(x).to(run.device) for x in h] for h in host]
        lists = [sbc.TensorList(d) for d in dev]
        R_list = sbc.TensorList(run.R)
        bound = sbc.sbc_msg_bound(sizes, p)
        msg = torch.zeros(bound, dtype=torch.uint8, device=run.device)
        R = [np.zeros(n, np.float32) for n in sizes]
        for s in order:
            want = o.compress_model(host[s], R, p)
            nbytes = sbc.sbc_compress(run.ctx, lists[s], R_list, p, msg)
            assert bytes(msg[:nbytes].cpu().numpy().tobytes()) == o.build_message(want), "set %d" % s
            R = [w.R_new for w in want]
            for t, w in enumerate(want):
                assert np.array_equal(run.R[t].cpu().numpy(), w.R_new.astype(np.float32)), (s, t)


def _planted_threshold_ties(n, k, seed_tensor):
    """Gaussian values with 40 more copies of the k-th largest and of the k-th smallest value at
    random places, so that both thresholds fall inside a group of equal values."""
    x = synth.gaussian_update(n, tensor=seed_tensor)
    g = synth.rng_for(8, 0, 0, seed_tensor)
    order = np.argsort(-x, kind="stable")
    hi, lo = x[order[k - 1]], x[order[n - k]]
    mid = order[2 * k: n - 2 * k]
    where = g.choice(mid, size=80, replace=False)
    x[where[:40]] = hi
    x[where[40:]] = lo
    return x


def test_grid_wide_selection():
    """Tensors that keep many entries take the grid-wide selection kernels (threshold lowered by
    option so that the oracle finishes in seconds): plain data, thresholds inside groups of
    equal values, and tie-heavy data that those kernels hand back to the one-workgroup kernel."""
    sizes = [100000, 300, 65536, 9000]
    p = 0.1
    for carry in (0, 1):
        with DeviceRun(sizes) as run:
            sbc.sbc_set_option(run.ctx, sbc.SBC_OPT_WIDE_MIN_KEPT, 6500)
            sbc.sbc_set_option(run.ctx, sbc.SBC_OPT_CARRY_FILTER_KEYS, carry)
            R = [np.zeros(n, np.float32) for n in sizes]
            for r in range(3):
                dWs = [synth.gaussian_update(n, round_=r, tensor=i) for i, n in enumerate(sizes)]
                res = check_round(run, dWs, R, p)
                # (with keys carried over from a round whose thresholds were much lower, the k-th entry
                # may lie beyond the window those kernels count in: they then hand the tensor back)
                assert carry and r > 0 or sbc.sbc_last_route(run.ctx) & sbc.SBC_ROUTE_WIDE
                R = [x.R_new for x in res]
    sizes = [200000, 80000]
    with DeviceRun(sizes) as run:
        sbc.sbc_set_option(run.ctx, sbc.SBC_OPT_WIDE_MIN_KEPT, 6500)
        dWs = [_planted_threshold_ties(n, int(p * n), i) for i, n in enumerate(sizes)]
        check_round(run, dWs, [np.zeros(n, np.float32) for n in sizes], p)
        assert sbc.sbc_last_route(run.ctx) & sbc.SBC_ROUTE_WIDE
    with DeviceRun(sizes) as run:
        sbc.sbc_set_option(run.ctx, sbc.SBC_OPT_WIDE_MIN_KEPT, 6500)
        dWs = [synth.palette_update(n, tensor=i) for i, n in enumerate(sizes)]
        check_round(run, dWs, [np.zeros(n, np.float32) for n in sizes], p)


def test_grid_wide_selection_four_rounds_at_the_default_threshold():
    """The 2^20-entry Gaussian tensor of configuration 1 (10485 kept entries: grid-wide kernels at
    the default threshold) over four rounds with the residual carried, alone (no other selection
    kernel runs in the call) and with a small tensor beside it."""
    p = 0.01
    for sizes in ([1 << 20], [1 << 20, 5000]):
        with DeviceRun(sizes) as run:
            R = [np.zeros(n, np.float32) for n in sizes]
            for r in range(4):
                dWs = [synth.gaussian_update(n, round_=r, tensor=i) for i, n in enumerate(sizes)]
                res = check_round(run, dWs, R, p, check_decode=(r in (0, 3)))
                assert res[0].k == 10485
                assert sbc.sbc_last_route(run.ctx) & sbc.SBC_ROUTE_WIDE
                R = [x.R_new for x in res]


def test_calls_of_grid_wide_tensors_only_that_need_the_second_pass():
    """A call whose tensors all take the grid-wide kernels runs no other selection kernel unless one
    of them cannot be finished there: a misleading sample (too few candidates: histogram route),
    and tie-heavy data (more equal entries at the threshold than those kernels rank: one workgroup)."""
    n = 400000
    x = (np.abs(synth.small_model_update([n], round_=4)[0]) * 1e-3).astype(np.float32)
    pos = sampled_positions(n, 0)
    x[pos[::200]] = 5.0                                      # every large entry lies where the sampler looks
    x[pos[1::200]] = -7.0
    with DeviceRun([n]) as run:
        sbc.sbc_set_option(run.ctx, sbc.SBC_OPT_WIDE_MIN_KEPT, 300)
        check_round(run, [x], [np.zeros(n, np.float32)], 0.001)               # k = 400
        assert main_route(run.ctx) & sbc.SBC_ROUTE_HISTOGRAM
    sizes = [200000, 80000]
    with DeviceRun(sizes) as run:
        sbc.sbc_set_option(run.ctx, sbc.SBC_OPT_WIDE_MIN_KEPT, 6500)
        R = [np.zeros(m, np.float32) for m in sizes]
        for r in range(2):
            dWs = [synth.palette_update(m, round_=r, tensor=i) for i, m in enumerate(sizes)]
            res = check_round(run, dWs, R, 0.1)
            R = [v.R_new for v in res]


def test_histogram_fallback_bitmap_and_grid_wide_tensors_in_one_call():
    """One call whose tensors take every route at once: tensor 0 keeps enough entries for the
    grid-wide kernels; tensor 1 keeps too many for the fused encoder and too few for those (one
    workgroup selects, positions go through the bitmap); tensor 2 has its large entries exactly
    where the sampler looks, so its filter keeps too few and the histogram route redoes it; tensor
    3 keeps more than the lists staged in LDS hold and is sorted and encoded by one workgroup."""
    sizes = [250000, 170000, 50000, 100000, 300]
    p = 0.1
    with DeviceRun(sizes) as run:
        sbc.sbc_set_option(run.ctx, sbc.SBC_OPT_WIDE_MIN_KEPT, 20000)
        R = [np.zeros(n, np.float32) for n in sizes]
        for r in range(2):
            dWs = [synth.gaussian_update(n, round_=r, tensor=i) for i, n in enumerate(sizes)]
            x = (np.abs(dWs[2]) * 1e-3).astype(np.float32)
            pos = sampled_positions(sizes[2], 2)
            x[pos[::8]] = 5.0 + r                                # 2048 large entries a side (k = 5000), all sampled
            x[pos[1::8]] = -7.0 - r
            dWs[2] = x
            res = check_round(run, dWs, R, p)
            route = sbc.sbc_last_route(run.ctx)
            assert route & sbc.SBC_ROUTE_HISTOGRAM and route & sbc.SBC_ROUTE_WIDE, route
            assert 16384 < res[1].k < 20000 <= res[0].k and 8192 < res[3].k <= 16384
            R = [x.R_new for x in res]


def test_more_wide_tensors_than_the_grid_wide_kernels_take():
    """70 tensors that each qualify for the grid-wide selection and for the tiled decoder: the
    selection takes 64 and hands the rest to the one-workgroup kernel, the decoder tiles 16 streams
    and leaves the rest to the one-workgroup decoder."""
    sizes = [70000 + 8 * i for i in range(70)]
    p = 0.1
    with DeviceRun(sizes) as run:
        sbc.sbc_set_option(run.ctx, sbc.SBC_OPT_WIDE_MIN_KEPT, 6500)
        R = [np.zeros(n, np.float32) for n in sizes]
        for r in range(2):
            dWs = [synth.gaussian_update(n, round_=r, tensor=i) for i, n in enumerate(sizes)]
            res = check_round(run, dWs, R, p)
            assert r > 0 or sbc.sbc_last_route(run.ctx) & sbc.SBC_ROUTE_WIDE     # (later rounds: see test_grid_wide_selection)
            assert all(x.k >= 6500 for x in res)
            R = [x.R_new for x in res]


def test_tensor_of_many_chunks():
    """A tensor of more than 1024 chunks (several rounds of every per-tensor scan over chunks),
    plain and tie-heavy (LDS queues overflow, chunks are read a second time)."""
    n = 8192 * 1100 + 5
    with DeviceRun([n, 70000]) as run:
        R = [np.zeros(n, np.float32), np.zeros(70000, np.float32)]
        for r in range(2):
            dWs = [synth.gaussian_update(n, round_=r), synth.gaussian_update(70000, round_=r, tensor=1)]
            res = check_round(run, dWs, R, 0.001, check_decode=(r == 0))
            R = [x.R_new for x in res]
        dWs = [synth.palette_update(n), synth.palette_update(70000, tensor=1)]
        check_round(run, dWs, R, 0.001, check_decode=False)


def test_tensor_of_several_scan_tiles():
    """A tensor encoded from the bitmap whose chunks span several tiles of the per-tensor scan
    (4096 chunks each), next to one of a single tile: bit offsets carry across tiles."""
    sizes = [8192 * 8200 + 77, 8192 * 900 + 1]
    with DeviceRun(sizes) as run:
        dWs = [synth.gaussian_update(n, tensor=i) for i, n in enumerate(sizes)]
        # a stretch of several tiles without any kept entry, and a tile whose first chunks are empty
        dWs[0][8192 * 1000: 8192 * 5200] = 0.0
        res = check_round(run, dWs, [np.zeros(n, np.float32) for n in sizes], 0.001)
        assert res[0].k > 6144 and res[1].k > 6144


def test_compact_context():
    """A context whose candidate lists hold a few times k entries instead of every entry: same
    results on ordinary data (also when carried keys let a flood pass that overflows the lists
    and sends the tensors through the histogram route), SBC_ECAPACITY before anything runs when p
    needs longer lists than the context has, and after the fact for data whose threshold value is
    shared by more entries than a list holds."""
    sizes = synth.numels(synth.resnet50_shapes())
    with DeviceRun(sizes, compact=True) as run:
        R = [np.zeros(n, np.float32) for n in sizes]
        for r in range(3):
            res = check_round(run, synth.resnet50_update(round_=r), R, 0.001, check_decode=(r == 0))
            R = [x.R_new for x in res]
        with pytest.raises(sbc.SbcError) as e:              # p = 0.2: the lists would need 1.6 entries per entry
            run.compress(synth.resnet50_update(round_=3), 0.2)
        assert e.value.code == sbc.SBC_ECAPACITY
    sizes = [300000, 64, 20000, 8193, 1]
    scales = [1.0, 1.0, 3000.0, 1.0, 1.0]                    # a jump in scale floods the lists behind carried keys
    with DeviceRun(sizes, compact=True) as run:
        R = [np.zeros(n, np.float32) for n in sizes]
        routes = []
        for r, sc in enumerate(scales):
            dWs = [(d * np.float32(sc)).astype(np.float32) for d in synth.small_model_update(sizes, round_=r)]
            res = check_round(run, dWs, R, 0.001)
            routes.append(main_route(run.ctx))
            R = [x.R_new for x in res]
        print("routes", routes)
        # (300000 entries: the lists hold 75000 per side; a flood beyond that is redone through the histogram route)
        assert routes[2] & sbc.SBC_ROUTE_HISTOGRAM and routes[2] & sbc.SBC_ROUTE_CARRIED_KEYS
    # a constant tensor: every entry equals the k-th, no list of a quarter of the entries holds them
    sizes = [200000, 3000]
    with DeviceRun(sizes, compact=True) as run:
        dWs = [np.full(200000, 0.5, np.float32), synth.gaussian_update(3000, tensor=1)]
        with pytest.raises(sbc.SbcError) as e:
            run.compress(dWs, 0.001)
        assert e.value.code == sbc.SBC_ECAPACITY
        # the context is usable afterwards
        for x in run.R:
            x.zero_()
        dWs = [synth.gaussian_update(n, tensor=i) for i, n in enumerate(sizes)]
        check_round(run, dWs, [np.zeros(n, np.float32) for n in sizes], 0.001)


def test_deferred_decode_status():
    """SBC_OPT_DEFER_DECODE_STATUS: decode calls only enqueue; results equal the waiting calls', a
    corrupt message among good ones is reported by sbc_decode_status, and the status starts afresh."""
    sizes = [40000, 64, 9000]
    p = 0.01
    clients = 4
    msgs, want = [], [np.zeros(n, np.float32) for n in sizes]
    with DeviceRun(sizes) as run:
        for c in range(clients):
            for r in run.R:
                r.zero_()
            dWs = synth.small_model_update(sizes, client=c)
            msg, nbytes = run.compress(dWs, p)
            msgs.append((msg, nbytes))
            res = o.compress_model(dWs, [np.zeros_like(d) for d in dWs], p)
            o.decode_accumulate(o.build_message(res), sizes, 1.0 / clients, want)
        sbc.sbc_set_option(run.ctx, sbc.SBC_OPT_DEFER_DECODE_STATUS, 1)
        sbc.sbc_decode_status(run.ctx)                                   # nothing outstanding: fine
        outs = [torch.zeros(n, dtype=torch.float32, device="cuda:0") for n in sizes]
        for msg, nbytes in msgs:
            sbc.sbc_decompress_accumulate(run.ctx, msg, nbytes, p, 1.0 / clients, outs)
        with pytest.raises(sbc.SbcError):                                # not while a status is outstanding
            sbc.sbc_set_option(run.ctx, sbc.SBC_OPT_DEFER_DECODE_STATUS, 0)
        sbc.sbc_decode_status(run.ctx)
        for t in range(len(sizes)):
            assert np.array_equal(outs[t].cpu().numpy(), want[t]), "tensor %d: deferred decode" % t
        # one corrupt message between good ones
        bad = msgs[1][0].clone()
        bad[32 + 4] += 1                                                 # nnz off by one
        guard = [torch.zeros(n + 64, dtype=torch.float32, device="cuda:0") for n in sizes]
        outs = [g[32:32 + n] for g, n in zip(guard, sizes)]
        sbc.sbc_decompress_accumulate(run.ctx, msgs[0][0], msgs[0][1], p, 1.0, outs)
        sbc.sbc_decompress_accumulate(run.ctx, bad, msgs[1][1], p, 1.0, outs)
        sbc.sbc_decompress_accumulate(run.ctx, msgs[2][0], msgs[2][1], p, 1.0, outs)
        with pytest.raises(sbc.SbcError) as e:
            sbc.sbc_decode_status(run.ctx)
        assert e.value.code == sbc.SBC_ECORRUPT
        for g, n in zip(guard, sizes):
            assert not g[:32].any() and not g[32 + n:].any(), "decode wrote out of bounds"
        # the status starts afresh, and other output buffers are picked up
        outs2 = [torch.zeros(n, dtype=torch.float32, device="cuda:0") for n in sizes]
        sbc.sbc_decompress_accumulate(run.ctx, msgs[3][0], msgs[3][1], p, 1.0, outs2)
        sbc.sbc_decode_status(run.ctx)
        sbc.sbc_set_option(run.ctx, sbc.SBC_OPT_DEFER_DECODE_STATUS, 0)
        outs3 = [torch.zeros(n, dtype=torch.float32, device="cuda:0") for n in sizes]
        sbc.sbc_decompress_accumulate(run.ctx, msgs[3][0], msgs[3][1], p, 1.0, outs3)
        for a, b in zip(outs2, outs3):
            assert torch.equal(a, b)


def test_compress_begin_end_interleaved_clients():
    """sbc_compress_begin / sbc_compress_end: three independent clients in flight on their own
    streams; every message and residual equals the oracle's, also on the histogram route."""
    sizes = [70000, 64, 20000, 8193]
    p = 0.01
    clients = 3
    runs = [DeviceRun(sizes) for _ in range(clients)]
    streams = [torch.cuda.Stream() for _ in range(clients)]
    try:
        sbc.sbc_set_option(runs[2].ctx, sbc.SBC_OPT_FORCE_EXACT_PATH, 1)      # completes in sbc_compress_end
        R = [[np.zeros(n, np.float32) for n in sizes] for _ in range(clients)]
        bound = sbc.sbc_msg_bound(sizes, p)
        with pytest.raises(sbc.SbcError):
            sbc.sbc_compress_end(runs[0].ctx)                                 # nothing pending
        for rnd in range(3):
            dWs = [synth.small_model_update(sizes, client=c, round_=rnd) for c in range(clients)]
            d_dW = [[torch.from_numpy(x).cuda() for x in dWs[c]] for c in range(clients)]
            msgs = [torch.zeros(bound, dtype=torch.uint8, device="cuda:0") for _ in range(clients)]
            torch.cuda.synchronize()
            for c in range(clients):
                sbc.sbc_compress_begin(runs[c].ctx, d_dW[c], runs[c].R, p, msgs[c], streams[c].cuda_stream)
            with pytest.raises(sbc.SbcError):                                 # one step at a time per context
                sbc.sbc_compress_begin(runs[0].ctx, d_dW[0], runs[0].R, p, msgs[0], streams[0].cuda_stream)
            with pytest.raises(sbc.SbcError):
                sbc.sbc_set_option(runs[0].ctx, sbc.SBC_OPT_CARRY_FILTER_KEYS, 1)
            for c in (1, 0, 2):
                nbytes = sbc.sbc_compress_end(runs[c].ctx)
                # (the size is known before the client's stream is idle; the copies below run on
                # another stream, so that stream is waited for first, as the header asks)
                streams[c].synchronize()
                res = o.compress_model(dWs[c], R[c], p)
                assert msgs[c][:nbytes].cpu().numpy().tobytes() == o.build_message(res), (rnd, c)
                for t, x in enumerate(res):
                    got = runs[c].R[t].cpu().numpy()
                    assert np.allclose(got, x.R_new, rtol=0, atol=1e-5 * max(abs(float(x.mu_signed)), 1e-30)), (rnd, c, t)
                    mu_pos, mu_neg, side, nnz, bit_len = sbc.sbc_last_tensor_stats(runs[c].ctx, t)
                    assert side == x.side and nnz == x.k
                R[c] = [x.R_new for x in res]
            assert main_route(runs[2].ctx) == sbc.SBC_ROUTE_HISTOGRAM
    finally:
        for r in runs:
            r.close()


def test_config3_in_the_benchmark_call_sequence():
    """The ResNet-50-shaped workload through the exact call sequence bench.py times: the client's
    next round is enqueued (begin) into the other message buffer before the server call on the
    current message, whose status is deferred; messages and the averaged update against the oracle."""
    sizes = synth.numels(synth.resnet50_shapes())
    p, scale, rounds = 1e-3, 1.0 / 32.0, 3
    bound = sbc.sbc_msg_bound(sizes, p)
    with DeviceRun(sizes) as run:
        sbc.sbc_set_option(run.ctx, sbc.SBC_OPT_DEFER_DECODE_STATUS, 1)
        msgs = [torch.zeros(bound, dtype=torch.uint8, device="cuda:0") for _ in range(2)]
        outs = [torch.zeros(n, dtype=torch.float32, device="cuda:0") for n in sizes]
        host_dW = [synth.resnet50_update(round_=r) for r in range(rounds)]
        d_dW = [[torch.from_numpy(x).cuda() for x in upd] for upd in host_dW]
        R_host = [np.zeros(n, np.float32) for n in sizes]
        want_out = [np.zeros(n, np.float32) for n in sizes]
        sbc.sbc_compress_begin(run.ctx, d_dW[0], run.R, p, msgs[0])
        for s in range(rounds):
            print("step", s, flush=True)
            nbytes = sbc.sbc_compress_end(run.ctx)
            got = msgs[s % 2][:nbytes].cpu().numpy().tobytes()
            if s + 1 < rounds:
                sbc.sbc_compress_begin(run.ctx, d_dW[s + 1], run.R, p, msgs[(s + 1) % 2])
            sbc.sbc_decompress_accumulate(run.ctx, msgs[s % 2], nbytes, p, scale, outs)
            res = o.compress_model(host_dW[s], R_host, p)
            want = o.build_message(res)
            assert got == want, "step %d: message differs" % s
            o.decode_accumulate(want, sizes, scale, want_out)
            R_host = [x.R_new for x in res]
        sbc.sbc_decode_status(run.ctx)
        for t in range(len(sizes)):
            assert np.array_equal(outs[t].cpu().numpy(), want_out[t]), "tensor %d: averaged update" % t
