"""Randomly drawn parity cases: tensor sizes, sparsity, data family, route thresholds and context
kind are drawn from a seeded generator; every round is compared with the oracle to the bar of
tests/test_gpu_parity.py (message bytes, mask and bitstream bit-exact).  The draw favours the
grid-wide selection kernels and the bitmap encoder, whose hand-backs and second passes depend on
where thresholds and ties happen to fall."""
import numpy as np
import pytest

from paper_1805_08768_amd import binding as sbc, synth
import parity_util
from parity_util import DeviceRun, check_round

pytestmark = pytest.mark.gpu

FAMILIES = ("gauss", "student", "palette", "model", "grow", "const", "sparse")


def _update(fam, g, sizes, case, r):
    if fam == "gauss":
        return [synth.gaussian_update(n, round_=r, tensor=i, client=case) for i, n in enumerate(sizes)]
    if fam == "student":
        return [synth.student_t_update(n, round_=r, tensor=i, client=case) for i, n in enumerate(sizes)]
    if fam == "palette":
        return [synth.palette_update(n, round_=r, tensor=i) for i, n in enumerate(sizes)]
    if fam == "grow":                                        # the scale triples every round: carried keys fall behind
        return [(synth.gaussian_update(n, round_=r, tensor=i, client=case) * np.float32(3.0 ** r)).astype(np.float32)
                for i, n in enumerate(sizes)]
    if fam == "const":                                       # every entry a tie
        return [np.full(n, np.float32(0.01 * (r + 1) * (-1) ** i), np.float32) for i, n in enumerate(sizes)]
    if fam == "sparse":                                      # mostly zeros
        out = []
        for n in sizes:
            x = np.zeros(n, np.float32)
            idx = g.integers(0, n, size=max(1, n // 50))
            x[idx] = g.standard_normal(len(idx)).astype(np.float32)
            out.append(x)
        return out
    return synth.small_model_update(sizes, round_=r)


@pytest.mark.parametrize("block", range(4))
def test_random_cases(block):
    for case in range(12 * block, 12 * block + 12):
        g = np.random.default_rng(77000 + case)
        sizes = [int(g.integers(20000, 400000)) for _ in range(int(g.integers(1, 4)))]
        if g.random() < 0.3:
            sizes.append(int(g.integers(1, 9000)))
        p = float(g.choice([0.001, 0.01, 0.03, 0.08, 0.15, 0.4]))
        wide_min = int(g.choice([300, 2000, 6500, 20000]))
        fam = str(g.choice(FAMILIES))
        sampled = bool(g.random() < 0.25)
        carry = int(g.random() < 0.8)
        compact = bool(g.random() < 0.3)
        parity_util.FUSED_STEP = int(g.random() < 0.2)
        print("case", case, sizes, "p", p, "wide_min", wide_min, fam, "sampled", sampled, "carry", carry,
              "compact", compact, "fused", parity_util.FUSED_STEP, flush=True)
        try:
            with DeviceRun(sizes, compact=compact, sampled=sampled) as run:
                sbc.sbc_set_option(run.ctx, sbc.SBC_OPT_WIDE_MIN_KEPT, wide_min)
                sbc.sbc_set_option(run.ctx, sbc.SBC_OPT_CARRY_FILTER_KEYS, carry)
                R = [np.zeros(n, np.float32) for n in sizes]
                for r in range(4):
                    try:
                        res = check_round(run, _update(fam, g, sizes, case, r), R, p, check_decode=(r % 2 == 0))
                    except sbc.SbcError as e:
                        # a compact context refuses what its short lists cannot hold (large p, all ties)
                        assert compact and e.code == sbc.SBC_ECAPACITY
                        break
                    R = [x.R_new for x in res]
        finally:
            parity_util.FUSED_STEP = 0
