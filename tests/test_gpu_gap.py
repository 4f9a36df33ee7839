"""GPU parity for 2-D gap packing across a downsampling layer (Section 3.2): the three-layer hand-off sequenced over
the C ABI (strided CAConv + merge into the gap, RAConv + gap sum, CAConv on the multiplexed format + gap sum) against
the oracle at every stage, the rotation counts of the cost table, and the decrypted formats against float64; plus the
batched rotate-and-sum entry point on its own."""
import sys

import numpy as np
import pytest

from he_inputs import sampling as S
from he_inputs.params import config_params, toy_params

pytestmark = pytest.mark.gpu


def _say(msg):
    print(msg, file=sys.__stdout__, flush=True)


def _case(prm, C_a, Hp, Wp, level, std, seed):
    from gpu_util import dev, host
    from oracle import gap as G
    from test_oracle_gap import check_handoff_stages, handoff_inputs
    from paper_2302_02407_amd import block as B
    from paper_2302_02407_amd.binding import HEContext
    d = handoff_inputs(prm, C_a, Hp, Wp, level, std, seed)
    geo, pw = d["geo"], d["pw"]
    _say("gap hand-off: running the oracle")
    want = G.downsample_handoff(d["orc"], geo, d["ct"], level, pw, d["evks"], progress=_say)
    ctx = HEContext.from_params(prm)
    for st, k in d["evks"].items():
        ctx.he_evk_register(ctx.galois_elt(st), dev(k))
    p1 = [dev(pw["p1"][o, t]) for o in range(geo.n1) for t in range(9)]
    p2 = [dev(pw["p2"][i, t]) for i in range(geo.n) for t in range(9)]
    p3 = [dev(pw["p3"][o, t]) for o in range(geo.n) for t in range(9)]
    ctx.he_counters_reset()
    _, got = B.downsample_handoff(ctx, C_a, Hp, Wp, geo.R0, level, dev(d["ct"]), p1, p2, dev(pw["mask_kappa"]), p3, dev(pw["mask_a"]),
                                  keep=True)
    cnt = ctx.he_counters()
    for name in ("l1_conv", "l1", "l3_conv", "l3"):
        for o in range(len(want[name])):
            assert (host(got[name][o]) == want[name][o]).all(), (name, o)
    for name in ("l2_conv", "l2"):
        assert (host(got[name]) == want[name]).all(), name
    log_ca, log_d, log_m, n = len(geo.ras_steps), int(np.log2(geo.d)), 1, geo.n
    # layer 1: Slide 8, merges n, RaS n*log2(C_a), replication n; layer 2: Slide 8, RaS_g + IR_g 2*log2(d');
    # layer 3: Slide 8, RaS n*log2(C_a), RaS_g + IR_g 2*n*log2(m')
    assert cnt["keyswitch"] == (8 + n + n * log_ca + n) + (8 + 2 * log_d) + (8 + n * log_ca + 2 * n * log_m), cnt
    assert cnt["rescale"] == geo.n1 + 1 + 1 + n + n and cnt["mac"] == 9 * geo.n1 + 9 * n + 1 + 9 * n + n
    err = check_handoff_stages(d, {k: ([host(t) for t in v] if isinstance(v, list) else host(v)) for k, v in got.items()}, level, prm.scale)
    _say("gap hand-off: max |dec - float64| over the three stages = %.3g" % err)


def test_handoff_small_ring():
    prm = toy_params(logN=10, q_bits=40, nq=7, p_bits=41, np_=3, dnum=3, scale=2.0 ** 30, hamming=32, seed=111)
    _case(prm, C_a=4, Hp=8, Wp=8, level=6, std=0.15, seed=111)


@pytest.mark.timeout(1100)
def test_handoff_resnet20_first_downsampling():
    """16 channels on 32x32 in format (m,d) = (1,2) -> 32 channels on 16x16 in format (2,4), N = 2^16, level 23 -> 18."""
    _case(config_params(4), C_a=16, Hp=32, Wp=32, level=23, std=(2.0 / (9 * 32)) ** 0.5, seed=7)


def test_ras_batched():
    from gpu_util import dev, host, zeros
    from oracle import gap as G
    from oracle import ckks_client as K
    from oracle.he_oracle import Oracle
    from paper_2302_02407_amd.binding import HEContext, HEError
    prm = toy_params(logN=9, q_bits=30, nq=6, p_bits=32, np_=2, dnum=3, hamming=16, seed=112)
    rng = S.make_rng(112)
    orc, ctx = Oracle.from_params(prm), HEContext.from_params(prm)
    cl = K.Client(orc, S.ternary_secret(rng, prm.N, prm.hamming))
    N, level = prm.N, 4
    steps = [1, 16, N // 2 - 3]
    evks = {s: cl.rotation_key(orc.galois_elt(s), S.uniform_limbs(rng, prm.moduli, N, prm.dnum), S.gaussian_error(rng, N, prm.sigma, prm.dnum))
            for s in steps}
    for s, k in evks.items():
        ctx.he_evk_register(ctx.galois_elt(s), dev(k))
    cts = [np.stack([S.uniform_limbs(rng, prm.q[:level + 1], N)[0] for _ in range(2)]) for _ in range(5)]
    d_cts = [dev(c) for c in cts]
    for use in (steps, steps[:2], steps[:1], []):
        outs = [zeros(2, level + 1, N) for _ in cts]
        ctx.he_counters_reset()
        ctx.he_ras(d_cts, level, use, outs)
        assert ctx.he_counters()["keyswitch"] == len(use) * len(cts)
        for c, o in zip(cts, outs):
            assert (host(o) == G.ras(orc, c, level, use, evks)).all(), use
    for c, dc in zip(cts, d_cts):
        assert (host(dc) == c).all()                                    # inputs untouched
    with pytest.raises(HEError):
        ctx.he_ras(d_cts, level, [2], [zeros(2, level + 1, N) for _ in cts])      # no key
    with pytest.raises(HEError):
        ctx.he_ras(d_cts[:1], level, [1], d_cts[:1])                               # output is the input
    ctx.he_ras([], level, [1], [])
