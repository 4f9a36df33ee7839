"""GPU parity of the fused CAConv -> Square -> RAConv block (Algorithm 3, he_ca_ra_block) against the oracle's
loop-for-loop version: one and two channel-aligned ciphertexts, every forwarding group size (same bits), with and
without the shared ModDown in Slide_1&Sum_f; operation counts; decrypted result against float64."""
import sys

import numpy as np
import pytest

from he_inputs.params import config_params, toy_params

pytestmark = pytest.mark.gpu


def _say(msg):
    print(msg, file=sys.__stdout__, flush=True)


def _case(prm, C_a, H, W, c_in, c_mid, level, std, seed, groups, deferred_modes=(False, True), hoisted_ras=False):
    from gpu_util import dev, host, zeros
    from oracle import block as OB
    from test_oracle_fused_block import check_fused_output, fused_inputs
    from paper_2302_02407_amd.binding import HEContext
    d = fused_inputs(prm, C_a, H, W, c_in, c_mid, level, std, seed, all_ras_multiples=hoisted_ras)
    orc, g_ca, g_ra, n_ca = d["orc"], d["g_ca"], d["g_ra"], d["n_ca"]
    n_ra, N = g_ca.n_out, prm.N
    ctx = HEContext.from_params(prm)
    for st, k in d["evks"].items():
        ctx.he_evk_register(ctx.galois_elt(st), dev(k))
    ctx.he_evk_register(0, dev(d["rlk"]))
    w_ca = [dev(d["p_ca"][j][k][t]) for j in range(n_ra) for k in range(n_ca) for t in range(9)]
    w_ra = [dev(d["p_ra"][l][j][t]) for l in range(n_ca) for j in range(n_ra) for t in range(9)]
    cts = [dev(c) for c in d["cts"]]
    n_ras = (C_a - 1) if hoisted_ras else len(g_ca.ras_steps)      # key switches of one rotate-and-sum
    ras_md = 1 if hoisted_ras else n_ras                            # its ModUps and ModDowns
    for deferred in deferred_modes:
        _say("fused block: running the oracle (n_ca=%d, n_ra=%d, one ModDown per output: %s)" % (n_ca, n_ra, deferred))
        want = OB.ca_ra_block(orc, g_ca, g_ra, d["cts"], level, d["p_ca"], d["p_ra"], d["evks"], d["rlk"], d["k_in"], deferred=deferred,
                              hoisted_ras=hoisted_ras)
        for group in groups:
            ctx.he_ws_reserve(ctx.he_ws_query_ca_ra_block(C_a, H, W, g_ca.R, 3, n_ca, n_ra, level, group, deferred, hoisted_ras))
            ws = ctx.he_ws_bytes()
            outs = [zeros(2, level - 2, N) for _ in range(n_ca)]
            ctx.he_counters_reset()
            ctx.he_ca_ra_block(C_a, H, W, g_ca.R, 3, level, d["k_in"], w_ca, w_ra, cts, outs, group=group, deferred=deferred,
                               hoisted_ras=hoisted_ras)
            cnt = ctx.he_counters()
            for l in range(n_ca):
                assert (host(outs[l]) == want[l]).all(), (deferred, group, l)
            assert ctx.he_ws_bytes() == ws
            # rotations: f^2-1 per input (Slide_f), log2(C_a) per intermediate (RaS), f^2-1 per output (Slide_1);
            # one relinearisation per intermediate
            assert cnt["keyswitch"] == 8 * n_ca + n_ras * n_ra + n_ra + 8 * n_ca, cnt
            assert cnt["modup"] == n_ca + ras_md * n_ra + n_ra + 8 * n_ca
            assert cnt["moddown"] == 8 * n_ca + ras_md * n_ra + n_ra + (n_ca if deferred else 8 * n_ca)
            assert cnt["mac"] == 2 * 9 * n_ca * n_ra and cnt["rescale"] == 2 * n_ra + n_ca
    err = check_fused_output(d, [host(o) for o in outs], level)
    _say("fused block: max |dec - float64| = %.3g" % err)


def test_fused_block_small_ring():
    prm = toy_params(logN=9, q_bits=40, nq=5, p_bits=41, np_=2, dnum=3, scale=2.0 ** 30, hamming=32, seed=97)
    _case(prm, C_a=4, H=4, W=4, c_in=4, c_mid=8, level=4, std=0.2, seed=97, groups=(1, 2, 0))
    _case(prm, C_a=4, H=4, W=4, c_in=8, c_mid=8, level=4, std=0.2, seed=98, groups=(1, 0))
    prm = toy_params(logN=10, q_bits=40, nq=5, p_bits=41, np_=2, dnum=3, scale=2.0 ** 30, hamming=32, seed=99)
    _case(prm, C_a=8, H=8, W=8, c_in=16, c_mid=8, level=4, std=0.1, seed=99, groups=(3,))     # R = 1, 8 intermediates, groups 3+3+2


@pytest.mark.timeout(1100)
def test_fused_block_resnet20_unit():
    """16 -> 16 -> 16 channels on 32x32 at N = 2^16 (one input ciphertext, 8 intermediates, level 23 -> 20): the
    algorithm's loop exactly (group 1), and all intermediates batched."""
    _case(config_params(3), C_a=16, H=32, W=32, c_in=16, c_mid=16, level=23, std=(2.0 / (9 * 16)) ** 0.5, seed=6,
          groups=(1, 0), deferred_modes=(True,))


def test_fused_block_hoisted_rotate_and_sum_small_ring():
    prm = toy_params(logN=9, q_bits=40, nq=5, p_bits=41, np_=2, dnum=3, scale=2.0 ** 30, hamming=32, seed=97)
    _case(prm, C_a=4, H=4, W=4, c_in=4, c_mid=8, level=4, std=0.2, seed=97, groups=(1, 0), hoisted_ras=True)


@pytest.mark.timeout(1100)
def test_fused_block_hoisted_rotate_and_sum_resnet20_unit():
    _case(config_params(3), C_a=16, H=32, W=32, c_in=16, c_mid=16, level=23, std=(2.0 / (9 * 16)) ** 0.5, seed=6,
          groups=(0,), deferred_modes=(True,), hoisted_ras=True)

