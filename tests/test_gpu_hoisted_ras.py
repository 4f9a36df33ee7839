"""GPU parity for the rotate-and-sum of he_conv2d evaluated as one hoisted sum of rotations per output
(hoisted_ras: one ModUp and one ModDown per output, keys shared by the outputs): bit-exact against the oracle on a
small ring, on a two-pass ring, with 32 channel blocks (31 terms: two launches of the inner products), with 57/59-bit moduli and a
single output, at N = 2^16 at level 5
(single digit) and on the ResNet-20 layer at level 23 (three digits, eight outputs in one launch set), with operation
counts; and
he_rotate_sum on one ciphertext repeated (terms that rotate the same polynomial share its ModUp)."""
import sys

import numpy as np
import pytest

from he_inputs import sampling as S
from he_inputs.params import config_params, toy_params

pytestmark = pytest.mark.gpu


def _say(msg):
    print(msg, file=sys.__stdout__, flush=True)


def _run(prm, C_a, H, W, c_out, level, w_std, tol, deferred_taps=False, seed=None):
    from gpu_util import dev, host, zeros
    from oracle import ckks_client as K
    from oracle import conv2d as CV
    from oracle.he_oracle import Oracle
    from paper_2302_02407_amd.binding import HEContext
    rng = S.make_rng(prm.seed if seed is None else seed)
    orc, ctx = Oracle.from_params(prm), HEContext.from_params(prm)
    cl = K.Client(orc, S.ternary_secret(rng, prm.N, prm.hamming))
    geo = CV.ConvGeometry(prm.N, C_a, H, W, c_out)
    x, wt = S.conv_tensors(rng, C_a, c_out, H, W, 3, w_std)
    base = geo.H * geo.W * geo.R
    steps = sorted(set(s for s in geo.tap_steps if s) | set(base * i for i in range(1, C_a)))
    evks = {st: cl.rotation_key(orc.galois_elt(st), S.uniform_limbs(rng, prm.moduli, prm.N, prm.dnum),
                                S.gaussian_error(rng, prm.N, prm.sigma, prm.dnum)) for st in steps}
    ct = cl.encrypt(geo.pack_input(x).astype(np.complex128), prm.scale, level,
                    S.uniform_limbs(rng, prm.q[:level + 1], prm.N)[0], S.gaussian_error(rng, prm.N, prm.sigma)[0])
    pts = (CV.encode_weights_raised if deferred_taps else CV.encode_weights)(orc, geo, wt, level, float(prm.q[level]))
    _say("hoisted rotate-and-sum parity: inputs ready (N=%d, %d keys), running the oracle" % (prm.N, len(evks)))
    want = CV.caconv(orc, geo, ct, level, pts, evks, progress=_say, deferred_taps=deferred_taps, hoisted_ras=True)
    for st, k in evks.items():
        ctx.he_evk_register(ctx.galois_elt(st), dev(k))
    weights = [dev(pts[o, t]) for o in range(geo.n_out) for t in range(9)]
    outs = [zeros(2, level, prm.N) for _ in range(geo.n_out)]
    d_ct = dev(ct)
    ctx.he_ws_reserve(ctx.he_ws_query_conv2d(C_a, H, W, geo.R, 3, level, geo.n_out, deferred_taps=deferred_taps, hoisted_ras=True))
    ws = ctx.he_ws_bytes()
    ctx.he_counters_reset()
    _say("hoisted rotate-and-sum parity: GPU call")
    ctx.he_conv2d(C_a, H, W, geo.R, 3, level, weights, d_ct, outs, deferred_taps=deferred_taps, hoisted_ras=True)
    cnt = ctx.he_counters()
    assert ctx.he_ws_bytes() == ws
    got = [host(o) for o in outs]
    for o in range(geo.n_out):
        assert (got[o] == want[o]).all(), o
    assert cnt["keyswitch"] == 8 + geo.n_out * (C_a - 1)
    assert cnt["modup"] == 1 + geo.n_out                                      # one per output, not one per step
    assert cnt["moddown"] == (geo.n_out if deferred_taps else 8) + geo.n_out
    dec, spread = geo.unpack_output([cl.decrypt(g, level - 1, prm.scale) for g in got])
    assert np.max(np.abs(dec - CV.conv2d_float(x, wt))) < tol and spread < tol


def test_small_ring_generic_path():
    prm = toy_params(logN=10, q_bits=40, nq=3, p_bits=41, np_=1, dnum=3, scale=2.0 ** 30, hamming=32, seed=80)
    _run(prm, C_a=4, H=4, W=4, c_out=16, level=2, w_std=0.1, tol=1e-3)


def test_two_pass_ring_with_deferred_taps():
    prm = toy_params(logN=13, q_bits=40, nq=4, p_bits=50, np_=2, dnum=2, scale=2.0 ** 30, hamming=32, seed=82)
    _run(prm, C_a=8, H=4, W=8, c_out=32, level=3, w_std=0.1, tol=1e-3, deferred_taps=True)


def test_thirty_two_channel_blocks_two_launches():
    # C_a = 32: rotations by multiples of N/64 slots leave the aligned blocks of 16 positions but stay inside the
    # 256-position tiles the inner products stage in LDS; 31 terms take two launches of at most 16 (the second continues
    # the stored accumulators)
    prm = toy_params(logN=12, q_bits=40, nq=4, p_bits=41, np_=2, dnum=2, scale=2.0 ** 30, hamming=32, seed=83)
    _run(prm, C_a=32, H=4, W=4, c_out=8, level=3, w_std=0.1, tol=1e-3)


def test_moduli_of_57_and_59_bits_single_output():
    # moduli wider than 54 bits take the 30-bit halves of the LDS-staged inner products (with their carry moves every
    # six products); one output ciphertext is the smallest register tile
    prm = toy_params(logN=11, q_bits=57, nq=3, p_bits=59, np_=2, dnum=2, scale=2.0 ** 45, hamming=32, seed=86)
    _run(prm, C_a=16, H=4, W=4, c_out=4, level=2, w_std=0.1, tol=1e-3)


def test_n65536_level5_single_digit():
    _run(config_params(3), C_a=16, H=32, W=32, c_out=4, level=5, w_std=(2.0 / (9 * 16)) ** 0.5, tol=1e-3, seed=85)


@pytest.mark.timeout(900)
def test_config3_resnet20_layer():
    _run(config_params(3), C_a=16, H=32, W=32, c_out=16, level=23, w_std=(2.0 / (9 * 16)) ** 0.5, tol=1e-3)


def test_rotate_sum_of_one_ciphertext_shares_its_modup():
    from gpu_util import dev, host, zeros
    from oracle import ckks_client as K
    from oracle.he_oracle import Oracle
    from paper_2302_02407_amd.binding import HEContext
    prm = config_params(3)
    rng = S.make_rng(86)
    orc, ctx = Oracle.from_params(prm), HEContext.from_params(prm)
    cl = K.Client(orc, S.ternary_secret(rng, prm.N, prm.hamming))
    N, level = prm.N, 7
    steps = [0, 5, 9, 1000]
    keys = {s: cl.rotation_key(orc.galois_elt(s), S.uniform_limbs(rng, prm.moduli, N, prm.dnum),
                               S.gaussian_error(rng, N, prm.sigma, prm.dnum)) for s in steps if s}
    for s, k in keys.items():
        ctx.he_evk_register(ctx.galois_elt(s), dev(k))
    ct = np.stack([S.uniform_limbs(rng, prm.q[:level + 1], N)[0] for _ in range(2)])
    want = orc.rotate_sum_deferred([ct] * len(steps), level, [orc.galois_elt(s) if s else 1 for s in steps], [keys.get(s) for s in steps])
    d = dev(ct)
    out = zeros(2, level + 1, N)
    ctx.he_counters_reset()
    ctx.he_rotate_sum([d] * len(steps), level, steps, out, deferred=True)
    assert (host(out) == want).all()
    cnt = ctx.he_counters()
    assert cnt["modup"] == 1 and cnt["moddown"] == 1 and cnt["keyswitch"] == 3
