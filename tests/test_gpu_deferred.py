"""GPU parity for sums of rotations that share one ModDown (he_rotate_sum with deferred != 0, and he_raconv with
deferred_moddown = 1): bit for bit against the oracle's rotate_sum_deferred / raconv(deferred=True), on the
stored-accumulator path (generic rings, and more than 16 rotated terms at N = 2^16) and on the N = 2^16 path that
computes the summed accumulator inside the ModDown transforms; decrypted results against the messages; counters."""
import sys

import numpy as np
import pytest

from he_inputs import sampling as S
from he_inputs.params import config_params, toy_params

pytestmark = pytest.mark.gpu


def _say(msg):
    print(msg, file=sys.__stdout__, flush=True)


def _setup(prm, seed):
    from oracle import ckks_client as K
    from oracle.he_oracle import Oracle
    from paper_2302_02407_amd.binding import HEContext
    rng = S.make_rng(seed)
    orc, ctx = Oracle.from_params(prm), HEContext.from_params(prm)
    cl = K.Client(orc, S.ternary_secret(rng, prm.N, prm.hamming))
    return rng, orc, ctx, cl


def _key(prm, rng, cl, g):
    return cl.rotation_key(g, S.uniform_limbs(rng, prm.moduli, prm.N, prm.dnum), S.gaussian_error(rng, prm.N, prm.sigma, prm.dnum))


def _rand_ct(prm, rng, level):
    return np.stack([S.uniform_limbs(rng, prm.q[:level + 1], prm.N)[0] for _ in range(2)])


def _sum_case(prm, seed, level, steps):
    """he_rotate_sum in both modes against the oracle on uniform ciphertexts."""
    from gpu_util import dev, host, zeros
    rng, orc, ctx, cl = _setup(prm, seed)
    N = prm.N
    gs = [orc.galois_elt(s) for s in steps]
    keys = {}
    for g in gs:
        if g != 1 and g not in keys:
            keys[g] = _key(prm, rng, cl, g)
            ctx.he_evk_register(g, dev(keys[g]))
    cts = [_rand_ct(prm, rng, level) for _ in steps]
    d_cts = [dev(c) for c in cts]
    want = orc.rotate_sum_deferred(cts, level, gs, [keys.get(g) for g in gs])
    out = zeros(2, level + 1, N)
    ctx.he_counters_reset()
    ctx.he_rotate_sum(d_cts, level, steps, out, deferred=True)
    cnt = ctx.he_counters()
    assert (host(out) == want).all(), ("deferred", prm.logN, level, steps)
    n_rot = sum(1 for g in gs if g != 1)
    assert cnt["keyswitch"] == n_rot and cnt["modup"] == n_rot and cnt["moddown"] == (1 if n_rot else 0)
    tbt = None
    for ct, g in zip(cts, gs):
        term = ct if g == 1 else orc.rotate(ct, level, g, keys[g])
        tbt = term if tbt is None else orc.add(tbt, term, level)
    ctx.he_counters_reset()
    ctx.he_rotate_sum(d_cts, level, steps, out, deferred=False)
    assert (host(out) == tbt).all(), ("term by term", prm.logN, level, steps)
    assert ctx.he_counters()["moddown"] == n_rot


@pytest.mark.parametrize("level", [5, 4, 2, 0])
def test_rotate_sum_small_ring(level):
    prm = toy_params(logN=9, q_bits=30, nq=6, p_bits=32, np_=2, dnum=3, hamming=16, seed=70)
    N = prm.N
    _sum_case(prm, 70 + level, level, [1, 0, 5, N // 2 - 3, 0, 7])           # rotated and plain terms mixed
    _sum_case(prm, 80 + level, level, [3])                                   # a single rotation
    _sum_case(prm, 90 + level, level, [0, 0])                                # nothing to switch
    _sum_case(prm, 100 + level, level, list(range(1, 21)))                   # 20 rotated terms: two groups of stored accumulators


def test_rotate_sum_two_pass_ring():
    prm = toy_params(logN=13, q_bits=40, nq=5, p_bits=50, np_=2, dnum=3, hamming=32, seed=71)
    _sum_case(prm, 71, 4, [1, 2, 0, 100])


@pytest.mark.parametrize("level,steps", [
    (22, [2, 62, 64, 66, 0, 32766, 32706, 32704, 32702]),     # the 9 taps of the 3x3 layer on 32x32 with R = 2
    (5, [1, 0, 2, 4]),
    (2, list(range(1, 18))),                                   # 17 rotated terms: the stored-accumulator path at N = 2^16
])
def test_rotate_sum_n65536(level, steps):
    _sum_case(config_params(3), 72 + level, level, steps)


def test_rotate_sum_n65536_widest_primes():
    """60-bit ciphertext primes: the partial sums of the fused inner products must stay canonical (twelve terms of
    lazily reduced partial sums would not fit 64 bits)."""
    prm = toy_params(logN=16, q_bits=60, nq=4, p_bits=59, np_=2, dnum=2, hamming=64, seed=73)
    _sum_case(prm, 73, 3, [1, 2, 3, 5, 7, 11, 13, 17, 19, 23, 29, 31, 0])


def test_rotate_sum_errors():
    from gpu_util import dev, zeros
    from paper_2302_02407_amd.binding import HEError
    prm = toy_params(logN=8, q_bits=30, nq=6, p_bits=32, np_=2, dnum=3, hamming=16, seed=73)
    rng, orc, ctx, cl = _setup(prm, 73)
    ct = dev(_rand_ct(prm, rng, 5))
    out = zeros(2, 6, prm.N)
    with pytest.raises(HEError) as e:
        ctx.he_rotate_sum([ct, ct], 5, [1, 2], out, deferred=True)            # no keys
    assert e.value.code == -3
    with pytest.raises(HEError):
        ctx.he_rotate_sum([ct], 5, [0], ct, deferred=True)                    # output is an input
    with pytest.raises(HEError):
        ctx.he_rotate_sum([], 5, [], out)                                     # no terms


def _raconv_case(prm, C_a, H, W, c_in, f, level, w_std, seed):
    from gpu_util import dev, host, zeros
    from oracle import conv2d as CV
    rng, orc, ctx, cl = _setup(prm, seed)
    N = prm.N
    geo = CV.RAGeometry(N, C_a, H, W, c_in, f=f)
    x = rng.uniform(-1.0, 1.0, size=(c_in, H, W))
    wt = rng.normal(0.0, w_std, size=(C_a, c_in, f, f))
    steps = sorted(set(s for s in geo.tap_steps if s))
    evks = {st: _key(prm, rng, cl, orc.galois_elt(st)) for st in steps}
    cts = [cl.encrypt(geo.pack_input(x, i).astype(np.complex128), prm.scale, level,
                      S.uniform_limbs(rng, prm.q[:level + 1], N)[0], S.gaussian_error(rng, N, prm.sigma)[0])
           for i in range(geo.n_in)]
    pts = CV.encode_ra_weights(orc, geo, wt, level, float(prm.q[level]))
    _say("raconv, one ModDown: running the oracle")
    want, inter = CV.raconv(orc, geo, cts, level, pts, evks, keep=True, deferred=True)
    for st, k in evks.items():
        ctx.he_evk_register(ctx.galois_elt(st), dev(k))
    weights = [dev(pts[i, t]) for i in range(geo.n_in) for t in range(f * f)]
    d_cts = [dev(c) for c in cts]
    ctx.he_ws_reserve(ctx.he_ws_query_raconv(geo.n_in, W, geo.R, f, level, deferred=True))
    ws = ctx.he_ws_bytes()
    out = zeros(2, level, N)
    ctx.he_counters_reset()
    ctx.he_raconv(W, geo.R, f, level, weights, d_cts, out, deferred=True)
    cnt = ctx.he_counters()
    got = host(out)
    assert ctx.he_ws_bytes() == ws
    assert (got == want).all()
    assert cnt["keyswitch"] == f * f - 1 and cnt["moddown"] == 1 and cnt["rescale"] == 1 and cnt["mac"] == geo.n_in * f * f
    # the pre-rescale sum through the stand-alone entry point equals the oracle's intermediate
    macs = [dev(m) for m in inter["mac"]]
    tot = zeros(2, level + 1, N)
    ctx.he_rotate_sum(macs, level, geo.tap_steps, tot, deferred=True)
    assert (host(tot) == inter["sum"]).all()
    # fewer transforms than one ModDown per tap
    ctx.he_counters_reset()
    ctx.he_raconv(W, geo.R, f, level, weights, d_cts, zeros(2, level, N), deferred=False)
    c2 = ctx.he_counters()
    assert c2["moddown"] == f * f - 1 and cnt["ntt_limbs"] < c2["ntt_limbs"] and cnt["intt_limbs"] < c2["intt_limbs"]
    z = cl.decrypt(got, level - 1, prm.scale).real.reshape(C_a, H, W, geo.R)
    assert np.max(np.abs(z.sum(axis=-1) - CV.conv2d_float(x, wt))) < 1e-3


def test_raconv_one_moddown_small_ring():
    prm = toy_params(logN=10, q_bits=40, nq=4, p_bits=41, np_=2, dnum=2, scale=2.0 ** 30, hamming=32, seed=95)
    _raconv_case(prm, C_a=8, H=8, W=8, c_in=8, f=3, level=3, w_std=0.2, seed=95)
    _raconv_case(prm, C_a=8, H=8, W=8, c_in=3, f=5, level=3, w_std=0.1, seed=98)      # 24 rotated taps


@pytest.mark.timeout(900)
def test_raconv_one_moddown_after_resnet20_layer():
    """8 ciphertexts of 2 channels each (16 channels, 32x32) at level 22 -> one ciphertext, N = 2^16: the eight
    tap rotations share one ModDown."""
    _raconv_case(config_params(3), C_a=16, H=32, W=32, c_in=16, f=3, level=22, w_std=(2.0 / (9 * 16)) ** 0.5, seed=3)
