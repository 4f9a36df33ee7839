"""Pin of the oracle's 2-D gap packing across a downsampling layer against float64: after each of the three layers
the decrypted ciphertexts hold conv(...) in the slot format the next layer expects - pi_RA with d' channels and m'
replicas after the strided CAConv and its hand-off, pi_CA in format (m', d') after RAConv and its gap sum, pi_RA again
after the CAConv on the multiplexed format - and the rotation counts are those of the cost table."""
import numpy as np

from he_inputs import sampling as S
from he_inputs.params import toy_params
from oracle import ckks_client as K
from oracle import gap as G
from oracle.he_oracle import Oracle


def handoff_inputs(prm, C_a, Hp, Wp, level, std, seed):
    rng = S.make_rng(seed)
    orc = Oracle.from_params(prm)
    cl = K.Client(orc, S.ternary_secret(rng, prm.N, prm.hamming))
    N = prm.N
    geo = G.GapGeometry(N, C_a, Hp, Wp, C_a, 2 * C_a)
    x = rng.uniform(-1.0, 1.0, size=(C_a, Hp, Wp))
    w1 = rng.normal(0.0, std, size=(2 * C_a, C_a, 3, 3))
    w2 = rng.normal(0.0, std, size=(2 * C_a, 2 * C_a, 3, 3))
    w3 = rng.normal(0.0, std, size=(2 * C_a, 2 * C_a, 3, 3))
    evks = {st: cl.rotation_key(orc.galois_elt(st), S.uniform_limbs(rng, prm.moduli, N, prm.dnum),
                                S.gaussian_error(rng, N, prm.sigma, prm.dnum)) for st in geo.all_steps()}
    ct = cl.encrypt(geo.g1.pack_input(x).astype(np.complex128), prm.scale, level,
                    S.uniform_limbs(rng, prm.q[:level + 1], N)[0], S.gaussian_error(rng, N, prm.sigma)[0])
    pw = G.encode_handoff_weights(orc, geo, w1, w2, w3, level)
    return dict(orc=orc, cl=cl, geo=geo, x=x, w1=w1, w2=w2, w3=w3, evks=evks, ct=ct, pw=pw)


def check_handoff_stages(d, st, level, scale, tol=1e-3):
    geo, cl = d["geo"], d["cl"]
    y1, y2, y3 = G.handoff_float(d["x"], d["w1"], d["w2"], d["w3"])
    worst = 0.0
    for o in range(geo.n):
        worst = max(worst, float(np.max(np.abs(cl.decrypt(st["l1"][o], level - 1, scale).real - geo.expect_ra_format(y1, o)))))
    worst = max(worst, float(np.max(np.abs(cl.decrypt(st["l2"], level - 3, scale).real - geo.expect_ca_format(y2)))))
    for o in range(geo.n):
        worst = max(worst, float(np.max(np.abs(cl.decrypt(st["l3"][o], level - 5, scale).real - geo.expect_ra_format(y3, o)))))
    assert worst < tol, worst
    return worst


def test_handoff_small_ring_matches_float():
    prm = toy_params(logN=10, q_bits=40, nq=7, p_bits=41, np_=3, dnum=3, scale=2.0 ** 30, hamming=32, seed=111)
    level = 6
    d = handoff_inputs(prm, C_a=4, Hp=8, Wp=8, level=level, std=0.15, seed=111)
    geo = d["geo"]
    assert (geo.R0, geo.d, geo.m, geo.n1, geo.n) == (2, 4, 2, 4, 2)
    st = G.downsample_handoff(d["orc"], geo, d["ct"], level, d["pw"], d["evks"])
    assert st["l3"][0].shape == (2, level - 4, prm.N)
    check_handoff_stages(d, st, level, prm.scale)
