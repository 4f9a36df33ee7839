"""Pins of the oracle's reordered RAConv (Algorithm 2) against float64: the chain CAConv -> RAConv equals two
plain convolutions in a row, with one channel per ciphertext (R = 1) and with two (R = 2, where the output
holds the partial sum of each replica class); and the reordered form equals the usual order (slide every
input, multiply, add) slot for slot."""
import numpy as np

from he_inputs import sampling as S
from he_inputs.params import toy_params
from oracle import ckks_client as K
from oracle import conv2d as CV
from oracle.he_oracle import Oracle


def _chain(C_a, H, W, c_mid, level):
    prm = toy_params(logN=10, q_bits=40, nq=4, p_bits=41, np_=2, dnum=2, scale=2.0 ** 30, hamming=32, seed=94)
    rng = S.make_rng(94)
    orc = Oracle.from_params(prm)
    cl = K.Client(orc, S.ternary_secret(rng, prm.N, prm.hamming))
    N = prm.N
    g1 = CV.ConvGeometry(N, C_a, H, W, c_mid, f=3)
    g2 = CV.RAGeometry(N, C_a, H, W, c_mid, f=3)
    assert g1.n_out == g2.n_in and g1.R == g2.R
    x, w1 = S.conv_tensors(rng, C_a, c_mid, H, W, 3, 0.2)
    w2 = rng.normal(0.0, 0.2, size=(C_a, c_mid, 3, 3))
    steps = sorted(set(s for s in g1.tap_steps if s) | set(g1.ras_steps) | set(s for s in g2.tap_steps if s))
    evks = {st: cl.rotation_key(orc.galois_elt(st), S.uniform_limbs(rng, prm.moduli, N, prm.dnum),
                                S.gaussian_error(rng, N, prm.sigma, prm.dnum)) for st in steps}
    ct = cl.encrypt(g1.pack_input(x).astype(np.complex128), prm.scale, level,
                    S.uniform_limbs(rng, prm.q[:level + 1], N)[0], S.gaussian_error(rng, N, prm.sigma)[0])
    p1 = CV.encode_weights(orc, g1, w1, level, float(prm.q[level]))
    mid = CV.caconv(orc, g1, ct, level, p1, evks)
    p2 = CV.encode_ra_weights(orc, g2, w2, level - 1, float(prm.q[level - 1]))
    out, inter = CV.raconv(orc, g2, mid, level - 1, p2, evks, keep=True)
    return prm, cl, g2, x, w1, w2, mid, p2, evks, out, inter, orc


def test_chain_one_channel_per_ciphertext():
    prm, cl, g2, x, w1, w2, mid, p2, evks, out, inter, orc = _chain(C_a=8, H=8, W=8, c_mid=8, level=3)
    assert g2.R == 1 and g2.n_in == 8 and out.shape == (2, 2, prm.N)
    y = CV.conv2d_float(CV.conv2d_float(x, w1), w2)                      # [C_a][H][W]
    z = cl.decrypt(out, 1, prm.scale).real.reshape(g2.C_a, g2.H, g2.W)
    assert np.max(np.abs(z - y)) < 1e-3


def test_chain_two_channels_per_ciphertext():
    prm, cl, g2, x, w1, w2, mid, p2, evks, out, inter, orc = _chain(C_a=4, H=8, W=8, c_mid=8, level=3)
    assert g2.R == 2 and g2.n_in == 4
    mid_f = CV.conv2d_float(x, w1)                                        # [c_mid][H][W]
    z = cl.decrypt(out, 1, prm.scale).real.reshape(g2.C_a, g2.H, g2.W, g2.R)
    for r in range(g2.R):
        chans = [c for c in range(8) if c % g2.R == r]                   # channels of replica class r
        part = CV.conv2d_float(mid_f[chans], w2[:, chans])
        assert np.max(np.abs(z[..., r] - part)) < 1e-3
    assert np.max(np.abs(z.sum(axis=-1) - CV.conv2d_float(mid_f, w2))) < 1e-3


def test_reordered_equals_usual_order():
    """Slide_f of every input, multiply by the un-rotated filter plaintexts, add (RAConv before reordering):
    same slots as the reordered form up to key-switching noise."""
    prm, cl, g2, x, w1, w2, mid, p2, evks, out, inter, orc = _chain(C_a=8, H=8, W=8, c_mid=8, level=3)
    level, mods = 2, [0, 1, 2]
    total = None
    for i in range(g2.n_in):
        for t, step in enumerate(g2.tap_steps):
            slid = mid[i] if step == 0 else orc.rotate(mid[i], level, orc.galois_elt(step), evks[step])
            m = K.encode(g2.filter_slots(w2, i, t).astype(np.complex128), prm.N, float(prm.q[level]))
            total = orc.ptct_mac(total, slid, orc.ntt(orc.reduce_signed(m, mods), mods), level, init=total is None)
    usual = cl.decrypt(orc.rescale(total, level), 1, prm.scale)
    assert np.max(np.abs(usual - cl.decrypt(out, 1, prm.scale))) < 1e-4
    # the count the paper gives: f^2-1 rotations for the reordered form against n_in*(f^2-1)
    assert sum(1 for s in g2.tap_steps if s) == 8


def test_gap_sum_and_replication_closes_the_cycle():
    """CAConv -> RAConv with two channels per ciphertext -> sum across the gap and re-replication: the result is
    the channel-aligned, replicated packing of conv(conv(x)), i.e. a valid input of the next CAConv."""
    from oracle import block as OB
    prm = toy_params(logN=10, q_bits=40, nq=5, p_bits=41, np_=2, dnum=3, scale=2.0 ** 30, hamming=32, seed=101)
    rng = S.make_rng(101)
    orc = Oracle.from_params(prm)
    cl = K.Client(orc, S.ternary_secret(rng, prm.N, prm.hamming))
    N, q, slots = prm.N, prm.q, prm.N // 2
    C_a, H, W, c, level = 4, 8, 8, 8, 4
    g1, g2 = CV.ConvGeometry(N, C_a, H, W, c, f=3), CV.RAGeometry(N, C_a, H, W, c, f=3)
    assert g2.R == 2
    x, w1 = S.conv_tensors(rng, C_a, c, H, W, 3, 0.2)
    w2 = rng.normal(0.0, 0.2, size=(C_a, c, 3, 3))
    steps = sorted(set(s for s in g1.tap_steps if s) | set(g1.ras_steps) | {1, slots - 1})
    evks = {st: cl.rotation_key(orc.galois_elt(st), S.uniform_limbs(rng, prm.moduli, N, prm.dnum),
                                S.gaussian_error(rng, N, prm.sigma, prm.dnum)) for st in steps}
    ct = cl.encrypt(g1.pack_input(x).astype(np.complex128), prm.scale, level,
                    S.uniform_limbs(rng, q[:level + 1], N)[0], S.gaussian_error(rng, N, prm.sigma)[0])
    mid = CV.caconv(orc, g1, ct, level, CV.encode_weights(orc, g1, w1, level, float(q[level])), evks)
    out = CV.raconv(orc, g2, mid, level - 1, CV.encode_ra_weights(orc, g2, w2, level - 1, float(q[level - 1])), evks)
    fin = OB.gap_sum_replicate(orc, out, level - 2, g2.R, OB.gap_mask(orc, g2, level - 2, float(q[level - 2])), evks)
    ref = CV.conv2d_float(CV.conv2d_float(x, w1), w2)
    assert np.max(np.abs(cl.decrypt(fin, level - 3, prm.scale).real - g1.pack_input(ref))) < 1e-3
