"""Pins of CAConv's Slide_f + MulFilter&Sum_f evaluated with one ModDown per output (the filter plaintexts
multiply the key-switch inner products over the raised basis; Algorithm 1 with the ModDown deferred across the
sum over the taps).

What fixes the function: (i) in exact integers on a tiny ring, the phase out0 + out1*s of every output equals
sum_t pt_t * sigma_{g_t}(c0 + c1*s) up to an error far below one ModDown rounding per tap times the plaintext
size (which is what the tap-by-tap order carries), so a dropped tap, a wrong Galois element or a plaintext taken
modulo the wrong prime fails; (ii) the plaintexts over the raised basis agree with the ordinary ones on the
ciphertext primes and are the same integer polynomial on the special primes; (iii) the whole layer decrypts to
the float64 convolution at the tolerance of the tap-by-tap order and agrees with it far below that tolerance;
(iv) with a single tap that does not rotate, nothing is switched and the result is the plain product."""
import numpy as np
import pytest

import pyref
from he_inputs import sampling as S
from he_inputs.params import config_params, toy_params
from oracle import ckks_client as K
from oracle import conv2d as CV
from oracle.he_oracle import Oracle


def _keys(o, cl, prm, rng, steps):
    return {st: cl.rotation_key(o.galois_elt(st), S.uniform_limbs(rng, prm.moduli, prm.N, prm.dnum),
                                S.gaussian_error(rng, prm.N, prm.sigma, prm.dnum)) for st in steps}


def _lift(orc, poly, qs):
    mods = list(range(len(qs)))
    c = orc.intt(poly, mods)
    out = []
    for n in range(orc.N):
        v, Q = pyref.crt([c[i][n] for i in mods], qs)
        out.append(pyref.center(v, Q))
    return out


def _sigma_int(poly, g, N, Q):
    out = [0] * N
    for i in range(N):
        t = (i * g) % (2 * N)
        if t < N:
            out[t] = (out[t] + poly[i]) % Q
        else:
            out[t - N] = (out[t - N] - poly[i]) % Q
    return out


@pytest.mark.parametrize("level", [2, 1])
def test_phase_relation_in_exact_integers(level):
    prm = toy_params(logN=5, q_bits=30, nq=3, p_bits=31, np_=2, dnum=3, scale=2.0 ** 20, hamming=8, seed=51)
    rng = S.make_rng(51 + level)
    orc = Oracle.from_params(prm)
    cl = K.Client(orc, S.ternary_secret(rng, prm.N, prm.hamming))
    N, qs = prm.N, prm.q[:level + 1]
    Q = int(np.prod([int(q) for q in qs], dtype=object))
    geo = CV.ConvGeometry(N, 2, 2, 2, 2)                       # R = 2, one output ciphertext, 9 taps
    x, wt = S.conv_tensors(rng, 2, 2, 2, 2, 3, 0.3)
    evks = _keys(orc, cl, prm, rng, sorted(set(s for s in geo.tap_steps if s)))
    ct = np.stack([S.uniform_limbs(rng, qs, N)[0] for _ in range(2)])      # any ciphertext: the relation is algebraic
    pt_scale = 2.0 ** 12
    pts = CV.encode_weights_raised(orc, geo, wt, level, pt_scale)
    outs = CV.slide_mac_deferred(orc, geo, ct, level, pts, evks)
    s = [int(v) for v in cl.s]

    def phase(c):
        c0, c1 = _lift(orc, c[0], qs), _lift(orc, c[1], qs)
        c1s = pyref.negacyclic_mul_int(c1, s)
        return [(c0[n] + c1s[n]) % Q for n in range(N)]

    ph = phase(ct)
    for o in range(geo.n_out):
        want = [0] * N
        for t, step in enumerate(geo.tap_steps):
            w = _lift(orc, pts[o, t, :level + 1], qs)           # the plaintext's integer polynomial (|coeff| << Q)
            rot = _sigma_int(ph, orc.galois_elt(step), N, Q)
            prod = pyref.negacyclic_mul_int(w, rot)
            want = [(want[n] + prod[n]) % Q for n in range(N)]
        got = phase(outs[o])
        noise = max(abs(pyref.center((got[n] - want[n]) % Q, Q)) for n in range(N))
        # one ModDown rounding (at most the number of special primes) plus key-switch noise scaled down by P: a
        # handful of units.  The tap-by-tap order carries one rounding per tap times the plaintext (2^14 here), so
        # this bound also shows that the ModDown really is taken once, after the products
        assert noise < 2 ** 8, noise
        assert max(abs(pyref.center(v, Q)) for v in want) > Q >> 6                           # not vacuous: noise is 2^-50 of it


def test_raised_plaintexts_are_the_same_polynomial():
    prm = toy_params(logN=5, q_bits=30, nq=3, p_bits=31, np_=2, dnum=3, scale=2.0 ** 20, hamming=8, seed=52)
    rng = S.make_rng(52)
    orc = Oracle.from_params(prm)
    geo = CV.ConvGeometry(prm.N, 2, 2, 2, 2)
    _, wt = S.conv_tensors(rng, 2, 2, 2, 2, 3, 0.3)
    level = 1
    a = CV.encode_weights(orc, geo, wt, level, 2.0 ** 12)
    b = CV.encode_weights_raised(orc, geo, wt, level, 2.0 ** 12)
    rm = orc.raised_moduli(level)
    assert b.shape[2] == len(rm) == level + 1 + 2
    assert (b[:, :, :level + 1] == a).all()
    # on the special primes: the centred integer polynomial recovered from the ciphertext primes, reduced
    qs = prm.q[:level + 1]
    for t in (0, 4, 8):
        w = _lift(orc, a[0, t], qs)
        for i, mi in enumerate(rm[level + 1:]):
            p = int(prm.moduli[mi])
            coef = orc.intt(b[0, t, level + 1 + i:level + 2 + i], [mi])[0]
            assert [int(v) for v in coef] == [v % p for v in w]


def _layer(prm, C_a, H, W, c_out, level, w_std, tol, seed):
    rng = S.make_rng(seed)
    o = Oracle.from_params(prm)
    cl = K.Client(o, S.ternary_secret(rng, prm.N, prm.hamming))
    geo = CV.ConvGeometry(prm.N, C_a, H, W, c_out)
    x, wt = S.conv_tensors(rng, C_a, c_out, H, W, 3, w_std)
    evks = _keys(o, cl, prm, rng, sorted(set(s for s in geo.tap_steps if s) | set(geo.ras_steps)))
    ct = cl.encrypt(geo.pack_input(x).astype(np.complex128), prm.scale, level,
                    S.uniform_limbs(rng, prm.q[:level + 1], prm.N)[0], S.gaussian_error(rng, prm.N, prm.sigma)[0])
    pts_r = CV.encode_weights_raised(o, geo, wt, level, float(prm.q[level]))
    outs = CV.caconv(o, geo, ct, level, pts_r, evks, deferred_taps=True)
    ref_order = CV.caconv(o, geo, ct, level, np.ascontiguousarray(pts_r[:, :, :level + 1]), evks)
    dec = [cl.decrypt(c, level - 1, prm.scale) for c in outs]
    dec_ref = [cl.decrypt(c, level - 1, prm.scale) for c in ref_order]
    got, spread = geo.unpack_output(dec)
    err = np.max(np.abs(got - CV.conv2d_float(x, wt)))
    assert err < tol and spread < tol, (err, spread)
    gap = max(np.max(np.abs(np.asarray(a) - np.asarray(b))) for a, b in zip(dec, dec_ref))
    assert gap < tol, gap
    assert any((a != b).any() for a, b in zip(outs, ref_order))          # a different rounding, not the same bits
    return gap, err


def test_layer_decrypts_to_float_convolution_tiny_ring():
    prm = toy_params(logN=6, q_bits=30, nq=3, p_bits=31, np_=1, dnum=3, scale=2.0 ** 24, hamming=8, seed=41)
    _layer(prm, C_a=2, H=2, W=2, c_out=2, level=2, w_std=0.3, tol=2e-3, seed=53)


def test_layer_decrypts_to_float_convolution_config0():
    _layer(config_params(0), C_a=4, H=8, W=8, c_out=4, level=2, w_std=0.1, tol=1e-3, seed=54)


def test_single_tap_is_the_plain_product():
    prm = toy_params(logN=5, q_bits=30, nq=3, p_bits=31, np_=2, dnum=3, scale=2.0 ** 20, hamming=8, seed=55)
    rng = S.make_rng(55)
    orc = Oracle.from_params(prm)
    level, N = 2, prm.N
    geo = CV.ConvGeometry(N, 2, 2, 2, 2, f=1)
    _, wt = S.conv_tensors(rng, 2, 2, 2, 2, 1, 0.3)
    ct = np.stack([S.uniform_limbs(rng, prm.q[:level + 1], N)[0] for _ in range(2)])
    pts = CV.encode_weights_raised(orc, geo, wt, level, 2.0 ** 12)
    out = CV.slide_mac_deferred(orc, geo, ct, level, pts, {})[0]
    want = orc.ptct_mac(None, ct, np.ascontiguousarray(pts[0, 0, :level + 1]), level, init=True)
    assert (out == want).all()


def test_hoisted_rotate_and_sum_is_the_same_sum():
    """RaS over C_a as one hoisted sum of its C_a - 1 rotations (one ModUp, one ModDown per output): decrypts to the
    float64 convolution, leaves the sum in every channel block, agrees with the stepwise form far below the
    tolerance and is not the same bits.  (The sum of rotations with one ModDown is pinned in exact integers by the
    tests of rotate_sum_deferred; that the hoisted form feeds it the right rotations is what this test fixes: a
    missing or repeated multiple of H*W*R breaks the replication across blocks.)"""
    prm = toy_params(logN=8, q_bits=40, nq=3, p_bits=41, np_=1, dnum=3, scale=2.0 ** 30, hamming=16, seed=56)
    rng = S.make_rng(56)
    o = Oracle.from_params(prm)
    cl = K.Client(o, S.ternary_secret(rng, prm.N, prm.hamming))
    level = 2
    geo = CV.ConvGeometry(prm.N, 8, 2, 2, 4)                    # C_a = 8: 7 rotations instead of 3 steps
    x, wt = S.conv_tensors(rng, 8, 4, 2, 2, 3, 0.2)
    base = geo.H * geo.W * geo.R
    steps = sorted(set(s for s in geo.tap_steps if s) | set(base * i for i in range(1, geo.C_a)))
    evks = _keys(o, cl, prm, rng, steps)
    ct = cl.encrypt(geo.pack_input(x).astype(np.complex128), prm.scale, level,
                    S.uniform_limbs(rng, prm.q[:level + 1], prm.N)[0], S.gaussian_error(rng, prm.N, prm.sigma)[0])
    pts = CV.encode_weights(o, geo, wt, level, float(prm.q[level]))
    a = CV.caconv(o, geo, ct, level, pts, evks, hoisted_ras=True)
    b = CV.caconv(o, geo, ct, level, pts, evks)
    da = [cl.decrypt(c, level - 1, prm.scale) for c in a]
    db = [cl.decrypt(c, level - 1, prm.scale) for c in b]
    got, spread = geo.unpack_output(da)
    assert np.max(np.abs(got - CV.conv2d_float(x, wt))) < 1e-3 and spread < 1e-3
    assert max(np.max(np.abs(np.asarray(u) - np.asarray(v))) for u, v in zip(da, db)) < 1e-3
    assert any((u != v).any() for u, v in zip(a, b))


def test_hoisted_rotate_and_sum_is_the_pinned_rotation_sum():
    """ras_hoisted writes the sum out with its single ModUp; it must be, bit for bit, rotate_sum_deferred (the function
    pinned in exact integers) applied to the ciphertext repeated C_a times with the Galois elements 1, g, g^2, ..."""
    prm = toy_params(logN=8, q_bits=40, nq=3, p_bits=41, np_=1, dnum=3, scale=2.0 ** 30, hamming=16, seed=57)
    rng = S.make_rng(57)
    o = Oracle.from_params(prm)
    cl = K.Client(o, S.ternary_secret(rng, prm.N, prm.hamming))
    geo = CV.ConvGeometry(prm.N, 8, 2, 2, 4)
    base = geo.H * geo.W * geo.R
    steps = [base * i for i in range(1, geo.C_a)]
    evks = _keys(o, cl, prm, rng, steps)
    for level in (2, 1):
        cur = np.stack([S.uniform_limbs(rng, prm.q[:level + 1], prm.N)[0] for _ in range(2)])
        a = CV.ras_hoisted(o, geo, cur, level, evks)
        b = o.rotate_sum_deferred([cur] * geo.C_a, level, [1] + [o.galois_elt(s) for s in steps], [None] + [evks[s] for s in steps])
        assert (a == b).all()

