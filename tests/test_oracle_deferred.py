"""Pins of the oracle's rotation sum with a deferred ModDown (Slide_1 & Sum_f of Algorithm 2 with one
ModDown for the whole sum) and of RAConv evaluated that way.

What fixes the function: (i) in exact integers on a tiny ring, out0 + out1*s equals the sum of the rotated
phases sigma_g(c0 + c1*s) up to a small error; (ii) its ModDown really is taken once, on the sum of the
accumulators: P*ks = A - [A]_P lifted, checked with Python integers from the accumulators re-derived here;
(iii) the decrypted result is the sum of the rolled messages; (iv) a term with g = 1 is added as is;
(v) a single term reproduces the ordinary rotation bit for bit; (vi) RAConv with it decrypts to the float64
convolution chain."""
import numpy as np
import pytest

import pyref
from he_inputs import sampling as S
from he_inputs.params import toy_params
from oracle import ckks_client as K
from oracle import conv2d as CV
from oracle.he_oracle import Oracle


def _setup(logN, seed, **kw):
    prm = toy_params(logN=logN, **kw)
    orc = Oracle.from_params(prm)
    rng = S.make_rng(seed)
    cl = K.Client(orc, S.ternary_secret(rng, prm.N, prm.hamming))
    return prm, orc, rng, cl


def _key(prm, rng, cl, g):
    return cl.rotation_key(g, S.uniform_limbs(rng, prm.moduli, prm.N, prm.dnum), S.gaussian_error(rng, prm.N, prm.sigma, prm.dnum))


def _lift(orc, poly, qs):
    """NTT-form limbs -> centred integer coefficients by CRT."""
    mods = list(range(len(qs)))
    c = orc.intt(poly, mods)
    out = []
    for n in range(orc.N):
        v, Q = pyref.crt([c[i][n] for i in mods], qs)
        out.append(pyref.center(v, Q))
    return out


@pytest.mark.parametrize("level", [5, 4, 2])
def test_phase_relation_in_exact_integers(level):
    prm, orc, rng, cl = _setup(4, 31)
    N, qs = prm.N, prm.q[:level + 1]
    Q = 1
    for q in qs:
        Q *= q
    steps = [1, 3, 0, N // 2 - 2]
    gs = [orc.galois_elt(s) for s in steps]
    evks = [None if g == 1 else _key(prm, rng, cl, g) for g in gs]
    cts = [np.stack([S.uniform_limbs(rng, qs, N)[0] for _ in range(2)]) for _ in steps]
    out = orc.rotate_sum_deferred(cts, level, gs, evks)
    s = [int(v) for v in cl.s]

    def phase(ct):
        c0, c1 = _lift(orc, ct[0], qs), _lift(orc, ct[1], qs)
        c1s = pyref.negacyclic_mul_int(c1, s)
        return [(c0[n] + c1s[n]) % Q for n in range(N)]

    want = [0] * N
    for ct, g in zip(cts, gs):
        ph = phase(ct)
        for i in range(N):                                   # sigma_g on integer coefficients: X^i -> X^(i g), X^N = -1
            t = (i * g) % (2 * N)
            if t < N:
                want[t] = (want[t] + ph[i]) % Q
            else:
                want[t - N] = (want[t - N] - ph[i]) % Q
    got = phase(out)
    noise = [pyref.center((got[n] - want[n]) % Q, Q) for n in range(N)]
    assert max(abs(v) for v in noise) < 2 ** 15, max(abs(v) for v in noise)
    assert max(abs(pyref.center(v, Q)) for v in want) > 2 ** 60          # the relation is not vacuous


def test_single_moddown_on_the_summed_accumulators():
    """ks_c = (A_c - lift([A_c]_P converted)) / P with A_c the sum of the per-term inner products, in Python
    integers: the conversion of the special-prime part is the fast one (x + u*P, 0 <= u < k), so
    P*ks_c = A_c - (a_P + u*P) for one u in [0, k) per coefficient, where a_P = [A_c]_P in [0, P)."""
    prm, orc, rng, cl = _setup(4, 32)
    N, level = prm.N, 5
    qs, ps = prm.q[:level + 1], prm.p
    P = 1
    for p in ps:
        P *= p
    steps = [1, 2, 5]
    gs = [orc.galois_elt(s) for s in steps]
    evks = [_key(prm, rng, cl, g) for g in gs]
    cts = [np.stack([S.uniform_limbs(rng, qs, N)[0] for _ in range(2)]) for _ in steps]
    out = orc.rotate_sum_deferred(cts, level, gs, evks)
    rm = orc.raised_moduli(level)
    mods = [prm.moduli[i] for i in rm]
    # the accumulators, re-derived term by term and summed in Python integers per limb
    A = np.zeros((2, len(rm), N), dtype=object)
    rot0 = np.zeros((level + 1, N), dtype=object)
    for ct, g, evk in zip(cts, gs, evks):
        ip = orc.inner_product(orc.automorph_ntt(orc.modup(ct[1], level), g), level, evk)
        A += ip.astype(object)
        rot0 += orc.automorph_ntt(ct[0], g).astype(object)
    for comp in range(2):
        Ared = np.stack([np.array([int(v) % mods[r] for v in A[comp][r]], dtype=np.uint64) for r in range(len(rm))])
        coef = orc.intt(Ared, rm)                                                    # coefficient form, every raised limb
        ks = out[comp].astype(object)
        if comp == 0:
            ks = (ks - rot0) % np.array(qs, dtype=object)[:, None]
        ksc = orc.intt(np.stack([np.array([int(v) for v in ks[r]], dtype=np.uint64) for r in range(level + 1)]), range(level + 1))
        for n in range(N):
            aP, _ = pyref.crt([coef[level + 1 + t][n] for t in range(len(ps))], ps)
            us = set()
            for r, q in enumerate(qs):
                u = [u for u in range(len(ps)) if (int(ksc[r][n]) * P - int(coef[r][n]) + aP + u * P) % q == 0]
                assert len(u) == 1, (comp, n, r)
                us.add(u[0])
            assert len(us) == 1


def test_decrypts_to_sum_of_rolled_messages_and_single_term_is_a_rotation():
    prm, orc, rng, cl = _setup(8, 33, q_bits=40, nq=6, p_bits=41, np_=2, dnum=3, scale=2.0 ** 30, hamming=16)
    N, level = prm.N, 5
    steps = [3, 0, N // 2 - 7, 16]
    gs = [orc.galois_elt(s) for s in steps]
    evks = [None if g == 1 else _key(prm, rng, cl, g) for g in gs]
    zs = [rng.uniform(-1, 1, N // 2) + 1j * rng.uniform(-1, 1, N // 2) for _ in steps]
    cts = [cl.encrypt(z, prm.scale, level, S.uniform_limbs(rng, prm.q[:level + 1], N)[0], S.gaussian_error(rng, N, prm.sigma)[0]) for z in zs]
    out = orc.rotate_sum_deferred(cts, level, gs, evks)
    want = sum(np.roll(z, -s) for z, s in zip(zs, steps))
    assert np.max(np.abs(cl.decrypt(out, level, prm.scale) - want)) < 1e-4
    # differs in bits from the term-by-term sum (ModDown does not distribute), agrees in value
    tbt = None
    for ct, g, evk in zip(cts, gs, evks):
        term = ct if g == 1 else orc.rotate(ct, level, g, evk)
        tbt = term if tbt is None else orc.add(tbt, term, level)
    assert not (tbt == out).all()
    assert np.max(np.abs(cl.decrypt(tbt, level, prm.scale) - cl.decrypt(out, level, prm.scale))) < 1e-5
    # one rotated term alone: identical to the ordinary rotation; only unrotated terms: their plain sum
    assert (orc.rotate_sum_deferred(cts[:1], level, gs[:1], evks[:1]) == orc.rotate(cts[0], level, gs[0], evks[0])).all()
    assert (orc.rotate_sum_deferred([cts[1], cts[1]], level, [1, 1], [None, None]) == orc.add(cts[1], cts[1], level)).all()


def test_raconv_deferred_matches_float_chain():
    prm = toy_params(logN=10, q_bits=40, nq=4, p_bits=41, np_=2, dnum=2, scale=2.0 ** 30, hamming=32, seed=94)
    rng = S.make_rng(95)
    orc = Oracle.from_params(prm)
    cl = K.Client(orc, S.ternary_secret(rng, prm.N, prm.hamming))
    N, C_a, H, W, c_mid, level = prm.N, 8, 8, 8, 8, 3
    g1 = CV.ConvGeometry(N, C_a, H, W, c_mid, f=3)
    g2 = CV.RAGeometry(N, C_a, H, W, c_mid, f=3)
    x, w1 = S.conv_tensors(rng, C_a, c_mid, H, W, 3, 0.2)
    w2 = rng.normal(0.0, 0.2, size=(C_a, c_mid, 3, 3))
    steps = sorted(set(s for s in g1.tap_steps if s) | set(g1.ras_steps) | set(s for s in g2.tap_steps if s))
    evks = {st: _key(prm, rng, cl, orc.galois_elt(st)) for st in steps}
    ct = cl.encrypt(g1.pack_input(x).astype(np.complex128), prm.scale, level,
                    S.uniform_limbs(rng, prm.q[:level + 1], N)[0], S.gaussian_error(rng, N, prm.sigma)[0])
    mid = CV.caconv(orc, g1, ct, level, CV.encode_weights(orc, g1, w1, level, float(prm.q[level])), evks)
    p2 = CV.encode_ra_weights(orc, g2, w2, level - 1, float(prm.q[level - 1]))
    out, inter = CV.raconv(orc, g2, mid, level - 1, p2, evks, deferred=True, keep=True)
    ref, inter_ref = CV.raconv(orc, g2, mid, level - 1, p2, evks, keep=True)
    y = CV.conv2d_float(CV.conv2d_float(x, w1), w2)
    z = cl.decrypt(out, 1, prm.scale).real.reshape(C_a, H, W)
    assert np.max(np.abs(z - y)) < 1e-3
    # before the rescale the two evaluation orders differ in bits (the rescale's rounding hides most of it) ...
    assert not (inter["sum"] == inter_ref["sum"]).all()
    assert np.max(np.abs(cl.decrypt(ref, 1, prm.scale).real.reshape(C_a, H, W) - z)) < 1e-5   # ... same message
