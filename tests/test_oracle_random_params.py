"""Randomised parameter sets (ring size, number of primes, digits, special primes, level) against the scheme's
semantics: Dec(Rot_r(Enc z)) = roll(z, -r), hoisted == single, Dec(Rescale(MulPt)) = z*w.  Seeded."""
import numpy as np
import pytest

from he_inputs import sampling as S
from he_inputs.params import toy_params
from oracle import ckks_client as K
from oracle.he_oracle import Oracle


def _draw(rng):
    logN = int(rng.integers(4, 9))
    nq = int(rng.integers(2, 8))
    dnum = int(rng.integers(1, nq + 1))
    alpha = -(-nq // dnum)
    np_ = int(rng.integers(alpha, alpha + 3))
    level = int(rng.integers(0, nq))
    return logN, nq, dnum, np_, level


@pytest.mark.parametrize("case", range(12))
def test_random_parameter_sets(case):
    rng = S.make_rng(1000 + case)
    logN, nq, dnum, np_, level = _draw(rng)
    prm = toy_params(logN=logN, q_bits=30, nq=nq, p_bits=31, np_=np_, dnum=dnum, scale=2.0 ** 22, hamming=min(8, 1 << (logN - 1)),
                     seed=1000 + case)
    o = Oracle.from_params(prm)
    cl = K.Client(o, S.ternary_secret(rng, prm.N, prm.hamming))
    N = prm.N
    z = rng.uniform(-1, 1, N // 2) + 1j * rng.uniform(-1, 1, N // 2)
    ct = cl.encrypt(z, prm.scale, level, S.uniform_limbs(rng, prm.q[:level + 1], N)[0], S.gaussian_error(rng, N, prm.sigma)[0])
    assert np.max(np.abs(cl.decrypt(ct, level, prm.scale) - z)) < 1e-3
    r = int(rng.integers(1, N // 2))
    g = o.galois_elt(r)
    key = cl.rotation_key(g, S.uniform_limbs(rng, prm.moduli, N, prm.dnum), S.gaussian_error(rng, N, prm.sigma, prm.dnum))
    rot = o.rotate(ct, level, g, key)
    # key-switching noise grows with the digit size relative to the special modulus; the sets drawn here keep
    # P at least as large as a digit, so the error stays at the scale of the encryption noise
    assert np.max(np.abs(cl.decrypt(rot, level, prm.scale) - np.roll(z, -r))) < 5e-3, (logN, nq, dnum, np_, level)
    assert (o.rotate_from_raised(ct, o.modup(ct[1], level), level, g, key) == rot).all()
    if level >= 1:
        w = rng.uniform(-1, 1, N // 2)
        mods = list(range(level + 1))
        pt = o.ntt(o.reduce_signed(K.encode(w.astype(np.complex128), N, float(prm.q[level])), mods), mods)
        prod = o.rescale(o.ptct_mac(None, ct, pt, level, init=True), level)
        assert np.max(np.abs(cl.decrypt(prod, level - 1, prm.scale) - z * w)) < 5e-3
