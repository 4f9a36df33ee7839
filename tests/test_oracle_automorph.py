"""Pins for the Galois automorphism: evaluation definition, composition, both forms agree."""
import numpy as np
import pytest

import pyref
from he_inputs import sampling as S
from he_inputs.params import config_params, toy_params
from oracle.he_oracle import Oracle


@pytest.mark.parametrize("logN", [3, 5])
def test_coef_form_is_substitution_x_to_x_g(logN):
    prm = toy_params(logN=logN, nq=2, np_=1)
    o = Oracle.from_params(prm)
    rng = S.make_rng(11)
    N = prm.N
    a = S.uniform_limbs(rng, prm.moduli, N)[0]
    for g in (5, 25 % (2 * N), 2 * N - 1, 3):
        out = o.automorph_coef(a, range(3), g)
        for i, q in enumerate(prm.moduli):
            psi = pyref.smallest_qnr_root(q, N)
            for e in (1, 3, 2 * N - 1):
                x = pow(psi, e, q)  # a root of X^N + 1
                assert pyref.poly_eval([int(v) for v in out[i]], x, q) == pyref.poly_eval([int(v) for v in a[i]], pow(x, g, q), q)


@pytest.mark.parametrize("logN", [4, 10])
def test_ntt_form_matches_coef_form_and_composes(logN):
    prm = toy_params(logN=logN, nq=2, np_=1)
    o = Oracle.from_params(prm)
    rng = S.make_rng(12)
    N = prm.N
    mods = [0, 1, 2]
    a = S.uniform_limbs(rng, prm.moduli, N)[0]
    A = o.ntt(a, mods)
    g, h = o.galois_elt(3), o.galois_elt(N // 2 - 5)
    for gg in (g, h, o.galois_conj):
        assert (o.ntt(o.automorph_coef(a, mods, gg), mods) == o.automorph_ntt(A, gg)).all()
    gh = g * h % (2 * N)
    assert (o.automorph_ntt(o.automorph_ntt(A, g), h) == o.automorph_ntt(A, gh)).all()
    assert (o.automorph_coef(o.automorph_coef(a, mods, g), mods, h) == o.automorph_coef(a, mods, gh)).all()
    # sigma_g is a ring homomorphism: sigma(a*b) = sigma(a)*sigma(b) (pointwise in NTT form)
    b = S.uniform_limbs(rng, prm.moduli, N)[0]
    B = o.ntt(b, mods)
    assert (o.automorph_ntt(o.pointwise_mul(A, B, mods), g) == o.pointwise_mul(o.automorph_ntt(A, g), o.automorph_ntt(B, g), mods)).all()
    # identity and inverse
    assert (o.automorph_ntt(A, 1) == A).all()
    ginv = pow(g, -1, 2 * N)
    assert (o.automorph_ntt(o.automorph_ntt(A, g), ginv) == A).all()


def test_forms_agree_n65536():
    prm = config_params(2)
    o = Oracle.from_params(prm)
    rng = S.make_rng(13)
    mods = [3, 31]
    a = S.uniform_limbs(rng, [prm.moduli[i] for i in mods], prm.N)[0]
    g = o.galois_elt(1 << 14)
    assert (o.ntt(o.automorph_coef(a, mods, g), mods) == o.automorph_ntt(o.ntt(a, mods), g)).all()


@pytest.mark.parametrize("logN", [9, 12, 16])
def test_rotations_by_multiples_of_n_over_512_stay_inside_blocks_of_256_positions(logN):
    """The layout fact that the LDS-staged hoisted sums rest on: in NTT form (bit-reversed evaluation order) a
    rotation by a multiple of N/2^(b+1) slots permutes every aligned block of 2^b positions within itself - b = 8 is a
    work group's tile, b = 4 holds for the rotate-and-sum amounts over up to 16 channel blocks - and a rotation by half
    that amount does not."""
    prm = toy_params(logN=logN, nq=1, np_=1) if logN < 16 else config_params(1)
    o = Oracle.from_params(prm)
    N = prm.N
    pos = np.arange(N, dtype=np.uint64)                     # out[n] = pos[src(n)] = src(n)
    for b in (8, 4):
        if N >> (b + 1) == 0:
            continue
        unit = N >> (b + 1)
        for mult in (1, 2, 3, (1 << b) - 1):
            src = o.automorph_ntt(pos, o.galois_elt(unit * mult)).astype(np.int64)
            assert sorted(src.tolist()) == list(range(N))
            assert ((src >> b) == (np.arange(N) >> b)).all(), (logN, b, mult)
        if unit >= 2:
            src = o.automorph_ntt(pos, o.galois_elt(unit // 2)).astype(np.int64)
            assert not ((src >> b) == (np.arange(N) >> b)).all()
