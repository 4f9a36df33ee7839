"""Pins for the oracle's negacyclic NTT: worked example, definition, convolution theorem,
round trip, linearity, root rule."""
import os

import numpy as np
import pytest

import pyref
from he_inputs import sampling as S
from he_inputs.params import config_params, toy_params
from oracle.he_oracle import Oracle, lib

GOLD = os.path.join(os.path.dirname(__file__), "golden", "ntt_n8_q17.txt")


def _gold():
    out = {}
    for line in open(GOLD):
        if line.startswith("#") or not line.strip():
            continue
        t = line.split()
        out[t[0]] = [int(x) for x in t[1:]]
    return out


def test_worked_example_n8_q17():
    g = _gold()
    o = Oracle(3, [17], [], 1)
    assert o.psi(0) == g["psi"][0] == pyref.smallest_qnr_root(17, 8)
    a = np.array(g["a"], dtype=np.uint64)
    # fixture is self-consistent with the definition (evaluation at odd powers of psi)
    assert [pyref.poly_eval(g["a"], pow(3, 2 * k + 1, 17), 17) for k in range(8)] == g["eval_natural"]
    assert [g["eval_natural"][pyref.brv(j, 3)] for j in range(8)] == g["ntt"]
    assert o.ntt(a.reshape(1, 8), [0])[0].tolist() == g["ntt"]
    assert o.ntt_def(a, 0).tolist() == g["ntt"]
    assert pyref.negacyclic_mul(g["a"], g["a"], 17) == g["a_squared"]
    sq = o.pointwise_mul(o.ntt(a.reshape(1, 8), [0]), o.ntt(a.reshape(1, 8), [0]), [0])
    assert o.intt(sq, [0])[0].tolist() == g["a_squared"]
    assert o.automorph_coef(a.reshape(1, 8), [0], 5)[0].tolist() == g["sigma5_coef"]
    assert o.automorph_ntt(np.array(g["ntt"], dtype=np.uint64).reshape(1, 8), 5)[0].tolist() == g["sigma5_ntt"]
    idx = o.automorph_ntt(np.arange(8, dtype=np.uint64).reshape(1, 8), 5)[0].tolist()
    assert idx == g["pi5"]


@pytest.mark.parametrize("logN", [1, 2, 4, 6])
def test_fast_ntt_equals_evaluation_definition(logN):
    prm = toy_params(logN=logN, nq=3, np_=1)
    o = Oracle.from_params(prm)
    rng = S.make_rng(100 + logN)
    a = S.uniform_limbs(rng, prm.moduli, prm.N)[0]
    mods = list(range(len(prm.moduli)))
    A = o.ntt(a, mods)
    for i, q in enumerate(prm.moduli):
        psi = pyref.smallest_qnr_root(q, prm.N)
        assert psi == o.psi(i)
        assert pow(psi, prm.N, q) == q - 1
        assert A[i].tolist() == pyref.ntt_by_evaluation([int(x) for x in a[i]], psi, q)
        assert o.ntt_def(a[i], i).tolist() == A[i].tolist()
    assert (o.intt(A, mods) == a).all()


def test_fast_ntt_equals_c_definition_n1024_wide_primes():
    # 54- and 60-bit primes exercise the full 128-bit product path
    from he_inputs.params import ntt_primes
    q = ntt_primes(54, 2048, 2) + ntt_primes(60, 2048, 1) + ntt_primes(62, 2048, 1)
    o = Oracle(10, q, [], 1)
    rng = S.make_rng(5)
    a = S.uniform_limbs(rng, q, 1024)[0]
    A = o.ntt(a, range(4))
    for i in range(4):
        assert (o.ntt_def(a[i], i) == A[i]).all()
    # spot-check entries against Python integers
    for i in range(4):
        psi = pyref.smallest_qnr_root(q[i], 1024)
        assert psi == o.psi(i)
        for j in (0, 1, 513, 1023):
            assert int(A[i][j]) == pyref.poly_eval([int(x) for x in a[i]], pow(psi, 2 * pyref.brv(j, 10) + 1, q[i]), q[i])


@pytest.mark.parametrize("logN", [3, 5])
def test_convolution_theorem_vs_schoolbook(logN):
    prm = toy_params(logN=logN, nq=2, np_=1)
    o = Oracle.from_params(prm)
    rng = S.make_rng(7)
    a = S.uniform_limbs(rng, prm.moduli, prm.N)[0]
    b = S.uniform_limbs(rng, prm.moduli, prm.N)[0]
    mods = list(range(3))
    c = o.intt(o.pointwise_mul(o.ntt(a, mods), o.ntt(b, mods), mods), mods)
    for i, q in enumerate(prm.moduli):
        ref = pyref.negacyclic_mul([int(x) for x in a[i]], [int(x) for x in b[i]], q)
        assert c[i].tolist() == ref
        assert o.negacyclic_mul_def(a[i], b[i], i).tolist() == ref


def test_convolution_theorem_n2048_c_schoolbook():
    from he_inputs.params import ntt_primes
    q = ntt_primes(54, 4096, 1) + ntt_primes(60, 4096, 1)
    o = Oracle(11, q, [], 1)
    rng = S.make_rng(8)
    a, b = S.uniform_limbs(rng, q, 2048)[0], S.uniform_limbs(rng, q, 2048)[0]
    c = o.intt(o.pointwise_mul(o.ntt(a, [0, 1]), o.ntt(b, [0, 1]), [0, 1]), [0, 1])
    for i in range(2):
        assert (c[i] == o.negacyclic_mul_def(a[i], b[i], i)).all()


def test_roundtrip_and_linearity_n65536():
    prm = config_params(1)
    o = Oracle.from_params(prm)
    rng = S.make_rng(1)
    mods = [0, 23, 24, 31]
    ms = [prm.moduli[i] for i in mods]
    a = S.uniform_limbs(rng, ms, prm.N)[0]
    b = S.uniform_limbs(rng, ms, prm.N)[0]
    A, B = o.ntt(a, mods), o.ntt(b, mods)
    assert (o.intt(A, mods) == a).all()
    s = np.stack([(a[i].astype(object) + b[i].astype(object)) % ms[i] for i in range(4)]).astype(np.uint64)
    Ssum = np.stack([(A[i].astype(object) + B[i].astype(object)) % ms[i] for i in range(4)]).astype(np.uint64)
    assert (o.ntt(s, mods) == Ssum).all()
    # X (the monomial) transforms to the evaluation points themselves
    x = np.zeros((1, prm.N), dtype=np.uint64)
    x[0, 1] = 1
    X = o.ntt(x, [0])[0]
    psi, q = o.psi(0), prm.q[0]
    for j in (0, 1, 2, 12345, 65535):
        assert int(X[j]) == pow(psi, 2 * pyref.brv(j, 16) + 1, q)
    assert pow(psi, prm.N, q) == q - 1


def test_scalar_helpers():
    L = lib()
    q = config_params(1).p[-1]
    for a, b in ((q - 1, q - 1), (123456789123456789 % q, 987654321987654321 % q)):
        assert L.orc_mulmod(a, b, q) == a * b % q
        assert L.orc_powmod(a, b, q) == pow(a, b, q)
        assert L.orc_invmod(a, q) == pow(a, -1, q)
