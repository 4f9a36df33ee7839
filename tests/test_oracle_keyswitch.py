"""Pins for ModUp / inner product / ModDown / key switch / rescale / MulPt against exact
integer (CRT) arithmetic on tiny rings."""
import numpy as np
import pytest

import pyref
from he_inputs import sampling as S
from he_inputs.params import toy_params
from oracle import ckks_client as K
from oracle.he_oracle import Oracle


def _setup(logN=4, seed=21, **kw):
    prm = toy_params(logN=logN, **kw)
    o = Oracle.from_params(prm)
    rng = S.make_rng(seed)
    return prm, o, rng


@pytest.mark.parametrize("level", [5, 4, 3, 2, 0])
def test_modup_is_x_plus_small_multiple_of_digit_product(level):
    prm, o, rng = _setup()
    N, alpha = prm.N, prm.alpha
    x = S.uniform_limbs(rng, prm.q[:level + 1], N)[0]          # coefficient form
    X = o.ntt(x, range(level + 1))
    raised = o.modup(X, level)
    rm = o.raised_moduli(level)
    beta = o.num_digits(level)
    assert raised.shape == (beta, level + 1 + len(prm.p), N)
    assert beta == -(-(level + 1) // alpha)
    for j in range(beta):
        coef = o.intt(raised[j], rm)
        lo, hi = j * alpha, min((j + 1) * alpha, level + 1)
        dmods = prm.q[lo:hi]
        for n in range(N):
            xv, Qj = pyref.crt([x[i][n] for i in range(lo, hi)], dmods)
            us = set()
            for r, mi in enumerate(rm):
                t = prm.moduli[mi]
                if lo <= r < hi:
                    assert int(coef[r][n]) == int(x[r][n])       # own limbs copied
                    continue
                # find u in [0, |D_j|) with out = x + u*Qj (mod t)
                u = [u for u in range(hi - lo + 1) if (xv + u * Qj) % t == int(coef[r][n])]
                assert len(u) == 1
                us.add(u[0])
            assert len(us) <= 1 and all(u < hi - lo for u in us)   # one overflow count for all targets


@pytest.mark.parametrize("level", [5, 3, 2])
def test_keyswitch_relation_and_noise(level):
    prm, o, rng = _setup(seed=22)
    N = prm.N
    s = S.ternary_secret(rng, N, prm.hamming)
    sp = S.ternary_secret(rng, N, prm.hamming)                   # arbitrary other key s'
    a = S.uniform_limbs(rng, prm.moduli, N, prm.dnum)
    e = S.gaussian_error(rng, N, 3.2, prm.dnum)
    evk = o.make_evk(s, sp, a, e)
    d = S.uniform_limbs(rng, prm.q[:level + 1], N)[0]           # NTT-form input
    o0, o1 = o.keyswitch(d, level, evk)
    mods = list(range(level + 1))
    dc, c0, c1 = o.intt(d, mods), o.intt(o0, mods), o.intt(o1, mods)
    qs = prm.q[:level + 1]
    Q = 1
    for q in qs:
        Q *= q
    D = [pyref.crt([dc[i][n] for i in mods], qs)[0] for n in range(N)]
    C0 = [pyref.crt([c0[i][n] for i in mods], qs)[0] for n in range(N)]
    C1 = [pyref.crt([c1[i][n] for i in mods], qs)[0] for n in range(N)]
    lhs = pyref.negacyclic_mul_int(C1, [int(v) for v in s])
    rhs = pyref.negacyclic_mul_int(D, [int(v) for v in sp])
    noise = [pyref.center((C0[n] + lhs[n] - rhs[n]) % Q, Q) for n in range(N)]
    # bound: digits * alpha * (q_max/P) * N * |e| terms + ModDown rounding (~ (1+h)/2 * k)
    assert max(abs(v) for v in noise) < 2 ** 14, max(abs(v) for v in noise)
    # the unreduced product d*s' is astronomically larger than the noise: the relation is not vacuous
    assert max(abs(pyref.center(v % Q, Q)) for v in rhs) > 2 ** 60


def test_evk_structure():
    prm, o, rng = _setup(seed=23)
    N, M = prm.N, len(prm.moduli)
    s = S.ternary_secret(rng, N, prm.hamming)
    sp = S.ternary_secret(rng, N, prm.hamming)
    a = S.uniform_limbs(rng, prm.moduli, N, prm.dnum)
    e = S.gaussian_error(rng, N, 3.2, prm.dnum)
    evk = o.make_evk(s, sp, a, e)
    P = 1
    for p in prm.p:
        P *= p
    allm = list(range(M))
    for j in range(prm.dnum):
        b = o.intt(evk[j, 0], allm)
        ac = o.intt(evk[j, 1], allm)
        for r in range(M):
            m = prm.moduli[r]
            a_s = pyref.negacyclic_mul([int(v) for v in ac[r]], [int(v) % m for v in s], m)
            in_digit = r < len(prm.q) and j * prm.alpha <= r < (j + 1) * prm.alpha
            for n in range(N):
                want = (-a_s[n] + int(e[j][n]) + (P * int(sp[n]) if in_digit else 0)) % m
                assert int(b[r][n]) == want


@pytest.mark.parametrize("level", [5, 2, 1])
def test_rescale_is_exact_rounded_division(level):
    prm, o, rng = _setup(seed=24)
    N = prm.N
    ct = np.stack([S.uniform_limbs(rng, prm.q[:level + 1], N)[0] for _ in range(2)])   # NTT form
    out = o.rescale(ct, level)
    qs = prm.q[:level + 1]
    ql = qs[-1]
    for comp in range(2):
        cin = o.intt(ct[comp], range(level + 1))
        cout = o.intt(out[comp], range(level))
        for n in range(N):
            c, Q = pyref.crt([cin[i][n] for i in range(level + 1)], qs)
            c = pyref.center(c, Q)
            r = (2 * c + ql) // (2 * ql)          # round half up of c/ql, exact integers
            for i in range(level):
                assert int(cout[i][n]) == r % qs[i]


def test_ptct_mac_pointwise_and_accumulates():
    prm, o, rng = _setup(seed=25)
    N, level = prm.N, 3
    qs = prm.q[:level + 1]
    ct = np.stack([S.uniform_limbs(rng, qs, N)[0] for _ in range(2)])
    ct2 = np.stack([S.uniform_limbs(rng, qs, N)[0] for _ in range(2)])
    pt, pt2 = S.uniform_limbs(rng, qs, N)[0], S.uniform_limbs(rng, qs, N)[0]
    acc = o.ptct_mac(None, ct, pt, level, init=True)
    acc2 = o.ptct_mac(acc, ct2, pt2, level, init=False)
    for comp in range(2):
        for i, q in enumerate(qs):
            for n in range(N):
                w1 = int(ct[comp][i][n]) * int(pt[i][n]) % q
                assert int(acc[comp][i][n]) == w1
                assert int(acc2[comp][i][n]) == (w1 + int(ct2[comp][i][n]) * int(pt2[i][n])) % q
    # init=True ignores previous contents
    assert (o.ptct_mac(acc2, ct, pt, level, init=True) == acc).all()
