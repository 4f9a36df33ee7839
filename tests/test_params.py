"""Workload parameter sets: the prime chains follow the stated rule and match the stored lists."""
import os

from he_inputs.params import config_params, is_prime, ntt_primes

GOLD = os.path.join(os.path.dirname(__file__), "golden", "primes.txt")


def _gold():
    out = {}
    for line in open(GOLD):
        if line.startswith("#") or not line.strip():
            continue
        t = line.split()
        b, logn = int(t[1]), int(t[2])
        out[t[0]] = [(1 << (b - 1)) + int(k) * (2 << logn) + 1 for k in t[3:]]
    return out


def _slow_is_prime(n):
    # Fermat + Euler checks to bases unrelated to the generator's Miller-Rabin bases
    for a in (41, 43, 47, 53, 59, 61, 67):
        if pow(a, n - 1, n) != 1:
            return False
    return True


def test_chains_match_golden():
    g = _gold()
    p0, p1 = config_params(0), config_params(1)
    assert p0.q == g["cfg0_q"] and p0.p == g["cfg0_p"]
    assert p1.q == g["cfg1_q"] and p1.p == g["cfg1_p"]
    for c in (2, 3, 4):
        pc = config_params(c)
        assert pc.q == p1.q and pc.p == p1.p and pc.dnum == 3 and pc.alpha == 8


def test_rule_smallest_primes_above_power_of_two():
    for bits, logn, cnt in ((40, 12, 3), (41, 12, 1), (54, 16, 24), (60, 16, 8)):
        two_n = 2 << logn
        ps = ntt_primes(bits, two_n, cnt)
        assert ps == sorted(ps) and len(set(ps)) == cnt
        c = (1 << (bits - 1)) + 1
        found = []
        while c <= ps[-1]:
            if _slow_is_prime(c):
                found.append(c)
            c += two_n
        assert found == ps  # nothing skipped, nothing composite
        for p in ps:
            assert p % two_n == 1 and p.bit_length() == bits and is_prime(p)


def test_special_modulus_covers_largest_digit():
    # hybrid key switching needs P >= every digit product Q_j
    for cfg in (0, 2):
        prm = config_params(cfg)
        P = 1
        for p in prm.p:
            P *= p
        a = prm.alpha
        for j in range(prm.dnum):
            Qj = 1
            for q in prm.q[j * a:(j + 1) * a]:
                Qj *= q
            assert P > Qj
        assert a == len(prm.p)
