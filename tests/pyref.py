"""Brute-force definitions in Python integers, used to pin the C oracle at tiny sizes.

Nothing here is shared with the oracle or the HIP path: it restates the mathematical
objects (polynomials in Z_q[X]/(X^N+1), CRT, rounding) directly.
"""
from functools import reduce


def brv(x, bits):
    return int(format(x, "0%db" % bits)[::-1], 2) if bits else 0


def negacyclic_mul(a, b, q):
    N = len(a)
    out = [0] * N
    for i in range(N):
        for j in range(N):
            k = i + j
            if k < N:
                out[k] = (out[k] + a[i] * b[j]) % q
            else:
                out[k - N] = (out[k - N] - a[i] * b[j]) % q
    return out


def negacyclic_mul_int(a, b):
    """Same over the integers (no modulus)."""
    N = len(a)
    out = [0] * N
    for i in range(N):
        for j in range(N):
            k = i + j
            if k < N:
                out[k] += a[i] * b[j]
            else:
                out[k - N] -= a[i] * b[j]
    return out


def poly_eval(a, x, q):
    acc = 0
    for c in reversed(a):
        acc = (acc * x + c) % q
    return acc


def ntt_by_evaluation(a, psi, q):
    """out[j] = a(psi^(2*brv(j)+1)) by Horner evaluation."""
    N = len(a)
    bits = N.bit_length() - 1
    return [poly_eval(a, pow(psi, 2 * brv(j, bits) + 1, q), q) for j in range(N)]


def smallest_qnr_root(q, N):
    c = 2
    while pow(c, (q - 1) // 2, q) != q - 1:
        c += 1
    return pow(c, (q - 1) // (2 * N), q)


def crt(residues, moduli):
    """Integer in [0, prod moduli) with the given residues."""
    M = reduce(lambda x, y: x * y, moduli, 1)
    x = 0
    for r, m in zip(residues, moduli):
        Mi = M // m
        x += int(r) * Mi * pow(Mi, -1, m)
    return x % M, M


def center(x, M):
    return x - M if x > M // 2 else x
