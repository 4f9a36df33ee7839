"""RNS-CKKS parameter sets of the five workloads (ring degree, prime chains, dnum, scale).

The paper fixes only the ring Z[X]/(X^N+1) with N = 2^15..2^17 and the existence of a
level/modulus chain (Section 2.1) and a decomposition number dnum for key switching
(Appendix, parameter-set table).  The concrete primes follow the workload statement:
"b-bit primes congruent to 1 mod 2N, the smallest such above 2^(b-1)".
"""
from dataclasses import dataclass, field
from typing import List

_MR_BASES = (2, 3, 5, 7, 11, 13, 17, 19, 23, 29, 31, 37)  # deterministic for n < 3.3e24


def is_prime(n: int) -> bool:
    """Deterministic Miller-Rabin for 64-bit integers."""
    if n < 2:
        return False
    for b in _MR_BASES:
        if n % b == 0:
            return n == b
    d, r = n - 1, 0
    while d % 2 == 0:
        d //= 2
        r += 1
    for a in _MR_BASES:
        x = pow(a, d, n)
        if x in (1, n - 1):
            continue
        for _ in range(r - 1):
            x = x * x % n
            if x == n - 1:
                break
        else:
            return False
    return True


def ntt_primes(bits: int, two_n: int, count: int) -> List[int]:
    """The `count` smallest primes q > 2^(bits-1) with q = 1 (mod two_n), ascending."""
    out = []
    c = (1 << (bits - 1)) + 1  # 2^(bits-1) is a multiple of two_n, so c = 1 mod two_n
    assert (c - 1) % two_n == 0
    while len(out) < count:
        if is_prime(c):
            out.append(c)
        c += two_n
    assert out[-1] < (1 << bits)
    return out


@dataclass
class HEParams:
    logN: int
    q: List[int]            # ciphertext primes q_0..q_L
    p: List[int]            # special primes p_0..p_{k-1}
    dnum: int
    scale: float            # ciphertext scale Delta
    hamming: int            # Hamming weight of the ternary secret
    sigma: float = 3.2      # error standard deviation
    seed: int = 0
    name: str = ""
    extra: dict = field(default_factory=dict)

    @property
    def N(self) -> int:
        return 1 << self.logN

    @property
    def alpha(self) -> int:
        return -(-len(self.q) // self.dnum)

    @property
    def moduli(self) -> List[int]:
        return list(self.q) + list(self.p)


def config_params(cfg: int) -> HEParams:
    """Parameter set of workload `cfg` (0..4)."""
    if cfg == 0:
        two_n = 2 << 12
        return HEParams(logN=12, q=ntt_primes(40, two_n, 3), p=ntt_primes(41, two_n, 1), dnum=3,
                        scale=2.0 ** 30, hamming=64, seed=0, name="tiny-conv-N4096")
    if cfg in (1, 2, 3, 4):
        two_n = 2 << 16
        q = ntt_primes(54, two_n, 24)
        p = ntt_primes(60, two_n, 8)
        return HEParams(logN=16, q=q, p=p, dnum=3, scale=2.0 ** 40, hamming=192, seed=cfg,
                        name={1: "ntt-batch", 2: "rotation-keyswitch", 3: "resnet20-conv",
                              4: "downsample-block"}[cfg])
    raise ValueError("config must be 0..4")


def toy_params(logN: int = 4, q_bits: int = 25, nq: int = 6, p_bits: int = 27, np_: int = 2,
               dnum: int = 3, scale: float = 2.0 ** 20, hamming: int = 4, seed: int = 7) -> HEParams:
    """Small parameter sets for brute-force checks (tiny rings, several digits, partial digits)."""
    two_n = 2 << logN
    return HEParams(logN=logN, q=ntt_primes(q_bits, two_n, nq), p=ntt_primes(p_bits, two_n, np_),
                    dnum=dnum, scale=scale, hamming=hamming, seed=seed, name="toy")
