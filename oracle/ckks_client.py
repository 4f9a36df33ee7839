"""Client side of RNS-CKKS for the oracle and the tests: encode/decode, key generation,
encryption, decryption.  TEST INFRASTRUCTURE ONLY (never on the HIP product path).

The paper excludes these from its timings (Section 4.1: measurement starts once plaintexts
and ciphertexts are resident) and names them only through the scheme (Section 2.1); the
definitions are the standard canonical-embedding ones:
  zeta = exp(i*pi/N); slot j <-> evaluation point zeta^(5^j mod 2N), j < N/2;
  encode(z, Delta): the real polynomial m with m(zeta^(5^j)) ~= Delta*z_j, rounded per
  coefficient;  decode: z_j = m(zeta^(5^j)) / Delta.
With this indexing the Galois map X -> X^(5^r) rotates the slot vector LEFT by r (the
direction the paper gives for CRot, Section 2.1) and X -> X^(2N-1) conjugates.
"""
import numpy as np

from .he_oracle import Oracle


def slot_exponents(N):
    """e_j = 5^j mod 2N for j < N/2."""
    e = np.empty(N // 2, dtype=np.int64)
    v = 1
    for j in range(N // 2):
        e[j] = v
        v = v * 5 % (2 * N)
    return e


def encode_def(z, N, scale):
    """Encoding by its O(N^2) definition: m_i = round((2*Delta/N) * Re sum_j z_j zeta^(-e_j i))."""
    z = np.asarray(z, dtype=np.complex128)
    e = slot_exponents(N)
    m = np.empty(N, dtype=np.int64)
    for i in range(N):
        ang = -np.pi * ((e * i) % (2 * N)) / N
        m[i] = int(np.rint((2.0 * scale / N) * np.sum(z.real * np.cos(ang) - z.imag * np.sin(ang))))
    return m


def decode_def(m, N, scale):
    """Decoding by its definition: z_j = m(zeta^(e_j)) / Delta, O(N^2)."""
    m = np.asarray(m, dtype=np.float64)
    e = slot_exponents(N)
    z = np.empty(N // 2, dtype=np.complex128)
    i = np.arange(N)
    for j in range(N // 2):
        ang = np.pi * ((e[j] * i) % (2 * N)) / N
        z[j] = np.sum(m * (np.cos(ang) + 1j * np.sin(ang))) / scale
    return z


def _odd_power_evals(m, N):
    """v[k] = m(zeta^(2k+1)), k < N, through one length-N FFT of the twisted coefficients."""
    i = np.arange(N)
    tw = np.exp(1j * np.pi * i / N)
    return np.fft.ifft(np.asarray(m, dtype=np.float64) * tw) * N


def encode(z, N, scale):
    """Same map as encode_def through an FFT (used at N = 2^12 / 2^16)."""
    z = np.asarray(z, dtype=np.complex128)
    assert z.shape == (N // 2,)
    e = slot_exponents(N)
    v = np.zeros(N, dtype=np.complex128)
    v[(e - 1) // 2] = z
    v[(2 * N - e - 1) // 2] = np.conj(z)
    i = np.arange(N)
    tw = np.exp(-1j * np.pi * i / N)
    m = (np.fft.fft(v) / N) * tw
    return np.rint(m.real * scale).astype(np.int64)


def decode(m, N, scale):
    e = slot_exponents(N)
    return _odd_power_evals(m, N)[(e - 1) // 2] / scale


def centered(res, q):
    """Canonical residues mod q -> signed representatives in (-q/2, q/2] as int64."""
    res = np.asarray(res, dtype=np.uint64)
    q = int(q)
    out = res.astype(np.int64)
    big = res > np.uint64(q // 2)
    out[big] = (res[big].astype(np.int64) - np.int64(q))
    return out


def automorph_signed(s, g):
    """sigma_g on a signed integer coefficient vector (X -> X^g, X^N = -1)."""
    s = np.asarray(s, dtype=np.int64)
    N = s.size
    out = np.zeros_like(s)
    for i in range(N):
        t = (i * g) % (2 * N)
        if t < N:
            out[t] = s[i]
        else:
            out[t - N] = -s[i]
    return out


class Client:
    """Holds a secret key and produces keys / ciphertexts from caller-supplied randomness."""

    def __init__(self, oracle: Oracle, secret):
        self.o = oracle
        self.s = np.ascontiguousarray(secret, dtype=np.int64)

    def rotation_key(self, g, a, e):
        """evk for s' = sigma_g(s); a: uniform [dnum][nq+np][N], e: errors [dnum][N]."""
        return self.o.make_evk(self.s, automorph_signed(self.s, g), a, e)

    def relin_key(self, a, e):
        """evk for s' = s^2 (negacyclic square of the secret, exact integers)."""
        N = self.o.N
        full = np.convolve(self.s, self.s)                   # length 2N-1, exact in int64
        s2 = full[:N].copy()
        s2[:N - 1] -= full[N:]
        return self.o.make_evk(self.s, s2, a, e)

    def encrypt(self, z, scale, level, a, e):
        m = encode(z, self.o.N, scale)
        return self.o.encrypt(m, self.s, a, e, level)

    def decrypt(self, ct, level, scale):
        """Decrypt on limb 0 alone (valid while |Delta*z| << q_0/2) and decode."""
        ph = self.o.phase(ct, level, self.s, limbs=(0,))[0]
        return decode(centered(ph, self.o.q[0]), self.o.N, scale)

    def decrypt_crt(self, ct, level, scale, limbs=2):
        """Decrypt on the first `limbs` limbs with an exact CRT lift (for scales near or above q_0)."""
        ph = self.o.phase(ct, level, self.s, limbs=tuple(range(limbs)))
        qs = [self.o.q[i] for i in range(limbs)]
        Q = 1
        for q in qs:
            Q *= q
        m = np.empty(self.o.N, dtype=np.float64)
        coef = [(Q // q) * pow(Q // q, -1, q) for q in qs]
        for n in range(self.o.N):
            v = sum(int(ph[i][n]) * coef[i] for i in range(limbs)) % Q
            if v > Q // 2:
                v -= Q
            m[n] = float(v)
        return decode(m, self.o.N, scale)
