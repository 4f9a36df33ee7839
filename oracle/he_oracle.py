"""ctypes binding of the plain-C CPU oracle (oracle/he_oracle.c).  TEST INFRASTRUCTURE ONLY.

Only tests, the smoke check and the benchmark's cpu_baseline leg may import this module; the
HIP library never does, and this module never imports the HIP binding.  Arrays are numpy
uint64 / int64, C-contiguous, limb-major [poly][limb][N].
"""
import ctypes as C
import os
import subprocess

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "he_oracle.c")
_LIB = os.path.join(_HERE, "libhe_oracle.so")

_u64p = C.POINTER(C.c_uint64)
_i64p = C.POINTER(C.c_int64)
_u32p = C.POINTER(C.c_uint32)


def build(force: bool = False) -> str:
    """Compile the oracle with gcc (plain C11, OpenMP over independent limbs)."""
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        subprocess.check_call(["gcc", "-O2", "-std=c11", "-fopenmp", "-shared", "-fPIC", "-o", _LIB, _SRC])
    return _LIB


_lib = None


def lib():
    global _lib
    if _lib is None:
        _lib = C.CDLL(build())
        _lib.orc_create.restype = C.c_void_p
        _lib.orc_create.argtypes = [C.c_uint32, _u64p, C.c_uint32, _u64p, C.c_uint32, C.c_uint32]
        _lib.orc_destroy.argtypes = [C.c_void_p]
        for name in ("orc_mulmod", "orc_powmod"):
            getattr(_lib, name).restype = C.c_uint64
            getattr(_lib, name).argtypes = [C.c_uint64] * 3
        _lib.orc_invmod.restype = C.c_uint64
        _lib.orc_invmod.argtypes = [C.c_uint64] * 2
        _lib.orc_find_psi.restype = C.c_uint64
        _lib.orc_find_psi.argtypes = [C.c_uint64, C.c_uint32]
        _lib.orc_psi.restype = C.c_uint64
        _lib.orc_psi.argtypes = [C.c_void_p, C.c_uint32]
        _lib.orc_num_digits.restype = C.c_uint32
        _lib.orc_num_digits.argtypes = [C.c_void_p, C.c_uint32]
        _lib.orc_num_threads.restype = C.c_int
    return _lib


def num_threads():
    """Threads the oracle's limb-parallel loops use (OpenMP default)."""
    return int(lib().orc_num_threads())


def _p(a, typ=_u64p):
    return a.ctypes.data_as(typ)


def _u64(a):
    a = np.ascontiguousarray(a, dtype=np.uint64)
    return a


def _idx(mod_idx):
    return np.ascontiguousarray(mod_idx, dtype=np.uint32)


class Oracle:
    """One RNS-CKKS parameter set: ring degree 2^logN, primes q_0..q_L, special primes p, dnum."""

    def __init__(self, logN, q, p, dnum):
        self.logN, self.N = int(logN), 1 << int(logN)
        self.q, self.p = [int(x) for x in q], [int(x) for x in p]
        self.nq, self.np_, self.dnum = len(self.q), len(self.p), int(dnum)
        self.alpha = -(-self.nq // self.dnum)
        self.moduli = self.q + self.p
        qa, pa = np.array(self.q, dtype=np.uint64), np.array(self.p if self.p else [0], dtype=np.uint64)
        self._h = lib().orc_create(self.logN, _p(qa), self.nq, _p(pa), self.np_, self.dnum)
        if not self._h:
            raise ValueError("bad oracle parameters")
        self._h = C.c_void_p(self._h)

    @classmethod
    def from_params(cls, prm):
        return cls(prm.logN, prm.q, prm.p, prm.dnum)

    def __del__(self):
        try:
            lib().orc_destroy(self._h)
        except Exception:
            pass

    # ---- parameters
    def psi(self, mi):
        return int(lib().orc_psi(self._h, mi))

    def num_digits(self, level):
        return int(lib().orc_num_digits(self._h, level))

    def raised_moduli(self, level):
        """Modulus indices of the raised basis at `level`: q_0..q_level, p_0..p_{k-1}."""
        return list(range(level + 1)) + [self.nq + t for t in range(self.np_)]

    # ---- transforms
    def ntt(self, data, mod_idx):
        d = _u64(data).copy().reshape(-1, self.N)
        mi = _idx(mod_idx)
        assert d.shape[0] == mi.size
        lib().orc_ntt(self._h, _p(d), _p(mi, _u32p), C.c_uint32(mi.size))
        return d.reshape(np.shape(data))

    def intt(self, data, mod_idx):
        d = _u64(data).copy().reshape(-1, self.N)
        mi = _idx(mod_idx)
        assert d.shape[0] == mi.size
        lib().orc_intt(self._h, _p(d), _p(mi, _u32p), C.c_uint32(mi.size))
        return d.reshape(np.shape(data))

    def ntt_def(self, a, mi):
        a = _u64(a)
        out = np.empty(self.N, dtype=np.uint64)
        lib().orc_ntt_def(self._h, C.c_uint32(mi), _p(a), _p(out))
        return out

    def negacyclic_mul_def(self, a, b, mi):
        a, b = _u64(a), _u64(b)
        out = np.empty(self.N, dtype=np.uint64)
        lib().orc_negacyclic_mul_def(C.c_uint64(self.moduli[mi]), C.c_uint32(self.N), _p(a), _p(b), _p(out))
        return out

    def pointwise_mul(self, a, b, mod_idx):
        a, b = _u64(a).reshape(-1, self.N), _u64(b).reshape(-1, self.N)
        mi = _idx(mod_idx)
        out = np.empty_like(a)
        lib().orc_pointwise_mul(self._h, _p(a), _p(b), _p(mi, _u32p), C.c_uint32(mi.size), _p(out))
        return out

    # ---- automorphism
    def automorph_coef(self, a, mod_idx, g):
        a = _u64(a).reshape(-1, self.N)
        mi = _idx(mod_idx)
        out = np.empty_like(a)
        lib().orc_automorph_coef(self._h, _p(a), _p(out), _p(mi, _u32p), C.c_uint32(mi.size), C.c_uint32(g))
        return out

    def automorph_ntt(self, a, g):
        a = _u64(a)
        flat = a.reshape(-1, self.N)
        out = np.empty_like(flat)
        lib().orc_automorph_ntt(self._h, _p(flat), _p(out), C.c_uint32(flat.shape[0]), C.c_uint32(g))
        return out.reshape(a.shape)

    def galois_elt(self, step):
        """Galois element of a left rotation by `step` slots (negative = right); 5^step mod 2N."""
        return pow(5, step % (self.N // 2), 2 * self.N)

    @property
    def galois_conj(self):
        return 2 * self.N - 1

    # ---- key switching
    def modup(self, poly, level):
        poly = _u64(poly)
        assert poly.shape == (level + 1, self.N)
        beta, R = self.num_digits(level), level + 1 + self.np_
        out = np.empty((beta, R, self.N), dtype=np.uint64)
        lib().orc_modup(self._h, _p(poly), C.c_uint32(level), _p(out))
        return out

    def inner_product(self, digits, level, evk):
        digits, evk = _u64(digits), _u64(evk)
        R = level + 1 + self.np_
        assert evk.shape == (self.dnum, 2, self.nq + self.np_, self.N)
        acc = np.empty((2, R, self.N), dtype=np.uint64)
        lib().orc_inner_product(self._h, _p(digits), C.c_uint32(level), _p(evk), _p(acc))
        return acc

    def moddown(self, acc, level):
        acc = _u64(acc)
        assert acc.shape == (level + 1 + self.np_, self.N)
        out = np.empty((level + 1, self.N), dtype=np.uint64)
        lib().orc_moddown(self._h, _p(acc), C.c_uint32(level), _p(out))
        return out

    def keyswitch(self, poly, level, evk):
        poly, evk = _u64(poly), _u64(evk)
        assert poly.shape == (level + 1, self.N)
        o0 = np.empty((level + 1, self.N), dtype=np.uint64)
        o1 = np.empty_like(o0)
        lib().orc_keyswitch(self._h, _p(poly), C.c_uint32(level), _p(evk), _p(o0), _p(o1))
        return o0, o1

    def rotate(self, ct, level, g, evk):
        ct, evk = _u64(ct), _u64(evk)
        assert ct.shape == (2, level + 1, self.N)
        out = np.empty_like(ct)
        lib().orc_rotate(self._h, _p(ct), C.c_uint32(level), C.c_uint32(g), _p(evk), _p(out))
        return out

    def rotate_from_raised(self, ct, raised, level, g, evk):
        ct, evk, raised = _u64(ct), _u64(evk), _u64(raised)
        out = np.empty_like(ct)
        lib().orc_rotate_from_raised(self._h, _p(ct), _p(raised), C.c_uint32(level), C.c_uint32(g), _p(evk), _p(out))
        return out

    def add_limbs(self, a, b, mod_idx):
        """a + b per limb, limb l modulo moduli[mod_idx[l]]."""
        a, b = _u64(a), _u64(b)
        mi = _idx(mod_idx)
        fa, fb = a.reshape(-1, self.N), b.reshape(-1, self.N)
        assert fa.shape == fb.shape and fa.shape[0] == mi.size
        out = np.empty_like(fa)
        lib().orc_add_limbs(self._h, _p(fa), _p(fb), _p(mi, _u32p), C.c_uint32(mi.size), _p(out))
        return out.reshape(a.shape)

    def rotate_sum_deferred(self, cts, level, gs, evks):
        """sum_t Rot(cts[t]; g_t) with the ModDown deferred across the sum (Slide_1 & Sum_f of the
        paper's Algorithm 2 evaluated with a single ModDown): every rotated term is raised and multiplied
        into its key on its own, the products are summed over the raised basis q_0..q_level, p_*, and only
        the sum is brought down:
            A_c   = sum_{t: g_t != 1} sum_j sigma_{g_t}(ModUp(c1_t)_j) * evk_t,j,c      (c = 0, 1)
            out   = ( sum_{t: g_t != 1} sigma_{g_t}(c0_t) + ModDown(A_0) + sum_{t: g_t = 1} c0_t ,
                      ModDown(A_1) + sum_{t: g_t = 1} c1_t ).
        The result decrypts to the same sum as rotating term by term, but its bits differ (ModDown does
        not distribute over sums), and it carries one ModDown's rounding instead of one per term.
        cts: ciphertexts [2][level+1][N]; gs: Galois elements; evks[t]: key of g_t (ignored where g_t = 1)."""
        L1, rm = level + 1, self.raised_moduli(level)
        qm = list(range(L1))
        acc = rot0 = plain = None
        for ct, g, evk in zip(cts, gs, evks):
            ct = _u64(ct)
            if g == 1:
                plain = ct if plain is None else self.add(plain, ct, level)
                continue
            raised = self.modup(ct[1], level)
            ip = self.inner_product(self.automorph_ntt(raised, g), level, evk)
            acc = ip if acc is None else self.add_limbs(acc, ip, rm + rm)
            r0 = self.automorph_ntt(ct[0], g)
            rot0 = r0 if rot0 is None else self.add_limbs(rot0, r0, qm)
        if acc is None:
            return plain
        out = np.stack([self.add_limbs(self.moddown(acc[0], level), rot0, qm), self.moddown(acc[1], level)])
        return out if plain is None else self.add(out, plain, level)

    # ---- MulPt accumulate, rescale, add
    def ptct_mac(self, acc, ct, pt, level, init):
        ct, pt = _u64(ct), _u64(pt)
        assert ct.shape == (2, level + 1, self.N) and pt.shape == (level + 1, self.N)
        acc = np.zeros_like(ct) if acc is None else _u64(acc).copy()
        lib().orc_ptct_mac(self._h, _p(acc), _p(ct), _p(pt), C.c_uint32(level), C.c_int(1 if init else 0))
        return acc

    def rescale(self, ct, level):
        ct = _u64(ct)
        assert ct.shape == (2, level + 1, self.N) and level >= 1
        out = np.empty((2, level, self.N), dtype=np.uint64)
        lib().orc_rescale(self._h, _p(ct), C.c_uint32(level), _p(out))
        return out

    def mulct(self, a, b, level, rlk):
        a, b, rlk = _u64(a), _u64(b), _u64(rlk)
        assert a.shape == b.shape == (2, level + 1, self.N)
        out = np.empty_like(a)
        lib().orc_mulct(self._h, _p(a), _p(b), C.c_uint32(level), _p(rlk), _p(out))
        return out

    def affine(self, ct, level, mul, add):
        """out_c[r] = ct_c[r]*mul[r] (+ add[r] on c0); mul/add are Python ints (any sign), reduced per limb."""
        ct = _u64(ct)
        m = np.array([int(mul[r]) % self.q[r] for r in range(level + 1)], dtype=np.uint64)
        a = np.array([int(add[r]) % self.q[r] for r in range(level + 1)], dtype=np.uint64)
        out = np.empty_like(ct)
        lib().orc_affine(self._h, _p(ct), C.c_uint32(level), _p(m), _p(a), _p(out))
        return out

    @staticmethod
    def drop_level(ct, level):
        """Forget limb q_level (no rounding, scale unchanged): [2][level+1][N] -> [2][level][N]."""
        return np.ascontiguousarray(_u64(ct)[:, :level, :])

    def add(self, a, b, level):
        a, b = _u64(a), _u64(b)
        out = np.empty_like(a)
        lib().orc_add(self._h, _p(a), _p(b), C.c_uint32(level), _p(out))
        return out

    def addpt(self, ct, pt, level):
        ct, pt = _u64(ct), _u64(pt)
        out = np.empty_like(ct)
        lib().orc_addpt(self._h, _p(ct), _p(pt), C.c_uint32(level), _p(out))
        return out

    # ---- client side
    def reduce_signed(self, m, mod_idx):
        m = np.ascontiguousarray(m, dtype=np.int64)
        mi = _idx(mod_idx)
        out = np.empty((mi.size, self.N), dtype=np.uint64)
        lib().orc_reduce_signed(self._h, _p(m, _i64p), _p(mi, _u32p), C.c_uint32(mi.size), _p(out))
        return out

    def make_evk(self, s, sprime, a, e):
        s = np.ascontiguousarray(s, dtype=np.int64)
        sprime = np.ascontiguousarray(sprime, dtype=np.int64)
        a = _u64(a)
        e = np.ascontiguousarray(e, dtype=np.int64)
        M = self.nq + self.np_
        assert a.shape == (self.dnum, M, self.N) and e.shape == (self.dnum, self.N)
        evk = np.empty((self.dnum, 2, M, self.N), dtype=np.uint64)
        lib().orc_make_evk(self._h, _p(s, _i64p), _p(sprime, _i64p), _p(a), _p(e, _i64p), _p(evk))
        return evk

    def encrypt(self, m, s, a, e, level):
        m = np.ascontiguousarray(m, dtype=np.int64)
        s = np.ascontiguousarray(s, dtype=np.int64)
        e = np.ascontiguousarray(e, dtype=np.int64)
        a = _u64(a)
        assert a.shape == (level + 1, self.N)
        ct = np.empty((2, level + 1, self.N), dtype=np.uint64)
        lib().orc_encrypt(self._h, _p(m, _i64p), _p(s, _i64p), _p(a), _p(e, _i64p), C.c_uint32(level), _p(ct))
        return ct

    def phase(self, ct, level, s, limbs=(0,)):
        """c0 + c1*s on the given limbs, coefficient form, canonical residues [len(limbs)][N]."""
        ct = _u64(ct)
        s = np.ascontiguousarray(s, dtype=np.int64)
        li = _idx(limbs)
        out = np.empty((li.size, self.N), dtype=np.uint64)
        lib().orc_phase(self._h, _p(ct), C.c_uint32(level), _p(s, _i64p), _p(li, _u32p), C.c_uint32(li.size), _p(out))
        return out
