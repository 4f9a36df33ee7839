"""ctypes binding of libhe_mi355x.so: same names as the C ABI, argument marshalling only.

Tensors are torch CUDA tensors of dtype uint64 (or int64 holding the same bits), contiguous,
limb-major [poly][limb][N].  Every step of the path runs in the library's HIP kernels; there
is no CPU fallback: if the library is missing or a call fails, an exception is raised.
"""
import ctypes as C
import os

import torch

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libhe_mi355x.so")

HE_OK = 0
_STATUS = {0: "HE_OK", -1: "HE_ERR_BADARG", -2: "HE_ERR_LEVEL", -3: "HE_ERR_NOKEY", -4: "HE_ERR_ALLOC", -5: "HE_ERR_HIP"}

EXPORTS = [
    "he_ctx_create", "he_ctx_destroy", "he_last_error", "he_ctx_psi", "he_counters", "he_counters_reset", "he_sync", "he_profile_begin", "he_profile_end",
    "he_ntt", "he_intt", "he_automorph", "he_evk_register", "he_keyswitch", "he_rotate_hoisted", "he_rotate_batch", "he_rotate",
    "he_conjugate", "he_ptct_mac", "he_add", "he_addpt", "he_mulct", "he_affine", "he_rescale", "he_conv2d", "he_raconv",
    "he_probe_alu", "he_build_id", "he_rotate_sum", "he_ws_query_raconv", "he_ca_ra_block", "he_ws_query_ca_ra_block", "he_ras", "he_ws_bytes", "he_ws_reserve", "he_ws_query_rotate_batch", "he_ws_query_conv2d", "he_rescale_noalloc", "he_ptct_mac_rot",
]


class HEError(RuntimeError):
    def __init__(self, code, msg):
        super().__init__("%s (%d): %s" % (_STATUS.get(code, "?"), code, msg))
        self.code = code


class Counters(C.Structure):
    _fields_ = [(n, C.c_uint64) for n in ("keyswitch", "modup", "ntt_limbs", "intt_limbs", "mac", "rescale", "automorph", "moddown")]


class Profile(C.Structure):
    _fields_ = [("transform_launches", C.c_uint64), ("transform_limb_passes", C.c_uint64),
                ("inner_product_digit_limbs", C.c_uint64), ("transform_ms", C.c_double),
                ("pass_launches", C.c_uint64 * 6), ("pass_limbs", C.c_uint64 * 6), ("pass_ms", C.c_double * 6),
                ("key_limbs_read", C.c_uint64)]


class AluProbe(C.Structure):
    _fields_ = [("fwd_butterflies_per_s", C.c_double), ("inv_butterflies_per_s", C.c_double),
                ("fwd_wide_butterflies_per_s", C.c_double)]


class ConvPlan(C.Structure):
    _fields_ = [("C_a", C.c_uint32), ("H", C.c_uint32), ("W", C.c_uint32), ("R", C.c_uint32), ("f", C.c_uint32),
                ("n_out", C.c_uint32), ("level", C.c_uint32), ("skip_ras", C.c_uint32), ("deferred_taps", C.c_uint32), ("hoisted_ras", C.c_uint32),
                ("h_d_weights", C.POINTER(C.c_void_p))]


class RaConvPlan(C.Structure):
    _fields_ = [("n_in", C.c_uint32), ("W", C.c_uint32), ("R", C.c_uint32), ("f", C.c_uint32), ("level", C.c_uint32),
                ("deferred_moddown", C.c_uint32), ("h_d_weights", C.POINTER(C.c_void_p))]


class BlockPlan(C.Structure):
    _fields_ = [("C_a", C.c_uint32), ("H", C.c_uint32), ("W", C.c_uint32), ("R", C.c_uint32), ("f", C.c_uint32),
                ("n_ca", C.c_uint32), ("n_ra", C.c_uint32), ("level", C.c_uint32), ("group", C.c_uint32),
                ("deferred_moddown", C.c_uint32), ("hoisted_ras", C.c_uint32), ("h_k_in", C.POINTER(C.c_uint64)),
                ("h_d_w_ca", C.POINTER(C.c_void_p)), ("h_d_w_ra", C.POINTER(C.c_void_p))]


_lib = None


def load():
    """Load the built library; raises if it is absent (build with __graft_entry__.build())."""
    global _lib
    if _lib is not None:
        return _lib
    if not os.path.exists(LIB_PATH):
        raise RuntimeError("libhe_mi355x.so is not built: run `python -m paper_2302_02407_amd.build`")
    lib = C.CDLL(LIB_PATH)
    vp, u32, i32 = C.c_void_p, C.c_uint32, C.c_int32
    u64p, u32p, i32p = C.POINTER(C.c_uint64), C.POINTER(C.c_uint32), C.POINTER(C.c_int32)
    sig = {
        "he_ctx_create": [C.POINTER(vp), u32, u64p, u32, u64p, u32, u32, vp],
        "he_ctx_destroy": [vp],
        "he_ctx_psi": [vp, u32, u64p],
        "he_counters": [vp, C.POINTER(Counters)],
        "he_counters_reset": [vp],
        "he_sync": [vp],
        "he_profile_begin": [vp],
        "he_profile_end": [vp, C.POINTER(Profile)],
        "he_probe_alu": [vp, C.POINTER(AluProbe)],
        "he_ntt": [vp, vp, u32p, u32],
        "he_intt": [vp, vp, u32p, u32],
        "he_automorph": [vp, vp, vp, u32p, u32, u32, i32],
        "he_evk_register": [vp, u32, vp],
        "he_keyswitch": [vp, vp, u32, u32, vp, vp],
        "he_rotate_hoisted": [vp, vp, u32, i32p, u32, C.POINTER(vp)],
        "he_rotate_batch": [vp, C.POINTER(vp), u32, u32, i32p, u32, C.POINTER(vp), i32],
        "he_rotate": [vp, vp, u32, i32, vp],
        "he_rotate_sum": [vp, C.POINTER(vp), u32, u32, i32p, vp, i32],
        "he_ws_query_raconv": [vp, C.POINTER(RaConvPlan), u64p],
        "he_ras": [vp, C.POINTER(vp), u32, u32, i32p, u32, C.POINTER(vp)],
        "he_conjugate": [vp, vp, u32, vp],
        "he_ptct_mac": [vp, vp, vp, vp, u32, i32],
        "he_add": [vp, vp, vp, u32, vp],
        "he_addpt": [vp, vp, vp, u32, vp],
        "he_rescale": [vp, vp, u32, vp],
        "he_mulct": [vp, vp, vp, u32, vp],
        "he_affine": [vp, vp, u32, u64p, u64p, vp],
        "he_conv2d": [vp, C.POINTER(ConvPlan), vp, C.POINTER(vp)],
        "he_raconv": [vp, C.POINTER(RaConvPlan), C.POINTER(vp), vp],
        "he_ca_ra_block": [vp, C.POINTER(BlockPlan), C.POINTER(vp), C.POINTER(vp)],
        "he_ws_query_ca_ra_block": [vp, C.POINTER(BlockPlan), u64p],
        "he_ws_bytes": [vp, u64p],
        "he_ws_reserve": [vp, C.c_uint64],
        "he_ws_query_rotate_batch": [vp, u32, u32, u32, i32, u64p],
        "he_ws_query_conv2d": [vp, C.POINTER(ConvPlan), u64p],
        "he_rescale_noalloc": [vp, vp, u32, vp],
        "he_ptct_mac_rot": [vp, vp, C.POINTER(C.c_void_p), C.POINTER(C.c_void_p), C.POINTER(u32), u32, u32, i32],
    }
    for name, args in sig.items():
        fn = getattr(lib, name)
        fn.argtypes = args
        fn.restype = i32
    lib.he_last_error.argtypes = [vp]
    lib.he_last_error.restype = C.c_char_p
    lib.he_build_id.argtypes = []
    lib.he_build_id.restype = C.c_char_p
    _lib = lib
    return lib


def _dev(t, what="tensor"):
    if not isinstance(t, torch.Tensor) or not t.is_cuda:
        raise TypeError("%s must be a CUDA tensor" % what)
    if t.dtype not in (torch.uint64, torch.int64):
        raise TypeError("%s must be uint64/int64" % what)
    if not t.is_contiguous():
        raise ValueError("%s must be contiguous" % what)
    return C.c_void_p(t.data_ptr())


def _need(t, n, what):
    """A buffer shorter than what the library will touch is the one mistake it cannot see itself."""
    if t.numel() < n:
        raise ValueError("%s holds %d elements, the call needs %d" % (what, t.numel(), n))


def _u32arr(xs):
    xs = [int(x) for x in xs]
    return (C.c_uint32 * max(1, len(xs)))(*xs), len(xs)


class HEContext:
    """One parameter set on the current device; all work goes to torch's current stream at creation."""

    def __init__(self, logN, q, p, dnum, stream=None):
        self._lib = load()
        if not torch.cuda.is_available():
            raise RuntimeError("no GPU visible: the HIP path has no CPU fallback")
        self.logN, self.N = int(logN), 1 << int(logN)
        self.q, self.p, self.dnum = [int(x) for x in q], [int(x) for x in p], int(dnum)
        self.nq, self.np_ = len(self.q), len(self.p)
        self.stream = torch.cuda.current_stream() if stream is None else stream
        qa = (C.c_uint64 * self.nq)(*self.q)
        pa = (C.c_uint64 * max(1, self.np_))(*(self.p or [0]))
        h = C.c_void_p()
        rc = self._lib.he_ctx_create(C.byref(h), self.logN, qa, self.nq, pa, self.np_, self.dnum,
                                     C.c_void_p(self.stream.cuda_stream))
        if rc != HE_OK:
            raise HEError(rc, self._lib.he_last_error(None).decode())
        self._h = h
        self._keys = {}   # keeps registered key tensors alive

    @classmethod
    def from_params(cls, prm, stream=None):
        return cls(prm.logN, prm.q, prm.p, prm.dnum, stream)

    def close(self):
        if getattr(self, "_h", None):
            self._lib.he_ctx_destroy(self._h)
            self._h = None

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass

    def _ck(self, rc):
        if rc != HE_OK:
            raise HEError(rc, self._lib.he_last_error(self._h).decode())

    # ---- parameters / bookkeeping
    def he_ctx_psi(self, mod_idx):
        v = C.c_uint64()
        self._ck(self._lib.he_ctx_psi(self._h, mod_idx, C.byref(v)))
        return v.value

    def he_counters(self):
        c = Counters()
        self._ck(self._lib.he_counters(self._h, C.byref(c)))
        return {n: getattr(c, n) for n, _ in Counters._fields_}

    def he_counters_reset(self):
        self._ck(self._lib.he_counters_reset(self._h))

    def he_sync(self):
        self._ck(self._lib.he_sync(self._h))

    def he_profile_begin(self):
        self._ck(self._lib.he_profile_begin(self._h))

    def he_profile_end(self):
        p = Profile()
        self._ck(self._lib.he_profile_end(self._h, C.byref(p)))
        return {n: (list(getattr(p, n)) if n.startswith("pass_") else getattr(p, n)) for n, _ in Profile._fields_}

    def he_probe_alu(self):
        p = AluProbe()
        self._ck(self._lib.he_probe_alu(self._h, C.byref(p)))
        return {n: getattr(p, n) for n, _ in AluProbe._fields_}

    def he_build_id(self):
        return self._lib.he_build_id().decode()

    def galois_elt(self, step):
        return pow(5, step % (self.N // 2), 2 * self.N)

    # ---- workspace
    def he_ws_bytes(self):
        v = C.c_uint64()
        self._ck(self._lib.he_ws_bytes(self._h, C.byref(v)))
        return v.value

    def he_ws_reserve(self, nbytes):
        self._ck(self._lib.he_ws_reserve(self._h, int(nbytes)))

    def he_ws_query_rotate_batch(self, level, n_ct, n_steps, hoisted=True):
        v = C.c_uint64()
        self._ck(self._lib.he_ws_query_rotate_batch(self._h, level, n_ct, n_steps, 1 if hoisted else 0, C.byref(v)))
        return v.value

    def he_ws_query_conv2d(self, C_a, H, W, R, f, level, n_out, deferred_taps=False, hoisted_ras=False):
        v = C.c_uint64()
        plan = ConvPlan(C_a, H, W, R, f, n_out, level, 0, 1 if deferred_taps else 0, 1 if hoisted_ras else 0, None)
        self._ck(self._lib.he_ws_query_conv2d(self._h, C.byref(plan), C.byref(v)))
        return v.value

    # ---- transforms
    def he_ntt(self, data, mod_idx):
        arr, n = _u32arr(mod_idx)
        _need(data, n * self.N, "data")
        self._ck(self._lib.he_ntt(self._h, _dev(data), arr, n))
        return data

    def he_intt(self, data, mod_idx):
        arr, n = _u32arr(mod_idx)
        _need(data, n * self.N, "data")
        self._ck(self._lib.he_intt(self._h, _dev(data), arr, n))
        return data

    def he_automorph(self, src, dst, mod_idx, galois_elt, ntt_form=True):
        arr, n = _u32arr(mod_idx)
        _need(src, n * self.N, "src")
        _need(dst, n * self.N, "dst")
        self._ck(self._lib.he_automorph(self._h, _dev(src), _dev(dst), arr, n, galois_elt, 1 if ntt_form else 0))
        return dst

    # ---- key switching
    def he_evk_register(self, galois_elt, evk):
        _need(evk, self.dnum * 2 * (self.nq + self.np_) * self.N, "evk")
        self._ck(self._lib.he_evk_register(self._h, galois_elt, _dev(evk)))
        self._keys[galois_elt] = evk

    def he_keyswitch(self, poly, level, galois_elt_of_key, out0, out1):
        for t, w in ((poly, "poly"), (out0, "out0"), (out1, "out1")):
            _need(t, (level + 1) * self.N, w)
        self._ck(self._lib.he_keyswitch(self._h, _dev(poly), level, galois_elt_of_key, _dev(out0), _dev(out1)))
        return out0, out1

    def he_rotate_hoisted(self, ct, level, steps, outs):
        steps = [int(s) for s in steps]
        if len(outs) != len(steps):
            raise ValueError("one output per step")
        for t in [ct] + list(outs):
            _need(t, 2 * (level + 1) * self.N, "ciphertext")
        sa = (C.c_int32 * max(1, len(steps)))(*steps)
        pa = (C.c_void_p * max(1, len(outs)))(*[_dev(o).value for o in outs])
        self._ck(self._lib.he_rotate_hoisted(self._h, _dev(ct), level, sa, len(steps), pa))
        return outs

    def he_rotate_batch(self, cts, level, steps, outs, hoisted=True):
        """outs[c*len(steps) + s] = CRot(cts[c]; steps[s])."""
        steps = [int(s) for s in steps]
        if len(outs) != len(cts) * len(steps):
            raise ValueError("need len(cts)*len(steps) outputs")
        for t in list(cts) + list(outs):
            _need(t, 2 * (level + 1) * self.N, "ciphertext")
        sa = (C.c_int32 * max(1, len(steps)))(*steps)
        ca = (C.c_void_p * max(1, len(cts)))(*[_dev(c).value for c in cts])
        oa = (C.c_void_p * max(1, len(outs)))(*[_dev(o).value for o in outs])
        self._ck(self._lib.he_rotate_batch(self._h, ca, len(cts), level, sa, len(steps), oa, 1 if hoisted else 0))
        return outs

    def he_rotate_sum(self, cts, level, steps, out, deferred=False):
        """out = sum_t CRot(cts[t]; steps[t]); deferred=True shares one ModDown across the sum."""
        steps = [int(s) for s in steps]
        if len(cts) != len(steps):
            raise ValueError("one step per ciphertext")
        for t in list(cts) + [out]:
            _need(t, 2 * (level + 1) * self.N, "ciphertext")
        sa = (C.c_int32 * max(1, len(steps)))(*steps)
        ca = (C.c_void_p * max(1, len(cts)))(*[_dev(c).value for c in cts])
        self._ck(self._lib.he_rotate_sum(self._h, ca, len(cts), level, sa, _dev(out), 1 if deferred else 0))
        return out

    def he_rotate(self, ct, level, step, out):
        _need(ct, 2 * (level + 1) * self.N, "ct")
        _need(out, 2 * (level + 1) * self.N, "out")
        self._ck(self._lib.he_rotate(self._h, _dev(ct), level, int(step), _dev(out)))
        return out

    def he_conjugate(self, ct, level, out):
        _need(ct, 2 * (level + 1) * self.N, "ct")
        _need(out, 2 * (level + 1) * self.N, "out")
        self._ck(self._lib.he_conjugate(self._h, _dev(ct), level, _dev(out)))
        return out

    # ---- MulPt accumulate / add / rescale
    def he_ptct_mac(self, acc, ct, pt, level, init):
        _need(acc, 2 * (level + 1) * self.N, "acc")
        _need(ct, 2 * (level + 1) * self.N, "ct")
        _need(pt, (level + 1) * self.N, "pt")
        self._ck(self._lib.he_ptct_mac(self._h, _dev(acc), _dev(ct), _dev(pt), level, 1 if init else 0))
        return acc

    def he_add(self, a, b, level, out):
        for t, w in ((a, "a"), (b, "b"), (out, "out")):
            _need(t, 2 * (level + 1) * self.N, w)
        self._ck(self._lib.he_add(self._h, _dev(a), _dev(b), level, _dev(out)))
        return out

    def he_addpt(self, ct, pt, level, out):
        _need(ct, 2 * (level + 1) * self.N, "ct")
        _need(pt, (level + 1) * self.N, "pt")
        _need(out, 2 * (level + 1) * self.N, "out")
        self._ck(self._lib.he_addpt(self._h, _dev(ct), _dev(pt), level, _dev(out)))
        return out

    def he_mulct(self, a, b, level, out):
        for t, w in ((a, "a"), (b, "b"), (out, "out")):
            _need(t, 2 * (level + 1) * self.N, w)
        self._ck(self._lib.he_mulct(self._h, _dev(a), _dev(b), level, _dev(out)))
        return out

    def he_affine(self, ct, level, mul, add, out):
        """mul/add: Python ints per limb (any sign); reduced to canonical residues here."""
        _need(ct, 2 * (level + 1) * self.N, "ct")
        _need(out, 2 * (level + 1) * self.N, "out")
        m = (C.c_uint64 * (level + 1))(*[int(mul[r]) % self.q[r] for r in range(level + 1)])
        a = (C.c_uint64 * (level + 1))(*[int(add[r]) % self.q[r] for r in range(level + 1)])
        self._ck(self._lib.he_affine(self._h, _dev(ct), level, m, a, _dev(out)))
        return out

    def he_rescale(self, ct, level, out):
        _need(ct, 2 * (level + 1) * self.N, "ct")
        _need(out, 2 * level * self.N, "out")
        self._ck(self._lib.he_rescale(self._h, _dev(ct), level, _dev(out)))
        return out

    def he_rescale_noalloc(self, ct, level, out):
        _need(ct, 2 * (level + 1) * self.N, "ct")
        _need(out, 2 * level * self.N, "out")
        self._ck(self._lib.he_rescale_noalloc(self._h, _dev(ct), level, _dev(out)))
        return out

    # ---- convolution
    def he_ras(self, cts, level, steps, outs):
        """outs[i] = cts[i] after ct <- ct + CRot(ct; s) for every s in steps, all ciphertexts batched."""
        steps = [int(s) for s in steps]
        if len(outs) != len(cts):
            raise ValueError("one output per ciphertext")
        for t in list(cts) + list(outs):
            _need(t, 2 * (level + 1) * self.N, "ciphertext")
        sa = (C.c_int32 * max(1, len(steps)))(*steps)
        ca = (C.c_void_p * max(1, len(cts)))(*[_dev(c).value for c in cts])
        oa = (C.c_void_p * max(1, len(outs)))(*[_dev(o).value for o in outs])
        self._ck(self._lib.he_ras(self._h, ca, len(cts), level, sa, len(steps), oa))
        return outs

    def he_conv2d(self, C_a, H, W, R, f, level, weights, ct_in, outs, skip_ras=False, deferred_taps=False, hoisted_ras=False):
        """weights: list of n_out*f*f device tensors [level+1][N] ([level+1+np][N], over the raised basis, with
        deferred_taps); outs: n_out tensors [2][level][N]."""
        n_out = len(outs)
        if len(weights) != n_out * f * f:
            raise ValueError("need n_out*f*f weight plaintexts")
        _need(ct_in, 2 * (level + 1) * self.N, "ct_in")
        for w in weights:
            _need(w, (level + 1 + (self.np_ if deferred_taps else 0)) * self.N, "weight plaintext")
        for o in outs:
            _need(o, 2 * level * self.N, "output")
        wa = (C.c_void_p * len(weights))(*[_dev(w).value for w in weights])
        oa = (C.c_void_p * n_out)(*[_dev(o).value for o in outs])
        plan = ConvPlan(C_a, H, W, R, f, n_out, level, 1 if skip_ras else 0, 1 if deferred_taps else 0, 1 if hoisted_ras else 0,
                        C.cast(wa, C.POINTER(C.c_void_p)))
        self._ck(self._lib.he_conv2d(self._h, C.byref(plan), _dev(ct_in), oa))
        return outs

    def he_ptct_mac_rot(self, acc, cts, pts, galois, level, init=True):
        """acc (= | +=) sum_i cts[i] * sigma_{galois[i]}(pts[i]) (plaintexts rotated on the fly)."""
        if not (len(cts) == len(pts) == len(galois)):
            raise ValueError("cts, pts and galois must have the same length")
        _need(acc, 2 * (level + 1) * self.N, "acc")
        for c in cts:
            _need(c, 2 * (level + 1) * self.N, "ciphertext")
        for p in pts:
            _need(p, (level + 1) * self.N, "plaintext")
        n = len(cts)
        ca = (C.c_void_p * max(1, n))(*[_dev(c).value for c in cts])
        pa = (C.c_void_p * max(1, n))(*[_dev(p).value for p in pts])
        ga = (C.c_uint32 * max(1, n))(*[int(g) for g in galois])
        self._ck(self._lib.he_ptct_mac_rot(self._h, _dev(acc), ca, pa, ga, n, level, 1 if init else 0))
        return acc

    def he_ws_query_raconv(self, n_in, W, R, f, level, deferred=False):
        v = C.c_uint64()
        plan = RaConvPlan(n_in, W, R, f, level, 1 if deferred else 0, None)
        self._ck(self._lib.he_ws_query_raconv(self._h, C.byref(plan), C.byref(v)))
        return v.value

    def he_raconv(self, W, R, f, level, weights, cts_in, out, deferred=False):
        """weights: list of n_in*f*f device tensors [level+1][N] (input-major); cts_in: n_in tensors
        [2][level+1][N]; out: [2][level][N]."""
        n_in = len(cts_in)
        if len(weights) != n_in * f * f:
            raise ValueError("need n_in*f*f weight plaintexts")
        for c in cts_in:
            _need(c, 2 * (level + 1) * self.N, "input")
        for w in weights:
            _need(w, (level + 1) * self.N, "weight plaintext")
        _need(out, 2 * level * self.N, "out")
        wa = (C.c_void_p * len(weights))(*[_dev(w).value for w in weights])
        ia = (C.c_void_p * n_in)(*[_dev(c).value for c in cts_in])
        plan = RaConvPlan(n_in, W, R, f, level, 1 if deferred else 0, C.cast(wa, C.POINTER(C.c_void_p)))
        self._ck(self._lib.he_raconv(self._h, C.byref(plan), ia, _dev(out)))
        return out

    def _block_plan(self, C_a, H, W, R, f, n_ca, n_ra, level, group, deferred, k_in, w_ca, w_ra, hoisted_ras=False):
        ka = (C.c_uint64 * level)(*[int(k_in) % self.q[r] for r in range(level)])
        ca = (C.c_void_p * max(1, len(w_ca)))(*[_dev(w).value for w in w_ca])
        ra = (C.c_void_p * max(1, len(w_ra)))(*[_dev(w).value for w in w_ra])
        plan = BlockPlan(C_a, H, W, R, f, n_ca, n_ra, level, group, 1 if deferred else 0, 1 if hoisted_ras else 0, ka,
                         C.cast(ca, C.POINTER(C.c_void_p)), C.cast(ra, C.POINTER(C.c_void_p)))
        return plan, (ka, ca, ra)

    def he_ws_query_ca_ra_block(self, C_a, H, W, R, f, n_ca, n_ra, level, group=0, deferred=False, hoisted_ras=False):
        v = C.c_uint64()
        plan, _keep = self._block_plan(C_a, H, W, R, f, n_ca, n_ra, level, group, deferred, 1, [], [], hoisted_ras)
        self._ck(self._lib.he_ws_query_ca_ra_block(self._h, C.byref(plan), C.byref(v)))
        return v.value

    def he_ca_ra_block(self, C_a, H, W, R, f, level, k_in, w_ca, w_ra, cts_in, outs, group=0, deferred=False, hoisted_ras=False):
        """Fused CAConv -> Square -> RAConv block.  w_ca: n_ra*n_ca*f*f plaintexts at `level` ([j][k][tap]); w_ra:
        n_ca*n_ra*f*f inversely rotated plaintexts at level-2 ([l][j][tap]); cts_in / outs: n_ca tensors at `level` /
        level-3; k_in: the integer lift before the square (reduced per limb here)."""
        n_ca = len(cts_in)
        if len(outs) != n_ca or len(w_ca) % (n_ca * f * f) or len(w_ra) != len(w_ca):
            raise ValueError("need n_ca outputs and n_ra*n_ca*f*f plaintexts for each convolution")
        n_ra = len(w_ca) // (n_ca * f * f)
        for c in cts_in:
            _need(c, 2 * (level + 1) * self.N, "input")
        for o in outs:
            _need(o, 2 * (level - 2) * self.N, "output")
        for w in w_ca:
            _need(w, (level + 1) * self.N, "CAConv weight plaintext")
        for w in w_ra:
            _need(w, (level - 1) * self.N, "RAConv weight plaintext")
        plan, _keep = self._block_plan(C_a, H, W, R, f, n_ca, n_ra, level, group, deferred, k_in, w_ca, w_ra, hoisted_ras)
        ia = (C.c_void_p * n_ca)(*[_dev(c).value for c in cts_in])
        oa = (C.c_void_p * n_ca)(*[_dev(o).value for o in outs])
        self._ck(self._lib.he_ca_ra_block(self._h, C.byref(plan), ia, oa))
        return outs
