"""Pins at the scheme level: encode/decode definition, Dec(Enc), Dec(Rot_r(Enc z)) = roll(z,-r),
conjugation, hoisted == single, MulPt + Rescale multiplies slot-wise."""
import numpy as np
import pytest

from he_inputs import sampling as S
from he_inputs.params import config_params, toy_params
from oracle import ckks_client as K
from oracle.he_oracle import Oracle


def test_encode_matches_definition_and_roundtrips():
    N, scale = 32, 2.0 ** 20
    rng = S.make_rng(31)
    z = rng.uniform(-1, 1, N // 2) + 1j * rng.uniform(-1, 1, N // 2)
    m = K.encode(z, N, scale)
    md = K.encode_def(z, N, scale)
    assert np.max(np.abs(m - md)) <= 1          # same rounding up to float noise at .5 boundaries
    assert np.max(np.abs(K.decode(m, N, scale) - z)) < 1e-4
    assert np.max(np.abs(K.decode_def(m, N, scale) - K.decode(m, N, scale))) < 1e-9
    # a single slot set to 1 encodes to the (scaled, rounded) basis polynomial of that slot
    e0 = np.zeros(N // 2, dtype=np.complex128)
    e0[3] = 1.0
    dec = K.decode(K.encode(e0, N, 2.0 ** 30), N, 2.0 ** 30)
    assert abs(dec[3] - 1) < 1e-6 and np.max(np.abs(np.delete(dec, 3))) < 1e-6


def _client(prm, rng):
    o = Oracle.from_params(prm)
    s = S.ternary_secret(rng, prm.N, prm.hamming)
    return o, K.Client(o, s)


@pytest.mark.parametrize("logN,level", [(4, 5), (4, 2), (6, 4)])
def test_rotation_and_conjugation_semantics(logN, level):
    prm = toy_params(logN=logN)
    rng = S.make_rng(32)
    o, cl = _client(prm, rng)
    N = prm.N
    z = rng.uniform(-1, 1, N // 2) + 1j * rng.uniform(-1, 1, N // 2)
    ct = cl.encrypt(z, prm.scale, level, S.uniform_limbs(rng, prm.q[:level + 1], N)[0], S.gaussian_error(rng, N)[0])
    assert np.max(np.abs(cl.decrypt(ct, level, prm.scale) - z)) < 1e-4
    raised = o.modup(ct[1], level)
    for r in (1, 2, N // 4, N // 2 - 1, -3):
        g = o.galois_elt(r)
        evk = cl.rotation_key(g, S.uniform_limbs(rng, prm.moduli, N, prm.dnum), S.gaussian_error(rng, N, 3.2, prm.dnum))
        rot = o.rotate(ct, level, g, evk)
        assert np.max(np.abs(cl.decrypt(rot, level, prm.scale) - np.roll(z, -r))) < 2e-4   # LEFT by r
        # hoisted (shared ModUp) and single rotations are the same bits
        assert (o.rotate_from_raised(ct, raised, level, g, evk) == rot).all()
    g = o.galois_conj
    evk = cl.rotation_key(g, S.uniform_limbs(rng, prm.moduli, N, prm.dnum), S.gaussian_error(rng, N, 3.2, prm.dnum))
    assert np.max(np.abs(cl.decrypt(o.rotate(ct, level, g, evk), level, prm.scale) - np.conj(z))) < 2e-4


def test_mulpt_rescale_multiplies_slots():
    prm = toy_params(logN=5)
    rng = S.make_rng(33)
    o, cl = _client(prm, rng)
    N, level = prm.N, 4
    z = rng.uniform(-1, 1, N // 2).astype(np.complex128)
    w = rng.uniform(-1, 1, N // 2).astype(np.complex128)
    ct = cl.encrypt(z, prm.scale, level, S.uniform_limbs(rng, prm.q[:level + 1], N)[0], S.gaussian_error(rng, N)[0])
    ql = float(prm.q[level])
    mods = list(range(level + 1))
    pt = o.ntt(o.reduce_signed(K.encode(w, N, ql), mods), mods)      # plaintext at scale q_level
    prod = o.rescale(o.ptct_mac(None, ct, pt, level, init=True), level)
    got = cl.decrypt(prod, level - 1, prm.scale)                     # scale Delta*q/q = Delta
    assert np.max(np.abs(got - z * w)) < 5e-4


def test_rotation_at_full_size_config2():
    prm = config_params(2)
    rng = S.make_rng(prm.seed)
    o, cl = _client(prm, rng)
    N, level = prm.N, 2            # low level keeps the CPU time small; key is full size
    z = rng.uniform(-1, 1, N // 2).astype(np.complex128)
    ct = cl.encrypt(z, prm.scale, level, S.uniform_limbs(rng, prm.q[:level + 1], N)[0], S.gaussian_error(rng, N)[0])
    g = o.galois_elt(1 << 14)
    evk = cl.rotation_key(g, S.uniform_limbs(rng, prm.moduli, N, prm.dnum), S.gaussian_error(rng, N, 3.2, prm.dnum))
    rot = o.rotate(ct, level, g, evk)
    err = np.abs(cl.decrypt(rot, level, prm.scale) - np.roll(z, -(1 << 14)))
    # ModDown without a rounding/overflow correction leaves an error polynomial with a
    # non-zero mean (-u, 0 <= u < k per coefficient); a constant-ish polynomial evaluates to
    # ~2N/pi at the slots whose root is nearest 1, so slot 0 carries ~k/2*(1+|s(zeta)|)*2N/pi/Delta.
    assert err.max() < 2e-5 and np.median(err) < 1e-7


def test_mulct_tensor_relin_and_affine():
    """MulCt: Dec(MulCt(Enc a, Enc b)) = a*b slot-wise, before the rescale (CRT lift at scale Delta^2)
    and after it; affine map (negate, integer multiple, constant add) against its slot meaning."""
    prm = toy_params(logN=5, q_bits=30, nq=6, p_bits=32, np_=2, dnum=3, scale=2.0 ** 25, hamming=8, seed=34)
    rng = S.make_rng(34)
    o, cl = _client(prm, rng)
    N, level = prm.N, 5
    za = rng.uniform(-1, 1, N // 2).astype(np.complex128)
    zb = rng.uniform(-1, 1, N // 2).astype(np.complex128)
    enc = lambda z: cl.encrypt(z, prm.scale, level, S.uniform_limbs(rng, prm.q[:level + 1], N)[0], S.gaussian_error(rng, N)[0])
    ca, cb = enc(za), enc(zb)
    rlk = cl.relin_key(S.uniform_limbs(rng, prm.moduli, N, prm.dnum), S.gaussian_error(rng, N, 3.2, prm.dnum))
    prod = o.mulct(ca, cb, level, rlk)
    res = o.rescale(prod, level)
    scale = prm.scale * prm.scale / prm.q[level]
    got = cl.decrypt(res, level - 1, scale)
    assert np.max(np.abs(got - za * zb)) < 2e-3
    # phase check of the relinearisation itself: Dec before rescale at scale Delta^2 with a CRT lift
    got2 = cl.decrypt_crt(prod, level, prm.scale * prm.scale, limbs=3)
    assert np.max(np.abs(got2 - za * zb)) < 2e-3
    # affine: -ct, 3*ct, ct + 1.5
    neg = o.affine(ca, level, [-1] * (level + 1), [0] * (level + 1))
    assert np.max(np.abs(cl.decrypt(neg, level, prm.scale) + za)) < 1e-4
    tri = o.affine(ca, level, [3] * (level + 1), [0] * (level + 1))
    assert np.max(np.abs(cl.decrypt(tri, level, prm.scale) - 3 * za)) < 1e-4
    k = int(round(1.5 * prm.scale))
    plus = o.affine(ca, level, [1] * (level + 1), [k] * (level + 1))
    assert np.max(np.abs(cl.decrypt(plus, level, prm.scale) - (za + 1.5))) < 1e-4
    # dropping a limb keeps the message
    low = o.drop_level(ca, level)
    assert np.max(np.abs(cl.decrypt(low, level - 1, prm.scale) - za)) < 1e-4


def test_addpt_adds_slots_and_prot_rotates_a_plaintext():
    """AddPt: Dec(AddPt(Enc z, Encode b)) = z + b.  PRot: the automorphism applied to an NTT-form plaintext
    is the encoding of the rotated vector (it equals encoding the rolled vector up to rounding)."""
    prm = toy_params(logN=6)
    rng = S.make_rng(35)
    o, cl = _client(prm, rng)
    N, level = prm.N, 3
    mods = list(range(level + 1))
    z = rng.uniform(-1, 1, N // 2)
    b = rng.uniform(-1, 1, N // 2)
    ct = cl.encrypt(z.astype(np.complex128), prm.scale, level, S.uniform_limbs(rng, prm.q[:level + 1], N)[0],
                    S.gaussian_error(rng, N, prm.sigma)[0])
    pt = o.ntt(o.reduce_signed(K.encode(b.astype(np.complex128), N, prm.scale), mods), mods)
    out = o.addpt(ct, pt, level)
    assert (out[1] == ct[1]).all()
    assert np.max(np.abs(cl.decrypt(out, level, prm.scale) - (z + b))) < 1e-3
    # PRot by r: sigma_{5^r} on the plaintext; multiplying by it acts on the slots rolled left by r
    r = 5
    rot = o.automorph_ntt(pt, o.galois_elt(r))
    want = o.ntt(o.reduce_signed(K.encode(np.roll(b, -r).astype(np.complex128), N, prm.scale), mods), mods)
    diff = K.centered(o.intt(rot, mods)[0], prm.q[0]) - K.centered(o.intt(want, mods)[0], prm.q[0])
    assert np.max(np.abs(diff)) <= 2             # same polynomial up to the rounding of the two encodings
