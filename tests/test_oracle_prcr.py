"""Pins of the PRCR reading for pointwise filters (oracle/prcr.py): (i) the channel-aligned form decrypts to the
float64 1x1 convolution as whole images; (ii) the replication-aligned form returns the rearranged format, segment by
segment; (iii) chained, they give conv(conv(x)); (iv) a reused plaintext rotated by k fragments is the plaintext one
would have encoded for the pair without reuse (so S plaintexts stand for S*S); (v) the rotation of a plaintext is a
pure permutation of its NTT-form residues (no key, no arithmetic)."""
import numpy as np

from he_inputs import sampling as S
from he_inputs.params import toy_params
from oracle import ckks_client as K
from oracle import prcr as PR
from oracle.ckks_client import encode
from oracle.he_oracle import Oracle


def _setup(seed, logN=8, Sg=4, H=8, W=4):
    prm = toy_params(logN=logN, q_bits=40, nq=4, p_bits=41, np_=1, dnum=2, scale=2.0 ** 30, hamming=16, seed=seed)
    rng = S.make_rng(seed)
    orc = Oracle.from_params(prm)
    cl = K.Client(orc, S.ternary_secret(rng, prm.N, prm.hamming))
    geo = PR.PrcrGeometry(prm.N, Sg, H, W)
    return prm, rng, orc, cl, geo


def _enc(cl, prm, rng, z, level):
    return cl.encrypt(np.asarray(z).astype(np.complex128), prm.scale, level, S.uniform_limbs(rng, prm.q[:level + 1], prm.N)[0],
                      S.gaussian_error(rng, prm.N, prm.sigma)[0])


def test_channel_aligned_form_gives_whole_images():
    prm, rng, orc, cl, geo = _setup(61)
    level = 3
    x = rng.uniform(-1, 1, (geo.S, geo.H, geo.W))
    wt = rng.normal(0, 0.4, (geo.S, geo.S))
    X = [_enc(cl, prm, rng, geo.pack_ca(x, k), level) for k in range(geo.S)]
    P = PR.encode_plaintexts(orc, geo, wt, level, float(prm.q[level]), "ca")
    F = PR.caconv_1x1(orc, geo, X, level, P)
    ref = np.einsum("oc,chw->ohw", wt, x)
    for o in range(geo.S):
        img, spread = geo.unpack_full(cl.decrypt(F[o], level - 1, prm.scale))
        assert np.max(np.abs(img - ref[o])) < 1e-4 and spread < 1e-4


def test_replication_aligned_form_returns_the_rearranged_format_and_chains():
    prm, rng, orc, cl, geo = _setup(62)
    level = 3
    x = rng.uniform(-1, 1, (geo.S, geo.H, geo.W))
    w1 = rng.normal(0, 0.4, (geo.S, geo.S))
    w2 = rng.normal(0, 0.4, (geo.S, geo.S))
    F = [_enc(cl, prm, rng, geo.pack_full(x[c]), level) for c in range(geo.S)]
    Q = PR.encode_plaintexts(orc, geo, w1, level, float(prm.q[level]), "ra")
    Y = PR.raconv_1x1(orc, geo, F, level, Q)
    mid = np.einsum("oc,chw->ohw", w1, x)
    got = geo.unpack_ca([cl.decrypt(y, level - 1, prm.scale) for y in Y])
    assert np.max(np.abs(got - mid)) < 1e-4
    # segment s of Y_k is channel (k+s) mod S and nothing else
    v = np.asarray(cl.decrypt(Y[1], level - 1, prm.scale)).real.reshape(geo.H, geo.W, geo.R)[:, :, 0]
    for s in range(geo.S):
        assert np.max(np.abs(v[s * geo.Hs:(s + 1) * geo.Hs] - mid[(1 + s) % geo.S, s * geo.Hs:(s + 1) * geo.Hs])) < 1e-4
    # ... which is what the channel-aligned form consumes
    P = PR.encode_plaintexts(orc, geo, w2, level - 1, float(prm.q[level - 1]), "ca")
    G = PR.caconv_1x1(orc, geo, Y, level - 1, P)
    ref = np.einsum("oc,chw->ohw", w2, mid)
    for o in range(geo.S):
        img, _ = geo.unpack_full(cl.decrypt(G[o], level - 2, prm.scale))
        assert np.max(np.abs(img - ref[o])) < 1e-4


def test_rotated_plaintext_is_the_plaintext_of_the_pair():
    prm, rng, orc, cl, geo = _setup(63)
    level, mods = 2, [0, 1, 2]
    wt = rng.normal(0, 0.4, (geo.S, geo.S))
    P = PR.encode_plaintexts(orc, geo, wt, level, 2.0 ** 20, "ca")
    for o in (0, 2):
        for k in range(geo.S):
            # the plaintext one would encode for (output o, input ciphertext k) without reuse
            direct = np.repeat(np.asarray([wt[o, (s + k) % geo.S] for s in range(geo.S)]), geo.frag)
            want = orc.ntt(orc.reduce_signed(encode(direct.astype(np.complex128), orc.N, 2.0 ** 20), mods), mods)
            got = P[o] if k == 0 else orc.automorph_ntt(P[o], orc.galois_elt(k * geo.frag))
            # equal as polynomials up to the rounding of the two encodings (at most one unit per coefficient)
            d = orc.intt(got, mods).astype(np.int64) - orc.intt(want, mods).astype(np.int64)
            q0 = int(prm.q[0])
            d0 = np.minimum(np.abs(d[0]), q0 - np.abs(d[0]))
            assert d0.max() <= 1, (o, k, d0.max())
    assert len(P) == geo.S                                           # S plaintexts for S*S (output, input) pairs


def test_plaintext_rotation_is_a_permutation_of_residues():
    prm, rng, orc, cl, geo = _setup(64)
    pt = S.uniform_limbs(rng, prm.q[:3], prm.N)[0]
    r = orc.automorph_ntt(pt, orc.galois_elt(geo.frag))
    for limb in range(3):
        assert sorted(pt[limb].tolist()) == sorted(r[limb].tolist())
    back = orc.automorph_ntt(r, orc.galois_elt(prm.N // 2 - geo.frag))
    assert (back == pt).all()
