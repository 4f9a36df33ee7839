"""GPU parity for PRCR on pointwise filters (paper Section 3.3): he_ptct_mac_rot (MulPt-accumulate with the plaintext
rotated on the fly) against the oracle's rotate-then-multiply, the two layer directions sequenced over the C ABI
against oracle/prcr.py bit for bit and against float64, and the entry point's argument checks."""
import numpy as np
import pytest

from he_inputs import sampling as S
from he_inputs.params import config_params, toy_params

pytestmark = pytest.mark.gpu


def _setup(prm, seed):
    from oracle import ckks_client as K
    from oracle.he_oracle import Oracle
    from paper_2302_02407_amd.binding import HEContext
    rng = S.make_rng(seed)
    orc, ctx = Oracle.from_params(prm), HEContext.from_params(prm)
    cl = K.Client(orc, S.ternary_secret(rng, prm.N, prm.hamming))
    return rng, orc, ctx, cl


@pytest.mark.parametrize("logN,n,level", [(10, 5, 2), (13, 20, 3), (16, 3, 5)])
def test_mac_with_rotated_plaintexts(logN, n, level):
    """n random (ciphertext, plaintext, Galois element) terms, uniform residues: one fused call (n > 16 takes two
    launches) equals rotating each plaintext and multiplying; then accumulation onto an existing value."""
    from gpu_util import dev, host, zeros
    from oracle import prcr as PR
    prm = config_params(2) if logN == 16 else toy_params(logN=logN, q_bits=40, nq=4, p_bits=41, np_=1, dnum=2, scale=2.0 ** 30,
                                                         hamming=16, seed=90 + logN)
    rng, orc, ctx, cl = _setup(prm, 90 + logN)
    N, qs = prm.N, prm.q[:level + 1]
    cts = [np.stack([S.uniform_limbs(rng, qs, N)[0] for _ in range(2)]) for _ in range(n)]
    pts = [S.uniform_limbs(rng, qs, N)[0] for _ in range(n)]
    gs = [1 if i == 1 else orc.galois_elt(int(rng.integers(1, N // 2))) for i in range(n)]
    gs[-1] = orc.galois_conj
    want = PR.mac_rotated_plaintexts(orc, cts, pts, gs, level)
    d_cts, d_pts = [dev(c) for c in cts], [dev(p) for p in pts]
    acc = zeros(2, level + 1, N)
    ctx.he_counters_reset()
    ctx.he_ptct_mac_rot(acc, d_cts, d_pts, gs, level, init=True)
    assert (host(acc) == want).all()
    assert ctx.he_counters()["mac"] == n
    ctx.he_ptct_mac_rot(acc, d_cts[:2], d_pts[:2], gs[:2], level, init=False)
    more = PR.mac_rotated_plaintexts(orc, cts[:2], pts[:2], gs[:2], level)
    assert (host(acc) == orc.add(want, more, level)).all()
    ctx.he_ptct_mac_rot(acc, [], [], [], level, init=True)
    assert not host(acc).any()


def _layers(prm, Sg, H, W, level, seed, tol):
    from gpu_util import dev, host, zeros
    from oracle import prcr as PR
    from paper_2302_02407_amd import block as blk
    rng, orc, ctx, cl = _setup(prm, seed)
    geo = PR.PrcrGeometry(prm.N, Sg, H, W)
    x = rng.uniform(-1, 1, (Sg, H, W))
    w1, w2 = rng.normal(0, 0.4, (Sg, Sg)), rng.normal(0, 0.4, (Sg, Sg))

    def enc(z, lv):
        return cl.encrypt(np.asarray(z).astype(np.complex128), prm.scale, lv, S.uniform_limbs(rng, prm.q[:lv + 1], prm.N)[0],
                          S.gaussian_error(rng, prm.N, prm.sigma)[0])
    # whole images -> rearranged format -> whole images: conv(conv(x))
    F = [enc(geo.pack_full(x[c]), level) for c in range(Sg)]
    Q = PR.encode_plaintexts(orc, geo, w1, level, float(prm.q[level]), "ra")
    P = PR.encode_plaintexts(orc, geo, w2, level - 1, float(prm.q[level - 1]), "ca")
    Y_want = PR.raconv_1x1(orc, geo, F, level, Q)
    G_want = PR.caconv_1x1(orc, geo, Y_want, level - 1, P)
    Y = blk.prcr_raconv_1x1(ctx, Sg, geo.frag, level, [dev(q) for q in Q], [dev(f) for f in F], [zeros(2, level, prm.N) for _ in range(Sg)])
    for k in range(Sg):
        assert (host(Y[k]) == Y_want[k]).all(), k
    G = blk.prcr_caconv_1x1(ctx, Sg, geo.frag, level - 1, [dev(p) for p in P], Y, [zeros(2, level - 1, prm.N) for _ in range(Sg)])
    ref = np.einsum("oc,chw->ohw", w2, np.einsum("oc,chw->ohw", w1, x))
    for o in range(Sg):
        got = host(G[o])
        assert (got == G_want[o]).all(), o
        img, spread = geo.unpack_full(cl.decrypt(got, level - 2, prm.scale))
        assert np.max(np.abs(img - ref[o])) < tol and spread < tol
    mid = geo.unpack_ca([cl.decrypt(host(y), level - 1, prm.scale) for y in Y])
    assert np.max(np.abs(mid - np.einsum("oc,chw->ohw", w1, x))) < tol


def test_layers_small_ring():
    prm = toy_params(logN=10, q_bits=40, nq=4, p_bits=41, np_=1, dnum=2, scale=2.0 ** 30, hamming=32, seed=95)
    _layers(prm, Sg=4, H=16, W=8, level=3, seed=95, tol=1e-4)


def test_layers_n65536_eight_segments():
    # the paper's |S| = 8 on a 64x64 image with 8 replicas at N = 2^16 (8 plaintexts stand for 64)
    _layers(config_params(3), Sg=8, H=64, W=64, level=4, seed=96, tol=1e-4)


def test_argument_checks():
    from gpu_util import dev, zeros
    from paper_2302_02407_amd.binding import HEError
    prm = toy_params(logN=10, q_bits=40, nq=3, p_bits=41, np_=1, dnum=3, scale=2.0 ** 30, hamming=32, seed=97)
    rng, orc, ctx, cl = _setup(prm, 97)
    N, level = prm.N, 2
    ct, pt, acc = zeros(2, level + 1, N), zeros(level + 1, N), zeros(2, level + 1, N)
    with pytest.raises(HEError):
        ctx.he_ptct_mac_rot(acc, [ct], [pt], [4], level)            # even Galois element
    with pytest.raises(HEError):
        ctx.he_ptct_mac_rot(acc, [ct], [pt], [2 * N + 1], level)    # not below 2N
    with pytest.raises(HEError):
        ctx.he_ptct_mac_rot(ct, [ct], [pt], [5], level)             # accumulator is an operand
    with pytest.raises(HEError):
        ctx.he_ptct_mac_rot(zeros(2, 4, N), [zeros(2, 4, N)], [zeros(4, N)], [5], 3)   # level above L
    ctx.he_ptct_mac_rot(acc, [ct], [pt], [5], level)
