"""Pin of the oracle's fused CAConv -> Square -> RAConv block in the loop order of Algorithm 3, with one and with
two channel-aligned ciphertexts, against float64: conv(conv(x, w1)^2, w2); and against the plain sequence of the
three layers where that exists (one input ciphertext)."""
import numpy as np
import pytest

from he_inputs import sampling as S
from he_inputs.params import toy_params
from oracle import block as OB
from oracle import ckks_client as K
from oracle import conv2d as CV
from oracle.he_oracle import Oracle


def fused_inputs(prm, C_a, H, W, c_in, c_mid, level, std, seed, all_ras_multiples=False):
    """Everything the block consumes, for n_CA = c_in / C_a input ciphertexts (shared with the GPU parity test).
    all_ras_multiples: also the keys of every multiple of H*W*R below C_a (the hoisted rotate-and-sum), drawn last."""
    rng = S.make_rng(seed)
    orc = Oracle.from_params(prm)
    cl = K.Client(orc, S.ternary_secret(rng, prm.N, prm.hamming))
    N, q = prm.N, prm.q
    n_ca = c_in // C_a
    g_ca, g_ra = CV.ConvGeometry(N, C_a, H, W, c_mid, f=3), CV.RAGeometry(N, C_a, H, W, c_mid, f=3)
    x = rng.uniform(-1.0, 1.0, size=(c_in, H, W))
    w1 = rng.normal(0.0, std, size=(c_mid, c_in, 3, 3))
    w2 = rng.normal(0.0, std, size=(c_in, c_mid, 3, 3))
    steps = sorted(set(s for s in g_ca.tap_steps if s) | set(g_ca.ras_steps))
    evks = {st: cl.rotation_key(orc.galois_elt(st), S.uniform_limbs(rng, prm.moduli, N, prm.dnum),
                                S.gaussian_error(rng, N, prm.sigma, prm.dnum)) for st in steps}
    rlk = cl.relin_key(S.uniform_limbs(rng, prm.moduli, N, prm.dnum), S.gaussian_error(rng, N, prm.sigma, prm.dnum))
    cts = [cl.encrypt(g_ca.pack_input(x[k * C_a:(k + 1) * C_a]).astype(np.complex128), prm.scale, level,
                      S.uniform_limbs(rng, q[:level + 1], N)[0], S.gaussian_error(rng, N, prm.sigma)[0]) for k in range(n_ca)]
    k_in = int(round(q[level - 1] / prm.scale))
    s_out = (prm.scale * k_in) ** 2 / q[level - 1]
    # p_ca[j][k]: filters of (intermediate j, input k); p_ra[l][j]: inversely rotated filters of (output l, intermediate j)
    p_ca = [[None] * n_ca for _ in range(g_ca.n_out)]
    for k in range(n_ca):
        pk = CV.encode_weights(orc, g_ca, w1[:, k * C_a:(k + 1) * C_a], level, float(q[level]))
        for j in range(g_ca.n_out):
            p_ca[j][k] = pk[j]
    p_ra = [[None] * g_ra.n_in for _ in range(n_ca)]
    for l in range(n_ca):
        pl = CV.encode_ra_weights(orc, g_ra, w2[l * C_a:(l + 1) * C_a], level - 2, float(q[level - 2]))
        for j in range(g_ra.n_in):
            p_ra[l][j] = pl[j]
    if all_ras_multiples:
        base = g_ca.H * g_ca.W * g_ca.R
        for i in range(1, C_a):
            if base * i not in evks:
                evks[base * i] = cl.rotation_key(orc.galois_elt(base * i), S.uniform_limbs(rng, prm.moduli, N, prm.dnum),
                                                 S.gaussian_error(rng, N, prm.sigma, prm.dnum))
    return dict(orc=orc, cl=cl, g_ca=g_ca, g_ra=g_ra, x=x, w1=w1, w2=w2, evks=evks, rlk=rlk, cts=cts, k_in=k_in,
                s_out=s_out, p_ca=p_ca, p_ra=p_ra, n_ca=n_ca)


def check_fused_output(d, outs, level, tol=1e-3):
    """Decrypted outputs against conv(conv(x, w1)^2, w2); with R channels per intermediate ciphertext each replica
    position r holds the partial sum over the intermediate channels of its class."""
    g = d["g_ra"]
    mid = CV.conv2d_float(d["x"], d["w1"]) ** 2
    worst = 0.0
    for l, out in enumerate(outs):
        z = d["cl"].decrypt_crt(out, level - 3, d["s_out"], limbs=2).real.reshape(g.C_a, g.H, g.W, g.R)
        w2l = d["w2"][l * g.C_a:(l + 1) * g.C_a]
        for r in range(g.R):
            chans = [c for c in range(mid.shape[0]) if c % g.R == r]
            worst = max(worst, float(np.max(np.abs(z[..., r] - CV.conv2d_float(mid[chans], w2l[:, chans])))))
    assert worst < tol, worst
    return worst


@pytest.mark.parametrize("c_in,deferred", [(4, False), (8, False), (8, True)])
def test_fused_block_matches_float(c_in, deferred):
    prm = toy_params(logN=9, q_bits=40, nq=5, p_bits=41, np_=2, dnum=3, scale=2.0 ** 30, hamming=32, seed=97)
    level = 4
    d = fused_inputs(prm, C_a=4, H=4, W=4, c_in=c_in, c_mid=8, level=level, std=0.2, seed=97)
    assert d["n_ca"] == c_in // 4 and d["g_ca"].R == 4 and d["g_ca"].n_out == 2
    outs = OB.ca_ra_block(d["orc"], d["g_ca"], d["g_ra"], d["cts"], level, d["p_ca"], d["p_ra"], d["evks"], d["rlk"], d["k_in"],
                          deferred=deferred)
    assert len(outs) == d["n_ca"] and outs[0].shape == (2, level - 2, prm.N)
    check_fused_output(d, outs, level)
    if c_in == 4 and not deferred:
        # one input ciphertext: identical to the plain sequence CAConv, Square, RAConv
        flat_ca = np.stack([d["p_ca"][j][0] for j in range(2)])
        flat_ra = np.stack([d["p_ra"][0][j] for j in range(2)])
        want, _ = OB.ca_square_ra(d["orc"], d["g_ca"], d["g_ra"], d["cts"][0], level, flat_ca, flat_ra, d["evks"], d["rlk"], d["k_in"])
        assert (outs[0] == want).all()


def test_block_with_hoisted_rotate_and_sum_matches_float():
    """The block with RaS over C_a as one hoisted sum of rotations per intermediate: same values as the stepwise
    form (conv(conv(x)^2) within the tolerance), other bits."""
    prm = toy_params(logN=9, q_bits=40, nq=5, p_bits=41, np_=2, dnum=3, scale=2.0 ** 30, hamming=32, seed=97)
    level = 4
    d = fused_inputs(prm, 4, 4, 4, 4, 8, level, 0.2, 97, all_ras_multiples=True)
    a = OB.ca_ra_block(d["orc"], d["g_ca"], d["g_ra"], d["cts"], level, d["p_ca"], d["p_ra"], d["evks"], d["rlk"], d["k_in"],
                       deferred=True, hoisted_ras=True)
    b = OB.ca_ra_block(d["orc"], d["g_ca"], d["g_ra"], d["cts"], level, d["p_ca"], d["p_ra"], d["evks"], d["rlk"], d["k_in"],
                       deferred=True)
    check_fused_output(d, a, level)
    assert any((u != v).any() for u, v in zip(a, b))

