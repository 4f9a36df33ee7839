"""Inputs and the float64 check (maximum absolute error) of the downsampling-block tests (shared by the CPU pin of the oracle's
block and the GPU parity test)."""
import numpy as np

from he_inputs import sampling as S
from oracle import ckks_client as K
from oracle.he_oracle import Oracle


def block_inputs(prm, C_a, H, W, c_out, level, std3, std1, all_ras_multiples=False):
    """Everything both sides consume: keys, the encrypted image, weight and merge plaintexts, constants.
    all_ras_multiples: also the keys of every multiple of H*W*R below C_a (hoisted rotate-and-sum), drawn last."""
    from oracle import block as OB
    from oracle import conv2d as CV
    rng = S.make_rng(prm.seed)
    orc = Oracle.from_params(prm)
    cl = K.Client(orc, S.ternary_secret(rng, prm.N, prm.hamming))
    N, q = prm.N, prm.q
    g3 = CV.ConvGeometry(N, C_a, H, W, c_out, f=3, stride=2)
    g1 = CV.ConvGeometry(N, C_a, H, W, c_out, f=1, stride=2)
    assert g3.n_out == g1.n_out <= C_a
    x, w3 = S.conv_tensors(rng, C_a, c_out, H, W, 3, std3)
    w1 = rng.normal(0.0, std1, size=(c_out, C_a, 1, 1))
    steps = sorted(set(s for s in g3.tap_steps if s) | set(g3.ras_steps))
    evks = {st: cl.rotation_key(orc.galois_elt(st), S.uniform_limbs(rng, prm.moduli, N, prm.dnum),
                                S.gaussian_error(rng, N, prm.sigma, prm.dnum)) for st in steps}
    rlk = cl.relin_key(S.uniform_limbs(rng, prm.moduli, N, prm.dnum), S.gaussian_error(rng, N, prm.sigma, prm.dnum))
    ct = cl.encrypt(g3.pack_input(x).astype(np.complex128), prm.scale, level,
                    S.uniform_limbs(rng, prm.q[:level + 1], N)[0], S.gaussian_error(rng, N, prm.sigma)[0])
    k_in, k3, s_out, k_short, ms_short = OB.block_scales(q, level, prm.scale)
    d = dict(orc=orc, cl=cl, g3=g3, g1=g1, x=x, w3=w3, w1=w1, evks=evks, rlk=rlk, ct=ct, k_in=k_in, k3=k3,
             s_out=s_out, k_short=k_short,
             p3=CV.encode_weights(orc, g3, w3, level, float(q[level])),
             p1=CV.encode_weights(orc, g1, w1, level, float(q[level])),
             m_main=OB.one_hot_masks(orc, g3, g3.n_out, level - 1, float(q[level - 1])),
             m_short=OB.one_hot_masks(orc, g3, g3.n_out, level - 1, ms_short))
    if all_ras_multiples:
        base = g3.H * g3.W * g3.R
        for i in range(1, C_a):
            if base * i not in evks:
                evks[base * i] = cl.rotation_key(orc.galois_elt(base * i), S.uniform_limbs(rng, prm.moduli, N, prm.dnum),
                                                 S.gaussian_error(rng, N, prm.sigma, prm.dnum))
    return d


def check_block_output(d, out, level, say=print):
    """Decrypted block output against float64: maximum absolute error below 1e-3 (the activation reaches
    |y| ~ 10^3, so the error relative to max(1, |y|) is reported beside it)."""
    from oracle import block as OB
    g3 = d["g3"]
    ref = OB.block_float(d["x"], d["w3"], d["w1"])
    z = d["cl"].decrypt_crt(out, level - 6, d["s_out"], limbs=2).real.reshape(g3.C_a, g3.H, g3.W, g3.R)
    worst_abs = worst_rel = 0.0
    for o in range(g3.n_out):
        for r in range(g3.R):
            y = ref[g3.out_channel(o, r)]
            err = np.abs(z[o, :, :, r] - y)
            worst_abs = max(worst_abs, float(err.max()))
            worst_rel = max(worst_rel, float((err / np.maximum(1.0, np.abs(y))).max()))
    if g3.n_out < g3.C_a:
        assert np.max(np.abs(z[g3.n_out:])) < 1e-3            # blocks nothing was merged into stay empty
    say("block: max |y| %.4g, max absolute error %.3g, max error relative to max(1,|y|) %.3g" % (np.abs(ref).max(), worst_abs, worst_rel))
    assert worst_abs < 1e-3
    return worst_abs, worst_rel
