"""GPU parity for the pieces of the downsampling block (workload 4): ct x ct multiply with relinearisation,
affine constants, strided and 1x1 channel-aligned convolutions, and the polynomial activation
p(p(u)), p(u) = 1.5u - 0.5u^3 composed from them.  Bit-exact vs the oracle; decrypted vs float64."""
import sys

import numpy as np
import pytest

from he_inputs import sampling as S
from he_inputs.params import config_params, toy_params

pytestmark = pytest.mark.gpu


def _say(msg):
    print(msg, file=sys.__stdout__, flush=True)


def _setup(prm, seed):
    from oracle import ckks_client as K
    from oracle.he_oracle import Oracle
    from paper_2302_02407_amd.binding import HEContext
    rng = S.make_rng(seed)
    orc, ctx = Oracle.from_params(prm), HEContext.from_params(prm)
    cl = K.Client(orc, S.ternary_secret(rng, prm.N, prm.hamming))
    return rng, orc, ctx, cl


def _enc(prm, rng, cl, z, scale, level):
    return cl.encrypt(np.asarray(z, dtype=np.complex128), scale, level, S.uniform_limbs(rng, prm.q[:level + 1], prm.N)[0],
                      S.gaussian_error(rng, prm.N, prm.sigma)[0])


@pytest.mark.parametrize("cfg,level", [("toy", 5), ("toy", 1), (4, 23), (4, 3)])
def test_mulct_and_affine(cfg, level):
    from gpu_util import dev, host, zeros
    prm = toy_params(logN=8, q_bits=30, nq=6, p_bits=32, np_=2, dnum=3, scale=2.0 ** 25, hamming=16, seed=90) if cfg == "toy" else config_params(cfg)
    rng, orc, ctx, cl = _setup(prm, 90)
    N = prm.N
    rlk = cl.relin_key(S.uniform_limbs(rng, prm.moduli, N, prm.dnum), S.gaussian_error(rng, N, prm.sigma, prm.dnum))
    ctx.he_evk_register(0, dev(rlk))
    za, zb = rng.uniform(-1, 1, N // 2), rng.uniform(-1, 1, N // 2)
    ca, cb = _enc(prm, rng, cl, za, prm.scale, level), _enc(prm, rng, cl, zb, prm.scale, level)
    out = zeros(2, level + 1, N)
    ctx.he_mulct(dev(ca), dev(cb), level, out)
    want = orc.mulct(ca, cb, level, rlk)
    assert (host(out) == want).all()
    if level >= 1:
        res = zeros(2, level, N)
        ctx.he_rescale(out, level, res)
        got = host(res)
        assert (got == orc.rescale(want, level)).all()
        scale = prm.scale * prm.scale / prm.q[level]
        assert np.max(np.abs(cl.decrypt(got, level - 1, scale) - za * zb)) < 1e-3
    # squaring in place (output aliases both inputs)
    sq = dev(ca)
    ctx.he_mulct(sq, sq, level, sq)
    assert (host(sq) == orc.mulct(ca, ca, level, rlk)).all()
    # affine: -x + 1.5, and 8*x
    k = int(round(1.5 * prm.scale))
    mul, add = [-1] * (level + 1), [k] * (level + 1)
    aff = zeros(2, level + 1, N)
    ctx.he_affine(dev(ca), level, mul, add, aff)
    assert (host(aff) == orc.affine(ca, level, mul, add)).all()
    assert np.max(np.abs(cl.decrypt(host(aff), level, prm.scale) - (1.5 - za))) < 1e-4
    ctx.he_affine(dev(ca), level, [8] * (level + 1), [0] * (level + 1), aff)
    assert (host(aff) == orc.affine(ca, level, [8] * (level + 1), [0] * (level + 1))).all()


def _conv_case(prm, C_a, H, W, c_out, f, stride, level, w_std, tol):
    from gpu_util import dev, host, zeros
    from oracle import conv2d as CV
    rng, orc, ctx, cl = _setup(prm, prm.seed)
    geo = CV.ConvGeometry(prm.N, C_a, H, W, c_out, f=f, stride=stride)
    x, wt = S.conv_tensors(rng, C_a, c_out, H, W, f, w_std)
    steps = sorted(set(s for s in geo.tap_steps if s) | set(geo.ras_steps))
    evks = {st: cl.rotation_key(orc.galois_elt(st), S.uniform_limbs(rng, prm.moduli, prm.N, prm.dnum),
                                S.gaussian_error(rng, prm.N, prm.sigma, prm.dnum)) for st in steps}
    ct = _enc(prm, rng, cl, geo.pack_input(x), prm.scale, level)
    pts = CV.encode_weights(orc, geo, wt, level, float(prm.q[level]))
    _say("conv f=%d stride=%d: running the oracle (%d outputs)" % (f, stride, geo.n_out))
    want = CV.caconv(orc, geo, ct, level, pts, evks, progress=_say)
    for st, k in evks.items():
        ctx.he_evk_register(ctx.galois_elt(st), dev(k))
    weights = [dev(pts[o, t]) for o in range(geo.n_out) for t in range(len(geo.taps))]
    outs = [zeros(2, level, prm.N) for _ in range(geo.n_out)]
    ctx.he_counters_reset()
    ctx.he_conv2d(geo.C_a, geo.H, geo.W, geo.R, f, level, weights, dev(ct), outs)
    cnt = ctx.he_counters()
    got = [host(o) for o in outs]
    for o in range(geo.n_out):
        assert (got[o] == want[o]).all(), o
    assert cnt["keyswitch"] == (f * f - 1) + geo.n_out * len(geo.ras_steps)
    dec, spread = geo.unpack_output([cl.decrypt(g, level - 1, prm.scale) for g in got])
    ref = CV.conv2d_float(x, wt)                   # stride-1 result; the strided layer keeps every s-th pixel in place
    mask = np.zeros_like(ref)
    mask[:, ::stride, ::stride] = 1.0              # void packing: skipped positions hold zero
    assert np.max(np.abs(dec - ref * mask)) < tol
    assert spread < tol


def test_strided_and_pointwise_conv_small_ring():
    prm = toy_params(logN=10, q_bits=40, nq=3, p_bits=41, np_=1, dnum=3, scale=2.0 ** 30, hamming=32, seed=91)
    _conv_case(prm, C_a=4, H=4, W=4, c_out=16, f=3, stride=2, level=2, w_std=0.1, tol=1e-3)
    _conv_case(prm, C_a=4, H=4, W=4, c_out=8, f=1, stride=2, level=2, w_std=0.1, tol=1e-3)
    _conv_case(prm, C_a=4, H=4, W=4, c_out=8, f=1, stride=1, level=1, w_std=0.1, tol=1e-3)


def _block_case(prm, C_a, H, W, c_out, level, std3, std1, hoisted_ras=False):
    """3x3 stride-2 CAConv -> merge -> p(p(u)), plus the 1x1 stride-2 shortcut -> merge, added: every stage
    bit-exact against the same sequence on the oracle, the decrypted result against float64."""
    from gpu_util import dev, host
    from oracle import block as OB
    from block_util import block_inputs, check_block_output
    from paper_2302_02407_amd import block as B
    from paper_2302_02407_amd.binding import HEContext
    d = block_inputs(prm, C_a, H, W, c_out, level, std3, std1, all_ras_multiples=hoisted_ras)
    ctx, g3, n_out = HEContext.from_params(prm), d["g3"], d["g3"].n_out
    _say("block: running the oracle (%d + %d output ciphertexts)" % (n_out, n_out))
    want = OB.downsampling_block(d["orc"], g3, d["g1"], d["ct"], level, d["p3"], d["p1"], d["m_main"], d["m_short"],
                                 d["evks"], d["rlk"], d["k_in"], d["k3"], d["k_short"], progress=_say, hoisted_ras=hoisted_ras)
    _say("block: oracle done, running the GPU path")
    for st, k in d["evks"].items():
        ctx.he_evk_register(ctx.galois_elt(st), dev(k))
    ctx.he_evk_register(0, dev(d["rlk"]))
    d3 = [dev(d["p3"][o, t]) for o in range(n_out) for t in range(9)]
    d1 = [dev(d["p1"][o, 0]) for o in range(n_out)]
    out, got = B.downsampling_block(ctx, C_a, H, W, g3.R, level, dev(d["ct"]), d3, d1, [dev(m) for m in d["m_main"]],
                                    [dev(m) for m in d["m_short"]], d["k_in"], d["k3"], d["k_short"], keep=True, hoisted_ras=hoisted_ras)
    got["out"] = out
    for name in ("conv3", "conv1"):
        for o in range(n_out):
            assert (host(got[name][o]) == want[name][o]).all(), (name, o)
    for name in ("merged", "u", "a1", "a2", "short", "out"):
        assert (host(got[name]) == want[name]).all(), name
    check_block_output(d, host(out), level, _say)


def test_downsampling_block_small_ring():
    prm = toy_params(logN=10, q_bits=40, nq=8, p_bits=41, np_=3, dnum=3, scale=2.0 ** 30, hamming=32, seed=93)
    _block_case(prm, C_a=4, H=4, W=4, c_out=16, level=7, std3=0.1, std1=0.3)


def test_downsampling_block_hoisted_rotate_and_sum_small_ring():
    prm = toy_params(logN=10, q_bits=40, nq=8, p_bits=41, np_=3, dnum=3, scale=2.0 ** 30, hamming=32, seed=93)
    _block_case(prm, C_a=4, H=4, W=4, c_out=16, level=7, std3=0.1, std1=0.3, hoisted_ras=True)


@pytest.mark.timeout(1100)
def test_downsampling_block_config4():
    """Workload 4 at full size: N = 2^16, 16 -> 32 channels on 32x32, stride 2, level 23, He-normal weights;
    16 output ciphertexts per convolution, block output at level 17."""
    prm = config_params(4)
    _block_case(prm, C_a=16, H=32, W=32, c_out=32, level=23, std3=(2.0 / (9 * 16)) ** 0.5, std1=(2.0 / 16) ** 0.5)


@pytest.mark.parametrize("cfg,level", [("toy", 5), (4, 23)])
def test_polynomial_activation_twice(cfg, level):
    """y = p(p(u)), p(u) = 1.5u - 0.5u^3 = 0.5*u*(3 - u^2), two levels per application: u2 = Rescale(MulCt(u,u)),
    w = 3 - u2 (affine), t = Rescale(MulCt(drop(u), w)); the factor 0.5 is carried in the scale.  The working
    scale is the prime size itself so that it survives the four multiplications."""
    import torch
    from gpu_util import dev, host, zeros
    prm = toy_params(logN=8, q_bits=30, nq=6, p_bits=32, np_=2, dnum=3, hamming=16, seed=92) if cfg == "toy" else config_params(cfg)
    rng, orc, ctx, cl = _setup(prm, 92)
    N = prm.N
    rlk = cl.relin_key(S.uniform_limbs(rng, prm.moduli, N, prm.dnum), S.gaussian_error(rng, N, prm.sigma, prm.dnum))
    ctx.he_evk_register(0, dev(rlk))
    u = rng.uniform(-1, 1, N // 2)
    scale = float(prm.q[level])                    # scale ~ q: Delta^2/q stays ~ q
    ct = _enc(prm, rng, cl, u, scale, level)
    d_ct = dev(ct)
    ref = u.copy()
    lv = level
    for rep in range(2):
        # ---- oracle
        u2 = orc.rescale(orc.mulct(ct, ct, lv, rlk), lv)
        s2 = scale * scale / prm.q[lv]
        k3 = int(round(3.0 * s2))
        w = orc.affine(u2, lv - 1, [-1] * lv, [k3] * lv)
        t = orc.rescale(orc.mulct(orc.drop_level(ct, lv), w, lv - 1, rlk), lv - 1)
        # ---- GPU, same sequence through the C ABI
        g_sq = zeros(2, lv + 1, N)
        ctx.he_mulct(d_ct, d_ct, lv, g_sq)
        g_u2 = zeros(2, lv, N)
        ctx.he_rescale(g_sq, lv, g_u2)
        assert (host(g_u2) == u2).all()
        ctx.he_affine(g_u2, lv - 1, [-1] * lv, [k3] * lv, g_u2)
        g_drop = d_ct[:, :lv, :].contiguous()      # forget limb q_lv (device-side slice, no arithmetic)
        g_prod = zeros(2, lv, N)
        ctx.he_mulct(g_drop, g_u2, lv - 1, g_prod)
        g_t = zeros(2, lv - 1, N)
        ctx.he_rescale(g_prod, lv - 1, g_t)
        assert (host(g_t) == t).all(), rep
        # ---- bookkeeping: t encodes u*(3-u^2) = 2 p(u) at scale scale*s2/q; halve by doubling the scale
        scale = 2.0 * scale * s2 / prm.q[lv - 1]
        ct, d_ct, lv = t, g_t, lv - 2
        ref = 1.5 * ref - 0.5 * ref ** 3
    got = cl.decrypt_crt(host(d_ct), lv, scale, limbs=2)
    tol = 1e-3
    assert np.max(np.abs(got.real - ref)) < tol
