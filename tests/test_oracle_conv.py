"""End-to-end pin of CAConv on the oracle: the decrypted output equals a direct float64
convolution (own loop and torch's conv2d), every C_a block holds the same result, and the
operation counts match the paper's cost table for CAConv."""
import numpy as np
import pytest
import torch

from he_inputs import sampling as S
from he_inputs.params import config_params, toy_params
from oracle import ckks_client as K
from oracle import conv2d as CV
from oracle.he_oracle import Oracle


def _keys(o, cl, prm, rng, steps):
    return {st: cl.rotation_key(o.galois_elt(st), S.uniform_limbs(rng, prm.moduli, prm.N, prm.dnum),
                                S.gaussian_error(rng, prm.N, prm.sigma, prm.dnum)) for st in steps}


def _run(prm, C_a, H, W, c_out, level, w_std, tol):
    rng = S.make_rng(prm.seed)
    o = Oracle.from_params(prm)
    cl = K.Client(o, S.ternary_secret(rng, prm.N, prm.hamming))
    geo = CV.ConvGeometry(prm.N, C_a, H, W, c_out)
    x, wt = S.conv_tensors(rng, C_a, c_out, H, W, 3, w_std)
    steps = sorted(set(s for s in geo.tap_steps if s) | set(geo.ras_steps))
    evks = _keys(o, cl, prm, rng, steps)
    ct = cl.encrypt(geo.pack_input(x).astype(np.complex128), prm.scale, level,
                    S.uniform_limbs(rng, prm.q[:level + 1], prm.N)[0], S.gaussian_error(rng, prm.N, prm.sigma)[0])
    pts = CV.encode_weights(o, geo, wt, level, float(prm.q[level]))   # plaintext scale q_level: output scale stays Delta
    outs = CV.caconv(o, geo, ct, level, pts, evks)
    assert len(outs) == geo.n_out
    dec = [cl.decrypt(c, level - 1, prm.scale) for c in outs]
    got, spread = geo.unpack_output(dec)
    ref = CV.conv2d_float(x, wt)
    tref = torch.nn.functional.conv2d(torch.from_numpy(x)[None], torch.from_numpy(wt), padding=1)[0].numpy()
    assert np.max(np.abs(ref - tref)) < 1e-12
    err = np.max(np.abs(got - ref))
    assert err < tol, err
    assert spread < tol          # rotate-and-sum leaves the sum replicated in every C_a block
    assert max(np.max(np.abs(np.asarray(d).imag)) for d in dec) < tol
    return geo


def test_caconv_tiny_ring():
    prm = toy_params(logN=6, q_bits=30, nq=3, p_bits=31, np_=1, dnum=3, scale=2.0 ** 24, hamming=8, seed=41)
    geo = _run(prm, C_a=2, H=2, W=2, c_out=2, level=2, w_std=0.3, tol=2e-3)
    assert geo.R == 4 and geo.n_out == 1


def test_caconv_config0():
    prm = config_params(0)
    geo = _run(prm, C_a=4, H=8, W=8, c_out=4, level=2, w_std=0.1, tol=1e-3)
    # CAConv cost (paper, cost table): f^2-1 Slide rotations + n_o*log2(C_a) RaS rotations, no IR
    assert geo.R == 8 and geo.n_out == 1
    assert sorted(s for s in geo.tap_steps if s) == sorted([8, 56, 64, 72, 2048 - 8, 2048 - 56, 2048 - 64, 2048 - 72])
    assert geo.ras_steps == [512, 1024]
    assert len([s for s in geo.tap_steps if s]) + geo.n_out * len(geo.ras_steps) == 10


def test_geometry_config3():
    geo = CV.ConvGeometry(1 << 16, 16, 32, 32, 16)
    assert geo.R == 2 and geo.n_out == 8
    assert sorted(min(s, 32768 - s) for s in geo.tap_steps if s) == [2, 2, 62, 62, 64, 64, 66, 66]
    assert geo.ras_steps == [2048, 4096, 8192, 16384]
    assert [geo.out_channel(3, r) for r in range(2)] == [6, 7]
    assert len([s for s in geo.tap_steps if s]) + geo.n_out * len(geo.ras_steps) == 40
