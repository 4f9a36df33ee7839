"""Pin of the oracle's downsampling block (MulCt + relinearisation, affine constants, strided and 1x1 CAConv,
one-hot merge, level drops, scale plan) against float64: conv, p(p(u)), shortcut, add computed directly."""
from block_util import block_inputs, check_block_output
from he_inputs.params import toy_params
from oracle import block as OB


def test_block_small_ring_matches_float():
    prm = toy_params(logN=10, q_bits=40, nq=8, p_bits=41, np_=3, dnum=3, scale=2.0 ** 30, hamming=32, seed=93)
    level = 7
    d = block_inputs(prm, C_a=4, H=4, W=4, c_out=16, level=level, std3=0.1, std1=0.3)
    st = OB.downsampling_block(d["orc"], d["g3"], d["g1"], d["ct"], level, d["p3"], d["p1"], d["m_main"], d["m_short"],
                               d["evks"], d["rlk"], d["k_in"], d["k3"], d["k_short"])
    assert st["out"].shape == (2, level - 5, prm.N)
    check_block_output(d, st["out"], level)
