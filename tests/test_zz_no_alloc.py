"""he_rescale_noalloc (static device scratch, no allocation) against he_rescale, through the C ABI:
two calls in a row, the second on a smaller input, bit for bit; plus the size limit."""
import numpy as np
import pytest

from he_inputs import sampling as S
from he_inputs.params import config_params, toy_params

pytestmark = pytest.mark.gpu


def _rand_ct(prm, rng, level):
    return np.stack([S.uniform_limbs(rng, prm.q[:level + 1], prm.N)[0] for _ in range(2)])


@pytest.mark.parametrize("cfg", ["n65536", "toy"])
def test_rescale_noalloc_matches_rescale_twice(cfg):
    import torch
    from gpu_util import dev, host, zeros
    from paper_2302_02407_amd.binding import HEContext, HEError
    prm = config_params(2) if cfg == "n65536" else toy_params(logN=10, q_bits=30, nq=6, p_bits=32, np_=2, dnum=3, hamming=16, seed=90)
    rng = S.make_rng(90)
    ctx = HEContext.from_params(prm)
    N = prm.N
    levels = (15, 6) if cfg == "n65536" else (5, 2)          # second call on a smaller input
    ws_before = ctx.he_ws_bytes()
    for level in levels:
        ct = dev(_rand_ct(prm, rng, level))
        want = zeros(2, level, N)
        ctx.he_rescale(ct, level, want)
        got = zeros(2, level, N)
        ctx.he_rescale_noalloc(ct, level, got)
        assert (host(got) == host(want)).all(), level
    assert ctx.he_ws_bytes() == ws_before                    # the context's workspace was not touched
    if cfg == "n65536":
        # the oracle agrees with both on the last (smaller) input
        from oracle.he_oracle import Oracle
        orc = Oracle.from_params(prm)
        assert (host(got) == orc.rescale(host(ct), levels[-1])).all()
        # beyond the static array: refused with a clear error, nothing enqueued
        big = dev(_rand_ct(prm, rng, 16))
        with pytest.raises(HEError) as e:
            ctx.he_rescale_noalloc(big, 16, zeros(2, 16, N))
        assert e.value.code == -1 and "scratch" in str(e.value)
    with pytest.raises(HEError):
        ctx.he_rescale_noalloc(ct, levels[-1], ct)            # output overlaps the input
    torch.cuda.synchronize()
