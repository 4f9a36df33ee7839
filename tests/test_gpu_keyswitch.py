"""GPU parity: key switching, rotations (single and hoisted), conjugation, MulPt-accumulate,
add and rescale vs the CPU oracle, bit-exact; plus Dec(Rot(Enc z)) = roll(z) on the GPU result."""
import sys

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


def _key(prm, rng, cl, g):
    return cl.rotation_key(g, S.uniform_limbs(rng, prm.moduli, prm.N, prm.dnum),
                           S.gaussian_error(rng, prm.N, prm.sigma, prm.dnum))


def _rand_ct(prm, rng, level):
    return np.stack([S.uniform_limbs(rng, prm.q[:level + 1], prm.N)[0] for _ in range(2)])


@pytest.mark.parametrize("level", [5, 4, 3, 2, 0])
def test_keyswitch_and_rotations_partial_digits(level):
    """6 primes, dnum 3 (alpha 2): levels with a partial last digit and fewer digits than dnum."""
    from gpu_util import dev, host, zeros
    prm = toy_params(logN=8, q_bits=30, nq=6, p_bits=32, np_=2, dnum=3, hamming=16, seed=60)
    rng, orc, ctx, cl = _setup(prm, 60 + level)
    N = prm.N
    steps = [1, 5, N // 2 - 3]
    keys = {s: _key(prm, rng, cl, orc.galois_elt(s)) for s in steps}
    for s, k in keys.items():
        ctx.he_evk_register(ctx.galois_elt(s), dev(k))
    ct = _rand_ct(prm, rng, level)
    # plain key switch of c1 with the key of step 1
    o0, o1 = zeros(level + 1, N), zeros(level + 1, N)
    ctx.he_keyswitch(dev(ct[1]), level, ctx.galois_elt(1), o0, o1)
    w0, w1 = orc.keyswitch(ct[1], level, keys[1])
    assert (host(o0) == w0).all() and (host(o1) == w1).all()
    # hoisted rotations (with a zero step and a negative step) == oracle == single rotations
    hs = [1, 0, 5, -3]
    outs = [zeros(2, level + 1, N) for _ in hs]
    ctx.he_rotate_hoisted(dev(ct), level, hs, outs)
    for s, o in zip(hs, outs):
        want = ct if s == 0 else orc.rotate(ct, level, orc.galois_elt(s), keys[s % (N // 2)])
        assert (host(o) == want).all(), s
        single = zeros(2, level + 1, N)
        ctx.he_rotate(dev(ct), level, s, single)
        assert (host(single) == want).all(), s


@pytest.mark.parametrize("cfg,level,n_ct,steps", [
    ("toy", 5, 5, [1, 5, 0, -3, 1]),
    ("toy", 2, 11, [5, 1]),
    (2, 23, 3, [1 << i for i in range(0, 15, 2)]),      # 24 jobs: several ModDown launch sets, shared keys
    (2, 4, 9, [1, 1 << 14]),                             # more sources than one ModUp wave
])
def test_rotate_batch_matches_single_calls_and_oracle(cfg, level, n_ct, steps):
    """he_rotate_batch, hoisted and not, equals he_rotate call by call (bit for bit) and the oracle on a sample."""
    from gpu_util import dev, host, zeros
    prm = (toy_params(logN=8, q_bits=30, nq=6, p_bits=32, np_=2, dnum=3, hamming=16, seed=63) if cfg == "toy"
           else config_params(cfg))
    rng, orc, ctx, cl = _setup(prm, 63)
    N = prm.N
    keys = {}
    for s in steps:
        g = orc.galois_elt(s)
        if g != 1 and g not in keys:
            keys[g] = _key(prm, rng, cl, g)
            ctx.he_evk_register(g, dev(keys[g]))
    cts = [_rand_ct(prm, rng, level) for _ in range(n_ct)]
    d_cts = [dev(c) for c in cts]
    ref = {}
    for c in range(n_ct):
        for i, s in enumerate(steps):
            o = zeros(2, level + 1, N)
            ctx.he_rotate(d_cts[c], level, s, o)
            ref[(c, i)] = host(o)
    for hoisted in (True, False):
        outs = [zeros(2, level + 1, N) for _ in range(n_ct * len(steps))]
        ctx.he_counters_reset()
        ctx.he_rotate_batch(d_cts, level, steps, outs, hoisted=hoisted)
        cnt = ctx.he_counters()
        nz = sum(1 for s in steps if orc.galois_elt(s) != 1)
        assert cnt["keyswitch"] == n_ct * nz
        assert cnt["modup"] == (n_ct if hoisted else n_ct * nz)
        for c in range(n_ct):
            for i, s in enumerate(steps):
                assert (host(outs[c * len(steps) + i]) == ref[(c, i)]).all(), (hoisted, c, s)
    for c, i in ((0, 0), (n_ct - 1, len(steps) - 1)):
        g = orc.galois_elt(steps[i])
        want = cts[c] if g == 1 else orc.rotate(cts[c], level, g, keys[g])
        assert (ref[(c, i)] == want).all()


@pytest.mark.timeout(900)
def test_config2_full_batch_as_benchmarked():
    """Workload 2 at the size and launch configuration bench.py times: 64 uniform ciphertexts at level 23,
    all 15 power-of-two steps through he_rotate_batch, singly and hoisted.  Every output of the two
    modes agrees bit for bit, two runs agree (determinism), and 4 ciphertexts x (15 steps + conjugation)
    equal the oracle."""
    import torch
    from gpu_util import dev, host, zeros
    prm = config_params(2)
    rng, orc, ctx, cl = _setup(prm, prm.seed)
    N, level, B = prm.N, 23, 64
    steps = [1 << i for i in range(15)]
    gen = torch.Generator(device="cuda")
    gen.manual_seed(2)

    def uniform(lead, moduli):
        cols = [torch.randint(0, int(m), tuple(lead) + (1, N), dtype=torch.int64, device="cuda", generator=gen) for m in moduli]
        return torch.cat(cols, dim=len(lead)).contiguous().view(torch.uint64)

    keys = {s: uniform((prm.dnum, 2), prm.moduli) for s in steps}     # uniform keys: parity does not need real ones
    for s in steps:
        ctx.he_evk_register(ctx.galois_elt(s), keys[s])
    cts = [uniform((2,), prm.q) for _ in range(B)]
    out_h = [zeros(2, level + 1, N) for _ in range(B * 15)]
    out_s = [zeros(2, level + 1, N) for _ in range(B * 15)]
    ctx.he_rotate_batch(cts, level, steps, out_h, hoisted=True)
    ctx.he_rotate_batch(cts, level, steps, out_s, hoisted=False)
    torch.cuda.synchronize()
    for a, b in zip(out_h, out_s):
        assert torch.equal(a, b)
    sums = [int(o.view(torch.int64).sum().item()) for o in out_h[::37]]
    ctx.he_rotate_batch(cts, level, steps, out_h, hoisted=True)
    torch.cuda.synchronize()
    assert sums == [int(o.view(torch.int64).sum().item()) for o in out_h[::37]]
    # the stated oracle subset: four seeded ciphertexts x all 15 steps + conjugation, bit for bit (the oracle
    # raises each ciphertext once and rotates from the raised digits, which its own pins show equals rotating singly)
    keys_h = {s: host(keys[s]) for s in steps}
    kc = uniform((prm.dnum, 2), prm.moduli)
    ctx.he_evk_register(2 * N - 1, kc)
    kc_h = host(kc)
    for c in (0, 17, 40, 63):
        ct_h = host(cts[c])
        raised = orc.modup(ct_h[1], level)
        for i, s in enumerate(steps):
            want = orc.rotate_from_raised(ct_h, raised, level, orc.galois_elt(s), keys_h[s])
            assert (host(out_h[c * 15 + i]) == want).all(), (c, s)
        oc = zeros(2, level + 1, N)
        ctx.he_conjugate(cts[c], level, oc)
        assert (host(oc) == orc.rotate_from_raised(ct_h, raised, level, orc.galois_conj, kc_h)).all(), (c, "conj")
        print("config 2: ciphertext %d, 15 steps + conjugation equal the oracle" % c, file=sys.__stdout__, flush=True)


def test_wide_digits_generic_conversion_path():
    """alpha = 10 > 8 source limbs per digit: the conversion kernel's chunked path (and a 60-limb raised basis)."""
    from gpu_util import dev, host, zeros
    prm = toy_params(logN=8, q_bits=30, nq=20, p_bits=32, np_=10, dnum=2, hamming=16, seed=62)
    rng, orc, ctx, cl = _setup(prm, 62)
    N = prm.N
    key = _key(prm, rng, cl, orc.galois_elt(3))
    ctx.he_evk_register(ctx.galois_elt(3), dev(key))
    for level in (19, 14, 9, 4):
        ct = _rand_ct(prm, rng, level)
        out = zeros(2, level + 1, N)
        ctx.he_rotate(dev(ct), level, 3, out)
        assert (host(out) == orc.rotate(ct, level, orc.galois_elt(3), key)).all(), level


def test_counters_and_errors():
    from gpu_util import dev, zeros
    from paper_2302_02407_amd.binding import HEError
    prm = toy_params(logN=8, q_bits=30, nq=6, p_bits=32, np_=2, dnum=3, hamming=16, seed=61)
    rng, orc, ctx, cl = _setup(prm, 61)
    N, level = prm.N, 5
    ct = dev(_rand_ct(prm, rng, level))
    out = zeros(2, level + 1, N)
    with pytest.raises(HEError) as e:
        ctx.he_rotate(ct, level, 1, out)                    # no key registered
    assert e.value.code == -3
    with pytest.raises(HEError) as e:
        ctx.he_rotate(zeros(2, 7, N), 6, 1, zeros(2, 7, N))  # level above L
    assert e.value.code == -2
    ctx.he_evk_register(ctx.galois_elt(1), dev(_key(prm, rng, cl, orc.galois_elt(1))))
    with pytest.raises(HEError):
        ctx.he_rotate(ct, level, 1, ct)                     # output overlaps input
    with pytest.raises(HEError):
        ctx.he_rescale(ct, 0, out)                          # cannot rescale at level 0
    with pytest.raises(HEError):
        ctx.he_keyswitch(ct[1], level, ctx.galois_elt(1), ct[1], out[1])   # output 0 is the input
    with pytest.raises(HEError):
        ctx.he_keyswitch(ct[1], level, ctx.galois_elt(1), out[0], out[0])  # the two outputs coincide
    # empty batches are no-ops
    ctx.he_counters_reset()
    ctx.he_rotate_hoisted(ct, level, [], [])
    ctx.he_rotate_batch([], level, [1], [])
    ctx.he_rotate_batch([ct], level, [], [], hoisted=False)
    assert ctx.he_counters()["keyswitch"] == 0 and ctx.he_counters()["modup"] == 0
    # only the zero step: plain copies, no key switch
    cp = zeros(2, level + 1, N)
    ctx.he_rotate_hoisted(ct, level, [0], [cp])
    assert (cp == ct).all() and ctx.he_counters()["keyswitch"] == 0
    ctx.he_counters_reset()
    ctx.he_rotate_hoisted(ct, level, [1, 0, 1], [zeros(2, level + 1, N) for _ in range(3)])
    c = ctx.he_counters()
    assert c["modup"] == 1 and c["keyswitch"] == 2
    # per key switch at level 5 (beta=3, R=8): iNTT 6 + 2*2, NTT 3*6 + 2*6
    assert c["intt_limbs"] == 6 + 2 * 4 and c["ntt_limbs"] == 18 + 2 * 12


@pytest.mark.parametrize("cfg,level", [(0, 2), (0, 1), (2, 23), (2, 9)])
def test_rotation_real_encryption(cfg, level):
    """Real keys and a real encryption at the workload's parameters: GPU == oracle bit for bit, and
    the GPU result decrypts to the rotated message."""
    from gpu_util import dev, host, zeros
    prm = config_params(cfg)
    rng, orc, ctx, cl = _setup(prm, prm.seed)
    N = prm.N
    z = rng.uniform(-1, 1, N // 2) + 1j * rng.uniform(-1, 1, N // 2)
    ct = cl.encrypt(z, prm.scale, level, S.uniform_limbs(rng, prm.q[:level + 1], N)[0], S.gaussian_error(rng, N, prm.sigma)[0])
    steps = [1, 1 << (prm.logN - 2)]
    # key-switch noise ~ beta*alpha*(q_max/P)*sqrt(N)*sigma/Delta: large at the tiny workload (one 41-bit
    # special prime against 40-bit digits, Delta = 2^30), small at N = 2^16 (P = 2^472, Delta = 2^40)
    tol = 1e-3 if cfg == 0 else 2e-5
    keys = {s: _key(prm, rng, cl, orc.galois_elt(s)) for s in steps}
    kc = _key(prm, rng, cl, orc.galois_conj)
    for s, k in keys.items():
        ctx.he_evk_register(ctx.galois_elt(s), dev(k))
    ctx.he_evk_register(2 * N - 1, dev(kc))
    outs = [zeros(2, level + 1, N) for _ in steps]
    ctx.he_rotate_hoisted(dev(ct), level, steps, outs)
    for s, o in zip(steps, outs):
        got = host(o)
        assert (got == orc.rotate(ct, level, orc.galois_elt(s), keys[s])).all()
        assert np.max(np.abs(cl.decrypt(got, level, prm.scale) - np.roll(z, -s))) < tol
    oc = zeros(2, level + 1, N)
    ctx.he_conjugate(dev(ct), level, oc)
    got = host(oc)
    assert (got == orc.rotate(ct, level, orc.galois_conj, kc)).all()
    assert np.max(np.abs(cl.decrypt(got, level, prm.scale) - np.conj(z))) < tol


def test_config2_uniform_ciphertexts_subset():
    """Workload 2 shape: uniform-random ciphertexts at level 23, rotated by power-of-two steps, singly and
    hoisted; a seeded subset is compared with the oracle, hoisted == single on all of it."""
    from gpu_util import dev, host, zeros
    prm = config_params(2)
    rng, orc, ctx, cl = _setup(prm, prm.seed)
    N, level = prm.N, 23
    steps = [1 << 0, 1 << 7, 1 << 14]
    keys = {s: _key(prm, rng, cl, orc.galois_elt(s)) for s in steps}
    for s, k in keys.items():
        ctx.he_evk_register(ctx.galois_elt(s), dev(k))
    for c in range(2):
        ct = _rand_ct(prm, rng, level)
        d = dev(ct)
        outs = [zeros(2, level + 1, N) for _ in steps]
        ctx.he_rotate_hoisted(d, level, steps, outs)
        raised = orc.modup(ct[1], level)
        for s, o in zip(steps, outs):
            single = zeros(2, level + 1, N)
            ctx.he_rotate(d, level, s, single)
            got = host(o)
            assert (got == host(single)).all()
            assert (got == orc.rotate_from_raised(ct, raised, level, orc.galois_elt(s), keys[s])).all(), (c, s)


@pytest.mark.parametrize("cfg,level", [(0, 2), (2, 23), (2, 1)])
def test_mac_add_rescale(cfg, level):
    from gpu_util import dev, host, zeros
    prm = config_params(cfg)
    rng, orc, ctx, cl = _setup(prm, 70 + cfg)
    N = prm.N
    ct, ct2 = _rand_ct(prm, rng, level), _rand_ct(prm, rng, level)
    pt, pt2 = S.uniform_limbs(rng, prm.q[:level + 1], N)[0], S.uniform_limbs(rng, prm.q[:level + 1], N)[0]
    pt[0, :5] = 0
    ct[0, 0, :5] = np.uint64(prm.q[0] - 1)
    acc = dev(np.full((2, level + 1, N), 12345, dtype=np.uint64))     # init must overwrite garbage
    ctx.he_ptct_mac(acc, dev(ct), dev(pt), level, init=True)
    w = orc.ptct_mac(None, ct, pt, level, init=True)
    assert (host(acc) == w).all()
    ctx.he_ptct_mac(acc, dev(ct2), dev(pt2), level, init=False)
    w = orc.ptct_mac(w, ct2, pt2, level, init=False)
    assert (host(acc) == w).all()
    s = zeros(2, level + 1, N)
    ctx.he_add(dev(ct), dev(ct2), level, s)
    assert (host(s) == orc.add(ct, ct2, level)).all()
    ap = zeros(2, level + 1, N)
    ctx.he_addpt(dev(ct), dev(pt), level, ap)
    assert (host(ap) == orc.addpt(ct, pt, level)).all()
    inplace = dev(ct)
    ctx.he_addpt(inplace, dev(pt2), level, inplace)
    assert (host(inplace) == orc.addpt(ct, pt2, level)).all()
    out = zeros(2, level, N)
    ctx.he_rescale(acc, level, out)
    assert (host(out) == orc.rescale(w, level)).all()


@pytest.mark.parametrize("q_bits,nq,p_bits,np_,dnum,levels", [
    (40, 12, 41, 1, 12, (11, 8, 5, 0)),     # alpha 1, one special prime; 12 and 9 digits take the unfused inner product
    (50, 6, 60, 3, 2, (5, 3, 2)),           # alpha 3 with 60-bit special primes, partial and single digits
    (57, 4, 58, 2, 2, (3, 1)),              # widest narrow-path primes (57 bits) and wide-path special primes
    (54, 6, 60, 2, 3, (5, 4, 2, 0)),        # alpha 2, three digits: three target sets in one single-launch conversion
])
def test_n65536_other_decompositions(q_bits, nq, p_bits, np_, dnum, levels):
    """The N = 2^16 kernels away from the benchmark's parameter set: other digit widths and counts (fused and
    unfused inner product), other prime sizes (lazy-reduction bounds), rotations singly, hoisted and summed."""
    from gpu_util import dev, host, zeros
    prm = toy_params(logN=16, q_bits=q_bits, nq=nq, p_bits=p_bits, np_=np_, dnum=dnum, hamming=64, seed=63)
    rng, orc, ctx, cl = _setup(prm, 63)
    N = prm.N
    steps = [1, 300]
    keys = {s: _key(prm, rng, cl, orc.galois_elt(s)) for s in steps}
    for s, k in keys.items():
        ctx.he_evk_register(ctx.galois_elt(s), dev(k))
    for level in levels:
        ct = _rand_ct(prm, rng, level)
        outs = [zeros(2, level + 1, N) for _ in steps]
        ctx.he_rotate_hoisted(dev(ct), level, steps, outs)
        for s, o in zip(steps, outs):
            want = orc.rotate(ct, level, orc.galois_elt(s), keys[s])
            assert (host(o) == want).all(), (level, s)
        single = zeros(2, level + 1, N)
        ctx.he_rotate(dev(ct), level, 300, single)
        assert (host(single) == host(outs[1])).all(), level
        o0, o1 = zeros(level + 1, N), zeros(level + 1, N)
        ctx.he_keyswitch(dev(ct[1]), level, ctx.galois_elt(1), o0, o1)
        w0, w1 = orc.keyswitch(ct[1], level, keys[1])
        assert (host(o0) == w0).all() and (host(o1) == w1).all(), level


@pytest.mark.parametrize("cfg", ["toy", 2])
def test_extreme_residues(cfg):
    """Worst cases for the lazy-reduction and 128-bit accumulation bounds: every residue of the ciphertext and of
    the key at m-1, at 0/m-1 alternating, and a ciphertext that is zero except for one coefficient; transforms,
    a hoisted rotation and a rescale must still equal the oracle bit for bit."""
    from gpu_util import dev, host, zeros
    prm = toy_params(logN=9, q_bits=30, nq=6, p_bits=32, np_=2, dnum=3, hamming=16, seed=64) if cfg == "toy" else config_params(cfg)
    rng, orc, ctx, cl = _setup(prm, 64)
    N, L1 = prm.N, len(prm.q)
    level = L1 - 1
    top = np.array(prm.moduli, dtype=np.uint64) - np.uint64(1)
    key = np.broadcast_to(top[None, None, :, None], (prm.dnum, 2, len(prm.moduli), N)).copy()
    key[:, :, :, 1::3] = 0
    g = orc.galois_elt(7)
    ctx.he_evk_register(g, dev(key))
    qtop = top[:L1]
    full = np.broadcast_to(qtop[None, :, None], (2, L1, N)).copy()
    alt = full.copy()
    alt[:, :, ::2] = 0
    spike = np.zeros((2, L1, N), dtype=np.uint64)
    spike[:, :, N - 1] = qtop[None, :]
    idx = list(range(L1)) * 2
    for name, ct in (("full", full), ("alternating", alt), ("spike", spike)):
        d = dev(ct.reshape(2 * L1, N))
        ctx.he_ntt(d, idx)
        assert (host(d) == orc.ntt(ct.reshape(2 * L1, N), idx)).all(), name
        ctx.he_intt(d, idx)
        assert (host(d) == ct.reshape(2 * L1, N)).all(), name
        d = dev(ct.reshape(2 * L1, N))
        ctx.he_intt(d, idx)
        assert (host(d) == orc.intt(ct.reshape(2 * L1, N), idx)).all(), name
        out = zeros(2, L1, N)
        ctx.he_rotate(dev(ct), level, 7, out)
        assert (host(out) == orc.rotate(ct, level, g, key)).all(), name
        res = zeros(2, level, N)
        ctx.he_rescale(dev(ct), level, res)
        assert (host(res) == orc.rescale(ct, level)).all(), name


@pytest.mark.parametrize("case", range(10))
def test_random_parameter_sets_match_oracle(case):
    """Seeded random ring sizes, prime counts, digit counts, special-prime counts and levels on the generic
    kernels: key switch, hoisted rotations with an add, rescale and ct x ct multiply, bit for bit."""
    from gpu_util import dev, host, zeros
    rng = S.make_rng(2000 + case)
    logN = int(rng.integers(8, 13))
    nq = int(rng.integers(2, 9))
    dnum = int(rng.integers(1, nq + 1))
    alpha = -(-nq // dnum)
    np_ = int(rng.integers(alpha, alpha + 3))
    level = int(rng.integers(0, nq))
    prm = toy_params(logN=logN, q_bits=int(rng.integers(28, 50)), nq=nq, p_bits=int(rng.integers(50, 60)), np_=np_, dnum=dnum,
                     hamming=16, seed=2000 + case)
    _, orc, ctx, cl = _setup(prm, 2000 + case)
    N = prm.N
    steps = [int(rng.integers(1, N // 2)) for _ in range(3)]
    keys = {s: _key(prm, rng, cl, orc.galois_elt(s)) for s in set(steps)}
    for s, k in keys.items():
        ctx.he_evk_register(ctx.galois_elt(s), dev(k))
    rlk = cl.relin_key(S.uniform_limbs(rng, prm.moduli, N, prm.dnum), S.gaussian_error(rng, N, prm.sigma, prm.dnum))
    ctx.he_evk_register(0, dev(rlk))
    ct, ct2 = _rand_ct(prm, rng, level), _rand_ct(prm, rng, level)
    outs = [zeros(2, level + 1, N) for _ in steps]
    ctx.he_rotate_hoisted(dev(ct), level, steps, outs)
    for s, o in zip(steps, outs):
        assert (host(o) == orc.rotate(ct, level, orc.galois_elt(s), keys[s])).all(), (logN, nq, dnum, np_, level, s)
    prod = zeros(2, level + 1, N)
    ctx.he_mulct(dev(ct), dev(ct2), level, prod)
    want = orc.mulct(ct, ct2, level, rlk)
    assert (host(prod) == want).all(), (logN, nq, dnum, np_, level)
    if level >= 1:
        res = zeros(2, level, N)
        ctx.he_rescale(prod, level, res)
        assert (host(res) == orc.rescale(want, level)).all()


@pytest.mark.parametrize("logN,q_bits,p_bits", [(13, 40, 50), (15, 54, 60), (17, 36, 59), (14, 57, 58)])
def test_two_pass_generic_rings_key_switching(logN, q_bits, p_bits):
    """Ring sizes above 2^12 other than 2^16 (the paper's N = 2^15 and 2^17 among them) run the generic
    transform in two passes with gathered sources, per-limb output scaling and the stand-alone ModDown
    epilogue: key switch, hoisted and single rotations, conjugation, rescale and ct x ct multiply against the
    oracle, at the top level (three digits, the last one partial) and at a level with two digits."""
    from gpu_util import dev, host, zeros
    prm = toy_params(logN=logN, q_bits=q_bits, nq=5, p_bits=p_bits, np_=2, dnum=3, hamming=64, seed=300 + logN)
    rng, orc, ctx, cl = _setup(prm, 300 + logN)
    N = prm.N
    steps = [1, N // 4 + 3]
    keys = {s: _key(prm, rng, cl, orc.galois_elt(s)) for s in steps}
    for s, k in keys.items():
        ctx.he_evk_register(ctx.galois_elt(s), dev(k))
    kc = _key(prm, rng, cl, orc.galois_conj)
    ctx.he_evk_register(2 * N - 1, dev(kc))
    rlk = cl.relin_key(S.uniform_limbs(rng, prm.moduli, N, prm.dnum), S.gaussian_error(rng, N, prm.sigma, prm.dnum))
    ctx.he_evk_register(0, dev(rlk))
    for level in (4, 2):
        ct, ct2 = _rand_ct(prm, rng, level), _rand_ct(prm, rng, level)
        o0, o1 = zeros(level + 1, N), zeros(level + 1, N)
        ctx.he_keyswitch(dev(ct[1]), level, ctx.galois_elt(1), o0, o1)
        w0, w1 = orc.keyswitch(ct[1], level, keys[1])
        assert (host(o0) == w0).all() and (host(o1) == w1).all(), (logN, level)
        outs = [zeros(2, level + 1, N) for _ in steps]
        ctx.he_rotate_hoisted(dev(ct), level, steps, outs)
        for s, o in zip(steps, outs):
            want = orc.rotate(ct, level, orc.galois_elt(s), keys[s])
            assert (host(o) == want).all(), (logN, level, s)
            single = zeros(2, level + 1, N)
            ctx.he_rotate(dev(ct), level, s, single)
            assert (host(single) == want).all(), (logN, level, s)
        oc = zeros(2, level + 1, N)
        ctx.he_conjugate(dev(ct), level, oc)
        assert (host(oc) == orc.rotate(ct, level, orc.galois_conj, kc)).all(), (logN, level)
        prod = zeros(2, level + 1, N)
        ctx.he_mulct(dev(ct), dev(ct2), level, prod)
        want = orc.mulct(ct, ct2, level, rlk)
        assert (host(prod) == want).all(), (logN, level)
        res = zeros(2, level, N)
        ctx.he_rescale(prod, level, res)
        assert (host(res) == orc.rescale(want, level)).all(), (logN, level)
    # a real encryption decrypts to the rotated message on this path too
    z = rng.uniform(-1, 1, N // 2) + 1j * rng.uniform(-1, 1, N // 2)
    scale = 2.0 ** (q_bits - 6)      # the un-rounded ModDown leaves up to ~2N/pi * k / scale in the slot nearest the real axis
    ct = cl.encrypt(z, scale, 4, S.uniform_limbs(rng, prm.q[:5], N)[0], S.gaussian_error(rng, N, prm.sigma)[0])
    out = zeros(2, 5, N)
    ctx.he_rotate(dev(ct), 4, 1, out)
    assert np.max(np.abs(cl.decrypt(host(out), 4, scale) - np.roll(z, -1))) < 1e-3


def test_low_levels_single_launch_conversions():
    """N = 2^16 at the low levels the networks run at, where a single key switch is a handful of limbs: the
    conversions take the single-launch column kernel (inverse column pass, basis conversion and forward column
    pass in one).  One full digit (levels 5, 7), two digits (8, 15: a one-limb and a full second digit), singly,
    hoisted in pairs and as a conjugation, bit for bit against the oracle; a batch of three rotations (large
    enough to take the separate kernels) must give the same bits as the single calls."""
    from gpu_util import dev, host, zeros
    prm = config_params(2)
    rng, orc, ctx, cl = _setup(prm, 77)
    N = prm.N
    steps = [1, 2, 4]
    keys = {s: _key(prm, rng, cl, orc.galois_elt(s)) for s in steps}
    kc = _key(prm, rng, cl, orc.galois_conj)
    for s, k in keys.items():
        ctx.he_evk_register(ctx.galois_elt(s), dev(k))
    ctx.he_evk_register(2 * N - 1, dev(kc))
    for level in (5, 7, 8, 15):
        print("level", level, flush=True)
        ct = _rand_ct(prm, rng, level)
        d = dev(ct)
        want = {s: orc.rotate(ct, level, orc.galois_elt(s), keys[s]) for s in steps}
        single = {}
        for s in steps:
            o = zeros(2, level + 1, N)
            ctx.he_rotate(d, level, s, o)
            single[s] = host(o)
            assert (single[s] == want[s]).all(), (level, s, "single")
        outs = [zeros(2, level + 1, N) for _ in range(2)]
        ctx.he_rotate_hoisted(d, level, steps[:2], outs)
        for s, o in zip(steps[:2], outs):
            assert (host(o) == want[s]).all(), (level, s, "hoisted pair")
        outs = [zeros(2, level + 1, N) for _ in steps]
        ctx.he_rotate_batch([d], level, steps, outs, hoisted=True)
        for s, o in zip(steps, outs):
            assert (host(o) == want[s]).all(), (level, s, "batch of three")
        oc = zeros(2, level + 1, N)
        ctx.he_conjugate(d, level, oc)
        assert (host(oc) == orc.rotate(ct, level, orc.galois_conj, kc)).all(), (level, "conj")
