"""Downsampling residual block on the oracle.  TEST INFRASTRUCTURE ONLY.

Shape of the paper's ResNet-20 first downsampling block (Section 4.1) built from the library
operations of Section 2.1: 3x3 stride-2 CAConv (Section 3.1; stride by void packing, Section
2.2), the n_out outputs merged into one ciphertext with one-hot channel-block plaintexts,
the polynomial activation p(p(u)), p(u) = 1.5u - 0.5u^3, and the 1x1 stride-2 shortcut
convolution (merged the same way) added to it.

Scale plan (a reading; the paper leaves scale management to its library): with Delta = 2^40
and 54-bit primes a ct x ct product rescales to 2^26 and would collapse on the next one, so
the activation runs at a working scale near the prime size: the merged convolution output is
multiplied by the integer round(q/Delta) (no level), each p is evaluated as u*(3 - u^2) with
the factor one half carried in the scale (two levels), and the shortcut is brought onto
exactly the resulting scale through the scale of its merge plaintexts and one integer factor.
"""
import numpy as np

from . import conv2d as CV
from .ckks_client import encode


def block_scales(q, level, delta):
    """Metadata only: (k_in, [k3 of step 1, k3 of step 2], scale of the block output, k_short,
    scale of the shortcut's merge plaintexts)."""
    lv = level - 2
    k_in = int(round(q[lv] / delta))
    s, k3 = delta * k_in, []
    for L in (lv, lv - 2):
        s2 = s * s / q[L]                      # scale of u^2 after its rescale
        k3.append(int(round(3.0 * s2)))
        s = 2.0 * s * s2 / q[L - 1]            # u*(3-u^2) = 2 p(u): halve by doubling the scale
    k_short = int(round(s / delta))
    return k_in, k3, s, k_short, q[level - 1] * s / (delta * k_short)


def one_hot_masks(orc, geo, n, level, scale):
    """Plaintext o (NTT form at `level`) is one on channel block o, zero elsewhere."""
    mods = list(range(level + 1))
    out = []
    for o in range(n):
        z = np.zeros((geo.C_a, geo.H * geo.W * geo.R))
        z[o] = 1.0
        out.append(orc.ntt(orc.reduce_signed(encode(z.reshape(-1).astype(np.complex128), orc.N, scale), mods), mods))
    return out


def merge(orc, outs, masks, level):
    acc = None
    for o in range(len(masks)):
        acc = orc.ptct_mac(acc, outs[o], masks[o], level, init=(o == 0))
    return orc.rescale(acc, level)


def activation_step(orc, u, level, k3, rlk):
    """u -> u*(3 - u^2): MulCt, Rescale, affine, MulCt with u one level down, Rescale."""
    w = orc.rescale(orc.mulct(u, u, level, rlk), level)
    w = orc.affine(w, level - 1, [-1] * level, [k3] * level)
    return orc.rescale(orc.mulct(orc.drop_level(u, level), w, level - 1, rlk), level - 1)


def downsampling_block(orc, g3, g1, ct, level, p3, p1, m_main, m_short, evks, rlk, k_in, k3, k_short, progress=None,
                       hoisted_ras=False):
    """Returns every stage: conv3, conv1 (lists), merged, u, a1, a2, short, out."""
    st = {"conv3": CV.caconv(orc, g3, ct, level, p3, evks, progress=progress, hoisted_ras=hoisted_ras)}
    st["conv1"] = CV.caconv(orc, g1, ct, level, p1, evks, hoisted_ras=hoisted_ras)
    lv = level - 2
    st["merged"] = merge(orc, st["conv3"], m_main, level - 1)
    st["u"] = orc.affine(st["merged"], lv, [k_in] * (lv + 1), [0] * (lv + 1))
    st["a1"] = activation_step(orc, st["u"], lv, k3[0], rlk)
    st["a2"] = activation_step(orc, st["a1"], lv - 2, k3[1], rlk)
    lo = lv - 4
    sh = merge(orc, st["conv1"], m_short, level - 1)
    for L in range(lv, lo, -1):
        sh = orc.drop_level(sh, L)
    st["short"] = orc.affine(sh, lo, [k_short] * (lo + 1), [0] * (lo + 1))
    st["out"] = orc.add(st["a2"], st["short"], lo)
    return st


def block_float(x, w3, w1):
    """float64 reference in the void-packed layout: [c_out][H][W], zero where the stride skips."""
    keep = np.zeros((w3.shape[0],) + x.shape[1:])
    keep[:, ::2, ::2] = 1.0

    def p(v):
        return 1.5 * v - 0.5 * v ** 3
    return p(p(CV.conv2d_float(x, w3) * keep)) + CV.conv2d_float(x, w1) * keep


# ---------------------------------------------------------------------------------------------
# CAConv -> Square -> RAConv (the unit of Algorithm 3).  Algorithm 3 forwards each CAConv output
# through Square into the RAConv accumulators as soon as it exists, to bound the number of live
# ciphertexts; the values it computes are those of the plain sequence below (modular sums do not
# depend on the order of accumulation).  Scale plan as above: the CAConv outputs are lifted to a
# scale near the prime size by an integer factor before the square.
def ca_square_ra(orc, g_ca, g_ra, ct, level, p_ca, p_ra, evks, rlk, k_in, progress=None):
    """ct at `level` -> (output ciphertext at level-3, list of squared intermediates at level-2)."""
    mids = CV.caconv(orc, g_ca, ct, level, p_ca, evks, progress=progress)
    lv = level - 1
    sq = []
    for m in mids:
        u = orc.affine(m, lv, [k_in] * (lv + 1), [0] * (lv + 1))
        sq.append(orc.rescale(orc.mulct(u, u, lv, rlk), lv))
    return CV.raconv(orc, g_ra, sq, lv - 1, p_ra, evks), sq


# ---------------------------------------------------------------------------------------------
# Sum across the gap dimension and re-replication after RAConv when each input ciphertext carried
# R > 1 channels (cost table of Section 3.1: RaS_g and IR_g, log2(m) rotations each; Section 3.4:
# one level for the multiplication with the mask).  RAConv leaves, in replica position r of every
# pixel, the partial sum over the input channels of class r.  RaS_g: w += Rot(w, 2^t), t < log2 R,
# gathers the total into position r = 0; a plaintext that is one at r = 0 and zero elsewhere
# (MulPt, Rescale) removes what the other positions picked up from neighbouring pixels; IR_g:
# w += Rot(w, -2^t) copies the total back into positions 1..R-1.  The result is a channel-aligned
# ciphertext with R equal replicas: the input format of the next CAConv.
def gap_mask(orc, geo, level, scale):
    z = np.zeros((geo.C_a * geo.H * geo.W, geo.R))
    z[:, 0] = 1.0
    mods = list(range(level + 1))
    return orc.ntt(orc.reduce_signed(encode(z.reshape(-1).astype(np.complex128), orc.N, scale), mods), mods)


def gap_sum_replicate(orc, ct, level, R, mask, evks):
    """ct [2][level+1][N] -> [2][level][N]; evks: slot-step -> key for steps 2^t and N/2 - 2^t, t < log2 R."""
    slots = orc.N // 2
    w = ct
    t = 1
    while t < R:
        w = orc.add(w, orc.rotate(w, level, orc.galois_elt(t), evks[t]), level)
        t <<= 1
    w = orc.rescale(orc.ptct_mac(None, w, mask, level, init=True), level)
    t = 1
    while t < R:
        w = orc.add(w, orc.rotate(w, level - 1, orc.galois_elt(slots - t), evks[slots - t]), level - 1)
        t <<= 1
    return w


# ---------------------------------------------------------------------------------------------
# The fused CAConv -> Square -> RAConv block, loop for loop as the paper's Algorithm 3 states it, for any
# number n_CA of channel-aligned ciphertexts: Slide_f of every input first; then, one replication-aligned
# intermediate j at a time, MulFilter&Sum_f over all inputs, RaS over C_a, Square, and its products with the
# inversely rotated RAConv filters added into the f^2 accumulators of every output (the forwarding that keeps
# only n_CA*f^2 ciphertexts alive); Slide_1&Sum_f of each output's accumulators last.  Rescales sit where the
# convolutions above put them (after MulFilter&Sum_f, after the square, after Slide_1&Sum_f), and the integer
# k_in lifts the CAConv output to the working scale of the square.
#
# Channel bookkeeping for n_CA > 1: input ciphertext k holds channels k*C_a .. (k+1)*C_a - 1 (one per block);
# intermediate j holds channel (j*R + r) mod c_mid in replica r of every block; output ciphertext l holds output
# channels l*C_a .. (l+1)*C_a - 1.  p_ca[j][k] are the f^2 filter plaintexts of (intermediate j, input k) at
# `level`; p_ra[l][j] the f^2 inversely rotated plaintexts of (output l, intermediate j) at level-2.
def ca_ra_block(orc, g_ca, g_ra, cts_in, level, p_ca, p_ra, evks, rlk, k_in, deferred=False, keep=False, hoisted_ras=False):
    n_ca, n_ra, taps = len(cts_in), g_ca.n_out, len(g_ca.taps)
    assert g_ra.n_in == n_ra and len(p_ca) == n_ra and len(p_ra) == n_ca
    lv = level - 1
    ct1 = []
    for ct in cts_in:                                                     # Slide_f of every input
        raised = orc.modup(ct[1], level)
        ct1.append([ct.copy() if st == 0 else orc.rotate_from_raised(ct, raised, level, orc.galois_elt(st), evks[st])
                    for st in g_ca.tap_steps])
    ct4 = [[None] * taps for _ in range(n_ca)]
    squares = []
    for j in range(n_ra):
        acc = None
        for k in range(n_ca):                                             # MulFilter&Sum_f over every input
            for t in range(taps):
                acc = orc.ptct_mac(acc, ct1[k][t], p_ca[j][k][t], level, init=acc is None)
        cur = orc.rescale(acc, level)
        if hoisted_ras and g_ca.C_a > 1:                                  # RaS over C_a as one hoisted sum of rotations
            cur = CV.ras_hoisted(orc, g_ca, cur, lv, evks)
        else:
            for st in g_ca.ras_steps:                                     # RaS over C_a
                cur = orc.add(cur, orc.rotate(cur, lv, orc.galois_elt(st), evks[st]), lv)
        u = orc.affine(cur, lv, [k_in] * (lv + 1), [0] * (lv + 1))
        sq = orc.rescale(orc.mulct(u, u, lv, rlk), lv)                    # Square
        squares.append(sq)
        for l in range(n_ca):                                             # forwarded into every output's accumulators
            for t in range(taps):
                ct4[l][t] = orc.ptct_mac(ct4[l][t], sq, p_ra[l][j][t], lv - 1, init=ct4[l][t] is None)
    outs = []
    gs = [orc.galois_elt(st) for st in g_ra.tap_steps]
    for l in range(n_ca):                                                 # Slide_1&Sum_f
        if deferred:
            total = orc.rotate_sum_deferred(ct4[l], lv - 1, gs, [evks.get(st) for st in g_ra.tap_steps])
        else:
            total = None
            for t, st in enumerate(g_ra.tap_steps):
                term = ct4[l][t] if st == 0 else orc.rotate(ct4[l][t], lv - 1, gs[t], evks[st])
                total = term if total is None else orc.add(total, term, lv - 1)
        outs.append(orc.rescale(total, lv - 1))
    return (outs, squares) if keep else outs
