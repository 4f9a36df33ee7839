"""Channel-aligned homomorphic convolution (CAConv) on the oracle.  TEST INFRASTRUCTURE ONLY.

Follows the paper's order of operations: Slide_f (the f^2 rotations of the input,
Algorithm 1 first subroutine), MulFilter&Sum_f (Algorithm 1 second subroutine) once per
output ciphertext, Rescale (one level per SISO, Section 3.4), then rotate-and-sum over the
outermost channel dimension C_a (Section 2.2 "RaS", Section 3.1 "CAConv"), which leaves the
sum replicated in every C_a block because rotation is cyclic.

Data format pi_CA = {C_a, H, W, R_g} with C_g = 1 (Section 3):
    slot(c, h, w, r) = ((c*H + h)*W + w)*R + r,   C_a*H*W*R = N/2,
every replica r holding the same input value x[c, h, w].
Output ciphertext o, replica r carries output channel co = (o*R + r) mod c_out.
"""
import numpy as np

from .ckks_client import encode
from .he_oracle import Oracle


class ConvGeometry:
    def __init__(self, N, C_a, H, W, c_out, f=3, stride=1):
        assert f % 2 == 1
        self.N, self.C_a, self.H, self.W, self.c_out, self.f, self.stride = N, C_a, H, W, c_out, f, stride
        slots = N // 2
        assert slots % (C_a * H * W) == 0
        self.R = slots // (C_a * H * W)
        self.n_out = -(-c_out // self.R)
        half = (f - 1) // 2
        # Slide_f amounts (Algorithm 1: r = w_i*(j1-(f-1)/2) + (j2-(f-1)/2)), times the inner stride R
        self.taps = [(dy, dx) for dy in range(-half, half + 1) for dx in range(-half, half + 1)]
        self.tap_steps = [((dy * W + dx) * self.R) % slots for dy, dx in self.taps]
        # RaS over C_a: strides H*W*R * 2^t
        self.ras_steps = [H * W * self.R * (1 << t) for t in range(int(np.log2(C_a)))]
        assert (1 << len(self.ras_steps)) == C_a

    def slot(self, c, h, w, r):
        return ((c * self.H + h) * self.W + w) * self.R + r

    def out_channel(self, o, r):
        return (o * self.R + r) % self.c_out

    def pack_input(self, x):
        """x[C_a][H][W] -> slot vector [N/2], each value replicated R times."""
        assert x.shape == (self.C_a, self.H, self.W)
        return np.repeat(x.reshape(-1), self.R).astype(np.float64)

    def weight_slots(self, wt, o, tap):
        """Slot vector of the filter plaintext for output ciphertext o and tap (dy,dx):
        Wt[co(o,r), c, dy+half, dx+half] where the tap reads inside the image, else 0
        (zero padding by masking); for stride s only output pixels with h,w multiples of s
        are kept."""
        dy, dx = self.taps[tap]
        half = (self.f - 1) // 2
        v = np.zeros((self.C_a, self.H, self.W, self.R), dtype=np.float64)
        for r in range(self.R):
            co = self.out_channel(o, r)
            for h in range(0, self.H):
                if not (0 <= h + dy < self.H) or h % self.stride:
                    continue
                for w in range(0, self.W):
                    if not (0 <= w + dx < self.W) or w % self.stride:
                        continue
                    v[:, h, w, r] = wt[co, :, dy + half, dx + half]
        return v.reshape(-1)

    def unpack_output(self, z_list):
        """Decoded slot vectors of the n_out outputs -> (out[c_out][H][W] from block c'=0,
        max spread over the C_a replicated blocks)."""
        out = np.zeros((self.c_out, self.H, self.W), dtype=np.float64)
        spread = 0.0
        for o, z in enumerate(z_list):
            v = np.asarray(z).real.reshape(self.C_a, self.H, self.W, self.R)
            spread = max(spread, float(np.max(np.abs(v - v[0:1]))))
            for r in range(self.R):
                out[self.out_channel(o, r)] = v[0, :, :, r]
        return out, spread


def encode_weights(orc: Oracle, geo: ConvGeometry, wt, level, pt_scale):
    """All n_out*f^2 filter plaintexts at `level`, NTT form: uint64 [n_out][f^2][level+1][N]."""
    mods = list(range(level + 1))
    pts = np.empty((geo.n_out, len(geo.taps), level + 1, orc.N), dtype=np.uint64)
    for o in range(geo.n_out):
        for t in range(len(geo.taps)):
            m = encode(geo.weight_slots(wt, o, t).astype(np.complex128), orc.N, pt_scale)
            pts[o, t] = orc.ntt(orc.reduce_signed(m, mods), mods)
    return pts


def encode_weights_raised(orc: Oracle, geo: ConvGeometry, wt, level, pt_scale):
    """The same filter plaintexts over the raised basis q_0..q_level, p_0..p_{k-1}: the integer polynomial of
    each encoding reduced modulo every one of those primes, NTT form: uint64 [n_out][f^2][level+1+k][N].  The
    first level+1 limbs equal encode_weights' (same polynomial, same primes)."""
    mods = orc.raised_moduli(level)
    pts = np.empty((geo.n_out, len(geo.taps), len(mods), orc.N), dtype=np.uint64)
    for o in range(geo.n_out):
        for t in range(len(geo.taps)):
            m = encode(geo.weight_slots(wt, o, t).astype(np.complex128), orc.N, pt_scale)
            pts[o, t] = orc.ntt(orc.reduce_signed(m, mods), mods)
    return pts


def slide_mac_deferred(orc: Oracle, geo: ConvGeometry, ct, level, pts_raised, evks, keep=False):
    """Slide_f and MulFilter&Sum_f of Algorithm 1 with the ModDown of the tap rotations deferred across the sum
    over the taps: the filter plaintexts multiply the key-switch inner products while these are still over the
    raised basis, and only each output's sum is brought down.  With (c0, c1) the input, d = ModUp(c1), g_t the
    Galois element of tap t and pt_{o,t} the plaintext of output o and tap t:
        A_t          = sum_j sigma_{g_t}(d_j) * evk_{g_t},j                       (both components, raised basis)
        ACC_o        = sum_{t: g_t != 1} pt_{o,t} * A_t                           (raised basis)
        out_o        = ( ModDown(ACC_o,0) + sum_{t: g_t != 1} pt_{o,t} * sigma_{g_t}(c0) + pt_{o,c} * c0 ,
                         ModDown(ACC_o,1) + pt_{o,c} * c1 )                       (c = the tap that does not rotate)
    which is the product-sum of the rotated inputs up to one ModDown rounding per output instead of one per
    tap scaled by the plaintext.  Returns the n_out accumulators [2][level+1][N] (before Rescale)."""
    L1, rm = level + 1, orc.raised_moduli(level)
    qm = list(range(L1))
    raised = orc.modup(ct[1], level)
    ips, rot0 = {}, {}
    for t, step in enumerate(geo.tap_steps):
        if step == 0:
            continue
        g = orc.galois_elt(step)
        ips[t] = orc.inner_product(orc.automorph_ntt(raised, g), level, evks[step])
        rot0[t] = orc.automorph_ntt(ct[0], g)
    outs, inter = [], {"ip": ips, "acc_raised": [], "plain": []}
    for o in range(geo.n_out):
        acc = None                                   # [2][R][N] over the raised basis
        p0 = None                                    # plain (un-switched) part of component 0, [L1][N]
        p1 = None
        for t, step in enumerate(geo.tap_steps):
            w_q = pts_raised[o, t, :L1]
            if step == 0:
                a = orc.pointwise_mul(ct[0], w_q, qm)
                p0 = a if p0 is None else orc.add_limbs(p0, a, qm)
                p1 = orc.pointwise_mul(ct[1], w_q, qm)
                continue
            term = np.stack([orc.pointwise_mul(ips[t][c], pts_raised[o, t], rm) for c in range(2)])
            acc = term if acc is None else orc.add_limbs(acc, term, rm + rm)
            a = orc.pointwise_mul(rot0[t], w_q, qm)
            p0 = a if p0 is None else orc.add_limbs(p0, a, qm)
        if acc is None:
            out = np.stack([p0, p1])
        else:
            o0 = orc.add_limbs(orc.moddown(acc[0], level), p0, qm)
            o1 = orc.moddown(acc[1], level)
            if p1 is not None:
                o1 = orc.add_limbs(o1, p1, qm)
            out = np.stack([o0, o1])
        inter["acc_raised"].append(acc)
        inter["plain"].append((p0, p1))
        outs.append(out)
    return (outs, inter) if keep else outs


def ras_hoisted(orc: Oracle, geo: ConvGeometry, cur, level, evks):
    """Rotate-and-sum over C_a (Section 2.2) as the sum of the C_a - 1 rotations of `cur` by i*H*W*R slots plus `cur`
    itself, the rotations sharing one ModUp (they rotate the same ciphertext) and one ModDown (rotate_sum_deferred):
    the same sum as the log2(C_a) rotate-and-add steps, with one ModDown rounding instead of log2(C_a)."""
    base = geo.H * geo.W * geo.R
    rm, qm = orc.raised_moduli(level), list(range(level + 1))
    raised = orc.modup(cur[1], level)                       # shared by all the rotations: they rotate the same ciphertext
    acc = rot0 = None
    for i in range(1, geo.C_a):
        g = orc.galois_elt(base * i)
        ip = orc.inner_product(orc.automorph_ntt(raised, g), level, evks[base * i])
        acc = ip if acc is None else orc.add_limbs(acc, ip, rm + rm)
        r0 = orc.automorph_ntt(cur[0], g)
        rot0 = r0 if rot0 is None else orc.add_limbs(rot0, r0, qm)
    out = np.stack([orc.add_limbs(orc.moddown(acc[0], level), rot0, qm), orc.moddown(acc[1], level)])
    return orc.add(out, cur, level)


def caconv(orc: Oracle, geo: ConvGeometry, ct, level, pts, evks, keep=False, progress=None, deferred_taps=False,
           hoisted_ras=False):
    """ct [2][level+1][N] -> list of n_out ciphertexts [2][level][N].

    evks: dict slot-step -> evaluation key of the Galois element 5^step.
    With keep=True also returns every intermediate (for limb-by-limb parity checks).
    deferred_taps: Slide_f and MulFilter&Sum_f share one ModDown per output (slide_mac_deferred); `pts` are
    then the plaintexts over the raised basis (encode_weights_raised).
    hoisted_ras: the rotate-and-sum as one hoisted sum of rotations per output (ras_hoisted); evks must then hold
    the keys of i*H*W*R for every i < C_a."""
    inter = {"slide": [], "mac": [], "rescaled": [], "ras": []}
    if deferred_taps:
        macs = slide_mac_deferred(orc, geo, ct, level, pts, evks)
        outs = []
        for o in range(geo.n_out):
            inter["mac"].append(macs[o])
            cur = orc.rescale(macs[o], level)
            inter["rescaled"].append(cur)
            steps_out = []
            if hoisted_ras and geo.C_a > 1:
                cur = ras_hoisted(orc, geo, cur, level - 1, evks)
                steps_out.append(cur)
            else:
                for step in geo.ras_steps:
                    rot = orc.rotate(cur, level - 1, orc.galois_elt(step), evks[step])
                    cur = orc.add(cur, rot, level - 1)
                    steps_out.append(cur)
            inter["ras"].append(steps_out)
            outs.append(cur)
            if progress:
                progress("oracle caconv (one ModDown per output): output %d/%d done" % (o + 1, geo.n_out))
        return (outs, inter) if keep else outs
    # Slide_f: all rotations of the one input share a single ModUp of c1 (same bits as
    # separate rotations by construction)
    raised = orc.modup(ct[1], level)
    slid = []
    for step in geo.tap_steps:
        if step == 0:
            slid.append(ct.copy())
        else:
            slid.append(orc.rotate_from_raised(ct, raised, level, orc.galois_elt(step), evks[step]))
    inter["slide"] = slid
    if progress:
        progress("oracle caconv: Slide_f done")
    outs = []
    for o in range(geo.n_out):
        acc = None
        for t in range(len(geo.taps)):
            acc = orc.ptct_mac(acc, slid[t], pts[o, t], level, init=(t == 0))
        inter["mac"].append(acc)
        cur = orc.rescale(acc, level)
        inter["rescaled"].append(cur)
        steps_out = []
        if hoisted_ras and geo.C_a > 1:
            cur = ras_hoisted(orc, geo, cur, level - 1, evks)
            steps_out.append(cur)
        else:
            for step in geo.ras_steps:
                rot = orc.rotate(cur, level - 1, orc.galois_elt(step), evks[step])
                cur = orc.add(cur, rot, level - 1)
                steps_out.append(cur)
        inter["ras"].append(steps_out)
        outs.append(cur)
        if progress:
            progress("oracle caconv: output %d/%d done" % (o + 1, geo.n_out))
    return (outs, inter) if keep else outs


def conv2d_float(x, wt, stride=1):
    """Direct float64 cross-correlation with zero 'same' padding (the plaintext reference)."""
    c_out, c_in, f, _ = wt.shape
    _, H, W = x.shape
    half = (f - 1) // 2
    out = np.zeros((c_out, H, W), dtype=np.float64)
    for co in range(c_out):
        for c in range(c_in):
            for dy in range(-half, half + 1):
                for dx in range(-half, half + 1):
                    h0, h1 = max(0, -dy), min(H, H - dy)
                    w0, w1 = max(0, -dx), min(W, W - dx)
                    out[co, h0:h1, w0:w1] += wt[co, c, dy + half, dx + half] * x[c, h0 + dy:h1 + dy, w0 + dx:w1 + dx]
    return out[:, ::stride, ::stride] if stride > 1 else out


# ---------------------------------------------------------------------------------------------
# Replication-aligned convolution with reordered SISO (Section 3.1 "RAConv", Algorithm 2).
#
# Input: n_in ciphertexts in the format CAConv leaves (pi_RA): ciphertext i holds, in every one of
# the C_a blocks, channel ch(i, r) = (i*R + r) mod c_in in replica position r.  Output: one
# ciphertext in pi_CA whose block c' holds output channel c':
#     out(c', h, w, r) = sum_i sum_taps Wt[c', ch(i, r), tap] * x_ch(i,r)(h+dy, w+dx),
# i.e. for R = 1 the whole convolution and for R > 1 the partial sum over the input channels of
# replica class r (the sum across the gap dimension belongs to gap packing, Section 3.2, and is
# not part of Algorithm 2).
#
# Order of operations (Algorithm 2): MulFilter&Sum_ci first - for each tap, the products of all
# inputs with filter plaintexts that were rotated the opposite way in advance, summed with
# additions only - then Slide_1&Sum_f: one rotation per off-centre tap and additions (f^2-1
# rotations in all, cost table of Section 3.1).  Reading: the single Rescale of the layer comes
# last, after the sum (the paper fixes one level per SISO, Section 3.4, not its position);
# rotating before the rescale divides the key-switching noise by q_l as well.
class RAGeometry:
    def __init__(self, N, C_a, H, W, c_in, f=3):
        assert f % 2 == 1
        self.N, self.C_a, self.H, self.W, self.c_in, self.f = N, C_a, H, W, c_in, f
        slots = N // 2
        assert slots % (C_a * H * W) == 0
        self.R = slots // (C_a * H * W)
        self.n_in = -(-c_in // self.R)
        half = (f - 1) // 2
        self.taps = [(dy, dx) for dy in range(-half, half + 1) for dx in range(-half, half + 1)]
        self.tap_steps = [((dy * W + dx) * self.R) % slots for dy, dx in self.taps]

    def in_channel(self, i, r):
        return (i * self.R + r) % self.c_in

    def pack_input(self, x, i):
        """Slot vector of input ciphertext i: channel ch(i, r) of x[c_in][H][W] in replica r of every block."""
        v = np.empty((self.C_a, self.H, self.W, self.R), dtype=np.float64)
        for r in range(self.R):
            v[:, :, :, r] = x[self.in_channel(i, r)][None, :, :]
        return v.reshape(-1)

    def filter_slots(self, wt, i, tap):
        """The plaintext that would multiply the slid input in the usual order: Wt[c', ch(i,r), tap] at
        slot (c', h, w, r) where the tap reads inside the image, else 0.  wt: [C_a][c_in][f][f]."""
        dy, dx = self.taps[tap]
        half = (self.f - 1) // 2
        v = np.zeros((self.C_a, self.H, self.W, self.R), dtype=np.float64)
        for r in range(self.R):
            ci = self.in_channel(i, r)
            for h in range(self.H):
                if not 0 <= h + dy < self.H:
                    continue
                for w in range(self.W):
                    if 0 <= w + dx < self.W:
                        v[:, h, w, r] = wt[:, ci, dy + half, dx + half]
        return v.reshape(-1)

    def weight_slots(self, wt, i, tap):
        """The same plaintext rotated the opposite way (Figure 'plaintexts inversely rotated'): it meets
        the input before the rotation by the tap amount, so its entry for output slot s sits at s + step."""
        return np.roll(self.filter_slots(wt, i, tap), self.tap_steps[tap])


def encode_ra_weights(orc: Oracle, geo: RAGeometry, wt, level, pt_scale):
    """uint64 [n_in][f^2][level+1][N], NTT form."""
    mods = list(range(level + 1))
    pts = np.empty((geo.n_in, len(geo.taps), level + 1, orc.N), dtype=np.uint64)
    for i in range(geo.n_in):
        for t in range(len(geo.taps)):
            m = encode(geo.weight_slots(wt, i, t).astype(np.complex128), orc.N, pt_scale)
            pts[i, t] = orc.ntt(orc.reduce_signed(m, mods), mods)
    return pts


def raconv(orc: Oracle, geo: RAGeometry, cts, level, pts, evks, keep=False, deferred=False):
    """cts: n_in ciphertexts [2][level+1][N] -> one ciphertext [2][level][N].

    deferred=True evaluates Slide_1 & Sum_f with one ModDown for the whole sum (Oracle.rotate_sum_deferred)
    instead of one per rotated tap: same message, different bits, less rounding."""
    inter = {"mac": [], "rot": []}
    for t in range(len(geo.taps)):
        acc = None
        for i in range(geo.n_in):
            acc = orc.ptct_mac(acc, cts[i], pts[i, t], level, init=(i == 0))
        inter["mac"].append(acc)
    if deferred:
        gs = [orc.galois_elt(step) for step in geo.tap_steps]
        total = orc.rotate_sum_deferred(inter["mac"], level, gs, [evks.get(step) for step in geo.tap_steps])
        inter["sum"] = total
        out = orc.rescale(total, level)
        return (out, inter) if keep else out
    total = None
    for t, step in enumerate(geo.tap_steps):
        term = inter["mac"][t] if step == 0 else orc.rotate(inter["mac"][t], level, orc.galois_elt(step), evks[step])
        inter["rot"].append(term)
        total = term if total is None else orc.add(total, term, level)
    inter["sum"] = total
    out = orc.rescale(total, level)
    return (out, inter) if keep else out
