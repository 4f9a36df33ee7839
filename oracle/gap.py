"""2-D gap packing across a downsampling layer on the oracle.  TEST INFRASTRUCTURE ONLY.

The paper (Section 3.2, "Data Formats for 2D Gap Packing"; cost table of Section 3.1, columns RaS_g and IR_g;
Section 4.3 for the schedule) packs the slots that a stride-2 convolution frees - the gap - with a mix of
multiplexed channels (m) and replicas (d); each convolution swaps the roles of the two gap dimensions, and m*d
quadruples at every downsampling layer (ResNet-20: (m,d) = (1,2) -> (2,4) -> (4,8)).  The text fixes the formats
pi_CA = {C_a, H, W, R_g, C_g}, pi_RA = {R_a, H, W, C_g, R_g} and the rotation counts; the slot assignment inside
the gap is a reading (stated below), chosen so that every step is one of the paper's operations.

Physical slot of block c, physical pixel (y, x), old replica r:  ((c*Hp + y)*Wp + x)*R0 + r.
After the stride-2 layer the logical pixel (h, w) owns the 2 x 2 x R0 slots (y, x, r) = (2h+a, 2w+b, r):
    channel position  kappa = b*R0 + r   (d' = 2*R0 contiguous slots),     replica position  a   (m' = 2).

Layer 1  CAConv, stride 2, format (1, R0) in:  Slide_f, MulFilter&Sum_f with void-packed filters (the paper's
         Figure of Section 2.2 (d)), Rescale - its c_out/R0 outputs hold R0 channels each at (a,b) = (0,0), zeros
         elsewhere.  Hand-off: pairs of outputs are merged into the gap, out[2o] + Rot(out[2o+1], one pixel
         right), which puts channel o*d' + kappa at position kappa; RaS over C_a (log2 C_a rotations) on the
         merged ciphertexts (half as many as before the merge); one more rotate-and-add, one physical row down,
         replicates over a.  Result: c_out/d' ciphertexts in pi_RA with C_g = d' channels, R_g = m' replicas.
Layer 2  RAConv (Algorithm 2) on the logical H/2 x W/2 grid: filter plaintext of (input i, tap) at slot
         (c', a, kappa) carries Wt[c'*m' + a, i*d' + kappa, tap] - the m' replicas multiplex m' output channels
         per block - then Slide_1&Sum_f (f^2-1 rotations by two physical pixels per logical one), Rescale,
         RaS_g over kappa (log2 d' rotations), mask kappa = 0 (MulPt, Rescale), IR_g (log2 d' rotations).
         Result: one ciphertext in pi_CA, format (m', d'): channel c*m' + a at block c, row parity a, d' replicas.
Layer 3  CAConv on format (m', d'): filter plaintext of (output o, tap) at (c, a, kappa) carries
         Wt[o*d' + kappa, c*m' + a, tap]; Slide_f, MulFilter&Sum_f, Rescale, RaS over C_a, RaS_g over a (log2 m'
         rotations by one physical row), mask a = 0, IR_g (log2 m').  Result: m'*C_a/d' ciphertexts in pi_RA,
         d' channels each, m' replicas - the counts of the cost table's CAConv row.
"""
import numpy as np

from . import block as OB
from . import conv2d as CV
from .ckks_client import encode


class Steps:
    """What the convolution routines of conv2d.py read from a geometry: taps, their slot amounts, RaS amounts."""

    def __init__(self, taps, tap_steps, ras_steps, n):
        self.taps, self.tap_steps, self.ras_steps = taps, tap_steps, ras_steps
        self.n_out = self.n_in = n


class GapGeometry:
    def __init__(self, N, C_a, Hp, Wp, c_in, c_out, f=3):
        slots = N // 2
        assert slots % (C_a * Hp * Wp) == 0 and Hp % 2 == 0 and Wp % 2 == 0 and f % 2 == 1
        self.N, self.slots, self.C_a, self.Hp, self.Wp, self.f = N, slots, C_a, Hp, Wp, f
        self.R0 = slots // (C_a * Hp * Wp)
        self.H, self.W = Hp // 2, Wp // 2                       # logical grid after the stride-2 layer
        self.d, self.m = 2 * self.R0, 2                         # (m', d') of the formats after the hand-off
        assert c_in == C_a and c_out == self.m * C_a and c_out % self.d == 0
        self.c_in, self.c_out = c_in, c_out
        self.g1 = CV.ConvGeometry(N, C_a, Hp, Wp, c_out, f=f, stride=2)      # layer 1: the void-packed strided layer
        self.n1 = self.g1.n_out                                 # outputs of layer 1 before the merge
        self.n = c_out // self.d                                # ciphertexts after the merge / outputs of layer 3
        half = (f - 1) // 2
        self.taps = [(dy, dx) for dy in range(-half, half + 1) for dx in range(-half, half + 1)]
        # one logical pixel = two physical ones
        self.tap_steps = [((dy * 2 * Wp + dx * 2) * self.R0) % slots for dy, dx in self.taps]
        self.ras_steps = list(self.g1.ras_steps)
        self.merge_step = slots - self.R0                       # one physical pixel to the right
        self.row_step = Wp * self.R0                            # one physical row (towards a = 0)
        self.ra = Steps(self.taps, self.tap_steps, [], self.n)                  # layer 2 as conv2d.raconv sees it
        self.ca = Steps(self.taps, self.tap_steps, self.ras_steps, self.n)      # layer 3 as conv2d.caconv sees it

    def all_steps(self):
        """Every rotation amount the three layers use (keys needed)."""
        s = set(st for st in self.g1.tap_steps if st) | set(self.ras_steps) | set(st for st in self.tap_steps if st)
        s |= {self.merge_step, self.slots - self.row_step, self.row_step}
        t = 1
        while t < self.d:
            s |= {t, self.slots - t}
            t <<= 1
        return sorted(s)

    # ---- slot views: [C_a][H][a][W][b][R0]
    def _view(self, v):
        return np.asarray(v).reshape(self.C_a, self.H, 2, self.W, 2, self.R0)

    def _valid(self, dy, dx):
        ok = np.zeros((self.H, self.W), dtype=bool)
        ok[max(0, -dy):min(self.H, self.H - dy), max(0, -dx):min(self.W, self.W - dx)] = True
        return ok

    def ra_filter_slots(self, wt, i, tap):
        """Layer 2, before the inverse rotation: Wt[c'*m + a, i*d + b*R0 + r, tap] at (c', h, a, w, b, r)."""
        dy, dx = self.taps[tap]
        half = (self.f - 1) // 2
        v = np.zeros((self.C_a, self.H, 2, self.W, 2, self.R0))
        ok = self._valid(dy, dx)
        for c in range(self.C_a):
            for a in range(2):
                for b in range(2):
                    for r in range(self.R0):
                        v[c, :, a, :, b, r] = ok * wt[c * self.m + a, i * self.d + b * self.R0 + r, dy + half, dx + half]
        return v.reshape(-1)

    def ra_weight_slots(self, wt, i, tap):
        return np.roll(self.ra_filter_slots(wt, i, tap), self.tap_steps[tap])

    def ca_weight_slots(self, wt, o, tap):
        """Layer 3: Wt[o*d + b*R0 + r, c*m + a, tap] at (c, h, a, w, b, r)."""
        dy, dx = self.taps[tap]
        half = (self.f - 1) // 2
        v = np.zeros((self.C_a, self.H, 2, self.W, 2, self.R0))
        ok = self._valid(dy, dx)
        for c in range(self.C_a):
            for a in range(2):
                for b in range(2):
                    for r in range(self.R0):
                        v[c, :, a, :, b, r] = ok * wt[o * self.d + b * self.R0 + r, c * self.m + a, dy + half, dx + half]
        return v.reshape(-1)

    def kappa0_mask_slots(self):
        v = np.zeros((self.C_a, self.H, 2, self.W, 2, self.R0))
        v[:, :, :, :, 0, 0] = 1.0
        return v.reshape(-1)

    def a0_mask_slots(self):
        v = np.zeros((self.C_a, self.H, 2, self.W, 2, self.R0))
        v[:, :, 0] = 1.0
        return v.reshape(-1)

    # ---- what each stage should decrypt to, given float tensors [channels][H][W]
    def expect_ra_format(self, y, o):
        """pi_RA ciphertext o: channel o*d + kappa at position kappa, every block and replica."""
        v = np.zeros((self.C_a, self.H, 2, self.W, 2, self.R0))
        for b in range(2):
            for r in range(self.R0):
                v[:, :, :, :, b, r] = y[o * self.d + b * self.R0 + r][None, :, None, :]
        return v.reshape(-1)

    def expect_ca_format(self, y):
        """pi_CA ciphertext: channel c*m + a at block c, row parity a, every kappa."""
        v = np.zeros((self.C_a, self.H, 2, self.W, 2, self.R0))
        for c in range(self.C_a):
            for a in range(2):
                v[c, :, a, :, :, :] = y[c * self.m + a][:, :, None, None]
        return v.reshape(-1)


def _encode_set(orc, level, scale, slot_vectors):
    mods = list(range(level + 1))
    return np.stack([orc.ntt(orc.reduce_signed(encode(np.asarray(v, dtype=np.complex128), orc.N, scale), mods), mods) for v in slot_vectors])


def encode_handoff_weights(orc, geo, w1, w2, w3, level):
    """Filter and mask plaintexts of the three layers at their levels (scale = the prime each Rescale drops)."""
    q = orc.q
    p1 = CV.encode_weights(orc, geo.g1, w1, level, float(q[level]))
    p2 = np.stack([_encode_set(orc, level - 1, float(q[level - 1]), [geo.ra_weight_slots(w2, i, t) for t in range(len(geo.taps))])
                   for i in range(geo.n)])
    mk = _encode_set(orc, level - 2, float(q[level - 2]), [geo.kappa0_mask_slots()])[0]
    p3 = np.stack([_encode_set(orc, level - 3, float(q[level - 3]), [geo.ca_weight_slots(w3, o, t) for t in range(len(geo.taps))])
                   for o in range(geo.n)])
    ma = _encode_set(orc, level - 4, float(q[level - 4]), [geo.a0_mask_slots()])[0]
    return dict(p1=p1, p2=p2, mask_kappa=mk, p3=p3, mask_a=ma)


def ras(orc, ct, level, steps, evks):
    """ct <- ct + Rot(ct, s) for every s in order."""
    for st in steps:
        ct = orc.add(ct, orc.rotate(ct, level, orc.galois_elt(st), evks[st]), level)
    return ct


def strided_gap_sum_replicate(orc, ct, level, count, stride, mask, evks):
    """Sum `count` gap positions that lie `stride` slots apart into the first (RaS_g), keep it (MulPt with the mask,
    Rescale), copy it back into the others (IR_g): level -> level-1."""
    slots = orc.N // 2
    fwd, back, t = [], [], 1
    while t < count:
        fwd.append(stride * t)
        back.append(slots - stride * t)
        t <<= 1
    w = ras(orc, ct, level, fwd, evks)
    w = orc.rescale(orc.ptct_mac(None, w, mask, level, init=True), level)
    return ras(orc, w, level - 1, back, evks)


def downsample_handoff(orc, geo, ct, level, pw, evks, progress=None):
    """The three layers; returns every stage: l1 (list, pi_RA), l2 (pi_CA, format (m', d')), l3 (list, pi_RA)."""
    say = progress or (lambda m: None)
    st = {}
    # layer 1: strided CAConv without its RaS, then the hand-off into the gap
    raised = orc.modup(ct[1], level)
    slid = [ct.copy() if s == 0 else orc.rotate_from_raised(ct, raised, level, orc.galois_elt(s), evks[s]) for s in geo.g1.tap_steps]
    outs = []
    for o in range(geo.n1):
        acc = None
        for t in range(len(geo.taps)):
            acc = orc.ptct_mac(acc, slid[t], pw["p1"][o, t], level, init=(t == 0))
        outs.append(orc.rescale(acc, level))
    st["l1_conv"] = outs
    lv = level - 1
    l1 = []
    for o in range(geo.n):
        mg = orc.add(outs[2 * o], orc.rotate(outs[2 * o + 1], lv, orc.galois_elt(geo.merge_step), evks[geo.merge_step]), lv)
        l1.append(ras(orc, mg, lv, geo.ras_steps + [geo.slots - geo.row_step], evks))
    st["l1"] = l1
    say("gap hand-off: layer 1 done")
    # layer 2: RAConv, then the sum over the channel positions and the re-replication
    ra = CV.raconv(orc, geo.ra, l1, lv, pw["p2"], evks)
    st["l2_conv"] = ra
    st["l2"] = OB.gap_sum_replicate(orc, ra, lv - 1, geo.d, pw["mask_kappa"], evks)
    say("gap hand-off: layer 2 done")
    # layer 3: CAConv on the multiplexed format, then RaS_g over a, mask, IR_g
    ca = CV.caconv(orc, geo.ca, st["l2"], lv - 2, pw["p3"], evks)
    st["l3_conv"] = ca
    st["l3"] = [strided_gap_sum_replicate(orc, c, lv - 3, geo.m, geo.row_step, pw["mask_a"], evks) for c in ca]
    say("gap hand-off: layer 3 done")
    return st


def handoff_float(x, w1, w2, w3):
    y1 = CV.conv2d_float(x, w1, stride=2)
    y2 = CV.conv2d_float(y1, w2)
    return y1, y2, CV.conv2d_float(y2, w3)
