"""PRCR (Section 3.3, "plaintext size reduction through image to ciphertext rearrangement") on the oracle, for
pointwise filters (f = 1, the case the paper's figure draws).  TEST INFRASTRUCTURE ONLY.

What the paper fixes: an image is split along its rows into S segments of H' = H/S rows; the channel-aligned format
becomes pi_CA' = {.., S, H', W, R}; a weight plaintext holds fragments of segment size arranged circularly and is
reused S times, each time multiplied with an input ciphertext and rotated by one fragment (a plaintext rotation, PRot
of Table 1: a slot permutation, no key); the sum over input channels restores image-size fragments; pi_RA is
unchanged, and the replication-aligned convolution, reusing its plaintexts the same way, returns pi_CA'.

The slot assignment is this reading (one image of H x W pixels per ciphertext, R replicas, S channels in and out):
    slot(s, h', w, r) = ((s*H' + h')*W + w)*R + r,            S*H'*W*R = N/2,   fragment = H'*W*R slots
    pi_CA' ciphertext X_k (k < S): segment s holds rows s*H'..(s+1)*H'-1 of channel (k + s) mod S
    pi_RA  ciphertext F_c       : the whole image of channel c
  CAConv' (X_* -> F_*):  plaintext P_o has Wt[o, s] on segment s;  F_o = sum_k X_k * PRot(P_o, k fragments)
      (rotating left by k fragments brings Wt[o, (s+k) mod S] onto segment s, where X_k holds channel (k+s) mod S)
  RAConv' (F_* -> Y_*):  plaintext Q_c has Wt[s, c] on segment s;  Y_k = sum_c F_c * PRot(Q_c, k fragments)
      (segment s of Y_k is then output channel (k+s) mod S: the format pi_CA' again)
Either way S plaintexts serve the S*S (output, input) pairs: the plaintext memory shrinks by S, at the price of S
plaintext rotations per plaintext.  Filters wider than one pixel would slide rows across segment borders, where a
pi_CA' ciphertext holds another channel; the paper does not say how it treats those borders, so only f = 1 is built.
"""
import numpy as np

from .ckks_client import encode
from .he_oracle import Oracle


class PrcrGeometry:
    def __init__(self, N, S, H, W):
        assert H % S == 0 and (N // 2) % (H * W) == 0
        self.N, self.S, self.H, self.W = N, S, H, W
        self.Hs = H // S
        self.R = (N // 2) // (H * W)
        self.frag = self.Hs * W * self.R                  # slots of one fragment; S fragments fill the ciphertext

    def pack_full(self, img):
        """img[H][W] -> slot vector (pi_RA: one whole channel image, R replicas)."""
        return np.repeat(np.asarray(img, dtype=np.float64).reshape(-1), self.R)

    def pack_ca(self, x, k):
        """x[S][H][W] -> slot vector of X_k: segment s = rows of channel (k+s) mod S."""
        rows = [x[(k + s) % self.S, s * self.Hs:(s + 1) * self.Hs] for s in range(self.S)]
        return self.pack_full(np.concatenate(rows, axis=0))

    def weights_ca(self, wt, o):
        """Slot vector of P_o: Wt[o, s] on segment s (wt[c_out][c_in])."""
        return np.repeat(np.asarray([wt[o, s] for s in range(self.S)], dtype=np.float64), self.frag)

    def weights_ra(self, wt, c):
        """Slot vector of Q_c: Wt[s, c] on segment s."""
        return np.repeat(np.asarray([wt[s, c] for s in range(self.S)], dtype=np.float64), self.frag)

    def unpack_full(self, z):
        v = np.asarray(z).real.reshape(self.H, self.W, self.R)
        return v[:, :, 0], float(np.max(np.abs(v - v[:, :, 0:1])))

    def unpack_ca(self, z_list):
        """Decoded X_* / Y_* -> channels [S][H][W]."""
        out = np.zeros((self.S, self.H, self.W))
        for k, z in enumerate(z_list):
            v = np.asarray(z).real.reshape(self.H, self.W, self.R)[:, :, 0]
            for s in range(self.S):
                out[(k + s) % self.S, s * self.Hs:(s + 1) * self.Hs] = v[s * self.Hs:(s + 1) * self.Hs]
        return out


def encode_plaintexts(orc: Oracle, geo: PrcrGeometry, wt, level, pt_scale, kind):
    """The S reusable plaintexts (kind 'ca': P_o, 'ra': Q_c), NTT form at `level`: uint64 [S][level+1][N]."""
    mods = list(range(level + 1))
    slots = geo.weights_ca if kind == "ca" else geo.weights_ra
    return np.stack([orc.ntt(orc.reduce_signed(encode(slots(wt, i).astype(np.complex128), orc.N, pt_scale), mods), mods)
                     for i in range(geo.S)])


def mac_rotated_plaintexts(orc: Oracle, cts, pts, gs, level):
    """sum_i cts[i] * sigma_{g_i}(pts[i]): the plaintext is permuted (PRot), the ciphertext is not."""
    acc = None
    for i, (ct, pt, g) in enumerate(zip(cts, pts, gs)):
        rp = pt if g == 1 else orc.automorph_ntt(pt, g)
        acc = orc.ptct_mac(acc, ct, rp, level, init=(i == 0))
    return acc


def caconv_1x1(orc: Oracle, geo: PrcrGeometry, X, level, P):
    """pi_CA' ciphertexts X[k] -> the S whole-image ciphertexts F[o] at level-1 (one Rescale)."""
    gs = [orc.galois_elt(k * geo.frag) for k in range(geo.S)]
    return [orc.rescale(mac_rotated_plaintexts(orc, X, [P[o]] * geo.S, gs, level), level) for o in range(geo.S)]


def raconv_1x1(orc: Oracle, geo: PrcrGeometry, F, level, Q):
    """Whole-image ciphertexts F[c] -> pi_CA' ciphertexts Y[k] at level-1."""
    out = []
    for k in range(geo.S):
        g = orc.galois_elt(k * geo.frag)
        out.append(orc.rescale(mac_rotated_plaintexts(orc, F, list(Q), [g] * geo.S, level), level))
    return out
