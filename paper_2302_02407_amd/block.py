"""Downsampling residual block composed from the C-ABI calls (sequencing and buffers only).

Shape of the paper's ResNet-20 first downsampling block (Section 4.1): a 3x3 stride-2
channel-aligned convolution, the polynomial activation applied to its output, and the 1x1
stride-2 shortcut convolution added to the result.  The stride lives in the weight
plaintexts (void packing, Section 2.2): positions that the stride skips are multiplied by
zero.  The n_out output ciphertexts of each convolution are brought into one ciphertext by
multiplying output o with a plaintext that is one on channel block o and zero elsewhere and
summing (one extra level).

Every plaintext and every integer constant comes from the caller, who keeps the scale
bookkeeping (Section 2.1: level and scale are metadata); nothing here touches a residue.
The activation is p(p(u)), p(u) = 1.5u - 0.5u^3, evaluated as t = u*(3 - u^2) with the factor
one half carried in the scale: two levels per application.
"""
import torch


class BufferPool:
    """Ciphertext buffers handed out in call order and reused across calls: a caller that runs the same block
    repeatedly (a serving loop, a timed region) allocates on the first pass only.  reset() rewinds to the first
    buffer; a buffer is reused only if the same position asks for the same level again."""

    def __init__(self):
        self._bufs, self._pos = [], 0

    def reset(self):
        self._pos = 0

    def ct(self, level, N):
        i = self._pos
        self._pos += 1
        if i < len(self._bufs) and self._bufs[i].shape == (2, level + 1, N):
            return self._bufs[i]
        t = torch.empty((2, level + 1, N), dtype=torch.uint64, device="cuda")
        if i < len(self._bufs):
            self._bufs[i] = t
        else:
            self._bufs.append(t)
        return t


_pool = None


def use_pool(pool):
    """Route the buffers of the functions below through `pool` (None: allocate afresh every time)."""
    global _pool
    _pool = pool
    if pool is not None:
        pool.reset()


def _ct(level, N):
    """Uninitialised ciphertext buffer (every use below overwrites it completely)."""
    if _pool is not None:
        return _pool.ct(level, N)
    return torch.empty((2, level + 1, N), dtype=torch.uint64, device="cuda")


def merge_outputs(ctx, outs, masks, level):
    """sum_o outs[o] (.) masks[o], rescaled: level -> level-1."""
    acc = _ct(level, ctx.N)
    for o, (ct, m) in enumerate(zip(outs, masks)):
        ctx.he_ptct_mac(acc, ct, m, level, init=(o == 0))
    return ctx.he_rescale(acc, level, _ct(level - 1, ctx.N))


def activation_step(ctx, u, level, k3):
    """u at `level` -> u*(3 - u^2) at level-2; k3 = the constant 3 at the scale of u^2 after its rescale."""
    N = ctx.N
    sq = ctx.he_mulct(u, u, level, _ct(level, N))
    w = ctx.he_rescale(sq, level, _ct(level - 1, N))
    ctx.he_affine(w, level - 1, [-1] * level, [k3] * level, w)
    u_low = _ct(level - 1, N)
    u_low.copy_(u[:, :level, :])                   # forget limb q_level (a slice, no arithmetic)
    prod = ctx.he_mulct(u_low, w, level - 1, _ct(level - 1, N))
    return ctx.he_rescale(prod, level - 1, _ct(level - 2, N))


def downsampling_block(ctx, C_a, H, W, R, level, ct_in, w3, w1, masks_main, masks_short, k_in, k3, k_short,
                       keep=False, hoisted_ras=False):
    """ct_in at `level` -> block output at level-6.

    w3 / w1: n_out*9 / n_out weight plaintexts at `level`; masks_*: n_out one-hot plaintexts at level-1;
    k_in: integer that lifts the merged main path to the activation's working scale; k3: the two
    constants of the activation steps; k_short: integer that lifts the merged shortcut to the scale
    of the activation's output.  With keep=True returns (out, dict of every intermediate).  hoisted_ras: the
    rotate-and-sum of both convolutions as one hoisted sum of rotations per output (see he_conv2d)."""
    N, n_out = ctx.N, len(masks_main)
    conv3 = ctx.he_conv2d(C_a, H, W, R, 3, level, w3, ct_in, [_ct(level - 1, N) for _ in range(n_out)], hoisted_ras=hoisted_ras)
    conv1 = ctx.he_conv2d(C_a, H, W, R, 1, level, w1, ct_in, [_ct(level - 1, N) for _ in range(n_out)], hoisted_ras=hoisted_ras)
    lv = level - 2
    merged = merge_outputs(ctx, conv3, masks_main, level - 1)
    u = ctx.he_affine(merged, lv, [k_in] * (lv + 1), [0] * (lv + 1), _ct(lv, N))
    a1 = activation_step(ctx, u, lv, k3[0])
    a2 = activation_step(ctx, a1, lv - 2, k3[1])
    short = merge_outputs(ctx, conv1, masks_short, level - 1)
    lo = lv - 4
    s_low = _ct(lo, N)
    s_low.copy_(short[:, :lo + 1, :])
    ctx.he_affine(s_low, lo, [k_short] * (lo + 1), [0] * (lo + 1), s_low)
    out = ctx.he_add(a2, s_low, lo, _ct(lo, N))
    if keep:
        return out, {"conv3": conv3, "conv1": conv1, "merged": merged, "u": u, "a1": a1, "a2": a2, "short": s_low}
    return out


def ca_square_ra(ctx, C_a, H, W, R, level, ct_in, w_ca, w_ra, k_in, n_mid, keep=False):
    """CAConv -> Square -> RAConv, the unit of the paper's fused block (Algorithm 3): ct_in at `level` ->
    one channel-aligned ciphertext at level-3.  w_ca: n_mid*9 plaintexts at `level`; w_ra: n_mid*9 inversely
    rotated plaintexts at level-2; k_in lifts the CAConv outputs to the working scale of the square.
    All n_mid intermediates are processed as one batch per stage (Algorithm 3 forwards them one by one
    to save memory; the values are the same)."""
    N = ctx.N
    lv = level - 1
    mids = ctx.he_conv2d(C_a, H, W, R, 3, level, w_ca, ct_in, [_ct(lv, N) for _ in range(n_mid)])
    sq = []
    for m in mids:
        ctx.he_affine(m, lv, [k_in] * (lv + 1), [0] * (lv + 1), m)
        ctx.he_mulct(m, m, lv, m)
        sq.append(ctx.he_rescale(m, lv, _ct(lv - 1, N)))
    out = ctx.he_raconv(W, R, 3, lv - 1, w_ra, sq, _ct(lv - 2, N))
    return (out, sq) if keep else out


def gap_sum_replicate(ctx, ct, level, R, mask):
    """After RAConv with R > 1 channels per input ciphertext: sum the R partial results of every pixel
    (log2 R rotations towards position 0), keep position 0 (MulPt with `mask`, Rescale), copy it back into
    the other R-1 positions (log2 R rotations the other way).  ct at `level` -> level-1, channel-aligned with
    R equal replicas (the input format of the next CAConv).  Needs keys for steps 2^t and N/2 - 2^t."""
    N, slots = ctx.N, ctx.N // 2
    w = ct
    t = 1
    while t < R:
        rot = ctx.he_rotate(w, level, t, _ct(level, N))
        w = ctx.he_add(w, rot, level, rot)
        t <<= 1
    acc = ctx.he_ptct_mac(_ct(level, N), w, mask, level, True)
    w = ctx.he_rescale(acc, level, _ct(level - 1, N))
    t = 1
    while t < R:
        rot = ctx.he_rotate(w, level - 1, slots - t, _ct(level - 1, N))
        w = ctx.he_add(w, rot, level - 1, rot)
        t <<= 1
    return w


def strided_gap_sum_replicate(ctx, cts, level, count, stride, mask):
    """For every ciphertext of the batch: sum `count` gap positions lying `stride` slots apart into the first
    (RaS_g: log2(count) rotations), keep it (MulPt with `mask`, Rescale), copy it back into the others (IR_g).
    level -> level-1.  Needs keys for stride*2^t and N/2 - stride*2^t."""
    N, slots = ctx.N, ctx.N // 2
    fwd, back, t = [], [], 1
    while t < count:
        fwd.append(stride * t)
        back.append(slots - stride * t)
        t <<= 1
    summed = ctx.he_ras(cts, level, fwd, [_ct(level, N) for _ in cts])
    kept = []
    for w in summed:
        acc = ctx.he_ptct_mac(_ct(level, N), w, mask, level, True)
        kept.append(ctx.he_rescale(acc, level, _ct(level - 1, N)))
    return ctx.he_ras(kept, level - 1, back, [_ct(level - 1, N) for _ in kept])


def downsample_handoff(ctx, C_a, Hp, Wp, R0, level, ct_in, p1, p2, mask_kappa, p3, mask_a, keep=False):
    """2-D gap packing across a stride-2 layer (Section 3.2), three layers on one input ciphertext in format
    (m, d) = (1, R0) with C_a channels on Hp x Wp:
      1. strided CAConv to 2*C_a channels (void-packed filters p1, 2*C_a/R0 outputs, no rotate-and-sum yet); pairs
         of outputs merged into the gap by one rotation each; rotate-and-sum over C_a on the merged ciphertexts and
         one more rotate-and-add that replicates over the freed rows: 2*C_a/(2*R0) ciphertexts carrying d' = 2*R0
         channels and m' = 2 replicas;
      2. RAConv on the logical Hp/2 x Wp/2 grid (p2) into one ciphertext, sum over the d' channel positions, mask,
         re-replication: format (m', d');
      3. CAConv on that multiplexed format (p3), rotate-and-sum over C_a, sum over the m' row positions, mask,
         re-replication.
    Levels: level -> level-1 -> level-3 -> level-5.  Returns the outputs of layer 3 (with keep=True every stage)."""
    N, slots = ctx.N, ctx.N // 2
    d, m = 2 * R0, 2
    n1, n = 2 * C_a // R0, 2 * C_a // d
    lv = level - 1
    ras_steps = []
    s = 1
    while s < C_a:
        ras_steps.append(Hp * Wp * R0 * s)
        s <<= 1
    row_step = Wp * R0
    conv1 = ctx.he_conv2d(C_a, Hp, Wp, R0, 3, level, p1, ct_in, [_ct(lv, N) for _ in range(n1)], skip_ras=True)
    merged = [ctx.he_rotate_sum([conv1[2 * o], conv1[2 * o + 1]], lv, [0, slots - R0], _ct(lv, N)) for o in range(n)]
    l1 = ctx.he_ras(merged, lv, ras_steps + [slots - row_step], [_ct(lv, N) for _ in range(n)])
    ra = ctx.he_raconv(Wp, 2 * R0, 3, lv, p2, l1, _ct(lv - 1, N))
    l2 = gap_sum_replicate(ctx, ra, lv - 1, d, mask_kappa)
    ca = ctx.he_conv2d(C_a, Hp // 2, Wp, 2 * R0, 3, lv - 2, p3, l2, [_ct(lv - 3, N) for _ in range(n)])
    l3 = strided_gap_sum_replicate(ctx, ca, lv - 3, m, row_step, mask_a)
    if keep:
        return l3, {"l1_conv": conv1, "l1": l1, "l2_conv": ra, "l2": l2, "l3_conv": ca, "l3": l3}
    return l3


def prcr_caconv_1x1(ctx, S, frag, level, plaintexts, cts_in, outs):
    """Pointwise convolution on the rearranged channel-aligned format (paper Section 3.3, PRCR): input ciphertext k
    holds, on row segment s, channel (k+s) mod S; plaintexts[o] holds Wt[o, s] on segment s and is reused for every
    input through a plaintext rotation by k fragments (`frag` slots each): out[o] = Rescale(sum_k cts_in[k] *
    PRot(plaintexts[o], k*frag)) is the whole image of output channel o.  S plaintexts serve the S*S pairs."""
    N = ctx.N
    gs = [ctx.galois_elt(k * frag) for k in range(S)]
    acc = _ct(level, N)
    for o in range(S):
        ctx.he_ptct_mac_rot(acc, cts_in, [plaintexts[o]] * S, gs, level, init=True)
        ctx.he_rescale(acc, level, outs[o])
    return outs


def prcr_raconv_1x1(ctx, S, frag, level, plaintexts, cts_in, outs):
    """The other direction: cts_in[c] is the whole image of channel c, plaintexts[c] holds Wt[s, c] on segment s;
    outs[k] = Rescale(sum_c cts_in[c] * PRot(plaintexts[c], k*frag)) is in the rearranged format again (segment s =
    output channel (k+s) mod S)."""
    N = ctx.N
    acc = _ct(level, N)
    for k in range(S):
        ctx.he_ptct_mac_rot(acc, cts_in, plaintexts, [ctx.galois_elt(k * frag)] * S, level, init=True)
        ctx.he_rescale(acc, level, outs[k])
    return outs

