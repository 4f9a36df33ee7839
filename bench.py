#!/usr/bin/env python3
"""Benchmark of the MI355X homomorphic-convolution hot path (one GPU).

Primary workload (BASELINE configs[2]): rotation / key-switch benchmark at N = 2^16, 24 ciphertext
limbs of 54 bits + 8 special primes of 60 bits, dnum = 3.  One step = a batch of ciphertexts, each
rotated by all 15 power-of-two steps 2^0..2^14, once singly (own ModUp per rotation) and once
hoisted (one shared ModUp), both through the batched entry point he_rotate_batch: 30 key switches
per ciphertext per step.  value = key switches / s.
The same run also reports the NTT round-trip rate of configs[1] and the he_conv2d latency of
configs[3] as extra fields, the roofline of the dominant kernel (the NTT tile kernel) from HIP
events around each of its launches, and the CPU oracle timed on a bounded sample.

All inputs are synthetic and seeded; ciphertexts, keys and plaintexts are uniform residues (what
real ones look like limb by limb), generated on the device, so the timed region starts with
everything resident in HBM.
"""
import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0   # MI355X published HBM3E bandwidth
TRAFFIC_FILE = os.path.join(ROOT, "profiles", "bench_rotation_n65536_hbm_traffic.md")
VALU_FILE = os.path.join(ROOT, "profiles", "bench_rotation_n65536_valu_instructions.md")


def _profile_constant(path, key, build_id):
    """A `key = integer` line of a committed rocprofv3 --pmc summary, or None if the file is absent or was
    taken on another build of the library (its `build_id = ...` line differs from the library being timed)."""
    try:
        val, stamp = None, None
        for line in open(path):
            if line.startswith(key):
                val = int(line.split("=")[1])
            if line.startswith("build_id"):
                stamp = line.split("=")[1].strip()
        return val if stamp == build_id else None
    except OSError:
        return None


def uniform_dev(torch, gen, moduli, N, lead=()):
    """uint64 device tensor [*lead][len(moduli)][N], limb i uniform in [0, moduli[i])."""
    cols = [torch.randint(0, int(m), tuple(lead) + (1, N), dtype=torch.int64, device="cuda", generator=gen)
            for m in moduli]
    return torch.cat(cols, dim=len(lead)).contiguous().view(torch.uint64)


def run_only(args, torch, ctx, prm, gen):
    """One extra workload in isolation: configs[1] NTT round trip or configs[3] CAConv."""
    N, level = prm.N, len(prm.q) - 1
    if args.only == "crot5":
        # one rotation of a 6-limb ciphertext (the levels the paper's networks work at), in isolation
        key = uniform_dev(torch, gen, prm.moduli, N, lead=(prm.dnum, 2))
        ctx.he_evk_register(ctx.galois_elt(1), key)
        lo_ct = uniform_dev(torch, gen, prm.q[:6], N, lead=(2,))
        lo_out = torch.empty_like(lo_ct)

        def fn():
            ctx.he_rotate(lo_ct, 5, 1, lo_out)
    elif args.only == "ntt":
        idx = list(range(level + 1)) * 16
        data = uniform_dev(torch, gen, prm.q, N, lead=(16,))

        def fn():
            ctx.he_ntt(data, idx)
            ctx.he_intt(data, idx)
    else:
        held = []                                        # the library keeps pointers to the keys, not copies
        for s in sorted(set(((dy * 32 + dx) * 2) % (N // 2) for dy in (-1, 0, 1) for dx in (-1, 0, 1)) - {0}
                        | {2048, 4096, 8192, 16384}):
            held.append(uniform_dev(torch, gen, prm.moduli, N, lead=(prm.dnum, 2)))
            ctx.he_evk_register(ctx.galois_elt(s), held[-1])
        hoisted_ras = args.only in ("convh", "conv5h")    # rotate-and-sum as one hoisted sum per output
        if hoisted_ras:
            for i in range(1, 16):
                if 2048 * i not in (2048, 4096, 8192, 16384):
                    held.append(uniform_dev(torch, gen, prm.moduli, N, lead=(prm.dnum, 2)))
                    ctx.he_evk_register(ctx.galois_elt(2048 * i), held[-1])
        if args.only in ("conv5", "conv5h"):             # the same layer on a 6-limb ciphertext
            level = 5
        ct = uniform_dev(torch, gen, prm.q[:level + 1], N, lead=(2,))
        weights = [uniform_dev(torch, gen, prm.q[:level + 1], N) for _ in range(8 * 9)]
        outs = [torch.empty((2, level, N), dtype=torch.uint64, device="cuda") for _ in range(8)]

        def fn():
            ctx.he_conv2d(16, 32, 32, 2, 3, level, weights, ct, outs, hoisted_ras=hoisted_ras)
        if args.only == "raconv":                        # reordered RAConv on 8 inputs, one ModDown per output
            lv = level - 1
            ins = [uniform_dev(torch, gen, prm.q[:lv + 1], N, lead=(2,)) for _ in range(8)]
            ra_w = [w[:lv + 1] for w in weights]
            ra_out = torch.empty((2, lv, N), dtype=torch.uint64, device="cuda")
            ctx.he_ws_reserve(ctx.he_ws_query_raconv(8, 32, 2, 3, lv, deferred=True))

            def fn():
                ctx.he_raconv(32, 2, 3, lv, ra_w, ins, ra_out, deferred=True)
    for _ in range(args.warmup):
        fn()
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(args.steps):
        fn()
    torch.cuda.synchronize()
    ms = (time.perf_counter() - t0) / args.steps * 1e3
    print(json.dumps({"workload": args.only, "steps": args.steps, "warmup": args.warmup, "ms": round(ms, 4)}))


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=3)
    ap.add_argument("--warmup", type=int, default=1)
    ap.add_argument("--batch", type=int, default=64, help="ciphertexts per step (configs[2] names 64)")
    ap.add_argument("--no-cpu", action="store_true", help="skip the oracle timing leg")
    ap.add_argument("--no-extras", action="store_true", help="skip the NTT and conv2d extra measurements")
    ap.add_argument("--only", choices=["ntt", "conv2d", "conv0", "crot5", "conv5", "raconv", "convh", "conv5h"], help="run just this extra workload --steps times (for profiling "
                    "it in isolation) and print its own small JSON line instead of the benchmark line")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build runs on one GPU only (no collectives, no sharding); use --gpus 1", file=sys.stderr)
        sys.exit(2)

    import torch
    from he_inputs.params import config_params
    from paper_2302_02407_amd.binding import HEContext

    if not torch.cuda.is_available():
        print("bench.py: no GPU visible; the HIP path has no CPU fallback", file=sys.stderr)
        sys.exit(1)
    torch.cuda.set_device(0)
    prm = config_params(2)
    N, L1, k = prm.N, len(prm.q), len(prm.p)
    level = L1 - 1
    ctx = HEContext.from_params(prm)
    gen = torch.Generator(device="cuda")
    gen.manual_seed(prm.seed)

    # a plain device copy of known size: the byte counters of a --pmc run are scaled by what they
    # read for this dispatch
    calib_src = torch.empty(64 << 20, dtype=torch.uint8, device="cuda")
    calib_dst = torch.empty_like(calib_src)
    calib_dst.copy_(calib_src)
    del calib_src, calib_dst

    if args.only == "conv0":
        # configs[0]: tiny CAConv at N = 2^12 in isolation (for a kernel trace of the latency path)
        prm0 = config_params(0)
        ctx0 = HEContext.from_params(prm0)
        N0, lv0 = prm0.N, len(prm0.q) - 1
        keys0 = []
        for s in sorted(set(((dy * 8 + dx) * 8) % (N0 // 2) for dy in (-1, 0, 1) for dx in (-1, 0, 1)) - {0} | {512, 1024}):
            keys0.append(uniform_dev(torch, gen, prm0.moduli, N0, lead=(prm0.dnum, 2)))
            ctx0.he_evk_register(ctx0.galois_elt(s), keys0[-1])
        ct0 = uniform_dev(torch, gen, prm0.q, N0, lead=(2,))
        w0 = [uniform_dev(torch, gen, prm0.q, N0) for _ in range(9)]
        out0 = [torch.empty((2, lv0, N0), dtype=torch.uint64, device="cuda")]
        for _ in range(args.warmup):
            ctx0.he_conv2d(4, 8, 8, 8, 3, lv0, w0, ct0, out0)
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for _ in range(args.steps):
            ctx0.he_conv2d(4, 8, 8, 8, 3, lv0, w0, ct0, out0)
        torch.cuda.synchronize()
        print(json.dumps({"workload": "conv0", "steps": args.steps, "warmup": args.warmup,
                          "us": round((time.perf_counter() - t0) / args.steps * 1e6, 2)}))
        return
    if args.only:
        run_only(args, torch, ctx, prm, gen)
        return

    steps15 = [1 << i for i in range(15)]
    keys = {}
    for s in steps15:
        keys[s] = uniform_dev(torch, gen, prm.moduli, N, lead=(prm.dnum, 2))
        ctx.he_evk_register(ctx.galois_elt(s), keys[s])
    B = args.batch
    cts = [uniform_dev(torch, gen, prm.q, N, lead=(2,)) for _ in range(B)]
    outs = [torch.empty((2, L1, N), dtype=torch.uint64, device="cuda") for _ in range(B * 15)]

    def step():
        ctx.he_rotate_batch(cts, level, steps15, outs, hoisted=False)   # singly: a ModUp per rotation
        ctx.he_rotate_batch(cts, level, steps15, outs, hoisted=True)    # hoisted: one ModUp per ciphertext

    ks_per_step = B * 30
    for _ in range(args.warmup):
        step()
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(args.steps):
        step()
    torch.cuda.synchronize()
    dt = time.perf_counter() - t0
    ms_per_step = dt / args.steps * 1e3
    value = ks_per_step * args.steps / dt

    # single vs hoisted rates, one ciphertext each, HIP events on the context's stream
    def timed(fn, reps=3):
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        fn()
        torch.cuda.synchronize()
        e0.record()
        for _ in range(reps):
            fn()
        e1.record()
        torch.cuda.synchronize()
        return e0.elapsed_time(e1) / reps


    # roofline of the dominant kernels: one more, identical step with an event pair around every
    # transform launch (kept out of the timed steps so the events do not perturb `value`)
    ctx.he_profile_begin()
    step()
    prof = ctx.he_profile_end()
    build_id = ctx.he_build_id()
    limb_bytes = N * 8
    passes_per_transform = 2 if prm.logN > 12 else 1
    # algorithmic bytes: a limb transform reads and writes its limb once (2*N*8 B = 1 MiB at N = 2^16);
    # it runs as two passes, each credited half: 0.5 MiB per limb pass and nothing else
    alg_bytes = prof["transform_limb_passes"] * (2.0 * limb_bytes) / passes_per_transform
    t_s = prof["transform_ms"] * 1e-3
    launches = max(1, prof["transform_launches"])
    achieved = alg_bytes / t_s / 1e9
    # per-limb-pass constants measured with rocprofv3 --pmc on this same command (profiles/); each summary is
    # stamped with the build it was taken on and is not quoted for any other build
    bplp = _profile_constant(TRAFFIC_FILE, "transform_bytes_per_limb_pass", build_id)
    ops = _profile_constant(VALU_FILE, "transform_valu_lane_ops_per_limb_pass", build_id)
    kinds = ["fwd_column", "fwd_row", "fwd_row_inner_product_moddown", "inv_row", "inv_row_inner_product", "inv_column"]
    by_pass = {}
    for i, name in enumerate(kinds):
        if prof["pass_launches"][i]:
            ms_i = prof["pass_ms"][i]
            by_pass[name] = {"launches": prof["pass_launches"][i], "limb_passes": prof["pass_limbs"][i],
                             "avg_launch_us": round(ms_i * 1e3 / prof["pass_launches"][i], 2),
                             "us_per_limb_pass": round(ms_i * 1e3 / prof["pass_limbs"][i], 4),
                             "frac": round(prof["pass_limbs"][i] * limb_bytes / (ms_i * 1e-3) / 1e9 / HBM_PEAK_GBS, 4)}
    roofline = {
        "kernel": "ntt16_* (the four passes of the N=2^16 transform, incl. the passes that carry the key-switch inner product and the ModDown epilogue)",
        "bound": "hbm",
        "achieved": round(achieved, 1),          # 0.5 MiB per limb pass / time, nothing else counted
        "peak": HBM_PEAK_GBS,
        "unit": "GB/s",
        "frac": round(achieved / HBM_PEAK_GBS, 4),
        "traffic": None if bplp is None else round(bplp * prof["transform_limb_passes"] / launches),
        "algorithmic_bytes_per_launch": round(alg_bytes / launches),
        "limb_passes_per_launch": round(prof["transform_limb_passes"] / launches, 2),
        "measured_GBps": None if bplp is None else round(bplp * prof["transform_limb_passes"] / t_s / 1e9, 1),
        "launches": prof["transform_launches"],
        "avg_launch_us": round(prof["transform_ms"] * 1e3 / launches, 2),
        "share_of_step": round(prof["transform_ms"] / ms_per_step, 3),
        "by_pass": by_pass,
        # the same with the raised-digit limbs the inner-product passes have to read added (N*8 B each; keys not counted)
        "frac_with_digit_reads": round((alg_bytes + prof["inner_product_digit_limbs"] * limb_bytes) / t_s / 1e9 / HBM_PEAK_GBS, 4),
        "build_id": build_id,
    }
    # second roof: vector-ALU issue.  Peak = radix-2 butterflies/s measured on this GPU in this run with the
    # passes' own register blocks running out of registers (he_probe_alu); achieved = butterflies of the
    # timed launches (N/2 * 8 stages per limb pass) / their time.  Narrow (q) and wide (special) primes
    # are weighted by their share of the limb passes; the inverse rate by the inverse passes' share.
    probe = ctx.he_probe_alu()
    bf_per_pass = (N // 2) * (prm.logN // passes_per_transform)
    inv_share = (prof["pass_limbs"][3] + prof["pass_limbs"][4] + prof["pass_limbs"][5]) / max(1, prof["transform_limb_passes"])
    fwd_rate = probe["fwd_butterflies_per_s"]
    inv_rate = probe["inv_butterflies_per_s"] or fwd_rate
    peak_bf = 1.0 / ((1.0 - inv_share) / fwd_rate + inv_share / inv_rate)
    ach_bf = prof["transform_limb_passes"] * bf_per_pass / t_s
    roofline["alu"] = {"achieved": round(ach_bf / 1e12, 3), "peak": round(peak_bf / 1e12, 3), "unit": "T butterfly/s",
                       "frac": round(ach_bf / peak_bf, 4),
                       "probe": {k_: round(v / 1e12, 3) for k_, v in probe.items()},
                       "note": "butterflies only; conversions, inner products and epilogues issued by the same kernels are extra ALU work not counted in achieved"}
    if ops is not None:
        roofline["alu"]["valu_lane_ops_per_limb_pass"] = ops
        roofline["alu"]["lane_ops_per_s_T"] = round(ops * prof["transform_limb_passes"] / t_s / 1e12, 2)

    extras = {}
    if not args.no_extras:
        # the two halves of the step on their own, and one ciphertext at a time through the plain entry points
        # (latency-oriented callers)
        ms_single = timed(lambda: ctx.he_rotate_batch(cts, level, steps15, outs, hoisted=False), reps=2)
        ms_hoisted = timed(lambda: ctx.he_rotate_batch(cts, level, steps15, outs, hoisted=True), reps=2)
        ms_one_single = timed(lambda: [ctx.he_rotate(cts[0], level, s, outs[i]) for i, s in enumerate(steps15)])
        ms_one_hoisted = timed(lambda: ctx.he_rotate_hoisted(cts[0], level, steps15, outs[:15]))
        # the whole key switch against the HBM roof.  Compulsory bytes of one key switch = input polynomial
        # (L1 limbs) + outputs (2*L1 limbs) + its share of the key (2*dnum*(L1+k) limbs).  Loop order of this
        # engine: rotations are ordered step-major within a wave of 8 raised sources and run in launch sets
        # of up to 10 jobs; jobs of a set that use the same key share one pass over it, so the key is counted
        # once per (launch set, key) - the engine reports those key limbs (key_limbs_read).  The own-key
        # figure (every key switch reads its whole key) is given beside it.
        own_bytes = (L1 + 2 * prm.dnum * (L1 + k) + 2 * L1) * limb_bytes
        sched_bytes = (3 * L1) * limb_bytes + prof["key_limbs_read"] * limb_bytes / ks_per_step
        rate_s, rate_h = 15 * B / (ms_single * 1e-3), 15 * B / (ms_hoisted * 1e-3)
        roofline["keyswitch"] = {
            "loop_order": "step-major; 8 sources raised per wave; launch sets of <= 10 jobs; one key pass per (launch set, key)",
            "bytes_as_scheduled": round(sched_bytes),
            "frac_single": round(rate_s * sched_bytes / 1e9 / HBM_PEAK_GBS, 4),
            "frac_hoisted": round(rate_h * sched_bytes / 1e9 / HBM_PEAK_GBS, 4),
            "bytes_own_key": own_bytes,
            "frac_single_own_key": round(rate_s * own_bytes / 1e9 / HBM_PEAK_GBS, 4),
            "frac_hoisted_own_key": round(rate_h * own_bytes / 1e9 / HBM_PEAK_GBS, 4),
        }
        extras.update({
            "single_keyswitch_per_s": round(15 * B / (ms_single * 1e-3), 1),
            "hoisted_keyswitch_per_s": round(15 * B / (ms_hoisted * 1e-3), 1),
            "one_ct_single_keyswitch_per_s": round(15 / (ms_one_single * 1e-3), 1),
            "one_ct_hoisted_keyswitch_per_s": round(15 / (ms_one_hoisted * 1e-3), 1),
        })
    if not args.no_extras:
        # configs[1]: NTT + iNTT round trip of 16 polys x 24 limbs; limb-GB/s counts the limb read and
        # written once per transform
        idx = list(range(L1)) * 16
        data = uniform_dev(torch, gen, prm.q, N, lead=(16,))

        def roundtrip():
            ctx.he_ntt(data, idx)
            ctx.he_intt(data, idx)

        ms_rt = timed(roundtrip, reps=10)
        extras["ntt_roundtrip_ms"] = round(ms_rt, 4)
        extras["ntt_limb_GBps"] = round(384 * N * 8 * 2 * 2 / (ms_rt * 1e-3) / 1e9, 1)
        extras["ntt_limb_frac_of_hbm_peak"] = round(extras["ntt_limb_GBps"] / HBM_PEAK_GBS, 4)
        del data
        # the streaming operations on one ciphertext at level 23, as GB/s of the bytes they must move
        ct_bytes = 2 * L1 * N * 8
        pt = uniform_dev(torch, gen, prm.q, N)
        acc = torch.empty_like(cts[0])
        ms = timed(lambda: ctx.he_ptct_mac(acc, cts[0], pt, level, False), reps=20)
        extras["ptct_mac_GBps"] = round((3 * ct_bytes + ct_bytes // 2) / (ms * 1e-3) / 1e9, 1)     # acc r+w, ct r, pt r
        ms = timed(lambda: ctx.he_automorph(cts[0].view(2 * L1, N), acc.view(2 * L1, N), list(range(L1)) * 2, 5, True), reps=20)
        extras["automorph_GBps"] = round(2 * ct_bytes / (ms * 1e-3) / 1e9, 1)
        ms = timed(lambda: ctx.he_add(cts[0], cts[1 % B], level, acc), reps=20)
        extras["add_GBps"] = round(3 * ct_bytes / (ms * 1e-3) / 1e9, 1)
        res = torch.empty((2, level, N), dtype=torch.uint64, device="cuda")
        extras["rescale_us"] = round(1e3 * timed(lambda: ctx.he_rescale(cts[0], level, res), reps=20), 1)
        # the paper's Table 1 operations, one ciphertext per call at level 23, in milliseconds
        if 0 not in keys:
            keys[0] = uniform_dev(torch, gen, prm.moduli, N, lead=(prm.dnum, 2))
            ctx.he_evk_register(0, keys[0])
        t1 = {}
        t1["AddPt"] = timed(lambda: ctx.he_addpt(cts[0], pt, level, acc), reps=20)
        t1["AddCt"] = timed(lambda: ctx.he_add(cts[0], cts[1 % B], level, acc), reps=20)
        t1["MulPt"] = timed(lambda: ctx.he_ptct_mac(acc, cts[0], pt, level, True), reps=20)
        t1["MulCt"] = timed(lambda: ctx.he_mulct(cts[0], cts[1 % B], level, acc), reps=10)
        t1["Rescale"] = timed(lambda: ctx.he_rescale(cts[0], level, res), reps=20)
        pt_rot = torch.empty_like(pt)
        t1["PRot"] = timed(lambda: ctx.he_automorph(pt, pt_rot, list(range(L1)), 5, True), reps=20)
        t1["CRot"] = timed(lambda: ctx.he_rotate(cts[0], level, 1, acc), reps=10)
        # the paper's networks work at levels <= 6: the same rotation on a 6-limb ciphertext
        lo_ct = cts[0][:, :6, :].contiguous()
        lo_out = torch.empty_like(lo_ct)
        t1["CRot_level5"] = timed(lambda: ctx.he_rotate(lo_ct, 5, 1, lo_out), reps=10)
        extras["table1_ms"] = {k_: round(v, 4) for k_, v in t1.items()}
        del lo_ct, lo_out
        del pt, acc, res, pt_rot
        # configs[3]: ResNet-20-shaped CAConv, 16 -> 16 channels on 32x32, R = 2, level 23
        conv_steps = sorted(set(((dy * 32 + dx) * 2) % (N // 2) for dy in (-1, 0, 1) for dx in (-1, 0, 1)) - {0}
                            | {2048, 4096, 8192, 16384})
        for s in conv_steps:
            if s not in keys:
                keys[s] = uniform_dev(torch, gen, prm.moduli, N, lead=(prm.dnum, 2))
                ctx.he_evk_register(ctx.galois_elt(s), keys[s])
        weights = [uniform_dev(torch, gen, prm.q, N) for _ in range(8 * 9)]
        conv_out = [torch.empty((2, level, N), dtype=torch.uint64, device="cuda") for _ in range(8)]
        ms_conv = timed(lambda: ctx.he_conv2d(16, 32, 32, 2, 3, level, weights, cts[0], conv_out), reps=2)
        extras["conv2d_ms"] = round(ms_conv, 3)
        # the same layer with Slide_f and MulFilter&Sum_f sharing one ModDown per output (plaintexts over the raised
        # basis); with n_out = f^2 - 1 = 8 this saves no ModDown here, it pays off for fewer outputs or wider filters
        w_raised = [uniform_dev(torch, gen, list(prm.q) + list(prm.p), N) for _ in range(8 * 9)]
        ctx.he_ws_reserve(ctx.he_ws_query_conv2d(16, 32, 32, 2, 3, level, 8, deferred_taps=True))
        extras["conv2d_one_moddown_per_output_ms"] = round(
            timed(lambda: ctx.he_conv2d(16, 32, 32, 2, 3, level, w_raised, cts[0], conv_out, deferred_taps=True), reps=2), 3)
        del w_raised
        # the same layer with the rotate-and-sum over C_a as one hoisted sum of its 15 rotations per output (one ModUp
        # and one ModDown per output instead of four of each; needs the keys of every multiple of H*W*R)
        for i in range(1, 16):
            s = 2048 * i
            if s not in keys:
                keys[s] = uniform_dev(torch, gen, prm.moduli, N, lead=(prm.dnum, 2))
                ctx.he_evk_register(ctx.galois_elt(s), keys[s])
        ctx.he_ws_reserve(ctx.he_ws_query_conv2d(16, 32, 32, 2, 3, level, 8, hoisted_ras=True))
        extras["conv2d_hoisted_ras_ms"] = round(
            timed(lambda: ctx.he_conv2d(16, 32, 32, 2, 3, level, weights, cts[0], conv_out, hoisted_ras=True), reps=3), 3)
        # the 32 -> 32 channel layer on 16x16 images of ResNet-20's second stage (C_a = 32, R = 4, 8 output
        # ciphertexts): 5 rotate-and-sum rounds in the paper's order, or one hoisted sum of 31 rotations per output
        # (two launches of the inner products: 16 + 15 terms)
        steps32 = sorted(set(((dy * 16 + dx) * 4) % (N // 2) for dy in (-1, 0, 1) for dx in (-1, 0, 1)) - {0}
                         | {1024 * i for i in range(1, 32)})
        for s in steps32:
            if s not in keys:
                keys[s] = uniform_dev(torch, gen, prm.moduli, N, lead=(prm.dnum, 2))
                ctx.he_evk_register(ctx.galois_elt(s), keys[s])
        ctx.he_ws_reserve(ctx.he_ws_query_conv2d(32, 16, 16, 4, 3, level, 8, hoisted_ras=True))
        extras["conv2d_32ch_ms"] = round(timed(lambda: ctx.he_conv2d(32, 16, 16, 4, 3, level, weights, cts[0], conv_out), reps=2), 3)
        extras["conv2d_32ch_hoisted_ras_ms"] = round(
            timed(lambda: ctx.he_conv2d(32, 16, 16, 4, 3, level, weights, cts[0], conv_out, hoisted_ras=True), reps=3), 3)
        # the 16 -> 16 layer on a 6-limb ciphertext (level 5, where the paper's networks run their convolutions)
        lo_w = [w[:6] for w in weights]
        lo_in = cts[0][:, :6, :].contiguous()
        lo_outs = [torch.empty((2, 5, N), dtype=torch.uint64, device="cuda") for _ in range(8)]
        extras["conv2d_level5_ms"] = round(timed(lambda: ctx.he_conv2d(16, 32, 32, 2, 3, 5, lo_w, lo_in, lo_outs), reps=5), 3)
        extras["conv2d_level5_hoisted_ras_ms"] = round(
            timed(lambda: ctx.he_conv2d(16, 32, 32, 2, 3, 5, lo_w, lo_in, lo_outs, hoisted_ras=True), reps=5), 3)
        del lo_w, lo_in, lo_outs
        # the layer that consumes those 8 outputs: reordered RAConv (Algorithm 2), 8 inputs x 9 taps at level 22
        ra_w = [w[:level] for w in weights]
        ra_out = torch.empty((2, level - 1, N), dtype=torch.uint64, device="cuda")
        ms_ra = timed(lambda: ctx.he_raconv(32, 2, 3, level - 1, ra_w, conv_out, ra_out), reps=5)
        extras["raconv_ms"] = round(ms_ra, 3)
        # the same layer with Slide_1&Sum_f sharing one ModDown across its eight rotations
        ctx.he_ws_reserve(ctx.he_ws_query_raconv(8, 32, 2, 3, level - 1, deferred=True))
        ms_ra = timed(lambda: ctx.he_raconv(32, 2, 3, level - 1, ra_w, conv_out, ra_out, deferred=True), reps=5)
        extras["raconv_one_moddown_ms"] = round(ms_ra, 3)
        # sum across the gap and re-replication after that RAConv (two channels per ciphertext): 2 rotations,
        # one mask multiplication, one rescale, level 21 -> 20
        from paper_2302_02407_amd import block as blk
        for s in (1, N // 2 - 1):
            if s not in keys:
                keys[s] = uniform_dev(torch, gen, prm.moduli, N, lead=(prm.dnum, 2))
                ctx.he_evk_register(ctx.galois_elt(s), keys[s])
        extras["gap_sum_replicate_ms"] = round(timed(lambda: blk.gap_sum_replicate(ctx, ra_out, level - 2, 2, ra_w[0]), reps=3), 3)
        # CAConv -> Square -> RAConv, the unit of the paper's fused block (Algorithm 3), level 23 -> 20
        if 0 not in keys:
            keys[0] = uniform_dev(torch, gen, prm.moduli, N, lead=(prm.dnum, 2))
            ctx.he_evk_register(0, keys[0])
        ra_w2 = [w[:level - 1] for w in weights]
        # through the library's fused entry point: all 8 intermediates forwarded as one batch, and one at a time
        # (the loop order of Algorithm 3, which keeps the fewest ciphertexts alive); Slide_1&Sum_f with one ModDown
        blk_out = [torch.empty((2, level - 2, N), dtype=torch.uint64, device="cuda")]
        ctx.he_ws_reserve(ctx.he_ws_query_ca_ra_block(16, 32, 32, 2, 3, 1, 8, level, 0, True))
        for name, grp in (("ca_square_ra_ms", 0), ("ca_square_ra_forward_one_ms", 1)):
            ms_unit = timed(lambda: ctx.he_ca_ra_block(16, 32, 32, 2, 3, level, 8192, weights, ra_w2, [cts[0]], blk_out,
                                                       group=grp, deferred=True), reps=3)
            extras[name] = round(ms_unit, 3)
        # all intermediates batched, rotate-and-sum over C_a as one hoisted sum per intermediate
        ctx.he_ws_reserve(ctx.he_ws_query_ca_ra_block(16, 32, 32, 2, 3, 1, 8, level, 0, True, True))
        extras["ca_square_ra_hoisted_ras_ms"] = round(
            timed(lambda: ctx.he_ca_ra_block(16, 32, 32, 2, 3, level, 8192, weights, ra_w2, [cts[0]], blk_out, group=0, deferred=True,
                                             hoisted_ras=True), reps=3), 3)
        del blk_out
        conv_weights_h = weights if not args.no_cpu else None
        del weights, conv_out, ra_w, ra_out, ra_w2
        # configs[4]: downsampling block, 16 -> 32 channels, stride 2: 3x3 and 1x1 CAConv (16 outputs each),
        # one-hot merges, p(p(u)) with four ct x ct multiplies, shortcut add (constants are arbitrary here:
        # the timing does not depend on values)
        w3 = [uniform_dev(torch, gen, prm.q, N) for _ in range(16 * 9)]
        w1 = [uniform_dev(torch, gen, prm.q, N) for _ in range(16)]
        masks = [uniform_dev(torch, gen, prm.q[:level], N) for _ in range(16)]
        pool = blk.BufferPool()                          # temporaries allocated once, outside the timed repetitions
        ctx.he_ws_reserve(ctx.he_ws_query_conv2d(16, 32, 32, 2, 3, level, 16))

        def run_block():
            blk.use_pool(pool)
            blk.downsampling_block(ctx, 16, 32, 32, 2, level, cts[0], w3, w1, masks, masks, 8192, [3 << 53, 3 << 55], 1 << 17)

        ms_blk = timed(run_block, reps=10)
        extras["downsampling_block_ms"] = round(ms_blk, 3)
        ctx.he_ws_reserve(ctx.he_ws_query_conv2d(16, 32, 32, 2, 3, level, 16, hoisted_ras=True))

        def run_block_h():
            blk.use_pool(pool)
            blk.downsampling_block(ctx, 16, 32, 32, 2, level, cts[0], w3, w1, masks, masks, 8192, [3 << 53, 3 << 55], 1 << 17,
                                   hoisted_ras=True)

        extras["downsampling_block_hoisted_ras_ms"] = round(timed(run_block_h, reps=10), 3)
        blk.use_pool(None)
        del pool
        del w3, w1, masks

    if not args.no_extras:
        # configs[0]: tiny CAConv, N = 2^12, 4 -> 4 channels on 8x8, R = 8, level 2 (latency in microseconds)
        prm0 = config_params(0)
        ctx0 = HEContext.from_params(prm0)
        N0, lv0 = prm0.N, len(prm0.q) - 1
        keys0 = []
        for s in sorted(set(((dy * 8 + dx) * 8) % (N0 // 2) for dy in (-1, 0, 1) for dx in (-1, 0, 1)) - {0} | {512, 1024}):
            keys0.append(uniform_dev(torch, gen, prm0.moduli, N0, lead=(prm0.dnum, 2)))
            ctx0.he_evk_register(ctx0.galois_elt(s), keys0[-1])
        ct0 = uniform_dev(torch, gen, prm0.q, N0, lead=(2,))
        w0 = [uniform_dev(torch, gen, prm0.q, N0) for _ in range(9)]
        out0 = [torch.empty((2, lv0, N0), dtype=torch.uint64, device="cuda")]
        extras["conv2d_config0_us"] = round(1e3 * timed(lambda: ctx0.he_conv2d(4, 8, 8, 8, 3, lv0, w0, ct0, out0), reps=20), 1)
        # one output and eight rotated taps: one ModDown instead of eight (through the general kernels, not the
        # single-launch ones the tap-by-tap order takes on this ring)
        w0r = [uniform_dev(torch, gen, list(prm0.q) + list(prm0.p), N0) for _ in range(9)]
        ctx0.he_ws_reserve(ctx0.he_ws_query_conv2d(4, 8, 8, 8, 3, lv0, 1, deferred_taps=True))
        extras["conv2d_config0_one_moddown_us"] = round(
            1e3 * timed(lambda: ctx0.he_conv2d(4, 8, 8, 8, 3, lv0, w0r, ct0, out0, deferred_taps=True), reps=20), 1)
        del ctx0

    cpu = None
    if not args.no_cpu:
        # the oracle as it stands, on the host cores, on a bounded sample of the same workload:
        # two ciphertexts, all 15 steps, singly and hoisted (60 of the step's 1920 key switches)
        import numpy as np
        from oracle.he_oracle import Oracle, num_threads
        orc = Oracle.from_params(prm)
        n_ct = min(2, B)
        cts_h = [cts[i].cpu().numpy() for i in range(n_ct)]
        keys_h = [keys[s].cpu().numpy() for s in steps15]
        t0 = time.perf_counter()
        for ct_h in cts_h:
            for i, s in enumerate(steps15):
                orc.rotate(ct_h, level, orc.galois_elt(s), keys_h[i])
            raised = orc.modup(ct_h[1], level)
            for i, s in enumerate(steps15):
                orc.rotate_from_raised(ct_h, raised, level, orc.galois_elt(s), keys_h[i])
        dt_cpu = time.perf_counter() - t0
        cpu = {"value": round(30 * n_ct / dt_cpu, 3), "unit": "keyswitch/s", "cores": num_threads(), "kind": "oracle",
               "sample": "%d ciphertexts x 15 steps, singly + hoisted (%d key switches, %.1f s)" % (n_ct, 30 * n_ct, dt_cpu)}
        if not args.no_extras:
            # the other workloads of the line above, once each on the oracle
            from oracle import conv2d as ocv
            a_h = np.stack([c.cpu().numpy().reshape(2 * L1, N) for c in cts[:8]]).reshape(16 * L1, N)
            idx_h = list(range(L1)) * 16
            t0 = time.perf_counter()
            orc.intt(orc.ntt(a_h, idx_h), idx_h)
            cpu["ntt_roundtrip_ms"] = round((time.perf_counter() - t0) * 1e3, 1)
            geo = ocv.ConvGeometry(N, 16, 32, 32, 16)
            ev = {st: keys[st].cpu().numpy() for st in set(geo.tap_steps) | set(geo.ras_steps) if st}
            pts = np.stack([w.cpu().numpy() for w in conv_weights_h]).reshape(8, 9, L1, N)
            t0 = time.perf_counter()
            ocv.caconv(orc, geo, cts_h[0], level, pts, ev)
            cpu["conv2d_ms"] = round((time.perf_counter() - t0) * 1e3, 1)

    out = {
        "metric": "HRot keyswitches/s", "value": round(value, 1), "unit": "keyswitch/s", "n_gpus": 1,
        "steps": args.steps, "warmup": args.warmup, "ms_per_step": round(ms_per_step, 3), "higher_is_better": True,
        "scaling": "weak", "vs_baseline": None, "dtype": "u64", "data": "synthetic",
        "config": {"workload": "configs[2] rotation/key-switch: N=2^16, 24x54-bit + 8x60-bit primes, dnum=3, "
                               "%d ciphertexts x 15 steps, singly and hoisted" % B,
                   "batch": B, "keyswitches_per_step": ks_per_step},
        "roofline": roofline, "cpu_baseline": cpu,
    }
    out.update(extras)
    print(json.dumps(out))


if __name__ == "__main__":
    main()
