#!/usr/bin/env python3
"""Benchmark of the RNS-CKKS key-switch hot path on one MI355X.

One "step" is one pass of the whole path over one batch of synthetic input at N=2^16, L=24, K=6,
dnum=4 (the shape of workload 2): a batch of 8 HMult+relinearisations (shared evaluation key)
followed by a batch of 8 rotations (shared Galois key) -- 16 key switches.  `value` is key
switches per second with every operand resident in HBM.  Extras report the other quantities the
metric names: NTT limbs/s on config 1 (16 x 24 limbs) and hoisted rotations/s on config 3.

The line also carries
  roofline     : the kernel with the largest share of the timed region (instantiations of one
                 kernel template that differ only in an operand mode count as that kernel and
                 are listed as `members`): its algorithmic bytes per launch over its mean launch
                 duration (HIP events recorded by the library on the launch stream, in a further
                 pass of the same K steps) against 8 TB/s, with the binding resource decided by
                 the counters of the committed profile; `largest_instantiation` gives the same
                 for the single instantiation with the largest share when that is another kernel;
  step_roofline: compulsory bytes and HBM-side counter bytes of the whole step over ms_per_step
                 against 8 TB/s (the figure the 60 % target speaks of);
  cpu_baseline : the CPU oracle, as it stands, on a bounded sample of the same workload.
"""
import argparse
import json
import os
import re
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0
# VALU issue peak: 256 CUs x 4 SIMDs, one wave64 instruction per 4 cycles at 2.4 GHz = 39.3 T lane-instructions/s
# (the same units and clock that give the published 78.6 TFLOP/s fp64 figure, an FMA counting two flops).
VALU_PEAK_TINSTR = 256 * 64 * 2.4e9 / 1e12

# Per-launch counters of the default workload come from the committed rocprofv3 --pmc summary (they are lab numbers of
# the run that wrote that file, not something this run observes): HBM-side bytes (FETCH_SIZE scaled by 2, the factor a
# plain copy of known size shows, plus WRITE_SIZE) and wave-level VALU instructions (SQ_INSTS_VALU).  Kernels that the
# file does not list report null.
_MIB = 1 << 20
TRAFFIC_SOURCE = "profiles/keyswitch_step_n16_l24_d4_hbm_traffic.txt"


def load_counter_table(path=None):
    """{kernel: (read MiB, write MiB, VALU wave-instructions)} parsed from the committed counter summary."""
    import re
    rows = {}
    try:
        with open(path or os.path.join(ROOT, TRAFFIC_SOURCE)) as f:
            for ln in f:
                m = re.match(r"^(\S.*?>)\s+([\d.]+)\s+([\d.]+)\s+(\d+)\s+(\d+)(?:\s+\d+)*\s*$", ln)
                if m:
                    rows[m.group(1)] = (float(m.group(2)), float(m.group(3)), int(m.group(5)))
    except OSError:
        pass
    return rows


MEASURED = load_counter_table()


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=100)
    ap.add_argument("--warmup", type=int, default=10)
    ap.add_argument("--no-extras", action="store_true", help="skip every extra measurement")
    ap.add_argument("--extras", default="overlap,concurrent,ntt,hoisted,config4,latency,levels,standalone",
                    help="comma-separated extra measurements: overlap (two streams inside each call), concurrent "
                         "(HMult and HRot batches on two caller streams), ntt (config 1), hoisted "
                         "(config 3 rotations, singly and doubly hoisted), config4 (32 rotations at L = 35, dnum = 5), latency (one "
                         "ciphertext at a time), levels (rescale, "
                         "merged rescale, level-13 operations, limb-wise arithmetic)")
    ap.add_argument("--no-cpu", action="store_true", help="skip the CPU oracle baseline")
    ap.add_argument("--no-overlap", action="store_true",
                    help="time the step with every kernel of a call on the caller's stream (the default lets the library "
                         "run the FP64 ModUp conversion on its internal second stream beside the special-limb inner product)")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build runs on one GPU only (no sharding, no collectives); use --gpus 1",
              file=sys.stderr)
        sys.exit(2)

    import numpy as np
    import torch
    from paper_2310_16530_amd import binding, synth

    if not torch.cuda.is_available():
        print("bench.py: no GPU visible; the HIP path has no CPU fallback", file=sys.stderr)
        sys.exit(2)
    torch.cuda.set_device(0)

    ps = synth.CFG2
    B = synth.CFG2_BATCH
    N, L, D, dnum = ps.N, ps.L, ps.L + ps.K, ps.dnum
    ctx = binding.Context(ps.logN, ps.L, ps.K, ps.dnum, ps.primes)
    overlap = not args.no_overlap
    ctx.set_overlap(overlap)

    def dev(a):
        return torch.from_numpy(np.ascontiguousarray(a).view(np.int64)).to("cuda:0")

    rng = synth.rng_for(2, 100)
    ct1 = dev(synth.uniform_residues(rng, ps.q_primes, N, lead=(B, 2)))
    ct2 = dev(synth.uniform_residues(rng, ps.q_primes, N, lead=(B, 2)))
    # key limbs of a fresh RLWE key are uniform residues; run time does not depend on the values
    evk = dev(synth.uniform_residues(rng, ps.primes, N, lead=(dnum, 2)))
    rk = dev(synth.uniform_residues(rng, ps.primes, N, lead=(dnum, 2)))
    g = synth.galois_element(1, ps.logN)
    out1 = torch.empty_like(ct1)
    out2 = torch.empty_like(ct1)

    def step():
        ctx.hmult_relin(ct1, ct2, evk, out1)
        ctx.hrot(ct1, g, rk, out2)

    # untimed: STARTUP steps that take the device from idle to its running clocks (the first steps after start-up are
    # 5-9 % slower), then the W warm-up steps asked for
    STARTUP = 30
    for _ in range(STARTUP + args.warmup):
        step()
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(args.steps):
        step()
    torch.cuda.synchronize()
    t1 = time.perf_counter()
    ms_per_step = (t1 - t0) * 1e3 / args.steps
    ks_per_step = 2 * B
    value = ks_per_step / (ms_per_step * 1e-3)
    # the same K steps once more, each bracketed by two events on the launch stream: median beside the mean
    evs = [(torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)) for _ in range(args.steps)]
    for e0, e1 in evs:
        e0.record()
        step()
        e1.record()
    torch.cuda.synchronize()
    per_step = sorted(e0.elapsed_time(e1) for e0, e1 in evs)
    ms_median = per_step[len(per_step) // 2] if len(per_step) % 2 else 0.5 * (per_step[len(per_step) // 2 - 1] + per_step[len(per_step) // 2])

    # ---- per-kernel pass: the same K steps with HIP events around every launch, every kernel on the caller's
    # stream: a duration measured while another kernel shares the chip says nothing about the kernel.  The
    # dominant kernel (the q-limb inner product that also ends the ModDown) runs alone in the timed
    # configuration as well: the second stream is joined before it.
    ctx.set_overlap(False)
    ctx.profile_enable(True)
    for _ in range(args.steps):
        step()
    torch.cuda.synchronize()
    prof = ctx.profile_read()
    ctx.profile_enable(False)
    kernels = {}
    total_ms = sum(v[1] for v in prof.values()) or 1.0
    for name, (n, ms, nbytes) in prof.items():
        if n:
            k = {"launches_per_step": n / args.steps, "avg_us": round(1e3 * ms / n, 2),
                 "share": round(ms / total_ms, 4), "alg_GBps": round(nbytes / ms / 1e6, 1)}
            mk = MEASURED.get(name) if B == synth.CFG2_BATCH else None
            if mk:
                k["hbm_traffic_GBps"] = round((mk[0] + mk[1]) * _MIB / (ms / n * 1e-3) / 1e9, 1)
                k["valu_issue_frac"] = round(mk[2] * 64 / (ms / n * 1e-3) / 1e12 / VALU_PEAK_TINSTR, 3)
            kernels[name] = k
    # Algorithmic lane-operations per launch of the two conversion kernels on FP64 limbs (the kernels that VALU
    # issue binds), from operation counts and the shortest exact FP64 sequences: a modular product of two
    # residues below 2^50 is 6 instructions (mul, fma for the low part, mul by 1/q, round, fma, add), a
    # multiply-accumulate 7, a butterfly 8 (product, add, sub), the reduction of an accumulator 3; a 60-bit source
    # is first brought below the target prime (4: mul by 1/q, round, fma, add of the low half) and then takes one
    # multiply-accumulate.  Every converted word then takes (log2 N - 8) / 2 butterflies of the first forward pass.
    bfly = 8 * (ps.logN - 8) // 2
    n_fp_q = sum(1 for q in ps.q_primes if q < 3 << 48)
    alg_lane_ops = {
        # ModUp: per ciphertext and coefficient, every digit writes the FP64 q-limbs it does not own
        "conv_fwd_strided_kernel<FpAr, 8, 1, 3, false>": B * N * dnum * (n_fp_q - ps.L // dnum) * (7 * (ps.L // dnum) + 3 + bfly),
        # ModDown: both components, every FP64 q-limb, K sources of 60 bits
        # ModDown on the matrix cores: 7 conversions + 12 FP64 operations recombine an output, then the butterflies
        "conv_mfma_kernel<8, 2, 2, 1>": B * 2 * N * n_fp_q * (19 + bfly),
    }
    for kname_, ops in alg_lane_ops.items():
        if kname_ in kernels:
            t = kernels[kname_]["avg_us"] * 1e-6
            kernels[kname_]["alg_lane_ops_frac"] = round(ops / t / 1e12 / VALU_PEAK_TINSTR, 3)
    # ---- roofline of the kernel with the largest share of the timed region.  The headline figure is the HBM one:
    # algorithmic bytes per launch (limbs the launch must read plus write once, tables excluded) over the mean launch
    # duration from HIP events, against 8 TB/s.  Which resource binds the kernel is decided by the counters of the
    # committed profile, evaluated at this run's duration: VALU issue fraction against HBM-traffic fraction.
    # A kernel is one __global__ template; instantiations that differ only in how an operand is formed (the own-digit
    # mode of the inner product, the gather mode of the first inverse pass) are launches of the same kernel, listed
    # under `members` with their own durations.  `largest_instantiation` carries the same figures for the single
    # instantiation with the largest share, when that is a different kernel.
    def family(name):
        m = re.match(r"^(ks_inner_kernel<\w+, \d+, )\d+(, \w+, \w+>)$", name) or \
            re.match(r"^(inv_contig_kernel<\w+, \d+, )\d+(>)$", name)
        return m.group(1) + "*" + m.group(2) if m else name

    def roofline_of(label, names):
        dn = sum(prof[k][0] for k in names)
        dms = sum(prof[k][1] for k in names)
        dbytes = sum(prof[k][2] for k in names)
        dur_s = dms / dn * 1e-3
        hbm_gbs = dbytes / dms / 1e6
        have = B == synth.CFG2_BATCH and all(k in MEASURED for k in names)
        # counters: mean per launch over the launches of this run
        traffic = int(sum((MEASURED[k][0] + MEASURED[k][1]) * _MIB * prof[k][0] for k in names) / dn) if have else None
        r = {"kernel": label, "bound": "hbm", "achieved": round(hbm_gbs, 1), "peak": HBM_PEAK_GBS, "unit": "GB/s",
             "frac": round(hbm_gbs / HBM_PEAK_GBS, 4), "traffic": traffic,
             "traffic_source": TRAFFIC_SOURCE if have else None,
             "alg_bytes_per_launch": dbytes // dn, "avg_launch_us": round(1e6 * dur_s, 2),
             "share_of_step": round(dms / total_ms, 3)}
        if len(names) > 1:
            r["members"] = {k: {"launches_per_step": prof[k][0] / args.steps,
                                "alg_bytes_per_launch": prof[k][2] // prof[k][0],
                                "avg_launch_us": round(1e3 * prof[k][1] / prof[k][0], 2),
                                "frac": round(prof[k][2] / prof[k][1] / 1e6 / HBM_PEAK_GBS, 4)} for k in names}
        if have:
            valu = sum(MEASURED[k][2] * prof[k][0] for k in names) / dn
            traffic_frac = traffic / dur_s / 1e9 / HBM_PEAK_GBS
            issue_frac = valu * 64 / dur_s / 1e12 / VALU_PEAK_TINSTR
            r["hbm_counter_traffic"] = {"GBps": round(traffic / dur_s / 1e9, 1), "frac": round(traffic_frac, 4)}
            r["valu_issue"] = {"wave_instructions_per_launch": int(valu), "frac": round(issue_frac, 4),
                               "peak": "256 CU x 4 SIMD x one wave64 instruction per 4 cycles x 2.4 GHz"}
            r["bound"] = "alu" if issue_frac > traffic_frac else "hbm"
            r["bound_decided_by"] = "valu_issue.frac vs hbm_counter_traffic.frac of the same kernel"
        if len(names) == 1 and names[0] in alg_lane_ops:  # secondary: the method's own FP64 operation count
            alg_t = alg_lane_ops[names[0]] / dur_s / 1e12
            r["alu_algorithmic"] = {"lane_ops_per_launch": alg_lane_ops[names[0]], "achieved_T_per_s": round(alg_t, 2),
                                    "peak_T_per_s": round(VALU_PEAK_TINSTR, 2), "frac": round(alg_t / VALU_PEAK_TINSTR, 4),
                                    "note": "shortest exact FP64 sequences counted by hand; not a hardware counter"}
        return r

    launched = [k for k, v in prof.items() if v[0]]
    fams = {}
    for k in launched:
        fams.setdefault(family(k), []).append(k)
    dfam = max(fams, key=lambda f: sum(prof[k][1] for k in fams[f]))
    roofline = roofline_of(dfam, sorted(fams[dfam]))
    dinst = max(launched, key=lambda k: prof[k][1])
    if [dinst] != fams[dfam]:
        roofline["largest_instantiation"] = roofline_of(dinst, [dinst])

    # ---- the whole step against the HBM roofline: compulsory bytes (operands, keys and results moved once: 6L limbs
    # per HMult, 4L per HRot, one key of 2*dnum*(L+K) limbs per batch) and the HBM-side counter bytes of every launch
    limb = 8 * N
    compulsory = (B * 6 * L + 2 * dnum * D + B * 4 * L + 2 * dnum * D) * limb
    step_roofline = {"compulsory_bytes_per_step": compulsory,
                     "compulsory_GBps": round(compulsory / ms_per_step / 1e6, 1),
                     "compulsory_frac": round(compulsory / ms_per_step / 1e6 / HBM_PEAK_GBS, 4),
                     "counter_bytes_per_step": None, "counter_GBps": None, "counter_frac": None,
                     "target_frac": 0.6, "traffic_source": None}
    if B == synth.CFG2_BATCH and all(k in MEASURED for k in prof):
        cb = sum((MEASURED[k][0] + MEASURED[k][1]) * _MIB * n / args.steps for k, (n, _ms, _b) in prof.items())
        step_roofline.update({"counter_bytes_per_step": int(cb), "counter_GBps": round(cb / ms_per_step / 1e6, 1),
                              "counter_frac": round(cb / ms_per_step / 1e6 / HBM_PEAK_GBS, 4),
                              "traffic_source": TRAFFIC_SOURCE})

    extra = {"hmult_relin_per_s": None, "hrot_per_s": None}
    # split of the step (separately timed, same launch configuration)
    for name, fn in (("hmult_relin_per_s", lambda: ctx.hmult_relin(ct1, ct2, evk, out1)),
                     ("hrot_per_s", lambda: ctx.hrot(ct1, g, rk, out2))):
        torch.cuda.synchronize()
        a = time.perf_counter()
        for _ in range(args.steps):
            fn()
        torch.cuda.synchronize()
        extra[name] = round(B * args.steps / (time.perf_counter() - a), 1)

    EXTRA_GROUPS = ("overlap", "concurrent", "ntt", "hoisted", "config4", "latency", "levels", "standalone")
    groups = () if args.no_extras else tuple(g for g in args.extras.split(",") if g)
    for gname in groups:
        if gname not in EXTRA_GROUPS:
            print("bench.py: unknown --extras group %r (choose from %s)" % (gname, ", ".join(EXTRA_GROUPS)), file=sys.stderr)
            sys.exit(2)
    extra_kernels = {}

    def timed(fn, reps=None, label=None, pctx=None):
        """Seconds per call over `reps` calls after 2 warm-up calls; with a label, a second event-timed pass
        records the per-kernel averages of that operation."""
        reps = reps or args.steps
        for _ in range(2):
            fn()
        torch.cuda.synchronize()
        a0 = time.perf_counter()
        for _ in range(reps):
            fn()
        torch.cuda.synchronize()
        per = (time.perf_counter() - a0) / reps
        if label:
            pctx = pctx or ctx
            pctx.profile_enable(True)
            for _ in range(reps):
                fn()
            torch.cuda.synchronize()
            pr = pctx.profile_read()
            pctx.profile_enable(False)
            extra_kernels[label] = {k: {"launches_per_call": n / reps, "avg_us": round(1e3 * ms / n, 2),
                                        "alg_GBps": round(nb / ms / 1e6, 1)} for k, (n, ms, nb) in pr.items() if n}
        return per

    # the extra measurements run with every kernel on the caller's stream unless they say otherwise
    if "overlap" in groups and overlap:
        extra["key_switches_per_s_without_overlap"] = round(ks_per_step / timed(step), 1)
    elif "overlap" in groups:
        # the same step with the optional two-stream execution inside each call (integer special-limb launches
        # beside the floating-point launches)
        ctx.set_overlap(True)
        extra["key_switches_per_s_with_overlap"] = round(ks_per_step / timed(step), 1)
        ctx.set_overlap(False)

    if "concurrent" in groups:
        # the two halves of the step are independent: HMult batch and HRot batch issued on two streams, each with
        # its own context (tables and workspace), so that compute-bound and memory-bound kernels of the two
        # operations overlap
        ctx2 = binding.Context(ps.logN, ps.L, ps.K, ps.dnum, ps.primes)
        st = [torch.cuda.Stream(), torch.cuda.Stream()]

        def step2():
            for q_ in st:
                q_.wait_stream(torch.cuda.current_stream())
            with torch.cuda.stream(st[0]):
                ctx.hmult_relin(ct1, ct2, evk, out1)
            with torch.cuda.stream(st[1]):
                ctx2.hrot(ct1, g, rk, out2)
            for q_ in st:
                torch.cuda.current_stream().wait_stream(q_)

        extra["key_switches_per_s_two_op_streams"] = round(ks_per_step / timed(step2), 1)
        del ctx2

    if "ntt" in groups:
        # config 1: 16 polynomials x 24 limbs, forward and inverse
        x = dev(synth.uniform_residues(rng, ps.q_primes, N, lead=(synth.CFG1_BATCH,)))
        limbs = synth.CFG1_BATCH * L
        for name, inv in (("ntt_fwd_limbs_per_s", False), ("ntt_inv_limbs_per_s", True)):
            dt = timed(lambda: ctx.ntt(x, 0, inverse=inv), label="ntt_inv" if inv else "ntt_fwd")
            extra[name] = round(limbs / dt, 1)
            # one transform reads and writes every limb once: 2 * 8N bytes per limb (compulsory)
            extra[name.replace("limbs_per_s", "effective_GBps")] = round(limbs * 2 * 8 * N / dt / 1e9, 1)
            # the two passes together move every limb four times
            extra[name.replace("limbs_per_s", "pass_traffic_GBps")] = round(limbs * 4 * 8 * N / dt / 1e9, 1)
        del x

    if "hoisted" in groups:
        # config 3: 17 hoisted rotations with plaintext MAC (keys are rolled copies of one uniform key)
        rots = synth.CFG3_ROTATIONS
        gs = [synth.galois_element(r, ps.logN) for r in rots]
        rks = [torch.roll(rk, shifts=i + 1, dims=-1).contiguous() for i in range(len(rots))]
        pt = torch.stack([torch.roll(ct1[0, 0], shifts=i, dims=-1) for i in range(len(rots))]).contiguous()
        ct = ct1[0].contiguous()
        o = torch.empty_like(ct)
        reps = max(1, args.steps // 4)
        dt = timed(lambda: ctx.hrot_hoisted_mac(ct, gs, rks, pt, o), reps, "hoisted_rot_mac")
        extra["hoisted_rot_mac_per_s"] = round(len(rots) / dt, 1)
        # the same 17 rotations double-hoisted: plaintexts on the extended basis, one ModDown for the sum
        ptx = torch.stack([torch.roll(evk[0, 0], shifts=i, dims=-1) for i in range(len(rots))]).contiguous()
        dt = timed(lambda: ctx.hrot_dh_mac(ct, gs, rks, ptx, o), reps, "double_hoisted_rot_mac")
        extra["double_hoisted_rot_mac_per_s"] = round(len(rots) / dt, 1)
        # bytes that must come from HBM per rotation: the key (2*dnum*(L+K) limbs) and the plaintext (L+K limbs)
        extra["double_hoisted_key_stream_GBps"] = round(len(rots) * (2 * dnum + 1) * D * 8 * N / dt / 1e9, 1)
        # baby-step giant-step transform with 8 x 4 = 32 diagonals: 8 baby rotations computed once in the extended
        # basis and shared by 4 giant steps, each followed by its own rotation
        n1, n2 = 8, 4
        bg = [synth.galois_element(r, ps.logN) for r in range(n1)]
        gg = [synth.galois_element(r * n1, ps.logN) for r in range(n2)]
        ptb = torch.stack([torch.roll(evk[0, 0], shifts=i, dims=-1) for i in range(n1 * n2)]).reshape(n2, n1, D, N).contiguous()
        dt = timed(lambda: ctx.lintrans_bsgs_at(L, ct, bg, rks[:n1], gg, rks[n1:n1 + n2], ptb, o), reps, "lintrans_bsgs_8x4")
        extra["bsgs_8x4_transforms_per_s"] = round(1.0 / dt, 1)
        extra["bsgs_8x4_diagonals_per_s"] = round(n1 * n2 / dt, 1)
        del rks, pt, ptx, ptb

    if "config4" in groups:
        # config 4: N = 2^16, L = 35, K = 7, dnum = 5; 32 rotations by +-2^i of one ciphertext with plaintext MAC
        # (a CoeffToSlot-shaped stage), singly and doubly hoisted.  32 keys of 210 MiB: rolled copies of one.
        ps4 = synth.CFG4
        ctx4 = binding.Context(ps4.logN, ps4.L, ps4.K, ps4.dnum, ps4.primes)
        rng4 = synth.rng_for(4, 100)
        rots4 = synth.CFG4_ROTATIONS
        gs4 = [synth.galois_element(r, ps4.logN) for r in rots4]
        key4 = dev(synth.uniform_residues(rng4, ps4.primes, N, lead=(ps4.dnum, 2)))
        rks4 = [torch.roll(key4, shifts=i + 1, dims=-1).contiguous() for i in range(len(rots4))]
        ct4 = dev(synth.uniform_residues(rng4, ps4.q_primes, N, lead=(2,)))
        ptx4 = torch.stack([torch.roll(key4[0, 0], shifts=i, dims=-1) for i in range(len(rots4))]).contiguous()
        pt4 = ptx4[:, :ps4.L].contiguous()
        o4 = torch.empty_like(ct4)
        reps = max(1, args.steps // 10)
        dt = timed(lambda: ctx4.hrot_hoisted_mac(ct4, gs4, rks4, pt4, o4), reps, "config4_hoisted_rot_mac", ctx4)
        extra["config4_hoisted_rot_mac_per_s"] = round(len(rots4) / dt, 1)
        dt = timed(lambda: ctx4.hrot_dh_mac(ct4, gs4, rks4, ptx4, o4), reps, "config4_double_hoisted_rot_mac", ctx4)
        extra["config4_double_hoisted_rot_mac_per_s"] = round(len(rots4) / dt, 1)
        extra["config4_double_hoisted_key_stream_GBps"] = round(
            len(rots4) * (2 * ps4.dnum + 1) * (ps4.L + ps4.K) * 8 * N / dt / 1e9, 1)
        # a factorised slot transform of the same shape: three baby-step giant-step stages of 8 x 4 diagonals at
        # levels 35, 34, 33, each followed by a rescale (ready plaintext diagonals, keys shared by the stages)
        n1, n2 = 8, 4
        stage_args = []
        stride = 1
        for s_ in range(3):
            ell = ps4.L - s_
            bg = [synth.galois_element(b * stride, ps4.logN) for b in range(n1)]
            gg = [synth.galois_element(g_ * n1 * stride, ps4.logN) for g_ in range(n2)]
            ptb = ptx4[:, :ell + ps4.K].reshape(n2, n1, ell + ps4.K, N).contiguous()
            stage_args.append((ell, bg, gg, ptb, torch.empty((2, ell, N), dtype=ct4.dtype, device=ct4.device),
                               torch.empty((1, 2, ell - 1, N), dtype=ct4.dtype, device=ct4.device)))
            stride *= n1 * n2

        def chain():
            x = ct4
            for ell, bg, gg, ptb, mid, low in stage_args:
                ctx4.lintrans_bsgs_at(ell, x, bg, rks4[:n1], gg, rks4[n1:n1 + n2], ptb, mid)
                ctx4.rescale(ell, mid.reshape(1, 2, ell, N), low)
                x = low[0]

        dt = timed(chain, reps, "config4_transform_chain_3x32", ctx4)
        extra["config4_transform_chain_3x32_per_s"] = round(1.0 / dt, 1)
        extra["config4_transform_chain_diagonals_per_s"] = round(3 * n1 * n2 / dt, 1)
        del ctx4, key4, rks4, ct4, ptx4, pt4, o4, stage_args

    if "latency" in groups:
        # one ciphertext at a time (the latency a single HMult or rotation sees, launch gaps included)
        a1, b1, o1 = ct1[:1].contiguous(), ct2[:1].contiguous(), torch.empty_like(ct1[:1])
        extra["hmult_relin_batch1_latency_us"] = round(1e6 * timed(lambda: ctx.hmult_relin(a1, b1, evk, o1), label="hmult_relin_batch1"), 1)
        extra["hrot_batch1_latency_us"] = round(1e6 * timed(lambda: ctx.hrot(a1, g, rk, o1)), 1)
        ctx.set_overlap(True)
        extra["hmult_relin_batch1_latency_us_with_overlap"] = round(1e6 * timed(lambda: ctx.hmult_relin(a1, b1, evk, o1)), 1)
        extra["hrot_batch1_latency_us_with_overlap"] = round(1e6 * timed(lambda: ctx.hrot(a1, g, rk, o1)), 1)
        ctx.set_overlap(False)
        r1 = torch.empty((1, 2, L - 1, N), dtype=ct1.dtype, device=ct1.device)
        extra["hmult_relin_rescale_batch1_latency_us"] = round(1e6 * timed(lambda: ctx.hmult_relin_rescale_at(L, a1, b1, evk, r1)), 1)
        del a1, b1, o1, r1

    if "levels" in groups:
        # levels below L: rescale of the batch at level 24, and the HMult+relin -> rescale pair a CNN layer
        # issues; then HMult+relin at level 13 (digits of 6, 6 and 1 limbs) with the same full-level key
        rs_out = torch.empty((B, 2, L - 1, N), dtype=ct1.dtype, device=ct1.device)
        dt = timed(lambda: ctx.rescale(L, ct1, rs_out), label="rescale")
        extra["rescale_per_s"] = round(B / dt, 1)
        # compulsory bytes of a rescale: read 2L limbs, write 2(L-1)
        extra["rescale_effective_GBps"] = round(B * (4 * L - 2) * 8 * N / dt / 1e9, 1)

        def mult_rescale():
            ctx.hmult_relin(ct1, ct2, evk, out1)
            ctx.rescale(L, out1, rs_out)

        extra["hmult_relin_rescale_per_s"] = round(B / timed(mult_rescale), 1)
        # the same pair with the rescale merged into the ModDown (one division by P * q_last)
        dt = timed(lambda: ctx.hmult_relin_rescale_at(L, ct1, ct2, evk, rs_out), label="hmult_relin_rescale_merged")
        extra["hmult_relin_rescale_merged_per_s"] = round(B / dt, 1)
        lv = 13
        a13 = ct1[:, :, :lv].contiguous()
        b13 = ct2[:, :, :lv].contiguous()
        o13 = torch.empty_like(a13)
        extra["hmult_relin_level13_per_s"] = round(B / timed(lambda: ctx.hmult_relin_at(lv, a13, b13, evk, o13)), 1)
        extra["hrot_level13_per_s"] = round(B / timed(lambda: ctx.hrot_at(lv, a13, g, rk, o13)), 1)
        # limb-wise arithmetic on the batch (HAdd and ciphertext x plaintext): 2 polynomials x L limbs per ciphertext
        pw_out = torch.empty_like(ct1)
        ptw = evk[0, 0, :L].contiguous().reshape(1, L, N)
        dt = timed(lambda: ctx.pointwise(binding.PW_ADD, ct1, ct2, pw_out), label="pointwise_add")
        extra["hadd_per_s"] = round(B / dt, 1)
        extra["hadd_effective_GBps"] = round(B * 6 * L * 8 * N / dt / 1e9, 1)
        dt = timed(lambda: ctx.pointwise(binding.PW_MUL, ct1, ptw, pw_out), label="pointwise_mul")
        extra["pmult_per_s"] = round(B / dt, 1)
        extra["pmult_effective_GBps"] = round((B * 4 + 1) * L * 8 * N / dt / 1e9, 1)
        del pw_out, ptw
        del a13, b13, o13, rs_out

    if "standalone" in groups:
        # the coefficient-form entry points as calls of their own (one element-parallel kernel each), on the batch
        xin = ct1[:, 0].contiguous()                                  # [B][L][N]
        up_out = torch.empty((B, dnum, D, N), dtype=ct1.dtype, device=ct1.device)
        dt = timed(lambda: ctx.modup(xin, up_out), label="modup")
        extra["modup_per_s"] = round(B / dt, 1)
        extra["modup_effective_GBps"] = round(B * (L + dnum * D) * 8 * N / dt / 1e9, 1)   # L limbs read, dnum*(L+K) written
        yin = up_out[:, :2].contiguous().reshape(B * 2, D, N)          # any residues below the primes will do
        dn_out = torch.empty((B * 2, L, N), dtype=ct1.dtype, device=ct1.device)
        dt = timed(lambda: ctx.moddown(yin, dn_out), label="moddown")
        extra["moddown_per_s"] = round(B * 2 / dt, 1)
        extra["moddown_effective_GBps"] = round(B * 2 * (D + L) * 8 * N / dt / 1e9, 1)
        am_out = torch.empty_like(ct1)
        for name, ev in (("automorph_eval", True), ("automorph_coeff", False)):
            dt = timed(lambda: ctx.automorph(ct1, g, ev, 0, am_out), label=name)
            extra[name + "_limbs_per_s"] = round(B * 2 * L / dt, 1)
            extra[name + "_effective_GBps"] = round(B * 2 * L * 2 * 8 * N / dt / 1e9, 1)
        del xin, up_out, yin, dn_out, am_out

    cpu = None
    if not args.no_cpu:
        import oracle
        P = oracle.Params.from_set(ps)
        h1, h2 = ct1[0].cpu().numpy().view(np.uint64), ct2[0].cpu().numpy().view(np.uint64)
        hk = evk.cpu().numpy().view(np.uint64)
        hr = rk.cpu().numpy().view(np.uint64)
        n_each = 0
        a = time.perf_counter()
        while n_each < 2 or time.perf_counter() - a < 10.0:  # about 10 s of CPU work, at least two of each
            oracle.hmult_relin(h1, h2, hk, P)
            oracle.hrot(h1, g, hr, P)
            n_each += 1
        dt = time.perf_counter() - a
        threads = oracle.threads()
        # the same pair once more on a single thread
        oracle.set_threads(1)
        a1 = time.perf_counter()
        oracle.hmult_relin(h1, h2, hk, P)
        oracle.hrot(h1, g, hr, P)
        dt1 = time.perf_counter() - a1
        oracle.set_threads(threads)
        cpu = {"value": round(2 * n_each / dt, 3), "unit": "key-switches/s", "cores": threads, "kind": "oracle",
               "sample": "%d HMult+relin and %d HRot of the same shape (1 ciphertext each, not the batch of 8), "
                         "OpenMP over limbs" % (n_each, n_each),
               "single_thread_value": round(2 / dt1, 3)}
        # the other workload shapes, a few seconds each (same oracle, all cores): transforms of workload 1, hoisted
        # rotations of workloads 3 and 4 (3 rotations each; the rate is per rotation), HMult of workload 0
        other = {}
        xs = h1[0][:16] if h1.shape[1] >= 16 else h1[0]
        a2 = time.perf_counter()
        oracle.ntt_batch(xs, P, 0)
        oracle.ntt_batch(xs, P, 0, inverse=True)
        other["ntt_limbs_per_s (workload 1 shape, %d limbs forward + inverse)" % xs.shape[0]] = round(2 * xs.shape[0] / (time.perf_counter() - a2), 1)
        gs3 = [synth.galois_element(r_, ps.logN) for r_ in synth.CFG3_ROTATIONS[:3]]
        a2 = time.perf_counter()
        oracle.hrot_hoisted_mac(h1, gs3, [hr, hk, hr], np.ascontiguousarray(h2[0][None].repeat(3, 0)), P)
        other["hoisted_rot_mac_per_s (workload 3 shape, 3 rotations)"] = round(3 / (time.perf_counter() - a2), 3)
        ps0 = synth.CFG0
        P0 = oracle.Params.from_set(ps0)
        r0 = synth.rng_for(0, 100)
        c0a = synth.uniform_residues(r0, ps0.q_primes, ps0.N, lead=(2,))
        c0b = synth.uniform_residues(r0, ps0.q_primes, ps0.N, lead=(2,))
        k0_ = synth.uniform_residues(r0, ps0.primes, ps0.N, lead=(ps0.dnum, 2))
        a2 = time.perf_counter()
        for _ in range(20):
            oracle.hmult_relin(c0a, c0b, k0_, P0)
        other["hmult_relin_per_s (workload 0 shape, N=2^12)"] = round(20 / (time.perf_counter() - a2), 1)
        ps4 = synth.CFG4
        P4 = oracle.Params.from_set(ps4)
        r4 = synth.rng_for(4, 101)
        c4 = synth.uniform_residues(r4, ps4.q_primes, ps4.N, lead=(2,))
        k4 = synth.uniform_residues(r4, ps4.primes, ps4.N, lead=(ps4.dnum, 2))
        p4 = synth.uniform_residues(r4, ps4.q_primes, ps4.N, lead=(2,))
        gs4_ = [synth.galois_element(r_, ps4.logN) for r_ in synth.CFG4_ROTATIONS[:2]]
        a2 = time.perf_counter()
        oracle.hrot_hoisted_mac(c4, gs4_, [k4, k4], p4, P4)
        other["hoisted_rot_mac_per_s (workload 4 shape, 2 rotations)"] = round(2 / (time.perf_counter() - a2), 3)
        cpu["other_workloads"] = other

    line = {
        "metric": "key-switches/sec (HMult+relin, HRot) at N=2^16,L=24",
        "value": round(value, 1),
        "unit": "key-switches/s",
        "n_gpus": 1,
        "steps": args.steps,
        "warmup": args.warmup,
        "ms_per_step": round(ms_per_step, 4),
        "ms_per_step_median": round(ms_median, 4),
        "startup_steps": STARTUP,
        "higher_is_better": True,
        "scaling": "weak",
        "vs_baseline": None,
        "dtype": "u64",
        "data": "synthetic",
        "config": {"workload": "configs[2] shape: N=2^16, L=24 fifty-bit limbs, K=6 sixty-bit special limbs, dnum=4; "
                               "one step = batch of 8 HMult+relin + batch of 8 HRot (16 key switches)",
                   "batch": B, "key_switches_per_step": ks_per_step, "overlap": overlap},
        "roofline": roofline,
        "step_roofline": step_roofline,
        "cpu_baseline": cpu,
        "kernels": kernels,
        "extra": extra,
        "extra_kernels": extra_kernels,
    }
    print(json.dumps(line))


if __name__ == "__main__":
    main()
