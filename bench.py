#!/usr/bin/env python3
"""Benchmark of the RNS-CKKS key-switch hot path on one MI355X.

One "step" is one pass of the whole path over one batch of synthetic input at N=2^16, L=24, K=6,
dnum=4 (BASELINE config 2's shape): a batch of 8 HMult+relinearisations (shared evaluation key)
followed by a batch of 8 rotations (shared Galois key) -- 16 key switches.  `value` is key
switches per second with every operand resident in HBM.  Extras report the other quantities the
metric names: NTT limbs/s on config 1 (16 x 24 limbs) and hoisted rotations/s on config 3.

The line also carries
  roofline     : the kernel with the largest share of the timed region, its algorithmic bytes per
                 launch over its mean launch duration (HIP events recorded by the library on the
                 launch stream, in a second pass of the same K steps) against 8 TB/s;
  cpu_baseline : the CPU oracle, as it stands, on a bounded sample of the same workload.
"""
import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0

# HBM bytes per launch (read + written) from rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE for the default workload,
# taken from profiles/keyswitch_step_n16_l24_d4_hbm_traffic.txt (FETCH_SIZE scaled by 2, the factor a plain
# copy of known size shows); None for kernels or workloads that were not measured.
_MIB = 1 << 20
MEASURED_TRAFFIC_BYTES = {
    "conv_fwd_strided_kernel<FpAr, 8, 1, 1>": int((97.5 + 288.0) * _MIB),
    "conv_fwd_strided_kernel<FpAr, 8, 2, 3>": int((78.1 + 194.0) * _MIB),
    "conv_fwd_strided_kernel<IntAr, 8, 1, 1>": int((156.0 + 96.0) * _MIB),
    "inv_contig_kernel<FpAr, 8, 1>": int((204.1 + 96.0) * _MIB),
    "inv_contig_kernel<FpAr, 8, 2>": int((108.1 + 96.0) * _MIB),
    "inv_strided_kernel<FpAr, 8>": int((96.6 + 96.0) * _MIB),
    "inv_strided_kernel<IntAr, 8>": int((48.5 + 48.0) * _MIB),
    "ks_final_kernel<FpAr, 8, 1>": int((984.7 + 192.0) * _MIB),
    "ks_final_kernel<FpAr, 8, 2>": int((504.3 + 192.0) * _MIB),
    "ks_inner_kernel<FpAr, 8, 1, false>": int((594.9 + 192.0) * _MIB),
    "ks_inner_kernel<FpAr, 8, 2, false>": int((497.5 + 192.0) * _MIB),
    "ks_inner_kernel<IntAr, 8, 1, false>": int((133.3 + 48.0) * _MIB),
    "ks_inner_kernel<IntAr, 8, 2, false>": int((133.5 + 48.0) * _MIB),
}


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=20)
    ap.add_argument("--warmup", type=int, default=3)
    ap.add_argument("--no-extras", action="store_true", help="skip the NTT and hoisted-rotation extras")
    ap.add_argument("--no-cpu", action="store_true", help="skip the CPU oracle baseline")
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

    for _ in range(args.warmup):
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

    # ---- per-kernel pass: the same K steps with HIP events around every launch
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
            kernels[name] = {"launches_per_step": n / args.steps, "avg_us": 1e3 * ms / n,
                             "share": ms / total_ms, "alg_GBps": nbytes / ms / 1e6}
    dom = max(prof.items(), key=lambda kv: kv[1][1])
    dname, (dn, dms, dbytes) = dom
    achieved = dbytes / dms / 1e6  # GB/s
    traffic = MEASURED_TRAFFIC_BYTES.get(dname) if (args.steps and B == synth.CFG2_BATCH) else None
    roofline = {"bound": "hbm", "kernel": dname, "achieved": round(achieved, 1), "peak": HBM_PEAK_GBS,
                "unit": "GB/s", "frac": round(achieved / HBM_PEAK_GBS, 4), "traffic": traffic,
                "alg_bytes_per_launch": dbytes // dn, "avg_launch_us": round(1e3 * dms / dn, 2),
                "share_of_step": round(dms / total_ms, 3)}

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

    if not args.no_extras:
        # config 1: 16 polynomials x 24 limbs, forward and inverse
        x = dev(synth.uniform_residues(rng, ps.q_primes, N, lead=(synth.CFG1_BATCH,)))
        limbs = synth.CFG1_BATCH * L
        for name, inv in (("ntt_fwd_limbs_per_s", False), ("ntt_inv_limbs_per_s", True)):
            for _ in range(2):
                ctx.ntt(x, 0, inverse=inv)
            torch.cuda.synchronize()
            a = time.perf_counter()
            for _ in range(args.steps):
                ctx.ntt(x, 0, inverse=inv)
            torch.cuda.synchronize()
            dt = (time.perf_counter() - a) / args.steps
            extra[name] = round(limbs / dt, 1)
            # one transform reads and writes every limb once: 2 * 8N bytes per limb (compulsory)
            extra[name.replace("limbs_per_s", "effective_GBps")] = round(limbs * 2 * 8 * N / dt / 1e9, 1)
        del x
        # config 3: 17 hoisted rotations with plaintext MAC (keys are rolled copies of one uniform key)
        rots = synth.CFG3_ROTATIONS
        gs = [synth.galois_element(r, ps.logN) for r in rots]
        rks = [torch.roll(rk, shifts=i + 1, dims=-1).contiguous() for i in range(len(rots))]
        pt = torch.stack([torch.roll(ct1[0, 0], shifts=i, dims=-1) for i in range(len(rots))]).contiguous()
        ct = ct1[0].contiguous()
        o = torch.empty_like(ct)
        ctx.hrot_hoisted_mac(ct, gs, rks, pt, o)
        torch.cuda.synchronize()
        a = time.perf_counter()
        reps = max(1, args.steps // 4)
        for _ in range(reps):
            ctx.hrot_hoisted_mac(ct, gs, rks, pt, o)
        torch.cuda.synchronize()
        extra["hoisted_rot_mac_per_s"] = round(len(rots) * reps / (time.perf_counter() - a), 1)
        del rks, pt

    cpu = None
    if not args.no_cpu:
        import oracle
        P = oracle.Params.from_set(ps)
        h1, h2 = ct1[0].cpu().numpy().view(np.uint64), ct2[0].cpu().numpy().view(np.uint64)
        hk = evk.cpu().numpy().view(np.uint64)
        hr = rk.cpu().numpy().view(np.uint64)
        n_each = 2
        a = time.perf_counter()
        for _ in range(n_each):
            oracle.hmult_relin(h1, h2, hk, P)
            oracle.hrot(h1, g, hr, P)
        dt = time.perf_counter() - a
        threads = int(os.environ.get("OMP_NUM_THREADS", os.cpu_count() or 1))
        cpu = {"value": round(2 * n_each / dt, 3), "unit": "key-switches/s", "cores": threads, "kind": "oracle",
               "sample": "%d HMult+relin and %d HRot of the same shape (1 ciphertext each, not the batch of 8), "
                         "OpenMP over limbs" % (n_each, n_each)}

    line = {
        "metric": "key-switches/sec (HMult+relin, HRot) at N=2^16,L=24",
        "value": round(value, 1),
        "unit": "key-switches/s",
        "n_gpus": 1,
        "steps": args.steps,
        "warmup": args.warmup,
        "ms_per_step": round(ms_per_step, 4),
        "higher_is_better": True,
        "scaling": "weak",
        "vs_baseline": None,
        "dtype": "u64",
        "data": "synthetic",
        "config": {"workload": "configs[2] shape: N=2^16, L=24 fifty-bit limbs, K=6 sixty-bit special limbs, dnum=4; "
                               "one step = batch of 8 HMult+relin + batch of 8 HRot (16 key switches)",
                   "batch": B, "key_switches_per_step": ks_per_step},
        "roofline": roofline,
        "cpu_baseline": cpu,
        "kernels": kernels,
        "extra": extra,
    }
    print(json.dumps(line))


if __name__ == "__main__":
    main()
