#!/usr/bin/env python3
"""Benchmark of the RNS-CKKS hot path on one MI355X.

A step is one batch of 64 HMult + relinearise + rescale at N = 2^16, 24 x 50-bit
ciphertext primes + 3 special primes, 8 key-switch digits of 3 primes (the
polynomial-activation workload shape), inputs resident in HBM.  Prints ONE JSON line.
Ciphertexts and the switching key are uniform residues drawn on the device: RLWE
ciphertexts and keys are pseudorandom and no kernel branches on data, so the time is
that of real ones (the parity tests, not this script, use real encryptions).
"""
import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

HBM_PEAK_GBPS = 8000.0        # MI355X HBM3E
FP64_PEAK_LANEOPS = 39.3e12   # 256 CU x 64 lanes x 2.4 GHz, one FP64 instruction per lane per clock


def uniform_residues(torch, moduli, lead, N, gen):
    """int64 tensor [*lead][len(moduli)][N] on the GPU, limb i uniform on [0, moduli[i])"""
    out = torch.empty(tuple(lead) + (len(moduli), N), dtype=torch.int64, device="cuda:0")
    for i, q in enumerate(moduli):
        out[..., i, :] = torch.randint(0, q, tuple(lead) + (N,), dtype=torch.int64, device="cuda:0", generator=gen)
    return out


def bytes_per_unit(name, N, level, k, alpha, batch):
    """algorithmic HBM bytes per unit of work of each kernel class (unit = one limb unless noted)"""
    E, beta = level + k, -(-level // alpha)
    w = 8 * N
    table = {
        # a limb transform reads and writes its limb once (16N bytes); it is done in two
        # kernels here, each credited with half of that
        "ntt_fwd_kernel<true>": w, "ntt_fwd_kernel<false>": w, "ntt_inv_kernel<false>": w, "ntt_inv_kernel<true>": w,
        "ntt_v2_kernel<false, true>": w, "ntt_v2_kernel<false, false>": w, "ntt_v2_kernel<true, false>": w, "ntt_v2_kernel<true, true>": w,
        "tensor_kernel": 7 * w,                       # 4 limbs in, 3 out
        "modup_kernel": w * (1.0 / E * min(alpha, level) + 1),   # per output limb: its share of the digit's source limbs + itself
        "inner_product_kernel": w * (beta + 2 + 2.0 * beta / batch),  # beta inputs, 2 outputs, key read once per batch
        "divround_conv_kernel": w * (1 + float(k) / level),
        "divround_final_kernel": 4 * w,               # x, tmp, addend in; out
        "automorphism_kernel": 2 * w,
        # fused kernels: the converted limb is written once (column-pass output) plus its share of the source limbs
        "conv_cols_kernel(ModUp)": w * (1 + float(level) / (beta * E - level)),
        "conv_cols_kernel(DivRound)": w * (1 + float(k) / level),
        "rows_inner_kernel": w * (beta + 2 + 2.0 * beta / batch),   # beta limbs in, 2 out, key once per batch
        "rows_final_kernel": 4 * w,                                  # column-pass output, x, addend in; out
        "elementwise kernels": 3 * w,
    }
    return table.get(name)


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=5)
    ap.add_argument("--warmup", type=int, default=2)
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-sweep", action="store_true", help="skip the plain transform sweep (keeps a profile to the timed steps)")
    ap.add_argument("--copy-probe", action="store_true",
                    help="also run one plain device copy of the input batch (known size) so that profiler byte counters can be scaled")
    args = ap.parse_args()
    if args.gpus != 1:
        sys.exit("bench.py: this build runs on ONE GPU; --gpus %d is not supported (every ciphertext is independent, "
                 "so the batch would simply be split across GPUs)" % args.gpus)

    import numpy as np
    import torch

    from paper_1911_11377_amd import ckksmi
    from paper_1911_11377_amd import workloads as wl

    if not torch.cuda.is_available():
        sys.exit("bench.py needs a GPU")
    p = wl.PRESETS["act_2e16"]
    level, batch, N = p.n_q, p.batch, p.N
    ctx = ckksmi.Context(p.logN, p.n_q, p.q_bits, p.k, p.special_bits, p.alpha, device=0)
    gen = torch.Generator(device="cuda:0")
    gen.manual_seed(wl.BASE_SEED + 4)
    a = uniform_residues(torch, ctx.q[:level], (batch, 2), N, gen)
    b = uniform_residues(torch, ctx.q[:level], (batch, 2), N, gen)
    evk = uniform_residues(torch, ctx.moduli, (ctx.beta_top, 2), N, gen)
    out = torch.empty((batch, 2, level - 1, N), dtype=torch.int64, device="cuda:0")
    ws = torch.empty(ctx.workspace_bytes(ckksmi.OP_HMUL_RELIN_RESCALE, level, batch) // 8, dtype=torch.int64, device="cuda:0")

    def step():
        ctx.hmul_relin_rescale(a, b, evk, out, level, batch, ws)

    for _ in range(args.warmup):
        step()
    torch.cuda.synchronize()
    ctx.profile_enable(True)
    t0 = time.perf_counter()
    for _ in range(args.steps):
        step()
    torch.cuda.synchronize()
    t1 = time.perf_counter()
    prof = ctx.profile_read()
    ctx.profile_enable(False)
    ms_per_step = (t1 - t0) * 1e3 / args.steps
    value = batch * args.steps / (t1 - t0)

    # ---- roofline of the dominant kernel (largest share of the timed region)
    kernels = {}
    for name, (ms, launches, units) in prof.items():
        bpu = bytes_per_unit(name, N, level, p.k, p.alpha, batch)
        kernels[name] = {"ms_total": round(ms, 3), "launches": launches, "avg_ms": round(ms / launches, 4),
                         "GBps": round(bpu * units / (ms * 1e-3) / 1e9, 1) if bpu else None}
    dom = max(prof, key=lambda n: prof[n][0])
    ms, launches, units = prof[dom]
    bpu = bytes_per_unit(dom, N, level, p.k, p.alpha, batch)
    achieved = bpu * units / (ms * 1e-3) / 1e9
    ntt_ms = sum(prof[n][0] for n in prof if n.startswith("ntt_"))
    ntt_limbs = sum(prof[n][2] for n in prof if n in ("ntt_fwd_kernel<false>", "ntt_inv_kernel<false>", "ntt_v2_kernel<false, false>", "ntt_v2_kernel<true, false>"))
    roofline = {"kernel": dom, "bound": "hbm", "achieved": round(achieved, 1), "peak": HBM_PEAK_GBPS, "unit": "GB/s",
                "frac": round(achieved / HBM_PEAK_GBPS, 4), "traffic": None,
                "avg_launch_ms": round(ms / launches, 4), "bytes_per_launch": bpu * units / launches,
                "all_transforms_GBps": round(16 * N * ntt_limbs / (ntt_ms * 1e-3) / 1e9, 1),
                "kernels": kernels}

    if args.copy_probe:
        probe = torch.empty_like(a)
        probe.copy_(a)  # reads and writes a.numel()*8 bytes
        torch.cuda.synchronize()
        del probe

    # ---- plain transform sweep: batch x 2 x (level + k) limbs, forward then inverse, in place
    idx = list(range(level)) + [p.n_q + m for m in range(p.k)]
    limbs = uniform_residues(torch, [ctx.moduli[t] for t in idx], (batch * 2,), N, gen)
    ntt = {}
    for name, fn in (() if args.no_sweep else (("fwd", ctx.ntt), ("inv", ctx.intt))):
        fn(limbs, idx, batch * 2)
        torch.cuda.synchronize()
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record()
        for _ in range(3):
            fn(limbs, idx, batch * 2)
        e1.record()
        torch.cuda.synchronize()
        gbps = 16.0 * N * len(idx) * batch * 2 * 3 / (e0.elapsed_time(e1) * 1e-3) / 1e9
        ntt[name] = {"GBps": round(gbps, 1), "frac_of_hbm_peak": round(gbps / HBM_PEAK_GBPS, 4)}
    del limbs

    # ---- the oracle on the host cores, on a bounded sample of the same workload
    cpu = None
    if not args.no_cpu_baseline:
        from concurrent.futures import ThreadPoolExecutor

        from oracle import oracle as orc

        cores = min(os.cpu_count() or 1, 16, batch)
        O = orc.Oracle(p.logN, p.n_q, p.q_bits, p.k, p.special_bits, p.alpha)
        assert O.moduli == ctx.moduli and O.psis == ctx.psis
        ha = a[:cores].cpu().numpy().view(np.uint64)
        hb = b[:cores].cpu().numpy().view(np.uint64)
        hk = evk.cpu().numpy().view(np.uint64)
        c0 = time.perf_counter()
        with ThreadPoolExecutor(cores) as ex:  # the C calls release the GIL
            res = list(ex.map(lambda i: O.hmul_relin_rescale(ha[i], hb[i], hk, level), range(cores)))
        c1 = time.perf_counter()
        got = out[:cores].cpu().numpy().view(np.uint64)
        match = all(np.array_equal(res[i], got[i]) for i in range(cores))
        cpu = {"value": round(cores / (c1 - c0), 4), "unit": "ops/s", "cores": cores, "kind": "oracle",
               "sample": "%d of the %d HMult+relin+rescale of one step, one per thread, same inputs" % (cores, batch),
               "matches_gpu_bits": bool(match)}

    line = {
        "metric": "HMult+relin+rescale ops/s at N=2^16", "value": round(value, 2), "unit": "ops/s", "n_gpus": 1,
        "steps": args.steps, "warmup": args.warmup, "ms_per_step": round(ms_per_step, 3), "higher_is_better": True,
        "scaling": "weak", "vs_baseline": None, "dtype": "f64", "data": "synthetic",
        "config": {"workload": "act_2e16: N=2^16, 24x50-bit primes + 3x51-bit special primes, 8 digits of 3, batch 64, level 24",
                   "op": "tensor -> key switch (ModUp, inner product, ModDown) -> add -> rescale"},
        "roofline": roofline, "ntt_sweep": ntt, "cpu_baseline": cpu,
    }
    print(json.dumps(line))


if __name__ == "__main__":
    main()
