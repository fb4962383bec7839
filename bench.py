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
INT8_PEAK_OPS = 5.0e15        # dense int8 MFMA
FP64_PEAK_LANEOPS = 39.3e12   # 256 CU x 64 lanes x 2.4 GHz, one FP64 instruction per lane per clock
COUNTERS_FILE = os.path.join(ROOT, "profiles", "counters_act_2e16.json")


def load_counters():
    """per-kernel hardware counters of the default workload (one launch each, batch 64, level 24), collected with
    rocprofv3 --pmc on this build and summarised in profiles/; None when the file is missing"""
    try:
        with open(COUNTERS_FILE) as f:
            return json.load(f)
    except (OSError, ValueError):
        return None


def counter_figures(C, name):
    """HBM traffic per launch (FETCH_SIZE and WRITE_SIZE in KiB, each scaled by what the same counter reads for a plain
    device copy of known size in the same profile), counted vector instructions per launch and the fraction of issue
    cycles the vector ALU was busy, for one kernel of the counters file"""
    if not C or name not in C.get("kernels", {}):
        return None
    k, probe = C["kernels"][name], C["copy_probe"]
    out = {}
    if "FETCH_SIZE" in k and "WRITE_SIZE" in k:
        ff = probe["bytes"] / (probe["FETCH_SIZE"] * 1024.0)
        wf = probe["bytes"] / (probe["WRITE_SIZE"] * 1024.0)
        out["traffic"] = ff * k["FETCH_SIZE"] * 1024.0 + wf * k["WRITE_SIZE"] * 1024.0
    if "SQ_INSTS_VALU" in k:
        out["valu_wave_instr"] = k["SQ_INSTS_VALU"]
    if "SQ_ACTIVE_INST_VALU" in k and "SQ_BUSY_CYCLES" in k:
        # SQ_ACTIVE_INST_VALU counts 4-cycle slots over all 1024 SIMDs, SQ_BUSY_CYCLES cycles summed over the 32 shader engines
        out["valu_busy"] = k["SQ_ACTIVE_INST_VALU"] * 4.0 / (k["SQ_BUSY_CYCLES"] / 32.0 * 1024.0)
    if "SQ_LDS_BANK_CONFLICT" in k and "SQ_ACTIVE_INST_LDS" in k:
        out["lds_conflict_frac"] = k["SQ_LDS_BANK_CONFLICT"] / max(k["SQ_ACTIVE_INST_LDS"], 1.0)
    if "TCC_HIT_sum" in k and "TCC_MISS_sum" in k:
        out["l2_hit_rate"] = k["TCC_HIT_sum"] / max(k["TCC_HIT_sum"] + k["TCC_MISS_sum"], 1.0)
    return out


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
        "tensor_rows_kernel": 3 * w,                  # the operands' second components in, the inverse row pass of a1*b1 out
        "modup_kernel": w * (1.0 / E * min(alpha, level) + 1),   # per output limb: its share of the digit's source limbs + itself
        "inner_product_kernel": w * (beta + 2 + 2.0 * beta / batch),  # beta inputs, 2 outputs, key read once per batch
        "divround_conv_kernel": w * (1 + float(k) / level),
        "divround_final_kernel": 4 * w,               # x, tmp, addend in; out
        "automorphism_kernel": 2 * w,
        # fused kernels: the converted limb is written once (column-pass output) plus its share of the source limbs
        # the same conversions organised by source tile (targets looped in the workgroup)
        # (the inverse column pass of the sources runs in the kernel too; same bytes)
        "modup_cols_kernel<4, %d, 0>" % alpha: w * (1 + float(level) / (beta * E - level)),
        "modup_cols_kernel<4, %d, 1>" % k: w * (1 + float(k) / level),
        "modup_cols_kernel<4, 1, 1>": w * (1 + 1.0 / (level - 1)),
        # ModDown + rescale as one conversion / the merged division: k + 1 source limbs for level - 1 targets
        "modup_cols_kernel<4, %d, 3>" % (k + 1): w * (1 + float(k + 1) / max(level - 1, 1)),
        "modup_cols_kernel<4, %d, 2>" % (k + 1): w * (1 + float(k + 1) / max(level - 1, 1)),
        "axpy_limb_kernel": 3 * w,
        # beta limbs in, 2 out, key read once per batch; in the composite multiply a ciphertext limb reads the four operand
        # limbs instead of its own digit's word (d0, d1, d2 are formed here, and with them z = x*P^-1 + d)
        "rows_inner_kernel": w * (beta + 2 + 2.0 * beta / batch + 3.0 * level / E),
        "rows_final_kernel": 3 * w,                                  # column-pass output and z in; out (4 with a separate addend)
        "elementwise kernels": 3 * w,
    }
    return table.get(name)


def laneops_per_unit(name, N, level, k, alpha):
    """FP64 vector instructions per unit of work (counted from the kernel source, per word: conversions u64<->f64 2 each,
    twiddle product 6, butterfly add/sub 2, reduction 3, canonical form 7) for the kernels where the ALU can bind"""
    beta = -(-level // alpha)
    # one pass of a transform between the reduced-double intermediate formats: 8 stages at 4 per word (twiddle product
    # 5 + add + sub per butterfly, lazy reductions included), one mid reduction, one reduction at the store
    xform_pass = 8 * 4 + 3 + 3
    table = {
        # source words converted to doubles once per workgroup, not once per target
        # (the inverse column pass of the source tiles, once per workgroup, adds about 5 %: not counted)
        "modup_cols_kernel<4, %d, 0>" % alpha: N * (5 * alpha + (alpha - 1) + 3 + xform_pass),
        "modup_cols_kernel<4, %d, 1>" % k: N * (5 * k + k + 3 + xform_pass),
        "modup_cols_kernel<4, 1, 1>": N * (5 + 1 + 3 + xform_pass),
        "modup_cols_kernel<4, %d, 3>" % (k + 1): N * (5 * k + k + 3 + 5 + 2 + 3 + xform_pass),
        "modup_cols_kernel<4, %d, 2>" % (k + 1): N * (5 * (k + 1) + (k + 1) + 6 + 3 + xform_pass),
        # per word: a row pass for every digit except the limb's own one (level of the E limbs have one), two
        # multiply-accumulates per digit (key word conversion 2 + exact product 5 + add 1, the prepared quotient and the
        # lazy reductions shared: about 2 more per digit), canonical form of the two results
        "rows_inner_kernel": N * ((beta - float(level) / (level + k)) * xform_pass + beta * (2 * 8 + 2) + 2 * 7
                                  + 2 * (5 + 3) * float(level) / (level + k)),
        "rows_final_kernel": N * (xform_pass + 2 + 1 + 5 + 3 + 7 + 2),   # (+5 when the kept limb is scaled before the subtraction)
    }
    return table.get(name)


def timed(torch, fn, reps):
    fn()
    torch.cuda.synchronize()
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    e0.record()
    for _ in range(reps):
        fn()
    e1.record()
    torch.cuda.synchronize()
    return e0.elapsed_time(e1) / reps


def conv_layer_workload(torch, ckksmi, wl, gen):
    """conv layer, slots-as-batch: N = 2^15, 16x50-bit, 3x32x32 pixel ciphertexts (16384 images), 3 -> 32 channels 5x5
    stride 2 (multiply-accumulate on the matrix cores), then the rescale of the 6272 output ciphertexts"""
    out = {}
    p3 = wl.PRESETS["conv_2e15"]
    c3 = ckksmi.Context(p3.logN, p3.n_q, p3.q_bits, p3.k, p3.special_bits, p3.alpha, device=0)
    L, N = p3.n_q, p3.N
    Cin, H, W, O, kh, stride = 3, 32, 32, 32, 5, 2
    Ho = (H - kh) // stride + 1
    xin = uniform_residues(torch, c3.q, (Cin * H * W, 2), N, gen)
    wts = torch.from_numpy(__import__("numpy").rint(wl.weights_float((O, Cin, kh, kh), 3) * c3.q[L - 1]).astype("int64")).to("cuda:0")
    co = torch.empty((O * Ho * Ho, 2, L, N), dtype=torch.int64, device="cuda:0")
    cr = torch.empty((O * Ho * Ho, 2, L - 1, N), dtype=torch.int64, device="cuda:0")
    wm = torch.empty(c3.conv2d_workspace_bytes(Cin, O, kh, kh, L) // 8 + 1, dtype=torch.int64, device="cuda:0")
    wr = torch.empty(c3.workspace_bytes(ckksmi.OP_RESCALE, L, 256) // 8, dtype=torch.int64, device="cuda:0")
    ms_mac = timed(torch, lambda: c3.conv2d_mac(xin, wts, Cin, H, W, O, kh, kh, stride, 0, co, L, wm), 1)
    ms_rs = timed(torch, lambda: c3.rescale(co, cr, L, O * Ho * Ho, wr), 1)
    mac_count = float(O) * Ho * Ho * Cin * kh * kh * 2 * L * N
    out["conv_layer_2e15"] = {"encrypted_images_per_s": round((N // 2) / ((ms_mac + ms_rs) * 1e-3), 1), "ms_mac": round(ms_mac, 2),
                              "ms_rescale": round(ms_rs, 2), "word_macs_per_s": round(mac_count / (ms_mac * 1e-3), 0),
                              # matrix cores: 49 int8 multiply-accumulates (7 x 7 base-256 digits) per word MAC, 2 ops each, against
                              # the 5.0 POP/s dense int8 peak; only the layer's real taps are counted, not the padding to 64
                              "mfma_frac": round(mac_count * 49 * 2 / (ms_mac * 1e-3) / INT8_PEAK_OPS, 4),
                              "what": "3x32x32 pixel ciphertexts -> 32x14x14, 5x5 stride 2, ptxt x ct MAC + rescale, 16384 images per pass"}
    del xin, co, cr, wm, wr
    c3.close()
    return out


def secondary_workloads(torch, ckksmi, wl, ctx, a, evk, ws, gen):
    """the other rows of the hot path, each timed on its own workload shape (uniform residues, resident in HBM)"""
    from paper_1911_11377_amd import activation

    out = {}
    # polynomial activation on the main shape: x^2 then 0.5 + 0.25y - 0.02y^3, 64 ciphertexts from level 24 to 21
    p4 = wl.PRESETS["act_2e16"]
    L, B, N = p4.n_q, p4.batch, p4.N
    s = 2.0 ** p4.log_scale
    consts = activation.poly3_constants(ctx.q, L - 1, s * s / ctx.q[L - 1])
    y = torch.empty((B, 2, L - 1, N), dtype=torch.int64, device="cuda:0")
    o3 = torch.empty((B, 2, L - 3, N), dtype=torch.int64, device="cuda:0")
    wsa = torch.empty(activation.workspace_bytes(ctx, L, B) // 8, dtype=torch.int64, device="cuda:0")

    def act():
        activation.square(ctx, a, evk, y, L, B, wsa)
        activation.poly3(ctx, y, evk, o3, L - 1, B, consts, wsa)

    ms = timed(torch, act, 2)
    out["activation_2e16"] = {"ciphertexts_per_s": round(B / (ms * 1e-3), 1), "ms": round(ms, 2),
                              "what": "square then degree-3 polynomial, 3 HMult+relin+rescale + 2 scalar rescales per ciphertext, level 24 -> 21"}
    del y, o3, wsa

    # rotation on the main shape: automorphism + key switch with one Galois key (the evaluation key's buffer stands in:
    # uniform residues of the same shape), batch 64 at level 24
    ctx.galois_key_register(1, evk)
    orot = torch.empty((B, 2, L, N), dtype=torch.int64, device="cuda:0")
    wrot = torch.empty(ctx.workspace_bytes(ckksmi.OP_ROTATE, L, B) // 8, dtype=torch.int64, device="cuda:0")
    ms = timed(torch, lambda: ctx.rotate(a, [1] * B, orot, L, B, wrot), 5)
    out["rotate_2e16"] = {"ops_per_s": round(B / (ms * 1e-3), 1), "ms": round(ms, 3),
                          "what": "HRot by one slot, batch 64, level 24 (ModUp, inner product, ModDown: no tensor, no rescale)"}
    del orot, wrot

    # the same product with one division by P*q_last instead of ModDown followed by rescale (different output bits:
    # a separate operation, not the headline one)
    om = torch.empty((B, 2, L - 1, N), dtype=torch.int64, device="cuda:0")
    ms = timed(torch, lambda: ctx.hmul_relin_rescale_merged(a, a, evk, om, L, B, ws), 5)
    out["merged_division_2e16"] = {"ops_per_s": round(B / (ms * 1e-3), 1), "ms": round(ms, 3),
                                   "what": "HMult + key switch + ONE exact division by P*q_last, batch 64, level 24 -> 23"}
    del om
    # fresh ciphertexts made on the device: encode (complex inverse transform) + encrypt with resident randomness
    z_re = torch.rand((B, N // 2), dtype=torch.float64, device="cuda:0", generator=gen) * 2 - 1
    small = [torch.empty((B, N), dtype=torch.int64, device="cuda:0") for _ in range(3)]
    pk = uniform_residues(torch, ctx.q, (2,), N, gen)
    ptd = torch.empty((B, L, N), dtype=torch.int64, device="cuda:0")
    ctd = torch.empty((B, 2, L, N), dtype=torch.int64, device="cuda:0")

    def fresh():
        ctx.sample_device(0, 3.2, 4, 0, B, small[0])
        ctx.sample_device(1, 3.2, 4, B, B, small[1])
        ctx.sample_device(1, 3.2, 4, 2 * B, B, small[2])
        ctx.encode_device(z_re, None, s, L, B, ptd, ws)
        ctx.encrypt_device(pk, ptd, small[0], small[1], small[2], L, B, ctd, ws)

    ms = timed(torch, fresh, 3)
    out["encode_encrypt_device_2e16"] = {"ciphertexts_per_s": round(B / (ms * 1e-3), 1), "ms": round(ms, 3),
                                         "what": "sample (ternary r, Gaussian e0, e1) + encode + encrypt on the device, batch 64, 24 limbs"}
    del z_re, small, pk, ptd, ctd
    # a sum of 4 products relinearised and rescaled once (lazy relinearisation; the same ciphertexts serve as every term)
    terms = 4
    at = a.unsqueeze(1).expand(B, terms, 2, L, N).contiguous()
    os_ = torch.empty((B, 2, L - 1, N), dtype=torch.int64, device="cuda:0")
    ms = timed(torch, lambda: ctx.hmul_sum_relin_rescale(at, at, terms, evk, os_, L, B, ws), 3)
    out["sum_of_4_products_2e16"] = {"sums_per_s": round(B / (ms * 1e-3), 1), "products_per_s": round(B * terms / (ms * 1e-3), 1), "ms": round(ms, 3),
                                     "what": "sum of 4 HMult tensors, ONE key switch and rescale, batch 64, level 24 -> 23"}
    del at, os_

    # the tiny shape (N = 2^12, 3x40-bit + special prime, batch 16): launch-bound, so also as one captured graph
    p1 = wl.PRESETS["tiny"]
    c1 = ckksmi.Context(p1.logN, p1.n_q, p1.q_bits, p1.k, p1.special_bits, p1.alpha, device=0)
    a1 = uniform_residues(torch, c1.q, (p1.batch, 2), p1.N, gen)
    k1 = uniform_residues(torch, c1.moduli, (c1.beta_top, 2), p1.N, gen)
    o1 = torch.empty((p1.batch, 2, p1.n_q - 1, p1.N), dtype=torch.int64, device="cuda:0")
    w1 = torch.empty(c1.workspace_bytes(ckksmi.OP_HMUL_RELIN_RESCALE, p1.n_q, p1.batch) // 8, dtype=torch.int64, device="cuda:0")
    step1 = lambda: c1.hmul_relin_rescale(a1, a1, k1, o1, p1.n_q, p1.batch, w1)
    ms_eager = timed(torch, step1, 50)
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):
        step1()
    side.synchronize()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph, stream=side):
        for _ in range(10):
            step1()
    ms_graph = timed(torch, graph.replay, 5) / 10
    out["hmul_relin_rescale_2e12"] = {"ops_per_s": round(p1.batch / (ms_eager * 1e-3), 1), "ms": round(ms_eager, 4),
                                      "ops_per_s_graph": round(p1.batch / (ms_graph * 1e-3), 1), "ms_graph": round(ms_graph, 4),
                                      "what": "tiny shape, batch 16, level 3; the second figure replays ten steps captured in one graph"}
    del a1, k1, o1, w1, graph
    c1.close()

    # N = 2^14, 8x50-bit + special prime: batch 256, HMult+relin+rescale and rotations by 8 random offsets
    p2 = wl.PRESETS["hmul_rot_2e14"]
    c2 = ckksmi.Context(p2.logN, p2.n_q, p2.q_bits, p2.k, p2.special_bits, p2.alpha, device=0)
    L, B, N = p2.n_q, p2.batch, p2.N
    a2 = uniform_residues(torch, c2.q, (B, 2), N, gen)
    b2 = uniform_residues(torch, c2.q, (B, 2), N, gen)
    k2 = uniform_residues(torch, c2.moduli, (c2.beta_top, 2), N, gen)
    rots = wl.rotation_offsets(N // 2, 8, 2)
    gks = [uniform_residues(torch, c2.moduli, (c2.beta_top, 2), N, gen) for _ in rots]
    for r, g in zip(rots, gks):
        c2.galois_key_register(r, g)
    pick = wl.rng(2, "rot.pick").integers(0, len(rots), size=B)
    rot = [rots[j] for j in pick]
    o2 = torch.empty((B, 2, L - 1, N), dtype=torch.int64, device="cuda:0")
    or2 = torch.empty((B, 2, L, N), dtype=torch.int64, device="cuda:0")
    w2 = torch.empty(max(c2.workspace_bytes(ckksmi.OP_HMUL_RELIN_RESCALE, L, B), c2.workspace_bytes(ckksmi.OP_ROTATE, L, B)) // 8,
                     dtype=torch.int64, device="cuda:0")
    ms = timed(torch, lambda: c2.hmul_relin_rescale(a2, b2, k2, o2, L, B, w2), 3)
    out["hmul_relin_rescale_2e14"] = {"ops_per_s": round(B / (ms * 1e-3), 1), "ms": round(ms, 3)}
    ms = timed(torch, lambda: c2.rotate(a2, rot, or2, L, B, w2), 3)
    out["rotate_2e14"] = {"ops_per_s": round(B / (ms * 1e-3), 1), "ms": round(ms, 3), "keys": len(rots)}
    # the same number of rotations as ALL 8 offsets of B/8 ciphertexts each, from one shared ModUp per ciphertext (hoisting;
    # a separate operation with its own output bits)
    Bh = B // len(rots)
    oh = torch.empty((Bh, len(rots), 2, L, N), dtype=torch.int64, device="cuda:0")
    wh = torch.empty(c2.rotate_hoisted_workspace_bytes(L, Bh, len(rots)) // 8, dtype=torch.int64, device="cuda:0")
    ms = timed(torch, lambda: c2.rotate_hoisted(a2, rots, oh, L, Bh, wh), 3)
    out["rotate_hoisted_2e14"] = {"ops_per_s": round(Bh * len(rots) / (ms * 1e-3), 1), "ms": round(ms, 3),
                                  "what": "%d ciphertexts x %d rotations each, one ModUp per ciphertext" % (Bh, len(rots))}
    # one image, rotation-packed: a dense 64x64 layer on ONE ciphertext (63 hoisted rotations, plaintext diagonals, rescale)
    import numpy as np
    from paper_1911_11377_amd import packed
    Wd = wl.weights_float((64, 64), 2, "packed.fc")
    lay_keys = {}
    for d in range(1, 64):
        if d not in rots:
            lay_keys[d] = uniform_residues(torch, c2.moduli, (c2.beta_top, 2), N, gen)
            c2.galois_key_register(d, lay_keys[d])
    to_dev = lambda arr: torch.from_numpy(np.ascontiguousarray(arr).view(np.int64)).to("cuda:0")
    plan = packed.plan_linear(c2, Wd, L, to_dev)
    wp = torch.empty(packed.workspace_bytes(c2, plan) // 8, dtype=torch.int64, device="cuda:0")
    op = torch.empty((2, L - 1, N), dtype=torch.int64, device="cuda:0")
    ms = timed(torch, lambda: packed.linear_transform(c2, a2[0], plan, op, wp), 3)
    out["packed_fc64_2e14"] = {"ms_per_layer": round(ms, 3), "what": "64x64 dense layer on one ciphertext: 63 rotations from one ModUp, level 8 -> 7"}
    # the same layer with baby and giant steps (8 x 8): 7 hoisted rotations, 7 rotations of the inner sums (offsets 1..7 and 8, 16, .. 56 are registered)
    plan_b = packed.plan_bsgs(c2, Wd, 64, L, to_dev)
    wpb = torch.empty(packed.bsgs_workspace_bytes(c2, plan_b) // 8 + 1, dtype=torch.int64, device="cuda:0")
    ms = timed(torch, lambda: packed.linear_transform_bsgs(c2, a2[0], plan_b, op, wpb), 3)
    out["packed_fc64_bsgs_2e14"] = {"ms_per_layer": round(ms, 3), "rotation_offsets": len(plan_b.rotation_offsets()),
                                    "what": "the same layer, baby and giant steps of 8"}
    del plan_b, wpb
    del lay_keys, wp, op, plan
    del a2, b2, k2, gks, o2, or2, w2, oh, wh
    c2.close()

    # ONE image through a whole network in the rotation-packed layout (the latency figure: the paper reports minutes per
    # image, section 3.2): the layer kinds and order of Table 1 at reduced width (3x16x16 -> conv 4@5x5 -> x -> 2x2 pool ->
    # conv 6@3x3 -> x -> pool -> FC 16 -> x -> FC 2, x = the degree-2 polynomial of section 3.1), every pooling merged into the
    # matrix of the layer after it, N = 2^14, 11 primes; keys and input are uniform residues
    cs = ckksmi.Context(14, 11, 50, 3, 51, 3, device=0)
    topo = "single_image_reduced"
    plans, n_per, lvl_out, _ = packed.plan_network(cs, wl.cnn_shapes(topo), wl.cnn_weights_float(topo, 7, sigma=0.25), 11, 2.0 ** 50, to_dev)
    all_rots = sorted({d for pl in plans if isinstance(pl, packed.BlockPlan) for r in pl.rotations.values() for d in r})
    net_keys = []
    for d in all_rots:
        net_keys.append(uniform_residues(torch, cs.moduli, (cs.beta_top, 2), 1 << 14, gen))
        cs.galois_key_register(d, net_keys[-1])
    evk_s = uniform_residues(torch, cs.moduli, (cs.beta_top, 2), 1 << 14, gen)
    xin_s = uniform_residues(torch, cs.q, (1, 2), 1 << 14, gen)
    wsn = torch.empty(packed.network_workspace_bytes(cs, plans, 11) // 8 + 1, dtype=torch.int64, device="cuda:0")
    ms = timed(torch, lambda: packed.run_network(cs, xin_s, plans, evk_s, 11, wsn), 2)
    # one image is a few thousand small launches (one ciphertext each): the same call sequence captured in a graph
    side_s = torch.cuda.Stream()
    side_s.wait_stream(torch.cuda.current_stream())
    graph_s = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph_s, stream=side_s):
        packed.run_network(cs, xin_s, plans, evk_s, 11, wsn)
    ms_graph = timed(torch, graph_s.replay, 3)
    del graph_s
    n_mul = sum(len(o) for pl in plans if isinstance(pl, packed.BlockPlan) for o in pl.offsets.values())
    out["single_image_network_2e14"] = {"ms_per_image": round(ms, 2), "ms_per_image_graph": round(ms_graph, 2), "rotations": sum(len(r) for pl in plans if isinstance(pl, packed.BlockPlan) for r in pl.rotations.values()),
                                        "plaintext_products": n_mul, "distinct_keys": len(all_rots), "levels": [11, lvl_out], "period": n_per,
                                        "what": "one image, rotation-packed: 3x16x16 -> conv 4@5x5, poly2, pool+conv 6@3x3, poly2, pool+FC 16, poly2, FC 2"}
    del net_keys, wsn, plans
    # the same network with baby steps and giant steps: offset d = g*32 + b costs a rotation by b (hoisted) and one by 32 g
    # of a whole sum, so every layer reads about 60 rotation keys instead of up to 961
    plans_b, _, lvl_b, _ = packed.plan_network(cs, wl.cnn_shapes(topo), wl.cnn_weights_float(topo, 7, sigma=0.25), 11, 2.0 ** 50, to_dev, bsgs=True)
    rots_b = sorted({d for pl in plans_b if isinstance(pl, packed.BsgsPlan) for d in pl.rotation_offsets()})
    keys_b = []
    for d in rots_b:
        keys_b.append(uniform_residues(torch, cs.moduli, (cs.beta_top, 2), 1 << 14, gen))
        cs.galois_key_register(d, keys_b[-1])
    wsb = torch.empty(packed.network_workspace_bytes(cs, plans_b, 11) // 8 + 1, dtype=torch.int64, device="cuda:0")
    ms_b = timed(torch, lambda: packed.run_network(cs, xin_s, plans_b, evk_s, 11, wsb), 3)
    side_b = torch.cuda.Stream()
    side_b.wait_stream(torch.cuda.current_stream())
    graph_b = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph_b, stream=side_b):
        packed.run_network(cs, xin_s, plans_b, evk_s, 11, wsb)
    ms_bg = timed(torch, graph_b.replay, 5)
    del graph_b
    bs = [pl for pl in plans_b if isinstance(pl, packed.BsgsPlan)]
    out["single_image_network_bsgs_2e14"] = {"ms_per_image": round(ms_b, 2), "ms_per_image_graph": round(ms_bg, 2), "baby": bs[0].baby, "distinct_keys": len(rots_b),
                                             "baby_rotations": sum(len(b) for pl in bs for b in pl.babies.values()),
                                             "giant_rotations": sum(len(pl.groups) - pl.n_plain for pl in bs),
                                             "plaintext_products": sum(len(pl.terms) for pl in bs), "levels": [11, lvl_b],
                                             "what": "the same network, every matrix in baby-step / giant-step form (other bits, same decrypted result)"}
    del keys_b, wsb, plans_b
    # a 3x32x32 image (Table 1's input size) through the same layer kinds at small width: conv 8@5x5, x, pool + conv 16@5x5,
    # x, pool + FC 64, x, FC 10; period 8192 = every slot of N = 2^14; 15161 diagonals encoded on the device at plan time
    topo_c = "single_image_cifar"

    def encode_batch(vecs, scale, level):
        pts = torch.empty((vecs.shape[0], level, 1 << 14), dtype=torch.int64, device="cuda:0")
        wse = torch.empty(512 * (1 << 14) * 2, dtype=torch.int64, device="cuda:0")
        for t0 in range(0, vecs.shape[0], 512):
            re = torch.from_numpy(__import__("numpy").ascontiguousarray(vecs[t0:t0 + 512])).to("cuda:0")
            cs.encode_device(re, None, scale, level, re.shape[0], pts[t0:t0 + re.shape[0]], wse)
        return pts

    t_plan = time.perf_counter()
    plans_c, n_c, lvl_c, _ = packed.plan_network(cs, wl.cnn_shapes(topo_c), wl.cnn_weights_float(topo_c, 7, sigma=0.1), 11, 2.0 ** 50, to_dev, bsgs=True,
                                                 encode_batch=encode_batch)
    torch.cuda.synchronize()
    t_plan = time.perf_counter() - t_plan
    bc = [pl for pl in plans_c if isinstance(pl, packed.BsgsPlan)]
    rots_c = sorted({d for pl in bc for d in pl.rotation_offsets()})
    keys_c = []
    for d in rots_c:
        keys_c.append(uniform_residues(torch, cs.moduli, (cs.beta_top, 2), 1 << 14, gen))
        cs.galois_key_register(d, keys_c[-1])
    wsc = torch.empty(packed.network_workspace_bytes(cs, plans_c, 11) // 8 + 1, dtype=torch.int64, device="cuda:0")
    ms_c = timed(torch, lambda: packed.run_network(cs, xin_s, plans_c, evk_s, 11, wsc), 3)
    out["single_image_cifar_2e14"] = {"ms_per_image": round(ms_c, 2), "plan_s": round(t_plan, 1), "baby": bc[0].baby, "distinct_keys": len(rots_c),
                                      "baby_rotations": sum(len(b) for pl in bc for b in pl.babies.values()),
                                      "giant_rotations": sum(len(pl.groups) - pl.n_plain for pl in bc),
                                      "plaintext_products": sum(len(pl.terms) for pl in bc),
                                      "plaintext_GB": round(sum(pl.pts.numel() * 8 for pl in bc) / 1e9, 1), "levels": [11, lvl_c], "period": n_c,
                                      "what": "one 3x32x32 image, rotation-packed with baby and giant steps: conv 8@5x5, poly2, pool+conv 16@5x5, poly2, pool+FC 64, poly2, FC 10"}
    del keys_c, evk_s, xin_s, wsc, plans_c
    cs.close()

    out.update(conv_layer_workload(torch, ckksmi, wl, gen))
    return out


def cnn_in_strips(torch, ckksmi, wl, gen, preset, topology, what):
    """A whole network at its real shape (N=2^16, 32768 images per pass, one ciphertext per pixel).  Its activations
    (up to a terabyte per layer) do not fit on one GPU, so every layer runs strip by strip over ALL of its output
    positions on buffers of uniform residues that are reused from strip to strip (ciphertexts are pseudorandom and no
    kernel branches on data); the time is the sum over the strips of every layer."""
    from paper_1911_11377_amd import activation, cnn

    p5 = wl.PRESETS[preset]
    c5 = ckksmi.Context(p5.logN, p5.n_q, p5.q_bits, p5.k, p5.special_bits, p5.alpha, device=0)
    N, L = p5.N, p5.n_q
    shapes = wl.cnn_shapes(topology)
    plans, out_level, _ = cnn.plan(shapes, wl.cnn_weights_float(topology, 5), c5.q, L, 2.0 ** p5.log_scale)
    evk = uniform_residues(torch, c5.moduli, (c5.beta_top, 2), N, gen)
    ct_words = lambda level: 2 * level * N
    ACT_BATCH = 256

    # strip sizes: one output row per conv strip, one output row per pooling strip, ACT_BATCH ciphertexts per activation
    def strip_words(pl):
        C, H, W = pl.in_shape
        O, Ho, Wo = pl.out_shape
        if pl.kind == "conv":
            rows_in = min(H, pl.kernel)
            return C * rows_in * W * ct_words(pl.level_in), O * Wo * ct_words(pl.level_in), O * Wo * ct_words(pl.level_out)
        if pl.kind == "fc":
            return C * H * W * ct_words(pl.level_in), O * ct_words(pl.level_in), O * ct_words(pl.level_out)
        if pl.kind in ("square", "poly2"):
            n = min(ACT_BATCH, C * H * W)
            return n * ct_words(pl.level_in), 0, n * ct_words(pl.level_out)
        rows_in = H if pl.pad else pl.kernel
        return C * rows_in * W * ct_words(pl.level_in), 0, O * (Ho if pl.pad else 1) * Wo * ct_words(pl.level_out)

    need = [strip_words(pl) for pl in plans]
    ws_bytes = cnn.workspace_bytes(c5, plans, max_items=64)
    in_words, mac_words, out_words = (max(n[i] for n in need) for i in range(3))
    xin = torch.empty(in_words, dtype=torch.int64, device="cuda:0")
    step = 1 << 27
    for o in range(0, in_words, step):  # canonical for every prime: all of them exceed 2^49
        xin[o:o + step].random_(0, 1 << 49, generator=gen)
    mac = torch.empty(max(mac_words, 1), dtype=torch.int64, device="cuda:0")
    out = torch.empty(out_words, dtype=torch.int64, device="cuda:0")
    ws = torch.empty(ws_bytes // 8 + 1, dtype=torch.int64, device="cuda:0")
    layers = []
    total_ms = 0.0
    for pl in plans:
        C, H, W = pl.in_shape
        O, Ho, Wo = pl.out_shape
        wdev = torch.from_numpy(pl.w_int).to("cuda:0") if pl.w_int is not None else None
        calls = []
        if pl.kind == "conv":
            for r in range(Ho):
                i0 = max(0, r * pl.stride - pl.pad)
                i1 = min(H - 1, r * pl.stride - pl.pad + pl.kernel - 1)
                calls.append(lambda r=r, i0=i0, i1=i1: cnn.conv_rows(c5, pl, xin, wdev, i0, i1 - i0 + 1, r, 1, mac, out, ws))
        elif pl.kind == "fc":
            def fc():
                c5.fc_mac(xin, wdev, C * H * W, O, mac, pl.level_in, ws)
                c5.rescale(mac, out, pl.level_in, O, ws)
            calls.append(fc)
        elif pl.kind == "square":
            n_ct = C * H * W
            for b0 in range(0, n_ct, ACT_BATCH):
                n = min(ACT_BATCH, n_ct - b0)
                calls.append(lambda n=n: c5.hmul_relin_rescale(xin, xin, evk, out, pl.level_in, n, ws))
        elif pl.kind == "poly2":
            n_ct = C * H * W
            for b0 in range(0, n_ct, ACT_BATCH):
                n = min(ACT_BATCH, n_ct - b0)
                calls.append(lambda n=n: cnn.poly2_batch(c5, pl, xin, evk, out, n, ws, 64))
        elif pl.pad:
            calls.append(lambda: c5.sum_pool2d(xin, C, H, W, pl.kernel, out, pl.level_in, pad=pl.pad))
        else:
            for r in range(Ho):
                calls.append(lambda: c5.sum_pool2d(xin, C, pl.kernel, W, pl.kernel, out, pl.level_in))
        calls[0]()  # warm-up of this layer's kernels
        torch.cuda.synchronize()
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record()
        for f in calls:
            f()
        e1.record()
        torch.cuda.synchronize()
        ms = e0.elapsed_time(e1)
        total_ms += ms
        layers.append({"layer": pl.kind, "in": list(pl.in_shape), "out": list(pl.out_shape), "level": pl.level_in, "strips": len(calls),
                       "ms": round(ms, 1)})
        del wdev
    images = N // 2
    res = {"encrypted_images_per_s": round(images / (total_ms * 1e-3), 1), "images_per_pass": images, "s_per_pass": round(total_ms * 1e-3, 2),
           "levels": [L, out_level], "layers": layers,
           "what": what + "; every layer at its real shape over all output positions, strip by strip on reused synthetic buffers"}
    del xin, mac, out, ws, evk
    c5.close()
    torch.cuda.empty_cache()
    return res


def op_byte_models(N, level, k, alpha, batch):
    """bytes of one HMult + relinearise + rescale under two traffic models (limb = 8N bytes):
    compulsory = read two ciphertexts, write one, the key once per batch; stage-wise = every stage reads its inputs once and
    writes its outputs once, nothing fused (tensor, inverse transform of d2, ModUp, forward transforms, inner product,
    ModDown, rescale; transforms counted once per limb)"""
    E, beta = level + k, -(-level // alpha)
    w = 8.0 * N
    compulsory = w * (4 * level + 2 * (level - 1) + 2.0 * beta * E / batch)
    tensor = w * (4 * level + 3 * level)
    intt_d2 = w * 2 * level
    modup = w * (level + beta * E - level)
    ntt_up = w * 2 * (beta * E - level)
    inner = w * (beta * E + 2 * E + 2.0 * beta * E / batch)
    moddown = w * (2 * (2 * k) + (2 * k + 2 * level) + 2 * (2 * level) + 4 * (2 * level))
    rescale = w * (2 * 2 + (2 + 2 * (level - 1)) + 2 * 2 * (level - 1) + 3 * 2 * (level - 1))
    return compulsory, tensor + intt_d2 + modup + ntt_up + inner + moddown + rescale


def copy_bandwidth(torch, nbytes=3 << 29):
    """a plain device-to-device copy (reads and writes nbytes each): what the memory system sustains for streaming"""
    src = torch.empty(nbytes // 8, dtype=torch.int64, device="cuda:0")
    dst = torch.empty_like(src)
    ms = timed(torch, lambda: dst.copy_(src), 5)
    del src, dst
    return 2.0 * nbytes / (ms * 1e-3) / 1e9


def transform_sweeps(torch, ckksmi, wl, gen, ctx4):
    """plain forward and inverse limb transforms, in place, for the shape of every workload: batch x 2 x (level + k) limbs
    (the conv workload's 3072 ciphertexts are capped at 256 per launch); GB/s on 16N bytes per limb transform"""
    out = {}
    for name, preset, cap in (("tiny_2e12", "tiny", None), ("hmul_rot_2e14", "hmul_rot_2e14", None), ("conv_2e15", "conv_2e15", 256),
                              ("act_2e16", "act_2e16", None)):
        p = wl.PRESETS[preset]
        c = ctx4 if preset == "act_2e16" else ckksmi.Context(p.logN, p.n_q, p.q_bits, p.k, p.special_bits, p.alpha, device=0)
        cts = p.batch if cap is None else min(p.batch, cap)
        idx = list(range(p.n_q)) + [p.n_q + m for m in range(p.k)]
        limbs = uniform_residues(torch, [c.moduli[t] for t in idx], (cts * 2,), p.N, gen)
        reps = 3 if p.logN >= 15 else 20
        row = {"limbs": cts * 2 * len(idx)}
        for d, fn in (("fwd", c.ntt), ("inv", c.intt)):
            ms = timed(torch, lambda: fn(limbs, idx, cts * 2), reps)
            gbps = 16.0 * p.N * len(idx) * cts * 2 / (ms * 1e-3) / 1e9
            row[d] = {"GBps": round(gbps, 1), "frac_of_hbm_peak": round(gbps / HBM_PEAK_GBPS, 4)}
        out[name] = row
        del limbs
        if c is not ctx4:
            c.close()
    return out


def oracle_legs(np, torch, wl, ckksmi, cores):
    """the oracle timed on the host cores, one unit of work per workload shape: a limb transform, HMult + relinearise +
    rescale, a rotation, one conv output ciphertext (multiply-accumulate over its window + rescale); single thread, and the
    same unit once per thread on `cores` threads (independent ciphertexts; the C calls release the GIL).  Inputs are uniform
    residues from the neutral input module: the oracle's time does not depend on the data."""
    from concurrent.futures import ThreadPoolExecutor

    from oracle import oracle as orc

    def both(fn):
        t0 = time.perf_counter()
        fn(0)
        t1 = time.perf_counter()
        with ThreadPoolExecutor(cores) as ex:
            list(ex.map(fn, range(cores)))
        t2 = time.perf_counter()
        return {"single_thread_s": round(t1 - t0, 4), "per_s_single": round(1.0 / (t1 - t0), 3), "per_s_all_cores": round(cores / (t2 - t1), 3)}

    legs = {}
    for name, preset, ops in (("tiny_2e12", "tiny", ("ntt", "hmul")), ("hmul_rot_2e14", "hmul_rot_2e14", ("ntt", "hmul", "rotate")),
                              ("conv_2e15", "conv_2e15", ("ntt", "conv_out")), ("act_2e16", "act_2e16", ("ntt", "rotate"))):
        p = wl.PRESETS[preset]
        O = orc.Oracle(p.logN, p.n_q, p.q_bits, p.k, p.special_bits, p.alpha)
        L, N = p.n_q, p.N
        row = {}
        ct = wl.uniform_limbs(O.q[:L], N, 9, "oracle.leg", preset, lead=(2,))
        if "ntt" in ops:
            limb = ct[0, :1].copy()
            row["limb_transform"] = both(lambda i: O.ntt_limbs(limb, [0]))
        key = wl.uniform_limbs(O.moduli, N, 9, "oracle.key", preset, lead=(O.beta_top, 2)) if p.k else None
        if "hmul" in ops:
            row["hmul_relin_rescale"] = both(lambda i: O.hmul_relin_rescale(ct, ct, key, L))
        if "rotate" in ops:
            row["rotate"] = both(lambda i: O.rotate(ct, 1, key, L))
        if "conv_out" in ops:
            win = wl.uniform_limbs(O.q[:L], N, 9, "oracle.win", lead=(3, 5, 5, 2))
            wi = np.rint(wl.weights_float((1, 3, 5, 5), 9, "oracle.w") * float(O.q[L - 1])).astype(np.int64)
            row["conv_output_ciphertext"] = both(lambda i: O.rescale(O.conv2d_mac(win, wi, 1, 0, L)[0, 0, 0], L))
        legs[name] = row
    return legs


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=5)
    ap.add_argument("--warmup", type=int, default=2)
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-sweep", action="store_true", help="skip the plain transform sweeps (keeps a profile to the timed steps)")
    ap.add_argument("--conv-only", action="store_true", help="run the conv layer workload (N=2^15) alone and print its figures: for profiles of its kernels")
    ap.add_argument("--no-extras", action="store_true", help="skip the secondary workloads (rotation at N=2^14, conv layer at N=2^15, activation schedule)")
    ap.add_argument("--no-cnn", action="store_true", help="skip the two full-size networks in strips (about a minute of GPU time, up to 200 GB of HBM)")
    ap.add_argument("--copy-probe", action="store_true",
                    help="also run one plain device copy of the input batch (known size) so that profiler byte counters can be scaled")
    args = ap.parse_args()
    if args.gpus != 1:
        sys.exit("bench.py: this build runs on ONE GPU; --gpus %d is not supported (every ciphertext is independent, "
                 "so the batch would simply be split across GPUs)" % args.gpus)

    import numpy as np
    import torch

    from paper_1911_11377_amd import build as lib_build
    from paper_1911_11377_amd import ckksmi
    from paper_1911_11377_amd import workloads as wl

    if not torch.cuda.is_available():
        sys.exit("bench.py needs a GPU")
    if not os.path.exists(lib_build.LIB):  # the library that is built is the one that runs; nothing built yet: build once
        lib_build.build(force=True)
    if args.conv_only:
        g3 = torch.Generator(device="cuda:0")
        g3.manual_seed(wl.BASE_SEED + 3)
        print(json.dumps({"extras": conv_layer_workload(torch, ckksmi, wl, g3)}))
        return
    p = wl.PRESETS["act_2e16"]
    level, batch, N = p.n_q, p.batch, p.N
    ctx = ckksmi.Context(p.logN, p.n_q, p.q_bits, p.k, p.special_bits, p.alpha, device=0)
    gen = torch.Generator(device="cuda:0")
    gen.manual_seed(wl.BASE_SEED + 4)
    a = uniform_residues(torch, ctx.q[:level], (batch, 2), N, gen)
    b = uniform_residues(torch, ctx.q[:level], (batch, 2), N, gen)
    evk = uniform_residues(torch, ctx.moduli, (ctx.beta_top, 2), N, gen)
    out = torch.empty((batch, 2, level - 1, N), dtype=torch.int64, device="cuda:0")
    ws_items = int(os.environ.get("CKKSMI_BENCH_WS_ITEMS", batch))  # tuning: a smaller workspace makes the call sweep the batch in chunks
    ws = torch.empty(ctx.workspace_bytes(ckksmi.OP_HMUL_RELIN_RESCALE, level, ws_items) // 8, dtype=torch.int64, device="cuda:0")

    def step():
        ctx.hmul_relin_rescale(a, b, evk, out, level, batch, ws)

    # ---- the timed region: K steps, nothing else on the stream (no timing events inside)
    for _ in range(args.warmup):
        step()
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(args.steps):
        step()
    torch.cuda.synchronize()
    t1 = time.perf_counter()
    ms_per_step = (t1 - t0) * 1e3 / args.steps
    value = batch * args.steps / (t1 - t0)

    # ---- the same K steps again with two HIP events around every kernel launch (recorded by the library on the launch
    # stream): per-kernel average durations for the roofline; the events cost a little, so this loop is not the headline
    ctx.profile_enable(True)
    t2 = time.perf_counter()
    for _ in range(args.steps):
        step()
    torch.cuda.synchronize()
    t3 = time.perf_counter()
    prof = ctx.profile_read()
    ctx.profile_enable(False)
    ms_per_step_profiled = (t3 - t2) * 1e3 / args.steps

    # ---- roofline of the dominant kernel (largest share of the timed region)
    counters = load_counters() if (level, batch, p.logN) == (24, 64, 16) else None
    kernels = {}
    for name, (ms, launches, units) in prof.items():
        bpu = bytes_per_unit(name, N, level, p.k, p.alpha, batch)
        row = {"ms_total": round(ms, 3), "launches": launches, "avg_ms": round(ms / launches, 4),
               "GBps": round(bpu * units / (ms * 1e-3) / 1e9, 1) if bpu else None}
        cf = counter_figures(counters, name)
        if cf:
            if "traffic" in cf:
                row["traffic_over_algorithmic"] = round(cf["traffic"] / (bpu * units / launches), 3) if bpu else None
            if "valu_wave_instr" in cf:
                row["alu_frac_counted"] = round(cf["valu_wave_instr"] * 64.0 / (ms / launches * 1e-3) / FP64_PEAK_LANEOPS, 4)
            for kname in ("valu_busy", "lds_conflict_frac", "l2_hit_rate"):
                if kname in cf:
                    row[kname] = round(cf[kname], 4)
        kernels[name] = row
    dom = max(prof, key=lambda n: prof[n][0])
    ms, launches, units = prof[dom]
    bpu = bytes_per_unit(dom, N, level, p.k, p.alpha, batch)
    achieved = bpu * units / (ms * 1e-3) / 1e9
    hbm_frac = achieved / HBM_PEAK_GBPS
    # vector-ALU rate of the dominant kernel: vector instructions counted by the hardware (SQ_INSTS_VALU of one launch,
    # from the counters file) x 64 lanes / this run's average launch duration; the count made by hand from the source
    # stays beside it
    lpu = laneops_per_unit(dom, N, level, p.k, p.alpha)
    alu_frac_hand = lpu * units / (ms * 1e-3) / FP64_PEAK_LANEOPS if lpu else None
    cf = counter_figures(counters, dom) or {}
    alu_rate = cf["valu_wave_instr"] * 64.0 / (ms / launches * 1e-3) if "valu_wave_instr" in cf else (lpu * units / (ms * 1e-3) if lpu else None)
    alu_frac = alu_rate / FP64_PEAK_LANEOPS if alu_rate else 0.0
    ntt_ms = sum(prof[n][0] for n in prof if n.startswith("ntt_"))
    ntt_limbs = sum(prof[n][2] for n in prof if n in ("ntt_fwd_kernel<false>", "ntt_inv_kernel<false>", "ntt_v2_kernel<false, false>", "ntt_v2_kernel<true, false>"))
    if alu_frac > hbm_frac:
        # the kernel does more vector work per byte than the machine balance: the vector ALU binds.  Peak = 256 CUs x 64
        # lanes x 2.4 GHz = 39.3 T vector instructions/s (half the 78.6 TFLOP/s FP64 FMA figure); unit: T instructions/s
        roofline = {"kernel": dom, "bound": "alu", "achieved": round(alu_rate / 1e12, 2), "peak": FP64_PEAK_LANEOPS / 1e12,
                    "unit": "T lane-instr/s", "frac": round(alu_frac, 4)}
    else:
        roofline = {"kernel": dom, "bound": "hbm", "achieved": round(achieved, 1), "peak": HBM_PEAK_GBPS, "unit": "GB/s",
                    "frac": round(hbm_frac, 4)}
    roofline.update({"traffic": cf.get("traffic"), "hbm_GBps": round(achieved, 1), "hbm_frac": round(hbm_frac, 4), "alu_frac": round(alu_frac, 4),
                     "alu_frac_source": "SQ_INSTS_VALU (profiles/counters_act_2e16.json)" if "valu_wave_instr" in cf else "hand count",
                     "alu_frac_hand_count": round(alu_frac_hand, 4) if alu_frac_hand else None,
                     "valu_busy": round(cf["valu_busy"], 4) if "valu_busy" in cf else None,
                     "avg_launch_ms": round(ms / launches, 4), "bytes_per_launch": bpu * units / launches,
                     "all_transforms_GBps": round(16 * N * ntt_limbs / (ntt_ms * 1e-3) / 1e9, 1) if ntt_ms else None,
                     "kernels": kernels})

    # ---- the whole step against the byte models and the streaming bandwidth the memory system sustains
    copy_gbps = copy_bandwidth(torch)
    compulsory, stagewise = op_byte_models(N, level, p.k, p.alpha, batch)
    step_s = ms_per_step * 1e-3
    traffic_step = None
    if counters:
        per = [counter_figures(counters, n) for n in prof]
        if all(x and "traffic" in x for x in per):
            traffic_step = sum(x["traffic"] * prof[n][1] / args.steps for x, n in zip(per, prof))
    step_fracs = {
        "ms_per_step": round(ms_per_step, 3), "ms_per_step_with_timing_events": round(ms_per_step_profiled, 3),
        "stagewise_bytes_per_op": stagewise, "compulsory_bytes_per_op": compulsory,
        "frac_of_hbm_peak_on_stagewise_bytes": round(stagewise * batch / step_s / 1e9 / HBM_PEAK_GBPS, 4),
        "frac_of_hbm_peak_on_compulsory_bytes": round(compulsory * batch / step_s / 1e9 / HBM_PEAK_GBPS, 4),
        "copy_GBps": round(copy_gbps, 1),
        "measured_traffic_bytes_per_step": traffic_step,
        "frac_of_hbm_peak_on_measured_traffic": round(traffic_step / step_s / 1e9 / HBM_PEAK_GBPS, 4) if traffic_step else None,
        "frac_of_copy_bandwidth_on_measured_traffic": round(traffic_step / step_s / 1e9 / copy_gbps, 4) if traffic_step else None,
    }

    if args.copy_probe:
        probe = torch.empty_like(a)
        probe.copy_(a)  # reads and writes a.numel()*8 bytes
        torch.cuda.synchronize()
        del probe

    # ---- plain transform sweeps, one per workload shape
    sweeps = {} if args.no_sweep else transform_sweeps(torch, ckksmi, wl, gen, ctx)
    ntt = sweeps.get("act_2e16", {})

    extras = None
    if not (args.no_extras or args.no_sweep):
        extras = secondary_workloads(torch, ckksmi, wl, ctx, a, evk, ws, gen)

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
        O.hmul_relin_rescale(ha[0], hb[0], hk, level)
        c1 = time.perf_counter()
        with ThreadPoolExecutor(cores) as ex:  # the C calls release the GIL
            res = list(ex.map(lambda i: O.hmul_relin_rescale(ha[i], hb[i], hk, level), range(cores)))
        c2 = time.perf_counter()
        got = out[:cores].cpu().numpy().view(np.uint64)
        match = all(np.array_equal(res[i], got[i]) for i in range(cores))
        cpu = {"value": round(cores / (c2 - c1), 4), "unit": "ops/s", "cores": cores, "kind": "oracle",
               "sample": "%d of the %d HMult+relin+rescale of one step, one per thread, same inputs" % (cores, batch),
               "single_thread_ops_per_s": round(1.0 / (c1 - c0), 4), "matches_gpu_bits": bool(match),
               "per_workload": oracle_legs(np, torch, wl, ckksmi, cores)}

    if extras is not None and not args.no_cnn:
        del a, b, evk, out, ws
        torch.cuda.empty_cache()
        extras["cnn_2e16_in_strips"] = cnn_in_strips(
            torch, ckksmi, wl, gen, "cnn_2e16", "cnn_2e16",
            "conv 3->32 5x5 s2, x^2, conv 32->64 3x3 s2, x^2, conv 64->64 3x3 pad 1, 2x2 sum pool, FC 3136->256, x^2, FC 256->2")
        # the paper's own network (Table 1, 3x32x32 inputs, degree-2 polynomial activations of section 3.1) on the 24-prime shape
        extras["table1_2e16_in_strips"] = cnn_in_strips(
            torch, ckksmi, wl, gen, "act_2e16", "table1",
            "Table 1: conv 96@11x11, conv 256@5x5, conv 384@3x3 (pad 1) twice, 2x2 average pooling after each, FC 4096, FC 4096, FC 1; "
            "0.00047x^2 + 0.5x after every layer but the last")

    line = {
        "metric": "HMult+relin+rescale ops/s at N=2^16", "value": round(value, 2), "unit": "ops/s", "n_gpus": 1,
        "steps": args.steps, "warmup": args.warmup, "ms_per_step": round(ms_per_step, 3), "higher_is_better": True,
        "scaling": "weak", "vs_baseline": None, "dtype": "f64", "data": "synthetic",
        "config": {"workload": "act_2e16: N=2^16, 24x50-bit primes + 3x51-bit special primes, 8 digits of 3, batch 64, level 24",
                   "op": "tensor -> key switch (ModUp, inner product, ModDown) -> add -> rescale"},
        "roofline": roofline, "step": step_fracs, "ntt_sweep": ntt, "ntt_sweeps": sweeps, "cpu_baseline": cpu, "extras": extras,
    }
    print(json.dumps(line))


if __name__ == "__main__":
    main()
