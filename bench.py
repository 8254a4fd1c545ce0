#!/usr/bin/env python3
"""Benchmark of the whole hot path on one MI355X.

One step = one pass of the batched ResNet-20 stage-3 block slice over one batch of synthetic input
(workload cfg5_resnet20_stage3: N = 2^16, 24 ciphertext limbs + 8 special primes, dnum 3, 64 -> 64
channels, 3x3 convolution on 8x8 images, batch 512 = 32768 slots per channel ciphertext), i.e.
he_conv_batched (64 shared decompositions, 512 hoisted rotations, the 64x576 multiply-accumulate,
64 rescales) followed by the degree-7 polynomial activation on every output channel (256
ciphertext products with relinearisation, 320 rescales).  All inputs are resident in HBM before
the timed region.  Prints ONE JSON line.

Inputs are seeded uniform residues of the right shapes (ciphertexts, switching keys, mask
plaintexts, integer weights): modular arithmetic has no data-dependent control flow, so timing does
not depend on the values; correctness on real ciphertexts is what the parity tests establish.
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0
# vector ALU peak: 256 CUs x 4 SIMDs x 16 lanes x 2.4 GHz = 39.3e12 lane-operations/s (32-bit integer or fp64 FMA alike)
ALU_PEAK_LANE_OPS = 256 * 4 * 16 * 2.4e9
# Kernels whose limiter is arithmetic, should one of them become the dominant kernel:
# a double-precision butterfly of the NTT = 10 fp64 operations (6 for the twiddle product, 2 for sum and
# difference, 2 for the amortised re-centring); the multiply-accumulate on the matrix cores = 49 digit
# products x 2 operations per modular multiply-add against the dense 8-bit integer peak.
ALU_KERNELS = {"ntt_fwd_lo": (10.0, "Gbutterfly/s"), "ntt_inv_lo": (10.0, "Gbutterfly/s")}
MFMA_KERNELS = {"weighted_sum": (98.0, 5.0e15)}   # int8 operations per modular multiply-add, peak int8 op/s
TRAFFIC_FILE = os.path.join(ROOT, "profiles", "pmc_traffic_cfg5_block_slice.txt")


def measured_traffic(kernel):
    """HBM bytes per launch of `kernel` from the committed rocprofv3 --pmc summary (FETCH_SIZE and
    WRITE_SIZE runs, scaled by the plain copy kernel), or None."""
    try:
        for line in open(TRAFFIC_FILE):
            f = line.split()
            if len(f) >= 4 and f[0] == kernel:
                return float(f[1]) + float(f[2])
    except OSError:
        pass
    return None


def parse_args():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=5)
    ap.add_argument("--warmup", type=int, default=1)
    ap.add_argument("--workload", default="cfg5_resnet20_stage3")
    ap.add_argument("--alignment", default="deferred_merged", choices=["direct", "four_keys", "deferred", "deferred_merged"],
                    help="convolution schedule: eight hoisted rotations with one ModDown each (direct), the paper's four-key "
                         "two-stage alignment, one ModDown per output channel after the sum (deferred), or that ModDown merged "
                         "with the rescale (deferred_merged, the default)")
    ap.add_argument("--two-step-activation", action="store_true",
                    help="activation with separate ModDown and rescale after every product (default: merged into one division)")
    ap.add_argument("--single-stream", action="store_true",
                    help="keep all work on one stream for the whole run (channel batches do not overlap): what the profiling runs use")
    ap.add_argument("--wide-weights", action="store_true",
                    help="do not state the bound on the integer weights (the multiply-accumulate then takes them as full residues)")
    ap.add_argument("--no-cpu-baseline", action="store_true", help="skip the oracle timing (profiling runs)")
    ap.add_argument("--no-kernel-timing", action="store_true", help="skip the per-kernel event pass")
    ap.add_argument("--no-microbench", action="store_true", help="skip the rotation and NTT microbenchmarks")
    ap.add_argument("--no-schedules", action="store_true", help="skip the other three convolution schedules")
    ap.add_argument("--rotations-only", action="store_true",
                    help="only the rotation microbenchmark (64 hoisted + 64 unhoisted rotations, three times each): for profiling runs")
    ap.add_argument("--ntt-only", action="store_true",
                    help="only the NTT microbenchmark (64 x 30 limb transforms at N = 2^16, forward and inverse, six times): for profiling runs")
    ap.add_argument("--fc-only", action="store_true", help="only the fully connected layer at the classifier's shape, ten times: for profiling runs")
    ap.add_argument("--downsample-only", action="store_true", help="only the down-sampling compaction (both schedules, three times each): for profiling runs")
    ap.add_argument("--prime-bits", type=int, default=50,
                    help="size of the primes for --ntt-only / --rotations-only (56: the 64-bit integer kernels instead of the double-precision ones)")
    ap.add_argument("--calibration-copy", action="store_true",
                    help="also run the library's plain copy kernel on one ciphertext (24 MiB in, 24 MiB out): the known-size "
                         "dispatch that hardware-counter runs are scaled by")
    return ap.parse_args()


def cpu_baseline(wl, params, alignment, act_merged):
    """Times the CPU oracle on a bounded sample of the same workload and schedule and extrapolates to one step."""
    import numpy as np
    from oracle import Oracle
    from workloads import conv_tap_offsets, uniform_residues
    orc = Oracle(params)
    level = params.num_q - 1
    q = params.moduli
    deferred = alignment.startswith("deferred")
    merged = alignment == "deferred_merged"
    ct = uniform_residues((2, level + 1, orc.N), q[:level + 1], "cpu_ct")
    key = uniform_residues((params.dnum, 2, orc.M, orc.N), q, "cpu_key")
    offs = conv_tap_offsets(wl.width)
    keys = {o: key for o in offs if o}
    q_mac = [q[t] for t in orc.ext_moduli_idx(level)] if deferred else list(q[:level + 1])
    pts = [uniform_residues((len(q_mac), orc.N), q_mac, "cpu_pt%d" % i) for i in range(9)]
    R_ALIGN, R_MAC, R_OUT, R_ACT = 8, 64, 8, 8              # repetitions: about 15 s of CPU work in all
    t0 = time.perf_counter()
    for _ in range(R_ALIGN):
        if deferred:
            aligned = orc.align_deferred(ct, level, wl.width, keys)
        elif alignment == "four_keys":
            aligned = orc.align_four_keys(ct, level, wl.width, keys)
        else:
            aligned = orc.align_direct(ct, level, wl.width, keys)
    t_align = (time.perf_counter() - t0) / R_ALIGN          # one input channel: its nine aligned copies
    t0 = time.perf_counter()
    for _ in range(R_MAC):
        acc = orc.mac_ext(pts, aligned, level) if deferred else orc.ptct_mac(pts, aligned, level)
    t_mac = (time.perf_counter() - t0) / R_MAC              # 9 taps of one (input, output) channel pair
    t0 = time.perf_counter()
    for _ in range(R_OUT):
        if merged:
            x = np.stack([orc.moddown_rescale(acc[0], level), orc.moddown_rescale(acc[1], level)])
        else:
            u = np.stack([orc.moddown(acc[0], level), orc.moddown(acc[1], level)]) if deferred else acc
            x = orc.rescale(u, level)
    t_out = (time.perf_counter() - t0) / R_OUT              # one output channel: (ModDown and) rescale
    t0 = time.perf_counter()
    for _ in range(R_ACT):
        (orc.poly_activation_merged if act_merged else orc.poly_activation)(x, level - 1, (3 << 40, -(5 << 40), 7 << 40, -(9 << 40)), key)
    t_act = (time.perf_counter() - t0) / R_ACT
    step = wl.c_in * t_align + wl.c_in * wl.c_out * t_mac + wl.c_out * (t_out + t_act)
    # the threads the oracle's OpenMP loops actually ran on, and the same sample once more on one thread (fewer repetitions)
    import ctypes
    gomp = ctypes.CDLL("libgomp.so.1")
    cores = int(gomp.omp_get_max_threads())
    gomp.omp_set_num_threads(1)
    t0 = time.perf_counter()
    aligned1 = orc.align_deferred(ct, level, wl.width, keys) if deferred else (
        orc.align_four_keys(ct, level, wl.width, keys) if alignment == "four_keys" else orc.align_direct(ct, level, wl.width, keys))
    s_align = time.perf_counter() - t0
    t0 = time.perf_counter()
    for _ in range(2):
        acc1 = orc.mac_ext(pts, aligned1, level) if deferred else orc.ptct_mac(pts, aligned1, level)
    s_mac = (time.perf_counter() - t0) / 2
    t0 = time.perf_counter()
    if merged:
        x1 = np.stack([orc.moddown_rescale(acc1[0], level), orc.moddown_rescale(acc1[1], level)])
    else:
        u1 = np.stack([orc.moddown(acc1[0], level), orc.moddown(acc1[1], level)]) if deferred else acc1
        x1 = orc.rescale(u1, level)
    s_out = time.perf_counter() - t0
    t0 = time.perf_counter()
    (orc.poly_activation_merged if act_merged else orc.poly_activation)(x1, level - 1, (3 << 40, -(5 << 40), 7 << 40, -(9 << 40)), key)
    s_act = time.perf_counter() - t0
    gomp.omp_set_num_threads(cores)
    step1 = wl.c_in * s_align + wl.c_in * wl.c_out * s_mac + wl.c_out * (s_out + s_act)
    return {
        "value": step * 1e3 / wl.batch, "unit": "ms/image", "cores": cores, "kind": "oracle",
        "single_thread": {"value": step1 * 1e3 / wl.batch, "unit": "ms/image", "cores": 1,
                          "sample": "one alignment (%.1f s), two 9-tap multiply-accumulates (%.2f s each), one output division (%.1f s), one "
                                    "activation (%.1f s) on one thread, extrapolated as above" % (s_align, s_mac, s_out, s_act)},
        "sample": ("oracle (%s schedule) timed at full size on %d input channels' alignments (%.2f s each), %d 9-tap "
                   "multiply-accumulates (%.3f s each), %d output channels' %srescale (%.2f s each) and %d degree-7 activations "
                   "(%.2f s each): %.0f s of CPU work, extrapolated to %d alignments, %d 9-tap MACs, %d output channels and activations"
                   % (alignment, R_ALIGN, t_align, R_MAC, t_mac, R_OUT, "ModDown + " if deferred else "", t_out, R_ACT, t_act,
                      R_ALIGN * t_align + R_MAC * t_mac + R_OUT * t_out + R_ACT * t_act, wl.c_in, wl.c_in * wl.c_out, wl.c_out)),
        "step_seconds_extrapolated": step,
    }


def rotation_microbench(hx, torch, ctx, ct, keys, level, N, ws, result, overlap=True):
    # rotation microbenchmark (24 limbs + 8 special primes, dnum 3): one ciphertext, 64 distinct offsets, 64 keys in
    # 64 separate 96 MiB buffers (their contents are clones of the eight seeded keys: only the addresses matter)
    n_rot_mb = 64
    from workloads import rotation_offsets
    mb_offs = rotation_offsets(n_rot_mb, N // 2)
    base_keys = [k for k in keys if k is not None]
    mb_keys = [hx.ckks_key_load(ctx, base_keys[i % len(base_keys)].tensor.clone(), hx.ckks_galois_element(ctx, r))
               for i, r in enumerate(mb_offs)]
    mb_outs = [hx.empty(2, level + 1, N) for _ in range(n_rot_mb)]
    for hoisted in (True, False):
        hx.ckks_ctx_set_overlap(ctx, overlap)
        hx.ckks_rotate_hoisted(ctx, ct, level, mb_offs, mb_keys, hoisted, outs=mb_outs, ws=ws)
        torch.cuda.synchronize()
        reps = 3
        t0 = time.perf_counter()
        for _ in range(reps):
            hx.ckks_rotate_hoisted(ctx, ct, level, mb_offs, mb_keys, hoisted, outs=mb_outs, ws=ws)
        torch.cuda.synchronize()
        dt = time.perf_counter() - t0
        name = "hoisted" if hoisted else "unhoisted"
        rate = n_rot_mb * reps / dt
        result["rotations_per_s_%s" % name] = rate
        # compulsory HBM traffic per rotation: key 96 MiB + c0 12 MiB + output 24 MiB (+ 24 MiB input when unhoisted)
        mib = (96 + 12 + 24) if hoisted else (96 + 24 + 24)
        result["rotation_%s_effective_GBs" % name] = rate * mib * 2**20 / 1e9
        result["rotation_%s_frac_of_hbm_peak" % name] = rate * mib * 2**20 / 1e9 / HBM_PEAK_GBS
    # where a hoisted rotation's time goes: every launch of one more call bracketed by events, all work on one stream
    hx.ckks_ctx_set_overlap(ctx, False)
    hx.ckks_prof_begin(ctx, None, max_launches=1 << 14)
    hx.ckks_rotate_hoisted(ctx, ct, level, mb_offs, mb_keys, True, outs=mb_outs, ws=ws)
    prof = hx.ckks_prof_end(ctx)
    prof.pop("dropped")
    inner = prof.get("key_inner", {"ms": 0.0, "bytes": 0.0})
    rest = sum(v["ms"] for k, v in prof.items() if k != "key_inner")
    result["rotation_hoisted_split"] = {
        "inner_product_us_per_rotation": 1e3 * inner["ms"] / n_rot_mb, "inner_product_GBs": inner["bytes"] / max(inner["ms"], 1e-9) / 1e6,
        "moddown_and_shared_modup_us_per_rotation": 1e3 * rest / n_rot_mb,
        "note": "one call of 64 rotations with every launch bracketed, no overlap between batches; the timed rate above lets batches overlap"}


def conv_microbench(hx, torch, name, result):
    """The convolution alone at another benchmark shape (deferred ModDown merged with the rescale, bounded weights)."""
    import numpy as np
    from workloads import CONFIGS, conv_tap_offsets, conv_weights, uniform_residues
    wl = CONFIGS[name]
    params = wl.params()
    ctx = hx.Context(params)
    N, level, q = params.n, params.num_q - 1, params.moduli
    M = params.num_q + params.num_p
    ins = [hx.from_host(uniform_residues((2, level + 1, N), q[:level + 1], name + "in%d" % c)) for c in range(wl.c_in)]
    offs = conv_tap_offsets(wl.width)
    keys = [hx.ckks_key_load(ctx, hx.from_host(uniform_residues((params.dnum, 2, M, N), q, name + "rk%d" % t)),
                             hx.ckks_galois_element(ctx, off)) if off else None for t, off in enumerate(offs)]
    q_mac = q[:level + 1] + q[params.num_q:]
    masks = hx.from_host(uniform_residues((9, len(q_mac), N), q_mac, name + "masks"))
    w_real = conv_weights(wl.c_out, wl.c_in, dist="he_normal").reshape(wl.c_out, wl.c_in, 9)
    k = q[level] * 2.0 ** 10 / 2.0 ** 28
    w_int = np.where(w_real >= 0, np.floor(w_real * k + 0.5), np.ceil(w_real * k - 0.5)).astype(np.int64)
    w_res = hx.from_host(np.stack([np.mod(w_int, qi).astype(np.uint64) for qi in q_mac], axis=-1))
    outs = [hx.empty(2, level, N) for _ in range(wl.c_out)]
    mode = hx.HE_CONV_DEFERRED_MERGED
    ws = torch.empty(hx.he_conv_workspace_bytes(ctx, wl.c_in, wl.c_out, wl.height, wl.width, wl.batch, level, mode), dtype=torch.uint8, device="cuda")
    run = lambda: hx.he_conv_batched(ctx, wl.height, wl.width, wl.batch, level, ins, keys, masks, w_res, wl.c_out, outs=outs, ws=ws,
                                     alignment=mode, weight_bits=hx.conv_weight_bits(w_int))
    run()
    torch.cuda.synchronize()
    reps = 5
    t0 = time.perf_counter()
    for _ in range(reps):
        run()
    torch.cuda.synchronize()
    ms = (time.perf_counter() - t0) / reps * 1e3
    result["conv_" + name] = {"ms_per_layer": ms, "ms_per_image": ms / wl.batch, "c_in": wl.c_in, "c_out": wl.c_out,
                              "image": "%dx%d" % (wl.height, wl.width), "batch": wl.batch, "limbs": params.num_q,
                              "special_primes": params.num_p, "schedule": "deferred_merged"}


def ntt_microbench(hx, torch, result, bits=50):
    from workloads import CONFIGS, make_params, uniform_residues
    # NTT microbenchmark: 64 polynomials x 30 limbs at N = 2^16, forward then inverse
    w2 = CONFIGS["cfg2_ntt"]
    p2 = make_params(w2.log_n, w2.num_q, w2.num_p, w2.dnum, bits=bits)
    ctx2 = hx.Context(p2)
    polys = hx.from_host(uniform_residues((64, p2.num_q, p2.n), p2.moduli, "cfg2"))
    idx2 = list(range(p2.num_q))
    hx.ckks_ntt_fwd(ctx2, polys, idx2)
    hx.ckks_ntt_inv(ctx2, polys, idx2)
    torch.cuda.synchronize()
    reps = 5
    t0 = time.perf_counter()
    for _ in range(reps):
        hx.ckks_ntt_fwd(ctx2, polys, idx2)
        hx.ckks_ntt_inv(ctx2, polys, idx2)
    torch.cuda.synchronize()
    dt = time.perf_counter() - t0
    result["ntt_limbs_per_s"] = 2 * 64 * p2.num_q * reps / dt          # forward and inverse limb transforms
    result["ntt_butterflies_per_s"] = result["ntt_limbs_per_s"] * (p2.n // 2) * p2.log_n


def fc_bench(hx, torch, ctx, params, ins, masks, base_keys, level, N, result):
    # batched fully connected layer at the classifier's shape: 64 -> 10 on 512 images (all N/2 slots), level 3,
    # base = ceil(sqrt(512)); every one of its 59 rotations has a key tensor of its own (random residues)
    fc_in, fc_out, fc_batch, fc_level, fc_base = 64, 10, 512, 3, 23
    fc_delta = fc_in - fc_out
    fc_offs = [[1 << t for t in range(6)], [-i for i in range(fc_out)], [l * fc_delta for l in range(fc_base)],
               [h * fc_base * fc_delta for h in range(-(-fc_batch // fc_base))]]
    fc_keys = [[None if r % (N // 2) == 0 else
                hx.ckks_key_load(ctx, base_keys[(7 * i + j) % len(base_keys)].tensor.clone(), hx.ckks_galois_element(ctx, r))
                for j, r in enumerate(offs)] for i, offs in enumerate(fc_offs)]
    fc_ct = ins[0][:, :fc_level + 1].contiguous()
    fc_w = torch.stack([masks[i % 9, :fc_level + 1] for i in range(fc_out)]).contiguous()
    fc_mm = masks[0, :fc_level].contiguous()
    fc_pm = torch.stack([masks[i % 9, :fc_level - 1] for i in range(fc_batch)]).contiguous()
    fc_b = masks[1, :fc_level - 2].contiguous()
    fc_o = hx.empty(2, fc_level - 2, N)
    fc_ws = hx.empty(hx.he_fc_workspace_bytes(ctx, fc_in, fc_out, fc_batch, fc_level, fc_base) // 8)
    run_fc = lambda: hx.he_fc_batched(ctx, fc_ct, fc_level, fc_in, fc_out, fc_batch, fc_base, fc_w, fc_mm, fc_pm, fc_b,
                                      *fc_keys, out=fc_o, ws=fc_ws)
    run_fc()
    torch.cuda.synchronize()
    reps = 10
    t0 = time.perf_counter()
    for _ in range(reps):
        run_fc()
    torch.cuda.synchronize()
    fc_dt = (time.perf_counter() - t0) / reps
    result["fc_layer_ms"] = fc_dt * 1e3
    result["fc_layer_ms_per_image"] = fc_dt * 1e3 / fc_batch
    result["fc_layer_shape"] = {"d_in": fc_in, "d_out": fc_out, "batch": fc_batch, "level": fc_level, "base": fc_base,
                                "key_switches": sum(k is not None for ks in fc_keys for k in ks) + (fc_out - 1) * 6}
    del fc_keys, fc_ws


def downsample_bench(hx, torch, ctx, params, ins, masks, base_keys, level, N, result):
    # down-sampling compaction at the stage-2 -> stage-3 transition: 64 channel ciphertexts of 128 images of 16x16 -> 8x8, at
    # the level the slice ends on.  Two re-layouts (inside the images, then whole images), in two configurations:
    #   direct    8 + 8 and 12 + 11 offsets, every rotation divided by P on its own (35 keys)
    #   deferred  16 + 4 and 32 + 4 offsets, divisions after the sums: first rotations are inner products only (52 keys)
    ds_level, ds_n, kp = level - 5, 64, params.num_p
    ds_in = [hx.empty(2, ds_level + 1, N).copy_(ins[i % len(ins)][:, :ds_level + 1]) for i in range(ds_n)]
    ds_plans = {
        "direct": (hx.HE_RELAYOUT_DIRECT, [([x for x in range(8)], [y * 24 for y in range(8)], 64),
                                            ([l * 192 for l in range(12)], [h * 12 * 192 for h in range(11)], 128)]),
        "deferred": (hx.HE_RELAYOUT_DEFERRED, [([y * 24 + x for y in range(2) for x in range(8)], [h * 48 for h in range(4)], 64),
                                                ([l * 192 for l in range(32)], [h * 32 * 192 for h in range(4)], 128)]),
    }
    for name, (sched, stages) in ds_plans.items():
        ds_ws = hx.empty(max(hx.he_relayout_workspace_bytes(ctx, ds_level - k, ds_n, len(lo), len(hi), sched)
                             for k, (lo, hi, _) in enumerate(stages)) // 8)
        ds_args = []
        for k, (lo, hi, n_pairs) in enumerate(stages):
            lv = ds_level - k
            mk = lambda offs, salt: [None if r % (N // 2) == 0 else
                                     hx.ckks_key_load(ctx, base_keys[(salt + j) % len(base_keys)].tensor.clone(), hx.ckks_galois_element(ctx, r))
                                     for j, r in enumerate(offs)]
            if sched == hx.HE_RELAYOUT_DEFERRED:   # masks on the extended basis: the live q-limbs, then the special primes
                pool = [torch.cat([masks[i, :lv + 1], masks[i, level + 1:level + 1 + kp]]).contiguous() for i in range(9)]
            else:
                pool = [masks[i, :lv + 1].contiguous() for i in range(9)]
            ms = [[(pool[(h * len(lo) + l) % 9] if h * len(lo) + l < n_pairs else None) for l in range(len(lo))] for h in range(len(hi))]
            ds_args.append((lv, lo, mk(lo, 3 * k), hi, mk(hi, 3 * k + 5), ms, [hx.empty(2, lv, N) for _ in range(ds_n)]))

        def run_ds():
            cur = ds_in
            for lv, lo, lk, hi, hk, ms, outs in ds_args:
                cur = hx.he_relayout_two_rotations(ctx, cur, lv, lo, lk, hi, hk, ms, schedule=sched, outs=outs, ws=ds_ws)
        run_ds()
        torch.cuda.synchronize()
        reps = 3
        t0 = time.perf_counter()
        for _ in range(reps):
            run_ds()
        torch.cuda.synchronize()
        ds_dt = (time.perf_counter() - t0) / reps
        result["downsample_%s" % name] = {
            "ms": ds_dt * 1e3, "ms_per_image": ds_dt * 1e3 / 128, "offsets": [[len(lo), len(hi)] for lo, hi, _ in stages],
            "keys": sum(1 for lo, hi, _ in stages for r in lo + hi if r % (N // 2)),
            "inner_products": ds_n * sum(1 for lo, hi, _ in stages for r in lo + hi if r % (N // 2))}
        del ds_args, ds_ws
    result["downsample_shape"] = {"channels": ds_n, "from": "16x16", "to": "8x8", "batch": 128, "level": ds_level}
    del ds_in


def main():
    args = parse_args()
    if args.gpus != 1:
        print("bench.py measures one GPU: this build has no multi-GPU path (run with --gpus 1)", file=sys.stderr)
        sys.exit(2)
    import torch
    if not torch.cuda.is_available():
        print("bench.py needs a GPU", file=sys.stderr)
        sys.exit(2)
    import paper_2604_16834_amd as hx
    from workloads import CONFIGS, conv_tap_offsets, uniform_residues

    if args.ntt_only:
        result = {"workload": "cfg2_ntt (the NTT microbenchmark of the default run)", "prime_bits": args.prime_bits}
        ntt_microbench(hx, torch, result, bits=args.prime_bits)
        print(json.dumps(result))
        return
    wl = CONFIGS[args.workload]
    params = wl.params()
    if args.prime_bits != 50:   # other prime sizes (the integer kernels above 2^50) for the microbenchmark-only runs
        from workloads import make_params
        params = make_params(wl.log_n, wl.num_q, wl.num_p, wl.dnum, bits=args.prime_bits)
    ctx = hx.Context(params)
    N, level, q = params.n, params.num_q - 1, params.moduli
    M = params.num_q + params.num_p
    t_setup = time.perf_counter()
    ins = [hx.from_host(uniform_residues((2, level + 1, N), q[:level + 1], "in%d" % c)) for c in range(wl.c_in)]
    offs = conv_tap_offsets(wl.width)
    keys = [hx.ckks_key_load(ctx, hx.from_host(uniform_residues((params.dnum, 2, M, N), q, "rk%d" % t)),
                             hx.ckks_galois_element(ctx, off)) if off else None for t, off in enumerate(offs)]
    rlk = hx.ckks_key_load(ctx, hx.from_host(uniform_residues((params.dnum, 2, M, N), q, "rlk")), 0)
    mode = {"direct": hx.HE_CONV_ALIGN_DIRECT, "four_keys": hx.HE_CONV_ALIGN_FOUR_KEYS, "deferred": hx.HE_CONV_DEFERRED_MODDOWN,
            "deferred_merged": hx.HE_CONV_DEFERRED_MERGED}[args.alignment]
    deferred = args.alignment.startswith("deferred")
    act_merged = not args.two_step_activation
    # operands of the multiply-accumulate live on the extended basis (q_0..q_level, p_0..) in the deferred schedule
    q_mac = (q[:level + 1] + q[params.num_q:]) if deferred else q[:level + 1]
    masks = hx.from_host(uniform_residues((9, len(q_mac), N), q_mac, "masks"))
    # integer weights as the layer has them: N(0, 2 / (9 C_in)) kernels times the weight scale q_level 2^10 / 2^28 (the
    # convolution's output then lands at scale 2^50), rounded: 31-bit integers, given by their residues
    import numpy as np
    from workloads import conv_weights
    w_real = conv_weights(wl.c_out, wl.c_in, dist="he_normal").reshape(wl.c_out, wl.c_in, 9)
    w_int = np.where(w_real >= 0, np.floor(w_real * (q[level] * 2.0 ** 10 / 2.0 ** 28) + 0.5), np.ceil(w_real * (q[level] * 2.0 ** 10 / 2.0 ** 28) - 0.5)).astype(np.int64)
    weight_bits = 0 if args.wide_weights else hx.conv_weight_bits(w_int)
    w_res = hx.from_host(np.stack([np.mod(w_int, qi).astype(np.uint64) for qi in q_mac], axis=-1))
    conv_out = [hx.empty(2, level, N) for _ in range(wl.c_out)]
    act_out = [hx.empty(2, level - 4, N) for _ in range(wl.c_out)]
    k_act = (3 << 40, -(5 << 40), 7 << 40, -(9 << 40))
    ws_bytes = max(hx.he_conv_workspace_bytes(ctx, wl.c_in, wl.c_out, wl.height, wl.width, wl.batch, level, mode),
                   hx.ckks_workspace_bytes(ctx, hx.binding.CKKS_OP_POLY_ACT, level - 1, wl.c_out))
    ws = torch.empty(ws_bytes, dtype=torch.uint8, device="cuda")
    torch.cuda.synchronize()
    print("[bench] setup %.1f s, workspace %.2f GiB" % (time.perf_counter() - t_setup, ws_bytes / 2**30), file=sys.stderr, flush=True)

    if args.fc_only or args.downsample_only:
        result = {"workload": "fc layer 64 -> 10 x 512 images at level 3" if args.fc_only else "down-sampling compaction 64 channels x 128 images 16x16 -> 8x8"}
        base_keys = [k for k in keys if k is not None]
        hx.ckks_ctx_set_overlap(ctx, not args.single_stream)
        (fc_bench if args.fc_only else downsample_bench)(hx, torch, ctx, params, ins, masks, base_keys, level, N, result)
        print(json.dumps(result))
        return
    if args.rotations_only:
        result = {"workload": "cfg3_rotations (the rotation microbenchmark of the default run)", "single_stream": bool(args.single_stream),
                  "prime_bits": args.prime_bits}
        rotation_microbench(hx, torch, ctx, ins[0], keys, level, N, ws, result, overlap=not args.single_stream)
        print(json.dumps(result))
        return

    def step():
        hx.he_conv_batched(ctx, wl.height, wl.width, wl.batch, level, ins, keys, masks, w_res, wl.c_out, outs=conv_out, ws=ws,
                           alignment=mode, weight_bits=weight_bits)
        hx.he_poly_act_deg7(ctx, conv_out, level - 1, k_act, rlk, outs=act_out, ws=ws, merged=act_merged)

    if args.single_stream:
        hx.ckks_ctx_set_overlap(ctx, False)
    for _ in range(args.warmup):
        step()
    # exactly K steps between two synchronisations; every step also sits between two HIP events on the caller's stream (no
    # host synchronisation inside), which give the per-step median
    evs = [torch.cuda.Event(enable_timing=True) for _ in range(args.steps + 1)]
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    evs[0].record()
    for i in range(args.steps):
        step()
        evs[i + 1].record()
    torch.cuda.synchronize()
    elapsed = time.perf_counter() - t0
    step_ms = sorted(evs[i].elapsed_time(evs[i + 1]) for i in range(args.steps))
    ms_median = step_ms[len(step_ms) // 2] if len(step_ms) % 2 else 0.5 * (step_ms[len(step_ms) // 2 - 1] + step_ms[len(step_ms) // 2])
    # the same K steps with every launch on the caller's stream: the per-kernel timings below are taken that way, because
    # the duration of a launch that shares the chip with a launch of another batch is not a property of its kernel
    hx.ckks_ctx_set_overlap(ctx, False)
    step()
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(args.steps):
        step()
    torch.cuda.synchronize()
    ms_single = (time.perf_counter() - t0) * 1e3 / args.steps
    ms_per_step = elapsed * 1e3 / args.steps
    print("[bench] %d steps, %.2f ms/step" % (args.steps, ms_per_step), file=sys.stderr, flush=True)

    n_rot = wl.c_in * 8
    n_keyswitch = n_rot + 4 * wl.c_out
    result = {
        "metric": "keyswitch rotations/s + amortised HE-conv ms/image at N=2^16; % peak HBM GB/s",
        "value": ms_per_step / wl.batch,
        "unit": "ms/image (amortised, conv 64->64 3x3 + degree-7 activation, batch 512)",
        "n_gpus": 1, "steps": args.steps, "warmup": args.warmup, "ms_per_step": ms_per_step,
        "higher_is_better": False, "scaling": "weak", "vs_baseline": None,
        "dtype": "u64 residues; fp64-exact butterflies and conversions; int8 MFMA digit products", "data": "synthetic",
        "config": {"workload": wl.name, "log_n": params.log_n, "limbs": params.num_q, "special_primes": params.num_p,
                   "dnum": params.dnum, "c_in": wl.c_in, "c_out": wl.c_out, "image": "%dx%d" % (wl.height, wl.width),
                   "batch": wl.batch, "rotations_per_step": n_rot, "keyswitches_per_step": n_keyswitch,
                   "conv_schedule": args.alignment, "activation": "merged_division" if act_merged else "two_step",
                   "channel_batches_overlap": not args.single_stream, "weight_bits": weight_bits},
        "ms_per_step_median_events": ms_median, "ms_per_step_min_events": step_ms[0], "ms_per_step_max_events": step_ms[-1],
        "ms_per_step_single_stream": ms_single,
        "kernel_timing": "per-kernel figures and the roofline are measured with all work on one stream (no overlap between channel batches)",
    }

    # per-kernel event timing over one more step (every launch bracketed on its own stream)
    if not args.no_kernel_timing:
        hx.ckks_prof_begin(ctx, None, max_launches=1 << 16)
        step()
        prof = hx.ckks_prof_end(ctx)
        dropped = prof.pop("dropped")
        total = sum(v["ms"] for v in prof.values())
        kernels = {}
        for name, v in sorted(prof.items(), key=lambda kv: -kv[1]["ms"]):
            kernels[name] = {"ms": round(v["ms"], 3), "launches": v["launches"], "avg_us": round(1e3 * v["ms"] / v["launches"], 2),
                             "GB/s": round(v["bytes"] / v["ms"] / 1e6, 1), "Gops/s": round(v["ops"] / v["ms"] / 1e6, 1)}
        result["kernels"] = kernels
        result["kernel_ms_total"] = round(total, 2)
        result["kernel_events_dropped"] = dropped
        dom = next(iter(kernels))
        # the dominant kernel class again, now bracketed inside a timed run of the same K steps
        hx.ckks_prof_begin(ctx, [dom], max_launches=1 << 16)
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for _ in range(args.steps):
            step()
        torch.cuda.synchronize()
        result["ms_per_step_with_events"] = (time.perf_counter() - t0) * 1e3 / args.steps
        v = hx.ckks_prof_end(ctx)[dom]
        secs = v["ms"] * 1e-3
        traffic = measured_traffic(dom)
        roof = {"kernel": dom, "launches": v["launches"], "avg_us": 1e6 * secs / v["launches"],
                "algorithmic_bytes_per_launch": v["bytes"] / v["launches"], "traffic": traffic,
                "traffic_source": "profiles/pmc_traffic_cfg5_block_slice.txt as committed (rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE scaled by a "
                                  "copy of known size); read from that file, not re-measured by this run",
                "hbm_GBs": v["bytes"] / secs / 1e9}
        if dom in MFMA_KERNELS:
            per, peak_ops = MFMA_KERNELS[dom]
            ach = v["ops"] * per / secs / 1e12
            roof.update({"bound": "mfma", "achieved": ach, "peak": peak_ops / 1e12, "unit": "TOP/s (int8)", "frac": ach / (peak_ops / 1e12)})
        elif dom in ALU_KERNELS:
            lane_ops, unit = ALU_KERNELS[dom]
            peak = ALU_PEAK_LANE_OPS / lane_ops / 1e9
            ach = v["ops"] / secs / 1e9
            hbm = v["bytes"] / secs / 1e9
            if hbm / HBM_PEAK_GBS > ach / peak:   # the roofline that binds is the one the kernel sits closer to
                roof.update({"bound": "hbm", "achieved": hbm, "peak": HBM_PEAK_GBS, "unit": "GB/s", "frac": hbm / HBM_PEAK_GBS,
                             "alu": {"achieved": ach, "peak": peak, "unit": unit, "frac": ach / peak}})
            else:
                roof.update({"bound": "alu", "achieved": ach, "peak": peak, "unit": unit, "frac": ach / peak,
                             "hbm": {"achieved": hbm, "peak": HBM_PEAK_GBS, "unit": "GB/s", "frac": hbm / HBM_PEAK_GBS}})
        else:
            ach = v["bytes"] / secs / 1e9
            roof.update({"bound": "hbm", "achieved": ach, "peak": HBM_PEAK_GBS, "unit": "GB/s", "frac": ach / HBM_PEAK_GBS})
        result["roofline"] = roof
        if "key_inner" in prof:   # the key inner products of the step, bracketed alone in K more steps (no other event pairs in the stream)
            hx.ckks_prof_begin(ctx, ["key_inner"], max_launches=1 << 16)
            for _ in range(args.steps):
                step()
            ki = hx.ckks_prof_end(ctx)["key_inner"]
            ach = ki["bytes"] / (ki["ms"] * 1e-3) / 1e9
            result["key_inner_hbm"] = {"achieved_GBs": ach, "frac_of_peak": ach / HBM_PEAK_GBS, "avg_us": 1e3 * ki["ms"] / ki["launches"],
                                       "launches": ki["launches"], "algorithmic_bytes_per_launch": ki["bytes"] / ki["launches"],
                                       "traffic": measured_traffic("key_inner"), "traffic_source": "profiles/pmc_traffic_cfg5_block_slice.txt as committed"}
        # a plain device-to-device copy of 2 GiB (the runtime's own copy kernel): what a read-once / write-once stream reaches here
        cp_src = torch.empty(1 << 28, dtype=torch.int64, device="cuda")
        cp_dst = torch.empty_like(cp_src)
        cp_dst.copy_(cp_src)
        c0, c1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        c0.record()
        for _ in range(10):
            cp_dst.copy_(cp_src)
        c1.record()
        torch.cuda.synchronize()
        copy_gbs = 10 * 2 * cp_src.numel() * 8 / (c0.elapsed_time(c1) * 1e-3) / 1e9
        del cp_src, cp_dst
        result["copy_ceiling"] = {"GB/s": copy_gbs, "frac_of_peak": copy_gbs / HBM_PEAK_GBS, "what": "device-to-device copy of 2 GiB, read + write bytes"}
        if result["roofline"].get("bound") == "hbm" or "hbm" in result["roofline"]:
            hb = result["roofline"]["achieved"] if result["roofline"]["bound"] == "hbm" else result["roofline"]["hbm"]["achieved"]
            result["roofline"]["frac_of_copy_ceiling"] = hb / copy_gbs

    if not args.no_schedules:
        # the same step under the other readings of where the divisions by P go (three steps each, one warm-up)
        sched = {args.alignment: ms_per_step}
        modes = {"direct": hx.HE_CONV_ALIGN_DIRECT, "four_keys": hx.HE_CONV_ALIGN_FOUR_KEYS, "deferred": hx.HE_CONV_DEFERRED_MODDOWN,
                 "deferred_merged": hx.HE_CONV_DEFERRED_MERGED}
        hx.ckks_ctx_set_overlap(ctx, not args.single_stream)
        for name, m in modes.items():
            if name in sched:
                continue
            ext = name.startswith("deferred")
            qm = (q[:level + 1] + q[params.num_q:]) if ext else q[:level + 1]
            mk = masks if ext == deferred else hx.from_host(uniform_residues((9, len(qm), N), qm, "masks_" + name))
            wr = w_res if ext == deferred else hx.from_host(np.stack([np.mod(w_int, qi).astype(np.uint64) for qi in qm], axis=-1))
            need = hx.he_conv_workspace_bytes(ctx, wl.c_in, wl.c_out, wl.height, wl.width, wl.batch, level, m)
            wsm = ws if need <= ws.numel() else torch.empty(need, dtype=torch.uint8, device="cuda")

            def other_step():
                hx.he_conv_batched(ctx, wl.height, wl.width, wl.batch, level, ins, keys, mk, wr, wl.c_out, outs=conv_out, ws=wsm,
                                   alignment=m, weight_bits=weight_bits)
                hx.he_poly_act_deg7(ctx, conv_out, level - 1, k_act, rlk, outs=act_out, ws=ws, merged=act_merged)
            other_step()
            torch.cuda.synchronize()
            t0 = time.perf_counter()
            for _ in range(3):
                other_step()
            torch.cuda.synchronize()
            sched[name] = (time.perf_counter() - t0) * 1e3 / 3
            del mk, wr, wsm
        result["schedules_ms_per_step"] = sched
        result["schedules_note"] = ("same activation (%s) in every row; direct = one ModDown per rotation (the literal reading of Eqs. 10-11), four_keys = "
                                    "the paper's two-stage alignment with four keys, deferred = one ModDown per output channel, deferred_merged = "
                                    "that ModDown merged with the rescale" % ("merged_division" if act_merged else "two_step"))

    if args.calibration_copy:   # a rotation by 0 slots is a plain copy of the ciphertext
        cal = hx.empty(2, level + 1, N)
        for _ in range(3):
            hx.ckks_rotate_hoisted(ctx, ins[0], level, [0], [None], True, outs=[cal], ws=ws)
        torch.cuda.synchronize()
        result["calibration_copy_bytes_each_way"] = 2 * (level + 1) * N * 8
    if args.no_microbench:
        if not args.no_cpu_baseline:
            result["cpu_baseline"] = cpu_baseline(wl, params, args.alignment, act_merged)
        print(json.dumps(result))
        return
    # ---- the two microbenchmark shapes, reported next to the headline value ------------------------
    rotation_microbench(hx, torch, ctx, ins[0], keys, level, N, ws, result, overlap=not args.single_stream)
    hx.ckks_ctx_set_overlap(ctx, not args.single_stream)
    base_keys = [k for k in keys if k is not None]
    # accumulator merge (the optimised pipeline's block-group transition): 4 intermediate ciphertexts with 8192
    # occupied slots each -> one full ciphertext, at the level the block slice leaves its outputs on
    acc_level, acc_g, acc_sts = level - 5, 4, 8192
    acc_in = [t[:, :acc_level + 1].contiguous() for t in ins[:acc_g]]
    acc_keys = [None] + [hx.ckks_key_load(ctx, base_keys[i].tensor, hx.ckks_galois_element(ctx, -i * acc_sts)) for i in range(1, acc_g)]
    acc_mask = masks[0, :acc_level + 1].contiguous()
    acc_out = hx.empty(2, acc_level, N)
    hx.he_accumulator_merge(ctx, acc_in, acc_level, acc_sts, acc_mask, acc_keys, out=acc_out, ws=ws)
    torch.cuda.synchronize()
    reps = 20
    t0 = time.perf_counter()
    for _ in range(reps):
        hx.he_accumulator_merge(ctx, acc_in, acc_level, acc_sts, acc_mask, acc_keys, out=acc_out, ws=ws)
    torch.cuda.synchronize()
    result["accumulator_merges_per_s"] = reps / (time.perf_counter() - t0)
    result["accumulator_merge_shape"] = {"g": acc_g, "sts": acc_sts, "level": acc_level}
    fc_bench(hx, torch, ctx, params, ins, masks, base_keys, level, N, result)
    downsample_bench(hx, torch, ctx, params, ins, masks, base_keys, level, N, result)
    # key staging: the block group's 9 keys (8 rotations + relinearisation) as b halves in pinned host memory (48 MiB
    # each) + seeds, copied and expanded on a side stream, alone and while the block slice runs on the main stream
    n_stage = 9
    host_b = [torch.empty(params.dnum, params.num_q + params.num_p, N, dtype=torch.int64).pin_memory() for _ in range(n_stage)]
    for i, t in enumerate(host_b):
        t.copy_(base_keys[i % len(base_keys)].tensor.view(params.dnum, 2, -1, N)[:, 0])
    staged = [hx.empty(params.dnum, 2, params.num_q + params.num_p, N) for _ in range(n_stage)]
    side = torch.cuda.Stream()
    stage_bytes = sum(t.numel() * 8 for t in host_b)

    def stage_once():
        side.wait_stream(torch.cuda.current_stream())
        hx.ckks_keyset_stage(ctx, host_b, list(range(100, 100 + n_stage)), staged, stream=side.cuda_stream)
    stage_once()
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    stage_once()
    torch.cuda.synchronize()
    alone = time.perf_counter() - t0
    t0 = time.perf_counter()
    stage_once()
    for _ in range(2):               # two block-slice steps on the main stream while the side stream stages
        step()
    torch.cuda.synchronize()
    both_dt = time.perf_counter() - t0
    result["key_staging"] = {"keys": n_stage, "host_bytes": stage_bytes, "device_key_bytes": 2 * stage_bytes,
                             "ms_alone": alone * 1e3, "host_link_GBs": stage_bytes / alone / 1e9,
                             "ms_two_steps_while_staging": both_dt * 1e3, "ms_two_steps": 2 * ms_per_step,
                             "staging_ms_hidden": alone * 1e3 + 2 * ms_per_step - both_dt * 1e3}
    del host_b, staged
    ntt_microbench(hx, torch, result)
    # the convolution of the first ResNet-20 stage (16 -> 16 channels on 32 images of 32x32, 20 limbs + 7 special primes)
    conv_microbench(hx, torch, "cfg4_resnet20_stage1", result)

    if not args.no_cpu_baseline:
        result["cpu_baseline"] = cpu_baseline(wl, params, args.alignment, act_merged)
    print(json.dumps(result))


if __name__ == "__main__":
    main()
