#!/usr/bin/env python3
"""Benchmark of the ct-pt MAC + lazy-rescale hot path at N = 2^14, L = 8 on one MI355X.

One step = one pass of the whole path over the two N = 2^14, L = 8 workloads, each layer as ONE
he_ct_pt_mac(HE_RESCALE) call:
  cfg4  conv 32x32x3 -> 16x16x16, 3x3, stride 2, same padding, scalar plaintexts:
        scalar-encode the 432 weights and 16 biases (Alg. 2), MAC + bias (Alg. 8 / 4),
        one lazy rescale per output ciphertext (Eq. (2)): 4096 rescaled ciphertexts
  cfg5  dense 256 -> 64 with full-polynomial plaintexts (Alg. 7), one rescale per output: 64
Inputs are synthetic (uniform residues, Gaussian weights), generated on the device before the timed
region.  Prints ONE JSON line.
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0
# 256 CUs x 64 lanes x 2.4 GHz: one 32x32(+64)-bit integer multiply(-add) per lane per clock
INT_MUL32_PEAK_TOPS = 256 * 64 * 2.4e9 / 1e12
MUL32_PER_MAC = 4          # a 64x64 -> 128-bit product is four 32x32 -> 64 multiply-adds
MUL32_PER_SHOUP = 10       # hi64(y*w') 4, lo64(y*w) 3, lo64(qh*q) 3
# HBM-side bytes per launch (read + written) of the main kernels come from rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE
# runs of this benchmark, scaled by a plain kernel of known size: counters cannot be read from inside this
# process, so they are taken from the summary of those runs, profiles/hbm_traffic.json, which names the commit
# it was measured at.
GIB = 1 << 30
TRAFFIC_FILE = os.path.join(ROOT, "profiles", "hbm_traffic.json")


def profiled_traffic():
    """{kernel: bytes per launch} and where the figures come from (None, None if the summary is absent)."""
    try:
        with open(TRAFFIC_FILE) as f:
            d = json.load(f)
    except (OSError, ValueError):
        return {}, None
    per = {k: int(v["fetch_bytes"] + v["write_bytes"]) for k, v in d.get("kernels", {}).items()}
    return per, {"file": "profiles/hbm_traffic.json", "commit": d.get("commit"), "counters": "rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE"}


def main() -> int:
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=10)
    ap.add_argument("--warmup", type=int, default=3)
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--only", default="", help="comma-separated phases to run (profiling aid; the JSON is then partial)")
    ap.add_argument("--calibrate-copy", action="store_true",
                    help="also run three plain elementwise kernels over 2 GiB (counter calibration for rocprofv3 --pmc)")
    ap.add_argument("--no-rates", dest="rates", action="store_false",
                    help="skip the he_measure_rate probes (keeps a profiler's kernel list to the path's own kernels)")
    ap.add_argument("--no-compare-arithmetic", dest="compare_arithmetic", action="store_false",
                    help="skip the timing of cfg4's rescale with integer butterflies only (keeps a kernel trace's averages to the step's own launches)")
    ap.add_argument("--no-all-configs", dest="all_configs", action="store_false",
                    help="skip the per-config report of the five layers")
    ap.add_argument("--cpu-sample-cfg4", type=int, default=1024, help="cfg4 outputs the oracle is timed on")
    ap.add_argument("--cpu-sample-cfg5", type=int, default=32, help="cfg5 outputs the oracle is timed on")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build runs on one GPU only (--gpus 1); no multi-GPU figure exists", file=sys.stderr)
        return 2

    import numpy as np
    import torch
    from paper_1908_04172_amd import he, workloads as wl

    if not torch.cuda.is_available():
        print("bench.py: no GPU", file=sys.stderr)
        return 1
    he.lib()
    dev = "cuda"
    c4, c5 = wl.config(4), wl.config(5)
    assert c4.q == c5.q and c4.N == c5.N
    N, L, q = c4.N, c4.L, c4.q
    ctx = he.Context(c4.log2N, q, device=0)
    p4, p5 = c4.plan, c5.plan
    hp4 = ctx.plan(p4.n_in, p4.n_out, p4.n_pt, p4.off, p4.term_ct, p4.term_pt)
    hp5 = ctx.plan(p5.n_in, p5.n_out, p5.n_pt, p5.off, p5.term_ct, p5.term_pt)

    # ---- inputs, resident in HBM before anything is timed
    ct4 = wl.uniform_residues_torch((p4.n_in, 2), q, N, c4.seed, dev)
    w4 = torch.from_numpy(wl.normal_values(p4.n_pt, c4.sigma, c4.seed + 100)).to(dev)
    b4 = torch.from_numpy(wl.normal_values(p4.n_out, c4.sigma, c4.seed + 200)).to(dev)
    ct5 = wl.uniform_residues_torch((p5.n_in, 2), q, N, c5.seed, dev)
    pt5 = wl.uniform_residues_torch((p5.n_pt,), q, N, c5.seed + 100, dev)
    wenc4 = torch.empty((p4.n_pt, L), dtype=torch.int64, device=dev)
    benc4 = torch.empty((p4.n_out, L), dtype=torch.int64, device=dev)
    acc4 = torch.empty((p4.n_out, 2, L, N), dtype=torch.int64, device=dev)
    out4 = torch.empty((p4.n_out, 2, L - 1, N), dtype=torch.int64, device=dev)
    acc5 = torch.empty((p5.n_out, 2, L, N), dtype=torch.int64, device=dev)
    out5 = torch.empty((p5.n_out, 2, L - 1, N), dtype=torch.int64, device=dev)
    ws4 = torch.empty(max(hp4.workspace_bytes(L, he.PT_SCALAR, 0), 256), dtype=torch.uint8, device=dev)
    scale = 2.0 ** c4.log2_scale

    wsf4 = torch.empty(max(hp4.workspace_bytes(L, he.PT_SCALAR, he.RESCALE), 256), dtype=torch.uint8, device=dev)
    wsf5 = torch.empty(max(hp5.workspace_bytes(L, he.PT_POLY, he.RESCALE), 256), dtype=torch.uint8, device=dev)

    # The timed step is the path as a user calls it: the scalar encoding, then ONE he_ct_pt_mac(HE_RESCALE) per layer
    # (MAC + bias + one lazy rescale per output).  The kernels inside such a call are timed in a second loop, which
    # issues the same launches as two calls (he_test_mac_for_rescale, then he_rescale) with events between them.
    step_phases = ["encode_cfg4", "layer_cfg4", "layer_cfg5"]
    phases = ["encode_cfg4", "mac_scalar_cfg4", "rescale_cfg4", "mac_poly_cfg5", "rescale_cfg5"]

    only = set(filter(None, args.only.split(",")))
    assert only <= set(phases), phases
    on = lambda name: not only or name in only

    def step(ev=None):
        def mark(i):
            if ev is not None:
                ev[i].record()
        mark(0)
        ctx.encode_scalar(w4, scale, out=wenc4)
        ctx.encode_scalar(b4, scale, out=benc4)
        mark(1)
        ctx.ct_pt_mac(hp4, ct4, wenc4, he.PT_SCALAR, bias=benc4, flags=he.RESCALE, out=out4, workspace=wsf4)
        mark(2)
        ctx.ct_pt_mac(hp5, ct5, pt5, he.PT_POLY, flags=he.RESCALE, out=out5, workspace=wsf5)
        mark(3)

    def kernels(ev=None):
        def mark(i):
            if ev is not None:
                ev[i].record()
        mark(0)
        if on("encode_cfg4"):
            ctx.encode_scalar(w4, scale, out=wenc4)
            ctx.encode_scalar(b4, scale, out=benc4)
        mark(1)
        if on("mac_scalar_cfg4"):
            ctx.mac_for_rescale(hp4, ct4, wenc4, he.PT_SCALAR, acc4, bias=benc4, workspace=ws4)
        mark(2)
        if on("rescale_cfg4"):
            ctx.rescale(acc4, out=out4k)
        mark(3)
        if on("mac_poly_cfg5"):
            ctx.mac_for_rescale(hp5, ct5, pt5, he.PT_POLY, acc5)
        mark(4)
        if on("rescale_cfg5"):
            ctx.rescale(acc5, out=out5k)
        mark(5)

    out4k, out5k = torch.empty_like(out4), torch.empty_like(out5)
    if only:                       # buffers the skipped phases would have produced
        ctx.encode_scalar(w4, scale, out=wenc4)
        ctx.encode_scalar(b4, scale, out=benc4)
        acc4.zero_()
        acc5.zero_()

    if args.calibrate_copy:        # a plain elementwise kernel: reads 2 GiB and writes 2 GiB per launch
        src = ct4[:1024]
        dst = torch.empty_like(src)
        for _ in range(3):
            torch.add(src, 1, out=dst)
        del dst
    step_ms = {}
    if not only:
        for _ in range(args.warmup):
            step()
        torch.cuda.synchronize()
        events = [[torch.cuda.Event(enable_timing=True) for _ in range(4)] for _ in range(args.steps)]
        t0 = time.perf_counter()
        for k in range(args.steps):
            step(events[k])
        torch.cuda.synchronize()
        wall = time.perf_counter() - t0
        ms_per_step = wall * 1e3 / args.steps
        step_ms = {name: float(np.median([events[k][i].elapsed_time(events[k][i + 1]) for k in range(args.steps)]))
                   for i, name in enumerate(step_phases)}
    for _ in range(args.warmup):
        kernels()
    torch.cuda.synchronize()
    events = [[torch.cuda.Event(enable_timing=True) for _ in range(6)] for _ in range(args.steps)]
    t0 = time.perf_counter()
    for k in range(args.steps):
        kernels(events[k])
    torch.cuda.synchronize()
    if only:
        ms_per_step = (time.perf_counter() - t0) * 1e3 / args.steps
    phase_ms = {name: float(np.median([events[k][i].elapsed_time(events[k][i + 1]) for k in range(args.steps)]))
                for i, name in enumerate(phases)}
    # the two-call form issues the launches of the one-call form: the same residues, bit for bit
    same_as_one_call = bool(only) or bool(torch.equal(out4k, out4) and torch.equal(out5k, out5))
    traffic, traffic_source = profiled_traffic()

    # ---- algorithmic work (per step)
    ct_bytes = 2 * L * N * 8
    out_bytes = 2 * (L - 1) * N * 8
    bytes4 = p4.n_in * ct_bytes + p4.n_out * out_bytes + (p4.n_pt + p4.n_out) * (8 + 8 * L)
    bytes5 = p5.n_pt * L * N * 8 + p5.n_in * ct_bytes + p5.n_out * out_bytes
    total_bytes = bytes4 + bytes5
    n_rescaled = p4.n_out + p5.n_out
    value = total_bytes / (ms_per_step * 1e-3) / 1e9

    def rescale_mul32(n_ct):
        butterflies = n_ct * 2 * L * (N // 2) * c4.log2N          # one INTT + L-1 NTTs per polynomial
        return (butterflies + n_ct * 2 * (L - 1) * N) * MUL32_PER_SHOUP
    rooflines = {}
    macs4 = p4.n_terms * 2 * L * N
    macs5 = p5.n_terms * 2 * L * N
    def alu(name, mul32):
        a = mul32 / (phase_ms[name] * 1e-3) / 1e12
        return {"kernel": name, "bound": "alu", "achieved": a, "peak": INT_MUL32_PEAK_TOPS, "unit": "Tmul32/s",
                "frac": a / INT_MUL32_PEAK_TOPS, "traffic": traffic.get(name)}
    def hbm(name, nbytes):
        a = nbytes / (phase_ms[name] * 1e-3) / 1e9
        return {"kernel": name, "bound": "hbm", "achieved": a, "peak": HBM_PEAK_GBS, "unit": "GB/s",
                "frac": a / HBM_PEAK_GBS, "traffic": traffic.get(name)}
    rooflines["mac_scalar_cfg4"] = alu("mac_scalar_cfg4", macs4 * MUL32_PER_MAC)   # the four-product definition of a term
    rooflines["rescale_cfg4"] = alu("rescale_cfg4", rescale_mul32(p4.n_out))
    # the full-polynomial MAC streams every plaintext residue once: HBM-bound
    mac5_bytes = p5.n_pt * L * N * 8 + p5.n_in * ct_bytes + p5.n_out * ct_bytes
    rooflines["mac_poly_cfg5"] = hbm("mac_poly_cfg5", mac5_bytes)
    rooflines["rescale_cfg5"] = alu("rescale_cfg5", rescale_mul32(p5.n_out))
    dominant = max(rooflines, key=lambda k: phase_ms[k])

    # ---- the same kernels against MEASURED register-resident rates of their own primitives
    # (he_measure_rate): time the arithmetic alone would take at that rate / time the kernel took
    rate_cache = {}
    def rate(kind, limb):
        if (kind, limb) not in rate_cache:
            rate_cache[(kind, limb)] = ctx.measure_rate(kind, limb) if args.rates and not only else float('nan')
        return rate_cache[(kind, limb)]
    mode = [2 if qi < (1 << 58) else 1 if qi < (1 << 61) else 0 for qi in q]
    fwd_kind = {0: he.RATE_BUTTERFLY_MODE0, 1: he.RATE_BUTTERFLY_MODE1, 2: he.RATE_BUTTERFLY_MODE2}
    bf = (N // 2) * c4.log2N
    def rescale_ideal_s(n_ct):
        # limbs below 2^50 are transformed on double-precision FMAs (forward: when the dropped modulus is at most twice theirs)
        last = L - 1
        fp = [qi < (1 << 50) for qi in q]
        inv = he.RATE_BUTTERFLY_FP64_INV if fp[last] else he.RATE_BUTTERFLY_INV if mode[last] else he.RATE_BUTTERFLY_MODE0
        per_poly = bf / rate(inv, last)
        for i in range(last):
            fwd = he.RATE_BUTTERFLY_FP64 if fp[i] and q[last] <= 2 * q[i] else fwd_kind[mode[i]]
            per_poly += bf / rate(fwd, i) + N / rate(he.RATE_SHOUP_EXACT, i)
        return 2 * n_ct * per_poly
    # the scalar MAC runs the three-product form of a term on the limbs that leave room for it
    three = [he.host_mac_three_product_terms(qi) >= max(int(x) for x in np.diff(p4.off.astype(np.int64))) for qi in q]
    def mac_ideal_s(plan, scalar):
        return sum(plan.n_terms * 2 * N / rate(he.RATE_MAC_TERM3 if scalar and three[i] else he.RATE_MAC_TERM, i) for i in range(L))
    ideal = {"mac_scalar_cfg4": mac_ideal_s(p4, True), "rescale_cfg4": rescale_ideal_s(p4.n_out),
             "mac_poly_cfg5": mac_ideal_s(p5, False), "rescale_cfg5": rescale_ideal_s(p5.n_out)}
    for name, r in rooflines.items():
        if args.rates and not only:
            r["arithmetic_ms_at_measured_rate"] = ideal[name] * 1e3
            r["frac_of_measured_rate"] = ideal[name] * 1e3 / phase_ms[name]
    names = ["mad32", "mac_term", "shoup_exact", "shoup_cheap", "butterfly_mode0", "butterfly_mode1",
             "butterfly_mode2", "butterfly_inverse", "mac_term_three_products", "butterfly_fp64", "butterfly_fp64_inverse"]
    measured_rates = {"unit": "G operations/s, register-resident, whole GPU",
                      "rates": {"%s@%dbit" % (names[k], q[limb].bit_length()): v / 1e9
                                for (k, limb), v in sorted(rate_cache.items(), reverse=True)}}

    result = {
        "metric": "ct-pt MAC GB/s (% HBM peak) + rescaled ciphertexts/sec at N=2^14, L=8",
        "value": value, "unit": "GB/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": ms_per_step, "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "u64", "data": "synthetic",
        "config": {"workload": "cfg4 (conv 32x32x3->16x16x16 3x3 s2 same, scalar pt: encode+MAC+bias+lazy rescale, "
                               "4096 outputs) + cfg5 (dense 256->64, full-poly pt: MAC+lazy rescale, 64 outputs), "
                               "N=2^14, L=8 (2x60-bit + 6x50-bit)",
                   "value_definition": "algorithmic bytes of the step (inputs once + outputs once) / step time",
                   "arithmetic": "residues are uint64; MAC, bias add and the rescale's combine step on 32-bit integer multiply-adds; "
                                 "the transforms of the 50-bit limbs on double-precision FMAs, those of the 60-bit limbs on integer "
                                 "Shoup butterflies (identical residues either way)",
                   "algorithmic_bytes_per_step": total_bytes},
        "pct_hbm_peak": 100.0 * value / HBM_PEAK_GBS,
        "rescaled_ct_per_s": n_rescaled / (ms_per_step * 1e-3),
        "rescale_only_ct_per_s": n_rescaled / ((phase_ms["rescale_cfg4"] + phase_ms["rescale_cfg5"]) * 1e-3),
        "mac_poly_cfg5_GBps": rooflines["mac_poly_cfg5"]["achieved"],
        "mac_poly_cfg5_pct_hbm_peak": 100.0 * rooflines["mac_poly_cfg5"]["frac"],
        "mac_scalar_cfg4_Tmac_per_s": macs4 / (phase_ms["mac_scalar_cfg4"] * 1e-3) / 1e12,
        "mac_poly_cfg5_Tmac_per_s": macs5 / (phase_ms["mac_poly_cfg5"] * 1e-3) / 1e12,
        "phase_ms": step_ms,
        "kernel_ms": phase_ms,
        "kernel_ms_what": "the launches of the two layer calls issued as he_test_mac_for_rescale + he_rescale with events between "
                          "them (median over the steps); outputs equal to the one-call form: %s" % same_as_one_call,
        "roofline": {k: v for k, v in rooflines[dominant].items()},
        "roofline_all": list(rooflines.values()),
        "traffic_source": traffic_source,
        "measured_rates": measured_rates if args.rates else None,
    }

    # ---- the oracle on the host cores, on a bounded sample of the same workload (before anything
    # below touches the inputs of the timed step)
    if only:
        result["partial"] = sorted(only)
    if not args.no_cpu_baseline and not only:
        import oracle
        threads = oracle.set_threads(0)
        psi = ctx.psi
        to_host = lambda t: t.cpu().numpy().view(np.uint64)
        idx = lambda t, ids: t[torch.as_tensor(np.asarray(ids, dtype=np.int64), device=t.device)]

        def compact(plan, outs):
            sub = plan.subset(outs)
            ct_ids, ct_inv = np.unique(sub.term_ct, return_inverse=True)
            pt_ids, pt_inv = np.unique(sub.term_pt, return_inverse=True)
            return sub.off, ct_inv.astype(np.uint32), pt_inv.astype(np.uint32), ct_ids, pt_ids

        s4 = list(range(0, p4.n_out, max(1, p4.n_out // args.cpu_sample_cfg4)))[: args.cpu_sample_cfg4]
        off, tc, tp, ct_ids, pt_ids = compact(p4, s4)
        h_ct, h_w, h_b = to_host(idx(ct4, ct_ids)), w4.cpu().numpy(), b4.cpu().numpy()
        t = time.perf_counter()
        wenc = oracle.encode_scalars(h_w, scale, q)
        benc = oracle.encode_scalars(h_b, scale, q)
        want4, _ = oracle.layer(h_ct, q, psi, off, tc, tp, wenc[pt_ids], oracle.PT_SCALAR, benc[s4])
        t4 = time.perf_counter() - t
        s5 = list(range(args.cpu_sample_cfg5))
        off, tc, tp, ct_ids, pt_ids = compact(p5, s5)
        h_ct, h_pt = to_host(idx(ct5, ct_ids)), to_host(idx(pt5, pt_ids))
        t = time.perf_counter()
        want5, _ = oracle.layer(h_ct, q, psi, off, tc, tp, h_pt, oracle.PT_POLY, None)
        t5 = time.perf_counter() - t
        # the timed GPU outputs must be the oracle's, bit for bit
        ok = np.array_equal(to_host(idx(out4, s4)), want4) and np.array_equal(to_host(idx(out5, s5)), want5)
        cpu_step_s = t4 * p4.n_out / len(s4) + t5 * p5.n_out / len(s5)
        # the serial program (one thread) on a few cfg4 outputs: the paper's single-operation tables are
        # single-threaded
        n1 = min(16, len(s4))
        off1, tc1, tp1, ct_ids1, pt_ids1 = compact(p4, s4[:n1])
        h_ct1 = to_host(idx(ct4, ct_ids1))
        oracle.set_threads(1)
        t = time.perf_counter()
        oracle.layer(h_ct1, q, psi, off1, tc1, tp1, wenc[pt_ids1], oracle.PT_SCALAR, benc[s4[:n1]])
        t1 = time.perf_counter() - t
        oracle.set_threads(0)
        result["cpu_baseline"] = {
            "one_thread_rescaled_ct_per_s": n1 / t1,
            "one_thread_sample": "%d cfg4 outputs (MAC of up to 27 terms + bias + rescale each), %.1f s" % (n1, t1),
            "value": total_bytes / cpu_step_s / 1e9, "unit": "GB/s", "cores": threads, "kind": "oracle",
            "sample": "%d of %d cfg4 outputs (%.1f s) + %d of %d cfg5 outputs (%.1f s), extrapolated linearly to "
                      "the whole step" % (len(s4), p4.n_out, t4, len(s5), p5.n_out, t5),
            "rescaled_ct_per_s": n_rescaled / cpu_step_s, "gpu_outputs_match_oracle": bool(ok)}
    # ---- the two plainly HBM-bound calls of the path, outside the timed step: Alg. 4 (scalar add, in
    # place on component 0) and Alg. 8 as one multiply per output (every ciphertext read once, written once)
    if not only:
        def timed(fn, reps=5):
            fn()
            torch.cuda.synchronize()
            ev = [torch.cuda.Event(enable_timing=True) for _ in range(reps + 1)]
            ev[0].record()
            for i in range(reps):
                fn()
                ev[i + 1].record()
            torch.cuda.synchronize()
            return float(np.mean([ev[i].elapsed_time(ev[i + 1]) for i in range(reps)]))
        # the copy ceiling of this machine, by the library every tensor here comes from: 2 GiB read + 2 GiB written
        cp_src, cp_dst = ct4[:1024], acc4[:1024]
        ms_copy = timed(lambda: cp_dst.copy_(cp_src))
        result["measured_copy_GBps"] = 2 * cp_src.numel() * 8 / (ms_copy * 1e-3) / 1e9
        n_add = p4.n_in
        pt_add = ctx.encode_scalar(torch.from_numpy(wl.normal_values(n_add, 0.1, 7)).to(dev), scale)
        ms_add = timed(lambda: ctx.ct_pt_add(ct4, pt_add, he.PT_SCALAR))
        add_bytes = n_add * L * N * 8 * 2                       # component 0 read + written
        n_str = 1024
        ids = np.arange(n_str, dtype=np.uint32)
        hps = ctx.plan(n_str, n_str, n_str, np.arange(n_str + 1, dtype=np.uint32), ids, ids)
        w_str = ctx.encode_scalar(torch.from_numpy(wl.normal_values(n_str, 0.1, 8)).to(dev), scale)
        ws_str = torch.empty(max(hps.workspace_bytes(L, he.PT_SCALAR, 0), 256), dtype=torch.uint8, device=dev)
        ms_str = timed(lambda: ctx.ct_pt_mac(hps, ct4[:n_str], w_str, he.PT_SCALAR, out=acc4[:n_str], workspace=ws_str))
        str_bytes = n_str * ct_bytes * 2
        result["hbm_bound_calls"] = {
            "ct_pt_add_scalar": {"ms": ms_add, "GBps": add_bytes / (ms_add * 1e-3) / 1e9,
                                 "pct_hbm_peak": 100 * add_bytes / (ms_add * 1e-3) / 1e9 / HBM_PEAK_GBS,
                                 "bytes": add_bytes, "what": "3072 ciphertexts, component 0 read and written in place"},
            "ct_pt_mac_one_term_per_output": {"ms": ms_str, "GBps": str_bytes / (ms_str * 1e-3) / 1e9,
                                              "pct_hbm_peak": 100 * str_bytes / (ms_str * 1e-3) / 1e9 / HBM_PEAK_GBS,
                                              "bytes": str_bytes, "what": "1024 ciphertexts times one scalar each: 2 GiB read, 2 GiB written"}}

    # ---- the two arithmetics of the transforms on the same launch: the limbs below 2^50 on double-precision FMAs (the
    # library's choice, timed above) against integer butterflies for every limb; the residues must be the same
    if not only and args.compare_arithmetic:
        ms_fp = timed(lambda: ctx.rescale(acc4, out=out4k))
        ctx.integer_transforms(True)
        out_int = torch.empty_like(out4k)
        ms_int = timed(lambda: ctx.rescale(acc4, out=out_int))
        ctx.integer_transforms(False)
        same = bool(torch.equal(out_int, out4k))
        del out_int
        result["rescale_cfg4_transform_arithmetic"] = {
            "ms_double_precision_below_2^50": ms_fp, "ms_integer_butterflies_only": ms_int, "same_residues": same,
            "what": "he_rescale on cfg4's accumulators with he_test_integer_transforms off / on"}

    # ---- the batched transforms on their own (he_ntt_fwd / he_ntt_inv over cfg4's 65 536 accumulator rows, in place)
    if not only:
        rows_t = p4.n_out * 2 * L
        bfl = rows_t * (N // 2) * c4.log2N
        acc4.copy_(wl.uniform_residues_torch((p4.n_out, 2), q, N, 31, dev))     # canonical residues
        ms_nf = timed(lambda: ctx.ntt_fwd(acc4))
        ms_ni = timed(lambda: ctx.ntt_inv(acc4))
        def at_rate(kinds):
            return sum((rows_t // L) * (N // 2) * c4.log2N / rate(kinds(i), i) for i in range(L)) * 1e3 if args.rates else None
        fp_l = [qi < (1 << 50) for qi in q]
        ideal_f = at_rate(lambda i: he.RATE_BUTTERFLY_FP64 if fp_l[i] else fwd_kind[mode[i]])
        ideal_i = at_rate(lambda i: he.RATE_BUTTERFLY_FP64_INV if fp_l[i] else he.RATE_BUTTERFLY_INV if mode[i] else he.RATE_BUTTERFLY_MODE0)
        result["transforms"] = {
            "rows": rows_t, "ntt_fwd_ms": ms_nf, "ntt_inv_ms": ms_ni,
            "ntt_fwd_T_butterflies_per_s": bfl / (ms_nf * 1e-3) / 1e12, "ntt_inv_T_butterflies_per_s": bfl / (ms_ni * 1e-3) / 1e12,
            "ntt_fwd_Tmul32_per_s": bfl * MUL32_PER_SHOUP / (ms_nf * 1e-3) / 1e12,
            "ntt_fwd_frac_of_integer_peak": bfl * MUL32_PER_SHOUP / (ms_nf * 1e-3) / 1e12 / INT_MUL32_PEAK_TOPS,
            "ntt_fwd_frac_of_measured_rate": None if ideal_f is None else ideal_f / ms_nf,
            "ntt_inv_frac_of_measured_rate": None if ideal_i is None else ideal_i / ms_ni,
            "GBps_fwd": rows_t * N * 16 / (ms_nf * 1e-3) / 1e9,
            "what": "he_ntt_fwd and he_ntt_inv in place over %d rows of N=2^14 (2 x 60-bit + 6 x 50-bit limbs); a butterfly counts "
                    "%d 32-bit multiplies as in the rescale's roofline" % (rows_t, MUL32_PER_SHOUP)}

    # ---- Alg. 1 on the GPU: the plaintext polynomials a layer like cfg5 consumes, encoded from slots
    if not only:
        n_vec = 1024
        zs = torch.randn((n_vec, N // 2), dtype=torch.complex128, device=dev, generator=torch.Generator(device=dev).manual_seed(9))
        enc_out = torch.empty((n_vec, L, N), dtype=torch.int64, device=dev)
        ms_enc = timed(lambda: ctx.encode_vector(zs, scale, out=enc_out))
        enc_bytes = n_vec * (N * 8 + L * N * 8)              # slots read once, residues written once
        result["encode_vector"] = {"ms": ms_enc, "vectors_per_s": n_vec / (ms_enc * 1e-3),
                                   "GBps": enc_bytes / (ms_enc * 1e-3) / 1e9,
                                   "pct_hbm_peak": 100 * enc_bytes / (ms_enc * 1e-3) / 1e9 / HBM_PEAK_GBS,
                                   "what": "%d vectors of N/2 complex slots -> [L][N] residues in NTT form (FFT kernel + "
                                           "NTT kernel); bytes = slots once + residues once" % n_vec}
        dec_out = torch.empty((n_vec, N // 2), dtype=torch.complex128, device=dev)
        dec_ws = torch.empty(n_vec * L * N * 8, dtype=torch.uint8, device=dev)
        ms_dec = timed(lambda: ctx.decode_vector(enc_out, scale, out=dec_out, workspace=dec_ws))
        result["decode_vector"] = {"ms": ms_dec, "vectors_per_s": n_vec / (ms_dec * 1e-3),
                                   "GBps": enc_bytes / (ms_dec * 1e-3) / 1e9,
                                   "max_abs_error_of_round_trip": float((dec_out - zs).abs().max().item()),
                                   "what": "the inverse map on the same %d polynomials (INTT kernel into the workspace + lift/FFT kernel); "
                                           "bytes = residues once + slots once" % n_vec}
        del zs, enc_out, dec_out, dec_ws

    # ---- every config as one fused layer call (encode, MAC + bias, one rescale per output): median of
    # 20 after 5 warm-ups.  cfg1-3 inputs are small enough to stay in the caches between repetitions.
    if not only and args.all_configs:
        per = []
        for k in (1, 2, 3, 4, 5):
            ck = wl.config(k)
            pk = ck.plan
            if k in (4, 5):
                cx, ctk = ctx, (ct4 if k == 4 else ct5)
            else:
                cx = he.Context(ck.log2N, ck.q, device=0)
                ctk = wl.uniform_residues_torch((pk.n_in, 2), ck.q, ck.N, ck.seed, dev)
            hp = hp4 if k == 4 else hp5 if k == 5 else cx.plan(pk.n_in, pk.n_out, pk.n_pt, pk.off, pk.term_ct, pk.term_pt)
            poly = ck.pt_kind == "poly"
            if poly:
                ptk, wk, bk = pt5, None, None
            else:
                wk = w4 if k == 4 else torch.from_numpy(wl.normal_values(pk.n_pt, ck.sigma, ck.seed + 100)).to(dev)
                bk = b4 if k == 4 else torch.from_numpy(wl.normal_values(pk.n_out, ck.sigma, ck.seed + 200)).to(dev)
            kind = he.PT_POLY if poly else he.PT_SCALAR
            outk = torch.empty((pk.n_out, 2, ck.L - 1, ck.N), dtype=torch.int64, device=dev)
            wsk = torch.empty(max(hp.workspace_bytes(ck.L, kind, he.RESCALE), 256), dtype=torch.uint8, device=dev)
            sc = 2.0 ** ck.log2_scale
            def layer():
                if poly:
                    cx.ct_pt_mac(hp, ctk, ptk, kind, flags=he.RESCALE, out=outk, workspace=wsk)
                else:
                    cx.ct_pt_mac(hp, ctk, cx.encode_scalar(wk, sc), kind, bias=cx.encode_scalar(bk, sc), flags=he.RESCALE,
                                 out=outk, workspace=wsk)
            for _ in range(5):
                layer()
            torch.cuda.synchronize()
            ev = [torch.cuda.Event(enable_timing=True) for _ in range(21)]
            ev[0].record()
            for i in range(20):
                layer()
                ev[i + 1].record()
            torch.cuda.synchronize()
            ms = float(np.median([ev[i].elapsed_time(ev[i + 1]) for i in range(20)]))
            ctb = 2 * ck.L * ck.N * 8
            outb = 2 * (ck.L - 1) * ck.N * 8
            ptb = pk.n_pt * ck.L * ck.N * 8 if poly else (pk.n_pt + pk.n_out) * 8 * ck.L
            b_min = pk.n_in * ctb + pk.n_out * outb + ptb
            per.append({"config": k, "N": ck.N, "L": ck.L, "outputs": pk.n_out, "mac_terms": pk.n_terms,
                        "ms": ms, "G_mac_residue_terms_per_s": pk.n_terms * 2 * ck.L * ck.N / (ms * 1e-3) / 1e9,
                        "rescaled_ct_per_s": pk.n_out / (ms * 1e-3),
                        "min_bytes_GBps": b_min / (ms * 1e-3) / 1e9,
                        "per_mac_streamed_GBps": pk.n_terms * ctb / (ms * 1e-3) / 1e9})
            del outk, wsk
        result["per_config"] = {"what": "encode + MAC + bias + rescale as one he_ct_pt_mac(HE_RESCALE) call per layer; "
                                        "min_bytes = inputs once + outputs once + plaintexts; per_mac_streamed = what one "
                                        "ciphertext read per multiply (the per-call formulation of Alg. 7/8) would move, "
                                        "which reuse lets exceed the HBM peak", "configs": per}

    # ---- packed 32-bit storage (moduli below 2^30, cfg1's parameter set: N = 2^12, two 30-bit limbs) next
    # to the 64-bit path on the same residues: a dense layer large enough to time, the streaming add, and
    # the rescale on its own
    if not only and args.all_configs:
        c1 = wl.config(1)
        cx = he.Context(c1.log2N, c1.q, device=0)
        K1, M1, n_big = 1024, 256, 8192
        pl = wl.dense_plan(K1, M1)
        hp1 = cx.plan(pl.n_in, pl.n_out, pl.n_pt, pl.off, pl.term_ct, pl.term_pt)
        sc1 = 2.0 ** c1.log2_scale
        big64 = wl.uniform_residues_torch((n_big, 2), c1.q, c1.N, 11, dev)
        big32 = cx.pack32(big64)
        w1 = cx.encode_scalar(torch.from_numpy(wl.normal_values(pl.n_pt, 0.1, 12)).to(dev), sc1)
        b1 = cx.encode_scalar(torch.from_numpy(wl.normal_values(pl.n_out, 0.1, 13)).to(dev), sc1)
        ws1 = torch.empty(max(hp1.workspace_bytes(c1.L, he.PT_SCALAR, he.RESCALE), 256), dtype=torch.uint8, device=dev)
        o64 = torch.empty((M1, 2, c1.L - 1, c1.N), dtype=torch.int64, device=dev)
        o32 = torch.empty((M1, 2, c1.L - 1, c1.N), dtype=torch.int32, device=dev)
        ms_l64 = timed(lambda: cx.ct_pt_mac(hp1, big64[:K1], w1, he.PT_SCALAR, bias=b1, flags=he.RESCALE, out=o64, workspace=ws1), 20)
        ms_l32 = timed(lambda: cx.ct_pt_mac32(hp1, big32[:K1], w1, he.PT_SCALAR, bias=b1, flags=he.RESCALE, out=o32, workspace=ws1), 20)
        same = bool(torch.equal(cx.unpack32(o32), o64))
        pa = cx.encode_scalar(torch.from_numpy(wl.normal_values(n_big, 0.1, 14)).to(dev), sc1)
        ms_a64 = timed(lambda: cx.ct_pt_add(big64, pa, he.PT_SCALAR), 20)
        ms_a32 = timed(lambda: cx.ct_pt_add32(big32, pa, he.PT_SCALAR), 20)
        r64 = torch.empty((n_big, 2, c1.L - 1, c1.N), dtype=torch.int64, device=dev)
        r32 = torch.empty((n_big, 2, c1.L - 1, c1.N), dtype=torch.int32, device=dev)
        ms_r64 = timed(lambda: cx.rescale(big64, out=r64), 10)
        ms_r32 = timed(lambda: cx.rescale32(big32, out=r32), 10)
        resid = n_big * c1.L * c1.N                              # residues of component 0 (read and written)
        res_b = lambda width, ms: n_big * 2 * (2 * c1.L - 1) * c1.N * width / (ms * 1e-3) / 1e9
        result["packed32"] = {
            "what": "cfg1's parameter set (N=2^12, two 30-bit limbs), the same residues stored as uint64 and as uint32",
            "dense_%dx%d_layer" % (K1, M1): {"ms_u64": ms_l64, "ms_u32": ms_l32, "speedup": ms_l64 / ms_l32,
                                              "outputs_equal": same,
                                              "G_mac_residue_terms_per_s_u32": K1 * M1 * 2 * c1.L * c1.N / (ms_l32 * 1e-3) / 1e9},
            "ct_pt_add_scalar_%d_ct" % n_big: {"ms_u64": ms_a64, "ms_u32": ms_a32,
                                                "GBps_u64": resid * 16 / (ms_a64 * 1e-3) / 1e9,
                                                "GBps_u32": resid * 8 / (ms_a32 * 1e-3) / 1e9,
                                                "G_residues_per_s_u64": resid / (ms_a64 * 1e-3) / 1e9,
                                                "G_residues_per_s_u32": resid / (ms_a32 * 1e-3) / 1e9},
            "rescale_%d_ct" % n_big: {"ms_u64": ms_r64, "ms_u32": ms_r32, "speedup": ms_r64 / ms_r32,
                                      "GBps_u64": res_b(8, ms_r64), "GBps_u32": res_b(4, ms_r32),
                                      "ct_per_s_u32": n_big / (ms_r32 * 1e-3)}}
        del big64, big32, r64, r32

    # ---- the x^2 activation (square + relinearise with the special prime + one rescale) at the benchmark's
    # parameters: ciphertexts on the first 7 limbs, the eighth limb as the special prime
    if not only and args.all_configs:
        n_sq = 256
        ct_sq = wl.uniform_residues_torch((n_sq, 2), q[:L - 1], N, 21, dev)
        evk = wl.uniform_residues_torch((L - 1, 2), q, N, 22, dev)
        out_sq = torch.empty_like(ct_sq)
        down_sq = torch.empty((n_sq, 2, L - 2, N), dtype=torch.int64, device=dev)
        ws_sq = torch.empty(ctx.square_relin_workspace_bytes(L - 1, n_sq), dtype=torch.uint8, device=dev)
        def activation():
            ctx.ct_square_relin(ct_sq, evk, out=out_sq, workspace=ws_sq)
            ctx.rescale(out_sq, out=down_sq)
        ms_sq = timed(activation, 5)
        ms_sq_only = timed(lambda: ctx.ct_square_relin(ct_sq, evk, out=out_sq, workspace=ws_sq), 5)
        result["square_relin"] = {
            "ms": ms_sq, "ms_without_the_rescale": ms_sq_only, "ciphertexts": n_sq, "ct_per_s": n_sq / (ms_sq * 1e-3),
            "us_per_ct": ms_sq * 1e3 / n_sq,
            "what": "he_ct_square_relin + he_rescale on %d ciphertexts, N=2^14, 7 limbs + special prime; the paper's "
                    "table of operation runtimes lists Square 2411 us + Relinearize 27681 us + Rescale 10189 us per "
                    "ciphertext at (2^14, 8) on its CPU" % n_sq}
        del ct_sq, evk, out_sq, down_sq, ws_sq

    # ---- ring degree 2^15: rows beyond the LDS (one stage over global memory + two half-size transforms per row)
    if not only and args.all_configs:
        N15, n15 = 1 << 15, 512
        q15 = wl.modulus_chain([60, 60] + [50] * 6, N15)
        ctx15 = he.Context(15, q15)
        ct15 = wl.uniform_residues_torch((n15, 2), q15, N15, 23, dev)
        out15 = torch.empty((n15, 2, L - 1, N15), dtype=torch.int64, device=dev)
        ms_r15 = timed(lambda: ctx15.rescale(ct15, out=out15), 5)
        ms_f15 = timed(lambda: ctx15.ntt_fwd(ct15), 5)
        bf15 = n15 * 2 * L * (N15 // 2) * 15
        result["ring_degree_2_15"] = {
            "rescale_ms": ms_r15, "rescaled_ct_per_s": n15 / (ms_r15 * 1e-3), "ntt_fwd_ms": ms_f15,
            "ntt_fwd_G_butterflies_per_s": bf15 / (ms_f15 * 1e-3) / 1e9,
            "what": "%d ciphertexts at N=2^15 with the moduli widths of the benchmark (2x60 + 6x50 bits): he_rescale, and "
                    "he_ntt_fwd over all %d rows" % (n15, n15 * 2 * L)}
        del ct15, out15
        ctx15.close()

    print(json.dumps(result))
    if not same_as_one_call:
        print("bench.py: the two-call form of a layer differs from he_ct_pt_mac(HE_RESCALE)", file=sys.stderr)
        return 3
    if not result.get("rescale_cfg4_transform_arithmetic", {}).get("same_residues", True):
        print("bench.py: integer and double-precision transforms disagree", file=sys.stderr)
        return 3
    if "cpu_baseline" in result and not result["cpu_baseline"]["gpu_outputs_match_oracle"]:
        print("bench.py: the timed GPU outputs differ from the oracle's", file=sys.stderr)
        return 3
    return 0


if __name__ == "__main__":
    sys.exit(main())
