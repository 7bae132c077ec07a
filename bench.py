#!/usr/bin/env python3
"""Benchmark of the BinaryAttention forward hot path on one MI355X.

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--workload NAME] [--no-configs]

One step = one pass of the whole hot path over one batch of synthetic input
already resident in HBM: binattn_pack_qk (sign words + mu of Q and K),
binattn_prepare_kv (V quantisation, key operand layout) and binattn_attend (the
fused attention kernel).  Prints ONE JSON line.

  value      attention TOPS-equiv = 4*B*H*N^2*d / step time (true d, no padding)
             of the headline workload (vit_hires), K steps after W warm-ups
  roofline   for the dominant kernel (the fused attention kernel), timed with
             events on the launch stream inside the timed region; the bound is
             the vector ALU: algorithmic lane-instructions per (query, key)
             pair x pairs / kernel time, against 256 CUs x 4 SIMDs x 16 lanes x
             2.4 GHz = 39.3 T lane-instructions/s
  configs    all five benchmark configurations under one protocol of their own
             (100 steps after 10 warm-ups: median and minimum per step and per
             kernel, a cold-cache variant, the single-launch form where it
             applies), each with t_bound = max(vector ALU, HBM, matrix cores)
             and the fraction of it that was reached
  cpu_baseline  the CPU oracle timed on this host on a bounded sample of rows
"""
from __future__ import annotations

import argparse
import json
import os
import re
import statistics
import subprocess
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

# Algorithmic vector-ALU work per (query, key) pair of the fused kernel, in issue
# slots of a 16-lane SIMD ("lane-instructions"): int->float of the logit, scale +
# bias FMA, bias unpack, running max, exponent FMA, row-sum add, round-to-byte
# (7 full-rate instructions) plus one exponential.  v_exp_f32 issues at half rate on
# this chip (measured with a dependent-free instruction stream: 2 slots), hence 7 + 2.
ALU_SLOTS_PER_PAIR = 7 + 2
# What this kernel's design actually needs per pair (the FP4 matrix-core logits arrive
# in fp32 with the bias already added; v_max3 takes two values per instruction; the
# sign offset of the byte codes costs a quarter instruction): unpack 1, scale 1,
# max 0.5, FMA 1, exp 2, add 1, round 1, xor 0.25.
ALU_SLOTS_PER_PAIR_STRICT = 7.75
ALU_PEAK_TLANEOPS = 256 * 4 * 16 * 2.4e9 / 1e12   # 39.32
MFMA_I8_PEAK_TOPS = 5033.0
MFMA_FP4_PEAK_TOPS = 10066.0
HBM_PEAK_GBS = 8000.0

CONFIG_STEPS, CONFIG_WARMUP = 100, 10


def parse():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=20)
    ap.add_argument("--warmup", type=int, default=3)
    ap.add_argument("--workload", default="vit_hires")
    ap.add_argument("--no-configs", action="store_true", help="skip the per-configuration table (profiling runs)")
    ap.add_argument("--others", action="store_true", help="accepted for compatibility: the configurations are always timed")
    ap.add_argument("--axial", action="store_true",
                    help="also time the workload with the in-kernel decomposed relative-position bias (extra field)")
    ap.add_argument("--relpos", action="store_true",
                    help="also time the workloads with the in-kernel relative-position table (extra field)")
    ap.add_argument("--sweep", choices=["hd128"], help="also time the head-dim-128 sequence-length sweep (extra field)")
    ap.add_argument("--sweep-bias", action="store_true", help="run the sweep with a dense bias (up to N = 16384)")
    ap.add_argument("--logits", action="store_true",
                    help="also time the three integer-logit variants of binattn_logits_debug (extra field)")
    ap.add_argument("--probe", action="store_true",
                    help="also measure the issue rate of the softmax's vector-ALU instructions (extra field)")
    ap.add_argument("--heads", action="store_true",
                    help="also time the two single-launch forms (8-wave / 4-wave workgroups) over the number of heads (extra field)")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-bias", action="store_true", help="run without the bias term (not the headline config)")
    ap.add_argument("--lut", action="store_true",
                    help="with --no-bias / --sweep: read the exponentials from the per-head table (BINATTN_FLAG_LUT)")
    ap.add_argument("--cpu-seconds", type=float, default=10.0, help="target CPU time of the oracle sample")
    return ap.parse_args()


def axial_grid(N):
    """Gy, Gx with Gy * Gx = N and Gx a power of two in [16, 256] (square when possible)."""
    import math
    gx = 1 << max(4, min(8, int(round(math.log2(max(N, 1)) / 2))))
    while gx > 16 and N % gx:
        gx //= 2
    return (N // gx, gx) if N % gx == 0 and N // gx <= 256 else None


def relpos_grid(N):
    """Gy, Gx with Gy * Gx = N, Gx a power of two in [16, 128] and Gy <= 128 (square when possible)."""
    g = axial_grid(N)
    return g if g and g[0] <= 128 and g[1] <= 128 else None


# ---- bounds ------------------------------------------------------------------------------
def bounds(w, with_bias=True):
    """Lower bounds (ms) of one step of workload `w`, from algorithmic work and published peaks.
    Fused kernel: the three units work side by side, so its bound is the largest of them."""
    B, H, N, d = w.B, w.H, w.N, w.d
    W = (d + 31) // 32
    pairs = w.pairs
    t_alu = ALU_SLOTS_PER_PAIR * pairs / (ALU_PEAK_TLANEOPS * 1e12) * 1e3
    # fused-kernel bytes: bias once per head (batch-shared), query sign words, key operand
    # (FP4 codes, d/2 bytes per key) + V codes once per head, output
    fused_bytes = (2 * H * N * N if with_bias else 0) + B * H * N * (W * 4 + 16 * ((d + 31) // 32) + d + 2 * d)
    t_hbm = fused_bytes / (HBM_PEAK_GBS * 1e9) * 1e3
    t_mfma = (2 * pairs * d / (MFMA_FP4_PEAK_TOPS * 1e12) + 2 * pairs * d / (MFMA_I8_PEAK_TOPS * 1e12)) * 1e3
    pack_bytes = 2 * B * H * N * d * 2 + 2 * B * H * N * W * 4
    prep_bytes = B * H * N * d * 2 + B * H * N * (d + 16 * ((d + 31) // 32)) + B * H * N * W * 4
    # the single-launch form reads Q, K, V and the bias once and writes the output
    one_bytes = 4 * B * H * N * d * 2 + (2 * H * N * N if with_bias else 0)
    t_fused = max(t_alu, t_hbm, t_mfma)
    return {
        "t_valu_ms": t_alu, "t_hbm_ms": t_hbm, "t_mfma_ms": t_mfma, "t_bound_fused_ms": t_fused,
        "t_bound_pack_ms": pack_bytes / (HBM_PEAK_GBS * 1e9) * 1e3,
        "t_bound_prepare_ms": prep_bytes / (HBM_PEAK_GBS * 1e9) * 1e3,
        "t_bound_single_launch_ms": max(t_alu, t_mfma, one_bytes / (HBM_PEAK_GBS * 1e9) * 1e3),
        "fused_hbm_bytes": fused_bytes, "pack_hbm_bytes": pack_bytes, "prepare_hbm_bytes": prep_bytes,
    }


class Buffers:
    """Inputs of one workload plus every buffer a step writes."""

    def __init__(self, name, with_bias=True, seed_shift=0):
        import torch
        from paper_2603_09582_amd import binding as ba
        from paper_2603_09582_amd import workloads as wl
        w = wl.WORKLOADS[name]
        if seed_shift:
            w = wl.Workload(w.name, w.B, w.H, w.N, w.d, w.seed + seed_shift, w.extra, w.note)
        self.w = w
        self.x = wl.make_inputs(w, device="cuda", with_bias=with_bias)
        B, H, N, d = w.B, w.H, w.N, w.d
        W = (d + 31) // 32
        dev = self.x.q.device
        self.q_bits = torch.empty(B, H, N, W, dtype=torch.int32, device=dev)
        self.k_bits = torch.empty_like(self.q_bits)
        self.mu_q = torch.empty(B, H, dtype=torch.float32, device=dev)
        self.mu_k = torch.empty_like(self.mu_q)
        self.out = torch.empty(B, H, N, d, dtype=torch.bfloat16, device=dev)
        self.ws = ba.alloc_workspace(B, H, N, d, dev)
        self.flags = 0


def three_calls(b, e=None, attend=None):
    """pack_qk, prepare_kv, attend on buffers `b`; `e`: four events recorded around the calls."""
    from paper_2603_09582_amd import binding as ba
    x = b.x
    if e: e[0].record()
    ba.pack_qk(x.q, x.k, b.q_bits, b.k_bits, b.mu_q, b.mu_k)
    if e: e[1].record()
    ba.prepare_kv(b.k_bits, x.v, b.ws)
    if e: e[2].record()
    if attend is not None:
        attend(b)
    else:
        ba.attend(b.q_bits, b.mu_q, b.mu_k, x.bias, x.scale, b.w.d, b.ws, out=b.out, flags=b.flags)
    if e: e[3].record()


def run_workload(name, steps, warmup, with_bias=True, axial=False, relpos=False, flags=0):
    """K steps after W warm-ups, four events per step inside the timed region (the headline protocol)."""
    import torch
    from paper_2603_09582_amd import binding as ba

    b = Buffers(name, with_bias=with_bias and not axial and not relpos)
    b.flags = flags
    w, x = b.w, b.x
    B, H, N, d = w.B, w.H, w.N, w.d
    W = (d + 31) // 32
    dev = x.q.device
    attend = None
    if axial:  # decomposed relative-position bias: two small tables per head instead of [H, N, N]
        Gy, Gx = axial_grid(N)
        gen = torch.Generator(device="cuda").manual_seed(w.seed + 1000)
        by = torch.randn(H, 2 * Gy - 1, generator=gen, device=dev) * 0.02
        bx = torch.randn(H, 2 * Gx - 1, generator=gen, device=dev) * 0.02
        attend = lambda b: ba.attend_axial(b.q_bits, b.mu_q, b.mu_k, by, bx, x.scale, d, b.ws, out=b.out)
    if relpos:  # the full relative-position table of each head instead of [H, N, N]
        Gy, Gx = relpos_grid(N)
        gen = torch.Generator(device="cuda").manual_seed(w.seed + 2000)
        table = torch.randn(H, 2 * Gy - 1, 2 * Gx - 1, generator=gen, device=dev) * 0.02
        attend = lambda b: ba.attend_relpos(b.q_bits, b.mu_q, b.mu_k, table, x.scale, d, b.ws, out=b.out)

    ev = [[torch.cuda.Event(enable_timing=True) for _ in range(4)] for _ in range(steps)]
    for _ in range(warmup):
        three_calls(b, attend=attend)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for i in range(steps):
        three_calls(b, ev[i], attend=attend)
    torch.cuda.synchronize()
    t1 = time.perf_counter()

    ms_step = (t1 - t0) * 1e3 / steps
    pack_ms = sum(e[0].elapsed_time(e[1]) for e in ev) / steps
    prep_ms = sum(e[1].elapsed_time(e[2]) for e in ev) / steps
    fused_ms = sum(e[2].elapsed_time(e[3]) for e in ev) / steps
    pairs = w.pairs
    bd = bounds(w, with_bias=with_bias and not axial and not relpos)
    res = {
        "workload": name, "B": B, "H": H, "N": N, "d": d,
        "ms_per_step": ms_step, "pack_ms": pack_ms, "prepare_ms": prep_ms, "fused_ms": fused_ms,
        "tops_equiv": w.equiv_ops / (ms_step * 1e-3) / 1e12,
        "fused_tops_equiv": w.equiv_ops / (fused_ms * 1e-3) / 1e12,
        # pack kernel: 2 B read per Q/K element + packed words written
        "pack_gbs": bd["pack_hbm_bytes"] / (pack_ms * 1e-3) / 1e9,
        "alu_tlaneops": ALU_SLOTS_PER_PAIR * pairs / (fused_ms * 1e-3) / 1e12,
        "mfma_tops_algorithmic": 4 * pairs * d / (fused_ms * 1e-3) / 1e12,
        "fused_hbm_bytes": bd["fused_hbm_bytes"],
        "bounds": bd,
    }
    res["fused_hbm_gbs"] = res["fused_hbm_bytes"] / (fused_ms * 1e-3) / 1e9
    return res, x


def med_min(v):
    return {"median": statistics.median(v), "min": min(v)}


def config_row(name, steps=CONFIG_STEPS, warmup=CONFIG_WARMUP):
    """One configuration under the table's protocol: `steps` steps after `warmup` warm-ups.
    Pass 1: start/end events per step and the wall clock (what a caller sees, launches included).
    Pass 2: events between the three calls (per-kernel times).  Pass 3 (short sequences only):
    the same step on a ring of distinct buffer sets larger than the 256 MB Infinity Cache, so
    that no step finds its inputs in a cache.  Pass 4 (N <= 256): the single-launch form."""
    import torch
    from paper_2603_09582_amd import binding as ba

    b = Buffers(name)
    w, x = b.w, b.x
    bd = bounds(w)

    def timed(fn, n, warm):
        for _ in range(warm):
            fn(0)
        torch.cuda.synchronize()
        ev = [(torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)) for _ in range(n)]
        t0 = time.perf_counter()
        for i in range(n):
            ev[i][0].record()
            fn(i)
            ev[i][1].record()
        torch.cuda.synchronize()
        wall = (time.perf_counter() - t0) * 1e3 / n
        return wall, [a.elapsed_time(c) for a, c in ev]

    wall, per = timed(lambda i: three_calls(b), steps, warmup)
    ev4 = [[torch.cuda.Event(enable_timing=True) for _ in range(4)] for _ in range(steps)]
    for i in range(steps):
        three_calls(b, ev4[i])
    torch.cuda.synchronize()
    kern = {"pack_qk": med_min([e[0].elapsed_time(e[1]) for e in ev4]),
            "prepare_kv": med_min([e[1].elapsed_time(e[2]) for e in ev4]),
            "attend": med_min([e[2].elapsed_time(e[3]) for e in ev4])}
    row = {
        "workload": name, "B": w.B, "H": w.H, "N": w.N, "d": w.d, "steps": steps, "warmup": warmup,
        "ms_per_step": med_min(per), "ms_per_step_wall_mean": wall,
        "kernels_ms": kern,
        "tops_equiv": w.equiv_ops / (statistics.median(per) * 1e-3) / 1e12,
        "fused_kernel_tops_equiv": w.equiv_ops / (kern["attend"]["median"] * 1e-3) / 1e12,
        "t_bound_ms": {"valu_9_slots": bd["t_valu_ms"], "hbm": bd["t_hbm_ms"], "mfma": bd["t_mfma_ms"],
                       "fused_kernel": bd["t_bound_fused_ms"], "pack_qk": bd["t_bound_pack_ms"],
                       "prepare_kv": bd["t_bound_prepare_ms"]},
        "fused_kernel_frac_of_bound": bd["t_bound_fused_ms"] / kern["attend"]["median"],
        # the step's bound: its three stages run one after the other
        "step_frac_of_bound": (bd["t_bound_fused_ms"] + bd["t_bound_pack_ms"] + bd["t_bound_prepare_ms"])
                              / statistics.median(per),
        "pack_gbs": bd["pack_hbm_bytes"] / (kern["pack_qk"]["median"] * 1e-3) / 1e9,
        "prepare_gbs": bd["prepare_hbm_bytes"] / (kern["prepare_kv"]["median"] * 1e-3) / 1e9,
    }
    if w.N <= 4096:   # cold caches: a ring of buffer sets larger than the last-level cache
        per_set = sum(t.numel() * t.element_size() for t in (x.q, x.k, x.v, x.bias, b.ws, b.out))
        nset = max(2, min(24, int(640e6 / per_set) + 1))
        ring = [b] + [Buffers(name, seed_shift=1000 * (i + 1)) for i in range(nset - 1)]
        _, cold = timed(lambda i: three_calls(ring[i % nset]), steps, nset)
        row["cold_cache"] = {"buffer_sets": nset, "bytes_per_set": per_set, "ms_per_step": med_min(cold)}
        del ring
    if w.N > 256:     # the same step through the one-call entry point (binattn_attention: three launches)
        one = lambda i: ba.attention(x.q, x.k, x.v, x.bias, x.scale, out=b.out, workspace=b.ws)
        wall1, per1 = timed(one, steps, warmup)
        # its first two launches read Q, K, V once (+ V a second time) and write the query sign
        # words and the operand images
        W = (w.d + 31) // 32
        t_io = (4 * w.B * w.H * w.N * w.d * 2 + w.B * w.H * w.N * (W * 4 + w.d + 16 * W)) / (HBM_PEAK_GBS * 1e9) * 1e3
        row["one_call"] = {"ms_per_step": med_min(per1), "ms_per_step_wall_mean": wall1,
                           "tops_equiv": w.equiv_ops / (statistics.median(per1) * 1e-3) / 1e12,
                           "t_bound_ms": bd["t_bound_fused_ms"] + t_io,
                           "frac_of_bound": (bd["t_bound_fused_ms"] + t_io) / statistics.median(per1)}
    if w.N <= 256:    # the whole step as one launch (binattn_forward_fused)
        one = lambda i: ba.forward_fused(x.q, x.k, x.v, x.bias, x.scale, out=b.out)
        wall1, per1 = timed(one, steps, warmup)
        row["single_launch"] = {"ms_per_step": med_min(per1), "ms_per_step_wall_mean": wall1,
                                "tops_equiv": w.equiv_ops / (statistics.median(per1) * 1e-3) / 1e12,
                                "t_bound_ms": bd["t_bound_single_launch_ms"],
                                "frac_of_bound": bd["t_bound_single_launch_ms"] / statistics.median(per1)}
        if w.B * w.H > 256:   # more heads than compute units: 4-wave workgroups by default; the 8-wave form beside it
            row["single_launch"]["workgroups"] = "4 waves, two per compute unit"
            one8 = lambda i: ba.forward_fused(x.q, x.k, x.v, x.bias, x.scale, out=b.out, flags=ba.FLAG_WIDE8)
            _, per8 = timed(one8, steps, warmup)
            row["single_launch"]["ms_per_step_8_wave_form"] = med_min(per8)
        else:
            row["single_launch"]["workgroups"] = "8 waves, one per head"
    if w.N % 8:       # the same bias in rows padded to a multiple of 8 elements: tiles staged through LDS
        import torch
        pitch = (w.N + 7) // 8 * 8
        store = torch.zeros(w.H, w.N, pitch, dtype=x.bias.dtype, device=x.bias.device)
        store[:, :, :w.N] = x.bias
        pb = store[:, :, :w.N]
        ev = lambda f: med_min(timed(f, steps, warmup)[1])
        row["bias_rows_padded_to_8_elements"] = {
            "row_pitch": pitch,
            "attend_ms": ev(lambda i: ba.attend(b.q_bits, b.mu_q, b.mu_k, pb, x.scale, w.d, b.ws, out=b.out)),
            "single_launch_ms": ev(lambda i: ba.forward_fused(x.q, x.k, x.v, pb, x.scale, out=b.out)),
            "note": "not the headline layout: the configuration's bias is [H, N, N] contiguous, read row by row into registers"}
        del store, pb
    # the fastest way through the library for this configuration, against that path's own bound
    cands = [("pack_qk + prepare_kv + attend", row["ms_per_step"]["median"], row["step_frac_of_bound"])]
    if "one_call" in row:
        cands.append(("binattn_attention (three launches)", row["one_call"]["ms_per_step"]["median"], row["one_call"]["frac_of_bound"]))
    if "single_launch" in row:
        cands.append(("binattn_forward_fused (one launch)", row["single_launch"]["ms_per_step"]["median"], row["single_launch"]["frac_of_bound"]))
    best = min(cands, key=lambda c: c[1])
    row["best"] = {"path": best[0], "ms_per_step": best[1], "frac_of_bound": best[2],
                   "tops_equiv": w.equiv_ops / (best[1] * 1e-3) / 1e12}
    del b
    torch.cuda.empty_cache()
    return row


def heads_rows(launches=60):
    """binattn_forward_fused with one 8-wave workgroup per head (BINATTN_FLAG_WIDE8) and with 4-wave
    workgroups (the default above 256 heads) over a range of head counts; microseconds per launch,
    events around `launches` back-to-back calls."""
    import torch
    from paper_2603_09582_amd import binding as ba
    from paper_2603_09582_amd import workloads as wl
    rows = []
    for (B, H, N, d) in [(18, 16, 256, 72), (24, 16, 256, 72), (32, 16, 256, 72), (48, 16, 256, 72), (64, 16, 256, 72),
                         (24, 12, 197, 64), (43, 12, 197, 64), (64, 12, 197, 64), (128, 12, 197, 64), (32, 16, 128, 64)]:
        x = wl.make_inputs(wl.custom_workload(B, H, N, d, 7), device="cuda")
        out = torch.empty_like(x.v)
        us = []
        for flags in (ba.FLAG_WIDE8, 0):
            for _ in range(5):
                ba.forward_fused(x.q, x.k, x.v, x.bias, x.scale, out=out, flags=flags)
            e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            e0.record()
            for _ in range(launches):
                ba.forward_fused(x.q, x.k, x.v, x.bias, x.scale, out=out, flags=flags)
            e1.record()
            torch.cuda.synchronize()
            us.append(e0.elapsed_time(e1) * 1e3 / launches)
        rows.append({"heads": B * H, "N": N, "d": d, "us_8_wave_form": us[0], "us_4_wave_form": us[1]})
        del x, out
    return rows


def logits_rows(steps=20):
    """The three forms of the integer logits (binattn_logits_debug, row-sum output so that no
    N x N store stream hides the difference) on a row slab of the two workloads named in the
    target, timed with events: popcount on the vector ALU, int8 MFMA, FP4 MFMA (the fused
    kernel's tile routine)."""
    import torch
    from paper_2603_09582_amd import binding as ba
    rows = []
    for name, r1 in (("dit_xl2_512", 1024), ("vit_hires", 4096)):
        b = Buffers(name, with_bias=False)
        w = b.w
        ba.pack_qk(b.x.q, b.x.k, b.q_bits, b.k_bits, b.mu_q, b.mu_k)
        pairs = w.B * w.H * r1 * w.N
        entry = {"workload": name, "rows": r1, "pairs": pairs}
        for label, var in (("popcount_valu", ba.LOGITS_POPCOUNT), ("mfma_i8", ba.LOGITS_MFMA_I8),
                           ("mfma_fp4", ba.LOGITS_MFMA_FP4)):
            var |= ba.LOGITS_ROWSUM
            for _ in range(3):
                out = ba.logits_debug(b.q_bits, b.k_bits, w.d, 0, r1, var, b.ws)
            ev = [(torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)) for _ in range(steps)]
            for e in ev:
                e[0].record()
                ba.logits_debug(b.q_bits, b.k_bits, w.d, 0, r1, var, b.ws)
                e[1].record()
            torch.cuda.synchronize()
            t = [a.elapsed_time(c) for a, c in ev]
            entry[label] = {"ms": med_min(t), "t_pairs_per_s": pairs / (statistics.median(t) * 1e-3) / 1e12}
            del out
        rows.append(entry)
        del b
        torch.cuda.empty_cache()
    return rows


def probe_rows(iters=4096, blocks=256 * 16, reps=3):
    """Issue rate of the vector-ALU instruction kinds of the softmax (binattn_probe_valu): T
    lane-instructions/s over the chip for each kind alone and mixed half and half with an FMA, a
    byte conversion, an exponential and an OR (a mix that runs faster than either kind alone
    shows that the two kinds issue side by side)."""
    import torch
    from paper_2603_09582_amd import binding as ba
    out = torch.empty(blocks * 256, dtype=torch.float32, device="cuda")

    def rate(op):
        ba.probe_valu(op, iters, blocks, out)
        ev = [(torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)) for _ in range(reps)]
        for e in ev:
            e[0].record()
            ba.probe_valu(op, iters, blocks, out)
            e[1].record()
        torch.cuda.synchronize()
        ms = statistics.median(a.elapsed_time(c) for a, c in ev)
        return blocks * 256 * ba.PROBE_CHAINS * iters / (ms * 1e-3) / 1e12

    rows = []
    for label, op in ba.PROBE_OPS.items():
        row = {"op": label, "alone": rate(op | (op << 8))}
        for partner in ba.PROBE_PARTNERS:
            if partner != label:
                row["with_" + partner] = rate(op | (ba.PROBE_OPS[partner] << 8))
        rows.append(row)
    # the softmax's own instruction mix on register data, 16 values per lane and step, with the LDS
    # per workgroup pinned so that 1, 2, 3 or 4 four-wave workgroups fit a compute unit
    out2 = torch.empty(256 * 16 * 256, dtype=torch.float32, device="cuda")
    for kib, waves in ((160, 1), (80, 2), (52, 3), (40, 4)):
        op, blk, it = ba.PROBE_SOFTMAX | (kib << 8), 256 * 4 * waves, 2048
        ba.probe_valu(op, it, blk, out2)
        ev = [(torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)) for _ in range(reps)]
        for e in ev:
            e[0].record()
            ba.probe_valu(op, it, blk, out2)
            e[1].record()
        torch.cuda.synchronize()
        ms = statistics.median(a.elapsed_time(c) for a, c in ev)
        rows.append({"op": "softmax_mix", "waves_per_simd": waves, "lds_kib_per_workgroup": kib,
                     "t_values_per_s": blk * 256 * 16 * it / (ms * 1e-3) / 1e12})
    return rows


def clock_from_probe():
    """Shader clock under a pure vector load, from the issue-rate probe: a dependent-free stream of
    v_fma_f32 at full occupancy issues one instruction per SIMD and 4 clocks, so lane-instructions/s
    / (256 CUs x 4 SIMDs x 16 lanes) is the clock the chip held (an estimate from below)."""
    import torch
    from paper_2603_09582_amd import binding as ba
    blocks, iters = 256 * 16, 2048
    out = torch.empty(blocks * 256, dtype=torch.float32, device="cuda")
    op = ba.PROBE_OPS["fma"] * 0x101
    ba.probe_valu(op, iters, blocks, out)
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    e0.record()
    ba.probe_valu(op, iters, blocks, out)
    e1.record()
    torch.cuda.synchronize()
    return blocks * 256 * ba.PROBE_CHAINS * iters / (e0.elapsed_time(e1) * 1e-3) / (256 * 4 * 16) / 1e9


def cpu_baseline(x, seconds):
    """Time the oracle (as it stands) on a bounded sample of this workload: query rows of head
    (0, 0), and once a whole head takes less than the budget, further whole heads."""
    import numpy as np
    import torch
    from oracle import binattn_oracle as orc

    w = x.workload
    N, d = w.N, w.d

    def bits(t):
        return t.cpu().contiguous().view(torch.int16).numpy().view(np.uint16)

    def run(b, h, n_rows):
        q, k, v = bits(x.q[b, h]), bits(x.k[b, h]), bits(x.v[b, h])
        rows = np.linspace(0, N - 1, n_rows).astype(np.int64)
        full = np.zeros((N, N), dtype=np.uint16)
        full[rows] = bits(x.bias[h][torch.as_tensor(rows, device=x.bias.device)])
        t0 = time.perf_counter()
        mu_q, mu_k = orc.abs_mean(q), orc.abs_mean(k)
        vq, delta = orc.quant_v(v)
        orc.sign_pack(q); orc.sign_pack(k)
        orc.attention_rows(q, k, v, full, x.scale, mu_q, mu_k, vq, delta, rows=rows, want=("O2",))
        return time.perf_counter() - t0

    probe_rows = min(N, 64)
    t_probe = run(0, 0, probe_rows)
    n_rows = int(min(N, max(probe_rows, probe_rows * seconds / max(t_probe, 1e-6))))
    t = run(0, 0, n_rows)
    total_rows, heads = n_rows, 1
    if n_rows == N:  # whole heads are cheap enough: add more until the budget is used
        for bh in range(1, w.B * w.H):
            if t >= seconds:
                break
            t += run(bh // w.H, bh % w.H, N)
            total_rows += N
            heads += 1
    ops = 4.0 * total_rows * N * d
    what = (f"{heads} whole head(s)" if n_rows == N else f"{n_rows} query rows of head (b=0,h=0)")
    return {"value": ops / t / 1e12, "unit": "TOPS-equiv", "cores": orc.num_threads(), "kind": "oracle",
            "sample": f"{what} of {w.name} ({total_rows} rows x all {N} keys), incl. each head's sign "
                      f"packing, mu and V quantisation; {t:.1f} s"}


def profile_record(workload, key="traffic_bytes_per_launch"):
    """A figure of the fused kernel as the committed rocprofv3 summary of this workload states it
    (a line `<key>: <number>`): HBM bytes per launch, executed lane-instructions per pair; or None."""
    path = os.path.join(ROOT, "profiles", f"binattn_kernels_{workload}.txt")
    try:
        m = re.search(r"^" + re.escape(key) + r"\s*:\s*([0-9.eE+]+)", open(path).read(), re.M)
        return float(m.group(1)) if m else None
    except OSError:
        return None


def clock_state():
    """Clocks and power as rocm-smi reports them (read-only), for the record.  Called before
    anything touches the GPU (a process that has initialised the GPU must not start other
    programs on this pool), and not at all under a profiler, which initialises the GPU first."""
    if any(k.startswith(("ROCPROF", "ROCP_")) for k in os.environ) or "rocprof" in os.environ.get("LD_PRELOAD", ""):
        return {"unavailable": "profiler run"}
    try:
        r = subprocess.run(["rocm-smi", "--showclocks", "--showpower", "--json"], capture_output=True,
                           text=True, timeout=20)
        card = next(iter(json.loads(r.stdout).values()))
        keep = {k: v for k, v in card.items() if any(s in k.lower() for s in ("sclk", "mclk", "fclk", "power"))}
        return keep or None
    except Exception as e:  # noqa: BLE001 - the record is optional
        return {"unavailable": type(e).__name__}


def main():
    a = parse()
    if a.gpus != 1:
        print("bench.py measures one GPU: this build has no multi-GPU path (each (batch, head) problem "
              "is independent and would shard over them, or over query rows, with no exchange step). Run with --gpus 1.", file=sys.stderr)
        sys.exit(2)
    clocks = clock_state()
    import torch
    assert torch.cuda.is_available(), "bench.py needs a GPU"
    from paper_2603_09582_amd import workloads as wl

    from paper_2603_09582_amd import binding as ba_
    lut_flag = ba_.FLAG_LUT if a.lut else 0
    res, x = run_workload(a.workload, a.steps, a.warmup, with_bias=not a.no_bias, flags=lut_flag)
    bd = res["bounds"]
    line = {
        "metric": "attention TOPS-equiv (4*B*H*N^2*d/s), whole hot path (pack_qk + prepare_kv + attend)",
        "value": res["tops_equiv"], "unit": "TOPS-equiv", "n_gpus": 1, "steps": a.steps, "warmup": a.warmup,
        "ms_per_step": res["ms_per_step"], "higher_is_better": True, "scaling": "weak",
        "vs_baseline": None,
        "dtype": "fp4 (e2m1, +-1.0 exact) x fp4 -> fp32 for Q.K^T (1-bit Q, K); u8 x s8 -> int32 for P.V "
                 "(as s8 x s8 on P - 128); fp32 softmax",
        "data": "synthetic",
        "config": {"workload": f"{a.workload} (B={res['B']}, H={res['H']}, N={res['N']}, d={res['d']}, bf16 Q/K/V, "
                               f"dense bf16 bias [H,N,N] shared over the batch, scale 1/sqrt(d))"},
        "kernels_ms": {"pack_qk": res["pack_ms"], "prepare_kv": res["prepare_ms"], "attend": res["fused_ms"]},
        "fused_kernel_tops_equiv": res["fused_tops_equiv"],
        "pack_kernel_gbs": res["pack_gbs"],
        "roofline": {"bound": "alu", "achieved": res["alu_tlaneops"], "peak": ALU_PEAK_TLANEOPS,
                     "unit": "T lane-instr/s", "frac": res["alu_tlaneops"] / ALU_PEAK_TLANEOPS,
                     "traffic": None if a.no_bias else profile_record(a.workload),
                     "kernel": "fused_kernel (binattn_attend)", "kernel_ms": res["fused_ms"],
                     "algorithmic_lane_instr_per_pair": ALU_SLOTS_PER_PAIR,
                     "frac_strict_count": res["alu_tlaneops"] / ALU_PEAK_TLANEOPS
                                          * ALU_SLOTS_PER_PAIR_STRICT / ALU_SLOTS_PER_PAIR,
                     "strict_lane_instr_per_pair": ALU_SLOTS_PER_PAIR_STRICT,
                     # what the SIMDs executed (SQ_INSTS_VALU x 64 / pairs, v_exp_f32 counted twice, from the
                     # committed rocprofv3 summary) and the fraction of the peak that is
                     "executed_lane_instr_per_pair": profile_record(a.workload, "executed_lane_instr_per_pair"),
                     "frac_executed": (None if profile_record(a.workload, "executed_lane_instr_per_pair") is None else
                                       res["alu_tlaneops"] / ALU_PEAK_TLANEOPS
                                       * profile_record(a.workload, "executed_lane_instr_per_pair") / ALU_SLOTS_PER_PAIR),
                     "algorithmic_hbm_bytes": res["fused_hbm_bytes"]},
        "roofline_other_bounds": {
            "t_valu_ms": bd["t_valu_ms"], "t_hbm_ms": bd["t_hbm_ms"], "t_mfma_ms": bd["t_mfma_ms"],
            "t_bound_ms": bd["t_bound_fused_ms"], "frac_of_t_bound": bd["t_bound_fused_ms"] / res["fused_ms"],
            "mfma_int8_frac": res["mfma_tops_algorithmic"] / MFMA_I8_PEAK_TOPS,
            "hbm_frac": res["fused_hbm_gbs"] / HBM_PEAK_GBS, "hbm_gbs": res["fused_hbm_gbs"]},
        "clocks": {"rocm_smi_before_the_run": clocks, "ghz_under_a_v_fma_stream": clock_from_probe(),
                   "ghz_under_the_fused_kernel_rocm_smi": 2.18,
                   "note": "the roofline peak assumes 2.4 GHz; rocm-smi --showclocks sampled during 1500 back-to-back "
                           "steps of this workload read 2175-2195 MHz (profiles/binattn_kernels_vit_hires.txt)"},
    }
    line["roofline"]["frac_at_the_clock_a_v_fma_stream_holds"] = (
        line["roofline"]["frac"] * 2.4 / line["clocks"]["ghz_under_a_v_fma_stream"])
    del x
    torch.cuda.empty_cache()
    if not a.no_configs and not a.no_bias:
        line["configs"] = [config_row(name) for name in wl.WORKLOAD_ORDER]
    if a.axial and axial_grid(wl.WORKLOADS[a.workload].N):
        r, xa = run_workload(a.workload, a.steps, a.warmup, axial=True)
        del xa
        torch.cuda.empty_cache()
        Gy, Gx = axial_grid(r["N"])
        line["axial_bias"] = {"grid": [Gy, Gx], "ms_per_step": r["ms_per_step"], "attend_ms": r["fused_ms"],
                              "tops_equiv": r["tops_equiv"], "fused_kernel_tops_equiv": r["fused_tops_equiv"],
                              "note": "b_ij = y[iy-jy] + x[ix-jx] from two fp32 tables per head held in LDS"}
    if a.relpos:
        rows = []
        for name in ("dit_xl2_256", "dit_xl2_512", "vit_hires"):
            if relpos_grid(wl.WORKLOADS[name].N) is None:
                continue
            r, xr = run_workload(name, max(5, a.steps), a.warmup, relpos=True)
            del xr
            torch.cuda.empty_cache()
            rows.append({"workload": name, "grid": list(relpos_grid(r["N"])), "ms_per_step": r["ms_per_step"],
                         "attend_ms": r["fused_ms"], "tops_equiv": r["tops_equiv"],
                         "fused_kernel_tops_equiv": r["fused_tops_equiv"],
                         "alu_frac": r["alu_tlaneops"] / ALU_PEAK_TLANEOPS})
        # ... and the whole layer in one launch where it applies (N <= 256)
        from paper_2603_09582_amd import binding as ba
        w256 = wl.WORKLOADS["dit_xl2_256"]
        x256 = wl.make_inputs(w256, device="cuda", with_bias=False)
        gen = torch.Generator(device="cuda").manual_seed(w256.seed + 2000)
        table = torch.randn(w256.H, 31, 31, generator=gen, device="cuda") * 0.02
        o256 = torch.empty_like(x256.q)
        n = max(5, a.steps)
        for _ in range(a.warmup):
            ba.forward_fused_relpos(x256.q, x256.k, x256.v, table, x256.scale, out=o256)
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for _ in range(n):
            ba.forward_fused_relpos(x256.q, x256.k, x256.v, table, x256.scale, out=o256)
        torch.cuda.synchronize()
        one_ms = (time.perf_counter() - t0) * 1e3 / n
        rows[0]["single_launch_ms_per_step"] = one_ms
        rows[0]["single_launch_tops_equiv"] = w256.equiv_ops / (one_ms * 1e-3) / 1e12
        del x256, o256
        # ... and from the bf16 tensors behind one call (binattn_attention_relpos), any N
        for row in rows:
            w = wl.WORKLOADS[row["workload"]]
            xw = wl.make_inputs(w, device="cuda", with_bias=False)
            Gy, Gx = relpos_grid(w.N)
            tb = torch.randn(w.H, 2 * Gy - 1, 2 * Gx - 1, generator=gen, device="cuda") * 0.02
            ow = torch.empty_like(xw.q)
            wsb = ba.alloc_workspace(w.B, w.H, w.N, w.d)
            for _ in range(a.warmup):
                ba.attention_relpos(xw.q, xw.k, xw.v, tb, xw.scale, out=ow, workspace=wsb)
            e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            e0.record()
            for _ in range(n):
                ba.attention_relpos(xw.q, xw.k, xw.v, tb, xw.scale, out=ow, workspace=wsb)
            e1.record()
            torch.cuda.synchronize()
            row["one_call_ms_per_step"] = e0.elapsed_time(e1) / n
            del xw, ow, wsb, tb
            torch.cuda.empty_cache()
        line["relpos_table_bias"] = {"note": "b_ij = table[iy-jy][ix-jx], fp32 table rows staged in LDS",
                                     "workloads": rows}
    if a.sweep:
        rows = []
        for name in wl.SWEEP_HD128:
            w = wl.WORKLOADS[name]
            if a.sweep_bias and w.N > 16384:
                continue
            r, xs = run_workload(name, max(5, a.steps), a.warmup, with_bias=a.sweep_bias, flags=lut_flag)
            del xs
            torch.cuda.empty_cache()
            r["bias"] = bool(a.sweep_bias)
            row = {k: r[k] for k in ("workload", "B", "H", "N", "d", "bias", "ms_per_step", "pack_ms",
                                     "prepare_ms", "fused_ms", "tops_equiv", "fused_tops_equiv")}
            row["t_bound_fused_ms"] = r["bounds"]["t_bound_fused_ms"]
            row["fused_kernel_frac_of_bound"] = r["bounds"]["t_bound_fused_ms"] / r["fused_ms"]
            rows.append(row)
        line["sweep_hd128"] = rows
    if a.logits:
        line["logits_variants"] = logits_rows()
    if a.probe:
        line["valu_issue_rates"] = probe_rows()
    if a.heads:
        line["single_launch_forms_vs_heads"] = heads_rows()
    if a.no_bias:
        line["config"]["workload"] += (" -- WITHOUT bias (diagnostic run), exponentials "
                                       + ("from the per-head table" if a.lut else "computed"))
    if not a.no_cpu_baseline and not a.no_bias:
        x = wl.make_inputs(wl.WORKLOADS[a.workload], device="cuda")   # the headline inputs again, for the CPU leg
        line["cpu_baseline"] = cpu_baseline(x, a.cpu_seconds)
    print(json.dumps(line))


if __name__ == "__main__":
    main()
