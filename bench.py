#!/usr/bin/env python3
"""Benchmark of the BinaryAttention forward hot path on one MI355X.

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--workload NAME] [--others]

One step = one pass of the whole hot path over one batch of synthetic input
already resident in HBM: binattn_pack_qk (sign words + mu of Q and K),
binattn_prepare_kv (V quantisation, key operand layout) and binattn_attend (the
fused attention kernel).  Prints ONE JSON line.

  value      attention TOPS-equiv = 4*B*H*N^2*d / step time (true d, no padding)
  roofline   for the dominant kernel (the fused attention kernel), timed with
             events on the launch stream inside the timed region; the bound is
             the vector ALU: algorithmic lane-instructions per (query, key)
             pair x pairs / kernel time, against 256 CUs x 4 SIMDs x 16 lanes x
             2.4 GHz = 39.3 T lane-instructions/s
  cpu_baseline  the CPU oracle timed on this host on a bounded sample of rows
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

# Algorithmic vector-ALU work per (query, key) pair of the fused kernel, in issue
# slots of a 16-lane SIMD ("lane-instructions"): bias unpack, scale, logit + bias,
# running max, exponent FMA, round-to-byte, row-sum add (7 full-rate instructions)
# plus one exponential.  v_exp_f32 issues at half rate on this chip (measured with
# a dependent-free instruction stream: 2 slots), hence 7 + 2.
ALU_SLOTS_PER_PAIR = 7 + 2
# The same list with what the kernel's design makes unnecessary taken out (the FP4
# matrix-core logits arrive in fp32 with the bias already added; v_max3 takes two
# values per instruction; the sign offset of the byte codes costs a quarter
# instruction): unpack 1, scale 1, max 0.5, FMA 1, exp 2, add 1, round 1, xor 0.25.
ALU_SLOTS_PER_PAIR_STRICT = 7.75
ALU_PEAK_TLANEOPS = 256 * 4 * 16 * 2.4e9 / 1e12   # 39.32
MFMA_I8_PEAK_TOPS = 5033.0
HBM_PEAK_GBS = 8000.0
# HBM bytes per launch of the fused kernel from rocprofv3 --pmc FETCH_SIZE and WRITE_SIZE
# (two runs of this file; KiB per dispatch, scaled by what the same counters read for a
# 512 MiB device-to-device copy: x2.0 and x1.0).  Summaries under profiles/.
FUSED_TRAFFIC_BYTES = {"vit_hires": 8.83e9 + 0.07e9}


def parse():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=20)
    ap.add_argument("--warmup", type=int, default=3)
    ap.add_argument("--workload", default="vit_hires")
    ap.add_argument("--others", action="store_true", help="also time the other workloads (extra field)")
    ap.add_argument("--axial", action="store_true",
                    help="also time the workload with the in-kernel decomposed relative-position bias (extra field)")
    ap.add_argument("--relpos", action="store_true",
                    help="also time the DiT workloads with the in-kernel relative-position table (extra field)")
    ap.add_argument("--sweep", choices=["hd128"], help="also time the head-dim-128 sequence-length sweep (extra field)")
    ap.add_argument("--sweep-bias", action="store_true", help="run the sweep with a dense bias (up to N = 16384)")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-bias", action="store_true", help="run without the bias term (not the headline config)")
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
    """Gy, Gx with Gy * Gx = N, Gx in {16, 32} and Gy <= 32 (the limits of binattn_attend_relpos)."""
    for gx in (32, 16):
        if N % gx == 0 and N // gx <= 32 and (gx == 16 or N // gx >= 16):
            return N // gx, gx
    return None


def run_workload(name, steps, warmup, with_bias=True, axial=False, relpos=False, graph=False):
    import torch
    from paper_2603_09582_amd import binding as ba
    from paper_2603_09582_amd import workloads as wl

    w = wl.WORKLOADS[name]
    x = wl.make_inputs(w, device="cuda", with_bias=with_bias and not axial and not relpos)
    B, H, N, d = w.B, w.H, w.N, w.d
    W = (d + 31) // 32
    dev = x.q.device
    q_bits = torch.empty(B, H, N, W, dtype=torch.int32, device=dev)
    k_bits = torch.empty_like(q_bits)
    mu_q = torch.empty(B, H, dtype=torch.float32, device=dev)
    mu_k = torch.empty_like(mu_q)
    out = torch.empty(B, H, N, d, dtype=torch.bfloat16, device=dev)
    ws = ba.alloc_workspace(B, H, N, d, dev)

    if axial:  # decomposed relative-position bias: two small tables per head instead of [H, N, N]
        Gy, Gx = axial_grid(N)
        gen = torch.Generator(device="cuda").manual_seed(w.seed + 1000)
        by = torch.randn(H, 2 * Gy - 1, generator=gen, device=dev) * 0.02
        bx = torch.randn(H, 2 * Gx - 1, generator=gen, device=dev) * 0.02

    if relpos:  # the full relative-position table of each head instead of [H, N, N]
        Gy, Gx = relpos_grid(N)
        gen = torch.Generator(device="cuda").manual_seed(w.seed + 2000)
        table = torch.randn(H, 2 * Gy - 1, 2 * Gx - 1, generator=gen, device=dev) * 0.02

    ev = [[torch.cuda.Event(enable_timing=True) for _ in range(4)] for _ in range(steps)]

    def step(e=None):
        if e: e[0].record()
        ba.pack_qk(x.q, x.k, q_bits, k_bits, mu_q, mu_k)
        if e: e[1].record()
        ba.prepare_kv(k_bits, x.v, ws)
        if e: e[2].record()
        if axial:
            ba.attend_axial(q_bits, mu_q, mu_k, by, bx, x.scale, d, ws, out=out)
        elif relpos:
            ba.attend_relpos(q_bits, mu_q, mu_k, table, x.scale, d, ws, out=out)
        else:
            ba.attend(q_bits, mu_q, mu_k, x.bias, x.scale, d, ws, out=out)
        if e: e[3].record()

    for _ in range(warmup):
        step()
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for i in range(steps):
        step(ev[i])
    torch.cuda.synchronize()
    t1 = time.perf_counter()

    ms_step = (t1 - t0) * 1e3 / steps
    pack_ms = sum(e[0].elapsed_time(e[1]) for e in ev) / steps
    prep_ms = sum(e[1].elapsed_time(e[2]) for e in ev) / steps
    fused_ms = sum(e[2].elapsed_time(e[3]) for e in ev) / steps
    pairs = w.pairs
    res = {
        "workload": name, "B": B, "H": H, "N": N, "d": d,
        "ms_per_step": ms_step, "pack_ms": pack_ms, "prepare_ms": prep_ms, "fused_ms": fused_ms,
        "tops_equiv": w.equiv_ops / (ms_step * 1e-3) / 1e12,
        "fused_tops_equiv": w.equiv_ops / (fused_ms * 1e-3) / 1e12,
        # pack kernel: 2 B read per Q/K element + packed words written
        "pack_gbs": (2 * B * H * N * d * 2 + 2 * B * H * N * W * 4) / (pack_ms * 1e-3) / 1e9,
        "alu_tlaneops": ALU_SLOTS_PER_PAIR * pairs / (fused_ms * 1e-3) / 1e12,
        "mfma_tops_algorithmic": 4 * pairs * d / (fused_ms * 1e-3) / 1e12,
        # fused-kernel algorithmic HBM bytes: bias once per head (batch-shared), sign words,
        # K operand + V codes once per head, output
        "fused_hbm_bytes": 2 * H * N * N + B * H * N * (W * 4 + 2 * 32 * W + 2 * d),
    }
    res["fused_hbm_gbs"] = res["fused_hbm_bytes"] / (fused_ms * 1e-3) / 1e9
    if N <= 256 and not axial and not relpos:  # the single-launch form of the same step (binattn_forward_fused)
        for _ in range(warmup):
            ba.forward_fused(x.q, x.k, x.v, x.bias, x.scale, out=out)
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for _ in range(steps):
            ba.forward_fused(x.q, x.k, x.v, x.bias, x.scale, out=out)
        torch.cuda.synchronize()
        one_ms = (time.perf_counter() - t0) * 1e3 / steps
        res["single_launch_ms_per_step"] = one_ms
        res["single_launch_tops_equiv"] = w.equiv_ops / (one_ms * 1e-3) / 1e12
    if graph and N <= 4096:
        # the same three calls captured once into a HIP graph and replayed: what a caller whose
        # loop is launch-bound gets (the library allocates nothing and never synchronises)
        side = torch.cuda.Stream()
        side.wait_stream(torch.cuda.current_stream())
        with torch.cuda.stream(side):
            step()
        torch.cuda.current_stream().wait_stream(side)
        torch.cuda.synchronize()
        g = torch.cuda.CUDAGraph()
        with torch.cuda.graph(g):
            step()
        for _ in range(warmup):
            g.replay()
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for _ in range(steps):
            g.replay()
        torch.cuda.synchronize()
        g_ms = (time.perf_counter() - t0) * 1e3 / steps
        res["graph_ms_per_step"] = g_ms
        res["graph_tops_equiv"] = w.equiv_ops / (g_ms * 1e-3) / 1e12
    return res, x


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


def main():
    a = parse()
    if a.gpus != 1:
        print("bench.py measures one GPU: this build has no multi-GPU path (each (batch, head) problem "
              "is independent and would shard over them, or over query rows, with no exchange step). Run with --gpus 1.", file=sys.stderr)
        sys.exit(2)
    import torch
    assert torch.cuda.is_available(), "bench.py needs a GPU"
    from paper_2603_09582_amd import workloads as wl

    res, x = run_workload(a.workload, a.steps, a.warmup, with_bias=not a.no_bias)
    line = {
        "metric": "attention TOPS-equiv (4*B*H*N^2*d/s), whole hot path (pack_qk + prepare_kv + attend)",
        "value": res["tops_equiv"], "unit": "TOPS-equiv", "n_gpus": 1, "steps": a.steps, "warmup": a.warmup,
        "ms_per_step": res["ms_per_step"], "higher_is_better": True, "scaling": "weak",
        "vs_baseline": None, "dtype": "int8 x int8 -> int32 contractions (1-bit Q,K; u8 P; s8 V), fp32 softmax",
        "data": "synthetic",
        "config": {"workload": f"{a.workload} (B={res['B']}, H={res['H']}, N={res['N']}, d={res['d']}, bf16 Q/K/V, "
                               f"dense bf16 bias [H,N,N] shared over the batch, scale 1/sqrt(d))"},
        "kernels_ms": {"pack_qk": res["pack_ms"], "prepare_kv": res["prepare_ms"], "attend": res["fused_ms"]},
        "fused_kernel_tops_equiv": res["fused_tops_equiv"],
        "pack_kernel_gbs": res["pack_gbs"],
        "roofline": {"bound": "alu", "achieved": res["alu_tlaneops"], "peak": ALU_PEAK_TLANEOPS,
                     "unit": "T lane-instr/s", "frac": res["alu_tlaneops"] / ALU_PEAK_TLANEOPS,
                     "traffic": None if a.no_bias else FUSED_TRAFFIC_BYTES.get(a.workload),
                     "kernel": "fused_kernel (binattn_attend)", "kernel_ms": res["fused_ms"],
                     "algorithmic_lane_instr_per_pair": ALU_SLOTS_PER_PAIR,
                     "frac_strict_count": res["alu_tlaneops"] / ALU_PEAK_TLANEOPS
                                          * ALU_SLOTS_PER_PAIR_STRICT / ALU_SLOTS_PER_PAIR,
                     "algorithmic_hbm_bytes": res["fused_hbm_bytes"]},
        "roofline_other_bounds": {
            "mfma_int8_frac": res["mfma_tops_algorithmic"] / MFMA_I8_PEAK_TOPS,
            "hbm_frac": res["fused_hbm_gbs"] / HBM_PEAK_GBS, "hbm_gbs": res["fused_hbm_gbs"]},
    }
    if a.others:
        others = []
        for name in wl.WORKLOAD_ORDER:
            if name == a.workload:
                continue
            del x
            torch.cuda.empty_cache()
            r, x = run_workload(name, max(5, a.steps), a.warmup, graph=True)
            r["alu_frac"] = r["alu_tlaneops"] / ALU_PEAK_TLANEOPS
            others.append(r)
        line["other_workloads"] = others
        del x
        torch.cuda.empty_cache()
        _, x = run_workload(a.workload, 1, 0)   # the headline inputs again, for the CPU leg
    if a.axial and axial_grid(wl.WORKLOADS[a.workload].N):
        del x
        torch.cuda.empty_cache()
        r, xa = run_workload(a.workload, a.steps, a.warmup, axial=True)
        del xa
        torch.cuda.empty_cache()
        Gy, Gx = axial_grid(r["N"])
        line["axial_bias"] = {"grid": [Gy, Gx], "ms_per_step": r["ms_per_step"], "attend_ms": r["fused_ms"],
                              "tops_equiv": r["tops_equiv"], "fused_kernel_tops_equiv": r["fused_tops_equiv"],
                              "note": "b_ij = y[iy-jy] + x[ix-jx] from two fp32 tables per head held in LDS"}
        _, x = run_workload(a.workload, 1, 0)
    if a.relpos:
        del x
        torch.cuda.empty_cache()
        rows = []
        for name in ("dit_xl2_256", "dit_xl2_512"):
            r, xr = run_workload(name, max(5, a.steps), a.warmup, relpos=True)
            del xr
            torch.cuda.empty_cache()
            rows.append({"workload": name, "grid": list(relpos_grid(r["N"])), "ms_per_step": r["ms_per_step"],
                         "attend_ms": r["fused_ms"], "tops_equiv": r["tops_equiv"],
                         "fused_kernel_tops_equiv": r["fused_tops_equiv"],
                         "alu_frac": r["alu_tlaneops"] / ALU_PEAK_TLANEOPS})
        # ... and the whole layer in one launch where it applies (N <= 256)
        import torch as _t
        from paper_2603_09582_amd import binding as _ba
        w256 = wl.WORKLOADS["dit_xl2_256"]
        x256 = wl.make_inputs(w256, device="cuda", with_bias=False)
        gen = _t.Generator(device="cuda").manual_seed(w256.seed + 2000)
        table = _t.randn(w256.H, 31, 31, generator=gen, device="cuda") * 0.02
        o256 = _t.empty_like(x256.q)
        for _ in range(a.warmup):
            _ba.forward_fused_relpos(x256.q, x256.k, x256.v, table, x256.scale, out=o256)
        _t.cuda.synchronize()
        t0 = time.perf_counter()
        for _ in range(max(5, a.steps)):
            _ba.forward_fused_relpos(x256.q, x256.k, x256.v, table, x256.scale, out=o256)
        _t.cuda.synchronize()
        one_ms = (time.perf_counter() - t0) * 1e3 / max(5, a.steps)
        rows[0]["single_launch_ms_per_step"] = one_ms
        rows[0]["single_launch_tops_equiv"] = w256.equiv_ops / (one_ms * 1e-3) / 1e12
        del x256, o256
        line["relpos_table_bias"] = {"note": "b_ij = table[iy-jy][ix-jx], the head's fp32 table held in LDS",
                                     "workloads": rows}
        _, x = run_workload(a.workload, 1, 0)
    if a.sweep:
        del x
        torch.cuda.empty_cache()
        rows = []
        for name in wl.SWEEP_HD128:
            w = wl.WORKLOADS[name]
            if a.sweep_bias and w.N > 16384:
                continue
            r, xs = run_workload(name, max(5, a.steps), a.warmup, with_bias=a.sweep_bias)
            del xs
            torch.cuda.empty_cache()
            r["bias"] = bool(a.sweep_bias)
            rows.append({k: r[k] for k in ("workload", "B", "H", "N", "d", "bias", "ms_per_step", "pack_ms",
                                           "prepare_ms", "fused_ms", "tops_equiv", "fused_tops_equiv")})
        line["sweep_hd128"] = rows
        _, x = run_workload(a.workload, 1, 0)
    if a.no_bias:
        line["config"]["workload"] += " -- WITHOUT bias (diagnostic run)"
    if not a.no_cpu_baseline and not a.no_bias:
        line["cpu_baseline"] = cpu_baseline(x, a.cpu_seconds)
    print(json.dumps(line))


if __name__ == "__main__":
    main()
