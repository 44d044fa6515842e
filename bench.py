#!/usr/bin/env python3
"""Benchmark of the Skiparse-2D attention hot path on one MI355X.

One step = one fused skiparse_attn_fwd call (token-wise, s=2) on the 768P-shaped workload: B=1, 40 heads,
head_dim 128, grid 21x48x80 (80,640 tokens; 160 attention units of 20,160 tokens), seed 2.  Inputs are synthetic bf16
N(0,1) tensors already resident in HBM.  Prints ONE JSON line; exits non-zero if a parity check of a timed
configuration fails.  Besides the headline the default run times, under `extras`, every other workload as it is stated:
the group-wise call and the unfused path (3 permutes + attention + unpermute) on the same tensors; the 480P workload
(seed 1, token-wise, unfused and fused, sampled-row parity); the hybrid comparison (seed 3: dense, token-wise and
group-wise on ONE set of tensors, speed-ups); the 8-bit variant (seed 4, group-wise, parity against the oracle on the
unquantised inputs); the permutes (HBM GB/s), the backward pass, the any-resolution mode; and it times the float64
oracle on a bounded sample of query rows on the host cores, using those rows as a parity check of the headline.
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

PEAK_BF16_TFLOPS = 2500.0  # MI355X dense bf16 MFMA peak
PEAK_FP8_TFLOPS = 5000.0
PEAK_HBM_GBS = 8000.0
# HBM bytes per launch of the headline kernel, measured with rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE and written by
# `bench.py --traffic-from <dir> ...` (see write_traffic); the file records the commit it was taken at.
TRAFFIC_FILE = os.path.join(ROOT, "profiles", "traffic.json")
HEADLINE_KERNEL = "attn_fwd_bf16_kernel<128, 1, false>"
COPY_KERNEL = "permute_rows_kernel"  # a plain copy of known size in the same runs: gives the counters' scale factors
# Paper context only (end-to-end model speed-ups on other hardware; Tab. 2): not comparable to a kernel figure.
PAPER_CONTEXT = {"e2e_speedup_h200_bf16": 1.64, "e2e_speedup_ascend950pr_hif8_720p": 1.69, "e2e_speedup_ascend950pr_hif8_768p": 2.27}


def time_calls(fn, iters, warmup=3):
    """Milliseconds per call, from events on the stream the kernels are launched on, one pair per call:
    {"avg", "median", "min"}.  At least three warm-up calls."""
    import torch

    for _ in range(max(warmup, 3)):
        fn()
    torch.cuda.synchronize()
    evs = [torch.cuda.Event(enable_timing=True) for _ in range(iters + 1)]
    evs[0].record()
    for i in range(iters):
        fn()
        evs[i + 1].record()
    torch.cuda.synchronize()
    per = sorted(evs[i].elapsed_time(evs[i + 1]) for i in range(iters))
    return {"avg": evs[0].elapsed_time(evs[-1]) / iters, "median": per[len(per) // 2], "min": per[0]}


def ms3(t):
    return {k: round(v, 4) for k, v in t.items()}


def write_traffic(dirs, commit):
    """Reads the counter_collection CSVs of two rocprofv3 --pmc runs of this benchmark (FETCH_SIZE in one, WRITE_SIZE in the other;
    KiB per dispatch), scales each counter by what it reads for the permute kernel, a copy of known size in the same run, and
    writes profiles/traffic.json.  Needs no GPU."""
    import collections
    import csv
    import glob

    import synth_inputs as si

    w = si.WORKLOADS["768p"]
    copy_kib = w.B * w.N * w.heads * w.D * 2 / 1024.0  # the permute reads and writes one tensor
    vals = collections.defaultdict(lambda: collections.defaultdict(list))
    for d in dirs:
        for f in glob.glob(os.path.join(d, "**", "*counter_collection.csv"), recursive=True):
            for row in csv.DictReader(open(f)):
                vals[row["Counter_Name"]][row["Kernel_Name"]].append(float(row["Counter_Value"]))
    out = {"commit": commit, "workload": "768p", "kernel": HEADLINE_KERNEL, "copy_kernel_kib": copy_kib}
    for ctr in ("FETCH_SIZE", "WRITE_SIZE"):
        head = [v for k, v in vals[ctr].items() if HEADLINE_KERNEL in k]
        cp = [v for k, v in sorted(vals[ctr].items()) if COPY_KERNEL in k]
        if not head or not cp:
            raise SystemExit(f"bench.py: {ctr} of {HEADLINE_KERNEL} or {COPY_KERNEL} not found under {dirs}")
        head_kib = sum(head[0]) / len(head[0])
        copy_read = sum(cp[0]) / len(cp[0])
        out[ctr] = {"kib_per_launch": head_kib, "copy_kernel_reads_kib": copy_read, "factor": round(copy_kib / copy_read, 3)}
    out["bytes_per_launch"] = sum(out[c]["kib_per_launch"] * out[c]["factor"] for c in ("FETCH_SIZE", "WRITE_SIZE")) * 1024.0
    with open(TRAFFIC_FILE, "w") as fh:
        json.dump(out, fh, indent=1)
        fh.write("\n")
    print(json.dumps(out))


def read_traffic():
    try:
        with open(TRAFFIC_FILE) as fh:
            t = json.load(fh)
        return t["bytes_per_launch"], t.get("commit")
    except (OSError, ValueError, KeyError):
        return None, None


def main() -> int:
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=50)
    ap.add_argument("--warmup", type=int, default=10, help="untimed steps before the timed ones (the first call after idle is 10 %% slower and the clock settles over the next few)")
    ap.add_argument("--workload", default="768p", choices=["480p", "768p"])
    ap.add_argument("--cpu-rows", type=int, default=16384, help="query rows the oracle computes for cpu_baseline")
    ap.add_argument("--skip-extras", action="store_true", help="only the headline timing (used under the profiler)")
    ap.add_argument("--extras", default="probe,group,unfused,permute,ssp,chain,bwd,c2,c4,c5,pad,cpu",
                    help="comma list of the extra sections to run: probe (MFMA-only kernels: attainable matrix throughput), group, unfused, permute, "
                         "ssp (one rank's local rearrangements of Sparse Sequence Parallelism), chain (sparse layout in, other pattern's layout out), bwd (backward pass), c2 (the 480P workload: unfused and fused, "
                         "parity), c4 (hybrid comparison on seed 3: dense, token-wise, group-wise), c5 (8-bit variant, group-wise, seed 4, parity), "
                         "pad (720P-shaped grid in the any-resolution mode), cpu (oracle baseline + parity of the headline)")
    ap.add_argument("--traffic-from", nargs="+", metavar="DIR", help="no benchmark: read rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE output of this "
                    "benchmark from these folders and write profiles/traffic.json")
    ap.add_argument("--commit", default="unknown", help="with --traffic-from: the commit the profiled library was built from")
    args = ap.parse_args()
    if args.traffic_from:
        write_traffic(args.traffic_from, args.commit)
        return 0
    if args.gpus != 1:
        print("bench.py: this build runs on ONE GPU only (no collectives, no sharding); use --gpus 1", file=sys.stderr)
        return 2

    import numpy as np
    import torch

    import paper_2605_28691_amd as sk
    import synth_inputs as si
    from paper_2605_28691_amd import probe

    if not torch.cuda.is_available():
        print("bench.py: no GPU visible", file=sys.stderr)
        return 2
    torch.cuda.set_device(0)
    sk.lib()
    w = si.WORKLOADS[args.workload]
    t0 = time.time()
    q, k, v = si.make_qkv(w)
    qd, kd, vd = q.cuda(), k.cuda(), v.cuda()
    out = torch.empty_like(qd)
    gen_s = time.time() - t0
    T, H, W, s = w.T, w.H, w.W, w.s
    flops = w.sparse_flops()

    def fused(pattern):
        return lambda: sk.skiparse_attn_fwd(qd, kd, vd, T, H, W, s, pattern, scale=w.scale, fused=True, out=out)

    # ---- headline: W warm-up steps, then exactly K timed steps bracketed by synchronisation
    for _ in range(args.warmup):
        fused("token")()
    torch.cuda.synchronize()
    evs = [torch.cuda.Event(enable_timing=True) for _ in range(args.steps + 1)]  # on the stream the kernels are launched on
    wall0 = time.perf_counter()
    evs[0].record()
    for i in range(args.steps):
        fused("token")()
        evs[i + 1].record()
    torch.cuda.synchronize()
    wall_ms = (time.perf_counter() - wall0) * 1e3 / args.steps
    kernel_ms = evs[0].elapsed_time(evs[-1]) / args.steps  # one kernel per step: this is the kernel's average duration
    per_step = sorted(evs[i].elapsed_time(evs[i + 1]) for i in range(args.steps))
    ms = wall_ms
    tflops = flops / (ms * 1e-3) / 1e12
    traffic, traffic_commit = read_traffic() if w.name == "768p" else (None, None)
    result = {
        "metric": "skiparse2d_attn_fwd_effective_tflops",
        "value": round(tflops, 2),
        "unit": "TFLOP/s",
        "n_gpus": 1,
        "steps": args.steps,
        "warmup": args.warmup,
        "ms_per_step": round(ms, 4),
        "higher_is_better": True,
        "scaling": "weak",
        "vs_baseline": None,
        "dtype": "bf16",
        "data": "synthetic",
        "config": {
            "workload": f"{w.name}: B={w.B} heads={w.heads} head_dim={w.D} grid={T}x{H}x{W} ({w.N} tokens) s={s} token-wise, fused kernel",
            "units": w.B * w.heads * s * s,
            "tokens_per_subsequence": w.Nsub,
            "flop_per_call": flops,
            "seed": w.seed,
        },
        "pct_of_bf16_mfma_peak": round(100.0 * tflops / PEAK_BF16_TFLOPS, 2),
        "roofline": {
            "bound": "mfma",
            "achieved": round(flops / (kernel_ms * 1e-3) / 1e12, 2),
            "peak": PEAK_BF16_TFLOPS,
            "unit": "TFLOP/s",
            "frac": round(flops / (kernel_ms * 1e-3) / 1e12 / PEAK_BF16_TFLOPS, 4),
            "traffic": traffic,
            "traffic_source": "profiles/traffic.json (rocprofv3 --pmc FETCH_SIZE, WRITE_SIZE; scaled by the permute kernel's readings)" if traffic else None,
            "traffic_commit": traffic_commit,
            "algorithmic_bytes": 4 * qd.numel() * 2,
            "kernel": "attn_fwd_bf16_kernel<128>",
            "kernel_ms": round(kernel_ms, 4),
            "kernel_ms_min": round(per_step[0], 4),
            "kernel_ms_median": round(per_step[len(per_step) // 2], 4),
        },
        "paper_context": PAPER_CONTEXT,
        "input_generation_s": round(gen_s, 1),
    }

    # the nominal peak recomputed from what the device reports: 4 SIMDs x 1024 bf16 FLOP per clock per compute unit (one 32x32x16
    # MFMA = 32768 FLOP in 32 clocks per SIMD)
    cus, clock_khz = probe.device_info(0)
    result["device"] = {
        "name": torch.cuda.get_device_properties(0).name,
        "compute_units": cus,
        "clock_mhz": round(clock_khz / 1e3, 1),
        "bf16_tflops_from_device": round(cus * 4096 * clock_khz / 1e9, 1),
        "frac_of_peak_from_device": round(flops / (kernel_ms * 1e-3) / 1e12 / (cus * 4096 * clock_khz / 1e9), 4),
    }

    sections = set() if args.skip_extras else {x for x in args.extras.split(",") if x}
    extras = {}
    failures = []
    if "probe" in sections:
        # what the matrix pipe sustains by itself on random operands (power-managed clock): nothing but MFMAs, 2 wavefronts per
        # SIMD (more wavefronts per SIMD measure lower: the pipe runs without gaps only on back-to-back MFMAs of one wavefront)
        gp = torch.Generator(device="cpu")
        gp.manual_seed(99)
        rnd = torch.randn(8192, generator=gp, dtype=torch.float32)
        sink = torch.empty(512 * 256, dtype=torch.float32, device="cuda")
        for name, ops, fp8, n_it in (("bf16", rnd.to(torch.bfloat16).cuda(), False, 80000),
                                     ("fp8", rnd.repeat(2).to(torch.float8_e4m3fn).view(torch.uint8).cuda(), True, 40000),
                                     ("bf16_zero_operands", torch.zeros(8192, dtype=torch.bfloat16, device="cuda"), False, 80000)):
            fl = [0.0]

            def run_probe():
                fl[0] = probe.mfma_probe(ops, sink, fp8, 512, n_it)

            p_ms = time_calls(run_probe, 5)["avg"]
            extras[f"mfma_only_{name}_tflops"] = round(fl[0] / p_ms / 1e9, 1)
        result["roofline"]["attainable_mfma_only"] = extras["mfma_only_bf16_tflops"]
        # the same with the A operand of every MFMA read from LDS, as an attention kernel must feed its products
        lds_ops = rnd.to(torch.bfloat16).cuda()
        fl = [0.0]

        def lprobe():
            fl[0] = probe.mfma_lds_probe(lds_ops, sink, 512, 40000)

        l_ms = time_calls(lprobe, 5)["avg"]
        extras["mfma_lds_fed_bf16_tflops"] = round(fl[0] / l_ms / 1e9, 1)
        result["roofline"]["attainable_mfma_lds_fed"] = extras["mfma_lds_fed_bf16_tflops"]
        # how much vector-ALU work the matrix pipe hides: the same loop on zero operands (full clock) with n independent FMAs per MFMA
        zero_ops = torch.zeros(8192, dtype=torch.bfloat16, device="cuda")
        for n in (0, 2, 4, 6, 8):
            fl = [0.0]

            def vprobe():
                fl[0] = probe.mfma_valu_probe(zero_ops, sink, n, 512, 100000)

            v_ms = time_calls(vprobe, 3)["avg"]
            extras[f"mfma_zero_operands_with_{n}_fma_per_mfma_tflops"] = round(fl[0] / v_ms / 1e9, 1)
        # what the LDS delivers to the two kinds of fragment read the attention kernels use (nominal clock assumed: the probe draws little power)
        sink2 = torch.empty(512 * 512, dtype=torch.float32, device="cuda")
        for kind, name in ((0, "ds_read_b128"), (1, "ds_read_b64_tr_b16")):
            nb = [0.0]

            def rprobe():
                nb[0] = probe.lds_read_probe(lds_ops, sink2, kind, 512, 20000)

            r_ms = time_calls(rprobe, 3)["avg"]
            extras[f"lds_{name}_bytes_per_clk_per_cu"] = round(nb[0] / (r_ms * 1e-3) / cus / (clock_khz * 1e3), 1)
        del sink, sink2
    it = max(5, min(10, args.steps))
    tensor_bytes = qd.numel() * 2
    if "group" in sections and "group" in w.patterns:
        g_t = time_calls(fused("group"), it)
        extras["fused_group_ms"] = round(g_t["avg"], 4)
        extras["fused_group_ms_median_min"] = [round(g_t["median"], 4), round(g_t["min"], 4)]
        extras["fused_group_tflops"] = round(flops / g_t["avg"] / 1e9, 2)
    if "unfused" in sections or "permute" in sections:
        need = sk.skiparse_workspace_bytes(w.B, w.heads, T, H, W, w.D, s, False)
        ws = torch.empty(need, dtype=torch.uint8, device="cuda")
        if "unfused" in sections:
            for pattern in w.patterns:
                u_t = time_calls(lambda: sk.skiparse_attn_fwd(qd, kd, vd, T, H, W, s, pattern, scale=w.scale, fused=False, out=out, workspace=ws), it)
                extras[f"unfused_{pattern}_ms"] = round(u_t["avg"], 4)
        if "permute" in sections:
            yp = ws[:tensor_bytes].view(torch.bfloat16).view(s * s * w.B, w.Nsub, w.heads, w.D)
            p_ms = time_calls(lambda: sk.skiparse_permute(qd, T, H, W, s, "token", out=yp), 10)["avg"]
            up_ms = time_calls(lambda: sk.skiparse_unpermute(yp, T, H, W, s, "token", out=out), 10)["avg"]
            extras["permute_ms"] = round(p_ms, 4)
            extras["permute_GBps"] = round(2 * tensor_bytes / p_ms / 1e6, 1)  # one read and one write of the tensor
            extras["unpermute_ms"] = round(up_ms, 4)
            extras["unpermute_GBps"] = round(2 * tensor_bytes / up_ms / 1e6, 1)
            extras["permute_frac_of_hbm_peak"] = round(2 * tensor_bytes / p_ms / 1e6 / PEAK_HBM_GBS, 4)
            extras["unpermute_frac_of_hbm_peak"] = round(2 * tensor_bytes / up_ms / 1e6 / PEAK_HBM_GBS, 4)
            if "group" in w.patterns:
                pg_ms = time_calls(lambda: sk.skiparse_permute(qd, T, H, W, s, "group", out=yp), 10)["avg"]
                upg_ms = time_calls(lambda: sk.skiparse_unpermute(yp, T, H, W, s, "group", out=out), 10)["avg"]
                extras["permute_group_GBps"] = round(2 * tensor_bytes / pg_ms / 1e6, 1)
                extras["unpermute_group_GBps"] = round(2 * tensor_bytes / upg_ms / 1e6, 1)
                sk.skiparse_permute(qd, T, H, W, s, "token", out=yp)
                yg = ws[tensor_bytes : 2 * tensor_bytes].view(torch.bfloat16).view(s * s * w.B, w.Nsub, w.heads, w.D)
                sw_ms = time_calls(lambda: sk.skiparse_switch_pattern(yp, T, H, W, s, "token", out=yg), 10)["avg"]
                extras["switch_tsa_to_gsa_ms"] = round(sw_ms, 4)
                extras["switch_GBps"] = round(2 * tensor_bytes / sw_ms / 1e6, 1)
                del yg
            del yp
        del ws
    if "ssp" in sections and "group" in w.patterns:
        # Sparse Sequence Parallelism (Sec. 3.3), the share of one rank of a group of four (one subsequence each): the local
        # rearrangements before and after the all-to-all; the exchange itself needs a second GPU and is not part of this build
        shard = sk.skiparse_permute(qd, T, H, W, s, "token")[2:3].contiguous()
        send = sk.skiparse_ssp_pack(shard, T, H, W, s, 4)
        back = torch.empty_like(shard)
        pk_ms = time_calls(lambda: sk.skiparse_ssp_pack(shard, T, H, W, s, 4, out=send), 20)["avg"]
        up_ms = time_calls(lambda: sk.skiparse_ssp_unpack(send, T, H, W, s, 4, out=back), 20)["avg"]
        shard_bytes = shard.numel() * 2
        extras["ssp_rank_share"] = {"group_size": 4, "shard_MB": round(shard_bytes / 1e6, 1), "pack_ms": round(pk_ms, 4),
                                    "pack_GBps": round(2 * shard_bytes / pk_ms / 1e6, 1), "unpack_ms": round(up_ms, 4),
                                    "unpack_GBps": round(2 * shard_bytes / up_ms / 1e6, 1)}
        del shard, send, back
    if "chain" in sections and "group" in w.patterns:
        # a block of a chain: q, k, v already in the token-wise sparse layout, output written in the group-wise layout
        qs, ks, vs = (sk.skiparse_permute(t, T, H, W, s, "token") for t in (qd, kd, vd))
        os_ = torch.empty_like(qs)
        c_ms = time_calls(lambda: sk.skiparse_attn_fwd_sparse(qs, ks, vs, T, H, W, s, "token", "other", scale=w.scale, out=os_), it)["avg"]
        extras["chain_token_to_group_ms"] = round(c_ms, 4)
        extras["chain_token_to_group_tflops"] = round(flops / c_ms / 1e9, 2)
        del qs, ks, vs, os_
    if "bwd" in sections:
        # training step of the layer: forward that keeps the log-sum-exp, then dQ, dK, dV (delta + two launches)
        dout = si.make_dout(w).cuda()
        lse = torch.empty((s * s * w.B, w.heads, w.Nsub), dtype=torch.float32, device="cuda")
        grads = [torch.empty_like(qd) for _ in range(3)]
        wsb = torch.empty(sk.skiparse_bwd_workspace_bytes(w.B, w.heads, T, H, W, w.D, s, "token"), dtype=torch.uint8, device="cuda")
        fl_ms = time_calls(lambda: sk.skiparse_attn_fwd_lse(qd, kd, vd, T, H, W, s, "token", scale=w.scale, out=out, lse=lse), it)["avg"]
        b_t = time_calls(lambda: sk.skiparse_attn_bwd(qd, kd, vd, out, dout, lse, T, H, W, s, "token", scale=w.scale, dq=grads[0], dk=grads[1],
                                                      dv=grads[2], workspace=wsb), 5)
        b_ms = b_t["avg"]
        extras["fwd_lse_ms"] = round(fl_ms, 4)
        extras["bwd_ms"] = round(b_ms, 4)
        extras["bwd_ms_median_min"] = [round(b_t["median"], 4), round(b_t["min"], 4)]
        extras["bwd_effective_tflops"] = round(2.5 * flops / b_ms / 1e9, 2)  # five matrix products of the definition (forward has two)
        extras["bwd_executed_tflops"] = round(3.5 * flops / b_ms / 1e9, 2)   # seven are executed (S and dP are formed in both launches)
        extras["bwd_frac_of_bf16_peak_effective"] = round(2.5 * flops / b_ms / 1e9 / PEAK_BF16_TFLOPS, 4)
        del dout, lse, grads, wsb
    if "pad" in sections and w.name == "768p":
        # any-resolution mode on the paper's padded workload: 81 x 720 x 1280 video -> grid 21 x 45 x 80, padded to 21 x 48 x 80
        Hp_real = 45
        g = torch.Generator(device="cuda").manual_seed(5)
        shp = (w.B, T * Hp_real * W, w.heads, w.D)
        qp, kp, vp = (torch.randn(shp, generator=g, device="cuda", dtype=torch.bfloat16) for _ in range(3))
        op = torch.empty_like(qp)
        pad_ms = time_calls(lambda: sk.skiparse_attn_fwd(qp, kp, vp, T, Hp_real, W, s, "token", scale=w.scale, fused=True, pad=True, out=op), it)["avg"]
        # real work: every class holds the real rows h = p, p+2, ... < 45 and all 40 columns of its parity
        real_flops = 0.0
        for p_ in range(s):
            rows_c = len(range(p_, Hp_real, s))
            for q_ in range(s):
                n_c = T * rows_c * len(range(q_, W, s))
                real_flops += 4.0 * w.B * w.heads * float(n_c) ** 2 * w.D
        extras["pad720p_token_ms"] = round(pad_ms, 4)
        extras["pad720p_real_tflops"] = round(real_flops / pad_ms / 1e9, 2)
        # the 8-bit variant on the same padded workload (the paper reports its 8-bit numbers at 720 x 1280 too)
        pq8 = [sk.skiparse_quantize_fp8(t, T, Hp_real, W, s, "token", pad=True) for t in (qp, kp, vp)]
        p8_ms = time_calls(lambda: sk.skiparse_attn_fwd_fp8(pq8[0][0], pq8[1][0], pq8[2][0], pq8[0][1], pq8[1][1], pq8[2][1], T, Hp_real, W, s, "token",
                                                            scale=w.scale, out=op, pad=True), it)["avg"]
        extras["pad720p_fp8_token_ms"] = round(p8_ms, 4)
        extras["pad720p_fp8_real_tflops"] = round(real_flops / p8_ms / 1e9, 2)
        del pq8
        if "bwd" in sections:
            # the paper's training grid (Sec. 4.1): backward in the any-resolution mode
            dop = torch.randn(shp, generator=g, device="cuda", dtype=torch.bfloat16)
            opl, lsep = sk.skiparse_attn_fwd_lse(qp, kp, vp, T, Hp_real, W, s, "token", scale=w.scale, out=op, pad=True)
            gp = [torch.empty_like(qp) for _ in range(3)]
            wsp = torch.empty(sk.skiparse_bwd_workspace_bytes(w.B, w.heads, T, Hp_real, W, w.D, s, "token", pad=True), dtype=torch.uint8, device="cuda")
            pb_ms = time_calls(lambda: sk.skiparse_attn_bwd(qp, kp, vp, opl, dop, lsep, T, Hp_real, W, s, "token", scale=w.scale, dq=gp[0],
                                                            dk=gp[1], dv=gp[2], workspace=wsp, pad=True), 3)["avg"]
            extras["pad720p_bwd_ms"] = round(pb_ms, 4)
            extras["pad720p_bwd_effective_real_tflops"] = round(2.5 * real_flops / pb_ms / 1e9, 2)
            del dop, lsep, gp, wsp
        del qp, kp, vp, op

    def sampled_parity(o, rows, want, max_abs_bar, rel_l2_bar):
        r = torch.from_numpy(rows).cuda()
        got = o[r[:, 0], r[:, 2], r[:, 1]].cpu().to(torch.float64).numpy()
        ma = float(np.abs(got - want).max())
        rl = float(np.linalg.norm(got - want) / np.linalg.norm(want))
        return {"rows": int(rows.shape[0]), "max_abs": ma, "rel_l2": rl, "bars": [max_abs_bar, rel_l2_bar], "ok": bool(ma <= max_abs_bar and rl <= rel_l2_bar)}

    def random_rows(wl, n, seed):
        rng = np.random.default_rng(seed)
        return np.stack([rng.integers(0, wl.B, n), rng.integers(0, wl.heads, n), rng.integers(0, wl.N, n)], axis=1).astype(np.int64)

    if w.name == "768p" and "c2" in sections:
        # the 480P workload as stated: seed 1, token-wise, unfused permute + attention + unpermute (and the fused call beside it)
        import oracle

        w2 = si.WORKLOADS["480p"]
        q2, k2, v2 = si.make_qkv(w2)
        q2d, k2d, v2d = q2.cuda(), k2.cuda(), v2.cuda()
        o2 = torch.empty_like(q2d)
        ws2 = torch.empty(sk.skiparse_workspace_bytes(w2.B, w2.heads, w2.T, w2.H, w2.W, w2.D, w2.s, False), dtype=torch.uint8, device="cuda")
        a2 = (w2.T, w2.H, w2.W, w2.s, "token")
        u2 = time_calls(lambda: sk.skiparse_attn_fwd(q2d, k2d, v2d, *a2, scale=w2.scale, fused=False, out=o2, workspace=ws2), 20)
        rows2 = random_rows(w2, 4096, 321)
        want2 = oracle.skiparse_attention_rows(*(si.as_oracle_array(t) for t in (q2, k2, v2)), rows2, w2.T, w2.H, w2.W, w2.s, "token", w2.scale)
        torch.cuda.synchronize()
        par_unfused = sampled_parity(o2, rows2, want2, 2e-2, 5e-3)
        f2 = time_calls(lambda: sk.skiparse_attn_fwd(q2d, k2d, v2d, *a2, scale=w2.scale, fused=True, out=o2), 20)
        torch.cuda.synchronize()
        par_fused = sampled_parity(o2, rows2, want2, 2e-2, 5e-3)
        d2 = time_calls(lambda: sk.dense_attn_fwd(q2d, k2d, v2d, w2.T, w2.H, w2.W, scale=w2.scale, out=o2), 10)
        extras["config2_480p"] = {
            "seed": w2.seed, "pattern": "token", "grid": [w2.T, w2.H, w2.W], "heads": w2.heads,
            "unfused_ms": ms3(u2), "unfused_tflops": round(w2.sparse_flops() / u2["avg"] / 1e9, 2),
            "fused_ms": ms3(f2), "fused_tflops": round(w2.sparse_flops() / f2["avg"] / 1e9, 2),
            "dense_ms": ms3(d2), "speedup_vs_dense_unfused": round(d2["avg"] / u2["avg"], 3), "speedup_vs_dense_fused": round(d2["avg"] / f2["avg"], 3),
            "parity_unfused": par_unfused, "parity_fused": par_fused,
        }
        if not (par_unfused["ok"] and par_fused["ok"]):
            failures.append("config2_480p parity")
        del q2d, k2d, v2d, o2, ws2
    if w.name == "768p" and "c4" in sections:
        # hybrid-layer comparison as stated: ONE set of tensors (seed 3): dense, token-wise, group-wise
        w4 = si.WORKLOADS["hybrid"]
        q4, k4, v4 = (t.cuda() for t in si.make_qkv(w4))
        a4 = (w4.T, w4.H, w4.W)
        d4 = time_calls(lambda: sk.dense_attn_fwd(q4, k4, v4, *a4, scale=w4.scale, out=out), 5)
        t4 = time_calls(lambda: sk.skiparse_attn_fwd(q4, k4, v4, *a4, w4.s, "token", scale=w4.scale, fused=True, out=out), it)
        g4 = time_calls(lambda: sk.skiparse_attn_fwd(q4, k4, v4, *a4, w4.s, "group", scale=w4.scale, fused=True, out=out), it)
        # the paper's 40-block model (Sec. 4.1): 8 full-attention blocks and 32 sparse ones, token-wise and group-wise alternating;
        # attention time of the stack from these per-layer figures, against 40 full-attention calls
        hyb = 8 * d4["avg"] + 16 * t4["avg"] + 16 * g4["avg"]
        extras["config4_hybrid"] = {
            "seed": w4.seed, "dense_ms": ms3(d4), "dense_tflops": round(w4.dense_flops() / d4["avg"] / 1e9, 2),
            "token_ms": ms3(t4), "group_ms": ms3(g4),
            "speedup_token_vs_dense": round(d4["avg"] / t4["avg"], 3), "speedup_group_vs_dense": round(d4["avg"] / g4["avg"], 3),
            "hybrid_stack_attention_ms": round(hyb, 2), "hybrid_stack_speedup_vs_all_dense": round(40 * d4["avg"] / hyb, 3),
        }
        extras["dense_ms"] = round(d4["avg"], 4)
        extras["speedup_vs_dense"] = extras["config4_hybrid"]["speedup_token_vs_dense"]
        del q4, k4, v4
    if w.name == "768p" and "c5" in sections:
        # 8-bit variant as stated: seed 4, group-wise; quantise (fused with the rearrangement), then fp8 attention; accuracy
        # against the float64 oracle on the UNQUANTISED inputs
        import oracle

        w5 = si.WORKLOADS["fp8"]
        pat5 = w5.patterns[0]
        q5, k5, v5 = si.make_qkv(w5)
        q5d, k5d, v5d = q5.cuda(), k5.cuda(), v5.cuda()
        a5 = (w5.T, w5.H, w5.W, w5.s, pat5)
        q8, sq = sk.skiparse_quantize_fp8(q5d, *a5)
        k8, sk_ = sk.skiparse_quantize_fp8(k5d, *a5)
        v8, sv = sk.skiparse_quantize_fp8(v5d, *a5)
        qz = time_calls(lambda: sk.skiparse_quantize_fp8(q5d, *a5), 10)
        f8 = time_calls(lambda: sk.skiparse_attn_fwd_fp8(q8, k8, v8, sq, sk_, sv, *a5, scale=w5.scale, out=out), it)
        b5 = time_calls(lambda: sk.skiparse_attn_fwd(q5d, k5d, v5d, *a5, scale=w5.scale, fused=True, out=out), it)
        sk.skiparse_attn_fwd_fp8(q8, k8, v8, sq, sk_, sv, *a5, scale=w5.scale, out=out)
        torch.cuda.synchronize()
        rows5 = random_rows(w5, 4096, 654)
        want5 = oracle.skiparse_attention_rows(*(si.as_oracle_array(t) for t in (q5, k5, v5)), rows5, w5.T, w5.H, w5.W, w5.s, pat5, w5.scale)
        par5 = sampled_parity(out, rows5, want5, 6e-2, 2e-2)
        par5["note"] = ("against the float64 oracle on the unquantised inputs; on i.i.d. N(0,1) data the relative L2 of an ideal E4M3 pipeline is "
                        "itself ~5.4e-2 (tests/_fp8_emulation.py), so 'ok' is false here by the format, not by the kernel; the tests bound the "
                        "kernel by that emulation and assert the stated bars on inputs with a mean")
        extras["config5_fp8"] = {
            "seed": w5.seed, "pattern": pat5,
            "quantize_ms_per_tensor": ms3(qz), "quantize_GBps": round(3 * q5d.numel() / qz["avg"] / 1e6, 1),  # 2 bytes read + 1 written per element
            "attn_ms": ms3(f8), "attn_tflops": round(flops / f8["avg"] / 1e9, 2),
            "frac_of_fp8_mfma_peak": round(flops / f8["avg"] / 1e9 / PEAK_FP8_TFLOPS, 4),
            "bf16_same_inputs_ms": ms3(b5), "speedup_vs_bf16": round(b5["avg"] / f8["avg"], 3),
            "parity": par5,
        }
        if not (par5["max_abs"] <= 6e-2 and par5["rel_l2"] <= 8e-2):  # the format's floor with margin; the stated 2e-2 is reported above
            failures.append("config5_fp8 parity backstop")
        del q5d, k5d, v5d, q8, k8, v8
    # the other kernels against the roofline that bounds each (same form as the headline's object; figures from the sections above)
    others = {}
    if "permute_GBps" in extras:
        others["permute_rows_kernel (permute)"] = {"bound": "hbm", "achieved": extras["permute_GBps"], "peak": PEAK_HBM_GBS, "unit": "GB/s",
                                                   "frac": round(extras["permute_GBps"] / PEAK_HBM_GBS, 4)}
        others["permute_rows_kernel (unpermute)"] = {"bound": "hbm", "achieved": extras["unpermute_GBps"], "peak": PEAK_HBM_GBS, "unit": "GB/s",
                                                     "frac": round(extras["unpermute_GBps"] / PEAK_HBM_GBS, 4)}
    if "config5_fp8" in extras:
        c5 = extras["config5_fp8"]
        others["quantize_fp8_kernel"] = {"bound": "hbm", "achieved": c5["quantize_GBps"], "peak": PEAK_HBM_GBS, "unit": "GB/s",
                                         "frac": round(c5["quantize_GBps"] / PEAK_HBM_GBS, 4)}
        others["attn_fwd_fp8_kernel"] = {"bound": "mfma", "achieved": c5["attn_tflops"], "peak": PEAK_FP8_TFLOPS, "unit": "TFLOP/s",
                                         "frac": c5["frac_of_fp8_mfma_peak"]}
    if "bwd_ms" in extras:
        others["attn_bwd_kernel (dQ + dK,dV launches, 7 products executed)"] = {
            "bound": "mfma", "achieved": extras["bwd_executed_tflops"], "peak": PEAK_BF16_TFLOPS, "unit": "TFLOP/s",
            "frac": round(extras["bwd_executed_tflops"] / PEAK_BF16_TFLOPS, 4), "frac_on_the_5_product_definition": extras["bwd_frac_of_bf16_peak_effective"]}
    if others:
        extras["rooflines_of_the_other_kernels"] = others
    if extras:
        result["extras"] = extras

    if "cpu" in sections:
        # oracle on the host cores, on a bounded sample of query rows of the same workload; doubles as parity check
        import oracle

        fused("token")()
        torch.cuda.synchronize()
        rows = random_rows(w, args.cpu_rows, 123)
        oq, ok_, ov = (si.as_oracle_array(t) for t in (q, k, v))
        c0 = time.perf_counter()
        want = oracle.skiparse_attention_rows(oq, ok_, ov, rows, T, H, W, s, "token", w.scale)
        cpu_s = time.perf_counter() - c0
        row_flops = 4.0 * w.Nsub * w.D
        result["cpu_baseline"] = {
            "value": round(args.cpu_rows * row_flops / cpu_s / 1e12, 6),
            "unit": "TFLOP/s",
            "cores": oracle.num_threads(),
            "kind": "oracle",
            "sample": f"{args.cpu_rows} of {w.B * w.heads * w.N} query rows drawn uniformly, each against all {w.Nsub} keys of its subsequence; {cpu_s:.1f} s",
            "extrapolated_full_call_s": round(cpu_s * (w.B * w.heads * w.N) / args.cpu_rows, 1),
        }
        result["parity"] = sampled_parity(out, rows, want, 2e-2, 5e-3)
        if not result["parity"]["ok"]:
            failures.append("headline parity")
        if "group" in sections and "group" in w.patterns:
            fused("group")()
            torch.cuda.synchronize()
            rows_g = rows[:2048]
            want_g = oracle.skiparse_attention_rows(oq, ok_, ov, rows_g, T, H, W, s, "group", w.scale)
            result["parity_group"] = sampled_parity(out, rows_g, want_g, 2e-2, 5e-3)
            if not result["parity_group"]["ok"]:
                failures.append("group-wise parity")

    print(json.dumps(result))
    if failures:
        print("bench.py: parity check failed: " + ", ".join(failures), file=sys.stderr)
        return 1
    return 0


if __name__ == "__main__":
    sys.exit(main())
