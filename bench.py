#!/usr/bin/env python3
"""Throughput of the per-device Transformer training step on one MI355X.

A step is one pass of the whole hot path over one batch of seeded synthetic input, with every
input already resident in HBM: block forward + backward (cfg3, cfg4), the same over a 2-layer
stack plus AdamW (cfg2), or the full fax_train_step (cfg5).  Default workload: cfg3, the
d_model=4096 block the throughput target is quoted on.

Prints ONE JSON line: tokens/s (whole job = this one GPU), model TFLOP/s and its fraction of the
bf16 MFMA peak, the roofline of the kernel that takes the most time (measured with HIP events on
the launch stream inside the library, see fax_timing_enable), and the CPU oracle timed on a
bounded sample of the same workload on this machine's host cores.
"""
import argparse
import json
import os
import sys
import time

import numpy as np

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

MFMA_BF16_PEAK_TFLOPS = 2516.6   # 256 CU x 2.4 GHz x 4096 flop/clk/CU, dense bf16
HBM_PEAK_GBS = 8000.0


def parse():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=20)
    ap.add_argument("--warmup", type=int, default=5)
    ap.add_argument("--config", default="cfg3", choices=["cfg2", "cfg3", "cfg4", "cfg5", "t1_5120", "t1_10240", "t1_16384", "fig4_124m"])
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--kernels", action="store_true", help="also print the per-kernel table to stderr")
    ap.add_argument("--graph", action="store_true",
                    help="capture one step (the same C-ABI calls) in a HIP graph and time its replays")
    ap.add_argument("--single-stream", action="store_true",
                    help="FAX_FLAG_SINGLE_STREAM: keep the weight gradients on the caller's stream (for comparison)")
    ap.add_argument("--deterministic", action="store_true",
                    help="FAX_FLAG_DETERMINISTIC (train-step workloads): ordered reduction for the embedding gradient")
    ap.add_argument("--no-ceilings", action="store_true", help="skip the measured MFMA-only and copy-kernel ceilings")
    ap.add_argument("--calib-copy", action="store_true",
                    help="first run a plain elementwise copy kernel (reads 256 MiB, writes 128 MiB): a known-size reference "
                         "for the HBM byte counters")
    return ap.parse_args()


def main():
    args = parse()
    if args.gpus != 1:
        print("bench.py: this build runs on ONE GPU; --gpus %d is not supported (no collectives are built). "
              "Run with --gpus 1." % args.gpus, file=sys.stderr)
        sys.exit(2)

    import torch
    import paper_2204_06514_amd as fax
    from workloads import get_config, make_block_inputs, make_stack_inputs, make_model_inputs, PARAM_NAMES
    from workloads.configs import ADAMW_DEFAULT, ModelShape

    dev = "cuda:0"
    torch.cuda.set_device(0)
    cfg = get_config(args.config)
    is_model = isinstance(cfg, ModelShape)
    sh = cfg.blk if is_model else cfg
    tp_share = sh.H * sh.dh != sh.D  # one tensor-parallel rank's share: the un-reduced partial sums are outputs too
    td = torch.bfloat16
    code = fax.FAX_BF16

    def up(a, dtype=td):
        return torch.from_numpy(np.ascontiguousarray(a, dtype=np.float32)).to(dev).to(dtype).contiguous()

    dims = fax.block_dims(sh.B, sh.S, sh.D, sh.H, sh.dh, sh.F, code, fax.FAX_GELU_TANH, sh.ln_eps,
                          (fax.FAX_FLAG_TP_PARTIAL if tp_share else 0) | (fax.FAX_FLAG_SINGLE_STREAM if args.single_stream else 0))
    base_flags = dims.flags
    hp = fax.FaxAdamW(**ADAMW_DEFAULT)
    T = sh.T

    if is_model:
        p, tok, lab = make_model_inputs(cfg, seed=0)
        top = ("tok_emb", "pos_emb", "lnf_g", "lnf_b")
        params = {k: up(p[k]) for k in top}
        params["blocks"] = [{k: up(bp[k]) for k in PARAM_NAMES} for bp in p["blocks"]]

        def like(fn):
            d = {k: fn(params[k]) for k in top}
            d["blocks"] = [{k: fn(b[k]) for k in PARAM_NAMES} for b in params["blocks"]]
            return d
        master = like(lambda t: t.float().clone())
        m = like(lambda t: torch.zeros(t.shape, dtype=torch.float32, device=dev))
        v = like(lambda t: torch.zeros(t.shape, dtype=torch.float32, device=dev))
        grads = like(lambda t: torch.empty(t.shape, dtype=torch.float32, device=dev))
        md = fax.FaxModelDims(dims, sh.L, cfg.V, cfg.S_max, fax.FAX_FLAG_DETERMINISTIC if args.deterministic else 0)
        wsb = fax.fax_train_workspace_bytes(md)
        ws = torch.empty(wsb, dtype=torch.uint8, device=dev)
        tokd, labd = torch.from_numpy(tok).to(dev), torch.from_numpy(lab).to(dev)
        loss = torch.zeros(4, device=dev)
        tabs = [fax.model_tensors(t) for t in (params, master, m, v, grads)]
        state = {"t": 0}

        def step():
            state["t"] += 1
            fax.fax_train_step(md, tabs[0], tabs[1], tabs[2], tabs[3], tabs[4], tokd, labd, hp, state["t"], loss, ws, wsb)
        flops = cfg.flops_fwd_bwd(True)
        flops_full = cfg.flops_fwd_bwd(False)
        what = "fax_train_step: embedding + %d blocks + final LN + tied head + CE + backward + AdamW" % sh.L
        ana = fax.fax_analyze(md)   # the static analyser's prediction for this model on one device, for comparison
        analysis = {"predicted_ms": round(ana.ms_step, 2), "predicted_ms_gemm": round(ana.ms_gemm, 2),
                    "predicted_ms_attention": round(ana.ms_attention, 2), "predicted_ms_bandwidth": round(ana.ms_bandwidth, 2),
                    "device_bytes": int(ana.bytes_total)}
    else:
        ps, x, dy = make_stack_inputs(sh, seed=0)
        pd = [{k: up(p[k]) for k in PARAM_NAMES} for p in ps]
        xs = [up(x)] + [torch.empty((sh.B, sh.S, sh.D), dtype=td, device=dev) for _ in range(sh.L)]
        dyd = up(dy)
        dcur = torch.empty_like(dyd)
        lay = fax.fax_block_saved_layout(dims)
        saved = [torch.empty(lay.total, dtype=torch.uint8, device=dev) for _ in range(sh.L)]
        wsb = fax.fax_block_workspace_bytes(dims)
        ws = torch.empty(wsb, dtype=torch.uint8, device=dev)
        gd = [{k: torch.empty(t.shape, dtype=torch.float32, device=dev) for k, t in p.items()} for p in pd]
        pa = torch.empty_like(dyd) if tp_share else None
        pm = torch.empty_like(dyd) if tp_share else None
        with_adam = args.config == "cfg2"
        if with_adam:
            master = [{k: t.float().clone() for k, t in p.items()} for p in pd]
            mo = [{k: torch.zeros_like(t) for k, t in p.items()} for p in master]
            vo = [{k: torch.zeros_like(t) for k, t in p.items()} for p in master]
        pt = [fax.block_tensors(p) for p in pd]
        gt = [fax.block_tensors(g) for g in gd]
        if with_adam:
            mt, mot, vot = ([fax.block_tensors(t) for t in ts] for ts in (master, mo, vo))
        state = {"t": 0}

        def step():
            for l in range(sh.L):
                fax.fax_block_fwd(dims, pt[l], xs[l], xs[l + 1], saved[l], pa, pm, ws, wsb)
            for l in reversed(range(sh.L)):
                fax.fax_block_bwd(dims, pt[l], xs[l], dyd if l == sh.L - 1 else dcur, saved[l], dcur, gt[l], 0, None, None, ws, wsb)
            if with_adam:
                state["t"] += 1
                for l in range(sh.L):
                    fax.fax_adamw_block_step(dims, mt[l], mot[l], vot[l], gt[l], pt[l], hp, state["t"])
        flops = sh.L * sh.block_flops_fwd_bwd(True)
        flops_full = sh.L * sh.block_flops_fwd_bwd(False)
        what = "%d x (fax_block_fwd + fax_block_bwd)%s" % (sh.L, " + fax_adamw_block_step per block (AdamW on every tensor)" if with_adam else "")

    if args.calib_copy:
        # an elementwise fp32 -> bf16 copy: reads exactly 2^28 bytes, writes exactly 2^27
        src = torch.zeros(1 << 26, dtype=torch.float32, device=dev)
        dst = torch.empty(1 << 26, dtype=torch.bfloat16, device=dev)
        for _ in range(3):
            dst.copy_(src)
        torch.cuda.synchronize()
        del src, dst

    timed_step = step
    if args.graph:
        for _ in range(2):  # first calls set kernel attributes: keep them out of the capture
            step()
        torch.cuda.synchronize()
        graph = torch.cuda.CUDAGraph()
        with torch.cuda.graph(graph):
            step()
        timed_step = graph.replay
    for _ in range(args.warmup):
        timed_step()
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(args.steps):
        timed_step()
    torch.cuda.synchronize()
    dt = (time.perf_counter() - t0) / args.steps

    # Second timed region with per-kernel HIP events on the launch stream.  Here every kernel goes to
    # the one stream (FAX_FLAG_SINGLE_STREAM): where the backward pass would run its weight gradients
    # on a second stream beside the input-gradient chain, the events around a kernel would span its
    # neighbour's time as well.  Same kernels, same launch shapes; only the timed region above carries
    # the headline.
    dims.flags = base_flags | fax.FAX_FLAG_SINGLE_STREAM
    if is_model:
        md.blk.flags = dims.flags
    for _ in range(2):
        step()
    torch.cuda.synchronize()
    t1 = time.perf_counter()
    fax.fax_timing_enable(1)
    for _ in range(args.steps):
        step()
    torch.cuda.synchronize()
    dt_single = (time.perf_counter() - t1) / args.steps
    rows = fax.fax_timing_report(64)
    fax.fax_timing_enable(0)
    dims.flags = base_flags
    if is_model:
        md.blk.flags = base_flags
    # fax_train_step also times its phases as wholes (forward / loss / backward / update, Fig. 4)
    phases = {r["name"][6:] + "_ms": round(r["ms"] / args.steps, 4) for r in rows if r["name"].startswith("phase_")}
    rows = [r for r in rows if not r["name"].startswith("phase_")]
    rows.sort(key=lambda r: -r["ms"])
    dom = rows[0]
    if dom["unit"] == 0:
        ach = dom["work"] / (dom["ms"] * 1e-3) / 1e12
        roof = {"kernel": dom["name"], "bound": "mfma", "achieved": round(ach, 2), "peak": MFMA_BF16_PEAK_TFLOPS,
                "unit": "TFLOP/s", "frac": round(ach / MFMA_BF16_PEAK_TFLOPS, 4), "traffic": None,
                "launches_per_step": dom["launches"] // args.steps,
                "avg_launch_ms": round(dom["ms"] / dom["launches"], 4),
                "flop_per_launch_avg": dom["work"] / dom["launches"]}
    else:
        ach = dom["work"] / (dom["ms"] * 1e-3) / 1e9
        roof = {"kernel": dom["name"], "bound": "hbm", "achieved": round(ach, 1), "peak": HBM_PEAK_GBS, "unit": "GB/s",
                "frac": round(ach / HBM_PEAK_GBS, 4), "traffic": None,
                "launches_per_step": dom["launches"] // args.steps,
                "avg_launch_ms": round(dom["ms"] / dom["launches"], 4),
                "bytes_per_launch_avg": dom["work"] / dom["launches"]}
    roof["traffic"] = committed_traffic(args.config, dom["name"])
    kernels = []
    for r in rows:
        per_step_ms = r["ms"] / args.steps
        rate = r["work"] / (r["ms"] * 1e-3) if r["ms"] > 0 else 0.0
        kernels.append({"name": r["name"], "launches_per_step": r["launches"] // args.steps,
                        "ms_per_step": round(per_step_ms, 4),
                        ("tflops" if r["unit"] == 0 else "gbs"): round(rate / (1e12 if r["unit"] == 0 else 1e9), 2)})
    if args.kernels:
        for k in kernels:
            print(json.dumps(k), file=sys.stderr)

    # Measured ceilings of this very GPU, after the timed regions: the matrix cores fed from registers
    # only (operands zero / random: the chip holds different clocks for the two) and a plain copy.
    ceilings = None
    if not args.no_ceilings:
        ceilings = measure_ceilings(fax, torch, dev)
        if roof["bound"] == "mfma":
            roof["frac_of_measured_mfma_random"] = round(roof["achieved"] / ceilings["mfma_bf16_random_tflops"], 4)
        else:
            roof["frac_of_measured_copy"] = round(roof["achieved"] / ceilings["copy_gbs"], 4)
        for k in kernels:
            if "tflops" in k:
                k["of_measured_mfma"] = round(k["tflops"] / ceilings["mfma_bf16_random_tflops"], 3)
            else:
                k["of_measured_copy"] = round(k["gbs"] / ceilings["copy_gbs"], 3)

    cpu = None
    if not args.no_cpu_baseline:
        cpu = cpu_baseline(args.config, cfg)

    tflops = flops / dt / 1e12
    out = {
        "metric": "tokens_per_sec", "value": round(T / dt, 1), "unit": "tokens/s", "n_gpus": 1,
        "steps": args.steps, "warmup": args.warmup, "ms_per_step": round(dt * 1e3, 4), "higher_is_better": True,
        "scaling": "weak", "vs_baseline": None, "dtype": "bf16", "data": "synthetic",
        "config": {"workload": "%s: %s; B=%d S=%d D=%d H=%dx%d F=%d L=%d%s" % (
            args.config, what, sh.B, sh.S, sh.D, sh.H, sh.dh, sh.F, sh.L, (" V=%d" % cfg.V) if is_model else "")},
        "model_tflops": round(tflops, 2), "mfma_peak_frac": round(tflops / MFMA_BF16_PEAK_TFLOPS, 4),
        "model_tflops_unhalved_attention": round(flops_full / dt / 1e12, 2),
        "model_flop_per_step": flops,
        "mfma_frac_of_measured": (round(tflops / ceilings["mfma_bf16_random_tflops"], 4) if ceilings else None),
        "ms_per_step_single_stream_with_kernel_events": round(dt_single * 1e3, 4),
        "roofline": roof, "ceilings": ceilings, "cpu_baseline": cpu, "phases": phases or None,
        "analysis": analysis if is_model else None, "kernels": kernels,
    }
    print(json.dumps(out))


def measure_ceilings(fax, torch, dev):
    """MFMA-only and copy-only kernels of the library, timed with its HIP events: what this GPU
    sustains when nothing but the matrix cores (256 workgroups of 4 waves, as the GEMM runs) or
    nothing but HBM is in the way."""
    sink = torch.zeros(4, device=dev)
    n = 1 << 30
    src = torch.empty(n, dtype=torch.uint8, device=dev).fill_(3)
    dst = torch.empty(n, dtype=torch.uint8, device=dev)
    cus = torch.cuda.get_device_properties(0).multi_processor_count
    iters = 40000          # 256 x 4 x 40000 x 16 MFMAs = 21.5 TFLOP: about 10 ms
    for seed in (0, 1):    # untimed first launches
        fax.fax_probe_mfma(cus, iters // 10, seed, sink)
    fax.fax_probe_copy(src, dst, n)
    torch.cuda.synchronize()
    fax.fax_timing_enable(1)
    for _ in range(3):
        fax.fax_probe_mfma(cus, iters, 0, sink)
        fax.fax_probe_mfma(cus, iters, 1, sink)
        fax.fax_probe_copy(src, dst, n)
    torch.cuda.synchronize()
    rows = {r["name"]: r for r in fax.fax_timing_report(16)}
    fax.fax_timing_enable(0)
    rate = lambda r: r["work"] / (r["ms"] * 1e-3)
    return {"mfma_bf16_zero_tflops": round(rate(rows["probe_mfma_zero"]) / 1e12, 1),
            "mfma_bf16_random_tflops": round(rate(rows["probe_mfma_random"]) / 1e12, 1),
            "copy_gbs": round(rate(rows["probe_copy"]) / 1e9, 1),
            "how": "fax_probe_mfma: %d workgroups x 4 waves x %d x 16 back-to-back 32x32x16 bf16 MFMAs on register operands "
                   "(zero / pseudo-random), fax_probe_copy: 1 GiB read + 1 GiB written; HIP events, 3 launches each" % (cus, iters)}


def committed_traffic(config, kernel):
    """HBM bytes per launch of `kernel` from the committed rocprofv3 --pmc summary (FETCH_SIZE and
    WRITE_SIZE runs, scaled by the copy-kernel calibration stated there), or None if not recorded."""
    import re
    path = os.path.join(ROOT, "profiles", "hbm_traffic_%s.txt" % config)
    if not os.path.exists(path):
        return None
    for line in open(path):
        m = re.match(r"^%s\s+traffic_bytes_per_launch\s*=\s*([0-9.eE+]+)" % re.escape(kernel), line)
        if m:
            return float(m.group(1))
    return None


def cpu_baseline(name, cfg):
    """The oracle as it stands, timed on this machine's host cores on a bounded sample."""
    from oracle import transformer as orc
    from workloads import make_block_inputs, make_model_inputs
    from workloads.configs import ModelShape
    try:
        from threadpoolctl import threadpool_info
        cores = max([i.get("num_threads", 1) for i in threadpool_info()] or [1])
    except Exception:
        cores = os.cpu_count()
    if isinstance(cfg, ModelShape):
        small = cfg.scaled(B=1, S=512, L=2, V=8192, S_max=512)
        p, tok, lab = make_model_inputs(small, seed=0)
        t0 = time.perf_counter()
        orc.model_loss_and_grads(p, tok, lab, small.blk.H, small.blk.dh)
        dt = time.perf_counter() - t0
        toks = small.blk.T
        sample = ("oracle loss+gradients of the same model cut to B=1, S=512, L=2, V=8192 (float64), one run; the whole "
                  "configuration would take more than ten minutes")
    elif name == "cfg3":
        # the whole configuration: about half a minute of float64 matrix products on 16 cores
        p, x, dy = make_block_inputs(cfg, seed=0)
        t0 = time.perf_counter()
        _, c = orc.block_fwd(x, p, cfg.H, cfg.dh)
        orc.block_bwd(dy, c, p)
        dt = time.perf_counter() - t0
        toks = cfg.T
        sample = "the whole workload, no sampling: oracle block forward+backward at B=%d, S=%d (float64), one run" % (cfg.B, cfg.S)
    else:
        S = min(cfg.S, 2048 if cfg.D <= 4096 else 1024 if cfg.D <= 12288 else 512)
        small = cfg.scaled(B=1, S=S, L=1)
        p, x, dy = make_block_inputs(small, seed=0)
        t0 = time.perf_counter()
        _, c = orc.block_fwd(x, p, small.H, small.dh)
        orc.block_bwd(dy, c, p)
        dt = time.perf_counter() - t0
        toks = small.T
        sample = ("oracle block forward+backward on one batch row (B=1, S=%d) of the same block (float64), one run; the "
                  "whole configuration would take minutes" % S)
    return {"value": round(toks / dt, 2), "unit": "tokens/s", "cores": int(cores), "kind": "oracle", "sample": sample,
            "seconds": round(dt, 2)}


if __name__ == "__main__":
    main()
