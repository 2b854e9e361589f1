#!/usr/bin/env python3
"""Benchmark of the RPTQ hot path on one MI355X.

A step is one pass of the whole path over one batch of synthetic input for the chosen
workload: for every quantization site, LayerNorm-in-cluster-order + per-cluster
quantization (one kernel), then the cluster-wise integer GEMM of every linear layer that
reads the site.  Inputs are resident in HBM before the timed region.  Prints one JSON
line: tokens/s of the whole step, the roofline record of the dominant kernel (measured
with HIP events around runs of its launches on the launch stream), and the CPU oracle timed on
the host cores on the same workload.

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--config i] [--no-cpu]
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

PEAK_INT8_TOPS = 5000.0      # MI355X dense int8 MFMA, TOP/s
PEAK_HBM_GBS = 8000.0        # MI355X HBM3E, GB/s
PEAK_BF16_TFLOPS = 2500.0     # MI355X dense bf16 MFMA, TFLOP/s (the first method of App. A.4, a row beyond the step)
EPS = 1e-5


def parse_args():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=None, help="timed steps (default: about 3 s of them)")
    ap.add_argument("--warmup", type=int, default=None, help="untimed steps before them (default: a quarter of --steps)")
    ap.add_argument("--ramp-s", type=float, default=1.0,
                    help="seconds of untimed steps before the warmup (the GPU clocks need about a second of load to settle)")
    ap.add_argument("--config", type=int, default=3,
                    help="index into BASELINE.json configs (default 3: the OPT-175b prefill layer, the largest "
                         "single-GPU workload; 4 is the decode layer, 0-2 the smaller ones)")
    ap.add_argument("--sets", type=int, default=4, help="distinct input/weight copies cycled through the steps")
    ap.add_argument("--no-cpu", action="store_true", help="skip the CPU oracle baseline")
    ap.add_argument("--unfused", action="store_true",
                    help="chained workloads: store fc1's bf16 output and quantize it with a second kernel "
                         "(rptq_cluster_gemm + rptq_ln_quant) instead of quantizing for the next site in "
                         "fc1's output stage (rptq_cluster_gemm_quant)")
    ap.add_argument("--graph", action="store_true",
                    help="record the steps (one per input set) into a HIP graph and replay it: the same kernels "
                         "without per-launch host work (steps is rounded down to a multiple of --sets)")
    ap.add_argument("--copy-probe-mib", type=int, default=0,
                    help="also run one device-to-device copy of this many MiB before the steps: a kernel of known "
                         "traffic, which a rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE run of this command uses to scale its byte counters")
    return ap.parse_args()


def main():
    args = parse_args()
    if args.gpus != 1:
        print("bench.py: this build runs on one GPU only (no collectives, no sharding); use --gpus 1", file=sys.stderr)
        sys.exit(2)

    import numpy as np
    import torch

    import paper_2304_01089_amd as rp
    import workloads as w

    rp.load_library()                       # no fallback: the HIP library must be built
    if not torch.cuda.is_available():
        print("bench.py: no GPU visible", file=sys.stderr)
        sys.exit(2)
    torch.cuda.set_device(0)
    cfg = w.CONFIGS[args.config]
    M, bits = cfg.M, cfg.bits

    def dev_bf16(x):
        return torch.from_numpy(w.bf16_bits(x).view(np.int16)).cuda().view(torch.bfloat16)

    # ---- setup (untimed): synthetic inputs, calibration, folding -----------------------------
    t_setup = time.time()
    sites = []
    host_sites = []
    # pass 1: inputs and calibration of every site.  A site without LayerNorm is the ReLU site
    # of an FFN: its input is the output of the first linear layer of the site before it, and it
    # is calibrated on that layer's output in the unquantized model (torch fp32, set-up only).
    for si, spec in enumerate(cfg.sites):
        seed = w.site_seed(args.config, si)
        if spec.layernorm:
            site = w.make_site(seed, spec.d, M, cfg.n_cal)
            gamma, beta = torch.from_numpy(site.gamma).cuda(), torch.from_numpy(site.beta).cuda()
            cal = rp.calibrate_site([dev_bf16(b) for b in site.cal], gamma, beta, EPS, False, spec.g, bits, seed=seed)
            xs = [dev_bf16(site.x)]
            for k in range(1, args.sets):       # further batches from the same channel model
                xs.append(dev_bf16(w.extra_batch(site, k, M)))
            Ws = [w.weight_matrix(seed + 500 + li, N, spec.d) for li, (_, N) in enumerate(spec.gemms)]
            sites.append(dict(spec=spec, cal=cal, run_cal=cal, xs=xs, relu=False, perm_out=[None] * len(Ws)))
            host_sites.append(dict(site=site, W=Ws))
        else:
            prev, hprev = sites[-1], host_sites[-1]
            pg, pb = torch.from_numpy(hprev["site"].gamma).cuda(), torch.from_numpy(hprev["site"].beta).cuda()
            W1 = torch.from_numpy(hprev["W"][0]).cuda()
            hcal = []
            for bch in hprev["site"].cal:
                xb = dev_bf16(bch).float()
                hcal.append((torch.nn.functional.layer_norm(xb, (xb.shape[1],), pg, pb, EPS) @ W1.T).to(torch.bfloat16))
            del W1
            cal = rp.calibrate_site(hcal, None, None, EPS, True, spec.g, bits, seed=seed)
            del hcal
            prev["row_perm_host"] = cal.perm
            if args.unfused:
                prev["perm_out"][0] = cal.perm      # fc1's rows leave in this site's cluster order
            else:
                prev["next_site"] = cal                 # ... and padded like it: fc1's output stage quantizes
            Ws = [w.weight_matrix(seed + 500 + li, N, spec.d) for li, (_, N) in enumerate(spec.gemms)]
            sites.append(dict(spec=spec, cal=cal, run_cal=rp.identity_site(cal), xs=None, relu=True,
                              perm_out=[None] * len(Ws)))
            host_sites.append(dict(site=None, W=Ws))
    # pass 2: folding and buffers
    for s, hs in zip(sites, host_sites):
        spec, cal = s["spec"], s["cal"]
        lins = []
        for li, (lname, N) in enumerate(spec.gemms):
            nxt = s.get("next_site") if li == 0 else None
            lin0 = rp.fold_linear(cal, torch.from_numpy(hs["W"][li]).cuda(), perm_out=s["perm_out"][li], next_site=nxt)
            copies = [lin0]
            for k in range(1, args.sets):
                c = rp.FoldedLinear(N=lin0.N, Wq=lin0.Wq.clone(), sW=lin0.sW.clone(), zW=lin0.zW.clone(),
                                    wsum=lin0.wsum, colterm=lin0.colterm.clone())
                copies.append(c)
            if nxt is None:
                ys = [torch.empty((M, N), dtype=torch.bfloat16, device="cuda") for _ in range(min(2, args.sets))]
                ws = None
            else:
                ys = None
                ws = torch.empty(rp.rptq_cluster_gemm_quant_workspace_bytes(M, lin0.N), dtype=torch.uint8, device="cuda")
            lins.append(dict(name=lname, N=N, copies=copies, ys=ys, next_site=nxt, workspace=ws))
        s["lins"] = lins
        s["codes"] = torch.empty(rp.rptq_codes_bytes(M, cal.k_padded, bits), dtype=torch.uint8, device="cuda")
        s["rowterm"] = torch.empty(M, dtype=torch.float32, device="cuda")
    torch.cuda.synchronize()
    t_setup = time.time() - t_setup

    # the launches of one step, in order: (stage name, launch(i)) with i the step index
    launches = []
    prev_ys = None
    fed_by_gemm = False                      # this site's codes are written by the previous product's output stage
    for si, s in enumerate(sites):
        cal = s["run_cal"]

        def ln_launch(i, s=s, cal=cal, prev_ys=prev_ys):
            x = s["xs"][i % args.sets] if s["xs"] is not None else prev_ys[i % len(prev_ys)]
            rp.rptq_ln_quant(x, M, cal.d, cal.gamma_pad, cal.beta_pad, EPS, s["relu"], cal.perm_pad,
                             cal.cluster_off, cal.s, cal.inv_s, cal.z, bits, s["codes"], None, s["rowterm"])
        if not fed_by_gemm:
            launches.append(("ln_quant:%s" % s["spec"].name, ln_launch))
        fed_by_gemm = False
        for lin in s["lins"]:
            if lin["next_site"] is not None:
                def gemm_launch(i, s=s, cal=cal, lin=lin, nxt=sites[si + 1]):
                    c, nc = lin["copies"][i % args.sets], lin["next_site"]
                    rp.rptq_cluster_gemm_quant(s["codes"], M, bits, c.Wq, c.N, cal.cluster_off, cal.s, c.sW, c.zW,
                                               c.colterm, s["rowterm"], True, nc.cluster_off, nc.s, nc.inv_s, nc.z,
                                               nc.bits, nxt["codes"], nxt["rowterm"], lin["workspace"])
                launches.append(("gemm_quant:%s" % lin["name"], gemm_launch))
                fed_by_gemm = True
                continue

            def gemm_launch(i, s=s, cal=cal, lin=lin):
                c = lin["copies"][i % args.sets]
                rp.rptq_cluster_gemm(s["codes"], M, bits, c.Wq, c.N, cal.cluster_off, cal.s, c.sW, c.zW, c.colterm,
                                     s["rowterm"], lin["ys"][i % len(lin["ys"])])
            launches.append(("gemm:%s" % lin["name"], gemm_launch))
        prev_ys = s["lins"][0]["ys"]

    def step(i):
        for _, fn in launches:
            fn(i)

    if args.copy_probe_mib > 0:
        src = torch.ones(args.copy_probe_mib << 20, dtype=torch.uint8, device="cuda")
        dst = torch.empty_like(src)
        dst.copy_(src)
        torch.cuda.synchronize()
        del src, dst

    # ---- whole-step throughput ------------------------------------------------------------------
    t_ramp = time.time()
    while time.time() - t_ramp < args.ramp_s:   # untimed: brings the clocks to their loaded state
        for i in range(50):
            step(i)
        torch.cuda.synchronize()
    if args.steps is None:                      # about three seconds of timed steps
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record()
        for i in range(4):
            step(i)
        e1.record()
        torch.cuda.synchronize()
        args.steps = int(min(2000, max(20, 3000.0 / max(e0.elapsed_time(e1) / 4, 1e-3))))
    if args.warmup is None:
        args.warmup = max(5, args.steps // 4)
    for i in range(args.warmup):
        step(i)
    torch.cuda.synchronize()
    t0 = torch.cuda.Event(enable_timing=True)
    t1 = torch.cuda.Event(enable_timing=True)
    if args.graph:
        graph = torch.cuda.CUDAGraph()
        with torch.cuda.graph(graph):           # (the eager warm-up above has done the one-time driver set-up)
            for i in range(args.sets):
                step(i)
        replays = max(1, args.steps // args.sets)
        args.steps = replays * args.sets
        for _ in range(3):
            graph.replay()
        torch.cuda.synchronize()
        t0.record()
        for _ in range(replays):
            graph.replay()
        t1.record()
    else:
        t0.record()
        for i in range(args.steps):
            step(i)
        t1.record()
    torch.cuda.synchronize()
    ms_per_step = t0.elapsed_time(t1) / args.steps
    tokens_per_s = M / (ms_per_step * 1e-3)

    # ---- per-kernel durations: HIP events around runs of R launches of one stage (the same launch
    # arguments and rotating input sets as in the steps; about K launches per stage in all).  Events
    # around single launches would add the gaps between dispatches to kernels this short.
    R = 20
    blocks = max(3, args.steps // R)
    stage_ms = {}
    for name, fn in launches:
        for i in range(5):
            fn(i)
        torch.cuda.synchronize()
        evs = []
        for bi in range(blocks):
            e0 = torch.cuda.Event(enable_timing=True)
            e1 = torch.cuda.Event(enable_timing=True)
            for i in range(5):          # keeps the GPU busy while the host queues the run behind it:
                step(i)                 # the run is then paced by the kernel, not by launch overhead
            e0.record()
            for i in range(R):
                fn(bi * R + i)
            e1.record()
            evs.append((e0, e1))
        torch.cuda.synchronize()
        stage_ms[name] = [e0.elapsed_time(e1) / R for e0, e1 in evs]
    # (a block that met a host-side stall is far outside the others and is dropped)
    def robust_mean(v):
        v = np.asarray(v, dtype=np.float64)
        return float(v[v <= 3.0 * np.median(v)].mean())
    stage_avg = {k: robust_mean(v) for k, v in stage_ms.items()}

    # ---- roofline of the dominant kernel ---------------------------------------------------------
    stage_info = {}
    for s in sites:
        d = s["spec"].d
        name = "ln_quant:%s" % s["spec"].name
        alg_bytes = M * (2 * d + d * bits / 8.0)
        stage_info[name] = dict(bound="hbm", work=alg_bytes, unit="GB/s", peak=PEAK_HBM_GBS, scale=1e-9)
        for lin in s["lins"]:
            if lin["next_site"] is not None:        # same product; the next site's quantizer rides in its output stage
                ops = 2.0 * M * lin["N"] * d
                stage_info["gemm_quant:%s" % lin["name"]] = dict(bound="mfma", work=ops, unit="TOP/s", peak=PEAK_INT8_TOPS, scale=1e-12)
                continue
            if M <= 32:
                # decode: the packed weights are streamed once; judged against HBM (unpadded algorithmic bytes)
                by = lin["N"] * d / 2.0 + M * d * bits / 8.0 + M * lin["N"] * 2.0
                stage_info["gemm:%s" % lin["name"]] = dict(bound="hbm", work=by, unit="GB/s", peak=PEAK_HBM_GBS, scale=1e-9)
            else:
                ops = 2.0 * M * lin["N"] * d
                stage_info["gemm:%s" % lin["name"]] = dict(bound="mfma", work=ops, unit="TOP/s", peak=PEAK_INT8_TOPS, scale=1e-12)
    # the same peaks from what the box reports: compute units x clock x 8192 int8 ops per clock and
    # unit (the 32x32x32 int8 MFMA: 65536 ops in 16 passes of 4 clocks on each of 4 matrix cores);
    # memory clock x bus width x 4 transfers per reported clock (HBM3E: 8 Gb/s per pin at the 2000 MHz the
    # runtime reports; 8192 pins)
    di = rp.rptq_device_info()
    box = dict(compute_units=di["compute_units"], clock_mhz=round(di["clock_khz"] / 1e3, 1),
               int8_tops=round(di["compute_units"] * di["clock_khz"] * 1e3 * 8192 / 1e12, 1),
               memory_clock_mhz=round(di["memory_clock_khz"] / 1e3, 1), memory_bus_bits=di["memory_bus_bits"],
               hbm_gbs=round(di["memory_clock_khz"] * 1e3 * 4 * di["memory_bus_bits"] / 8 / 1e9, 1))
    dominant = max(stage_avg, key=lambda k: stage_avg[k])
    info = stage_info[dominant]
    achieved = info["work"] / (stage_avg[dominant] * 1e-3) * info["scale"]
    traffic = None
    tpath = os.path.join(ROOT, "profiles", "traffic.json")
    if os.path.exists(tpath):
        try:
            traffic = json.load(open(tpath)).get("config%d" % args.config, {}).get(dominant)
        except Exception:
            traffic = None
    roofline = dict(kernel=dominant, bound=info["bound"], achieved=round(achieved, 3), peak=info["peak"],
                    unit=info["unit"], frac=round(achieved / info["peak"], 4), traffic=traffic,
                    avg_launch_ms=round(stage_avg[dominant], 5), peak_from_box=box)
    stages = {}
    for k, ms in stage_avg.items():
        si = stage_info[k]
        ach = si["work"] / (ms * 1e-3) * si["scale"]
        stages[k] = dict(ms=round(ms, 5), ms_median=round(float(np.median(stage_ms[k])), 5),
                         ms_max=round(float(np.max(stage_ms[k])), 5), bound=si["bound"], achieved=round(ach, 3),
                         unit=si["unit"], frac=round(ach / si["peak"], 4))

    # ---- rows beyond the step: key/value-cache codes (Sec. 5.1 settings W4A4KV / W4A3KV / W3A3KV) ----------
    # The first site's input stands in for a key tensor of the layer's width (heads of 128 channels, 4
    # clusters per head as in Sec. 5.3's ablation outcome); not part of ms_per_step.
    next_rows = {}
    d0 = sites[0]["spec"].d
    if sites[0]["xs"] is not None and d0 % 128 == 0:
        H = d0 // 128
        xk = sites[0]["xs"][0]
        kmin = xk.float().amin(dim=0).cpu().numpy() + np.float32(0)
        kmax = xk.float().amax(dim=0).cpu().numpy() + np.float32(0)
        hc = rp.rptq_cluster_heads([kmin], [kmax], H, 4, bits, seed=1)
        table = torch.empty(rp.rptq_kv_table_bytes(d0), dtype=torch.uint8, device="cuda")
        rp.rptq_kv_tables(hc["perm"], hc["cluster_off"], hc["s"][0], hc["inv_s"][0], hc["z"][0], d0, H, 4, table)
        kcodes = torch.empty(M * d0 * bits // 8, dtype=torch.uint8, device="cuda")
        kback = torch.empty((M, d0), dtype=torch.bfloat16, device="cuda")
        kv_bytes = M * (2.0 * d0 + d0 * bits / 8.0)
        for kname, kfn in (("kv_quant", lambda i: rp.rptq_kv_quant(sites[0]["xs"][i % args.sets], M, d0, table, bits, kcodes)),
                           ("kv_dequant", lambda i: rp.rptq_kv_dequant(kcodes, M, d0, table, bits, kback))):
            for i in range(5):
                kfn(i)
            torch.cuda.synchronize()
            ts = []
            for bi in range(5):
                e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
                e0.record()
                for i in range(R):
                    kfn(bi * R + i)
                e1.record()
                torch.cuda.synchronize()
                ts.append(e0.elapsed_time(e1) / R)
            ms = robust_mean(ts)
            gbs = kv_bytes / (ms * 1e-3) * 1e-9
            next_rows[kname] = dict(ms=round(ms, 5), bound="hbm", achieved=round(gbs, 1), unit="GB/s",
                                    frac=round(gbs / PEAK_HBM_GBS, 4), tokens=M, d=d0, heads=H, bits=bits)

    # ... the reorder fused into LayerNorm the way Sec. 4.2 words it (original channel order, the reorder index
    # offsets the write address: one int8 per code, then a packing kernel), beside the LDS-gather kernel of the step
    if sites[0]["xs"] is not None:
        s0, cal0 = sites[0], sites[0]["cal"]
        g0, b0 = torch.from_numpy(host_sites[0]["site"].gamma).cuda(), torch.from_numpy(host_sites[0]["site"].beta).cuda()
        ws0 = torch.empty(rp.rptq_ln_quant_scatter_workspace_bytes(M, d0, cal0.k_padded) + 256, dtype=torch.uint8, device="cuda")
        ws0 = ws0[(-ws0.data_ptr()) % 256:]
        codes_sc = torch.empty_like(s0["codes"])

        def sc_fn(i):
            rp.rptq_ln_quant_scatter(s0["xs"][i % args.sets], M, d0, g0, b0, EPS, False, cal0.perm_pad, cal0.cluster_off,
                                     cal0.inv_s, cal0.z, bits, codes_sc, ws0)
        for i in range(3):
            sc_fn(i)
        torch.cuda.synchronize()
        ts = []
        for bi in range(5):
            e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            e0.record()
            for i in range(R):
                sc_fn(i)
            e1.record()
            torch.cuda.synchronize()
            ts.append(e0.elapsed_time(e1) / R)
        ms = robust_mean(ts)
        gbs = M * (2.0 * d0 + d0 * bits / 8.0) / (ms * 1e-3) * 1e-9
        next_rows["ln_quant_scatter:%s" % s0["spec"].name] = dict(
            ms=round(ms, 5), bound="hbm", achieved=round(gbs, 1), unit="GB/s", frac=round(gbs / PEAK_HBM_GBS, 4),
            gather_kernel_ms=round(stage_avg["ln_quant:%s" % s0["spec"].name], 5))
        del ws0, codes_sc

    # ... and the product with one weight parameter pair per (output channel, input cluster), App. A.4 as
    # printed, on the last site's first linear layer (at most 32 clusters): per-cluster row sums + product
    s_last, hs_last = sites[-1], host_sites[-1]
    if s_last["cal"].g_eff <= 32 and s_last["lins"][0]["ys"] is not None:
        cal_l, lin_l = s_last["run_cal"], s_last["lins"][0]
        Wl = torch.from_numpy(hs_last["W"][0]).cuda()
        lcw = rp.fold_linear_cw(s_last["cal"], Wl)
        del Wl
        rsums = torch.empty(rp.rptq_cw_rowsum_bytes(M, cal_l.g_eff) // 4, dtype=torch.float32, device="cuda")
        ycw = lin_l["ys"][0]
        d_l, N_l = s_last["spec"].d, lin_l["N"]

        def cw_sums(i):
            rp.rptq_cluster_rowsums(s_last["codes"], M, bits, cal_l.cluster_off, cal_l.s, cal_l.z, rsums)

        def cw_gemm(i):
            rp.rptq_cluster_gemm_cw(s_last["codes"], M, bits, lcw.Wq, lcw.N, cal_l.cluster_off, lcw.scale_tab,
                                    lcw.cross_tab, lcw.colterm, rsums, ycw)
        cw_sums(0)
        for kname, kfn, work, peak, unit, scale, bound in (
                ("cluster_rowsums:%s" % lin_l["name"], cw_sums, M * d_l * bits / 8.0, PEAK_HBM_GBS, "GB/s", 1e-9, "hbm"),
                ("gemm_cw:%s" % lin_l["name"], cw_gemm, 2.0 * M * N_l * d_l,
                 PEAK_HBM_GBS if M <= 32 else PEAK_INT8_TOPS, "GB/s" if M <= 32 else "TOP/s", 1e-9 if M <= 32 else 1e-12,
                 "hbm" if M <= 32 else "mfma")):
            if kname.startswith("gemm_cw") and M <= 32:
                work = N_l * d_l / 2.0 + M * d_l * bits / 8.0 + M * N_l * 2.0
            for i in range(3):
                kfn(i)
            torch.cuda.synchronize()
            ts = []
            for bi in range(5):
                e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
                e0.record()
                for i in range(R):
                    kfn(i)
                e1.record()
                torch.cuda.synchronize()
                ts.append(e0.elapsed_time(e1) / R)
            ms = robust_mean(ts)
            ach = work / (ms * 1e-3) * scale
            next_rows[kname] = dict(ms=round(ms, 5), bound=bound, achieved=round(ach, 1), unit=unit, frac=round(ach / peak, 4))
        del lcw

    # ... and the first method of App. A.4 on the same layer: de-quantize the codes to bf16 (per call), bf16 matrix
    # cores with fp32 accumulation (weights de-quantized once, offline); judged against the bf16 peak
    if s_last["lins"][0]["ys"] is not None:
        cal_l, lin_l = s_last["run_cal"], s_last["lins"][0]
        d_l, N_l, kp_l = s_last["spec"].d, lin_l["N"], cal_l.k_padded
        if N_l % 4 == 0 and (N_l + M) * kp_l * 2 < 8e9:
            fl = lin_l["copies"][0]
            w_hat = torch.empty((N_l, kp_l), dtype=torch.bfloat16, device="cuda")
            x_hat = torch.empty((M, kp_l), dtype=torch.bfloat16, device="cuda")
            rp.rptq_dequant_weights(fl.Wq, N_l, cal_l.cluster_off, fl.sW, fl.zW, w_hat)
            y1 = lin_l["ys"][0]

            def m1_dequant(i):
                rp.rptq_dequant_codes(s_last["codes"], M, bits, cal_l.cluster_off, cal_l.s, cal_l.z, x_hat)

            def m1_gemm(i):
                rp.rptq_gemm_bf16(x_hat, w_hat, M, N_l, kp_l, y1)
            m1_dequant(0)
            for kname, kfn, work, peak, unit, scale, bound in (
                    ("method1_dequant_codes:%s" % lin_l["name"], m1_dequant, M * (d_l * bits / 8.0 + 2.0 * d_l), PEAK_HBM_GBS,
                     "GB/s", 1e-9, "hbm"),
                    ("method1_gemm_bf16:%s" % lin_l["name"], m1_gemm, 2.0 * M * N_l * d_l, PEAK_BF16_TFLOPS, "TFLOP/s", 1e-12,
                     "mfma")):
                for i in range(3):
                    kfn(i)
                torch.cuda.synchronize()
                ts = []
                for bi in range(5):
                    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
                    e0.record()
                    for i in range(R if M > 32 else 5):
                        kfn(i)
                    e1.record()
                    torch.cuda.synchronize()
                    ts.append(e0.elapsed_time(e1) / (R if M > 32 else 5))
                ms = robust_mean(ts)
                ach = work / (ms * 1e-3) * scale
                next_rows[kname] = dict(ms=round(ms, 5), bound=bound, achieved=round(ach, 1), unit=unit, frac=round(ach / peak, 4))
            del w_hat, x_hat

    # ---- CPU oracle on the host cores (reported baseline) -----------------------------------------
    cpu = None
    if not args.no_cpu:
        from oracle import rptq_oracle as o
        cores = len(os.sched_getaffinity(0))
        if os.environ.get("OMP_NUM_THREADS", "").isdigit():      # numpy's BLAS threads: what the oracle really uses
            cores = min(cores, int(os.environ["OMP_NUM_THREADS"]))
        rows = M
        budget_flops = 1.2e12                     # keeps the leg to roughly 10-30 s of CPU work
        flops_per_row = sum(2.0 * N * s["spec"].d for s in sites for (_, N) in s["spec"].gemms)
        rows = int(max(16, min(M, budget_flops // flops_per_row)))
        # the oracle keeps the per-cluster integers [g, rows, N] (int64): bound that array to about 8 GB
        rows = int(max(16, min(rows, 8e9 // (8 * max(s["spec"].g * N for s in sites for (_, N) in s["spec"].gemms)))))
        # offline work, untimed: Eq. 1-2 per output row.  Rows are independent, so the oracle's function is
        # called on row blocks (bounded memory) from a thread pool.
        from concurrent.futures import ThreadPoolExecutor

        def quantize_rows(Wh, perm_in, perm_out):
            order = np.arange(Wh.shape[0]) if perm_out is None else np.asarray(perm_out)
            blocks = [order[r0:r0 + 2048] for r0 in range(0, len(order), 2048)]
            with ThreadPoolExecutor(max_workers=cores) as pool:
                parts = list(pool.map(lambda rws: o.quantize_weights(Wh[rws], perm_in), blocks))
            return tuple(np.concatenate([p[k] for p in parts]) for k in range(4))
        wqs = [[quantize_rows(Wh, s["cal"].perm, s.get("row_perm_host") if li == 0 else None)
                for li, Wh in enumerate(hs["W"])] for s, hs in zip(sites, host_sites)]
        tc = time.perf_counter()
        hidden = None
        for s, hs, wl in zip(sites, host_sites, wqs):
            cal = s["cal"]
            if s["relu"]:        # input already in this site's cluster order (fc1's rows were permuted offline)
                codes, xsum, _ = o.ln_quant(hidden, None, None, EPS, True, None, cal.cluster_off, cal.inv_s, cal.z, bits)
            else:
                codes, xsum, _ = o.ln_quant(hs["site"].x[:rows], hs["site"].gamma, hs["site"].beta, EPS, False,
                                            cal.perm, cal.cluster_off, cal.inv_s, cal.z, bits)
            for li, (wq, sW, _, zW) in enumerate(wl):
                _, _, Y = o.cluster_gemm_int(codes, wq, cal.cluster_off, cal.s, cal.z, sW, zW)
                if li == 0:
                    hidden = w.round_to_bf16(Y.astype(np.float32))
        online = max(time.perf_counter() - tc, 1e-9)
        cpu = dict(value=round(rows / online, 2), unit="tokens/s", cores=cores, kind="oracle",
                   sample="%d of %d tokens, all sites and GEMMs of the workload, numpy float64/int64 oracle "
                          "(offline weight quantization excluded)" % (rows, M), seconds=round(online, 3))

    out = {
        "metric": "tokens/s for LN+quant+cluster-GEMM per layer; % HBM GB/s or int8 MFMA peak",
        "value": round(tokens_per_s, 1),
        "unit": "tokens/s",
        "n_gpus": 1,
        "steps": args.steps,
        "warmup": args.warmup,
        "ms_per_step": round(ms_per_step, 5),
        "higher_is_better": True,
        "scaling": "weak",
        "vs_baseline": None,
        "dtype": "int8",
        "data": "synthetic",
        "config": {"workload": "configs[%d]: %s, M=%d, A%d, sites=%s" % (
            args.config, cfg.name, M, bits,
            ";".join("%s(d=%d,g=%d)->%s" % (s.name, s.d, s.g, ",".join("%s %dx%d" % (n, N, s.d) for n, N in s.gemms))
                     for s in cfg.sites)),
            "input_sets": args.sets, "y_dtype": "bf16", "setup_s": round(t_setup, 2), "hip_graph": bool(args.graph),
            "next_site_quantized_in_output_stage": any(l["next_site"] is not None for s in sites for l in s["lins"])},
        "roofline": roofline,
        "stages": stages,
        "cpu_baseline": cpu,
        "next_rows": next_rows,
    }
    print(json.dumps(out))


if __name__ == "__main__":
    main()
