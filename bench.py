#!/usr/bin/env python3
"""Benchmark of the QSpec W4 linear-layer hot path on one MI355X.

Workload (configuration 2 of the build's table): the four linear layers of a
Llama-7B-shaped decoder block (qkv 4096->12288, o 4096->4096, gate_up
4096->22016, down 11008->4096), int4 weights with fp16 group scales (g=128),
batch 8, draft length gamma=3.  One *step* is one draft pass (activation
quantiser + W4A4 GEMM at M=8 for every linear) plus one verify pass (W4A16
GEMM at M=32 for every linear) over `--layers` decoder blocks with distinct
weight blobs (default 32 = the whole model, 3.3 GB of packed weights, so
every weight byte comes from HBM and not from the 256 MB last-level cache).
Weight packing runs once before the timed region (it is off the token path)
and is reported separately.

Prints ONE JSON line:  value = algorithmic bytes of a step / time, in TB/s.
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

HBM_PEAK_GBS = 8000.0          # MI355X published HBM3E bandwidth
MFMA_PEAK_TFLOPS = {"w4a16": 2500.0, "w4a4": 5000.0}   # published dense fp16 / int8 matrix peaks


def alg_bytes_w4a16(M, N, K):
    G = K // 128
    return N * K // 2 + 2 * N * G + 2 * M * K + 2 * M * N


def alg_bytes_w4a4(M, N, K):
    G = K // 128
    return N * K // 2 + 2 * N * G + M * K // 2 + 4 * M * G + 2 * M * N


def alg_bytes_quant(M, K):
    return 2 * M * K + M * K // 2 + 4 * M * (K // 128)


def main() -> int:
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=50)
    ap.add_argument("--warmup", type=int, default=5)
    ap.add_argument("--layers", type=int, default=0,
                    help="decoder blocks with distinct weights per step (default: 32 for configs 1-3, 8 for 4, 4 for 5; "
                         "always far more packed weights than the 256 MB last-level cache holds)")
    ap.add_argument("--config", type=int, default=2, help="workload configuration (2 = headline)")
    ap.add_argument("--no-graph", action="store_true", help="launch eagerly instead of replaying HIP graphs")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--vendor-context", action="store_true",
                    help="also time torch.matmul (the vendor library's plain fp16 GEMM, fp16 weights, no quantisation) "
                         "on this configuration's verify-mode shapes: a yardstick for what the machine sustains, not a target")
    ap.add_argument("--prefill", action="store_true",
                    help="also time both modes at 1024 and 2048 tokens (prefill-sized M) in extra_rows_M256_M512")
    ap.add_argument("--no-extra", action="store_true",
                    help="skip the rows at 256 and 512 tokens, the verify-mode pass at the draft M and the fused producers (profiling runs: their "
                         "launches would mix into the kernel statistics)")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build runs on ONE GPU only (no collectives, no sharding); "
              "run with --gpus 1", file=sys.stderr)
        return 2

    import numpy as np
    import torch

    from paper_2410_11305_amd import binding as B
    from paper_2410_11305_amd import synth

    if not torch.cuda.is_available():
        print("bench.py: no GPU visible", file=sys.stderr)
        return 3
    B.lib()
    torch.cuda.set_device(0)
    dev = torch.device("cuda:0")
    cfg = synth.CONFIGS[args.config]
    Md, Mv = cfg.draft_M, cfg.verify_M
    lins = list(cfg.layers)
    L = args.layers or {4: 8, 5: 4}.get(args.config, 32)
    to = lambda a: torch.from_numpy(np.ascontiguousarray(a)).to(dev)

    # ---- inputs: block 0 from the seeded NumPy recipe, further blocks drawn on
    # the GPU with a seeded torch generator (same distributions), all packed by
    # the library itself.
    gen = torch.Generator(device=dev)
    gen.manual_seed(10000 * args.config + 99)
    blobs = [[None] * len(lins) for _ in range(L)]
    t_pack = 0.0
    pack_bytes = 0
    for i, lin in enumerate(lins):
        N, K = lin.N, lin.K
        for l in range(L):
            if l == 0:
                codes = to(synth.weight_codes(args.config, i, N, K))
                scales = to(synth.weight_scales(args.config, i, N, K))
            else:
                codes = torch.randint(-8, 8, (N, K), dtype=torch.int8, device=dev, generator=gen)
                scales = (torch.rand((N, K // 128), device=dev, generator=gen) * 0.008 + 0.002).half()
            out = torch.empty(B.packed_weight_bytes(N, K), dtype=torch.uint8, device=dev)
            e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            e0.record()
            B.pack_weights(codes, scales, out)
            e1.record()
            e1.synchronize()
            if l > 0:
                t_pack += e0.elapsed_time(e1) * 1e-3
                pack_bytes += N * K + 2 * N * (K // 128) + out.numel()
            blobs[l][i] = out
            del codes, scales
    xd = [to(synth.activations(args.config, i, Md, lin.K, verify=False)) for i, lin in enumerate(lins)]
    xv = [to(synth.activations(args.config, i, Mv, lin.K, verify=True)) for i, lin in enumerate(lins)]
    qa = [torch.empty((Md, lin.K // 2), dtype=torch.uint8, device=dev) for lin in lins]
    sa = [torch.empty((Md, lin.K // 128), dtype=torch.float32, device=dev) for lin in lins]
    yd = [torch.empty((Md, lin.N), dtype=torch.float16, device=dev) for lin in lins]
    yv = [torch.empty((Mv, lin.N), dtype=torch.float16, device=dev) for lin in lins]
    ws_bytes = max([B.workspace_bytes(Md, l.N, l.K) for l in lins] + [B.workspace_bytes(Mv, l.N, l.K) for l in lins] + [16])
    ws = B.alloc_workspace(ws_bytes)

    # one plain device copy of known size (256 MiB read + 256 MiB written): the
    # reference point that scales the FETCH_SIZE / WRITE_SIZE counters in profiles
    cal_src = torch.empty(256 << 20, dtype=torch.uint8, device=dev)
    cal_dst = torch.empty_like(cal_src)
    cal_dst.copy_(cal_src)
    torch.cuda.synchronize()
    del cal_src, cal_dst

    # ---- the passes
    def run_quant():
        for _ in range(L):
            for i in range(len(lins)):
                B.quant_act(xd[i], qa[i], sa[i])

    def run_w4a4():
        for l in range(L):
            for i, lin in enumerate(lins):
                B.gemm_w4a4(blobs[l][i], qa[i], sa[i], lin.N, y=yd[i], workspace=ws)

    def run_draft():
        for l in range(L):
            for i, lin in enumerate(lins):
                B.quant_act(xd[i], qa[i], sa[i])
                B.gemm_w4a4(blobs[l][i], qa[i], sa[i], lin.N, y=yd[i], workspace=ws)

    def run_verify():
        for l in range(L):
            for i, lin in enumerate(lins):
                B.gemm_w4a16(blobs[l][i], xv[i], lin.N, y=yv[i], workspace=ws)

    def run_w4a16_at_draft_M():
        for l in range(L):
            for i, lin in enumerate(lins):
                B.gemm_w4a16(blobs[l][i], xd[i], lin.N, y=yd[i], workspace=ws)

    def run_step():
        run_draft()
        run_verify()

    def one_kind(fn_name, i):
        lin = lins[i]

        def f():
            for l in range(L):
                if fn_name == "w4a4":
                    B.gemm_w4a4(blobs[l][i], qa[i], sa[i], lin.N, y=yd[i], workspace=ws)
                else:
                    B.gemm_w4a16(blobs[l][i], xv[i], lin.N, y=yv[i], workspace=ws)
        return f

    use_graph = not args.no_graph

    def make_runner(fn):
        """Returns a callable that enqueues fn's launches on the current stream
        (replaying a captured HIP graph unless --no-graph)."""
        fn()                       # eager once: first-call effects stay out of the capture
        torch.cuda.synchronize()
        if not use_graph:
            return fn
        g = torch.cuda.CUDAGraph()
        with torch.cuda.graph(g):
            fn()
        torch.cuda.synchronize()
        return g.replay

    def time_runner(run, reps, warm):
        for _ in range(warm):
            run()
        torch.cuda.synchronize()
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record()
        for _ in range(reps):
            run()
        e1.record()
        torch.cuda.synchronize()
        return e0.elapsed_time(e1) * 1e-3 / reps       # seconds per run

    # ---- headline: K steps, wall clock bracketed by synchronize
    step = make_runner(run_step)
    for _ in range(args.warmup):
        step()
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(args.steps):
        step()
    torch.cuda.synchronize()
    t_step = (time.perf_counter() - t0) / args.steps

    bytes_draft = sum(alg_bytes_quant(Md, l.K) + alg_bytes_w4a4(Md, l.N, l.K) for l in lins) * L
    bytes_verify = sum(alg_bytes_w4a16(Mv, l.N, l.K) for l in lins) * L
    bytes_step = bytes_draft + bytes_verify
    value = bytes_step / t_step / 1e12

    # ---- per-call and per-kernel durations: HIP events on the launch stream around a
    # replayed graph that holds only that call's L launches (distinct weight blobs)
    reps = max(3, min(20, args.steps // 5))
    t_q = time_runner(make_runner(run_quant), reps, 2)
    t_4 = time_runner(make_runner(run_w4a4), reps, 2)
    # (profiling runs skip this pass: its launches are further instances of the verify-mode kernels
    # and would mix into their statistics)
    t_16d = None if args.no_extra else time_runner(make_runner(run_w4a16_at_draft_M), reps, 2)
    calls = {}
    kernels = {"quant_act_kernel": dict(launches=L * len(lins), seconds=t_q, flops=0, mode="quant",
                                        bytes=sum(alg_bytes_quant(Md, l.K) for l in lins) * L)}
    for i, lin in enumerate(lins):
        for kind, M, ab in (("w4a4", Md, alg_bytes_w4a4), ("w4a16", Mv, alg_bytes_w4a16)):
            t = time_runner(make_runner(one_kind(kind, i)), reps, 2)          # L launches
            calls[f"{lin.name}.{kind}.M{M}"] = dict(us=round(t / L * 1e6, 3),
                                                    TBps=round(ab(M, lin.N, lin.K) * L / t / 1e12, 3))
            name = B.describe_kernel(kind == "w4a4", M, lin.N, lin.K)          # the profiler's symbol
            k = kernels.setdefault(name, dict(launches=0, seconds=0.0, bytes=0, flops=0, mode=kind))
            k["launches"] += L
            k["seconds"] += t
            k["bytes"] += ab(M, lin.N, lin.K) * L
            k["flops"] += 2 * M * lin.N * lin.K * L
    # The roofline object is for the dominant KERNEL, i.e. one __global__ template in
    # one mode; its instances (tiles per workgroup and the like, chosen per layer
    # shape) are separate symbols to the profiler and are added up here.  The
    # profile summaries carry the same family rows.
    def family(sym):
        if sym.startswith("gemm_stream_kernel<"):
            return "gemm_stream_kernel<" + ",".join(sym.split("<")[1].split(",")[:2]) + ", *>"
        return sym.split("<")[0] + ("<*>" if "<" in sym else "")
    families = {}
    for sym, v in kernels.items():
        f = families.setdefault(family(sym), dict(launches=0, seconds=0.0, bytes=0, flops=0, mode=v["mode"], symbols=[]))
        for key in ("launches", "seconds", "bytes", "flops"):
            f[key] += v[key]
        f["symbols"].append(sym)
    dom = max(families, key=lambda k: families[k]["seconds"])
    kd = families[dom]
    # which roof bounds that kernel: the one its algorithmic work takes longer to reach
    t_hbm = kd["bytes"] / (HBM_PEAK_GBS * 1e9)
    t_mfma = kd["flops"] / (MFMA_PEAK_TFLOPS.get(kd["mode"], 1.0) * 1e12) if kd["flops"] else 0.0
    # HBM traffic per launch of that kernel from the committed counter summary (if it covers it)
    traffic = None
    try:
        with open(os.path.join(ROOT, "profiles", "hbm_traffic.json")) as f:
            per = json.load(f).get("bytes_per_launch", {})
        if all(sym in per for sym in kd["symbols"]):       # launch-weighted mean over the family's symbols
            traffic = int(sum(per[sym] * kernels[sym]["launches"] for sym in kd["symbols"]) / kd["launches"])
    except (OSError, ValueError):
        pass
    if t_mfma > t_hbm:
        peak = MFMA_PEAK_TFLOPS[kd["mode"]]
        achieved = kd["flops"] / kd["seconds"] / 1e12
        roofline = dict(bound="mfma", kernel=dom, symbols=kd["symbols"], achieved=round(achieved, 1), peak=peak,
                        unit="TFLOP/s" if kd["mode"] == "w4a16" else "TOP/s")
    else:
        peak = HBM_PEAK_GBS
        achieved = kd["bytes"] / kd["seconds"] / 1e9
        roofline = dict(bound="hbm", kernel=dom, symbols=kd["symbols"], achieved=round(achieved, 1), peak=peak, unit="GB/s")
    roofline.update(frac=round(achieved / peak, 4), traffic=traffic,
                    avg_launch_us=round(kd["seconds"] / kd["launches"] * 1e6, 3),
                    alg_bytes_per_launch=kd["bytes"] // kd["launches"],
                    alg_flops_per_launch=kd["flops"] // kd["launches"])

    # ---- extra rows: both modes at 256 and 512 tokens on this configuration's layers (no
    # configuration drafts more than 128 tokens; these rows show the draft-mode kernel in
    # the matrix-bound regime next to the verify-mode kernel at the same shape)
    extra = {}
    for Mx in (() if args.no_extra else ((256, 512, 1024, 2048) if args.prefill else (256, 512))):
        xx = [torch.randn((Mx, lin.K), device=dev, generator=gen).half() for lin in lins]
        qx = [B.quant_act(t) for t in xx]
        yx = [torch.empty((Mx, lin.N), dtype=torch.float16, device=dev) for lin in lins]
        wsx = B.alloc_workspace(max([B.workspace_bytes(Mx, l.N, l.K) for l in lins] + [16]))
        Lx = min(L, 4)
        for i, lin in enumerate(lins):
            for kind in ("w4a4", "w4a16"):
                def f(i=i, lin=lin, kind=kind):
                    for l in range(Lx):
                        if kind == "w4a4":
                            B.gemm_w4a4(blobs[l][i], qx[i][0], qx[i][1], lin.N, y=yx[i], workspace=wsx)
                        else:
                            B.gemm_w4a16(blobs[l][i], xx[i], lin.N, y=yx[i], workspace=wsx)
                t = time_runner(make_runner(f), 3, 1) / Lx
                extra[f"{lin.name}.{kind}.M{Mx}"] = dict(
                    us=round(t * 1e6, 2),
                    mfma_frac=round(2 * Mx * lin.N * lin.K / t / 1e12 / MFMA_PEAK_TFLOPS[kind], 4))
        del xx, qx, yx, wsx

    # ---- optional yardstick: the vendor library's plain fp16 GEMM on the verify-mode shapes
    vendor = None
    if args.vendor_context:
        vendor = {}
        for i, lin in enumerate(lins):
            Rv = max(2, int(1.2e9 // (lin.N * lin.K * 2)) + 1)           # rotate over more fp16 weight bytes than the last-level cache holds
            Wv = [(torch.randn((lin.N, lin.K), device=dev, generator=gen) * 0.03).half() for _ in range(Rv)]
            yvv = torch.empty((Mv, lin.N), dtype=torch.float16, device=dev)
            t = time_runner(make_runner(lambda: [torch.matmul(xv[i], W.t(), out=yvv) for W in Wv]), 3, 1) / Rv
            vendor[f"{lin.name}.fp16.M{Mv}"] = dict(us=round(t * 1e6, 2), TFLOPs=round(2 * Mv * lin.N * lin.K / t / 1e12, 1),
                                                     weight_TBps=round(lin.N * lin.K * 2 / t / 1e12, 2))
            del Wv, yvv

    # ---- the steps after the verify pass (greedy acceptance, KV-cache overwrite): not part
    # of the step above, timed on their own at this configuration's batch and draft length
    lg_h, dr_h, _ = synth.accept_inputs(args.config)
    Bn, rows, V = lg_h.shape
    kvD, kvS = lins[0].K, 2048                       # one K (or V) row of a decoder block; cache length 2048
    lg, dr = to(lg_h), to(dr_h)
    n_acc = torch.empty((Bn,), dtype=torch.int32, device=dev)
    out_tok = torch.empty((Bn, rows), dtype=torch.int32, device=dev)
    ws_acc = torch.empty(max(B.accept_workspace_bytes(Bn, rows - 1, V), 16), dtype=torch.uint8, device=dev)
    kv_new = torch.randn((Bn, rows, kvD), device=dev, generator=gen).half()
    kv_cache = torch.zeros((Bn, kvS, kvD), dtype=torch.float16, device=dev)
    kv_pos = torch.randint(0, kvS - rows, (Bn,), device=dev, generator=gen).to(torch.int32)
    n_rep_small = 16
    t_acc = time_runner(make_runner(lambda: [B.greedy_accept(lg, dr, n_acc, out_tok, ws_acc) for _ in range(n_rep_small)]),
                        reps, 2) / n_rep_small
    t_kv = time_runner(make_runner(lambda: [B.kv_overwrite(kv_cache, kv_new, n_acc, kv_pos) for _ in range(n_rep_small)]),
                       reps, 2) / n_rep_small
    acc_bytes = Bn * rows * V * 2 + Bn * (rows - 1) * 4 + Bn * (rows + 1) * 4
    kv_bytes = int((n_acc.sum().item() + Bn) * kvD * 2 * 2)

    def time_fused_producers():
        # ---- the fused producers of draft-mode activations (RMSNorm + quantiser, SiLU*up +
        # quantiser): beside the step as well, against the quantiser alone on the same shape
        # and against the unfused pair with torch's own producer kernels in front of it
        px_h, pw_h, pgu_h = synth.producer_inputs(args.config)
        px, pw, pgu = to(px_h), to(pw_h), to(pgu_h)
        Kh, Ii = px.shape[1], pgu.shape[1] // 2
        pq_h = (torch.empty((Md, Kh // 2), dtype=torch.uint8, device=dev), torch.empty((Md, Kh // 128), dtype=torch.float32, device=dev))
        pq_i = (torch.empty((Md, Ii // 2), dtype=torch.uint8, device=dev), torch.empty((Md, Ii // 128), dtype=torch.float32, device=dev))
        ph = torch.empty((Md, Kh), dtype=torch.float16, device=dev)
        pi = torch.empty((Md, Ii), dtype=torch.float16, device=dev)

        def torch_rms():
            return torch.nn.functional.rms_norm(px, (Kh,), pw, synth.RMS_EPS)

        def torch_silu():
            return torch.nn.functional.silu(pgu[:, :Ii]) * pgu[:, Ii:]

        def per_call(f):
            return time_runner(make_runner(lambda: [f() for _ in range(n_rep_small)]), reps, 2) / n_rep_small * 1e6

        fused_producers = {
            "M": Md, "hidden": Kh, "intermediate": Ii,
            "rmsnorm_quant_us": round(per_call(lambda: B.rmsnorm_quant(px, pw, synth.RMS_EPS, pq_h[0], pq_h[1])), 3),
            "quant_act_alone_hidden_us": round(per_call(lambda: B.quant_act(ph, pq_h[0], pq_h[1])), 3),
            "torch_rms_norm_then_quant_act_us": round(per_call(lambda: B.quant_act(torch_rms(), pq_h[0], pq_h[1])), 3),
            "silu_mul_quant_us": round(per_call(lambda: B.silu_mul_quant(pgu, pq_i[0], pq_i[1])), 3),
            "quant_act_alone_intermediate_us": round(per_call(lambda: B.quant_act(pi, pq_i[0], pq_i[1])), 3),
            "torch_silu_mul_then_quant_act_us": round(per_call(lambda: B.quant_act(torch_silu(), pq_i[0], pq_i[1])), 3),
            # with the per-group Hadamard rotation in front of the quantiser
            "hadamard_quant_hidden_us": round(per_call(lambda: B.hadamard_quant(ph, pq_h[0], pq_h[1])), 3),
            "rmsnorm_rotate_quant_us": round(per_call(lambda: B.rmsnorm_quant(px, pw, synth.RMS_EPS, pq_h[0], pq_h[1], rotate=True)), 3),
            "silu_mul_rotate_quant_us": round(per_call(lambda: B.silu_mul_quant(pgu, pq_i[0], pq_i[1], rotate=True)), 3),
        }
        # the reordering quantiser (outlier channels last, one outlier group at 239 levels as two 4-bit
        # groups) and what the extra group costs the draft-mode GEMM of the first layer
        order = np.argsort(-np.abs(px_h.astype(np.float64)).mean(axis=0), kind="stable")
        pperm = to(np.concatenate([np.sort(order[128:]), np.sort(order[:128])]).astype(np.int32))
        Kx = Kh + 128
        pq_x = (torch.empty((Md, Kx // 2), dtype=torch.uint8, device=dev), torch.empty((Md, Kx // 128), dtype=torch.float32, device=dev))
        fused_producers["reorder_quant_hidden_us"] = round(per_call(lambda: B.reorder_quant(px, pperm, 1, pq_x[0], pq_x[1])), 3)
        lin0 = lins[0]
        blobs_x = []
        for l in range(L):
            cx = torch.randint(-8, 8, (lin0.N, Kx), dtype=torch.int8, device=dev, generator=gen)
            sx = (torch.rand((lin0.N, Kx // 128), device=dev, generator=gen) * 0.008 + 0.002).half()
            blobs_x.append(B.pack_weights(cx, sx))
            del cx, sx
        B.reorder_quant(px, pperm, 1, pq_x[0], pq_x[1])
        B.quant_act(px, pq_h[0], pq_h[1])
        y0 = torch.empty((Md, lin0.N), dtype=torch.float16, device=dev)
        ws_x = B.alloc_workspace(max(B.workspace_bytes(Md, lin0.N, Kx), B.workspace_bytes(Md, lin0.N, Kh), 16))
        t_kx = time_runner(make_runner(lambda: [B.gemm_w4a4(b, pq_x[0], pq_x[1], lin0.N, y=y0, workspace=ws_x) for b in blobs_x]), reps, 2) / L
        t_k = time_runner(make_runner(lambda: [B.gemm_w4a4(blobs[l][0], pq_h[0], pq_h[1], lin0.N, y=y0, workspace=ws_x) for l in range(L)]), reps, 2) / L
        fused_producers["draft_gemm_first_layer_us"] = {"K": round(t_k * 1e6, 3), "K_plus_one_outlier_group": round(t_kx * 1e6, 3)}
        del blobs_x

        # the MLP of a decoder block as the draft pass runs it: RMSNorm -> gate/up -> SiLU*up -> down,
        # fused producers (4 launches) against torch's producers + the plain quantiser (6 launches)
        i_gu = next(i for i, l in enumerate(lins) if l.name == "gate_up") if len(lins) == 4 else None
        if i_gu is not None and lins[i_gu].N == 2 * Ii and lins[3].K == Ii and lins[i_gu].K == Kh:
            ygu = torch.empty((Md, 2 * Ii), dtype=torch.float16, device=dev)
            ydn = torch.empty((Md, lins[3].N), dtype=torch.float16, device=dev)

            def mlp_fused():
                for l in range(L):
                    B.rmsnorm_quant(px, pw, synth.RMS_EPS, pq_h[0], pq_h[1])
                    B.gemm_w4a4(blobs[l][i_gu], pq_h[0], pq_h[1], 2 * Ii, y=ygu, workspace=ws)
                    B.silu_mul_quant(ygu, pq_i[0], pq_i[1])
                    B.gemm_w4a4(blobs[l][3], pq_i[0], pq_i[1], lins[3].N, y=ydn, workspace=ws)

            def mlp_unfused():
                for l in range(L):
                    B.quant_act(torch_rms(), pq_h[0], pq_h[1])
                    B.gemm_w4a4(blobs[l][i_gu], pq_h[0], pq_h[1], 2 * Ii, y=ygu, workspace=ws)
                    B.quant_act(torch.nn.functional.silu(ygu[:, :Ii]) * ygu[:, Ii:], pq_i[0], pq_i[1])
                    B.gemm_w4a4(blobs[l][3], pq_i[0], pq_i[1], lins[3].N, y=ydn, workspace=ws)

            fused_producers["draft_mlp_block_us"] = {
                "fused_producers": round(time_runner(make_runner(mlp_fused), reps, 2) / L * 1e6, 2),
                "torch_producers_plus_quant_act": round(time_runner(make_runner(mlp_unfused), reps, 2) / L * 1e6, 2)}
        fused_producers["silu_mul_quant_GBps"] = round((Md * Ii * 4 + Md * Ii // 2 + Md * (Ii // 128) * 4)
                                                       / fused_producers["silu_mul_quant_us"] / 1e3, 1)
        return fused_producers

    # (their quantiser and GEMM launches would mix into the kernel statistics of a profiling run)
    fused_producers = None if args.no_extra else time_fused_producers()

    after_verify = {
        "greedy_accept": dict(B=Bn, gamma=rows - 1, V=V, us=round(t_acc * 1e6, 3), launches=2,
                              GBps=round(acc_bytes / t_acc / 1e9, 1), hbm_frac=round(acc_bytes / t_acc / 1e9 / HBM_PEAK_GBS, 4),
                              accepted_per_cycle=round(float(n_acc.float().mean().item()), 3)),
        "kv_overwrite": dict(B=Bn, gamma=rows - 1, D=kvD, S=kvS, us=round(t_kv * 1e6, 3), launches=1,
                             GBps=round(kv_bytes / t_kv / 1e9, 1)),
    }

    # ---- CPU baseline: the oracle on one decoder block (bounded sample)
    cpu = None
    if not args.no_cpu_baseline:
        from oracle import qspec_oracle as orc
        try:
            from threadpoolctl import threadpool_info
            cores = max([p.get("num_threads", 1) for p in threadpool_info()] + [1])
        except Exception:
            cores = os.cpu_count() or 1
        host = []
        for i, lin in enumerate(lins):
            host.append((synth.weight_codes(args.config, i, lin.N, lin.K),
                         synth.weight_scales(args.config, i, lin.N, lin.K),
                         synth.activations(args.config, i, Md, lin.K, verify=False),
                         synth.activations(args.config, i, Mv, lin.K, verify=True)))
        # one decoder block is the unit; repeat it until about 10 s of oracle time
        c0 = time.perf_counter()
        n_rep = 0
        while True:
            for codes, scales, hxd, hxv in host:
                q, s = orc.quant_act(hxd)
                orc.gemm_w4a4(q, s, codes, scales)
                orc.gemm_w4a16(hxv, codes, scales)
            n_rep += 1
            c_t = time.perf_counter() - c0
            if c_t >= 10.0 or n_rep >= L:
                break
        cpu = dict(value=round(bytes_step / L * n_rep / c_t / 1e12, 6), unit="TB/s", cores=int(cores),
                   kind="oracle",
                   sample=f"{n_rep} of the {L} decoder blocks of one step (4 linears each, draft M={Md} + "
                          f"verify M={Mv}), {c_t:.1f} s of NumPy float64 oracle",
                   seconds_per_block=round(c_t / n_rep, 3))

    out = {
        "metric": "W4A4 & W4A16 GEMM us/call, achieved HBM TB/s + MFMA % at draft/verify M",
        "value": round(value, 4),
        "unit": "TB/s",
        "n_gpus": 1,
        "steps": args.steps,
        "warmup": args.warmup,
        "ms_per_step": round(t_step * 1e3, 4),
        "higher_is_better": True,
        "scaling": "weak",
        "vs_baseline": None,
        "dtype": "int4 weights; int8 MFMA/int32 (draft), fp16 MFMA/fp32 (verify)",
        "data": "synthetic",
        "config": {"workload": f"config {args.config} ({cfg.label}): Llama-shaped decoder linears x {L} blocks, "
                               f"draft W4A4 M={Md} (+quant_act), verify W4A16 M={Mv}",
                   "layers": L, "launch": "hip-graph" if use_graph else "eager",
                   "alg_bytes_per_step": bytes_step},
        "roofline": roofline,
        "cpu_baseline": cpu,
        "kernels": {k: dict(avg_us=round(v["seconds"] / v["launches"] * 1e6, 3),
                            GBps=round(v["bytes"] / v["seconds"] / 1e9, 1),
                            TOPS=round(v["flops"] / v["seconds"] / 1e12, 2)) for k, v in kernels.items()},
        "calls": calls,
        "same_shape": {"w4a4_draft_pass_us": round((t_4 + t_q) * 1e6, 1),
                       "w4a16_at_draft_M_pass_us": None if t_16d is None else round(t_16d * 1e6, 1)},
        "pack_weights_GBps": round(pack_bytes / t_pack / 1e9, 1) if t_pack > 0 else None,
        "after_verify": after_verify,
        "fused_producers": fused_producers,
        "extra_rows_M256_M512": extra,
        "vendor_fp16_gemm_context": vendor,
    }
    print(json.dumps(out))
    return 0


if __name__ == "__main__":
    sys.exit(main())
