#!/usr/bin/env python3
"""Benchmark of the QSpec W4 linear-layer hot path on one MI355X.

Workloads: the five configurations of the build's table (Llama-shaped decoder
linears, int4 weights with fp16 group scales, g = 128).  For a configuration one
*step* is one draft pass (activation quantiser + W4A4 GEMM at M = batch for every
linear) plus one verify pass (W4A16 GEMM at M = batch * (gamma + 1) for every
linear) over `layers` decoder blocks with distinct weight blobs (more packed
weights than the 256 MB last-level cache holds, so weight bytes come from HBM),
replayed as one HIP graph.  Weight packing runs once before the timed region (it
is off the token path) and is reported separately.

The default run measures ALL five configurations in one process.  The headline
(`value`, `ms_per_step`, `roofline`, `cpu_baseline` at the top level) is the
largest one, configuration 5 (Llama-70B-shaped, batch 128); `configs` holds the
same objects for every configuration, `ceilings` what the machine itself sustains
(bare streaming reads, matrix-instruction loops) measured by a bench-only HIP
library in the same run.

Prints ONE JSON line:  value = algorithmic bytes of a step / time, in TB/s.
"""
from __future__ import annotations

import argparse
import ctypes
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0          # MI355X published HBM3E bandwidth
MFMA_PEAK_TFLOPS = {"w4a16": 2500.0, "w4a4": 5000.0}   # published dense fp16 / int8 matrix peaks
DEFAULT_LAYERS = {1: 32, 2: 32, 3: 32, 4: 8, 5: 4}
CEIL_LIB = os.path.join(ROOT, "paper_2410_11305_amd", "libqspec_ceilings.so")


def alg_bytes_w4a16(M, N, K):
    G = K // 128
    return N * K // 2 + 2 * N * G + 2 * M * K + 2 * M * N


def alg_bytes_w4a4(M, N, K):
    G = K // 128
    return N * K // 2 + 2 * N * G + M * K // 2 + 4 * M * G + 2 * M * N


def alg_bytes_quant(M, K):
    return 2 * M * K + M * K // 2 + 4 * M * (K // 128)


def family(sym):
    """The kernel template and mode a profiler symbol belongs to (its instances differ in
    tiles per workgroup and the like, chosen per layer shape)."""
    if sym.startswith("gemm_stream_kernel<"):
        return "gemm_stream_kernel<" + ",".join(sym.split("<")[1].split(",")[:2]) + ", *>"
    return sym.split("<")[0] + ("<*>" if "<" in sym else "")


class Bench:
    def __init__(self, args):
        import numpy as np
        import torch
        from paper_2410_11305_amd import binding as B
        from paper_2410_11305_amd import synth
        self.np, self.torch, self.B, self.synth, self.args = np, torch, B, synth, args
        self.dev = torch.device("cuda:0")
        self.use_graph = not args.no_graph
        self.blob_cache = {}           # (N, K) -> list of packed blobs (blocks 1.. drawn on the GPU)
        self.t_pack, self.pack_bytes = 0.0, 0
        try:
            with open(os.path.join(ROOT, "profiles", "hbm_traffic.json")) as f:
                self.traffic_table = json.load(f).get("by_config", {})
        except (OSError, ValueError):
            self.traffic_table = {}

    def to(self, a):
        return self.torch.from_numpy(self.np.ascontiguousarray(a)).to(self.dev)

    # ---- launching and timing
    def make_runner(self, fn):
        """A callable that enqueues fn's launches on the current stream (a replayed HIP graph
        unless --no-graph)."""
        torch = self.torch
        fn()                       # eager once: first-call effects stay out of the capture
        torch.cuda.synchronize()
        if not self.use_graph:
            return fn
        g = torch.cuda.CUDAGraph()
        with torch.cuda.graph(g):
            fn()
        torch.cuda.synchronize()
        return g.replay

    def time_runner(self, run, reps, warm):
        """Seconds per run: HIP events on the launch stream around `reps` runs."""
        torch = self.torch
        for _ in range(warm):
            run()
        torch.cuda.synchronize()
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record()
        for _ in range(reps):
            run()
        e1.record()
        torch.cuda.synchronize()
        return e0.elapsed_time(e1) * 1e-3 / reps

    # ---- inputs
    def blobs_for(self, ci, li, N, K, L, gen):
        """L packed blobs of an [N, K] layer: block 0 from the seeded NumPy recipe of
        configuration ci, further blocks drawn on the GPU (same distributions), all packed by
        the library itself.  Configurations with the same layer shapes share them."""
        torch, B = self.torch, self.B
        have = self.blob_cache.setdefault((N, K), [])
        while len(have) < L:
            l = len(have)
            if l == 0:
                codes = self.to(self.synth.weight_codes(ci, li, N, K))
                scales = self.to(self.synth.weight_scales(ci, li, N, K))
            else:
                codes = torch.randint(-8, 8, (N, K), dtype=torch.int8, device=self.dev, generator=gen)
                scales = (torch.rand((N, K // 128), device=self.dev, generator=gen) * 0.008 + 0.002).half()
            out = torch.empty(B.packed_weight_bytes(N, K), dtype=torch.uint8, device=self.dev)
            e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            e0.record()
            B.pack_weights(codes, scales, out)
            e1.record()
            e1.synchronize()
            if l > 0:
                self.t_pack += e0.elapsed_time(e1) * 1e-3
                self.pack_bytes += N * K + 2 * N * (K // 128) + out.numel()
            have.append(out)
            del codes, scales
        return have[:L]

    def drop_blobs_except(self, shapes):
        for key in list(self.blob_cache):
            if key not in shapes:
                del self.blob_cache[key]
        self.torch.cuda.empty_cache()

    # ---- one configuration
    def run_config(self, ci, extras):
        np, torch, B, synth, args = self.np, self.torch, self.B, self.synth, self.args
        dev = self.dev
        cfg = synth.CONFIGS[ci]
        Md, Mv = cfg.draft_M, cfg.verify_M
        lins = list(cfg.layers)
        L = args.layers or DEFAULT_LAYERS[ci]
        gen = torch.Generator(device=dev)
        gen.manual_seed(10000 * ci + 99)
        self.drop_blobs_except({(l.N, l.K) for l in lins})
        blobs = [self.blobs_for(ci, i, lin.N, lin.K, L, gen) for i, lin in enumerate(lins)]     # [layer][block]
        xd = [self.to(synth.activations(ci, i, Md, lin.K, verify=False)) for i, lin in enumerate(lins)]
        xv = [self.to(synth.activations(ci, i, Mv, lin.K, verify=True)) for i, lin in enumerate(lins)]
        qa = [torch.empty((Md, lin.K // 2), dtype=torch.uint8, device=dev) for lin in lins]
        sa = [torch.empty((Md, lin.K // 128), dtype=torch.float32, device=dev) for lin in lins]
        qav = [torch.empty((Mv, lin.K // 2), dtype=torch.uint8, device=dev) for lin in lins]
        sav = [torch.empty((Mv, lin.K // 128), dtype=torch.float32, device=dev) for lin in lins]
        yd = [torch.empty((Md, lin.N), dtype=torch.float16, device=dev) for lin in lins]
        yv = [torch.empty((Mv, lin.N), dtype=torch.float16, device=dev) for lin in lins]
        ws_bytes = max([B.workspace_bytes(M, l.N, l.K) for l in lins for M in (Md, Mv)] + [16])
        ws = B.alloc_workspace(ws_bytes)
        nl = len(lins)
        # Layers whose draft-mode product runs on the tiled kernel take their activation codes in
        # the quantiser's widened format (same codes and scales, one byte per code): quantiser
        # and GEMM of such a layer are the *_wide entry points, everywhere in this benchmark.
        wide_d = [B.w4a4_takes_wide(Md, lin.N, lin.K) for lin in lins]
        wide_v = [B.w4a4_takes_wide(Mv, lin.N, lin.K) for lin in lins]
        qa8 = [torch.empty((Md, lin.K), dtype=torch.int8, device=dev) if w else None for lin, w in zip(lins, wide_d)]
        qav8 = [torch.empty((Mv, lin.K), dtype=torch.int8, device=dev) if w else None for lin, w in zip(lins, wide_v)]

        def quant(i, verify=False):
            src, q, q8, s, wide = (xv, qav, qav8, sav, wide_v) if verify else (xd, qa, qa8, sa, wide_d)
            if wide[i]:
                B.quant_act_wide(src[i], q8[i], s[i])
            else:
                B.quant_act(src[i], q[i], s[i])

        def w4a4(i, l, verify=False):
            q, q8, s, y, wide = (qav, qav8, sav, yv, wide_v) if verify else (qa, qa8, sa, yd, wide_d)
            if wide[i]:
                B.gemm_w4a4_wide(blobs[i][l], q8[i], s[i], lins[i].N, y=y[i], workspace=ws)
            else:
                B.gemm_w4a4(blobs[i][l], q[i], s[i], lins[i].N, y=y[i], workspace=ws)

        def run_quant(M_is_verify=False):
            for _ in range(L):
                for i in range(nl):
                    quant(i, M_is_verify)

        def run_w4a4(M_is_verify=False):
            for l in range(L):
                for i in range(nl):
                    w4a4(i, l, M_is_verify)

        def run_draft():
            for l in range(L):
                for i in range(nl):
                    quant(i)
                    w4a4(i, l)

        def run_w4a16(M_is_verify=True):
            x, y = (xv, yv) if M_is_verify else (xd, yd)
            for l in range(L):
                for i, lin in enumerate(lins):
                    B.gemm_w4a16(blobs[i][l], x[i], lin.N, y=y[i], workspace=ws)

        def run_step():
            run_draft()
            run_w4a16(True)

        def one_kind(kind, i):
            lin = lins[i]

            def f():
                for l in range(L):
                    if kind == "w4a4":
                        w4a4(i, l)
                    else:
                        B.gemm_w4a16(blobs[i][l], xv[i], lin.N, y=yv[i], workspace=ws)
            return f

        # ---- the step: K steps, wall clock bracketed by synchronize
        step = self.make_runner(run_step)
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
        flops_step = sum(2 * (Md + Mv) * l.N * l.K for l in lins) * L

        # ---- per-call and per-kernel durations: HIP events on the launch stream around a
        # replayed graph that holds only that call's L launches (distinct weight blobs)
        reps = max(3, min(20, args.steps // 4))
        t_q = self.time_runner(self.make_runner(run_quant), reps, 2)
        calls = {}
        kernels = {"quant_act_kernel": dict(launches=L * nl, seconds=t_q, flops=0, mode="quant",
                                            bytes=sum(alg_bytes_quant(Md, l.K) for l in lins) * L)}
        for i, lin in enumerate(lins):
            for kind, M, ab in (("w4a4", Md, alg_bytes_w4a4), ("w4a16", Mv, alg_bytes_w4a16)):
                t = self.time_runner(self.make_runner(one_kind(kind, i)), reps, 2)          # L launches
                fl = 2 * M * lin.N * lin.K
                calls[f"{lin.name}.{kind}.M{M}"] = dict(
                    us=round(t / L * 1e6, 3), TBps=round(ab(M, lin.N, lin.K) * L / t / 1e12, 3),
                    hbm_frac=round(ab(M, lin.N, lin.K) * L / t / 1e9 / HBM_PEAK_GBS, 4),
                    mfma_frac=round(fl * L / t / 1e12 / MFMA_PEAK_TFLOPS[kind], 4))
                name = B.describe_kernel(kind == "w4a4", M, lin.N, lin.K)          # the profiler's symbol
                if kind == "w4a4" and wide_d[i]:
                    name = name.replace(", false>", ", true>")                     # (the instance that takes widened codes)
                k = kernels.setdefault(name, dict(launches=0, seconds=0.0, bytes=0, flops=0, mode=kind))
                k["launches"] += L
                k["seconds"] += t
                k["bytes"] += ab(M, lin.N, lin.K) * L
                k["flops"] += fl * L
        # The roofline object is for the dominant KERNEL, i.e. one __global__ template in one
        # mode; its instances are separate symbols to the profiler and are added up here (the
        # profile summaries carry the same family rows).
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
        # HBM traffic per launch of that kernel from the committed counter summary of THIS
        # configuration (launch-weighted mean over the family's symbols), if it covers them
        traffic = None
        per = self.traffic_table.get(str(ci), {})
        if kd["symbols"] and all(sym in per for sym in kd["symbols"]):
            traffic = int(sum(per[sym] * kernels[sym]["launches"] for sym in kd["symbols"]) / kd["launches"])
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
                        alg_flops_per_launch=kd["flops"] // kd["launches"],
                        share_of_step=round(kd["seconds"] / max(sum(v["seconds"] for v in families.values()), 1e-30), 3))

        # ---- both modes at the same M (one pass over the configuration's blocks; the draft
        # side includes its quantiser launches), at the draft M and at the verify M
        same = None
        if not args.no_extra:
            t_4d = self.time_runner(self.make_runner(run_w4a4), reps, 2)
            t_16d = self.time_runner(self.make_runner(lambda: run_w4a16(False)), reps, 2)
            run_quant(True)
            t_qv = self.time_runner(self.make_runner(lambda: run_quant(True)), reps, 2)
            t_4v = self.time_runner(self.make_runner(lambda: run_w4a4(True)), reps, 2)
            t_16v = self.time_runner(self.make_runner(lambda: run_w4a16(True)), reps, 2)
            fl_d = sum(2 * Md * l.N * l.K for l in lins) * L
            fl_v = sum(2 * Mv * l.N * l.K for l in lins) * L
            same = {
                f"M{Md}": {"w4a4_gemm_pass_us": round(t_4d * 1e6, 1), "quant_act_pass_us": round(t_q * 1e6, 1),
                           "w4a16_pass_us": round(t_16d * 1e6, 1),
                           "w4a4_gemm_over_w4a16": round(t_16d / t_4d, 3),
                           "w4a4_mfma_frac": round(fl_d / t_4d / 1e12 / MFMA_PEAK_TFLOPS["w4a4"], 4),
                           "w4a16_mfma_frac": round(fl_d / t_16d / 1e12 / MFMA_PEAK_TFLOPS["w4a16"], 4)},
                f"M{Mv}": {"w4a4_gemm_pass_us": round(t_4v * 1e6, 1), "quant_act_pass_us": round(t_qv * 1e6, 1),
                           "w4a16_pass_us": round(t_16v * 1e6, 1),
                           "w4a4_gemm_over_w4a16": round(t_16v / t_4v, 3),
                           "w4a4_mfma_frac": round(fl_v / t_4v / 1e12 / MFMA_PEAK_TFLOPS["w4a4"], 4),
                           "w4a16_mfma_frac": round(fl_v / t_16v / 1e12 / MFMA_PEAK_TFLOPS["w4a16"], 4)},
            }

        cpu = None if args.no_cpu_baseline else self.cpu_baseline(ci, lins, Md, Mv, extras.get("cpu_seconds", 3.0))

        out = {
            "workload": f"config {ci} ({cfg.label}): Llama-shaped decoder linears x {L} blocks, "
                        f"draft W4A4 M={Md} (+quant_act), verify W4A16 M={Mv}",
            "layers": L, "launch": "hip-graph" if self.use_graph else "eager",
            "value": round(bytes_step / t_step / 1e12, 4), "unit": "TB/s",
            "ms_per_step": round(t_step * 1e3, 4),
            "alg_bytes_per_step": bytes_step, "alg_flops_per_step": flops_step,
            "TOPS": round(flops_step / t_step / 1e12, 1),
            "roofline": roofline,
            "cpu_baseline": cpu,
            "kernels": {k: dict(avg_us=round(v["seconds"] / v["launches"] * 1e6, 3),
                                GBps=round(v["bytes"] / v["seconds"] / 1e9, 1),
                                TOPS=round(v["flops"] / v["seconds"] / 1e12, 2)) for k, v in kernels.items()},
            "calls": calls,
            "widened_activation_format": {"draft_M": {lin.name: bool(w) for lin, w in zip(lins, wide_d)},
                                          "verify_M": {lin.name: bool(w) for lin, w in zip(lins, wide_v)}},
            "same_shape": same,
        }
        if extras.get("rows_256_512"):
            out["extra_rows_M256_M512"] = self.extra_rows(lins, blobs, L, gen, (256, 512, 1024, 2048) if args.prefill else (256, 512))
        if extras.get("stream_read"):
            out["bare_read"] = self.bare_reads(lins, blobs, L, Md)
        if extras.get("vendor"):
            out["vendor_fp16_gemm_context"] = self.vendor_context(lins, xv, Mv, gen)
        if extras.get("after_verify"):
            out["after_verify"] = self.after_verify(ci, lins, gen, reps)
        if extras.get("fused_producers"):
            out["fused_producers"] = self.fused_producers(ci, lins, blobs, L, Md, gen, reps, ws)
        return out

    # ---- extra rows: both modes at 256 and 512 tokens on a configuration's layers
    def extra_rows(self, lins, blobs, L, gen, Ms):
        torch, B, dev = self.torch, self.B, self.dev
        extra = {}
        for Mx in Ms:
            xx = [torch.randn((Mx, lin.K), device=dev, generator=gen).half() for lin in lins]
            wide = [B.w4a4_takes_wide(Mx, lin.N, lin.K) for lin in lins]
            qx = [B.quant_act_wide(t) if w else B.quant_act(t) for t, w in zip(xx, wide)]
            yx = [torch.empty((Mx, lin.N), dtype=torch.float16, device=dev) for lin in lins]
            wsx = B.alloc_workspace(max([B.workspace_bytes(Mx, l.N, l.K) for l in lins] + [16]))
            Lx = min(L, 4)
            for i, lin in enumerate(lins):
                for kind in ("w4a4", "w4a16"):
                    def f(i=i, lin=lin, kind=kind):
                        for l in range(Lx):
                            if kind == "w4a4":
                                (B.gemm_w4a4_wide if wide[i] else B.gemm_w4a4)(blobs[i][l], qx[i][0], qx[i][1], lin.N, y=yx[i], workspace=wsx)
                            else:
                                B.gemm_w4a16(blobs[i][l], xx[i], lin.N, y=yx[i], workspace=wsx)
                    t = self.time_runner(self.make_runner(f), 3, 1) / Lx
                    extra[f"{lin.name}.{kind}.M{Mx}"] = dict(
                        us=round(t * 1e6, 2),
                        mfma_frac=round(2 * Mx * lin.N * lin.K / t / 1e12 / MFMA_PEAK_TFLOPS[kind], 4))
            del xx, qx, yx, wsx
        return extra

    # ---- ceilings (bench-only HIP library, built by build())
    def ceil_lib(self):
        L = ctypes.CDLL(CEIL_LIB)
        vp, ci, sz = ctypes.c_void_p, ctypes.c_int, ctypes.c_size_t
        L.ceil_stream_read.restype = ci
        L.ceil_stream_read.argtypes = [vp, sz, ci, vp, vp]
        L.ceil_mfma.restype = ci
        L.ceil_mfma.argtypes = [ci, vp, ci, ci, vp, vp]
        L.ceil_empty.restype = ci
        L.ceil_empty.argtypes = [vp]
        L.ceil_quant_prologue.restype = ci
        L.ceil_quant_prologue.argtypes = [vp, ci, ci, ci, vp, vp]
        return L

    def bare_reads(self, lins, blobs, L, Md):
        """A bare streaming read of each layer's packed weights (the same rotating blobs, one
        launch per blob, the tile-to-workgroup split of the streaming kernel's plan): what one
        launch can reach at most on these byte counts."""
        torch, B = self.torch, self.B
        C = self.ceil_lib()
        sink = torch.zeros(16, dtype=torch.int32, device=self.dev)
        out = {}
        for i, lin in enumerate(lins):
            G = lin.K // 128
            name = B.describe_kernel(True, Md, lin.N, lin.K)
            nbytes = lin.N * lin.K // 2            # the code tiles; whole 1 KB tiles
            if name.startswith("gemm_stream_kernel"):
                per = int(name.split(",")[-1].strip(" >")) * G       # NT tiles per workgroup over all of K
            else:
                per = max(1, nbytes // 1024 // 2048)                 # tiled kernels: about 2048 workgroups
            nt = per / G

            def f(i=i, nbytes=nbytes, per=per):
                s = torch.cuda.current_stream().cuda_stream
                for l in range(L):
                    rc = C.ceil_stream_read(blobs[i][l].data_ptr(), nbytes, per, sink.data_ptr(), s)
                    assert rc == 0, rc
            t = self.time_runner(self.make_runner(f), 5, 2) / L
            out[lin.name] = dict(bytes=nbytes, us=round(t * 1e6, 3), TBps=round(nbytes / t / 1e12, 3),
                                 hbm_frac=round(nbytes / t / 1e9 / HBM_PEAK_GBS, 4), tiles_per_workgroup=per)
        return out

    def machine_ceilings(self):
        torch = self.torch
        C = self.ceil_lib()
        dev = self.dev
        out = {}
        s = lambda: torch.cuda.current_stream().cuda_stream
        n_empty = 64
        t = self.time_runner(self.make_runner(lambda: [C.ceil_empty(s()) for _ in range(n_empty)]), 10, 2) / n_empty
        out["empty_kernel_in_graph_us"] = round(t * 1e6, 3)
        gen = torch.Generator(device=dev)
        gen.manual_seed(7)
        ops_f16 = torch.randn((8 << 20,), device=dev, generator=gen).half()                       # 16 MiB of random fp16
        ops_i8 = torch.randint(-128, 128, (16 << 20,), dtype=torch.int8, device=dev, generator=gen)
        ops_const = torch.full((8 << 20,), 1.0, dtype=torch.float16, device=dev)
        # operands distributed as the kernels' own: a thread of the loop takes units 0..3 of its
        # 8 x 16 bytes as A and units 4..7 as B.  Verify mode: A = fp16(code * scale), B = the
        # input recipe's activations (one channel in a hundred 20x); draft mode: 16 * code, the
        # form the draft kernels feed the matrix unit
        # (the clock this part holds depends on how many operand bits toggle)
        n = (1 << 20) // 8
        w16 = (torch.randint(-8, 8, (n, 4, 8), device=dev, generator=gen).float() *
               (torch.rand((n, 4, 1), device=dev, generator=gen) * 0.008 + 0.002).half().float()).half()
        x16 = (torch.randn((n, 4, 8), device=dev, generator=gen) *
               torch.where(torch.rand((n, 4, 8), device=dev, generator=gen) < 0.01, 20.0, 1.0)).half()
        ops_verify = torch.cat([w16, x16], dim=1).contiguous()
        ops_draft = (torch.cat([torch.randint(-7, 8, (n, 4, 16), dtype=torch.int8, device=dev, generator=gen),
                                torch.randint(-8, 8, (n, 4, 16), dtype=torch.int8, device=dev, generator=gen)], dim=1) * 16).contiguous()
        ops_zero = torch.zeros((8 << 20,), dtype=torch.float16, device=dev)
        sink = torch.zeros(16, dtype=torch.float32, device=dev)
        blocks, iters, waves = 256, 2000, 8
        f16_flop, i8_flop = 2 * 32 * 32 * 16, 2 * 32 * 32 * 32
        C.ceil_mfma(0, ops_f16.data_ptr(), blocks, iters, sink.data_ptr(), s())       # (the first loop after start-up times slow)
        for key, kind, ops, flop, peak in (("mfma_f16_32x32x16_random_operands", 0, ops_f16, f16_flop, 2500.0),
                                           ("mfma_f16_32x32x16_constant_operands", 0, ops_const, f16_flop, 2500.0),
                                           ("mfma_f16_32x32x16_zero_operands", 0, ops_zero, f16_flop, 2500.0),
                                           ("mfma_f16_32x32x16_verify_mode_operands", 0, ops_verify, f16_flop, 2500.0),
                                           ("mfma_i8_32x32x32_random_operands", 1, ops_i8, i8_flop, 5000.0),
                                           ("mfma_i8_32x32x32_draft_mode_operands", 1, ops_draft, i8_flop, 5000.0),
                                           ("mfma_i8_plus_group_rescale_2fma_per_output", 2, ops_i8, i8_flop, 5000.0),
                                           ("mfma_i8_draft_mode_operands_plus_group_rescale", 2, ops_draft, i8_flop, 5000.0)):
            def f(kind=kind, ops=ops):
                rc = C.ceil_mfma(kind, ops.data_ptr(), blocks, iters, sink.data_ptr(), s())
                assert rc == 0, rc
            t = self.time_runner(self.make_runner(f), 5, 2)
            tops = blocks * waves * iters * 16 * flop / t / 1e12
            out[key] = dict(TOPS=round(tops, 1), frac_of_published_peak=round(tops / peak, 4), us=round(t * 1e6, 1))
        # what a quantiser fused into the small-M draft GEMM would add to that kernel (every one of
        # its workgroups would quantise all of x), against the separate quantiser launch it would save
        B = self.B
        fused = {}
        n_rep = 16
        for M, K in ((8, 4096), (8, 11008), (32, 4096), (32, 11008)):
            x = torch.randn((M, K), device=dev, generator=gen).half()
            scratch = torch.empty(256 * (M * K // 2 + M * K // 32), dtype=torch.uint8, device=dev)
            qa = torch.empty((M, K // 2), dtype=torch.uint8, device=dev)
            sa = torch.empty((M, K // 128), dtype=torch.float32, device=dev)

            def f(x=x, M=M, K=K, scratch=scratch):
                for _ in range(n_rep):
                    rc = C.ceil_quant_prologue(x.data_ptr(), M, K, 256, scratch.data_ptr(), s())
                    assert rc == 0, rc
            t_in = self.time_runner(self.make_runner(f), 5, 2) / n_rep
            t_sep = self.time_runner(self.make_runner(lambda x=x, qa=qa, sa=sa: [B.quant_act(x, qa, sa) for _ in range(n_rep)]), 5, 2) / n_rep
            fused[f"M{M}.K{K}"] = dict(every_workgroup_quantises_all_of_x_us=round(t_in * 1e6, 2),
                                       separate_quant_act_launch_us=round(t_sep * 1e6, 2))
        out["quantiser_inside_small_M_draft_gemm"] = fused
        return out

    # ---- optional yardstick: the vendor library's plain fp16 GEMM on the verify-mode shapes
    def vendor_context(self, lins, xv, Mv, gen):
        torch, dev = self.torch, self.dev
        vendor = {}
        for i, lin in enumerate(lins):
            Rv = max(2, int(1.2e9 // (lin.N * lin.K * 2)) + 1)           # rotate over more fp16 weight bytes than the last-level cache holds
            Wv = [(torch.randn((lin.N, lin.K), device=dev, generator=gen) * 0.03).half() for _ in range(Rv)]
            yvv = torch.empty((Mv, lin.N), dtype=torch.float16, device=dev)
            t = self.time_runner(self.make_runner(lambda: [torch.matmul(xv[i], W.t(), out=yvv) for W in Wv]), 3, 1) / Rv
            vendor[f"{lin.name}.fp16.M{Mv}"] = dict(us=round(t * 1e6, 2), TFLOPs=round(2 * Mv * lin.N * lin.K / t / 1e12, 1),
                                                     weight_TBps=round(lin.N * lin.K * 2 / t / 1e12, 2))
            del Wv, yvv
        return vendor

    # ---- the steps after the verify pass (greedy acceptance, KV-cache overwrite): not part
    # of the step, timed on their own at the configuration's batch and draft length
    def after_verify(self, ci, lins, gen, reps):
        torch, B, dev, synth = self.torch, self.B, self.dev, self.synth
        lg_h, dr_h, _ = synth.accept_inputs(ci)
        Bn, rows, V = lg_h.shape
        kvD, kvS = lins[0].K, 2048                       # one K (or V) row of a decoder block; cache length 2048
        lg, dr = self.to(lg_h), self.to(dr_h)
        n_acc = torch.empty((Bn,), dtype=torch.int32, device=dev)
        out_tok = torch.empty((Bn, rows), dtype=torch.int32, device=dev)
        ws_acc = torch.empty(max(B.accept_workspace_bytes(Bn, rows - 1, V), 16), dtype=torch.uint8, device=dev)
        kv_new = torch.randn((Bn, rows, kvD), device=dev, generator=gen).half()
        kv_cache = torch.zeros((Bn, kvS, kvD), dtype=torch.float16, device=dev)
        kv_pos = torch.randint(0, kvS - rows, (Bn,), device=dev, generator=gen).to(torch.int32)
        n_rep = 16
        t_acc = self.time_runner(self.make_runner(lambda: [B.greedy_accept(lg, dr, n_acc, out_tok, ws_acc) for _ in range(n_rep)]),
                                 reps, 2) / n_rep
        t_kv = self.time_runner(self.make_runner(lambda: [B.kv_overwrite(kv_cache, kv_new, n_acc, kv_pos) for _ in range(n_rep)]),
                                reps, 2) / n_rep
        acc_bytes = Bn * rows * V * 2 + Bn * (rows - 1) * 4 + Bn * (rows + 1) * 4
        kv_bytes = int((n_acc.sum().item() + Bn) * kvD * 2 * 2)
        return {
            "greedy_accept": dict(B=Bn, gamma=rows - 1, V=V, us=round(t_acc * 1e6, 3), launches=2,
                                  GBps=round(acc_bytes / t_acc / 1e9, 1), hbm_frac=round(acc_bytes / t_acc / 1e9 / HBM_PEAK_GBS, 4),
                                  accepted_per_cycle=round(float(n_acc.float().mean().item()), 3)),
            "kv_overwrite": dict(B=Bn, gamma=rows - 1, D=kvD, S=kvS, us=round(t_kv * 1e6, 3), launches=1,
                                 GBps=round(kv_bytes / t_kv / 1e9, 1)),
        }

    # ---- the fused producers of draft-mode activations, beside the step: against the
    # quantiser alone on the same shape and against the unfused pair with torch's producers
    def fused_producers(self, ci, lins, blobs, L, Md, gen, reps, ws):
        np, torch, B, dev, synth = self.np, self.torch, self.B, self.dev, self.synth
        px_h, pw_h, pgu_h = synth.producer_inputs(ci)
        px, pw, pgu = self.to(px_h), self.to(pw_h), self.to(pgu_h)
        Kh, Ii = px.shape[1], pgu.shape[1] // 2
        pq_h = (torch.empty((Md, Kh // 2), dtype=torch.uint8, device=dev), torch.empty((Md, Kh // 128), dtype=torch.float32, device=dev))
        pq_i = (torch.empty((Md, Ii // 2), dtype=torch.uint8, device=dev), torch.empty((Md, Ii // 128), dtype=torch.float32, device=dev))
        ph = torch.empty((Md, Kh), dtype=torch.float16, device=dev)
        pi = torch.empty((Md, Ii), dtype=torch.float16, device=dev)
        n_rep = 16

        def torch_rms():
            return torch.nn.functional.rms_norm(px, (Kh,), pw, synth.RMS_EPS)

        def torch_silu():
            return torch.nn.functional.silu(pgu[:, :Ii]) * pgu[:, Ii:]

        def per_call(f):
            return self.time_runner(self.make_runner(lambda: [f() for _ in range(n_rep)]), reps, 2) / n_rep * 1e6

        out = {
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
        pperm = self.to(np.concatenate([np.sort(order[128:]), np.sort(order[:128])]).astype(np.int32))
        Kx = Kh + 128
        pq_x = (torch.empty((Md, Kx // 2), dtype=torch.uint8, device=dev), torch.empty((Md, Kx // 128), dtype=torch.float32, device=dev))
        out["reorder_quant_hidden_us"] = round(per_call(lambda: B.reorder_quant(px, pperm, 1, pq_x[0], pq_x[1])), 3)
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
        t_kx = self.time_runner(self.make_runner(lambda: [B.gemm_w4a4(b, pq_x[0], pq_x[1], lin0.N, y=y0, workspace=ws_x) for b in blobs_x]), reps, 2) / L
        t_k = self.time_runner(self.make_runner(lambda: [B.gemm_w4a4(blobs[0][l], pq_h[0], pq_h[1], lin0.N, y=y0, workspace=ws_x) for l in range(L)]), reps, 2) / L
        out["draft_gemm_first_layer_us"] = {"K": round(t_k * 1e6, 3), "K_plus_one_outlier_group": round(t_kx * 1e6, 3)}
        del blobs_x

        # the MLP of a decoder block as the draft pass runs it: RMSNorm -> gate/up -> SiLU*up -> down,
        # fused producers (4 launches) against torch's producers + the plain quantiser (6 launches)
        i_gu = next(i for i, l in enumerate(lins) if l.name == "gate_up") if len(lins) == 4 else None
        if i_gu is not None and lins[i_gu].N == 2 * Ii and lins[3].K == Ii and lins[i_gu].K == Kh:
            ygu = torch.empty((Md, 2 * Ii), dtype=torch.float16, device=dev)
            ydn = torch.empty((Md, lins[3].N), dtype=torch.float16, device=dev)

            # (a consumer that runs on the tiled kernel gets its codes in the widened format,
            # straight from the fused producer)
            wide_gu = B.w4a4_takes_wide(Md, 2 * Ii, Kh)
            wide_dn = B.w4a4_takes_wide(Md, lins[3].N, Ii)
            q8_h = torch.empty((Md, Kh), dtype=torch.int8, device=dev) if wide_gu else None
            q8_i = torch.empty((Md, Ii), dtype=torch.int8, device=dev) if wide_dn else None

            def mlp_fused():
                for l in range(L):
                    if wide_gu:
                        B.rmsnorm_quant(px, pw, synth.RMS_EPS, q8_h, pq_h[1], wide=True)
                        B.gemm_w4a4_wide(blobs[i_gu][l], q8_h, pq_h[1], 2 * Ii, y=ygu, workspace=ws)
                    else:
                        B.rmsnorm_quant(px, pw, synth.RMS_EPS, pq_h[0], pq_h[1])
                        B.gemm_w4a4(blobs[i_gu][l], pq_h[0], pq_h[1], 2 * Ii, y=ygu, workspace=ws)
                    if wide_dn:
                        B.silu_mul_quant(ygu, q8_i, pq_i[1], wide=True)
                        B.gemm_w4a4_wide(blobs[3][l], q8_i, pq_i[1], lins[3].N, y=ydn, workspace=ws)
                    else:
                        B.silu_mul_quant(ygu, pq_i[0], pq_i[1])
                        B.gemm_w4a4(blobs[3][l], pq_i[0], pq_i[1], lins[3].N, y=ydn, workspace=ws)

            def mlp_unfused():
                for l in range(L):
                    B.quant_act(torch_rms(), pq_h[0], pq_h[1])
                    B.gemm_w4a4(blobs[i_gu][l], pq_h[0], pq_h[1], 2 * Ii, y=ygu, workspace=ws)
                    B.quant_act(torch.nn.functional.silu(ygu[:, :Ii]) * ygu[:, Ii:], pq_i[0], pq_i[1])
                    B.gemm_w4a4(blobs[3][l], pq_i[0], pq_i[1], lins[3].N, y=ydn, workspace=ws)

            out["draft_mlp_block_us"] = {
                "fused_producers": round(self.time_runner(self.make_runner(mlp_fused), reps, 2) / L * 1e6, 2),
                "torch_producers_plus_quant_act": round(self.time_runner(self.make_runner(mlp_unfused), reps, 2) / L * 1e6, 2)}
            # the same block with gate/up -> SiLU*up + quantiser -> down as ONE persistent launch
            # (2 launches per block instead of 4), where the kernel takes the shape
            if Md <= 32:
                try:
                    ws_m = B.alloc_workspace(B.mlp_draft_workspace_bytes(Md, Kh, Ii))
                    st_m = torch.zeros(1, dtype=torch.int32, device=dev)

                    def mlp_persistent():
                        for l in range(L):
                            B.rmsnorm_quant(px, pw, synth.RMS_EPS, pq_h[0], pq_h[1])
                            B.mlp_draft(blobs[i_gu][l], blobs[3][l], pq_h[0], pq_h[1], Kh, Ii, ws_m, st_m, ygu, pq_i[0], pq_i[1], ydn)

                    t_p = self.time_runner(self.make_runner(mlp_persistent), reps, 2) / L * 1e6
                    out["draft_mlp_block_us"]["persistent_launch"] = round(t_p, 2)
                    out["draft_mlp_block_us"]["persistent_launch_gave_up"] = int(st_m.item())
                    mlp_bytes = alg_bytes_w4a4(Md, 2 * Ii, Kh) + alg_bytes_w4a4(Md, Kh, Ii)
                    out["draft_mlp_block_us"]["hbm_frac_of_the_two_gemms"] = {
                        "separate_launches": round(mlp_bytes / (out["draft_mlp_block_us"]["fused_producers"] * 1e-6) / 1e9 / HBM_PEAK_GBS, 4),
                        "persistent_launch": round(mlp_bytes / (t_p * 1e-6) / 1e9 / HBM_PEAK_GBS, 4)}
                except B.QSpecError as e:
                    out["draft_mlp_block_us"]["persistent_launch"] = str(e)
        out["silu_mul_quant_GBps"] = round((Md * Ii * 4 + Md * Ii // 2 + Md * (Ii // 128) * 4) / out["silu_mul_quant_us"] / 1e3, 1)
        return out

    # ---- CPU baseline: the oracle as it stands on a bounded sample of the configuration
    def cpu_baseline(self, ci, lins, Md, Mv, budget_s):
        """The NumPy float64 oracle (BLAS threads of the host) on column chunks of the
        configuration's layers, round-robin over the layers, until about budget_s seconds of
        oracle time: quantiser + draft-mode product at M = Md and verify-mode product at M = Mv
        for each chunk.  Throughput in the step's unit (algorithmic bytes of the columns done)."""
        np, synth = self.np, self.synth
        from oracle import qspec_oracle as orc
        try:
            from threadpoolctl import threadpool_info
            cores = max([p.get("num_threads", 1) for p in threadpool_info()] + [1])
        except Exception:
            cores = os.cpu_count() or 1
        chunk = 512
        host = []
        for i, lin in enumerate(lins):
            n_rows = min(lin.N, 32 * chunk)             # the sample never needs more rows than this
            rng_codes = synth.weight_codes(ci, i, lin.N, lin.K)[:n_rows] if lin.N * lin.K <= (1 << 28) else None
            if rng_codes is None:                       # very large layers: draw the sampled rows only (same distribution)
                rng = np.random.default_rng(10000 * ci + 100 * i)
                rng_codes = rng.integers(-8, 8, size=(n_rows, lin.K), dtype=np.int8)
                scales = rng.uniform(0.002, 0.01, size=(n_rows, lin.K // 128)).astype(np.float16)
            else:
                scales = synth.weight_scales(ci, i, lin.N, lin.K)[:n_rows]
            host.append((rng_codes, scales, synth.activations(ci, i, Md, lin.K, verify=False),
                         synth.activations(ci, i, Mv, lin.K, verify=True)))
        done = [0] * len(lins)          # columns done per layer (counted on through repeats of the sampled rows)
        c0 = time.perf_counter()
        quantised = {}
        bytes_done = 0.0
        while time.perf_counter() - c0 < budget_s:
            for i, lin in enumerate(lins):
                codes, scales, hxd, hxv = host[i]
                if i not in quantised:
                    quantised[i] = orc.quant_act(hxd)
                    bytes_done += alg_bytes_quant(Md, lin.K)
                q, s = quantised[i]
                start = done[i] % (codes.shape[0] - codes.shape[0] % chunk or codes.shape[0])
                cols = np.arange(start, min(start + chunk, codes.shape[0]))
                orc.gemm_w4a4_columns(q, s, codes, scales, cols)
                orc.gemm_w4a16_columns(hxv, codes, scales, cols)
                done[i] += len(cols)
                bytes_done += len(cols) / lin.N * (alg_bytes_w4a4(Md, lin.N, lin.K) + alg_bytes_w4a16(Mv, lin.N, lin.K))
                if time.perf_counter() - c0 >= budget_s:
                    break
        c_t = time.perf_counter() - c0
        return dict(value=round(bytes_done / c_t / 1e12, 6), unit="TB/s", cores=int(cores), kind="oracle",
                    sample=f"{', '.join(str(d) for d in done)} output columns (chunks of {chunk}) of the "
                           f"{len(lins)} layer(s) of one decoder block (quantiser + draft product at M={Md}, verify "
                           f"product at M={Mv}), {c_t:.1f} s of the NumPy float64 oracle on BLAS threads",
                    seconds=round(c_t, 2))


def main() -> int:
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=20)
    ap.add_argument("--warmup", type=int, default=5)
    ap.add_argument("--layers", type=int, default=0,
                    help="decoder blocks with distinct weights per step (default: 32 for configs 1-3, 8 for 4, 4 for 5; "
                         "always far more packed weights than the 256 MB last-level cache holds)")
    ap.add_argument("--configs", type=str, default="1,2,3,4,5", help="workload configurations to measure")
    ap.add_argument("--config", type=int, default=0, help="measure this configuration only (it is then the headline)")
    ap.add_argument("--headline", type=int, default=5, help="the configuration whose step is the top-level value")
    ap.add_argument("--no-graph", action="store_true", help="launch eagerly instead of replaying HIP graphs")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--vendor-context", action="store_true",
                    help="also time torch.matmul (the vendor library's plain fp16 GEMM, fp16 weights, no quantisation) "
                         "on the verify-mode shapes: a yardstick for what the machine sustains, not a target")
    ap.add_argument("--prefill", action="store_true",
                    help="also time both modes at 1024 and 2048 tokens (prefill-sized M) in extra_rows_M256_M512")
    ap.add_argument("--no-extra", action="store_true",
                    help="the steps and per-call timings only (profiling runs: the extra rows' launches would mix "
                         "into the kernel statistics)")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build runs on ONE GPU only (no collectives, no sharding); "
              "run with --gpus 1", file=sys.stderr)
        return 2

    import torch

    from paper_2410_11305_amd import binding as B

    if not torch.cuda.is_available():
        print("bench.py: no GPU visible", file=sys.stderr)
        return 3
    B.lib()
    torch.cuda.set_device(0)
    bench = Bench(args)
    todo = [args.config] if args.config else sorted({int(c) for c in args.configs.split(",")})
    headline = args.config or (args.headline if args.headline in todo else todo[-1])

    # one plain device copy of known size (256 MiB read + 256 MiB written): the reference
    # point that scales the FETCH_SIZE / WRITE_SIZE counters in the profile summaries
    cal_src = torch.empty(256 << 20, dtype=torch.uint8, device=bench.dev)
    cal_dst = torch.empty_like(cal_src)
    cal_dst.copy_(cal_src)
    torch.cuda.synchronize()
    del cal_src, cal_dst

    ceilings = None
    if not args.no_extra:
        ceilings = bench.machine_ceilings()
    results = {}
    for ci in todo:
        extras = {}
        if not args.no_extra:
            extras["stream_read"] = True
            extras["rows_256_512"] = ci in (2, 5) or len(todo) == 1
            extras["vendor"] = args.vendor_context
            extras["after_verify"] = ci == headline or ci == 2
            extras["fused_producers"] = ci == headline or ci == 2
        extras["cpu_seconds"] = 12.0 if ci == headline else 2.5
        results[ci] = bench.run_config(ci, extras)
    if ceilings is not None:
        ceilings["bare_read_of_packed_weights"] = {str(ci): r.pop("bare_read") for ci, r in results.items() if "bare_read" in r}

    h = results[headline]
    out = {
        "metric": "W4A4 & W4A16 GEMM us/call, achieved HBM TB/s + MFMA % at draft/verify M",
        "value": h["value"],
        "unit": "TB/s",
        "n_gpus": 1,
        "steps": args.steps,
        "warmup": args.warmup,
        "ms_per_step": h["ms_per_step"],
        "higher_is_better": True,
        "scaling": "weak",
        "vs_baseline": None,
        "dtype": "int4 weights; int8 MFMA/int32 (draft), fp16 MFMA/fp32 (verify)",
        "data": "synthetic",
        "config": {"workload": h["workload"], "layers": h["layers"], "launch": h["launch"],
                   "alg_bytes_per_step": h["alg_bytes_per_step"], "alg_flops_per_step": h["alg_flops_per_step"],
                   "measured_configs": todo},
        "roofline": h["roofline"],
        "cpu_baseline": h["cpu_baseline"],
        "pack_weights_GBps": round(bench.pack_bytes / bench.t_pack / 1e9, 1) if bench.t_pack > 0 else None,
        "ceilings": ceilings,
        "configs": {str(ci): r for ci, r in results.items()},
    }
    print(json.dumps(out))
    return 0


if __name__ == "__main__":
    sys.exit(main())
