#!/usr/bin/env python3
"""Benchmark of the W4A4 MXFP4 linear hot path on one MI355X.

One "step" is one pass of the whole online path, batq_linear = fused transform + clip +
MXFP4 quantise of the activations followed by the MXFP4 x MXFP4 GEMM, over one batch of
synthetic activations that is already resident in HBM.  Prints ONE JSON line.

The timed loop rotates over enough distinct (X, workspace, Y) buffer sets that the
footprint exceeds twice the 256 MB last-level cache, so the activation kernel is
measured against HBM and not against the cache.

Method: after the warm-up, the loop of --steps steps is timed --repeats times (each repeat
bracketed by a device synchronisation); ms_per_step and value are the median repeat, the
fastest and slowest are reported beside it.  Kernel durations come from HIP events on the
launch stream around --steps launches of the kernel alone, again the median of the repeats.
The shader clock and board power the tool `rocm-smi` shows while the step loop runs are
recorded in `clock_state` (the matrix kernels run at the board's power limit, so the clock
explains most of the spread between boxes and runs).
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

PEAK_FP4_TFLOPS = 10100.0    # MI355X dense MXFP4 MFMA
PEAK_FP8_TFLOPS = 5000.0     # MI355X dense FP8 MFMA: the rate of a block-scaled instruction with an 8-bit operand
PEAK_HBM_GBS = 8000.0        # MI355X HBM3E


def _die(msg: str, code: int = 2):
    print(msg, file=sys.stderr)
    sys.exit(code)


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=200)
    ap.add_argument("--warmup", type=int, default=20)
    ap.add_argument("--workload", type=int, default=2, choices=[0, 1, 2, 3, 4],
                    help="which synthetic configuration is the timed workload (default: 8B-class prefill up/gate)")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--repeats", type=int, default=5, help="timed repeats of the --steps loop; the median is reported")
    ap.add_argument("--also", type=str, default="0,1,3,4",
                    help="comma list of other configs to time briefly ('' = none); all five are in the line by default")
    ap.add_argument("--no-clock-state", action="store_true", help="do not call rocm-smi")
    ap.add_argument("--no-w4a8", action="store_true", help="skip the W4A8 side measurement")
    ap.add_argument("--no-two-streams", action="store_true",
                    help="skip the two-stream side measurement (its overlapping kernels distort a kernel trace)")
    ap.add_argument("--no-kv", action="store_true", help="skip the key/value-cache side measurement")
    ap.add_argument("--no-mlp", action="store_true", help="skip the MLP-block side measurement (gate/up, SwiGLU, down)")
    ap.add_argument("--no-gemm-over-m", action="store_true",
                    help="skip the GEMM-time-over-token-count table (16 to 1024 rows on the two headline weight shapes)")
    ap.add_argument("--no-ceilings", action="store_true", help="skip the measured-ceiling tool (register-only MFMA "
                    "loop, streaming HBM kernels)")
    args = ap.parse_args()
    if args.gpus != 1 or int(os.environ.get("WORLD_SIZE", "1")) != 1:
        _die("bench.py: this build runs on ONE GPU only (no collectives, no sharding); run with --gpus 1")

    import numpy as np
    import torch

    import batq_inputs as bi
    import paper_2603_16590_amd as B

    if not torch.cuda.is_available():
        _die("bench.py: no GPU visible; the HIP path has no CPU fallback")
    torch.cuda.set_device(0)

    def to_dev(a, dtype):
        if dtype == "bf16":
            return torch.from_numpy(np.ascontiguousarray(a).view(np.int16)).view(torch.bfloat16).cuda()
        return torch.from_numpy(np.ascontiguousarray(a, dtype=np.float32)).cuda()

    def run_config(cfg: int, steps: int, warmup: int, a8: bool = False, repeats: int = 5, rotate_weights: bool = True):
        # a8: the W4A8 variant of the same layer (MXFP8 activations, same MXFP4 weights)
        linear = B.batq_linear_a8w4 if a8 else B.batq_linear
        quantize = B.batq_quantize_act_mxfp8 if a8 else B.batq_quantize_act
        gemm = B.batq_gemm_a8w4 if a8 else B.batq_gemm_mxfp4
        w = bi.make_workload(cfg)
        t = B.Transform(w.K, w.G, w.P, w.clip)
        wh = B.batq_prepare_weight(t, to_dev(w.W, w.dtype))
        ydt = torch.bfloat16 if w.out_dtype == "bf16" else torch.float32
        xbytes = 2 if w.dtype == "bf16" else 4
        ybytes = 2 if w.out_dtype == "bf16" else 4
        # workspace of a step: codes, scales and (shapes that want them) the partial sums of the GEMM's K parts
        wsz = B.batq_linear_workspace_for(wh, w.M, 8 if a8 else 4)
        per_set = w.M * w.K * xbytes + wsz + w.M * w.N * ybytes
        nsets = max(2, min(64, -(-(600 << 20) // per_set)))
        X0 = to_dev(w.X, w.dtype)
        Xs = [X0] + [X0.clone() for _ in range(nsets - 1)]
        Ws = [torch.empty(max(wsz, 16), dtype=torch.uint8, device="cuda") for _ in range(nsets)]
        Ys = [torch.empty((w.M, w.N), dtype=ydt, device="cuda") for _ in range(nsets)]
        cb = B.batq_code8_bytes(w.M, w.K) if a8 else B.batq_code_bytes(w.M, w.K)
        sb = B.batq_scale_bytes(w.M, w.K)
        parts_at = -(-(cb + sb) // 256) * 256
        codes = [wk[:cb] for wk in Ws]
        scales = [wk[cb: cb + sb] for wk in Ws]

        def step(i):
            j = i % nsets
            linear(t, wh, Xs[j], Y=Ys[j], workspace=Ws[j])

        def median(v):
            v = sorted(v)
            return v[len(v) // 2] if len(v) % 2 else 0.5 * (v[len(v) // 2 - 1] + v[len(v) // 2])

        for i in range(warmup):
            step(i)
        step_ms = []
        for _ in range(repeats):
            torch.cuda.synchronize()
            t0 = time.perf_counter()
            for i in range(steps):
                step(i)
            torch.cuda.synchronize()
            step_ms.append((time.perf_counter() - t0) * 1e3 / steps)
        ms_step = median(step_ms)

        # the same steps handed to two streams in turn (independent batches, as a server with more than one
        # request in flight would): the tail of one step's GEMM overlaps with the head of the next step
        ms_step_two = None
        if not args.no_two_streams:
            two = [torch.cuda.Stream(), torch.cuda.Stream()]
            for i in range(warmup):
                with torch.cuda.stream(two[i & 1]):
                    step(i)
            two_ms = []
            for _ in range(repeats):
                torch.cuda.synchronize()
                t0 = time.perf_counter()
                for i in range(steps):
                    with torch.cuda.stream(two[i & 1]):
                        step(i)
                torch.cuda.synchronize()
                two_ms.append((time.perf_counter() - t0) * 1e3 / steps)
            ms_step_two = median(two_ms)

        # per-kernel durations: HIP events on the stream the kernels are launched on, median of the repeats
        def timed(fn, n):
            for i in range(min(warmup, 10)):
                fn(i)
            out = []
            for _ in range(repeats):
                e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
                torch.cuda.synchronize()
                e0.record()
                for i in range(n):
                    fn(i)
                e1.record()
                e1.synchronize()
                out.append(e0.elapsed_time(e1) / n)
            return median(out), min(out), max(out)

        # the quantiser alone touches only X and the codes: rotate over enough sets of those that their footprint
        # exceeds twice the 256 MB memory-side cache
        nq = max(nsets, min(64, -(-(600 << 20) // (w.M * w.K * xbytes + wsz))))
        for _ in range(nq - nsets):
            Xs.append(X0.clone())
            Ws.append(torch.empty(max(wsz, 16), dtype=torch.uint8, device="cuda"))
        qcodes = [wk[:cb] for wk in Ws]
        qscales = [wk[cb: cb + sb] for wk in Ws]
        parts = [wk[parts_at:] if wk.numel() > parts_at else None for wk in Ws]
        ms_quant, ms_quant_min, ms_quant_max = timed(lambda i: quantize(t, Xs[i % nq], qcodes[i % nq], qscales[i % nq]), steps)
        ms_gemm, ms_gemm_min, ms_gemm_max = timed(
            lambda i: gemm(codes[i % nsets], scales[i % nsets], wh, w.M, Y=Ys[i % nsets], workspace=parts[i % nsets]), steps)
        ms_quant_warm, _, _ = timed(lambda i: quantize(t, Xs[0], codes[0], scales[0]), steps)
        # the GEMM with the weights coming from HBM: enough copies of the prepared weight taking turns that their
        # footprint exceeds the 256 MB memory-side cache (the figure above re-reads one weight, which stays in it)
        wbytes = w.K * w.N * (0.5 + 1.0 / 32)
        nw = max(10, -(-(300 << 20) // int(wbytes))) if rotate_weights else 0
        ms_gemm_rot = None
        if nw:
            wcodes, wscales = wh.export()
            whs = [wh] + [B.batq_weight_import(wcodes, wscales, w.K, w.N) for _ in range(nw - 1)]
            del wcodes, wscales
            ms_gemm_rot, _, _ = timed(
                lambda i: gemm(codes[i % nsets], scales[i % nsets], whs[i % nw], w.M, Y=Ys[i % nsets],
                               workspace=parts[i % nsets]), steps)
            del whs

        flops = 2.0 * w.M * w.K * w.N
        qbytes = w.M * w.K * (xbytes + (1.0 if a8 else 0.5) + 1.0 / 32)
        res = {
            "workload": f"cfg{cfg}:{w.name} M={w.M} K={w.K} N={w.N} x={w.dtype} y={w.out_dtype}",
            "ms_per_step": ms_step, "ms_per_step_min": min(step_ms), "ms_per_step_max": max(step_ms),
            "repeats": repeats, "steps_per_repeat": steps,
            "linear_tflops": flops / ms_step / 1e9,
            "ms_per_step_two_streams": ms_step_two,
            "linear_tflops_two_streams": flops / ms_step_two / 1e9 if ms_step_two else None,
            "quant_ms": ms_quant, "quant_gbs": qbytes / ms_quant / 1e6,
            "quant_gbs_cache_warm": qbytes / ms_quant_warm / 1e6,
            "quant_ms_min": ms_quant_min, "quant_ms_max": ms_quant_max,
            "gemm_ms": ms_gemm, "gemm_ms_min": ms_gemm_min, "gemm_ms_max": ms_gemm_max,
            "gemm_tflops": flops / ms_gemm / 1e9,
            "gemm_ms_rotating_weights": ms_gemm_rot, "weight_copies": nw,
            "gemm_tflops_rotating_weights": flops / ms_gemm_rot / 1e9 if ms_gemm_rot else None,
            "gemm_frac_of_fp4_peak": flops / ms_gemm / 1e9 / PEAK_FP4_TFLOPS,
            "quant_frac_of_hbm_peak": qbytes / ms_quant / 1e6 / PEAK_HBM_GBS,
            "buffer_sets": nsets, "quant_buffer_sets": nq,
        }
        return w, t, wh, res, flops, qbytes

    w, t, wh, res, flops, qbytes = run_config(args.workload, args.steps, args.warmup, repeats=args.repeats)

    # the dominant kernel of the step decides which roofline is reported first
    gemm_dominant = res["gemm_ms"] >= res["quant_ms"]
    roof_gemm = {"kernel": "gemm_tiled", "bound": "mfma", "achieved": res["gemm_tflops"], "peak": PEAK_FP4_TFLOPS,
                 "unit": "TFLOP/s", "frac": res["gemm_tflops"] / PEAK_FP4_TFLOPS, "traffic": None}
    roof_quant = {"kernel": "quant_act_mfma", "bound": "hbm", "achieved": res["quant_gbs"], "peak": PEAK_HBM_GBS,
                  "unit": "GB/s", "frac": res["quant_gbs"] / PEAK_HBM_GBS, "traffic": None}
    # HBM traffic per launch is not measured in this run: it comes from the stored rocprofv3 --pmc profile
    # (FETCH_SIZE / WRITE_SIZE, calibrated on a copy kernel), whose file says which commit it was taken at
    traffic_file = os.path.join(ROOT, "profiles", "pmc_traffic.json")
    traffic_source = None
    if os.path.exists(traffic_file):
        try:
            stored = json.load(open(traffic_file))
            tr = stored.get(f"cfg{args.workload}", {})
            roof_gemm["traffic"] = tr.get("gemm_tiled")
            roof_quant["traffic"] = tr.get("quant_act_mfma")
            traffic_source = {"file": "profiles/pmc_traffic.json", "kind": "stored rocprofv3 --pmc profile, not this run",
                              "measured_at_commit": stored.get("measured_at_commit")}
        except Exception:
            pass
    roof_gemm["traffic_source"] = roof_quant["traffic_source"] = traffic_source
    roof_gemm.update({"ms": res["gemm_ms"], "ms_min": res["gemm_ms_min"], "ms_max": res["gemm_ms_max"],
                      "achieved_rotating_weights": res["gemm_tflops_rotating_weights"]})
    roof_quant.update({"ms": res["quant_ms"], "ms_min": res["quant_ms_min"], "ms_max": res["quant_ms_max"]})

    # Shader clock and board power while the step loop runs (rocm-smi is slow, so half a second of steps is
    # queued first); best effort: the headline numbers do not depend on it.
    clock_state = None
    if not args.no_clock_state:
        import re
        import shutil
        import subprocess
        smi = shutil.which("rocm-smi") or "/opt/rocm/bin/rocm-smi"
        try:
            Xc = to_dev(w.X, w.dtype)
            Yc = torch.empty((w.M, w.N), dtype=torch.bfloat16 if w.out_dtype == "bf16" else torch.float32, device="cuda")
            wk = torch.empty(max(B.batq_linear_workspace_for(wh, w.M), 16), dtype=torch.uint8, device="cuda")
            for _ in range(int(0.6 / max(res["ms_per_step"] * 1e-3, 1e-6))):
                B.batq_linear(t, wh, Xc, Y=Yc, workspace=wk)
            out = subprocess.run([smi, "-d", "0", "--showclocks", "--showpower", "--showmaxpower", "--showtemp"],
                                 capture_output=True, text=True, timeout=30).stdout
            torch.cuda.synchronize()
            def grab(pat):
                m = re.search(pat, out)
                return m.group(1) if m else None
            clock_state = {
                "source": "rocm-smi while the step loop runs",
                "sclk": grab(r"sclk clock level[^\n]*?\((\d+Mhz)\)"),
                "mclk": grab(r"mclk clock level[^\n]*?\((\d+Mhz)\)"),
                "power_w": grab(r"Graphics Package Power \(W\):\s*([\d.]+)") or grab(r"Power \(W\):\s*([\d.]+)"),
                "power_cap_w": grab(r"Max Graphics Package Power \(W\):\s*([\d.]+)"),
                "junction_temp_c": grab(r"Temperature \(Sensor junction\) \(C\):\s*([\d.]+)"),
            }
            del Xc, Yc, wk
        except Exception as e:
            clock_state = {"error": str(e)}

    # Small-M shapes (cfg0: 64 tokens, cfg1: 16 tokens, the decode shape): the GEMM is one pass over the weight
    # codes, so it is reported as a streaming rate over the weight's codes and scales, with enough copies of the
    # weight taking turns to exceed the memory-side cache (at least 32).  The kernels take a few microseconds, less
    # than a launch from Python, so they are timed as replays of a captured graph of one call per weight copy.
    def small_config(cfg: int):
        w1 = bi.make_workload(cfg)
        t1_ = B.Transform(w1.K, w1.G, w1.P, w1.clip)
        Wd1 = to_dev(w1.W, w1.dtype)
        wbytes = w1.K * w1.N * (0.5 + 1.0 / 32)
        ncopy = max(32, min(512, -(-(300 << 20) // int(wbytes))))
        first = B.batq_prepare_weight(t1_, Wd1)
        wcodes, wscales = first.export()
        whs = [first] + [B.batq_weight_import(wcodes, wscales, w1.K, w1.N) for _ in range(ncopy - 1)]
        X1 = to_dev(w1.X, w1.dtype)
        ws1_ = torch.empty(max(B.batq_linear_workspace_for(first, w1.M), 16), dtype=torch.uint8, device="cuda")
        cb1, sb1 = B.batq_code_bytes(w1.M, w1.K), B.batq_scale_bytes(w1.M, w1.K)
        pa1 = -(-(cb1 + sb1) // 256) * 256
        parts1 = ws1_[pa1:] if ws1_.numel() > pa1 else None
        ydt = torch.bfloat16 if w1.out_dtype == "bf16" else torch.float32
        Y1 = torch.empty((w1.M, w1.N), dtype=ydt, device="cuda")
        side = torch.cuda.Stream()

        def graph_us(fn):
            with torch.cuda.stream(side):
                for i in range(ncopy):
                    fn(i)
            side.synchronize()
            gr = torch.cuda.CUDAGraph()
            with torch.cuda.graph(gr, stream=side):
                for i in range(ncopy):
                    fn(i)
            gr.replay()
            torch.cuda.synchronize()
            out = []
            for _ in range(args.repeats):
                e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
                e0.record()
                for _ in range(4):
                    gr.replay()
                e1.record()
                e1.synchronize()
                out.append(e0.elapsed_time(e1) / (4 * ncopy) * 1e3)
            return sorted(out)[len(out) // 2]

        us_lin = graph_us(lambda i: B.batq_linear(t1_, whs[i], X1, Y=Y1, workspace=ws1_))
        us_q = graph_us(lambda i: B.batq_quantize_act(t1_, X1, ws1_[:cb1], ws1_[cb1:cb1 + sb1]))
        us_g = graph_us(lambda i: B.batq_gemm_mxfp4(ws1_[:cb1], ws1_[cb1:cb1 + sb1], whs[i], w1.M, Y=Y1, workspace=parts1))
        xb = 2 if w1.dtype == "bf16" else 4
        res1 = {"workload": f"cfg{cfg}:{w1.name} M={w1.M} K={w1.K} N={w1.N} x={w1.dtype} y={w1.out_dtype}",
                "linear_us": us_lin, "linear_tflops": 2.0 * w1.M * w1.K * w1.N / us_lin / 1e6,
                "quant_us": us_q, "quant_gbs": w1.M * w1.K * (xb + 0.5 + 1.0 / 32) / us_q / 1e3,
                "gemm_us": us_g, "gemm_weight_stream_gbs": wbytes / us_g / 1e3,
                "gemm_frac_of_hbm_peak": wbytes / us_g / 1e3 / PEAK_HBM_GBS, "weight_copies": ncopy,
                "note": "graph replays of one call per weight copy (launch gaps between dependent kernels included), "
                        "median of the repeats; the GEMM streams the weight once, so it is rated in GB/s over the "
                        "weight codes and scales"}
        del whs, Wd1, first, wcodes, wscales
        torch.cuda.empty_cache()
        return res1

    also = {}
    for c in [int(x) for x in args.also.split(",") if x.strip() != ""]:
        if c == args.workload:
            continue
        if c in (0, 1):
            also[f"cfg{c}"] = small_config(c)
            continue
        _, _, _, r, _, _ = run_config(c, max(10, args.steps // 4), max(3, args.warmup // 4), repeats=args.repeats)
        also[f"cfg{c}"] = r
        torch.cuda.empty_cache()

    # the W4A8 variant of the same workload (MXFP8 activations): its matrix instructions run at the FP8 rate
    w4a8 = None
    if not args.no_w4a8:
        _, _, _, r8, _, _ = run_config(args.workload, max(10, args.steps // 4), max(3, args.warmup // 4), a8=True,
                                       repeats=args.repeats, rotate_weights=False)
        r8["gemm_frac_of_fp8_rate_peak"] = r8["gemm_tflops"] / PEAK_FP8_TFLOPS
        r8["quant_frac_of_hbm_peak"] = r8["quant_gbs"] / PEAK_HBM_GBS
        w4a8 = r8
        torch.cuda.empty_cache()

    # The MLP block the two headline shapes come from (hidden 4096, intermediate 14336; cfg2 = gate/up, cfg3 =
    # down): P_up quantise -> gate/up GEMM -> silu(gate) * up -> P_down quantise -> down GEMM, with the gated
    # activation (a) left to a separate elementwise pass, (b) fused into the down projection's quantiser,
    # (c) fused into the gate/up GEMM's epilogue.  Side measurement; the headline value is the single layer.
    mlp = None
    if not args.no_mlp and args.workload in (2, 3):
        Mm, D, Fh = 2048, 4096, 14336
        rng = np.random.default_rng(7)

        def mk(K):
            nbk = K // 32
            G = (np.eye(4) + 0.05 * rng.standard_normal((4, 4))).astype(np.float32)
            P = (np.eye(8)[None] + 0.05 * rng.standard_normal((nbk, 8, 8))).astype(np.float32)
            return B.Transform(K, G, P, rng.uniform(0.85, 1.0, nbk).astype(np.float32))

        t_up, t_down = mk(D), mk(Fh)
        gen = torch.Generator(device="cuda")
        gen.manual_seed(7)
        Wg = (torch.randn((D, Fh), device="cuda", generator=gen) * 0.02).to(torch.bfloat16)
        Wu = (torch.randn((D, Fh), device="cuda", generator=gen) * 0.02).to(torch.bfloat16)
        Wd = (torch.randn((Fh, D), device="cuda", generator=gen) * 0.02).to(torch.bfloat16)
        w_gu = B.batq_prepare_weight_gate_up(t_up, Wg, Wu)
        w_d = B.batq_prepare_weight(t_down, Wd)
        del Wg, Wu, Wd
        Xm = torch.randn((Mm, D), device="cuda", generator=gen).to(torch.bfloat16)
        ws1 = torch.empty(B.batq_linear_workspace_for(w_gu, Mm), dtype=torch.uint8, device="cuda")
        ws2 = torch.empty(B.batq_linear_workspace_for(w_d, Mm), dtype=torch.uint8, device="cuda")
        GU = torch.empty((Mm, 2 * Fh), dtype=torch.bfloat16, device="cuda")
        Hh = torch.empty((Mm, Fh), dtype=torch.bfloat16, device="cuda")
        Ym = torch.empty((Mm, D), dtype=torch.bfloat16, device="cuda")
        # in the interleaved weight gate and up alternate in groups of 32 columns: views for the unfused chains
        GU3 = GU.view(Mm, Fh // 32, 2, 32)

        def chain_separate():
            B.batq_linear(t_up, w_gu, Xm, Y=GU, workspace=ws1)
            torch.mul(torch.nn.functional.silu(GU3[:, :, 0, :]), GU3[:, :, 1, :], out=Hh.view(Mm, Fh // 32, 32))
            B.batq_linear(t_down, w_d, Hh, Y=Ym, workspace=ws2)

        def chain_epilogue():
            B.batq_linear_glu(t_up, w_gu, Xm, H=Hh, workspace=ws1)
            B.batq_linear(t_down, w_d, Hh, Y=Ym, workspace=ws2)

        def time_chain(fn, n=20):
            for _ in range(3):
                fn()
            torch.cuda.synchronize()
            e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            e0.record()
            for _ in range(n):
                fn()
            e1.record()
            e1.synchronize()
            return e0.elapsed_time(e1) / n

        ms_sep, ms_epi = time_chain(chain_separate), time_chain(chain_epilogue)
        mlp = {"shape": f"{Mm} tokens, hidden {D}, intermediate {Fh}", "flops": 6.0 * Mm * D * Fh,
               "ms_separate_activation_pass": ms_sep, "ms_gated_epilogue": ms_epi,
               "tflops_gated_epilogue": 6.0 * Mm * D * Fh / ms_epi / 1e9}
        del w_gu, w_d, GU, Hh, Ym, ws1, ws2, Xm
        torch.cuda.empty_cache()

    # Key/value-cache helpers (Sec. 3.2): a cache of 32768 tokens x 8 heads x 128 channels written by the
    # quantiser (KV4 and KV8) and read back as bf16, and the query-side transform at the headline token count.
    # Rates are algorithmic bytes (input + output of the call) over the time per call, 20 calls back to back
    # (sizes at which a kernel outlasts the issue of the next call from Python).
    kv = None
    if not args.no_kv:
        Mk, Kk, Mq, Kq = 32768, 1024, 8192, 4096
        rk = np.random.default_rng(77)
        Gk, Pk, ck = bi.make_factors(Kk // 32, rk, rk, rk, 0.7)
        Gq, Pq, _ = bi.make_factors(Kq // 32, rk, rk, rk, 0.7)
        tk, tq = B.Transform(Kk, Gk, Pk, ck), B.Transform(Kq, Gq, Pq, None)
        Xk = torch.randn((Mk, Kk), device="cuda").to(torch.bfloat16)
        Xq = torch.randn((Mq, Kq), device="cuda").to(torch.bfloat16)
        Ok = torch.empty_like(Xk)
        Oq = torch.empty_like(Xq)

        def per_call_us(fn, n=20):
            for _ in range(3):
                fn()
            torch.cuda.synchronize()
            best = None
            for _ in range(3):
                e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
                e0.record()
                for _ in range(n):
                    fn()
                e1.record()
                e1.synchronize()
                us = e0.elapsed_time(e1) / n * 1e3
                best = us if best is None else min(best, us)
            return best

        kv = {"cache": f"{Mk} tokens x {Kk} channels (8 heads x 128), bf16 in / out", "query": f"{Mq} x {Kq} bf16"}
        for bits in (4, 8):
            cbytes = Mk * Kk * ((0.5 if bits == 4 else 1.0) + 1.0 / 32)
            kc = torch.empty(B.batq_code8_bytes(Mk, Kk) if bits == 8 else B.batq_code_bytes(Mk, Kk), dtype=torch.uint8,
                             device="cuda")
            ksc = torch.empty(B.batq_scale_bytes(Mk, Kk), dtype=torch.uint8, device="cuda")
            if bits == 4:
                us_w = per_call_us(lambda: B.batq_quantize_act(tk, Xk, kc, ksc))
            else:
                kc, ksc = B.batq_quantize_act_ex(tk, Xk, act_bits=8)
                us_w = per_call_us(lambda: B.batq_quantize_act_ex(tk, Xk, act_bits=8))
            us_r = per_call_us(lambda: B.batq_dequantize(kc, ksc, Mk, Kk, bits, out=Ok))
            kv[f"kv{bits}"] = {"quantize_us": us_w, "quantize_gbs": (Mk * Kk * 2 + cbytes) / us_w / 1e3,
                               "dequantize_us": us_r, "dequantize_gbs": (Mk * Kk * 2 + cbytes) / us_r / 1e3}
        us_a = per_call_us(lambda: B.batq_transform_apply(tq, Xq, B.APPLY_INVERSE_T, out=Oq))
        us_ak = per_call_us(lambda: B.batq_transform_apply(tk, Xk, B.APPLY_INVERSE, out=Ok))
        kv["apply_inverse_t_query_us"] = us_a
        kv["apply_inverse_t_query_gbs"] = Mq * Kq * 4 / us_a / 1e3
        kv["apply_inverse_cache_shape_us"] = us_ak
        kv["apply_inverse_cache_shape_gbs"] = Mk * Kk * 4 / us_ak / 1e3
        del Xk, Xq, Ok, Oq
        torch.cuda.empty_cache()

    # GEMM time over the token count M on the two headline weight shapes, weights in HBM: 20 copies of the weight
    # take turns, the 20 calls are replayed as one captured graph (so the gaps between dependent launches are in the
    # figure), each call with the workspace batq_gemm_workspace() asks for.  One pass over the weight's codes and
    # scales at the measured read ceiling is the floor for small M.
    over_m = None
    if not args.no_gemm_over_m:
        over_m = {"note": "us per GEMM call, graph replays of 20 calls over 20 weight copies, median of the repeats; "
                          "weight_stream_us = weight codes and scales / 5.5 TB/s", "shapes": {}}
        gen = torch.Generator(device="cuda")
        gen.manual_seed(11)
        side = torch.cuda.Stream()
        for Kw, Nw in ((4096, 14336), (14336, 4096)):
            nbw = Kw // 32
            rw = np.random.default_rng(Kw)
            Gw, Pw, cw = bi.make_factors(nbw, rw, rw, rw, 0.85)
            tw = B.Transform(Kw, Gw, Pw, cw)
            first = B.batq_prepare_weight(tw, (torch.randn((Kw, Nw), device="cuda", generator=gen) * 0.02).to(torch.bfloat16))
            wcodes, wscales = first.export()
            whs = [first] + [B.batq_weight_import(wcodes, wscales, Kw, Nw) for _ in range(19)]
            row = {}
            for Mw in (16, 64, 128, 256, 512, 1024):
                Xw = torch.randn((Mw, Kw), device="cuda", generator=gen).to(torch.bfloat16)
                xc_ = torch.empty(B.batq_code_bytes(Mw, Kw), dtype=torch.uint8, device="cuda")
                xs_ = torch.empty(B.batq_scale_bytes(Mw, Kw), dtype=torch.uint8, device="cuda")
                B.batq_quantize_act(tw, Xw, xc_, xs_)
                need = B.batq_gemm_workspace(first, Mw)
                work = torch.empty(need, dtype=torch.uint8, device="cuda") if need else None
                Yw = torch.empty((Mw, Nw), dtype=torch.bfloat16, device="cuda")
                with torch.cuda.stream(side):
                    for i in range(20):
                        B.batq_gemm_mxfp4(xc_, xs_, whs[i], Mw, Y=Yw, workspace=work)
                side.synchronize()
                gr = torch.cuda.CUDAGraph()
                with torch.cuda.graph(gr, stream=side):
                    for i in range(20):
                        B.batq_gemm_mxfp4(xc_, xs_, whs[i], Mw, Y=Yw, workspace=work)
                gr.replay()
                torch.cuda.synchronize()
                out = []
                for _ in range(args.repeats):
                    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
                    e0.record()
                    for _ in range(10):
                        gr.replay()
                    e1.record()
                    e1.synchronize()
                    out.append(e0.elapsed_time(e1) / 200 * 1e3)
                row[str(Mw)] = sorted(out)[len(out) // 2]
                del gr
            over_m["shapes"][f"K={Kw} N={Nw}"] = {"us": row, "weight_stream_us": Kw * Nw * (0.5 + 1.0 / 32) / 5.5e6}
            del whs, first, wcodes, wscales
            torch.cuda.empty_cache()

    ceilings = None
    tool = os.path.join(ROOT, "paper_2603_16590_amd", "batq_ceilings")
    if not args.no_ceilings and os.path.exists(tool):
        import subprocess
        torch.cuda.synchronize()
        try:
            out = subprocess.run([tool], capture_output=True, text=True, timeout=120)
            ceilings = json.loads(out.stdout.strip().splitlines()[-1])
        except Exception as e:  # the headline numbers do not depend on it
            ceilings = {"error": str(e)}

    cpu = None
    if not args.no_cpu_baseline:
        from oracle import batq_oracle as o
        # bounded sample: at most 2048 rows x 16384 output columns (the whole of cfg2), a few
        # seconds to tens of seconds of oracle work on the host cores
        ms_rows = min(w.M, 2048)
        ns_cols = min(w.N, 16384)
        Xs_ = w.X_f32()[:ms_rows]
        Wc, Wsc = o.prepare_weight(w.W_f32()[:, :ns_cols], w.G, w.P)          # offline, not timed
        # repeated until about ten seconds of oracle work have been timed
        t_quant = t_total = 0.0
        reps = 0
        while t_total < 10.0 and reps < 50:
            c0 = time.perf_counter()
            xc, xs = o.quantize_act(Xs_, w.G, w.P, w.clip)
            c1 = time.perf_counter()
            o.gemm(xc, xs, Wc, Wsc)
            c2 = time.perf_counter()
            t_quant += c1 - c0
            t_total += c2 - c0
            reps += 1
        try:
            from threadpoolctl import threadpool_info
            blas_threads = max([p.get("num_threads", 1) for p in threadpool_info()] or [1])
        except Exception:
            blas_threads = len(os.sched_getaffinity(0))
        cpu = {
            "value": reps * 2.0 * ms_rows * w.K * ns_cols / t_total / 1e12, "unit": "TFLOP/s",
            "cores": int(min(blas_threads, len(os.sched_getaffinity(0)))), "kind": "oracle",
            "sample": f"{ms_rows} rows x {ns_cols} output columns of the same workload "
                      f"(oracle quantize_act + fp64 dequantise/matmul; weights prepared beforehand), "
                      f"{reps} passes",
            "quant_gbs": ms_rows * w.K * ((2 if w.dtype == 'bf16' else 4) + 0.5 + 1 / 32) * reps / t_quant / 1e9,
            "seconds": t_total,
        }

    line = {
        "metric": "W4A4 MXFP4 linear TFLOP/s incl. online transform+quantize",
        "value": res["linear_tflops"], "unit": "TFLOP/s",
        "n_gpus": 1, "steps": args.steps, "warmup": args.warmup, "ms_per_step": res["ms_per_step"],
        "repeats": args.repeats, "ms_per_step_min": res["ms_per_step_min"], "ms_per_step_max": res["ms_per_step_max"],
        "timing": "median of `repeats` timed loops of `steps` steps each, synchronised on both sides",
        "clock_state": clock_state,
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "mxfp4 (e2m1 x e8m0), fp32 accumulate", "data": "synthetic",
        "config": {"workload": res["workload"], "block": 32, "gpk": "G4x4 (x) P8x8", "buffer_sets": res["buffer_sets"]},
        "two_streams": {"ms_per_step": res["ms_per_step_two_streams"], "value": res["linear_tflops_two_streams"],
                        "note": "same steps issued to two streams in turn; the headline value is the one-stream figure"},
        "quantize_gbs": res["quant_gbs"], "quantize_gbs_cache_warm": res["quant_gbs_cache_warm"],
        "gemm_tflops": res["gemm_tflops"], "quant_ms": res["quant_ms"], "gemm_ms": res["gemm_ms"],
        "gemm_tflops_rotating_weights": res["gemm_tflops_rotating_weights"],
        "roofline": roof_gemm if gemm_dominant else roof_quant,
        "roofline_other": roof_quant if gemm_dominant else roof_gemm,
        "measured_ceilings": ceilings,
        "cpu_baseline": cpu,
        "also": also,
        "w4a8": w4a8,
        "mlp_block": mlp,
        "gemm_over_m": over_m,
        "kv_cache": kv,
    }
    print(json.dumps(line))


if __name__ == "__main__":
    main()
