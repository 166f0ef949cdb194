#!/usr/bin/env python3
"""Benchmark of the single-GPU MoE layer hot path (forward + backward) on one MI355X.

A step is one pass of the whole path -- gate/top-k/capacity, dispatch, expert FFNs (grouped GEMM),
combine, and the full backward -- over one batch of synthetic tokens already resident in HBM.
Prints ONE JSON line: whole-job tokens/s, the roofline of the dominant kernel family (the bf16 MFMA
grouped GEMM of the experts, timed live with HIP events) and the CPU oracle timed on a bounded
sample of the same workload on the host cores.

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--workload mixtral] [--no-cpu-baseline]
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

PEAK_BF16_TFLOPS = 2500.0   # MI355X dense bf16 MFMA
PEAK_HBM_GBS = 8000.0       # MI355X HBM3E
# HBM bytes per step of the six expert-GEMM launches at the Mixtral shape, from the rocprofv3 --pmc
# FETCH_SIZE / WRITE_SIZE runs summarised in profiles/gg_mfma_kernel_mixtral_hbm_traffic.md (scaled by
# the factors a plain 1 GiB copy gives: 2.0 and 1.0).  Algorithmic bytes for the same launches: 22.3e9.
MEASURED_GEMM_TRAFFIC = {"mixtral": {"read": 67.8e9, "written": 8.1e9}}


def parse():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=10)
    ap.add_argument("--warmup", type=int, default=3)
    ap.add_argument("--workload", default="mixtral", choices=["tiny", "gpt2", "mixtral", "finegrained", "switch"])
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-breakdown", action="store_true")
    ap.add_argument("--chunks", type=int, default=0,
                    help="also time the layer run in this many chunks (moe_layer_fwd_chunked / moe_layer_bwd_chunked, "
                         "dispatch of the next chunk on a second stream); reported beside the headline figure")
    ap.add_argument("--fit-expert-model", action="store_true",
                    help="time the expert FFN on 1/r of the rows of every expert, r = 1, 2, 4, 8, 16, and fit the linear model "
                         "t = alpha + (n / r) * beta of FSMoE Sec. 4.1; reports the fit and what Algorithm 1 picks on one GPU")
    ap.add_argument("--graph", action="store_true",
                    help="also time the step replayed from a HIP graph that holds moe_layer_fwd + moe_layer_bwd (the calls allocate "
                         "nothing and never synchronise, so they can be captured); reported beside the headline figure")
    ap.add_argument("--gates", action="store_true",
                    help="also time a layer step with each of the other gates of FSMoE Sec. 2.1 at the same shape (sigmoid, noisy, "
                         "X-MoE with a 256-wide projection, expert choice with the same number of expert rows); reported "
                         "beside the headline figure, the counterpart on one GPU of the paper's comparison of gates (Table 6)")
    ap.add_argument("--no-calibrate", action="store_true",
                    help="skip the measured peaks that the line carries beside the nominal ones: the vendor library's plain bf16 "
                         "GEMM (torch.matmul, about 0.7 s per operand layout) and the bandwidth of a plain 1 GiB device copy")
    ap.add_argument("--calibrate-gemm", action="store_true", help="accepted for compatibility: the measured peaks are on by default")
    ap.add_argument("--calibrate-copy", action="store_true",
                    help="also run one plain 1 GiB device copy before the timed region (a known-size reference for rocprofv3 byte counters)")
    return ap.parse_args()


def library_gemm_reference(torch, m=32768, n=4096, k=14336, secs=0.7):
    """Sustained TFLOP/s of torch.matmul (the vendor library) in bf16 on dense products of the size of the Mixtral
    expert products with all experts merged, one per operand layout of the path:
      NN: A [m,k] . B [k,n], B row-major             (forward: xe.W1, hh.W2)
      NT: A [m,k] . W^T with W [n,k]                 (backward of the inputs: dq.W2^T, da.W1^T)
      TN: A^T . B with A [m,k'], B [m,n], k' = k     (weight gradients: hh^T.dq, contraction over the m rows)"""
    out = {}
    for name in ("NN", "NT", "TN"):
        a = torch.randn(m, k, device="cuda", dtype=torch.bfloat16)
        if name == "NN":
            b = torch.randn(k, n, device="cuda", dtype=torch.bfloat16) * 0.02
            c = torch.empty(m, n, device="cuda", dtype=torch.bfloat16)
            fn = lambda: torch.matmul(a, b, out=c)
        elif name == "NT":
            b = torch.randn(n, k, device="cuda", dtype=torch.bfloat16) * 0.02
            c = torch.empty(m, n, device="cuda", dtype=torch.bfloat16)
            bt = b.t()
            fn = lambda: torch.matmul(a, bt, out=c)
        else:
            b = torch.randn(m, n, device="cuda", dtype=torch.bfloat16)
            c = torch.empty(k, n, device="cuda", dtype=torch.bfloat16)
            at = a.t()
            fn = lambda: torch.matmul(at, b, out=c)
        fn()
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        rates = []
        while time.perf_counter() - t0 < secs:
            e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            e0.record()
            for _ in range(10):
                fn()
            e1.record()
            torch.cuda.synchronize()
            rates.append(2.0 * m * n * k * 10 / e0.elapsed_time(e1) / 1e9)
        half = rates[len(rates) // 2:]
        out[name] = round(sum(half) / len(half), 1)
        del a, b, c
    return {"what": f"torch.matmul bf16, {m} x {n} x {k} (NN, NT) and {k} x {n} x {m} (TN), sustained, TFLOP/s", **out}


def copy_bandwidth(torch, gib=1, reps=10):
    """Bandwidth of a plain device-to-device copy of `gib` GiB (bytes read + bytes written per second, GB/s): what the
    HBM sustains on this machine for the simplest streaming kernel."""
    src = torch.empty(gib << 30, dtype=torch.uint8, device="cuda").fill_(1)
    dst = torch.empty_like(src)
    dst.copy_(src)
    torch.cuda.synchronize()
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    e0.record()
    for _ in range(reps):
        dst.copy_(src)
    e1.record()
    torch.cuda.synchronize()
    ms = e0.elapsed_time(e1) / reps
    del src, dst
    return round(2.0 * (gib << 30) / ms / 1e6, 1)


def fit_expert_model(torch, cfg, w, d, b, xe, a1, a3, hh, count, timed, reps, fwd_flop):
    """FSMoE Sec. 4.1: t_exp,r = alpha_exp + (n_exp / r) * beta_exp, fitted by least squares on the measured time of
    moe_expert_ffn_fwd / _bwd over the first 1/r of the rows of every expert (n_exp in TFLOP of the whole layer)."""
    import numpy as np
    import paper_2501_10714_amd as moe
    res = {}
    rs = [1, 2, 4, 8, 16]
    for phase, flop in (("fwd", fwd_flop), ("bwd", 2 * fwd_flop)):
        ts = []
        for r in rs:
            cnt = torch.div(count, r, rounding_mode="floor")
            off = torch.zeros(w.E + 1, dtype=torch.int32, device="cuda")
            off[1:] = torch.cumsum(cnt, 0)
            if phase == "fwd":
                ts.append(timed(lambda: moe.moe_expert_ffn_fwd(cfg, xe, off, d["w1"], d["w3"], d["w2"], b.q, b.a1, b.a3, b.hh, b.ws), reps))
            else:
                ts.append(timed(lambda: moe.moe_expert_ffn_bwd(cfg, b.dq, xe, off, d["w1"], d["w3"], d["w2"], a1, a3, hh, b.dxe,
                                                               b.dw1, b.dw3, b.dw2, b.ws), reps))
        x = np.array([flop / 1e12 / r for r in rs])
        y = np.array(ts)
        beta, alpha = np.polyfit(x, y, 1)
        resid = y - (alpha + beta * x)
        m = moe.PipelineModel(0, 0, 0, 0, 0, 0, 0, 0, 0, max(alpha, 0.0), beta, flop / 1e12, 0.0)
        r_opt, t_opt, case = moe.moe_find_pipeline_degree(m, 16)
        res[phase] = {"r": rs, "ms": [round(t, 3) for t in ts], "alpha_ms": round(float(alpha), 4),
                      "beta_ms_per_tflop": round(float(beta), 4), "n_tflop": round(flop / 1e12, 3),
                      "max_abs_residual_ms": round(float(np.abs(resid).max()), 4),
                      "algorithm1_one_gpu": {"r": r_opt, "t_ms": round(t_opt, 3), "case": case}}
    return res


def device_inputs(w, torch):
    """Synthetic inputs drawn on the device (same shapes and distributions as the parity inputs)."""
    import moe_synth as S
    g = torch.Generator(device="cuda")
    g.manual_seed(1000 + w.seed)
    dt = torch.bfloat16 if w.dtype == S.DT_BF16 else torch.float32

    def normal(shape, std):
        out = torch.empty(shape, dtype=dt, device="cuda")
        flat = out.view(-1)
        step = 1 << 26
        for i in range(0, flat.numel(), step):          # chunked: no fp32 temporary of the whole tensor
            n = min(step, flat.numel() - i)
            flat[i:i + n] = (torch.randn(n, generator=g, device="cuda", dtype=torch.float32) * std).to(dt)
        return out

    d = {"x": normal((w.N, w.M), w.x_std), "dy": normal((w.N, w.M), w.x_std), "w_gate": normal((w.M, w.E), 0.02),
         "w1": normal((w.E, w.M, w.H), 0.02), "w2": normal((w.E, w.H, w.M), 0.02),
         "w3": normal((w.E, w.M, w.H), 0.02) if w.gated else None}
    bg = S.draw_b_gate(w)
    d["b_gate"] = None if bg is None else torch.from_numpy(bg).cuda()
    return d


def main():
    args = parse()
    if args.gpus != 1:
        print("bench.py: this build is the one-GPU hot path; it has no multi-GPU mode (--gpus must be 1)", file=sys.stderr)
        sys.exit(2)
    import numpy as np
    import torch
    import moe_synth as S
    import paper_2501_10714_amd as moe
    from paper_2501_10714_amd.buffers import Buffers, make_cfg   # allocation only; the oracle is loaded by cpu_baseline() alone

    moe.load()                                           # fails loudly when the HIP library is missing
    torch.cuda.set_device(0)
    w = S.WORKLOADS[args.workload]
    cfg = make_cfg(w)
    d = device_inputs(w, torch)
    b = Buffers(w, cfg)
    has_bias = d["b_gate"] is not None

    def fwd():
        moe.moe_layer_fwd(cfg, d["x"], d["w_gate"], d["b_gate"], d["w1"], d["w3"], d["w2"], b.y, b.saved, b.ws)

    def bwd():
        moe.moe_layer_bwd(cfg, d["dy"], d["x"], d["w_gate"], d["w1"], d["w3"], d["w2"], b.saved, b.dx, b.dw_gate,
                          b.db_gate if has_bias else None, b.dw1, b.dw3, b.dw2, b.ws)

    library_gemm = copy_gbs = None
    if not args.no_calibrate:
        library_gemm = library_gemm_reference(torch)
        copy_gbs = copy_bandwidth(torch)
        torch.cuda.empty_cache()
    if args.calibrate_copy:
        src = torch.empty(1 << 30, dtype=torch.uint8, device="cuda").fill_(1)
        dst = torch.empty_like(src)
        dst.copy_(src)                                   # reads 1 GiB, writes 1 GiB
        torch.cuda.synchronize()
        del src, dst
    for _ in range(args.warmup):
        fwd(); bwd()
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(args.steps):
        fwd(); bwd()
    torch.cuda.synchronize()
    ms_per_step = (time.perf_counter() - t0) * 1e3 / args.steps

    # ---- kept rows (A) and algorithmic work of the expert GEMMs
    offs = moe.saved_view(cfg, b.saved, "offsets", torch.int32).cpu().numpy()
    count = np.diff(offs)
    A = int(offs[-1])
    per_row = (6 if w.gated else 4) * w.M * w.H           # forward FLOP per kept row
    flop_fwd, flop_bwd = A * per_row, 2 * A * per_row

    # ---- per-call timing with HIP events on the launch stream (torch's current stream)
    def timed(fn, reps):
        ev0, ev1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        fn(); torch.cuda.synchronize()
        ev0.record()
        for _ in range(reps):
            fn()
        ev1.record(); torch.cuda.synchronize()
        return ev0.elapsed_time(ev1) / reps

    sv = lambda name, dt: moe.saved_view(cfg, b.saved, name, dt)
    tdt = b.y.dtype
    i32, f32 = torch.int32, torch.float32
    xe = sv("xe", tdt).view(w.N * w.k, w.M); q = sv("q", tdt).view(w.N * w.k, w.M)
    a1 = sv("a1", tdt).view(w.N * w.k, w.H); hh = sv("hh", tdt).view(w.N * w.k, w.H)
    a3 = sv("a3", tdt).view(w.N * w.k, w.H) if w.gated else None
    row_of = sv("row_of", i32); offsets = sv("offsets", i32); topk_w = sv("topk_w", f32)
    reps = max(3, args.steps // 2)
    t_ffn_fwd = timed(lambda: moe.moe_expert_ffn_fwd(cfg, xe, offsets, d["w1"], d["w3"], d["w2"], b.q, b.a1, b.a3, b.hh, b.ws), reps)
    moe.moe_combine_bwd(cfg, d["dy"], q, topk_w, row_of, b.dq, b.dtopk_w)
    t_ffn_bwd = timed(lambda: moe.moe_expert_ffn_bwd(cfg, b.dq, xe, offsets, d["w1"], d["w3"], d["w2"], a1, a3, hh,
                                                     b.dxe, b.dw1, b.dw3, b.dw2, b.ws), reps)
    gemm_ms = t_ffn_fwd + t_ffn_bwd
    achieved = (flop_fwd + flop_bwd) / (gemm_ms * 1e-3) / 1e12
    roofline = {"bound": "mfma", "kernel": "gg_mfma64_kernel / gg_mfma_kernel (bf16 grouped GEMM, 2 forward + 4 backward launches per step)",
                "achieved": round(achieved, 1), "peak": PEAK_BF16_TFLOPS, "unit": "TFLOP/s",
                "frac": round(achieved / PEAK_BF16_TFLOPS, 4),
                "traffic": (lambda t: None if t is None else t["read"] + t["written"])(MEASURED_GEMM_TRAFFIC.get(w.name)),
                "flop_per_step": flop_fwd + flop_bwd, "ms_per_step": round(gemm_ms, 3),
                "fwd": {"ms": round(t_ffn_fwd, 3), "tflops": round(flop_fwd / t_ffn_fwd / 1e9, 1)},
                "bwd": {"ms": round(t_ffn_bwd, 3), "tflops": round(flop_bwd / t_ffn_bwd / 1e9, 1)}}

    out = {"metric": "MoE layer fwd+bwd tokens/s (%s-shape, 1 GPU)" % w.name, "value": round(w.N / (ms_per_step * 1e-3), 1),
           "unit": "tokens/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
           "ms_per_step": round(ms_per_step, 3), "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
           "dtype": "bf16" if w.dtype == S.DT_BF16 else "f32", "data": "synthetic",
           "config": {"workload": "%s: N=%d M=%d E=%d H=%d k=%d f=%s act=%d renormalize=%d residual=%d" % (
               w.name, w.N, w.M, w.E, w.H, w.k, S.capacity_factor_text(w), w.act, w.renormalize, w.add_residual),
               "kept_rows": A, "rows_per_expert_min_max": [int(count.min()), int(count.max())]},
           "expert_gemm_tflops": round(achieved, 1), "roofline": roofline}
    if library_gemm is not None:
        # measured peaks of this machine beside the nominal ones the fractions above are taken against
        out["library_gemm_reference"] = library_gemm
        out["measured_peaks"] = {"copy_GBps": copy_gbs, "copy_frac_of_nominal_hbm": round(copy_gbs / PEAK_HBM_GBS, 3),
                                 "library_gemm_best_TFLOPs": max(library_gemm[k] for k in ("NN", "NT", "TN")),
                                 "expert_gemm_vs_library_best": round(achieved / max(library_gemm[k] for k in ("NN", "NT", "TN")), 3)}
    if args.fit_expert_model:
        out["expert_model"] = fit_expert_model(torch, cfg, w, d, b, xe, a1, a3, hh, torch.from_numpy(count).to("cuda"), timed, reps, flop_fwd)
    if args.chunks > 1:
        aux = torch.cuda.Stream()

        def step_chunked():
            moe.moe_layer_fwd_chunked(cfg, d["x"], d["w_gate"], d["b_gate"], d["w1"], d["w3"], d["w2"], b.y, b.saved, b.ws,
                                      args.chunks, aux)
            moe.moe_layer_bwd_chunked(cfg, d["dy"], d["x"], d["w_gate"], d["w1"], d["w3"], d["w2"], b.saved, b.dx,
                                      b.dw_gate, b.db_gate if has_bias else None, b.dw1, b.dw3, b.dw2, b.ws, args.chunks)

        for _ in range(args.warmup):
            step_chunked()
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for _ in range(args.steps):
            step_chunked()
        torch.cuda.synchronize()
        ms_c = (time.perf_counter() - t0) * 1e3 / args.steps
        out["chunked"] = {"n_chunks": args.chunks, "streams": 2, "ms_per_step": round(ms_c, 3),
                          "tokens_per_s": round(w.N / ms_c * 1e3, 1)}

    if args.graph:
        graph = torch.cuda.CUDAGraph()
        with torch.cuda.graph(graph):
            fwd(); bwd()
        for _ in range(args.warmup):
            graph.replay()
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for _ in range(args.steps):
            graph.replay()
        torch.cuda.synchronize()
        ms_g = (time.perf_counter() - t0) * 1e3 / args.steps
        out["graph"] = {"ms_per_step": round(ms_g, 4), "tokens_per_s": round(w.N / ms_g * 1e3, 1)}

    if args.gates:
        out["gates"] = time_gates(torch, moe, S, w, d, args, ms_per_step)

    if not args.no_breakdown:
        bpe = 2 if w.dtype == S.DT_BF16 else 4
        N, M, E, k = w.N, w.M, w.E, w.k
        calls = {
            "route": (lambda: moe.moe_route(cfg, d["x"], d["w_gate"], d["b_gate"], b.logits, b.probs, b.topk_idx, b.topk_w,
                                            b.pos, b.row_of, b.count, b.offsets, b.src_of_row, b.ws),
                      N * M * bpe + M * E * bpe + N * (8 * E + 16 * k) + 4 * (2 * E + 1)),
            "dispatch": (lambda: moe.moe_dispatch(cfg, d["x"], row_of, b.xe), N * M * bpe + 4 * N * k + A * M * bpe),
            "combine": (lambda: moe.moe_combine(cfg, q, topk_w, row_of, d["x"], b.y), A * M * bpe + 8 * N * k + N * M * bpe),
            "combine_bwd": (lambda: moe.moe_combine_bwd(cfg, d["dy"], q, topk_w, row_of, b.dq, b.dtopk_w),
                            N * M * bpe + 2 * A * M * bpe + 4 * N * k),
            "dispatch_bwd": (lambda: moe.moe_dispatch_bwd(cfg, b.dxe, row_of, d["dy"], b.dx), A * M * bpe + N * M * bpe),
            "route_bwd": (lambda: moe.moe_route_bwd(cfg, d["x"], d["w_gate"], sv("probs", f32), sv("topk_idx", i32),
                                                    sv("pos", i32), b.dtopk_w, b.dw_gate,
                                                    b.db_gate if has_bias else None, b.dx, b.ws),
                          3 * N * M * bpe + 8 * N * E + M * E * bpe),
        }
        br = {}
        for name, (fn, nbytes) in calls.items():
            ms = timed(fn, reps)
            br[name] = {"ms": round(ms, 4), "GB/s": round(nbytes / ms / 1e6, 1), "hbm_frac": round(nbytes / ms / 1e6 / PEAK_HBM_GBS, 3)}
        br["expert_ffn_fwd"] = {"ms": round(t_ffn_fwd, 3)}
        br["expert_ffn_bwd"] = {"ms": round(t_ffn_bwd, 3)}
        out["breakdown"] = br

    if not args.no_cpu_baseline:
        out["cpu_baseline"] = cpu_baseline(w)
    print(json.dumps(out), flush=True)


def time_gates(torch, moe, S, w, d, args, ms_default):
    """ms per layer step (forward + backward) with each gate of Sec. 2.1, same N, M, H, E and expert weights."""
    from paper_2501_10714_amd.buffers import Buffers, make_cfg
    dt = d["x"].dtype
    i32, f32 = torch.int32, torch.float32
    names = [("logits", f32), ("probs", f32), ("topk_idx", i32), ("topk_w", f32), ("pos", i32), ("row_of", i32),
             ("count", i32), ("offsets", i32), ("src_of_row", i32)]

    def clock(step):
        for _ in range(args.warmup):
            step()
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for _ in range(args.steps):
            step()
        torch.cuda.synchronize()
        return round((time.perf_counter() - t0) * 1e3 / args.steps, 3)

    res = {"as_configured (renormalize=%d)" % w.renormalize: round(ms_default, 3)}
    g = torch.Generator(device="cuda")
    g.manual_seed(77)
    rnd = lambda shape, std: (torch.randn(shape, generator=g, device="cuda", dtype=torch.float32) * std)

    def fused(wl):
        cfg = make_cfg(wl)
        b = Buffers(wl, cfg)

        def step():
            moe.moe_layer_fwd(cfg, d["x"], d["w_gate"], d["b_gate"], d["w1"], d["w3"], d["w2"], b.y, b.saved, b.ws)
            moe.moe_layer_bwd(cfg, d["dy"], d["x"], d["w_gate"], d["w1"], d["w3"], d["w2"], b.saved, b.dx, b.dw_gate,
                              b.db_gate if d["b_gate"] is not None else None, b.dw1, b.dw3, b.dw2, b.ws)
        t = clock(step)
        del b
        torch.cuda.empty_cache()
        return t

    res["sigmoid"] = fused(S.scaled(w, renormalize=2))
    if w.E <= 8:   # one slot per expert; every expert keeps N k / E tokens: the same number of expert rows
        res["expert_choice (%d tokens per expert)" % (w.N * w.k // w.E)] = fused(
            S.scaled(w, k=w.E, f=float(w.k) / w.E, renormalize=3))

    cfg = make_cfg(w)
    b = Buffers(w, cfg)
    v = {n: moe.saved_view(cfg, b.saved, n, t) for n, t in names}
    route_out = [v[n] for n, _ in names[1:]]
    # noisy gate: the draws are an input
    w_noise = rnd((w.M, w.E), 0.02).to(dt)
    noise = rnd((w.N, w.E), 1.0)
    nl = torch.empty(w.N, w.E, dtype=f32, device="cuda")
    dw_noise = torch.empty_like(b.dw_gate)

    def step_noisy():
        moe.moe_route_noisy(cfg, d["x"], d["w_gate"], d["b_gate"], w_noise, noise, v["logits"], nl, *route_out, b.ws)
        moe.moe_layer_fwd_routed(cfg, d["x"], d["w1"], d["w3"], d["w2"], b.y, b.saved, b.ws)
        moe.moe_layer_bwd_routed(cfg, d["dy"], d["w1"], d["w3"], d["w2"], b.saved, b.dx, b.dw1, b.dw3, b.dw2, b.dtopk_w, b.ws)
        moe.moe_route_noisy_bwd(cfg, d["x"], d["w_gate"], w_noise, noise, nl, v["probs"], v["topk_idx"], v["pos"], b.dtopk_w,
                                b.dw_gate, b.db_gate if d["b_gate"] is not None else None, dw_noise, b.dx, b.ws)
    res["noisy"] = clock(step_noisy)
    # X-MoE: 256-wide projection, cosine scores
    dp = 256
    w_proj = rnd((w.M, dp), 0.02).to(dt)
    w_emb = rnd((dp, w.E), 0.5).to(dt)
    proj = torch.empty(w.N, dp, dtype=f32, device="cuda")
    ws_x = torch.empty(moe.moe_route_xmoe_workspace_bytes(cfg, dp), dtype=torch.uint8, device="cuda")
    dw_proj = torch.empty(w.M, dp, dtype=dt, device="cuda")
    dw_emb = torch.empty(dp, w.E, dtype=dt, device="cuda")

    def step_xmoe():
        moe.moe_route_xmoe(cfg, d["x"], w_proj, w_emb, dp, proj, v["logits"], *route_out, ws_x)
        moe.moe_layer_fwd_routed(cfg, d["x"], d["w1"], d["w3"], d["w2"], b.y, b.saved, b.ws)
        moe.moe_layer_bwd_routed(cfg, d["dy"], d["w1"], d["w3"], d["w2"], b.saved, b.dx, b.dw1, b.dw3, b.dw2, b.dtopk_w, b.ws)
        moe.moe_route_xmoe_bwd(cfg, d["x"], w_proj, w_emb, dp, proj, v["probs"], v["topk_idx"], v["pos"], b.dtopk_w, dw_proj,
                               dw_emb, b.dx, ws_x)
    res["xmoe (d_proj=%d)" % dp] = clock(step_xmoe)
    return res


def cpu_baseline(w):
    """The oracle, as it stands, timed on the host cores.  The two small shapes (tiny, gpt2) run the full oracle on the
    full workload, on all threads and on one.  The larger shapes run a bounded sample of the workload: the same layer
    (full d_model, d_hidden, k, activation, gate) on fewer tokens and, to bound the weight memory, on min(E, max(k, 2))
    experts; per-token arithmetic is that of the full workload."""
    import numpy as np
    import moe_synth as S
    from oracle import moe_oracle as O
    try:
        import threadpoolctl
        cores = max((p.get("num_threads", 1) for p in threadpoolctl.threadpool_info()), default=1)
    except Exception:
        threadpoolctl = None
        cores = os.cpu_count() or 1

    def run(ws, cap):
        d = S.draw_all(ws)
        f = {k: (None if v is None else S.to_f64(v)) for k, v in d.items()}
        t0 = time.perf_counter()
        fwd = O.layer_fwd(f["x"], f["w_gate"], f["b_gate"], f["w1"], f["w3"], f["w2"], ws.k, cap, ws.act, ws.renormalize,
                          ws.add_residual)
        O.layer_bwd(f["dy"], f["x"], f["w_gate"], f["b_gate"], f["w1"], f["w3"], f["w2"], fwd, ws.act, ws.renormalize,
                    ws.add_residual)
        return time.perf_counter() - t0

    per_token = 3 * (6 if w.gated else 4) * w.M * w.H * w.k      # fwd+bwd FLOP per token
    if w.N * per_token <= 2e12:                                  # tiny, gpt2: the whole workload
        cap = 0 if w.f is None else O.capacity(w.N, w.E, w.k, w.f)
        dt = run(w, cap)
        out = {"value": round(w.N / dt, 2), "unit": "tokens/s", "cores": int(cores), "kind": "oracle",
               "sample": "the full workload (%d tokens, %d experts), fwd+bwd in fp64 numpy, %.2f s" % (w.N, w.E, dt)}
        if threadpoolctl is not None:
            with threadpoolctl.threadpool_limits(limits=1):
                dt1 = run(w, cap)
            out["one_thread"] = {"value": round(w.N / dt1, 2), "unit": "tokens/s", "seconds": round(dt1, 2)}
        return out
    e_s = min(w.E, max(w.k, 2))
    n_s = int(max(64, min(w.N, 1.5e13 / per_token)))             # about 15 TFLOP of fp64 work
    ws = S.scaled(w, N=n_s, E=e_s, f=None, bias="none")
    dt = run(ws, 0)
    return {"value": round(n_s / dt, 2), "unit": "tokens/s", "cores": int(cores), "kind": "oracle",
            "sample": "%d tokens, %d of %d experts, full M=%d H=%d k=%d, fwd+bwd in fp64 numpy, %.1f s" % (
                n_s, e_s, w.E, w.M, w.H, w.k, dt)}


if __name__ == "__main__":
    main()
