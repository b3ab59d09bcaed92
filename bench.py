#!/usr/bin/env python3
"""Benchmark of the MDN chunkwise hot path on one MI355X.

A step = one forward (keeping the correction values for the backward) + one backward of the whole
layer-shaped batch, through the C ABI.  Default workload: the 1.3B-layer training shape
(B=4, T=4096, H=16, dk=dv=128, C=64, bf16 storage, fp32 states), the configuration the headline
metric (fwd+bwd tokens/s, % of bf16 MFMA peak) is quoted on.  Inputs are synthetic and resident
in HBM before the timed region.  Prints ONE JSON line.
"""
import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

PEAK_BF16_TFLOPS = 2500.0   # MI355X dense bf16 MFMA
PEAK_F32_TFLOPS = 157.3     # fp32 matrix
PEAK_HBM_GBS = 8000.0


def flops_per_tokhd(C, dk, dv):
    """Algorithmic flops per token per head of each kernel (dense C x C tiles, causal half not
    exploited), following the step list of the chunkwise algorithm."""
    tri = 2.0 * C * C / 3.0
    return {
        "intra_fwd": 8 * C * dk + 2 * C * dv + tri,      # masked products, solve, T V / T diag(a^-) P / T diag(b^-) P of the paper's step list
        "scan_fwd": 12 * dk * dv + 2 * C * dv,           # V~, inter read-out, S'/M' update, intra output
        "intra_bwd": 8 * C * dk + tri,                   # recomputed products, solve, the two P products
        "rebuild": 4 * dk * dv,                          # S'/M' update lines only
        "scan_bwd": 12 * dk * dv + 2 * C * dv,           # dV~, dS, dM
        "grad": 8 * C * dk + 6 * C * dv + 12 * dk * dv,  # chunk-parallel gradients
    }


def bytes_per_tokhd(C, dk, dv, es, keep):
    """Bytes per token per head that each kernel must move once in this decomposition (es = bytes of a
    stored element; gates and coefficients are fp32).  `keep`: the training forward also writes the
    reverse pass's operands and the chunk-start states."""
    coef = 8 * 4                                          # one row of 8 fp32 coefficients per token
    kt_fwd = dk * es if es == 4 else 0                    # K^T for the forward scan: 16-bit storage makes it on chip
    fwd_ops = kt_fwd + 2 * C * es + coef                  # (K^T,) T, Bm, coefficient block
    rev_ops = (2 * dk + 2 * C) * es + coef                # K^T, Q^T, Bm^T, T^T, coefficient block
    states = 2 * dk * dv * es // C                        # S, M of one chunk, per token
    qk = 2 * dk * es
    return {
        "intra_fwd": qk + 16 + (2 * C * es + rev_ops if keep else fwd_ops),
        "scan_fwd": fwd_ops + qk + dv * es + 2 * dv * es + (states if keep else 0),   # + q, k, v; V~ and o out
        "intra_bwd": qk + 16 + rev_ops,
        "rebuild": dk * es + dv * es + coef + states,
        "scan_bwd": rev_ops + dk * es + dv * es + dv * es + states,                   # + k, dO; dv, dstates out
        # q, k, V~, dO, dV and both state pairs in; dq, dk and the gate gradients out (with 16-bit storage K^T and Q^T
        # come out of the k, q tiles on chip; the fp32 path still reads them: 2 dk es more)
        "grad": 2 * dk * es + 3 * dv * es + 2 * states + 16 + 2 * dk * es + 12 + (2 * dk * es if es == 4 else 0),
    }


def read_traffic(path):
    """Measured HBM bytes per launch {kernel: fetch + write}, from the `traffic` lines of a profiles/ summary."""
    out = {}
    try:
        for line in open(path):
            p = line.split()
            if len(p) == 4 and p[0] == "traffic":
                out[p[1]] = int(p[2]) + int(p[3])
    except OSError:
        pass
    return out


def decode_bench(args, torch, binding, synth):
    """One decode token per sequence through mdn_recurrent_step: HBM-bound on reading and writing S and M (fp32)."""
    B, H, dk = args.decode, 16, 128
    w = synth.custom(B=B, T=64, H=H, dk=dk, dv=dk, dtype="bf16", seed=7)
    t = synth.to_device(w)
    tok = {k: t[k][:, :1].contiguous() for k in ("q", "k", "v", "beta", "alpha", "mu")}
    S = torch.zeros((B, H, dk, dk), dtype=torch.float32, device="cuda")
    M = torch.zeros_like(S)
    o = None

    def step():
        nonlocal o
        o = binding.mdn_recurrent_step(tok["q"], tok["k"], tok["v"], tok["beta"], tok["alpha"], tok["mu"], S, M,
                                       scale=w.scale, out=o)

    for _ in range(args.warmup):
        step()
    torch.cuda.synchronize()
    binding.profile_begin()
    t0 = time.perf_counter()
    for _ in range(args.steps):
        step()
    torch.cuda.synchronize()
    wall = time.perf_counter() - t0
    ms, cnt = binding.profile_end()["recurrent"]
    avg = ms / max(cnt, 1)
    nbytes = 4 * B * H * dk * dk * 4  # S and M, read and written once, fp32
    gbs = nbytes / (avg * 1e-3) / 1e9
    print(json.dumps({
        "metric": "MDN recurrent step (decode) tokens/sec", "value": round(B * args.steps / wall, 1), "unit": "tokens/s",
        "n_gpus": 1, "steps": args.steps, "warmup": args.warmup, "ms_per_step": round(wall * 1e3 / args.steps, 4),
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None, "dtype": "f32", "data": "synthetic",
        "config": {"workload": f"decode_B{B}_H{H}_d{dk}", "B": B, "T": 1, "H": H, "dk": dk, "dv": dk},
        "roofline": {"kernel": "recurrent", "bound": "hbm", "achieved": round(gbs, 1), "peak": PEAK_HBM_GBS,
                     "unit": "GB/s", "frac": round(gbs / PEAK_HBM_GBS, 5), "traffic": None},
        "kernels": {"recurrent": {"avg_ms": round(avg, 4), "launches": cnt}}, "cpu_baseline": None}))


def handoff_bench(args, torch, binding, synth):
    """Prefill -> decode hand-off: mdn_chunk_fwd over T_ctx tokens (inference mode: nothing kept for a backward)
    leaves S, M; mdn_recurrent_step then decodes from them, one token per call and in blocks of 8 tokens per call.
    The decode cost does not depend on T_ctx (Fig. 4, left: the state has a fixed size), the prefill cost is linear."""
    B, H, dk = args.handoff, 16, 128
    rows = []
    for T_ctx in (1024, 4096, 16384):
        w = synth.custom(B=B, T=T_ctx, H=H, dk=dk, dv=dk, dtype="bf16", seed=11)
        t = synth.to_device(w)
        names = ("q", "k", "v", "beta", "alpha", "mu")
        tok1 = {k: t[k][:, :1].contiguous() for k in names}   # the decode tokens: synthetic, like the prompt's
        tok8 = {k: t[k][:, :8].contiguous() for k in names}
        out = None

        def prefill():
            nonlocal out
            out = binding.mdn_chunk_fwd(*(t[k] for k in names), scale=w.scale, out=out, workspace=out and out["workspace"])

        def timed(fn, n):
            for _ in range(max(args.warmup // 2, 1)):
                fn()
            torch.cuda.synchronize()
            t0 = time.perf_counter()
            for _ in range(n):
                fn()
            torch.cuda.synchronize()
            return (time.perf_counter() - t0) * 1e3 / n

        ms_prefill = timed(prefill, max(args.steps // 4, 2))
        S, M = out["S"].clone(), out["M"].clone()
        o1 = o8 = None

        def dec1():
            nonlocal o1
            o1 = binding.mdn_recurrent_step(*(tok1[k] for k in names), S, M, scale=w.scale, out=o1)

        def dec8():
            nonlocal o8
            o8 = binding.mdn_recurrent_step(*(tok8[k] for k in names), S, M, scale=w.scale, out=o8)

        ms1 = timed(dec1, args.steps * 4)
        ms8 = timed(dec8, args.steps * 2)
        rows.append({"T_ctx": T_ctx, "prefill_ms": round(ms_prefill, 4),
                     "prefill_tokens_per_s": round(B * T_ctx / (ms_prefill * 1e-3), 1),
                     "decode_ms_per_token": round(ms1, 4), "decode_block8_ms_per_token": round(ms8 / 8, 4)})
        del t, out, S, M
        torch.cuda.empty_cache()
    nbytes = 4 * B * H * dk * dk * 4
    gbs = nbytes / (rows[-1]["decode_ms_per_token"] * 1e-3) / 1e9
    print(json.dumps({
        "metric": "MDN decode latency after prefill hand-off", "value": rows[-1]["decode_ms_per_token"], "unit": "ms/token",
        "n_gpus": 1, "steps": args.steps, "warmup": args.warmup, "ms_per_step": rows[-1]["decode_ms_per_token"],
        "higher_is_better": False, "scaling": "weak", "vs_baseline": None, "dtype": "f32", "data": "synthetic",
        "config": {"workload": f"handoff_B{B}_H{H}_d{dk}", "B": B, "H": H, "dk": dk, "dv": dk},
        "roofline": {"kernel": "recurrent", "bound": "hbm", "achieved": round(gbs, 1), "peak": PEAK_HBM_GBS,
                     "unit": "GB/s", "frac": round(gbs / PEAK_HBM_GBS, 5), "traffic": None},
        "by_context": rows, "cpu_baseline": None}))


def varlen_bench(args, torch, binding, synth):
    """Packed variable-length batches, forward + backward (the backward rebuilds states and operands): the batch as one
    stream of tokens (no per-sequence states asked for) against the same batch run sequence by sequence."""
    total, H, dk = args.varlen, 16, 128
    rows = []
    for nseq in (8, 64, 256):
        L = total // nseq
        w = synth.custom(B=1, T=nseq * L, H=H, dk=dk, dv=dk, dtype="bf16", seed=5, backward=True)
        t = synth.to_device(w)
        cu = [i * L for i in range(nseq + 1)]
        names = ("q", "k", "v", "beta", "alpha", "mu")
        row = {"sequences": nseq, "tokens_each": L}
        for one_stream in (True, False):
            def step():
                f = binding.mdn_chunk_fwd_varlen(*(t[k] for k in names), cu, scale=w.scale, save_vt=True,
                                                 want_states=not one_stream)
                binding.mdn_chunk_bwd_varlen(*(t[k] for k in names), f["vt"], t["dO"], cu, scale=w.scale,
                                             want_state_grads=not one_stream)
            for _ in range(2):
                step()
            torch.cuda.synchronize()
            t0 = time.perf_counter()
            n = max(args.steps // 5, 2)
            for _ in range(n):
                step()
            torch.cuda.synchronize()
            ms = (time.perf_counter() - t0) * 1e3 / n
            key = "one_stream" if one_stream else "sequence_by_sequence"
            row[key + "_ms"] = round(ms, 3)
            row[key + "_tokens_per_s"] = round(nseq * L / (ms * 1e-3), 1)
        # prefill of the same batch as prompts: forward only, final states of every sequence wanted (zero initial
        # states: the stream form plus one batch of last chunks; with initial states given: sequence by sequence)
        zeros = torch.zeros((nseq, H, dk, dk), dtype=torch.float32, device="cuda")
        for one_stream in (True, False):
            def prefill():
                binding.mdn_chunk_fwd_varlen(*(t[k] for k in names), cu, scale=w.scale,
                                             S0=None if one_stream else zeros, M0=None if one_stream else zeros)
            for _ in range(2):
                prefill()
            torch.cuda.synchronize()
            t0 = time.perf_counter()
            n = max(args.steps // 5, 2)
            for _ in range(n):
                prefill()
            torch.cuda.synchronize()
            ms = (time.perf_counter() - t0) * 1e3 / n
            key = "prefill_one_stream" if one_stream else "prefill_sequence_by_sequence"
            row[key + "_ms"] = round(ms, 3)
            row[key + "_tokens_per_s"] = round(nseq * L / (ms * 1e-3), 1)
        rows.append(row)
        del t, zeros
        torch.cuda.empty_cache()
    print(json.dumps({
        "metric": "MDN packed variable-length batch fwd+bwd tokens/sec", "value": rows[1]["one_stream_tokens_per_s"],
        "unit": "tokens/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup, "ms_per_step": rows[1]["one_stream_ms"],
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None, "dtype": "bf16", "data": "synthetic",
        "config": {"workload": f"varlen_{total}tokens_H{H}_d{dk}", "H": H, "dk": dk, "dv": dk}, "roofline": None,
        "by_batch": rows, "cpu_baseline": None}))


def layer_ops_bench(args, torch, binding):
    """The elementwise operations around the delta rule (gate parameterisation, front end, back end) and their adjoints
    at the 1.3B layer shape: streaming kernels, HBM-bound.  Wall-clock rates here include the binding's output
    allocations; `rocprofv3 --kernel-trace --stats` on this command gives the kernels' own durations."""
    B, T, H, d = 4, 4096, 16, 128
    g = torch.Generator(device="cuda").manual_seed(0)
    r = lambda: torch.randn((B, T, H, d), device="cuda", generator=g).to(torch.bfloat16)
    xq, xk, xv, dq, dk, dv, o, gg, dy = (r() for _ in range(9))
    dh = torch.rand(H, device="cuda", generator=g)
    w = torch.rand(d, device="cuda", generator=g) + 0.5
    xs = [torch.randn((B, T, H), device="cuda", generator=g) for _ in range(8)]
    par = [torch.rand(H, device="cuda", generator=g) + 0.2 for _ in range(4)]
    row = B * T * H * d * 2
    ops = (("frontend_fwd", lambda: binding.mdn_frontend_fwd(xq, xk, xv, dh), 6 * row),
           ("frontend_bwd", lambda: binding.mdn_frontend_bwd(xq, xk, xv, dh, dq, dk, dv), 9 * row),
           ("epilogue_fwd", lambda: binding.mdn_epilogue_fwd(o, gg, w), 3 * row),
           ("epilogue_bwd", lambda: binding.mdn_epilogue_bwd(o, gg, w, dy), 5 * row),
           ("gates_fwd", lambda: binding.mdn_gates_fwd(*xs[:4], *par, 0.8, 8.0), 8 * B * T * H * 4),
           ("gates_bwd", lambda: binding.mdn_gates_bwd(*xs[:4], *par, 0.8, 8.0, *xs[4:]), 12 * B * T * H * 4))
    rows = {}
    for name, f, nbytes in ops:
        for _ in range(args.warmup):
            f()
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for _ in range(args.steps):
            f()
        torch.cuda.synchronize()
        ms = (time.perf_counter() - t0) * 1e3 / args.steps
        rows[name] = {"bytes": nbytes, "wall_ms": round(ms, 4), "wall_gbs": round(nbytes / ms / 1e6, 1)}
    best = max(rows, key=lambda k: rows[k]["wall_gbs"])
    print(json.dumps({
        "metric": "MDN layer elementwise operations, streaming rate", "value": rows[best]["wall_gbs"], "unit": "GB/s",
        "n_gpus": 1, "steps": args.steps, "warmup": args.warmup, "ms_per_step": rows[best]["wall_ms"],
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None, "dtype": "bf16", "data": "synthetic",
        "config": {"workload": f"layer_ops_B{B}_T{T}_H{H}_d{d}", "B": B, "T": T, "H": H, "d": d},
        "roofline": {"kernel": best, "bound": "hbm", "achieved": rows[best]["wall_gbs"], "peak": PEAK_HBM_GBS, "unit": "GB/s",
                     "frac": round(rows[best]["wall_gbs"] / PEAK_HBM_GBS, 5), "traffic": None},
        "by_op": rows, "cpu_baseline": None}))


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=20)
    ap.add_argument("--warmup", type=int, default=5)
    ap.add_argument("--config", type=int, default=3, help="measurement configuration 0..4 (default: 1.3B fwd+bwd)")
    ap.add_argument("--forward-only", action="store_true")
    ap.add_argument("--recompute", action="store_true",
                    help="forward keeps only the correction values: the backward reconstructs the chunk-start "
                         "states and recomputes its chunk-local operands (default: the forward keeps both)")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-kernel-events", action="store_true", help="do not bracket kernels with HIP events")
    ap.add_argument("--event-period", type=int, default=3,
                    help="bracket every N-th kernel launch of the timed region with a HIP event pair (1: every launch, which "
                         "costs ~3 %% of the step; 3 walks through the 4 (or 16) launches of a step, step after step)")
    ap.add_argument("--decode", type=int, default=0, metavar="BATCH",
                    help="instead of the training step, time mdn_recurrent_step: one token for BATCH sequences x 16 heads "
                         "x 128x128 states (the decode regime of the recurrent form); prints its own JSON line")
    ap.add_argument("--handoff", type=int, default=0, metavar="BATCH",
                    help="instead of the training step: prefill BATCH sequences x 16 heads x d128 of 1024 / 4096 / 16384 "
                         "tokens with mdn_chunk_fwd, then decode from the states it leaves (mdn_recurrent_step, one token "
                         "and 8 tokens per call); prints its own JSON line with the decode latency per context length")
    ap.add_argument("--varlen", type=int, default=0, metavar="TOKENS",
                    help="packed variable-length batches of TOKENS tokens in 8, 64, 256 equal sequences (16 heads, d = 128)")
    ap.add_argument("--layer-ops", action="store_true",
                    help="instead of the training step: the elementwise operations around the delta rule (gates, front end, "
                         "back end) and their adjoints at B=4, T=4096, H=16, d=128")
    ap.add_argument("--calibration-copy-mib", type=int, default=0,
                    help="after the timed region, also run one plain device copy of this many MiB (the known-size "
                         "kernel that the FETCH_SIZE / WRITE_SIZE counters of a rocprofv3 --pmc run are scaled by)")
    args = ap.parse_args()
    if args.gpus != 1 or int(os.environ.get("WORLD_SIZE", "1")) != 1:
        print("bench.py: this build runs on ONE GPU only (the path has no multi-GPU part); use --gpus 1",
              file=sys.stderr)
        sys.exit(2)

    import numpy as np
    import torch
    from paper_2605_05838_amd import binding, synth

    if not torch.cuda.is_available():
        print("bench.py: no GPU visible", file=sys.stderr)
        sys.exit(2)
    torch.cuda.set_device(0)
    if args.layer_ops:
        return layer_ops_bench(args, torch, binding)
    if args.decode:
        return decode_bench(args, torch, binding, synth)
    if args.varlen:
        return varlen_bench(args, torch, binding, synth)
    if args.handoff:
        return handoff_bench(args, torch, binding, synth)
    w = synth.config(args.config)
    do_bwd = w.backward and not args.forward_only
    t = synth.to_device(w)

    fout, bout = {}, {}
    fws = bws = None
    keep = do_bwd and not args.recompute

    def step():
        nonlocal fout, bout, fws, bws
        f = binding.mdn_chunk_fwd(t["q"], t["k"], t["v"], t["beta"], t["alpha"], t["mu"], eta=t["eta"], S0=t["S0"],
                                  M0=t["M0"], scale=w.scale, save_vt=do_bwd, save_states=keep, save_operands=keep,
                                  workspace=fws, out=fout)
        fws, fout = f["workspace"], f
        if do_bwd:
            g = binding.mdn_chunk_bwd(t["q"], t["k"], t["v"], t["beta"], t["alpha"], t["mu"], f["vt"], t["dO"],
                                      eta=t["eta"], S0=t["S0"], M0=t["M0"], states=f["states"],
                                      operands=f["operands"], scale=w.scale, workspace=bws, out=bout)
            bws, bout = g["workspace"], g

    for _ in range(args.warmup):
        step()
    torch.cuda.synchronize()
    if not args.no_kernel_events:
        binding.profile_begin(args.event_period)
    ev0, ev1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    ev0.record()
    for _ in range(args.steps):
        step()
    ev1.record()
    torch.cuda.synchronize()
    wall = time.perf_counter() - t0
    kern = {} if args.no_kernel_events else binding.profile_end(with_launch_counts=True)
    if args.calibration_copy_mib:
        src = torch.empty(args.calibration_copy_mib << 20, dtype=torch.uint8, device="cuda").fill_(1)
        dst = torch.empty_like(src)
        torch.cuda.synchronize()
        dst.copy_(src)
        torch.cuda.synchronize()
    ms_per_step = wall * 1e3 / args.steps
    tokens_per_s = w.tokens * args.steps / wall

    # ---- per-kernel figures.  A call may launch a kernel several times per step (segments of the sequence, the
    # partial last chunk); the algorithmic flops and bytes of a step are shared among those launches, so a kernel is
    # priced per STEP: (work of one step) / (summed duration of its launches in one step), which is also
    # (work per launch) / (average launch duration) when the step's work is split evenly.
    tokhd = w.B * w.T * w.H
    fl = flops_per_tokhd(w.C, w.dk, w.dv)
    by = bytes_per_tokhd(w.C, w.dk, w.dv, 2 if w.dtype == "bf16" else 4, keep)
    peak = PEAK_BF16_TFLOPS if w.dtype == "bf16" else PEAK_F32_TFLOPS
    kernels = {}
    for name, (ms, cnt, launched) in kern.items():
        if cnt and name in fl:
            lps = launched / args.steps          # launches per step (all of them)
            per_step = ms / cnt * lps            # average bracketed launch x launches per step
            tfl = fl[name] * tokhd / (per_step * 1e-3) / 1e12
            gbs = by[name] * tokhd / (per_step * 1e-3) / 1e9
            kernels[name] = {"ms_per_step": round(per_step, 4), "launches_per_step": round(lps, 2),
                             "avg_launch_ms": round(ms / cnt, 4), "launches_timed": cnt,
                             "gflop_per_launch": round(fl[name] * tokhd / lps / 1e9, 3),
                             "mib_per_launch": round(by[name] * tokhd / lps / 2 ** 20, 1),
                             "tflops": round(tfl, 2), "frac_mfma": round(tfl / peak, 5),
                             "gbs": round(gbs, 1), "frac_hbm": round(gbs / PEAK_HBM_GBS, 5)}
    roofline = roofline_hbm = None
    if kernels:
        dom = max(kernels, key=lambda k: kernels[k]["ms_per_step"])
        # measured HBM bytes per launch come from rocprofv3 counter runs (FETCH_SIZE, WRITE_SIZE, scaled by what the
        # same counters read for a plain copy), which cannot run inside a timed run: the figure is read from the
        # committed summary of such runs of this same command, and only the default run of config 3 has one
        traffic, source = None, None
        if args.config == 3 and keep:
            source = "profiles/step_c3_hbm_traffic.md"
            traffic = read_traffic(os.path.join(ROOT, source)).get(dom)
        roofline = {"kernel": dom, "bound": "mfma", "achieved": kernels[dom]["tflops"], "peak": peak,
                    "unit": "TFLOP/s", "frac": kernels[dom]["frac_mfma"], "traffic": traffic, "traffic_source": source}
        roofline_hbm = {"kernel": dom, "bound": "hbm", "achieved": kernels[dom]["gbs"], "peak": PEAK_HBM_GBS,
                        "unit": "GB/s", "frac": kernels[dom]["frac_hbm"], "traffic": traffic, "traffic_source": source}
    # the whole path: the ALGORITHMIC step list (state reconstruction and the second chunk-local pass included, also
    # when the forward kept their results and they are not launched) and the flops of the kernels actually launched
    steps_fwd, steps_bwd = ("intra_fwd", "scan_fwd"), ("intra_bwd", "rebuild", "scan_bwd", "grad")
    total_flops = sum(fl[k] for k in steps_fwd + (steps_bwd if do_bwd else ())) * tokhd
    executed = [k for k in steps_fwd + (steps_bwd if do_bwd else ())
                if not (keep and k in ("intra_bwd", "rebuild"))]
    executed_flops = sum(fl[k] for k in executed) * tokhd
    path_tflops = total_flops / (ms_per_step * 1e-3) / 1e12
    path_tflops_executed = executed_flops / (ms_per_step * 1e-3) / 1e12
    for name, kd in kernels.items():
        assert kd["frac_mfma"] <= 1.0 and kd["frac_hbm"] <= 1.0, (name, kd)
    assert path_tflops / peak <= 1.0

    # ---- CPU baseline: the fp64 oracle as it stands, on the host cores: the whole workload on all cores (best of
    # three), and a sample of its (batch, head) pairs on one thread
    cpu = None
    if not args.no_cpu_baseline:
        from oracle import mdn_oracle as orc
        a = {k: (None if v is None else np.asarray(v, dtype=np.float64)) for k, v in w.arrays.items()}

        def oracle_pass(x, nthreads):
            c0 = time.perf_counter()
            r = orc.forward(x["q"], x["k"], x["v"], x["alpha"], x["beta"], x["mu"], eta=x["eta"], S0=x["S0"], M0=x["M0"],
                            scale=w.scale, nthreads=nthreads)
            if do_bwd:
                orc.backward(x["q"], x["k"], x["v"], x["alpha"], x["beta"], x["mu"], x["dO"], eta=x["eta"], S0=x["S0"],
                             M0=x["M0"], scale=w.scale, nthreads=nthreads)
            return time.perf_counter() - c0, r["threads"]

        runs = [oracle_pass(a, 0) for _ in range(3)]
        csec, threads = min(r[0] for r in runs), runs[0][1]
        # one thread: the first batch element, two heads (pairs are independent and cost the same)
        nh = min(2, w.H)
        one = {k: (None if v is None else np.ascontiguousarray(v[:1, :nh] if k in ("S0", "M0") else v[:1, :, :nh]))
               for k, v in a.items()}
        sec1, _ = oracle_pass(one, 1)
        what = "forward+backward" if do_bwd else "forward"
        cpu = {"value": round(w.tokens / csec, 1), "unit": "tokens/s", "cores": threads, "kind": "oracle",
               "sample": f"the full workload ({w.B}x{w.T} tokens, {w.H} heads, fp64, {what}), best of 3: {csec:.1f} s",
               "one_thread": {"value": round(w.T * nh / w.H / sec1, 1), "unit": "tokens/s", "cores": 1,
                              "sample": f"{nh} of the {w.B * w.H} (batch, head) pairs ({w.T} tokens each, {what}): "
                                        f"{sec1:.1f} s; a layer token is {w.H} heads"}}

    line = {
        "metric": "MDN layer fwd+bwd tokens/sec at 1.3B shape; % bf16 MFMA peak" if do_bwd and args.config == 3
        else f"MDN layer {'fwd+bwd' if do_bwd else 'fwd'} tokens/sec",
        "value": round(tokens_per_s, 1), "unit": "tokens/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": round(ms_per_step, 4), "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": w.dtype, "data": "synthetic",
        "config": {"workload": w.name, "B": w.B, "T": w.T, "H": w.H, "dk": w.dk, "dv": w.dv, "C": w.C,
                   "pass": "fwd+bwd" if do_bwd else "fwd", "forward_keeps_states_and_operands": bool(keep)},
        "path_tflops": round(path_tflops, 2), "path_frac_of_mfma_peak": round(path_tflops / peak, 5),
        "path_tflops_executed": round(path_tflops_executed, 2),
        "path_frac_of_mfma_peak_executed": round(path_tflops_executed / peak, 5),
        "gpu_event_ms_per_step": round(ev0.elapsed_time(ev1) / args.steps, 4),
        "roofline": roofline, "roofline_hbm": roofline_hbm, "kernels": kernels, "cpu_baseline": cpu,
    }
    print(json.dumps(line))


if __name__ == "__main__":
    main()
