#!/usr/bin/env python3
"""Benchmark of the arithmetic-sampling decode path on one MI355X.

One "step" is one whole as_decode call of the headline configuration
(V=32128, d=512, bf16, B=16 prompts x N=64 codes = 1024 rows, T=64 decode steps,
temperature 0.7, EOS sticky): lattice init, then per decode step the logits
GEMM and the fused sampling kernel.  Inputs (weights, prompts, shifts) are
synthetic, seeded and already resident in HBM when timing starts.

Prints ONE JSON line: whole-job code-steps/s, plus
  roofline      the fused sampling kernel (the dominant HBM-bound kernel): its
                algorithmic bytes per launch over its average launch duration,
                taken from the dispatch's own HIP events during the timed region
  roofline_cold the same kernel launched alone over >1 GiB of rotating logits
                buffers, so no row can be served from the 256 MB Infinity Cache
  roofline_16x_rows  (only with --rows16x) the same kernel, one launch over
                16x the rows (1 GiB)
  fused_decode  the decode without the logits round trip (as_decode_fused)
  encode        the encode direction over the decoded sequences (as_encode)
  ancestral     the ancestral-sampling mode and the lattice estimator
  logits_gemm   the MFMA logits kernel: achieved TFLOP/s against the bf16 peak
  cpu_baseline  the fp64 CPU oracle timed on this machine's host cores on a bounded
                sample of the same workload
  other_configs compact legs for the other benchmark configurations at their full shapes
                (configs[2] run twice, top-k=40 and top-p=0.9; configs[3]; configs[4]): whole-decode
                code-steps/s, the sampling kernel's launch time and fraction of the HBM peak,
                the logits kernel's launch time (skipped with --no-legs)
"""
import argparse
import hashlib
import json
import os
import sys
import time

import numpy as np

HBM_PEAK_GBS = 8000.0          # MI355X HBM3E, published
MFMA_BF16_PEAK_TFLOPS = 2500.0  # MI355X dense bf16, published


def spread(samples_ms):
    """median / p10 / p90 of single launch durations, in microseconds"""
    if len(samples_ms) == 0:
        return None
    q = np.percentile(np.asarray(samples_ms, dtype=np.float64) * 1e3, [50, 10, 90])
    return {"median_us": float(q[0]), "p10_us": float(q[1]), "p90_us": float(q[2]), "launches": int(len(samples_ms))}


def up(a):
    import torch
    if a.dtype == np.uint16:
        return torch.from_numpy(a.view(np.int16)).cuda().view(torch.bfloat16)
    return torch.from_numpy(a).cuda()


def sampling_kernel_name(V, ldt, top_k, top_p, temp=1.0):
    """Which kernel finishes the sampling step for this shape (the choice the library makes)."""
    has_k, has_p = 0 < top_k < V, 0.0 < top_p < 1.0
    tile = V <= (32768 if ldt == "bf16" else 16384) and V % (8 if ldt == "bf16" else 4) == 0
    first_chunk_reference_ok = 1.4426950408889634 / temp <= 4.0      # (the library's kTileMaxScale)
    if tile and ldt == "bf16" and has_k and top_k <= 48:
        return ("topk_tile_kernel (top-k%s and the sampling step in one launch, row resident in registers), "
                "as launched inside as_decode" % (" + nucleus" if has_p else ""))
    if tile and ldt == "bf16" and has_p and not has_k and first_chunk_reference_ok:
        return ("nucleus_tile_kernel (nucleus and the sampling step in one launch, logits counted by stored value), "
                "as launched inside as_decode")
    if V <= 32768 and has_k and top_k <= 128:
        return "threshold_resident_kernel with the sampling step fused (top-k, candidates ranked in LDS), as launched inside as_decode"
    if has_k or has_p:
        return "threshold kernel, then the sampling-step kernel, as launched inside as_decode"
    if tile and first_chunk_reference_ok:
        return "step_tile_kernel (fused sampling step, one-tile rows), as launched inside as_decode"
    return "step_kernel (fused sampling step), as launched inside as_decode"


def active_rows(tokens, eos):
    """Rows still running at each decode step, averaged over the steps (finished rows are not read)."""
    tk = tokens.cpu().numpy().reshape(-1, tokens.shape[-1])
    T = tk.shape[1]
    active = np.ones(tk.shape, dtype=bool)
    for t in range(1, T):
        active[:, t] = active[:, t - 1] & (tk[:, t - 1] != eos)
    return float(active.sum()) / T


def compact_leg(cfg_id, top_k, top_p, steps, warmup):
    """One whole-decode measurement of another configuration at its full shape, with the kernels' own times."""
    import torch
    from paper_2210_15458_amd import binding as B
    from paper_2210_15458_amd import synth
    cfg = synth.CONFIGS[cfg_id]
    V, d, Bn, N, T, temp, eos = cfg["V"], cfg["d"], cfg["B"], cfg["N"], cfg["T"], cfg["temp"], cfg["eos_id"]
    R = Bn * N
    E, U = synth.bigram_weights(V, d, seed=0, dtype=cfg["dtype"])
    Ed, Ud = up(E), up(U)
    del E, U
    model = B.Model(Ed, Ud, scale=cfg["scale"])
    del Ud
    prompts, u = up(synth.prompts(Bn, V, seed=1)), up(synth.shifts(Bn, seed=2))
    ctx = B.Ctx(R, V, torch.bfloat16)
    tokens = torch.empty((Bn, N, T), dtype=torch.int32, device="cuda")
    for _ in range(warmup):
        B.as_decode(ctx, model, prompts, N, T, u, temp, top_k, top_p, eos, tokens)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(steps):
        B.as_decode(ctx, model, prompts, N, T, u, temp, top_k, top_p, eos, tokens)
    torch.cuda.synchronize()
    t1 = time.perf_counter()
    ctx.profile(True)
    for _ in range(steps):
        B.as_decode(ctx, model, prompts, N, T, u, temp, top_k, top_p, eos, tokens)
    torch.cuda.synchronize()
    step_samples, gemm_samples, thr_samples = ctx.profile_samples(0), ctx.profile_samples(1), ctx.profile_samples(2)
    ctx.profile_read(0); ctx.profile_read(1); ctx.profile_read(2)
    ctx.profile(False)
    act = active_rows(tokens, eos)
    bytes_per_row = V * 2 + 18
    # the sampling step of a launch: the kernel that finishes it, plus the threshold kernel where that is separate
    samp_us = float(np.mean(step_samples)) * 1e3 + (float(np.mean(thr_samples)) * 1e3 if len(thr_samples) else 0.0)
    ach = act * bytes_per_row / (samp_us * 1e-6) / 1e9
    out = {
        "workload": f"configs[{cfg_id}] {cfg['name']}: as_decode V={V} d={d} bf16, B={Bn} N={N} (R={R}) T={T} "
                    f"temp={temp} top_k={top_k} top_p={top_p} eos={eos}",
        "value": R * T * steps / (t1 - t0), "unit": "code-steps/s", "decodes_timed": steps,
        "ms_per_decode": (t1 - t0) / steps * 1e3,
        "sampling": {"kernel": sampling_kernel_name(V, "bf16", top_k, top_p, temp), "bound": "hbm",
                     "avg_launch_us": samp_us, "spread": spread(step_samples), "achieved": ach, "peak": HBM_PEAK_GBS,
                     "unit": "GB/s", "frac": ach / HBM_PEAK_GBS, "bytes_per_code_step": bytes_per_row,
                     "active_rows_per_launch": act},
        "logits_gemm": {"avg_launch_us": float(np.mean(gemm_samples)) * 1e3, "spread": spread(gemm_samples),
                        "achieved": 2.0 * R * d * V / (float(np.mean(gemm_samples)) * 1e-3) / 1e12,
                        "peak": MFMA_BF16_PEAK_TFLOPS, "unit": "TFLOP/s"}}
    out["logits_gemm"]["frac"] = out["logits_gemm"]["achieved"] / MFMA_BF16_PEAK_TFLOPS
    if len(thr_samples):
        out["sampling"]["threshold_kernel_us"] = float(np.mean(thr_samples)) * 1e3
    if top_k <= 0 and not (0.0 < top_p < 1.0) and R <= 4096:
        # the same decode without the logits round trip (no logit modifiers; logits stay fp32 on chip)
        for _ in range(warmup):
            B.as_decode_fused(ctx, model, prompts, N, T, u, temp, eos, tokens)
        torch.cuda.synchronize()
        f0 = time.perf_counter()
        for _ in range(steps):
            B.as_decode_fused(ctx, model, prompts, N, T, u, temp, eos, tokens)
        torch.cuda.synchronize()
        f1 = time.perf_counter()
        ctx.profile(True)
        B.as_decode_fused(ctx, model, prompts, N, T, u, temp, eos, tokens)
        torch.cuda.synchronize()
        fs, fg = ctx.profile_samples(0), ctx.profile_samples(1)
        ctx.profile_read(0); ctx.profile_read(1)
        ctx.profile(False)
        out["fused_decode"] = {"value": R * T * steps / (f1 - f0), "unit": "code-steps/s",
                               "ms_per_decode": (f1 - f0) / steps * 1e3,
                               "logits_kernel_us": float(np.mean(fg)) * 1e3, "sampling_kernel_us": float(np.mean(fs)) * 1e3}
    ctx.close()
    model.close()
    del Ed, tokens
    torch.cuda.empty_cache()
    return out


def source_stamp():
    """Hash of the sources the sampling kernel is built from (ties a stored counter reading to the kernel timed)."""
    here = os.path.join(os.path.dirname(os.path.abspath(__file__)), "paper_2210_15458_amd", "csrc")
    h = hashlib.sha256()
    for name in ("as_step.hip", "as_tile.hpp", "as_row.hpp", "as_common.hpp"):
        with open(os.path.join(here, name), "rb") as f:
            h.update(f.read())
    return h.hexdigest()[:16]


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=20)
    ap.add_argument("--warmup", type=int, default=3)
    ap.add_argument("--config", type=int, default=1, help="index into the benchmark configurations")
    ap.add_argument("--top-k", type=int, default=None, help="override the configuration's top_k (0 = off)")
    ap.add_argument("--top-p", type=float, default=None, help="override the configuration's top_p (1 = off)")
    ap.add_argument("--logits", choices=["bf16", "f32"], default=None,
                    help="storage type of the logits between the two kernels (default: the configuration's)")
    ap.add_argument("--no-cpu", action="store_true", help="skip the CPU oracle leg")
    ap.add_argument("--no-cold", action="store_true", help="skip the cold (rotating buffers) kernel leg")
    ap.add_argument("--no-legs", action="store_true", help="skip the compact legs for the other configurations")
    ap.add_argument("--only-leg", default=None,
                    help="run nothing but one compact leg (configs2_topk, configs2_nucleus, configs3, configs4) "
                         "and print it: for kernel traces and counter runs of that configuration")
    ap.add_argument("--rows16x", action="store_true",
                    help="add the leg that runs the sampling kernel once over 16x the rows (its launches carry the "
                         "same kernel name, so a kernel trace of a run with this flag averages over both sizes)")
    ap.add_argument("--copy-calibration", action="store_true",
                    help="also run plain device copies of a known size (256 MiB each), the yardstick for "
                         "reading rocprofv3's FETCH_SIZE / WRITE_SIZE counters")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build runs on one GPU only (codes are independent, so more GPUs would each "
              "run this same path on their share of the codes); use --gpus 1", file=sys.stderr)
        return 2

    import torch
    from paper_2210_15458_amd import binding as B
    from paper_2210_15458_amd import synth

    legs = {"configs2_topk": (2, 40, 1.0, 3), "configs2_nucleus": (2, 0, 0.9, 3), "configs3": (3, 0, 1.0, 2),
            "configs4": (4, 0, 1.0, 2)}
    if args.only_leg:
        cid, k_, p_, n_ = legs[args.only_leg]
        print(json.dumps({args.only_leg: compact_leg(cid, k_, p_, n_, 1)}))
        return 0

    cfg = synth.CONFIGS[args.config]
    V, d, Bn, N, T = cfg["V"], cfg["d"], cfg["B"], cfg["N"], cfg["T"]
    temp, top_k, top_p, eos = cfg["temp"], cfg["top_k"], cfg["top_p"], cfg["eos_id"]
    if args.top_k is not None:
        top_k = args.top_k
    if args.top_p is not None:
        top_p = args.top_p
    R = Bn * N
    ldt = args.logits or cfg["dtype"]
    tdt = torch.bfloat16 if ldt == "bf16" else torch.float32
    esz = 2 if ldt == "bf16" else 4

    E, U = synth.bigram_weights(V, d, seed=0, dtype=cfg["dtype"])
    Ed, Ud = up(E), up(U)
    model = B.Model(Ed, Ud, scale=cfg["scale"])
    del Ud
    prompts = up(synth.prompts(Bn, V, seed=1))
    u = up(synth.shifts(Bn, seed=2))
    ctx = B.Ctx(R, V, tdt)
    tokens = torch.empty((Bn, N, T), dtype=torch.int32, device="cuda")

    def decode():
        B.as_decode(ctx, model, prompts, N, T, u, temp, top_k, top_p, eos, tokens)

    for _ in range(args.warmup):
        decode()
    torch.cuda.synchronize()
    # timed region: K whole decodes, nothing else on the stream
    t0 = time.perf_counter()
    for _ in range(args.steps):
        decode()
    torch.cuda.synchronize()
    t1 = time.perf_counter()

    # a longer region of the same work (the K-step figure moves by a few per cent from box to box and run to run)
    long_steps = max(100, args.steps)
    t4 = time.perf_counter()
    for _ in range(long_steps):
        decode()
    torch.cuda.synchronize()
    t5 = time.perf_counter()

    # the same region once more with a start/stop event attached to every kernel
    # dispatch (this costs some launch throughput, so it is kept out of `value`)
    ctx.profile(True)
    t2 = time.perf_counter()
    for _ in range(args.steps):
        decode()
    torch.cuda.synchronize()
    t3 = time.perf_counter()
    step_samples = ctx.profile_samples(0)
    gemm_samples = ctx.profile_samples(1)
    step_ms, step_n, step_drop = ctx.profile_read(0)
    gemm_ms, gemm_n, _ = ctx.profile_read(1)
    thr_ms, thr_n, _ = ctx.profile_read(2)
    ctx.profile(False)

    wall = t1 - t0
    code_steps = R * T * args.steps
    # rows that were still running, per launch: finished rows are not read
    active_rows_per_launch = active_rows(tokens, eos)
    bytes_per_row = V * esz + 18           # the logits row + code in/out, token, flags
    step_avg_us = step_ms / max(step_n, 1) * 1e3
    achieved = active_rows_per_launch * bytes_per_row / (step_avg_us * 1e-6) / 1e9 if step_n else None

    out = {
        "metric": "code-steps/sec and sampling-kernel HBM GB/s (% peak), V=32128, N*B=1024",
        "value": code_steps / wall,
        "unit": "code-steps/s",
        "n_gpus": 1,
        "steps": args.steps,
        "warmup": args.warmup,
        "ms_per_step": wall / args.steps * 1e3,
        "higher_is_better": True,
        "scaling": "weak",
        "vs_baseline": None,
        "dtype": "f32",
        "data": "synthetic",
        "config": {"workload": f"configs[{args.config}] {cfg['name']}: as_decode V={V} d={d} {cfg['dtype']} "
                               f"weights, {ldt} logits, B={Bn} N={N} (R={R}) T={T} temp={temp} top_k={top_k} "
                               f"top_p={top_p} eos={eos}; one step = one whole decode ({R * T} code-steps)",
                   "storage": ldt, "rows": R, "decode_steps": T,
                   "value_with_dispatch_events": code_steps / (t3 - t2),
                   "value_over_a_longer_region": {"steps": long_steps, "value": R * T * long_steps / (t5 - t4),
                                                  "ms_per_step": (t5 - t4) / long_steps * 1e3}},
        "roofline": {
            "kernel": sampling_kernel_name(V, ldt, top_k, top_p, temp),
            "bound": "hbm", "achieved": achieved, "peak": HBM_PEAK_GBS, "unit": "GB/s",
            "frac": (achieved / HBM_PEAK_GBS) if achieved else None, "traffic": None,
            "avg_launch_us": step_avg_us, "launches": step_n, "untimed_launches": step_drop,
            "bytes_per_code_step": bytes_per_row, "active_rows_per_launch": active_rows_per_launch,
            "note": "rows follow the logits GEMM that just wrote them, so part of each row can come from "
                    "the Infinity Cache rather than HBM; see roofline_cold for the HBM-only figure"},
        "logits_gemm": {
            "bound": "mfma", "avg_launch_us": gemm_ms / max(gemm_n, 1) * 1e3, "launches": gemm_n,
            "achieved": (2.0 * R * d * V / (gemm_ms / max(gemm_n, 1) * 1e-3) / 1e12) if gemm_n else None,
            "peak": MFMA_BF16_PEAK_TFLOPS, "unit": "TFLOP/s"},
    }
    if out["logits_gemm"]["achieved"]:
        out["logits_gemm"]["frac"] = out["logits_gemm"]["achieved"] / MFMA_BF16_PEAK_TFLOPS
    out["roofline"]["spread"] = spread(step_samples)
    out["logits_gemm"]["spread"] = spread(gemm_samples)
    if len(step_samples) == T * args.steps and T >= 4:
        # by position in the decode: the first step (every row of a prompt starts from the same token, so the
        # logits rows repeat N times) against the second half (rows have gone their own ways; some have finished)
        by_step = np.asarray(step_samples).reshape(args.steps, T)
        out["roofline"]["first_step"] = spread(by_step[:, 0])
        out["roofline"]["late_steps"] = spread(by_step[:, T // 2:].ravel())
    if thr_n:
        out["threshold_kernel"] = {"avg_launch_us": thr_ms / thr_n * 1e3, "launches": thr_n}

    # ---- the same decode without the logits round trip (no logit modifiers; logits stay fp32 on chip)
    if top_k <= 0 and not (0.0 < top_p < 1.0) and cfg["dtype"] == "bf16" and V <= 32768:
        tokens_f = torch.empty_like(tokens)
        for _ in range(args.warmup):
            B.as_decode_fused(ctx, model, prompts, N, T, u, temp, eos, tokens_f)
        torch.cuda.synchronize()
        f0 = time.perf_counter()
        for _ in range(args.steps):
            B.as_decode_fused(ctx, model, prompts, N, T, u, temp, eos, tokens_f)
        torch.cuda.synchronize()
        f1 = time.perf_counter()
        ctx.profile_read(0); ctx.profile_read(1)
        ctx.profile(True)
        for _ in range(3):
            B.as_decode_fused(ctx, model, prompts, N, T, u, temp, eos, tokens_f)
        fs_ms, fs_n, _ = ctx.profile_read(0)
        fg_ms, fg_n, _ = ctx.profile_read(1)
        ctx.profile(False)
        same = float((tokens_f[:, :, 0] == tokens[:, :, 0]).float().mean().item())
        out["fused_decode"] = {
            "what": "as_decode_fused: logits kernel leaves 8 bytes per 32 logits, sampling kernel recomputes the "
                    "one group its code falls into",
            "value": code_steps / (f1 - f0), "unit": "code-steps/s", "ms_per_step": (f1 - f0) / args.steps * 1e3,
            "logits_kernel_us": fg_ms / max(fg_n, 1) * 1e3, "sampling_kernel_us": fs_ms / max(fs_n, 1) * 1e3,
            "first_tokens_equal_to_unfused_bf16_decode": same}

    # ---- encode direction (sequence -> code interval) over the sequences just decoded
    lo = torch.empty(R, dtype=torch.float64, device="cuda")
    width = torch.empty(R, dtype=torch.float64, device="cuda")
    B.as_encode(ctx, model, prompts, N, T, tokens, temp, top_k, top_p, eos, lo, width)
    torch.cuda.synchronize()
    ctx.profile_read(3)
    ctx.profile(True)
    e0 = time.perf_counter()
    for _ in range(3):
        B.as_encode(ctx, model, prompts, N, T, tokens, temp, top_k, top_p, eos, lo, width)
    torch.cuda.synchronize()
    e1 = time.perf_counter()
    iv_ms, iv_n, _ = ctx.profile_read(3)
    ctx.profile_read(1); ctx.profile_read(2)
    ctx.profile(False)
    iv_us = iv_ms / max(iv_n, 1) * 1e3
    out["encode"] = {
        "kernel": "interval_tile_kernel (the single-tile sampling kernel with a lookup of the given token in place of the search), inside as_encode",
        "avg_launch_us": iv_us, "launches": iv_n, "bound": "hbm",
        "achieved": active_rows_per_launch * bytes_per_row / (iv_us * 1e-6) / 1e9 if iv_n else None,
        "peak": HBM_PEAK_GBS, "unit": "GB/s",
        "code_steps_per_s_with_dispatch_events": code_steps / args.steps * 3 / (e1 - e0)}
    if out["encode"]["achieved"]:
        out["encode"]["frac"] = out["encode"]["achieved"] / HBM_PEAK_GBS

    # ---- ancestral mode (fresh uniforms per step, same kernels) and the lattice estimator over the decoded batch
    uniforms = torch.from_numpy(synth.uniform_codes(T * R, seed=6)).cuda()
    tokens_a = torch.empty_like(tokens)
    B.as_decode_ancestral(ctx, model, prompts, N, T, uniforms, temp, top_k, top_p, eos, tokens_a)
    torch.cuda.synchronize()
    a0 = time.perf_counter()
    for _ in range(3):
        B.as_decode_ancestral(ctx, model, prompts, N, T, uniforms, temp, top_k, top_p, eos, tokens_a)
    torch.cuda.synchronize()
    a1 = time.perf_counter()
    score = torch.linspace(0.0, 1.0, V, dtype=torch.float32, device="cuda")
    est = torch.empty(Bn, dtype=torch.float64, device="cuda")
    B.as_estimate_mean(ctx, tokens, score, eos, est)
    torch.cuda.synchronize()
    m0 = time.perf_counter()
    for _ in range(20):
        B.as_estimate_mean(ctx, tokens, score, eos, est)
    torch.cuda.synchronize()
    m1 = time.perf_counter()
    out["ancestral"] = {
        "what": "as_decode_ancestral (the caller's uniforms[t, r] as codes, kernels unchanged); as_estimate_mean "
                "over the lattice decode's tokens (additive per-token score, fp64, one value per prompt)",
        "value": code_steps / args.steps * 3 / (a1 - a0), "unit": "code-steps/s",
        "estimate_mean_us_per_call": (m1 - m0) / 20 * 1e6}

    if args.copy_calibration:
        src_t = torch.empty(256 * 2 ** 20, dtype=torch.uint8, device="cuda").random_()
        dst_t = torch.empty_like(src_t)
        for _ in range(10):
            dst_t.copy_(src_t)
        torch.cuda.synchronize()
        out["copy_calibration"] = {"bytes_read_per_launch": src_t.numel(), "bytes_written_per_launch": src_t.numel(),
                                   "launches": 10}
        del src_t, dst_t

    # ---- measured HBM traffic of the sampling kernel, if a counter run has been recorded
    traffic_file = os.path.join(os.path.dirname(os.path.abspath(__file__)), "profiles", "step_kernel_traffic.json")
    if os.path.exists(traffic_file) and args.config == 1 and top_k <= 0 and not (0.0 < top_p < 1.0) and ldt == "bf16":
        with open(traffic_file) as f:
            tr = json.load(f)
        # a counter reading of another build of the kernel says nothing about the one timed here
        if tr.get("source_stamp") == source_stamp():
            out["roofline"]["traffic"] = tr.get("traffic_bytes_per_launch")
            out["roofline"]["traffic_source"] = tr.get("source")
        else:
            out["roofline"]["traffic_source"] = ("no counter reading of this build of the kernel is stored "
                                                 "(profiles/step_kernel_traffic.json is of another one)")

    # ---- cold leg: the sampling kernel alone, rotating over > 1 GiB of logits
    if not args.no_cold:
        ld = (V + 7) // 8 * 8
        nbuf = max(2, int(np.ceil((1.25 * 2 ** 30) / (R * ld * esz))))
        bufs = torch.empty((nbuf, R, ld), dtype=tdt, device="cuda")
        prev = prompts.repeat_interleave(N).contiguous()
        for i in range(nbuf):
            # distinct, realistic rows in every buffer: logits of a shifted token set
            B.as_bigram_logits(ctx, model, ((prev + 977 * i) % V).to(torch.int32).contiguous(), bufs[i])
        codes = up(synth.uniform_codes(R, seed=4))
        tok = torch.empty(R, dtype=torch.int32, device="cuda")
        cout = torch.empty(R, dtype=torch.float32, device="cuda")
        torch.cuda.synchronize()
        reps = 8
        for i in range(nbuf):                       # warm-up pass (code, not data: buffers keep rotating)
            B.as_step(ctx, bufs[i], codes, temp, top_k, top_p, tok, cout)
        torch.cuda.synchronize()
        ctx.profile_read(0)
        ctx.profile(True)
        for _ in range(reps):
            for i in range(nbuf):
                B.as_step(ctx, bufs[i], codes, temp, top_k, top_p, tok, cout)
        cold_samples = ctx.profile_samples(0)
        ms, n, _ = ctx.profile_read(0)
        ctx.profile(False)
        us = ms / n * 1e3
        ach = R * bytes_per_row / (us * 1e-6) / 1e9
        out["roofline_cold"] = {
            "spread": spread(cold_samples),
            "kernel": "step_kernel alone, rotating over %d logits buffers (%.2f GiB)" % (
                nbuf, nbuf * R * ld * esz / 2 ** 30),
            "bound": "hbm", "achieved": ach, "peak": HBM_PEAK_GBS, "unit": "GB/s", "frac": ach / HBM_PEAK_GBS,
            "avg_launch_us": us, "launches": n, "code_steps_per_s": R / (us * 1e-6)}
        del bufs

    # ---- the same kernel where a launch is long enough to amortise its fixed costs: 16x the rows, one launch
    # over a 1 GiB logits buffer (nothing of it fits the Infinity Cache by the time it is read again)
    if args.rows16x and args.config == 1:
        Rl = 16 * R
        ld = (V + 7) // 8 * 8
        ctxl = B.Ctx(Rl, V, tdt)
        big = torch.empty((Rl, ld), dtype=tdt, device="cuda")
        prevl = ((prompts.repeat_interleave(N).repeat(16) + 131 * torch.arange(Rl, device="cuda", dtype=torch.int32))
                 % V).to(torch.int32).contiguous()
        B.as_bigram_logits(ctxl, model, prevl, big)
        codesl = up(synth.uniform_codes(Rl, seed=5))
        tokl = torch.empty(Rl, dtype=torch.int32, device="cuda")
        coutl = torch.empty(Rl, dtype=torch.float32, device="cuda")
        for _ in range(3):
            B.as_step(ctxl, big, codesl, temp, top_k, top_p, tokl, coutl)
        torch.cuda.synchronize()
        ctxl.profile_read(0)
        ctxl.profile(True)
        for _ in range(20):
            B.as_step(ctxl, big, codesl, temp, top_k, top_p, tokl, coutl)
        ms, n, _ = ctxl.profile_read(0)
        ctxl.profile(False)
        us = ms / n * 1e3
        ach = Rl * bytes_per_row / (us * 1e-6) / 1e9
        out["roofline_16x_rows"] = {
            "kernel": "step_kernel alone, one launch over %d rows (%.2f GiB of logits)" % (Rl, Rl * ld * esz / 2 ** 30),
            "bound": "hbm", "achieved": ach, "peak": HBM_PEAK_GBS, "unit": "GB/s", "frac": ach / HBM_PEAK_GBS,
            "avg_launch_us": us, "launches": n, "code_steps_per_s": Rl / (us * 1e-6)}
        del big
        ctxl.close()

    # ---- CPU oracle on a bounded sample of the same workload (reported, not a target)
    if not args.no_cpu:
        import oracle
        nthreads = min(os.cpu_count() or 1, int(os.environ.get("OMP_NUM_THREADS", "0") or 0) or (os.cpu_count() or 1))
        ld = (V + 7) // 8 * 8
        prev = prompts.repeat_interleave(N).contiguous()
        logits = torch.empty((R, ld), dtype=tdt, device="cuda")
        B.as_bigram_logits(ctx, model, prev, logits)
        torch.cuda.synchronize()
        stored = logits.view(torch.int16).cpu().numpy().view(np.uint16) if tdt == torch.bfloat16 else logits.cpu().numpy()
        codes = synth.uniform_codes(R, seed=4).astype(np.float64)
        sample_rows = R
        oracle.step(stored[:64], codes[:64], temp=temp, top_k=top_k, top_p=top_p, V=V, nthreads=nthreads)  # warm
        c0 = time.perf_counter()
        reps = 0
        while True:
            oracle.step(stored[:sample_rows], codes[:sample_rows], temp=temp, top_k=top_k, top_p=top_p, V=V,
                        nthreads=nthreads)
            reps += 1
            if time.perf_counter() - c0 > 1.5:
                break
        c1 = time.perf_counter()
        # the same on one thread, over fewer rows
        one_rows = min(R, 64)
        o0 = time.perf_counter()
        one_reps = 0
        while True:
            oracle.step(stored[:one_rows], codes[:one_rows], temp=temp, top_k=top_k, top_p=top_p, V=V, nthreads=1)
            one_reps += 1
            if time.perf_counter() - o0 > 0.5:
                break
        o1 = time.perf_counter()
        out["cpu_baseline"] = {
            "one_thread": {"value": one_rows * one_reps / (o1 - o0), "unit": "code-steps/s",
                           "sample": f"the first {one_rows} rows, {one_reps} repetitions, {o1 - o0:.2f} s"},
            "value": sample_rows * reps / (c1 - c0), "unit": "code-steps/s", "cores": nthreads, "kind": "oracle",
            "sample": f"oracle step (fp64) over the {sample_rows} rows of the first decode step's logits, "
                      f"{reps} repetitions, {nthreads} OpenMP threads, {c1 - c0:.2f} s wall; sampling step "
                      f"only (the oracle's fp64 logits GEMM is not included)"}

    ctx.close()
    model.close()
    del Ed, tokens
    torch.cuda.empty_cache()

    # ---- the other configurations at their full shapes, compactly
    if not args.no_legs and args.config == 1:
        out["other_configs"] = {}
        for name, (cid, k_, p_, n_) in legs.items():
            out["other_configs"][name] = compact_leg(cid, k_, p_, n_, 1)

    print(json.dumps(out))
    return 0


if __name__ == "__main__":
    sys.exit(main())
