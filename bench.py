#!/usr/bin/env python3
"""Benchmark of the PVF round on one MI355X.

A "step" is one PVF round: one batched forward over the backbone canvas and its live drafts,
followed by the decision epilogue (stage 1 over the window logits, stage 2 verify / commit /
propose).  The default workload is the LLaDA-8B-shaped bf16 random-init model, batch 1,
256 prompt + 256 masked tokens, block 32, tau_high 0.9, K = 4, planning vocabulary 512 ids
(third entry of the benchmark's configs).  Weights and prompts are generated on the device
before the timed region, so every input is resident in HBM when timing starts; the timed rounds
decode eight seeded prompts one after the other (a finished canvas is followed by the next prompt).

Prints ONE JSON line.  `value` = tokens committed during the timed rounds / wall time.
Extra objects:
  roofline           dominant kernel (bf16 MFMA GEMM): algorithmic FLOPs / HIP-event time summed
                     over every GEMM launch of the timed rounds, against 2.5 PFLOP/s
  roofline_epilogue  stage 1 on bf16 logits [8 x 256, 126464] (second entry of configs), rotating
                     over 4 buffers (2 GB) so that the 256 MB cache cannot serve repeats
  cpu_baseline       the CPU oracle timed on this host on a bounded sample and extrapolated
  threshold_decoding the same library with K = 0 (confidence-threshold decoding) for the ratios
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

PEAK_BF16_TFLOPS = 2500.0      # MI355X dense bf16 MFMA
PEAK_HBM_GBS = 8000.0          # MI355X HBM3E
LOGIT_SCALE = 12.0             # calibrated once: K=0 decoding of this model lands at 4.6 tokens/forward,
                               # inside the 3.5-6.4 range the paper's confidence-threshold baseline shows
# HBM-side bytes per launch (L2 fills + write-backs) from rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE passes over
# this script, scaled by what the counters read for a plain 256 MiB copy; the passes and the arithmetic are in
# profiles/bench_c3_llada8b_pmc_hbm_traffic.txt
TRAFFIC_GEMM = 412.0e6         # mean over the GEMM launches of the timed mix (algorithmic: 179.4e6)
TRAFFIC_STAGE1 = 518.5e6       # [2048, 126464] bf16 logits (algorithmic: 518.0e6)


# full-batch forwards: sequences per forward, canvas length, window rows per canvas
FULL_BATCH = {"c3_5x512": (5, 512, 64), "c4_9x1280": (9, 1280, 128), "c5_80x1024": (80, 1024, 64)}


def parse():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=240)
    ap.add_argument("--warmup", type=int, default=5)
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-epilogue", action="store_true")
    ap.add_argument("--no-decodes", action="store_true",
                    help="only the timed rounds and the stage-1 measurement: skip the whole decodes (PVF, K = 0, with and "
                         "without K/V cache) and the full-batch forward timing; used for profiling runs")
    ap.add_argument("--all-configs", action="store_true",
                    help="also time one full-batch forward of the 9 x 1280 and 80 x 1024 configurations")
    ap.add_argument("--forward-only", choices=sorted(FULL_BATCH), default=None,
                    help="time nothing but min(--steps, 20) full-batch forwards of the named configuration and print that figure "
                         "(one JSON line); used for profiling runs of the larger configurations")
    ap.add_argument("--pmc-reference", action="store_true",
                    help="also run a plain device-to-device copy of 256 MiB (reference for scaling "
                         "rocprofv3 FETCH_SIZE / WRITE_SIZE readings)")
    return ap.parse_args()


def timed_rounds(ctx, B, cfg, prompts, bitmap, steps, warmup, torch):
    """Runs warmup + steps rounds of a continuing decode; a finished canvas is followed by the next prompt
    of the list (a random model's trajectory, hence its tokens per round, varies a lot from prompt to prompt)."""
    st = B.State(1, cfg)
    ctx.state_init(st, prompts[0])
    n_seq, which = 1, 0

    def one_round():
        nonlocal n_seq, which
        ctx.round(st, bitmap, n_seq)
        nd, dn, nc = st.n_drafts.cpu(), st.done.cpu(), st.n_commit.cpu()      # per-round status read-back
        committed = int(nc.sum())
        used = n_seq
        if int(dn[0]):
            which = (which + 1) % len(prompts)
            ctx.state_init(st, prompts[which])
            n_seq = 1
        else:
            n_seq = 1 + int(nd[0])
        return committed, used

    for _ in range(warmup):
        one_round()
    torch.cuda.synchronize()
    ctx.profile_begin()
    t0 = time.perf_counter()
    tokens = seqs = 0
    for _ in range(steps):
        c, u = one_round()
        tokens += c
        seqs += u
    torch.cuda.synchronize()
    dt = time.perf_counter() - t0
    prof = ctx.profile_end()
    return dt, tokens, seqs, prof


def epilogue_roofline(B, torch, iters=24):
    import numpy as np
    V, rows, mask_id = 126464, 8 * 256, 126336
    bufs = []
    for i in range(4):
        t = torch.empty(rows, V, dtype=torch.bfloat16, device="cuda")
        B.fill_normal(t, 1234 + i, 0.0, 1.0)
        bufs.append(t)
    conf = torch.empty(rows, dtype=torch.float32, device="cuda")
    tok = torch.empty(rows, dtype=torch.int32, device="cuda")
    for b in bufs:
        B.stage1(b, mask_id, 1.0, conf, tok)
    torch.cuda.synchronize()
    us = []
    for it in range(iters // 4):
        # four back-to-back launches (one per buffer) between a pair of events on the launch stream,
        # so that the host's submission latency is not charged to the kernel
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record()
        for b in bufs:
            B.stage1(b, mask_id, 1.0, conf, tok)              # launched on torch's current stream
        e1.record()
        torch.cuda.synchronize()
        us.append(e0.elapsed_time(e1) * 1e3 / len(bufs))
    us = np.array(us)
    algo = rows * V * 2 + rows * 8
    ach = algo / (us.mean() * 1e-6) / 1e9
    return {"kernel": "stage1_vec_kernel<bf16>", "workload": "bf16 logits [8x256, 126464], threshold 0.9",
            "bound": "hbm", "achieved": round(ach, 1), "peak": PEAK_HBM_GBS, "unit": "GB/s",
            "frac": round(ach / PEAK_HBM_GBS, 4), "traffic": TRAFFIC_STAGE1,
            "us_mean": round(float(us.mean()), 2), "us_median": round(float(np.median(us)), 2),
            "us_min": round(float(us.min()), 2), "us_p90": round(float(np.percentile(us, 90)), 2),
            "algorithmic_bytes": algo, "launches": iters}


def cpu_baseline(dims, T, R, canv_per_round, tpf, threads):
    """Times the oracle on a bounded sample: one transformer layer of one T-token canvas at the
    full widths plus the output head and stage 1 on the R window rows; extrapolates to a round."""
    import numpy as np
    from oracle import pvf_oracle as O
    from synth import inputs as S
    small_vocab = 4096                                     # embedding rows actually indexed by the sample
    shape = S.ModelShape(n_layers=1, d_model=dims["d_model"], n_heads=dims["n_heads"], d_ff=dims["d_ff"],
                         vocab=small_vocab, mask_id=small_vocab - 1, rope_theta=dims["rope_theta"])
    w = S.make_weights(shape, seed=7)
    rng = np.random.default_rng(8)
    w["out_head"] = rng.standard_normal((dims["vocab"], dims["d_model"]), dtype=np.float32) * np.float32(0.02)
    tokens = S.make_prompt(9, T, small_vocab, small_vocab - 1)
    tokens[T // 2:] = small_vocab - 1
    rows = np.arange(T - R, T)
    mc1 = O.ModelCfg(1, shape.d_model, shape.n_heads, shape.d_ff, dims["vocab"], dims["mask_id"], shape.rms_eps, shape.rope_theta)
    mc0 = O.ModelCfg(0, shape.d_model, shape.n_heads, shape.d_ff, dims["vocab"], dims["mask_id"], shape.rms_eps, shape.rope_theta)
    t0 = time.perf_counter(); O.forward_hidden(tokens, w, mc1); t_layer = time.perf_counter() - t0
    t0 = time.perf_counter(); lg = O.forward(tokens, w, mc0, rows=rows); t_head = time.perf_counter() - t0
    t0 = time.perf_counter(); O.stage1(lg, LOGIT_SCALE, dims["mask_id"]); t_s1 = time.perf_counter() - t0
    t_canvas = t_head + dims["n_layers"] * t_layer + t_s1
    t_round = canv_per_round * t_canvas
    return {"value": round(tpf / t_round, 4), "unit": "tokens/s", "cores": threads, "kind": "oracle",
            "sample": f"oracle.forward on one {T}-token canvas with 1 of {dims['n_layers']} layers at full width "
                      f"({t_layer:.2f} s) + final norm, output head on {R} rows ({t_head:.2f} s) and stage 1 "
                      f"({t_s1:.3f} s); extrapolated x{dims['n_layers']} layers x {canv_per_round:.2f} canvases "
                      f"per round at the measured tokens per round ({tpf:.2f})",
            "seconds_per_round_extrapolated": round(t_round, 2)}


def forward_full_batch(ctx, W, dims, S, T, R, torch, iters):
    """One forward over S full canvases (every draft slot live): ms, TFLOP/s and share of the bf16 peak."""
    tokens = W.random_prompts(S, T, dims["vocab"], dims["mask_id"], seed=7)
    rows = torch.arange(T - R, T, dtype=torch.int32, device="cuda")[None].repeat(S, 1).contiguous()
    for _ in range(2):
        ctx.forward(tokens, rows)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(iters):
        ctx.forward(tokens, rows)
    torch.cuda.synchronize()
    dt = (time.perf_counter() - t0) / iters
    fl = W.flops_per_round(dims, S, T, R)
    return {"ms": round(dt * 1e3, 2), "tflops": round(fl / dt / 1e12, 1), "frac_of_bf16_peak": round(fl / dt / 1e12 / PEAK_BF16_TFLOPS, 4)}


def main():
    a = parse()
    if a.gpus != 1:
        print("bench.py: this build runs on one GPU only (no collectives, no sharding); use --gpus 1", file=sys.stderr)
        sys.exit(2)
    import torch
    from paper_2601_12247_amd import binding as B, workloads as W
    if not torch.cuda.is_available():
        print("bench.py: no GPU visible", file=sys.stderr)
        sys.exit(1)
    B.lib()                                                 # fails loudly if libpvf.so is missing
    dims = dict(W.LLADA_8B)
    K, bl, P, Gn = 4, 32, 256, 256
    T, R = P + Gn, 2 * bl
    weights = W.random_model(dims, seed=0)
    if a.forward_only:
        S_, T_, R_ = FULL_BATCH[a.forward_only]
        c2 = W.make_context(dims, weights, max_seqs=S_, max_T=T_, max_rows=R_)
        print(json.dumps({"forward_full_batch": {a.forward_only: forward_full_batch(c2, W, dims, S_, T_, R_, torch, min(a.steps, 20))}}))
        return
    ctx = W.make_context(dims, weights, max_seqs=1 + K, max_T=T, max_rows=R)
    prompts = [W.random_prompts(1, P, dims["vocab"], dims["mask_id"], seed=1 + i) for i in range(8)]
    n_dec = 4                                               # whole decodes per setting for the TPF / NFE figures
    bitmap = W.random_plan_bitmap(512, dims["vocab"], dims["mask_id"], seed=2)
    cfg = B.DecodeCfg(block_len=bl, prompt_len=P, gen_len=Gn, K=K, tau_high=0.9, logit_scale=LOGIT_SCALE)
    torch.cuda.synchronize()

    dt, tokens, seqs, prof = timed_rounds(ctx, B, cfg, prompts, bitmap, a.steps, a.warmup, torch)
    g = prof["gemm"]
    gemm_tflops = g["flops"] / (g["ms"] * 1e-3) / 1e12 if g["ms"] else 0.0
    tpf = tokens / a.steps
    flops_total = W.flops_per_round(dims, 1, T, R) * seqs          # per canvas x canvases forwarded

    # whole decodes of the first n_dec prompts for TPF / NFE, PVF and K = 0
    def decode_all(c, warm=False):
        tot = {"rounds": 0, "ms": 0.0, "seqs": 0, "base": 0, "plan": 0, "ar": 0}
        for pr in prompts[:n_dec]:
            if warm:
                ctx.decode(B.State(1, c), pr, bitmap)                       # cache allocation, tile shapes
            out, st_ = ctx.decode(B.State(1, c), pr, bitmap)
            assert int((out == dims["mask_id"]).sum()) == 0
            tot["rounds"] += st_.rounds; tot["ms"] += st_.ms_total; tot["seqs"] += st_.seq_forwards
            tot["base"] += st_.n_base; tot["plan"] += st_.n_plan; tot["ar"] += st_.n_ar
        return tot

    s_pvf = s_thr = None
    if not a.no_decodes:
        s_pvf = decode_all(cfg)
        s_thr = decode_all(B.DecodeCfg(block_len=bl, prompt_len=P, gen_len=Gn, K=0, tau_high=0.9, logit_scale=LOGIT_SCALE))

    res = {
        "metric": "committed_tokens_per_s", "value": round(tokens / dt, 2), "unit": "tokens/s",
        "n_gpus": 1, "steps": a.steps, "warmup": a.warmup, "ms_per_step": round(dt / a.steps * 1e3, 3),
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None, "dtype": "bf16", "data": "synthetic",
        "config": {"workload": "LLaDA-8B-shaped random-init bf16 denoiser (32 layers, d 4096, 32 heads, ff 12288, "
                               "vocab 126464), batch 1, prompt 256 + 256 masked, block 32, tau_high 0.9, K=4, "
                               "planning vocabulary 512 ids, full-canvas forward (no KV cache)",
                   "logit_scale": LOGIT_SCALE, "tau_plan": [cfg.tau_plan_lo, cfg.tau_plan_hi], "tau_ar": cfg.tau_ar_lo},
        "tokens_per_forward": round(tpf, 3), "forwards_per_s": round(a.steps / dt, 3),
        "canvases_per_forward": round(seqs / a.steps, 3),
        "forward_tflops_whole_round": round(flops_total / dt / 1e12, 1),
        "roofline": {"kernel": "gemm_bf16_mfma_kernel", "bound": "mfma", "achieved": round(gemm_tflops, 1),
                     "peak": PEAK_BF16_TFLOPS, "unit": "TFLOP/s", "frac": round(gemm_tflops / PEAK_BF16_TFLOPS, 4),
                     "traffic": TRAFFIC_GEMM, "launches": int(g["launches"]),
                     "avg_launch_us": round(g["ms"] * 1e3 / max(1, g["launches"]), 2),
                     "algorithmic_flops_per_launch": round(g["flops"] / max(1, g["launches"])),
                     "algorithmic_bytes_per_launch": round(g["bytes"] / max(1, g["launches"])),
                     "gemm_share_of_step_time": round(g["ms"] * 1e-3 / dt, 4),
                     "attention_tflops": round(prof["attention"]["flops"] / max(prof["attention"]["ms"], 1e-9) / 1e9, 1),
                     "stage1_gbs_in_round": round(prof["stage1"]["bytes"] / max(prof["stage1"]["ms"], 1e-9) / 1e6, 1)},
        "paper_context": "paper: up to 2.3x tokens/s over confidence-threshold decoding on LLaDA-8B-Instruct, "
                         "one NVIDIA H200, trained weights, KV cache; not comparable with random-init weights",
    }
    if s_pvf is not None:
        gen = n_dec * Gn
        res.update({
        "pvf_decode": {"prompts": n_dec, "nfe": s_pvf["rounds"], "tokens_per_forward": round(gen / s_pvf["rounds"], 3),
                       "tokens_per_s": round(gen / s_pvf["ms"] * 1e3, 2), "canvases_forwarded": s_pvf["seqs"],
                       "committed_by_threshold": s_pvf["base"], "by_planning": s_pvf["plan"], "by_ar": s_pvf["ar"]},
        "threshold_decoding": {"prompts": n_dec, "nfe": s_thr["rounds"], "tokens_per_forward": round(gen / s_thr["rounds"], 3),
                               "tokens_per_s": round(gen / s_thr["ms"] * 1e3, 2)}})
        res["pvf_vs_threshold"] = {"tpf_ratio": round(s_thr["rounds"] / s_pvf["rounds"], 3),
                                   "tokens_per_s_ratio": round(res["pvf_decode"]["tokens_per_s"] /
                                                               res["threshold_decoding"]["tokens_per_s"], 3)}
        # the same decodes with the block-level K/V cache (the setting of the paper's tokens/s; approximate)
        kv = {}
        for name, k in (("pvf", K), ("threshold", 0)):
            c = B.DecodeCfg(block_len=bl, prompt_len=P, gen_len=Gn, K=k, tau_high=0.9, logit_scale=LOGIT_SCALE, kv_cache=1)
            s_kv = decode_all(c, warm=(name == "pvf"))
            kv[name] = {"prompts": n_dec, "nfe": s_kv["rounds"], "tokens_per_s": round(gen / s_kv["ms"] * 1e3, 2),
                        "ms_per_round": round(s_kv["ms"] / s_kv["rounds"], 3), "canvases_forwarded": s_kv["seqs"]}
        res["kv_cache_decode"] = kv
    if not a.no_decodes:
        res["forward_full_batch"] = {"c3_5x512": forward_full_batch(ctx, W, dims, 1 + K, T, R, torch, 10)}
    if a.all_configs and not a.no_decodes:
        del ctx
        torch.cuda.empty_cache()
        for name in ("c4_9x1280", "c5_80x1024"):
            S_, T_, R_ = FULL_BATCH[name]
            c2 = W.make_context(dims, weights, max_seqs=S_, max_T=T_, max_rows=R_)
            res["forward_full_batch"][name] = forward_full_batch(c2, W, dims, S_, T_, R_, torch, 3)
            del c2
            torch.cuda.empty_cache()
        ctx = None
    if not a.no_epilogue:
        res["roofline_epilogue"] = epilogue_roofline(B, torch)
    if not a.no_cpu_baseline:
        try:
            from threadpoolctl import threadpool_info
            threads = max([p.get("num_threads", 1) for p in threadpool_info()] + [1])
        except Exception:
            threads = os.cpu_count() or 1
        res["cpu_baseline"] = cpu_baseline(dims, T, R, seqs / a.steps, tpf, threads)
    if a.pmc_reference:
        src = torch.empty(256 * 1024 * 1024 // 2, dtype=torch.bfloat16, device="cuda")
        B.fill_normal(src, 99, 0.0, 1.0)
        dst = torch.empty_like(src)
        for _ in range(3):
            dst.copy_(src)
        torch.cuda.synchronize()
    print(json.dumps(res))


if __name__ == "__main__":
    main()
