#!/usr/bin/env python3
"""Benchmark of the DWDP MoE-layer hot path on one MI355X.

A step is one dwdp_moe_forward (route -> permute -> quantise -> grouped GEMM gate/up+SwiGLU
-> grouped GEMM down -> combine) over one batch of seeded synthetic tokens with all inputs
and weights resident in HBM.  Default workload: the DeepSeek-R1-shaped decode layer, T=64.
Prints ONE JSON line (see the fields below); `roofline` is for the dominant kernel measured
with HIP events on the compute stream inside the timed region; `cpu_baseline` is the CPU
oracle timed on a bounded sample of the same workload on this host.
"""
import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0        # MI355X HBM3E, published
FP8_PEAK_TFLOPS = 5000.0     # MI355X dense FP8 MFMA, published
# HBM bytes per launch of the dominant kernel from the committed rocprofv3 counter runs (profiles/:
# FETCH_SIZE x 2.0 + WRITE_SIZE, calibrated against a 1 GiB copy), keyed by (workload, seed, T); None
# when this configuration was not profiled.
PROFILED_TRAFFIC = {("decode", 1, 64): (2325711 * 2 + 1238) * 1024,
                    ("prefill", 1, 8192): (4361665 * 2 + 152102) * 1024}


def parse():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=50)
    ap.add_argument("--warmup", type=int, default=10)
    ap.add_argument("--workload", default="decode", choices=["decode", "prefill", "skew", "pipeline", "tiny"])
    ap.add_argument("--T", type=int, default=None, help="override the workload's token count")
    ap.add_argument("--seed", type=int, default=1)
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--cpu-sample-tokens", type=int, default=16,
                    help="tokens of the workload the CPU oracle is timed on (about 10-20 s of host work at 16)")
    ap.add_argument("--slice-mib", type=int, default=1, help="pipeline workload: prefetch slice size in MiB")
    ap.add_argument("--stream-max-rows", type=int, default=None,
                    help="override the library's kernel-selection threshold (dwdp_set_stream_max_rows)")
    ap.add_argument("--copy-engine", type=int, default=1, help="pipeline workload: 0 hipMemcpyAsync per slice, "
                                                               "1 copy-plan kernel")
    ap.add_argument("--copy-wgs", type=int, default=512, help="pipeline workload: workgroups of the copy-plan kernel")
    ap.add_argument("--weights", default="fp8", choices=["fp8", "mxfp4"],
                    help="expert weight format of the decode/prefill/skew workloads: block-scaled FP8 (the "
                         "headline configuration) or MXFP4 (FP4 codes with a power-of-two scale per 32)")
    ap.add_argument("--window-pad-ms", type=float, default=0.0,
                    help="pipeline workload: extra compute per layer (a spin kernel on the compute stream) standing "
                         "in for the attention that shares the paper's compute window")
    ap.add_argument("--pullers", type=int, default=1,
                    help="pipeline workload: with N > 1, time N contexts (stand-ins for N ranks) that pull the "
                         "same layer from the same source pool at once, over slice sizes and both copy engines")
    ap.add_argument("--merge-baseline", action="store_true",
                    help="pipeline workload: merge resident and staged experts into one contiguous image before "
                         "every layer (the naive split-weight baseline) instead of reading them in place")
    ap.add_argument("--calib-copy-mib", type=int, default=0,
                    help="after the timed region run one plain device copy of this many MiB (a known-size "
                         "reference dispatch for scaling rocprofv3 FETCH_SIZE / WRITE_SIZE counters)")
    return ap.parse_args()


def cpu_baseline(cfg, x, logits, bias, w, n_tok):
    """Time the oracle (as it stands) on the first n_tok tokens of the workload."""
    import numpy as np
    from oracle import moe_oracle as mo
    try:
        from threadpoolctl import threadpool_info
        cores = max([p.get("num_threads", 1) for p in threadpool_info()] or [1])
    except Exception:
        cores = 1
    spec = mo.spec_from(cfg)
    lg = logits.float().cpu().numpy()
    bs = None if bias is None else bias.float().cpu().numpy()
    xs = x.float().cpu().numpy()
    ids, _ = mo.route(lg[:n_tok], bs, spec)
    need = sorted(set(int(e) for e in ids.reshape(-1)) | ({cfg.E} if cfg.has_shared else set()))
    ex = [None] * w.n
    for e in need:     # host copies of the bytes are input staging, not oracle work
        if w.s13 is None:
            ex[e] = mo.ExpertNumpy(w.w13[e].float().cpu().numpy(), w.w2[e].float().cpu().numpy())
        else:
            ex[e] = mo.ExpertNumpy(w.w13[e].cpu().numpy(), w.w2[e].cpu().numpy(), w.s13[e].cpu().numpy(),
                                   w.s2[e].cpu().numpy())
    t0 = time.perf_counter()
    ref = mo.moe_forward(xs[:n_tok], lg[:n_tok], bs, ex, spec)
    dt = time.perf_counter() - t0
    return {"value": n_tok / dt, "unit": "tokens/s", "cores": int(cores), "kind": "oracle",
            "sample": f"first {n_tok} tokens of the workload ({len(need)} experts dequantised), {dt:.1f} s"}, ref


def main():
    args = parse()
    if args.gpus != 1:
        print("bench.py measures one GPU: this build has no multi-GPU path (run with --gpus 1)", file=sys.stderr)
        sys.exit(2)
    import torch
    from paper_2604_01621_amd import binding, inputs

    assert torch.cuda.is_available(), "bench.py needs a GPU"
    dev = torch.device("cuda:0")
    torch.cuda.set_device(dev)

    if args.workload == "pipeline":
        from paper_2604_01621_amd import pipeline_bench
        out = pipeline_bench.run_pullers(args) if args.pullers > 1 else pipeline_bench.run(args)
        print(json.dumps(out))
        return

    cfg, x, logits, bias = inputs.make_layer_inputs(args.workload, args.seed, device=dev, T=args.T)
    if args.weights == "mxfp4" and cfg.w_dtype == inputs.W_FP8:
        import dataclasses
        cfg = dataclasses.replace(cfg, w_dtype=inputs.W_MXFP4)
    w = inputs.make_expert_weights(cfg, args.seed, device=dev)
    stream = torch.cuda.Stream()
    ctx = binding.Context(cfg, stream=stream)
    if args.stream_max_rows is not None:
        ctx.dwdp_set_stream_max_rows(args.stream_max_rows)
    wp = ctx.pack_experts(w)          # one-off weight preparation, outside the timed region
    table = binding.expert_table(wp)
    y = torch.empty(cfg.T, cfg.H, dtype=torch.bfloat16, device=dev)
    torch.cuda.synchronize()

    for _ in range(args.warmup):
        ctx.dwdp_moe_forward(0, x, logits, bias, table, y)
    torch.cuda.synchronize()
    ctx.dwdp_profile_enable(True)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(args.steps):
        ctx.dwdp_moe_forward(0, x, logits, bias, table, y)
    torch.cuda.synchronize()
    dt = time.perf_counter() - t0
    stage_ms, n_calls = ctx.dwdp_profile_read()
    ctx.dwdp_profile_enable(False)
    stage_ms = {k: v / max(n_calls, 1) for k, v in stage_ms.items()}

    if args.calib_copy_mib > 0:
        src = torch.ones(args.calib_copy_mib << 20, dtype=torch.uint8, device=dev)
        dst = torch.empty_like(src)
        torch.cuda.synchronize()
        dst.copy_(src)
        torch.cuda.synchronize()
        del src, dst

    n_off = cfg.E + 1 + cfg.has_shared
    off = ctx.workspace("offsets", (n_off,), torch.int32).cpu().numpy()
    counts = off[1:] - off[:-1]
    active = int((counts > 0).sum())
    pairs = int(counts.sum())
    ms_per_step = dt / args.steps * 1e3

    fp8 = cfg.w_dtype == inputs.W_FP8
    mx = cfg.w_dtype == inputs.W_MXFP4
    el = 1 if fp8 else 2
    if mx:      # packed codes + packed scales as the kernels read them
        b13 = 2 * cfg.I * cfg.H // 2 + binding.mx_scale_bytes(2 * cfg.I, cfg.H)
        b2 = cfg.H * cfg.I // 2 + binding.mx_scale_bytes(cfg.H, cfg.I)
    else:
        b13 = 2 * cfg.I * cfg.H * el + (4 * (2 * cfg.I // 128) * (cfg.H // 128) if fp8 else 0)
        b2 = cfg.H * cfg.I * el + (4 * (cfg.H // 128) * (cfg.I // 128) if fp8 else 0)
    # which kernel family serves which expert (the library's default threshold: 16 rows)
    smr = args.stream_max_rows if args.stream_max_rows is not None else 16
    if not (fp8 or mx) or cfg.T <= smr:
        smr = 1 << 30
    n_stream = int(((counts > 0) & (counts <= smr)).sum())
    n_tile = int((counts > smr).sum())
    rows_tile = int(counts[counts > smr].sum())

    def roofline(stage_stream, stage_tile, bytes_per_expert, flops_per_row, label):
        """Roofline entry for the kernel family that does most of one GEMM stage's work."""
        t_s, t_t = stage_ms[stage_stream], stage_ms.get(stage_tile, 0.0)
        tile = n_tile > n_stream          # the family that serves more experts does more of the work
        t = t_t if tile else t_s
        n_exp = n_tile if tile else n_stream
        kern = ("LDS-tiled " if tile else "weight-streaming ") + label
        compute_bound = tile and rows_tile / max(n_tile, 1) >= 128
        if compute_bound:
            ach = rows_tile * flops_per_row / (t * 1e-3) / 1e12
            # the same launch against the HBM roofline: every listed expert's weights read once
            hbm = n_tile * bytes_per_expert / (t * 1e-3) / 1e9
            return {"bound": "mfma", "kernel": kern, "achieved": ach, "peak": FP8_PEAK_TFLOPS, "unit": "TFLOP/s",
                    "frac": ach / FP8_PEAK_TFLOPS, "traffic": None,
                    "algorithmic_flops_per_launch": rows_tile * flops_per_row, "avg_launch_ms": t,
                    "hbm_read_once_gbs": hbm, "hbm_frac": hbm / HBM_PEAK_GBS}
        ach = n_exp * bytes_per_expert / (t * 1e-3) / 1e9
        return {"bound": "hbm", "kernel": kern, "achieved": ach, "peak": HBM_PEAK_GBS, "unit": "GB/s",
                "frac": ach / HBM_PEAK_GBS, "traffic": None, "algorithmic_bytes_per_launch": n_exp * bytes_per_expert,
                "experts_in_launch": n_exp, "avg_launch_ms": t}

    roof = roofline("gemm1", "gemm1_tile", b13, 2 * 2 * cfg.I * cfg.H, "GEMM-1 (gate/up + SwiGLU)")
    roof2 = roofline("gemm2", "gemm2_tile", b2, 2 * cfg.I * cfg.H, "GEMM-2 (down)")
    if args.stream_max_rows is None and not mx:
        roof["traffic"] = PROFILED_TRAFFIC.get((args.workload, args.seed, cfg.T))

    out = {
        "metric": "moe_layer_tokens_per_s", "value": cfg.T / (ms_per_step * 1e-3), "unit": "tokens/s",
        "n_gpus": 1, "steps": args.steps, "warmup": args.warmup, "ms_per_step": ms_per_step,
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "fp8_e4m3" if fp8 else ("mxfp4 weights x fp8_e4m3 activations" if mx else "bf16"), "data": "synthetic",
        "config": {"workload": f"{args.workload}: DeepSeek-R1-shaped MoE layer" if args.workload != "tiny"
                   else "tiny bf16 MoE layer", "T": cfg.T, "H": cfg.H, "I": cfg.I, "E": cfg.E, "K": cfg.K,
                   "shared_experts": cfg.has_shared, "active_expert_slots": active, "token_expert_pairs": pairs,
                   "weights": "FP8 e4m3 + fp32 128x128 block scales, all resident" if fp8 else
                   ("MXFP4 (E2M1 + E8M0 per 32), all resident" if mx else "bf16, all resident")},
        "roofline": roof, "roofline_gemm2": roof2, "stage_ms": stage_ms,
        "experts_streamed": n_stream, "experts_tiled": n_tile,
        "layer_weight_gbs": active * (b13 + b2) / (ms_per_step * 1e-3) / 1e9,
    }
    if not args.no_cpu_baseline:
        n_tok = min(args.cpu_sample_tokens, cfg.T)
        cb, ref = cpu_baseline(cfg, x, logits, bias, w, n_tok)
        out["cpu_baseline"] = cb
        from oracle import moe_oracle as mo
        err, l2 = mo.error_metrics(y[:n_tok].float().cpu().numpy(), ref)
        out["sample_max_rel_err"] = err
    print(json.dumps(out))
    ctx.close()


if __name__ == "__main__":
    main()
