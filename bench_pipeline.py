"""Benchmark legs of the split-weight prefetch pipeline workload (4 layers, T=256, 64 resident +
192 staged experts per layer).  Used by bench.py: as the third leg of its default run and as
`--workload pipeline` (with the sweeps: slice size, copy engine, window padding, several pullers)."""
from __future__ import annotations

import sys
import threading
import time

import torch

from paper_2604_01621_amd import binding, inputs, pipeline

HBM_PEAK_GBS = 8000.0
N_LAYERS, N_RESIDENT, N_PEERS = 4, 64, 3


def overlap_fraction(spans):
    """Share of the copy spans' total duration during which some GEMM span is running (the
    timeline view of overlap; it does not say that the copy cost nothing, see hidden_fraction)."""
    gemm = sorted((a, b) for k, _, a, b in spans if k == 1)
    merged = []
    for a, b in gemm:
        if merged and a <= merged[-1][1]:
            merged[-1][1] = max(merged[-1][1], b)
        else:
            merged.append([a, b])
    tot = hid = 0.0
    for k, _, a, b in spans:
        if k != 0:
            continue
        tot += b - a
        for ga, gb in merged:
            lo, hi = max(a, ga), min(b, gb)
            if hi > lo:
                hid += hi - lo
    return (hid / tot if tot > 0 else 0.0), tot


def hidden_fraction(ms_per_layer: float, compute_alone_ms: float, copy_alone_ms: float):
    """(exposed copy time per layer, share of the copy's stand-alone time that the pipeline hides).

    exposed = what a layer costs with the prefetch running beyond what it costs without;
    hidden = 1 - exposed / copy_alone, clipped to [0, 1].  With T = max(T_compute, T_prefetch)
    (paper Section 3) a fully hidden copy has exposed = 0 when compute is the longer of the two."""
    exposed = max(ms_per_layer - compute_alone_ms, 0.0)
    hidden = 1.0 - exposed / copy_alone_ms if copy_alone_ms > 0 else 0.0
    return exposed, min(max(hidden, 0.0), 1.0)


class PipelineRig:
    """Context, split-weight layer stack and per-layer inputs of the pipeline workload."""

    def __init__(self, seed: int, T: int = None, T_max: int = None, copy_engine: int = 1, copy_wgs: int = 65535,
                 slice_bytes: int = 1 << 20, keep_logical_layer0: bool = False, dev=None,
                 n_resident: int = N_RESIDENT, n_peers: int = N_PEERS):
        self.dev = dev or torch.device("cuda:0")
        cfg = inputs.WORKLOADS["pipeline"]
        self.cfg = cfg if T is None else cfg.with_T(T)
        self.seed, self.slice_bytes = seed, slice_bytes
        self.engine, self.copy_wgs = copy_engine, copy_wgs
        self.stream = torch.cuda.Stream()
        self.ctx = binding.Context(self.cfg, n_layers=N_LAYERS, stream=self.stream,
                                   T_max=max(self.cfg.T, T_max or 0))
        self.ctx.dwdp_set_copy_engine(copy_engine, copy_wgs)
        self.n_resident, self.n_peers = n_resident, n_peers
        self.layers = pipeline.SplitWeightLayers(self.ctx, self.cfg, N_LAYERS, n_resident, n_peers, seed=seed,
                                                 device=self.dev)
        if keep_logical_layer0:
            self.layers.logical[1:] = [None] * (N_LAYERS - 1)
        else:
            self.layers.drop_logical()
        torch.cuda.empty_cache()
        self.xs, self.lgs, self.bs, self.ys = [], [], [], []
        for l in range(N_LAYERS):
            x = inputs.make_activations(self.cfg, seed + 10 + l, device=self.dev)
            self.xs.append(x)
            self.lgs.append(inputs.make_gate_logits(self.cfg, x, seed + 10 + l))
            self.bs.append(inputs.make_bias(self.cfg, seed + 10 + l, device=self.dev, kind="small"))
            self.ys.append(torch.empty(self.cfg.T, self.cfg.H, dtype=torch.bfloat16, device=self.dev))
        for l in range(N_LAYERS):      # device plans built here: no allocation inside the timed loops
            src, dst, nb = self.layers.prefetch_args(l)
            self.ctx.dwdp_prepare_prefetch(l, src, dst, nb, n_peers, pipeline.N_PARAMS, slice_bytes)
        torch.cuda.synchronize()

    def set_copy_workgroups(self, n: int):
        self.copy_wgs = n
        self.ctx.dwdp_set_copy_engine(self.engine, n)

    def close(self):
        self.ctx.close()

    def measure(self, steps: int, warmup: int, pad_ms: float = 0.0, merge: bool = False):
        ctx, cfg, layers, stream, dev = self.ctx, self.cfg, self.layers, self.stream, self.dev
        slice_bytes = self.slice_bytes
        if merge:
            # naive baseline of paper Section 4.2: before each layer's GEMMs, copy its resident and staged
            # experts into one contiguous image and run the same kernels on that
            n = cfg.n_slots
            m_w13 = torch.empty(n, 2 * cfg.I, cfg.H, dtype=torch.uint8, device=dev)
            m_s13 = torch.empty(n, 2 * cfg.I // 128, cfg.H // 128, dtype=torch.float32, device=dev)
            m_w2 = torch.empty(n, cfg.H, cfg.I, dtype=torch.uint8, device=dev)
            m_s2 = torch.empty(n, cfg.H // 128, cfg.I // 128, dtype=torch.float32, device=dev)
            tables_host = [t.cpu().contiguous() for t in layers.tables]
            merged_dev = ctx.dwdp_merge_experts(0, tables_host[0], m_w13, m_s13, m_w2, m_s2).to(dev)
            torch.cuda.synchronize()

        # Stand-in for the rest of the compute window of a layer (the paper's window also holds the next
        # layer's attention, Section 3): a spin kernel of one wavefront on the compute stream, no memory traffic.
        pad_cycles = 0
        if pad_ms > 0:
            with torch.cuda.stream(stream):
                probe = 20_000_000
                e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
                torch.cuda._sleep(probe)                      # warm
                e0.record(stream)
                torch.cuda._sleep(probe)
                e1.record(stream)
            torch.cuda.synchronize()
            pad_cycles = int(probe * pad_ms / e0.elapsed_time(e1))

        def forward(l):
            if pad_cycles:
                with torch.cuda.stream(stream):
                    torch.cuda._sleep(pad_cycles)
            if merge:
                ctx.dwdp_merge_experts(l, tables_host[l], m_w13, m_s13, m_w2, m_s2)
                ctx.dwdp_moe_forward(l, self.xs[l], self.lgs[l], self.bs[l], merged_dev, self.ys[l])
            else:
                ctx.dwdp_moe_forward(l, self.xs[l], self.lgs[l], self.bs[l], layers.tables[l], self.ys[l])

        def loop(n_iter, with_prefetch=True):
            # steady state: the prefetch of the next iteration's layer 0 runs under this iteration's last layer
            for it in range(n_iter):
                for l in range(N_LAYERS):
                    if with_prefetch:
                        nxt = (l + 1) % N_LAYERS
                        if not (it == n_iter - 1 and l == N_LAYERS - 1):
                            layers.prefetch(ctx, nxt, slice_bytes)
                    forward(l)

        # compute alone (staging already holds valid experts after one warm pass) and copy alone
        layers.prefetch(ctx, 0, slice_bytes)
        loop(max(warmup, 1))
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        loop(steps, with_prefetch=False)
        torch.cuda.synchronize()
        compute_alone_ms = (time.perf_counter() - t0) * 1e3 / (steps * N_LAYERS)
        n_copy = 4
        y_dummy = torch.empty(0, cfg.H, dtype=torch.bfloat16, device=dev)
        t0 = time.perf_counter()
        for i in range(n_copy):
            layers.prefetch(ctx, i % 2, slice_bytes)
            ctx.dwdp_moe_forward(i % 2, self.xs[0][:0], self.lgs[0][:0], self.bs[0], layers.tables[i % 2], y_dummy)
        torch.cuda.synchronize()
        copy_alone_ms = (time.perf_counter() - t0) * 1e3 / n_copy

        # timed steady-state pipeline
        layers.prefetch(ctx, 0, slice_bytes)
        torch.cuda.synchronize()
        ctx.dwdp_timeline_enable(True)
        ctx.dwdp_profile_enable(True)
        t0 = time.perf_counter()
        loop(steps)
        torch.cuda.synchronize()
        dt = time.perf_counter() - t0
        stage_ms, n_calls = ctx.dwdp_profile_read()
        spans = ctx.dwdp_timeline_read()
        ctx.dwdp_timeline_enable(False)
        ctx.dwdp_profile_enable(False)
        frac, copy_ms_total = overlap_fraction(spans)
        n_copies = sum(1 for s in spans if s[0] == 0)
        ms_per_layer = dt * 1e3 / (steps * N_LAYERS)
        stage_ms = {k: v / max(n_calls, 1) for k, v in stage_ms.items()}
        off = ctx.workspace("offsets", (cfg.E + 2,), torch.int32).cpu().numpy()
        active = int(((off[1:] - off[:-1]) > 0).sum())
        eb = inputs.expert_bytes(cfg)
        pf_bytes = layers.prefetch_bytes()
        exposed, hidden = hidden_fraction(ms_per_layer, compute_alone_ms, copy_alone_ms)
        traffic = active * eb + 2 * pf_bytes       # weights read once by the GEMMs + the copy's read and write
        return {
            "T": cfg.T, "layers": N_LAYERS, "steps": steps, "slice_bytes": slice_bytes,
            "resident_experts": self.n_resident, "peers": self.n_peers,
            "copy_engine": "copy-plan kernel, %d workgroups" % self.copy_wgs if self.engine == 1
            else "hipMemcpyAsync per slice",
            "split_weights": "merged into one contiguous image before every layer (naive baseline)" if merge
            else "read in place through the expert-pointer table",
            "prefetch_bytes_per_layer": pf_bytes, "active_expert_slots": active, "window_pad_ms": pad_ms,
            "ms_per_layer": ms_per_layer, "compute_alone_ms_per_layer": compute_alone_ms,
            "copy_alone_ms_per_layer": copy_alone_ms, "copy_alone_gbs": pf_bytes / (copy_alone_ms * 1e-3) / 1e9,
            "exposed_copy_ms_per_layer": exposed, "hidden_frac": hidden,
            "ideal_ms_per_layer_max_of_both": max(compute_alone_ms, copy_alone_ms),
            "overlap_frac_timeline": frac, "avg_copy_ms": copy_ms_total / max(n_copies, 1), "copies": n_copies,
            "hbm_bytes_per_layer": traffic, "hbm_gbs": traffic / (ms_per_layer * 1e-3) / 1e9,
            "hbm_frac": traffic / (ms_per_layer * 1e-3) / 1e9 / HBM_PEAK_GBS,
            "stage_ms": stage_ms,
        }


def run(args):
    rig = PipelineRig(args.seed, T=args.T, copy_engine=getattr(args, "copy_engine", 1),
                      copy_wgs=getattr(args, "copy_wgs", 65535), slice_bytes=getattr(args, "slice_mib", 1) << 20,
                      n_resident=getattr(args, "resident", N_RESIDENT), n_peers=getattr(args, "peers", N_PEERS))
    if getattr(args, "stream_max_rows", None) is not None:
        rig.ctx.dwdp_set_stream_max_rows(args.stream_max_rows)
    m = rig.measure(args.steps, args.warmup, pad_ms=float(getattr(args, "window_pad_ms", 0.0) or 0.0),
                    merge=bool(getattr(args, "merge_baseline", False)))
    cfg = rig.cfg
    out = {
        "metric": "moe_layer_tokens_per_s", "value": cfg.T / (m["ms_per_layer"] * 1e-3), "unit": "tokens/s",
        "n_gpus": 1, "steps": args.steps, "warmup": args.warmup, "ms_per_step": m["ms_per_layer"] * N_LAYERS,
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None, "dtype": "fp8_e4m3", "data": "synthetic",
        "config": {"workload": "pipeline: 4 DeepSeek-R1-shaped MoE layers, %d resident + %d staged experts each"
                               % (rig.n_resident, cfg.E - rig.n_resident),
                   "T": cfg.T, "layers": N_LAYERS, "slice_bytes": m["slice_bytes"],
                   "active_expert_slots": m["active_expert_slots"], "copy_engine": m["copy_engine"],
                   "split_weights": m["split_weights"], "prefetch_bytes_per_layer": m["prefetch_bytes_per_layer"]},
        "roofline": {"bound": "hbm", "kernel": "whole layer: grouped GEMMs reading every expert once + the next "
                                               "layer's copy (read and write)",
                     "achieved": m["hbm_gbs"], "peak": HBM_PEAK_GBS, "unit": "GB/s", "frac": m["hbm_frac"],
                     "traffic": None, "algorithmic_bytes_per_launch": m["hbm_bytes_per_layer"],
                     "avg_launch_ms": m["ms_per_layer"]},
        "pipeline": m,
    }
    rig.close()
    return out


def run_pullers(args):
    """Several pullers on one source (paper Section 4.3: many-to-one contention and the sliced,
    peer-interleaved copy order of Section 4.3.2), emulated on one GPU: every puller is a context of
    its own (own copy stream, own landing buffer, issued from a host thread of its own) and all
    of them fetch the same layer's non-resident experts from the same pool at the same time.
    Reports, per copy engine, slice size and peer order, when each puller's copies were done."""
    dev = torch.device("cuda:0")
    cfg = inputs.WORKLOADS["pipeline"]
    n_res, n_peers, P = N_RESIDENT, N_PEERS, args.pullers
    ctxs = [binding.Context(cfg, n_layers=1, stream=torch.cuda.Stream()) for _ in range(P)]
    layers = pipeline.SplitWeightLayers(ctxs[0], cfg, 1, n_res, n_peers, seed=args.seed, device=dev)
    layers.drop_logical()
    torch.cuda.empty_cache()
    stagings = [layers.staging[0]] + [layers.new_puller_staging(dev) for _ in range(P - 1)]
    tables = [layers.puller_table(0, st, dev) for st in stagings]
    copy_streams = [torch.cuda.ExternalStream(c.copy_stream_handle()) for c in ctxs]
    x0 = torch.empty(0, cfg.H, dtype=torch.bfloat16, device=dev)
    lg0 = torch.empty(0, cfg.E, dtype=torch.float32, device=dev)
    b0 = inputs.make_bias(cfg, args.seed, device=dev, kind="zero")
    pf_bytes = layers.prefetch_bytes()
    reps = max(2, min(args.steps, 5))

    def one_round(engine, slice_bytes, rotated, active):
        for c in ctxs:
            c.dwdp_set_copy_engine(engine, min(getattr(args, "copy_wgs", 512), 512))
        torch.cuda.synchronize()
        e0 = torch.cuda.Event(enable_timing=True)
        evs = [torch.cuda.Event(enable_timing=True) for _ in range(active)]
        gate = threading.Barrier(active)
        errs = []

        def pull(p):
            try:
                gate.wait()
                layers.puller_prefetch(ctxs[p], 0, stagings[p], slice_bytes, first_peer=(p % n_peers) if rotated else 0)
                evs[p].record(copy_streams[p])
            except Exception as ex:      # surfaced after the join
                errs.append(ex)

        e0.record(torch.cuda.current_stream())
        th = [threading.Thread(target=pull, args=(p,)) for p in range(active)]
        for t in th:
            t.start()
        for t in th:
            t.join()
        if errs:
            raise errs[0]
        for p in range(active):     # T = 0 layer: takes the buffer and releases it for the next round
            ctxs[p].dwdp_moe_forward(0, x0, lg0, b0, tables[p], x0)
        torch.cuda.synchronize()
        return [e0.elapsed_time(ev) for ev in evs]

    rows = []
    for engine in (1, 0):
        for slice_mib in (1, 16, 256):
            for active, rotated in ((1, False), (P, False), (P, True)):
                one_round(engine, slice_mib << 20, rotated, active)     # warm: plans cached, pages touched
                t = [one_round(engine, slice_mib << 20, rotated, active) for _ in range(reps)]
                done = [sum(r[p] for r in t) / reps for p in range(active)]
                rows.append({"copy_engine": "copy-plan kernel" if engine == 1 else "hipMemcpyAsync per slice",
                             "slice_mib": slice_mib, "pullers": active,
                             "peer_order": "rotated per puller" if rotated else "same for all",
                             "done_ms": [round(v, 3) for v in done],
                             "last_done_ms": round(max(done), 3),
                             "spread": round((max(done) - min(done)) / max(done), 3),
                             "aggregate_gbs": round(active * pf_bytes / (max(done) * 1e-3) / 1e9, 1)})
                print(rows[-1], flush=True, file=sys.stderr)
    ref = next(r for r in rows if r["copy_engine"] == "copy-plan kernel" and r["slice_mib"] == 1
               and r["pullers"] == P and r["peer_order"] == "rotated per puller")
    out = {"metric": "multi_puller_prefetch_last_done_ms", "value": ref["last_done_ms"], "unit": "ms", "n_gpus": 1,
           "steps": reps, "warmup": 1, "ms_per_step": ref["last_done_ms"], "higher_is_better": False,
           "scaling": "weak", "vs_baseline": None, "dtype": "u8", "data": "synthetic",
           "config": {"workload": "pipeline layer 0: %d pullers x 192 staged experts from one 3-peer pool" % P,
                      "prefetch_bytes_per_puller": pf_bytes}, "rows": rows}
    for c in ctxs:
        c.close()
    return out
