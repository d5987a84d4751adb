"""GPU tests of the split-weight prefetch pipeline (paper Section 2 double buffering,
Section 4.2 multi-buffer grouped GEMM): results must not depend on where an expert lives,
a layer must never read a staging buffer before its copies have landed, and a staging
buffer must not be overwritten before its reader is done."""
import numpy as np
import pytest
import torch

from oracle import moe_oracle as mo
from oracle import prefetch_oracle as po
from paper_2604_01621_amd import inputs
from tests.util import experts_numpy, row_tolerance, to_np, tolerance

pytestmark = pytest.mark.gpu

N_LAYERS, N_RES, N_PEERS = 4, 4, 3


@pytest.fixture(scope="module")
def env(gpu_device):
    from paper_2604_01621_amd import binding, pipeline
    cfg = inputs.small_fp8_layer(T=24)
    ctx = binding.Context(cfg, n_layers=N_LAYERS)
    layers = pipeline.SplitWeightLayers(ctx, cfg, N_LAYERS, N_RES, N_PEERS, seed=100)
    xs, lgs, bs = [], [], []
    for l in range(N_LAYERS):
        x = inputs.make_activations(cfg, 200 + l)
        xs.append(x.cuda())
        lgs.append(inputs.make_gate_logits(cfg, x, 200 + l).cuda())
        bs.append(inputs.make_bias(cfg, 200 + l, kind="small").cuda())
    yield binding, pipeline, cfg, ctx, layers, xs, lgs, bs
    ctx.close()


def _reference_outputs(ctx, cfg, layers, xs, lgs, bs):
    """Every layer computed with a table that reads the peer pool in place (no staging)."""
    out = []
    for l in range(N_LAYERS):
        y = torch.empty(cfg.T, cfg.H, dtype=torch.bfloat16, device="cuda")
        ctx.dwdp_moe_forward(l, xs[l], lgs[l], bs[l], layers.all_resident_table(l), y)
        torch.cuda.synchronize()
        out.append(y)
    return out


@pytest.mark.parametrize("engine", [0, 1])
@pytest.mark.parametrize("slice_bytes", [0, 4096, 100000, 1000])
def test_pipeline_poisoned_and_delayed(env, slice_bytes, engine):
    binding, pipeline, cfg, ctx, layers, xs, lgs, bs = env
    print("pipeline slice", slice_bytes, "engine", engine, flush=True)
    ctx.dwdp_set_copy_engine(engine, 24)
    ref = _reference_outputs(ctx, cfg, layers, xs, lgs, bs)
    copy_stream = torch.cuda.ExternalStream(ctx.copy_stream_handle())
    ys = [[torch.empty(cfg.T, cfg.H, dtype=torch.bfloat16, device="cuda") for _ in range(N_LAYERS)] for _ in range(2)]
    for b in range(2):
        layers.poison_staging(b)
    torch.cuda.synchronize()
    done = {}

    def poison_then_prefetch(l, it):
        b = l % 2
        prev = done.get(b)
        with torch.cuda.stream(copy_stream):
            if prev is not None:
                copy_stream.wait_event(prev)      # the test's own ordering for its poison writes
            layers.poison_staging(b)
            torch.cuda._sleep(20_000_000)         # copies arrive late: the layer has to wait for them
        layers.prefetch(ctx, l, slice_bytes)

    # issue order of the layer-ahead schedule
    sched = po.pipeline_schedule(N_LAYERS)
    for it in range(2):
        for kind, l, b, dep in sched:
            if kind == "prefetch":
                poison_then_prefetch(l, it)
            else:
                ctx.dwdp_moe_forward(l, xs[l], lgs[l], bs[l], layers.tables[l], ys[it][l])
                ev = torch.cuda.Event()
                ev.record(torch.cuda.current_stream())
                done[b] = ev
    torch.cuda.synchronize()
    ctx.dwdp_set_copy_engine(0)
    for it in range(2):
        for l in range(N_LAYERS):
            got = ys[it][l].float().cpu().numpy()
            assert np.isfinite(got).all(), (it, l)
            np.testing.assert_array_equal(got, ref[l].float().cpu().numpy())


@pytest.mark.parametrize("engine", [0, 1])
@pytest.mark.parametrize("smr", [0, 16, 1 << 30])
def test_buffer_not_overwritten_before_its_reader_is_done(env, smr, engine):
    """Write-after-read half of the double-buffer protocol (paper Section 2: a staging buffer is
    reused only once the MoE block that reads it is done).  The compute stream is held back by a
    bounded spin so that layer 0's GEMMs have not started when layer 2's prefetch -- other
    weights, same buffer -- is issued; the test itself orders nothing: only the library's wait
    for the buffer's reader keeps layer 0 from reading layer 2's experts.  Run for every kernel
    family split (the second chain's end is part of "done")."""
    binding, pipeline, cfg, ctx, layers, xs, lgs, bs = env
    print("write-after-read, stream_max_rows", smr, "engine", engine, flush=True)
    ctx.dwdp_set_stream_max_rows(smr)
    ctx.dwdp_set_copy_engine(engine, 24)
    try:
        ref = _reference_outputs(ctx, cfg, layers, xs, lgs, bs)
        y0 = torch.empty(cfg.T, cfg.H, dtype=torch.bfloat16, device="cuda")
        y2 = torch.empty_like(y0)
        torch.cuda.synchronize()
        layers.prefetch(ctx, 0, 4096)
        torch.cuda._sleep(60_000_000)              # compute stream (the context's: the default stream) held back
        ctx.dwdp_moe_forward(0, xs[0], lgs[0], bs[0], layers.tables[0], y0)
        layers.prefetch(ctx, 2, 4096)              # same staging buffer, issued while layer 0 is still waiting to run
        ctx.dwdp_moe_forward(2, xs[2], lgs[2], bs[2], layers.tables[2], y2)
        torch.cuda.synchronize()
        np.testing.assert_array_equal(y0.float().cpu().numpy(), ref[0].float().cpu().numpy())
        np.testing.assert_array_equal(y2.float().cpu().numpy(), ref[2].float().cpu().numpy())
        assert not np.array_equal(ref[0].float().cpu().numpy(), ref[2].float().cpu().numpy())
    finally:
        ctx.dwdp_set_stream_max_rows(16)
        ctx.dwdp_set_copy_engine(0)


def test_pipeline_layers_match_oracle(env):
    binding, pipeline, cfg, ctx, layers, xs, lgs, bs = env
    print("pipeline vs oracle", flush=True)
    ys = [torch.empty(cfg.T, cfg.H, dtype=torch.bfloat16, device="cuda") for _ in range(N_LAYERS)]
    for kind, l, b, dep in po.pipeline_schedule(N_LAYERS):
        if kind == "prefetch":
            layers.prefetch(ctx, l, 1 << 16)
        else:
            ctx.dwdp_moe_forward(l, xs[l], lgs[l], bs[l], layers.tables[l], ys[l])
    torch.cuda.synchronize()
    spec = mo.spec_from(cfg)
    for l in range(N_LAYERS):
        ref = mo.moe_forward(to_np(xs[l]), to_np(lgs[l]), to_np(bs[l]), experts_numpy(layers.logical[l]), spec)
        err, l2 = mo.error_metrics(ys[l].float().cpu().numpy(), ref)
        assert mo.error_metric_rows(ys[l].float().cpu().numpy(), ref) <= row_tolerance(cfg)     # token by token as well
        print(f"  layer {l}: max-rel {err:.3e}", flush=True)
        assert err <= tolerance(cfg)


@pytest.mark.parametrize("engine", [0, 1])
def test_two_pullers_share_one_source(env, engine):
    """Two contexts (the pullers of two ranks, paper Section 4.3) fetch the same layer from the
    same peers at the same time, each in its own peer order and into its own landing buffer:
    both layers equal the in-place reference bit for bit."""
    binding, pipeline, cfg, ctx, layers, xs, lgs, bs = env
    print("two pullers, engine", engine, flush=True)
    l = 1
    ref = _reference_outputs(ctx, cfg, layers, xs, lgs, bs)[l].float().cpu().numpy()
    ctx2 = binding.Context(cfg, n_layers=N_LAYERS)
    try:
        st2 = layers.new_puller_staging()
        table2 = layers.puller_table(l, st2)
        for c in (ctx, ctx2):
            c.dwdp_set_copy_engine(engine, 24)
        layers.poison_staging(l % 2)
        layers.poison_staging(l % 2, st2)
        torch.cuda.synchronize()
        layers.puller_prefetch(ctx, l, layers.staging[l % 2], 4096, first_peer=0)
        layers.puller_prefetch(ctx2, l, st2, 4096, first_peer=1)
        y1 = torch.empty(cfg.T, cfg.H, dtype=torch.bfloat16, device="cuda")
        y2 = torch.empty_like(y1)
        ctx.dwdp_moe_forward(l, xs[l], lgs[l], bs[l], layers.tables[l], y1)
        ctx2.dwdp_moe_forward(l, xs[l], lgs[l], bs[l], table2, y2)
        torch.cuda.synchronize()
        np.testing.assert_array_equal(y1.float().cpu().numpy(), ref)
        np.testing.assert_array_equal(y2.float().cpu().numpy(), ref)
    finally:
        ctx2.close()
        ctx.dwdp_set_copy_engine(0)


@pytest.mark.parametrize("engine,wgs", [(0, 0), (1, 1), (1, 7), (1, 65535)])
@pytest.mark.parametrize("slice_bytes", [0, 1000, 262144 + 48])
def test_copy_plan_moves_exact_bytes(gpu_device, engine, wgs, slice_bytes):
    """The copy plan by itself (paper Section 4.3.2, Listing 1: every parameter of every peer,
    slice by slice): odd lengths, addresses that are not multiples of 16, a parameter of zero
    bytes; with one workgroup walking the whole plan, a few, and one per piece (the copy kernel's
    two workgroup shapes).  Every destination equals its source byte for byte and the guard bytes
    around each destination keep their pattern."""
    from paper_2604_01621_amd import binding
    print("copy plan engine", engine, "workgroups", wgs, "slice", slice_bytes, flush=True)
    cfg = inputs.small_fp8_layer(T=8)
    ctx = binding.Context(cfg, n_layers=2)
    n_peers, n_params, guard = 3, 3, 256
    sizes = [1_000_003, 0, 300_016]
    g = torch.Generator().manual_seed(5)
    srcs, dsts, src_ptrs, dst_ptrs = [], [], [], []
    for q in range(n_peers):
        for prm in range(n_params):
            n = sizes[prm]
            off_s, off_d = (q * 5 + prm) % 16, (q * 3 + prm * 7) % 16      # mixed alignments, some both 0 mod 16
            if q == 0:
                off_s = off_d = 0
            sb = torch.randint(0, 256, (n + off_s + 16,), dtype=torch.uint8, generator=g).cuda()
            db = torch.full((n + off_d + 2 * guard,), 0xA5, dtype=torch.uint8, device="cuda")
            srcs.append((sb, off_s))
            dsts.append((db, off_d))
            src_ptrs.append(sb.data_ptr() + off_s)
            dst_ptrs.append(db.data_ptr() + guard + off_d)
    ctx.dwdp_set_copy_engine(engine, wgs if engine == 1 else 256)
    ctx.dwdp_prefetch_layer(0, src_ptrs, dst_ptrs, sizes, n_peers, n_params, slice_bytes)
    torch.cuda.current_stream().wait_stream(torch.cuda.ExternalStream(ctx.copy_stream_handle()))
    torch.cuda.synchronize()
    for i, ((sb, off_s), (db, off_d)) in enumerate(zip(srcs, dsts)):
        n = sizes[i % n_params]
        got = db.cpu().numpy()
        np.testing.assert_array_equal(got[guard + off_d:guard + off_d + n], sb.cpu().numpy()[off_s:off_s + n], err_msg=str(i))
        assert (got[:guard + off_d] == 0xA5).all() and (got[guard + off_d + n:] == 0xA5).all(), i
    ctx.close()


def test_prefetch_protocol_errors(env):
    binding, pipeline, cfg, ctx, layers, xs, lgs, bs = env
    print("pipeline protocol", flush=True)
    torch.cuda.synchronize()
    layers.prefetch(ctx, 0, 0)
    with pytest.raises(binding.DwdpError) as ei:
        layers.prefetch(ctx, 2, 0)                 # buffer 0 still holds layer 0
    assert ei.value.status == binding.ESTATE
    y = torch.empty(cfg.T, cfg.H, dtype=torch.bfloat16, device="cuda")
    ctx.dwdp_moe_forward(0, xs[0], lgs[0], bs[0], layers.tables[0], y)     # consumes it
    layers.prefetch(ctx, 2, 0)
    ctx.dwdp_moe_forward(2, xs[2], lgs[2], bs[2], layers.tables[2], y)
    torch.cuda.synchronize()
    with pytest.raises(binding.DwdpError) as ei:
        src, dst, nb = layers.prefetch_args(0)
        ctx.dwdp_prefetch_layer(N_LAYERS, src, dst, nb, N_PEERS, pipeline.N_PARAMS, 0)     # no such layer
    assert ei.value.status == binding.EINVAL


def test_merged_copy_equals_mixed_table(env):
    """The naive baseline (merge into one contiguous buffer, paper Section 4.2) gives the same bits."""
    binding, pipeline, cfg, ctx, layers, xs, lgs, bs = env
    print("merge baseline", flush=True)
    l = 1
    layers.prefetch(ctx, l, 0)
    y_mixed = torch.empty(cfg.T, cfg.H, dtype=torch.bfloat16, device="cuda")
    ctx.dwdp_moe_forward(l, xs[l], lgs[l], bs[l], layers.tables[l], y_mixed)
    torch.cuda.synchronize()
    n = cfg.n_slots
    w13 = torch.empty(n, 2 * cfg.I, cfg.H, dtype=torch.uint8, device="cuda")
    w2 = torch.empty(n, cfg.H, cfg.I, dtype=torch.uint8, device="cuda")
    s13 = torch.empty(n, 2 * cfg.I // 128, cfg.H // 128, device="cuda")
    s2 = torch.empty(n, cfg.H // 128, cfg.I // 128, device="cuda")
    merged = ctx.dwdp_merge_experts(l, layers.tables[l].cpu().contiguous(), w13, s13, w2, s2)
    y_merged = torch.empty_like(y_mixed)
    ctx.dwdp_moe_forward(l, xs[l], lgs[l], bs[l], merged.cuda(), y_merged)
    torch.cuda.synchronize()
    assert merged[1, 0] - merged[0, 0] == 2 * cfg.I * cfg.H            # contiguous
    np.testing.assert_array_equal(y_merged.float().cpu().numpy(), y_mixed.float().cpu().numpy())


def test_non_divisible_group_with_redundant_experts(gpu_device):
    """A DWDP group whose size does not divide the expert count (paper Section 2, last
    paragraphs): 16 experts over 3 ranks -> every rank keeps 6 (neighbouring ranks overlap in
    one expert) and pulls 5 from each of its 2 peers.  Only the pointer table and the prefetch
    lists change; results must equal the all-in-place reference bit for bit."""
    from paper_2604_01621_amd import binding, pipeline
    print("non-divisible placement", flush=True)
    cfg = inputs.small_fp8_layer(T=40)
    n_layers, n_res, n_peers = 2, 6, 2
    ctx = binding.Context(cfg, n_layers=n_layers)
    layers = pipeline.SplitWeightLayers(ctx, cfg, n_layers, n_res, n_peers, seed=300)
    assert layers.per == 5 and layers.ranges == [(6, 11), (11, 16)]
    eb = inputs.expert_bytes(cfg)
    assert layers.prefetch_bytes() == 10 * eb          # 10 of 16 experts pulled per layer, 6 + shared resident
    ctx.dwdp_set_copy_engine(1, 16)
    for b in range(2):
        layers.poison_staging(b)
    ys, refs, ins = [], [], []
    for l in range(n_layers):
        x = inputs.make_activations(cfg, 310 + l).cuda()
        lg = inputs.make_gate_logits(cfg, x.cpu(), 310 + l).cuda()
        y = torch.empty(cfg.T, cfg.H, dtype=torch.bfloat16, device="cuda")
        ref = torch.empty_like(y)
        layers.prefetch(ctx, l, 3000)
        ctx.dwdp_moe_forward(l, x, lg, None, layers.tables[l], y)
        ctx.dwdp_moe_forward(l, x, lg, None, layers.all_resident_table(l), ref)
        ys.append(y)
        refs.append(ref)
        ins.append((x, lg))
    torch.cuda.synchronize()
    ctx.dwdp_set_copy_engine(0)
    spec = mo.spec_from(cfg)
    for l in range(n_layers):
        got = ys[l].float().cpu().numpy()
        assert np.isfinite(got).all()
        np.testing.assert_array_equal(got, refs[l].float().cpu().numpy())
        # and against the oracle, which knows nothing of placements: the layer's logical weights by value
        x, lg = ins[l]
        want = mo.moe_forward(to_np(x), to_np(lg), None, experts_numpy(layers.logical[l]), spec)
        err, l2 = mo.error_metrics(got, want)
        rows = mo.error_metric_rows(got, want)
        print(f"  layer {l}: max-rel {err:.3e} per-row {rows:.3e}", flush=True)
        assert err <= tolerance(cfg) and rows <= row_tolerance(cfg)
    ctx.close()
