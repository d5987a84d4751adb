"""GPU parity: the HIP path through the C ABI against the CPU oracle on the same seeded inputs.

Bars: routing ids and permutation bit-exact; routing weights to fp32 rounding; layer output
max|y-ref|/max|ref| <= 2e-2 (FP8 weights) or 5e-3 (bf16 weights).
"""
import numpy as np
import pytest
import torch

from oracle import moe_oracle as mo
from paper_2604_01621_amd import inputs
from tests.util import experts_numpy, gpu_forward, row_tolerance, to_np, tolerance

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def binding(gpu_device):
    from paper_2604_01621_amd import binding as b
    return b


def _route_case(binding, cfg, logits, bias):
    dev = "cuda"
    ctx = binding.Context(cfg)
    ids = torch.full((cfg.T, cfg.K), -1, dtype=torch.int32, device=dev)
    w = torch.zeros(cfg.T, cfg.K, dtype=torch.float32, device=dev)
    ctx.dwdp_route(logits.to(dev), None if bias is None else bias.to(dev), ids, w)
    torch.cuda.synchronize()
    rid, rw = mo.route(to_np(logits), to_np(bias), mo.spec_from(cfg))
    np.testing.assert_array_equal(ids.cpu().numpy(), rid)
    np.testing.assert_allclose(w.cpu().numpy(), rw, rtol=2e-6, atol=0)
    ctx.close()
    return ids


@pytest.mark.parametrize("seed", [0, 1])
def test_route_tiny_softmax(binding, seed):
    cfg, x, logits, bias = inputs.make_layer_inputs("tiny", seed)
    print("route tiny seed", seed, flush=True)
    _route_case(binding, cfg, logits, bias)


@pytest.mark.parametrize("T", [1, 5, 64, 1000])
def test_route_r1_sigmoid_group_limited(binding, T):
    print("route r1 T", T, flush=True)
    cfg, x, logits, bias = inputs.make_layer_inputs("decode", 3, T=T)
    _route_case(binding, cfg, logits, bias)


def test_route_zipf_and_normal_logits(binding):
    print("route skew/prefill", flush=True)
    cfg, x, logits, bias = inputs.make_layer_inputs("skew", 4, T=700)
    _route_case(binding, cfg, logits, bias)
    cfg, x, logits, bias = inputs.make_layer_inputs("prefill", 4, T=900)
    _route_case(binding, cfg, logits, bias)


def test_route_small_group_shapes_and_ties(binding):
    print("route small/ties", flush=True)
    cfg = inputs.small_fp8_layer(T=77)
    x = inputs.make_activations(cfg, 9)
    logits = inputs.make_gate_logits(cfg, x, 9)
    _route_case(binding, cfg, logits, inputs.make_bias(cfg, 9, kind="small"))
    _route_case(binding, cfg, logits, None)
    # exact ties everywhere: lower index must win on both sides
    _route_case(binding, cfg, torch.zeros(cfg.T, cfg.E), torch.zeros(cfg.E))
    q = torch.round(logits * 2) / 2          # heavily quantised logits: many ties
    _route_case(binding, cfg, q, torch.zeros(cfg.E))


@pytest.mark.parametrize("T,has_shared", [(0, 1), (1, 1), (64, 1), (1024, 0), (1025, 1), (5000, 1)])
def test_permute_bit_exact(binding, T, has_shared):
    print("permute T", T, "shared", has_shared, flush=True)
    cfg = inputs.r1_layer(T)
    cfg = inputs.MoEConfig(**{**cfg.__dict__, "has_shared": has_shared})
    spec = mo.spec_from(cfg)
    g = torch.Generator().manual_seed(T + 1)
    # K distinct experts per token, arbitrary order
    ids = torch.stack([torch.randperm(cfg.E, generator=g)[:cfg.K] for _ in range(T)]).to(torch.int32) if T else \
        torch.zeros(0, cfg.K, dtype=torch.int32)
    ctx = binding.Context(cfg, T_max=max(T, 1))
    n_off = cfg.E + 1 + has_shared
    off = torch.full((n_off,), -7, dtype=torch.int32, device="cuda")
    perm = torch.full((T * cfg.K,), -1, dtype=torch.int32, device="cuda")
    inv = torch.full((T * cfg.K,), -1, dtype=torch.int32, device="cuda")
    ctx.dwdp_permute(ids.cuda(), off, perm, inv)
    torch.cuda.synchronize()
    roff, rperm, rinv = mo.permute(ids.numpy(), spec)
    np.testing.assert_array_equal(off.cpu().numpy(), roff)
    np.testing.assert_array_equal(perm.cpu().numpy(), rperm)
    np.testing.assert_array_equal(inv.cpu().numpy(), rinv)
    ctx.close()


def test_permute_skewed_histogram(binding):
    print("permute skew", flush=True)
    cfg, x, logits, bias = inputs.make_layer_inputs("skew", 2, T=2048)
    ids = _route_case(binding, cfg, logits, bias)
    ctx = binding.Context(cfg)
    off = torch.zeros(cfg.E + 2, dtype=torch.int32, device="cuda")
    perm = torch.zeros(cfg.T * cfg.K, dtype=torch.int32, device="cuda")
    inv = torch.zeros_like(perm)
    ctx.dwdp_permute(ids, off, perm, inv)
    torch.cuda.synchronize()
    roff, rperm, rinv = mo.permute(ids.cpu().numpy(), mo.spec_from(cfg))
    np.testing.assert_array_equal(off.cpu().numpy(), roff)
    np.testing.assert_array_equal(perm.cpu().numpy(), rperm)
    np.testing.assert_array_equal(inv.cpu().numpy(), rinv)
    counts = np.diff(roff[:cfg.E + 1])
    assert counts.max() > 10 * cfg.T * cfg.K / cfg.E
    ctx.close()


def test_pack_fp8_weight_layout(binding):
    """Tile-major packing against the layout the header documents, written out in numpy."""
    print("pack layout", flush=True)
    cfg = inputs.small_fp8_layer(T=1)
    ctx = binding.Context(cfg)
    rows, cols = 48, 384
    g = torch.Generator().manual_seed(0)
    src = torch.randint(0, 256, (2, rows, cols), generator=g, dtype=torch.int32).to(torch.uint8)
    dst = torch.zeros_like(src).cuda()
    ctx.dwdp_pack_fp8_weight(src.cuda(), dst)
    torch.cuda.synchronize()
    s = src.numpy()
    # [m, tr, r, kb, q, half, b] -> [m, tr, kb, half, q, r, b]
    want = s.reshape(2, rows // 16, 16, cols // 128, 4, 2, 16).transpose(0, 1, 3, 5, 4, 2, 6).reshape(2, rows, cols)
    np.testing.assert_array_equal(dst.cpu().numpy(), want)
    ctx.close()


def _layer_case(binding, cfg, x, logits, bias, w, check_intermediates=False, stream_max_rows=None, schedule=None):
    dev = "cuda"
    wd = inputs.ExpertWeights(w.w13.to(dev), w.w2.to(dev), None if w.s13 is None else w.s13.to(dev),
                              None if w.s2 is None else w.s2.to(dev))
    ctx = binding.Context(cfg)
    if stream_max_rows is not None:
        ctx.dwdp_set_stream_max_rows(stream_max_rows)
    if schedule is not None:
        ctx.dwdp_set_tile_schedule(schedule)
    wp = ctx.pack_experts(wd)              # stays referenced: the table below holds raw addresses into it
    table = binding.expert_table(wp)
    xd, ld = x.to(dev), logits.to(dev)
    bd = None if bias is None else bias.to(dev)
    y = gpu_forward(ctx, cfg, xd, ld, bd, table)
    spec = mo.spec_from(cfg)
    ref = mo.moe_forward(to_np(x), to_np(logits), to_np(bias), experts_numpy(w), spec)
    err, l2 = mo.error_metrics(y.float().cpu().numpy(), ref)
    assert mo.error_metric_rows(y.float().cpu().numpy(), ref) <= row_tolerance(cfg)     # token by token as well
    print(f"  T={cfg.T} H={cfg.H} I={cfg.I} E={cfg.E}: max-rel {err:.3e} l2-rel {l2:.3e}", flush=True)
    assert np.isfinite(y.float().cpu().numpy()).all()
    assert err <= tolerance(cfg), (err, l2)
    # the persistent tiled GEMM's error word: no bounded device-side wait gave up
    assert int(ctx.workspace("sched", (32,), torch.int32)[16]) == 0
    if check_intermediates:
        rid, rw = mo.route(to_np(logits), to_np(bias), spec)
        np.testing.assert_array_equal(ctx.workspace("topk_ids", (cfg.T, cfg.K), torch.int32).cpu().numpy(), rid)
        roff, rperm, rinv = mo.permute(rid, spec)
        np.testing.assert_array_equal(ctx.workspace("perm", (cfg.T * cfg.K,), torch.int32).cpu().numpy(), rperm)
        np.testing.assert_array_equal(
            ctx.workspace("offsets", (cfg.E + 1 + cfg.has_shared,), torch.int32).cpu().numpy(), roff)
        if cfg.w_dtype == inputs.W_FP8:
            # activation quantisation decides integer codes from exact bf16 inputs in fp32 on both
            # sides: bit-exact
            _, codes, scales = mo.qdq_act(to_np(x))
            np.testing.assert_array_equal(ctx.workspace("xs", (cfg.T, cfg.H // 128), torch.float32).cpu().numpy(),
                                          scales)
            got = ctx.workspace("xq", (cfg.T, cfg.H), torch.uint8).cpu().numpy()
            nz = (codes & 0x7F) != 0         # +-0 may differ in sign bit only
            np.testing.assert_array_equal(got[nz], codes[nz])
            assert ((got[~nz] & 0x7F) == 0).all()
    ctx.close()
    return y


@pytest.mark.parametrize("seed", [0, 1, 2])
def test_layer_tiny_bf16(binding, seed):
    print("layer tiny seed", seed, flush=True)
    cfg, x, logits, bias = inputs.make_layer_inputs("tiny", seed)
    w = inputs.make_expert_weights(cfg, seed)
    _layer_case(binding, cfg, x, logits, bias, w, check_intermediates=True)


@pytest.mark.parametrize("smr", [0, 16, 1 << 30])
@pytest.mark.parametrize("T", [1, 7, 48, 333])
def test_layer_small_fp8(binding, T, smr):
    """Scaled-down sigmoid/group-limited FP8 layer: several 16-token tiles with a ragged tail,
    experts without tokens, shared expert.  smr selects the kernels: 0 = LDS-tiled for every
    expert, 16 = the default split, 2^30 = weight-streaming for every expert."""
    print("layer small fp8 T", T, "stream_max_rows", smr, flush=True)
    cfg = inputs.small_fp8_layer(T=T)
    x = inputs.make_activations(cfg, T)
    logits = inputs.make_gate_logits(cfg, x, T)
    bias = inputs.make_bias(cfg, T, kind="small")
    w = inputs.make_expert_weights(cfg, T)
    _layer_case(binding, cfg, x, logits, bias, w, check_intermediates=True, stream_max_rows=smr)


@pytest.mark.parametrize("smr", [0, 1 << 30])
@pytest.mark.parametrize("H,I,T", [(1536, 1024, 37), (1408, 640, 20), (640, 384, 300), (256, 2304, 20),
                                   (384, 1536, 33)])
def test_layer_fp8_long_k(binding, H, I, T, smr):
    """K loops of several pipeline rounds plus a remainder (H/128 = 12, 11, 5, 2 or 3; I/128 = 8,
    5, 3, 18 or 12: the streaming GEMM-2 stages its operand in chunks of 16 K blocks, so 18 runs
    two chunks), output rows not a multiple of the 256-row workgroup tile, on both kernel
    families."""
    print("layer fp8 long-k", H, I, T, smr, flush=True)
    cfg = inputs.small_fp8_layer(T=T, H=H, I=I, E=8, K=2, n_group=1, topk_group=1)
    x = inputs.make_activations(cfg, 21)
    logits = inputs.make_gate_logits(cfg, x, 21)
    w = inputs.make_expert_weights(cfg, 21)
    _layer_case(binding, cfg, x, logits, None, w, check_intermediates=True, stream_max_rows=smr)


@pytest.mark.parametrize("T", [31, 32, 33, 64, 287, 288, 289, 320, 577])
def test_layer_fp8_tile_boundaries(binding, T):
    """Row counts at the edges of the LDS-tiled kernel's units (32-token tiles of the matrix
    instruction, 288-token workgroup tiles): the shared expert holds exactly T rows, the routed
    experts ragged shares of 2T, every expert on the tiled kernels."""
    print("layer fp8 tile boundaries T", T, flush=True)
    cfg = inputs.small_fp8_layer(T=T, H=256, I=128, E=8, K=2, n_group=1, topk_group=1)
    x = inputs.make_activations(cfg, 100 + T)
    logits = inputs.make_gate_logits(cfg, x, 100 + T)
    w = inputs.make_expert_weights(cfg, 100 + T)
    _layer_case(binding, cfg, x, logits, None, w, check_intermediates=True, stream_max_rows=0)


@pytest.mark.parametrize("smr", [64, 1 << 30])
@pytest.mark.parametrize("T", [17, 31, 32, 33, 63, 64, 65, 127, 128, 129, 288])
def test_layer_fp8_row_group_boundaries(binding, T, smr):
    """Row counts at the edges of the multi-tile streaming items (16-token tiles, groups of 64
    rows): the shared expert holds exactly T rows, the routed experts ragged shares of 2T.
    With the default threshold (64) experts above it go to the tiled kernels, with 2^30 every
    expert is streamed, in one to five row groups."""
    print("layer fp8 row groups T", T, "stream_max_rows", smr, flush=True)
    cfg = inputs.small_fp8_layer(T=T, H=384, I=256, E=8, K=2, n_group=1, topk_group=1)
    x = inputs.make_activations(cfg, 500 + T)
    logits = inputs.make_gate_logits(cfg, x, 500 + T)
    w = inputs.make_expert_weights(cfg, 500 + T)
    _layer_case(binding, cfg, x, logits, None, w, check_intermediates=True, stream_max_rows=smr)


def test_layer_fp8_many_mtiles(binding):
    """Enough 288-row M tiles (35: 11 of the shared expert, about 3 per routed expert) for the tiled
    kernels' paired numbering of M tiles, which small layers do not reach."""
    print("layer fp8 many M tiles", flush=True)
    cfg = inputs.small_fp8_layer(T=3000, H=256, I=128, E=8, K=2, n_group=1, topk_group=1)
    x = inputs.make_activations(cfg, 77)
    logits = inputs.make_gate_logits(cfg, x, 77)
    w = inputs.make_expert_weights(cfg, 77)
    _layer_case(binding, cfg, x, logits, None, w, check_intermediates=True, stream_max_rows=0)


@pytest.mark.parametrize("T,H,I", [(3000, 256, 128), (700, 640, 384)])
def test_tile_schedules_give_the_same_bits(binding, T, H, I):
    """One workgroup per item, persistent launches per GEMM, and ONE persistent launch for both
    tiled GEMMs (down-projection items wait on device-side counters for their rows' gate/up
    items): identical output, and the scheduler's error word stays clear."""
    print("tile schedules T", T, flush=True)
    cfg = inputs.small_fp8_layer(T=T, H=H, I=I, E=8, K=2, n_group=1, topk_group=1)
    x = inputs.make_activations(cfg, 78)
    logits = inputs.make_gate_logits(cfg, x, 78)
    w = inputs.make_expert_weights(cfg, 78)
    ys = [_layer_case(binding, cfg, x, logits, None, w, stream_max_rows=0, schedule=m).float().cpu().numpy()
          for m in (0, 1, 2)]
    np.testing.assert_array_equal(ys[1], ys[0])
    np.testing.assert_array_equal(ys[2], ys[0])


def test_few_tiled_experts_join_the_row_groups(binding):
    """Default threshold, a layer whose only expert above 64 rows is the shared one (200 rows, one
    M tile): the list builder sends it to the row-group items instead of a whole-unit workgroup
    launch; same function, checked against the oracle like every other case."""
    print("few tiled experts", flush=True)
    cfg = inputs.small_fp8_layer(T=200, H=384, I=256, E=16, K=2, n_group=1, topk_group=1)
    x = inputs.make_activations(cfg, 79)
    logits = inputs.make_gate_logits(cfg, x, 79)
    w = inputs.make_expert_weights(cfg, 79)
    _layer_case(binding, cfg, x, logits, None, w, check_intermediates=True)


@pytest.mark.parametrize("T", [200, 500])
def test_layer_maximum_expert_and_topk_counts(binding, T):
    """The largest routing set-up the library accepts (1024 experts, top-32, 8 groups of 128) on a
    narrow layer: routing ids, permutation and output, with the permutation on one workgroup
    (T = 200) and on several (T = 500)."""
    print("layer E=1024 K=32 T", T, flush=True)
    cfg = inputs.small_fp8_layer(T=T, H=128, I=128, E=1024, K=32, n_group=8, topk_group=4)
    x = inputs.make_activations(cfg, 300 + T)
    logits = inputs.make_gate_logits(cfg, x, 300 + T)
    bias = inputs.make_bias(cfg, 300 + T, kind="small")
    w = inputs.make_expert_weights(cfg, 300 + T)
    _layer_case(binding, cfg, x, logits, bias, w, check_intermediates=True)


def test_layer_small_fp8_no_shared_and_empty(binding):
    print("layer small fp8 no shared / T=0", flush=True)
    cfg = inputs.small_fp8_layer(T=40, has_shared=0, E=32, n_group=4, topk_group=2, K=4, H=384, I=128)
    x = inputs.make_activations(cfg, 5)
    logits = inputs.make_gate_logits(cfg, x, 5)
    w = inputs.make_expert_weights(cfg, 5)
    _layer_case(binding, cfg, x, logits, None, w, check_intermediates=True)
    # T = 0: accepted, nothing written
    ctx = binding.Context(cfg)
    wd = inputs.ExpertWeights(w.w13.cuda(), w.w2.cuda(), w.s13.cuda(), w.s2.cuda())
    y = torch.empty(0, cfg.H, dtype=torch.bfloat16, device="cuda")
    wp = ctx.pack_experts(wd)
    ctx.dwdp_moe_forward(0, x[:0].cuda(), logits[:0].cuda(), None, binding.expert_table(wp), y)
    torch.cuda.synchronize()
    ctx.close()


def test_error_paths(binding):
    print("error paths", flush=True)
    cfg = inputs.small_fp8_layer(T=8)
    ctx = binding.Context(cfg, n_layers=2)
    x = torch.zeros(9, cfg.H, dtype=torch.bfloat16, device="cuda")
    lg = torch.zeros(9, cfg.E, device="cuda")
    y = torch.zeros(9, cfg.H, dtype=torch.bfloat16, device="cuda")
    tbl = torch.zeros(cfg.n_slots, 4, dtype=torch.int64, device="cuda")
    with pytest.raises(binding.DwdpError) as ei:
        ctx.dwdp_moe_forward(0, x, lg, None, tbl, y)            # T > T_max
    assert ei.value.status == binding.ESHAPE
    with pytest.raises(binding.DwdpError) as ei:
        ctx.dwdp_moe_forward(2, x[:4], lg[:4], None, tbl, y)    # layer out of range
    assert ei.value.status == binding.EINVAL
    with pytest.raises(binding.DwdpError) as ei:
        ctx.dwdp_moe_forward(0, x[:4], lg[:4], None, None, y)   # NULL table
    assert ei.value.status == binding.EINVAL
    ctx.close()
