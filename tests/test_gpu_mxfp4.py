"""GPU parity of the MXFP4-weight path (FP4 E2M1 codes with E8M0 scales per 32 along K, FP8
activations) against the oracle, through the C ABI."""
import dataclasses

import numpy as np
import pytest
import torch

from oracle import moe_oracle as mo
from paper_2604_01621_amd import inputs
from tests.util import experts_numpy, row_tolerance, to_np, tolerance

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def binding(gpu_device):
    from paper_2604_01621_amd import binding as b
    return b


def test_pack_layout(binding):
    """dwdp_pack_mxfp4_weight against the layout its header documents, written out index by index."""
    print("mxfp4 pack layout", flush=True)
    cfg = dataclasses.replace(inputs.small_fp8_layer(T=1), w_dtype=inputs.W_MXFP4)
    ctx = binding.Context(cfg)
    rows, cols = 32, 640                         # 5 K blocks: two scale groups, the second padded
    g = torch.Generator().manual_seed(0)
    codes = torch.randint(0, 256, (1, rows, cols // 2), generator=g, dtype=torch.int32).to(torch.uint8)
    scales = torch.randint(100, 140, (1, rows, cols // 32), generator=g, dtype=torch.int32).to(torch.uint8)
    co = torch.zeros_like(codes).cuda()
    so = torch.zeros(1, binding.mx_scale_bytes(rows, cols), dtype=torch.uint8, device="cuda")
    ctx.dwdp_pack_mxfp4_weight(codes.cuda(), scales.cuda(), co, so)
    torch.cuda.synchronize()
    c, s = codes[0].numpy(), scales[0].numpy()
    nkb, ng = cols // 128, (cols // 128 + 3) // 4
    want_c = np.zeros(rows * cols // 2, dtype=np.uint8)
    want_s = np.full(binding.mx_scale_bytes(rows, cols), 127, dtype=np.uint8)
    for tr in range(rows // 16):
        for kb in range(nkb):
            for q in range(4):
                for r in range(16):
                    base = ((tr * nkb + kb) * 64 + q * 16 + r) * 16
                    want_c[base:base + 16] = c[tr * 16 + r, kb * 64 + q * 16: kb * 64 + q * 16 + 16]
                    want_s[((tr * ng + kb // 4) * 64 + q * 16 + r) * 4 + kb % 4] = s[tr * 16 + r, kb * 4 + q]
    np.testing.assert_array_equal(co.cpu().numpy().reshape(-1), want_c)
    np.testing.assert_array_equal(so.cpu().numpy().reshape(-1), want_s)
    ctx.close()


def _case(binding, cfg, seed, bias_kind="small", stream_max_rows=None):
    x = inputs.make_activations(cfg, seed)
    logits = inputs.make_gate_logits(cfg, x, seed)
    bias = None if bias_kind is None else inputs.make_bias(cfg, seed, kind=bias_kind)
    w = inputs.make_expert_weights(cfg, seed)
    wd = inputs.ExpertWeights(w.w13.cuda(), w.w2.cuda(), w.s13.cuda(), w.s2.cuda())
    ctx = binding.Context(cfg)
    if stream_max_rows is not None:
        ctx.dwdp_set_stream_max_rows(stream_max_rows)
    wp = ctx.pack_experts(wd)
    table = binding.expert_table(wp)
    y = torch.empty(cfg.T, cfg.H, dtype=torch.bfloat16, device="cuda")
    ctx.dwdp_moe_forward(0, x.cuda(), logits.cuda(), None if bias is None else bias.cuda(), table, y)
    torch.cuda.synchronize()
    spec = mo.spec_from(cfg)
    ref = mo.moe_forward(to_np(x), to_np(logits), to_np(bias), experts_numpy(w), spec)
    got = y.float().cpu().numpy()
    assert np.isfinite(got).all()
    err, l2 = mo.error_metrics(got, ref)
    assert mo.error_metric_rows(got, ref) <= row_tolerance(cfg)     # token by token as well
    print(f"  T={cfg.T} H={cfg.H} I={cfg.I} E={cfg.E}: max-rel {err:.3e} l2-rel {l2:.3e}", flush=True)
    assert err <= tolerance(cfg), (err, l2)
    ctx.close()


@pytest.mark.parametrize("smr", [0, 16, 1 << 30])
@pytest.mark.parametrize("T", [1, 7, 48, 333])
def test_layer_small_mxfp4(binding, T, smr):
    """The scaled-down sigmoid / group-limited layer with MXFP4 weights: several 16-token passes
    with a ragged tail, experts without tokens, shared expert.  smr selects the kernels: 0 =
    LDS-tiled for every expert, 16 = the default split, 2^30 = weight-streaming for every expert."""
    print("layer small mxfp4 T", T, "stream_max_rows", smr, flush=True)
    cfg = dataclasses.replace(inputs.small_fp8_layer(T=T), w_dtype=inputs.W_MXFP4)
    _case(binding, cfg, T, stream_max_rows=smr)


@pytest.mark.parametrize("smr", [0, 1 << 30])
@pytest.mark.parametrize("H,I,T", [(1536, 1024, 37), (1408, 640, 20), (640, 384, 300), (128, 128, 5), (256, 2304, 20)])
def test_layer_mxfp4_long_k(binding, H, I, T, smr):
    """K loops of 1..18 blocks: scale groups of four K blocks with a partial last group (11, 5,
    3, 1 blocks), odd numbers of two-block pipeline stages, on both kernel families."""
    print("layer mxfp4 long-k", H, I, T, smr, flush=True)
    cfg = dataclasses.replace(inputs.small_fp8_layer(T=T, H=H, I=I, E=8, K=2, n_group=1, topk_group=1),
                              w_dtype=inputs.W_MXFP4)
    _case(binding, cfg, 21, bias_kind=None, stream_max_rows=smr)


def test_full_size_decode_mxfp4(binding):
    """DeepSeek-R1 layer shape (H=7168, I=2048, 256+1 experts, top-8) at T=64 with MXFP4 weights:
    routing and permutation bit-exact on every token, output on sampled tokens."""
    print("full-size decode mxfp4: generating 257 experts on the GPU", flush=True)
    cfg, x, logits, bias = inputs.make_layer_inputs("decode", 1, device="cuda")
    cfg = dataclasses.replace(cfg, w_dtype=inputs.W_MXFP4)
    w = inputs.make_expert_weights(cfg, 1, device="cuda")
    ctx = binding.Context(cfg)
    wp = ctx.pack_experts(w)
    table = binding.expert_table(wp)
    y = torch.empty(cfg.T, cfg.H, dtype=torch.bfloat16, device="cuda")
    ctx.dwdp_moe_forward(0, x, logits, bias, table, y)
    torch.cuda.synchronize()
    spec = mo.spec_from(cfg)
    rid, _ = mo.route(to_np(logits), to_np(bias), spec)
    np.testing.assert_array_equal(ctx.workspace("topk_ids", (cfg.T, cfg.K), torch.int32).cpu().numpy(), rid)
    roff, rperm, _ = mo.permute(rid, spec)
    np.testing.assert_array_equal(ctx.workspace("perm", (cfg.T * cfg.K,), torch.int32).cpu().numpy(), rperm)
    toks = [0, 31, 63]
    need = sorted({int(e) for t in toks for e in rid[t]} | {cfg.E})
    ref = mo.moe_forward(to_np(x), to_np(logits), to_np(bias), experts_numpy(w, only=need), spec, tokens=toks)
    got = y[toks].float().cpu().numpy()
    err, l2 = mo.error_metrics(got, ref)
    assert mo.error_metric_rows(got, ref) <= row_tolerance(cfg)     # token by token as well
    print(f"  max-rel {err:.3e} l2-rel {l2:.3e}", flush=True)
    assert np.isfinite(y.float().cpu().numpy()).all()
    assert err <= tolerance(cfg), (err, l2)
    ctx.close()


def test_full_size_prefill_mxfp4(binding):
    """The same layer shape at T=8192 with MXFP4 weights (every expert on the LDS-tiled kernels, in
    the launch configuration `bench.py --workload prefill --weights mxfp4` times): routing and
    permutation bit-exact on every token, output on sampled tokens."""
    print("full-size prefill mxfp4: generating 257 experts on the GPU", flush=True)
    cfg, x, logits, bias = inputs.make_layer_inputs("prefill", 1, device="cuda")
    cfg = dataclasses.replace(cfg, w_dtype=inputs.W_MXFP4)
    w = inputs.make_expert_weights(cfg, 1, device="cuda")
    ctx = binding.Context(cfg)
    wp = ctx.pack_experts(w)
    table = binding.expert_table(wp)
    y = torch.empty(cfg.T, cfg.H, dtype=torch.bfloat16, device="cuda")
    ctx.dwdp_moe_forward(0, x, logits, bias, table, y)
    torch.cuda.synchronize()
    spec = mo.spec_from(cfg)
    rid, _ = mo.route(to_np(logits), to_np(bias), spec)
    np.testing.assert_array_equal(ctx.workspace("topk_ids", (cfg.T, cfg.K), torch.int32).cpu().numpy(), rid)
    roff, rperm, _ = mo.permute(rid, spec)
    np.testing.assert_array_equal(ctx.workspace("perm", (cfg.T * cfg.K,), torch.int32).cpu().numpy(), rperm)
    toks = [0, 4097, 8191]
    need = sorted({int(e) for t in toks for e in rid[t]} | {cfg.E})
    ref = mo.moe_forward(to_np(x), to_np(logits), to_np(bias), experts_numpy(w, only=need), spec, tokens=toks)
    got = y[toks].float().cpu().numpy()
    err, l2 = mo.error_metrics(got, ref)
    assert mo.error_metric_rows(got, ref) <= row_tolerance(cfg)     # token by token as well
    print(f"  max-rel {err:.3e} l2-rel {l2:.3e}", flush=True)
    assert np.isfinite(y.float().cpu().numpy()).all()
    assert err <= tolerance(cfg), (err, l2)
    ctx.close()
