"""Parity at the full DeepSeek-R1 layer shape (H=7168, I=2048, E=256+1, top-8), in the launch
configuration bench.py times.  Routing and permutation are compared on every token
(bit-exact); the layer output is compared on sampled tokens whose rows the oracle computes
one by one (it dequantises only the experts those tokens use)."""
import numpy as np
import pytest
import torch

from oracle import moe_oracle as mo
from paper_2604_01621_amd import inputs
from tests.util import experts_numpy, to_np, tolerance

pytestmark = pytest.mark.gpu
SEED = 1


@pytest.fixture(scope="module")
def r1(gpu_device):
    from paper_2604_01621_amd import binding
    cfg = inputs.r1_layer(8192)
    print("generating 257 R1-shaped experts on the GPU", flush=True)
    w = inputs.make_expert_weights(cfg, SEED, device="cuda")
    ctx = binding.Context(cfg)
    wp = ctx.pack_experts(w)
    table = binding.expert_table(wp)
    yield binding, ctx, w, wp, table
    ctx.close()


def _check(r1, name, T, sample):
    binding, ctx, w, wp, table = r1
    cfg, x, logits, bias = inputs.make_layer_inputs(name, SEED, device="cuda", T=T)
    spec = mo.spec_from(cfg)
    y = torch.empty(cfg.T, cfg.H, dtype=torch.bfloat16, device="cuda")
    ctx.dwdp_moe_forward(0, x, logits, bias, table, y)
    torch.cuda.synchronize()
    # routing + permutation: every token, bit-exact
    rid, rw = mo.route(to_np(logits), to_np(bias), spec)
    np.testing.assert_array_equal(ctx.workspace("topk_ids", (cfg.T, cfg.K), torch.int32).cpu().numpy(), rid)
    np.testing.assert_allclose(ctx.workspace("topk_w", (cfg.T, cfg.K), torch.float32).cpu().numpy(), rw, rtol=2e-6)
    roff, rperm, rinv = mo.permute(rid, spec)
    np.testing.assert_array_equal(ctx.workspace("offsets", (cfg.E + 2,), torch.int32).cpu().numpy(), roff)
    np.testing.assert_array_equal(ctx.workspace("perm", (cfg.T * cfg.K,), torch.int32).cpu().numpy(), rperm)
    np.testing.assert_array_equal(ctx.workspace("inv_perm", (cfg.T * cfg.K,), torch.int32).cpu().numpy(), rinv)
    counts = np.diff(roff[:cfg.E + 1])
    # sampled tokens: the given ones plus one token of the most and of the least loaded expert
    hot, cold = int(np.argmax(counts)), int(np.argmin(np.where(counts > 0, counts, 1 << 30)))
    toks = set(sample)
    for e in (hot, cold):
        toks.add(int(rperm[roff[e]]) // cfg.K)
    toks = sorted(toks)
    need = sorted({int(e) for t in toks for e in rid[t]} | {cfg.E})
    print(f"  {name} T={T}: {len(toks)} sampled tokens, {len(need)} experts for the oracle; "
          f"rows/expert min {counts.min()} max {counts.max()}", flush=True)
    ref = mo.moe_forward(to_np(x), to_np(logits), to_np(bias), experts_numpy(w, only=need), spec, tokens=toks)
    got = y[toks].float().cpu().numpy()
    err, l2 = mo.error_metrics(got, ref)
    print(f"  max-rel {err:.3e} l2-rel {l2:.3e}", flush=True)
    assert np.isfinite(y.float().cpu().numpy()).all()
    assert err <= tolerance(cfg), (err, l2)
    return counts


def test_decode_T64(r1):
    print("full-size decode", flush=True)
    _check(r1, "decode", 64, [0, 31, 63])


def test_prefill_T8192(r1):
    print("full-size prefill", flush=True)
    counts = _check(r1, "prefill", 8192, [0, 4097, 8191])
    assert counts.min() > 150 and counts.max() < 400           # uniform routing


def test_skew_T2048(r1):
    print("full-size skew", flush=True)
    counts = _check(r1, "skew", 2048, [5, 2047])
    assert counts.max() > 10 * 2048 * 8 / 256                   # hottest expert > 10x the mean


def test_pipeline_T256_mixed_table(r1):
    """T=256 with 64 resident + 192 staged experts: the staged copy must give the same bits as
    reading the peer pool in place, and match the oracle on sampled tokens."""
    print("full-size pipeline layer", flush=True)
    binding, ctx, w, wp, table = r1
    cfg, x, logits, bias = inputs.make_layer_inputs("pipeline", SEED, device="cuda")
    n_res, n_peers, per = 64, 3, 64
    # staging buffer: the 192 non-resident experts, copied by the library's prefetch in 1 MiB slices
    st13, st2 = torch.full_like(wp.w13[n_res:cfg.E], 0xFF), torch.full_like(wp.w2[n_res:cfg.E], 0xFF)
    ss13, ss2 = torch.full_like(wp.s13[n_res:cfg.E], float("nan")), torch.full_like(wp.s2[n_res:cfg.E], float("nan"))
    src, dst, nbytes = [], [], None
    for p in range(n_peers):
        lo = n_res + p * per
        parts_src = [wp.w13[lo:lo + per], wp.s13[lo:lo + per], wp.w2[lo:lo + per], wp.s2[lo:lo + per]]
        parts_dst = [st13[p * per:(p + 1) * per], ss13[p * per:(p + 1) * per], st2[p * per:(p + 1) * per],
                     ss2[p * per:(p + 1) * per]]
        src += [t.data_ptr() for t in parts_src]
        dst += [t.data_ptr() for t in parts_dst]
        nbytes = [t.numel() * t.element_size() for t in parts_src]
    rows = []
    for e in range(cfg.E + 1):
        if e < n_res or e == cfg.E:
            rows.append([wp.w13[e].data_ptr(), wp.s13[e].data_ptr(), wp.w2[e].data_ptr(), wp.s2[e].data_ptr()])
        else:
            i = e - n_res
            rows.append([st13[i].data_ptr(), ss13[i].data_ptr(), st2[i].data_ptr(), ss2[i].data_ptr()])
    mixed = torch.tensor(rows, dtype=torch.int64).cuda()
    torch.cuda.synchronize()
    ctx.dwdp_prefetch_layer(0, src, dst, nbytes, n_peers, 4, 1 << 20)
    y_mixed = torch.empty(cfg.T, cfg.H, dtype=torch.bfloat16, device="cuda")
    ctx.dwdp_moe_forward(0, x, logits, bias, mixed, y_mixed)
    y_res = torch.empty_like(y_mixed)
    ctx.dwdp_moe_forward(0, x, logits, bias, table, y_res)
    torch.cuda.synchronize()
    np.testing.assert_array_equal(y_mixed.float().cpu().numpy(), y_res.float().cpu().numpy())
    spec = mo.spec_from(cfg)
    rid, _ = mo.route(to_np(logits), to_np(bias), spec)
    toks = [0, 255]
    need = sorted({int(e) for t in toks for e in rid[t]} | {cfg.E})
    ref = mo.moe_forward(to_np(x), to_np(logits), to_np(bias), experts_numpy(w, only=need), spec, tokens=toks)
    err, l2 = mo.error_metrics(y_mixed[toks].float().cpu().numpy(), ref)
    print(f"  max-rel {err:.3e}", flush=True)
    assert err <= tolerance(cfg)
