"""Pins for the oracle's expert MLP, combine and whole-layer output, and the prefetch oracle."""
import os

import numpy as np
import pytest
import torch

from oracle import moe_oracle as mo
from oracle import prefetch_oracle as po
from paper_2604_01621_amd import inputs

GOLDEN = os.path.join(os.path.dirname(__file__), "golden")


def experts_numpy(w: inputs.ExpertWeights):
    out = []
    for e in range(w.n):
        if w.s13 is None:
            out.append(mo.ExpertNumpy(w.w13[e].float().numpy(), w.w2[e].float().numpy()))
        else:
            out.append(mo.ExpertNumpy(w.w13[e].numpy(), w.w2[e].numpy(), w.s13[e].numpy(), w.s2[e].numpy()))
    return out


def _lib_dense(w: inputs.ExpertWeights, e: int):
    """Expert e as fp64 torch matrices using library decode only."""
    if w.s13 is None:
        return w.w13[e].double(), w.w2[e].double()
    a = w.w13[e].view(torch.float8_e4m3fn).double() * w.s13[e].double().repeat_interleave(128, 0).repeat_interleave(128, 1)
    b = w.w2[e].view(torch.float8_e4m3fn).double() * w.s2[e].double().repeat_interleave(128, 0).repeat_interleave(128, 1)
    return a, b


def test_bf16_expert_is_three_library_matmuls():
    cfg, x, logits, bias = inputs.make_layer_inputs("tiny", 0)
    w = inputs.make_expert_weights(cfg, 0)
    spec = mo.spec_from(cfg)
    ex = experts_numpy(w)
    for e in (0, 5):
        w13, w2 = _lib_dense(w, e)
        xd = x.double()
        g = xd @ w13[:cfg.I].t()
        u = xd @ w13[cfg.I:].t()
        ref = (torch.nn.functional.silu(g) * u) @ w2.t()
        got = mo.expert_mlp(x.float().numpy(), ex[e], spec)
        assert got.shape == (cfg.T, cfg.H)
        np.testing.assert_allclose(got, ref.numpy(), rtol=1e-10, atol=1e-14)


def test_tiny_layer_vs_independent_dense_sum():
    """Layer output == dense sum over the selected experts, computed with library ops only
    (torch.topk + torch.softmax + matmul), no permutation."""
    cfg, x, logits, bias = inputs.make_layer_inputs("tiny", 1)
    w = inputs.make_expert_weights(cfg, 1)
    spec = mo.spec_from(cfg)
    y = mo.moe_forward(x.float().numpy(), logits.numpy(), None, experts_numpy(w), spec)
    tv, ti = torch.topk(logits.double(), cfg.K, dim=1)
    tw = torch.softmax(tv, dim=1)
    ref = torch.zeros(cfg.T, cfg.H, dtype=torch.float64)
    for t in range(cfg.T):
        for k in range(cfg.K):
            w13, w2 = _lib_dense(w, int(ti[t, k]))
            gu = w13 @ x[t].double()
            h = torch.nn.functional.silu(gu[:cfg.I]) * gu[cfg.I:]
            ref[t] += tw[t, k] * (w2 @ h)
    np.testing.assert_allclose(y, ref.numpy(), rtol=1e-6, atol=1e-8)  # routing weights are fp32
    yb = mo.moe_forward_bruteforce(x.float().numpy(), logits.numpy(), None, experts_numpy(w), spec)
    np.testing.assert_allclose(y, yb, rtol=1e-9, atol=1e-14)


def test_uniform_router_reduces_to_mean_of_experts():
    """K = E with equal logits: every weight is 1/E and the layer is the mean of all expert MLPs."""
    cfg = inputs.MoEConfig(T=5, H=128, I=128, E=4, K=4)
    x = inputs.make_activations(cfg, 3)
    w = inputs.make_expert_weights(cfg, 3, std=0.1)
    spec = mo.spec_from(cfg)
    y = mo.moe_forward(x.float().numpy(), np.zeros((cfg.T, cfg.E), np.float32), None, experts_numpy(w), spec)
    ref = torch.zeros(cfg.T, cfg.H, dtype=torch.float64)
    for e in range(cfg.E):
        w13, w2 = _lib_dense(w, e)
        gu = x.double() @ w13.t()
        ref += (torch.nn.functional.silu(gu[:, :cfg.I]) * gu[:, cfg.I:]) @ w2.t() / cfg.E
    np.testing.assert_allclose(y, ref.numpy(), rtol=1e-9, atol=1e-14)


def test_fp8_layer_vs_independent_reference():
    """FP8 layer with shared expert: independent per-token reference built from library
    pieces (torch float8 cast for both weight decode and activation encode)."""
    cfg = inputs.small_fp8_layer(T=12)
    seed = 4
    x = inputs.make_activations(cfg, seed)
    logits = inputs.make_gate_logits(cfg, x, seed)
    bias = inputs.make_bias(cfg, seed, kind="small")
    w = inputs.make_expert_weights(cfg, seed)
    spec = mo.spec_from(cfg)
    y = mo.moe_forward(x.float().numpy(), logits.numpy(), bias.numpy(), experts_numpy(w), spec)
    ids, tw = mo.route(logits.numpy(), bias.numpy(), spec)      # routing pinned elsewhere

    def qdq_lib(v):                                   # v fp64 [n]; library e4m3 cast
        g = v.float().view(-1, 128)
        amax = g.abs().amax(dim=1, keepdim=True)
        sc = torch.where(amax > 0, amax / 448.0, torch.ones_like(amax))
        q = (g / sc).clamp(-448, 448).to(torch.float8_e4m3fn).double()
        return (q * sc.double()).view(-1)

    ref = torch.zeros(cfg.T, cfg.H, dtype=torch.float64)
    for t in range(cfg.T):
        xq = qdq_lib(x[t].double())
        sel = [(int(ids[t, k]), float(tw[t, k])) for k in range(cfg.K)] + [(cfg.E, 1.0)]
        for e, wk in sel:
            w13, w2 = _lib_dense(w, e)
            gu = w13 @ xq
            h = torch.nn.functional.silu(gu[:cfg.I]) * gu[cfg.I:]
            ref[t] += wk * (w2 @ qdq_lib(h))
    np.testing.assert_allclose(y, ref.numpy(), rtol=1e-9, atol=1e-12)
    yb = mo.moe_forward_bruteforce(x.float().numpy(), logits.numpy(), bias.numpy(), experts_numpy(w), spec)
    np.testing.assert_allclose(y, yb, rtol=1e-9, atol=1e-12)
    # token subset evaluation gives the same rows
    sub = mo.moe_forward(x.float().numpy(), logits.numpy(), bias.numpy(), experts_numpy(w), spec, tokens=[3, 7])
    np.testing.assert_allclose(sub, y[[3, 7]], rtol=1e-11, atol=1e-14)


def test_fp8_closed_form_identity_expert():
    """Weights chosen so the answer is known in closed form: W_gate = a*I, W_up = b*I,
    W_down = I (all exactly representable), x on the e4m3 grid with amax 448.  Then
    o = QDQ(silu(a x) * b x) and the only inexact step is the second quantisation, whose
    error is bounded by 2^-4 relative."""
    H = I = 128
    spec = mo.LayerSpec(H=H, I=I, E=1, K=1, w_dtype=mo.W_FP8)
    eye = np.zeros((H, H), np.uint8)
    eye[np.arange(H), np.arange(H)] = 0x38           # 1.0
    w13 = np.concatenate([eye, eye], axis=0)
    a, b = 0.5, 0.03125
    s13 = np.array([[a], [b]], np.float32)
    ex = mo.ExpertNumpy(w13, eye.copy(), s13, np.ones((1, 1), np.float32))
    rng = np.random.default_rng(0)
    codes = rng.integers(1, 127, size=(3, H)).astype(np.uint8)
    codes[:, 0] = 0x7E
    x = mo.E4M3_TABLE[codes] * (1.0 / 64)
    x[:, 1::2] *= -1
    o = mo.expert_mlp(x, ex, spec)
    h = (a * x) / (1 + np.exp(-a * x)) * (b * x)
    err = np.abs(o - h)
    amax = np.abs(h).max(axis=1, keepdims=True)
    assert (err <= np.maximum(np.abs(h) * 2.0 ** -4, amax / 448 * 2.0 ** -10) * (1 + 1e-5)).all()
    assert np.abs(o).max() > 0


# ------------------------------------------------------------------ prefetch oracle

def test_contention_pmf_matches_printed_table():
    rows = [l.split() for l in open(os.path.join(GOLDEN, "table2_contention.txt")) if l.strip() and l[0] != "#"]
    assert len(rows) == 6
    for r in rows:
        N = int(r[0])
        printed = [float(v) for v in r[1:]]
        pmf = [100 * p for p in po.contention_pmf(N)]
        assert len(pmf) == N - 1
        assert abs(sum(pmf) - 100) < 1e-9
        for got, want in zip(pmf, printed):
            # printed with 2 decimals / 2-3 significant digits
            assert abs(got - want) <= max(0.006, 0.06 * want), (N, got, want)
    assert po.pull_service_time(3.0, 4) == 1.0


def test_copy_plan_matches_hand_worked_listing():
    want = [tuple(int(v) for v in l.split()) for l in open(os.path.join(GOLDEN, "listing1_plan.txt"))
            if l.strip() and l[0] != "#"]
    src = {peer: [1000 * peer + 100 * p for p in range(2)] for peer in (1, 2, 3)}
    dst = {peer: [50000 + 1000 * peer + 100 * p for p in range(2)] for peer in (1, 2, 3)}
    plan = po.copy_plan([10, 4], [1, 2, 3], 4, src, dst)
    assert plan == want
    assert po.n_slices(10, 4) == 3 and po.n_slices(4, 4) == 1 and po.n_slices(5, 4) == 2


@pytest.mark.parametrize("M,s,peers", [([1000, 24, 7], 64, [2, 0]), ([5], 100, [1]), ([256, 256], 128, [3, 1, 2])])
def test_copy_plan_invariants(M, s, peers):
    src = {q: [10 ** 6 * (q + 1) + 10 ** 4 * p for p in range(len(M))] for q in peers}
    dst = {q: [10 ** 8 + 10 ** 6 * (q + 1) + 10 ** 4 * p for p in range(len(M))] for q in peers}
    plan = po.copy_plan(M, peers, s, src, dst)
    assert len(plan) == sum(po.n_slices(m, s) for m in M) * len(peers)
    assert sum(c for _, _, c in plan) == sum(M) * len(peers)
    # every (peer, parameter) region is tiled exactly once, same offsets on both sides
    for q in peers:
        for p, m in enumerate(M):
            segs = sorted((d - dst[q][p], c) for d, sr, c in plan
                          if dst[q][p] <= d < dst[q][p] + m and sr - src[q][p] == d - dst[q][p])
            pos = 0
            for off, c in segs:
                assert off == pos and 0 < c <= s
                pos += c
            assert pos == m
    # consecutive copies rotate over the peers in the given order
    for i, (d, sr, c) in enumerate(plan):
        q = peers[i % len(peers)]
        assert any(src[q][p] <= sr < src[q][p] + M[p] for p in range(len(M)))


def test_pipeline_schedule_double_buffering():
    steps = po.pipeline_schedule(5)
    pos = {(s[0], s[1]): i for i, s in enumerate(steps)}
    for kind, l, buf, dep in steps:
        assert buf == l % 2
        if kind == "moe":
            assert dep == ("prefetch", l) and pos[dep] < pos[("moe", l)]
            if l + 1 < 5:       # next layer's copy is issued before this layer's compute: it runs under it
                assert pos[("prefetch", l + 1)] < pos[("moe", l)]
        else:
            if l >= 2:          # the buffer is reused only after its previous reader finished
                assert dep == ("moe", l - 2) and pos[dep] < pos[("prefetch", l)]
            else:
                assert dep is None
