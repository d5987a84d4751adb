"""Pins of the comparators and reports every parity assertion goes through: the two error
metrics (hand-valued), the selection-margin report (hand-built scores), the whole-layer
brute force with MXFP4 weights, and the report-only reference without activation quantisation."""
import dataclasses

import numpy as np
import torch

from oracle import moe_oracle as mo
from paper_2604_01621_amd import inputs


def test_error_metrics_hand_values():
    ref = np.array([[3.0, -4.0], [0.0, 0.5]])
    y = np.array([[3.0, -3.0], [0.25, 0.5]])
    # |d| = [[0, 1], [0.25, 0]]; max|ref| = 4; ||d|| = sqrt(1.0625); ||ref|| = sqrt(25.25)
    mx, l2 = mo.error_metrics(y, ref)
    assert mx == 0.25
    assert abs(l2 - np.sqrt(1.0625 / 25.25)) < 1e-15
    # row by row: row 0 -> 1/4, row 1 -> 0.25/0.5; the small row dominates
    assert mo.error_metric_rows(y, ref) == 0.5
    # symmetric in sign, zero for equal inputs, not symmetric in its arguments (normalised by ref)
    assert mo.error_metrics(ref, ref) == (0.0, 0.0) and mo.error_metric_rows(ref, ref) == 0.0
    assert mo.error_metrics(-y, -ref)[0] == 0.25
    assert mo.error_metrics(ref, y)[0] == 1.0 / 3.0


def test_error_metric_rows_zero_reference_row():
    ref = np.array([[0.0, 0.0], [1.0, 2.0]])
    assert mo.error_metric_rows(np.array([[0.0, 0.0], [1.0, 2.0]]), ref) == 0.0
    assert mo.error_metric_rows(np.array([[1e-9, 0.0], [1.0, 2.0]]), ref) == np.inf


def test_route_margins_hand_built():
    """Softmax scoring selects on the raw logits, so the margins can be set by hand."""
    spec = mo.LayerSpec(H=128, I=128, E=8, K=2, n_group=4, topk_group=2, score_fn=mo.SCORE_SOFTMAX)
    one = np.float32(1.0)
    up = np.nextafter(one, np.float32(2.0))                    # 1 + 1 ulp
    up3 = np.float32(1.0 + 3 * 2.0 ** -23)
    #           g0          g1         g2           g3
    z = np.array([[4.0, 4.0, 3.0, one, up3, up, 0.0, 0.0],     # groups: 8, 4, 2+4ulp, 0
                  [5.0, 0.0, 4.0, 0.0, 3.0, 0.0, 2.0, 0.0]], np.float32)
    em, gm = mo.route_margins(z, None, spec)
    # token 0: kept groups 0 and 1 (scores 8 and 4); candidates 4, 4, 3, 1 -> K-th = 4, next = 3
    assert em[0] == (4.0 - 3.0) / np.spacing(np.float32(4.0))
    # last kept group 4.0 against best dropped 2 + 4 ulp(1): exact gap over the spacing at 4
    assert gm[0] == (4.0 - float(up3 + up)) / np.spacing(np.float32(4.0))
    # token 1: groups 5, 4 kept; candidates 5, 4, 0, 0 -> gap 4 at spacing(4)
    assert em[1] == 4.0 / np.spacing(np.float32(4.0)) and gm[1] == 1.0 / np.spacing(np.float32(4.0))
    # an exact tie has margin 0; a one-ulp gap has margin 1
    spec1 = mo.LayerSpec(H=128, I=128, E=4, K=1, score_fn=mo.SCORE_SOFTMAX)
    em, gm = mo.route_margins(np.array([[one, one, 0.0, 0.0], [up, one, 0.0, 0.0]], np.float32), None, spec1)
    assert list(em) == [0.0, 1.0] and np.all(np.isinf(gm))


def test_route_margins_agree_with_route_on_sigmoid_scores():
    """The margin report uses the selection scores route() selects on: perturbing the runner-up
    by more than the reported margin changes the selection, by less does not."""
    cfg = inputs.small_fp8_layer(T=6)
    spec = mo.spec_from(cfg)
    x = inputs.make_activations(cfg, 5)
    z = inputs.make_gate_logits(cfg, x, 5).numpy()
    b = inputs.make_bias(cfg, 5, kind="small").numpy()
    em, gm = mo.route_margins(z, b, spec)
    assert em.shape == (cfg.T,) and np.all(em > 0) and np.all(gm > 0) and np.all(np.isfinite(em))
    ids, _ = mo.route(z, b, spec)
    # recompute the K-th / (K+1)-th gap independently from the selected ids
    s = (1.0 / (1.0 + np.exp(-z.astype(np.float64)))).astype(np.float32)
    c = (s + b).astype(np.float32)
    gs = cfg.E // cfg.n_group
    for t in range(cfg.T):
        kept = sorted({int(e) // gs for e in ids[t]})
        gscore = [np.sort(c[t, g * gs:(g + 1) * gs])[-2:].sum(dtype=np.float32) for g in range(cfg.n_group)]
        kept_all = list(np.argsort(-np.array(gscore), kind="stable")[:cfg.topk_group])
        assert set(kept) <= set(int(g) for g in kept_all)
        cand = np.concatenate([c[t, g * gs:(g + 1) * gs] for g in kept_all])
        rest = np.sort(np.setdiff1d(cand, c[t, ids[t]]))[::-1]
        kth = c[t, ids[t, -1]]
        want = (float(kth) - float(rest[0])) / float(np.spacing(max(abs(kth), abs(rest[0]))))
        assert abs(em[t] - want) <= 1e-9 * max(want, 1.0)


def test_mxfp4_layer_bruteforce_equals_permuted_evaluation():
    """Whole layer with MXFP4 weights: the token-by-token evaluation (no permutation) equals the
    expert-by-expert one; both quantise the activations (FP8 activations beside MXFP4 weights)."""
    cfg = dataclasses.replace(inputs.small_fp8_layer(T=7, H=256, I=128, E=8, K=2, n_group=2, topk_group=1),
                              w_dtype=inputs.W_MXFP4)
    w = inputs.make_expert_weights(cfg, 11)
    spec = mo.spec_from(cfg)
    ex = [mo.ExpertNumpy(w.w13[e].numpy(), w.w2[e].numpy(), w.s13[e].numpy(), w.s2[e].numpy()) for e in range(w.n)]
    x = inputs.make_activations(cfg, 11)
    z = inputs.make_gate_logits(cfg, x, 11).numpy()
    b = inputs.make_bias(cfg, 11, kind="small").numpy()
    y = mo.moe_forward(x.float().numpy(), z, b, ex, spec)
    yb = mo.moe_forward_bruteforce(x.float().numpy(), z, b, ex, spec)
    np.testing.assert_allclose(y, yb, rtol=1e-9, atol=1e-13)
    # and it is not the un-quantised function: dropping the activation quantisation moves the result
    y_nq = mo.moe_forward(x.float().numpy(), z, b, ex, spec, act_quant=False)
    d = mo.error_metrics(y, y_nq)[0]
    assert 1e-3 < d < 0.2


def test_unquantised_activation_reference_is_plain_weight_only_layer():
    """act_quant=False == dequantised FP8 weights applied to the raw bf16 activations with
    library matmuls; the quantised layer lies within a few per cent of it."""
    cfg = inputs.small_fp8_layer(T=9)
    seed = 6
    x = inputs.make_activations(cfg, seed)
    z = inputs.make_gate_logits(cfg, x, seed)
    b = inputs.make_bias(cfg, seed, kind="small")
    w = inputs.make_expert_weights(cfg, seed)
    spec = mo.spec_from(cfg)
    ex = [mo.ExpertNumpy(w.w13[e].numpy(), w.w2[e].numpy(), w.s13[e].numpy(), w.s2[e].numpy()) for e in range(w.n)]
    y_nq = mo.moe_forward(x.float().numpy(), z.numpy(), b.numpy(), ex, spec, act_quant=False)
    ids, tw = mo.route(z.numpy(), b.numpy(), spec)
    ref = torch.zeros(cfg.T, cfg.H, dtype=torch.float64)
    for t in range(cfg.T):
        for e, wk in [(int(ids[t, k]), float(tw[t, k])) for k in range(cfg.K)] + [(cfg.E, 1.0)]:
            w13 = w.w13[e].view(torch.float8_e4m3fn).double() * w.s13[e].double().repeat_interleave(128, 0).repeat_interleave(128, 1)
            w2 = w.w2[e].view(torch.float8_e4m3fn).double() * w.s2[e].double().repeat_interleave(128, 0).repeat_interleave(128, 1)
            gu = w13 @ x[t].double()
            ref[t] += wk * (w2 @ (torch.nn.functional.silu(gu[:cfg.I]) * gu[cfg.I:]))
    np.testing.assert_allclose(y_nq, ref.numpy(), rtol=1e-9, atol=1e-12)
    y = mo.moe_forward(x.float().numpy(), z.numpy(), b.numpy(), ex, spec)
    assert 5e-3 < mo.error_metrics(y, y_nq)[0] < 0.15
