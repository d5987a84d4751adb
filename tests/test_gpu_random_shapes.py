"""Seeded random small layers against the oracle: shapes, routing set-ups, kernel-selection
thresholds, tile schedules and bias kinds that the hand-picked cases do not enumerate (K loops of 1..6 blocks,
1..40 experts per kernel family, token counts around the 16-, 64- and 288-row tile edges)."""
import random

import numpy as np
import pytest
import torch

from oracle import moe_oracle as mo
from paper_2604_01621_amd import inputs
from tests.util import experts_numpy, row_tolerance, to_np, tolerance

pytestmark = pytest.mark.gpu


def _case(rng):
    n_group = rng.choice([1, 2, 4])
    per_group = rng.choice([2, 4, 8])
    E = n_group * per_group
    topk_group = rng.randint(1, n_group)
    K = rng.randint(1, min(8, topk_group * per_group))
    return dict(T=rng.choice([1, 2, 3, 15, 16, 17, 31, 33, 64, 100, 290, 577, 700]), H=128 * rng.randint(1, 6),
                I=128 * rng.randint(1, 5), E=E, K=K, n_group=n_group, topk_group=topk_group,
                has_shared=rng.choice([0, 1])), rng.choice([0, 1, 5, 16, 16, 40, 64, 64, 100, 1 << 30]), \
        rng.choice(["none", "small", "zipf"]), rng.randint(0, 10 ** 6), rng.choice([0, 0, 1, 2])


@pytest.mark.parametrize("sweep_seed", [11, 12, 13, 14])
def test_random_small_layers(gpu_device, sweep_seed):
    from paper_2604_01621_amd import binding
    rng = random.Random(sweep_seed)
    for case in range(16):
        shape, smr, bias_kind, seed, schedule = _case(rng)
        print("random layer", sweep_seed, case, shape, "stream_max_rows", smr, "bias", bias_kind, "seed", seed,
              "tile schedule", schedule, flush=True)
        cfg = inputs.small_fp8_layer(**shape)
        x = inputs.make_activations(cfg, seed)
        logits = inputs.make_gate_logits(cfg, x, seed)
        bias = None if bias_kind == "none" else inputs.make_bias(cfg, seed, kind=bias_kind)
        w = inputs.make_expert_weights(cfg, seed)
        wd = inputs.ExpertWeights(w.w13.cuda(), w.w2.cuda(), w.s13.cuda(), w.s2.cuda())
        ctx = binding.Context(cfg)
        ctx.dwdp_set_stream_max_rows(smr)
        ctx.dwdp_set_tile_schedule(schedule)
        wp = ctx.pack_experts(wd)
        table = binding.expert_table(wp)
        y = torch.empty(cfg.T, cfg.H, dtype=torch.bfloat16, device="cuda")
        ctx.dwdp_moe_forward(0, x.cuda(), logits.cuda(), None if bias is None else bias.cuda(), table, y)
        torch.cuda.synchronize()
        spec = mo.spec_from(cfg)
        rid, _ = mo.route(to_np(logits), to_np(bias), spec)
        np.testing.assert_array_equal(ctx.workspace("topk_ids", (cfg.T, cfg.K), torch.int32).cpu().numpy(), rid)
        _, rperm, _ = mo.permute(rid, spec)
        np.testing.assert_array_equal(ctx.workspace("perm", (cfg.T * cfg.K,), torch.int32).cpu().numpy(), rperm)
        ref = mo.moe_forward(to_np(x), to_np(logits), to_np(bias), experts_numpy(w), spec)
        got = y.float().cpu().numpy()
        assert np.isfinite(got).all()
        err, l2 = mo.error_metrics(got, ref)
        assert mo.error_metric_rows(got, ref) <= row_tolerance(cfg)     # token by token as well
        assert err <= tolerance(cfg), (shape, smr, bias_kind, seed, err, l2)
        ctx.close()
