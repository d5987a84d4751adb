"""Pins of the oracle's MXFP4 decoding against what the OCP Microscaling Formats (MX) v1.0
specification fixes, and of the MXFP4 expert MLP against independent evaluations."""
import dataclasses

import numpy as np
import torch

from oracle import moe_oracle as mo
from paper_2604_01621_amd import inputs


def test_e2m1_value_set():
    # OCP MX v1.0, FP4 E2M1: exponent bias 1, no Inf/NaN, max normal 6.0, min normal 1.0, subnormal 0.5
    want = [0.0, 0.5, 1.0, 1.5, 2.0, 3.0, 4.0, 6.0]
    assert [mo.e2m1_decode(c) for c in range(8)] == want
    assert [mo.e2m1_decode(8 + c) for c in range(1, 8)] == [-v for v in want[1:]]
    assert mo.e2m1_decode(8) == 0.0 and np.signbit(mo.e2m1_decode(8))          # negative zero
    assert np.all(np.isfinite(mo.E2M1_TABLE))
    # generic form: (-1)^s * 2^(e-1) * (1 + m/2) for e > 0
    for c in range(16):
        s, e, m = c >> 3, (c >> 1) & 3, c & 1
        v = (0.5 * m) if e == 0 else 2.0 ** (e - 1) * (1 + m / 2)
        assert mo.E2M1_TABLE[c] == (-v if s else v)


def test_e8m0_scale():
    # E8M0: unsigned exponent, bias 127, value 2^(x-127); 0xFF is NaN; 0 is 2^-127 (no zero)
    x = np.array([0, 1, 126, 127, 128, 254, 255], dtype=np.uint8)
    v = mo.e8m0_decode(x)
    assert v[3] == 1.0 and v[4] == 2.0 and v[2] == 0.5
    assert v[0] == 2.0 ** -127 and v[5] == 2.0 ** 127 and np.isnan(v[6])
    assert np.all(np.diff(np.log2(v[:6])) == np.array([1, 125, 1, 1, 126]))


def test_dequant_layout_low_nibble_first_and_block_of_32():
    # element 2i in the low nibble of byte i; one scale per 32 consecutive elements of a row
    packed = np.zeros((2, 32), dtype=np.uint8)       # 64 elements per row: two scale blocks
    packed[0, 0] = 0x72                               # elements 0, 1 = codes 2 (1.0), 7 (6.0)
    packed[0, 16] = 0x0F                              # element 32 = code 15 (-6.0), element 33 = 0
    packed[1, 31] = 0x30                              # element 63 = code 3 (1.5)
    scales = np.array([[127, 129], [120, 126]], dtype=np.uint8)
    w = mo.dequant_mxfp4(packed, scales)
    assert w.shape == (2, 64)
    assert w[0, 0] == 1.0 and w[0, 1] == 6.0
    assert w[0, 32] == -24.0 and w[0, 33] == 0.0      # second block: x 2^2
    assert w[1, 63] == 0.75                           # 1.5 x 2^-1
    assert np.count_nonzero(w) == 4


def test_generated_weights_decode_close_to_their_source():
    """The generator's MXFP4 data decodes (by the oracle) to within half a grid step of the
    fp32 values it was made from: ties the two sides' nibble order, block size and scale bias."""
    g = torch.Generator().manual_seed(3)
    w = torch.randn(16, 256, generator=g) * 0.02
    packed, scales = inputs._quant_mxfp4(w)
    assert packed.shape == (16, 128) and scales.shape == (16, 8)
    deq = mo.dequant_mxfp4(packed.numpy(), scales.numpy())
    blk_scale = mo.e8m0_decode(scales.numpy())
    src = w.numpy().astype(np.float64).reshape(16, 8, 32)
    err = np.abs(deq.reshape(16, 8, 32) - src) / blk_scale[:, :, None]
    q = np.abs(src) / blk_scale[:, :, None]
    assert np.all(err[q <= 6] <= 1.0 + 1e-12)      # half of the widest grid gap (4 .. 6)
    assert np.all(q < 8) and np.all(err[q > 6] < 2.0)   # the top of the block's binade saturates at 6
    # block maxima are representable without saturation loss beyond one step and use the top binade
    amax = np.abs(deq).reshape(16, 8, 32).max(axis=2)
    assert np.all(amax >= 4 * blk_scale) and np.all(amax <= 6 * blk_scale)


def test_mxfp4_expert_mlp_equals_dense_evaluation():
    cfg = dataclasses.replace(inputs.small_fp8_layer(T=5, H=256, I=128, E=4, K=2, n_group=1, topk_group=1,
                                                     has_shared=0), w_dtype=inputs.W_MXFP4)
    w = inputs.make_expert_weights(cfg, 9)
    spec = mo.spec_from(cfg)
    ex = mo.ExpertNumpy(w.w13[1].numpy(), w.w2[1].numpy(), w.s13[1].numpy(), w.s2[1].numpy())
    x = inputs.make_activations(cfg, 9).float().numpy()
    got = mo.expert_mlp(x, ex, spec)
    # the same with everything written out: decode weights element by element, quantise, multiply
    W13 = np.zeros((2 * cfg.I, cfg.H))
    for r in range(2 * cfg.I):
        for c in range(cfg.H):
            byte = int(w.w13[1, r, c // 2])
            code = (byte >> 4) if (c & 1) else (byte & 15)
            W13[r, c] = mo.e2m1_decode(code) * 2.0 ** (int(w.s13[1, r, c // 32]) - 127)
    W2 = mo.dequant_mxfp4(w.w2[1].numpy(), w.s2[1].numpy())
    xq = mo.qdq_act(x)[0]
    gu = xq @ W13.T
    h = mo.qdq_act(gu[:, :cfg.I] / (1 + np.exp(-gu[:, :cfg.I])) * gu[:, cfg.I:])[0]
    np.testing.assert_allclose(got, h @ W2.T, rtol=1e-12, atol=1e-15)
