"""Seeded synthetic inputs for the DWDP MoE-layer hot path.

This module only *draws data*: activations, router logits, router bias and
expert weights with the shapes and value distributions of a DeepSeek-R1-shaped
MoE layer.  It holds none of the layer's arithmetic (no routing, no
permutation, no expert MLP, no activation quantisation) and is the one piece of
code that both the CPU oracle's tests and the HIP path's tests call, so that
both sides consume byte-identical inputs.

The FP8 weight bytes are produced with the library cast
``Tensor.to(torch.float8_e4m3fn)`` (OCP e4m3, finite-only, max 448); neither the
oracle's nor the kernels' own codecs are used here.

Workloads (names used by tests and bench):
  tiny      T=16   H=256  I=128  E=8   top-2 softmax, bf16 weights, no shared expert
  decode    T=64   H=7168 I=2048 E=256 top-8 sigmoid, group-limited (8 groups, keep 4),
                   routed scale 2.5, one shared expert, FP8 block-scaled weights
  prefill   same layer, T=8192, logits ~ N(0,1) (uniform routing)
  skew      same layer, T=2048, Zipf(1.2) router bias
  pipeline  same layer, T=256, 4 layers, 64 resident + 192 "peer" experts per layer
"""
from __future__ import annotations

import dataclasses
import math
from typing import Dict, Optional

import torch

SCORE_SOFTMAX = 0
SCORE_SIGMOID = 1
W_BF16 = 0
W_FP8 = 1
W_MXFP4 = 2        # FP4 E2M1 codes, one E8M0 scale per 32 elements along K (OCP MX)
MX_BLOCK = 32
BLOCK = 128          # side of a weight scale block; also the activation quantisation group
E4M3_MAX = 448.0


@dataclasses.dataclass(frozen=True)
class MoEConfig:
    """Shape and routing parameters of one MoE layer (mirrors the C struct dwdp_config)."""
    T: int
    H: int
    I: int
    E: int
    K: int
    n_group: int = 1
    topk_group: int = 1
    has_shared: int = 0
    score_fn: int = SCORE_SOFTMAX
    routed_scale: float = 1.0
    w_dtype: int = W_BF16

    @property
    def n_slots(self) -> int:
        """Expert slots in the pointer table: E routed (+1 shared)."""
        return self.E + (1 if self.has_shared else 0)

    def with_T(self, T: int) -> "MoEConfig":
        return dataclasses.replace(self, T=T)


def r1_layer(T: int) -> MoEConfig:
    """DeepSeek-R1-shaped MoE layer at T tokens."""
    return MoEConfig(T=T, H=7168, I=2048, E=256, K=8, n_group=8, topk_group=4, has_shared=1,
                     score_fn=SCORE_SIGMOID, routed_scale=2.5, w_dtype=W_FP8)


WORKLOADS: Dict[str, MoEConfig] = {
    "tiny": MoEConfig(T=16, H=256, I=128, E=8, K=2),
    "decode": r1_layer(64),
    "prefill": r1_layer(8192),
    "skew": r1_layer(2048),
    "pipeline": r1_layer(256),
}

# Slope of the Zipf router bias of the "skew" workload: b_e = ZIPF_BETA * (-1.2 ln rank_e),
# shifted to zero mean.  The value was chosen once, offline, so that with the seeded gate
# logits the most popular expert receives more than ten times the mean token count; the
# tests re-check that property on the realised histogram.
ZIPF_S = 1.2
ZIPF_BETA = 0.12


def _gen(seed: int, device) -> torch.Generator:
    g = torch.Generator(device=device)
    g.manual_seed(int(seed))
    return g


def make_activations(cfg: MoEConfig, seed: int, device="cpu") -> torch.Tensor:
    """x ~ N(0,1), bf16 [T,H]."""
    g = _gen(seed * 7919 + 1, device)
    return torch.randn(cfg.T, cfg.H, generator=g, device=device, dtype=torch.float32).to(torch.bfloat16)


def make_gate_logits(cfg: MoEConfig, x: torch.Tensor, seed: int) -> torch.Tensor:
    """Router logits z = x W_g^T with W_g ~ N(0, 0.02), fp32 [T,E].

    The gate projection is a dense GEMM outside the hot path; it is evaluated here
    once (fp64 accumulate, rounded once to fp32) so both sides see the same logits.
    """
    device = x.device
    g = _gen(seed * 7919 + 2, device)
    wg = torch.randn(cfg.E, cfg.H, generator=g, device=device, dtype=torch.float32) * 0.02
    return (x.to(torch.float64) @ wg.to(torch.float64).t()).to(torch.float32).contiguous()


def make_normal_logits(cfg: MoEConfig, seed: int, device="cpu") -> torch.Tensor:
    """Router logits ~ N(0,1) drawn directly (uniform routing), fp32 [T,E]."""
    g = _gen(seed * 7919 + 3, device)
    return torch.randn(cfg.T, cfg.E, generator=g, device=device, dtype=torch.float32)


def make_bias(cfg: MoEConfig, seed: int, device="cpu", kind: str = "small") -> Optional[torch.Tensor]:
    """Router selection bias, fp32 [E].

    kind="none"  -> None (softmax workloads)
    kind="zero"  -> zeros
    kind="small" -> N(0, 0.05): a load-balancing bias of realistic magnitude
    kind="zipf"  -> expert popularity ~ Zipf(1.2) over a seeded random ranking of the experts
    """
    if kind == "none":
        return None
    if kind == "zero":
        return torch.zeros(cfg.E, dtype=torch.float32, device=device)
    g = _gen(seed * 7919 + 4, "cpu")
    if kind == "small":
        return (torch.randn(cfg.E, generator=g, dtype=torch.float32) * 0.05).to(device)
    if kind == "zipf":
        rank = torch.randperm(cfg.E, generator=g).to(torch.float64) + 1.0
        b = ZIPF_BETA * (-ZIPF_S * torch.log(rank))
        b = b - b.mean()
        return b.to(torch.float32).to(device)
    raise ValueError(kind)


@dataclasses.dataclass
class ExpertWeights:
    """Weights of n expert slots in the logical layouts the C-ABI documents.

    w13 [n, 2I, H]  rows 0..I-1 = gate projection, rows I..2I-1 = up projection
    w2  [n, H, I]   down projection
    FP8: dtype uint8 (e4m3 bytes), s13 fp32 [n, 2I/128, H/128], s2 fp32 [n, H/128, I/128]
    bf16: dtype bfloat16, s13 = s2 = None
    """
    w13: torch.Tensor
    w2: torch.Tensor
    s13: Optional[torch.Tensor]
    s2: Optional[torch.Tensor]

    @property
    def n(self) -> int:
        return self.w13.shape[0]


def _quant_block_fp8(w: torch.Tensor):
    """fp32 [R,C] -> (uint8 [R,C], fp32 [R/128,C/128]); scale = block amax / 448."""
    R, C = w.shape
    wb = w.view(R // BLOCK, BLOCK, C // BLOCK, BLOCK)
    amax = wb.abs().amax(dim=(1, 3))
    scale = torch.where(amax > 0, amax / E4M3_MAX, torch.ones_like(amax))
    q = (wb / scale[:, None, :, None]).clamp_(-E4M3_MAX, E4M3_MAX)
    codes = q.to(torch.float8_e4m3fn).view(torch.uint8).view(R, C)
    return codes, scale.to(torch.float32)


def _quant_mxfp4(w: torch.Tensor):
    """fp32 [R,C] -> (packed E2M1 codes uint8 [R,C/2], E8M0 scales uint8 [R,C/32]).

    Input synthesis only (how random weights become MXFP4 test data; the layer's arithmetic
    starts from the codes): shared exponent = floor(log2(block amax)) - 2 (2 = exponent of
    the largest E2M1 value, 6 = 1.5 * 2^2), elements rounded to the nearest E2M1 value, ties
    to the even code, saturating at +-6.
    """
    R, C = w.shape
    wb = w.view(R, C // MX_BLOCK, MX_BLOCK)
    amax = wb.abs().amax(dim=2)
    e = torch.where(amax > 0, torch.floor(torch.log2(amax)) - 2, torch.zeros_like(amax)).clamp_(-127, 127)
    q = (wb / torch.exp2(e)[:, :, None]).abs()
    # thresholds between neighbouring magnitudes 0, .5, 1, 1.5, 2, 3, 4, 6; `up` = the tie goes to the upper
    # neighbour (its code is the even one)
    code = torch.zeros_like(q, dtype=torch.uint8)
    for thr, up in ((0.25, False), (0.75, True), (1.25, False), (1.75, True), (2.5, False), (3.5, True), (5.0, False)):
        code += ((q > thr) | ((q == thr) & up)).to(torch.uint8)
    code |= (wb < 0).to(torch.uint8) << 3
    code = code.view(R, C)
    packed = (code[:, 0::2] | (code[:, 1::2] << 4)).contiguous()
    return packed, (e + 127).to(torch.uint8)


def make_expert_weights(cfg: MoEConfig, seed: int, device="cpu", n: Optional[int] = None,
                        std: float = 0.02) -> ExpertWeights:
    """W ~ N(0, std) per expert slot; FP8 workloads quantise per 128x128 block so that the
    codes of every block span the full +-448 range."""
    n = cfg.n_slots if n is None else n
    H, I = cfg.H, cfg.I
    g = _gen(seed * 7919 + 5, device)
    if cfg.w_dtype == W_BF16:
        w13 = torch.empty(n, 2 * I, H, dtype=torch.bfloat16, device=device)
        w2 = torch.empty(n, H, I, dtype=torch.bfloat16, device=device)
        for e in range(n):
            w13[e] = (torch.randn(2 * I, H, generator=g, device=device) * std).to(torch.bfloat16)
            w2[e] = (torch.randn(H, I, generator=g, device=device) * std).to(torch.bfloat16)
        return ExpertWeights(w13, w2, None, None)
    assert H % BLOCK == 0 and I % BLOCK == 0
    if cfg.w_dtype == W_MXFP4:
        w13 = torch.empty(n, 2 * I, H // 2, dtype=torch.uint8, device=device)
        w2 = torch.empty(n, H, I // 2, dtype=torch.uint8, device=device)
        s13 = torch.empty(n, 2 * I, H // MX_BLOCK, dtype=torch.uint8, device=device)
        s2 = torch.empty(n, H, I // MX_BLOCK, dtype=torch.uint8, device=device)
        for e in range(n):
            w13[e], s13[e] = _quant_mxfp4(torch.randn(2 * I, H, generator=g, device=device) * std)
            w2[e], s2[e] = _quant_mxfp4(torch.randn(H, I, generator=g, device=device) * std)
        return ExpertWeights(w13, w2, s13, s2)
    w13 = torch.empty(n, 2 * I, H, dtype=torch.uint8, device=device)
    w2 = torch.empty(n, H, I, dtype=torch.uint8, device=device)
    s13 = torch.empty(n, 2 * I // BLOCK, H // BLOCK, dtype=torch.float32, device=device)
    s2 = torch.empty(n, H // BLOCK, I // BLOCK, dtype=torch.float32, device=device)
    for e in range(n):
        w13[e], s13[e] = _quant_block_fp8(torch.randn(2 * I, H, generator=g, device=device) * std)
        w2[e], s2[e] = _quant_block_fp8(torch.randn(H, I, generator=g, device=device) * std)
    return ExpertWeights(w13, w2, s13, s2)


def expert_bytes(cfg: MoEConfig) -> int:
    """HBM bytes of one expert's weights (codes + scales): the unit of the decode roofline."""
    H, I = cfg.H, cfg.I
    if cfg.w_dtype == W_BF16:
        return 2 * (2 * I * H + H * I)
    if cfg.w_dtype == W_MXFP4:
        return 3 * I * H // 2 + 3 * I * H // MX_BLOCK
    return 3 * I * H + 4 * ((2 * I // BLOCK) * (H // BLOCK) + (H // BLOCK) * (I // BLOCK))


def flops_per_pair(cfg: MoEConfig) -> int:
    """Useful FLOPs of one (token, expert) pair: three H x I projections."""
    return 3 * 2 * cfg.H * cfg.I


def make_layer_inputs(name: str, seed: int, device="cpu", T: Optional[int] = None):
    """(cfg, x, logits, bias) of a named workload; T overrides the token count."""
    cfg = WORKLOADS[name]
    if T is not None:
        cfg = cfg.with_T(T)
    x = make_activations(cfg, seed, device)
    if name == "tiny":
        return cfg, x, make_gate_logits(cfg, x, seed), None
    if name == "prefill":
        return cfg, x, make_normal_logits(cfg, seed, device), make_bias(cfg, seed, device, "zero")
    if name == "skew":
        return cfg, x, make_gate_logits(cfg, x, seed), make_bias(cfg, seed, device, "zipf")
    return cfg, x, make_gate_logits(cfg, x, seed), make_bias(cfg, seed, device, "small")


def small_fp8_layer(T=48, H=512, I=256, E=16, K=4, n_group=4, topk_group=2, has_shared=1) -> MoEConfig:
    """A scaled-down sigmoid / group-limited / FP8 layer the oracle finishes in seconds."""
    return MoEConfig(T=T, H=H, I=I, E=E, K=K, n_group=n_group, topk_group=topk_group,
                     has_shared=has_shared, score_fn=SCORE_SIGMOID, routed_scale=2.5, w_dtype=W_FP8)


def split_peers(n_routed: int, n_resident: int, n_peers: int):
    """Expert-id ranges of a DWDP placement: [0,n_resident) local, the rest split evenly over peers."""
    rest = n_routed - n_resident
    assert rest % n_peers == 0
    per = rest // n_peers
    return [(n_resident + p * per, n_resident + (p + 1) * per) for p in range(n_peers)]


def zipf_expected_hot_ratio(E: int = 256, s: float = ZIPF_S) -> float:
    """Hottest-to-mean probability ratio of a Zipf(s) law over E items (documentation aid)."""
    z = sum(r ** -s for r in range(1, E + 1))
    return (1.0 / z) * E
