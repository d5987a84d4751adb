"""CPU oracle for the DWDP MoE-layer hot path.  TEST INFRASTRUCTURE ONLY.

A plain, slow, obviously-correct numpy implementation of what one rank's MoE
layer computes: router top-k, permutation by expert, block-scaled FP8 (or MXFP4, or
bf16) expert MLP with SwiGLU, weighted combine.  Floating point is fp64 unless a step
fixes a precision (stated at the step).  Only tests, the smoke check and the
benchmark's cpu_baseline leg may import this package; it shares no code with the
HIP path and never imports it.

Where the definitions come from.  The paper (Section 2, "Methodology Overview";
Section 4.2, "Eliminating Split-Weight Merge Overhead") fixes *where* expert
weights live and that the grouped GEMM reads them from several buffers; it
delegates the MoE arithmetic itself to the DeepSeek-V3/R1 architecture
(Section 5.1, "Hardware, Software Stack, and Model").  The arithmetic below is
therefore the public DeepSeek-V3 MoE definition with the readings listed per
function.  The buffer placement does not change the function computed, so the
oracle takes each expert's weights by value.

Parity pins (tests/test_oracle_*.py): brute-force per-token selection, closed
forms for the e4m3 codec, library softmax / matmul special cases, permutation
invariants, dense-sum identity for combine (FP8 and MXFP4 weights), hand-valued
cases for the error metrics and the selection-margin report, a library-matmul
evaluation of the report-only reference without activation quantisation.
The absolute MoE output values have
no printed worked example in the paper: "parity unpinned" by the paper for
moe_forward's numeric output, pinned only by the identities above.
"""
from __future__ import annotations

import math
from dataclasses import dataclass
from typing import List, Optional, Sequence, Tuple

import numpy as np

SCORE_SOFTMAX = 0
SCORE_SIGMOID = 1
W_BF16 = 0
W_FP8 = 1
W_MXFP4 = 2


@dataclass(frozen=True)
class LayerSpec:
    """Routing and shape parameters of the layer (the oracle's own copy of the config)."""
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


def spec_from(cfg) -> LayerSpec:
    """Build a LayerSpec from any object with the same attribute names."""
    return LayerSpec(H=cfg.H, I=cfg.I, E=cfg.E, K=cfg.K, n_group=cfg.n_group, topk_group=cfg.topk_group,
                     has_shared=cfg.has_shared, score_fn=cfg.score_fn, routed_scale=cfg.routed_scale,
                     w_dtype=cfg.w_dtype)


# --------------------------------------------------------------------------------------
# FP8 e4m3 (OCP "fn" variant: 4 exponent bits, bias 7, 3 mantissa bits, no infinities,
# S.1111.111 = NaN, largest finite 448).  Written from the format definition.
# --------------------------------------------------------------------------------------

def e4m3_decode(code: int) -> float:
    """Value of one e4m3 byte."""
    sign = -1.0 if (code & 0x80) else 1.0
    exp = (code >> 3) & 0xF
    man = code & 0x7
    if exp == 0xF and man == 0x7:
        return math.nan
    if exp == 0:
        return sign * (man / 8.0) * 2.0 ** -6
    return sign * (1.0 + man / 8.0) * 2.0 ** (exp - 7)


E4M3_TABLE = np.array([e4m3_decode(c) for c in range(256)], dtype=np.float64)
# The 127 finite non-negative values in increasing order (codes 0x00..0x7E).
_E4M3_POS = E4M3_TABLE[:127].copy()


def e4m3_encode(v: np.ndarray) -> np.ndarray:
    """Round-to-nearest-even onto the e4m3 grid, saturating at +-448.  Returns uint8 codes.

    Nearest grid point by search over the sorted table; an exact midpoint goes to the
    neighbour with even code (even mantissa), which is IEEE round-half-even.
    """
    v = np.asarray(v, dtype=np.float64)
    a = np.minimum(np.abs(v), 448.0)
    hi = np.searchsorted(_E4M3_POS, a, side="left")          # first grid value >= a
    hi = np.minimum(hi, 126)
    lo = np.maximum(hi - 1, 0)
    d_lo = a - _E4M3_POS[lo]
    d_hi = _E4M3_POS[hi] - a
    pick_hi = (d_hi < d_lo) | ((d_hi == d_lo) & (hi % 2 == 0))
    code = np.where(pick_hi, hi, lo).astype(np.uint8)
    neg = np.signbit(v)
    return np.where(neg, code | 0x80, code).astype(np.uint8)


def qdq_act(v: np.ndarray, group: int = 128) -> Tuple[np.ndarray, np.ndarray, np.ndarray]:
    """Dynamic activation quantisation, per row and per `group` contiguous elements.

    Decision precision is fp32 (the precision the kernels use for it): v is taken as fp32,
    scale = fp32(amax) / fp32(448) (1.0 when the group is all zero), q = fp32(v / scale),
    code = RNE e4m3(q).  Returns (dequantised fp64 values, uint8 codes, fp32 scales [rows, n/group]).
    """
    v32 = np.asarray(v, dtype=np.float32)
    rows, n = v32.shape
    assert n % group == 0
    g = v32.reshape(rows, n // group, group)
    amax = np.abs(g).max(axis=2)
    scale = np.where(amax > 0, amax / np.float32(448.0), np.float32(1.0)).astype(np.float32)
    q = (g / scale[:, :, None]).astype(np.float32)
    codes = e4m3_encode(q)
    deq = E4M3_TABLE[codes] * scale[:, :, None].astype(np.float64)
    return deq.reshape(rows, n), codes.reshape(rows, n), scale


def dequant_blocks(codes: np.ndarray, scales: np.ndarray, block: int = 128) -> np.ndarray:
    """fp64 matrix from e4m3 bytes [R,C] and fp32 scales [R/block, C/block]."""
    R, C = codes.shape
    w = E4M3_TABLE[codes]
    s = np.repeat(np.repeat(scales.astype(np.float64), block, axis=0), block, axis=1)
    return w * s[:R, :C]


# --------------------------------------------------------------------------------------
# MXFP4 weights (OCP Microscaling Formats v1.0): elements are FP4 E2M1 (1 sign, 2 exponent
# bits with bias 1, 1 mantissa bit: magnitudes 0, 0.5, 1, 1.5, 2, 3, 4, 6), blocks of 32
# consecutive elements along K share one E8M0 scale 2^(byte - 127) (0xFF = NaN).  This is
# the AMD-native analogue of the NVFP4 weights the paper's model uses (its Section 5.1); the
# paper itself fixes no FP4 arithmetic, so the format definition is the specification.
# Storage: two codes per byte, element 2i in the low nibble of byte i.
# --------------------------------------------------------------------------------------

def e2m1_decode(code: int) -> float:
    """Value of one 4-bit E2M1 code."""
    sign = -1.0 if (code & 0x8) else 1.0
    exp = (code >> 1) & 0x3
    man = code & 0x1
    if exp == 0:
        return sign * 0.5 * man                     # subnormal: 0 or 0.5
    return sign * (1.0 + 0.5 * man) * 2.0 ** (exp - 1)


E2M1_TABLE = np.array([e2m1_decode(c) for c in range(16)], dtype=np.float64)


def e8m0_decode(code: np.ndarray) -> np.ndarray:
    """2^(code - 127) for uint8 codes; 255 is NaN."""
    c = np.asarray(code).astype(np.int64)
    return np.where(c == 255, np.nan, np.ldexp(1.0, c - 127))


def dequant_mxfp4(packed: np.ndarray, scales: np.ndarray, block: int = 32) -> np.ndarray:
    """fp64 matrix [R,C] from packed E2M1 codes uint8 [R,C/2] and E8M0 scales uint8 [R,C/block]."""
    R, half = packed.shape
    C = 2 * half
    codes = np.empty((R, C), dtype=np.uint8)
    codes[:, 0::2] = packed & 0xF
    codes[:, 1::2] = packed >> 4
    return E2M1_TABLE[codes] * np.repeat(e8m0_decode(scales), block, axis=1)[:, :C]


# --------------------------------------------------------------------------------------
# Router
# --------------------------------------------------------------------------------------

def _argsort_desc_stable(c: np.ndarray) -> np.ndarray:
    """Indices by descending value; equal values keep the lower index first."""
    return np.argsort(-c, kind="stable")


def route(logits: np.ndarray, bias: Optional[np.ndarray], spec: LayerSpec):
    """Router top-k.  Returns (topk_ids int32 [T,K], topk_w fp32 [T,K]).

    Sigmoid scoring (DeepSeek-V3 style):
      s_e = fp32( 1 / (1 + exp(-fp64(z_e))) )      evaluated in fp64, rounded once
      c_e = fp32(s_e + b_e)                        selection score; the bias only selects
      group score = fp32 sum of the two largest c_e of the group (groups = contiguous E/n_group)
      keep the topk_group best groups, then the K best c_e among their experts
      w_k = s_{e_k} / (sum_j s_{e_j} + 1e-20) * routed_scale        (un-biased scores)
    Softmax scoring: selection on the raw logits (softmax is monotone), no bias, and
      w = softmax over the K selected logits times routed_scale (equal to the full softmax
      renormalised over the selection).
    Ties go to the lower expert / group index; ids are listed by descending selection score.
    """
    z = np.asarray(logits, dtype=np.float32)
    T, E = z.shape
    assert E == spec.E
    K = spec.K
    ids = np.zeros((T, K), dtype=np.int32)
    w = np.zeros((T, K), dtype=np.float32)
    gs = E // spec.n_group
    for t in range(T):
        if spec.score_fn == SCORE_SIGMOID:
            s = (1.0 / (1.0 + np.exp(-z[t].astype(np.float64)))).astype(np.float32)
            c = s + bias.astype(np.float32) if bias is not None else s.copy()
        else:
            s = None
            c = z[t].copy()
        c = c.astype(np.float32)
        masked = c.astype(np.float64)
        if spec.n_group > 1:
            gscore = np.zeros(spec.n_group, dtype=np.float32)
            for g in range(spec.n_group):
                grp = np.sort(c[g * gs:(g + 1) * gs])[::-1]
                gscore[g] = np.float32(grp[0]) + np.float32(grp[1])
            keep = _argsort_desc_stable(gscore)[:spec.topk_group]
            allowed = np.zeros(E, dtype=bool)
            for g in keep:
                allowed[g * gs:(g + 1) * gs] = True
            masked = np.where(allowed, masked, -np.inf)
        sel = _argsort_desc_stable(masked)[:K]
        ids[t] = sel
        if spec.score_fn == SCORE_SIGMOID:
            sv = s[sel].astype(np.float64)
            w[t] = (sv / (sv.sum() + 1e-20) * spec.routed_scale).astype(np.float32)
        else:
            zv = z[t][sel].astype(np.float64)
            ex = np.exp(zv - zv.max())
            w[t] = (ex / ex.sum() * spec.routed_scale).astype(np.float32)
    return ids, w


# --------------------------------------------------------------------------------------
# Permutation by expert
# --------------------------------------------------------------------------------------

def permute(topk_ids: np.ndarray, spec: LayerSpec):
    """Stable counting sort of the flat (token, slot) index f = t*K + k by expert id.

    Returns (expert_offsets int32 [E+1 (+1 if shared)], perm int32 [T*K], inv_perm int32 [T*K]):
      rows expert_offsets[e] .. expert_offsets[e+1]-1 of the sorted order belong to expert e,
      perm[r] = f of sorted row r, inv_perm[f] = r.  Within an expert rows keep increasing f
      (hence increasing token).  With a shared expert one more group follows the routed ones:
      rows T*K + t for t = 0..T-1, so expert_offsets[E+1] = T*K + T.
    """
    T, K = topk_ids.shape
    flat = topk_ids.reshape(-1)
    counts = np.zeros(spec.E, dtype=np.int64)
    for e in flat:
        counts[e] += 1
    n_off = spec.E + 1 + (1 if spec.has_shared else 0)
    offsets = np.zeros(n_off, dtype=np.int32)
    for e in range(spec.E):
        offsets[e + 1] = offsets[e] + counts[e]
    if spec.has_shared:
        offsets[spec.E + 1] = T * K + T
    cursor = offsets[:spec.E].astype(np.int64).copy()
    perm = np.zeros(T * K, dtype=np.int32)
    inv = np.zeros(T * K, dtype=np.int32)
    for f in range(T * K):
        e = flat[f]
        r = cursor[e]
        cursor[e] += 1
        perm[r] = f
        inv[f] = r
    return offsets, perm, inv


# --------------------------------------------------------------------------------------
# Expert MLP and the layer
# --------------------------------------------------------------------------------------

@dataclass
class ExpertNumpy:
    """One expert's weights, logical layouts: w13 [2I,H] (gate rows then up rows), w2 [H,I].
    FP8: uint8 codes + fp32 scales per 128x128 block.  MXFP4: packed E2M1 codes (two per byte
    along the second axis) + uint8 E8M0 scales per 32 elements.  bf16: float arrays holding
    bf16 values."""
    w13: np.ndarray
    w2: np.ndarray
    s13: Optional[np.ndarray] = None
    s2: Optional[np.ndarray] = None

    def dense(self) -> Tuple[np.ndarray, np.ndarray]:
        if self.s13 is None:
            return self.w13.astype(np.float64), self.w2.astype(np.float64)
        if self.s13.dtype == np.uint8:
            return dequant_mxfp4(self.w13, self.s13), dequant_mxfp4(self.w2, self.s2)
        return dequant_blocks(self.w13, self.s13), dequant_blocks(self.w2, self.s2)


def silu(g: np.ndarray) -> np.ndarray:
    return g / (1.0 + np.exp(-g))


def expert_mlp(x_rows: np.ndarray, expert: ExpertNumpy, spec: LayerSpec, act_quant: bool = True) -> np.ndarray:
    """o = W_down ( QDQ( silu(W_gate x~) * (W_up x~) ) ),  x~ = QDQ(x), rows of x_rows at once.

    QDQ is the per-token, per-128 e4m3 activation quantisation and exists for FP8 and MXFP4
    weights (the matrix cores need an FP8 activation operand beside them, so the quantisation
    is part of the function both sides compute); for bf16 weights it is the identity.  fp64
    everywhere else.

    act_quant=False drops both QDQ steps: the same dequantised weights applied to the
    un-quantised activations.  That is the other reading of "bf16 activations, FP8 weights"
    (a weight-only-quantised layer); it is never the parity reference, tests and the
    benchmark only REPORT the distance of the GPU result to it, so that the cost of
    quantising the activations stays visible.
    """
    I = spec.I
    w13, w2 = expert.dense()
    xr = np.asarray(x_rows, dtype=np.float64)
    quantised = act_quant and spec.w_dtype in (W_FP8, W_MXFP4)
    if quantised:
        xr = qdq_act(xr)[0]
    gu = xr @ w13.T
    h = silu(gu[:, :I]) * gu[:, I:]
    if quantised:
        h = qdq_act(h)[0]
    return h @ w2.T


def moe_forward(x: np.ndarray, logits: np.ndarray, bias: Optional[np.ndarray],
                experts: Sequence[Optional[ExpertNumpy]], spec: LayerSpec,
                tokens: Optional[Sequence[int]] = None, act_quant: bool = True) -> np.ndarray:
    """y_t = sum_k w_{t,k} * MLP_{e_{t,k}}(x_t)  (+ MLP_shared(x_t), weight 1, not scaled).

    experts[e] for e < E are routed experts, experts[E] the shared one.  Works expert by
    expert over the permuted rows (one dequantised expert in memory at a time).  `tokens`
    restricts the output to a subset of tokens (experts none of them selects may be None).
    act_quant: see expert_mlp (False = report-only reference without activation quantisation).
    Returns fp64 [len(tokens) or T, H].
    """
    T = x.shape[0]
    ids, w = route(logits, bias, spec)
    tok = np.arange(T) if tokens is None else np.asarray(list(tokens), dtype=np.int64)
    pos = {int(t): i for i, t in enumerate(tok)}
    y = np.zeros((len(tok), spec.H), dtype=np.float64)
    offsets, perm, _ = permute(ids, spec)
    xf = np.asarray(x, dtype=np.float64)
    for e in range(spec.E):
        rows = perm[offsets[e]:offsets[e + 1]]
        rows = [f for f in rows if (f // spec.K) in pos]
        if not rows:
            continue
        ts = np.array([f // spec.K for f in rows])
        ks = np.array([f % spec.K for f in rows])
        o = expert_mlp(xf[ts], experts[e], spec, act_quant)
        for i in range(len(rows)):
            y[pos[int(ts[i])]] += float(w[ts[i], ks[i]]) * o[i]
    if spec.has_shared:
        o = expert_mlp(xf[tok], experts[spec.E], spec, act_quant)
        y += o
    return y


def moe_forward_bruteforce(x, logits, bias, experts, spec: LayerSpec) -> np.ndarray:
    """The same function written token by token with no permutation at all: for each token,
    sort its scores, loop over the chosen experts, add.  Used to pin moe_forward/permute."""
    T = x.shape[0]
    ids, w = route(logits, bias, spec)
    y = np.zeros((T, spec.H), dtype=np.float64)
    dense = [ex.dense() if ex is not None else None for ex in experts]
    quantised = spec.w_dtype in (W_FP8, W_MXFP4)     # FP8 activations beside FP8 and MXFP4 weights
    for t in range(T):
        xt = np.asarray(x[t], dtype=np.float64)[None, :]
        if quantised:
            xt = qdq_act(xt)[0]
        chosen = [(int(ids[t, k]), float(w[t, k])) for k in range(spec.K)]
        if spec.has_shared:
            chosen.append((spec.E, 1.0))
        for e, wk in chosen:
            w13, w2 = dense[e]
            g = w13[:spec.I] @ xt[0]
            u = w13[spec.I:] @ xt[0]
            h = (g / (1.0 + np.exp(-g)) * u)[None, :]
            if quantised:
                h = qdq_act(h)[0]
            y[t] += wk * (w2 @ h[0])
    return y


def error_metrics(y: np.ndarray, ref: np.ndarray) -> Tuple[float, float]:
    """(max |y-ref| / max |ref|, ||y-ref||_2 / ||ref||_2): the parity metric and an L2 companion."""
    y = np.asarray(y, dtype=np.float64)
    ref = np.asarray(ref, dtype=np.float64)
    d = np.abs(y - ref)
    return float(d.max() / np.abs(ref).max()), float(np.linalg.norm(y - ref) / np.linalg.norm(ref))


def error_metric_rows(y: np.ndarray, ref: np.ndarray) -> float:
    """max over rows t of ( max_i |y[t,i]-ref[t,i]| / max_i |ref[t,i]| ): the same metric taken
    token by token, so that a token whose output is small cannot hide behind a large one.
    Rows of ref that are entirely zero are compared absolutely (their error must be zero to pass)."""
    y = np.asarray(y, dtype=np.float64)
    ref = np.asarray(ref, dtype=np.float64)
    y = y.reshape(-1, y.shape[-1])
    ref = ref.reshape(-1, ref.shape[-1])
    d = np.abs(y - ref).max(axis=1)
    m = np.abs(ref).max(axis=1)
    rel = np.where(m > 0, d / np.where(m > 0, m, 1.0), np.where(d > 0, np.inf, 0.0))
    return float(rel.max()) if rel.size else 0.0


def route_margins(logits: np.ndarray, bias: Optional[np.ndarray], spec: LayerSpec) -> Tuple[np.ndarray, np.ndarray]:
    """How close each token's selection is to a different outcome, in units of fp32 spacing.

    Returns (expert_margin [T], group_margin [T]): the gap between the K-th selected and the
    best unselected selection score among the kept groups, and between the last kept and the
    best dropped group score (inf when nothing is dropped), each divided by the fp32 spacing
    (ulp) at the larger of the two magnitudes.  A margin of 0 is an exact tie (decided by the
    index rule); margins of a few ulp mark tokens whose ids would change under a one-ulp
    difference of the sigmoid between two exp implementations.  Uses the same score
    definitions as route().
    """
    z = np.asarray(logits, dtype=np.float32)
    T, E = z.shape
    gs = E // spec.n_group
    em = np.full(T, np.inf)
    gm = np.full(T, np.inf)

    def ulps(a, b):
        big = np.float32(max(abs(float(a)), abs(float(b)), np.finfo(np.float32).tiny))
        return abs(float(a) - float(b)) / float(np.spacing(big))

    for t in range(T):
        if spec.score_fn == SCORE_SIGMOID:
            s = (1.0 / (1.0 + np.exp(-z[t].astype(np.float64)))).astype(np.float32)
            c = (s + bias.astype(np.float32)).astype(np.float32) if bias is not None else s
        else:
            c = z[t]
        allowed = np.ones(E, dtype=bool)
        if spec.n_group > 1:
            gscore = np.zeros(spec.n_group, dtype=np.float32)
            for g in range(spec.n_group):
                top = np.sort(c[g * gs:(g + 1) * gs])[::-1]
                gscore[g] = np.float32(top[0]) + np.float32(top[1])
            order = _argsort_desc_stable(gscore)
            if spec.topk_group < spec.n_group:
                gm[t] = ulps(gscore[order[spec.topk_group - 1]], gscore[order[spec.topk_group]])
            allowed[:] = False
            for g in order[:spec.topk_group]:
                allowed[g * gs:(g + 1) * gs] = True
        cand = np.sort(c[allowed])[::-1]
        if len(cand) > spec.K:
            em[t] = ulps(cand[spec.K - 1], cand[spec.K])
    return em, gm
