"""Split-weight layer stack for the prefetch pipeline: device buffers and pointer tables only.

One rank of a DWDP group (paper Section 2): each layer keeps `n_resident` routed experts
(plus the shared expert) in a resident buffer; the other routed experts live in a separate
HBM pool that plays the peers (`n_peers` equal shards).  Two staging buffers receive a
layer's non-resident experts one layer ahead.  A layer's pointer table mixes resident and
staging addresses and is fixed once the buffers exist, because layer l always stages into
buffer l % 2.

Per (peer, layer) the pulled data are four contiguous parameters (paper Section 4.3.2 calls
them "parameters p"): W13 codes, W13 scales, W2 codes, W2 scales of that peer's experts.
Everything here is allocation and pointer arithmetic; the copies and the compute are the
library's (dwdp_prefetch_layer, dwdp_moe_forward).
"""
from __future__ import annotations

from typing import List, Optional

import torch

from . import inputs
from .inputs import ExpertWeights, MoEConfig

N_PARAMS = 4  # w13 codes, w13 scales, w2 codes, w2 scales


class _Shard:
    """Experts [lo, hi) of one layer stored as four contiguous parameter regions."""

    def __init__(self, cfg: MoEConfig, n: int, device):
        H, I = cfg.H, cfg.I
        self.n = n
        self.w13 = torch.empty(n, 2 * I, H, dtype=torch.uint8, device=device)
        self.s13 = torch.empty(n, 2 * I // 128, H // 128, dtype=torch.float32, device=device)
        self.w2 = torch.empty(n, H, I, dtype=torch.uint8, device=device)
        self.s2 = torch.empty(n, H // 128, I // 128, dtype=torch.float32, device=device)

    def params(self):
        return [self.w13, self.s13, self.w2, self.s2]

    def ptrs(self) -> List[int]:
        return [p.data_ptr() for p in self.params()]

    def nbytes(self) -> List[int]:
        return [p.numel() * p.element_size() for p in self.params()]

    def fill_from(self, w: ExpertWeights, lo: int, hi: int):
        self.w13.copy_(w.w13[lo:hi])
        self.s13.copy_(w.s13[lo:hi])
        self.w2.copy_(w.w2[lo:hi])
        self.s2.copy_(w.s2[lo:hi])

    def row(self, i: int) -> List[int]:
        return [self.w13[i].data_ptr(), self.s13[i].data_ptr(), self.w2[i].data_ptr(), self.s2[i].data_ptr()]


class SplitWeightLayers:
    def __init__(self, ctx, cfg: MoEConfig, n_layers: int, n_resident: int, n_peers: int, seed: int, device="cuda"):
        assert cfg.w_dtype == inputs.W_FP8 and cfg.has_shared == 1
        self.cfg, self.n_layers, self.n_resident, self.n_peers = cfg, n_layers, n_resident, n_peers
        self.ranges = inputs.split_peers(cfg.E, n_resident, n_peers)
        per = self.ranges[0][1] - self.ranges[0][0]
        self.per = per
        # resident: experts [0, n_resident) then the shared expert
        self.resident = [_Shard(cfg, n_resident + 1, device) for _ in range(n_layers)]
        self.peer = [[_Shard(cfg, per, device) for _ in range(n_peers)] for _ in range(n_layers)]
        self.staging = [[_Shard(cfg, per, device) for _ in range(n_peers)] for _ in range(2)]
        self.logical: List[Optional[ExpertWeights]] = [None] * n_layers
        self.seeds = [seed + l for l in range(n_layers)]
        for l in range(n_layers):
            w = inputs.make_expert_weights(cfg, self.seeds[l], device=device)
            wp = ctx.pack_experts(w)
            res = self.resident[l]
            idx = list(range(n_resident)) + [cfg.E]
            res.w13.copy_(wp.w13[idx])
            res.s13.copy_(wp.s13[idx])
            res.w2.copy_(wp.w2[idx])
            res.s2.copy_(wp.s2[idx])
            for p, (lo, hi) in enumerate(self.ranges):
                self.peer[l][p].fill_from(wp, lo, hi)
            del wp
            self.logical[l] = w
        torch.cuda.synchronize()
        self.tables = [self._table(l, device) for l in range(n_layers)]

    def drop_logical(self):
        """Free the row-major copies kept for the oracle (large workloads)."""
        self.logical = [None] * self.n_layers

    def _table(self, l: int, device, staging=None) -> torch.Tensor:
        cfg = self.cfg
        staging = self.staging[l % 2] if staging is None else staging
        rows = []
        for e in range(cfg.E):
            if e < self.n_resident:
                rows.append(self.resident[l].row(e))
            else:
                p = (e - self.n_resident) // self.per
                rows.append(staging[p].row(e - self.ranges[p][0]))
        rows.append(self.resident[l].row(self.n_resident))      # shared expert
        return torch.tensor(rows, dtype=torch.int64).to(device)

    def new_puller_staging(self, device="cuda") -> List[_Shard]:
        """One more staging buffer over the same peers: the landing area of another puller (a
        second context standing for another rank that pulls from the same sources)."""
        return [_Shard(self.cfg, self.per, device) for _ in range(self.n_peers)]

    def puller_table(self, l: int, staging, device="cuda") -> torch.Tensor:
        """Layer l's table for a puller that stages into `staging` (from new_puller_staging)."""
        return self._table(l, device, staging)

    def puller_prefetch(self, ctx, l: int, staging, slice_bytes: int, first_peer: int = 0):
        """dwdp_prefetch_layer(l) of context `ctx` into `staging`, peers visited in the order
        first_peer, first_peer + 1, ... (paper Section 4.3.2: every puller walks its own peer order)."""
        src, dst = [], []
        for i in range(self.n_peers):
            p = (first_peer + i) % self.n_peers
            src += self.peer[l][p].ptrs()
            dst += staging[p].ptrs()
        ctx.dwdp_prefetch_layer(l, src, dst, self.peer[l][0].nbytes(), self.n_peers, N_PARAMS, slice_bytes)

    def all_resident_table(self, l: int, device="cuda") -> torch.Tensor:
        """Table of the same layer reading the peer pool in place (reference for equivalence tests)."""
        rows = []
        for e in range(self.cfg.E):
            if e < self.n_resident:
                rows.append(self.resident[l].row(e))
            else:
                p = (e - self.n_resident) // self.per
                rows.append(self.peer[l][p].row(e - self.ranges[p][0]))
        rows.append(self.resident[l].row(self.n_resident))
        return torch.tensor(rows, dtype=torch.int64).to(device)

    def prefetch_args(self, l: int):
        """(src, dst, bytes) for dwdp_prefetch_layer(l): index peer * N_PARAMS + p."""
        src, dst = [], []
        for p in range(self.n_peers):
            src += self.peer[l][p].ptrs()
            dst += self.staging[l % 2][p].ptrs()
        return src, dst, self.peer[l][0].nbytes()

    def prefetch_bytes(self) -> int:
        return self.n_peers * sum(self.peer[0][0].nbytes())

    def prefetch(self, ctx, l: int, slice_bytes: int):
        src, dst, nb = self.prefetch_args(l)
        ctx.dwdp_prefetch_layer(l, src, dst, nb, self.n_peers, N_PARAMS, slice_bytes)

    def poison_staging(self, b: int, staging=None):
        """Fill staging buffer b (or the given puller's landing buffer) with 0xFF bytes (e4m3 NaN
        codes, NaN scales) on the current stream."""
        for sh in (self.staging[b] if staging is None else staging):
            sh.w13.fill_(0xFF)
            sh.w2.fill_(0xFF)
            sh.s13.view(torch.uint8).fill_(0xFF)
            sh.s2.view(torch.uint8).fill_(0xFF)
