"""CPU oracle for the DWDP prefetch side.  TEST INFRASTRUCTURE ONLY.

Covers the host-side pieces the paper does define:
  * the batched prefetch-copy plan in round-robin slice order (Section 4.3.2, Listing 1),
  * the contention-level distribution of the random asynchronous model (Section 4.3.1,
    Eqs. (1)-(2), Table 2),
  * the layer-ahead double-buffered schedule (Section 2): which staging buffer a layer
    uses and what each copy / compute step has to wait for.
Nothing here is imported by the product path.
"""
from __future__ import annotations

from math import comb
from typing import List, Sequence, Tuple


def copy_plan(prefetch_size: Sequence[int], peers: Sequence[int], slice_bytes: int,
              src_base, dst_base) -> List[Tuple[int, int, int]]:
    """Ordered list of (dst, src, chunk) copies (Section 4.3.2, Listing 1).

    prefetch_size[p] = M, bytes to pull of parameter p from *each* remote peer;
    peers = remote peers in the fixed round-robin order of this rank;
    src_base[peer][p] = address of the peer's region of parameter p (peer pointer plus the
    source offset of the pulled shard); dst_base[peer][p] = local staging address for it.
    Every pull is cut into ceil(M / s) slices; slice offsets are the outer loop and the
    peers the inner loop, so consecutive copies come from different source ranks.
    """
    assert slice_bytes > 0
    n_peers = len(peers)
    plan = []
    for p, M in enumerate(prefetch_size):
        # Copy i of this parameter moves slice i // n_peers of the pull from peer i % n_peers:
        # the slice index changes slowest, so each round of n_peers copies visits every source once.
        for i in range(n_slices(M, slice_bytes) * n_peers):
            k, q = divmod(i, n_peers)
            lo = k * slice_bytes
            plan.append((dst_base[peers[q]][p] + lo, src_base[peers[q]][p] + lo, min(slice_bytes, M - lo)))
    return plan


def n_slices(M: int, s: int) -> int:
    """K = ceil(M / s) (Section 4.3.2)."""
    return -(-M // s)


def contention_pmf(N: int) -> List[float]:
    """Pr[C = c] for c = 1..N-1 in a DWDP group of N ranks (Section 4.3.1).

    After the tagged rank picks a source, each of the other N-2 ranks picks the same one
    with probability 1/(N-1); X ~ Binomial(N-2, 1/(N-1)) and C = X + 1.
    """
    n, p = N - 2, 1.0 / (N - 1)
    return [comb(n, c - 1) * p ** (c - 1) * (1 - p) ** (n - (c - 1)) for c in range(1, N)]


def pull_service_time(T_total: float, N: int) -> float:
    """tau = T / (N - 1): ideal service time of one of the N-1 serial pulls (Eq. (1))."""
    return T_total / (N - 1)


def pipeline_schedule(n_layers: int, n_buffers: int = 2):
    """Symbolic layer-ahead schedule (Section 2).

    Returns a list of steps in issue order; each step is
      ("prefetch", l, buffer, wait_for)  copy of layer l's remote experts into `buffer`,
                                         legal only once `wait_for` = ("moe", l - n_buffers)
                                         has finished (None for the first n_buffers layers),
      ("moe", l, buffer, wait_for)       MoE block of layer l, reading `buffer`,
                                         legal only once ("prefetch", l) has finished.
    The prefetch of layer l+1 is issued before the MoE block of layer l so that it runs
    underneath it; layer l's staging buffer is l mod n_buffers and is released (reusable)
    once its MoE block is done.
    """
    steps = []

    def prefetch(l):
        dep = ("moe", l - n_buffers) if l - n_buffers >= 0 else None
        steps.append(("prefetch", l, l % n_buffers, dep))

    prefetch(0)
    for l in range(n_layers):
        if l + 1 < n_layers:
            prefetch(l + 1)
        steps.append(("moe", l, l % n_buffers, ("prefetch", l)))
    return steps
