"""Host-side checks that need no GPU: the library loads, exports every symbol the header
declares, and the copy-plan builder follows the round-robin slice order of the paper's
Section 4.3.2 (Listing 1) -- compared with the oracle's plan and the hand-worked fixture."""
import ctypes as C
import os
import re

import pytest

from oracle import prefetch_oracle as po
from paper_2604_01621_amd import binding

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def test_library_exports_every_declared_symbol():
    hdr = open(os.path.join(ROOT, "include", "dwdp.h")).read()
    names = set(re.findall(r"\b(dwdp_[a-z_0-9]+)\s*\(", hdr))
    names -= {"dwdp_ctx"}
    assert {"dwdp_route", "dwdp_permute", "dwdp_moe_forward", "dwdp_prefetch_layer"} <= names
    lib = C.CDLL(binding.LIB_PATH)
    for n in sorted(names):
        assert hasattr(lib, n), f"{n} declared in dwdp.h but not exported"


def test_struct_layouts_match_header():
    assert C.sizeof(binding.dwdp_expert_ptrs) == 32
    assert C.sizeof(binding.dwdp_config) == 48


def test_copy_plan_matches_fixture_and_oracle():
    want = [tuple(int(v) for v in l.split()) for l in open(os.path.join(ROOT, "tests", "golden", "listing1_plan.txt"))
            if l.strip() and l[0] != "#"]
    peers = [1, 2, 3]
    src = [1000 * q + 100 * p for q in peers for p in range(2)]
    dst = [50000 + 1000 * q + 100 * p for q in peers for p in range(2)]
    plan = binding.build_copy_plan(src, dst, [10, 4], 3, 2, 4)
    assert plan == want


@pytest.mark.parametrize("M,s,n_peers", [([1000, 24, 7], 64, 2), ([5], 100, 1), ([256, 256, 0, 3], 128, 3),
                                          ([1 << 20, 12345], 0, 3), ([], 16, 2), ([8], 16, 0)])
def test_copy_plan_vs_oracle(M, s, n_peers):
    n_params = len(M)
    src = [10 ** 9 * (q + 1) + 10 ** 7 * p for q in range(n_peers) for p in range(n_params)]
    dst = [10 ** 12 + 10 ** 9 * (q + 1) + 10 ** 7 * p for q in range(n_peers) for p in range(n_params)]
    plan = binding.build_copy_plan(src, dst, M, n_peers, n_params, s)
    srcd = {q: src[q * n_params:(q + 1) * n_params] for q in range(n_peers)}
    dstd = {q: dst[q * n_params:(q + 1) * n_params] for q in range(n_peers)}
    s_eff = s if s else max(max(M, default=1), 1)
    want = po.copy_plan(M, list(range(n_peers)), s_eff, srcd, dstd)
    assert plan == want


def test_create_rejects_bad_shapes_without_gpu():
    """Argument errors are detected before any HIP call, so this runs on a CPU-only host."""
    lib = binding.lib
    h = C.c_void_p()
    good = dict(T_max=4, H=256, I=128, E=8, K=2, n_group=1, topk_group=1, has_shared=0, score_fn=0,
                routed_scale=1.0, w_dtype=0, n_layers=1)
    for bad, code in [(dict(H=200), binding.ESHAPE), (dict(K=9), binding.ESHAPE), (dict(E=2048), binding.ESHAPE),
                      (dict(n_group=3), binding.ESHAPE), (dict(score_fn=7), binding.EINVAL),
                      (dict(n_layers=0), binding.EINVAL), (dict(n_group=8, topk_group=1, K=2), binding.ESHAPE),
                      (dict(w_dtype=5), binding.EINVAL)]:
        cfg = binding.dwdp_config(**{**good, **bad})
        assert lib.dwdp_create(C.byref(cfg), None, C.byref(h)) == code, bad
        assert lib.dwdp_last_error(None)
        assert not h.value
    assert lib.dwdp_create(None, None, C.byref(h)) == binding.EINVAL
    assert lib.dwdp_route(None, None, None, 0, None, None) == binding.EINVAL


def test_permute_static_rejects_bad_arguments_without_gpu():
    """The allocation-free permutation checks its arguments and its scratch limit before any HIP call."""
    lib = binding.lib
    one = C.c_void_p(16)       # any non-NULL value: rejected calls never touch the pointers
    assert lib.dwdp_permute_static(one, -1, 8, 2, 0, None, one, one, one) == binding.EINVAL
    assert lib.dwdp_permute_static(one, 4, 0, 2, 0, None, one, one, one) == binding.EINVAL
    assert lib.dwdp_permute_static(one, 4, 8, 2, 2, None, one, one, one) == binding.EINVAL
    assert lib.dwdp_permute_static(one, 4, 2048, 2, 0, None, one, one, one) == binding.ESHAPE
    assert lib.dwdp_permute_static(one, 4, 8, 9, 0, None, one, one, one) == binding.ESHAPE
    assert lib.dwdp_permute_static(one, 4, 8, 2, 0, None, None, one, one) == binding.EINVAL
    assert lib.dwdp_permute_static(None, 4, 8, 2, 0, None, one, one, one) == binding.EINVAL
    # scratch limit: ceil(T / 128) * E * 4 bytes must fit DWDP_STATIC_SCRATCH_BYTES = 1 MiB
    assert lib.dwdp_permute_static(one, 131072 + 1, 256, 8, 1, None, one, one, one) == binding.ESHAPE
    assert b"scratch" in lib.dwdp_last_error(None)
