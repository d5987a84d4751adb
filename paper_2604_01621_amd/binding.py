"""ctypes binding of libdwdp.so: argument marshalling only.

Function names match the C entry points declared in include/dwdp.h.  Tensors are torch
tensors used as device memory; every step of the path runs inside the library's kernels.
Importing this module fails loudly when the library has not been built: there is no
Python or CPU fallback.
"""
from __future__ import annotations

import ctypes as C
import os
from typing import List, Optional, Sequence

import torch

from .inputs import MoEConfig, ExpertWeights

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libdwdp.so")

OK, EINVAL, ESHAPE, ENOMEM, EHIP, ESTATE = range(6)
DEFAULT_STREAM_MAX_ROWS = 64     # the library's default kernel-selection threshold (dwdp_set_stream_max_rows)
STAGES = ("route", "permute", "quant", "gemm1", "gemm2", "combine", "gemm1_tile", "gemm2_tile")
WS = {"topk_ids": 0, "topk_w": 1, "offsets": 2, "perm": 3, "inv_perm": 4, "xq": 5, "xs": 6, "hq": 7, "hs": 8, "yp": 9, "sched": 10}


class dwdp_config(C.Structure):
    _fields_ = [("T_max", C.c_int32), ("H", C.c_int32), ("I", C.c_int32), ("E", C.c_int32), ("K", C.c_int32),
                ("n_group", C.c_int32), ("topk_group", C.c_int32), ("has_shared", C.c_int32),
                ("score_fn", C.c_int32), ("routed_scale", C.c_float), ("w_dtype", C.c_int32),
                ("n_layers", C.c_int32)]


class dwdp_expert_ptrs(C.Structure):
    _fields_ = [("w13", C.c_void_p), ("s13", C.c_void_p), ("w2", C.c_void_p), ("s2", C.c_void_p)]


class DwdpError(RuntimeError):
    def __init__(self, status: int, msg: str):
        super().__init__(f"dwdp status {status}: {msg}")
        self.status = status


def _load() -> C.CDLL:
    if not os.path.exists(LIB_PATH):
        raise ImportError(f"{LIB_PATH} is missing: build it with `python -m paper_2604_01621_amd.build` "
                          "(there is no fallback path)")
    lib = C.CDLL(LIB_PATH)
    vp, i32, sz = C.c_void_p, C.c_int32, C.c_size_t
    lib.dwdp_create.argtypes = [C.POINTER(dwdp_config), vp, C.POINTER(vp)]
    lib.dwdp_destroy.argtypes = [vp]
    lib.dwdp_destroy.restype = None
    lib.dwdp_last_error.argtypes = [vp]
    lib.dwdp_last_error.restype = C.c_char_p
    lib.dwdp_route.argtypes = [vp, vp, vp, i32, vp, vp]
    lib.dwdp_permute.argtypes = [vp, vp, i32, vp, vp, vp]
    lib.dwdp_moe_forward.argtypes = [vp, i32, vp, vp, vp, i32, vp, vp]
    lib.dwdp_prefetch_layer.argtypes = [vp, i32, C.POINTER(vp), C.POINTER(vp), C.POINTER(sz), i32, i32, sz]
    lib.dwdp_prepare_prefetch.argtypes = [vp, i32, C.POINTER(vp), C.POINTER(vp), C.POINTER(sz), i32, i32, sz]
    lib.dwdp_permute_static.argtypes = [vp, i32, i32, i32, i32, vp, vp, vp, vp]
    lib.dwdp_build_copy_plan.argtypes = [C.POINTER(vp), C.POINTER(vp), C.POINTER(sz), i32, i32, sz,
                                         C.POINTER(vp), C.POINTER(vp), C.POINTER(sz), sz, C.POINTER(sz)]
    lib.dwdp_merge_experts.argtypes = [vp, i32, C.POINTER(dwdp_expert_ptrs), i32, vp, vp, vp, vp,
                                       C.POINTER(dwdp_expert_ptrs)]
    lib.dwdp_set_stream_max_rows.argtypes = [vp, i32]
    lib.dwdp_set_tile_schedule.argtypes = [vp, i32]
    lib.dwdp_set_tile_share.argtypes = [vp, i32]
    lib.dwdp_set_copy_engine.argtypes = [vp, i32, i32]
    lib.dwdp_pack_fp8_weight.argtypes = [vp, vp, vp, C.c_int64, C.c_int64]
    lib.dwdp_pack_mxfp4_weight.argtypes = [vp, vp, vp, vp, vp, C.c_int64, C.c_int64]
    lib.dwdp_profile_enable.argtypes = [vp, i32]
    lib.dwdp_profile_read.argtypes = [vp, C.POINTER(C.c_float), C.POINTER(i32)]
    lib.dwdp_timeline_enable.argtypes = [vp, i32]
    fp, ip = C.POINTER(C.c_float), C.POINTER(i32)
    lib.dwdp_timeline_read.argtypes = [vp, ip, ip, fp, fp, i32, ip]
    lib.dwdp_workspace_ptr.argtypes = [vp, i32]
    lib.dwdp_workspace_ptr.restype = vp
    lib.dwdp_copy_stream.argtypes = [vp]
    lib.dwdp_copy_stream.restype = vp
    return lib


lib = _load()


def _ptr(t: Optional[torch.Tensor]):
    if t is None:
        return None
    assert t.is_contiguous()
    return C.c_void_p(t.data_ptr())


def build_copy_plan(src: Sequence[int], dst: Sequence[int], nbytes: Sequence[int], n_peers: int, n_params: int,
                    slice_bytes: int):
    """dwdp_build_copy_plan: returns [(dst, src, chunk), ...] (host only, no GPU needed)."""
    vp, sz = C.c_void_p, C.c_size_t
    n = n_peers * n_params
    a_src = (vp * max(n, 1))(*[vp(v) for v in src])
    a_dst = (vp * max(n, 1))(*[vp(v) for v in dst])
    a_b = (sz * max(n_params, 1))(*nbytes)
    cnt = sz(0)
    st = lib.dwdp_build_copy_plan(a_src, a_dst, a_b, n_peers, n_params, slice_bytes, None, None, None, 0, C.byref(cnt))
    if st != OK:
        raise DwdpError(st, "dwdp_build_copy_plan")
    m = cnt.value
    pd, ps, pb = (vp * max(m, 1))(), (vp * max(m, 1))(), (sz * max(m, 1))()
    st = lib.dwdp_build_copy_plan(a_src, a_dst, a_b, n_peers, n_params, slice_bytes, pd, ps, pb, m, C.byref(cnt))
    if st != OK:
        raise DwdpError(st, "dwdp_build_copy_plan")
    return [(pd[i] or 0, ps[i] or 0, pb[i]) for i in range(m)]


def mx_scale_bytes(rows: int, cols: int) -> int:
    """Bytes of the packed MXFP4 scales of one [rows, cols] matrix (see dwdp_pack_mxfp4_weight)."""
    return (rows // 16) * ((cols // 128 + 3) // 4) * 256


def expert_table(weights: ExpertWeights, device=None) -> torch.Tensor:
    """Pointer table (int64 [n,4] = rows of dwdp_expert_ptrs) for experts stored back to back."""
    rows = []
    for e in range(weights.n):
        rows.append([weights.w13[e].data_ptr(), weights.s13[e].data_ptr() if weights.s13 is not None else 0,
                     weights.w2[e].data_ptr(), weights.s2[e].data_ptr() if weights.s2 is not None else 0])
    t = torch.tensor(rows, dtype=torch.int64).to(device if device is not None else weights.w13.device)
    # The table holds raw addresses.  It keeps the tensors they point into alive, so that
    # expert_table(ctx.pack_experts(w)) does not leave it pointing at freed (and soon reused) memory.
    t._dwdp_keepalive = weights
    return t


def dwdp_permute_static(topk_ids: torch.Tensor, E: int, K: int, has_shared: int, expert_offsets: torch.Tensor,
                        perm: torch.Tensor, inv_perm: torch.Tensor, stream: Optional[torch.cuda.Stream] = None):
    """The context-free, allocation-free permutation (see dwdp.h); topk_ids int32 [T,K]."""
    s = C.c_void_p(stream.cuda_stream) if stream is not None else None
    st = lib.dwdp_permute_static(_ptr(topk_ids), topk_ids.shape[0], E, K, has_shared, s, _ptr(expert_offsets),
                                 _ptr(perm), _ptr(inv_perm))
    if st != OK:
        raise DwdpError(st, (lib.dwdp_last_error(None) or b"").decode())


class Context:
    """Owns one dwdp_ctx.  Methods are the C entry points with tensors in place of pointers."""

    def __init__(self, cfg: MoEConfig, n_layers: int = 1, stream: Optional[torch.cuda.Stream] = None,
                 T_max: Optional[int] = None):
        self.cfg = cfg
        self.c = dwdp_config(T_max if T_max is not None else cfg.T, cfg.H, cfg.I, cfg.E, cfg.K, cfg.n_group,
                             cfg.topk_group, cfg.has_shared, cfg.score_fn, cfg.routed_scale, cfg.w_dtype, n_layers)
        self.stream = stream
        handle = C.c_void_p()
        s = C.c_void_p(stream.cuda_stream) if stream is not None else None
        st = lib.dwdp_create(C.byref(self.c), s, C.byref(handle))
        if st != OK:
            raise DwdpError(st, (lib.dwdp_last_error(None) or b"").decode())
        self.h = handle

    def close(self):
        if getattr(self, "h", None):
            lib.dwdp_destroy(self.h)
            self.h = None

    def __del__(self):
        # at interpreter shutdown the module globals may already be gone; the process is ending
        # and the driver reclaims the context's device memory
        if lib is not None:
            self.close()

    def _check(self, st: int):
        if st != OK:
            raise DwdpError(st, (lib.dwdp_last_error(self.h) or b"").decode())

    def dwdp_route(self, logits, bias, topk_ids, topk_w):
        self._check(lib.dwdp_route(self.h, _ptr(logits), _ptr(bias), logits.shape[0], _ptr(topk_ids), _ptr(topk_w)))

    def dwdp_permute(self, topk_ids, expert_offsets, perm, inv_perm):
        self._check(lib.dwdp_permute(self.h, _ptr(topk_ids), topk_ids.shape[0], _ptr(expert_offsets), _ptr(perm),
                                     _ptr(inv_perm)))

    def dwdp_moe_forward(self, layer, x, logits, bias, table, y):
        self._check(lib.dwdp_moe_forward(self.h, layer, _ptr(x), _ptr(logits), _ptr(bias), x.shape[0], _ptr(table),
                                         _ptr(y)))

    def dwdp_prefetch_layer(self, layer, src: Sequence[int], dst: Sequence[int], nbytes: Sequence[int], n_peers: int,
                            n_params: int, slice_bytes: int):
        vp, sz = C.c_void_p, C.c_size_t
        n = n_peers * n_params
        a_src = (vp * max(n, 1))(*[vp(v) for v in src])
        a_dst = (vp * max(n, 1))(*[vp(v) for v in dst])
        a_b = (sz * max(n_params, 1))(*nbytes)
        self._check(lib.dwdp_prefetch_layer(self.h, layer, a_src, a_dst, a_b, n_peers, n_params, slice_bytes))

    def dwdp_prepare_prefetch(self, layer, src: Sequence[int], dst: Sequence[int], nbytes: Sequence[int], n_peers: int,
                              n_params: int, slice_bytes: int):
        vp, sz = C.c_void_p, C.c_size_t
        n = n_peers * n_params
        a_src = (vp * max(n, 1))(*[vp(v) for v in src])
        a_dst = (vp * max(n, 1))(*[vp(v) for v in dst])
        a_b = (sz * max(n_params, 1))(*nbytes)
        self._check(lib.dwdp_prepare_prefetch(self.h, layer, a_src, a_dst, a_b, n_peers, n_params, slice_bytes))

    def dwdp_merge_experts(self, layer: int, table_host: torch.Tensor, w13_out, s13_out, w2_out,
                           s2_out) -> torch.Tensor:
        n = table_host.shape[0]
        assert table_host.device.type == "cpu" and table_host.dtype == torch.int64 and table_host.is_contiguous()
        src = C.cast(table_host.data_ptr(), C.POINTER(dwdp_expert_ptrs))
        merged = torch.zeros(n, 4, dtype=torch.int64)
        dst = C.cast(merged.data_ptr(), C.POINTER(dwdp_expert_ptrs))
        self._check(lib.dwdp_merge_experts(self.h, layer, src, n, _ptr(w13_out), _ptr(s13_out), _ptr(w2_out), _ptr(s2_out),
                                           dst))
        return merged

    def dwdp_set_copy_engine(self, mode: int, n_workgroups: int = 256):
        """mode 0: hipMemcpyAsync per plan entry; mode 1: one copy-plan kernel of n_workgroups."""
        self._check(lib.dwdp_set_copy_engine(self.h, mode, n_workgroups))

    def dwdp_set_stream_max_rows(self, max_rows: int):
        self._check(lib.dwdp_set_stream_max_rows(self.h, max_rows))

    def dwdp_set_tile_schedule(self, mode: int):
        """0: one workgroup per item; 1: persistent per GEMM; 2: persistent, both GEMMs in one launch."""
        self._check(lib.dwdp_set_tile_schedule(self.h, mode))

    def dwdp_set_tile_share(self, n_workgroups: int):
        self._check(lib.dwdp_set_tile_share(self.h, n_workgroups))

    def dwdp_pack_fp8_weight(self, src: torch.Tensor, dst: torch.Tensor):
        """src uint8 [..., rows, cols] row-major matrices -> dst (same shape) tile-major, matrix by matrix."""
        assert src.shape == dst.shape and src.dtype == torch.uint8 and dst.dtype == torch.uint8
        rows, cols = src.shape[-2], src.shape[-1]
        n = src.numel() // (rows * cols) if rows * cols else 0
        s2, d2 = src.reshape(n, rows, cols), dst.reshape(n, rows, cols)
        for i in range(n):
            self._check(lib.dwdp_pack_fp8_weight(self.h, _ptr(s2[i]), _ptr(d2[i]), rows, cols))

    def dwdp_pack_mxfp4_weight(self, codes: torch.Tensor, scales: torch.Tensor, codes_out: torch.Tensor,
                               scales_out: torch.Tensor):
        """codes uint8 [n, rows, cols/2], scales uint8 [n, rows, cols/32] -> streaming layouts, matrix by matrix."""
        n, rows, half = codes.shape
        cols = 2 * half
        assert scales.shape == (n, rows, cols // 32) and codes_out.shape == codes.shape
        assert scales_out.shape == (n, mx_scale_bytes(rows, cols))
        for i in range(n):
            self._check(lib.dwdp_pack_mxfp4_weight(self.h, _ptr(codes[i]), _ptr(scales[i]), _ptr(codes_out[i]),
                                                   _ptr(scales_out[i]), rows, cols))

    def pack_experts(self, w: ExpertWeights) -> ExpertWeights:
        """Device copy of `w` in the layout the kernels read: FP8 codes tile-major (scales
        shared, not copied), MXFP4 codes and scales in their streaming layouts, bf16 weights
        unchanged."""
        if w.s13 is None:
            return w
        if w.s13.dtype == torch.uint8:      # MXFP4
            n, r13, c13 = w.w13.shape[0], w.w13.shape[1], 2 * w.w13.shape[2]
            r2, c2 = w.w2.shape[1], 2 * w.w2.shape[2]
            p13, p2 = torch.empty_like(w.w13), torch.empty_like(w.w2)
            q13 = torch.empty(n, mx_scale_bytes(r13, c13), dtype=torch.uint8, device=w.w13.device)
            q2 = torch.empty(n, mx_scale_bytes(r2, c2), dtype=torch.uint8, device=w.w13.device)
            torch.cuda.synchronize()
            self.dwdp_pack_mxfp4_weight(w.w13, w.s13, p13, q13)
            self.dwdp_pack_mxfp4_weight(w.w2, w.s2, p2, q2)
            if self.stream is not None:
                self.stream.synchronize()
            else:
                torch.cuda.synchronize()
            return ExpertWeights(p13, p2, q13, q2)
        p13, p2 = torch.empty_like(w.w13), torch.empty_like(w.w2)
        torch.cuda.synchronize()      # `w` may still be being written on another stream
        self.dwdp_pack_fp8_weight(w.w13, p13)
        self.dwdp_pack_fp8_weight(w.w2, p2)
        if self.stream is not None:
            self.stream.synchronize()
        else:
            torch.cuda.synchronize()
        return ExpertWeights(p13, p2, w.s13, w.s2)

    def dwdp_profile_enable(self, on: bool):
        self._check(lib.dwdp_profile_enable(self.h, 1 if on else 0))

    def dwdp_profile_read(self):
        ms = (C.c_float * len(STAGES))()
        n = C.c_int32(0)
        self._check(lib.dwdp_profile_read(self.h, ms, C.byref(n)))
        return {name: ms[i] for i, name in enumerate(STAGES)}, n.value

    def dwdp_timeline_enable(self, on: bool):
        self._check(lib.dwdp_timeline_enable(self.h, 1 if on else 0))

    def dwdp_timeline_read(self):
        """[(kind, layer, start_ms, end_ms), ...] with kind 0 = copy span, 1 = GEMM span."""
        cap = 4096
        kind, layer = (C.c_int32 * cap)(), (C.c_int32 * cap)()
        a, b = (C.c_float * cap)(), (C.c_float * cap)()
        n = C.c_int32(0)
        self._check(lib.dwdp_timeline_read(self.h, kind, layer, a, b, cap, C.byref(n)))
        return [(kind[i], layer[i], a[i], b[i]) for i in range(min(n.value, cap))]

    def workspace(self, name: str, shape, dtype) -> torch.Tensor:
        """Copy of a workspace buffer (device-to-device) as a tensor of the given shape/dtype."""
        ptr = lib.dwdp_workspace_ptr(self.h, WS[name])
        out = torch.empty(shape, dtype=dtype, device="cuda")
        if out.numel():
            assert ptr
            nbytes = out.numel() * out.element_size()
            torch.cuda.synchronize()
            _hip_memcpy_d2d(out.data_ptr(), ptr, nbytes)
        return out

    def copy_stream_handle(self) -> int:
        return lib.dwdp_copy_stream(self.h) or 0


_hiprt = None


def _hip_memcpy_d2d(dst: int, src: int, nbytes: int):
    """Synchronous device-to-device copy through the HIP runtime (test/inspection helper)."""
    global _hiprt
    if _hiprt is None:
        _hiprt = C.CDLL("libamdhip64.so")
        _hiprt.hipMemcpy.argtypes = [C.c_void_p, C.c_void_p, C.c_size_t, C.c_int]
    err = _hiprt.hipMemcpy(C.c_void_p(dst), C.c_void_p(src), nbytes, 3)
    if err != 0:
        raise RuntimeError(f"hipMemcpy failed with {err}")
