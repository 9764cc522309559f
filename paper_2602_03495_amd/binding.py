"""Thin ctypes binding of libmoe_mi355x.so: the same entry points as include/moe_layer.h, taking torch
device tensors.  Argument marshalling only -- every step of the layer runs in the library's HIP kernels.
There is no fallback: a missing library or a non-zero return code raises."""
from __future__ import annotations

import ctypes as C
import os
from dataclasses import dataclass
from typing import Optional

import torch

from .build import LIB

FFN_AUTO, FFN_TILED, FFN_SKINNY = 0, 1, 2
NORM_NONE, NORM_RENORM = 0, 1
MAX_EXPERTS, MAX_TOPK = 128, 8        # MOE_MAX_EXPERTS, MOE_MAX_TOPK of include/moe_layer.h

EXPORTS = ["moe_strerror", "moe_workspace_bytes", "moe_route", "moe_predict_workload", "moe_expert_ffn",
           "moe_expert_ffn_stage", "moe_combine", "moe_dense_route", "moe_shared_gate", "moe_pack_weights",
           "moe_expert_times", "moe_greedy_assign", "moe_cache_step", "moe_res_vec_workspace_bytes",
           "moe_res_vec_accumulate", "moe_res_vec_finish", "moe_route_predict", "moe_append_shared",
           "moe_expert_ffn_static", "moe_static_scratch_bytes", "moe_debug_set_trace", "moe_route_shared"]


class MoeShape(C.Structure):
    _fields_ = [("T", C.c_int32), ("d", C.c_int32), ("N", C.c_int32), ("k", C.c_int32), ("I", C.c_int32),
                ("ffn_path", C.c_int32), ("weight_layout", C.c_int32)]


class MoeError(RuntimeError):
    pass


_lib = None


def load_library():
    """dlopen the in-tree library; raises if it has not been built."""
    global _lib
    if _lib is None:
        if not os.path.exists(LIB):
            raise MoeError(f"{LIB} is missing: run `python -c 'import __graft_entry__ as g; g.build()'` first")
        _lib = C.CDLL(LIB)
        _lib.moe_strerror.restype = C.c_char_p
        _lib.moe_strerror.argtypes = [C.c_int]
        for name in EXPORTS[1:]:
            getattr(_lib, name).restype = C.c_int
        _lib.moe_res_vec_workspace_bytes.restype = C.c_size_t
        _lib.moe_static_scratch_bytes.restype = C.c_size_t
    return _lib


def _check(rc: int, what: str):
    if rc != 0:
        raise MoeError(f"{what} failed: {load_library().moe_strerror(rc).decode()} (code {rc})")


def _ptr(t: Optional[torch.Tensor], dtype=None):
    if t is None:
        return C.c_void_p(0)
    if not t.is_cuda or not t.is_contiguous():
        raise MoeError("expected a contiguous device tensor")
    if dtype is not None and t.dtype != dtype:
        raise MoeError(f"expected dtype {dtype}, got {t.dtype}")
    return C.c_void_p(t.data_ptr())


def _stream():
    return C.c_void_p(torch.cuda.current_stream().cuda_stream)


WEIGHTS_ROWMAJOR, WEIGHTS_PACKED = 0, 1      # MOE_WEIGHTS_* of include/moe_layer.h


def shape(T: int, d: int, N: int, k: int, I: int, ffn_path: int = FFN_AUTO, weight_layout: int = WEIGHTS_PACKED) -> MoeShape:
    """weight_layout states what the expert weight tensors passed with this shape hold; the default is what
    moe_pack_weights (LayerWeights.upload) produces, the only layout the kernels read."""
    return MoeShape(T, d, N, k, I, ffn_path, weight_layout)


def workspace_bytes(s: MoeShape) -> int:
    n = C.c_size_t(0)
    _check(load_library().moe_workspace_bytes(C.byref(s), C.byref(n)), "moe_workspace_bytes")
    return int(n.value)


def alloc_workspace(s: MoeShape, device="cuda") -> torch.Tensor:
    return torch.empty(workspace_bytes(s) + 256, dtype=torch.uint8, device=device)


def _ws_ptr(ws: Optional[torch.Tensor]):
    if ws is None:
        return C.c_void_p(0)
    p = ws.data_ptr()
    return C.c_void_p((p + 255) & ~255)


@dataclass
class Routing:
    topk_idx: torch.Tensor   # [T,k] int32
    topk_w: torch.Tensor     # [T,k] float32
    counts: torch.Tensor     # [N] int32
    offsets: torch.Tensor    # [N+1] int32
    perm: torch.Tensor       # [T*k] int32
    inv_perm: torch.Tensor   # [T*k] int32


def alloc_routing(s: MoeShape, device="cuda") -> Routing:
    R = s.T * s.k
    i32 = dict(dtype=torch.int32, device=device)
    return Routing(torch.empty((s.T, s.k), **i32), torch.empty((s.T, s.k), dtype=torch.float32, device=device),
                   torch.empty(s.N, **i32), torch.empty(s.N + 1, **i32), torch.empty(R, **i32), torch.empty(R, **i32))


def moe_route(s: MoeShape, h, gate_w, gate_bias, norm_mode: int, out: Routing, ws: Optional[torch.Tensor]) -> Routing:
    rc = load_library().moe_route(C.byref(s), _ptr(h, torch.bfloat16), _ptr(gate_w, torch.bfloat16),
                                  _ptr(gate_bias, torch.float32), C.c_int(norm_mode), _ptr(out.topk_idx, torch.int32),
                                  _ptr(out.topk_w, torch.float32), _ptr(out.counts, torch.int32),
                                  _ptr(out.offsets, torch.int32), _ptr(out.perm, torch.int32),
                                  _ptr(out.inv_perm, torch.int32), _ws_ptr(ws), _stream())
    _check(rc, "moe_route")
    return out


def moe_predict_workload(s: MoeShape, h, res_vec, next_gate_w, next_gate_bias, p: int, pred_counts, top_experts,
                         ws: torch.Tensor):
    rc = load_library().moe_predict_workload(C.byref(s), _ptr(h, torch.bfloat16), _ptr(res_vec, torch.float32),
                                             _ptr(next_gate_w, torch.bfloat16), _ptr(next_gate_bias, torch.float32),
                                             C.c_int(p), _ptr(pred_counts, torch.int32), _ptr(top_experts, torch.int32),
                                             _ws_ptr(ws), _stream())
    _check(rc, "moe_predict_workload")
    return pred_counts, top_experts


def moe_route_predict(s: MoeShape, h, gate_w, gate_bias, norm_mode: int, r, res_vec, next_gate_w, next_gate_bias, p: int,
                      pred_counts, top_experts, ws: torch.Tensor):
    rc = load_library().moe_route_predict(C.byref(s), _ptr(h, torch.bfloat16), _ptr(gate_w, torch.bfloat16),
                                          _ptr(gate_bias, torch.float32), C.c_int(norm_mode), _ptr(r.topk_idx, torch.int32),
                                          _ptr(r.topk_w, torch.float32), _ptr(r.counts, torch.int32),
                                          _ptr(r.offsets, torch.int32), _ptr(r.perm, torch.int32),
                                          _ptr(r.inv_perm, torch.int32), _ptr(res_vec, torch.float32),
                                          _ptr(next_gate_w, torch.bfloat16), _ptr(next_gate_bias, torch.float32), C.c_int(p),
                                          _ptr(pred_counts, torch.int32), _ptr(top_experts, torch.int32), _ws_ptr(ws), _stream())
    _check(rc, "moe_route_predict")
    return r


class ResVecCalibration:
    """Device buffers of one res_vec calibration: float64 running sum [d], scratch, token count."""

    def __init__(self, d: int, device="cuda"):
        lib = load_library()
        self.d, self.n_total = d, 0
        self.acc = torch.zeros(d, dtype=torch.float64, device=device)
        self.ws = torch.empty(int(lib.moe_res_vec_workspace_bytes(C.c_int(d))), dtype=torch.uint8, device=device)
        self.res_vec = torch.empty(d, dtype=torch.float32, device=device)

    def accumulate(self, h_cur: torch.Tensor, h_next: torch.Tensor):
        n = h_cur.shape[0]
        assert h_cur.shape == h_next.shape == (n, self.d)
        rc = load_library().moe_res_vec_accumulate(C.c_int(n), C.c_int(self.d), _ptr(h_cur, torch.bfloat16),
                                                   _ptr(h_next, torch.bfloat16), _ptr(self.acc, torch.float64),
                                                   C.c_void_p(self.ws.data_ptr()), _stream())
        _check(rc, "moe_res_vec_accumulate")
        self.n_total += n

    def finish(self) -> torch.Tensor:
        rc = load_library().moe_res_vec_finish(C.c_int(self.d), _ptr(self.acc, torch.float64), C.c_int64(self.n_total),
                                               _ptr(self.res_vec, torch.float32), _stream())
        _check(rc, "moe_res_vec_finish")
        return self.res_vec


def moe_expert_ffn(s: MoeShape, h, perm, offsets, counts, w1, w3, w2, expert_mask, y, ws: torch.Tensor):
    rc = load_library().moe_expert_ffn(C.byref(s), _ptr(h, torch.bfloat16), _ptr(perm, torch.int32),
                                       _ptr(offsets, torch.int32), _ptr(counts, torch.int32), _ptr(w1, torch.bfloat16),
                                       _ptr(w3, torch.bfloat16), _ptr(w2, torch.bfloat16), _ptr(expert_mask, torch.uint8),
                                       _ptr(y, torch.bfloat16), _ws_ptr(ws), _stream())
    _check(rc, "moe_expert_ffn")
    return y


def moe_expert_ffn_static(s: MoeShape, h, perm, offsets, counts, w1, w3, w2, expert_mask, y):
    """moe_expert_ffn on the library's static scratch array (no workspace argument, no allocation)."""
    rc = load_library().moe_expert_ffn_static(C.byref(s), _ptr(h, torch.bfloat16), _ptr(perm, torch.int32),
                                              _ptr(offsets, torch.int32), _ptr(counts, torch.int32), _ptr(w1, torch.bfloat16),
                                              _ptr(w3, torch.bfloat16), _ptr(w2, torch.bfloat16), _ptr(expert_mask, torch.uint8),
                                              _ptr(y, torch.bfloat16), _stream())
    _check(rc, "moe_expert_ffn_static")
    return y


TRACE_MAX_BLOCKS = 65536


def moe_debug_set_trace(records: Optional[torch.Tensor]):
    """records: zeroed int64 device tensor of 2 * TRACE_MAX_BLOCKS * 8 elements, or None to switch the timeline off."""
    if records is not None and (records.dtype != torch.int64 or records.numel() < 2 * TRACE_MAX_BLOCKS * 8):
        raise MoeError("timeline buffer: int64, 2 * 65536 * 8 elements")
    _check(load_library().moe_debug_set_trace(_ptr(records)), "moe_debug_set_trace")


def static_scratch_bytes() -> int:
    return int(load_library().moe_static_scratch_bytes())


STAGE_UP, STAGE_DOWN, STAGE_ALL = 1, 2, 3


def moe_expert_ffn_stage(s: MoeShape, h, perm, offsets, counts, w1, w3, w2, expert_mask, y, ws: torch.Tensor, stages: int):
    rc = load_library().moe_expert_ffn_stage(C.byref(s), _ptr(h, torch.bfloat16), _ptr(perm, torch.int32),
                                             _ptr(offsets, torch.int32), _ptr(counts, torch.int32),
                                             _ptr(w1, torch.bfloat16), _ptr(w3, torch.bfloat16), _ptr(w2, torch.bfloat16),
                                             _ptr(expert_mask, torch.uint8), _ptr(y, torch.bfloat16), _ws_ptr(ws),
                                             C.c_int(stages), _stream())
    _check(rc, "moe_expert_ffn_stage")
    return y


def moe_combine(s: MoeShape, y, topk_idx, topk_w, inv_perm, expert_mask, shared_y, n_shared: int, shared_scale, out):
    rc = load_library().moe_combine(C.byref(s), _ptr(y, torch.bfloat16), _ptr(topk_idx, torch.int32),
                                    _ptr(topk_w, torch.float32), _ptr(inv_perm, torch.int32),
                                    _ptr(expert_mask, torch.uint8), _ptr(shared_y, torch.bfloat16), C.c_int(n_shared),
                                    _ptr(shared_scale, torch.float32), _ptr(out, torch.bfloat16), _stream())
    _check(rc, "moe_combine")
    return out


def moe_pack_weights(src: torch.Tensor, dst: Optional[torch.Tensor] = None) -> torch.Tensor:
    """Pack row-major [n_mats, rows, K] bf16 matrices into the MFMA-fragment order the FFN kernels read."""
    n_mats, rows, K = src.shape
    if dst is None:
        dst = torch.empty_like(src)
    rc = load_library().moe_pack_weights(C.c_int(n_mats), C.c_int(rows), C.c_int(K), _ptr(src, torch.bfloat16),
                                         _ptr(dst, torch.bfloat16), _stream())
    _check(rc, "moe_pack_weights")
    return dst


def expert_times(counts, cached, trans_time: float, gpu_compute, cpu_compute):
    """Per-expert execution times on either side (Section "Greedy Assignment Strategy") from profiled time tables indexed
    by workload: returns (t_gpu, t_cpu) float32 arrays.  cached: uint8 [N] or None."""
    import numpy as np
    c = np.ascontiguousarray(counts, np.int32)
    g, p = np.ascontiguousarray(gpu_compute, np.float32), np.ascontiguousarray(cpu_compute, np.float32)
    assert g.size == p.size and g.size >= 1
    ca = None if cached is None else np.ascontiguousarray(cached, np.uint8)
    t_gpu, t_cpu = np.zeros(c.size, np.float32), np.zeros(c.size, np.float32)
    f = C.POINTER(C.c_float)
    _check(load_library().moe_expert_times(C.c_int(c.size), c.ctypes.data_as(C.POINTER(C.c_int32)),
                                           None if ca is None else ca.ctypes.data_as(C.POINTER(C.c_uint8)),
                                           C.c_float(trans_time), g.ctypes.data_as(f), p.ctypes.data_as(f), C.c_int(g.size - 1),
                                           t_gpu.ctypes.data_as(f), t_cpu.ctypes.data_as(f)), "moe_expert_times")
    return t_gpu, t_cpu


def greedy_assign(t_gpu, t_cpu):
    """Alg. 1 on host arrays: returns (G, C, T_gpu, T_cpu) with G, C as uint8 numpy arrays."""
    import numpy as np
    tg, tc = np.ascontiguousarray(t_gpu, np.float32), np.ascontiguousarray(t_cpu, np.float32)
    N = tg.size
    G, Cc = np.zeros(N, np.uint8), np.zeros(N, np.uint8)
    Tg, Tc = C.c_float(0), C.c_float(0)
    f, b = C.POINTER(C.c_float), C.POINTER(C.c_uint8)
    _check(load_library().moe_greedy_assign(C.c_int(N), tg.ctypes.data_as(f), tc.ctypes.data_as(f), G.ctypes.data_as(b),
                                            Cc.ctypes.data_as(b), C.byref(Tg), C.byref(Tc)), "moe_greedy_assign")
    return G, Cc, Tg.value, Tc.value


CACHE_ALWAYS, CACHE_GUARDED = 0, 1      # MOE_CACHE_ALWAYS (Alg. 2 as printed), MOE_CACHE_GUARDED (variant)


class ExpertCache:
    """Alg. 2 state of one layer, advanced by moe_cache_step."""

    def __init__(self, N: int, on_gpu_ids, w_size: int, u_size: int, mode: int = CACHE_ALWAYS):
        import numpy as np
        self.N, self.w_size, self.u_size, self.mode = N, w_size, u_size, mode
        self.score = np.zeros(N, np.int64)
        self.on_gpu = np.zeros(N, np.uint8)
        self.on_gpu[list(on_gpu_ids)] = 1
        self.step_in_window = C.c_int32(0)
        self._ev = np.full(max(u_size, 1), -1, np.int32)
        self._ld = np.full(max(u_size, 1), -1, np.int32)

    def step(self, workload):
        import numpy as np
        w = np.ascontiguousarray(workload, np.int32)
        n = C.c_int32(0)
        i32, i64, u8 = C.POINTER(C.c_int32), C.POINTER(C.c_int64), C.POINTER(C.c_uint8)
        _check(load_library().moe_cache_step(C.c_int(self.N), C.c_int(self.w_size), C.c_int(self.u_size),
                                             C.c_int(self.mode), w.ctypes.data_as(i32), self.score.ctypes.data_as(i64),
                                             self.on_gpu.ctypes.data_as(u8), C.byref(self.step_in_window),
                                             self._ev.ctypes.data_as(i32), self._ld.ctypes.data_as(i32), C.byref(n)),
               "moe_cache_step")
        return [(int(self._ev[j]), int(self._ld[j])) for j in range(n.value)]


def moe_dense_route(s: MoeShape, counts, offsets, perm):
    rc = load_library().moe_dense_route(C.byref(s), _ptr(counts, torch.int32), _ptr(offsets, torch.int32),
                                        _ptr(perm, torch.int32), _stream())
    _check(rc, "moe_dense_route")


def moe_shared_gate(s: MoeShape, h, w_sg, scale):
    rc = load_library().moe_shared_gate(C.byref(s), _ptr(h, torch.bfloat16), _ptr(w_sg, torch.bfloat16),
                                        _ptr(scale, torch.float32), _stream())
    _check(rc, "moe_shared_gate")
    return scale


def moe_append_shared(s: MoeShape, n_shared: int, h, w_sg, r: Routing, out: Routing) -> Routing:
    """Tables of the layer with its shared experts appended as experts N.. and slots k.. (out: shapes of N+n_shared, k+n_shared)."""
    i32 = torch.int32
    rc = load_library().moe_append_shared(C.byref(s), C.c_int(n_shared), _ptr(h, torch.bfloat16), _ptr(w_sg, torch.bfloat16),
                                          _ptr(r.topk_idx, i32), _ptr(r.topk_w, torch.float32), _ptr(r.counts, i32),
                                          _ptr(r.offsets, i32), _ptr(r.perm, i32), _ptr(r.inv_perm, i32),
                                          _ptr(out.topk_idx, i32), _ptr(out.topk_w, torch.float32), _ptr(out.counts, i32),
                                          _ptr(out.offsets, i32), _ptr(out.perm, i32), _ptr(out.inv_perm, i32), _stream())
    _check(rc, "moe_append_shared")
    return out


def moe_route_shared(s: MoeShape, n_shared: int, h, gate_w, gate_bias, norm_mode: int, w_sg, r: Routing, out: Routing,
                     ws: Optional[torch.Tensor]) -> Routing:
    """moe_route + moe_append_shared in one call (one launch fewer at decode sizes); fills r and out, returns out."""
    i32 = torch.int32
    rc = load_library().moe_route_shared(C.byref(s), C.c_int(n_shared), _ptr(h, torch.bfloat16), _ptr(gate_w, torch.bfloat16),
                                         _ptr(gate_bias, torch.float32), C.c_int(norm_mode), _ptr(w_sg, torch.bfloat16),
                                         _ptr(r.topk_idx, i32), _ptr(r.topk_w, torch.float32), _ptr(r.counts, i32),
                                         _ptr(r.offsets, i32), _ptr(r.perm, i32), _ptr(r.inv_perm, i32),
                                         _ptr(out.topk_idx, i32), _ptr(out.topk_w, torch.float32), _ptr(out.counts, i32),
                                         _ptr(out.offsets, i32), _ptr(out.perm, i32), _ptr(out.inv_perm, i32), _ws_ptr(ws), _stream())
    _check(rc, "moe_route_shared")
    return out
