"""CPU oracle of the MoE expert layer -- TEST INFRASTRUCTURE ONLY.

Thin ctypes access to ``moe_oracle.c`` (plain C, double accumulation, one token and one expert at a
time).  Only the tests, the smoke check and the CPU-baseline leg of the benchmark may import this
package; the HIP library never does, and this package never imports the HIP library.

Arrays: bf16 tensors are ``uint16`` bit patterns, indices ``int32``, weights/logits ``float32``,
expert and layer outputs ``float64``.
"""
from __future__ import annotations

import ctypes as C
import os
import subprocess
from typing import Optional, Sequence

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "moe_oracle.c")
_LIB = os.path.join(_HERE, "libmoe_oracle.so")
_lib = None


def build(force: bool = False) -> str:
    """Compile the oracle with gcc (no fast-math, so the sums are evaluated as written)."""
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        cmd = ["gcc", "-O2", "-fopenmp", "-fPIC", "-shared", "-std=c99", "-Wall", "-Wextra",
               "-o", _LIB, _SRC, "-lm"]
        subprocess.run(cmd, check=True)
    return _LIB


def _p(a: Optional[np.ndarray], ctype):
    if a is None:
        return None
    return a.ctypes.data_as(C.POINTER(ctype))


def _u16(a):
    a = np.ascontiguousarray(a)
    assert a.dtype == np.uint16, a.dtype
    return a


def lib():
    global _lib
    if _lib is None:
        build()
        _lib = C.CDLL(_LIB)
        _lib.oracle_num_threads.restype = C.c_int
    return _lib


def num_threads() -> int:
    return int(lib().oracle_num_threads())


def logits(h, gate_w, bias=None, res_vec=None) -> np.ndarray:
    """[T,N] float32 gate logits of ``h`` (or of ``h + res_vec``) under ``gate_w`` [N,d]."""
    h, gate_w = _u16(h), _u16(gate_w)
    T, d = h.shape
    N = gate_w.shape[0]
    assert gate_w.shape[1] == d
    b = None if bias is None else np.ascontiguousarray(bias, dtype=np.float32)
    r = None if res_vec is None else np.ascontiguousarray(res_vec, dtype=np.float32)
    out = np.empty((T, N), dtype=np.float32)
    lib().oracle_logits(C.c_int(T), C.c_int(d), C.c_int(N), _p(h, C.c_uint16), _p(gate_w, C.c_uint16),
                        _p(b, C.c_float), _p(r, C.c_float), _p(out, C.c_float))
    return out


def select(lg: np.ndarray, k: int, norm_mode: int):
    """(topk_idx [T,k] int32, topk_w [T,k] float32) from logits [T,N]."""
    lg = np.ascontiguousarray(lg, dtype=np.float32)
    T, N = lg.shape
    assert 1 <= k <= N
    idx = np.empty((T, k), dtype=np.int32)
    w = np.empty((T, k), dtype=np.float32)
    lib().oracle_select(C.c_int(T), C.c_int(N), C.c_int(k), _p(lg, C.c_float), C.c_int(norm_mode),
                        _p(idx, C.c_int32), _p(w, C.c_float))
    return idx, w


def histogram(topk_idx: np.ndarray, N: int) -> np.ndarray:
    idx = np.ascontiguousarray(topk_idx, dtype=np.int32)
    counts = np.empty(N, dtype=np.int32)
    lib().oracle_histogram(C.c_int(idx.size), C.c_int(N), _p(idx, C.c_int32), _p(counts, C.c_int32))
    return counts


def top_p(counts: np.ndarray, p: int) -> np.ndarray:
    counts = np.ascontiguousarray(counts, dtype=np.int32)
    top = np.empty(p, dtype=np.int32)
    lib().oracle_top_p(C.c_int(counts.size), _p(counts, C.c_int32), C.c_int(p), _p(top, C.c_int32))
    return top


def route(h, gate_w, bias, k: int, norm_mode: int):
    """(logits, topk_idx, topk_w, counts) of one layer."""
    lg = logits(h, gate_w, bias)
    idx, w = select(lg, k, norm_mode)
    return lg, idx, w, histogram(idx, gate_w.shape[0])


def predict_workload(h, res_vec, next_gate_w, next_bias, k: int, p: int):
    """(pred_logits, pred_idx, pred_counts, top_p): next layer's gate on h + res_vec, token counts per
    predicted expert, and the p highest-workload experts."""
    lg = logits(h, next_gate_w, next_bias, res_vec)
    idx, _ = select(lg, k, 0)
    cnt = histogram(idx, next_gate_w.shape[0])
    return lg, idx, cnt, top_p(cnt, p)


def expert_rows(h, topk_idx, w1, w3, w2, mask=None, tokens: Optional[Sequence[int]] = None) -> np.ndarray:
    """[n_tok, k, d] float64: the output of each selected expert for each listed token (zeros where
    the expert's mask bit is off)."""
    h, w1, w3, w2 = _u16(h), _u16(w1), _u16(w3), _u16(w2)
    idx = np.ascontiguousarray(topk_idx, dtype=np.int32)
    T, d = h.shape
    N, I, _ = w1.shape
    k = idx.shape[1]
    assert w3.shape == (N, I, d) and w2.shape == (N, d, I) and idx.shape[0] == T
    toks = np.arange(T, dtype=np.int32) if tokens is None else np.ascontiguousarray(tokens, dtype=np.int32)
    m = None if mask is None else np.ascontiguousarray(mask, dtype=np.uint8)
    y = np.empty((toks.size, k, d), dtype=np.float64)
    lib().oracle_expert_rows(C.c_int(d), C.c_int(N), C.c_int(k), C.c_int(I), _p(h, C.c_uint16),
                             _p(idx, C.c_int32), _p(w1, C.c_uint16), _p(w3, C.c_uint16), _p(w2, C.c_uint16),
                             _p(m, C.c_uint8), C.c_int(toks.size), _p(toks, C.c_int32), _p(y, C.c_double))
    return y


def layer(h, topk_idx, topk_w, w1, w3, w2, mask=None, shared=None, shared_mode: int = 0,
          tokens: Optional[Sequence[int]] = None) -> np.ndarray:
    """[n_tok, d] float64 layer output (Eq. 2 over the masked-on experts, plus shared experts).

    ``shared`` = (sw1, sw3, sw2, w_sg) or None; ``shared_mode`` 1: weight 1, 2: sigmoid(h . w_sg).
    """
    h, w1, w3, w2 = _u16(h), _u16(w1), _u16(w3), _u16(w2)
    idx = np.ascontiguousarray(topk_idx, dtype=np.int32)
    tw = np.ascontiguousarray(topk_w, dtype=np.float32)
    T, d = h.shape
    N, I, _ = w1.shape
    k = idx.shape[1]
    assert w3.shape == (N, I, d) and w2.shape == (N, d, I) and idx.shape == tw.shape and idx.shape[0] == T
    toks = np.arange(T, dtype=np.int32) if tokens is None else np.ascontiguousarray(tokens, dtype=np.int32)
    m = None if mask is None else np.ascontiguousarray(mask, dtype=np.uint8)
    sw1 = sw3 = sw2 = wsg = None
    n_sh = I_sh = 0
    if shared is not None and shared_mode != 0:
        sw1, sw3, sw2, wsg = shared
        sw1, sw3, sw2 = _u16(sw1), _u16(sw3), _u16(sw2)
        n_sh, I_sh = sw1.shape[0], sw1.shape[1]
        if shared_mode == 2:
            wsg = _u16(wsg)
    else:
        shared_mode = 0
    out = np.empty((toks.size, d), dtype=np.float64)
    lib().oracle_layer(C.c_int(d), C.c_int(N), C.c_int(k), C.c_int(I), _p(h, C.c_uint16), _p(idx, C.c_int32),
                       _p(tw, C.c_float), _p(w1, C.c_uint16), _p(w3, C.c_uint16), _p(w2, C.c_uint16),
                       _p(m, C.c_uint8), C.c_int(shared_mode), C.c_int(n_sh), C.c_int(I_sh),
                       _p(sw1, C.c_uint16), _p(sw3, C.c_uint16), _p(sw2, C.c_uint16), _p(wsg, C.c_uint16),
                       C.c_int(toks.size), _p(toks, C.c_int32), _p(out, C.c_double))
    return out


def shared_scale(h, w_sg) -> np.ndarray:
    """[T] float64: weight of a sigmoid-gated shared expert, c(t) = 1 / (1 + exp(-(h[t,:] . w_sg))), the shared-expert
    term of Eq. 2 for the model whose shared expert carries a gate of its own (model table, Section "Experimental
    Setup").  Plain NumPy in float64 from the bf16-valued inputs."""
    hb, wb = _u16(h), _u16(w_sg)
    x = (hb.astype(np.uint32) << 16).view(np.float32).astype(np.float64)
    g = (wb.astype(np.uint32) << 16).view(np.float32).astype(np.float64)
    return 1.0 / (1.0 + np.exp(-(x @ g)))


def res_vec(h_cur, h_next) -> np.ndarray:
    """[d] float32: mean over calibration tokens of h_next - h_cur."""
    a, b = _u16(h_cur), _u16(h_next)
    assert a.shape == b.shape
    n, d = a.shape
    out = np.empty(d, dtype=np.float32)
    lib().oracle_res_vec(C.c_int(n), C.c_int(d), _p(a, C.c_uint16), _p(b, C.c_uint16), _p(out, C.c_float))
    return out
