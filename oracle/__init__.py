"""ctypes front end of the CPU oracle (oracle/lq_oracle.c).

TEST INFRASTRUCTURE ONLY: imported by tests/, by the smoke check and by the benchmark's
CPU-baseline leg.  Nothing in the GPU package imports this, and this imports nothing from it.
Inputs and outputs are numpy arrays; bfloat16 tensors travel as uint16 bit patterns.
"""
from __future__ import annotations

import ctypes
import os
import subprocess
from dataclasses import dataclass
from typing import List, Optional, Sequence

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "lq_oracle.c")
_LIB = os.path.join(_HERE, "liblq_oracle.so")
_lib = None


def build(force: bool = False) -> str:
    """Compile the oracle with the host C compiler (no GPU toolchain involved)."""
    stale = (not os.path.exists(_LIB)) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC)
    if force or stale:
        tmp = _LIB + f".tmp{os.getpid()}"
        subprocess.run(["gcc", "-O3", "-march=native", "-fopenmp", "-fPIC", "-shared", "-Wall", "-Wextra",
                        "-o", tmp, _SRC], check=True)
        os.replace(tmp, _LIB)
    return _LIB


def _load():
    global _lib
    if _lib is None:
        build()
        L = ctypes.CDLL(_LIB)
        i32, i64, vp = ctypes.c_int32, ctypes.c_int64, ctypes.c_void_p
        L.lq_oracle_build_segments.restype = i32
        L.lq_oracle_build_segments.argtypes = [vp, vp, i32, vp, i32, vp, vp, vp, vp, vp]
        L.lq_oracle_forward.restype = None
        L.lq_oracle_forward.argtypes = [vp, i64, vp, i64, i32, i32, i32, vp, vp, vp, vp, i32, vp, vp, vp, vp, vp, vp]
        L.lq_oracle_backward.restype = None
        L.lq_oracle_backward.argtypes = [vp, i64, vp, i64, vp, i64, i32, i32, i32, vp, vp, vp, vp, i32,
                                         vp, vp, vp, vp, vp, vp, vp, vp]
        L.lq_oracle_num_threads.restype = i32
        u32 = ctypes.c_uint32
        L.lq_oracle_dropout_keep.restype = i32
        L.lq_oracle_dropout_keep.argtypes = [u32, i32, i32, u32]
        L.lq_oracle_dropout_rows.restype = None
        L.lq_oracle_dropout_rows.argtypes = [vp, i64, vp, i64, i32, i32, vp, vp, i32, u32, u32]
        L.lq_oracle_kind_offsets.restype = None
        L.lq_oracle_kind_offsets.argtypes = [vp, vp, i32, vp]
        L.lq_oracle_split_rows.restype = None
        L.lq_oracle_split_rows.argtypes = [vp, i64, i32, vp, i32, vp]
        L.lq_oracle_concat_rows.restype = None
        L.lq_oracle_concat_rows.argtypes = [vp, i32, vp, i32, vp, i64]
        _lib = L
    return _lib


def num_threads() -> int:
    return int(_load().lq_oracle_num_threads())


def _p(a: Optional[np.ndarray]):
    return None if a is None else a.ctypes.data_as(ctypes.c_void_p)


def _ptr_table(arrs: Sequence[np.ndarray]):
    tab = (ctypes.c_void_p * max(len(arrs), 1))()
    for i, a in enumerate(arrs):
        tab[i] = a.ctypes.data
    return tab


@dataclass
class Segments:
    perm: np.ndarray         # int32[n_live]      token indices, grouped by (kind, adapter), stable
    seg_starts: np.ndarray   # int32[n_seg + 1]   positions in perm
    seg_adapter: np.ndarray  # int32[n_seg]
    seg_kind: np.ndarray     # uint8[n_seg]
    h_offsets: np.ndarray    # int64[n_seg + 1]   element offsets into the saved-h buffer

    @property
    def n_segments(self) -> int:
        return int(self.seg_adapter.shape[0])

    @property
    def h_elems(self) -> int:
        return int(self.h_offsets[-1])


def build_segments(token_adapter, token_kind, ranks) -> Segments:
    ta = np.ascontiguousarray(token_adapter, dtype=np.int32)
    tk = np.ascontiguousarray(token_kind, dtype=np.uint8)
    rk = np.ascontiguousarray(ranks, dtype=np.int32)
    T = ta.shape[0]
    perm = np.zeros(max(T, 1), np.int32)
    starts = np.zeros(T + 1, np.int32)
    sad = np.zeros(max(T, 1), np.int32)
    skd = np.zeros(max(T, 1), np.uint8)
    hoff = np.zeros(T + 1, np.int64)
    n = _load().lq_oracle_build_segments(_p(ta), _p(tk), T, _p(rk), rk.shape[0], _p(perm), _p(starts), _p(sad),
                                         _p(skd), _p(hoff))
    n_live = int(starts[n])
    return Segments(perm[:n_live].copy(), starts[:n + 1].copy(), sad[:n].copy(), skd[:n].copy(), hoff[:n + 1].copy())


def token_h_offsets(seg: Segments, ranks, n_tokens: int) -> np.ndarray:
    """Element offset of each fine-tune token's saved h row (-1 for every other token)."""
    out = np.full(n_tokens, -1, np.int64)
    for s in range(seg.n_segments):
        if seg.seg_kind[s] != 0:
            continue
        r = int(ranks[seg.seg_adapter[s]])
        for p in range(int(seg.seg_starts[s]), int(seg.seg_starts[s + 1])):
            out[seg.perm[p]] = int(seg.h_offsets[s]) + (p - int(seg.seg_starts[s])) * r
    return out


@dataclass
class ForwardResult:
    y: np.ndarray            # float64[T, d_out]
    h: np.ndarray            # float64[h_elems]  saved (unscaled) h of fine-tune rows, metadata layout
    segments: Segments


def forward(x, y0, A: List[np.ndarray], B: List[np.ndarray], ranks, scales, token_adapter, token_kind,
            token_scales=None) -> ForwardResult:
    """token_scales: optional float32[T]; when given it replaces scales[adapter] for every token (the dynamic,
    per-request scale of Section 3.3)."""
    x = np.ascontiguousarray(x, dtype=np.uint16)
    y0 = np.ascontiguousarray(y0, dtype=np.uint16)
    A = [np.ascontiguousarray(a, dtype=np.uint16) for a in A]
    B = [np.ascontiguousarray(b, dtype=np.uint16) for b in B]
    rk = np.ascontiguousarray(ranks, dtype=np.int32)
    sc = np.ascontiguousarray(scales, dtype=np.float32)
    ta = np.ascontiguousarray(token_adapter, dtype=np.int32)
    tk = np.ascontiguousarray(token_kind, dtype=np.uint8)
    T, d_in = x.shape
    d_out = y0.shape[1]
    for a, b, r in zip(A, B, rk):
        assert a.shape == (r, d_in) and b.shape == (r, d_out)
    seg = build_segments(ta, tk, rk)
    hoff = token_h_offsets(seg, rk, T)
    y = np.zeros((T, d_out), np.float64)
    h = np.zeros(max(seg.h_elems, 1), np.float64)
    At, Bt = _ptr_table(A), _ptr_table(B)
    ts = None if token_scales is None else np.ascontiguousarray(token_scales, dtype=np.float32)
    assert ts is None or ts.shape == (T,)
    _load().lq_oracle_forward(_p(x), d_in, _p(y0), d_out, T, d_in, d_out, At, Bt, _p(rk), _p(sc), rk.shape[0],
                              _p(ta), _p(tk), _p(hoff), _p(ts), _p(y), _p(h))
    return ForwardResult(y, h[:seg.h_elems], seg)


@dataclass
class BackwardResult:
    dA: List[np.ndarray]     # float64[r, d_in] per adapter
    dB: List[np.ndarray]     # float64[r, d_out] per adapter
    dx: np.ndarray           # float64[T, d_in]
    g: np.ndarray            # float64[h_elems]  dy B^T of fine-tune rows (unscaled), metadata layout


def backward(x, dy, dx0, A, B, ranks, scales, token_adapter, token_kind, token_scales=None) -> BackwardResult:
    x = np.ascontiguousarray(x, dtype=np.uint16)
    dy = np.ascontiguousarray(dy, dtype=np.uint16)
    dx0 = None if dx0 is None else np.ascontiguousarray(dx0, dtype=np.uint16)
    A = [np.ascontiguousarray(a, dtype=np.uint16) for a in A]
    B = [np.ascontiguousarray(b, dtype=np.uint16) for b in B]
    rk = np.ascontiguousarray(ranks, dtype=np.int32)
    sc = np.ascontiguousarray(scales, dtype=np.float32)
    ta = np.ascontiguousarray(token_adapter, dtype=np.int32)
    tk = np.ascontiguousarray(token_kind, dtype=np.uint8)
    T, d_in = x.shape
    d_out = dy.shape[1]
    seg = build_segments(ta, tk, rk)
    hoff = token_h_offsets(seg, rk, T)
    dA = [np.zeros((int(r), d_in), np.float64) for r in rk]
    dB = [np.zeros((int(r), d_out), np.float64) for r in rk]
    dx = np.zeros((T, d_in), np.float64)
    g = np.zeros(max(seg.h_elems, 1), np.float64)
    ts = None if token_scales is None else np.ascontiguousarray(token_scales, dtype=np.float32)
    assert ts is None or ts.shape == (T,)
    _load().lq_oracle_backward(_p(x), d_in, _p(dy), d_out, _p(dx0), d_in, T, d_in, d_out, _ptr_table(A), _ptr_table(B),
                               _p(rk), _p(sc), rk.shape[0], _p(ta), _p(tk), _p(hoff), _p(ts),
                               _ptr_table(dA), _ptr_table(dB), _p(dx), _p(g))
    return BackwardResult(dA, dB, dx, g[:seg.h_elems])


# ---- LoRA dropout on the fine-tuning rows, row split / concatenation of Algorithm 1 ------------------------------
def dropout_threshold(p: float) -> int:
    """The 16-bit threshold of the dropout contract: an element is kept iff its 16-bit field is >= p * 65536 rounded
    to the nearest integer, the product and the rounding (add one half, truncate) taken in fp32."""
    return int(np.float32(p) * np.float32(65536.0) + np.float32(0.5))


def dropout_keep(seed: int, t: int, k: int, threshold: int) -> bool:
    return bool(_load().lq_oracle_dropout_keep(seed & 0xffffffff, t, k, threshold))


def dropout_rows(x, token_adapter, token_kind, n_adapters: int, seed: int, p: float) -> np.ndarray:
    """m * x on the live fine-tuning rows (bf16 bit patterns), every other row copied."""
    x = np.ascontiguousarray(x, dtype=np.uint16)
    ta = np.ascontiguousarray(token_adapter, dtype=np.int32)
    tk = np.ascontiguousarray(token_kind, dtype=np.uint8)
    out = np.empty_like(x)
    T, d = x.shape
    _load().lq_oracle_dropout_rows(_p(x), d, _p(out), d, T, d, _p(ta), _p(tk), n_adapters, seed & 0xffffffff, dropout_threshold(p))
    return out


def kind_offsets(seg: Segments) -> np.ndarray:
    """int32[4]: where the fine-tune, prefill and decode rows start in the segment order, and the number of live rows."""
    out = np.zeros(4, np.int32)
    starts = np.ascontiguousarray(seg.seg_starts, np.int32)
    kinds = np.ascontiguousarray(seg.seg_kind, np.uint8) if seg.n_segments else np.zeros(1, np.uint8)
    _load().lq_oracle_kind_offsets(_p(starts), _p(kinds), seg.n_segments, _p(out))
    return out


def split_rows(src, seg: Segments) -> np.ndarray:
    """The live rows of src in segment order (the three kinds back to back), uint16[n_live, d]."""
    src = np.ascontiguousarray(src, dtype=np.uint16)
    perm = np.ascontiguousarray(seg.perm, np.int32)
    out = np.zeros((perm.shape[0], src.shape[1]), np.uint16)
    _load().lq_oracle_split_rows(_p(src), src.shape[1], src.shape[1], _p(perm), perm.shape[0], _p(out))
    return out


def concat_rows(parts, seg: Segments, dst) -> np.ndarray:
    """dst with its live rows replaced by the rows of parts (inverse of split_rows); other rows untouched."""
    parts = np.ascontiguousarray(parts, dtype=np.uint16)
    perm = np.ascontiguousarray(seg.perm, np.int32)
    out = np.ascontiguousarray(dst, dtype=np.uint16).copy()
    _load().lq_oracle_concat_rows(_p(parts), parts.shape[1], _p(perm), perm.shape[0], _p(out), out.shape[1])
    return out
