"""Thin ctypes binding over liblqlora.so (include/lqlora.h).  Argument marshalling only: every step
of the path runs in the library's HIP kernels.  PyTorch is used for device memory and streams.

There is no fallback: if the library has not been built (python -m paper_2511_00101_amd.build)
loading raises, and every entry point raises LqError on a non-zero status.
"""
from __future__ import annotations

import ctypes
import os
from dataclasses import dataclass
from typing import List, Optional, Sequence

import numpy as np
import torch

LQ_OK, LQ_ERR_INVALID_ARG, LQ_ERR_UNSUPPORTED, LQ_ERR_WORKSPACE, LQ_ERR_HIP = range(5)
LQ_SEG_FINETUNE, LQ_SEG_PREFILL, LQ_SEG_DECODE = 0, 1, 2
LQ_VARIANT_SPLIT, LQ_VARIANT_FUSED, LQ_VARIANT_SHRINK_ONLY, LQ_VARIANT_EXPAND_ONLY, LQ_VARIANT_SLAB, LQ_VARIANT_AUTO = 0, 1, 2, 3, 4, 5
LQ_MAX_RANK = 128
LQ_MAX_GROUP = 4
LQ_STATIC_WORKSPACE_BYTES = 4096 + (32 << 20)

LIB_PATH = os.path.join(os.path.dirname(os.path.abspath(__file__)), "liblqlora.so")
_lib = None

_i32, _i64, _vp, _sz = ctypes.c_int32, ctypes.c_int64, ctypes.c_void_p, ctypes.c_size_t

_SIGNATURES = {
    "lora_status_string": (ctypes.c_char_p, [ctypes.c_int]),
    "lora_workspace_bytes": (_sz, [_i32, _i32, _i32, _i32, _i32]),
    "lora_build_workspace_bytes": (_sz, [_i32, _i32]),
    "lora_build_segments": (ctypes.c_int, [_vp, _vp, _i32, _vp, _i32, _vp, _vp, _vp, _vp, _vp, _vp, _i32, _vp, _sz, _vp]),
    "lora_forward_workspace_bytes": (_sz, [_i32, _i32, _i32, _i32, _i32]),
    "lora_segmented_forward": (ctypes.c_int, [_vp, _i64, _vp, _i64, _i32, _i32, _vp, _vp, _vp, _vp, _vp, _i32, _i32,
                                              _vp, _i32, _vp, _vp, _vp, _vp, _i32, _vp, _vp, _i32, _vp, _sz, _vp]),
    "lora_forward_group_workspace_bytes": (_sz, [_i32, _i32, _i32]),
    "lora_segmented_forward_group": (ctypes.c_int, [_vp, _i64, _i32, _i32, _vp, _vp, _vp, _vp, _vp, _vp, _vp, _vp, _vp, _i32, _i32,
                                                    _vp, _i32, _vp, _vp, _vp, _vp, _i32, _vp, _i32, _vp, _sz, _vp]),
    "lora_segmented_forward_static": (ctypes.c_int, [_vp, _i64, _vp, _i64, _i32, _i32, _vp, _vp, _vp, _vp, _vp, _i32, _i32,
                                                     _vp, _i32, _vp, _vp, _vp, _vp, _i32, _vp, _vp, _i32, _vp, _vp]),
    "lora_backward_workspace_bytes": (_sz, [_i32, _i32, _i32, _i32, _i32]),
    "lora_segmented_backward": (ctypes.c_int, [_vp, _i64, _vp, _i64, _vp, _i64, _i32, _i32, _vp, _vp, _vp, _vp,
                                               _vp, _vp, _vp, _i32, _i32, _vp, _i32, _vp, _vp, _vp, _vp, _i32,
                                               _vp, _vp, _i32, _vp, _sz, _vp]),
    "lora_dropout_rows": (ctypes.c_int, [_vp, _i64, _vp, _i64, _i32, _vp, _vp, _i32, _i32, ctypes.c_uint32, ctypes.c_float, _vp]),
    "lora_kind_offsets": (ctypes.c_int, [_vp, _vp, _vp, _i32, _vp, _vp]),
    "lora_split_rows": (ctypes.c_int, [_vp, _i64, _i32, _vp, _i32, _vp, _vp, _i32, _vp, _vp]),
    "lora_concat_rows": (ctypes.c_int, [_vp, _i32, _vp, _i32, _vp, _vp, _i32, _vp, _i64, _vp]),
    "lora_profile_enable": (ctypes.c_int, [_i32]),
    "lora_profile_read": (ctypes.c_int, [_vp, _vp, _i32]),
}
KERNEL_NAMES = ("build", "shrink", "expand", "forward_fused", "wgrad", "wreduce", "forward_slab")


class LqError(RuntimeError):
    def __init__(self, status: int, where: str):
        self.status = status
        super().__init__(f"{where}: {lora_status_string(status)} (status {status})")


def lib() -> ctypes.CDLL:
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise RuntimeError(f"{LIB_PATH} is missing: build it with `python -m paper_2511_00101_amd.build` "
                               "(there is no CPU fallback)")
        L = ctypes.CDLL(LIB_PATH)
        for name, (res, args) in _SIGNATURES.items():
            fn = getattr(L, name)
            fn.restype, fn.argtypes = res, args
        _lib = L
    return _lib


def exported_symbols() -> List[str]:
    return list(_SIGNATURES)


def _ptr(t: Optional[torch.Tensor]) -> Optional[int]:
    return None if t is None else t.data_ptr()


def _stream(stream) -> Optional[int]:
    if stream is None:
        stream = torch.cuda.current_stream()
    if isinstance(stream, torch.cuda.Stream):
        return stream.cuda_stream
    return int(stream) or None


def lora_status_string(status: int) -> str:
    return lib().lora_status_string(int(status)).decode()


def lora_workspace_bytes(n_tokens: int, n_adapters: int, max_rank: int, d_in: int, d_out: int) -> int:
    return int(lib().lora_workspace_bytes(n_tokens, n_adapters, max_rank, d_in, d_out))


def lora_build_workspace_bytes(n_tokens: int, n_adapters: int) -> int:
    return int(lib().lora_build_workspace_bytes(n_tokens, n_adapters))


def lora_forward_workspace_bytes(n_tokens: int, max_rank: int, d_in: int, d_out: int, variant: int) -> int:
    return int(lib().lora_forward_workspace_bytes(n_tokens, max_rank, d_in, d_out, variant))


def lora_backward_workspace_bytes(n_tokens: int, n_adapters: int, max_rank: int, d_in: int, d_out: int) -> int:
    return int(lib().lora_backward_workspace_bytes(n_tokens, n_adapters, max_rank, d_in, d_out))


@dataclass
class SegmentTables:
    """Device buffers the builder fills and the forward/backward read."""
    perm: torch.Tensor         # int32[n_tokens]
    seg_starts: torch.Tensor   # int32[max_segments + 1]
    seg_adapter: torch.Tensor  # int32[max_segments]
    seg_kind: torch.Tensor     # uint8[max_segments]
    h_offsets: torch.Tensor    # int64[max_segments + 1]
    n_segments: torch.Tensor   # int32[1]
    max_segments: int
    n_tokens: int

    @staticmethod
    def empty(n_tokens: int, n_adapters: int, device="cuda", max_segments: Optional[int] = None) -> "SegmentTables":
        if max_segments is None:
            max_segments = min(n_tokens, 3 * n_adapters)
        dev = torch.device(device)
        return SegmentTables(
            perm=torch.zeros(max(n_tokens, 1), dtype=torch.int32, device=dev),
            seg_starts=torch.zeros(max_segments + 1, dtype=torch.int32, device=dev),
            seg_adapter=torch.zeros(max(max_segments, 1), dtype=torch.int32, device=dev),
            seg_kind=torch.zeros(max(max_segments, 1), dtype=torch.uint8, device=dev),
            h_offsets=torch.zeros(max_segments + 1, dtype=torch.int64, device=dev),
            n_segments=torch.zeros(1, dtype=torch.int32, device=dev),
            max_segments=max_segments, n_tokens=n_tokens)

    def to_host(self):
        """Copies the tables back (synchronises); trims to the live part."""
        n = int(self.n_segments.item())
        starts = self.seg_starts[: n + 1].cpu().numpy()
        n_live = int(starts[n]) if n >= 0 else 0
        return dict(perm=self.perm[:n_live].cpu().numpy(), seg_starts=starts,
                    seg_adapter=self.seg_adapter[:n].cpu().numpy(), seg_kind=self.seg_kind[:n].cpu().numpy(),
                    h_offsets=self.h_offsets[: n + 1].cpu().numpy(), n_segments=n)


class PreparedCall:
    """An entry point with its arguments marshalled once: for loops that repeat the same call (the tensors must stay
    alive and in place; the stream is the one that was current when the call was prepared)."""

    def __init__(self, fn, args, where: str):
        self.fn, self.args, self.where = fn, args, where

    def __call__(self) -> None:
        st = self.fn(*self.args)
        if st != LQ_OK:
            raise LqError(st, self.where)


def _build_segments_args(token_adapter, token_kind, ranks, out, workspace, stream):
    n_tokens = int(token_adapter.shape[0])
    n_adapters = int(ranks.shape[0])
    assert token_adapter.dtype == torch.int32 and token_kind.dtype == torch.uint8 and ranks.dtype == torch.int32
    assert token_adapter.is_contiguous() and token_kind.is_contiguous() and ranks.is_contiguous()
    return (_ptr(token_adapter) if n_tokens else None, _ptr(token_kind) if n_tokens else None,
            n_tokens, _ptr(ranks), n_adapters,
            _ptr(out.perm), _ptr(out.seg_starts), _ptr(out.seg_adapter), _ptr(out.seg_kind),
            _ptr(out.h_offsets), _ptr(out.n_segments), out.max_segments,
            _ptr(workspace), 0 if workspace is None else workspace.numel() * workspace.element_size(),
            _stream(stream))


def lora_build_segments(token_adapter: torch.Tensor, token_kind: torch.Tensor, ranks: torch.Tensor,
                        out: SegmentTables, workspace: Optional[torch.Tensor] = None, stream=None) -> SegmentTables:
    st = lib().lora_build_segments(*_build_segments_args(token_adapter, token_kind, ranks, out, workspace, stream))
    if st != LQ_OK:
        raise LqError(st, "lora_build_segments")
    return out


def prepare_build_segments(token_adapter, token_kind, ranks, out, workspace=None, stream=None) -> PreparedCall:
    return PreparedCall(lib().lora_build_segments, _build_segments_args(token_adapter, token_kind, ranks, out, workspace, stream),
                        "lora_build_segments")


@dataclass
class AdapterTable:
    """Per-adapter weights of one linear layer, kept as separate tensors (never concatenated) plus the
    device pointer tables the library takes.  Swapping an adapter = rewriting one pointer."""
    A: List[torch.Tensor]      # bf16 [r, d_in]
    B: List[torch.Tensor]      # bf16 [r, d_out]
    ranks: torch.Tensor        # int32[n]
    scales: torch.Tensor       # float32[n]
    A_ptrs: torch.Tensor       # int64[n]
    B_ptrs: torch.Tensor       # int64[n]
    max_rank: int

    @staticmethod
    def from_tensors(A: Sequence[torch.Tensor], B: Sequence[torch.Tensor], scales, device="cuda") -> "AdapterTable":
        dev = torch.device(device)
        A = [a.contiguous() for a in A]
        B = [b.contiguous() for b in B]
        ranks = torch.tensor([a.shape[0] for a in A], dtype=torch.int32, device=dev)
        sc = torch.as_tensor(np.asarray(scales, dtype=np.float32)).to(dev)
        ap = torch.tensor([a.data_ptr() for a in A], dtype=torch.int64, device=dev)
        bp = torch.tensor([b.data_ptr() for b in B], dtype=torch.int64, device=dev)
        return AdapterTable(list(A), list(B), ranks, sc, ap, bp, max(int(a.shape[0]) for a in A))

    @property
    def n_adapters(self) -> int:
        return len(self.A)


def _token_scales_ptr(token_scales, n_tokens):
    if token_scales is None:
        return None
    assert token_scales.dtype == torch.float32 and token_scales.is_contiguous() and token_scales.numel() == n_tokens
    return token_scales.data_ptr()


def _forward_args(x, y, adapters, seg, h_out, workspace, variant, use_perm, stream, token_scales=None):
    assert x.dtype == torch.bfloat16 and y.dtype == torch.bfloat16
    assert x.stride(1) == 1 and y.stride(1) == 1
    n_tokens, d_in = int(x.shape[0]), int(x.shape[1])
    d_out = int(y.shape[1])
    return (_ptr(x), x.stride(0), _ptr(y), y.stride(0), d_in, d_out,
            _ptr(adapters.A_ptrs), _ptr(adapters.B_ptrs), _ptr(adapters.ranks), _ptr(adapters.scales),
            _token_scales_ptr(token_scales, n_tokens), adapters.n_adapters, adapters.max_rank,
            _ptr(seg.perm) if use_perm else None, n_tokens,
            _ptr(seg.seg_starts), _ptr(seg.seg_adapter), _ptr(seg.seg_kind), _ptr(seg.n_segments), seg.max_segments,
            _ptr(h_out), _ptr(seg.h_offsets) if h_out is not None else None,
            variant, _ptr(workspace), 0 if workspace is None else workspace.numel() * workspace.element_size(), _stream(stream))


def lora_segmented_forward(x: torch.Tensor, y: torch.Tensor, adapters: AdapterTable, seg: SegmentTables,
                           h_out: Optional[torch.Tensor], workspace: torch.Tensor,
                           variant: int = LQ_VARIANT_SPLIT, use_perm: bool = True, stream=None,
                           token_scales: Optional[torch.Tensor] = None) -> None:
    st = lib().lora_segmented_forward(*_forward_args(x, y, adapters, seg, h_out, workspace, variant, use_perm, stream,
                                                     token_scales))
    if st != LQ_OK:
        raise LqError(st, "lora_segmented_forward")


def lora_forward_group_workspace_bytes(n_proj: int, n_tokens: int, max_rank: int) -> int:
    return int(lib().lora_forward_group_workspace_bytes(n_proj, n_tokens, max_rank))


def _group_args(x, ys, adapters, seg, h_outs, workspace, variant, use_perm, stream, token_scales):
    """Arguments of lora_segmented_forward_group; the host arrays are returned as well (they must outlive the call)."""
    n = len(ys)
    assert n == len(adapters) and 1 <= n <= LQ_MAX_GROUP and (h_outs is None or len(h_outs) == n)
    assert x.dtype == torch.bfloat16 and x.stride(1) == 1 and all(y.dtype == torch.bfloat16 and y.stride(1) == 1 for y in ys)
    a0 = adapters[0]
    assert all(ad.n_adapters == a0.n_adapters and ad.max_rank == a0.max_rank for ad in adapters)
    n_tokens, d_in = int(x.shape[0]), int(x.shape[1])
    hy = (ctypes.c_void_p * n)(*[y.data_ptr() for y in ys])
    hld = (ctypes.c_int64 * n)(*[y.stride(0) for y in ys])
    hd = (ctypes.c_int32 * n)(*[int(y.shape[1]) for y in ys])
    hA = (ctypes.c_void_p * n)(*[ad.A_ptrs.data_ptr() for ad in adapters])
    hB = (ctypes.c_void_p * n)(*[ad.B_ptrs.data_ptr() for ad in adapters])
    hh = None if h_outs is None else (ctypes.c_void_p * n)(*[_ptr(h) for h in h_outs])
    keep = (hy, hld, hd, hA, hB, hh)
    cast = lambda a: None if a is None else ctypes.cast(a, ctypes.c_void_p)
    args = (_ptr(x), x.stride(0), d_in, n, cast(hy), cast(hld), cast(hd), cast(hA), cast(hB), cast(hh),
            _ptr(a0.ranks), _ptr(a0.scales), _token_scales_ptr(token_scales, n_tokens), a0.n_adapters, a0.max_rank,
            _ptr(seg.perm) if use_perm else None, n_tokens,
            _ptr(seg.seg_starts), _ptr(seg.seg_adapter), _ptr(seg.seg_kind), _ptr(seg.n_segments), seg.max_segments,
            _ptr(seg.h_offsets) if h_outs is not None else None,
            variant, _ptr(workspace), workspace.numel() * workspace.element_size(), _stream(stream))
    return args, keep


def lora_segmented_forward_group(x: torch.Tensor, ys: Sequence[torch.Tensor], adapters: Sequence[AdapterTable],
                                 seg: SegmentTables, h_outs: Optional[Sequence[Optional[torch.Tensor]]],
                                 workspace: torch.Tensor, variant: int = LQ_VARIANT_FUSED, use_perm: bool = True, stream=None,
                                 token_scales: Optional[torch.Tensor] = None) -> None:
    """Several linear layers that read the same x (q, k, v; gate, up) in one call.  The adapter tables of the
    layers must agree in the number of adapters, their ranks and their scales (those of adapters[0] are used)."""
    args, keep = _group_args(x, ys, adapters, seg, h_outs, workspace, variant, use_perm, stream, token_scales)
    st = lib().lora_segmented_forward_group(*args)
    del keep
    if st != LQ_OK:
        raise LqError(st, "lora_segmented_forward_group")


def prepare_forward_group(x, ys, adapters, seg, h_outs, workspace, variant=LQ_VARIANT_FUSED, use_perm=True, stream=None,
                          token_scales=None) -> PreparedCall:
    args, keep = _group_args(x, ys, adapters, seg, h_outs, workspace, variant, use_perm, stream, token_scales)
    call = PreparedCall(lib().lora_segmented_forward_group, args, "lora_segmented_forward_group")
    call.keep = keep   # the host arrays the arguments point to
    return call


def lora_segmented_forward_static(x: torch.Tensor, y: torch.Tensor, adapters: AdapterTable, seg: SegmentTables,
                                  h_out: Optional[torch.Tensor], error_word: Optional[torch.Tensor] = None,
                                  variant: int = LQ_VARIANT_SPLIT, use_perm: bool = True, stream=None,
                                  token_scales: Optional[torch.Tensor] = None) -> None:
    """The forward with the library's own device array as workspace (allocates nothing)."""
    args = _forward_args(x, y, adapters, seg, h_out, None, variant, use_perm, stream, token_scales)
    assert error_word is None or error_word.dtype == torch.int32
    st = lib().lora_segmented_forward_static(*args[:23], _ptr(error_word), args[25])   # all but the workspace pair
    if st != LQ_OK:
        raise LqError(st, "lora_segmented_forward_static")


def prepare_forward(x, y, adapters, seg, h_out, workspace, variant=LQ_VARIANT_SPLIT, use_perm=True, stream=None,
                    token_scales=None) -> PreparedCall:
    return PreparedCall(lib().lora_segmented_forward,
                        _forward_args(x, y, adapters, seg, h_out, workspace, variant, use_perm, stream, token_scales),
                        "lora_segmented_forward")


def lora_segmented_backward(x: torch.Tensor, dy: torch.Tensor, dx: torch.Tensor, adapters: AdapterTable,
                            dA_ptrs: Optional[torch.Tensor], dB_ptrs: Optional[torch.Tensor], seg: SegmentTables,
                            h_saved: torch.Tensor, workspace: torch.Tensor, variant: int = LQ_VARIANT_FUSED,
                            use_perm: bool = True, stream=None, token_scales: Optional[torch.Tensor] = None) -> None:
    assert x.dtype == torch.bfloat16 and dy.dtype == torch.bfloat16 and dx.dtype == torch.bfloat16
    n_tokens, d_in = int(x.shape[0]), int(x.shape[1])
    d_out = int(dy.shape[1])
    st = lib().lora_segmented_backward(
        _ptr(x), x.stride(0), _ptr(dy), dy.stride(0), _ptr(dx), dx.stride(0), d_in, d_out,
        _ptr(adapters.A_ptrs), _ptr(adapters.B_ptrs), _ptr(dA_ptrs), _ptr(dB_ptrs),
        _ptr(adapters.ranks), _ptr(adapters.scales), _token_scales_ptr(token_scales, n_tokens),
        adapters.n_adapters, adapters.max_rank,
        _ptr(seg.perm) if use_perm else None, n_tokens,
        _ptr(seg.seg_starts), _ptr(seg.seg_adapter), _ptr(seg.seg_kind), _ptr(seg.n_segments), seg.max_segments,
        _ptr(h_saved), _ptr(seg.h_offsets), variant, _ptr(workspace), workspace.numel() * workspace.element_size(),
        _stream(stream))
    if st != LQ_OK:
        raise LqError(st, "lora_segmented_backward")


def lora_dropout_rows(x: torch.Tensor, out: torch.Tensor, token_adapter: torch.Tensor, token_kind: torch.Tensor,
                      n_adapters: int, seed: int, p: float, stream=None) -> None:
    """out = mask * x on the fine-tuning rows (copy elsewhere); out may be x itself."""
    assert x.dtype == torch.bfloat16 and out.dtype == torch.bfloat16 and x.shape == out.shape
    assert x.stride(1) == 1 and out.stride(1) == 1
    st = lib().lora_dropout_rows(_ptr(x), x.stride(0), _ptr(out), out.stride(0), int(x.shape[1]), _ptr(token_adapter),
                                 _ptr(token_kind), int(x.shape[0]), n_adapters, seed & 0xffffffff, float(p), _stream(stream))
    if st != LQ_OK:
        raise LqError(st, "lora_dropout_rows")


def lora_kind_offsets(seg: SegmentTables, out: Optional[torch.Tensor] = None, stream=None) -> torch.Tensor:
    out = torch.zeros(4, dtype=torch.int32, device=seg.perm.device) if out is None else out
    st = lib().lora_kind_offsets(_ptr(seg.seg_starts), _ptr(seg.seg_kind), _ptr(seg.n_segments), seg.max_segments, _ptr(out),
                                 _stream(stream))
    if st != LQ_OK:
        raise LqError(st, "lora_kind_offsets")
    return out


def lora_split_rows(src: torch.Tensor, seg: SegmentTables, parts: torch.Tensor, use_perm: bool = True, stream=None) -> None:
    assert src.dtype == torch.bfloat16 and parts.dtype == torch.bfloat16 and parts.is_contiguous() and src.stride(1) == 1
    st = lib().lora_split_rows(_ptr(src), src.stride(0), int(src.shape[1]), _ptr(seg.perm) if use_perm else None,
                               int(src.shape[0]), _ptr(seg.seg_starts), _ptr(seg.n_segments), seg.max_segments, _ptr(parts),
                               _stream(stream))
    if st != LQ_OK:
        raise LqError(st, "lora_split_rows")


def lora_concat_rows(parts: torch.Tensor, seg: SegmentTables, dst: torch.Tensor, use_perm: bool = True, stream=None) -> None:
    assert dst.dtype == torch.bfloat16 and parts.dtype == torch.bfloat16 and parts.is_contiguous() and dst.stride(1) == 1
    st = lib().lora_concat_rows(_ptr(parts), int(dst.shape[1]), _ptr(seg.perm) if use_perm else None, int(dst.shape[0]),
                                _ptr(seg.seg_starts), _ptr(seg.n_segments), seg.max_segments, _ptr(dst), dst.stride(0),
                                _stream(stream))
    if st != LQ_OK:
        raise LqError(st, "lora_concat_rows")


# ---- plumbing between numpy bf16 bit patterns and device tensors ------------------------------------------------
def bf16_from_bits(bits: np.ndarray, device="cuda") -> torch.Tensor:
    return torch.from_numpy(np.ascontiguousarray(bits).view(np.int16)).view(torch.bfloat16).to(device)


def bits_from_bf16(t: torch.Tensor) -> np.ndarray:
    return t.detach().contiguous().view(torch.int16).cpu().numpy().view(np.uint16)


def workspace(n_bytes: int, device="cuda") -> torch.Tensor:
    return torch.zeros((max(n_bytes, 4096) + 7) // 8, dtype=torch.int64, device=device)


LQ_DEVICE_ERR_BAD_SEGMENT = 1      # a segment was skipped: adapter id, rank, matrix pointer or row range unusable
LQ_DEVICE_ERR_BARRIER_TIMEOUT = 2  # the single-launch kernel's device-wide wait ran out: y / dx were left untouched


class LqDeviceError(RuntimeError):
    """The kernels reported a problem in the workspace's error word (the library itself never synchronises)."""

    def __init__(self, bits: int, where: str):
        names = [n for b, n in ((LQ_DEVICE_ERR_BAD_SEGMENT, "bad segment table entry (segment skipped)"),
                                (LQ_DEVICE_ERR_BARRIER_TIMEOUT, "device-wide wait timed out (outputs left untouched; "
                                 "use LQ_VARIANT_SLAB or LQ_VARIANT_SPLIT when the device is shared)")) if bits & b]
        super().__init__(f"{where}: device error word {bits:#x}: " + "; ".join(names or ["unknown bits"]))
        self.bits = bits


def device_error_word(workspace_or_word: torch.Tensor) -> int:
    """The error word of a workspace (its first 32 bits) or of a one-element int32 tensor; waits for the stream."""
    t = workspace_or_word.view(-1)[:1]
    return int(t.view(torch.int32)[0].item()) & 0xffffffff


def raise_on_device_error(workspace_or_word: torch.Tensor, where: str = "lqlora") -> None:
    """Checked mode for callers that can afford a synchronisation: raises LqDeviceError if the kernels that used this
    workspace set a bit of its error word.  The word is left as it is (the caller zeroes the header to clear it)."""
    bits = device_error_word(workspace_or_word)
    if bits:
        raise LqDeviceError(bits, where)


def lora_profile_enable(on: bool) -> None:
    """Start (or stop) timing the library's own launches; either way what was recorded is discarded."""
    st = lib().lora_profile_enable(1 if on else 0)
    if st != LQ_OK:
        raise LqError(st, "lora_profile_enable")


def lora_profile_read() -> dict:
    """Waits for the recorded launches; {kernel name: (summed microseconds, launches)} since recording started."""
    n = len(KERNEL_NAMES)
    total = (ctypes.c_double * n)()
    count = (ctypes.c_int64 * n)()
    st = lib().lora_profile_read(ctypes.cast(total, ctypes.c_void_p), ctypes.cast(count, ctypes.c_void_p), n)
    if st != LQ_OK:
        raise LqError(st, "lora_profile_read")
    return {name: (float(total[i]), int(count[i])) for i, name in enumerate(KERNEL_NAMES)}
