"""The C-ABI library loads, exports every symbol include/lqlora.h declares, and rejects bad host
arguments before launching anything (so these run without a GPU)."""
import ctypes
import os
import re

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


@pytest.fixture(scope="module")
def lqlib():
    from paper_2511_00101_amd import binding
    if not os.path.exists(binding.LIB_PATH):
        from paper_2511_00101_amd import build
        build.build_library()
    return binding


def declared_functions():
    text = open(os.path.join(ROOT, "include", "lqlora.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(lora_[a-z_]+)\s*\(", text)))


def test_header_symbols_are_exported_and_bound(lqlib):
    names = declared_functions()
    assert len(names) >= 7
    L = lqlib.lib()
    for n in names:
        assert hasattr(L, n), n
    assert sorted(lqlib.exported_symbols()) == names


def test_status_strings(lqlib):
    assert lqlib.lora_status_string(0) == "ok"
    assert len({lqlib.lora_status_string(i) for i in range(5)}) == 5


def test_workspace_sizes(lqlib):
    a = lqlib.lora_forward_workspace_bytes(256, 16, 4096, 4096, 0)
    b = lqlib.lora_forward_workspace_bytes(512, 16, 4096, 4096, 0)
    assert 256 <= a < b
    assert lqlib.lora_build_workspace_bytes(100, 64) >= 256
    c = lqlib.lora_backward_workspace_bytes(1024, 4, 16, 512, 768)
    assert c > lqlib.lora_forward_workspace_bytes(1024, 16, 512, 768, 0)
    # the one-size-fits-all answer is the largest of the per-call ones
    for (T, n_ad, r, d_in, d_out) in ((1024, 4, 16, 512, 768), (256, 64, 16, 4096, 4096), (100000, 2000, 128, 64, 64), (0, 1, 1, 8, 8)):
        each = [lqlib.lora_build_workspace_bytes(T, n_ad), lqlib.lora_backward_workspace_bytes(T, n_ad, r, d_in, d_out)]
        each += [lqlib.lora_forward_workspace_bytes(T, r, d_in, d_out, v) for v in range(4)]
        assert lqlib.lora_workspace_bytes(T, n_ad, r, d_in, d_out) == max(each)


def test_host_validation_returns_codes_without_launching(lqlib):
    L = lqlib.lib()
    one = ctypes.c_void_p(0x1000)        # never dereferenced: validation fails first
    al = ctypes.c_void_p(0x2000)

    def fwd(x=one, ldx=64, y=al, ldy=64, d_in=64, d_out=64, n_ad=2, max_rank=8, T=4, max_seg=4, variant=0,
            ws=ctypes.c_void_p(0x4000), ws_bytes=1 << 30):
        return L.lora_segmented_forward(x, ldx, y, ldy, d_in, d_out, one, one, one, one, None, n_ad, max_rank, one, T,
                                        one, one, one, one, max_seg, None, None, variant, ws, ws_bytes, None)

    assert fwd(d_in=0) == lqlib.LQ_ERR_INVALID_ARG
    assert fwd(x=None) == lqlib.LQ_ERR_INVALID_ARG
    assert fwd(ldx=32) == lqlib.LQ_ERR_INVALID_ARG
    assert fwd(variant=9) == lqlib.LQ_ERR_INVALID_ARG
    assert fwd(y=one) == lqlib.LQ_ERR_INVALID_ARG              # x aliases y
    assert fwd(d_in=60, ldx=64) == lqlib.LQ_ERR_UNSUPPORTED      # not a multiple of 8
    assert fwd(max_rank=129) == lqlib.LQ_ERR_UNSUPPORTED
    assert fwd(x=ctypes.c_void_p(0x1004)) == lqlib.LQ_ERR_UNSUPPORTED   # misaligned
    assert fwd(ws=None) == lqlib.LQ_ERR_WORKSPACE
    assert fwd(ws_bytes=16) == lqlib.LQ_ERR_WORKSPACE
    assert fwd(T=0) == lqlib.LQ_OK                                # empty batch: nothing to do, nothing launched

    def bwd(x=one, dy=al, dx=ctypes.c_void_p(0x3000), d_in=64, d_out=64, ldx=64, T=4, ws=ctypes.c_void_p(0x4000),
            ws_bytes=1 << 30, max_rank=8, variant=1):
        return L.lora_segmented_backward(x, ldx, dy, 64, dx, 64, d_in, d_out, one, one, None, None, one, one, None, 2, max_rank,
                                         one, T, one, one, one, one, 4, None, None, variant, ws, ws_bytes, None)

    assert bwd(variant=2) == lqlib.LQ_ERR_INVALID_ARG            # only the two-launch and the single-launch forms
    assert bwd(d_in=0) == lqlib.LQ_ERR_INVALID_ARG
    assert bwd(dx=one) == lqlib.LQ_ERR_INVALID_ARG               # dx aliases x
    assert bwd(ldx=8) == lqlib.LQ_ERR_INVALID_ARG
    assert bwd(max_rank=200) == lqlib.LQ_ERR_UNSUPPORTED
    assert bwd(ws_bytes=100) == lqlib.LQ_ERR_WORKSPACE
    assert bwd(T=0) == lqlib.LQ_OK

    def bld(T=4, n_ad=2, max_seg=4, ranks=one):
        return L.lora_build_segments(one, one, T, ranks, n_ad, one, one, one, one, one, one, max_seg, None, 0, None)

    assert bld(T=-1) == lqlib.LQ_ERR_INVALID_ARG
    assert bld(n_ad=0) == lqlib.LQ_ERR_INVALID_ARG
    assert bld(ranks=None) == lqlib.LQ_ERR_INVALID_ARG
    assert bld(max_seg=3) == lqlib.LQ_ERR_INVALID_ARG             # tables too small for min(T, 3 * n_adapters)
    assert bld(n_ad=5000, max_seg=4) == lqlib.LQ_ERR_UNSUPPORTED
    assert bld(T=100000, n_ad=2000, max_seg=6000) == lqlib.LQ_ERR_WORKSPACE   # needs the global histogram
