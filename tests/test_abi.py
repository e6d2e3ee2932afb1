"""Host-only checks of the C-ABI library: it loads, exports every symbol the
header declares, and rejects bad arguments before anything is launched."""
import ctypes
import os
import re

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
HEADER = os.path.join(ROOT, "include", "gqa_decode.h")
LIB = os.path.join(ROOT, "paper_2510_07356_amd", "libgqa_decode.so")


@pytest.fixture(scope="module")
def lib():
    if not os.path.exists(LIB):
        from paper_2510_07356_amd.build import build_library
        build_library()
    from paper_2510_07356_amd import binding
    return binding


def declared_functions():
    text = open(HEADER).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(gqa_(?:decode|timer|cascade|prefill)_\w+)\s*\(", text)))


def test_header_and_library_agree(lib):
    names = declared_functions()
    assert set(names) == set(lib.EXPORTS)
    raw = ctypes.CDLL(LIB)
    for n in names:
        assert hasattr(raw, n), n


def test_curation_header_and_library_agree(lib):
    text = re.sub(r"/\*.*?\*/", "", open(os.path.join(ROOT, "include", "concur_curation.h")).read(), flags=re.S)
    names = sorted(set(re.findall(r"\b(concur_\w+)\s*\(", text)))
    assert set(names) == set(lib.CURATION_EXPORTS) and len(names) == 7
    raw = ctypes.CDLL(LIB)
    for n in names:
        assert hasattr(raw, n), n


def test_timer_rejects_bad_arguments():
    raw = ctypes.CDLL(LIB)
    raw.gqa_timer_read_calls.argtypes = [ctypes.c_void_p, ctypes.c_int32, ctypes.c_void_p, ctypes.c_void_p, ctypes.c_void_p]
    assert raw.gqa_timer_read_calls(None, 4, None, None, None) == -1
    raw.gqa_timer_read.argtypes = [ctypes.c_void_p, ctypes.c_void_p, ctypes.c_void_p]
    assert raw.gqa_timer_read(None, None, None) == -1


def test_version_and_strerror(lib):
    assert lib.gqa_decode_version() >= 100
    assert lib.gqa_decode_strerror(0) == "ok"
    for code in (-1, -2, -3, -4, -99):
        assert lib.gqa_decode_strerror(code)


def params(lib, **kw):
    p = lib.gqa_decode_params()
    p.batch, p.num_q_heads, p.num_kv_heads, p.head_dim = 4, 40, 8, 128
    p.max_kv_len, p.page_size, p.block_table_stride, p.chunk_tokens = 4096, 0, 0, 0
    p.scale, p.kernel_variant = 0.088, 0
    p.q_stride_b, p.q_stride_h = 40 * 128, 128
    p.k_stride_b, p.k_stride_h, p.k_stride_t = 8 * 4096 * 128, 4096 * 128, 128
    p.v_stride_b, p.v_stride_h, p.v_stride_t = 8 * 4096 * 128, 4096 * 128, 128
    for k, v in kw.items():
        setattr(p, k, v)
    return p


def test_workspace_size_covers_all_partials(lib):
    """One partial slot per (share, row) piece: slots >= shares + rows, each
    holding G * (128 + 2) floats."""
    p = params(lib, chunk_tokens=256)
    info = lib.gqa_decode_plan_info(p)
    assert info.share_tokens == 256
    shares = 4 * 8 * (4096 // 256)
    assert info.partial_slots >= shares + 4 * 8
    assert lib.gqa_decode_workspace_bytes(p) >= info.partial_slots * 5 * (128 + 2) * 4 + 4 * 5
    auto = lib.gqa_decode_plan_info(params(lib))
    assert auto.share_tokens == 0 and auto.partial_slots >= 4 * 8
    small = lib.gqa_decode_plan_info(params(lib, chunk_tokens=64, max_kv_len=32768, batch=128))
    assert small.partial_slots >= 128 * 8 * (32768 // 64) + 128 * 8


@pytest.mark.parametrize("kw,code", [
    (dict(batch=0), -1), (dict(num_q_heads=41), -1), (dict(max_kv_len=-1), -1),
    (dict(chunk_tokens=48), -1), (dict(kernel_variant=7), -1), (dict(scale=float("nan")), -1),
    (dict(head_dim=64), -2), (dict(num_q_heads=8 * 17), -2), (dict(page_size=24), -2),
    (dict(page_size=8), -2), (dict(num_q_heads=8 * 16, kernel_variant=1), -2),
    (dict(page_size=16, block_table_stride=10), -1),
])
def test_bad_shapes_are_rejected(lib, kw, code):
    p = params(lib, **kw)
    assert lib.gqa_decode_workspace_bytes(p) == 0
    with pytest.raises(lib.GqaError) as e:
        lib.gqa_decode_plan_info(p)
    assert e.value.status == code


def test_bad_pointers_and_workspace_are_rejected_before_launch(lib):
    """Null / misaligned pointers and short workspaces return an error code; no
    HIP call is made on these paths, so this runs without a GPU."""
    raw = lib._lib
    p = params(lib)
    need = lib.gqa_decode_workspace_bytes(p)
    good = 0x10000            # never dereferenced on these paths
    def call(q=good, k=good, v=good, lens=good, bt=None, out=good, ws=good, ws_bytes=need, pp=p):
        return raw.gqa_decode_attn(ctypes.byref(pp), q, k, v, lens, bt, None, out, None, ws, ws_bytes, None)
    assert call(q=None) == -1 and call(k=None) == -1 and call(v=None) == -1
    assert call(lens=None) == -1 and call(out=None) == -1 and call(ws=None) == -1
    assert call(q=good + 2) == -1 and call(ws=good + 16) == -1
    assert call(bt=good) == -1                                  # block table without paging
    assert call(ws_bytes=need - 1) == -3
    assert call(pp=params(lib, k_stride_t=132)) == -1           # rows not 16-byte aligned
    assert call(pp=params(lib, page_size=16, block_table_stride=256)) == -1   # paging without table
    assert raw.gqa_decode_attn(None, good, good, good, good, None, None, good, None, good, need, None) == -1


def test_append_rejects_bad_arguments_before_launch(lib):
    raw = lib._lib
    p = lib.gqa_append_params()
    p.batch, p.num_q_heads, p.num_kv_heads, p.head_dim = 2, 40, 8, 128
    p.max_kv_len, p.page_size, p.block_table_stride, p.rope_positions = 512, 0, 0, 512
    p.q_stride_b, p.q_stride_h = 40 * 128, 128
    p.k_stride_b, p.k_stride_h, p.k_stride_t = 8 * 512 * 128, 512 * 128, 128
    p.v_stride_b, p.v_stride_h, p.v_stride_t = 8 * 512 * 128, 512 * 128, 128
    g = 0x10000
    def call(pp=p, q=g, cs=g, bt=None):
        return raw.gqa_decode_kv_append(ctypes.byref(pp), q, g, g, g, g, g, g, bt, cs, None)
    assert call(q=None) == -1
    assert call(bt=g) == -1                                  # block table without paging
    p.rope_positions = 100
    assert call() == -1                                      # table shorter than the length bound
    p.rope_positions = 512
    p.head_dim = 64
    assert call() == -2
    p.head_dim = 128
    p.page_size = 24
    assert call() == -2
    assert raw.gqa_decode_kv_append(None, g, g, g, g, g, g, g, None, None, None) == -1
