"""gqa_decode_attn_static (the entry point that allocates nothing: partial results go to the
library's built-in per-device scratch buffer) against gqa_decode_attn with a caller-owned
workspace, through the C ABI: two calls in a row on the same device, the second on a smaller
batch, so the second call finds the first one's partial results in the buffer."""
import ctypes

import numpy as np
import pytest

from oracle import decode_attn
from paper_2510_07356_amd import workloads as wl

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def binding():
    from paper_2510_07356_amd import binding as b
    return b


def both_entry_points(binding, w, chunk_tokens=0):
    import torch
    dev = binding.to_device(w)
    params = binding.make_params(dev["q"], dev["k"], dev["v"], w.max_kv_len, w.scale, w.page_size,
                                 dev["block_table"], chunk_tokens, 0)
    shape = (w.batch, w.num_q_heads, w.head_dim)
    ref_out = torch.full(shape, float("nan"), dtype=torch.float32, device="cuda:0")
    ref_lse = torch.full(shape[:2], float("nan"), dtype=torch.float32, device="cuda:0")
    ws = torch.full((binding.gqa_decode_workspace_bytes(params),), 0xFF, dtype=torch.uint8, device="cuda:0")
    binding.gqa_decode_attn(params, dev["q"], dev["k"], dev["v"], dev["kv_lens"], dev["block_table"], None,
                            ref_out, ref_lse, ws)
    out = torch.full(shape, float("nan"), dtype=torch.float32, device="cuda:0")
    lse = torch.full(shape[:2], float("nan"), dtype=torch.float32, device="cuda:0")
    binding.gqa_decode_attn_static(params, dev["q"], dev["k"], dev["v"], dev["kv_lens"], dev["block_table"],
                                   out, lse)
    torch.cuda.synchronize()
    return out, lse, ref_out, ref_lse


def check_against_oracle(w, out, lse):
    ref = decode_attn(w.q, w.k, w.v, w.kv_lens, w.scale, block_table=w.block_table, page_size=w.page_size)
    got = out.double().cpu().numpy()
    err = got - ref.out
    assert np.isfinite(got).all()
    assert np.abs(err).max() <= 1e-2 and np.linalg.norm(err) / np.linalg.norm(ref.out) <= 5e-3
    live = w.kv_lens > 0
    assert np.abs(lse.double().cpu().numpy()[live] - ref.lse[live]).max() <= 4e-3


def test_two_calls_in_a_row_match_the_workspace_entry_point(binding):
    import torch
    binding.gqa_decode_init()
    assert binding.gqa_decode_static_scratch_bytes() == 32 << 20
    # first call: ragged batch, several shares per row and several rows per share
    big = wl.make_contiguous("static_big", 41, 12, 40, 8, [3000, 1, 517, 2048, 0, 999, 64, 4097, 33, 1500, 2500, 700])
    out, lse, ref_out, ref_lse = both_entry_points(binding, big)
    assert torch.equal(out, ref_out) and torch.equal(lse, ref_lse)
    check_against_oracle(big, out, lse)
    # second call, smaller and paged: the buffer still holds the first call's partial results
    small = wl.make_paged("static_small", 42, 3, 32, 8, [130, 16, 257], table_width=32)
    out, lse, ref_out, ref_lse = both_entry_points(binding, small)
    assert torch.equal(out, ref_out) and torch.equal(lse, ref_lse)
    check_against_oracle(small, out, lse)
    # third: fixed share length (other slot arithmetic), smaller again
    tiny = wl.make_contiguous("static_tiny", 43, 2, 40, 8, [95, 31])
    out, lse, ref_out, ref_lse = both_entry_points(binding, tiny, chunk_tokens=32)
    assert torch.equal(out, ref_out) and torch.equal(lse, ref_lse)
    check_against_oracle(tiny, out, lse)


def test_limit_and_argument_errors(binding):
    import torch
    w = wl.make_contiguous("static_err", 44, 2, 40, 8, [64, 64])
    dev = binding.to_device(w)
    out = torch.empty((2, 40, 128), dtype=torch.float32, device="cuda:0")
    # a share per 32 tokens of a huge bound: more partial results than the buffer holds
    params = binding.make_params(dev["q"], dev["k"], dev["v"], 1 << 22, w.scale, 0, None, 32, 0)
    with pytest.raises(binding.GqaError) as e:
        binding.gqa_decode_attn_static(params, dev["q"], dev["k"], dev["v"], dev["kv_lens"], None, out, None)
    assert e.value.status == binding.GQA_ERR_SCRATCH_LIMIT
    params = binding.make_params(dev["q"], dev["k"], dev["v"], 64, w.scale, 0, None, 0, 0)
    rc = binding._lib.gqa_decode_attn_static(ctypes.byref(params), None, dev["k"].data_ptr(), dev["v"].data_ptr(),
                                             dev["kv_lens"].data_ptr(), None, out.data_ptr(), None, None)
    assert rc == binding.GQA_ERR_INVALID_ARG
    torch.cuda.synchronize()
