"""GPU parity of the KV-append + rotary step against the oracle: bit for bit (the rotation is
evaluated in fp64 on both sides and rounded once), then one whole decode step (append, attention)."""
import numpy as np
import pytest

from oracle import decode_attn, kv_append
from paper_2510_07356_amd import workloads as wl

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def binding():
    from paper_2510_07356_amd import binding as b
    return b


def rope_table(positions, D=128, theta=1.0e6):
    d = np.arange(D // 2, dtype=np.float64)
    ang = np.arange(positions, dtype=np.float64)[:, None] * theta ** (-2.0 * d / D)[None, :]
    return np.concatenate([np.cos(ang), np.sin(ang)], axis=1).astype(np.float32)


def new_rows(seed, B, Hkv, D=128):
    rng = np.random.default_rng(seed)
    return (wl.f32_to_bf16_bits(rng.standard_normal((B, Hkv, D)).astype(np.float32)),
            wl.f32_to_bf16_bits(rng.standard_normal((B, Hkv, D)).astype(np.float32)))


def to_bits(t):
    import torch
    return t.contiguous().view(torch.int16).cpu().numpy().view(np.uint16)


def run_append(binding, w, k_new, v_new, table):
    import torch
    dev = binding.to_device(w)
    q_out = torch.empty_like(dev["q"])
    kn = binding._bf16_view(k_new).to("cuda:0")
    vn = binding._bf16_view(v_new).to("cuda:0")
    cs = torch.from_numpy(table).to("cuda:0") if table is not None else None
    binding.gqa_decode_kv_append(dev["q"], q_out, kn, vn, dev["k"], dev["v"], dev["kv_lens"], w.max_kv_len,
                                 dev["block_table"], w.page_size, cs)
    torch.cuda.synchronize()
    return dev, q_out


@pytest.mark.parametrize("rotary", [False, True])
@pytest.mark.parametrize("layout", ["head_major", "token_major"])
@pytest.mark.parametrize("paged", [False, True])
def test_append_is_bit_exact(binding, rotary, layout, paged):
    import torch
    lens = [1, 17, 0, 300, 64, 1000]
    if paged:
        w = wl.make_paged("app_paged", 200, 6, 40, 8, lens, table_width=64, layout=layout)
    else:
        w = wl.make_contiguous("app", 200, 6, 40, 8, lens, cache_len=1000, layout=layout)
    k_new, v_new = new_rows(201, 6, 8)
    table = rope_table(1000) if rotary else None
    dev, q_out = run_append(binding, w, k_new, v_new, table)
    q_ref = kv_append(w.q, k_new, v_new, w.k, w.v, w.kv_lens, cos_sin=table,
                      block_table=w.block_table, page_size=w.page_size)      # updates w.k / w.v in place
    np.testing.assert_array_equal(to_bits(q_out), q_ref)
    # compare the caches through their logical index (strides may differ between host and device)
    got_k = to_bits(dev["k"]); got_v = to_bits(dev["v"])
    np.testing.assert_array_equal(got_k, np.ascontiguousarray(w.k))
    np.testing.assert_array_equal(got_v, np.ascontiguousarray(w.v))
    if rotary:
        assert not np.array_equal(q_ref[3], w.q[3])
    del torch


def test_append_in_place_query(binding):
    import torch
    w = wl.make_contiguous("app_inplace", 202, 3, 40, 8, [5, 900, 33], cache_len=900)
    k_new, v_new = new_rows(203, 3, 8)
    table = rope_table(900)
    dev = binding.to_device(w)
    kn = binding._bf16_view(k_new).to("cuda:0")
    vn = binding._bf16_view(v_new).to("cuda:0")
    binding.gqa_decode_kv_append(dev["q"], dev["q"], kn, vn, dev["k"], dev["v"], dev["kv_lens"], 900,
                                 None, 0, torch.from_numpy(table).to("cuda:0"))
    q_ref = kv_append(w.q, k_new, v_new, w.k, w.v, w.kv_lens, cos_sin=table)
    np.testing.assert_array_equal(to_bits(dev["q"]), q_ref)


@pytest.mark.parametrize("paged", [False, True])
def test_one_decode_step_append_then_attend(binding, paged):
    """The new token's K/V are appended (with rotary) and attention runs over the grown cache."""
    import torch
    lens = [700, 33, 1, 2048]
    if paged:
        w = wl.make_paged("step_paged", 204, 4, 40, 8, lens, table_width=128)
    else:
        w = wl.make_contiguous("step", 204, 4, 40, 8, lens, cache_len=2048)
    k_new, v_new = new_rows(205, 4, 8)
    table = rope_table(2048)
    dev, q_out = run_append(binding, w, k_new, v_new, table)
    dev["q"] = q_out
    out, lse = binding.run_workload(w, dev=dev)
    q_ref = kv_append(w.q, k_new, v_new, w.k, w.v, w.kv_lens, cos_sin=table,
                      block_table=w.block_table, page_size=w.page_size)
    ref = decode_attn(q_ref, w.k, w.v, w.kv_lens, w.scale, block_table=w.block_table, page_size=w.page_size)
    err = out.double().cpu().numpy() - ref.out
    assert np.isfinite(err).all()
    assert np.abs(err).max() <= 1e-2 and np.linalg.norm(err) / np.linalg.norm(ref.out) <= 5e-3
    assert np.abs(lse.double().cpu().numpy() - ref.lse).max() <= 4e-3
    del torch


def test_append_rounding_over_the_whole_bf16_range(binding):
    """Operands and table entries whose rotated results land below the normal bf16 range (sub-normal
    grid, signed zeros), on ties, beyond the largest finite value, and on NaN: the kernel's bits must
    equal the oracle's for every element."""
    import torch
    B, Hq, Hkv, D = 6, 8, 8, 128
    rng = np.random.default_rng(230)

    def spread(shape):
        # bf16 bit patterns with exponents over the whole range, both signs; a few special values
        bits = rng.integers(0, 0x7F80, size=shape).astype(np.uint16) | (rng.integers(0, 2, size=shape).astype(np.uint16) << 15)
        flat = bits.reshape(-1)
        flat[::97] = 0x0080            # smallest normal
        flat[1::97] = 0x8000           # -0
        flat[2::97] = 0x7F7F           # largest finite
        flat[3::211] = 0x7F80          # +inf
        flat[4::211] = 0x7FC1          # NaN
        return bits

    lens = [1, 2, 3, 4, 5, 6]
    w = wl.make_contiguous("app_range", 231, B, Hq, Hkv, lens, cache_len=8)
    w.q = spread((B, Hq, D))
    k_new, v_new = spread((B, Hkv, D)), spread((B, Hkv, D))
    # pairs whose difference cancels into lower binades: second half equal to the first up to a few ulps
    k_new[:, :, D // 2:] = k_new[:, :, :D // 2] ^ rng.integers(0, 4, size=(B, Hkv, D // 2)).astype(np.uint16)
    table = rng.uniform(-1, 1, size=(8, D)).astype(np.float32)
    table[0, :D // 2] = (rng.integers(0, 257, size=D // 2) / 256.0).astype(np.float32)      # dyadic: ties on the 2^-133 grid
    table[0, D // 2:] = 0.0
    table[1] = 1.0                                                                           # x - y, y + x
    table[2, :D // 2] = (2.0 ** -rng.integers(0, 140, size=D // 2).astype(np.float64)).astype(np.float32)   # down to fp32 sub-normals
    dev, q_out = run_append(binding, w, k_new, v_new, table)
    q_ref = kv_append(w.q, k_new, v_new, w.k, w.v, w.kv_lens, cos_sin=table)
    got_q = to_bits(q_out)
    np.testing.assert_array_equal(got_q, q_ref)
    np.testing.assert_array_equal(to_bits(dev["k"]), np.ascontiguousarray(w.k))
    np.testing.assert_array_equal(to_bits(dev["v"]), np.ascontiguousarray(w.v))
    mag = q_ref & 0x7FFF
    assert ((mag > 0) & (mag < 0x0080)).sum() > 20, "the case must reach the sub-normal grid"
    assert (mag == 0).any() and (mag == 0x7F80).any() and (q_ref == 0x7FC0).any()
    del torch
