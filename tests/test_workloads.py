"""The seeded input generators: bf16 rounding (both code paths of f32_to_bf16_bits give the same
bits, and those bits are round-to-nearest-even), determinism of the five named configurations and
the structure of a paged pool."""
from fractions import Fraction

import numpy as np
import pytest

from paper_2510_07356_amd import workloads as wl


def _numpy_path(x):
    """The integer-arithmetic path of f32_to_bf16_bits, taken whatever the array size."""
    x = np.asarray(x, dtype=np.float32)
    out = np.empty(x.shape, dtype=np.uint16).reshape(-1)
    flat = x.reshape(-1)
    step = (1 << 16) - 1                       # below the size at which the other path takes over
    for i in range(0, flat.size, step):
        out[i:i + step] = wl.f32_to_bf16_bits(flat[i:i + step])
    return out.reshape(x.shape)


def _interesting_values():
    rng = np.random.default_rng(5)
    normals = rng.standard_normal(1 << 17).astype(np.float32)
    # every kind of tie and near-tie: bf16 value + (0, just below half, half, just above half) of a step,
    # over many exponents, both signs; sub-normal floats; the largest finite values
    hi = rng.integers(0, 0x7F7F, size=1 << 15).astype(np.uint32) << 16
    lows = np.array([0x0000, 0x7FFF, 0x8000, 0x8001, 0xFFFF, 0x0001], dtype=np.uint32)
    ties = (hi[:, None] | lows[None, :]).reshape(-1)
    ties = np.concatenate([ties, ties | np.uint32(0x80000000)])
    special = np.array([0x00000000, 0x80000000, 0x00000001, 0x00008000, 0x00018000, 0x007FFFFF,
                        0x7F7F0000, 0x7F7F7FFF], dtype=np.uint32)
    return np.concatenate([normals, ties.view(np.float32), special.view(np.float32)])


def test_torch_and_numpy_rounding_paths_agree_bit_for_bit():
    pytest.importorskip("torch")
    x = _interesting_values()
    assert x.size >= 1 << 16                    # large enough for the fused path
    fused = wl.f32_to_bf16_bits(x)
    plain = _numpy_path(x)
    np.testing.assert_array_equal(fused, plain)


def test_rounding_is_nearest_even_in_exact_arithmetic():
    x = _interesting_values()
    rng = np.random.default_rng(6)
    pick = np.concatenate([rng.integers(0, x.size, size=3000), np.arange(x.size - 8, x.size)])
    got = _numpy_path(x[pick])
    back = wl.bf16_bits_to_f32(got)
    for xv, gb, bv in zip(x[pick], got, back):
        if not np.isfinite(bv):                 # rounded up past the largest finite bf16
            assert abs(Fraction(float(xv))) >= Fraction(2) ** 128 - Fraction(2) ** 119
            continue
        exact, mine = Fraction(float(xv)), Fraction(float(bv))
        lo = wl.bf16_bits_to_f32(np.uint16(gb - 1 if (gb & 0x7FFF) else gb))
        hi = wl.bf16_bits_to_f32(np.uint16(gb + 1))
        for other in (lo, hi):                  # no neighbour is closer; on a tie the even pattern wins
            if np.isfinite(other) and float(other) != float(bv):
                d_other, d_mine = abs(Fraction(float(other)) - exact), abs(mine - exact)
                assert d_mine < d_other or (d_mine == d_other and gb % 2 == 0), (xv, hex(gb))


def test_named_configurations_are_reproducible_and_shaped_as_stated():
    a, b = wl.make_config(0), wl.make_config(0)
    for name in ("q", "k", "v", "kv_lens"):
        np.testing.assert_array_equal(getattr(a, name), getattr(b, name))
    assert (a.batch, a.num_q_heads, a.num_kv_heads, a.head_dim, int(a.kv_lens[0])) == (1, 40, 8, 128, 512)
    assert a.kv_bytes == 2_097_152
    assert np.float32(a.scale) == np.float32(1.0 / np.sqrt(128.0))


def test_paged_pool_is_a_permutation_and_padding_is_poison():
    lens = [17, 16, 1, 40, 0]
    p = wl.make_paged("pool", 9, 5, 8, 2, lens, head_dim=8, page_size=16)
    used = [p.block_table[b, : -(-L // 16)] for b, L in enumerate(lens)]
    flat = np.concatenate(used)
    assert len(set(flat.tolist())) == len(flat) and flat.min() >= 0 and flat.max() < p.k.shape[0]
    for b, L in enumerate(lens):
        assert np.all(p.block_table[b, -(-L // 16):] == -1)
        if L % 16:
            blk = p.block_table[b, L // 16]
            assert np.all(p.k[blk, :, L % 16:] == wl.BF16_POISON) and np.all(p.v[blk, :, L % 16:] == wl.BF16_POISON)
