"""Pins for the fp64 oracle: nothing here re-uses the oracle's own code.

Each test fixes the oracle to something the definition of softmax attention
(or plain mathematics) determines on its own: brute force in pure Python on
tiny inputs, closed forms, a hand-derived worked example, invariants, and a
float64 library routine as a third opinion.  The set is chosen so that a
dropped term, a wrong sign, a wrong head/group index, a transposed operand or
a wrong stride/page computation fails at least one of them.
"""
import math
import os

import numpy as np
import pytest

from oracle import decode_attn
from paper_2510_07356_amd.workloads import (BF16_POISON, bf16_bits_to_f32, f32_to_bf16_bits,
                                           make_contiguous, make_paged)

GOLDEN = os.path.join(os.path.dirname(__file__), "golden")


def bits(x):
    """Values that are exactly representable in bf16 -> bit patterns (checked)."""
    x = np.asarray(x, dtype=np.float32)
    b = f32_to_bf16_bits(x)
    assert np.array_equal(bf16_bits_to_f32(b), x), "test value not representable in bf16"
    return b


def small_ints(rng, shape, lo=-4, hi=4, step=0.25):
    """Random multiples of `step`: exact in bf16, exact products and short sums in fp64."""
    n = int(round((hi - lo) / step))
    return (rng.integers(0, n + 1, size=shape) * step + lo).astype(np.float32)


def brute_force(q, k, v, lens, scale, group):
    """Pure-Python softmax attention: exp(s)/sum exp(s) with no maximum
    subtracted, exactly rounded sums (math.fsum).  q [B][Hq][D]; k, v
    [B][Hkv][T][D] as nested lists of Python floats."""
    out, lse, wts = [], [], []
    for b in range(len(q)):
        ob, lb, wb = [], [], []
        for h in range(len(q[b])):
            g = h // group
            s = [scale * math.fsum(q[b][h][d] * k[b][g][j][d] for d in range(len(q[b][h])))
                 for j in range(lens[b])]
            e = [math.exp(x) for x in s]
            z = math.fsum(e)
            w = [x / z for x in e]
            ob.append([math.fsum(w[j] * v[b][g][j][d] for j in range(lens[b]))
                       for d in range(len(q[b][h]))])
            lb.append(math.log(z))
            wb.append(w)
        out.append(ob), lse.append(lb), wts.append(wb)
    return out, lse, wts


# --------------------------------------------------------------------------- brute force

@pytest.mark.parametrize("seed,B,Hq,Hkv,D,lens", [
    (0, 1, 1, 1, 1, [1]),
    (1, 2, 4, 2, 4, [5, 3]),
    (2, 2, 6, 2, 3, [1, 4]),
    (3, 3, 4, 4, 2, [2, 5, 1]),
    (4, 1, 8, 2, 8, [7]),
])
@pytest.mark.parametrize("layout", ["head_major", "token_major"])
def test_brute_force_contiguous(seed, B, Hq, Hkv, D, lens, layout):
    rng = np.random.default_rng(seed)
    T = max(lens) + 2                      # cache longer than any sequence; tail is poison
    q = small_ints(rng, (B, Hq, D), -2, 2)
    k = small_ints(rng, (B, Hkv, T, D), -2, 2)
    v = small_ints(rng, (B, Hkv, T, D))
    scale = 0.375
    kb, vb = bits(k), bits(v)
    for b, L in enumerate(lens):
        kb[b, :, L:, :] = BF16_POISON
        vb[b, :, L:, :] = BF16_POISON
    if layout == "token_major":
        kb = np.ascontiguousarray(kb.transpose(0, 2, 1, 3)).transpose(0, 2, 1, 3)
        vb = np.ascontiguousarray(vb.transpose(0, 2, 1, 3)).transpose(0, 2, 1, 3)
    res = decode_attn(bits(q), kb, vb, np.array(lens), scale, want_weights=True)
    ref_o, ref_l, ref_w = brute_force(q.tolist(), k.tolist(), v.tolist(), lens, scale, Hq // Hkv)
    np.testing.assert_allclose(res.out, np.array(ref_o), rtol=0, atol=2e-14)
    np.testing.assert_allclose(res.lse, np.array(ref_l), rtol=0, atol=2e-14)
    for b, L in enumerate(lens):
        np.testing.assert_allclose(res.weights[b, :, :L], np.array(ref_w[b]), rtol=0, atol=1e-15)


@pytest.mark.parametrize("layout", ["head_major", "token_major"])
@pytest.mark.parametrize("page", [2, 4])
def test_brute_force_paged(layout, page):
    rng = np.random.default_rng(11)
    B, Hq, Hkv, D = 3, 4, 2, 4
    lens = [5, 1, 8]
    nblk = [-(-L // page) for L in lens]
    total = sum(nblk)
    perm = rng.permutation(total + 2)[:total]
    pool_k = np.full((total + 2, Hkv, page, D), BF16_POISON, dtype=np.uint16)
    pool_v = pool_k.copy()
    table = np.full((B, max(nblk) + 1), -1, dtype=np.int32)
    q = small_ints(rng, (B, Hq, D), -2, 2)
    k_log = small_ints(rng, (B, Hkv, max(lens), D), -2, 2)
    v_log = small_ints(rng, (B, Hkv, max(lens), D))
    off = 0
    for b, L in enumerate(lens):
        for i in range(nblk[b]):
            blk = perm[off + i]
            table[b, i] = blk
            for s in range(page):
                j = i * page + s
                if j < L:
                    pool_k[blk, :, s, :] = bits(k_log[b, :, j, :])
                    pool_v[blk, :, s, :] = bits(v_log[b, :, j, :])
        off += nblk[b]
    if layout == "token_major":
        pool_k = np.ascontiguousarray(pool_k.transpose(0, 2, 1, 3)).transpose(0, 2, 1, 3)
        pool_v = np.ascontiguousarray(pool_v.transpose(0, 2, 1, 3)).transpose(0, 2, 1, 3)
    res = decode_attn(bits(q), pool_k, pool_v, np.array(lens), 0.5, block_table=table, page_size=page)
    ref_o, ref_l, _ = brute_force(q.tolist(), k_log.tolist(), v_log.tolist(), lens, 0.5, Hq // Hkv)
    np.testing.assert_allclose(res.out, np.array(ref_o), rtol=0, atol=2e-14)
    np.testing.assert_allclose(res.lse, np.array(ref_l), rtol=0, atol=2e-14)


# --------------------------------------------------------------------------- worked example, closed forms

def test_golden_three_keys():
    rows = {}
    with open(os.path.join(GOLDEN, "three_keys_ln2.txt")) as f:
        for line in f:
            if line.startswith("#") or not line.strip():
                continue
            key, *vals = line.split()
            rows[key] = np.array([float(x) for x in vals])
    q = bits(rows["q"].reshape(1, 1, 2))
    k = bits(rows["k"].reshape(1, 1, 3, 2))
    v = bits(rows["v"].reshape(1, 1, 3, 2))
    res = decode_attn(q, k, v, np.array([3]), math.log(2.0), want_weights=True)
    np.testing.assert_allclose(res.weights[0, 0], rows["weights"], rtol=0, atol=1e-15)
    np.testing.assert_allclose(res.out[0, 0], rows["out"], rtol=0, atol=1e-15)
    np.testing.assert_allclose(res.lse[0, 0], rows["lse"][0], rtol=0, atol=1e-15)


def test_single_key_returns_its_value_row():
    rng = np.random.default_rng(5)
    w = make_contiguous("one", 5, 3, 4, 2, [1, 1, 1], head_dim=8)
    res = decode_attn(w.q, w.k, w.v, w.kv_lens, w.scale, want_weights=True)
    vf = bf16_bits_to_f32(w.v).astype(np.float64)
    for h in range(4):
        np.testing.assert_array_equal(res.out[:, h, :], vf[:, h // 2, 0, :])
    np.testing.assert_array_equal(res.weights[..., 0], 1.0)
    # LSE of a single key is its scaled score
    qf, kf = bf16_bits_to_f32(w.q).astype(np.float64), bf16_bits_to_f32(w.k).astype(np.float64)
    for b in range(3):
        for h in range(4):
            s = w.scale * math.fsum(qf[b, h] * kf[b, h // 2, 0])
            assert abs(res.lse[b, h] - s) < 1e-14
    del rng


def test_scale_zero_gives_mean_of_values():
    w = make_contiguous("mean", 6, 2, 6, 3, [9, 4], head_dim=16)
    res = decode_attn(w.q, w.k, w.v, w.kv_lens, 0.0, want_weights=True)
    vf = bf16_bits_to_f32(w.v).astype(np.float64)
    for b, L in enumerate([9, 4]):
        for h in range(6):
            np.testing.assert_allclose(res.out[b, h], vf[b, h // 2, :L].mean(axis=0), atol=1e-15)
            np.testing.assert_allclose(res.weights[b, h, :L], 1.0 / L, atol=1e-16)
            assert abs(res.lse[b, h] - math.log(L)) < 1e-15


def test_two_keys_log3_gives_quarter_and_three_quarters():
    q, k = bits([[[1.0]]]), bits([[[[0.0], [1.0]]]])
    v = bits([[[[8.0], [-8.0]]]])
    res = decode_attn(q, k, v, np.array([2]), math.log(3.0), want_weights=True)
    np.testing.assert_allclose(res.weights[0, 0], [0.25, 0.75], atol=1e-16)
    assert abs(res.out[0, 0, 0] - (-4.0)) < 1e-15
    assert abs(res.lse[0, 0] - math.log(4.0)) < 1e-15


def test_sign_of_scores():
    """A key aligned with q must outweigh a key opposed to it (a flipped sign
    in the exponent or in the dot product reverses this)."""
    q = bits([[[2.0, 0.0]]])
    k = bits([[[[1.0, 0.0], [-1.0, 0.0]]]])
    v = bits([[[[1.0, 0.0], [0.0, 1.0]]]])
    res = decode_attn(q, k, v, np.array([2]), 1.0)
    e = math.exp(4.0)
    np.testing.assert_allclose(res.out[0, 0], [e / (1 + e), 1 / (1 + e)], atol=1e-15)


def test_empty_sequence_is_zero_row_and_minus_inf():
    w = make_contiguous("empty", 7, 3, 4, 2, [0, 3, 0], head_dim=8, cache_len=4)
    res = decode_attn(w.q, w.k, w.v, w.kv_lens, w.scale)
    assert np.all(res.out[[0, 2]] == 0.0) and np.all(np.isneginf(res.lse[[0, 2]]))
    assert np.all(np.isfinite(res.out[1])) and np.all(np.isfinite(res.lse[1]))


# --------------------------------------------------------------------------- invariants

def _case(seed=21, B=3, Hq=10, Hkv=2, D=16, lens=(37, 1, 64), **kw):
    return make_contiguous("inv", seed, B, Hq, Hkv, list(lens), head_dim=D, **kw)


def test_weights_sum_to_one_and_are_positive():
    w = _case()
    res = decode_attn(w.q, w.k, w.v, w.kv_lens, w.scale, want_weights=True)
    for b, L in enumerate(w.kv_lens):
        assert np.all(res.weights[b, :, :L] > 0.0)
        np.testing.assert_allclose(res.weights[b, :, :L].sum(axis=-1), 1.0, atol=1e-14)
        assert np.all(res.weights[b, :, L:] == 0.0)


def test_identical_keys_give_mean_of_values():
    w = _case()
    k = w.k.copy()
    k[:, :, :, :] = k[:, :, :1, :]
    res = decode_attn(w.q, k, w.v, w.kv_lens, w.scale)
    vf = bf16_bits_to_f32(w.v).astype(np.float64)
    for b, L in enumerate(w.kv_lens):
        for h in range(w.num_q_heads):
            np.testing.assert_allclose(res.out[b, h], vf[b, h // 5, :L].mean(axis=0), atol=1e-14)


def test_single_dominant_key_returns_its_value_row():
    w = _case(scale=1.0)
    D = w.head_dim
    q = bits(np.full((3, 10, D), 2.0))
    k = bits(np.zeros((3, 2, 64, D)))
    hot = [17, 0, 63]
    for b, j in enumerate(hot):
        k[b, :, j, :] = bits(np.full(D, 2.0))          # score 4*D = 64 above all others (0)
    res = decode_attn(q, k, w.v, w.kv_lens, 1.0)
    vf = bf16_bits_to_f32(w.v).astype(np.float64)
    for b, j in enumerate(hot):
        for h in range(10):
            np.testing.assert_allclose(res.out[b, h], vf[b, h // 5, j], rtol=0, atol=1e-15 * 64)


def test_permuting_kv_order_changes_nothing():
    w = _case()
    rng = np.random.default_rng(3)
    k, v = w.k.copy(), w.v.copy()
    for b, L in enumerate(w.kv_lens):
        p = rng.permutation(L)
        k[b, :, :L] = w.k[b][:, p]
        v[b, :, :L] = w.v[b][:, p]
    a = decode_attn(w.q, w.k, w.v, w.kv_lens, w.scale)
    c = decode_attn(w.q, k, v, w.kv_lens, w.scale)
    np.testing.assert_allclose(a.out, c.out, rtol=0, atol=1e-14)
    np.testing.assert_allclose(a.lse, c.lse, rtol=0, atol=1e-14)


def test_gqa_equals_mha_with_repeated_kv_heads():
    w = _case()
    G = w.num_q_heads // w.num_kv_heads
    a = decode_attn(w.q, w.k, w.v, w.kv_lens, w.scale)
    c = decode_attn(w.q, np.repeat(w.k, G, axis=1), np.repeat(w.v, G, axis=1), w.kv_lens, w.scale)
    np.testing.assert_array_equal(a.out, c.out)
    # the interleaved map h % Hkv would give something else:
    kk = np.tile(w.k, (1, G, 1, 1))
    d = decode_attn(w.q, kk, np.tile(w.v, (1, G, 1, 1)), w.kv_lens, w.scale)
    assert np.abs(a.out - d.out).max() > 1e-3


def test_identical_queries_in_a_group_give_identical_rows():
    w = _case()
    q = w.q.copy()
    q[:, 0:5] = q[:, 0:1]
    res = decode_attn(q, w.k, w.v, w.kv_lens, w.scale)
    for h in range(1, 5):
        np.testing.assert_array_equal(res.out[:, h], res.out[:, 0])
    assert np.abs(res.out[:, 5] - res.out[:, 0]).max() > 1e-3      # other group: other keys


def test_output_lies_in_convex_hull_of_values():
    w = _case()
    res = decode_attn(w.q, w.k, w.v, w.kv_lens, w.scale)
    vf = bf16_bits_to_f32(w.v).astype(np.float64)
    for b, L in enumerate(w.kv_lens):
        for h in range(w.num_q_heads):
            lo, hi = vf[b, h // 5, :L].min(axis=0), vf[b, h // 5, :L].max(axis=0)
            assert np.all(res.out[b, h] >= lo - 1e-14) and np.all(res.out[b, h] <= hi + 1e-14)


def test_padding_is_never_read():
    w = _case(cache_len=80)
    a = decode_attn(w.q, w.k, w.v, w.kv_lens, w.scale)
    assert np.all(np.isfinite(a.out)) and np.all(np.isfinite(a.lse))
    k2 = w.k.copy()
    for b, L in enumerate(w.kv_lens):
        k2[b, :, L:] = 0
    c = decode_attn(w.q, k2, w.v, w.kv_lens, w.scale)
    np.testing.assert_array_equal(a.out, c.out)


def test_paged_equals_contiguous_for_any_block_order():
    lens = [37, 16, 1, 50]
    c = make_contiguous("c", 31, 4, 8, 2, lens, head_dim=16)
    ref = decode_attn(c.q, c.k, c.v, c.kv_lens, c.scale)
    for permute in (False, True):
        for layout in ("head_major", "token_major"):
            p = make_paged("p", 31, 4, 8, 2, lens, head_dim=16, permute=permute, layout=layout)
            got = decode_attn(p.q, p.k, p.v, p.kv_lens, p.scale, block_table=p.block_table,
                              page_size=p.page_size)
            np.testing.assert_array_equal(ref.out, got.out)
            np.testing.assert_array_equal(ref.lse, got.lse)


def test_split_and_lse_merge_reproduces_one_shot():
    """Attention over [0, L) equals the log-sum-exp weighted merge of attention
    over [0, c) and [c, L): pins LSE (base e, of the scaled scores)."""
    w = _case(lens=(64, 33, 50))
    full = decode_attn(w.q, w.k, w.v, w.kv_lens, w.scale)
    for cut in (1, 16, 31):
        a = decode_attn(w.q, w.k[:, :, :cut], w.v[:, :, :cut], np.full(3, cut), w.scale)
        rest = w.kv_lens - cut
        c = decode_attn(w.q, w.k[:, :, cut:], w.v[:, :, cut:], rest, w.scale)
        big = np.maximum(a.lse, c.lse)
        wa, wc = np.exp(a.lse - big), np.exp(c.lse - big)
        merged = (wa[..., None] * a.out + wc[..., None] * c.out) / (wa + wc)[..., None]
        np.testing.assert_allclose(merged, full.out, rtol=0, atol=1e-14)
        np.testing.assert_allclose(big + np.log(wa + wc), full.lse, rtol=0, atol=1e-14)


def test_shift_of_all_scores_moves_lse_only():
    """Adding a constant c to every score (one extra q/k coordinate) leaves the
    output unchanged and moves LSE by exactly c."""
    w = _case(D=16, scale=0.5)
    q, k = w.q.copy(), w.k.copy()
    q[:, :, 0] = bits(np.float32(4.0))
    k[:, :, :, 0] = bits(np.float32(0.0))
    a = decode_attn(q, k, w.v, w.kv_lens, 0.5)
    k[:, :, :, 0] = bits(np.float32(1.5))            # every score grows by 0.5 * 4 * 1.5 = 3
    c = decode_attn(q, k, w.v, w.kv_lens, 0.5)
    np.testing.assert_allclose(a.out, c.out, rtol=0, atol=1e-13)
    np.testing.assert_allclose(c.lse - a.lse, 3.0, rtol=0, atol=1e-13)


# --------------------------------------------------------------------------- library third opinion

@pytest.mark.parametrize("layout", ["head_major", "token_major"])
def test_matches_float64_library_softmax(layout):
    torch = pytest.importorskip("torch")
    w = make_contiguous("lib", 41, 2, 10, 2, [300, 129], head_dim=128, layout=layout)
    res = decode_attn(w.q, w.k, w.v, w.kv_lens, w.scale)
    qf = torch.from_numpy(bf16_bits_to_f32(w.q).astype(np.float64))
    kf = torch.from_numpy(bf16_bits_to_f32(np.ascontiguousarray(w.k)).astype(np.float64))
    vf = torch.from_numpy(bf16_bits_to_f32(np.ascontiguousarray(w.v)).astype(np.float64))
    for b, L in enumerate(w.kv_lens):
        kk = kf[b, :, :L].repeat_interleave(5, dim=0)           # [Hq, L, D]
        vv = vf[b, :, :L].repeat_interleave(5, dim=0)
        s = torch.einsum("hd,hjd->hj", qf[b], kk) * w.scale
        o = torch.einsum("hj,hjd->hd", torch.softmax(s, dim=-1), vv)
        np.testing.assert_allclose(res.out[b], o.numpy(), rtol=0, atol=1e-13)
        np.testing.assert_allclose(res.lse[b], torch.logsumexp(s, dim=-1).numpy(), rtol=0, atol=1e-12)


def test_thread_count_does_not_change_the_result():
    w = _case()
    a = decode_attn(w.q, w.k, w.v, w.kv_lens, w.scale, threads=1)
    c = decode_attn(w.q, w.k, w.v, w.kv_lens, w.scale, threads=4)
    np.testing.assert_array_equal(a.out, c.out)
    assert a.threads == 1 and 1 <= c.threads <= 4


# --------------------------------------------------------------------------- append + rotary oracle

from oracle import kv_append  # noqa: E402


def rope_table(positions, D, theta=1.0e6):
    """cos/sin of pos * theta^(-2d/D), d < D/2, computed in float64 and stored as fp32 [positions, D]."""
    d = np.arange(D // 2, dtype=np.float64)
    ang = np.arange(positions, dtype=np.float64)[:, None] * theta ** (-2.0 * d / D)[None, :]
    return np.concatenate([np.cos(ang), np.sin(ang)], axis=1).astype(np.float32)


def test_append_without_rotary_is_a_bit_exact_scatter():
    w = make_contiguous("app", 51, 3, 8, 2, [5, 0, 9], head_dim=8, cache_len=10)
    rng = np.random.default_rng(1)
    k_new = f32_to_bf16_bits(rng.standard_normal((3, 2, 8)).astype(np.float32))
    v_new = f32_to_bf16_bits(rng.standard_normal((3, 2, 8)).astype(np.float32))
    for layout in ("head_major", "token_major"):
        k, v = w.k.copy(), w.v.copy()
        if layout == "token_major":
            k = np.ascontiguousarray(k.transpose(0, 2, 1, 3)).transpose(0, 2, 1, 3)
            v = np.ascontiguousarray(v.transpose(0, 2, 1, 3)).transpose(0, 2, 1, 3)
        k0, v0 = k.copy(), v.copy()
        q_out = kv_append(w.q, k_new, v_new, k, v, w.kv_lens)
        np.testing.assert_array_equal(q_out, w.q)
        for b, L in enumerate(w.kv_lens):
            if L > 0:
                np.testing.assert_array_equal(k[b, :, L - 1], k_new[b])
                np.testing.assert_array_equal(v[b, :, L - 1], v_new[b])
                k0[b, :, L - 1] = k_new[b]
                v0[b, :, L - 1] = v_new[b]
        np.testing.assert_array_equal(k, k0)          # nothing else was touched (empty sequence included)
        np.testing.assert_array_equal(v, v0)


def test_append_paged_lands_in_the_block_the_table_names():
    lens = [17, 16, 1, 40]
    p = make_paged("app_p", 52, 4, 8, 2, lens, head_dim=8, page_size=16)
    rng = np.random.default_rng(2)
    k_new = f32_to_bf16_bits(rng.standard_normal((4, 2, 8)).astype(np.float32))
    v_new = f32_to_bf16_bits(rng.standard_normal((4, 2, 8)).astype(np.float32))
    k0, v0 = p.k.copy(), p.v.copy()
    kv_append(p.q, k_new, v_new, p.k, p.v, p.kv_lens, block_table=p.block_table, page_size=16)
    for b, L in enumerate(lens):
        blk, slot = p.block_table[b, (L - 1) // 16], (L - 1) % 16
        k0[blk, :, slot] = k_new[b]
        v0[blk, :, slot] = v_new[b]
    np.testing.assert_array_equal(p.k, k0)
    np.testing.assert_array_equal(p.v, v0)


def test_rotary_identity_and_quarter_turn():
    """cos=1, sin=0 leaves q and k unchanged; cos=0, sin=1 maps (x, y) -> (-y, x) for the pair
    (d, d + D/2): pins the pairing and the sign of the rotation."""
    D = 8
    rng = np.random.default_rng(3)
    q = f32_to_bf16_bits(rng.standard_normal((2, 4, D)).astype(np.float32))
    k_new = f32_to_bf16_bits(rng.standard_normal((2, 2, D)).astype(np.float32))
    v_new = f32_to_bf16_bits(rng.standard_normal((2, 2, D)).astype(np.float32))
    lens = np.array([3, 1])
    ident = np.zeros((4, D), np.float32); ident[:, :D // 2] = 1.0
    kc = np.zeros((2, 2, 4, D), np.uint16); vc = kc.copy()
    np.testing.assert_array_equal(kv_append(q, k_new, v_new, kc, vc, lens, cos_sin=ident), q)
    np.testing.assert_array_equal(kc[0, :, 2], k_new[0])
    quarter = np.zeros((4, D), np.float32); quarter[:, D // 2:] = 1.0
    kc[:] = 0
    q_out = kv_append(q, k_new, v_new, kc, vc, lens, cos_sin=quarter)
    qf, of = bf16_bits_to_f32(q), bf16_bits_to_f32(q_out)
    np.testing.assert_array_equal(of[..., :D // 2], -qf[..., D // 2:])
    np.testing.assert_array_equal(of[..., D // 2:], qf[..., :D // 2])
    kf, ko = bf16_bits_to_f32(k_new[1]), bf16_bits_to_f32(kc[1, :, 0])
    np.testing.assert_array_equal(ko[..., :D // 2], -kf[..., D // 2:])
    np.testing.assert_array_equal(ko[..., D // 2:], kf[..., :D // 2])
    np.testing.assert_array_equal(vc[1, :, 0], v_new[1])            # V is never rotated


def test_rotary_exact_cases_match_rational_arithmetic():
    """Small integers and dyadic cos/sin: every result is exactly representable in bf16, so the
    oracle must return exactly x*c - y*s and y*c + x*s (the table row used is kv_len - 1)."""
    from fractions import Fraction
    D = 4
    rng = np.random.default_rng(4)
    q = rng.integers(-8, 9, size=(3, 2, D)).astype(np.float32)
    kn = rng.integers(-8, 9, size=(3, 1, D)).astype(np.float32)
    table = (rng.integers(-4, 5, size=(6, D)) * 0.25).astype(np.float32)
    lens = np.array([6, 2, 4])
    kc = np.zeros((3, 1, 6, D), np.uint16); vc = kc.copy()
    q_out = bf16_bits_to_f32(kv_append(bits(q), bits(kn), bits(kn), kc, vc, lens, cos_sin=table))
    for b in range(3):
        pos = lens[b] - 1
        for src, got in ((q[b], q_out[b]), (kn[b], bf16_bits_to_f32(kc[b, :, pos]))):
            for h in range(src.shape[0]):
                for d in range(D // 2):
                    c, s = Fraction(float(table[pos, d])), Fraction(float(table[pos, D // 2 + d]))
                    x, y = Fraction(float(src[h, d])), Fraction(float(src[h, d + D // 2]))
                    assert Fraction(float(got[h, d])) == x * c - y * s
                    assert Fraction(float(got[h, d + D // 2])) == y * c + x * s


def test_rotary_rounds_to_nearest_even_bf16():
    D = 2
    table = np.array([[1.0, 1.0]], np.float32)                     # cos = 1, sin = 1: x' = x - y
    kc = np.zeros((1, 1, 1, D), np.uint16); vc = kc.copy()
    cases = [(0x3F80, 2.0 ** -8, 0x3F80),      # 1 + 2^-8: tie between 0x3F80 and 0x3F81 -> even 0x3F80
             (0x3F81, 2.0 ** -8, 0x3F82),      # 1 + 3*2^-8: tie between 0x3F81 and 0x3F82 -> even 0x3F82
             (0x3F80, 2.0 ** -9, 0x3F80),      # below the tie
             (0x3F80, 3 * 2.0 ** -9, 0x3F81)]  # above the tie
    for xbits, y, want in cases:
        q = np.array([[[xbits, int(bits(np.float32(-y)))]]], np.uint16)
        out = kv_append(q, q[:, :1], q[:, :1], kc, vc, np.array([1]), cos_sin=table)
        assert out[0, 0, 0] == want, (hex(xbits), y, hex(out[0, 0, 0]))


def test_rotary_scores_depend_on_relative_position_only():
    """<R_m q, R_n k> is a function of m - n: shifting both positions changes the dot product only
    by bf16 rounding.  A rotation in the wrong direction for one of the two breaks this."""
    D = 64
    table = rope_table(64, D, theta=100.0)
    rng = np.random.default_rng(6)
    q = f32_to_bf16_bits(rng.standard_normal((1, 1, D)).astype(np.float32))
    kn = f32_to_bf16_bits(rng.standard_normal((1, 1, D)).astype(np.float32))
    dots = []
    for shift in (0, 7, 30):
        kc = np.zeros((1, 1, 64, D), np.uint16); vc = kc.copy()
        kv_append(q, kn, kn, kc, vc, np.array([5 + shift]), cos_sin=table)       # key at position 4 + shift
        qr = kv_append(q, kn, kn, kc.copy(), vc, np.array([21 + shift]), cos_sin=table)   # query at 20 + shift
        dots.append(float(bf16_bits_to_f32(qr[0, 0]).astype(np.float64) @
                          bf16_bits_to_f32(kc[0, 0, 4 + shift]).astype(np.float64)))
    scale = float(np.linalg.norm(bf16_bits_to_f32(q)) * np.linalg.norm(bf16_bits_to_f32(kn)))
    assert max(dots) - min(dots) < 2.0 ** -7 * scale
    # and the rotation is not the identity: the unrotated dot product differs
    plain = float(bf16_bits_to_f32(q[0, 0]).astype(np.float64) @ bf16_bits_to_f32(kn[0, 0]).astype(np.float64))
    assert abs(plain - dots[0]) > 2.0 ** -7 * scale


def test_rotary_matches_float64_rotate_half_formula():
    torch = pytest.importorskip("torch")
    D = 128
    table = rope_table(300, D)
    rng = np.random.default_rng(7)
    q = f32_to_bf16_bits(rng.standard_normal((4, 6, D)).astype(np.float32))
    kn = f32_to_bf16_bits(rng.standard_normal((4, 2, D)).astype(np.float32))
    lens = np.array([300, 1, 77, 150])
    kc = np.zeros((4, 2, 300, D), np.uint16); vc = kc.copy()
    got = bf16_bits_to_f32(kv_append(q, kn, kn, kc, vc, lens, cos_sin=table)).astype(np.float64)
    x = torch.from_numpy(bf16_bits_to_f32(q).astype(np.float64))
    cos = torch.from_numpy(table[lens - 1, :D // 2].astype(np.float64)).repeat(1, 2)[:, None, :]
    sin = torch.from_numpy(table[lens - 1, D // 2:].astype(np.float64)).repeat(1, 2)[:, None, :]
    rot = torch.cat([-x[..., D // 2:], x[..., :D // 2]], dim=-1)
    want = (x * cos + rot * sin).numpy()
    # correct rounding to 8 significant bits: every element within half a bf16 step of the exact value
    assert np.all(np.abs(got - want) <= 2.0 ** -8 * np.abs(want) * (1 + 1e-12))
    assert np.abs(got - want).max() > 0.0


def _round_to_bf16_rational(value: float) -> int:
    """Independent nearest-even rounding of a double to a bf16 bit pattern in exact rational
    arithmetic: the bf16 grid around |value| has spacing 2^(max(e, -126) - 7) with
    2^e <= |value| < 2^(e+1); anything at or beyond 2^128 - 2^119 (half a step above the largest
    bf16) is infinity."""
    from fractions import Fraction
    import math
    if math.isnan(value):
        return 0x7FC0
    sign = 0x8000 if math.copysign(1.0, value) < 0 else 0
    if math.isinf(value):
        return sign | 0x7F80
    a = abs(Fraction(value))
    if a == 0:
        return sign
    e = a.numerator.bit_length() - a.denominator.bit_length()
    if Fraction(2) ** e > a:
        e -= 1
    assert Fraction(2) ** e <= a < Fraction(2) ** (e + 1)
    step = Fraction(2) ** (max(e, -126) - 7)
    n, rem = divmod(a, step)
    n = int(n)
    if rem * 2 > step or (rem * 2 == step and n % 2 == 1):
        n += 1
    # n * step on the bf16 grid: magnitude bits are n + 128 * (max(e, -126) + 126) once the hidden bit is
    # accounted for (sub-normal: n itself; normal: exponent field e + 127, mantissa n - 128)
    if e < -126:
        mag = n                       # n = 128 is the smallest normal number 0x0080
    else:
        mag = ((e + 127) << 7) + (n - 128)      # a mantissa carry (n = 256) rolls into the exponent
    return sign | (0x7F80 if mag >= 0x7F80 else mag)


def _rotate_one(xbits, ybits, c, s):
    """Oracle results (x', y') for one pair (x, y) rotated with cos = c, sin = s (fp32 values)."""
    D = 2
    table = np.array([[c, s]], np.float32)
    kc = np.zeros((1, 1, 1, D), np.uint16); vc = kc.copy()
    q = np.array([[[xbits, ybits]]], np.uint16)
    out = kv_append(q, q[:, :1], q[:, :1], kc, vc, np.array([1]), cos_sin=table)
    np.testing.assert_array_equal(kc[0, 0, 0], out[0, 0])            # the key takes the same path as the query
    return int(out[0, 0, 0]), int(out[0, 0, 1])


def test_rotary_rounding_below_the_normal_range():
    """bf16 results below 2^-126 sit on a grid of fixed spacing 2^-133 (sub-normal numbers) and
    are rounded to nearest even on THAT grid, not truncated.  x = 2^-126 (0x0080) times a
    dyadic cosine lands exactly where the case needs it."""
    tiny = 0x0080
    f = np.float32
    # half the smallest normal number is the sub-normal 64 * 2^-133
    assert _rotate_one(tiny, 0, f(0.5), f(0.0))[0] == 0x0040
    # exact sub-normals survive: k * 2^-133
    for kq in (1, 2, 3, 64, 127):
        assert _rotate_one(tiny, 0, f(kq / 128.0), f(0.0))[0] == kq
    # ties (k + 1/2) * 2^-133 go to the even neighbour
    assert _rotate_one(tiny, 0, f(0.5 / 128.0), f(0.0))[0] == 0x0000        # 0.5 -> 0
    assert _rotate_one(tiny, 0, f(1.5 / 128.0), f(0.0))[0] == 0x0002        # 1.5 -> 2
    assert _rotate_one(tiny, 0, f(2.5 / 128.0), f(0.0))[0] == 0x0002        # 2.5 -> 2
    assert _rotate_one(tiny, 0, f(126.5 / 128.0), f(0.0))[0] == 0x007E
    assert _rotate_one(tiny, 0, f(127.5 / 128.0), f(0.0))[0] == 0x0080      # up into the normal range
    # just off a tie: decided by the exact value (a truncating implementation gets these wrong)
    assert _rotate_one(tiny, 0, f(2.5 / 128.0 * (1 + 2.0 ** -20)), f(0.0))[0] == 0x0003
    assert _rotate_one(tiny, 0, f(1.5 / 128.0 * (1 - 2.0 ** -20)), f(0.0))[0] == 0x0001
    assert _rotate_one(tiny, 0, f(0.75 / 128.0), f(0.0))[0] == 0x0001
    # negative results keep their sign, also when they round to zero
    assert _rotate_one(tiny | 0x8000, 0, f(3 / 128.0), f(0.0))[0] == 0x8003
    assert _rotate_one(tiny | 0x8000, 0, f(0.25 / 128.0), f(0.0))[0] == 0x8000
    # y' = y cos + x sin takes the same path
    assert _rotate_one(tiny, 0, f(0.0), f(1.5 / 128.0))[1] == 0x0002


def test_rotary_rounding_of_zero_infinity_and_nan():
    f = np.float32
    one, big = 0x3F80, 0x7F7F                                  # 1.0, the largest finite bf16
    assert _rotate_one(0x0000, 0x0000, f(1.0), f(0.0)) == (0x0000, 0x0000)
    # (-0) * 1 - (+0) * 0 = -0; (+0) * 1 + (-0) * 0 = +0 (round-to-nearest sign rules of IEEE 754)
    assert _rotate_one(0x8000, 0x0000, f(1.0), f(0.0)) == (0x8000, 0x0000)
    # exact cancellation gives +0
    assert _rotate_one(one, one, f(1.0), f(1.0))[0] == 0x0000
    # overflow: big + big = 2^129 (1 - 2^-8) rounds to infinity; big * 1 stays finite
    assert _rotate_one(big, big | 0x8000, f(1.0), f(1.0))[0] == 0x7F80
    assert _rotate_one(big | 0x8000, big, f(1.0), f(1.0))[0] == 0xFF80
    assert _rotate_one(big, 0, f(1.0), f(0.0))[0] == big
    # big = 2^128 - 2^120, the grid step there is 2^120: big + 2^119 is a tie whose even neighbour is
    # 2^128 = infinity; big + 1.5 * 2^118 is below the tie and stays; big + 1.5 * 2^119 is above it
    assert _rotate_one(big, 0x7B00, f(1.0), f(-1.0))[0] == 0x7F80            # 0x7B00 = 2^119
    assert _rotate_one(big, 0x7AC0, f(1.0), f(-1.0))[0] == big               # 0x7AC0 = 1.5 * 2^118
    assert _rotate_one(big, 0x7B40, f(1.0), f(-1.0))[0] == 0x7F80            # 0x7B40 = 1.5 * 2^119
    # infinities pass through; inf * 0 and inf - inf are NaN, stored as the one quiet NaN 0x7FC0
    assert _rotate_one(0x7F80, 0, f(1.0), f(0.0)) == (0x7F80, 0x7FC0)       # x' = inf - 0, y' = 0 + inf * 0
    assert _rotate_one(0x7F80, 0, f(2.0), f(1.0)) == (0x7F80, 0x7F80)
    assert _rotate_one(0xFF80, 0, f(2.0), f(1.0)) == (0xFF80, 0xFF80)
    assert _rotate_one(0x7F80, 0x7F80, f(1.0), f(1.0))[0] == 0x7FC0
    assert _rotate_one(0x7FC1, 0, f(1.0), f(1.0)) == (0x7FC0, 0x7FC0)
    assert _rotate_one(0xFFFF, 0, f(1.0), f(1.0)) == (0x7FC0, 0x7FC0)


def test_rotary_rounding_matches_rational_rounding_over_the_whole_range():
    """Seeded sweep over magnitudes from far below the sub-normal range to overflow: the fp64
    expression x c - y s (Python floats are IEEE doubles and never contract) rounded to bf16 in
    exact rational arithmetic must equal the oracle's bits."""
    rng = np.random.default_rng(11)
    n = 4000
    # bf16 operands with exponents spread over the whole range, fp32 cos/sin in [-1, 1] and a few larger
    xb = rng.integers(0, 0x7F80, size=n).astype(np.uint16) | (rng.integers(0, 2, size=n).astype(np.uint16) << 15)
    yb = rng.integers(0, 0x7F80, size=n).astype(np.uint16) | (rng.integers(0, 2, size=n).astype(np.uint16) << 15)
    # half of the pairs: y close to x in magnitude so that the difference cancels into lower binades
    yb[: n // 2] = (xb[: n // 2] & 0x7FFF) ^ rng.integers(0, 8, size=n // 2).astype(np.uint16)
    c = rng.uniform(-1, 1, size=n).astype(np.float32)
    s = rng.uniform(-1, 1, size=n).astype(np.float32)
    c[::7] = np.float32(1.0); s[::7] = np.float32(1.0)
    c[::11] = (rng.integers(1, 256, size=len(c[::11])) / 128.0).astype(np.float32); s[::11] = 0
    D = 2
    q = np.stack([xb, yb], axis=-1)[:, None, :]                       # [n, 1, 2]
    table = np.zeros((n, D), np.float32)
    table[:, 0], table[:, 1] = c, s
    kc = np.zeros((n, 1, 1, D), np.uint16)
    out = np.empty((n, 2), np.uint16)
    for i in range(n):                                                 # one call per pair: position 0, own table row
        o = kv_append(q[i:i + 1], q[i:i + 1, :1], q[i:i + 1, :1], kc[i:i + 1], kc[i:i + 1].copy(),
                      np.array([1]), cos_sin=table[i:i + 1])
        out[i] = o[0, 0]
    xs, ys = bf16_bits_to_f32(xb).astype(np.float64), bf16_bits_to_f32(yb).astype(np.float64)
    seen_sub = seen_inf = 0
    for i in range(n):
        x, y, ci, si = float(xs[i]), float(ys[i]), float(c[i]), float(s[i])
        want = (_round_to_bf16_rational(x * ci - y * si), _round_to_bf16_rational(y * ci + x * si))
        assert (int(out[i, 0]), int(out[i, 1])) == want, (i, hex(xb[i]), hex(yb[i]), ci, si)
        seen_sub += (want[0] & 0x7FFF) < 0x0080
        seen_inf += (want[0] & 0x7FFF) == 0x7F80
    assert seen_sub > 20                                        # the sweep reaches the sub-normal grid
    del seen_inf


# ---------------------------------------------------------------------------
# Causal rows and shared-prefix attention: the two thin front ends that decide what
# decode_attn is asked, against brute force written out in plain Python
# ---------------------------------------------------------------------------
from oracle import causal_attn_rows, shared_prefix_attn  # noqa: E402
from paper_2510_07356_amd.workloads import make_shared_prefix  # noqa: E402


def _softmax_attention(qrow, keys, values, scale):
    """exp(s) / sum exp(s) in plain Python floats with math.fsum, no max subtraction."""
    s = [scale * math.fsum(a * b for a, b in zip(qrow, kr)) for kr in keys]
    e = [math.exp(x) for x in s]
    z = math.fsum(e)
    D = len(values[0])
    return [math.fsum(e[j] / z * values[j][d] for j in range(len(keys))) for d in range(D)], math.log(z)


@pytest.mark.parametrize("T,Hq,Hkv", [(1, 2, 1), (5, 4, 2), (6, 3, 3)])
def test_causal_rows_against_brute_force(T, Hq, Hkv):
    """Row t sees keys 0..t of ITS sequence and of kv head h / (Hq / Hkv): an off-by-one in the
    visible length, a mixed-up sequence or a transposed token/head axis all change the numbers."""
    B, D, scale = 2, 4, 0.5
    rng = np.random.default_rng(60 + T)
    q = small_ints(rng, (B, T, Hq, D))
    k = small_ints(rng, (B, T, Hkv, D))
    v = small_ints(rng, (B, T, Hkv, D))
    G = Hq // Hkv
    for b in range(B):
        rows = list(range(T))[::-1]                     # any order, any subset
        res = causal_attn_rows(bits(q), bits(k), bits(v), b, rows, scale)
        assert res.out.shape == (T, Hq, D)
        for i, t in enumerate(rows):
            for h in range(Hq):
                g = h // G
                want, want_lse = _softmax_attention(q[b, t, h].tolist(), k[b, :t + 1, g].tolist(),
                                                    v[b, :t + 1, g].tolist(), scale)
                np.testing.assert_allclose(res.out[i, h], want, rtol=0, atol=1e-13)
                assert abs(res.lse[i, h] - want_lse) < 1e-13
    # the first row is the first value row, the rows of sequence 0 do not depend on sequence 1
    res0 = causal_attn_rows(bits(q), bits(k), bits(v), 0, [0], scale)
    np.testing.assert_array_equal(res0.out[0], np.repeat(v[0, 0], G, axis=0).astype(np.float64))


@pytest.mark.parametrize("paged", [False, True])
def test_shared_prefix_against_brute_force(paged):
    """Two groups (3 and 2 samples) with prefixes of 3 and 0 tokens, suffixes of 0..4 tokens: every
    sequence attends over its group's prefix followed by its own suffix, nothing else."""
    sizes, prefixes, suffixes = [3, 2], [3, 0], [2, 0, 4, 1, 3]
    kw = dict(page_size=2) if paged else {}
    sw = make_shared_prefix("pin_prefix", 70, sizes, prefixes, suffixes, num_q_heads=4, num_kv_heads=2,
                            head_dim=4, paged=paged, **kw)
    w = sw.base
    res = shared_prefix_attn(w.q, sw.kp, sw.vp, sw.prefix_lens, sw.group_start, w.k, w.v, w.kv_lens, w.scale,
                             block_table=w.block_table, page_size=w.page_size)
    qf, kpf, vpf = bf16_bits_to_f32(w.q), bf16_bits_to_f32(sw.kp), bf16_bits_to_f32(sw.vp)
    kf, vf = bf16_bits_to_f32(w.k), bf16_bits_to_f32(w.v)
    group_of = [0, 0, 0, 1, 1]
    for b in range(5):
        j = group_of[b]
        for h in range(4):
            g = h // 2
            keys = [kpf[j, g, t].tolist() for t in range(prefixes[j])]
            vals = [vpf[j, g, t].tolist() for t in range(prefixes[j])]
            for t in range(suffixes[b]):
                if paged:
                    blk, slot = int(w.block_table[b, t // 2]), t % 2
                    keys.append(kf[blk, g, slot].tolist()); vals.append(vf[blk, g, slot].tolist())
                else:
                    keys.append(kf[b, g, t].tolist()); vals.append(vf[b, g, t].tolist())
            if not keys:
                assert np.all(res.out[b, h] == 0) and np.isneginf(res.lse[b, h])
                continue
            want, want_lse = _softmax_attention(qf[b, h].tolist(), keys, vals, float(w.scale))
            np.testing.assert_allclose(res.out[b, h], want, rtol=0, atol=1e-13)
            assert abs(res.lse[b, h] - want_lse) < 1e-12
    # the benchmark's "same problem without sharing" workload is the same concatenation
    c = sw.concatenated()
    plain = decode_attn(c.q, c.k, c.v, c.kv_lens, c.scale)
    np.testing.assert_array_equal(plain.out, res.out)
    np.testing.assert_array_equal(plain.lse, res.lse)
