"""GPU parity of causal prefill attention.  Row t of causal attention is, by definition, the decode
attention of query t over the first t + 1 keys, so the (pinned) decode oracle serves through
oracle.causal_attn_rows (itself pinned against a brute-force causal attention in
tests/test_oracle_pins.py).  Small cases check every row; the 32,768-token case checks sampled rows."""
import numpy as np
import pytest

from oracle import causal_attn_rows as oracle_rows
from paper_2510_07356_amd import workloads as wl

pytestmark = pytest.mark.gpu

MAX_ABS, REL_L2, LSE_ABS = 1e-2, 5e-3, 4e-3


@pytest.fixture(scope="module")
def binding():
    from paper_2510_07356_amd import binding as b
    return b


def make_inputs(seed, B, T, Hq, Hkv, D=128):
    rng = np.random.default_rng(seed)
    q = wl.f32_to_bf16_bits(rng.standard_normal((B, T, Hq, D), dtype=np.float32))
    k = wl.f32_to_bf16_bits(rng.standard_normal((B, T, Hkv, D), dtype=np.float32))
    v = wl.f32_to_bf16_bits(rng.standard_normal((B, T, Hkv, D), dtype=np.float32))
    return q, k, v


def run(binding, q, k, v, scale):
    import torch
    dq, dk, dv = (binding._bf16_view(x).to("cuda:0") for x in (q, k, v))
    B, T, Hq, D = q.shape
    out = torch.full((B, T, Hq, D), float("nan"), dtype=torch.float32, device="cuda:0")
    lse = torch.full((B, T, Hq), float("nan"), dtype=torch.float32, device="cuda:0")
    binding.gqa_prefill_attn(dq, dk, dv, scale, out, lse)
    torch.cuda.synchronize()
    return out, lse


def check_rows(out, lse, ref, b, rows, tag):
    got = out[b].double().cpu().numpy()[rows]
    assert np.isfinite(got).all(), f"{tag}: non-finite"
    err = got - ref.out
    max_abs = np.abs(err).max()
    rel = np.linalg.norm(err) / np.linalg.norm(ref.out)
    worst = max(np.linalg.norm(err[i]) / np.linalg.norm(ref.out[i]) for i in range(len(rows)))
    print(f"{tag}: rows={len(rows)} max_abs={max_abs:.3e} rel_l2={rel:.3e} worst_row_rel_l2={worst:.3e}", flush=True)
    assert max_abs <= MAX_ABS and rel <= REL_L2 and worst <= REL_L2, tag
    gl = lse[b].double().cpu().numpy()[rows]
    assert np.abs(gl - ref.lse).max() <= LSE_ABS, f"{tag}: lse"


@pytest.mark.parametrize("T", [1, 31, 64, 257, 700])
def test_every_row_small(binding, T):
    scale = float(np.float32(1.0 / np.sqrt(128)))
    q, k, v = make_inputs(400 + T, 2, T, 10, 2)
    out, lse = run(binding, q, k, v, scale)
    for b in range(2):
        rows = np.arange(T)
        check_rows(out, lse, oracle_rows(q, k, v, b, rows, scale), b, rows, f"prefill_T{T}_b{b}")


def test_first_row_is_the_first_value_row(binding):
    scale = 0.25
    q, k, v = make_inputs(450, 1, 300, 8, 8)
    out, _ = run(binding, q, k, v, scale)
    np.testing.assert_array_equal(out[0, 0].cpu().numpy(), wl.bf16_bits_to_f32(v[0, 0]))


@pytest.mark.parametrize("scale", [0.0, -0.05, 1.5])
def test_zero_negative_and_large_scale(binding, scale):
    """scale 0: every row is the running mean of the values (the mask must not rely on -inf * 0);
    a negative scale prefers the smallest raw scores; a large one makes the softmax nearly one-hot."""
    q, k, v = make_inputs(455, 1, 300, 10, 2)
    out, lse = run(binding, q, k, v, scale)
    rows = np.arange(300)
    check_rows(out, lse, oracle_rows(q, k, v, 0, rows, scale), 0, rows, f"prefill_scale_{scale}")


def test_outlier_keys_move_the_running_maximum(binding):
    """A few key rows scaled by 8 (as in the long-sequence decode configuration): rows after an outlier
    are dominated by it, the running maximum jumps late in the walk and the accumulators are rescaled."""
    scale = float(np.float32(1.0 / np.sqrt(128)))
    T = 600
    q, k, v = make_inputs(456, 1, T, 10, 2)
    kf = wl.bf16_bits_to_f32(k)
    for t in (5, 130, 131, 383, 599):
        kf[0, t] *= 8.0
    k = wl.f32_to_bf16_bits(kf)
    out, lse = run(binding, q, k, v, scale)
    rows = np.arange(T)
    check_rows(out, lse, oracle_rows(q, k, v, 0, rows, scale), 0, rows, "prefill_outliers")


@pytest.mark.parametrize("growth", [1.0, 4.0, 11.0])
def test_scores_that_keep_growing_along_the_sequence(binding, growth):
    """Keys aligned with the queries and growing with the token index: the largest score of a row rises by
    `growth` binary orders of magnitude per 32 tokens, so the exponent reference of the online softmax lags
    behind the maximum (weights above 1 for growth 1 and 4) or has to follow it at every step (growth 11)."""
    scale = float(np.float32(1.0 / np.sqrt(128)))
    T = 700
    rng = np.random.default_rng(457)
    u = rng.standard_normal(128).astype(np.float32)
    per_token = growth / 32.0 / (scale * np.log2(np.e)) / float(u @ u)      # raw score rises by this per token
    q = wl.f32_to_bf16_bits(np.broadcast_to(u, (1, T, 10, 128)) + 0.1 * rng.standard_normal((1, T, 10, 128), dtype=np.float32))
    ramp = (np.arange(T, dtype=np.float32) * per_token)[None, :, None, None] * u
    k = wl.f32_to_bf16_bits(ramp + 0.1 * rng.standard_normal((1, T, 2, 128), dtype=np.float32))
    v = wl.f32_to_bf16_bits(rng.standard_normal((1, T, 2, 128), dtype=np.float32))
    out, lse = run(binding, q, k, v, scale)
    rows = np.arange(T)
    check_rows(out, lse, oracle_rows(q, k, v, 0, rows, scale), 0, rows, f"prefill_growing_{growth}")


def test_strided_inputs_and_group_sizes(binding):
    """Token-major projections sliced out of a fused QKV buffer, group sizes 1, 4 and 16."""
    import torch
    scale = float(np.float32(1.0 / np.sqrt(128)))
    for Hq, Hkv in ((4, 4), (16, 4), (16, 1)):
        T = 200
        q, k, v = make_inputs(460 + Hq + Hkv, 1, T, Hq, Hkv)
        fused = torch.zeros((1, T, Hq + 2 * Hkv, 128), dtype=torch.bfloat16, device="cuda:0")
        fused[:, :, :Hq] = binding._bf16_view(q).to("cuda:0")
        fused[:, :, Hq:Hq + Hkv] = binding._bf16_view(k).to("cuda:0")
        fused[:, :, Hq + Hkv:] = binding._bf16_view(v).to("cuda:0")
        out = torch.empty((1, T, Hq, 128), dtype=torch.float32, device="cuda:0")
        lse = torch.empty((1, T, Hq), dtype=torch.float32, device="cuda:0")
        binding.gqa_prefill_attn(fused[:, :, :Hq], fused[:, :, Hq:Hq + Hkv], fused[:, :, Hq + Hkv:], scale, out, lse)
        rows = np.arange(T)
        check_rows(out, lse, oracle_rows(q, k, v, 0, rows, scale), 0, rows, f"prefill_fused_{Hq}_{Hkv}")


@pytest.mark.parametrize("Hq,Hkv", [(32, 16), (16, 16), (6, 3), (9, 9), (24, 12)])
def test_kv_head_counts_beyond_and_off_the_xcd_count(binding, Hq, Hkv):
    """KV heads are dealt to the 8 XCDs: more than 8 (two heads per XCD), fewer, and counts that are
    not a multiple of 8 (workgroups whose head does not exist leave at once)."""
    scale = float(np.float32(1.0 / np.sqrt(128)))
    T = 300
    q, k, v = make_inputs(480 + Hq + Hkv, 2, T, Hq, Hkv)
    out, lse = run(binding, q, k, v, scale)
    rows = np.arange(T)
    for b in range(2):
        check_rows(out, lse, oracle_rows(q, k, v, b, rows, scale), b, rows, f"prefill_heads_{Hq}_{Hkv}_b{b}")


def test_long_sequence_sampled_rows(binding):
    """32,768 tokens, the 32B head shape: sampled rows (block edges, the diagonal of every kind of
    tile, the last rows) against the oracle."""
    scale = float(np.float32(1.0 / np.sqrt(128)))
    T = 32768
    q, k, v = make_inputs(470, 1, T, 40, 8)
    out, lse = run(binding, q, k, v, scale)
    rng = np.random.default_rng(1)
    rows = np.unique(np.concatenate([[0, 1, 31, 32, 63, 64, 255, 256, 257, 16383, 16384, T - 257, T - 256, T - 1],
                                     rng.integers(0, T, size=50)]))
    check_rows(out, lse, oracle_rows(q, k, v, 0, rows, scale), 0, rows, "prefill_32k")


def test_ragged_prompt_batch(binding):
    """Prompts of different lengths in one padded batch: every row below a sequence's length matches the
    oracle, rows beyond it (and a whole empty sequence) are left untouched."""
    import torch
    B, T, Hq, Hkv = 5, 700, 40, 8
    lens = [700, 1, 300, 0, 257]
    q, k, v = make_inputs(31, B, T, Hq, Hkv)
    scale = float(np.float32(1.0 / np.sqrt(128)))
    dq, dk, dv = (binding._bf16_view(x).to("cuda:0") for x in (q, k, v))
    # poison what lies beyond each sequence: it must not be read
    for b, L in enumerate(lens):
        dk[b, L:] = float("nan")
        dv[b, L:] = float("nan")
        dq[b, L:] = float("nan")
    out = torch.full((B, T, Hq, 128), float("nan"), dtype=torch.float32, device="cuda:0")
    lse = torch.full((B, T, Hq), float("nan"), dtype=torch.float32, device="cuda:0")
    binding.gqa_prefill_attn(dq, dk, dv, scale, out, lse, seq_lens=torch.tensor(lens, dtype=torch.int32, device="cuda:0"))
    torch.cuda.synchronize()
    for b, L in enumerate(lens):
        if L > 0:
            rows = np.arange(L)
            check_rows(out, lse, oracle_rows(q, k, v, b, rows, scale), b, rows, f"ragged b={b} len={L}")
        assert torch.isnan(out[b, L:]).all() and torch.isnan(lse[b, L:]).all(), f"b={b}: rows beyond the length were written"
