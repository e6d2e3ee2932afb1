"""A whole decode step (KV append with rotary, then attention) captured once in a HIP graph and
replayed as the sequences grow.  The launch shape of the attention kernels does not depend on the
lengths (the KV stream is cut into equal shares on the device), so one captured graph serves every
step; each replay is checked against the oracle and against the same step run eagerly, with
ordinary eager work and synchronisation between the replays."""
import numpy as np
import pytest

from oracle import decode_attn, kv_append
from paper_2510_07356_amd import workloads as wl

pytestmark = pytest.mark.gpu

STEPS = 4


@pytest.fixture(scope="module")
def binding():
    from paper_2510_07356_amd import binding as b
    return b


def rope_table(positions, D=128, theta=1.0e6):
    d = np.arange(D // 2, dtype=np.float64)
    ang = np.arange(positions, dtype=np.float64)[:, None] * theta ** (-2.0 * d / D)[None, :]
    return np.concatenate([np.cos(ang), np.sin(ang)], axis=1).astype(np.float32)


def step_inputs(seed, B, Hq, Hkv, D=128):
    rng = np.random.default_rng(seed)
    bits = lambda shape: wl.f32_to_bf16_bits(rng.standard_normal(shape).astype(np.float32))
    return bits((B, Hq, D)), bits((B, Hkv, D)), bits((B, Hkv, D))


@pytest.mark.parametrize("paged", [False, True])
def test_captured_decode_step_replays(binding, paged):
    import torch
    # paged lengths leave room for STEPS more tokens inside each sequence's last page
    lens = [700, 33, 1, 2049 - 16, 0, 1500]
    B, Hq, Hkv = len(lens), 40, 8
    grown = [l + STEPS for l in lens]
    if paged:
        w = wl.make_paged("graph_paged", 300, B, Hq, Hkv, grown, table_width=160)
    else:
        w = wl.make_contiguous("graph", 300, B, Hq, Hkv, grown, cache_len=2048 + 64)
    cap = max(grown)                      # the length bound the captured launches are sized for
    w.kv_lens[:] = np.asarray(lens, dtype=np.int32)
    table = rope_table(cap)
    dev = binding.to_device(w)
    cs = torch.from_numpy(table).to("cuda:0")
    q_in = torch.empty_like(dev["q"])
    q_rot = torch.empty_like(dev["q"])
    k_new = torch.empty((B, Hkv, 128), dtype=torch.bfloat16, device="cuda:0")
    v_new = torch.empty_like(k_new)
    params = binding.make_params(q_rot, dev["k"], dev["v"], cap, w.scale, w.page_size,
                                 dev["block_table"], 0, 0)
    ws = torch.empty(binding.gqa_decode_workspace_bytes(params), dtype=torch.uint8, device="cuda:0")
    out = torch.empty((B, Hq, 128), dtype=torch.float32, device="cuda:0")
    lse = torch.empty((B, Hq), dtype=torch.float32, device="cuda:0")

    def decode_step():
        binding.gqa_decode_kv_append(q_in, q_rot, k_new, v_new, dev["k"], dev["v"], dev["kv_lens"], cap,
                                     dev["block_table"], w.page_size, cs)
        binding.gqa_decode_attn(params, q_rot, dev["k"], dev["v"], dev["kv_lens"], dev["block_table"], None,
                                out, lse, ws)

    def load_step(step):
        q, kn, vn = step_inputs(310 + step, B, Hq, Hkv)
        q_in.copy_(binding._bf16_view(q).to("cuda:0"))
        k_new.copy_(binding._bf16_view(kn).to("cuda:0"))
        v_new.copy_(binding._bf16_view(vn).to("cuda:0"))
        # a sequence that is empty stays empty; the others grow by the token being appended
        w.kv_lens[:] = np.where(np.asarray(lens) > 0, np.asarray(lens) + step + 1, 0).astype(np.int32)
        dev["kv_lens"].copy_(torch.from_numpy(w.kv_lens))
        return q, kn, vn

    # the first call on a device queries its properties: keep that outside the capture
    load_step(-1)
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):
        decode_step()
    torch.cuda.current_stream().wait_stream(side)
    torch.cuda.synchronize()
    # that warm-up appended a token at position lens[b] - 1 + 0; restore the cache
    fresh = binding.to_device(w)
    dev["k"].copy_(fresh["k"])
    dev["v"].copy_(fresh["v"])
    torch.cuda.synchronize()

    graph = torch.cuda.CUDAGraph()
    load_step(0)
    with torch.cuda.graph(graph):
        decode_step()
    # capture only records; undo nothing, run every step through replay

    for step in range(STEPS):
        q, kn, vn = load_step(step)
        out.fill_(float("nan"))
        lse.fill_(float("nan"))
        graph.replay()
        torch.cuda.synchronize()
        got, got_lse = out.double().cpu().numpy(), lse.double().cpu().numpy()
        w.q = q
        q_ref = kv_append(q, kn, vn, w.k, w.v, w.kv_lens, cos_sin=table,
                          block_table=w.block_table, page_size=w.page_size)
        ref = decode_attn(q_ref, w.k, w.v, w.kv_lens, w.scale, block_table=w.block_table, page_size=w.page_size)
        err = got - ref.out
        assert np.isfinite(got).all(), step
        assert np.abs(err).max() <= 1e-2 and np.linalg.norm(err) / np.linalg.norm(ref.out) <= 5e-3, step
        live = np.asarray(lens) > 0
        assert np.abs(got_lse[live] - ref.lse[live]).max() <= 4e-3, step
        assert np.all(got[~live] == 0) and np.all(np.isneginf(got_lse[~live])), step
        # eager work between replays: the same step again, eagerly (the append rewrites the same rows
        # with the same values), must reproduce the replay bit for bit
        eager_out = torch.empty_like(out)
        keep = out.clone()
        decode_step()
        torch.cuda.synchronize()
        eager_out.copy_(out)
        assert torch.equal(eager_out, keep), step
