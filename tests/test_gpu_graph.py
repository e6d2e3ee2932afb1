"""A whole decode step (KV append with rotary, then attention) captured once in a HIP graph and
replayed as the sequences grow.  The launch shape of the attention kernels does not depend on the
lengths (the KV stream is cut into equal shares on the device), so one captured graph serves every
step; each replay is checked against the oracle and against the same step run eagerly, with
ordinary eager work and synchronisation between the replays."""
import numpy as np
import pytest

from oracle import decode_attn, kv_append, shared_prefix_attn
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


def replay_and_compare(graph, eager, outputs, replays=3):
    """Replays `graph` several times with eager work and synchronisation in between; every replay
    must reproduce, bit for bit, what the same calls give when run eagerly."""
    import torch
    eager()
    torch.cuda.synchronize()
    want = [t.clone() for t in outputs]
    for r in range(replays):
        for t in outputs:
            t.fill_(float("nan"))
        graph.replay()
        torch.cuda.synchronize()
        for t, w in zip(outputs, want):
            assert torch.equal(t, w), f"replay {r}"
        eager()                      # the program's own eager work between replays
        torch.cuda.synchronize()


def test_captured_prefill_shared_prefix_and_static_calls(binding):
    """After gqa_decode_init() the other entry points can be captured too: causal prefill (its LDS
    limit is a per-device attribute set at init), the shared-prefix call, and the call that uses the
    built-in scratch buffer.  Run alone, these are the first calls of the process on these entry points."""
    import torch
    binding.gqa_decode_init()
    scale = float(np.float32(1.0 / np.sqrt(128)))
    rng = np.random.default_rng(77)
    bits = lambda shape: binding._bf16_view(wl.f32_to_bf16_bits(rng.standard_normal(shape).astype(np.float32))).to("cuda:0")

    # prefill, ragged batch of two prompts
    pq, pk, pv = bits((2, 300, 10, 128)), bits((2, 300, 2, 128)), bits((2, 300, 2, 128))
    p_lens = torch.tensor([300, 129], dtype=torch.int32, device="cuda:0")
    p_out = torch.zeros((2, 300, 10, 128), dtype=torch.float32, device="cuda:0")
    p_lse = torch.zeros((2, 300, 10), dtype=torch.float32, device="cuda:0")

    # shared prefix: 2 prompts x 3 samples
    sw = wl.make_shared_prefix("graph_casc", 320, [3, 3], [200, 65], [40, 1, 300, 0, 77, 130])
    sdev = binding.shared_prefix_to_device(sw)
    cp = binding.make_cascade_params(sdev["q"], sdev["k"], sdev["v"], sdev["kp"], sdev["vp"], sw.base.max_kv_len,
                                     int(sw.prefix_lens.max()), 2, sw.base.scale)
    s_ws = torch.empty(binding.gqa_cascade_workspace_bytes(cp), dtype=torch.uint8, device="cuda:0")
    s_out = torch.zeros((6, 40, 128), dtype=torch.float32, device="cuda:0")
    s_lse = torch.zeros((6, 40), dtype=torch.float32, device="cuda:0")

    def casc():         # marshalled at call time: the call goes to the stream that is current then
        binding.CascadeCall(cp, sdev["q"], sdev["kp"], sdev["vp"], sdev["prefix_lens"], sdev["group_start"],
                            sw.group_start, sdev["k"], sdev["v"], sdev["kv_lens"], None, s_out, s_lse, s_ws)()

    # plain decode on the built-in scratch buffer
    w = wl.make_contiguous("graph_static", 321, 3, 40, 8, [900, 31, 257])
    dev = binding.to_device(w)
    params = binding.make_params(dev["q"], dev["k"], dev["v"], w.max_kv_len, w.scale)
    d_out = torch.zeros((3, 40, 128), dtype=torch.float32, device="cuda:0")
    d_lse = torch.zeros((3, 40), dtype=torch.float32, device="cuda:0")

    def calls():
        binding.gqa_prefill_attn(pq, pk, pv, scale, p_out, p_lse, seq_lens=p_lens)
        casc()
        binding.gqa_decode_attn_static(params, dev["q"], dev["k"], dev["v"], dev["kv_lens"], None, d_out, d_lse)

    torch.cuda.synchronize()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph):
        calls()
    # rows of the second prompt beyond its length are not written: compare the written part only
    p_out[1, 129:] = 0
    p_lse[1, 129:] = 0

    def eager():
        calls()
        p_out[1, 129:] = 0
        p_lse[1, 129:] = 0

    def replay_outputs():
        return [p_out[0], p_out[1, :129], p_lse[0], p_lse[1, :129], s_out, s_lse, d_out, d_lse]

    # torch.equal on views: materialise through the helper's clone()
    replay_and_compare(graph, eager, replay_outputs())

    # and the results are the right ones
    ref = decode_attn(w.q, w.k, w.v, w.kv_lens, w.scale)
    err = d_out.double().cpu().numpy() - ref.out
    assert np.abs(err).max() <= 1e-2 and np.linalg.norm(err) / np.linalg.norm(ref.out) <= 5e-3
    ref = shared_prefix_attn(sw.base.q, sw.kp, sw.vp, sw.prefix_lens, sw.group_start, sw.base.k, sw.base.v,
                             sw.base.kv_lens, sw.base.scale)
    err = s_out.double().cpu().numpy() - ref.out
    assert np.abs(err).max() <= 1e-2 and np.linalg.norm(err) / np.linalg.norm(ref.out) <= 5e-3
