"""GPU parity: the HIP library (through its C ABI) against the fp64 oracle,
element by element, on the same seeded bf16 inputs.

Tolerances (bf16 inputs, fp32 accumulation, probabilities rounded to bf16 on
the matrix-core path): max-abs error <= 1e-2 and relative L2 error <= 5e-3
over the whole output of a case; additionally the worst single sequence must
meet the same relative-L2 bound, and no output may be non-finite.  LSE is
compared with an absolute bound of 4e-3 (its normaliser is summed from
bf16-rounded weights, each within 2^-9 of the exact one).
"""
import numpy as np
import pytest

from oracle import decode_attn
from paper_2510_07356_amd import workloads as wl

pytestmark = pytest.mark.gpu

MAX_ABS = 1e-2
REL_L2 = 5e-3
LSE_ABS = 4e-3


@pytest.fixture(scope="module")
def binding():
    from paper_2510_07356_amd import binding as b
    return b


def oracle_of(w):
    return decode_attn(w.q, w.k, w.v, w.kv_lens, w.scale, block_table=w.block_table, page_size=w.page_size)


def check(w, out, lse, ref, tag=""):
    got = out.double().cpu().numpy()
    assert np.all(np.isfinite(got)), f"{tag}: non-finite output"
    err = got - ref.out
    max_abs = np.abs(err).max()
    rel = np.linalg.norm(err) / max(np.linalg.norm(ref.out), 1e-30)
    per_seq = [np.linalg.norm(err[b]) / np.linalg.norm(ref.out[b])
               for b in range(w.batch) if w.kv_lens[b] > 0]
    worst = max(per_seq) if per_seq else 0.0
    print(f"{tag or w.name}: max_abs={max_abs:.3e} rel_l2={rel:.3e} worst_seq_rel_l2={worst:.3e}", flush=True)
    assert max_abs <= MAX_ABS, f"{tag}: max-abs {max_abs}"
    assert rel <= REL_L2, f"{tag}: rel-L2 {rel}"
    assert worst <= REL_L2, f"{tag}: worst per-sequence rel-L2 {worst}"
    for b in range(w.batch):
        if w.kv_lens[b] == 0:
            assert np.all(got[b] == 0.0)
    if lse is not None:
        gl = lse.double().cpu().numpy()
        empty = w.kv_lens == 0
        assert np.all(np.isneginf(gl[empty]))
        assert np.abs(gl[~empty] - ref.lse[~empty]).max(initial=0.0) <= LSE_ABS, f"{tag}: lse"


# --------------------------------------------------------------------------- small cases, every output compared

SMALL_LENS = [1, 17, 64, 65, 200, 333, 0, 1025]          # empty, single, tile edges, ragged tails, > 2 chunks


@pytest.mark.parametrize("variant", [0, 1])
@pytest.mark.parametrize("layout", ["head_major", "token_major"])
@pytest.mark.parametrize("chunk", [0, 64, 256])
def test_small_contiguous(binding, variant, layout, chunk):
    w = wl.make_contiguous("small", 100, len(SMALL_LENS), 40, 8, SMALL_LENS, cache_len=1100, layout=layout)
    ref = oracle_of(w)
    for host in (True, False):
        out, lse = binding.run_workload(w, chunk_tokens=chunk, kernel_variant=variant, use_host_lens=host)
        check(w, out, lse, ref, f"small/{layout}/v{variant}/c{chunk}/host{int(host)}")


@pytest.mark.parametrize("variant", [0, 1])
@pytest.mark.parametrize("layout", ["head_major", "token_major"])
@pytest.mark.parametrize("page", [16, 64])
def test_small_paged(binding, variant, layout, page):
    w = wl.make_paged("small_paged", 101, len(SMALL_LENS), 32, 8, SMALL_LENS, page_size=page,
                      table_width=1100 // page + 3, layout=layout)
    ref = oracle_of(w)
    for chunk in (0, 128):
        out, lse = binding.run_workload(w, chunk_tokens=chunk, kernel_variant=variant)
        check(w, out, lse, ref, f"paged{page}/{layout}/v{variant}/c{chunk}")


@pytest.mark.parametrize("hq,hkv,variants", [(8, 8, (0, 1)), (8, 4, (0, 1)), (24, 8, (0, 1)), (7, 1, (0, 1)),
                                             (64, 8, (0, 1)), (32, 2, (0,)), (12, 1, (0,))])
def test_group_sizes(binding, hq, hkv, variants):
    lens = [300, 31, 129]
    w = wl.make_contiguous("groups", 102, 3, hq, hkv, lens)
    ref = oracle_of(w)
    for variant in variants:
        out, lse = binding.run_workload(w, chunk_tokens=128, kernel_variant=variant)
        check(w, out, lse, ref, f"G{hq // hkv}/v{variant}")


def test_split_count_does_not_change_the_result_much_and_runs_are_deterministic(binding):
    w = wl.make_contiguous("splits", 103, 2, 40, 8, [4000, 2500])
    ref = oracle_of(w)
    dev = binding.to_device(w)
    outs = []
    for chunk in (64, 128, 512, 4096):
        out, lse = binding.run_workload(w, dev=dev, chunk_tokens=chunk)
        check(w, out, lse, ref, f"splits/c{chunk}")
        again, _ = binding.run_workload(w, dev=dev, chunk_tokens=chunk)
        assert bool((out == again).all()), "same plan, different bits"
        outs.append(out)


def test_extreme_scores(binding):
    """One key dominates by a huge margin, others are far below: exercises the
    rescale and underflow paths (weights that round to zero, no NaN)."""
    w = wl.make_contiguous("extreme", 104, 2, 40, 8, [2000, 700], outlier_fraction=0.002, outlier_gain=32.0,
                           scale=1.0)
    ref = oracle_of(w)
    for variant in (0, 1):
        out, lse = binding.run_workload(w, chunk_tokens=128, kernel_variant=variant)
        check(w, out, lse, ref, f"extreme/v{variant}")


def test_zero_and_negative_scale(binding):
    w0 = wl.make_contiguous("scale0", 105, 2, 40, 8, [500, 77], scale=0.0)
    wn = wl.make_contiguous("scaleneg", 105, 2, 40, 8, [500, 77], scale=-0.25)
    for w in (w0, wn):
        ref = oracle_of(w)
        for variant in (0, 1):
            out, lse = binding.run_workload(w, kernel_variant=variant)
            check(w, out, lse, ref, f"{w.name}/v{variant}")


def test_strided_q_and_no_lse(binding):
    import torch
    w = wl.make_contiguous("strided_q", 106, 3, 40, 8, [100, 260, 5])
    ref = oracle_of(w)
    dev = binding.to_device(w)
    wide = torch.zeros((3, 40, 256), dtype=torch.bfloat16, device="cuda:0")
    wide[:, :, :128] = dev["q"]
    dev["q"] = wide[:, :, :128]
    out, lse = binding.run_workload(w, dev=dev, want_lse=False)
    assert lse is None
    check(w, out, None, ref, "strided_q")


# --------------------------------------------------------------------------- the five configurations, full size

@pytest.mark.parametrize("index", [0, 1, 2, 3, 4])
def test_named_configs_full_size(binding, index):
    """Every output element of every named configuration, in the launch
    configuration the benchmark times (default variant, library-chosen split,
    host lengths given)."""
    w = wl.make_config(index)
    ref = oracle_of(w)
    dev = binding.to_device(w)
    out, lse = binding.run_workload(w, dev=dev)
    check(w, out, lse, ref, f"config{index}:{w.name}")
    if index in (0, 2):          # the plain fp32 path and the token-major layout on the same data
        out, lse = binding.run_workload(w, dev=dev, kernel_variant=1)
        check(w, out, lse, ref, f"config{index}:{w.name}/valu")
    del dev
    if index in (0, 1):
        wt = wl.make_config(index, layout="token_major")
        out, lse = binding.run_workload(wt)
        check(wt, out, lse, ref, f"config{index}:{w.name}/token_major")
