"""GPU parity of shared-prefix (cascade) decode attention against the oracle
(oracle.shared_prefix_attn: the same problem without sharing, one private cache per sequence holding
the prefix of its group followed by its suffix; pinned against brute force in
tests/test_oracle_pins.py).  Tolerances as in test_gpu_parity.py."""
import numpy as np
import pytest

from oracle import shared_prefix_attn
from paper_2510_07356_amd import workloads as wl

pytestmark = pytest.mark.gpu

MAX_ABS, REL_L2, LSE_ABS = 1e-2, 5e-3, 4e-3


@pytest.fixture(scope="module")
def binding():
    from paper_2510_07356_amd import binding as b
    return b


def oracle_reference(sw):
    w = sw.base
    return shared_prefix_attn(w.q, sw.kp, sw.vp, sw.prefix_lens, sw.group_start, w.k, w.v, w.kv_lens, w.scale,
                              block_table=w.block_table, page_size=w.page_size)


def check(sw, out, lse, tag):
    ref = oracle_reference(sw)
    full_lens = np.repeat(sw.prefix_lens, np.diff(sw.group_start)).astype(np.int64) + sw.base.kv_lens
    got = out.double().cpu().numpy()
    assert np.isfinite(got).all(), f"{tag}: non-finite"
    err = got - ref.out
    max_abs = np.abs(err).max()
    rel = np.linalg.norm(err) / max(np.linalg.norm(ref.out), 1e-30)
    worst = max([np.linalg.norm(err[b]) / np.linalg.norm(ref.out[b]) for b in range(sw.base.batch) if full_lens[b] > 0],
                default=0.0)
    print(f"{tag}: max_abs={max_abs:.3e} rel_l2={rel:.3e} worst_seq_rel_l2={worst:.3e}", flush=True)
    assert max_abs <= MAX_ABS and rel <= REL_L2 and worst <= REL_L2, tag
    gl = lse.double().cpu().numpy()
    empty = full_lens == 0
    assert np.all(got[empty] == 0.0) and np.all(np.isneginf(gl[empty]))
    assert np.abs(gl[~empty] - ref.lse[~empty]).max(initial=0.0) <= LSE_ABS, f"{tag}: lse"


@pytest.mark.parametrize("paged", [False, True])
@pytest.mark.parametrize("layout", ["head_major", "token_major"])
def test_small_groups(binding, paged, layout):
    """Group sizes 1..12 (1 to 4 MFMA column blocks with G = 5), empty prefixes, empty suffixes,
    an entirely empty sequence, ragged tile tails."""
    sizes = [1, 3, 4, 7, 12, 2]
    prefixes = [100, 33, 0, 257, 64, 1]
    rng = np.random.default_rng(3)
    suffixes = rng.integers(0, 300, size=sum(sizes))
    suffixes[0] = 0
    suffixes[5] = 0          # group 2 has no prefix: this sequence is empty altogether
    suffixes[9] = 1
    sw = wl.make_shared_prefix("casc_small", 300, sizes, prefixes, suffixes, paged=paged, layout=layout)
    for chunk in (0, 32, 256):
        out, lse = binding.run_shared_prefix(sw, chunk_tokens=chunk)
        check(sw, out, lse, f"casc_small/{layout}/paged{int(paged)}/c{chunk}")


def test_group_of_four_heads_sixteen_samples(binding):
    sw = wl.make_shared_prefix("casc_g4", 301, [16, 5], [700, 90], list(range(1, 22)), num_q_heads=32,
                               num_kv_heads=8)
    check(sw, *binding.run_shared_prefix(sw), "casc_g4")


def test_single_group_equals_plain_attention_when_prefix_is_empty(binding):
    """No prefix at all: the cascade entry point must reproduce the plain one."""
    lens = [500, 31, 1200]
    sw = wl.make_shared_prefix("casc_noprefix", 302, [3], [0], lens)
    out, lse = binding.run_shared_prefix(sw)
    check(sw, out, lse, "casc_noprefix")
    plain, plain_lse = binding.run_workload(sw.base)
    assert float((out - plain).abs().max()) <= 2e-3


@pytest.mark.parametrize("scale", [0.0, -0.05, 1.5])
@pytest.mark.parametrize("paged", [False, True])
def test_zero_negative_and_large_scale(binding, scale, paged):
    """scale 0: the mean over prefix and suffix together; a negative scale; a nearly one-hot softmax
    whose winner may sit in the prefix or in the suffix."""
    sw = wl.make_shared_prefix("casc_scale", 304, [5, 2, 1], [300, 40, 0], [120, 1, 0, 77, 500, 64, 9, 200],
                               paged=paged, scale=scale)
    check(sw, *binding.run_shared_prefix(sw), f"casc_scale_{scale}_paged{int(paged)}")


@pytest.mark.parametrize("paged", [False, True])
def test_groups_without_sequences(binding, paged):
    """group_start may repeat a value: a group with no sequence (its prefix is never read), at the
    start, in the middle and at the end of the list."""
    sizes = [0, 3, 0, 0, 2, 4, 0]
    prefixes = [500, 100, 64, 0, 33, 257, 90]
    suffixes = [40, 0, 130, 1, 65, 300, 31, 32, 0]
    sw = wl.make_shared_prefix("casc_holes", 305, sizes, prefixes, suffixes, paged=paged)
    for chunk in (0, 64):
        check(sw, *binding.run_shared_prefix(sw, chunk_tokens=chunk), f"casc_holes/paged{int(paged)}/c{chunk}")


@pytest.mark.parametrize("groups", [63, 64, 65, 150])
def test_many_groups(binding, groups):
    """More groups than a wavefront has lanes: the search for a sequence's group then takes several
    rounds of 64 (63 is the largest list the combine kernel handles in one)."""
    rng = np.random.default_rng(groups)
    sizes = rng.integers(0, 4, size=groups)
    sizes[0], sizes[-1] = 2, 1
    prefixes = rng.integers(0, 200, size=groups)
    suffixes = rng.integers(0, 150, size=int(sizes.sum()))
    sw = wl.make_shared_prefix(f"casc_many{groups}", 306 + groups, list(sizes), list(prefixes), list(suffixes),
                               paged=bool(groups % 2))
    check(sw, *binding.run_shared_prefix(sw), f"casc_many{groups}")


def test_too_large_group_is_rejected(binding):
    sw = wl.make_shared_prefix("casc_big", 303, [13], [64], [10] * 13)       # 13 * 5 = 65 query rows > 64
    with pytest.raises(binding.GqaError) as e:
        binding.run_shared_prefix(sw)
    assert e.value.status == binding.GQA_ERR_UNSUPPORTED


def test_sampling_batch_full_size(binding):
    """The benchmark workload: 12 prompts x 5 samples, every output element."""
    sw = wl.make_sampling_batch()
    out, lse = binding.run_shared_prefix(sw)
    check(sw, out, lse, "sampling_12x5")
    sw10 = wl.make_sampling_batch(seed=6, tasks=6, samples=10)
    out, lse = binding.run_shared_prefix(sw10)
    check(sw10, out, lse, "sampling_6x10")


def random_cascade_case(rng):
    hkv = int(rng.choice([1, 2, 3, 8]))
    group = int(rng.choice([1, 2, 4, 5, 8, 16]))
    n_groups = int(rng.choice([1, 2, 7, 20, 70]))
    most = max(64 // group, 1)                                   # a group serves at most 64 query rows
    sizes = rng.integers(0, min(most, 12) + 1, size=n_groups)
    if sizes.sum() == 0:
        sizes[0] = 1
    top_p = int(rng.choice([0, 40, 700, 3000]))
    top_s = int(rng.choice([40, 300, 2000]))
    prefixes = rng.integers(0, top_p + 1, size=n_groups)
    suffixes = rng.integers(0, top_s + 1, size=int(sizes.sum()))
    kind = rng.random(len(suffixes))
    suffixes = np.where(kind < 0.15, 0, np.where(kind < 0.25, 1, suffixes))
    return dict(hkv=hkv, group=group, sizes=sizes, prefixes=prefixes, suffixes=suffixes,
                paged=bool(rng.random() < 0.5), layout=str(rng.choice(["head_major", "token_major"])),
                chunk=int(rng.choice([0, 0, 32, 96, 512])),
                scale=float(rng.choice([1.0 / np.sqrt(128), 0.25, -0.05])))


@pytest.mark.parametrize("seed", list(range(16)))
def test_random_shared_prefix_shape(binding, seed):
    """Seeded random group counts and sizes (groups without sequences, up to 64 query rows per group), prefix
    and suffix lengths (empty ones, single tokens), head counts, layouts, paging, fixed and automatic splits."""
    rng = np.random.Generator(np.random.PCG64([901, seed]))
    c = random_cascade_case(rng)
    print(f"seed={seed} Hkv={c['hkv']} G={c['group']} groups={len(c['sizes'])} B={int(c['sizes'].sum())} "
          f"prefix[max]={int(c['prefixes'].max())} suffix[max]={int(c['suffixes'].max(initial=0))} paged={c['paged']} "
          f"layout={c['layout']} chunk={c['chunk']} scale={c['scale']:.4f}", flush=True)
    sw = wl.make_shared_prefix(f"casc_rand{seed}", 2000 + seed, list(c["sizes"]), list(c["prefixes"]),
                               list(c["suffixes"]), num_q_heads=c["hkv"] * c["group"], num_kv_heads=c["hkv"],
                               paged=c["paged"], layout=c["layout"], scale=c["scale"])
    check(sw, *binding.run_shared_prefix(sw, chunk_tokens=c["chunk"]), f"casc_rand{seed}")
