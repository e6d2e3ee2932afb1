"""Seeded random shapes through the C ABI against the oracle: batch sizes, head counts, group sizes,
length mixes (empty sequences, single tokens, ragged tails), page sizes, memory layouts, fixed and
automatic splits, both kernel variants.  Every output element is compared; each case prints its
parameters first so that a failure names it."""
import numpy as np
import pytest

from paper_2510_07356_amd import workloads as wl
from test_gpu_parity import check, oracle_of

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def binding():
    from paper_2510_07356_amd import binding as b
    return b


def random_case(rng):
    hkv = int(rng.choice([1, 2, 3, 8]))
    group = int(rng.choice([1, 2, 4, 5, 8, 16]))
    batch = int(rng.choice([1, 2, 5, 17, 70, 130]))
    top = int(rng.choice([40, 300, 1500, 5000]))
    lens = rng.integers(0, top + 1, size=batch)
    kind = rng.random(batch)
    lens = np.where(kind < 0.1, 0, np.where(kind < 0.2, 1, lens)).astype(np.int32)
    if batch * hkv * int(lens.max(initial=0)) > 3_000_000:          # keep the oracle's share of the run short
        lens = np.minimum(lens, 3_000_000 // (batch * hkv)).astype(np.int32)
    paged = bool(rng.random() < 0.5)
    layout = str(rng.choice(["head_major", "token_major"]))
    variant = int(rng.random() < 0.3) if group <= 8 else 0
    chunk = int(rng.choice([0, 0, 32, 96, 512]))
    page = int(rng.choice([16, 32, 128]))
    scale = float(rng.choice([1.0 / np.sqrt(128), 0.25, -0.05]))
    return dict(hkv=hkv, group=group, batch=batch, lens=lens, paged=paged, layout=layout, variant=variant,
                chunk=chunk, page=page, scale=scale)


@pytest.mark.parametrize("seed", list(range(24)))
def test_random_shape(binding, seed):
    rng = np.random.Generator(np.random.PCG64([900, seed]))
    c = random_case(rng)
    print(f"seed={seed} B={c['batch']} Hkv={c['hkv']} G={c['group']} lens[max]={int(c['lens'].max(initial=0))} "
          f"paged={c['paged']} page={c['page']} layout={c['layout']} variant={c['variant']} chunk={c['chunk']} "
          f"scale={c['scale']:.4f}", flush=True)
    hq = c["hkv"] * c["group"]
    if c["paged"]:
        width = max(-(-int(c["lens"].max(initial=0)) // c["page"]), 1) + int(rng.integers(0, 3))
        w = wl.make_paged(f"rand{seed}", 1000 + seed, c["batch"], hq, c["hkv"], c["lens"], page_size=c["page"],
                          table_width=width, layout=c["layout"], scale=c["scale"])
    else:
        cache = max(int(c["lens"].max(initial=0)), 1) + int(rng.integers(0, 40))
        w = wl.make_contiguous(f"rand{seed}", 1000 + seed, c["batch"], hq, c["hkv"], c["lens"], cache_len=cache,
                               layout=c["layout"], scale=c["scale"])
    out, lse = binding.run_workload(w, chunk_tokens=c["chunk"], kernel_variant=c["variant"],
                                    use_host_lens=bool(seed % 2))
    check(w, out, lse, oracle_of(w), f"rand{seed}")
