"""GPU parity on seeded random configurations: the decode step, the prompt-encoding attention and the projections,
each through the runners of the hand-picked tests, on shapes nobody picked: layer counts and warmup placements,
head counts and group sizes, both head dimensions, batch sizes that are not multiples of anything, ragged lengths
with zeros and page edges, contiguous and paged caches, both pairing rules, forced split sizes.  The seeds are
fixed, so every run sees the same cases."""
import os

import numpy as np
import pytest

from paper_2405_10637_amd import synth

from test_gpu_parity_small import run_case
from test_gpu_prefill import run_prefill
from test_gpu_project import run_project

pytestmark = pytest.mark.gpu

# more cases on demand: LCKV_RANDOM_CASES=10 multiplies the number of seeds by 10
MORE = int(os.environ.get("LCKV_RANDOM_CASES", "1"))


def random_workload(rng, name, dtype=None, max_B=9):
    L = int(rng.integers(1, 7))
    warm = tuple(int(l) for l in np.flatnonzero(rng.random(L) < 0.35))
    if len(warm) == L and L > 1 and rng.random() < 0.7:           # mostly keep at least one condensed layer
        warm = warm[:-1]
    Hkv = int(rng.choice([1, 2, 3, 4]))
    G = int(rng.choice([1, 1, 2, 4, 8]))
    D = int(rng.choice([64, 128]))
    B = int(rng.integers(1, max_B + 1))
    dtype = dtype or ("bf16" if rng.random() < 0.8 else "f32")
    return synth.Workload(name, dtype, L=L, w=len(warm), Hq=Hkv * G, Hkv=Hkv, D=D, B=B, T=1, sigma=1.0,
                          seed=int(rng.integers(1, 1 << 30)), paged=bool(rng.random() < 0.5), warm=warm)


def random_lens(rng, B, top):
    special = [0, 1, 15, 16, 17, 31, 32, 33, top - 1, top]
    return np.array([int(rng.choice(special)) if rng.random() < 0.4 else int(rng.integers(0, top + 1))
                     for _ in range(B)], np.int32)


@pytest.mark.parametrize("seed", range(16 * MORE))
def test_decode_step_random_config(seed):
    rng = np.random.default_rng(9000 + seed)
    wl = random_workload(rng, "rnd-decode-%d" % seed)
    top = int(rng.choice([40, 100, 200]))
    lens = random_lens(rng, wl.B, top)
    split = int(rng.choice([0, 16, 32, 64]))
    rule = int(rng.integers(0, 2))
    waves = int(rng.choice([0, 0, 4, 8, 16]))                      # workgroup width of the bf16 kernel (fp32 ignores it)
    run_case(wl.with_(T=top), lens, top + 8, rule=rule, split_tokens=split, steps=2, waves=waves)


@pytest.mark.parametrize("seed", range(12 * MORE))
def test_prefill_random_config(seed):
    rng = np.random.default_rng(9100 + seed)
    wl = random_workload(rng, "rnd-prefill-%d" % seed, max_B=4)
    S = int(rng.choice([24, 70, 129, 200, 300]))
    lens = np.minimum(random_lens(rng, wl.B, S), S)
    tile = int(rng.choice([0, 2, 4])) if wl.dtype == "bf16" else 0
    run_prefill(wl.with_(T=S), S, lens, tile=tile, T_cap=(S + 15) // 16 * 16)


@pytest.mark.parametrize("seed", range(10 * MORE))
def test_projection_random_config(seed):
    rng = np.random.default_rng(9200 + seed)
    wl = random_workload(rng, "rnd-project-%d" % seed, max_B=int(rng.choice([4, 40, 140])))
    hidden = int(rng.choice([256, 512, 768])) if wl.dtype == "bf16" else int(rng.choice([40, 96, 256]))
    top = 40
    lens = np.minimum(random_lens(rng, wl.B, top), top - 1)      # the new token needs a free position
    run_project(wl.with_(T=top), hidden, lens, 48, rope_base=float(rng.choice([10000.0, 500000.0, 0.0])))


@pytest.mark.parametrize("seed", range(8 * MORE))
def test_sink_window_policy_random_config(seed):
    from test_gpu_streaming import run_streaming
    rng = np.random.default_rng(9300 + seed)
    wl = random_workload(rng, "rnd-stream-%d" % seed, max_B=4)
    sink = int(rng.choice([0, 1, 4, 7]))
    window = int(rng.choice([9, 16, 23, 40]))
    lens0 = np.minimum(random_lens(rng, wl.B, sink + window), sink + window)
    steps = int(rng.integers(window + 2, 3 * window))               # past the capacity: the ring wraps
    run_streaming(wl.with_(T=sink + window), sink, window, lens0, steps, rule=int(rng.integers(0, 2)),
                  split_tokens=int(rng.choice([0, 16])))
