"""GPU parity on seeded random tensors of many families and sizes: the whole pipeline against the
oracle, element by element (the same checks as tests/test_gpu_parity.py)."""
import numpy as np
import pytest
import torch

from paper_2306_11800_amd import synth
from test_gpu_parity import run_pipeline

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def ctx():
    from paper_2306_11800_amd import api
    c = api.Context(torch.device("cuda:0"))
    yield c
    c.close()


def family(rng, kind, n):
    if kind == 0:    # heavy tails
        x = 0.02 * rng.standard_t(3, n)
    elif kind == 1:  # all positive and tiny (second moments)
        x = np.abs(rng.normal(0, 1e-6, n)) ** 2
    elif kind == 2:  # all negative
        x = -np.abs(rng.normal(0, 0.3, n))
    elif kind == 3:  # huge dynamic range
        x = rng.normal(0, 1, n) * np.exp2(rng.integers(-100, 100, n))
    elif kind == 4:  # powers of two only (many equal values, keys on bin edges)
        x = np.exp2(rng.integers(-12, 4, n)) * rng.choice([-1.0, 1.0], n)
    elif kind == 5:  # mostly zeros of both signs
        x = rng.normal(0, 1e-3, n)
        x[rng.random(n) < 0.9] = 0.0
        x[rng.random(n) < 0.05] = -0.0
    elif kind == 6:  # denormals next to ordinary values
        x = rng.normal(0, 1, n)
        tiny = rng.random(n) < 0.3
        x[tiny] = rng.normal(0, 1e-41, int(tiny.sum()))
    elif kind == 7:  # a ramp with a few outliers
        x = np.linspace(-1, 1, n)
        x[rng.integers(0, n, max(1, n // 500))] *= 1000.0
    elif kind == 8:  # quantised to a coarse lattice: long runs of equal values
        x = np.round(rng.normal(0, 1, n) * 8) / 8
    else:            # two far clusters
        x = np.where(rng.random(n) < 0.5, rng.normal(-5, 0.01, n), rng.normal(7, 1e-4, n))
    return x.astype(np.float32)


def step(rng, x, kind):
    y = x.copy()
    m = rng.random(x.size) < (0.3 if kind % 2 else 1.0)
    y[m] = (y[m] * (1 + rng.normal(0, 1e-3, int(m.sum())))).astype(np.float32)
    return y


@pytest.mark.parametrize("seed", [101, 102, 103])
def test_families_full_grid(ctx, seed):
    rng = np.random.default_rng(seed)
    sizes = [int(s) for s in rng.choice([3, 130, 1023, 4097, 12289, 16385, 40_000, 65_537, 131_072,
                                         200_003], 10, replace=False)]
    prevs = [family(rng, k, n) for k, n in enumerate(sizes)]
    curs = [step(rng, x, k) for k, x in enumerate(prevs)]
    run_pipeline(ctx, prevs, curs, synth.grid_full(), synth.EPS_DEFAULT, want_perm=(seed % 2 == 1))


def test_chunk_boundaries_of_the_delta(ctx):
    """Sizes around one delta chunk (64 tiles of 12288 elements) and one tile."""
    rng = np.random.default_rng(104)
    sizes = [786_431, 786_432, 786_433, 12_287, 12_288, 24_577]
    prevs = [family(rng, k % 3, n) for k, n in enumerate(sizes)]
    curs = [step(rng, x, k) for k, x in enumerate(prevs)]
    run_pipeline(ctx, prevs, curs, synth.grid_small(), synth.EPS_DEFAULT, want_perm=False)


@pytest.mark.parametrize("mode", ["sampled", "sampled_all_missed"])
def test_sampled_first_sweep(mode, monkeypatch):
    """Large tensors read one tile in eight in the first sweep and predict where the thresholds
    fall; INSHR_SAMPLE_MIN_N=1 does that for every tensor, INSHR_SAMPLE_FORCE_MISS=1 treats every
    prediction as wrong (both exact sweeps are then repeated).  The last tensor's sampled tiles are
    a hundred times larger than the others, so its predictions are wrong by themselves.  Results
    must not depend on any of this."""
    import os
    from paper_2306_11800_amd import api
    env = {"INSHR_SAMPLE_MIN_N": "1"}
    if mode == "sampled_all_missed":
        env["INSHR_SAMPLE_FORCE_MISS"] = "1"
    with monkeypatch.context() as m:  # (whatever the variables were before comes back afterwards)
        for k, v in env.items():
            m.setenv(k, v)
        c = api.Context(torch.device("cuda:0"))
    rng = np.random.default_rng(105)
    sizes = [5, 16_384, 40_000, 131_072, 200_003, 300_001, 16_384 * 24 + 77]
    prevs = [family(rng, k, n) for k, n in zip([0, 5, 3, 6, 8, 9, 0], sizes)]
    biased = prevs[-1].reshape(-1)
    for tile in range(0, biased.size // 16_384, 8):
        biased[tile * 16_384:(tile + 1) * 16_384] *= 100.0
    curs = [step(rng, x, k) for k, x in enumerate(prevs)]
    run_pipeline(c, prevs, curs, synth.grid_full(), synth.EPS_DEFAULT, want_perm=False)
    # a NaN / an Inf in a tile that the sampled sweep does not read is still found
    for bad in (np.nan, np.inf, -np.inf):
        x = prevs[3].copy()
        x[3 * 16_384 + 5] = bad
        with pytest.raises(api.InshrError) as e:
            c.search([torch.from_numpy(x).to("cuda:0")], synth.grid_small(), synth.EPS_DEFAULT)
        assert e.value.code == -3
    c.close()
