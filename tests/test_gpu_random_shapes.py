"""Randomised packed shapes: many clips of arbitrary lengths (including empty and one-token
clips, lengths around every tile size), odd head counts, both head dims; the whole
rope -> forward -> backward path against the oracle."""
import numpy as np
import pytest

from paper_2503_12964_amd import workloads as W
from tests import parity_utils as U
from tests.test_gpu_parity import _assert_parity, _run_fwd_bwd

pytestmark = pytest.mark.gpu


def _random_workload(seed):
    rng = np.random.default_rng(seed)
    hd = (64, 128)[seed % 2]
    heads = int(rng.choice([1, 3, 5]))
    n_clips = int(rng.integers(3, 40))
    grids = []
    for _ in range(n_clips):
        kind = rng.integers(0, 6)
        if kind == 0:
            grids.append((0, 1, 1))                               # empty clip
        elif kind == 1:
            grids.append((1, 1, 1))                               # one token
        elif kind == 2:                                           # around a tile boundary
            n = int(rng.choice([31, 32, 33, 63, 64, 65, 127, 128, 129, 255, 256, 257]))
            grids.append((1, 1, n))
        else:
            grids.append((int(rng.integers(1, 5)), int(rng.integers(1, 13)), int(rng.integers(1, 13))))
    dims = (16, 24, 24) if hd == 64 else (32, 48, 48)
    return W.Workload(f"rand{seed}", tuple(grids), heads, hd, dims, seed=100 + seed)


@pytest.mark.parametrize("seed", range(8))
def test_random_packed_shapes(seed):
    wl = _random_workload(seed)
    if wl.total_tokens == 0:
        pytest.skip("all clips empty")
    gpu, host = _run_fwd_bwd(wl, rope=True)
    # short clips make outputs O(|v|): bound the absolute error relative to max(1, |ref|)
    _assert_parity(wl, gpu, host, relative_maxabs=True)


def _random_long_workload(seed):
    """A few clips of arbitrary length up to 6,000 tokens (many ring turns and every remainder of
    the unrolled loops), some of them empty, tiny, or a token or two around a tile multiple."""
    rng = np.random.default_rng(1000 + seed)
    hd = 128 if seed % 4 else 64
    grids = []
    for _ in range(int(rng.integers(1, 12))):
        kind = rng.integers(0, 5)
        if kind == 0:
            n = int(rng.integers(0, 3))
        elif kind == 1:
            n = int(rng.choice([32, 64, 96, 128, 192, 256, 384, 512, 768, 1024])) + int(rng.integers(-2, 3))
        else:
            n = int(rng.integers(1, 6000))
        grids.append((1, 1, n) if n else (0, 1, 1))
    dims = (16, 24, 24) if hd == 64 else (32, 48, 48)
    return W.Workload(f"long{seed}", tuple(grids), int(rng.choice([1, 2, 3])), hd, dims, seed=5000 + seed)


@pytest.mark.parametrize("seed", [201, 203, 228, 237])
def test_random_long_clips(seed):
    wl = _random_long_workload(seed)
    gpu, host = _run_fwd_bwd(wl, rope=True)
    _assert_parity(wl, gpu, host, relative_maxabs=True)


def test_maximum_number_of_clips():
    # 256 clips (the table's capacity) of 1..40 tokens
    rng = np.random.default_rng(7)
    grids = tuple((1, 1, int(n)) for n in rng.integers(1, 41, size=256))
    wl = W.Workload("max_clips", grids, 2, 128, (32, 48, 48), seed=77)
    gpu, host = _run_fwd_bwd(wl, rope=True)
    _assert_parity(wl, gpu, host, relative_maxabs=True)
