"""Seeded random shapes through the whole decode step on the GPU against the CPU oracle:
batch, heads, group size, sequence length (1 to 6000, log-uniform), rank d (any multiple of a
16-byte chunk, so both the matrix-core and the vector scoring kernels are hit), k, storage
type, select mode, ragged or uniform lengths, with or without the folded append, cache
capacity beyond S, and the kernel sequence (library's choice, split, fused where allowed)."""
import numpy as np
import pytest

from paper_2406_02542_amd import api, synth
from tests.test_gpu_step import run_step_case

pytestmark = pytest.mark.gpu


def random_case(seed):
    rng = np.random.default_rng(77000 + seed)
    dtype = "bf16" if rng.random() < 0.7 else "f32"
    G = int(rng.choice([1, 1, 2, 4, 8]))
    Hkv = int(rng.integers(1, 4))
    B = int(rng.integers(1, 6))
    S = int(np.exp(rng.uniform(0.0, np.log(6000.0))))
    step = 8 if dtype == "bf16" else 4
    d = int(rng.integers(1, 128 // step + 1)) * step
    k = int(rng.integers(1, S + 1))
    mode = int(rng.integers(0, 2))
    ragged = bool(rng.integers(0, 2))
    append = bool(rng.integers(0, 2))
    S_cap = S + int(rng.integers(0, 40))
    w = synth.Workload(f"rand{seed}", B, G * Hkv, Hkv, 128, S, dtype, d, k, seed=88000 + seed)
    paths = [0, api.PATH_SPLIT]
    if G == 1 and k <= 2048:
        paths.append(api.PATH_FUSED)
    path = int(rng.choice(paths))
    return w, mode, ragged, append, path, S_cap


@pytest.mark.parametrize("seed", range(32))
def test_random_shape(seed):
    w, mode, ragged, append, path, S_cap = random_case(seed)
    run_step_case(w, mode, ragged, append, path=path, S_cap=S_cap)


def random_grouped_case(seed):
    """Shapes the single-launch grouped-query kernel accepts (bf16, one selection per KV group,
    d in {16, 32, 64}, up to 16384 rows, k <= 2048), with every option it has."""
    rng = np.random.default_rng(99000 + seed)
    G = int(rng.choice([2, 4, 8]))
    Hkv = int(rng.integers(1, 4))
    B = int(rng.integers(1, 5))
    S = int(np.exp(rng.uniform(0.0, np.log(16384.0))))
    d = int(rng.choice([16, 32, 64]))
    k = int(rng.integers(1, min(S, 2048) + 1))
    ragged = bool(rng.integers(0, 2))
    append = bool(rng.integers(0, 2))
    page_rows = int(rng.choice([0, 0, 256, 512, 1024]))
    S_cap = None if page_rows else S + int(rng.integers(0, 40))
    w = synth.Workload(f"rand_g{seed}", B, G * Hkv, Hkv, 128, S, "bf16", d, k, seed=99500 + seed)
    return w, ragged, append, S_cap, page_rows


def random_cluster_case(seed):
    """Shapes the launch with several blocks per unit accepts (bf16, one selection per KV group,
    d in {16, 32, 64}, at most 128 units, slices of at most 16384 rows), with every option it has:
    1 to 60000 rows, so that slices run from a single row (and empty ones) to several thousand."""
    rng = np.random.default_rng(123000 + seed)
    G = int(rng.choice([2, 4, 8]))
    Hkv = int(rng.choice([1, 2, 3, 8]))
    B = int(rng.integers(1, 6))
    S = int(np.exp(rng.uniform(0.0, np.log(60000.0))))
    d = int(rng.choice([16, 32, 64]))
    k = int(rng.integers(1, min(S, 6000) + 1))
    ragged = bool(rng.integers(0, 2))
    append = bool(rng.integers(0, 2))
    page_rows = int(rng.choice([0, 0, 1024, 2048]))  # (at most 64 pages per sequence)
    S_cap = None if page_rows else S + int(rng.integers(0, 40))
    w = synth.Workload(f"rand_c{seed}", B, G * Hkv, Hkv, 128, S, "bf16", d, k, seed=123500 + seed)
    return w, ragged, append, S_cap, page_rows


@pytest.mark.parametrize("seed", range(20))
def test_random_shape_grouped_cluster(seed):
    w, ragged, append, S_cap, page_rows = random_cluster_case(seed)
    run_step_case(w, 1, ragged, append, path=api.PATH_CLUSTER, S_cap=S_cap, page_rows=page_rows)


@pytest.mark.parametrize("seed", range(24))
def test_random_shape_grouped_single_kernel(seed):
    w, ragged, append, S_cap, page_rows = random_grouped_case(seed)
    run_step_case(w, 1, ragged, append, path=api.PATH_FUSED, S_cap=S_cap, page_rows=page_rows)
