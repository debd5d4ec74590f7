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
