"""GPU parity at the benchmark's full sizes, in the same launch configuration bench.py
times.  The oracle recomputes a sample of (batch, KV head) units one by one; properties
that hold at any size (index validity, ordering) are checked on every unit."""
import numpy as np
import pytest

import torch

from oracle import loki_oracle as O
from paper_2406_02542_amd import api, synth
from tests.parity import OUT_TOL, TORCH_DT, DeviceCase, check_dense, check_loki, check_out

pytestmark = pytest.mark.gpu


def say(msg):
    print(msg, flush=True)


def _sample_units(w, n, seed=0):
    rng = np.random.default_rng(seed)
    all_units = [(b, h) for b in range(w.B) for h in range(w.Hkv)]
    pick = rng.choice(len(all_units), size=min(n, len(all_units)), replace=False)
    units = [all_units[i] for i in sorted(pick)]
    # always include the first and the last unit (grid edges)
    for u in (all_units[0], all_units[-1]):
        if u not in units:
            units.append(u)
    return units


def _all_index_sets_valid(idx, S):
    idx = idx.astype(np.int64)
    assert idx.min() >= 0 and idx.max() < S
    assert np.all(np.diff(idx, axis=-1) > 0)


@pytest.mark.parametrize("name,modes,n_units", [
    ("llama2_7b", (0,), 24),
    ("llama3_8b_gqa", (0, 1), 8),
    ("long_gqa", (0, 1), 3),
])
def test_full_size_config(name, modes, n_units):
    w = synth.paper_configs()[name]
    say(f"generating {w}")
    x = synth.make_inputs(w, threads=16)
    case = DeviceCase(w, x)
    units = _sample_units(w, n_units, seed=len(name))
    for mode in modes:
        out, idx = case.run_loki(mode)
        _all_index_sets_valid(idx, w.S)
        assert np.all(np.isfinite(out))
        say(f"{name} mode {mode}: {check_loki(case, mode, units=units, out_gpu=out, idx_gpu=idx)}")
        if w.G == 1:
            # the library's choice above is the one-kernel path; pin the split path too
            out2, idx2 = case.run_loki(mode, path=api.PATH_SPLIT)
            assert np.array_equal(idx, idx2)
            say(f"{name} mode {mode} split path: "
                f"{check_loki(case, mode, units=units, out_gpu=out2, idx_gpu=idx2)}")
        elif mode == 1:
            # grouped heads, one selection per group, 128 / 32 units: the library's choice is the
            # single launch with 2 / 8 cooperating blocks per unit; pin every sequence that takes
            # the shape and require the same index lists
            others = [("split", api.PATH_SPLIT)] + ([("one block per unit", api.PATH_FUSED)] if w.S <= 16384 else [])
            for label, p in others:
                out2, idx2 = case.run_loki(mode, path=p)
                assert np.array_equal(idx, idx2)
                say(f"{name} mode 1, {label}: "
                    f"{check_loki(case, mode, units=units, out_gpu=out2, idx_gpu=idx2)}")
            out3, idx3 = case.run_loki(mode, path=api.PATH_CLUSTER)
            assert np.array_equal(idx, idx3) and np.array_equal(out, out3)
    out = case.run_dense()
    assert np.all(np.isfinite(out))
    say(f"{name} dense: {check_dense(case, units=units[:4], out_gpu=out)}")
    # Appendix E, Algorithm 2 at the same size (grouped heads: the matrix-core kernel)
    lay = case.layout
    ws = torch.empty(api.loki_workspace_bytes(lay, w.S, w.d, 0, -2), dtype=torch.uint8, device="cuda")
    outp = torch.full((w.B, w.Hq, w.D), float("nan"), dtype=TORCH_DT[w.dtype], device="cuda")
    api.loki_pca_attn(lay, case.q, case.P, case.klo, case.v, w.S, w.d, ws, outp)
    torch.cuda.synchronize()
    got = outp.float().cpu().numpy().astype(np.float64)
    assert np.all(np.isfinite(got))
    ref = O.pca_attention_batch(x["q"], x["P"], x["khat"], x["v"], w.d, units=units[:4])
    worst = 0.0
    for b, h in units[:4]:
        for hq in range(h * w.G, (h + 1) * w.G):
            worst = max(worst, check_out(got[b, hq], ref[b, hq], w.dtype, f"{name} PCAAttn b={b} hq={hq}"))
    say(f"{name} PCAAttn: max_err {worst:.3e} over {4 * w.G} heads")
    assert worst <= OUT_TOL[w.dtype]


def test_full_size_large_share_sweep():
    """Config 5: batch 64, 64 query / 8 KV heads, S=8192, d in {16,32,64} x k_f in
    {1/16, 1/8, 1/4}; the cache content is shared, the slab split is rebuilt per d."""
    base = synth.paper_configs()["large_share"]
    say(f"generating {base}")
    x = synth.make_inputs(base, threads=16)
    units = _sample_units(base, 3, seed=5)
    for d in (16, 32, 64):
        case = DeviceCase(base.replace(d=d), x)
        for k in (512, 1024, 2048):
            case.w = base.replace(d=d, k=k, name=f"large_share_d{d}_k{k}")
            for mode in (0, 1):
                out, idx = case.run_loki(mode)
                _all_index_sets_valid(idx, base.S)
                say(f"{case.w.name} mode {mode}: "
                    f"{check_loki(case, mode, units=units, out_gpu=out, idx_gpu=idx)}")
                if mode == 1:
                    # the library's choice above is the single-launch grouped-query kernel (512
                    # units); pin the split path too and require the same index lists
                    out2, idx2 = case.run_loki(mode, path=api.PATH_SPLIT)
                    assert np.array_equal(idx, idx2)
                    say(f"{case.w.name} mode 1 split path: "
                        f"{check_loki(case, mode, units=units, out_gpu=out2, idx_gpu=idx2)}")
                    out3, idx3 = case.run_loki(mode, path=api.PATH_FUSED)
                    assert np.array_equal(idx, idx3) and np.array_equal(out, out3)
        if d == 16:
            say(f"dense: {check_dense(case, units=units[:2])}")
        del case
