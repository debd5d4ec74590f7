"""GPU parity: the HIP path, called through the C ABI, against the CPU oracle on the same
seeded inputs.  Sizes here are ones the oracle finishes in seconds; they span several tiles
of every kernel and ragged tails.  Full benchmark sizes are in test_gpu_full_size.py."""
import numpy as np
import pytest
import torch

from oracle import loki_oracle as O
from paper_2406_02542_amd import api, synth
from tests.parity import (DeviceCase, OUT_TOL, TORCH_DT, check_dense, check_loki, gqa_single_kernel_ok,
                          to_dev)

pytestmark = pytest.mark.gpu


def _case(name, B, Hq, Hkv, S, dtype, d, k, **kw):
    w = synth.Workload(name, B, Hq, Hkv, 128, S, dtype, d, k, **kw)
    return w, synth.make_inputs(w)


def say(msg):
    print(msg, flush=True)


# ------------------------------------------------------------------ whole path --
def test_tiny_config_fp32():
    """Config 1: batch 1, 8 heads, S=1024, fp32, d=32, k=256."""
    w = synth.paper_configs()["tiny"]
    say(f"case {w}")
    case = DeviceCase(w, synth.make_inputs(w))
    for path in (0, api.PATH_SPLIT, api.PATH_FUSED):
        st = check_loki(case, 0, path=path)
        say(f"loki path {path:#x} {st}")
        assert st["max_err"] <= 1e-5
    say(f"dense {check_dense(case)}")


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
@pytest.mark.parametrize("shape", [
    # (B, Hq, Hkv, S, d, k)
    (2, 4, 4, 1500, 32, 300),     # MHA, ragged S, several score/select tiles
    (1, 8, 2, 3001, 16, 517),     # GQA G=4, odd sizes
    (1, 8, 1, 2048, 64, 256),     # GQA G=8
    (3, 2, 1, 700, 32, 699),      # G=2, k = S-1
])
@pytest.mark.parametrize("mode", [0, 1])
def test_loki_matches_oracle(dtype, shape, mode):
    B, Hq, Hkv, S, d, k = shape
    w, x = _case(f"p_{dtype}_{S}", B, Hq, Hkv, S, dtype, d, k, seed=1000 + S + d)
    say(f"case {w} mode {mode}")
    case = DeviceCase(w, x, S_cap=S + 37)  # capacity larger than the live rows
    say(f"loki {check_loki(case, mode)}")
    say(f"loki split {check_loki(case, mode, path=api.PATH_SPLIT)}")
    if Hq == Hkv:
        say(f"loki fused {check_loki(case, mode, path=api.PATH_FUSED)}")
    elif gqa_single_kernel_ok(w, mode):
        say(f"loki grouped single-kernel {check_loki(case, mode, path=api.PATH_FUSED)}")


@pytest.mark.parametrize("shape", [
    # (B, Hq, Hkv, S, d, k)
    (2, 8, 2, 4096, 32, 1024),    # G=4: 16 keys per thread in the select stage
    (1, 16, 2, 8192, 16, 2048),   # G=8: 32 keys per thread, largest index list
    (1, 8, 1, 8190, 64, 511),     # G=8, two loads per row tile, ragged tail
    (2, 4, 2, 16384, 32, 2048),   # G=2: the 512-thread form (one block per CU)
    (1, 8, 2, 12001, 16, 1500),   # 512-thread form, odd length
    (1, 4, 1, 5, 32, 3),          # fewer rows than one wave step
    (1, 8, 1, 33, 64, 33),        # k = S
])
def test_grouped_single_kernel_matches_oracle_and_split_path(shape):
    """One selection per KV group in one launch (grouped heads, bf16): against the oracle, and
    the same index lists as the split path."""
    B, Hq, Hkv, S, d, k = shape
    w, x = _case(f"gq_{S}_{d}", B, Hq, Hkv, S, "bf16", d, k, seed=1500 + S + d + k)
    say(f"case {w}")
    assert gqa_single_kernel_ok(w, 1)
    case = DeviceCase(w, x, S_cap=S + 11)
    of, jf = case.run_loki(1, path=api.PATH_FUSED)
    os_, js = case.run_loki(1, path=api.PATH_SPLIT)
    say(f"single kernel {check_loki(case, 1, out_gpu=of, idx_gpu=jf)}")
    say(f"split {check_loki(case, 1, out_gpu=os_, idx_gpu=js)}")
    assert np.array_equal(jf, js)
    assert np.max(np.abs(of - os_)) <= 8e-3


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
def test_dense_matches_oracle(dtype):
    for (B, Hq, Hkv, S) in [(2, 4, 4, 1500), (1, 8, 2, 3001), (1, 8, 1, 2048), (2, 2, 1, 77)]:
        w, x = _case(f"dn_{dtype}_{S}", B, Hq, Hkv, S, dtype, 32, 1, seed=2000 + S)
        say(f"case {w}")
        say(f"dense {check_dense(DeviceCase(w, x, S_cap=S + 5))}")


# ------------------------------------------------------------------- edge cases --
@pytest.mark.parametrize("dtype", ["f32", "bf16"])
@pytest.mark.parametrize("S,d,k", [
    (1, 32, 1),         # a single cached token
    (2, 32, 2),
    (65, 32, 64),       # one row past a wave tile
    (257, 8, 1),        # k = 1; one 16-byte chunk per slab row in bf16
    (1000, 128, 100),   # d = D: the Exact-TopK case, empty residual slab
    (1000, 96, 250),    # slab row is not a power-of-two number of chunks
    (640, 32, 640),     # k = S: equals dense attention
    (5000, 32, 4999),
])
def test_edge_shapes(dtype, S, d, k):
    w, x = _case(f"e_{dtype}_{S}_{d}", 1, 4, 2, S, dtype, d, k, seed=3000 + S + d + k)
    say(f"case {w}")
    case = DeviceCase(w, x)
    for mode in (0, 1):
        say(f"mode {mode} {check_loki(case, mode)}")
    if k == S:
        # k = S: Loki equals dense attention of the same q over the unrotated keys
        # K = Khat P^T (Lemma 4.1), whatever d is
        out, _ = case.run_loki(0)
        K = np.einsum("bhsj,hij->bhsi", x["khat"].astype(np.float64), x["P"].astype(np.float64))
        dn = O.dense_decode_batch(x["q"], K, x["v"])
        from tests.parity import check_out
        check_out(out, dn, dtype, "k = S against dense attention over the unrotated keys")


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
@pytest.mark.parametrize("S,d,k", [
    (1, 32, 1), (2, 32, 2), (65, 32, 64), (257, 8, 1), (1000, 128, 100), (1000, 96, 250),
    (640, 32, 640), (5000, 32, 2048), (8192, 16, 2048), (8191, 64, 1),
])
def test_edge_shapes_single_kernel_and_split_paths(dtype, S, d, k):
    """Hq == Hkv: the same shapes through the one-kernel path and through the split path;
    the selected sets must be identical and the outputs agree to fp32 rounding."""
    w, x = _case(f"f_{dtype}_{S}_{d}", 2, 3, 3, S, dtype, d, k, seed=3500 + S + d + k)
    say(f"case {w}")
    case = DeviceCase(w, x)
    of, jf = case.run_loki(0, path=api.PATH_FUSED)
    os_, js = case.run_loki(0, path=api.PATH_SPLIT)
    say(f"fused {check_loki(case, 0, out_gpu=of, idx_gpu=jf)}")
    say(f"split {check_loki(case, 0, out_gpu=os_, idx_gpu=js)}")
    assert np.array_equal(jf, js)
    assert np.max(np.abs(of - os_)) <= (1e-6 if dtype == "f32" else 8e-3)


def test_single_kernel_path_limits():
    """Pinning the one-kernel path outside its limits is refused, not silently rerouted."""
    for (Hq, Hkv, S, k, mode) in [(4, 2, 512, 64, 0), (2, 2, 8193, 64, 0), (2, 2, 8192, 2049, 0),
                                  (4, 2, 16385, 64, 1), (4, 2, 4096, 2049, 1)]:
        w, x = _case("lim", 1, Hq, Hkv, S, "bf16", 32, k, seed=3600)
        case = DeviceCase(w, x)
        with pytest.raises(api.LokiError) as e:
            case.run_loki(mode, path=api.PATH_FUSED)
        assert e.value.status == 2
        check_loki(case, mode)  # the default route still works


@pytest.mark.parametrize("S,k,G", [
    (8193, 700, 1),      # just past the one-kernel limit: 1024-thread register-resident select
    (16384, 2048, 2),
    (16385, 1000, 1),    # first size of the streaming select, S % 4 != 0
    (20000, 1250, 4),
    (50001, 3000, 1),
    (70000, 35000, 2),   # half of everything selected
])
def test_long_sequences(S, k, G):
    w, x = _case(f"long_{S}", 1, 2 * G, 2, S, "bf16", 16, k, seed=3700 + S)
    say(f"case {w}")
    case = DeviceCase(w, x)
    for mode in ((0, 1) if G > 1 else (0,)):
        say(f"mode {mode} {check_loki(case, mode)}")


@pytest.mark.parametrize("S", [1100000, 1100001])
def test_sequence_beyond_the_chunked_select(S):
    """More than 64 chunks of 16384 rows: one block per head streams the scores four times
    (select_stream_kernel), with and without 16-byte-aligned score rows."""
    w, x = _case(f"huge_{S}", 1, 1, 1, S, "bf16", 16, 5000, seed=3900 + S % 7)
    say(f"case {w}")
    say(f"{check_loki(DeviceCase(w, x), 0)}")


def test_long_sequence_with_massive_ties():
    """S = 40000 with an all-zero cache and with only 7 distinct key rows: the threshold bin
    overflows every candidate buffer, the plain digit passes must take over."""
    w, x = _case("long_ties", 1, 2, 2, 40000, "f32", 32, 17001, seed=3800)
    x0 = dict(x)
    x0["khat"] = np.zeros_like(x["khat"])
    out, idx = DeviceCase(w, x0).run_loki(0)
    for h in range(2):
        assert idx[0, h].tolist() == list(range(17001))
    x7 = dict(x)
    x7["khat"] = np.tile(x["khat"][:, :, :7, :], (1, 1, 40000 // 7 + 1, 1))[:, :, :40000, :].copy()
    case = DeviceCase(w, x7)
    st = check_loki(case, 0)
    say(f"7 distinct rows: {st}")
    assert st["heads_with_swaps"] == 0


def test_ties_go_to_lowest_position():
    """All-zero cache: every score ties, the first k positions must be selected and the
    output is the mean of the first k value rows.  Then planted duplicate rows."""
    w, x = _case("ties", 1, 2, 2, 3000, "f32", 32, 1100, seed=4000)
    x0 = dict(x)
    x0["khat"] = np.zeros_like(x["khat"])
    case = DeviceCase(w, x0)
    for path in (api.PATH_SPLIT, api.PATH_FUSED):
        out, idx = case.run_loki(0, path=path)
        for h in range(2):
            assert idx[0, h].tolist() == list(range(1100))
            np.testing.assert_allclose(out[0, h],
                                       x["v"][0, h, :1100].astype(np.float64).mean(axis=0), atol=1e-5)
    # duplicates: rows 100.. are copies of rows 0..99 cyclically, so every score has 30 equals
    xd = dict(x)
    kd = x["khat"].copy()
    kd[:, :, 100:, :] = np.tile(kd[:, :, :100, :], (1, 1, 29, 1))
    xd["khat"] = kd
    case = DeviceCase(w, xd)
    out, idx = case.run_loki(0, path=api.PATH_SPLIT)
    outf, idxf = case.run_loki(0, path=api.PATH_FUSED)
    assert np.array_equal(idx, idxf)
    # equal rows give bit-identical GPU scores, so the tie rule decides: sets must be exact
    # unless rows of *different* value fall within rounding of each other at the threshold
    st = check_loki(case, 0, out_gpu=out, idx_gpu=idx)
    say(f"duplicates {st}")
    for h in range(2):
        sel = set(idx[0, h].tolist())
        for p in idx[0, h].tolist():
            base = p % 100
            lower = [base + 100 * j for j in range((p - base) // 100)]
            # if a copy at position p is selected, all its earlier copies are selected too
            assert all(lp in sel for lp in lower)


@pytest.mark.parametrize("S,k", [(3000, 1100), (8192, 2048), (12000, 900)])
def test_grouped_single_kernel_ties(S, k):
    """The single-launch grouped-query kernel with equal scores: an all-zero cache (the threshold
    bin holds every row: its candidate list overflows and the plain selection over all keys takes
    over), planted duplicates (30 equal rows per score: the candidate-list route with ties inside
    it), and a cache whose rows take 7 distinct values.  Lowest position wins; the index lists must
    equal the split path's."""
    w, x = _case(f"gq_ties_{S}", 1, 8, 2, S, "bf16", 32, k, seed=4100 + S)
    x0 = dict(x)
    x0["khat"] = np.zeros_like(x["khat"])
    out, idx = DeviceCase(w, x0).run_loki(1, path=api.PATH_FUSED)
    for h in range(2):
        assert idx[0, h].tolist() == list(range(k))
    for reps in (100, 7):
        xd = dict(x)
        kd = x["khat"].copy()
        kd[:, :, reps:, :] = np.tile(kd[:, :, :reps, :], (1, 1, S // reps + 1, 1))[:, :, :S - reps, :]
        xd["khat"] = kd
        case = DeviceCase(w, xd)
        outs, idxs = case.run_loki(1, path=api.PATH_SPLIT)
        outf, idxf = case.run_loki(1, path=api.PATH_FUSED)
        assert np.array_equal(idxs, idxf)
        st = check_loki(case, 1, out_gpu=outf, idx_gpu=idxf)
        say(f"{reps} distinct rows: {st}")
        assert st["heads_with_swaps"] == 0


@pytest.mark.parametrize("shape", [(1, 8, 2, 3000, 32, 500), (4, 32, 8, 4000, 32, 700), (2, 16, 8, 2500, 16, 300),
                                   (16, 16, 8, 6000, 64, 1000), (3, 8, 4, 1000, 32, 1000),
                                   (1, 16, 2, 20000, 32, 2500), (2, 8, 1, 50000, 16, 4000)])
def test_cluster_matches_oracle_and_split_path(shape):
    """The launch with several blocks per unit (2, 4 or 8, by the number of units): outputs against
    the oracle, index lists identical to the split path's (the same matrix-core scoring)."""
    B, Hq, Hkv, S, d, k = shape
    w, x = _case(f"cluster_{Hq}_{Hkv}_{S}", B, Hq, Hkv, S, "bf16", d, k, seed=7000 + S)
    case = DeviceCase(w, x)
    outc, idxc = case.run_loki(1, path=api.PATH_CLUSTER)
    _, idxs = case.run_loki(1, path=api.PATH_SPLIT)
    assert np.array_equal(idxc, idxs)
    st = check_loki(case, 1, out_gpu=outc, idx_gpu=idxc)
    say(f"{w.name}: {st}")
    assert st["heads_with_swaps"] == 0


@pytest.mark.parametrize("S,k", [(3000, 1100), (12000, 900), (40000, 5000)])
def test_cluster_ties(S, k):
    """Equal scores across the blocks of a unit: an all-zero cache (every row ties: all three
    histogram exchanges run and each block takes what the blocks before it leave), planted
    duplicates (ties inside the candidate exchange) and a cache whose rows take 7 distinct
    values.  Lowest position wins; the index lists must equal the split path's."""
    w, x = _case(f"cluster_ties_{S}", 1, 8, 2, S, "bf16", 32, k, seed=4100 + S)
    x0 = dict(x)
    x0["khat"] = np.zeros_like(x["khat"])
    out, idx = DeviceCase(w, x0).run_loki(1, path=api.PATH_CLUSTER)
    for h in range(2):
        assert idx[0, h].tolist() == list(range(k))
    for reps in (100, 7):
        xd = dict(x)
        kd = x["khat"].copy()
        kd[:, :, reps:, :] = np.tile(kd[:, :, :reps, :], (1, 1, S // reps + 1, 1))[:, :, :S - reps, :]
        xd["khat"] = kd
        case = DeviceCase(w, xd)
        _, idxs = case.run_loki(1, path=api.PATH_SPLIT)
        outc, idxc = case.run_loki(1, path=api.PATH_CLUSTER)
        assert np.array_equal(idxs, idxc)
        st = check_loki(case, 1, out_gpu=outc, idx_gpu=idxc)
        say(f"{reps} distinct rows: {st}")
        assert st["heads_with_swaps"] == 0


def test_cluster_on_a_workspace_the_caller_cleared_once():
    """With LOKI_WORKSPACE_ZEROED the launch clears nothing in front: it relies on the control
    words at the start of the workspace being zero, and leaves them zero.  Calls of two shapes
    (8 and 4 blocks per unit, different numbers of units) share one cleared workspace, take
    turns ten times, and must each time equal the call that asks for nothing (bit for bit);
    calls on other kernel sequences in between write the rest of the workspace."""
    wa, xa = _case("cluster_ws_a", 1, 8, 2, 9000, "bf16", 32, 900, seed=8101)
    wb, xb = _case("cluster_ws_b", 5, 32, 8, 3000, "bf16", 16, 400, seed=8102)
    ca, cb = DeviceCase(wa, xa), DeviceCase(wb, xb)
    ref = {}
    for name, c in (("a", ca), ("b", cb)):
        ref[name] = c.run_loki(1, path=api.PATH_CLUSTER)
    n = max(api.loki_workspace_bytes(c.layout, c.w.S, c.w.d, c.w.k, 1) for c in (ca, cb))
    ws = torch.zeros(n, dtype=torch.uint8, device="cuda")
    for it in range(10):
        for name, c in (("a", ca), ("b", cb)):
            w = c.w
            out = torch.full((w.B, w.Hq, w.D), float("nan"), dtype=torch.bfloat16, device="cuda")
            idx = torch.full((w.B, w.Hkv, w.k), -7, dtype=torch.int32, device="cuda")
            api.loki_decode_attn(c.layout, c.q, c.P, c.klo, c.khi, c.v, w.S, w.d, w.k,
                                 1 | api.PATH_CLUSTER | api.WORKSPACE_ZEROED, ws, out, idx)
            if it % 3 == 1:  # another kernel sequence on the same workspace
                api.loki_decode_attn(c.layout, c.q, c.P, c.klo, c.khi, c.v, w.S, w.d, w.k,
                                     1 | api.PATH_SPLIT | api.WORKSPACE_ZEROED, ws,
                                     torch.empty_like(out), None)
            torch.cuda.synchronize()
            assert np.array_equal(out.float().cpu().numpy().astype(np.float64), ref[name][0]), (it, name)
            assert np.array_equal(idx.cpu().numpy(), ref[name][1]), (it, name)
    # the control words are zero again
    assert int(ws[:128 * 144 * 4].view(torch.int32).abs().max()) == 0


def test_cluster_wait_gives_up_cleanly():
    """The blocks of a unit wait for each other with a bounded number of polls.  With the bound
    set to one poll by the host, blocks that find a partner late give up: the launch must still
    end, and every unit's output is then either NaN (for all its heads) or the regular result.
    With the default restored the same call is regular again."""
    w, x = _case("cluster_give_up", 2, 16, 4, 20000, "bf16", 32, 2000, seed=7777)
    case = DeviceCase(w, x)
    ref, idx_ref = case.run_loki(1, path=api.PATH_CLUSTER)
    assert np.all(np.isfinite(ref))
    api.loki_debug_cluster_spin_limit(1)
    try:
        out, _ = case.run_loki(1, path=api.PATH_CLUSTER)
    finally:
        api.loki_debug_cluster_spin_limit(0)
    gave_up = 0
    for b in range(w.B):
        for h in range(w.Hkv):
            o = out[b, h * w.G:(h + 1) * w.G]
            if np.all(np.isnan(o)):
                gave_up += 1
            else:
                assert np.array_equal(o, ref[b, h * w.G:(h + 1) * w.G])
    say(f"units that gave up with a one-poll limit: {gave_up} of {w.B * w.Hkv}")
    again, idx_again = case.run_loki(1, path=api.PATH_CLUSTER)
    assert np.array_equal(again, ref) and np.array_equal(idx_again, idx_ref)

    # On a workspace the caller vouches for (LOKI_WORKSPACE_ZEROED: nothing is cleared in front of
    # a launch) a give-up leaves its mark: later launches refuse (NaN everywhere) instead of
    # trusting the flags it left behind, until the caller has zeroed the workspace again.
    ws = torch.zeros(api.loki_workspace_bytes(case.layout, w.S, w.d, w.k, 1), dtype=torch.uint8, device="cuda")

    def run_vouched():
        o = torch.full((w.B, w.Hq, w.D), float("nan"), dtype=torch.bfloat16, device="cuda")
        api.loki_decode_attn(case.layout, case.q, case.P, case.klo, case.khi, case.v, w.S, w.d, w.k,
                             1 | api.PATH_CLUSTER | api.WORKSPACE_ZEROED, ws, o, None)
        torch.cuda.synchronize()
        return o.float().cpu().numpy().astype(np.float64)

    assert np.array_equal(run_vouched(), ref)
    assert not api.loki_cluster_gave_up(ws)
    api.loki_debug_cluster_spin_limit(1)
    try:
        o1 = run_vouched()
    finally:
        api.loki_debug_cluster_spin_limit(0)
    # the library says so itself: the mark is there exactly when some unit came back as NaN
    assert api.loki_cluster_gave_up(ws) == bool(np.isnan(o1).any())
    if np.isnan(o1).any():
        assert np.all(np.isnan(run_vouched()))
        ws.zero_()
    assert np.array_equal(run_vouched(), ref)
    assert not api.loki_cluster_gave_up(ws)


def test_heavy_hitters_are_selected():
    """The peaked-attention recipe of the long-context config at reduced size: the planted
    positions carry > 90 % of the mass and must all be among the selected rows."""
    w = synth.paper_configs()["long_gqa"].replace(B=1, Hq=8, Hkv=2, S=20000, k=1250)
    x = synth.make_inputs(w)
    case = DeviceCase(w, x)
    for mode in (0, 1):
        out, idx = case.run_loki(mode)
        say(f"mode {mode} {check_loki(case, mode, out_gpu=out, idx_gpu=idx)}")
        for h in range(2):
            planted = set(synth.heavy_positions(w, h).tolist())
            for hs in (range(4 * h, 4 * h + 4) if mode == 0 else [h]):
                assert planted <= set(idx[0, hs].tolist())


def _pca_attn_gpu(case):
    w = case.w
    ws = torch.empty(api.loki_workspace_bytes(case.layout, w.S, w.d, 0, -2), dtype=torch.uint8, device="cuda")
    out = torch.full((w.B, w.Hq, w.D), float("nan"), dtype=TORCH_DT[w.dtype], device="cuda")
    api.loki_pca_attn(case.layout, case.q, case.P, case.klo, case.v, w.S, w.d, ws, out)
    torch.cuda.synchronize()
    return out.float().cpu().numpy().astype(np.float64)


@pytest.mark.parametrize("G", [4, 8])
def test_peaked_attention_grouped_heads(G):
    """Outputs of magnitude 0.1 - 1 on the matrix-core paths (grouped heads, bf16): the peaked
    recipe of the long-context workload, both select modes, the single-launch kernel, the dense
    baseline and PCAAttn, all under the bound that scales with the result."""
    w = synth.paper_configs()["long_gqa"].replace(B=2, Hq=2 * G, Hkv=2, S=6000, k=750, name=f"peaked_g{G}")
    x = synth.make_inputs(w)
    case = DeviceCase(w, x)
    for mode in (0, 1):
        say(f"G={G} mode {mode} {check_loki(case, mode, path=api.PATH_SPLIT)}")
    say(f"G={G} single kernel {check_loki(case, 1, path=api.PATH_FUSED)}")
    say(f"G={G} dense {check_dense(case)}")
    from tests.parity import check_out
    ref = O.pca_attention_batch(x["q"], x["P"], x["khat"], x["v"], w.d)
    say(f"G={G} PCAAttn max_err {check_out(_pca_attn_gpu(case), ref, 'bf16', 'PCAAttn'):.3e}")
    assert np.max(np.abs(ref)) > 0.2  # the point of the case: results are not tiny


@pytest.mark.parametrize("heavy", [False, True])
def test_scaled_bound_rejects_plausible_mistakes(heavy):
    """The bound that scales with the result tells a right matrix-core attention from a plausibly
    wrong one: the mistakes are planted in the expected value on the CPU (softmax in base 2
    without the log2(e) factor; the 32-row tile that holds the heaviest row left out), never in a
    kernel.  Gather over a
    shared selection, dense baseline and PCAAttn, 8 heads per KV head, bf16."""
    from tests.parity import out_bound
    base = synth.paper_configs()["long_gqa"] if heavy else synth.paper_configs()["llama2_7b"]
    w = base.replace(B=1, Hq=8, Hkv=1, S=4096, d=32, k=1024, name=f"mut_{heavy}")
    x = synth.make_inputs(w)
    case = DeviceCase(w, x)
    out, idx = case.run_loki(1, path=api.PATH_SPLIT)
    dn = case.run_dense()
    pc = _pca_attn_gpu(case)
    Kh, V, P = x["khat"][0, 0].astype(np.float64), x["v"][0, 0].astype(np.float64), x["P"][0]
    rows_all = np.arange(w.S)

    def attend(qvec, K, rows, scale_factor=1.0):
        logits = (K[rows] @ qvec) / np.sqrt(w.D) * scale_factor
        return O.softmax(logits) @ V[rows]

    for hq in range(w.Hq):
        qhat = O.rotate_query(x["q"][0, hq], P)
        qlo = qhat.copy(); qlo[w.d:] = 0.0
        sel = idx[0, 0].astype(np.int64)
        # (the dense baseline is given the cache as it is and the query as it is: Eq. 1 on them)
        cases = [("gather", out[0, hq], qhat, sel),
                 ("dense", dn[0, hq], x["q"][0, hq].astype(np.float64), rows_all),
                 ("PCAAttn", pc[0, hq], qlo, rows_all)]
        for name, got, qv, rows in cases:
            good = attend(qv, Kh, rows)
            assert np.all(np.abs(got - good) <= out_bound(good, "bf16")), (name, hq)
            wrong_base = attend(qv, Kh, rows, scale_factor=np.log(2.0))   # exp2 without log2(e)
            # the 32-row tile of the list that holds the row with the largest weight, left out
            t0 = int(np.argmax(Kh[rows] @ qv)) // 32 * 32
            wrong_tile = attend(qv, Kh, np.concatenate([rows[:t0], rows[t0 + 32:]]))
            for label, wrong in (("base-2 softmax", wrong_base), ("a 32-row tile left out", wrong_tile)):
                assert np.any(np.abs(got - wrong) > out_bound(wrong, "bf16")), \
                    f"{name} head {hq}: the bound accepts {label}"
    say(f"heavy={heavy}: both planted mistakes rejected on every head and path")


def test_deterministic():
    w, x = _case("det", 2, 8, 2, 4096, "bf16", 32, 1024, seed=5000)
    case = DeviceCase(w, x)
    a, ia = case.run_loki(0)
    b, ib = case.run_loki(0)
    assert np.array_equal(a, b) and np.array_equal(ia, ib)
    assert np.array_equal(case.run_dense(), case.run_dense())


def test_out_idx_optional():
    w, x = _case("noidx", 1, 4, 4, 900, "bf16", 32, 200, seed=5001)
    case = DeviceCase(w, x)
    a, _ = case.run_loki(0, want_idx=True)
    b, none = case.run_loki(0, want_idx=False)
    assert none is None and np.array_equal(a, b)


# -------------------------------------------------------------------- rotate_keys --
@pytest.mark.parametrize("dtype", ["f32", "bf16"])
def test_rotate_keys_matches_oracle(dtype):
    """Khat = K P rounded to storage.  bf16: within one unit in the last place everywhere and
    exactly equal for >= 99.9 % of the elements (fp32 accumulation against the oracle's
    float64 can only flip a rounding that sits within ~1e-6 relative of a tie).  fp32: within
    fp32 accumulation error of the float64 product."""
    w = synth.Workload("rot", 2, 4, 2, 128, 777, dtype, 32, 8, seed=6000)
    P = synth.make_P(w)
    K = synth.make_unrotated_keys(w, P)
    say(f"case {w}")
    lay = api.make_layout(w.B, w.Hq, w.Hkv, 128, w.d, 1000, TORCH_DT[dtype])
    klo, khi, _ = api.alloc_cache(lay)
    klo.fill_(5.0)
    khi.fill_(5.0)
    Pd = torch.from_numpy(P).cuda()
    # prefill of 700 rows at position 3, then appends of 1 and 76 rows
    pos = 3
    for n_new, lo in ((700, 0), (1, 700), (76, 701)):
        chunk = to_dev(K[:, :, lo:lo + n_new, :], dtype)
        api.loki_rotate_keys(lay, chunk, Pd, klo, khi, pos + lo, n_new)
    torch.cuda.synchronize()
    got = torch.cat([klo, khi], dim=-1).float().cpu().numpy().astype(np.float64)
    assert np.all(got[:, :, :pos] == 5.0) and np.all(got[:, :, pos + 777:] == 5.0)
    ref64 = O.rotate_keys_batch(K, P)
    ref = O.to_storage(ref64, dtype)
    g = got[:, :, pos:pos + 777]
    if dtype == "bf16":
        exact = np.mean(g == ref)
        # one unit in the last place of bf16 (8 significant bits) at the reference's magnitude,
        # plus the fp32 accumulation error of the 128-term dot product, which dominates for
        # elements that cancel to nearly zero: 1e-6 * sum_i |k_i| |P_ij|
        ulp = 2.0 ** (np.floor(np.log2(np.maximum(np.abs(ref), 1e-30))) - 7)
        mag = np.einsum("bhsi,hij->bhsj", np.abs(K.astype(np.float64)), np.abs(P.astype(np.float64)))
        excess = np.abs(g - ref) - (ulp * 1.0000001 + 1e-6 * mag)
        say(f"exact fraction {exact:.6f}; worst excess over (1 ulp + fp32 accumulation) {excess.max():.3e}")
        assert excess.max() <= 0
        assert exact >= 0.999
    else:
        # fp32 storage: the kernel's fp32 accumulation of 128 terms against the unrounded
        # float64 product, relative to the row norm (sqrt(128) * 2^-24 ~ 7e-7)
        err = np.abs(g - ref64) / np.linalg.norm(ref64, axis=-1, keepdims=True)
        say(f"max relative-to-row-norm error {err.max():.3e}")
        assert err.max() < 2e-6


def test_rotate_then_decode_chain():
    """K -> loki_rotate_keys -> loki_decode_attn on the GPU-rotated cache, compared with
    the oracle run on that same cache content and, through Lemma 4.1 with d = D and k = S,
    with dense attention on the unrotated keys."""
    w = synth.Workload("chain", 1, 4, 2, 128, 1200, "bf16", 32, 300, seed=7000)
    P = synth.make_P(w)
    K = synth.make_unrotated_keys(w, P)
    x = {"P": P, "q": synth.make_q(w, P), "v": synth.make_v(w)}
    lay = api.make_layout(w.B, w.Hq, w.Hkv, 128, w.d, w.S, torch.bfloat16)
    klo, khi, v = api.alloc_cache(lay)
    Pd = torch.from_numpy(P).cuda()
    api.loki_rotate_keys(lay, to_dev(K, "bf16"), Pd, klo, khi, 0, w.S)
    torch.cuda.synchronize()
    x["khat"] = torch.cat([klo, khi], dim=-1).float().cpu().numpy()
    case = DeviceCase(w, x)
    say(f"chain {check_loki(case, 0)}")
    # Lemma 4.1: full-rank, full-k Loki on the rotated cache ~ dense attention on unrotated
    # keys; the rotated cache was rounded to bf16, so allow that rounding in the logits.
    wfull = w.replace(d=128, k=w.S)
    lay2 = api.make_layout(w.B, w.Hq, w.Hkv, 128, 128, w.S, torch.bfloat16)
    klo2, _, _ = api.alloc_cache(lay2)
    api.loki_rotate_keys(lay2, to_dev(K, "bf16"), Pd, klo2, None, 0, w.S)
    ws = api.alloc_workspace(lay2, w.S, 128, w.S, 0)
    out = torch.empty((1, 4, 128), dtype=torch.bfloat16, device="cuda")
    api.loki_decode_attn(lay2, case.q, Pd, klo2, None, case.v, w.S, 128, w.S, 0, ws, out)
    torch.cuda.synchronize()
    ref = O.dense_decode_batch(x["q"], K, x["v"])
    assert np.max(np.abs(out.float().cpu().numpy() - ref)) < 3e-2
    del wfull


def test_errors_surface_as_exceptions():
    w, x = _case("err", 1, 2, 2, 128, "bf16", 32, 16, seed=8000)
    case = DeviceCase(w, x)
    ws = torch.empty(256, dtype=torch.uint8, device="cuda")
    out = torch.empty((1, 2, 128), dtype=torch.bfloat16, device="cuda")
    with pytest.raises(api.LokiError) as e:
        api.loki_decode_attn(case.layout, case.q, case.P, case.klo, case.khi, case.v, 128, 32, 16, 0,
                             ws, out)
    assert e.value.status == 4
    with pytest.raises(api.LokiError):
        api.loki_decode_attn(case.layout, case.q, case.P, case.klo, case.khi, case.v, 128, 32, 129, 0,
                             ws, out)


@pytest.mark.gpu
def test_stream_read_probe_runs():
    """The measurement aid reads a buffer (whole words and a ragged word count) without error."""
    buf = torch.arange(1 << 20, dtype=torch.int32, device="cuda")
    api.loki_stream_read(buf, buf.numel() * 4)
    api.loki_stream_read(buf, 16 * 1237)
    torch.cuda.synchronize()
