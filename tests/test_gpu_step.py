"""GPU parity of the whole decode step (loki_decode_step: per-sequence lengths and the
cache append of the current token folded into the decode launches; Algorithm 1 lines 2-9)
and of dense_decode_step, against the CPU oracle.

Protocol.  The rows the GPU appended are read back and checked on their own against the
oracle's rotation (bf16: one unit in the last place plus fp32 accumulation, as for
loki_rotate_keys; values bit-exact); they are then put into the oracle's cache, so that a
last-place difference in the new key cannot cascade into the selection, and the oracle's
step (without append) is compared with the GPU's outputs and index lists under the usual
tolerances, sequence by sequence with each sequence's own length and k.  Rows past a
sequence's end hold 3e4 in K and -3e4 in V on the GPU: any use of them would show."""
import numpy as np
import pytest
import torch

from oracle import loki_oracle as O
from paper_2406_02542_amd import api, synth
from tests.parity import OUT_TOL, TORCH_DT, check_index_set, check_out, to_dev

pytestmark = pytest.mark.gpu


def say(msg):
    print(msg, flush=True)


def run_step_case(w, mode, ragged, append, path=0, lens=None, ks=None, S_cap=None, use_ks=True,
                  boost_tail=0, page_rows=0):
    """page_rows > 0: the same case on a paged cache (random physical pages, a third of the pool
    unused); the pools are mapped back to the contiguous layout for the checks below."""
    x = synth.make_inputs(w)
    st = synth.make_step_inputs(w, x["P"], ragged=ragged)
    if lens is not None:
        st["seq_lens"] = np.asarray(lens, np.int32)
        st["ks"] = np.minimum(np.maximum(1, (w.k * st["seq_lens"].astype(np.int64)) // w.S),
                              np.minimum(st["seq_lens"], w.k)).astype(np.int32)
    if boost_tail:
        # the last `boost_tail` rows of every sequence point along the first query head's rotated
        # query (low-rank columns), so they are certain to be selected by that head
        for b in range(w.B):
            n = int(st["seq_lens"][b])
            for h in range(w.Hkv):
                qhat = O.rotate_query(x["q"][b, h * w.G], x["P"][h])
                row = np.zeros(w.D)
                row[:w.d] = 8.0 * qhat[:w.d] / max(np.linalg.norm(qhat[:w.d]), 1e-9)
                x["khat"][b, h, max(0, n - boost_tail):n] = O.to_storage(row, w.dtype)
    if ks is not None:
        st["ks"] = np.asarray(ks, np.int32)
    lens_np, ks_np = st["seq_lens"], st["ks"]
    if not use_ks:
        ks_np = np.minimum(lens_np, w.k).astype(np.int32)
    S_cap = S_cap or w.S
    pages_per_seq = 0
    if page_rows:
        pages_per_seq = (w.S + page_rows - 1) // page_rows
        S_cap = pages_per_seq * page_rows
    say(f"case {w} mode {mode} path {path:#x} ragged {ragged} append {append} page_rows {page_rows} "
        f"lens {lens_np.tolist()[:8]} ks {ks_np.tolist()[:8]}")
    tdt = TORCH_DT[w.dtype]
    lay = api.make_layout(w.B, w.Hq, w.Hkv, w.D, w.d, S_cap, tdt)
    klo, khi, v = api.alloc_cache(lay)
    klo.fill_(3e4)
    v.fill_(-3e4)
    if khi is not None:
        khi.fill_(3e4)
    kh = to_dev(x["khat"], w.dtype)
    vv = to_dev(x["v"], w.dtype)
    for b in range(w.B):
        n = int(lens_np[b]) - (1 if append else 0)  # the append fills the last row itself
        klo[b, :, :n] = kh[b, :, :n, :w.d]
        if khi is not None:
            khi[b, :, :n] = kh[b, :, :n, w.d:]
        v[b, :, :n] = vv[b, :, :n]
    q = to_dev(x["q"], w.dtype)
    P = torch.from_numpy(x["P"]).cuda()
    ws = api.alloc_workspace(lay, w.S, w.d, w.k, mode)
    out = torch.full((w.B, w.Hq, w.D), float("nan"), dtype=tdt, device="cuda")
    eff_mode = 0 if w.G == 1 else mode
    hsel = w.Hq if eff_mode == 0 else w.Hkv
    idx = torch.full((w.B, hsel, w.k), -7, dtype=torch.int32, device="cuda")
    step_kw = dict(
        seq_lens=torch.from_numpy(lens_np).cuda() if ragged or lens is not None else None,
        ks=torch.from_numpy(ks_np).cuda() if use_ks and (ragged or lens is not None or ks is not None) else None,
        k_new=to_dev(st["k_new"], w.dtype) if append else None,
        v_new=to_dev(st["v_new"], w.dtype) if append else None)
    if page_rows:
        n_pages = w.B * pages_per_seq * 3 // 2 + 1
        perm = np.random.default_rng(w.seed).permutation(n_pages)[:w.B * pages_per_seq].astype(np.int32)
        table = torch.from_numpy(perm.reshape(w.B, pages_per_seq)).cuda()

        def to_pool(c, fill):  # [B, Hkv, S_cap, W] -> [n_pages, Hkv, page_rows, W]
            pool = torch.full((n_pages, w.Hkv, page_rows, c.shape[-1]), fill, dtype=tdt, device="cuda")
            pool[table.view(-1).long()] = c.view(w.B, w.Hkv, pages_per_seq, page_rows, -1).permute(
                0, 2, 1, 3, 4).reshape(w.B * pages_per_seq, w.Hkv, page_rows, -1)
            return pool

        def from_pool(pool):
            return pool[table.view(-1).long()].view(w.B, pages_per_seq, w.Hkv, page_rows, -1).permute(
                0, 2, 1, 3, 4).reshape(w.B, w.Hkv, S_cap, -1).contiguous()

        pklo, pv = to_pool(klo, 3e4), to_pool(v, -3e4)
        pkhi = to_pool(khi, 3e4) if khi is not None else None
        api.loki_decode_step(lay, q, P, pklo, pkhi, pv, w.S, w.d, w.k, mode | path, ws, out, idx,
                             page_table=table, page_rows=page_rows, n_pages=n_pages, **step_kw)
        torch.cuda.synchronize()
        klo, v = from_pool(pklo), from_pool(pv)
        khi = from_pool(pkhi) if pkhi is not None else None
    else:
        api.loki_decode_step(lay, q, P, klo, khi, v, w.S, w.d, w.k, mode | path, ws, out, idx, **step_kw)
    torch.cuda.synchronize()
    out_g = out.float().cpu().numpy().astype(np.float64)
    idx_g = idx.cpu().numpy()

    khat = x["khat"].astype(np.float64).copy()
    vref = x["v"].astype(np.float64).copy()
    if append:
        kcat = torch.cat([klo, khi], dim=-1) if khi is not None else klo
        for b in range(w.B):
            r = int(lens_np[b]) - 1
            got_k = kcat[b, :, r].float().cpu().numpy().astype(np.float64)
            got_v = v[b, :, r].float().cpu().numpy().astype(np.float64)
            np.testing.assert_array_equal(got_v, st["v_new"][b].astype(np.float64))
            for h in range(w.Hkv):
                ref64 = O.rotate_keys(st["k_new"][b, h][None, :], x["P"][h])[0]
                ref = O.to_storage(ref64, w.dtype)
                if w.dtype == "bf16":
                    ulp = 2.0 ** (np.floor(np.log2(np.maximum(np.abs(ref), 1e-30))) - 7)
                    mag = np.abs(st["k_new"][b, h].astype(np.float64)) @ np.abs(x["P"][h].astype(np.float64))
                    assert np.all(np.abs(got_k[h] - ref) <= ulp * 1.0000001 + 1e-6 * mag), (b, h)
                else:
                    assert np.max(np.abs(got_k[h] - ref64)) / np.linalg.norm(ref64) < 2e-6, (b, h)
            khat[b, :, r] = got_k
            vref[b, :, r] = got_v
            # nothing else was written
            if r + 1 < S_cap:
                assert torch.all(kcat[b, :, r + 1:] == 3e4) and torch.all(v[b, :, r + 1:] == -3e4)
            if r > 0:
                assert torch.equal(kcat[b, :, :r], kh[b, :, :r]) and torch.equal(v[b, :, :r], vv[b, :, :r])
    out_o, idx_o, sc_o, _, _ = O.loki_decode_step(x["q"], x["P"], khat, vref, w.d, w.k, eff_mode,
                                                  seq_lens=lens_np, ks=ks_np)
    tol = OUT_TOL[w.dtype]
    swaps, max_err = 0, 0.0
    for b in range(w.B):
        S_b, k_b = int(lens_np[b]), int(ks_np[b])
        for h in range(w.Hkv):
            qheads = range(h * w.G, (h + 1) * w.G)
            same = {}
            for hs in (qheads if eff_mode == 0 else [h]):
                assert np.all(idx_g[b, hs, k_b:] == -1), f"b={b} head={hs}: index list not padded with -1"
                same[hs] = check_index_set(idx_g[b, hs, :k_b], idx_o[b, hs, :k_b], sc_o[b, hs, :S_b], S_b,
                                           k_b, f"{w.name} b={b} sel_head={hs}")
            for hq in qheads:
                hs = hq if eff_mode == 0 else h
                ref = out_o[b, hq]
                if not same[hs]:
                    swaps += 1
                    qhat = O.rotate_query(x["q"][b, hq], x["P"][h])
                    ref = O.attend_selected(qhat, khat[b, h, :S_b], vref[b, h, :S_b],
                                            idx_g[b, hs, :k_b].astype(np.int64))
                err = check_out(out_g[b, hq], ref, w.dtype, f"{w.name} b={b} hq={hq}")
                max_err = max(max_err, err)
    say(f"   max_err {max_err:.3e} heads_with_swaps {swaps}")
    return out_g, idx_g


# ------------------------------------------------------------- one query head per KV head --
@pytest.mark.parametrize("path", [api.PATH_FUSED, api.PATH_SPLIT])
@pytest.mark.parametrize("ragged,append", [(True, False), (False, True), (True, True)])
def test_step_fp32_mha(path, ragged, append):
    w = synth.Workload("step_f32", 5, 4, 4, 128, 1500, "f32", 32, 300, seed=9100)
    run_step_case(w, 0, ragged, append, path=path)


@pytest.mark.parametrize("path", [api.PATH_FUSED, api.PATH_SPLIT])
@pytest.mark.parametrize("S,k", [(4096, 1024), (6000, 700)])
def test_step_bf16_mha(path, S, k):
    """S = 4096: 8 keys per thread in the fused select; 6000: 16.  Ragged and appending."""
    w = synth.Workload("step_bf16", 6, 8, 8, 128, S, "bf16", 32, k, seed=9200)
    run_step_case(w, 0, True, True, path=path)


@pytest.mark.parametrize("path", [api.PATH_FUSED, api.PATH_SPLIT])
def test_step_append_into_short_sequences(path):
    """The new row lies inside the range the fused kernel pre-loads before it rotates
    (first 1024 rows): sequence lengths 1, 2, 300, 1024, 1025 and the full 2048."""
    w = synth.Workload("step_short", 6, 2, 2, 128, 2048, "bf16", 32, 64, seed=9300)
    run_step_case(w, 0, True, True, path=path, lens=[2048, 1, 2, 300, 1024, 1025])


def test_step_full_rank_cache_has_no_residual_slab():
    """d = D: the whole rotated key goes to the low-rank slab (Exact-TopK of Section 5)."""
    w = synth.Workload("step_dD", 3, 4, 4, 128, 900, "bf16", 128, 100, seed=9400)
    run_step_case(w, 0, True, True)


def test_step_default_k_is_min_of_k_and_length():
    """ks = NULL: a sequence shorter than k keeps all its rows."""
    w = synth.Workload("step_defk", 4, 2, 2, 128, 1024, "f32", 32, 512, seed=9500)
    run_step_case(w, 0, True, False, lens=[1024, 100, 512, 513], use_ks=False)


# ------------------------------------------------------------------------ grouped queries --
@pytest.mark.parametrize("mode", [0, 1])
@pytest.mark.parametrize("G,dtype", [(4, "bf16"), (8, "bf16"), (2, "bf16"), (4, "f32")])
def test_step_gqa(mode, G, dtype):
    """Split path: matrix-core and vector scoring, resident select, vector and matrix-core
    gather, with several gather splits whose tail blocks are empty for short sequences."""
    w = synth.Workload(f"step_g{G}", 4, 2 * G, 2, 128, 5000, dtype, 32, 1200, seed=9600 + G)
    run_step_case(w, mode, True, True)


@pytest.mark.parametrize("G,S,k", [(4, 5000, 1200), (8, 8192, 2048), (2, 12000, 700)])
def test_step_gqa_single_kernel_ragged(G, S, k):
    """Grouped heads, one selection per KV group, one launch: per-sequence lengths and k."""
    w = synth.Workload(f"step_gq{G}", 4, 2 * G, 2, 128, S, "bf16", 32, k, seed=9650 + G)
    run_step_case(w, 1, True, False, path=api.PATH_FUSED)
    run_step_case(w, 1, True, False, path=api.PATH_FUSED, lens=[S, 1, 2, 257])


@pytest.mark.parametrize("G,S,k,d", [(2, 700, 100, 32), (4, 4096, 512, 16), (8, 8192, 1024, 64),
                                     (4, 12000, 1500, 32)])
def test_step_gqa_single_kernel_append(G, S, k, d):
    """Grouped heads, one launch, the current token's key and value appended by the same launch
    (Algorithm 1 lines 3-4 folded in): uniform and per-sequence lengths; sequences of one and two
    rows, where the appended row is certain to be selected and lies in the rows the kernel
    requests before it has written them (they must be read again)."""
    w = synth.Workload(f"step_gq{G}_app", 4, 2 * G, 2, 128, S, "bf16", d, k, seed=9670 + G)
    run_step_case(w, 1, False, True, path=api.PATH_FUSED)
    run_step_case(w, 1, True, True, path=api.PATH_FUSED)
    run_step_case(w, 1, True, True, path=api.PATH_FUSED, lens=[S, 1, 2, 257])


@pytest.mark.parametrize("G,B,Hkv,S,k,d", [(4, 3, 2, 1500, 300, 32), (8, 5, 8, 9000, 1200, 16),
                                             (2, 2, 2, 30000, 3000, 64), (4, 16, 8, 2000, 256, 32)])
def test_step_gqa_cluster(G, B, Hkv, S, k, d):
    """Several cooperating blocks per unit (8, 4, 8 and 2 of them): per-sequence lengths, so that
    slices differ from sequence to sequence; the append, written by the block whose slice holds
    the last row; both; and sequences so short that most blocks of a unit hold no row at all."""
    w = synth.Workload(f"step_cluster_g{G}", B, G * Hkv, Hkv, 128, S, "bf16", d, k, seed=G * 1000 + S)
    for ragged, append in [(True, False), (False, True), (True, True)]:
        run_step_case(w, 1, ragged, append, path=api.PATH_CLUSTER)
    lens = ([1, 2, 65, S, 64, 129, 3, S - 1] * 2)[:B]
    run_step_case(w, 1, True, True, path=api.PATH_CLUSTER, lens=lens, S_cap=S + 13)


@pytest.mark.parametrize("mode", [0, 1])
def test_step_long_sequences_multiblock_select(mode):
    """S_max = 40000 (three chunks of the multi-block select): one full sequence, one inside
    the first chunk, one ending just past a chunk boundary."""
    w = synth.Workload("step_long", 3, 4, 1, 128, 40000, "bf16", 16, 2500, seed=9700)
    run_step_case(w, mode, True, True, lens=[40000, 9000, 16385 + 16384])


@pytest.mark.parametrize("append", [False, True])
@pytest.mark.parametrize("mode", [0, 1])
def test_step_multiblock_select_short_sequences_not_multiple_of_four(mode, append):
    """Sequences that end before the last chunk of the multi-block select and whose length is
    not a multiple of four: the chunks past their end must count no row (they once re-read the
    sequence's last rows, which moved the threshold and left ranks of the index list unwritten)."""
    w = synth.Workload("step_long_odd", 4, 4, 1, 128, 40000, "bf16", 16, 2500, seed=9710)
    run_step_case(w, mode, True, append, lens=[40000, 9001, 16387, 3], boost_tail=4)


# ------------------------------------------------------------------- identities and errors --
def test_step_without_options_equals_decode_attn_bitwise():
    w = synth.Workload("step_id", 2, 8, 2, 128, 3000, "bf16", 32, 500, seed=9800)
    x = synth.make_inputs(w)
    lay = api.make_layout(w.B, w.Hq, w.Hkv, 128, w.d, w.S, torch.bfloat16)
    klo, khi, v = api.alloc_cache(lay)
    kh = to_dev(x["khat"], "bf16")
    klo.copy_(kh[..., :w.d]); khi.copy_(kh[..., w.d:]); v.copy_(to_dev(x["v"], "bf16"))
    q, P = to_dev(x["q"], "bf16"), torch.from_numpy(x["P"]).cuda()
    for mode in (0, 1):
        ws = api.alloc_workspace(lay, w.S, w.d, w.k, mode)
        o1 = torch.empty((w.B, w.Hq, 128), dtype=torch.bfloat16, device="cuda")
        o2 = torch.empty_like(o1)
        api.loki_decode_attn(lay, q, P, klo, khi, v, w.S, w.d, w.k, mode, ws, o1)
        api.loki_decode_step(lay, q, P, klo, khi, v, w.S, w.d, w.k, mode, ws, o2)
        torch.cuda.synchronize()
        assert torch.equal(o1, o2)
        # uniform lengths given explicitly change nothing either
        lens = torch.full((w.B,), w.S, dtype=torch.int32, device="cuda")
        api.loki_decode_step(lay, q, P, klo, khi, v, w.S, w.d, w.k, mode, ws, o2, seq_lens=lens)
        torch.cuda.synchronize()
        assert torch.equal(o1, o2)


def test_step_rejects_half_an_append():
    w = synth.Workload("step_err", 1, 2, 2, 128, 64, "bf16", 32, 16, seed=9900)
    lay = api.make_layout(1, 2, 2, 128, 32, 64, torch.bfloat16)
    klo, khi, v = api.alloc_cache(lay)
    q = torch.zeros((1, 2, 128), dtype=torch.bfloat16, device="cuda")
    P = torch.zeros((2, 128, 128), device="cuda")
    ws = api.alloc_workspace(lay, 64, 32, 16, 0)
    out = torch.empty_like(q)
    kn = torch.zeros((1, 2, 128), dtype=torch.bfloat16, device="cuda")
    with pytest.raises(api.LokiError) as e:
        api.loki_decode_step(lay, q, P, klo, khi, v, 64, 32, 16, 0, ws, out, k_new=kn)
    assert e.value.status == 1


# --------------------------------------------------------------------------- dense baseline --
@pytest.mark.parametrize("G,dtype", [(1, "bf16"), (4, "bf16"), (8, "bf16"), (2, "f32")])
def test_dense_step_ragged(G, dtype):
    w = synth.Workload(f"dense_g{G}", 4, 2 * G, 2, 128, 3000, dtype, 32, 8, seed=9950 + G)
    x = synth.make_inputs(w)
    lens = synth.make_step_inputs(w, x["P"])["seq_lens"]
    say(f"case {w} lens {lens.tolist()}")
    tdt = TORCH_DT[dtype]
    lay = api.make_layout(w.B, w.Hq, w.Hkv, 128, w.d, w.S, tdt)
    kfull = torch.full((w.B, w.Hkv, w.S, 128), 3e4, dtype=tdt, device="cuda")
    v = torch.full((w.B, w.Hkv, w.S, 128), -3e4, dtype=tdt, device="cuda")
    kh, vv = to_dev(x["khat"], dtype), to_dev(x["v"], dtype)
    for b in range(w.B):
        kfull[b, :, :lens[b]] = kh[b, :, :lens[b]]
        v[b, :, :lens[b]] = vv[b, :, :lens[b]]
    ws = torch.empty(max(api.loki_workspace_bytes(lay, w.S, 0, 0, -1), 256), dtype=torch.uint8, device="cuda")
    out = torch.full((w.B, w.Hq, 128), float("nan"), dtype=tdt, device="cuda")
    api.dense_decode_step(lay, to_dev(x["q"], dtype), kfull, v, w.S, torch.from_numpy(lens).cuda(), ws, out)
    torch.cuda.synchronize()
    got = out.float().cpu().numpy().astype(np.float64)
    for b in range(w.B):
        ref = O.dense_decode_batch(x["q"][b:b + 1], x["khat"][b:b + 1, :, :lens[b]], x["v"][b:b + 1, :, :lens[b]])
        check_out(got[b], ref[0], dtype, f"dense ragged b={b}")


# ------------------------------------------------- paged cache, judged by the oracle directly --
@pytest.mark.parametrize("G,mode,path,page_rows", [(1, 0, api.PATH_FUSED, 256), (1, 0, api.PATH_SPLIT, 512),
                                                   (4, 0, api.PATH_SPLIT, 256), (4, 1, api.PATH_SPLIT, 1024),
                                                   (8, 1, api.PATH_SPLIT, 256), (4, 1, api.PATH_FUSED, 256),
                                                   (8, 1, api.PATH_FUSED, 1024), (2, 1, api.PATH_FUSED, 512),
                                                   (4, 1, api.PATH_CLUSTER, 256), (8, 1, api.PATH_CLUSTER, 1024),
                                                   (2, 1, api.PATH_CLUSTER, 512)])
def test_step_paged_cache_against_oracle(G, mode, path, page_rows):
    """The whole step (ragged, appending) on a paged cache against the oracle itself, not only
    against the contiguous layout: outputs, index lists and the appended rows."""
    w = synth.Workload(f"step_paged_g{G}", 4, 2 * G, 2, 128, 3000, "bf16", 32, 700, seed=9660 + G + mode)
    run_step_case(w, mode, True, True, path=path, page_rows=page_rows)


# ---------------------------------------------------------------- PCAAttn (Algorithm 2) --
@pytest.mark.parametrize("G,dtype,d,S", [(1, "f32", 32, 1500), (1, "bf16", 32, 4096), (2, "bf16", 16, 3001),
                                         (4, "bf16", 64, 5000), (8, "bf16", 32, 2000), (4, "f32", 128, 700),
                                         (1, "bf16", 128, 1000), (8, "bf16", 48, 2500), (4, "bf16", 8, 1300),
                                         (4, "bf16", 104, 900), (8, "bf16", 128, 700)])
def test_pca_attn(G, dtype, d, S):
    """softmax(qhat[:d] Klo^T / sqrt(D)) V over all rows; the residual slab is never passed."""
    w = synth.Workload(f"pca_g{G}", 3, 2 * G, 2, 128, S, dtype, d, 8, seed=9990 + G)
    x = synth.make_inputs(w)
    say(f"case {w}")
    tdt = TORCH_DT[dtype]
    lay = api.make_layout(w.B, w.Hq, w.Hkv, 128, d, S + 5, tdt)
    klo, _, v = api.alloc_cache(lay)
    klo.fill_(3e4); v.fill_(-3e4)
    kh = to_dev(x["khat"], dtype)
    klo[:, :, :S] = kh[..., :d]
    v[:, :, :S] = to_dev(x["v"], dtype)
    ws = torch.empty(api.loki_workspace_bytes(lay, S, d, 0, -2), dtype=torch.uint8, device="cuda")
    out = torch.full((w.B, w.Hq, 128), float("nan"), dtype=tdt, device="cuda")
    api.loki_pca_attn(lay, to_dev(x["q"], dtype), torch.from_numpy(x["P"]).cuda(), klo, v, S, d, ws, out)
    torch.cuda.synchronize()
    ref = O.pca_attention_batch(x["q"], x["P"], x["khat"], x["v"], d)
    err = check_out(out.float().cpu().numpy(), ref, dtype, f"PCAAttn G={G} d={d}")
    say(f"   max_err {err:.3e}")


# ------------------------------------------------------------------------- graph capture --
@pytest.mark.parametrize("G,mode,path", [(1, 0, 0), (4, 0, 0), (4, 1, 0), (4, 1, api.PATH_FUSED),
                                         (4, 1, api.PATH_CLUSTER)])
def test_decode_step_replays_from_a_captured_graph(G, mode, path):
    """The library allocates nothing and records no memset, so a step can be captured once and
    replayed: every replay (with eager work and synchronisations in between, and with the
    inputs changed in place) must equal the eager result on the same inputs bit for bit.  (The
    launch with cooperating blocks clears its meeting flags with a kernel of its own, which is
    part of the captured sequence.)"""
    w = synth.Workload(f"graph_g{G}", 2, 2 * G, 2, 128, 3000, "bf16", 32, 600, seed=9970 + G)
    x = synth.make_inputs(w)
    st = synth.make_step_inputs(w, x["P"])
    lay = api.make_layout(w.B, w.Hq, w.Hkv, 128, w.d, w.S, torch.bfloat16)
    klo, khi, v = api.alloc_cache(lay)
    kh = to_dev(x["khat"], "bf16")
    klo.copy_(kh[..., :w.d]); khi.copy_(kh[..., w.d:]); v.copy_(to_dev(x["v"], "bf16"))
    q, P = to_dev(x["q"], "bf16"), torch.from_numpy(x["P"]).cuda()
    lens, ks = torch.from_numpy(st["seq_lens"]).cuda(), torch.from_numpy(st["ks"]).cuda()
    k_new, v_new = to_dev(st["k_new"], "bf16"), to_dev(st["v_new"], "bf16")
    ws = api.alloc_workspace(lay, w.S, w.d, w.k, mode)
    out_g = torch.zeros((w.B, w.Hq, 128), dtype=torch.bfloat16, device="cuda")
    out_e = torch.zeros_like(out_g)

    def step(out):
        api.loki_decode_step(lay, q, P, klo, khi, v, w.S, w.d, w.k, mode | path, ws, out, None,
                             seq_lens=lens, ks=ks, k_new=k_new, v_new=v_new)

    step(out_e)  # warm-up outside the capture (first-launch set-up of the kernels)
    torch.cuda.synchronize()
    side = torch.cuda.Stream()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.stream(side):
        graph.capture_begin()
        step(out_g)
        graph.capture_end()
    torch.cuda.synchronize()
    gen = torch.Generator(device="cuda").manual_seed(5)
    for it in range(4):
        # new query and new token in place: the graph reads them through the same pointers
        q.copy_(torch.randn(q.shape, device="cuda", generator=gen).to(torch.bfloat16))
        k_new.copy_((0.3 * torch.randn(k_new.shape, device="cuda", generator=gen)).to(torch.bfloat16))
        v_new.copy_(torch.randn(v_new.shape, device="cuda", generator=gen).to(torch.bfloat16))
        torch.cuda.synchronize()
        out_g.zero_()
        graph.replay()
        torch.cuda.synchronize()
        step(out_e)
        torch.cuda.synchronize()
        assert torch.equal(out_g, out_e), f"replay {it} differs from the eager step"
        assert torch.isfinite(out_g.float()).all()


# ------------------------------------------------------- several new tokens per sequence --
@pytest.mark.parametrize("G,dtype,mode,m,B", [(1, "bf16", 0, 3, 3), (4, "bf16", 0, 3, 3), (4, "bf16", 1, 3, 3),
                                              (2, "f32", 0, 3, 3), (4, "bf16", 0, 5, 3), (8, "bf16", 1, 3, 3),
                                              (1, "bf16", 0, 17, 3), (2, "bf16", 1, 9, 3), (8, "bf16", 0, 2, 3),
                                              (4, "bf16", 0, 3, 4), (2, "f32", 0, 2, 4), (1, "bf16", 0, 4, 4)])
def test_step_with_several_new_tokens_per_sequence(G, dtype, mode, m, B):
    """queries_per_seq = m (chunked / speculative decoding): token j of a sequence is appended
    at its own row and attends up to and including it; entries of one sequence share its
    cache.  Same protocol as the single-token cases.  On a bf16 cache the m G query heads of
    a KV head are scored as tiles of 16 columns: the cases cover a partly filled tile, two
    tiles, and a last tile with one token.  With 4 sequences (8 cached KV heads) the gather
    renumbers its blocks per XCD."""
    w = synth.Workload(f"multi_g{G}", B, 2 * G, 2, 128, 2500, dtype, 32, 400, seed=14000 + G)
    wq = w.replace(B=B * m)
    x = synth.make_inputs(w)
    xq = synth.make_inputs(wq.replace(S=8))   # only its q is used
    st = synth.make_step_inputs(wq, x["P"])    # k_new, v_new for B m entries
    rows = np.array([2500, 700, 1337, 2011][:B])   # rows of each sequence after the chunk
    lens = np.array([rows[b] - (m - 1 - j) for b in range(B) for j in range(m)], np.int32)
    ks = np.maximum(1, (w.k * lens.astype(np.int64)) // w.S).astype(np.int32)
    say(f"case {w} m {m} mode {mode} lens {lens.tolist()} ks {ks.tolist()}")
    tdt = TORCH_DT[dtype]
    lay = api.make_layout(B, w.Hq, w.Hkv, 128, w.d, w.S, tdt)
    klo, khi, v = api.alloc_cache(lay)
    klo.fill_(3e4); khi.fill_(3e4); v.fill_(-3e4)
    kh, vv = to_dev(x["khat"], dtype), to_dev(x["v"], dtype)
    for b in range(B):
        n = int(rows[b]) - m
        klo[b, :, :n] = kh[b, :, :n, :w.d]; khi[b, :, :n] = kh[b, :, :n, w.d:]; v[b, :, :n] = vv[b, :, :n]
    lay_ws = api.make_layout(B * m, w.Hq, w.Hkv, 128, w.d, w.S, tdt)
    ws = api.alloc_workspace(lay_ws, w.S, w.d, w.k, mode)
    out = torch.full((B * m, w.Hq, 128), float("nan"), dtype=tdt, device="cuda")
    hsel = w.Hq if mode == 0 or G == 1 else w.Hkv
    idx = torch.full((B * m, hsel, w.k), -7, dtype=torch.int32, device="cuda")
    api.loki_decode_step(lay, to_dev(xq["q"], dtype), torch.from_numpy(x["P"]).cuda(), klo, khi, v, w.S,
                         w.d, w.k, mode, ws, out, idx, seq_lens=torch.from_numpy(lens).cuda(),
                         ks=torch.from_numpy(ks).cuda(), k_new=to_dev(st["k_new"], dtype),
                         v_new=to_dev(st["v_new"], dtype), queries_per_seq=m)
    torch.cuda.synchronize()
    out_g = out.float().cpu().numpy().astype(np.float64)
    idx_g = idx.cpu().numpy()
    # the GPU's appended rows (checked against the oracle's rotation) go into the oracle's cache
    kcat = torch.cat([klo, khi], dim=-1).float().cpu().numpy().astype(np.float64)
    khat, vref = x["khat"].astype(np.float64).copy(), x["v"].astype(np.float64).copy()
    for e in range(B * m):
        b, r = e // m, int(lens[e]) - 1
        for h in range(w.Hkv):
            ref64 = O.rotate_keys(st["k_new"][e, h][None, :], x["P"][h])[0]
            ref = O.to_storage(ref64, dtype)
            if dtype == "bf16":
                ulp = 2.0 ** (np.floor(np.log2(np.maximum(np.abs(ref), 1e-30))) - 7)
                mag = np.abs(st["k_new"][e, h].astype(np.float64)) @ np.abs(x["P"][h].astype(np.float64))
                assert np.all(np.abs(kcat[b, h, r] - ref) <= ulp * 1.0000001 + 1e-6 * mag)
            else:
                assert np.max(np.abs(kcat[b, h, r] - ref64)) / np.linalg.norm(ref64) < 2e-6
        khat[b, :, r] = kcat[b, :, r]
        vref[b, :, r] = st["v_new"][e].astype(np.float64)
        assert np.array_equal(v[b, :, r].float().cpu().numpy(), st["v_new"][e])
    for b in range(B):
        assert torch.all(klo[b, :, rows[b]:] == 3e4) and torch.all(v[b, :, rows[b]:] == -3e4)
    eff_mode = 0 if G == 1 else mode
    out_o, idx_o, sc_o, _, _ = O.loki_decode_step(xq["q"], x["P"], khat, vref, w.d, w.k, eff_mode,
                                                  seq_lens=lens, ks=ks, queries_per_seq=m)
    tol, max_err = OUT_TOL[dtype], 0.0
    for e in range(B * m):
        S_e, k_e, b = int(lens[e]), int(ks[e]), e // m
        for h in range(w.Hkv):
            qheads = range(h * G, (h + 1) * G)
            same = {}
            for hs in (qheads if eff_mode == 0 else [h]):
                assert np.all(idx_g[e, hs, k_e:] == -1)
                same[hs] = check_index_set(idx_g[e, hs, :k_e], idx_o[e, hs, :k_e], sc_o[e, hs, :S_e], S_e, k_e,
                                           f"entry {e} sel_head {hs}")
            for hq in qheads:
                hs = hq if eff_mode == 0 else h
                ref = out_o[e, hq]
                if not same[hs]:
                    qhat = O.rotate_query(xq["q"][e, hq], x["P"][h])
                    ref = O.attend_selected(qhat, khat[b, h, :S_e], vref[b, h, :S_e], idx_g[e, hs, :k_e].astype(np.int64))
                err = check_out(out_g[e, hq], ref, dtype, f"entry {e} hq {hq}")
                max_err = max(max_err, err)
    say(f"   max_err {max_err:.3e}")


def _multi_token_vs_single_token_steps(Bs, Hq, Hkv, S, d, k, mode, m, seed):
    """One step with queries_per_seq = m against m single-token steps one after the other (the
    form the oracle covers), on random bf16 caches.  Index lists must be identical when both
    forms score with the same matrix-core arithmetic (grouped heads, d a power of two above
    16); otherwise the two score kernels differ in accumulation order and a list may differ by
    swaps at the threshold.  Outputs agree to the output tolerance (the two forms split the k
    rows over a different number of blocks)."""
    G = Hq // Hkv
    tdt = torch.bfloat16
    g = torch.Generator(device="cuda").manual_seed(seed)
    rnd = lambda *shape, scale=1.0: (scale * torch.randn(shape, device="cuda", generator=g)).to(tdt)
    klo0, khi0, v0 = rnd(Bs, Hkv, S, d, scale=2.0), rnd(Bs, Hkv, S, 128 - d, scale=0.5), rnd(Bs, Hkv, S, 128)
    q, k_new, v_new = rnd(Bs, m, Hq, 128), rnd(Bs, m, Hkv, 128), rnd(Bs, m, Hkv, 128)
    Pm = torch.linalg.qr(torch.randn((Hkv, 128, 128), device="cuda", generator=g))[0].contiguous()
    rows = torch.randint(max(S // 3, m), S + 1, (Bs,), device="cuda", generator=g, dtype=torch.int32)
    rows[0] = S
    lens = (rows[:, None] - (m - 1 - torch.arange(m, device="cuda", dtype=torch.int32))[None, :]).contiguous()
    ks = torch.clamp((k * lens.long()) // S, min=1).to(torch.int32).contiguous()
    say(f"Bs {Bs} Hq {Hq} Hkv {Hkv} S {S} d {d} k {k} mode {mode} m {m} rows {rows.tolist()}")
    lay = api.make_layout(Bs, Hq, Hkv, 128, d, S, tdt)
    laym = api.make_layout(Bs * m, Hq, Hkv, 128, d, S, tdt)
    ws = api.alloc_workspace(laym, S, d, k, mode)
    hsel = Hq if mode == 0 or G == 1 else Hkv
    sel = mode | api.PATH_SPLIT

    ca = [t.clone() for t in (klo0, khi0, v0)]
    out_a = torch.full((Bs, m, Hq, 128), float("nan"), dtype=tdt, device="cuda")
    idx_a = torch.full((Bs, m, hsel, k), -7, dtype=torch.int32, device="cuda")
    api.loki_decode_step(lay, q.view(Bs * m, Hq, 128), Pm, *ca, S, d, k, sel, ws, out_a.view(Bs * m, Hq, 128),
                         idx_a.view(Bs * m, hsel, k), seq_lens=lens.view(-1), ks=ks.view(-1),
                         k_new=k_new.view(Bs * m, Hkv, 128), v_new=v_new.view(Bs * m, Hkv, 128), queries_per_seq=m)
    cb = [t.clone() for t in (klo0, khi0, v0)]
    out_b, idx_b = torch.empty_like(out_a), torch.empty_like(idx_a)
    for j in range(m):
        o = torch.full((Bs, Hq, 128), float("nan"), dtype=tdt, device="cuda")
        ix = torch.full((Bs, hsel, k), -7, dtype=torch.int32, device="cuda")
        api.loki_decode_step(lay, q[:, j].contiguous(), Pm, *cb, S, d, k, sel, ws, o, ix,
                             seq_lens=lens[:, j].contiguous(), ks=ks[:, j].contiguous(),
                             k_new=k_new[:, j].contiguous(), v_new=v_new[:, j].contiguous())
        out_b[:, j], idx_b[:, j] = o, ix
    torch.cuda.synchronize()
    for a, b in zip(ca, cb):
        assert torch.equal(a, b)  # the appended rows
    assert torch.isfinite(out_a.float()).all()
    same_arithmetic = G > 1 and d > 16 and (d & (d - 1)) == 0
    if same_arithmetic:
        assert torch.equal(idx_a, idx_b)
    else:
        ia, ib = idx_a.cpu().numpy(), idx_b.cpu().numpy()
        worst = 0
        for e in np.ndindex(ia.shape[:3]):
            la, lb = set(ia[e][ia[e] >= 0].tolist()), set(ib[e][ib[e] >= 0].tolist())
            assert len(la) == len(lb)
            worst = max(worst, len(la - lb))
        say(f"   most rows swapped in one list: {worst}")
        assert worst <= 2
    err = float((out_a.float() - out_b.float()).abs().max())
    say(f"   max |out difference| {err:.3e}")
    assert err <= OUT_TOL["bf16"]


@pytest.mark.parametrize("Hq,Hkv,mode,m", [(32, 8, 0, 4), (32, 8, 1, 4), (32, 8, 1, 3), (32, 32, 0, 4)])
def test_multi_token_step_equals_single_token_steps_at_full_size(Hq, Hkv, mode, m):
    """At a size the oracle cannot walk: 16 sequences, S = 8192, k = 1024."""
    _multi_token_vs_single_token_steps(16, Hq, Hkv, 8192, 32, 1024, mode, m, 77 + Hq + mode + m)


@pytest.mark.parametrize("seed", range(16))
def test_multi_token_step_equals_single_token_steps_on_random_shapes(seed):
    """Odd shapes: any number of sequences and KV heads (the XCD renumbering of the gather
    pads the grid), 1 to 8 heads per KV head, 2 to 9 tokens (partly filled and several score
    tiles), slab widths on both score kernels, either selection mode."""
    rng = np.random.default_rng(5000 + seed)
    Hkv = int(rng.choice([1, 2, 3, 4, 8]))
    G = int(rng.choice([1, 2, 4, 8]))
    Bs = int(rng.integers(1, 8))
    m = int(rng.integers(2, 10))
    S = int(rng.integers(300, 5000))
    d = int(rng.choice([8, 16, 24, 32, 64]))
    k = int(rng.integers(1, max(2, S // 3)))
    mode = int(rng.integers(0, 2))
    _multi_token_vs_single_token_steps(Bs, Hkv * G, Hkv, S, d, k, mode, m, 6000 + seed)


# -------------------------------------------------------------------------- paged cache --
@pytest.mark.parametrize("G,dtype,mode,page_rows,m,path", [
    (1, "bf16", 0, 256, 1, api.PATH_SPLIT), (4, "bf16", 0, 1024, 1, api.PATH_SPLIT),
    (4, "bf16", 1, 256, 1, api.PATH_SPLIT), (8, "bf16", 1, 512, 1, api.PATH_SPLIT),
    (2, "f32", 0, 256, 1, api.PATH_SPLIT), (4, "bf16", 0, 256, 2, api.PATH_SPLIT),
    (4, "bf16", 1, 512, 5, api.PATH_SPLIT), (1, "bf16", 0, 256, 3, api.PATH_SPLIT),
    (1, "bf16", 0, 256, 1, api.PATH_FUSED), (1, "bf16", 0, 2048, 1, api.PATH_FUSED),
    (1, "f32", 0, 512, 1, api.PATH_FUSED), (4, "bf16", 1, 256, 1, api.PATH_FUSED),
    (8, "bf16", 1, 2048, 1, api.PATH_FUSED), (2, "bf16", 1, 512, 1, api.PATH_FUSED),
    (4, "bf16", 1, 256, 1, api.PATH_CLUSTER), (8, "bf16", 1, 1024, 1, api.PATH_CLUSTER)])
def test_paged_cache_equals_contiguous_cache(G, dtype, mode, page_rows, m, path):
    """The same rows scattered over randomly ordered physical pages (with unused pages in
    between) give bit-identical outputs, index lists and appended rows, on either kernel
    sequence: the page table changes where a row lives, not what is computed.  The contiguous
    reference is itself checked against the oracle by the tests above."""
    w = synth.Workload(f"paged_g{G}", 3, 2 * G, 2, 128, 3000, dtype, 32, 500, seed=15000 + G)
    _paged_vs_contiguous(w, mode, page_rows, m, path, [3000, 800, 1537])


@pytest.mark.parametrize("seed", range(12))
def test_paged_cache_equals_contiguous_cache_on_random_shapes(seed):
    rng = np.random.default_rng(7000 + seed)
    Hkv = int(rng.choice([1, 2, 3, 4]))
    G = int(rng.choice([1, 2, 4, 8]))
    B = int(rng.integers(1, 6))
    m = int(rng.choice([1, 1, 2, 3, 6]))
    S = int(rng.integers(400, 5000))
    d = int(rng.choice([8, 16, 32, 64]))
    dtype = "bf16" if rng.random() < 0.75 else "f32"
    k = int(rng.integers(1, max(2, min(S // 3, 2000))))
    mode = int(rng.integers(0, 2))
    page_rows = int(rng.choice([256, 512, 1024, 2048]))
    fused_ok = m == 1 and (S + page_rows - 1) // page_rows <= 32 and (
        G == 1 or (mode == 1 and dtype == "bf16" and d in (16, 32, 64) and k <= 2048))
    path = api.PATH_FUSED if (fused_ok and rng.random() < 0.5) else api.PATH_SPLIT
    rows = [S] + [int(rng.integers(max(m, 2), S + 1)) for _ in range(B - 1)]
    w = synth.Workload(f"paged_rnd{seed}", B, Hkv * G, Hkv, 128, S, dtype, d, k, seed=17000 + seed)
    _paged_vs_contiguous(w, mode, page_rows, m, path, rows)


def _paged_vs_contiguous(w, mode, page_rows, m, path, rows):
    B, G, dtype = w.B, w.G, w.dtype
    x = synth.make_inputs(w)
    wq = w.replace(B=B * m)
    st = synth.make_step_inputs(wq, x["P"])
    q = to_dev(synth.make_inputs(wq.replace(S=8))["q"], dtype)
    rows = np.array(rows)
    lens = np.array([rows[b] - (m - 1 - j) for b in range(B) for j in range(m)], np.int32)
    ks = np.maximum(1, (w.k * lens.astype(np.int64)) // w.S).astype(np.int32)
    say(f"paged case {w} mode {mode} page_rows {page_rows} m {m} path {path:#x} rows {rows.tolist()}")
    tdt = TORCH_DT[dtype]
    pages_per_seq = (w.S + page_rows - 1) // page_rows
    S_cap = pages_per_seq * page_rows
    lay = api.make_layout(B, w.Hq, w.Hkv, 128, w.d, S_cap, tdt)
    klo, khi, v = api.alloc_cache(lay)
    klo.fill_(3e4); khi.fill_(3e4); v.fill_(-3e4)
    kh, vv = to_dev(x["khat"], dtype), to_dev(x["v"], dtype)
    for b in range(B):
        n = int(rows[b]) - m
        klo[b, :, :n] = kh[b, :, :n, :w.d]; khi[b, :, :n] = kh[b, :, :n, w.d:]; v[b, :, :n] = vv[b, :, :n]
    # pools: every logical page gets a random physical page; a third of the pool stays unused
    n_pages = B * pages_per_seq * 3 // 2 + 1
    perm = np.random.default_rng(5).permutation(n_pages)[:B * pages_per_seq].astype(np.int32)
    table = torch.from_numpy(perm.reshape(B, pages_per_seq)).cuda()

    def to_pool(c):  # [B, Hkv, S_cap, W] -> [n_pages, Hkv, page_rows, W]
        pool = torch.full((n_pages, w.Hkv, page_rows, c.shape[-1]), 7.0, dtype=tdt, device="cuda")
        pool[table.view(-1).long()] = c.view(B, w.Hkv, pages_per_seq, page_rows, -1).permute(0, 2, 1, 3, 4).reshape(
            B * pages_per_seq, w.Hkv, page_rows, -1)
        return pool

    def from_pool(pool):
        return pool[table.view(-1).long()].view(B, pages_per_seq, w.Hkv, page_rows, -1).permute(0, 2, 1, 3, 4).reshape(
            B, w.Hkv, S_cap, -1)

    pklo, pkhi, pv = to_pool(klo), to_pool(khi), to_pool(v)
    lay_ws = api.make_layout(B * m, w.Hq, w.Hkv, 128, w.d, S_cap, tdt)
    ws = api.alloc_workspace(lay_ws, w.S, w.d, w.k, mode)
    hsel = w.Hq if mode == 0 or G == 1 else w.Hkv
    P = torch.from_numpy(x["P"]).cuda()
    common = dict(seq_lens=torch.from_numpy(lens).cuda(), ks=torch.from_numpy(ks).cuda(),
                  k_new=to_dev(st["k_new"], dtype), v_new=to_dev(st["v_new"], dtype), queries_per_seq=m)
    out_c = torch.full((B * m, w.Hq, 128), float("nan"), dtype=tdt, device="cuda")
    idx_c = torch.full((B * m, hsel, w.k), -7, dtype=torch.int32, device="cuda")
    api.loki_decode_step(lay, q, P, klo, khi, v, w.S, w.d, w.k, mode | path, ws, out_c, idx_c, **common)
    out_p = torch.full_like(out_c, float("nan"))
    idx_p = torch.full_like(idx_c, -7)
    api.loki_decode_step(lay, q, P, pklo, pkhi, pv, w.S, w.d, w.k, mode | path, ws, out_p, idx_p,
                         page_table=table, page_rows=page_rows, n_pages=n_pages, **common)
    torch.cuda.synchronize()
    assert torch.isfinite(out_c.float()).all()
    assert torch.equal(out_p, out_c)
    assert torch.equal(idx_p, idx_c)
    assert torch.equal(from_pool(pklo), klo) and torch.equal(from_pool(pkhi), khi) and torch.equal(from_pool(pv), v)
    unused = np.setdiff1d(np.arange(n_pages), perm)
    assert torch.all(pklo[torch.from_numpy(unused).cuda().long()] == 7.0)


def test_paged_cache_rejects_bad_geometry():
    lay = api.make_layout(1, 2, 2, 128, 32, 1024, torch.bfloat16)
    z = lambda *s: torch.zeros(s, dtype=torch.bfloat16, device="cuda")
    pool_lo, pool_hi, pool_v = z(4, 2, 256, 32), z(4, 2, 256, 96), z(4, 2, 256, 128)
    q, out, P = z(1, 2, 128), z(1, 2, 128), torch.zeros((2, 128, 128), device="cuda")
    ws = api.alloc_workspace(lay, 1024, 32, 64, 0)
    table = torch.zeros((1, 4), dtype=torch.int32, device="cuda")
    for kw, status in ((dict(page_rows=200, n_pages=4), 1),      # not a power of two
                       (dict(page_rows=128, n_pages=4), 1),      # below the scoring block granularity
                       (dict(page_rows=256, n_pages=0), 1)):
        with pytest.raises((api.LokiError, ValueError)) as e:
            api.loki_decode_step(lay, q, P, pool_lo, pool_hi, pool_v, 1024, 32, 64, 0, ws, out,
                                 page_table=table, **kw)
        if isinstance(e.value, api.LokiError):
            assert e.value.status == status
    short = torch.zeros((1, 3), dtype=torch.int32, device="cuda")  # 3 pages x 256 rows < S
    with pytest.raises(api.LokiError) as e:
        api.loki_decode_step(lay, q, P, pool_lo, pool_hi, pool_v, 1024, 32, 64, 0, ws, out,
                             page_table=short, page_rows=256, n_pages=4)
    assert e.value.status == 1


@pytest.mark.parametrize("dtype", ["bf16", "f32"])
def test_paged_key_rotation_equals_contiguous(dtype):
    """loki_rotate_keys_paged writes bit for bit what loki_rotate_keys writes, at the rows the
    page table names; pages it does not name stay untouched."""
    B, Hkv, page_rows, pps = 3, 2, 256, 5
    S_cap = pps * page_rows
    w = synth.Workload("paged_rot", B, Hkv, Hkv, 128, 1100, dtype, 32, 8, seed=16000)
    P = synth.make_P(w)
    K = synth.make_unrotated_keys(w, P)
    tdt = TORCH_DT[dtype]
    lay = api.make_layout(B, Hkv, Hkv, 128, 32, S_cap, tdt)
    klo, khi, _ = api.alloc_cache(lay)
    klo.fill_(5.0); khi.fill_(5.0)
    n_pages = B * pps + 4
    perm = np.random.default_rng(6).permutation(n_pages)[:B * pps].astype(np.int32)
    table = torch.from_numpy(perm.reshape(B, pps)).cuda()
    pklo = torch.full((n_pages, Hkv, page_rows, 32), 5.0, dtype=tdt, device="cuda")
    pkhi = torch.full((n_pages, Hkv, page_rows, 96), 5.0, dtype=tdt, device="cuda")
    Pd = torch.from_numpy(P).cuda()
    for lo, n_new in ((0, 1000), (1000, 1), (1001, 99)):  # prefill at position 7, then appends
        chunk = to_dev(K[:, :, lo:lo + n_new], dtype)
        api.loki_rotate_keys(lay, chunk, Pd, klo, khi, 7 + lo, n_new)
        api.loki_rotate_keys_paged(lay, chunk, Pd, pklo, pkhi, table, page_rows, n_pages, 7 + lo, n_new)
    torch.cuda.synchronize()

    def from_pool(pool):
        return pool[table.view(-1).long()].view(B, pps, Hkv, page_rows, -1).permute(0, 2, 1, 3, 4).reshape(
            B, Hkv, S_cap, -1)

    assert torch.equal(from_pool(pklo), klo) and torch.equal(from_pool(pkhi), khi)
    assert not torch.all(klo == 5.0)
    unused = torch.from_numpy(np.setdiff1d(np.arange(n_pages), perm)).cuda().long()
    assert torch.all(pklo[unused] == 5.0) and torch.all(pkhi[unused] == 5.0)
