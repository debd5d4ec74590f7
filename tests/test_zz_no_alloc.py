"""GPU test of loki_decode_attn_static, the entry point for callers that cannot allocate: it
must give what loki_decode_attn gives on a caller-owned workspace, on two calls in a row that
share the library's built-in scratch buffer, the second with a smaller input."""
import ctypes

import numpy as np
import pytest
import torch

from paper_2406_02542_amd import api, synth
from tests.parity import TORCH_DT, to_dev

pytestmark = pytest.mark.gpu


def say(msg):
    print(msg, flush=True)


def _inputs(w):
    x = synth.make_inputs(w)
    tdt = TORCH_DT[w.dtype]
    lay = api.make_layout(w.B, w.Hq, w.Hkv, w.D, w.d, w.S, tdt)
    klo, khi, v = api.alloc_cache(lay)
    kh = to_dev(x["khat"], w.dtype)
    klo.copy_(kh[..., :w.d])
    khi.copy_(kh[..., w.d:])
    v.copy_(to_dev(x["v"], w.dtype))
    return lay, to_dev(x["q"], w.dtype), torch.from_numpy(x["P"]).cuda(), klo, khi, v


def _both(w, mode):
    """(out, idx) of loki_decode_attn and of loki_decode_attn_static through the raw C ABI."""
    lay, q, P, klo, khi, v = _inputs(w)
    tdt = TORCH_DT[w.dtype]
    hsel = w.Hq if (mode & 1) == 0 or w.G == 1 else w.Hkv
    ws = api.alloc_workspace(lay, w.S, w.d, w.k, mode)
    o_ref = torch.full((w.B, w.Hq, w.D), float("nan"), dtype=tdt, device="cuda")
    i_ref = torch.full((w.B, hsel, w.k), -7, dtype=torch.int32, device="cuda")
    api.loki_decode_attn(lay, q, P, klo, khi, v, w.S, w.d, w.k, mode, ws, o_ref, i_ref)
    o_st = torch.full_like(o_ref, float("nan"))
    i_st = torch.full_like(i_ref, -7)
    L = api.lib()
    vp = ctypes.c_void_p
    rc = L.loki_decode_attn_static(ctypes.byref(lay), vp(q.data_ptr()), vp(P.data_ptr()),
                                   vp(klo.data_ptr()), vp(khi.data_ptr()), vp(v.data_ptr()), w.S, w.d,
                                   w.k, mode, vp(o_st.data_ptr()), vp(i_st.data_ptr()),
                                   vp(torch.cuda.current_stream().cuda_stream))
    assert rc == 0, api.status_string(rc)
    torch.cuda.synchronize()
    return o_ref, i_ref, o_st, i_st


@pytest.mark.parametrize("mode", [api.PATH_SPLIT | 0, 1, api.PATH_CLUSTER | 1])
def test_static_scratch_entry_point_matches_decode_attn(mode):
    # (with cooperating blocks per unit the built-in buffer also holds the blocks' meeting flags:
    # it starts as zeros, every launch leaves them zero, and no clearing kernel runs in front)
    big = synth.Workload("na_big", 2, 8, 2, 128, 3000, "bf16", 32, 500, seed=7700)
    small = synth.Workload("na_small", 1, 8, 2, 128, 700, "bf16", 32, 90, seed=7701)
    for w in (big, small):  # two calls in a row on the shared buffer, the second one smaller
        say(f"case {w} mode {mode:#x}")
        o_ref, i_ref, o_st, i_st = _both(w, mode)
        assert torch.equal(i_ref, i_st)                       # index lists: bit-exact
        assert int(i_st.min()) >= 0 and int(i_st.max()) < w.S
        assert torch.equal(o_ref, o_st)                       # same kernels, same inputs: same bits
        assert bool(torch.isfinite(o_st.float()).all())


def test_static_scratch_entry_point_refuses_large_shapes():
    """A shape whose workspace exceeds the built-in buffer is refused on the host."""
    lay = api.make_layout(64, 64, 8, 128, 32, 8192, torch.bfloat16)
    assert api.loki_workspace_bytes(lay, 8192, 32, 1024, 0) > api.STATIC_SCRATCH_BYTES
    p = ctypes.c_void_p(0x10000)  # aligned, never dereferenced: the call returns before any launch
    rc = api.lib().loki_decode_attn_static(ctypes.byref(lay), p, p, p, p, p, 8192, 32, 1024, 0, p,
                                           None, None)
    assert rc == 6 and "scratch" in api.status_string(rc)
