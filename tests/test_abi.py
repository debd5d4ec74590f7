"""Host-only checks of the C ABI: the library loads, exports every symbol the header
declares, sizes caches and workspaces, and rejects bad arguments before any launch.
No compute call is made, so no GPU is needed."""
import ctypes
import os
import re

import pytest
import torch

from paper_2406_02542_amd import api

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def _declared_functions():
    text = open(os.path.join(ROOT, "include", "loki.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    names = re.findall(r"^\s*(?:const\s+char\s*\*|int)\s+(\w+)\s*\(", text, flags=re.M)
    return sorted(set(names))


def test_library_exports_every_declared_symbol():
    names = _declared_functions()
    for expected in ("loki_rotate_keys", "loki_decode_attn", "dense_decode_attn",
                     "loki_cache_bytes", "loki_workspace_bytes", "loki_status_string",
                     "loki_version", "loki_profile_create", "loki_profile_read"):
        assert expected in names
    L = api.lib()
    for n in names:
        assert hasattr(L, n), f"{n} declared in include/loki.h but not exported"
    assert api.version() >= 100
    assert api.status_string(0) == "ok"
    assert "workspace" in api.status_string(4)


def test_layout_struct_matches_header():
    assert ctypes.sizeof(api.Layout) == 7 * 4
    assert [f[0] for f in api.Layout._fields_] == ["B", "Hq", "Hkv", "D", "d_split", "S_cap", "dtype"]


def test_step_args_struct_matches_header():
    assert [f[0] for f in api.StepArgs._fields_] == ["seq_lens", "ks", "k_new", "v_new", "queries_per_seq",
                                                     "page_rows", "page_table", "pages_per_seq", "n_pages"]
    assert ctypes.sizeof(api.StepArgs) == 4 * 8 + 2 * 4 + 8 + 2 * 4


def test_cache_and_workspace_sizes():
    lay = api.make_layout(16, 32, 32, 128, 32, 4096, torch.bfloat16)
    klo, khi, v = api.loki_cache_bytes(lay)
    rows = 16 * 32 * 4096
    assert (klo, khi, v) == (rows * 32 * 2, rows * 96 * 2, rows * 128 * 2)
    assert klo + khi == v  # the split cache holds each key exactly once (Section 4.2)
    ws = api.loki_workspace_bytes(lay, 4096, 32, 1024, 0)
    assert ws >= 16 * 32 * (4096 * 4 + 1024 * 4 + 128 * 4)
    assert ws % 256 == 0
    lay32 = api.make_layout(1, 8, 8, 128, 32, 1024, torch.float32)
    assert api.loki_cache_bytes(lay32) == (8 * 1024 * 32 * 4, 8 * 1024 * 96 * 4, 8 * 1024 * 128 * 4)
    assert api.loki_workspace_bytes(lay32, 1024, 0, 0, -1) >= 0


def _status(fn, *a):
    return fn(*a)


def test_rejects_bad_arguments_before_launch():
    L = api.lib()
    lay = api.make_layout(2, 8, 2, 128, 32, 512, torch.bfloat16)
    n = ctypes.c_size_t()
    by = ctypes.byref
    # size queries
    assert L.loki_workspace_bytes(by(lay), 0, 32, 1, 0, by(n)) == 1      # S < 1
    assert L.loki_workspace_bytes(by(lay), 513, 32, 1, 0, by(n)) == 1    # S > S_cap
    assert L.loki_workspace_bytes(by(lay), 512, 32, 0, 0, by(n)) == 1    # k < 1
    assert L.loki_workspace_bytes(by(lay), 512, 32, 513, 0, by(n)) == 1  # k > S
    assert L.loki_workspace_bytes(by(lay), 512, 16, 8, 0, by(n)) == 2    # d != d_split
    assert L.loki_workspace_bytes(by(lay), 512, 32, 8, 7, by(n)) == 1    # bad mode
    assert L.loki_workspace_bytes(None, 512, 32, 8, 0, by(n)) == 1
    bad = api.Layout(2, 8, 3, 128, 32, 512, 1)
    assert L.loki_workspace_bytes(by(bad), 512, 32, 8, 0, by(n)) == 1    # Hq % Hkv
    bad = api.Layout(2, 8, 2, 64, 32, 512, 1)
    assert L.loki_workspace_bytes(by(bad), 512, 32, 8, 0, by(n)) == 2    # D != 128
    bad = api.Layout(2, 8, 2, 128, 12, 512, 1)
    assert L.loki_workspace_bytes(by(bad), 512, 12, 8, 0, by(n)) == 2    # 24-byte slab rows
    bad = api.Layout(2048, 32, 32, 128, 32, 512, 1)
    assert L.loki_workspace_bytes(by(bad), 512, 32, 8, 0, by(n)) == 2    # B * Hq beyond the grid limit
    bad = api.Layout(2, 8, 2, 128, 32, 512, 9)
    assert L.loki_workspace_bytes(by(bad), 512, 32, 8, 0, by(n)) == 2    # dtype
    # compute entry points: every failure below is detected on the host, nothing is launched
    p = 0x10000  # a non-null, aligned, never dereferenced address
    assert L.loki_decode_attn(by(lay), None, p, p, p, p, 512, 32, 8, 0, p, 1 << 30, p, None, None) == 1
    assert L.loki_decode_attn(by(lay), p, p, p, p, p, 512, 32, 600, 0, p, 1 << 30, p, None, None) == 1
    assert L.loki_decode_attn(by(lay), p, p, p, p, p, 600, 32, 8, 0, p, 1 << 30, p, None, None) == 1
    assert L.loki_decode_attn(by(lay), p, p, p, p, p, 512, 64, 8, 0, p, 1 << 30, p, None, None) == 2
    assert L.loki_decode_attn(by(lay), p + 4, p, p, p, p, 512, 32, 8, 0, p, 1 << 30, p, None, None) == 3
    assert L.loki_decode_attn(by(lay), p, p, p, p, p, 512, 32, 8, 0, p + 16, 1 << 30, p, None, None) == 3
    assert L.loki_decode_attn(by(lay), p, p, p, p, p, 512, 32, 8, 0, p, 16, p, None, None) == 4
    assert L.loki_decode_attn(by(lay), p, p, p, None, p, 512, 32, 8, 0, p, 1 << 30, p, None, None) == 1
    assert L.loki_rotate_keys(by(lay), p, p, p, p, 500, 13, None) == 1   # pos + n_new > S_cap
    assert L.loki_rotate_keys(by(lay), p, p, p, p, -1, 1, None) == 1
    assert L.loki_rotate_keys(by(lay), p, None, p, p, 0, 1, None) == 1
    assert L.dense_decode_attn(by(lay), p, p, p, 0, p, 1 << 30, p, None) == 1
    assert L.dense_decode_attn(by(lay), p, p + 2, p, 512, p, 1 << 30, p, None) == 3
    assert L.dense_decode_attn(by(lay), p, p, p, 512, p, 0, p, None) == 4
    flag = ctypes.c_int32(7)
    assert L.loki_cluster_gave_up(None, ctypes.byref(flag), None) == 1
    assert L.loki_cluster_gave_up(p, None, None) == 1
    assert L.loki_cluster_gave_up(p + 8, ctypes.byref(flag), None) == 3
    assert L.loki_stream_read(None, 1024, None) == 1
    assert L.loki_stream_read(p, 0, None) == 1
    assert L.loki_stream_read(p, 1000, None) == 1    # not a multiple of 16
    assert L.loki_stream_read(p + 8, 1024, None) == 1  # misaligned


def test_binding_refuses_cpu_tensors():
    lay = api.make_layout(1, 1, 1, 128, 32, 64, torch.float32)
    t = torch.zeros(128)
    with pytest.raises(ValueError):
        api.dense_decode_attn(lay, t, torch.zeros(64 * 128), torch.zeros(64 * 128), 64, None, t)
