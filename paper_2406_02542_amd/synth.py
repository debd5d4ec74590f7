"""Seeded synthetic inputs for Loki decode attention (numpy only).

This module is the one piece of code that both the CPU oracle's tests and the
HIP path's tests/benchmarks use: it produces *data* (queries, PCA bases, key and
value caches) and holds none of the method's arithmetic.  Nothing here imports
the oracle or the HIP binding.

Recipe (stands in for the real model keys the paper's micro-benchmark ran on,
Section 6.4 / Figure 7: a Llama-2-13B-shaped attention layer; the paper's key
property is a fast-decaying PCA spectrum, Section 3 / Appendix A.1):

* ``P_h``: Q factor of a D x D matrix of N(0,1) draws, signs fixed so that the
  diagonal of R is positive; one per KV head (or one shared by all heads).
  Columns are the "principal components", most important first.  Stored fp32.
* rotated keys ``Khat[s, i] = c * sqrt(sigma_i^2 + nu)`` with ``c ~ N(0,1)``,
  ``sigma_i = exp(-i / tau)``, ``i = 0..D-1``: the same law as
  ``(c' * sigma) + eps`` with ``eps ~ N(0, nu)`` because both terms are
  independent centred Gaussians.  Unrotated keys, where a test needs them, are
  ``K = Khat_unrounded @ P_h^T``.
* ``q``, ``V`` ~ N(0,1).
* "heavy" variant: 64 planted key positions per (batch, KV head) are pushed
  along the direction ``w = P_h (sigma/|sigma|)`` by ``gamma`` and every query of
  the group is ``beta * w + N(0, I)``, which gives a peaked attention
  distribution on those positions.
* every array is rounded (round-to-nearest-even) to the storage dtype and
  returned as float32 holding exactly-representable values, so the GPU side can
  cast to bf16 without a second rounding and the oracle reads the same numbers.
"""
from __future__ import annotations

import dataclasses
from concurrent.futures import ThreadPoolExecutor
from typing import Optional

import numpy as np

BASE_SEED = 240602542


@dataclasses.dataclass(frozen=True)
class Workload:
    """Shape and generator parameters of one synthetic decode-attention case."""

    name: str
    B: int
    Hq: int
    Hkv: int
    D: int
    S: int
    dtype: str  # "f32" | "bf16"
    d: int
    k: int
    tau: float = 20.0
    noise_var: float = 0.01
    shared_P: bool = False
    heavy: bool = False
    seed: int = BASE_SEED

    @property
    def G(self) -> int:
        return self.Hq // self.Hkv

    @property
    def elem_bytes(self) -> int:
        return 4 if self.dtype == "f32" else 2

    def replace(self, **kw) -> "Workload":
        return dataclasses.replace(self, **kw)


def paper_configs() -> dict:
    """The five benchmark configurations (shapes follow the paper's
    micro-benchmark set-up in Section 5 / Section 6.4, scaled to GQA and long
    context); config 5 is a sweep and is returned at d=32, k_f=0.125."""
    return {
        "tiny": Workload("tiny", 1, 8, 8, 128, 1024, "f32", 32, 256, tau=20.0,
                         shared_P=True, seed=BASE_SEED + 0),
        "llama2_7b": Workload("llama2_7b", 16, 32, 32, 128, 4096, "bf16", 32, 1024,
                              tau=20.0, seed=BASE_SEED + 1),
        "llama3_8b_gqa": Workload("llama3_8b_gqa", 16, 32, 8, 128, 16384, "bf16", 32, 2048,
                                  tau=25.0, seed=BASE_SEED + 2),
        "long_gqa": Workload("long_gqa", 4, 32, 8, 128, 131072, "bf16", 16, 8192,
                             tau=20.0, heavy=True, seed=BASE_SEED + 3),
        "large_share": Workload("large_share", 64, 64, 8, 128, 8192, "bf16", 32, 1024,
                                tau=20.0, seed=BASE_SEED + 4),
    }


def large_share_sweep() -> list:
    """Config 5's nine (d, k_f) points."""
    base = paper_configs()["large_share"]
    out = []
    for d in (16, 32, 64):
        for kf in (0.0625, 0.125, 0.25):
            out.append(base.replace(name=f"large_share_d{d}_k{int(base.S * kf)}",
                                    d=d, k=int(base.S * kf)))
    return out


# --------------------------------------------------------------------------
# storage rounding (the generator's own; the oracle and the kernels have theirs)
# --------------------------------------------------------------------------
def round_bf16(x: np.ndarray) -> np.ndarray:
    """Round float32 values to the nearest bfloat16 (ties to even); the result
    is float32 whose low 16 mantissa bits are zero."""
    x = np.ascontiguousarray(x, dtype=np.float32)
    u = x.view(np.uint32)
    r = (u + np.uint32(0x7FFF) + ((u >> np.uint32(16)) & np.uint32(1))) & np.uint32(0xFFFF0000)
    return r.view(np.float32)


def round_storage(x: np.ndarray, dtype: str) -> np.ndarray:
    if dtype == "bf16":
        return round_bf16(x)
    if dtype == "f32":
        return np.ascontiguousarray(x, dtype=np.float32)
    raise ValueError(f"unknown storage dtype {dtype!r}")


# --------------------------------------------------------------------------
# generators
# --------------------------------------------------------------------------
def _rng(seed: int, tensor_id: int, unit: int = 0) -> np.random.Generator:
    return np.random.Generator(np.random.Philox(key=[(seed << 20) ^ tensor_id, unit]))


_T_P, _T_K, _T_V, _T_Q, _T_HEAVY, _T_LEN, _T_KNEW, _T_VNEW = 1, 2, 3, 4, 5, 6, 7, 8


def spectrum(D: int, tau: float) -> np.ndarray:
    """Planted standard deviations sigma_i = exp(-i/tau), i = 0..D-1 (float64)."""
    return np.exp(-np.arange(D, dtype=np.float64) / tau)


def orthogonal_basis(seed: int, head: int, D: int) -> np.ndarray:
    """One D x D orthogonal matrix (float64): Q of a Gaussian matrix with the
    sign convention diag(R) > 0."""
    a = _rng(seed, _T_P, head).standard_normal((D, D))
    qm, rm = np.linalg.qr(a)
    return qm * np.sign(np.diag(rm))[None, :]


def make_P(w: Workload) -> np.ndarray:
    """[Hkv, D, D] float32."""
    if w.shared_P:
        p = orthogonal_basis(w.seed, 0, w.D)
        return np.broadcast_to(p, (w.Hkv, w.D, w.D)).astype(np.float32).copy()
    return np.stack([orthogonal_basis(w.seed, h, w.D) for h in range(w.Hkv)]).astype(np.float32)


def heavy_positions(w: Workload, unit: int, n: int = 64) -> np.ndarray:
    return np.sort(_rng(w.seed, _T_HEAVY, unit).choice(w.S, size=min(n, w.S), replace=False))


HEAVY_GAMMA = 4.0
HEAVY_BETA = 32.0


def _khat_unit_f32(w: Workload, unit: int) -> np.ndarray:
    """Unrounded rotated keys of one (batch, KV head) unit, [S, D] float32."""
    scale = np.sqrt(spectrum(w.D, w.tau) ** 2 + w.noise_var).astype(np.float32)
    x = _rng(w.seed, _T_K, unit).standard_normal((w.S, w.D), dtype=np.float32)
    x *= scale[None, :]
    if w.heavy:
        sig = spectrum(w.D, w.tau)
        what = (sig / np.linalg.norm(sig)).astype(np.float32)
        x[heavy_positions(w, unit)] += np.float32(HEAVY_GAMMA) * what[None, :]
    return x


def _parallel_units(fn, n_units: int, threads: int):
    if threads <= 1 or n_units <= 1:
        return [fn(u) for u in range(n_units)]
    with ThreadPoolExecutor(max_workers=threads) as ex:
        return list(ex.map(fn, range(n_units)))


def make_khat(w: Workload, threads: int = 8) -> np.ndarray:
    """Rotated key cache [B, Hkv, S, D], storage-rounded float32."""
    out = np.empty((w.B * w.Hkv, w.S, w.D), dtype=np.float32)

    def fill(u):
        out[u] = round_storage(_khat_unit_f32(w, u), w.dtype)

    _parallel_units(fill, w.B * w.Hkv, threads)
    return out.reshape(w.B, w.Hkv, w.S, w.D)


def make_unrotated_keys(w: Workload, P: np.ndarray, threads: int = 8) -> np.ndarray:
    """Keys in the model's own basis, K = Khat_unrounded @ P_h^T, storage-rounded
    float32 [B, Hkv, S, D].  Meant for small cases (it is the input of
    ``loki_rotate_keys``)."""
    out = np.empty((w.B * w.Hkv, w.S, w.D), dtype=np.float32)

    def fill(u):
        h = u % w.Hkv
        k = _khat_unit_f32(w, u).astype(np.float64) @ P[h].astype(np.float64).T
        out[u] = round_storage(k.astype(np.float32), w.dtype)

    _parallel_units(fill, w.B * w.Hkv, threads)
    return out.reshape(w.B, w.Hkv, w.S, w.D)


def make_v(w: Workload, threads: int = 8) -> np.ndarray:
    """Value cache [B, Hkv, S, D], storage-rounded float32."""
    out = np.empty((w.B * w.Hkv, w.S, w.D), dtype=np.float32)

    def fill(u):
        out[u] = round_storage(
            _rng(w.seed, _T_V, u).standard_normal((w.S, w.D), dtype=np.float32), w.dtype)

    _parallel_units(fill, w.B * w.Hkv, threads)
    return out.reshape(w.B, w.Hkv, w.S, w.D)


def make_q(w: Workload, P: Optional[np.ndarray] = None) -> np.ndarray:
    """Queries [B, Hq, D] in the model's own (unrotated) basis, storage-rounded
    float32.  The heavy variant needs ``P`` to place the planted direction."""
    q = _rng(w.seed, _T_Q).standard_normal((w.B, w.Hq, w.D))
    if w.heavy:
        if P is None:
            raise ValueError("heavy workloads need P to build queries")
        sig = spectrum(w.D, w.tau)
        u = sig / np.linalg.norm(sig)
        for h in range(w.Hq):
            wdir = P[h // w.G].astype(np.float64) @ u
            q[:, h, :] += HEAVY_BETA * wdir[None, :]
    return round_storage(q.astype(np.float32), w.dtype)


def split_cache(khat: np.ndarray, d: int):
    """Split [..., S, D] rotated keys into the low-rank slab [..., S, d] and the
    residual slab [..., S, D-d] (both contiguous copies)."""
    return np.ascontiguousarray(khat[..., :d]), np.ascontiguousarray(khat[..., d:])


def make_inputs(w: Workload, threads: int = 8) -> dict:
    """All decode-step inputs of a workload: q, P, Khat (rotated cache), V."""
    P = make_P(w)
    return {
        "P": P,
        "q": make_q(w, P),
        "khat": make_khat(w, threads),
        "v": make_v(w, threads),
    }


def make_step_inputs(w: Workload, P: np.ndarray, ragged: bool = True, min_frac: float = 0.25) -> dict:
    """Per-sequence sizes and the current token's key / value for a whole decode step.

    * ``seq_lens`` [B] int32: a length mix of a serving batch, S * u with u uniform in
      [min_frac, 1]; sequence 0 is full (S) and, with B > 1, sequence 1 is the shortest
      allowed, so both ends are always present.  ``ragged=False``: all S.
    * ``ks`` [B] int32: max(1, floor(k_f * seq_len)) with k_f = k / S (Section 4.2
      states k as a fraction of the sequence).
    * ``k_new`` [B, Hkv, D]: one more key per unit from the cache's law, in the model's
      own basis (unrounded rotated draw @ P_h^T), storage-rounded float32.
    * ``v_new`` [B, Hkv, D] ~ N(0,1), storage-rounded float32."""
    g = _rng(w.seed, _T_LEN)
    lo = max(1, int(np.ceil(min_frac * w.S)))
    lens = g.integers(lo, w.S + 1, size=w.B).astype(np.int32) if ragged else np.full(w.B, w.S, np.int32)
    if ragged:
        lens[0] = w.S
        if w.B > 1:
            lens[1] = lo
    ks = np.maximum(1, (w.k * lens.astype(np.int64)) // w.S)  # floor(k_f * seq_len) in integers
    ks = np.minimum(ks, np.minimum(lens, w.k)).astype(np.int32)
    scale = np.sqrt(spectrum(w.D, w.tau) ** 2 + w.noise_var)
    c = _rng(w.seed, _T_KNEW).standard_normal((w.B, w.Hkv, w.D)) * scale[None, None, :]
    k_new = np.einsum("bhj,hij->bhi", c, P.astype(np.float64))  # c @ P_h^T
    v_new = _rng(w.seed, _T_VNEW).standard_normal((w.B, w.Hkv, w.D))
    return {"seq_lens": lens, "ks": ks,
            "k_new": round_storage(k_new.astype(np.float32), w.dtype),
            "v_new": round_storage(v_new.astype(np.float32), w.dtype)}
