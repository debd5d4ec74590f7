"""CPU oracle for Loki decode attention — TEST INFRASTRUCTURE, not the product.

A plain, slow, float64 numpy statement of what the hot path computes, written
from the paper (Loki: Low-rank Keys for Efficient Sparse Attention,
arXiv 2406.02542).  It shares no code with the HIP kernels and must never be
imported by the product path; only tests, the smoke check and the benchmark's
CPU-baseline leg use it.

Loki is an approximation of dense attention, so the oracle is Algorithm 1 taken
step by step in the paper's order and notation (no blocking, no fusion):

  line 3   qhat = q P                                  -> rotate_query
  line 3-4 khat = k P, appended to the cache           -> rotate_keys
  line 5   a_approx = qhat[:d] . Khat[:, :d]^T         -> approx_scores
  line 6   indices = topk(a_approx, k)                 -> topk_indices
  line 7-9 softmax(qhat Khat'^T / sqrt(D)) V'          -> attend_selected

and Eq. 1 (Section 2) for dense attention                -> dense_attention.

Readings of points the paper leaves open (each is also listed in the design
notes): the softmax of line 8 runs over the selected rows only (the prose of
Section 4.2 says the exact scores use the selected keys); the ranking scores
are unscaled and compared by signed value; ties go to the lowest position; no
mean-centring; P's columns are the components, most important first, and the
row-vector convention qhat = q P is used; V is never rotated.

Grouped-query attention (not treated by the paper, whose Algorithm 1 is per
query head): ``select_mode=0`` lets every query head pick its own k rows from
its KV head's cache (the literal reading); ``select_mode=1`` picks one set per
KV head from the maximum over the group's scores and every query head of the
group attends over that set.  Mode 1 is this build's own definition: parity
unpinned by the paper, pinned only by its reduction to mode 0 when G = 1.

Pins (tests/test_oracle_pins.py): d=D,k=S equals Eq. 1 on unrotated inputs
(Lemma 4.1); k=S equals Eq. 1 for any d; a hand-worked 2-D example with exact
rational softmax weights (tests/golden/); brute-force top-k; closed forms
(V=1, Khat=0, indicator V); permutation symmetry; Exact-TopK at d=D; the
planted spectrum recovered by an eigendecomposition; Eq. 2 on a geometric
spectrum; the printed 2.6x of the cost model.
"""
from __future__ import annotations

import math

import numpy as np

SELECT_PER_QUERY_HEAD = 0
SELECT_PER_KV_GROUP = 1


# ---------------------------------------------------------------------------
# storage rounding (the oracle's own implementation)
# ---------------------------------------------------------------------------
def to_bf16(x) -> np.ndarray:
    """Round to the nearest bfloat16, ties to even; returns float64 values that
    are exactly representable in bfloat16.  Input is first rounded to float32
    (float64 -> float32 -> bfloat16 double rounding can differ from a direct
    rounding only when the float64 value sits within 2^-29 relative of a
    bfloat16 tie, which the tests treat as a one-ulp case)."""
    f = np.asarray(x, dtype=np.float64).astype(np.float32)
    bits = f.view(np.uint32).astype(np.uint64)
    lsb = (bits >> np.uint64(16)) & np.uint64(1)
    bits = (bits + np.uint64(0x7FFF) + lsb) >> np.uint64(16) << np.uint64(16)
    return bits.astype(np.uint32).view(np.float32).astype(np.float64)


def to_storage(x, dtype: str) -> np.ndarray:
    if dtype == "bf16":
        return to_bf16(x)
    if dtype == "f32":
        return np.asarray(x, dtype=np.float64).astype(np.float32).astype(np.float64)
    raise ValueError(dtype)


# ---------------------------------------------------------------------------
# Eq. 1 — dense decode attention for one query head
# ---------------------------------------------------------------------------
def softmax(z: np.ndarray) -> np.ndarray:
    z = np.asarray(z, dtype=np.float64)
    e = np.exp(z - np.max(z))
    return e / np.sum(e)


def dense_attention(q, K, V) -> np.ndarray:
    """y = softmax(q K^T / sqrt(D)) V   (Section 2, Eq. 1).  q [D], K,V [S,D]."""
    q = np.asarray(q, dtype=np.float64)
    K = np.asarray(K, dtype=np.float64)
    V = np.asarray(V, dtype=np.float64)
    D = q.shape[0]
    return softmax((K @ q) / math.sqrt(D)) @ V


# ---------------------------------------------------------------------------
# Algorithm 1, one query head
# ---------------------------------------------------------------------------
def rotate_query(q, P) -> np.ndarray:
    """qhat = q P  (Algorithm 1 line 3; Lemma 4.1's transform)."""
    return np.asarray(q, dtype=np.float64) @ np.asarray(P, dtype=np.float64)


def rotate_keys(K, P) -> np.ndarray:
    """Khat = K P for a block of rows (Algorithm 1 lines 3-4), float64,
    not yet rounded to the cache's storage type.  K [n, D], P [D, D]."""
    return np.asarray(K, dtype=np.float64) @ np.asarray(P, dtype=np.float64)


def approx_scores(qhat, Khat, d: int) -> np.ndarray:
    """a_approx = qhat[:d] Khat[:, :d]^T  (Algorithm 1 line 5): unscaled."""
    qhat = np.asarray(qhat, dtype=np.float64)
    Khat = np.asarray(Khat, dtype=np.float64)
    return Khat[:, :d] @ qhat[:d]


def topk_indices(a, k: int) -> np.ndarray:
    """Positions of the k largest entries of a (Algorithm 1 line 6), returned in
    ascending position order; among equal scores the lowest position wins."""
    a = np.asarray(a, dtype=np.float64)
    order = np.argsort(-a, kind="stable")  # stable: equal scores keep position order
    return np.sort(order[:k])


def attend_selected(qhat, Khat, V, indices) -> np.ndarray:
    """Exact attention over the selected rows in the rotated space
    (Algorithm 1 lines 7-9): softmax(qhat Khat'^T / sqrt(D)) V'."""
    qhat = np.asarray(qhat, dtype=np.float64)
    Kp = np.asarray(Khat, dtype=np.float64)[indices]
    Vp = np.asarray(V, dtype=np.float64)[indices]
    D = qhat.shape[0]
    return softmax((Kp @ qhat) / math.sqrt(D)) @ Vp


def loki_attention(q, P, Khat, V, d: int, k: int):
    """Algorithm 1 lines 3 and 5-9 for one query head (the new key is assumed
    already appended).  Returns (out [D], indices [k], a_approx [S])."""
    qhat = rotate_query(q, P)
    a = approx_scores(qhat, Khat, d)
    idx = topk_indices(a, k)
    return attend_selected(qhat, Khat, V, idx), idx, a


# ---------------------------------------------------------------------------
# batched forms with grouped-query heads
# ---------------------------------------------------------------------------
def loki_decode_batch(q, P, Khat, V, d: int, k: int, select_mode: int = 0,
                      units=None):
    """q [B,Hq,D], P [Hkv,D,D], Khat,V [B,Hkv,S,D].

    Returns (out [B,Hq,D], idx [B,Hsel,k], scores [B,Hsel,S]) in float64 /
    int64, with Hsel = Hq (mode 0) or Hkv (mode 1).  ``units`` optionally
    restricts the work to a list of (b, kv_head) pairs; other entries stay NaN /
    -1."""
    B, Hq, D = q.shape
    Hkv = P.shape[0]
    G = Hq // Hkv
    S = Khat.shape[2]
    Hsel = Hq if select_mode == SELECT_PER_QUERY_HEAD else Hkv
    out = np.full((B, Hq, D), np.nan)
    idx = np.full((B, Hsel, k), -1, dtype=np.int64)
    scores = np.full((B, Hsel, S), np.nan)
    todo = units if units is not None else [(b, h) for b in range(B) for h in range(Hkv)]
    for b, h in todo:
        Kh = np.asarray(Khat[b, h], dtype=np.float64)
        Vh = np.asarray(V[b, h], dtype=np.float64)
        qhats = [rotate_query(q[b, h * G + g], P[h]) for g in range(G)]
        a = [approx_scores(qh, Kh, d) for qh in qhats]
        if select_mode == SELECT_PER_QUERY_HEAD:
            for g in range(G):
                hq = h * G + g
                sel = topk_indices(a[g], k)
                idx[b, hq] = sel
                scores[b, hq] = a[g]
                out[b, hq] = attend_selected(qhats[g], Kh, Vh, sel)
        else:
            group = np.max(np.stack(a), axis=0)
            sel = topk_indices(group, k)
            idx[b, h] = sel
            scores[b, h] = group
            for g in range(G):
                out[b, h * G + g] = attend_selected(qhats[g], Kh, Vh, sel)
    return out, idx, scores


def loki_decode_step(q, P, Khat, V, d: int, k_max: int, select_mode: int = 0,
                     seq_lens=None, ks=None, k_new=None, v_new=None, storage: str = "f32",
                     units=None, queries_per_seq: int = 1):
    """The whole step of Algorithm 1 (lines 2-9), sequence by sequence.

    Entry e of the batch holds seq_lens[e] rows (default: all S of Khat) and keeps ks[e] of
    them (default min(k_max, seq_lens[e])).  With k_new / v_new [E,Hkv,D] given, row
    seq_lens[e]-1 of each (entry, KV head) first becomes the rotated new key, rounded to
    the storage type (lines 3-4), and the new value.  Each entry is then
    loki_decode_batch on its own rows.

    queries_per_seq = m > 1: m consecutive entries (the last m tokens of one sequence)
    share one cached sequence: q [B m,Hq,D] against Khat, V [B,Hkv,S,D]; all their rows are
    appended first, then entry e attends over the first seq_lens[e] rows of sequence e // m
    (its causal limit).

    Returns (out [E,Hq,D], idx [E,Hsel,k_max] padded with -1, scores [E,Hsel,S]
    NaN past each entry's end, Khat, V): the last two are copies of the caches
    after the append."""
    E, Hq, D = q.shape
    Hkv = P.shape[0]
    S = Khat.shape[2]
    m = queries_per_seq
    assert E == Khat.shape[0] * m
    Hsel = Hq if select_mode == SELECT_PER_QUERY_HEAD else Hkv
    Khat = np.array(Khat, dtype=np.float64, copy=True)
    V = np.array(V, dtype=np.float64, copy=True)
    out = np.full((E, Hq, D), np.nan)
    idx = np.full((E, Hsel, k_max), -1, dtype=np.int64)
    scores = np.full((E, Hsel, S), np.nan)
    S_of = [S if seq_lens is None else int(seq_lens[e]) for e in range(E)]
    if k_new is not None:
        for e in range(E):
            for h in range(Hkv):
                if units is None or (e, h) in units:
                    Khat[e // m, h, S_of[e] - 1] = to_storage(rotate_keys(k_new[e, h][None, :], P[h])[0], storage)
                    V[e // m, h, S_of[e] - 1] = v_new[e, h]
    for e in range(E):
        S_e = S_of[e]
        k_e = min(k_max, S_e) if ks is None else int(ks[e])
        assert 1 <= k_e <= min(k_max, S_e) <= S
        heads = [h for h in range(Hkv) if units is None or (e, h) in units]
        c = e // m
        o, i, a = loki_decode_batch(q[e:e + 1], P, Khat[c:c + 1, :, :S_e], V[c:c + 1, :, :S_e], d,
                                    k_e, select_mode, units=[(0, h) for h in heads])
        out[e] = o[0]
        idx[e, :, :k_e] = i[0]
        scores[e, :, :S_e] = a[0]
    return out, idx, scores, Khat, V


def pca_attention(q, P, Khat, V, d: int) -> np.ndarray:
    """PCAAttn (Appendix E, Algorithm 2): the weights come from the first d rotated
    columns alone, over every row, still scaled by 1/sqrt(D):
    softmax(qhat[:d] Khat[:, :d]^T / sqrt(D)) V."""
    qhat = rotate_query(q, P)
    D = qhat.shape[0]
    return softmax(approx_scores(qhat, Khat, d) / math.sqrt(D)) @ np.asarray(V, dtype=np.float64)


def pca_attention_batch(q, P, Khat, V, d: int, units=None) -> np.ndarray:
    """PCAAttn for every query head; q [B,Hq,D], P [Hkv,D,D], Khat,V [B,Hkv,S,D]."""
    B, Hq, D = q.shape
    Hkv = P.shape[0]
    G = Hq // Hkv
    out = np.full((B, Hq, D), np.nan)
    todo = units if units is not None else [(b, h) for b in range(B) for h in range(Hkv)]
    for b, h in todo:
        for g in range(G):
            out[b, h * G + g] = pca_attention(q[b, h * G + g], P[h], Khat[b, h], V[b, h], d)
    return out


def dense_decode_batch(q, K, V, units=None) -> np.ndarray:
    """Eq. 1 for every query head; q [B,Hq,D], K,V [B,Hkv,S,D]."""
    B, Hq, D = q.shape
    Hkv = K.shape[1]
    G = Hq // Hkv
    out = np.full((B, Hq, D), np.nan)
    todo = units if units is not None else [(b, h) for b in range(B) for h in range(Hkv)]
    for b, h in todo:
        for g in range(G):
            out[b, h * G + g] = dense_attention(q[b, h * G + g], K[b, h], V[b, h])
    return out


def rotate_keys_batch(K, P) -> np.ndarray:
    """K [B,Hkv,n,D], P [Hkv,D,D] -> Khat float64, unrounded."""
    K = np.asarray(K, dtype=np.float64)
    out = np.empty_like(K)
    for h in range(K.shape[1]):
        for b in range(K.shape[0]):
            out[b, h] = rotate_keys(K[b, h], P[h])
    return out


# ---------------------------------------------------------------------------
# Section 3.1 / Section 4.2 helpers
# ---------------------------------------------------------------------------
def pca_basis(keys):
    """PCA of a set of keys [N, D] (Section 3.1): eigenvalues of the sample
    covariance in decreasing order and the matching eigenvectors as columns."""
    X = np.asarray(keys, dtype=np.float64)
    Xc = X - X.mean(axis=0, keepdims=True)
    cov = (Xc.T @ Xc) / (X.shape[0] - 1)
    lam, vec = np.linalg.eigh(cov)
    order = np.argsort(lam)[::-1]
    return lam[order], vec[:, order]


def rank_at(eigenvalues, v: float) -> int:
    """Rank@v (Section 3.1, Eq. 2): the smallest d whose leading normalised
    eigenvalues sum to at least v/100."""
    lam = np.sort(np.asarray(eigenvalues, dtype=np.float64))[::-1]
    lam = lam / lam.sum()
    running = 0.0
    for d, value in enumerate(lam, start=1):
        running += value
        if running >= v / 100.0:
            return d
    return len(lam)


def layer_rank_at(eigenvalues, v: float) -> float:
    """Rank_l@v (Section 3.1, below Eq. 2): Rank_{l,h}@v averaged over the heads of a layer;
    ``eigenvalues`` is [heads, D]."""
    lam = np.asarray(eigenvalues, dtype=np.float64)
    return float(np.mean([rank_at(lam[h], v) for h in range(lam.shape[0])]))


def layer_width(eigenvalues, v: float, multiple: int = 1) -> int:
    """Variable-width policy of Appendix B.2: a layer's d follows its explained variance.
    Reading: d is Rank_l@v of the layer, taken up to the next whole number and then to the
    next multiple of the cache layout's granularity, at most D."""
    lam = np.asarray(eigenvalues, dtype=np.float64)
    D = lam.shape[-1]
    d = int(math.ceil(layer_rank_at(lam, v)))
    d = -(-d // multiple) * multiple
    return min(d, D)


def jaccard(a, b) -> float:
    """|A n B| / |A u B| of two index sets (Section 6.3 compares the selection of Loki with
    that of exact top-k this way); negative entries are padding."""
    A = {int(x) for x in a if x >= 0}
    B = {int(x) for x in b if x >= 0}
    return len(A & B) / len(A | B) if (A or B) else 1.0


def theoretical_speedup(D: int, S: int, d: int, k: int, exact: bool = True) -> float:
    """Section 4.2 cost model: 2DS / (dS + 2Dk + 2D^2), or its large-S limit
    1 / (d_f/2 + k_f) when ``exact`` is False."""
    if exact:
        return (2.0 * D * S) / (d * S + 2.0 * D * k + 2.0 * D * D)
    return 1.0 / ((d / D) / 2.0 + k / S)
