"""ctypes binding of the plain-C fp64 oracle (test infrastructure, not product code).

The oracle is the plain definition of the modelled retrieval step of the paper's
State Selector / Optimization Selector (Section 3): cosine of the decoded stored bits,
optional tag filter ``(qmask & tag) != 0``, full sort by (score desc, index asc),
first k, padded with (-1, -inf).  All arithmetic lives in ``kb_oracle.c``; this file
only marshals numpy arrays.
"""
from __future__ import annotations

import ctypes
import os
import subprocess

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "kb_oracle.c")
_LIB = os.path.join(_HERE, "libkb_oracle.so")

F32, BF16, FP8_E4M3 = 0, 1, 2
_ELEM_BYTES = {F32: 4, BF16: 2, FP8_E4M3: 1}

_lib = None


def build(force: bool = False) -> str:
    """Compile kb_oracle.c with gcc into libkb_oracle.so beside it."""
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        subprocess.check_call(
            ["gcc", "-O2", "-fopenmp", "-shared", "-fPIC", "-Wall", "-Wextra", "-o", _LIB, _SRC, "-lm"]
        )
    return _LIB


def lib() -> ctypes.CDLL:
    global _lib
    if _lib is None:
        L = ctypes.CDLL(build())
        vp, i64, i32, dbl = ctypes.c_void_p, ctypes.c_int64, ctypes.c_int, ctypes.c_double
        L.oracle_decode_bf16.restype = dbl
        L.oracle_decode_bf16.argtypes = [ctypes.c_uint16]
        L.oracle_decode_e4m3.restype = dbl
        L.oracle_decode_e4m3.argtypes = [ctypes.c_uint8]
        L.oracle_score_matrix.restype = i32
        L.oracle_score_matrix.argtypes = [vp, i32, vp, i64, i64, vp, i32, i64, vp]
        L.oracle_select.restype = i64
        L.oracle_select.argtypes = [vp, i64, vp, i32, ctypes.c_uint64, i64, vp, vp]
        L.oracle_query.restype = i32
        L.oracle_query.argtypes = [vp, i32, vp, vp, i64, i64, vp, i32, i64, vp, i64, vp, vp, vp]
        L.oracle_philox4x32_10.restype = None
        L.oracle_philox4x32_10.argtypes = [vp, vp, vp]
        L.oracle_uniform.restype = dbl
        L.oracle_uniform.argtypes = [ctypes.c_uint64, ctypes.c_uint32, ctypes.c_uint64]
        L.oracle_gumbel.restype = dbl
        L.oracle_gumbel.argtypes = [ctypes.c_uint64, ctypes.c_uint32, ctypes.c_uint64]
        L.oracle_selection_keys.restype = i32
        L.oracle_selection_keys.argtypes = [vp, i64, i64, vp, dbl, ctypes.c_uint64, i64, vp]
        L.oracle_encode_e4m3.restype = ctypes.c_uint8
        L.oracle_encode_e4m3.argtypes = [ctypes.c_float]
        L.oracle_quantize_rows.restype = i32
        L.oracle_quantize_rows.argtypes = [vp, i32, i64, i64, vp, vp]
        L.oracle_num_threads.restype = i32
        L.oracle_num_threads.argtypes = []
        _lib = L
    return _lib


def _bits(a: np.ndarray, dtype: int, name: str) -> np.ndarray:
    """Stored bits as a C-contiguous array of the right element width (no value conversion)."""
    want = {F32: (np.float32,), BF16: (np.uint16,), FP8_E4M3: (np.uint8,)}[dtype]
    a = np.ascontiguousarray(a)
    if a.dtype.type not in want:
        raise TypeError(f"{name}: dtype code {dtype} needs {want[0].__name__} bits, got {a.dtype}")
    if a.ndim != 2:
        raise ValueError(f"{name} must be 2-D")
    return a


def _ptr(a):
    return None if a is None else a.ctypes.data_as(ctypes.c_void_p)


def decode_bf16(bits: int) -> float:
    return lib().oracle_decode_bf16(int(bits))


def decode_e4m3(code: int) -> float:
    return lib().oracle_decode_e4m3(int(code))


def encode_e4m3(y: float) -> int:
    return lib().oracle_encode_e4m3(float(y))


def quantize_rows(rows, dtype: int):
    """(codes uint8 [n, d], scale float32 [n]) of float32 / bf16-bit rows: per-row scale max|x| / 448, nearest e4m3 code."""
    rows = _bits(rows, dtype, "rows")
    n, d = rows.shape
    codes = np.empty((n, d), dtype=np.uint8)
    scale = np.empty(n, dtype=np.float32)
    rc = lib().oracle_quantize_rows(_ptr(rows), dtype, n, d, _ptr(codes), _ptr(scale))
    if rc:
        raise RuntimeError(f"oracle_quantize_rows failed ({rc})")
    return codes, scale


def num_threads() -> int:
    return lib().oracle_num_threads()


def score_matrix(keys, key_dtype, queries, q_dtype, row_scale=None) -> np.ndarray:
    """[Q, N] fp64 cosine scores of the stored bits."""
    keys = _bits(keys, key_dtype, "keys")
    queries = _bits(queries, q_dtype, "queries")
    N, d = keys.shape
    Q, dq = queries.shape
    if d != dq:
        raise ValueError("keys and queries disagree on d")
    if row_scale is not None:
        row_scale = np.ascontiguousarray(row_scale, dtype=np.float32)
        assert row_scale.shape == (N,)
    out = np.empty((Q, N), dtype=np.float64)
    rc = lib().oracle_score_matrix(_ptr(keys), key_dtype, _ptr(row_scale), N, d, _ptr(queries), q_dtype, Q, _ptr(out))
    if rc:
        raise RuntimeError(f"oracle_score_matrix failed ({rc})")
    return out


def select(scores, k, tags=None, qmask=None):
    """Top-k of one query's score vector; returns (index int64[k], score float64[k], n_candidates)."""
    scores = np.ascontiguousarray(scores, dtype=np.float64)
    assert scores.ndim == 1
    use_mask = qmask is not None
    if use_mask:
        tags = np.ascontiguousarray(tags, dtype=np.uint64)
        assert tags.shape == scores.shape
    idx = np.empty(k, dtype=np.int64)
    sc = np.empty(k, dtype=np.float64)
    n = lib().oracle_select(_ptr(scores), scores.shape[0], _ptr(tags) if use_mask else None, int(use_mask),
                            int(qmask) if use_mask else 0, k, _ptr(idx), _ptr(sc))
    if n < 0:
        raise RuntimeError("oracle_select failed")
    return idx, sc, int(n)


def philox4x32_10(ctr, key):
    """One call of the counter-based generator: four 32-bit words from a 4-word counter and a 2-word key."""
    c = np.ascontiguousarray(ctr, dtype=np.uint32)
    kk = np.ascontiguousarray(key, dtype=np.uint32)
    assert c.shape == (4,) and kk.shape == (2,)
    out = np.empty(4, dtype=np.uint32)
    lib().oracle_philox4x32_10(_ptr(c), _ptr(kk), _ptr(out))
    return out


def uniform(seed: int, query: int, entry: int) -> float:
    return lib().oracle_uniform(seed, query, entry)


def gumbel(seed: int, query: int, entry: int) -> float:
    return lib().oracle_gumbel(seed, query, entry)


def selection_keys(scores, gain, temperature: float, seed: int, first_query: int = 0) -> np.ndarray:
    """Keys of the weighted random selection, float64 [Q, N]: score / T + ln(gain) + Gumbel(seed, query, entry)."""
    scores = np.ascontiguousarray(scores, dtype=np.float64)
    assert scores.ndim == 2
    gain = np.ascontiguousarray(gain, dtype=np.float32)
    assert gain.shape == (scores.shape[1],)
    keys = np.empty_like(scores)
    rc = lib().oracle_selection_keys(_ptr(scores), scores.shape[0], scores.shape[1], _ptr(gain), float(temperature), seed,
                                     first_query, _ptr(keys))
    if rc != 0:
        raise RuntimeError(f"oracle_selection_keys failed ({rc})")
    return keys


# ---- knowledge-base maintenance: the numeric side of the paper's ParameterUpdate step (Section 3, the outer loop of
# Algorithm 2: after the rollouts the predicted gains in the knowledge base are revised from the measured ones), and
# removal of entries (knowledge-base management, named as future work in the paper's conclusion).  The paper gives
# neither a formula; the model: predicted gains move towards observed gains by an exponential moving average, a
# removed entry is never a candidate again, and compaction closes the gaps without changing the order of the rest.

def update_gain(gain, indices, values, alpha: float) -> np.ndarray:
    """gain[i] <- (1 - alpha) * gain[i] + alpha * value for each (i, value) pair, in fp64, pairs taken in order;
    an index outside [0, len(gain)) (the -1 padding of a result list) is skipped.  Returns a float64 copy."""
    g = np.array(gain, dtype=np.float64)
    for i, v in zip(np.asarray(indices).tolist(), np.asarray(values, dtype=np.float64).tolist()):
        if 0 <= i < g.shape[0]:
            g[i] = (1.0 - alpha) * g[i] + alpha * v
    return g


def without_removed(scores, removed) -> np.ndarray:
    """Scores (or selection keys) [Q, N] with every removed entry's column at -inf: never a candidate (select skips -inf)."""
    out = np.array(scores, dtype=np.float64)
    out[:, np.asarray(removed, dtype=bool)] = -np.inf
    return out


def compact(removed, *arrays):
    """Stable removal: (index_map int32 [n]: new index of each old entry or -1, [a[live] for a in arrays])."""
    removed = np.asarray(removed, dtype=bool)
    index_map = np.full(removed.shape[0], -1, dtype=np.int32)
    nxt = 0
    for i in range(removed.shape[0]):
        if not removed[i]:
            index_map[i] = nxt
            nxt += 1
    live = np.flatnonzero(~removed)
    return index_map, [np.ascontiguousarray(np.asarray(a)[live]) for a in arrays]


# ---- two-stage retrieval: the paper's knowledge base is a hierarchy, states first and each state's candidate
# optimizations below it (Section 3, the knowledge-base format figure and the walk through one task: the state is
# matched first, its optimizations are looked at afterwards).  Numeric model: entries are grouped into clusters
# ("states"), rows of cluster c are [offsets[c], offsets[c+1]); a query first ranks the cluster centroids like any
# other keys, keeps the best `nprobe` clusters, and the exact retrieval then runs over the rows of those clusters
# only.  An approximation of the exact retrieval by construction; its quality is reported as recall@k.

def restricted_to_clusters(scores, cluster_offsets, probe) -> np.ndarray:
    """scores [Q, N] with, for query r, every row outside the clusters probe[r, :] at -inf (never a candidate).
    Entries of probe outside [0, C) (the -1 padding of a result list) are skipped."""
    out = np.full(np.shape(scores), -np.inf, dtype=np.float64)
    scores = np.asarray(scores, dtype=np.float64)
    off = np.asarray(cluster_offsets, dtype=np.int64)
    C = off.shape[0] - 1
    for r in range(scores.shape[0]):
        for c in np.asarray(probe[r]).tolist():
            if 0 <= c < C:
                out[r, off[c]:off[c + 1]] = scores[r, off[c]:off[c + 1]]
    return out


def two_stage(keys, key_dtype, centroids, centroid_dtype, cluster_offsets, queries, q_dtype, nprobe, k, row_scale=None,
              tags=None, qmask=None):
    """(index [Q, k], score [Q, k], probe [Q, nprobe], restricted scores [Q, N]): centroid ranking, then exact
    retrieval over the rows of the nprobe best clusters."""
    probe, _ = query(centroids, centroid_dtype, queries, q_dtype, nprobe)
    full = restricted_to_clusters(score_matrix(keys, key_dtype, queries, q_dtype, row_scale=row_scale), cluster_offsets, probe)
    Q = full.shape[0]
    idx = np.empty((Q, k), dtype=np.int64)
    sc = np.empty((Q, k), dtype=np.float64)
    for r in range(Q):
        idx[r], sc[r], _ = select(full[r], k, tags=tags, qmask=None if qmask is None else qmask[r])
    return idx, sc, probe, full


def recall_at_k(found, exact) -> float:
    """Mean over queries of |found ∩ exact| / |exact| (valid entries only; a query with no exact entry counts as 1)."""
    tot = 0.0
    for f, e in zip(np.asarray(found), np.asarray(exact)):
        e = set(int(x) for x in e if x >= 0)
        f = set(int(x) for x in f if x >= 0)
        tot += 1.0 if not e else len(e & f) / len(e)
    return tot / len(found)


def query(keys, key_dtype, queries, q_dtype, k, row_scale=None, tags=None, qmask=None, return_scores=False):
    """Full retrieval.  Returns (index int64[Q,k], score float64[Q,k][, scores float64[Q,N]])."""
    keys = _bits(keys, key_dtype, "keys")
    queries = _bits(queries, q_dtype, "queries")
    N, d = keys.shape
    Q, dq = queries.shape
    if d != dq:
        raise ValueError("keys and queries disagree on d")
    if row_scale is not None:
        row_scale = np.ascontiguousarray(row_scale, dtype=np.float32)
        assert row_scale.shape == (N,)
    if qmask is not None:
        if tags is None:
            raise ValueError("qmask given for an untagged knowledge base")
        tags = np.ascontiguousarray(tags, dtype=np.uint64)
        qmask = np.ascontiguousarray(qmask, dtype=np.uint64)
        assert tags.shape == (N,) and qmask.shape == (Q,)
    idx = np.empty((Q, k), dtype=np.int64)
    sc = np.empty((Q, k), dtype=np.float64)
    full = np.empty((Q, N), dtype=np.float64) if return_scores else None
    rc = lib().oracle_query(_ptr(keys), key_dtype, _ptr(row_scale), _ptr(tags) if qmask is not None else None, N, d,
                            _ptr(queries), q_dtype, Q, _ptr(qmask), k, _ptr(idx), _ptr(sc), _ptr(full))
    if rc:
        raise RuntimeError(f"oracle_query failed ({rc})")
    return (idx, sc, full) if return_scores else (idx, sc)
