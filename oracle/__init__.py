"""CPU oracle for Sparse Causal Flash Attention -- TEST INFRASTRUCTURE ONLY.

Only ``tests/``, ``__graft_entry__.smoke()`` and the ``cpu_baseline`` leg of
``bench.py`` may import this package.  It shares no code with the HIP path and
never imports it.

Floating-point part: ``scfa_oracle.c`` (plain C, fp64), the definition of masked
causal softmax attention and its derivatives written out on the original,
unpermuted tensors (paper Sec. 3: the method computes exact attention under the mask, no approximation,
so the oracle is that computation's plain definition).

Integer part (this file, numpy): the stable sort by bucket and the compaction
of kept tokens (paper Sec. 3.1, 3.2 and the pre-processing of App. B.2), the
tile ranges of Alg. 1 and Alg. 2 taken in the paper's order, and brute-force
tile occupancy.

Bucketing (numpy, fp64): the cross-polytope LSH the paper adopts for its hash-sparse
experiments (Sec. 4.2 "Hashing mechanism": the scheme of Andoni et al. with a chosen number
of hash codes), in the form the benchmark definition states: argmax over [xR, -xR].

Conventions: tensors are ``[S, T, d]`` float64 with ``S`` the flattened
(batch, head) segments; labels are ``[S, T]`` int32 (bucket ids for the hash
variant, 0/1 keep flags for QK-dropping).
"""
from __future__ import annotations

import ctypes
import os
import subprocess
import sys

import numpy as np

HASH = 0
QKDROP = 1

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "scfa_oracle.c")
_LIB = os.path.join(_HERE, "libscfa_oracle.so")
_lib = None


def build(force: bool = False) -> str:
    """Compile the C oracle with gcc (fp64, OpenMP over independent outputs)."""
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        # no -ffast-math: the oracle keeps IEEE semantics and the written summation order
        cmd = ["gcc", "-O2", "-fopenmp", "-fPIC", "-shared", "-std=c11", "-Wall", "-Wextra",
               "-o", _LIB, _SRC, "-lm"]
        subprocess.run(cmd, check=True)
    return _LIB


def _load():
    global _lib
    if _lib is None:
        build()
        lib = ctypes.CDLL(_LIB)
        dp = ctypes.POINTER(ctypes.c_double)
        ip = ctypes.POINTER(ctypes.c_int32)
        ci, cd = ctypes.c_int, ctypes.c_double
        lib.scfa_oracle_forward_rows.argtypes = [dp, dp, dp, ip, ip, ci, ci, ci, ci, cd,
                                                 ip, ci, dp, dp, dp, dp]
        lib.scfa_oracle_forward_rows.restype = None
        lib.scfa_oracle_probs.argtypes = [dp, dp, ip, ip, ci, ci, ci, ci, cd, dp]
        lib.scfa_oracle_probs.restype = None
        lib.scfa_oracle_row_stats.argtypes = [dp, dp, dp, dp, ip, ip, ci, ci, ci, ci, cd,
                                              dp, dp, dp]
        lib.scfa_oracle_row_stats.restype = None
        lib.scfa_oracle_dq_rows.argtypes = [dp, dp, dp, dp, ip, ip, ci, ci, ci, ci, cd,
                                            ip, ci, dp]
        lib.scfa_oracle_dq_rows.restype = None
        lib.scfa_oracle_dkdv_rows.argtypes = [dp, dp, dp, dp, ip, ip, ci, ci, ci, ci, cd,
                                              dp, dp, dp, ip, ci, dp, dp]
        lib.scfa_oracle_dkdv_rows.restype = None
        lib.scfa_oracle_count_pairs.argtypes = [ip, ip, ci, ci, ci]
        lib.scfa_oracle_count_pairs.restype = ctypes.c_longlong
        _lib = lib
    return _lib


def _f64(a):
    a = np.ascontiguousarray(a, dtype=np.float64)
    return a, a.ctypes.data_as(ctypes.POINTER(ctypes.c_double))


def _i32(a):
    a = np.ascontiguousarray(a, dtype=np.int32)
    return a, a.ctypes.data_as(ctypes.POINTER(ctypes.c_int32))


def _seg_args(Q, K, V, lab_q, lab_k):
    Q = np.ascontiguousarray(Q, dtype=np.float64)
    K = np.ascontiguousarray(K, dtype=np.float64)
    V = np.ascontiguousarray(V, dtype=np.float64)
    lab_q = np.ascontiguousarray(lab_q, dtype=np.int32)
    lab_k = np.ascontiguousarray(lab_k, dtype=np.int32)
    assert Q.ndim == 3 and Q.shape == K.shape == V.shape, "expect [S,T,d] with T_Q == T_KV"
    assert lab_q.shape == Q.shape[:2] and lab_k.shape == Q.shape[:2]
    return Q, K, V, lab_q, lab_k


# --------------------------------------------------------------------------
# floating point: masked causal attention, forward and backward
# --------------------------------------------------------------------------

def attention_forward(Q, K, V, lab_q, lab_k, variant, tau, strict=False, rows=None,
                      return_stats=False):
    """O and LSE of the definition in ``scfa_oracle.c`` (paper Sec. 3).

    ``rows``: optional 1-D list of query positions; then only those rows are
    computed (the same rows in every segment) and the outputs are
    ``[S, len(rows), d]`` / ``[S, len(rows)]``.
    """
    lib = _load()
    Q, K, V, lab_q, lab_k = _seg_args(Q, K, V, lab_q, lab_k)
    S, T, d = Q.shape
    rows = np.arange(T, dtype=np.int32) if rows is None else np.asarray(rows, dtype=np.int32)
    rows, rows_p = _i32(rows)
    n = rows.shape[0]
    O = np.zeros((S, n, d)); LSE = np.zeros((S, n)); M = np.zeros((S, n)); L = np.zeros((S, n))
    dp = ctypes.POINTER(ctypes.c_double)
    for s in range(S):
        lib.scfa_oracle_forward_rows(_f64(Q[s])[1], _f64(K[s])[1], _f64(V[s])[1],
                                     _i32(lab_q[s])[1], _i32(lab_k[s])[1],
                                     int(variant), int(bool(strict)), T, d, float(tau),
                                     rows_p, n,
                                     O[s].ctypes.data_as(dp), LSE[s].ctypes.data_as(dp),
                                     M[s].ctypes.data_as(dp), L[s].ctypes.data_as(dp))
    if return_stats:
        return O, LSE, M, L
    return O, LSE


def attention_probs(Q, K, lab_q, lab_k, variant, tau, strict=False):
    """Dense P ``[S, T, T]`` (zeros where masked); small T only."""
    lib = _load()
    Q = np.ascontiguousarray(Q, dtype=np.float64)
    K = np.ascontiguousarray(K, dtype=np.float64)
    lab_q = np.ascontiguousarray(lab_q, dtype=np.int32)
    lab_k = np.ascontiguousarray(lab_k, dtype=np.int32)
    S, T, d = Q.shape
    P = np.zeros((S, T, T))
    dp = ctypes.POINTER(ctypes.c_double)
    for s in range(S):
        lib.scfa_oracle_probs(_f64(Q[s])[1], _f64(K[s])[1], _i32(lab_q[s])[1], _i32(lab_k[s])[1],
                              int(variant), int(bool(strict)), T, d, float(tau),
                              P[s].ctypes.data_as(dp))
    return P


def row_stats(Q, K, V, dO, lab_q, lab_k, variant, tau, strict=False):
    """m, l, D per query row, ``[S, T]`` each (D_i = sum_j P_ij <dO_i, V_j>)."""
    lib = _load()
    Q, K, V, lab_q, lab_k = _seg_args(Q, K, V, lab_q, lab_k)
    dO = np.ascontiguousarray(dO, dtype=np.float64)
    S, T, d = Q.shape
    m = np.zeros((S, T)); l = np.zeros((S, T)); D = np.zeros((S, T))
    dp = ctypes.POINTER(ctypes.c_double)
    for s in range(S):
        lib.scfa_oracle_row_stats(_f64(Q[s])[1], _f64(K[s])[1], _f64(V[s])[1], _f64(dO[s])[1],
                                  _i32(lab_q[s])[1], _i32(lab_k[s])[1],
                                  int(variant), int(bool(strict)), T, d, float(tau),
                                  m[s].ctypes.data_as(dp), l[s].ctypes.data_as(dp),
                                  D[s].ctypes.data_as(dp))
    return m, l, D


def attention_backward(Q, K, V, dO, lab_q, lab_k, variant, tau, strict=False,
                       q_rows=None, k_rows=None):
    """dQ, dK, dV of the definition (derivatives of ``attention_forward``).

    ``q_rows`` / ``k_rows``: optional row subsets (same in every segment) for
    dQ and for dK, dV; outputs then have that many rows.
    """
    lib = _load()
    Q, K, V, lab_q, lab_k = _seg_args(Q, K, V, lab_q, lab_k)
    dO = np.ascontiguousarray(dO, dtype=np.float64)
    assert dO.shape == Q.shape
    S, T, d = Q.shape
    q_rows = np.arange(T, dtype=np.int32) if q_rows is None else np.asarray(q_rows, dtype=np.int32)
    k_rows = np.arange(T, dtype=np.int32) if k_rows is None else np.asarray(k_rows, dtype=np.int32)
    q_rows, q_rows_p = _i32(q_rows)
    k_rows, k_rows_p = _i32(k_rows)
    nq, nk = q_rows.shape[0], k_rows.shape[0]
    dQ = np.zeros((S, nq, d)); dK = np.zeros((S, nk, d)); dV = np.zeros((S, nk, d))
    m, l, D = row_stats(Q, K, V, dO, lab_q, lab_k, variant, tau, strict)
    dp = ctypes.POINTER(ctypes.c_double)
    for s in range(S):
        args = (_f64(Q[s])[1], _f64(K[s])[1], _f64(V[s])[1], _f64(dO[s])[1],
                _i32(lab_q[s])[1], _i32(lab_k[s])[1],
                int(variant), int(bool(strict)), T, d, float(tau))
        lib.scfa_oracle_dq_rows(*args, q_rows_p, nq, dQ[s].ctypes.data_as(dp))
        lib.scfa_oracle_dkdv_rows(*args, m[s].ctypes.data_as(dp), l[s].ctypes.data_as(dp),
                                  D[s].ctypes.data_as(dp), k_rows_p, nk,
                                  dK[s].ctypes.data_as(dp), dV[s].ctypes.data_as(dp))
    return dQ, dK, dV


def count_allowed_pairs(lab_q, lab_k, variant, strict=False):
    """Number of allowed (query, key) pairs, summed over segments."""
    lib = _load()
    lab_q = np.ascontiguousarray(lab_q, dtype=np.int32)
    lab_k = np.ascontiguousarray(lab_k, dtype=np.int32)
    S, T = lab_q.shape
    return sum(int(lib.scfa_oracle_count_pairs(_i32(lab_q[s])[1], _i32(lab_k[s])[1],
                                               int(variant), int(bool(strict)), T))
               for s in range(S))


# --------------------------------------------------------------------------
# integer passes
# --------------------------------------------------------------------------

def sort_by_bucket(bucket, nb):
    """Stable sort of positions by bucket id, per segment (paper Sec. 3.2; the
    pre-processing of App. B.2 sorts the bucket ids with a stable sort).

    Returns ``idx`` (original position of every sorted row), ``bucket_sorted``
    and ``off`` with ``off[s, b]`` = number of tokens of segment ``s`` whose
    bucket id is below ``b`` (``[S, nb+1]``).
    """
    bucket = np.asarray(bucket, dtype=np.int32)
    idx = np.argsort(bucket, axis=-1, kind="stable").astype(np.int32)
    bucket_sorted = np.take_along_axis(bucket, idx, axis=-1)
    S = bucket.shape[0]
    off = np.zeros((S, nb + 1), dtype=np.int32)
    for s in range(S):
        for b in range(nb + 1):
            off[s, b] = int(np.sum(bucket[s] < b))
    return idx, bucket_sorted, off


def compact_keep(keep):
    """Positions of kept tokens in increasing order, then positions of dropped
    tokens in increasing order (paper App. B.2: a stable descending sort of the
    keep flag), and the kept count per segment."""
    keep = np.asarray(keep)
    S, T = keep.shape
    idx = np.zeros((S, T), dtype=np.int32)
    count = np.zeros((S,), dtype=np.int32)
    for s in range(S):
        kept = np.flatnonzero(keep[s] != 0)
        dropped = np.flatnonzero(keep[s] == 0)
        idx[s, :kept.size] = kept
        idx[s, kept.size:] = dropped
        count[s] = kept.size
    return idx, count


def allowed_mask(lab_q, lab_k, variant, strict=False):
    """Dense boolean mask ``[T, T]`` of one segment in ORIGINAL coordinates."""
    lab_q = np.asarray(lab_q); lab_k = np.asarray(lab_k)
    T = lab_q.shape[0]
    i = np.arange(T)[:, None]; j = np.arange(T)[None, :]
    causal = (j < i) if strict else (j <= i)
    if variant == HASH:
        return causal & (lab_q[:, None] == lab_k[None, :])
    return causal & (lab_q[:, None] != 0) & (lab_k[None, :] != 0)


def _per_tile(x, B):
    """Smallest and largest entry of every block of B consecutive entries (the last block may be short)."""
    x = np.asarray(x)
    starts = np.arange(0, x.shape[0], B)
    return np.minimum.reduceat(x, starts), np.maximum.reduceat(x, starts)


def paper_tile_ranges_qk(q_idx, k_idx, Bm, Bn):
    """Key-tile range ``[0, end)`` per query tile under the QK-sparse rule (paper Sec. 3.1, Alg. 1): a key
    tile is visited iff its earliest key is not later than the query tile's latest query, and ``end`` is
    the NUMBER of such tiles (the compacted keys are in increasing order, so they form a prefix).
    ``q_idx`` / ``k_idx`` are the (padded) index vectors of the compacted tensors of ONE segment."""
    _, q_last = _per_tile(q_idx, Bm)
    k_first, _ = _per_tile(k_idx, Bn)
    return [(0, int(np.count_nonzero(k_first <= ql))) for ql in q_last]


def paper_tile_ranges_hash(q_idx, k_idx, q_hash, k_hash, Bm, Bn):
    """Key-tile range ``[start, end)`` per query tile under the hash rule (paper Sec. 3.2, Alg. 2), on the
    bucket-sorted vectors of ONE segment.  Buckets first: tiles all of whose keys lie in buckets below the
    query tile's lowest bucket are skipped (their number is ``start``), and the tiles that begin in a
    bucket not above the query tile's highest one number ``end_hash``.  Causality second: inside
    ``[start, end_hash)`` the range stops after the last tile whose earliest key is not later than the
    tile's latest query; when no tile qualifies the paper's rule leaves the range at ``end_hash``."""
    _, q_last = _per_tile(q_idx, Bm)
    qh_lo, qh_hi = _per_tile(q_hash, Bm)
    k_first, _ = _per_tile(k_idx, Bn)
    kh_lo, kh_hi = _per_tile(k_hash, Bn)
    out = []
    for i in range(q_last.shape[0]):
        start = int(np.count_nonzero(kh_hi < qh_lo[i]))
        end_hash = int(np.count_nonzero(kh_lo <= qh_hi[i]))
        seen = np.flatnonzero(k_first[start:end_hash] <= q_last[i])
        out.append((start, start + int(seen[-1]) + 1 if seen.size else end_hash))
    return out


def tile_occupancy(mask_perm, Bm, Bn):
    """Brute force: ``occ[i, j]`` is True iff tile (i, j) of a dense boolean
    matrix (already in permuted / compacted coordinates) holds an allowed pair."""
    mask_perm = np.asarray(mask_perm, dtype=bool)
    nq, nk = mask_perm.shape
    ni, nj = -(-nq // Bm), -(-nk // Bn)
    occ = np.zeros((ni, nj), dtype=bool)
    for i in range(ni):
        for j in range(nj):
            occ[i, j] = mask_perm[i * Bm:(i + 1) * Bm, j * Bn:(j + 1) * Bn].any()
    return occ


if __name__ == "__main__":
    print(build(force="--force" in sys.argv))


# ---------------------------------------------------------------------------
# LSH bucketing (the step in front of the hash-sparse path)
# ---------------------------------------------------------------------------

def lsh_projections(x, R, H):
    """x [S,T,d], R [H,d,r] -> [S,T,2r] float64: for segment s = b*H + h the row x[s,t,:] times
    R[h], followed by its negation (cross-polytope LSH: the 2r vertices +-e_c of the rotated
    space, Sec. 4.2 "Hashing mechanism")."""
    x = np.asarray(x, np.float64)
    R = np.asarray(R, np.float64)
    S, T, d = x.shape
    assert R.shape[0] == H and R.shape[1] == d and S % H == 0
    out = np.empty((S, T, 2 * R.shape[2]), np.float64)
    for s in range(S):
        p = x[s] @ R[s % H]
        out[s, :, :R.shape[2]] = p
        out[s, :, R.shape[2]:] = -p
    return out


def lsh_buckets(x, R, H):
    """Bucket id = index of the largest entry of [xR, -xR]; the lowest index wins a tie.
    Returns (bucket int32 [S,T], margin float64 [S,T]) with margin = largest minus second
    largest entry (a caller comparing against lower-precision arithmetic uses it to set
    aside rows whose decision is within rounding)."""
    ext = lsh_projections(x, R, H)
    b = np.argmax(ext, axis=-1).astype(np.int32)
    part = np.partition(ext, -2, axis=-1)
    return b, part[..., -1] - part[..., -2]
