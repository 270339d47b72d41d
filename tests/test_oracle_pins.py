"""Pins for the CPU oracle: everything here checks ``oracle/`` against something
other than itself -- values the paper prints (Fig. 1), library routines on
special cases, closed forms, invariants, finite differences and brute force.

Each pin names the mistake it would catch.
"""
import itertools
import json
import math
import os

import numpy as np
import pytest
import torch

import oracle
from oracle import HASH, QKDROP


def rnd(seed, *shape):
    return np.random.default_rng(seed).standard_normal(shape)


@pytest.fixture(scope="module")
def fig1(golden_dir):
    with open(os.path.join(golden_dir, "fig1_worked_example.json")) as f:
        return json.load(f)


# ---------------------------------------------------------------- Fig. 1 pins

def test_fig1_qk_sparse_kept_sets_and_row_counts(fig1):
    """Fig. 1 top row.  Catches: exclusive instead of inclusive causality,
    causality on compacted instead of original positions, wrong compaction order."""
    g = fig1["qk_sparse"]
    T = fig1["T"]
    keep_q = np.ones((1, T), np.uint8); keep_q[0, g["dropped_queries"]] = 0
    keep_k = np.ones((1, T), np.uint8); keep_k[0, g["dropped_keys"]] = 0
    q_idx, nq = oracle.compact_keep(keep_q)
    k_idx, nk = oracle.compact_keep(keep_k)
    assert q_idx[0, :nq[0]].tolist() == g["kept_queries"]
    assert k_idx[0, :nk[0]].tolist() == g["kept_keys"]
    assert sorted(q_idx[0, nq[0]:].tolist()) == g["dropped_queries"]
    M = oracle.allowed_mask(keep_q[0], keep_k[0], QKDROP)
    counts = [int(M[i].sum()) for i in g["kept_queries"]]
    assert counts == g["allowed_keys_per_compacted_row"]
    # the same counts from the probabilities of the floating-point oracle
    P = oracle.attention_probs(rnd(0, 1, T, 4), rnd(1, 1, T, 4), keep_q, keep_k, QKDROP, 0.5)[0]
    assert [(P[i] > 0).sum() for i in g["kept_queries"]] == g["allowed_keys_per_compacted_row"]
    for i in g["dropped_queries"]:
        assert not P[i].any()
    for j in g["dropped_keys"]:
        assert not P[:, j].any()


def test_fig1_hash_sparse_sort_and_cells(fig1):
    """Fig. 1 bottom row.  Catches: unstable sort, wrong bucket order, a mask that
    drops the bucket test or the causal test, transposed query/key roles."""
    g = fig1["hash_sparse"]
    T = fig1["T"]
    bq = np.array([g["query_bucket_by_position"]], np.int32)
    bk = np.array([g["key_bucket_by_position"]], np.int32)
    q_idx, q_sorted, q_off = oracle.sort_by_bucket(bq, 3)
    k_idx, k_sorted, k_off = oracle.sort_by_bucket(bk, 3)
    assert q_idx[0].tolist() == g["sorted_query_positions"]
    assert k_idx[0].tolist() == g["sorted_key_positions"]
    assert q_sorted[0].tolist() == g["sorted_query_buckets"]
    assert k_sorted[0].tolist() == g["sorted_key_buckets"]
    assert q_off[0].tolist() == [0, 2, 5, 8] and k_off[0].tolist() == [0, 2, 6, 8]
    M = oracle.allowed_mask(bq[0], bk[0], HASH)
    Mp = M[np.ix_(q_idx[0], k_idx[0])]          # sorted coordinates: [query row, key col]
    cells = sorted((int(c), int(r)) for r, c in zip(*np.nonzero(Mp)))
    assert cells == sorted(tuple(x) for x in g["computed_cells_keycol_queryrow"])
    P = oracle.attention_probs(rnd(2, 1, T, 4), rnd(3, 1, T, 4), bq, bk, HASH, 0.5)[0]
    assert np.array_equal(P > 0, M)


# ------------------------------------------------- library routine special cases

def _torch_dense(Q, K, V, mask, tau):
    """softmax(tau QK^T + mask) V with library ops; rows without keys -> 0."""
    Q, K, V = (torch.from_numpy(np.asarray(a, dtype=np.float64)) for a in (Q, K, V))
    s = tau * Q @ K.transpose(-1, -2)
    m = torch.from_numpy(mask)
    s = s.masked_fill(~m, -math.inf)
    has = m.any(-1, keepdim=True)
    p = torch.softmax(torch.where(has, s, torch.zeros_like(s)), -1) * m
    lse = torch.where(has[..., 0], torch.logsumexp(torch.where(has, s, torch.zeros_like(s)), -1),
                      torch.full(s.shape[:-1], -math.inf, dtype=torch.float64))
    return p @ V, lse


def test_one_bucket_is_plain_causal_attention_library():
    """nb = 1 reduces to torch's scaled_dot_product_attention(is_causal=True).
    Catches: wrong scale, transposed operands, off-by-one causality, wrong normaliser."""
    S, T, d = 2, 37, 8
    Q, K, V = rnd(10, S, T, d), rnd(11, S, T, d), rnd(12, S, T, d)
    lab = np.zeros((S, T), np.int32)
    O, LSE = oracle.attention_forward(Q, K, V, lab, lab, HASH, 1 / math.sqrt(d))
    ref = torch.nn.functional.scaled_dot_product_attention(
        torch.from_numpy(Q), torch.from_numpy(K), torch.from_numpy(V), is_causal=True)
    np.testing.assert_allclose(O, ref.numpy(), rtol=0, atol=1e-12)
    s = (torch.from_numpy(Q) @ torch.from_numpy(K).transpose(-1, -2)) / math.sqrt(d)
    s = s.masked_fill(~torch.tril(torch.ones(T, T, dtype=torch.bool)), -math.inf)
    np.testing.assert_allclose(LSE, torch.logsumexp(s, -1).numpy(), rtol=0, atol=1e-12)


def test_keep_all_is_plain_causal_attention_library():
    S, T, d = 1, 29, 6
    Q, K, V = rnd(13, S, T, d), rnd(14, S, T, d), rnd(15, S, T, d)
    keep = np.ones((S, T), np.uint8)
    O, _ = oracle.attention_forward(Q, K, V, keep, keep, QKDROP, 0.3)
    ref = torch.nn.functional.scaled_dot_product_attention(
        torch.from_numpy(Q), torch.from_numpy(K), torch.from_numpy(V), is_causal=True, scale=0.3)
    np.testing.assert_allclose(O, ref.numpy(), rtol=0, atol=1e-12)


@pytest.mark.parametrize("variant", [HASH, QKDROP])
def test_general_mask_matches_library_softmax(variant):
    """Arbitrary labels vs torch softmax with an explicit mask (different code path:
    library softmax / logsumexp over the dense masked matrix)."""
    S, T, d = 3, 41, 5
    Q, K, V = rnd(20, S, T, d), rnd(21, S, T, d), rnd(22, S, T, d)
    rng = np.random.default_rng(23)
    if variant == HASH:
        lq = rng.integers(0, 3, (S, T)).astype(np.int32); lk = rng.integers(0, 3, (S, T)).astype(np.int32)
    else:
        lq = (rng.random((S, T)) < 0.6).astype(np.uint8); lk = (rng.random((S, T)) < 0.4).astype(np.uint8)
    O, LSE = oracle.attention_forward(Q, K, V, lq, lk, variant, 0.7)
    for s in range(S):
        M = oracle.allowed_mask(lq[s], lk[s], variant)
        o_ref, lse_ref = _torch_dense(Q[s], K[s], V[s], M, 0.7)
        np.testing.assert_allclose(O[s], o_ref.numpy(), rtol=0, atol=1e-12)
        fin = np.isfinite(lse_ref.numpy())
        np.testing.assert_allclose(LSE[s][fin], lse_ref.numpy()[fin], rtol=0, atol=1e-12)
        assert np.all(np.isneginf(LSE[s][~fin]))
        assert not O[s][~fin].any()            # stranded queries give zero vectors (Sec. 3.1)
        assert (~fin).any() or variant == HASH


def test_hash_equals_per_bucket_causal_attention():
    """Closed decomposition: the hash result equals plain attention run separately on each
    bucket's sub-sequences (queries of bucket b against keys of bucket b) with the
    non-square causal mask on original positions.  Catches a mask that leaks across
    buckets or uses sorted instead of original positions."""
    T, d, nb = 64, 8, 4
    Q, K, V = rnd(30, 1, T, d), rnd(31, 1, T, d), rnd(32, 1, T, d)
    rng = np.random.default_rng(33)
    bq = rng.integers(0, nb, (1, T)).astype(np.int32); bk = rng.integers(0, nb, (1, T)).astype(np.int32)
    O, _ = oracle.attention_forward(Q, K, V, bq, bk, HASH, 0.4)
    for b in range(nb):
        qi = np.flatnonzero(bq[0] == b); ki = np.flatnonzero(bk[0] == b)
        m = torch.from_numpy(ki[None, :] <= qi[:, None])
        rows = m.any(-1).numpy()
        ref = torch.nn.functional.scaled_dot_product_attention(
            torch.from_numpy(Q[0, qi][rows]), torch.from_numpy(K[0, ki]), torch.from_numpy(V[0, ki]),
            attn_mask=m[torch.from_numpy(rows)], scale=0.4)
        np.testing.assert_allclose(O[0, qi][rows], ref.numpy(), rtol=0, atol=1e-12)
        assert not O[0, qi][~rows].any()


def test_qkdrop_equals_attention_on_hand_compacted_tensors():
    """QK-dropping equals masked attention on the compacted tensors (Sec. 3.1), with the
    mask taken on original positions; dropped queries give zero."""
    T, d = 48, 8
    Q, K, V = rnd(40, 1, T, d), rnd(41, 1, T, d), rnd(42, 1, T, d)
    rng = np.random.default_rng(43)
    kq = (rng.random((1, T)) < 0.5).astype(np.uint8); kk = (rng.random((1, T)) < 0.5).astype(np.uint8)
    O, _ = oracle.attention_forward(Q, K, V, kq, kk, QKDROP, 0.35)
    qi = np.flatnonzero(kq[0]); ki = np.flatnonzero(kk[0])
    m = torch.from_numpy(ki[None, :] <= qi[:, None])
    rows = m.any(-1).numpy()
    ref = torch.nn.functional.scaled_dot_product_attention(
        torch.from_numpy(Q[0, qi][rows]), torch.from_numpy(K[0, ki]), torch.from_numpy(V[0, ki]),
        attn_mask=m[torch.from_numpy(rows)], scale=0.35)
    np.testing.assert_allclose(O[0, qi][rows], ref.numpy(), rtol=0, atol=1e-12)
    assert not O[0, np.flatnonzero(kq[0] == 0)].any()


# --------------------------------------------------------- closed forms / invariants

def test_first_row_closed_form():
    """Row 0 sees only key 0: O[0] = V[0] and LSE[0] = tau <Q0,K0> exactly."""
    T, d = 9, 4
    Q, K, V = rnd(50, 1, T, d), rnd(51, 1, T, d), rnd(52, 1, T, d)
    lab = np.zeros((1, T), np.int32)
    O, LSE = oracle.attention_forward(Q, K, V, lab, lab, HASH, 0.5)
    np.testing.assert_allclose(O[0, 0], V[0, 0], rtol=0, atol=1e-15)
    assert abs(LSE[0, 0] - 0.5 * float(Q[0, 0] @ K[0, 0])) < 1e-14


def test_equal_scores_give_uniform_average():
    """With K = 0 every allowed key has score 0: O_i is the mean of the allowed V rows and
    LSE_i = ln(#allowed).  Catches a wrong normaliser or a max subtracted twice."""
    T, d = 12, 3
    Q, V = rnd(60, 1, T, d), rnd(61, 1, T, d)
    K = np.zeros((1, T, d))
    rng = np.random.default_rng(62)
    bq = rng.integers(0, 2, (1, T)).astype(np.int32); bk = rng.integers(0, 2, (1, T)).astype(np.int32)
    O, LSE = oracle.attention_forward(Q, K, V, bq, bk, HASH, 1.0)
    M = oracle.allowed_mask(bq[0], bk[0], HASH)
    for i in range(T):
        n = M[i].sum()
        if n:
            np.testing.assert_allclose(O[0, i], V[0][M[i]].mean(0), atol=1e-14)
            assert abs(LSE[0, i] - math.log(n)) < 1e-14
        else:
            assert not O[0, i].any() and np.isneginf(LSE[0, i])


@pytest.mark.parametrize("variant", [HASH, QKDROP])
def test_probability_rows_sum_to_one_or_zero(variant):
    S, T, d = 2, 33, 4
    Q, K = rnd(70, S, T, d), rnd(71, S, T, d)
    rng = np.random.default_rng(72)
    lq = rng.integers(0, 2, (S, T)).astype(np.int32); lk = rng.integers(0, 2, (S, T)).astype(np.int32)
    P = oracle.attention_probs(Q, K, lq, lk, variant, 0.9)
    for s in range(S):
        M = oracle.allowed_mask(lq[s], lk[s], variant)
        sums = P[s].sum(-1)
        np.testing.assert_allclose(sums[M.any(-1)], 1.0, atol=1e-13)
        assert not sums[~M.any(-1)].any()
        assert not P[s][~M].any()


def test_bucket_relabelling_and_segment_shuffle_invariance():
    """Renaming bucket ids by a bijection leaves O unchanged; permuting the (batch, head)
    segments permutes the result the same way."""
    S, T, d, nb = 3, 40, 4, 4
    Q, K, V = rnd(80, S, T, d), rnd(81, S, T, d), rnd(82, S, T, d)
    rng = np.random.default_rng(83)
    bq = rng.integers(0, nb, (S, T)).astype(np.int32); bk = rng.integers(0, nb, (S, T)).astype(np.int32)
    O, LSE = oracle.attention_forward(Q, K, V, bq, bk, HASH, 0.5)
    perm = np.array([2, 0, 3, 1], np.int32)
    O2, LSE2 = oracle.attention_forward(Q, K, V, perm[bq], perm[bk], HASH, 0.5)
    assert np.array_equal(O, O2) and np.array_equal(LSE, LSE2)
    sp = np.array([1, 2, 0])
    O3, _ = oracle.attention_forward(Q[sp], K[sp], V[sp], bq[sp], bk[sp], HASH, 0.5)
    assert np.array_equal(O3, O[sp])


def test_row_subset_matches_full():
    S, T, d = 2, 50, 4
    Q, K, V = rnd(90, S, T, d), rnd(91, S, T, d), rnd(92, S, T, d)
    lab = np.random.default_rng(93).integers(0, 3, (S, T)).astype(np.int32)
    O, LSE = oracle.attention_forward(Q, K, V, lab, lab, HASH, 0.5)
    rows = [0, 7, 49, 23]
    Or, Lr = oracle.attention_forward(Q, K, V, lab, lab, HASH, 0.5, rows=rows)
    assert np.array_equal(Or, O[:, rows]) and np.array_equal(Lr, LSE[:, rows])
    dO = rnd(94, S, T, d)
    dQ, dK, dV = oracle.attention_backward(Q, K, V, dO, lab, lab, HASH, 0.5)
    dQr, dKr, dVr = oracle.attention_backward(Q, K, V, dO, lab, lab, HASH, 0.5, q_rows=rows, k_rows=rows)
    assert np.array_equal(dQr, dQ[:, rows]) and np.array_equal(dKr, dK[:, rows]) and np.array_equal(dVr, dV[:, rows])


# --------------------------------------------------------------------- gradients

def _labels(variant, rng, S, T):
    if variant == HASH:
        return rng.integers(0, 3, (S, T)).astype(np.int32), rng.integers(0, 3, (S, T)).astype(np.int32)
    return (rng.random((S, T)) < 0.6).astype(np.uint8), (rng.random((S, T)) < 0.6).astype(np.uint8)


@pytest.mark.parametrize("variant", [HASH, QKDROP])
def test_backward_matches_torch_autograd(variant):
    """Gradients vs torch.autograd through library ops on the dense masked formula.
    Catches: a dropped D term, a missing tau, swapped dK/dQ operands, wrong sign."""
    S, T, d = 2, 24, 5
    tau = 0.45
    Q, K, V, dO = rnd(100, S, T, d), rnd(101, S, T, d), rnd(102, S, T, d), rnd(103, S, T, d)
    lq, lk = _labels(variant, np.random.default_rng(104), S, T)
    dQ, dK, dV = oracle.attention_backward(Q, K, V, dO, lq, lk, variant, tau)
    for s in range(S):
        q, k, v = (torch.tensor(a[s], dtype=torch.float64, requires_grad=True) for a in (Q, K, V))
        M = torch.from_numpy(oracle.allowed_mask(lq[s], lk[s], variant))
        sc = (tau * q @ k.T).masked_fill(~M, -math.inf)
        has = M.any(-1, keepdim=True)
        p = torch.softmax(torch.where(has, sc, torch.zeros_like(sc)), -1) * M
        (p @ v * torch.from_numpy(dO[s])).sum().backward()
        np.testing.assert_allclose(dQ[s], q.grad.numpy(), rtol=0, atol=1e-12)
        np.testing.assert_allclose(dK[s], k.grad.numpy(), rtol=0, atol=1e-12)
        np.testing.assert_allclose(dV[s], v.grad.numpy(), rtol=0, atol=1e-12)


@pytest.mark.parametrize("variant", [HASH, QKDROP])
def test_backward_matches_finite_differences(variant):
    """Central differences of L = sum(O * dO) through the oracle's own forward."""
    S, T, d = 1, 7, 3
    tau = 0.8
    Q, K, V, dO = rnd(110, S, T, d), rnd(111, S, T, d), rnd(112, S, T, d), rnd(113, S, T, d)
    lq, lk = _labels(variant, np.random.default_rng(114), S, T)
    dQ, dK, dV = oracle.attention_backward(Q, K, V, dO, lq, lk, variant, tau)

    def loss(q, k, v):
        return float((oracle.attention_forward(q, k, v, lq, lk, variant, tau)[0] * dO).sum())

    eps = 1e-6
    for X, G, which in ((Q, dQ, 0), (K, dK, 1), (V, dV, 2)):
        for t in range(T):
            for c in range(d):
                args = [Q.copy(), K.copy(), V.copy()]
                args[which][0, t, c] += eps
                up = loss(*args)
                args[which][0, t, c] -= 2 * eps
                dn = loss(*args)
                fd = (up - dn) / (2 * eps)
                assert abs(fd - G[0, t, c]) < 1e-6 * max(1.0, abs(fd)), (which, t, c)


def test_backward_identities():
    """D_i = <dO_i, O_i>; dS rows sum to zero (so dQ_i is orthogonal to nothing it should
    not be); dropped / stranded rows get zero gradients."""
    S, T, d = 2, 30, 4
    tau = 0.5
    Q, K, V, dO = rnd(120, S, T, d), rnd(121, S, T, d), rnd(122, S, T, d), rnd(123, S, T, d)
    rng = np.random.default_rng(124)
    kq = (rng.random((S, T)) < 0.5).astype(np.uint8); kk = (rng.random((S, T)) < 0.5).astype(np.uint8)
    O, _ = oracle.attention_forward(Q, K, V, kq, kk, QKDROP, tau)
    m, l, D = oracle.row_stats(Q, K, V, dO, kq, kk, QKDROP, tau)
    np.testing.assert_allclose(D, (dO * O).sum(-1), atol=1e-13)
    dQ, dK, dV = oracle.attention_backward(Q, K, V, dO, kq, kk, QKDROP, tau)
    assert not dQ[kq == 0].any() and not dK[kk == 0].any() and not dV[kk == 0].any()
    # sum_j dS_ij = 0  =>  sum over all keys of dV-like test: use V = ones => dP const => dS = 0
    ones = np.ones_like(V)
    dQ1, dK1, _ = oracle.attention_backward(Q, K, ones, dO, kq, kk, QKDROP, tau)
    np.testing.assert_allclose(dQ1, 0, atol=1e-13)
    np.testing.assert_allclose(dK1, 0, atol=1e-13)


# ------------------------------------------------------------------ brute force

def _brute(Q, K, V, lq, lk, variant, tau):
    """Literal loops with math.exp (no numpy broadcasting, no shared helper)."""
    T, d = len(Q), len(Q[0])
    O = [[0.0] * d for _ in range(T)]
    LSE = [-math.inf] * T
    for i in range(T):
        sc = {}
        for j in range(T):
            ok = j <= i and ((lq[i] == lk[j]) if variant == HASH else (lq[i] != 0 and lk[j] != 0))
            if ok:
                sc[j] = tau * sum(Q[i][c] * K[j][c] for c in range(d))
        if not sc:
            continue
        mx = max(sc.values())
        den = sum(math.exp(x - mx) for x in sc.values())
        for j, x in sc.items():
            w = math.exp(x - mx) / den
            for c in range(d):
                O[i][c] += w * V[j][c]
        LSE[i] = mx + math.log(den)
    return np.array(O), np.array(LSE)


def test_brute_force_all_bucket_assignments_tiny():
    """Every assignment of T=4 queries and keys to nb=2 buckets (256 cases) and every
    keep pattern, against literal Python loops."""
    T, d = 4, 2
    Q, K, V = rnd(130, 1, T, d), rnd(131, 1, T, d), rnd(132, 1, T, d)
    for variant in (HASH, QKDROP):
        for lq in itertools.product(range(2), repeat=T):
            for lk in itertools.product(range(2), repeat=T):
                a = np.array([lq], np.int32); b = np.array([lk], np.int32)
                O, LSE = oracle.attention_forward(Q, K, V, a, b, variant, 0.6)
                Ob, Lb = _brute(Q[0].tolist(), K[0].tolist(), V[0].tolist(), lq, lk, variant, 0.6)
                np.testing.assert_allclose(O[0], Ob, atol=1e-14)
                fin = np.isfinite(Lb)
                np.testing.assert_allclose(LSE[0][fin], Lb[fin], atol=1e-14)
                assert np.all(np.isneginf(LSE[0][~fin]))


def test_brute_force_random_t16():
    T, d = 16, 3
    for seed in range(4):
        Q, K, V = rnd(140 + seed, 1, T, d), rnd(150 + seed, 1, T, d), rnd(160 + seed, 1, T, d)
        rng = np.random.default_rng(170 + seed)
        lq = rng.integers(0, 3, (1, T)).astype(np.int32); lk = rng.integers(0, 3, (1, T)).astype(np.int32)
        O, LSE = oracle.attention_forward(Q, K, V, lq, lk, HASH, 0.5)
        Ob, Lb = _brute(Q[0].tolist(), K[0].tolist(), V[0].tolist(), lq[0].tolist(), lk[0].tolist(), HASH, 0.5)
        np.testing.assert_allclose(O[0], Ob, atol=1e-14)


def test_strict_variant_excludes_self():
    """strict=True removes the diagonal (App. B.1: ">=" replaced by ">"): row 0 is stranded."""
    T, d = 10, 3
    Q, K, V = rnd(180, 1, T, d), rnd(181, 1, T, d), rnd(182, 1, T, d)
    lab = np.zeros((1, T), np.int32)
    O, LSE = oracle.attention_forward(Q, K, V, lab, lab, HASH, 0.5, strict=True)
    assert not O[0, 0].any() and np.isneginf(LSE[0, 0])
    np.testing.assert_allclose(O[0, 1], V[0, 0], atol=1e-15)
    M = oracle.allowed_mask(lab[0], lab[0], HASH, strict=True)
    assert not np.diag(M).any() and M[3, 2] and not M[2, 3]


def test_count_pairs_matches_mask():
    rng = np.random.default_rng(190)
    lq = rng.integers(0, 4, (2, 57)).astype(np.int32); lk = rng.integers(0, 4, (2, 57)).astype(np.int32)
    n = oracle.count_allowed_pairs(lq, lk, HASH)
    assert n == sum(int(oracle.allowed_mask(lq[s], lk[s], HASH).sum()) for s in range(2))


# ------------------------------------------------------------ integer oracles

def test_sort_by_bucket_against_python_sorted():
    rng = np.random.default_rng(200)
    b = rng.integers(0, 5, (3, 101)).astype(np.int32)
    idx, bs, off = oracle.sort_by_bucket(b, 5)
    for s in range(3):
        ref = sorted(range(101), key=lambda t: (int(b[s, t]), t))   # (bucket, position) order
        assert idx[s].tolist() == ref
        assert bs[s].tolist() == [int(b[s, t]) for t in ref]
        assert off[s].tolist() == [sum(int(x) < c for x in b[s]) for c in range(6)]


def test_paper_tile_ranges_regular_case_is_lower_triangular():
    """With no sparsity the tile set coincides with FlashAttention's (Fig. 2, left):
    query tile i computes key tiles 0..i."""
    T, B = 64, 8
    idx = np.arange(T)
    assert oracle.paper_tile_ranges_qk(idx, idx, B, B) == [(0, i + 1) for i in range(T // B)]
    h = np.zeros(T, np.int32)
    assert oracle.paper_tile_ranges_hash(idx, idx, h, h, B, B) == [(0, i + 1) for i in range(T // B)]


def test_paper_tile_ranges_cover_occupied_tiles():
    """The ranges of Alg. 1 / Alg. 2 are supersets of the occupied tiles (brute force)."""
    rng = np.random.default_rng(210)
    T, B = 96, 8
    for _ in range(5):
        bq = rng.integers(0, 4, (1, T)).astype(np.int32); bk = rng.integers(0, 4, (1, T)).astype(np.int32)
        qi, qs, _ = oracle.sort_by_bucket(bq, 4); ki, ks, _ = oracle.sort_by_bucket(bk, 4)
        Mp = oracle.allowed_mask(bq[0], bk[0], HASH)[np.ix_(qi[0], ki[0])]
        occ = oracle.tile_occupancy(Mp, B, B)
        rg = oracle.paper_tile_ranges_hash(qi[0], ki[0], qs[0], ks[0], B, B)
        for i, (a, e) in enumerate(rg):
            cols = np.flatnonzero(occ[i])
            assert all(a <= c < e for c in cols)
        kq = (rng.random((1, T)) < 0.5).astype(np.uint8); kk = (rng.random((1, T)) < 0.5).astype(np.uint8)
        qi, nq = oracle.compact_keep(kq); ki, nk = oracle.compact_keep(kk)
        qv, kv = qi[0, :nq[0]], ki[0, :nk[0]]
        Mp = oracle.allowed_mask(kq[0], kk[0], QKDROP)[np.ix_(qv, kv)]
        occ = oracle.tile_occupancy(Mp, B, B)
        rg = oracle.paper_tile_ranges_qk(qv, kv, B, B)
        for i, (a, e) in enumerate(rg):
            assert all(a <= c < e for c in np.flatnonzero(occ[i]))


# ---------------------------------------------------------------- LSH bucketing pins

def test_lsh_axis_aligned_projection_is_signed_argmax_abs():
    """With R = the first r columns of the identity, [xR, -xR] = [x_0..x_{r-1}, -x_0..-x_{r-1}]:
    the bucket is the coordinate of largest magnitude, offset by r when it is negative
    (catches a transposed R, a missing negated half, a wrong concatenation order)."""
    d, r, T = 8, 4, 200
    x = rnd(21, 2, T, d)
    R = np.zeros((1, d, r)); R[0, :r, :r] = np.eye(r)
    b, margin = oracle.lsh_buckets(x, R, 1)
    c = np.argmax(np.abs(x[..., :r]), axis=-1)
    expect = np.where(np.take_along_axis(x[..., :r], c[..., None], -1)[..., 0] >= 0, c, c + r)
    assert np.array_equal(b, expect) and (margin >= 0).all()


def test_lsh_hand_example_and_tie_rule():
    """x = (1, 2), R = [[1, 0], [0, 1]]: [1, 2, -1, -2] -> bucket 1; x = (-3, 1): [-3, 1, 3, -1] -> 2;
    x = (1, 1): a tie between entries 0 and 1 -> the lowest index; x = 0: every entry ties -> 0."""
    R = np.eye(2)[None]
    x = np.array([[[1.0, 2.0], [-3.0, 1.0], [1.0, 1.0], [0.0, 0.0]]])
    b, margin = oracle.lsh_buckets(x, R, 1)
    assert b[0].tolist() == [1, 2, 0, 0]
    assert margin[0].tolist() == [1.0, 2.0, 0.0, 0.0]


def test_lsh_invariances_and_per_head_projection():
    """Positive scaling leaves the bucket, negation moves it to the antipodal vertex (c <-> c + r);
    segment s uses the projection of head s % H (catches indexing R by batch instead of head)."""
    H, d, r, T = 3, 16, 4, 300
    x = rnd(22, 2 * H, T, d)
    R = rnd(23, H, d, r)
    b, _ = oracle.lsh_buckets(x, R, H)
    assert np.array_equal(oracle.lsh_buckets(3.7 * x, R, H)[0], b)
    assert np.array_equal(oracle.lsh_buckets(-x, R, H)[0], (b + r) % (2 * r))
    for s in range(2 * H):
        assert np.array_equal(oracle.lsh_buckets(x[s:s + 1], R[s % H:s % H + 1], 1)[0][0], b[s])
    # with orthonormal columns the projections of Gaussian rows are i.i.d. N(0,1): all 2r vertices
    # are equally likely (12000 rows: three standard deviations of a frequency are below 0.01)
    Q = np.linalg.qr(rnd(24, d, d))[0][None, :, :r]
    bu, _ = oracle.lsh_buckets(rnd(25, 1, 12000, d), Q, 1)
    counts = np.bincount(bu.ravel(), minlength=2 * r) / bu.size
    assert np.abs(counts - 1.0 / (2 * r)).max() < 0.012


def test_lsh_matches_generator_of_the_benchmark_inputs():
    """The workload generator draws its bucket ids with its own implementation of the same rule;
    the two agree wherever the decision is not within rounding."""
    from paper_2306_01160_amd import workloads as W
    wl = W.hash_lsh(9, 2, 3, 256, 64, 8)
    Rm = np.random.default_rng(5).standard_normal((3, 64, 4)).astype(np.float32)
    got = W.lsh_buckets(wl.q, Rm).reshape(6, 256)
    ref, margin = oracle.lsh_buckets(wl.q.reshape(6, 256, 64), Rm, 3)
    clear = margin > 1e-9
    assert clear.mean() > 0.99 and np.array_equal(got[clear], ref[clear])
