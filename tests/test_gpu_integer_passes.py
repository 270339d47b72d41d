"""GPU integer passes vs the oracle, bit-exact: stable sort by bucket, compaction,
row gather, and validity of the tile-skip schedule."""
import numpy as np
import pytest
import torch

import oracle
from paper_2306_01160_amd import binding as sc

pytestmark = pytest.mark.gpu
DEV = "cuda:0"


def _t(a):
    return torch.from_numpy(np.ascontiguousarray(a)).to(DEV)


@pytest.mark.parametrize("S,T,nb", [(1, 8, 3), (3, 1, 1), (2, 63, 4), (5, 1000, 16), (4, 8192, 16),
                                    (2, 16384, 8), (1, 32768, 256), (3, 4097, 7), (2, 2048, 1)])
def test_sort_by_bucket_bit_exact(S, T, nb):
    rng = np.random.default_rng(S * 1000003 + T * 31 + nb)
    b = rng.integers(0, nb, (S, T)).astype(np.int32)
    if nb > 2:
        b[b == 1] = 0        # leave a bucket empty
    idx, bs, off = sc.scfa_sort_by_bucket(_t(b), nb)
    ridx, rbs, roff = oracle.sort_by_bucket(b, nb)
    assert np.array_equal(idx.cpu().numpy(), ridx)
    assert np.array_equal(bs.cpu().numpy(), rbs)
    assert np.array_equal(off.cpu().numpy(), roff)


def test_sort_fig1_example(golden_dir):
    import json, os
    g = json.load(open(os.path.join(golden_dir, "fig1_worked_example.json")))["hash_sparse"]
    bq = np.array([g["query_bucket_by_position"]], np.int32)
    bk = np.array([g["key_bucket_by_position"]], np.int32)
    qi, qs, _ = sc.scfa_sort_by_bucket(_t(bq), 3)
    ki, ks, _ = sc.scfa_sort_by_bucket(_t(bk), 3)
    assert qi.cpu().numpy()[0].tolist() == g["sorted_query_positions"]
    assert ki.cpu().numpy()[0].tolist() == g["sorted_key_positions"]
    assert qs.cpu().numpy()[0].tolist() == g["sorted_query_buckets"]
    assert ks.cpu().numpy()[0].tolist() == g["sorted_key_buckets"]


def test_sort_clamps_out_of_range_ids():
    b = np.array([[5, -3, 1, 0, 7, 1]], np.int32)
    idx, bs, off = sc.scfa_sort_by_bucket(_t(b), 2)
    ridx, rbs, roff = oracle.sort_by_bucket(np.clip(b, 0, 1), 2)
    assert np.array_equal(idx.cpu().numpy(), ridx) and np.array_equal(bs.cpu().numpy(), rbs)
    assert np.array_equal(off.cpu().numpy(), roff)


@pytest.mark.parametrize("shape,nb,n_bad", [((1, 6), 2, 3), ((3, 1000), 16, 0), ((4, 40000), 8, 1234), ((2, 1), 1, 1)])
def test_count_invalid_buckets(shape, nb, n_bad):
    """The validating call counts exactly the ids the sort would clamp."""
    rng = np.random.default_rng(nb * 31 + n_bad)
    b = rng.integers(0, nb, shape).astype(np.int32)
    flat = b.reshape(-1)
    where = rng.choice(flat.size, n_bad, replace=False)
    flat[where] = np.where(rng.random(n_bad) < 0.5, -1 - rng.integers(0, 1000, n_bad), nb + rng.integers(0, 1000, n_bad))
    got = sc.scfa_count_invalid_buckets(_t(b), nb)
    assert int(got.item()) == int(((b < 0) | (b >= nb)).sum()) == n_bad
    # the counter is overwritten, not accumulated
    got2 = sc.scfa_count_invalid_buckets(_t(np.zeros(shape, np.int32)), nb)
    assert int(got2.item()) == 0


@pytest.mark.parametrize("S,T,p", [(1, 8, 0.5), (2, 1, 1.0), (3, 100, 0.0), (4, 2048, 0.5), (16, 32768, 0.3),
                                   (2, 5000, 1.0), (3, 777, 0.1)])
def test_compact_keep_bit_exact(S, T, p):
    rng = np.random.default_rng(S * 7 + T)
    keep = (rng.random((S, T)) < p).astype(np.uint8)
    keep[keep != 0] = rng.integers(1, 255, int(keep.sum())).astype(np.uint8)   # any non-zero value = kept
    idx, cnt = sc.scfa_compact_keep(_t(keep))
    ridx, rcnt = oracle.compact_keep(keep)
    assert np.array_equal(cnt.cpu().numpy(), rcnt)
    assert np.array_equal(idx.cpu().numpy(), ridx)


def test_compact_fig1_example(golden_dir):
    import json, os
    g = json.load(open(os.path.join(golden_dir, "fig1_worked_example.json")))["qk_sparse"]
    kq = np.ones((1, 8), np.uint8); kq[0, g["dropped_queries"]] = 0
    kk = np.ones((1, 8), np.uint8); kk[0, g["dropped_keys"]] = 0
    qi, nq = sc.scfa_compact_keep(_t(kq)); ki, nk = sc.scfa_compact_keep(_t(kk))
    assert qi.cpu().numpy()[0, :int(nq[0])].tolist() == g["kept_queries"]
    assert ki.cpu().numpy()[0, :int(nk[0])].tolist() == g["kept_keys"]


@pytest.mark.parametrize("dtype,d", [(torch.bfloat16, 64), (torch.bfloat16, 128), (torch.float32, 64)])
def test_gather_rows_bit_exact(dtype, d):
    S, T = 3, 1237
    rng = np.random.default_rng(d)
    x = torch.from_numpy(rng.standard_normal((S, T, d)).astype(np.float32)).to(DEV).to(dtype)
    idx = np.stack([rng.permutation(T) for _ in range(S)]).astype(np.int32)
    out = sc.scfa_gather_rows(x, _t(idx))
    ref = torch.gather(x, 1, _t(idx).long()[..., None].expand(-1, -1, d))
    assert torch.equal(out, ref)
    # with counts: rows beyond count[s] are untouched
    cnt = np.array([0, 500, T], np.int32)
    sentinel = torch.full_like(x, 7.0)
    out2 = sc.scfa_gather_rows(x, _t(idx), _t(cnt), out=sentinel.clone())
    for s in range(S):
        assert torch.equal(out2[s, :cnt[s]], ref[s, :cnt[s]])
        assert torch.equal(out2[s, cnt[s]:], sentinel[s, cnt[s]:])


def test_gather_rows_bf16_to_f16_compute_format():
    """bf16 -> fp16 on the way (IEEE, round to nearest even): equals torch's conversion bit for bit,
    including values below the fp16 normal range, values above its maximum (which become infinite: an input
    outside the compute format must show in the results) and NaN (which stays NaN)."""
    S, T, d = 2, 777, 64
    rng = np.random.default_rng(9)
    x = rng.standard_normal((S, T, d)).astype(np.float32)
    x[0, :5] *= 1e-6          # fp16 denormals / flush
    x[1, :3] *= 1e6           # beyond 65504: +-inf
    x[1, 5, 7] = np.nan
    xb = torch.from_numpy(x).to(DEV).to(torch.bfloat16)
    idx = np.stack([rng.permutation(T) for _ in range(S)]).astype(np.int32)
    out = sc.scfa_gather_rows(xb, _t(idx), to_f16=True)
    assert out.dtype == torch.float16
    ref = torch.gather(xb, 1, _t(idx).long()[..., None].expand(-1, -1, d)).float().to(torch.float16)
    assert torch.isinf(ref).any() and torch.isnan(ref).any()
    assert torch.equal(out.view(torch.int16), ref.view(torch.int16))     # bit patterns: NaN compares unequal to itself


def test_gather_rows_scaled_queries():
    """A gather with a scale multiplies in fp32 before the one rounding to the output format:
    equals torch's float multiply + conversion bit for bit."""
    S, T, d = 2, 515, 64
    rng = np.random.default_rng(11)
    x = rng.standard_normal((S, T, d)).astype(np.float32)
    idx = np.stack([rng.permutation(T) for _ in range(S)]).astype(np.int32)
    scale = float(np.float32(0.125) * np.float32(1.4426950408889634))
    xb = torch.from_numpy(x).to(DEV).to(torch.bfloat16)
    g = torch.gather(xb, 1, _t(idx).long()[..., None].expand(-1, -1, d)).float()
    out = sc.scfa_gather_rows(xb, _t(idx), to_f16=True, scale=scale)
    assert torch.equal(out, (g * scale).to(torch.float16))
    xf = torch.from_numpy(x).to(DEV)
    gf = torch.gather(xf, 1, _t(idx).long()[..., None].expand(-1, -1, d))
    assert torch.equal(sc.scfa_gather_rows(xf, _t(idx), scale=scale), gf * scale)


@pytest.mark.parametrize("S,T,nb", [(1, 8, 3), (3, 4097, 7), (2, 16384, 8), (5, 1000, 16)])
def test_pair_entry_points_match_single_calls(S, T, nb):
    """Query and key side in one launch: same results as two separate calls, bit for bit."""
    rng = np.random.default_rng(S + T + nb)
    bq = rng.integers(0, nb, (S, T)).astype(np.int32)
    bk = rng.integers(0, nb, (S, T)).astype(np.int32)
    (qi, qs, qo, qkey), (ki, ks, ko, kkey) = sc.scfa_sort_by_bucket_pair(_t(bq), _t(bk), nb)
    for got, key, b in (((qi, qs, qo), qkey, bq), ((ki, ks, ko), kkey, bk)):
        ref = oracle.sort_by_bucket(b, nb)
        for a, r in zip(got, ref):
            assert np.array_equal(a.cpu().numpy(), r)
        # sort key of a sorted row = the pair it was ordered by, bucket << 24 | position
        assert np.array_equal(key.cpu().numpy().astype(np.int64) & 0xffffffff, (ref[1].astype(np.int64) << 24) | ref[0])
        single = sc.scfa_sort_by_bucket(_t(b), nb, want_sort_key=True)
        assert torch.equal(single[3], key) and torch.equal(single[0], got[0])
    kq = (rng.random((S, T)) < 0.6).astype(np.uint8)
    kk = (rng.random((S, T)) < 0.3).astype(np.uint8)
    (cqi, cnq), (cki, cnk) = sc.scfa_compact_keep_pair(_t(kq), _t(kk))
    for (gi, gn), keep in (((cqi, cnq), kq), ((cki, cnk), kk)):
        ri, rn = oracle.compact_keep(keep)
        assert np.array_equal(gi.cpu().numpy(), ri) and np.array_equal(gn.cpu().numpy(), rn)
    # fused Q/K/V gather against the single-tensor gather
    d = 64
    q, k, v = (torch.from_numpy(rng.standard_normal((S, T, d)).astype(np.float32)).to(DEV).to(torch.bfloat16)
               for _ in range(3))
    scale = float(np.float32(0.125) * np.float32(1.4426950408889634))
    for nq_, nk_ in ((None, None), (cnq, cnk)):
        i_q, i_k = (qi, ki) if nq_ is None else (cqi, cki)
        sent = [torch.full((S, T, d), 3.0, dtype=torch.float16, device=DEV) for _ in range(3)]
        r_q = sc.scfa_gather_rows(q, i_q, nq_, out=sent[0].clone(), to_f16=True, scale=scale)
        r_k = sc.scfa_gather_rows(k, i_k, nk_, out=sent[1].clone(), to_f16=True)
        r_v = sc.scfa_gather_rows(v, i_k, nk_, out=sent[2].clone(), to_f16=True)
        g_q, g_k, g_v = sc.scfa_gather_qkv(q, k, v, i_q, i_k, nq_, nk_, to_f16=True, q_scale=scale)
        for s_ in range(S):
            a, b = (T, T) if nq_ is None else (int(nq_[s_]), int(nk_[s_]))
            assert torch.equal(g_q[s_, :a], r_q[s_, :a])
            assert torch.equal(g_k[s_, :b], r_k[s_, :b]) and torch.equal(g_v[s_, :b], r_v[s_, :b])


@pytest.mark.parametrize("S,T,nb", [(1, 65536, 16), (3, 20000, 256), (2, 8192, 1), (1, 32768 + 77, 7), (40, 8192, 8),
                                    (5, 16384, 33), (3, 12000, 5), (2, 16385, 9)])
def test_chunked_sort_equals_single_workgroup_sort(S, T, nb):
    """Long sequences are cut into chunks sorted by several workgroups (above 16384 tokens only when scratch
    is given; up to there every workgroup counts the other chunks itself): same bits with and without
    scratch and as the oracle, for the sort and the compaction."""
    rng = np.random.default_rng(S * 7 + T + nb)
    b = rng.integers(0, nb, (S, T)).astype(np.int32)
    b[0, : T // 3] = nb - 1                          # a long run of one key across chunk borders
    assert sc.scfa_sort_workspace_bytes(S, T, nb) > 0 or S * 2 >= 256
    a = sc.scfa_sort_by_bucket(_t(b), nb, want_sort_key=True, use_ws=True)
    c = sc.scfa_sort_by_bucket(_t(b), nb, want_sort_key=True, use_ws=False)
    for x, y in zip(a, c):
        assert torch.equal(x, y)
    ref = oracle.sort_by_bucket(b, nb)
    for x, r in zip(a[:3], ref):
        assert np.array_equal(x.cpu().numpy(), r)
    (qa, _, oa, ka), (qb, _, ob, kb) = sc.scfa_sort_by_bucket_pair(_t(b), _t(b[:, ::-1].copy()), nb, want_sorted=False)
    (qc, _, oc, kc), (qd, _, od, kd) = sc.scfa_sort_by_bucket_pair(_t(b), _t(b[:, ::-1].copy()), nb, want_sorted=False, use_ws=False)
    assert torch.equal(qa, qc) and torch.equal(qb, qd) and torch.equal(oa, oc) and torch.equal(ob, od)
    assert torch.equal(ka, kc) and torch.equal(kb, kd) and torch.equal(qa, a[0])
    keep = (rng.random((S, T)) < 0.4).astype(np.uint8)
    i1, n1 = sc.scfa_compact_keep(_t(keep), use_ws=True)
    i2, n2 = sc.scfa_compact_keep(_t(keep), use_ws=False)
    ri, rn = oracle.compact_keep(keep)
    assert torch.equal(i1, i2) and torch.equal(n1, n2)
    assert np.array_equal(n1.cpu().numpy(), rn)
    for s_ in range(S):
        assert np.array_equal(i1[s_, : rn[s_]].cpu().numpy(), ri[s_, : rn[s_]])


# ------------------------------------------------------------------ LSH bucketing

@pytest.mark.parametrize("S,H,T,d,nb,dtype", [(4, 2, 1000, 64, 8, torch.bfloat16), (3, 3, 777, 128, 16, torch.bfloat16),
                                               (2, 1, 4096, 64, 2, torch.bfloat16), (2, 2, 513, 64, 64, torch.float32),
                                               (1, 1, 1, 64, 4, torch.bfloat16), (2, 2, 300, 128, 256, torch.float32),
                                               (2, 2, 5000, 64, 64, torch.bfloat16), (3, 1, 70001, 64, 6, torch.bfloat16),
                                               (2, 2, 2500, 128, 64, torch.bfloat16), (2, 1, 700, 64, 66, torch.bfloat16)])
def test_lsh_buckets_against_oracle(S, H, T, d, nb, dtype):
    """argmax over [xR, -xR]: an integer decided by floating point.  The kernel decides in fp32, the
    oracle in fp64, so: wherever the oracle's two largest candidates are further apart than fp32
    rounding of a d-term dot product can move them, the ids are equal; everywhere, the id the
    kernel picked is a candidate within that rounding of the oracle's maximum."""
    rng = np.random.default_rng(S * 100 + T + nb)
    x = torch.from_numpy(rng.standard_normal((S, T, d)).astype(np.float32)).to(DEV).to(dtype)
    y = torch.from_numpy(rng.standard_normal((S, T, d)).astype(np.float32)).to(DEV).to(dtype)
    R = rng.standard_normal((H, d, nb // 2)).astype(np.float32)
    bx, by = sc.scfa_lsh_buckets(x, y, _t(R), H, nb)
    bx1 = sc.scfa_lsh_buckets(x, None, _t(R), H, nb)
    assert torch.equal(bx, bx1)
    for t, got in ((x, bx), (y, by)):
        x64 = t.float().cpu().numpy().astype(np.float64)
        ref, margin = oracle.lsh_buckets(x64, R, H)
        ext = oracle.lsh_projections(x64, R, H)
        got = got.cpu().numpy()
        assert got.min() >= 0 and got.max() < nb
        eps = 64 * np.finfo(np.float32).eps * np.abs(x64).sum(-1) * np.abs(R).max()     # generous fp32 bound
        clear = margin > eps
        assert clear.mean() > 0.95
        assert np.array_equal(got[clear], ref[clear])
        picked = np.take_along_axis(ext, got[..., None].astype(np.int64), -1)[..., 0]
        assert (picked >= ext.max(-1) - eps).all()


def test_lsh_buckets_exact_ties_take_the_lowest_index():
    """Rows and projections of small integers: every product and sum is exact in fp32, so ties are
    real ties and the ids must equal the oracle's bit for bit."""
    rng = np.random.default_rng(3)
    S, H, T, d, nb = 2, 2, 640, 64, 8
    x = torch.from_numpy(rng.integers(-2, 3, (S, T, d)).astype(np.float32)).to(DEV).to(torch.bfloat16)
    x[0, :4] = 0                                     # all candidates tie at zero -> bucket 0
    R = rng.integers(-1, 2, (H, d, nb // 2)).astype(np.float32)
    got = sc.scfa_lsh_buckets(x, None, _t(R), H, nb).cpu().numpy()
    ref, margin = oracle.lsh_buckets(x.float().cpu().numpy(), R, H)
    assert (margin == 0).sum() > 10                  # the case does contain ties
    assert np.array_equal(got, ref)


# ------------------------------------------------------------------ schedule

def _check_order(live):
    """items come bucket pair by bucket pair; inside a pair the ranged side's count never grows"""
    group = live[:, 5] // 2
    assert np.all(np.diff(group) >= 0), "items must be grouped by bucket pair"
    same = np.diff(group) == 0
    assert np.all(np.diff(live[:, 3])[same] <= 0), "inside a bucket pair items must be ordered by decreasing work"


def _check_schedule(variant, lab_q, lab_k, nb, tiles, strict=False):
    """Several schedules are correct; check what must hold: every allowed pair is covered
    exactly once, claimed mask-free regions are mask-free, ranges are tight, items are
    ordered by bucket pair and by decreasing work inside a pair, counters match the emitted items.
    An item of several small buckets spans exactly the rows of those buckets on both sides,
    fits one tile of the tiled side and claims no mask-free region."""
    fm, fn, bn, bm = tiles
    S, T = lab_q.shape
    if variant == sc.SCFA_HASH:
        q_idx, _, q_off = sc.scfa_sort_by_bucket(_t(lab_q), nb)
        k_idx, _, k_off = sc.scfa_sort_by_bucket(_t(lab_k), nb)
        rq, _, _ = oracle.sort_by_bucket(lab_q, nb); rk, _, _ = oracle.sort_by_bucket(lab_k, nb)
        nq = np.full(S, T); nk = np.full(S, T)
        ovar = oracle.HASH
    else:
        q_idx, q_off = sc.scfa_compact_keep(_t(lab_q))
        k_idx, k_off = sc.scfa_compact_keep(_t(lab_k))
        rq, nq = oracle.compact_keep(lab_q); rk, nk = oracle.compact_keep(lab_k)
        ovar = oracle.QKDROP
    assert np.array_equal(q_idx.cpu().numpy(), rq) and np.array_equal(k_idx.cpu().numpy(), rk)
    fwd, bwd, cnt = sc.scfa_block_ranges(variant, q_idx, k_idx, q_off, k_off, nb, tiles,
                                         flags=sc.SCFA_FLAG_STRICT_CAUSAL if strict else 0)
    torch.cuda.synchronize()
    fwd, bwd, cnt = fwd.cpu().numpy(), bwd.cpu().numpy(), cnt.cpu().numpy()
    qo, ko = q_off.cpu().numpy(), k_off.cpu().numpy()
    merged = 0
    for s in range(S):
        M = oracle.allowed_mask(lab_q[s], lab_k[s], ovar, strict=strict)[np.ix_(rq[s], rk[s])]   # permuted coordinates
        M[nq[s]:, :] = False; M[:, nk[s]:] = False
        # forward list
        covered = np.zeros(T, bool)
        items = fwd[s]
        live = items[items[:, 1] > 0]
        assert np.all(items[len(live):] == 0), "unused items must trail and be zero"
        _check_order(live)
        tiles_f = 0; rect_f = 0
        for qb, qc, kb, kc, kn, bucket, nbk, _ in live:
            assert 0 < qc <= fm and 0 <= kn <= kc and nbk >= 1
            assert not covered[qb:qb + qc].any(); covered[qb:qb + qc] = True
            sub = M[qb:qb + qc]
            assert not sub[:, :kb].any() and not sub[:, kb + kc:].any(), "allowed pair outside the key range"
            assert sub[:, kb:kb + kn].all(), "mask-free prefix contains a masked pair"
            if nbk > 1:
                merged += 1
                assert kn == 0
                assert (qb, qb + qc) == (qo[s, bucket], qo[s, bucket + nbk]) and (kb, kb + kc) == (ko[s, bucket], ko[s, bucket + nbk])
            else:
                if kc:
                    assert sub[:, kb + kc - 1].any(), "key range is not tight"
                if kn < kc:
                    assert not sub[:, kb + kn].all(), "mask-free prefix is not maximal"
            tiles_f += -(-kc // fn); rect_f += qc * kc
        assert np.array_equal(covered[:nq[s]], np.ones(nq[s], bool)) and not covered[nq[s]:].any()
        # backward list
        covered = np.zeros(T, bool)
        items = bwd[s]
        live = items[items[:, 1] > 0]
        assert np.all(items[len(live):] == 0)
        _check_order(live)
        tiles_b = 0; rect_b = 0
        for kb, kc, qb, qc, qm, bucket, nbk, _ in live:
            assert 0 < kc <= bn and 0 <= qm <= qc and nbk >= 1
            assert not covered[kb:kb + kc].any(); covered[kb:kb + kc] = True
            sub = M[:, kb:kb + kc]
            assert not sub[:qb].any() and not sub[qb + qc:].any(), "allowed pair outside the query range"
            assert sub[qb + qm:qb + qc].all(), "unmasked query rows contain a masked pair"
            if nbk > 1:
                merged += 1
                assert qm == qc
                assert (qb, qb + qc) == (qo[s, bucket], qo[s, bucket + nbk]) and (kb, kb + kc) == (ko[s, bucket], ko[s, bucket + nbk])
            else:
                if qc:
                    assert sub[qb].any(), "query range is not tight"
                if qm:
                    assert not sub[qb + qm - 1].all()
            tiles_b += -(-qc // bm); rect_b += qc * kc
        assert np.array_equal(covered[:nk[s]], np.ones(nk[s], bool)) and not covered[nk[s]:].any()
        assert cnt[s].tolist() == [tiles_f, rect_f, tiles_b, rect_b]
    return merged


@pytest.mark.parametrize("S,T,nb", [(2, 700, 4), (1, 2048, 16), (3, 300, 1), (1, 129, 3), (2, 64, 8), (2, 1000, 64),
                                     (1, 4096, 256), (2, 1500, 24)])
def test_schedule_hash(S, T, nb):
    rng = np.random.default_rng(T + nb)
    bq = rng.integers(0, nb, (S, T)).astype(np.int32)
    bk = rng.integers(0, nb, (S, T)).astype(np.int32)
    if nb > 2:
        bk[bk == 2] = 0          # a bucket present in Q but absent in K
        bq[bq == 1] = 0          # and one present in K but absent in Q
    merged = _check_schedule(sc.SCFA_HASH, bq, bk, nb, sc.scfa_tile_config(64, sc.SCFA_BF16))
    assert (merged > 0) == (T / nb < 64), "buckets smaller than a tile are put together, larger ones are not"


@pytest.mark.parametrize("S,T,pq,pk", [(2, 900, 0.5, 0.5), (1, 2048, 0.3, 0.7), (2, 257, 1.0, 1.0),
                                       (2, 300, 0.0, 0.5), (2, 300, 0.5, 0.0)])
def test_schedule_qkdrop(S, T, pq, pk):
    rng = np.random.default_rng(T)
    kq = (rng.random((S, T)) < pq).astype(np.uint8)
    kk = (rng.random((S, T)) < pk).astype(np.uint8)
    _check_schedule(sc.SCFA_QKDROP, kq, kk, 1, sc.scfa_tile_config(64, sc.SCFA_BF16))


@pytest.mark.parametrize("S,T,nb", [(2, 700, 4), (1, 129, 3), (1, 1024, 1)])
def test_schedule_strict_causal(S, T, nb):
    """Strictly-earlier keys only (App. B.1's ">"): same validity conditions against the strict mask,
    for both variants; queries and keys share their labels in the second case (shared projections)."""
    rng = np.random.default_rng(T * 3 + nb)
    bq = rng.integers(0, nb, (S, T)).astype(np.int32)
    bk = rng.integers(0, nb, (S, T)).astype(np.int32)
    tiles = sc.scfa_tile_config(64, sc.SCFA_BF16)
    _check_schedule(sc.SCFA_HASH, bq, bk, nb, tiles, strict=True)
    _check_schedule(sc.SCFA_HASH, bq, bq, nb, tiles, strict=True)
    kq = (rng.random((S, T)) < 0.5).astype(np.uint8)
    _check_schedule(sc.SCFA_QKDROP, kq, kq, 1, tiles, strict=True)


@pytest.mark.parametrize("T,nb,strict", [(50001, 16, False), (70000, 5, True), (300000, 3, False)])
def test_schedule_long_sequences(T, nb, strict):
    """Sequences whose index vector does not fit in LDS are searched in two levels (every 2^k-th
    entry in LDS, then a few steps in global memory): every range end of every single-bucket item
    must equal what numpy's searchsorted gives on the oracle's sorted index vectors."""
    rng = np.random.default_rng(T)
    S = 2
    bq = rng.integers(0, nb, (S, T)).astype(np.int32); bk = rng.integers(0, nb, (S, T)).astype(np.int32)
    fm, fn, bn, bm = tiles = sc.scfa_tile_config(64, sc.SCFA_BF16)
    q_idx, _, q_off = sc.scfa_sort_by_bucket(_t(bq), nb)
    k_idx, _, k_off = sc.scfa_sort_by_bucket(_t(bk), nb)
    fwd, bwd, cnt = sc.scfa_block_ranges(sc.SCFA_HASH, q_idx, k_idx, q_off, k_off, nb, tiles,
                                         flags=sc.SCFA_FLAG_STRICT_CAUSAL if strict else 0)
    fwd, bwd = fwd.cpu().numpy(), bwd.cpu().numpy()
    qi, ki, qo, ko = (a.cpu().numpy() for a in (q_idx, k_idx, q_off, k_off))
    le, lt = ("left", "right") if strict else ("right", "left")     # searchsorted side for "<=" and "<" (swapped when strict)
    for s in range(S):
        live = fwd[s][fwd[s][:, 1] > 0]
        assert live[:, 1].sum() == T and (live[:, 6] == 1).all()
        for qb, qc, kb, kc, kn, b, _, _ in live:
            keys = ki[s, ko[s, b]:ko[s, b + 1]]
            assert kb == ko[s, b]
            assert kc == np.searchsorted(keys, qi[s, qb + qc - 1], side=le)
            assert kn == np.searchsorted(keys, qi[s, qb], side=le)
        live = bwd[s][bwd[s][:, 1] > 0]
        assert live[:, 1].sum() == T
        for kb, kc, qb, qc, qm, b, _, _ in live:
            qs = qi[s, qo[s, b]:qo[s, b + 1]]
            first = np.searchsorted(qs, ki[s, kb], side=lt)
            assert qb == qo[s, b] + first and qc == len(qs) - first
            assert qm == max(0, np.searchsorted(qs, ki[s, kb + kc - 1], side=lt) - first)


def test_schedule_regular_case_is_lower_triangular():
    """No sparsity: the computed tile set coincides with FlashAttention's (Fig. 2, left),
    and never exceeds what the paper's Alg. 2 range rule computes."""
    T = 1024
    fm, fn, bn, bm = tiles = sc.scfa_tile_config(64, sc.SCFA_BF16)
    lab = np.zeros((1, T), np.int32)
    q_idx, _, q_off = sc.scfa_sort_by_bucket(_t(lab), 1)
    fwd, bwd, cnt = sc.scfa_block_ranges(sc.SCFA_HASH, q_idx, q_idx, q_off, q_off, 1, tiles)
    fwd = fwd.cpu().numpy()[0]
    live = fwd[fwd[:, 1] > 0]
    got = sorted((int(qb) // fm, -(-int(kc) // fn)) for qb, qc, kb, kc, kn, *_ in live)
    assert got == [(i, (i + 1) * fm // fn) for i in range(T // fm)]
    ref = oracle.paper_tile_ranges_hash(np.arange(T), np.arange(T), lab[0], lab[0], fm, fn)
    assert int(cnt[0, 0]) == sum(e - a for a, e in ref)


def test_schedule_computes_no_more_than_paper_rule():
    """On LSH-like bucket sizes the bucket-anchored tiles cover no more area than the
    ranges of Alg. 2 with the same tile shape (the paper notes its tiles straddle bucket
    boundaries, App. C)."""
    S, T, nb = 2, 4096, 16
    fm, fn, bn, bm = tiles = sc.scfa_tile_config(64, sc.SCFA_BF16)
    rng = np.random.default_rng(5)
    bq = rng.integers(0, nb, (S, T)).astype(np.int32); bk = rng.integers(0, nb, (S, T)).astype(np.int32)
    q_idx, q_bs, q_off = sc.scfa_sort_by_bucket(_t(bq), nb)
    k_idx, k_bs, k_off = sc.scfa_sort_by_bucket(_t(bk), nb)
    _, _, cnt = sc.scfa_block_ranges(sc.SCFA_HASH, q_idx, k_idx, q_off, k_off, nb, tiles)
    for s in range(S):
        ref = oracle.paper_tile_ranges_hash(q_idx[s].cpu().numpy(), k_idx[s].cpu().numpy(),
                                            q_bs[s].cpu().numpy(), k_bs[s].cpu().numpy(), fm, fn)
        assert int(cnt[s, 0]) <= sum(e - a for a, e in ref)


# ------------------------------------------------------------------ measurement aids

def test_occupancy_query():
    """Workgroups per compute unit as the runtime derives them from registers and LDS: at least one
    for every attention kernel (a launch would otherwise fail), and no more than the LDS ring allows."""
    for kernel, ring_bytes in (("fwd", 3 * (64 * 64 * 4 + 256)), ("bwd_dkdv", 3 * 17664), ("bwd_dq", 3 * (64 * 64 * 4 + 256))):
        n64, n128 = sc.scfa_prof_occupancy(kernel, 64), sc.scfa_prof_occupancy(kernel, 128)
        print(kernel, n64, n128)
        assert 1 <= n128 <= n64 <= (160 * 1024) // ring_bytes
