"""GPU attention (forward and backward, both variants) vs the fp64 oracle, element by
element in ORIGINAL order, at sizes that span several tiles and ragged tails, on the
degenerate cases, and at the five benchmark configurations.

Tolerances (bf16 inputs, fp32 accumulation): max-abs 2e-2 on O, dQ, dK, dV and 1e-3 on
the logsumexp; fp32 path: 1e-4 on O and 1e-5 on the logsumexp.
"""
import numpy as np
import pytest
import torch

from paper_2306_01160_amd import workloads as W

from gpu_util import assert_within, compare_backward, compare_forward, run_gpu

pytestmark = pytest.mark.gpu


def _full_check(wl, backward=True):
    o, lse, grads, ctx = run_gpu(wl, backward=backward)
    errs = compare_forward(wl, o, lse)
    if backward:
        errs.update(compare_backward(wl, grads))
    print(wl.name, {k: f"{v:.2e}" for k, v in errs.items()})
    assert_within(errs, wl.dtype)
    return errs


# --------------------------------------------------------------- small / ragged

def test_config1_hash_fp32_forward():
    _full_check(W.config1(), backward=False)


@pytest.mark.parametrize("T,nb,d", [(256, 4, 64), (333, 3, 64), (1000, 2, 128), (130, 1, 64), (64, 8, 128),
                                    (1, 1, 64), (700, 16, 64), (500, 64, 64)])
def test_hash_fp32_forward_shapes(T, nb, d):
    _full_check(W.hash_uniform(100 + T, 1, 2, T, d, nb, dtype="f32", passes="fwd"), backward=False)


@pytest.mark.parametrize("T,nb,d", [(256, 4, 64), (333, 3, 64), (1000, 2, 128), (130, 1, 64), (2049, 1, 64),
                                    (64, 8, 128), (1, 1, 64), (700, 16, 64), (1500, 4, 128)])
def test_hash_bf16_forward_backward_shapes(T, nb, d):
    _full_check(W.hash_uniform(200 + T, 2, 2, T, d, nb))


@pytest.mark.parametrize("T,nb,d,strict", [(1000, 64, 64, False), (1111, 200, 128, False), (2048, 256, 64, False),
                                           (900, 48, 64, True), (300, 256, 128, True)])
def test_hash_bf16_buckets_smaller_than_a_tile(T, nb, d, strict):
    """Many buckets of a few rows each: the schedule puts consecutive buckets into one work item and
    the kernels tell them apart by the sort keys in every tile."""
    wl = W.hash_uniform(800 + T, 1, 3, T, d, nb)
    wl.meta["strict"] = strict
    _full_check(wl)


def test_hash_bf16_small_and_large_buckets_mixed():
    """Bucket sizes from one row to several tiles in one segment (sizes like 1 / rank), and
    buckets that have queries but no keys and the reverse."""
    rng = np.random.default_rng(9)
    wl = W.hash_uniform(9, 1, 2, 3000, 64, 40)
    p = 1.0 / np.arange(1, 41); p /= p.sum()
    wl.lab_q[...] = rng.choice(40, size=wl.lab_q.shape, p=p).astype(np.int32)
    wl.lab_k[...] = rng.choice(40, size=wl.lab_k.shape, p=p).astype(np.int32)
    wl.lab_k[wl.lab_k == 17] = 3
    wl.lab_q[wl.lab_q == 30] = 31
    _full_check(wl)


@pytest.mark.parametrize("T,pq,pk,d", [(512, 0.5, 0.5, 64), (777, 0.3, 0.7, 64), (1025, 1.0, 1.0, 64),
                                       (900, 0.7, 0.2, 128), (65, 0.5, 0.5, 128)])
def test_qkdrop_bf16_forward_backward_shapes(T, pq, pk, d):
    _full_check(W.qkdrop_bernoulli(300 + T, 1, 3, T, d, pq, pk))


def test_qkdrop_fp32_forward():
    _full_check(W.qkdrop_bernoulli(7, 1, 2, 300, 64, 0.5, 0.5, dtype="f32", passes="fwd"), backward=False)


def test_scores_growing_along_the_sequence():
    """Scores that rise by ~40 base-2 units from the first key to the last: the forward's reference
    maximum, taken from a row's first tiles, falls far behind and has to be raised several times
    (probabilities computed against a stale reference leave the fp16 range; the kernel has to
    notice, and redo the tile).  The forward forms <q, k> from the inputs' own values and scales in
    fp32, so the logsumexp of ~30 still meets the plain 1e-3 bound."""
    T, d = 1500, 64
    wl = W.hash_uniform(31, 1, 2, T, d, 1)
    rng = np.random.default_rng(31)
    u = np.where(rng.random(d) < 0.5, -1.0, 1.0).astype(np.float32)
    ramp = (np.arange(T, dtype=np.float32) / T)[:, None]
    wl.q[...] = u                                          # tau <q, k_j> = 8 * 3.75 * j / T
    wl.k[...] = W.round_to_bf16((np.float32(3.75) * ramp * u).astype(np.float32))
    o, lse, grads, _ = run_gpu(wl)
    errs = compare_forward(wl, o, lse)
    errs.update(compare_backward(wl, grads))
    print(wl.name, {k: f"{v:.2e}" for k, v in errs.items()})
    lse_max = float(np.abs(lse.cpu().numpy()).max())
    assert lse_max > 25.0
    assert errs["LSE"] <= 1e-3
    assert max(errs["O"], errs["dQ"], errs["dK"], errs["dV"]) <= 2e-2


# --------------------------------------------------------------- strictly-causal mask

def _strict(wl, shared_qk=False):
    wl.meta["strict"] = True
    if shared_qk:      # keys = queries and one set of labels (the paper's shared-projection setting)
        wl.k = wl.q.copy()
        wl.lab_k = wl.lab_q.copy()
    return wl


@pytest.mark.parametrize("T,nb,d,shared", [(700, 4, 64, False), (1500, 2, 128, False), (1029, 8, 64, True),
                                           (130, 1, 64, True)])
def test_strict_causal_hash_bf16(T, nb, d, shared):
    """App. B.1's ">" mask: a token does not attend itself; the first query of each bucket is stranded."""
    wl = _strict(W.hash_uniform(500 + T, 1, 2, T, d, nb), shared)
    errs = _full_check(wl)
    if shared:   # with shared labels the first token of every bucket has no earlier key
        o, lse, _, _ = run_gpu(wl, backward=False)
        lab = wl.lab_q.reshape(wl.S, wl.T)
        for s in range(wl.S):
            for b in np.unique(lab[s]):
                first = int(np.flatnonzero(lab[s] == b)[0])
                assert np.isneginf(lse.cpu().numpy().reshape(wl.S, wl.T)[s, first])


@pytest.mark.parametrize("T,pq,pk,d", [(777, 0.5, 0.5, 64), (600, 1.0, 1.0, 128)])
def test_strict_causal_qkdrop_bf16(T, pq, pk, d):
    _full_check(_strict(W.qkdrop_bernoulli(600 + T, 1, 2, T, d, pq, pk)))


def test_strict_causal_fp32_forward():
    _full_check(_strict(W.hash_uniform(77, 1, 2, 300, 64, 3, dtype="f32", passes="fwd")), backward=False)


# --------------------------------------------------------------- seeded random shapes

@pytest.mark.parametrize("seed", range(12))
def test_seeded_random_shapes(seed):
    """Shapes, sparsity, variant and mask form drawn from a seeded generator: ragged lengths, bucket
    counts from 1 to 40 (more buckets than a tile has rows), keep rates from 5 % to 100 %."""
    rng = np.random.default_rng(1000 + seed)
    T = int(rng.integers(1, 2600))
    d = int(rng.choice([64, 128]))
    B, H = int(rng.integers(1, 3)), int(rng.integers(1, 4))
    strict = bool(rng.integers(0, 2))
    if rng.integers(0, 2):
        wl = W.hash_uniform(seed, B, H, T, d, int(rng.integers(1, 41)))
    else:
        wl = W.qkdrop_bernoulli(seed, B, H, T, d, float(rng.uniform(0.05, 1.0)), float(rng.uniform(0.05, 1.0)))
    wl.meta["strict"] = strict
    _full_check(wl)


@pytest.mark.parametrize("seed", range(2000, 2024))
def test_seeded_random_shapes_many_buckets(seed):
    """As above with up to 256 buckets (rows that see one or two keys: the logsumexp is then a single
    score), bucket sizes skewed like 1 / rank, and keep rates down to 2 %."""
    rng = np.random.default_rng(seed)
    T = int(rng.integers(1, 3000))
    d = int(rng.choice([64, 128]))
    B, H = int(rng.integers(1, 3)), int(rng.integers(1, 4))
    strict = bool(rng.integers(0, 2))
    kind = int(rng.integers(0, 3))
    if kind == 0:
        wl = W.hash_uniform(seed, B, H, T, d, int(rng.integers(1, 257)))
    elif kind == 1:
        nb = int(rng.integers(2, 129))
        wl = W.hash_uniform(seed, B, H, T, d, nb)
        p = 1.0 / np.arange(1, nb + 1); p /= p.sum()
        wl.lab_q[...] = rng.choice(nb, size=wl.lab_q.shape, p=p).astype(np.int32)
        wl.lab_k[...] = rng.choice(nb, size=wl.lab_k.shape, p=p).astype(np.int32)
    else:
        wl = W.qkdrop_bernoulli(seed, B, H, T, d, float(rng.uniform(0.02, 1.0)), float(rng.uniform(0.02, 1.0)))
    wl.meta["strict"] = strict
    _full_check(wl)


# --------------------------------------------------------------- degenerate cases

def test_bucket_present_in_q_but_absent_in_k_gives_zero_rows():
    wl = W.hash_uniform(41, 1, 2, 400, 64, 4)
    wl.lab_k[wl.lab_k == 2] = 3          # no key in bucket 2: those queries are stranded
    wl.lab_q[wl.lab_q == 1] = 0          # no query in bucket 1: those keys get zero gradients
    o, lse, grads, _ = run_gpu(wl)
    stranded = wl.lab_q == 2
    assert stranded.any()
    assert not o.float().cpu().numpy()[stranded].any()
    assert np.isneginf(lse.cpu().numpy()[stranded]).all()
    assert not grads[0].cpu().numpy()[stranded].any()
    orphan_keys = wl.lab_k == 1
    assert not grads[1].cpu().numpy()[orphan_keys].any() and not grads[2].cpu().numpy()[orphan_keys].any()
    errs = compare_forward(wl, o, lse); errs.update(compare_backward(wl, grads))
    assert_within(errs, wl.dtype)


def test_queries_and_keys_in_disjoint_buckets():
    """No query shares a bucket with any key: every output row is zero, every LSE is -inf, every
    gradient is zero (large and small buckets, i.e. own and shared work items)."""
    for T, nb in ((900, 4), (700, 64)):
        wl = W.hash_uniform(43, 1, 2, T, 64, nb)
        wl.lab_q[...] = (wl.lab_q // 2) * 2            # queries in even buckets
        wl.lab_k[...] = (wl.lab_k // 2) * 2 + 1        # keys in odd buckets
        o, lse, grads, _ = run_gpu(wl)
        assert not o.float().cpu().numpy().any()
        assert np.isneginf(lse.cpu().numpy()).all()
        for g in grads:
            assert not g.cpu().numpy().any()


def test_more_buckets_than_tokens():
    """256 buckets for 100 tokens: most buckets are empty, the rest hold one or two rows."""
    wl = W.hash_uniform(44, 2, 2, 100, 128, 256)
    wl.lab_k[...] = wl.lab_q                          # shared labels so that some pairs exist
    _full_check(wl)
    wl.meta["strict"] = True
    _full_check(wl)


def test_zero_kept_keys_and_zero_kept_queries():
    wl = W.qkdrop_bernoulli(42, 1, 2, 300, 64, 0.5, 0.5)
    wl.lab_k[0, 0, :] = 0                # head 0: every key dropped
    wl.lab_q[0, 1, :] = 0                # head 1: every query dropped
    o, lse, grads, _ = run_gpu(wl)
    assert not o.float().cpu().numpy().any()
    assert np.isneginf(lse.cpu().numpy()).all()
    for g in grads:
        assert not g.cpu().numpy().any()
    errs = compare_forward(wl, o, lse); errs.update(compare_backward(wl, grads))
    assert_within(errs, wl.dtype)


def test_first_kept_query_before_first_kept_key():
    wl = W.qkdrop_bernoulli(43, 1, 1, 200, 64, 1.0, 1.0)
    wl.lab_k[0, 0, :50] = 0              # queries 0..49 are kept but have no key
    o, lse, grads, _ = run_gpu(wl)
    assert not o.float().cpu().numpy()[0, 0, :50].any()
    errs = compare_forward(wl, o, lse); errs.update(compare_backward(wl, grads))
    assert_within(errs, wl.dtype)


@pytest.mark.parametrize("T,d,pq,pk", [(500, 64, 0.5, 0.5), (1300, 128, 0.3, 0.7), (2100, 64, 0.9, 0.1)])
def test_outputs_do_not_depend_on_previous_buffer_contents(T, d, pq, pk):
    """Outputs are fully written, the rows of dropped tokens included: poison-filled output buffers give the same result."""
    from paper_2306_01160_amd import binding as sc
    from gpu_util import to_gpu
    from paper_2306_01160_amd import pipeline
    wl = W.qkdrop_bernoulli(44, 1, 2, T, d, pq, pk)
    q, k, v, do, lq, lk = to_gpu(wl)
    o1, lse1, ctx = pipeline.qkdrop_forward(q, k, v, lq, lk, wl.tau)
    g1 = pipeline.qkdrop_backward(ctx, do)
    o2 = torch.full_like(o1, float("nan")); lse2 = torch.full_like(lse1, float("nan"))
    sc.scfa_qkdrop_attn_fwd(ctx.q_p, ctx.k_p, ctx.v_p, ctx.q_idx, ctx.k_idx, ctx.n_q, ctx.fwd_work, 1, 2, wl.tau,
                            o_out=o2, lse_out=lse2)
    outs = tuple(torch.full_like(g, float("nan")) for g in g1)
    g2 = pipeline.qkdrop_backward(ctx, do, outs=outs)
    torch.cuda.synchronize()
    assert torch.equal(o1, o2) and torch.equal(lse1, lse2)
    for a, b in zip(g1, g2):
        assert torch.equal(a, b)
    for g, lab in ((g2[0], lq), (g2[1], lk), (g2[2], lk)):
        assert not g.reshape(-1, d)[lab.reshape(-1) == 0].any()
    assert not o2.reshape(-1, d)[lq.reshape(-1) == 0].any()


def test_two_runs_are_bit_identical():
    """No float atomics anywhere: the path is deterministic."""
    wl = W.hash_lsh(45, 1, 2, 2048, 64, 8)
    o1, l1, g1, _ = run_gpu(wl)
    o2, l2, g2, _ = run_gpu(wl)
    assert torch.equal(o1, o2) and torch.equal(l1, l2)
    for a, b in zip(g1, g2):
        assert torch.equal(a, b)


def test_side_stream_gives_the_same_bits():
    """All work is enqueued on the caller's stream: a whole forward + backward issued on a second
    stream (default priority), with the per-kernel event timers switched on, returns bit for bit
    what the default stream returns."""
    from paper_2306_01160_amd import binding as sc
    for wl in (W.hash_uniform(46, 1, 2, 1300, 64, 6), W.qkdrop_bernoulli(47, 1, 2, 900, 128, 0.6, 0.4)):
        o1, l1, g1, _ = run_gpu(wl)
        side = torch.cuda.Stream()
        side.wait_stream(torch.cuda.current_stream())
        sc.scfa_prof_reset(); sc.scfa_prof_enable(True)
        with torch.cuda.stream(side):
            o2, l2, g2, _ = run_gpu(wl)
        sc.scfa_prof_enable(False)
        ms, n = sc.scfa_prof_read("fwd")
        sc.scfa_prof_reset()
        torch.cuda.synchronize()
        assert n == 1 and ms > 0.0
        assert torch.equal(o1, o2) and torch.equal(l1, l2)
        for a, b in zip(g1, g2):
            assert torch.equal(a, b)


def test_hip_graph_replays_match_eager():
    """The library neither allocates nor synchronises nor clears memory with memset nodes, so a whole
    forward + backward can be captured in a HIP graph.  Three replays, each after the inputs were
    overwritten in place and with eager work in between, must equal the eager result bit for bit."""
    from paper_2306_01160_amd import pipeline
    from gpu_util import to_gpu
    wl = W.hash_uniform(48, 1, 2, 1500, 64, 6)
    q, k, v, do, lq, lk = to_gpu(wl)

    def run():
        o, lse, ctx = pipeline.hash_forward(q, k, v, lq, lk, wl.nb, wl.tau)
        return (o, lse) + tuple(pipeline.hash_backward(ctx, do))

    run()                                            # first launches set kernel attributes: not under capture
    torch.cuda.synchronize()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph):
        captured = run()
    gen = torch.Generator(device=q.device); gen.manual_seed(5)
    for rep in range(3):
        q.copy_(torch.randn(q.shape, device=q.device, generator=gen).to(q.dtype))
        lq.copy_(torch.randint(0, wl.nb, lq.shape, device=q.device, generator=gen, dtype=torch.int32))
        graph.replay()
        torch.cuda.synchronize()
        got = [t.clone() for t in captured]
        want = run()                                 # eager work between the replays
        torch.cuda.synchronize()
        for a, b in zip(got, want):
            assert torch.equal(a, b), f"replay {rep} differs from the eager result"


# --------------------------------------------------------------- benchmark configurations

def test_config2_qkdrop_bf16():
    _full_check(W.config2())


def test_config3_hash_lsh_T8192():
    _full_check(W.config3())


def test_config4_hash_lsh_T16384():
    _full_check(W.config4())


def test_config4_dense_twin_sampled():
    """nb = 1 (dense causal) at T = 16384: the oracle checks sampled rows of two heads."""
    wl = W.config4(nb=1)
    o, lse, grads, _ = run_gpu(wl)
    rows = np.unique(np.concatenate([np.arange(0, 130), np.arange(8000, 8130), np.arange(16384 - 130, 16384),
                                     np.random.default_rng(0).integers(0, 16384, 64)])).astype(np.int32)
    segs = [0, 17]
    errs = compare_forward(wl, o, lse, segs=segs, rows=rows)
    errs.update(compare_backward(wl, grads, segs=segs, q_rows=rows, k_rows=rows))
    print(wl.name, errs)
    assert_within(errs, wl.dtype)


def test_config5_qkdrop_T32768_d128_sampled():
    """B=1, H=16, T=32768, d=128, keep 0.5 (queries) / 0.3 (keys): sampled rows of three heads."""
    wl = W.config5()
    o, lse, grads, _ = run_gpu(wl)
    rows = np.unique(np.concatenate([np.arange(0, 200), np.arange(20000, 20100), np.arange(32768 - 200, 32768),
                                     np.random.default_rng(1).integers(0, 32768, 100)])).astype(np.int32)
    segs = [0, 7, 15]
    errs = compare_forward(wl, o, lse, segs=segs, rows=rows)
    errs.update(compare_backward(wl, grads, segs=segs, q_rows=rows, k_rows=rows))
    print(wl.name, errs)
    assert_within(errs, wl.dtype)
    # dropped rows are exactly zero everywhere
    dq = grads[0].cpu().numpy()
    assert not dq[wl.lab_q == 0].any()
    assert not o.float().cpu().numpy()[wl.lab_q == 0].any()


def test_hash_T65536_sampled():
    """The longest sequence of the speed-up sweep (B=1, H=2, T=65536, d=64, 16 uniformly random
    buckets): sampled rows of one head; the schedule's index vector no longer fits in LDS here."""
    T = 65536
    wl = W.hash_uniform(65, 1, 2, T, 64, 16)
    o, lse, grads, _ = run_gpu(wl)
    rows = np.unique(np.concatenate([np.arange(0, 140), np.arange(40000, 40100), np.arange(T - 140, T),
                                     np.random.default_rng(2).integers(0, T, 100)])).astype(np.int32)
    segs = [1]
    errs = compare_forward(wl, o, lse, segs=segs, rows=rows)
    errs.update(compare_backward(wl, grads, segs=segs, q_rows=rows, k_rows=rows))
    print(wl.name, errs)
    assert_within(errs, wl.dtype)


def test_hash_T262144_sampled():
    """Four times the longest sequence of the sweep (B=1, H=1, T=262144, d=64, 128 uniformly random buckets):
    byte offsets inside the segment pass 2^25, the sort runs in 64 chunks, the schedule holds 2176 items per
    list; sampled rows against the oracle."""
    T = 262144
    wl = W.hash_uniform(66, 1, 1, T, 64, 128)
    o, lse, grads, _ = run_gpu(wl)
    rows = np.unique(np.concatenate([np.arange(0, 140), np.arange(200000, 200100), np.arange(T - 140, T),
                                     np.random.default_rng(3).integers(0, T, 100)])).astype(np.int32)
    segs = [0]
    errs = compare_forward(wl, o, lse, segs=segs, rows=rows)
    errs.update(compare_backward(wl, grads, segs=segs, q_rows=rows, k_rows=rows))
    print(wl.name, errs)
    assert_within(errs, wl.dtype)

