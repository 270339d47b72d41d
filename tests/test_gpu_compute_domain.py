"""The fp16 compute format of the bf16 path: inputs far from N(0,1) scale.

The kernels convert bf16 inputs to fp16 (exact for magnitudes in [2^-17, 65504]) and run the
contractions on fp16 matrix instructions with fp32 accumulation.  These tests leave unit scale:
everything scaled by 2^8 / 2^-8 where the method stays well conditioned, outlier rows of magnitude
1e3 in K, in V and in Q, gradients of magnitude 1e-6, logits in the thousands.  The benchmark states
max-abs bounds (2e-2 on O and the gradients, 1e-3 on the logsumexp) for N(0,1) inputs, whose outputs are
of order one; for outputs of another size the same bounds are applied relative to the largest reference
magnitude of the tensor (and, for the logsumexp, never below four units in the last place of an fp32 of
its size).  Beyond the format's range the library must not return finite nonsense: those cases check
that the results are non-finite.
"""
import numpy as np
import pytest
import torch

import oracle
from gpu_util import labels, oracle_variant, run_gpu, seg64
from paper_2306_01160_amd import workloads as W

pytestmark = pytest.mark.gpu

REL = {"O": 5e-3, "dQ": 5e-3, "dK": 5e-3, "dV": 5e-3}   # of max |reference|; 2e-2 absolute at max |ref| = 4


def _errors(wl):
    o, lse, grads, _ = run_gpu(wl)
    S, T, d = wl.S, wl.T, wl.d
    lq, lk = labels(wl)
    Q, K, V, dO = (seg64(wl, a) for a in (wl.q, wl.k, wl.v, wl.do))
    O_ref, L_ref = oracle.attention_forward(Q, K, V, lq, lk, oracle_variant(wl), wl.tau)
    dQ_ref, dK_ref, dV_ref = oracle.attention_backward(Q, K, V, dO, lq, lk, oracle_variant(wl), wl.tau)
    got = {"O": o.float().cpu().numpy().reshape(S, T, d), "dQ": grads[0].cpu().numpy().reshape(S, T, d),
           "dK": grads[1].cpu().numpy().reshape(S, T, d), "dV": grads[2].cpu().numpy().reshape(S, T, d)}
    ref = {"O": O_ref, "dQ": dQ_ref, "dK": dK_ref, "dV": dV_ref}
    lg = lse.cpu().numpy().reshape(S, T)
    return got, ref, lg, L_ref


def _check(wl, names=("O", "dQ", "dK", "dV")):
    got, ref, lg, L_ref = _errors(wl)
    fin = np.isfinite(L_ref)
    assert np.array_equal(np.isfinite(lg), fin)
    lse_tol = np.maximum(1e-3, 4 * np.spacing(np.abs(L_ref[fin]).astype(np.float32)).astype(np.float64))
    assert np.all(np.abs(lg[fin] - L_ref[fin]) <= lse_tol), float(np.abs(lg[fin] - L_ref[fin]).max())
    for n in names:
        assert np.isfinite(got[n]).all(), f"{n} has non-finite values"
        scale = float(np.abs(ref[n]).max())
        err = float(np.abs(got[n] - ref[n]).max())
        assert err <= REL[n] * scale, f"{n}: max-abs error {err:.3g} against max |ref| {scale:.3g}"


def _scaled(wl, sq=1.0, sk=1.0, sv=1.0, sdo=1.0):
    wl.q = W.round_to_bf16(wl.q * np.float32(sq))
    wl.k = W.round_to_bf16(wl.k * np.float32(sk))
    wl.v = W.round_to_bf16(wl.v * np.float32(sv))
    wl.do = W.round_to_bf16(wl.do * np.float32(sdo))
    return wl


def _base(d, variant):
    if variant == "hash":
        return W.hash_uniform(31, 1, 2, 1024, d, 4)
    return W.qkdrop_bernoulli(32, 1, 2, 1100, d, 0.6, 0.5)


@pytest.mark.parametrize("d", [64, 128])
@pytest.mark.parametrize("variant", ["hash", "qkdrop"])
def test_everything_scaled_down_by_2_to_8(d, variant):
    """values of a few 1e-3: part of them subnormal in fp16; logits ~1e-4: a near-uniform softmax"""
    _check(_scaled(_base(d, variant), 2.0 ** -8, 2.0 ** -8, 2.0 ** -8, 2.0 ** -8))


@pytest.mark.parametrize("d", [64, 128])
@pytest.mark.parametrize("variant", ["hash", "qkdrop"])
def test_values_and_gradients_scaled_up_by_2_to_8(d, variant):
    """|V| and |dO| in the hundreds: O, D and dP - D in the thousands"""
    _check(_scaled(_base(d, variant), 1.0, 1.0, 256.0, 256.0))


@pytest.mark.parametrize("d", [64, 128])
def test_logits_in_the_thousands(d):
    """Q and K scaled by 2^4: logits up to ~1e3, a sharply peaked softmax; the recomputed scores of the
    backward must be as exact as the forward's"""
    _check(_scaled(_base(d, "hash"), 16.0, 16.0, 1.0, 1.0))


@pytest.mark.parametrize("d", [64, 128])
@pytest.mark.parametrize("which", ["k", "v", "q"])
def test_outlier_rows_of_magnitude_1e3(d, which):
    wl = _base(d, "hash")
    a = getattr(wl, which)
    a[:, :, 100, :] *= 1000.0
    a[:, :, 700, :] *= 1000.0
    setattr(wl, which, W.round_to_bf16(a))
    _check(wl)


@pytest.mark.parametrize("d", [64, 128])
def test_upstream_gradient_of_magnitude_1e_minus_6(d):
    _check(_scaled(_base(d, "qkdrop"), 1.0, 1.0, 1.0, 1e-6))


def test_values_beyond_the_fp16_range_give_non_finite_outputs():
    """one V row of magnitude 1e5 (a legal bf16 value, no fp16 value): the rows that attend it must not
    come back finite"""
    wl = _base(64, "hash")
    wl.v[:, :, 100, :] = np.float32(1.0e5)
    wl.v = W.round_to_bf16(wl.v)
    o, lse, grads, _ = run_gpu(wl)
    og = o.float().cpu().numpy().reshape(wl.S, wl.T, wl.d)
    lq, lk = labels(wl)
    for s in range(wl.S):
        sees = (lq[s] == lk[s, 100]) & (np.arange(wl.T) >= 100)      # queries that attend key 100
        assert sees.any()
        assert not np.isfinite(og[s][sees]).all(axis=1).any(), "a row attending the out-of-range value is finite"
    assert np.isfinite(lse.cpu().numpy()[np.isfinite(lse.cpu().numpy())]).all()   # the logsumexp does not involve V


def test_nan_in_an_input_reaches_the_output():
    wl = _base(64, "hash")
    wl.k[0, 0, 50, 3] = np.nan
    o, lse, grads, _ = run_gpu(wl, backward=False)
    og = o.float().cpu().numpy().reshape(wl.S, wl.T, wl.d)
    lq, lk = labels(wl)
    sees = (lq[0] == lk[0, 50]) & (np.arange(wl.T) >= 50)
    assert np.isnan(og[0][sees]).any(axis=1).all(), "NaN in a key must show in every row that attends it"
    assert np.isfinite(og[1]).all()                                  # the other segment is untouched


def test_logits_beyond_the_backward_range_give_non_finite_gradients():
    """everything scaled by 2^8: logits of ~3e5, |LSE| / tau beyond what the backward's aux rows hold.  The forward
    is still exact (one-hot softmax); the gradients must not come back finite."""
    wl = _scaled(_base(64, "hash"), 256.0, 256.0, 256.0, 256.0)
    got, ref, lg, L_ref = _errors(wl)
    fin = np.isfinite(L_ref)
    assert np.abs(L_ref[fin]).max() * 8 > 2.1e6                       # the case is out of range
    assert np.all(np.abs(lg[fin] - L_ref[fin]) <= 4 * np.spacing(np.abs(L_ref[fin]).astype(np.float32)))
    assert float(np.abs(got["O"] - ref["O"]).max()) <= REL["O"] * float(np.abs(ref["O"]).max())
    big = fin & (np.abs(np.where(fin, L_ref, 0.0)) * 8 > 2.2e6)       # rows clearly beyond the range (LSE / tau, tau = 1/8)
    assert big.sum() >= 4
    for n in ("dQ",):
        g = got[n]
        assert not np.isfinite(g[big]).all(axis=-1).any(), f"{n}: an out-of-range row came back finite"
    assert not np.isfinite(got["dK"]).all() and not np.isfinite(got["dV"]).all()
