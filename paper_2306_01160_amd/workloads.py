"""Seeded synthetic inputs shaped like the paper's workloads.

This module only draws inputs (numpy, CPU).  It holds none of the method's
arithmetic and imports neither the HIP binding nor the CPU oracle; tests and
the benchmark feed the same arrays to both sides.

Shapes and distributions follow the paper's "runtime in a vacuum" experiments
(random Q, K, V; bucket ids or drop decisions "given for free", Sec. 4.2 and
4.3) and its language-model setup (12 heads of 64 dimensions, T = 8192 and
16384, Sec. 4.1).  They stand in for activations of models trained on the
paper's datasets, which are not available here.

All floating-point tensors are returned as float32 arrays whose values are
exactly representable in the workload's dtype (bf16 values are rounded to
nearest-even first), so that widening them to fp64 for the oracle and
narrowing them to bf16 for the GPU are both exact.
"""
from __future__ import annotations

from dataclasses import dataclass, field

import numpy as np

HASH = "hash"
QKDROP = "qkdrop"


def round_to_bf16(x: np.ndarray) -> np.ndarray:
    """Round float32 values to the nearest bfloat16 (ties to even); returns float32."""
    x = np.ascontiguousarray(x, dtype=np.float32)
    u = x.view(np.uint32)
    rounded = (u + np.uint32(0x7FFF) + ((u >> np.uint32(16)) & np.uint32(1))) & np.uint32(0xFFFF0000)
    return rounded.view(np.float32)


def bf16_bits(x: np.ndarray) -> np.ndarray:
    """uint16 bit patterns of float32 values that are already bf16-representable."""
    x = np.ascontiguousarray(x, dtype=np.float32)
    u = x.view(np.uint32)
    assert not np.any(u & np.uint32(0xFFFF)), "values are not bf16-representable"
    return (u >> np.uint32(16)).astype(np.uint16)


def lsh_buckets(x: np.ndarray, R: np.ndarray) -> np.ndarray:
    """Cross-polytope style bucket ids: argmax over [xR, -xR] (ties -> lowest index).

    ``x`` is ``[B, H, T, d]``, ``R`` is ``[H, d, nb/2]`` (one projection per head,
    applied separately to every row).  The paper adopts the LSH scheme of Andoni
    et al. (Sec. 4.2, "Hashing mechanism") without printing the formula; this is
    the form the benchmark configuration states.
    """
    proj = np.einsum("bhtd,hdr->bhtr", x.astype(np.float64), R.astype(np.float64))
    both = np.concatenate([proj, -proj], axis=-1)
    return np.argmax(both, axis=-1).astype(np.int32)


@dataclass
class Workload:
    name: str
    variant: str            # HASH or QKDROP
    dtype: str              # "bf16" or "f32"
    B: int
    H: int
    T: int
    d: int
    nb: int                 # number of buckets (hash); 1 for QK-dropping
    q: np.ndarray           # [B,H,T,d] float32 (values exact in `dtype`)
    k: np.ndarray
    v: np.ndarray
    do: np.ndarray          # upstream gradient, same shape
    lab_q: np.ndarray       # [B,H,T] int32 bucket ids (hash) or uint8 keep flags (qkdrop)
    lab_k: np.ndarray
    passes: str = "fwd+bwd"
    meta: dict = field(default_factory=dict)

    @property
    def S(self) -> int:
        return self.B * self.H

    @property
    def tau(self) -> float:
        # softmax scale 1/sqrt(d), the default of the paper's interface (App. B.2)
        return 1.0 / float(np.sqrt(self.d))


def _normal(rng, shape, scale, dtype):
    x = (rng.standard_normal(shape, dtype=np.float32) * np.float32(scale)).astype(np.float32)
    return round_to_bf16(x) if dtype == "bf16" else x


def hash_uniform(seed, B, H, T, d, nb, dtype="bf16", scale=1.0, name=None, passes="fwd+bwd"):
    """Bucket ids drawn independently and uniformly in {0..nb-1} for every query
    and every key (the paper's vacuum benchmark, Sec. 4.2)."""
    rng = np.random.default_rng(seed)
    shape = (B, H, T, d)
    q, k, v, do = (_normal(rng, shape, scale, dtype) for _ in range(4))
    lab_q = rng.integers(0, nb, size=(B, H, T), dtype=np.int32)
    lab_k = rng.integers(0, nb, size=(B, H, T), dtype=np.int32)
    return Workload(name or f"hash_uniform_T{T}_nb{nb}", HASH, dtype, B, H, T, d, nb,
                    q, k, v, do, lab_q, lab_k, passes, {"seed": seed, "buckets": "uniform"})


def hash_lsh(seed, B, H, T, d, nb, dtype="bf16", scale=1.0, name=None, passes="fwd+bwd"):
    """Bucket ids from the LSH ``argmax([xR, -xR])`` with a d x nb/2 Gaussian R per
    head, applied to the (rounded) query and key rows separately.  nb = 1 puts
    every token in bucket 0: the dense causal twin."""
    rng = np.random.default_rng(seed)
    shape = (B, H, T, d)
    q, k, v, do = (_normal(rng, shape, scale, dtype) for _ in range(4))
    if nb == 1:
        lab_q = np.zeros((B, H, T), dtype=np.int32)
        lab_k = np.zeros((B, H, T), dtype=np.int32)
    else:
        assert nb % 2 == 0
        R = rng.standard_normal((H, d, nb // 2), dtype=np.float32)
        lab_q = lsh_buckets(q, R)
        lab_k = lsh_buckets(k, R)
    return Workload(name or f"hash_lsh_T{T}_nb{nb}", HASH, dtype, B, H, T, d, nb,
                    q, k, v, do, lab_q, lab_k, passes, {"seed": seed, "buckets": "lsh"})


def qkdrop_bernoulli(seed, B, H, T, d, keep_q, keep_k, dtype="bf16", scale=1.0, name=None,
                     passes="fwd+bwd"):
    """Every query / key is kept independently per (batch, head) with the given
    probabilities (the paper's random dropping, Sec. 4.3)."""
    rng = np.random.default_rng(seed)
    shape = (B, H, T, d)
    q, k, v, do = (_normal(rng, shape, scale, dtype) for _ in range(4))
    lab_q = (rng.random((B, H, T)) < keep_q).astype(np.uint8)
    lab_k = (rng.random((B, H, T)) < keep_k).astype(np.uint8)
    return Workload(name or f"qkdrop_T{T}_q{keep_q}_k{keep_k}", QKDROP, dtype, B, H, T, d, 1,
                    q, k, v, do, lab_q, lab_k, passes,
                    {"seed": seed, "keep_q": keep_q, "keep_k": keep_k})


# ---- the five benchmark configurations -----------------------------------

def config1():
    """Hash, forward only, fp32: B=1, H=1, T=256, d=64, nb=4, uniform buckets."""
    return hash_uniform(1, 1, 1, 256, 64, 4, dtype="f32", name="c1_hash_fp32_T256", passes="fwd")


def config2(B=4, H=8, T=2048):
    """QK-dropping, fwd+bwd, bf16: B=4, H=8, T=2048, d=64, keep 0.5 / 0.5."""
    return qkdrop_bernoulli(2, B, H, T, 64, 0.5, 0.5, name=f"c2_qkdrop_T{T}")


def config3(B=4, H=12, T=8192):
    """Hash (LSH, nb=16), fwd+bwd, bf16: B=4, H=12, T=8192, d=64."""
    return hash_lsh(3, B, H, T, 64, 16, name=f"c3_hash_T{T}_nb16")


def config4(B=2, H=12, T=16384, nb=8):
    """Hash (LSH, nb=8), fwd+bwd, bf16, values 0.5*N(0,1): B=2, H=12, T=16384, d=64.
    nb=1 is the dense causal twin of the same shape."""
    return hash_lsh(4, B, H, T, 64, nb, scale=0.5, name=f"c4_hash_T{T}_nb{nb}")


def config5(B=1, H=16, T=32768, keep_q=0.5, keep_k=0.3, seed=5):
    """QK-dropping, long sequence, fwd+bwd, bf16: B=1, H=16, T=32768, d=128."""
    return qkdrop_bernoulli(seed, B, H, T, 128, keep_q, keep_k,
                            name=f"c5_qkdrop_T{T}_q{keep_q}_k{keep_k}")


CONFIG5_SWEEP = (1.0, 0.7, 0.5, 0.3, 0.1)
