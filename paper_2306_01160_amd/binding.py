"""ctypes binding of libscfa.so: one Python function per C entry point, same names.

Argument marshalling only: tensors are torch CUDA tensors (PyTorch provides device
memory and the stream), pointers and sizes are passed through unchanged, outputs are
allocated here with ``torch.empty``.  Every step of the path runs in the library's
kernels.  There is no fallback: if the library is missing or a call fails, an
exception is raised.
"""
from __future__ import annotations

import ctypes
import os

import torch

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.environ.get("SCFA_LIB", os.path.join(_HERE, "libscfa.so"))

SCFA_OK = 0
SCFA_EINVAL, SCFA_EUNSUPPORTED, SCFA_EWORKSPACE, SCFA_EHIP = -1, -2, -3, -4
SCFA_BF16, SCFA_F32, SCFA_F16 = 0, 1, 2
SCFA_HASH, SCFA_QKDROP = 0, 1
SCFA_FLAG_STRICT_CAUSAL = 1
SCFA_WORK_STRIDE = 8
KERNEL_IDS = {"sort": 0, "compact": 1, "gather": 2, "ranges": 3, "fwd": 4, "bwd_prep": 5,
              "bwd_dkdv": 6, "bwd_dq": 7, "fill": 8, "lsh": 9}

EXPORTS = [
    "scfa_version", "scfa_last_hip_error", "scfa_error_string", "scfa_sort_by_bucket", "scfa_sort_by_bucket_static",
    "scfa_count_invalid_buckets", "scfa_sort_by_bucket_pair", "scfa_compact_keep_pair", "scfa_gather_qkv", "scfa_lsh_buckets",
    "scfa_compact_keep", "scfa_gather_rows", "scfa_block_ranges", "scfa_num_work_items",
    "scfa_tile_config", "scfa_hash_attn_fwd", "scfa_qkdrop_attn_fwd",
    "scfa_attn_bwd_workspace_bytes", "scfa_sort_workspace_bytes", "scfa_hash_attn_bwd", "scfa_qkdrop_attn_bwd",
    "scfa_prof_enable", "scfa_prof_reset", "scfa_prof_read", "scfa_prof_occupancy",
]


class ScfaError(RuntimeError):
    pass


_lib = None


def lib():
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise ScfaError(f"{LIB_PATH} is missing: build it with `python -m paper_2306_01160_amd.build`")
        L = ctypes.CDLL(LIB_PATH)
        vp, ci, cf, sz = ctypes.c_void_p, ctypes.c_int, ctypes.c_float, ctypes.c_size_t
        L.scfa_version.restype = ci
        L.scfa_last_hip_error.restype = ci
        L.scfa_error_string.restype = ctypes.c_char_p
        L.scfa_error_string.argtypes = [ci]
        L.scfa_sort_by_bucket.argtypes = [vp, ci, ci, ci, vp, vp, vp, vp, vp, sz, vp]
        L.scfa_sort_by_bucket_static.argtypes = [vp, ci, ci, ci, vp, vp, vp, vp, vp]
        L.scfa_count_invalid_buckets.argtypes = [vp, ctypes.c_longlong, ci, vp, vp]
        L.scfa_compact_keep.argtypes = [vp, ci, ci, vp, vp, vp, sz, vp]
        L.scfa_lsh_buckets.argtypes = [vp, vp, vp, ci, ci, ci, ci, ci, ci, vp, vp, vp]
        L.scfa_sort_by_bucket_pair.argtypes = [vp, vp, ci, ci, ci, vp, vp, vp, vp, vp, vp, vp, vp, vp, sz, vp]
        L.scfa_compact_keep_pair.argtypes = [vp, vp, ci, ci, vp, vp, vp, vp, vp, sz, vp]
        L.scfa_gather_qkv.argtypes = [vp, vp, vp, vp, vp, vp, vp, ci, ci, ci, ci, ci, ctypes.c_float, vp, vp, vp, vp]
        L.scfa_gather_rows.argtypes = [vp, vp, vp, ci, ci, ci, ci, ci, ctypes.c_float, vp, vp]
        L.scfa_block_ranges.argtypes = [ci, vp, vp, vp, vp, ci, ci, ci, ci, ci, ci, ci, ci, vp, vp, vp, vp]
        L.scfa_num_work_items.argtypes = [ci, ci, ci]
        ip = ctypes.POINTER(ci)
        L.scfa_tile_config.argtypes = [ci, ci, ip, ip, ip, ip]
        L.scfa_hash_attn_fwd.argtypes = [vp, vp, vp, vp, vp, vp, ci, ci, ci, ci, ci, ci, cf, ci, vp, vp, vp, vp]
        L.scfa_qkdrop_attn_fwd.argtypes = [vp, vp, vp, vp, vp, vp, vp, ci, ci, ci, ci, ci, ci, cf, ci, vp, vp, vp, vp]
        L.scfa_attn_bwd_workspace_bytes.argtypes = [ci, ci, ci, ci]
        L.scfa_attn_bwd_workspace_bytes.restype = sz
        L.scfa_sort_workspace_bytes.argtypes = [ci, ci, ci]
        L.scfa_sort_workspace_bytes.restype = sz
        L.scfa_hash_attn_bwd.argtypes = [vp, vp, vp, vp, vp, vp, ci, vp, ci, vp, vp, vp, vp,
                                         ci, ci, ci, ci, ci, cf, ci, vp, vp, vp, vp, sz, vp]
        L.scfa_qkdrop_attn_bwd.argtypes = [vp, vp, vp, vp, vp, vp, vp, vp, ci, vp, ci, vp, vp, vp, vp,
                                           ci, ci, ci, ci, ci, cf, ci, vp, vp, vp, vp, sz, vp]
        L.scfa_prof_enable.argtypes = [ci]
        L.scfa_prof_read.argtypes = [ci, ctypes.POINTER(ctypes.c_double), ip]
        L.scfa_prof_occupancy.argtypes = [ci, ci, ip]
        for name in EXPORTS:
            fn = getattr(L, name)
            if name not in ("scfa_error_string", "scfa_attn_bwd_workspace_bytes", "scfa_sort_workspace_bytes"):
                fn.restype = ci
        _lib = L
    return _lib


def _check(rc: int, what: str):
    if rc != SCFA_OK:
        L = lib()
        msg = L.scfa_error_string(rc).decode()
        extra = f" (hipError {L.scfa_last_hip_error()})" if rc == SCFA_EHIP else ""
        raise ScfaError(f"{what}: {msg}{extra}")


def _ptr(t):
    if t is None:
        return None
    assert t.is_cuda and t.is_contiguous(), "expect contiguous CUDA tensors"
    return t.data_ptr()


def _stream():
    return torch.cuda.current_stream().cuda_stream


def dtype_code(t: torch.Tensor) -> int:
    if t.dtype in (torch.bfloat16, torch.float16):   # fp16 = compute format of bf16 tensors
        return SCFA_BF16
    if t.dtype == torch.float32:
        return SCFA_F32
    raise ScfaError(f"unsupported dtype {t.dtype}")


def _out_dtype(x_perm: torch.Tensor):
    """O has the dtype of the original tensors: bf16 when the permuted copies are fp16."""
    return torch.bfloat16 if x_perm.dtype == torch.float16 else x_perm.dtype


# ---------------------------------------------------------------- entry points

def scfa_version() -> int:
    return lib().scfa_version()


def scfa_num_work_items(T: int, nb: int, tile: int) -> int:
    return lib().scfa_num_work_items(T, nb, tile)


def scfa_tile_config(d: int, dtype: int):
    a, b, c, e = (ctypes.c_int() for _ in range(4))
    _check(lib().scfa_tile_config(d, dtype, ctypes.byref(a), ctypes.byref(b), ctypes.byref(c), ctypes.byref(e)),
           "scfa_tile_config")
    return a.value, b.value, c.value, e.value


def scfa_lsh_buckets(x_q: torch.Tensor, x_k, R: torch.Tensor, H: int, nb: int):
    """x_q, x_k [S,T,d] (x_k may be None), R [H,d,nb/2] float32 -> bucket ids int32 [S,T] (one or two)."""
    S, T, d = x_q.shape
    assert R.dtype == torch.float32 and tuple(R.shape) == (H, d, nb // 2)
    out = torch.empty((2 if x_k is not None else 1, S, T), dtype=torch.int32, device=x_q.device)
    _check(lib().scfa_lsh_buckets(_ptr(x_q), _ptr(x_k), _ptr(R), S, H, T, d, nb, dtype_code(x_q), _ptr(out[0]),
                                  _ptr(out[1]) if x_k is not None else None, _stream()), "scfa_lsh_buckets")
    return (out[0], out[1]) if x_k is not None else out[0]


def scfa_sort_workspace_bytes(S, T, nb) -> int:
    return int(lib().scfa_sort_workspace_bytes(S, T, nb))


def _sort_ws(S, T, nb, device, use_ws):
    """Scratch for the chunked sort of long sequences (None: one workgroup per segment)."""
    need = scfa_sort_workspace_bytes(S, T, nb) if use_ws else 0
    return (torch.empty((need,), dtype=torch.uint8, device=device), need) if need else (None, 0)


def scfa_sort_by_bucket(bucket: torch.Tensor, nb: int, want_sort_key=False, use_ws=True):
    """bucket [S,T] int32 -> idx [S,T], bucket_sorted [S,T], off [S,nb+1] (all int32); with
    want_sort_key also the [S,T] sort keys bucket << 24 | position (uint32 bits in an int32 tensor)."""
    S, T = bucket.shape
    idx = torch.empty_like(bucket)
    bsorted = torch.empty_like(bucket)
    off = torch.empty((S, nb + 1), dtype=torch.int32, device=bucket.device)
    key = torch.empty_like(bucket) if want_sort_key else None
    ws, ws_bytes = _sort_ws(S, T, nb, bucket.device, use_ws)
    _check(lib().scfa_sort_by_bucket(_ptr(bucket), S, T, nb, _ptr(idx), _ptr(bsorted), _ptr(off), _ptr(key),
                                     _ptr(ws), ws_bytes, _stream()), "scfa_sort_by_bucket")
    return (idx, bsorted, off, key) if want_sort_key else (idx, bsorted, off)


def scfa_sort_by_bucket_static(bucket: torch.Tensor, nb: int, idx: torch.Tensor, bsorted, off: torch.Tensor, key):
    """The sort with the library's own scratch: outputs are passed in (the call allocates nothing)."""
    S, T = bucket.shape
    _check(lib().scfa_sort_by_bucket_static(_ptr(bucket), S, T, nb, _ptr(idx), _ptr(bsorted), _ptr(off), _ptr(key),
                                            _stream()), "scfa_sort_by_bucket_static")


def scfa_count_invalid_buckets(bucket: torch.Tensor, nb: int) -> torch.Tensor:
    """Number of ids outside [0, nb) as a one-element int32 device tensor (not synchronised)."""
    out = torch.empty(1, dtype=torch.int32, device=bucket.device)
    _check(lib().scfa_count_invalid_buckets(_ptr(bucket), bucket.numel(), nb, _ptr(out), _stream()),
           "scfa_count_invalid_buckets")
    return out


def scfa_compact_keep(keep: torch.Tensor, use_ws=True):
    """keep [S,T] uint8 -> idx [S,T] int32 (kept then dropped positions), count [S] int32."""
    S, T = keep.shape
    idx = torch.empty((S, T), dtype=torch.int32, device=keep.device)
    count = torch.empty((S,), dtype=torch.int32, device=keep.device)
    ws, ws_bytes = _sort_ws(S, T, 2, keep.device, use_ws)
    _check(lib().scfa_compact_keep(_ptr(keep), S, T, _ptr(idx), _ptr(count), _ptr(ws), ws_bytes, _stream()),
           "scfa_compact_keep")
    return idx, count


def scfa_sort_by_bucket_pair(bucket_q: torch.Tensor, bucket_k: torch.Tensor, nb: int, want_sorted=True, use_ws=True):
    """Both sides of one attention call in one launch ->
    (q_idx, q_sorted, q_off, q_sort_key), (k_idx, k_sorted, k_off, k_sort_key)."""
    S, T = bucket_q.shape
    assert bucket_k.shape == bucket_q.shape
    both = torch.empty((2, S, T), dtype=torch.int32, device=bucket_q.device)
    srt = torch.empty((2, S, T), dtype=torch.int32, device=bucket_q.device) if want_sorted else None
    off = torch.empty((2, S, nb + 1), dtype=torch.int32, device=bucket_q.device)
    key = torch.empty((2, S, T), dtype=torch.int32, device=bucket_q.device)
    ws, ws_bytes = _sort_ws(S, T, nb, bucket_q.device, use_ws)
    _check(lib().scfa_sort_by_bucket_pair(_ptr(bucket_q), _ptr(bucket_k), S, T, nb, _ptr(both[0]),
                                          _ptr(srt[0]) if want_sorted else None, _ptr(off[0]), _ptr(key[0]),
                                          _ptr(both[1]), _ptr(srt[1]) if want_sorted else None, _ptr(off[1]),
                                          _ptr(key[1]), _ptr(ws), ws_bytes, _stream()),
           "scfa_sort_by_bucket_pair")
    return ((both[0], srt[0] if want_sorted else None, off[0], key[0]),
            (both[1], srt[1] if want_sorted else None, off[1], key[1]))


def scfa_compact_keep_pair(keep_q: torch.Tensor, keep_k: torch.Tensor, use_ws=True):
    """Both sides of one attention call in one launch -> (q_idx, n_q), (k_idx, n_k)."""
    S, T = keep_q.shape
    assert keep_k.shape == keep_q.shape
    idx = torch.empty((2, S, T), dtype=torch.int32, device=keep_q.device)
    cnt = torch.empty((2, S), dtype=torch.int32, device=keep_q.device)
    ws, ws_bytes = _sort_ws(S, T, 2, keep_q.device, use_ws)
    _check(lib().scfa_compact_keep_pair(_ptr(keep_q), _ptr(keep_k), S, T, _ptr(idx[0]), _ptr(cnt[0]), _ptr(idx[1]),
                                        _ptr(cnt[1]), _ptr(ws), ws_bytes, _stream()), "scfa_compact_keep_pair")
    return (idx[0], cnt[0]), (idx[1], cnt[1])


def scfa_gather_qkv(q, k, v, q_idx, k_idx, n_q=None, n_k=None, to_f16=False, q_scale=1.0):
    """Permuted / compacted Q (times q_scale), K, V in one launch; inputs [S,T,d]."""
    S, T, d = q.shape
    odt = torch.float16 if to_f16 else q.dtype
    out = torch.empty((3, S, T, d), dtype=odt, device=q.device)
    out_code = SCFA_F16 if to_f16 else dtype_code(q)
    _check(lib().scfa_gather_qkv(_ptr(q), _ptr(k), _ptr(v), _ptr(q_idx), _ptr(k_idx), _ptr(n_q), _ptr(n_k), S, T, d,
                                 dtype_code(q), out_code, float(q_scale), _ptr(out[0]), _ptr(out[1]), _ptr(out[2]),
                                 _stream()), "scfa_gather_qkv")
    return out[0], out[1], out[2]


def scfa_gather_rows(x: torch.Tensor, idx: torch.Tensor, count=None, out=None, to_f16=False, scale=1.0):
    """x [S,T,d], idx [S,T] -> out [S,T,d] with out[s,r] = scale * x[s, idx[s,r]] for r < count[s] (or T).
    to_f16: bf16 input is written in the fp16 compute format of the attention kernels."""
    S, T, d = x.shape
    if out is None:
        out = torch.empty(x.shape, dtype=torch.float16 if to_f16 else x.dtype, device=x.device)
    out_code = SCFA_F16 if to_f16 else dtype_code(x)
    _check(lib().scfa_gather_rows(_ptr(x), _ptr(idx), _ptr(count), S, T, d, dtype_code(x), out_code, float(scale),
                                  _ptr(out), _stream()), "scfa_gather_rows")
    return out


def scfa_block_ranges(variant, q_idx, k_idx, q_off, k_off, nb, tiles, want_bwd=True, want_counters=True, flags=0):
    """-> fwd_work [S,n_fwd,8], bwd_work [S,n_bwd,8] or None, counters [S,4] int64 or None."""
    S, T = q_idx.shape
    fm, fn, bn, bm = tiles
    n_fwd = scfa_num_work_items(T, nb, fm)
    n_bwd = scfa_num_work_items(T, nb, bn)
    dev = q_idx.device
    fwd = torch.empty((S, n_fwd, SCFA_WORK_STRIDE), dtype=torch.int32, device=dev)
    bwd = torch.empty((S, n_bwd, SCFA_WORK_STRIDE), dtype=torch.int32, device=dev) if want_bwd else None
    cnt = torch.empty((S, 4), dtype=torch.int64, device=dev) if want_counters else None
    _check(lib().scfa_block_ranges(variant, _ptr(q_idx), _ptr(k_idx), _ptr(q_off), _ptr(k_off), S, T, nb,
                                   fm, fn, bn, bm, int(flags), _ptr(fwd), _ptr(bwd), _ptr(cnt), _stream()),
           "scfa_block_ranges")
    return fwd, bwd, cnt


def scfa_hash_attn_fwd(q_perm, k_perm, v_perm, q_sort_key, k_sort_key, fwd_work, B, H, sm_scale, o_out=None, lse_out=None,
                       o_f16_out=None, flags=0):
    S, T, d = q_perm.shape
    assert S == B * H
    o = torch.empty((B, H, T, d), dtype=_out_dtype(q_perm), device=q_perm.device) if o_out is None else o_out
    lse = torch.empty((B, H, T), dtype=torch.float32, device=q_perm.device) if lse_out is None else lse_out
    _check(lib().scfa_hash_attn_fwd(_ptr(q_perm), _ptr(k_perm), _ptr(v_perm), _ptr(q_sort_key), _ptr(k_sort_key),
                                    _ptr(fwd_work), fwd_work.shape[1], B, H, T, d, dtype_code(q_perm),
                                    float(sm_scale), int(flags), _ptr(o), _ptr(lse), _ptr(o_f16_out), _stream()),
           "scfa_hash_attn_fwd")
    return o, lse


def scfa_qkdrop_attn_fwd(q_c, k_c, v_c, q_idx, k_idx, n_q, fwd_work, B, H, sm_scale, o_out=None, lse_out=None,
                         o_f16_out=None, flags=0):
    S, T, d = q_c.shape
    assert S == B * H
    o = torch.empty((B, H, T, d), dtype=_out_dtype(q_c), device=q_c.device) if o_out is None else o_out
    lse = torch.empty((B, H, T), dtype=torch.float32, device=q_c.device) if lse_out is None else lse_out
    _check(lib().scfa_qkdrop_attn_fwd(_ptr(q_c), _ptr(k_c), _ptr(v_c), _ptr(q_idx), _ptr(k_idx), _ptr(n_q),
                                      _ptr(fwd_work), fwd_work.shape[1], B, H, T, d, dtype_code(q_c),
                                      float(sm_scale), int(flags), _ptr(o), _ptr(lse), _ptr(o_f16_out), _stream()),
           "scfa_qkdrop_attn_fwd")
    return o, lse


def scfa_attn_bwd_workspace_bytes(S, T, d, dtype) -> int:
    return int(lib().scfa_attn_bwd_workspace_bytes(S, T, d, dtype))


def _bwd_outputs(B, H, T, d, dev, outs):
    if outs is not None:
        return outs
    return tuple(torch.empty((B, H, T, d), dtype=torch.float32, device=dev) for _ in range(3))


def scfa_hash_attn_bwd(q_perm, k_perm, v_perm, q_sort_key, k_sort_key, fwd_work, bwd_work, o, lse, d_o, B, H, sm_scale,
                       ws=None, outs=None, o_f16=None, flags=0):
    S, T, d = q_perm.shape
    dt = dtype_code(q_perm)
    need = scfa_attn_bwd_workspace_bytes(S, T, d, dt)
    if ws is None:
        ws = torch.empty((need,), dtype=torch.uint8, device=q_perm.device)
    dq, dk, dv = _bwd_outputs(B, H, T, d, q_perm.device, outs)
    _check(lib().scfa_hash_attn_bwd(_ptr(q_perm), _ptr(k_perm), _ptr(v_perm), _ptr(q_sort_key), _ptr(k_sort_key),
                                    _ptr(fwd_work), fwd_work.shape[1], _ptr(bwd_work), bwd_work.shape[1],
                                    _ptr(o), _ptr(o_f16), _ptr(lse), _ptr(d_o), B, H, T, d, dt, float(sm_scale),
                                    int(flags), _ptr(dq), _ptr(dk), _ptr(dv), _ptr(ws), ws.numel(), _stream()),
           "scfa_hash_attn_bwd")
    return dq, dk, dv


def scfa_qkdrop_attn_bwd(q_c, k_c, v_c, q_idx, k_idx, n_q, n_k, fwd_work, bwd_work, o, lse, d_o, B, H, sm_scale,
                         ws=None, outs=None, o_f16=None, flags=0):
    S, T, d = q_c.shape
    dt = dtype_code(q_c)
    need = scfa_attn_bwd_workspace_bytes(S, T, d, dt)
    if ws is None:
        ws = torch.empty((need,), dtype=torch.uint8, device=q_c.device)
    dq, dk, dv = _bwd_outputs(B, H, T, d, q_c.device, outs)
    _check(lib().scfa_qkdrop_attn_bwd(_ptr(q_c), _ptr(k_c), _ptr(v_c), _ptr(q_idx), _ptr(k_idx), _ptr(n_q),
                                      _ptr(n_k), _ptr(fwd_work), fwd_work.shape[1], _ptr(bwd_work),
                                      bwd_work.shape[1], _ptr(o), _ptr(o_f16), _ptr(lse), _ptr(d_o), B, H, T, d, dt,
                                      float(sm_scale), int(flags), _ptr(dq), _ptr(dk), _ptr(dv), _ptr(ws), ws.numel(),
                                      _stream()), "scfa_qkdrop_attn_bwd")
    return dq, dk, dv


def scfa_prof_enable(on: bool) -> int:
    return lib().scfa_prof_enable(1 if on else 0)


def scfa_prof_reset():
    _check(lib().scfa_prof_reset(), "scfa_prof_reset")


def scfa_prof_occupancy(kernel: str, d: int) -> int:
    """Workgroups of an attention kernel ("fwd", "bwd_dkdv", "bwd_dq") resident per compute unit."""
    n = ctypes.c_int(0)
    _check(lib().scfa_prof_occupancy(KERNEL_IDS[kernel], int(d), ctypes.byref(n)), "scfa_prof_occupancy")
    return n.value


def scfa_prof_read(kernel: str):
    ms, n = ctypes.c_double(), ctypes.c_int()
    _check(lib().scfa_prof_read(KERNEL_IDS[kernel], ctypes.byref(ms), ctypes.byref(n)), "scfa_prof_read")
    return ms.value, n.value
