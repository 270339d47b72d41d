"""The allocation-free sort entry point against the workspace one (bit-exact), called through
the C ABI twice in a row on one device, the second time with a smaller input."""
import ctypes

import numpy as np
import pytest
import torch

from paper_2306_01160_amd import binding as sc

pytestmark = pytest.mark.gpu


def _raw_sort_ws(bucket, nb):
    """scfa_sort_by_bucket through the raw ABI with a caller workspace."""
    L = sc.lib()
    S, T = bucket.shape
    dev = bucket.device
    idx, srt, key = (torch.full((S, T), -7, dtype=torch.int32, device=dev) for _ in range(3))
    off = torch.full((S, nb + 1), -7, dtype=torch.int32, device=dev)
    need = int(L.scfa_sort_workspace_bytes(S, T, nb))
    ws = torch.empty((max(need, 1),), dtype=torch.uint8, device=dev)
    rc = L.scfa_sort_by_bucket(bucket.data_ptr(), S, T, nb, idx.data_ptr(), srt.data_ptr(), off.data_ptr(),
                               key.data_ptr(), ws.data_ptr(), need, torch.cuda.current_stream().cuda_stream)
    assert rc == sc.SCFA_OK
    return idx, srt, off, key, need


def _raw_sort_static(bucket, nb):
    L = sc.lib()
    S, T = bucket.shape
    dev = bucket.device
    idx, srt, key = (torch.full((S, T), -9, dtype=torch.int32, device=dev) for _ in range(3))
    off = torch.full((S, nb + 1), -9, dtype=torch.int32, device=dev)
    rc = L.scfa_sort_by_bucket_static(bucket.data_ptr(), S, T, nb, idx.data_ptr(), srt.data_ptr(), off.data_ptr(),
                                      key.data_ptr(), torch.cuda.current_stream().cuda_stream)
    assert rc == sc.SCFA_OK, sc.lib().scfa_error_string(rc)
    return idx, srt, off, key


def test_static_scratch_sort_matches_workspace_sort_twice():
    dev = torch.device("cuda:0")
    rng = np.random.default_rng(77)
    # (S, T, nb): both long enough to be cut into chunks (the path that uses the scratch array);
    # the second call is smaller and leaves most of the first call's counters in the array
    for S, T, nb in ((3, 20000, 16), (2, 9001, 5)):
        bucket = torch.from_numpy(rng.integers(0, nb, size=(S, T), dtype=np.int32)).to(dev)
        ref = _raw_sort_ws(bucket, nb)
        assert ref[4] > 0, "the case must use the chunked sort"
        got = _raw_sort_static(bucket, nb)
        torch.cuda.synchronize()
        for name, a, b in zip(("idx", "bucket_sorted", "bucket_off", "sort_key"), ref[:4], got):
            assert torch.equal(a, b), f"{name} differs at S={S} T={T} nb={nb}"
        # and against the definition: a stable sort of the positions by bucket id
        order = np.argsort(bucket.cpu().numpy(), axis=1, kind="stable").astype(np.int32)
        assert np.array_equal(got[0].cpu().numpy(), order)


def test_static_scratch_sort_rejects_what_does_not_fit():
    L = sc.lib()
    one = ctypes.c_void_p(256)   # never dereferenced: the size check fails first
    # 65 segments x 4 chunks x 256 buckets x 4 bytes > 256 KiB
    assert int(L.scfa_sort_workspace_bytes(65, 16384, 256)) > 256 * 1024
    assert L.scfa_sort_by_bucket_static(one, 65, 16384, 256, one, one, one, None, None) == sc.SCFA_EWORKSPACE
    assert L.scfa_sort_by_bucket_static(None, 1, 8, 2, None, None, None, None, None) == sc.SCFA_EINVAL
