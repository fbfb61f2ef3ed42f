"""The cache test for callers that cannot allocate: cdf_cache_filter_static keeps its scratch in a
static device array of the library. Its results must equal cdf_cache_filter's (and the oracle's)
bit for bit, on two calls in a row that share the array, the second on a smaller input."""
import ctypes

import numpy as np
import pytest
import torch

pytestmark = pytest.mark.gpu
DEV = "cuda:0"


def make_rows(R, F, dtype, seed):
    g = torch.Generator().manual_seed(seed)
    cached = torch.randn(R, F, generator=g)
    rate = torch.rand(R, 1, generator=g) * 0.08
    cur = cached * (1 + rate * torch.randn(R, F, generator=g))
    same = torch.rand(R, generator=g) < 0.3
    cur[same] = cached[same]
    cached[torch.rand(R, generator=g) < 0.05] = 0
    return cur.to(dtype), cached.to(dtype)


def to_np(t):
    t = t.detach().cpu()
    if t.dtype == torch.bfloat16:
        return t.view(torch.int16).numpy().view(np.uint16).copy()
    return t.numpy().copy()


@pytest.mark.parametrize("dtype,norm", [(torch.float32, 0), (torch.bfloat16, 0), (torch.float32, 1)])
def test_static_scratch_filter_equals_the_workspace_one(oracle, dtype, norm):
    import paper_2408_00232_amd as cdf
    cdf.binding.load()
    assert torch.cuda.is_available()
    # the first call spans several thousand blocks of counts (a vector pass of the scan and a ragged
    # rest); the second is smaller, so stale counts of the first call sit right behind what it uses
    for call, (R, F) in enumerate([(64 * 8192 + 64 * 37 + 11, 8), (3001, 100)]):
        cur, cached = make_rows(R, F, dtype, seed=100 * call + norm)
        dcur, dcached = cur.to(DEV), cached.to(DEV)
        outs = []
        for static in (True, False):
            mask = torch.full((R,), 7, dtype=torch.uint8, device=DEV)
            idx = torch.full((R,), -1, dtype=torch.int32, device=DEV)
            n_sent = torch.full((1,), -1, dtype=torch.int32, device=DEV)
            if static:
                cdf.cdf_cache_filter_static(dcur, dcached, 0.05, norm, mask, idx, n_sent)
            else:
                ws = torch.zeros(cdf.cdf_workspace_bytes(R, F, 1), dtype=torch.uint8, device=DEV)
                cdf.cdf_cache_filter(dcur, dcached, 0.05, norm, mask, idx, n_sent, ws)
            torch.cuda.synchronize()
            outs.append((int(n_sent.item()), to_np(mask), to_np(idx)))
        (n_s, mask_s, idx_s), (n_w, mask_w, idx_w) = outs
        assert 0 < n_w < R and n_s == n_w
        np.testing.assert_array_equal(mask_s, mask_w)
        np.testing.assert_array_equal(idx_s[:n_s], idx_w[:n_w])
        assert (idx_s[n_s:] == -1).all()                     # nothing written past the count
        omask, oidx = oracle.cache_filter(to_np(cur), to_np(cached), 0.05, norm)
        np.testing.assert_array_equal(mask_s, omask)
        np.testing.assert_array_equal(idx_s[:n_s], oidx)


def test_static_scratch_filter_limits():
    import paper_2408_00232_amd as cdf
    lib = cdf.binding.load()
    n = torch.full((1,), -1, dtype=torch.int32, device=DEV)
    # empty input: the count is defined, nothing else is touched
    e = torch.zeros(0, 16, device=DEV)
    cdf.cdf_cache_filter_static(e, e, 0.1, 0, None, None, n)
    torch.cuda.synchronize()
    assert int(n.item()) == 0
    # beyond the static array: refused on the host, nothing launched
    rc = lib.cdf_cache_filter_static(None, None, ctypes.c_int32((8 << 20) + 1), ctypes.c_int32(4), ctypes.c_int64(4),
                                     0, ctypes.c_float(0.1), 0, None, None, ctypes.c_void_p(n.data_ptr()), None)
    assert rc == cdf.ERR_UNSUPPORTED and b"static scratch" in lib.cdf_last_error()
