"""The allocation-free count of correct predictions (slp_count_correct_static) against the entry point it is a variant
of (slp_count_correct) and against the oracle, through the C ABI: two calls in a row, the second on a smaller input,
then the limit and an accumulate call.  Nothing may pass through the caching allocator during the calls (the HIP
runtime's own lazy loading of the library's code object on a first launch is not the library's doing and is not
measured)."""

import ctypes

import numpy as np
import pytest
import torch

from oracle import segment as osg
from paper_2403_11204_amd import api

pytestmark = pytest.mark.gpu
DEV = "cuda"


def make_case(batch, classes, dtype, seed):
    g = np.random.default_rng(seed)
    Z = (g.integers(-8, 9, size=(batch, classes)) / 4.0).astype(np.float32)       # coarse grid: equal maxima occur
    y = g.integers(0, classes, batch).astype(np.int32)
    y[: batch // 2] = np.argmax(Z[: batch // 2], axis=1)
    t = torch.from_numpy(Z).to(DEV)
    t = (t.to(torch.bfloat16) if dtype == api.BF16 else t).contiguous()
    return t, torch.from_numpy(y).to(DEV), osg.count_correct(t.float().cpu().numpy(), y)


@pytest.mark.parametrize("dtype", [api.F32, api.BF16])
def test_static_count_equals_the_caller_scratch_count(dtype):
    L = api.lib()
    big = make_case(65536, 47, dtype, 1)        # the limit: every entry of the static array is used
    small = make_case(1410, 47, dtype, 2)       # then a smaller input: stale partial counts must not be read
    out_s = torch.full((1,), -1, dtype=torch.int64, device=DEV)
    out_r = torch.full((1,), -1, dtype=torch.int64, device=DEV)
    scratch = torch.empty(65536 // 4, dtype=torch.int32, device=DEV)
    torch.cuda.synchronize()
    reserved = torch.cuda.memory_reserved()
    st = ctypes.c_void_p(torch.cuda.current_stream().cuda_stream)
    for Z, y, ref in (big, small):
        B, C = Z.shape
        rc = L.slp_count_correct_static(api._ptr(Z), api._ptr(y), B, C, dtype, 0, api._ptr(out_s), st)
        assert rc == 0, L.slp_last_error()
        rc = L.slp_count_correct(api._ptr(Z), api._ptr(y), B, C, dtype, api._ptr(scratch), scratch.numel() * 4, 0, api._ptr(out_r), st)
        assert rc == 0, L.slp_last_error()
        assert int(out_s.item()) == int(out_r.item()) == ref and 0 < ref < B
    # accumulate on top of the last count
    Z, y, ref = small
    assert L.slp_count_correct_static(api._ptr(Z), api._ptr(y), Z.shape[0], Z.shape[1], dtype, 1, api._ptr(out_s), st) == 0
    assert int(out_s.item()) == 2 * ref
    torch.cuda.synchronize()
    assert torch.cuda.memory_reserved() == reserved                 # nothing went through torch's allocator
    # beyond the limit: refused on the host, nothing launched
    Zb = torch.zeros((65537, 2), dtype=Z.dtype, device=DEV)
    yb = torch.zeros(65537, dtype=torch.int32, device=DEV)
    assert L.slp_count_correct_static(api._ptr(Zb), api._ptr(yb), 65537, 2, dtype, 0, api._ptr(out_s), st) == -2
    assert b"limit" in L.slp_last_error()
    assert int(out_s.item()) == 2 * ref
