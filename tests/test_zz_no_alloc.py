"""scar_select_topk_static - the selection for callers that cannot allocate - against
scar_select_topk, index for index, on calls in a row that share the library's one scratch
array: a large input first (more than 2,048 tiles: the separate scan kernel), then smaller
ones, float and 64-bit integer keys, so that what an earlier call left in the array would
show if a later call relied on it."""
import ctypes

import numpy as np
import pytest
import torch

import oracle
from paper_1810_07354_amd import scar
from gpu_util import DEV, idx_host

pytestmark = pytest.mark.gpu


def keys(n, kind, seed):
    r = np.random.default_rng(seed)
    if kind == "f32":
        return torch.from_numpy(r.standard_gamma(0.5, size=n).astype(np.float32)).to(DEV)
    if kind == "f32_ties":
        return torch.from_numpy(r.integers(0, 50, size=n).astype(np.float32)).to(DEV)
    return torch.from_numpy(r.integers(0, 40, size=n, dtype=np.int64)).to(DEV)


def test_static_selection_equals_the_workspace_one_on_calls_in_a_row():
    cases = [(5_000_000, 1_234_567, "f32", 1), (300_000, 30_000, "f32", 2), (20_000, 19_999, "f32_ties", 3),
             (1_000_000, 100_000, "i64", 4), (100_000, 5_000, "i64", 5), (17_000, 1, "f32", 6),
             (4_300_000, 4_299_999, "f32_ties", 7), (16_385, 8_000, "i64", 8)]
    for n, k, kind, seed in cases:
        print("static select n=%d k=%d keys=%s" % (n, k, kind), flush=True)
        s = keys(n, kind, seed)
        want = scar.select_topk(s, k, scar.new_workspace(n, DEV))
        got = torch.full((k,), -1, dtype=torch.int32, device=DEV)
        scar.select_topk_static(s, k, out=got)
        torch.cuda.synchronize()
        assert torch.equal(got, want)
    # the smallest of them once more against the oracle itself
    s = keys(20_000, "f32_ties", 3)
    got = scar.select_topk_static(s, 777)
    np.testing.assert_array_equal(idx_host(got), oracle.select_topk(s.cpu().numpy().astype(np.float64), 777))


def test_static_selection_argument_errors():
    L_ = scar.lib()
    s = keys(100, "f32", 9)
    out = torch.empty(100, dtype=torch.int32, device=DEV)
    vp = ctypes.c_void_p
    st = vp(torch.cuda.current_stream().cuda_stream)
    too_many = scar.STATIC_MAX_BLOCKS + 1
    # beyond the fixed scratch: refused on the host (the pointers are never touched)
    assert L_.scar_select_topk_static(scar.SCORE_F32, vp(s.data_ptr()), too_many, 10, vp(out.data_ptr()), st) == -2
    assert L_.scar_select_topk_static(scar.SCORE_F32, vp(s.data_ptr()), 100, 101, vp(out.data_ptr()), st) == -1
    assert L_.scar_select_topk_static(7, vp(s.data_ptr()), 100, 10, vp(out.data_ptr()), st) == -1
    assert L_.scar_select_topk_static(scar.SCORE_F32, vp(0), 100, 10, vp(out.data_ptr()), st) == -1
    assert L_.scar_select_topk_static(scar.SCORE_F32, vp(s.data_ptr()), 100, 0, vp(0), st) == 0
    torch.cuda.synchronize()
