"""The benchmark's own workload at full size (2^30 elements, 1,024-element blocks; f32, its
bf16 copy, and f32 with a bf16 checkpoint), through the same entry points and launch
configuration as bench.py.

The whole store is brought to the host and the oracle (OpenMP over blocks) runs the whole
cycle on it: every one of the 1,048,576 scores is compared, the selection is checked by both
rules (exactly the oracle's choice on the GPU's own scores; against the oracle's float64
scores within the band around its k-th score), and after the commit and after the recovery
every byte of c and of x is compared with the oracle's host mirrors.  The by-layer variant of
the store (96 tensors) is treated the same way."""
import numpy as np
import pytest
import torch

import oracle
from paper_1810_07354_amd import scar
from paper_1810_07354_amd import workloads as wl
from gpu_util import (DEV, REL_TOL, assert_norm_matches, assert_scores_match, assert_selection_matches,
                      idx_dev, idx_host, to_host)

pytestmark = pytest.mark.gpu

N_ELEMS, L = 1 << 30, 1024
NB = N_ELEMS // L
ORACLE_THREADS = 16


def same_bits(t: torch.Tensor, host: np.ndarray) -> bool:
    """Device tensor against a host mirror, bit for bit, a slab at a time (bfloat16 as uint16)."""
    step = 1 << 28
    for lo in range(0, t.numel(), step):
        if not np.array_equal(to_host(t[lo:lo + step]), host[lo:lo + step]):
            return False
    return True


@pytest.mark.parametrize("dtype", [wl.F32, wl.BF16, wl.F32_BF16C])
def test_flat_store_full_size(dtype):
    print("full size dtype=%d: generate" % dtype, flush=True)
    x, c = wl.flat_like_torch(DEV, seed=4, n_elems=N_ELEMS)
    if dtype == wl.BF16:
        x, c = x.to(torch.bfloat16), c.to(torch.bfloat16)
    elif dtype == wl.F32_BF16C:
        c = c.to(torch.bfloat16)
    k, n_lost = wl.k_of_fraction(0.10, NB), NB // 8
    ws = scar.new_workspace(NB, DEV)
    hx, hc = to_host(x), to_host(c)
    score_kind = wl.F32          # float scores whatever the store holds
    oracle.set_num_threads(ORACLE_THREADS)
    try:
        # ---- scores: every block against the oracle
        print("scores", flush=True)
        s = scar.block_scores(x, c, L)
        s_ref = oracle.block_scores(dtype, hx, hc, L)
        assert_scores_match(s, s_ref, score_kind)
        s_h = s.cpu().numpy()
        # sum of all scores = squared norm of a full recovery (Appendix A.3), both from the oracle
        full_ref = oracle.perturbation_norm(dtype, hx, hc, L)
        assert abs(s_ref.sum() - full_ref[0]) <= 1e-9 * full_ref[0]
        full = scar.read_norm(scar.perturbation_norm(x, c, L, None, ws))
        assert_norm_matches(full, full_ref, score_kind)

        # ---- selection: both rules on all 2^20 keys
        print("select", flush=True)
        idx = scar.select_topk(s, k, ws)
        idx_h = idx_host(idx)
        assert_selection_matches(idx_h, s_h, s_ref, k)

        # ---- commit: the oracle advances its mirror, every byte of c and x compared
        print("commit", flush=True)
        scar.checkpoint_commit(x, c, L, idx)
        oracle.checkpoint_commit(dtype, hx, hc, L, idx_h)
        assert same_bits(c, hc), "c differs from the oracle's mirror after the commit"
        assert same_bits(x, hx), "the commit changed x"

        # ---- partial recovery with the fused norm
        print("recover", flush=True)
        lost = wl.random_lost_blocks(NB, n_lost, 4 + 1000)
        got = scar.read_norm(scar.partial_recover(x, c, L, idx_dev(lost), ws))
        want = oracle.partial_recover(dtype, hx, hc, L, lost)
        assert_norm_matches(got, want, score_kind)
        assert got[1] <= full[1] * (1 + REL_TOL)                      # Theorem 4.1
        assert same_bits(x, hx), "x differs from the oracle's mirror after the recovery"
        assert same_bits(c, hc), "the recovery changed c"
    finally:
        oracle.set_num_threads(1)


@pytest.mark.parametrize("log2_elems", [26, 27])
def test_scores_in_the_occupancy_limited_launch(log2_elems):
    """2^26 and 2^27 float32 elements in 1,024-element blocks: 65,536 / 131,072 workgroup-sized
    launches, the size from which the score scan limits its workgroups per compute unit - the
    launch the benchmark's store uses - with every score compared with the oracle."""
    n = 1 << log2_elems
    print("occupancy-limited scores n=2^%d" % log2_elems, flush=True)
    x, c = wl.flat_like_torch(DEV, seed=40 + log2_elems, n_elems=n)
    hx, hc = to_host(x), to_host(c)
    oracle.set_num_threads(ORACLE_THREADS)
    try:
        for dtype in (wl.F32, wl.BF16, wl.F32_BF16C):
            if dtype == wl.BF16:
                xd, cd = x.to(torch.bfloat16), c.to(torch.bfloat16)
            elif dtype == wl.F32_BF16C:
                xd, cd = x, c.to(torch.bfloat16)
            else:
                xd, cd = x, c
            for bl in (512, 1024, 2048):
                s = scar.block_scores(xd, cd, bl)
                s_ref = oracle.block_scores(dtype, to_host(xd) if dtype == wl.BF16 else hx,
                                            to_host(cd) if dtype != wl.F32 else hc, bl)
                assert_scores_match(s, s_ref, wl.F32)
    finally:
        oracle.set_num_threads(1)


def test_by_layer_store_full_size():
    """The by-layer benchmark workload (2^30 f32 in 96 tensors of very unequal length) through
    the variable-length entry points; here the oracle runs the whole cycle on the full store."""
    print("by-layer full size: generate", flush=True)
    sizes = wl.mixed_layer_sizes(96, N_ELEMS, seed=6)
    sizes[np.argmax(sizes)] += N_ELEMS - sizes.sum()
    off_h = np.concatenate([[0], np.cumsum(sizes)]).astype(np.uint64)
    nb = sizes.size
    x, c = wl.flat_like_torch(DEV, seed=4, n_elems=N_ELEMS)
    for j in range(3):
        wl.drift_torch(x, 7000 + j, 0.10, 1024)
    off = torch.from_numpy(off_h.astype(np.int64)).to(DEV)
    k = wl.k_of_fraction(0.10, nb)
    lost = wl.random_lost_blocks(nb, 12, 4 + 1000)
    ws, ws_sel = scar.new_var_workspace(nb, DEV), scar.new_workspace(nb, DEV)
    hx, hc = x.cpu().numpy(), c.cpu().numpy()
    oracle.set_num_threads(8)
    try:
        print("scores", flush=True)
        s = scar.var_block_scores(x, c, off, ws)
        s_ref = oracle.var_block_scores(wl.F32, hx, hc, off_h)
        s_h = s.cpu().numpy()
        np.testing.assert_allclose(s_h.astype(np.float64), s_ref, rtol=REL_TOL, atol=0)

        print("select", flush=True)
        idx = scar.select_topk(s, k, ws_sel)
        idx_h = idx_host(idx)
        np.testing.assert_array_equal(idx_h, oracle.select_topk(s_h.astype(np.float64), k))

        print("commit", flush=True)
        scar.var_checkpoint_commit(x, c, off, idx, ws)
        oracle.var_checkpoint_commit(wl.F32, hx, hc, off_h, idx_h)
        assert torch.equal(c.cpu(), torch.from_numpy(hc))
        assert torch.equal(x.cpu(), torch.from_numpy(hx))

        print("recover", flush=True)
        full = scar.read_norm(scar.var_perturbation_norm(x, c, off, None, ws))
        want_full = oracle.var_perturbation_norm(wl.F32, hx, hc, off_h)
        assert abs(full[1] - want_full[1]) <= REL_TOL * want_full[1]
        got = scar.read_norm(scar.var_partial_recover(x, c, off, idx_dev(lost), ws))
        want = oracle.var_partial_recover(wl.F32, hx, hc, off_h, lost)
        assert abs(got[0] - want[0]) <= REL_TOL * want[0]
        assert abs(got[1] - want[1]) <= REL_TOL * want[1]
        assert got[1] <= full[1] * (1 + REL_TOL)                      # Theorem 4.1
        assert torch.equal(x.cpu(), torch.from_numpy(hx))
        assert torch.equal(c.cpu(), torch.from_numpy(hc))
    finally:
        oracle.set_num_threads(1)
