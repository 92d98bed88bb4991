"""The benchmark's own workload at full size (2^30 elements, 1,024-element blocks, f32 and
its bf16 copy), through the same entry points and launch configuration as bench.py.

The oracle cannot run 2 x 4 GiB in seconds, so it checks what it can compute one by one -
the scores of ~1,000 sampled blocks, the whole top-k on the GPU's scores (1M keys), the
commit on the sampled blocks, the norm over all 131,072 lost blocks - and properties that
hold at any size cover the rest (every byte outside K / S unchanged, every byte inside
copied, sum of scores = squared full-recovery norm).  The by-layer variant of the store has
only 96 blocks, so there the oracle runs the whole cycle on the full host copy."""
import numpy as np
import pytest
import torch

import oracle
from paper_1810_07354_amd import scar
from paper_1810_07354_amd import workloads as wl
from gpu_util import DEV, REL_TOL, idx_dev, idx_host, to_host

pytestmark = pytest.mark.gpu

N_ELEMS, L = 1 << 30, 1024
NB = N_ELEMS // L


def rows_to_host(t, rows):
    """Blocks `rows` of device store t as one contiguous host store (bf16 as uint16 bits)."""
    sel = t.view(NB, L)[torch.from_numpy(rows.astype(np.int64)).to(DEV)].contiguous()
    return to_host(sel).reshape(-1)


def bits(t):
    """A view that torch.equal compares bit for bit (bfloat16 as int16)."""
    return t.view(torch.int16) if t.dtype == torch.bfloat16 else t


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
    oracle.set_num_threads(8)
    try:
        # ---- scores: sampled blocks through the oracle
        print("scores", flush=True)
        s = scar.block_scores(x, c, L)
        r = np.random.default_rng(11)
        sample = np.unique(np.concatenate([r.choice(NB, size=1024, replace=False), [0, 1, NB - 2, NB - 1]]))
        ref = oracle.block_scores(dtype, rows_to_host(x, sample), rows_to_host(c, sample), L)
        s_h = s.cpu().numpy()
        np.testing.assert_allclose(s_h[sample].astype(np.float64), ref, rtol=REL_TOL, atol=0)
        # sum of all scores = squared norm of a full recovery (Appendix A.3)
        full = scar.read_norm(scar.perturbation_norm(x, c, L, None, ws))
        assert abs(s_h.astype(np.float64).sum() - full[0]) <= REL_TOL * full[0]

        # ---- selection: the whole top-k on the GPU's own scores
        print("select", flush=True)
        idx = scar.select_topk(s, k, ws)
        idx_h = idx_host(idx)
        np.testing.assert_array_equal(idx_h, oracle.select_topk(s_h.astype(np.float64), k))

        # ---- commit: sampled blocks through the oracle, everything else by property
        print("commit", flush=True)
        c_before = c.clone()
        scar.checkpoint_commit(x, c, L, idx)
        chosen = np.zeros(NB, dtype=bool)
        chosen[idx_h] = True
        sub_x, sub_c = rows_to_host(x, sample), rows_to_host(c_before, sample)
        oracle.checkpoint_commit(dtype, sub_x, sub_c, L, np.nonzero(chosen[sample])[0].astype(np.uint32))
        np.testing.assert_array_equal(rows_to_host(c, sample), sub_c)
        expect = c_before
        idx_l = idx.long()
        expect.view(NB, L)[idx_l] = x.view(NB, L)[idx_l].to(c.dtype)     # torch rounds to nearest even too
        assert torch.equal(bits(c), bits(expect))
        del expect, c_before

        # ---- partial recovery with the fused norm: the norm over all lost blocks by the oracle
        print("recover", flush=True)
        lost = wl.random_lost_blocks(NB, n_lost, 4 + 1000)
        lost_d = idx_dev(lost)
        hx, hc = rows_to_host(x, lost), rows_to_host(c, lost)
        want = oracle.perturbation_norm(dtype, hx, hc, L)
        x_before = x.clone()
        got = scar.read_norm(scar.partial_recover(x, c, L, lost_d, ws))
        assert abs(got[0] - want[0]) <= REL_TOL * want[0]
        assert abs(got[1] - want[1]) <= REL_TOL * want[1]
        assert got[1] <= full[1] * (1 + REL_TOL)                      # Theorem 4.1 (after the commit the
        lost_l = lost_d.long()                                         # full norm only shrank, so compare
        x_before.view(NB, L)[lost_l] = c.view(NB, L)[lost_l].to(x.dtype)   # with the pre-commit one)
        assert torch.equal(bits(x), bits(x_before))
        if dtype != wl.F32_BF16C:
            np.testing.assert_array_equal(rows_to_host(x, lost[:256]), hc[:256 * L])
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
