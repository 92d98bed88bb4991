"""Document-length-scaled total variation (Section 5.1 "LDA", Appendix C) on the GPU against
the oracle: per-block distances, the norm alone, the norm fused into a partial recovery, and a
whole prioritized checkpoint + recovery cycle on document-topic rows."""
import numpy as np
import pytest
import torch

import oracle
from paper_1810_07354_amd import scar
from paper_1810_07354_amd import workloads as wl
from gpu_util import (DEV, REL_TOL, assert_selection_matches, idx_dev, idx_host, to_dev, to_host)

pytestmark = pytest.mark.gpu
F32, BF16 = wl.F32, wl.BF16


def rows(dtype, nb, L, seed, ragged=True):
    r = np.random.default_rng(seed)
    n = nb * L - (L // 3 if ragged else 0)
    c = r.dirichlet(np.full(L, 0.3), size=nb).astype(np.float32).ravel()[:n]
    x = np.where(r.random(n) < 0.3, c + r.normal(0, 0.01, size=n).astype(np.float32), c).astype(np.float32)
    if dtype == BF16:
        x, c = wl.f32_to_bf16_bits(x), wl.f32_to_bf16_bits(c)
    return x, c


def close(got, want):
    np.testing.assert_allclose(np.asarray(got, dtype=np.float64), want, rtol=REL_TOL, atol=0)


def norm_close(got, want):
    assert got[2] == 0 and want[2] == 0
    assert abs(got[0] - want[0]) <= REL_TOL * max(want[0], 1e-300)
    assert abs(got[1] - want[1]) <= REL_TOL * max(want[1], 1e-300)
    assert got[0] == got[1]


@pytest.mark.parametrize("dtype", [F32, BF16])
@pytest.mark.parametrize("L", [1, 5, 37, 100, 256, 1000, 4096, 5000])
@pytest.mark.parametrize("weighted", [False, True])
def test_tv_calls(dtype, L, weighted):
    nb = 300 if L < 2000 else 50
    hx, hc = rows(dtype, nb, L, seed=L + dtype)
    nbk = oracle.n_blocks_of(hx.size, L)
    r = np.random.default_rng(L)
    hw = r.integers(5, 3000, size=nbk).astype(np.float32) if weighted else None
    w = torch.from_numpy(hw).to(DEV) if weighted else None
    print("tv dtype=%d L=%d weighted=%s" % (dtype, L, weighted), flush=True)
    x, c = to_dev(hx, dtype), to_dev(hc, dtype)
    ws = scar.new_workspace(nbk, DEV)
    s = scar.tv_block_scores(x, c, L, w)
    close(s.cpu().numpy(), oracle.tv_block_scores(dtype, hx, hc, L, hw))
    full = scar.read_norm(scar.tv_perturbation_norm(x, c, L, None, ws, w))
    norm_close(full, oracle.tv_perturbation_norm(dtype, hx, hc, L, hw))
    S = np.unique(np.append(r.permutation(nbk)[: nbk // 2], nbk - 1)).astype(np.uint32)
    r.shuffle(S)
    pre = scar.read_norm(scar.tv_perturbation_norm(x, c, L, idx_dev(S), ws, w))
    got = scar.read_norm(scar.tv_partial_recover(x, c, L, idx_dev(S), ws, w))
    want = oracle.tv_partial_recover(dtype, hx, hc, L, S, hw)
    norm_close(got, want)
    assert pre == got
    assert got[1] <= full[1] * (1 + REL_TOL)
    np.testing.assert_array_equal(to_host(x), hx)
    np.testing.assert_array_equal(to_host(c), hc)
    assert scar.read_norm(scar.tv_partial_recover(x, c, L, idx_dev(S), ws, w)) == (0.0, 0.0, 0)
    empty = torch.zeros(0, dtype=torch.int32, device=DEV)
    assert scar.read_norm(scar.tv_perturbation_norm(x, c, L, empty, ws, w)) == (0.0, 0.0, 0)


@pytest.mark.parametrize("dtype", [F32, BF16])
@pytest.mark.parametrize("row_bytes", [16, 80, 400, 512, 20, 36, 100, 404, 2004])
@pytest.mark.parametrize("weighted", [False, True])
def test_tv_scores_of_many_short_rows(dtype, row_bytes, weighted):
    # enough rows of 16 ... 512 bytes for the scan that reads whole runs of rows; last row short
    L = row_bytes // (2 if dtype == BF16 else 4)
    nb = 9001
    hx, hc = rows(dtype, nb, L, seed=row_bytes + dtype)
    assert oracle.n_blocks_of(hx.size, L) == nb
    hw = np.random.default_rng(L).integers(5, 3000, size=nb).astype(np.float32) if weighted else None
    w = torch.from_numpy(hw).to(DEV) if weighted else None
    print("tv short rows dtype=%d L=%d weighted=%s" % (dtype, L, weighted), flush=True)
    s = scar.tv_block_scores(to_dev(hx, dtype), to_dev(hc, dtype), L, w)
    close(s.cpu().numpy(), oracle.tv_block_scores(dtype, hx, hc, L, hw))


def test_tv_unaligned_bases():
    L, nb = 37, 400
    hx, hc = rows(F32, nb, L, seed=3)
    hx, hc = np.concatenate([[0], hx]).astype(np.float32), np.concatenate([[0], hc]).astype(np.float32)
    x, c = to_dev(hx, F32)[1:], to_dev(hc, F32)[1:]
    hw = np.arange(1, oracle.n_blocks_of(hx.size - 1, L) + 1, dtype=np.float32)
    s = scar.tv_block_scores(x, c, L, torch.from_numpy(hw).to(DEV))
    close(s.cpu().numpy(), oracle.tv_block_scores(F32, hx[1:].copy(), hc[1:].copy(), L, hw))


@pytest.mark.parametrize("dtype", [F32, BF16])
def test_tv_cycle_on_document_topic_rows(dtype):
    # prioritized checkpoint of the documents that moved furthest in scaled total variation,
    # then loss and recovery of a quarter of them
    w = wl.doc_topic_like(docs=6000, topics=100, dtype=dtype)
    L, hw = w.block_len, w.extra["lengths"]
    hx, hc = w.x.copy(), w.c.copy()
    x, c, dw = to_dev(hx, dtype), to_dev(hc, dtype), torch.from_numpy(hw).to(DEV)
    ws = scar.new_workspace(w.n_blocks, DEV)
    s = scar.tv_block_scores(x, c, L, dw)
    s_ref = oracle.tv_block_scores(dtype, hx, hc, L, hw)
    close(s.cpu().numpy(), s_ref)
    idx = scar.select_topk(s, w.k, ws)
    assert_selection_matches(idx_host(idx), s.cpu().numpy(), s_ref, w.k)
    before = scar.read_norm(scar.tv_perturbation_norm(x, c, L, None, ws, dw))
    scar.checkpoint_commit(x, c, L, idx)
    oracle.checkpoint_commit(dtype, hx, hc, L, idx_host(idx))
    np.testing.assert_array_equal(to_host(c), hc)
    after = scar.read_norm(scar.tv_perturbation_norm(x, c, L, None, ws, dw))
    norm_close(after, oracle.tv_perturbation_norm(dtype, hx, hc, L, hw))
    # the commit removed exactly the chosen documents' distances from the whole-store norm
    assert abs((before[0] - after[0]) - s_ref[idx_host(idx)].sum()) <= 10 * REL_TOL * before[0]
    got = scar.read_norm(scar.tv_partial_recover(x, c, L, idx_dev(w.lost), ws, dw))
    norm_close(got, oracle.tv_partial_recover(dtype, hx, hc, L, w.lost, hw))
    np.testing.assert_array_equal(to_host(x), hx)


def test_tv_argument_errors():
    x = torch.zeros(64, dtype=torch.int32, device=DEV)
    with pytest.raises(scar.ScarError):
        scar.tv_block_scores(x, x.clone(), 8)
    xf = torch.zeros(64, device=DEV)
    with pytest.raises(ValueError):
        scar.tv_block_scores(xf, xf.clone(), 8, torch.ones(3, device=DEV))
    with pytest.raises(scar.ScarError):
        scar.tv_block_scores(xf, xf.clone().to(torch.bfloat16), 8)


def test_tv_large_store_and_long_lists():
    # 400,000 documents x 64 topics: the wide-workgroup recovery launch in this norm
    nb, L = 400_000, 64
    hx, hc = rows(F32, nb, L, seed=9, ragged=False)
    hw = np.random.default_rng(1).integers(5, 3000, size=nb).astype(np.float32)
    x, c, w = to_dev(hx, F32), to_dev(hc, F32), torch.from_numpy(hw).to(DEV)
    ws = scar.new_workspace(nb, DEV)
    oracle.set_num_threads(8)
    try:
        close(scar.tv_block_scores(x, c, L, w).cpu().numpy(), oracle.tv_block_scores(F32, hx, hc, L, hw))
        S = np.random.default_rng(2).permutation(nb)[: (3 * nb) // 4].astype(np.uint32)
        got = scar.read_norm(scar.tv_partial_recover(x, c, L, idx_dev(S), ws, w))
        norm_close(got, oracle.tv_partial_recover(F32, hx, hc, L, S, hw))
    finally:
        oracle.set_num_threads(1)
    np.testing.assert_array_equal(to_host(x), hx)


def test_tv_cycle_at_the_benchmark_size():
    # the total-variation workload of bench.py (2,000,000 documents x 100 topics, weighted) in
    # the benchmark's launch configuration: every score, the whole selection, the commit and
    # the recovery with its norm against the oracle on the full host copy
    import os
    import sys
    sys.path.insert(0, os.path.dirname(os.path.dirname(os.path.abspath(__file__))))
    import bench
    x, c, L, k, n_lost, lost_of, _drift, label, lengths = bench.make_doctopic(DEV)
    print(label, flush=True)
    nb = x.numel() // L
    hx, hc, hw = to_host(x), to_host(c), lengths.cpu().numpy()
    ws = scar.new_workspace(nb, DEV)
    oracle.set_num_threads(8)
    try:
        s = scar.tv_block_scores(x, c, L, lengths)
        s_ref = oracle.tv_block_scores(F32, hx, hc, L, hw)
        close(s.cpu().numpy(), s_ref)
        idx = scar.select_topk(s, k, ws)
        assert_selection_matches(idx_host(idx), s.cpu().numpy(), s_ref, k)
        scar.checkpoint_commit(x, c, L, idx)
        oracle.checkpoint_commit(F32, hx, hc, L, idx_host(idx))
        assert torch.equal(c, torch.from_numpy(hc).to(DEV))
        lost = lost_of(0)
        pre = scar.read_norm(scar.tv_perturbation_norm(x, c, L, idx_dev(lost), ws, lengths))
        got = scar.read_norm(scar.tv_partial_recover(x, c, L, idx_dev(lost), ws, lengths))
        norm_close(got, oracle.tv_partial_recover(F32, hx, hc, L, lost, hw))
        assert pre == got                                   # the norm alone, bit for bit
        assert torch.equal(x, torch.from_numpy(hx).to(DEV))
    finally:
        oracle.set_num_threads(1)


@pytest.mark.parametrize("seed", range(4))
def test_tv_random_layouts(seed):
    # seeded random stores (element type, row length, row count, weights or none, short last
    # row, x and c one element into their allocations or not) through the three calls
    r = np.random.default_rng(2000 + seed)
    for case in range(8):
        dtype = int(r.choice([F32, BF16]))
        L = int(np.exp(r.uniform(0, np.log(3000))))
        nb = int(np.exp(r.uniform(np.log(3), np.log(40_000))))
        nb = max(2, min(nb, 3_000_000 // L))
        hx, hc = rows(dtype, nb, L, seed=seed * 100 + case, ragged=bool(r.integers(0, 2)))
        nbk = oracle.n_blocks_of(hx.size, L)
        off = int(r.choice([0, 0, 1]))
        x = to_dev(np.concatenate([np.zeros(off, dtype=hx.dtype), hx]), dtype)[off:]
        c = to_dev(np.concatenate([np.zeros(off, dtype=hc.dtype), hc]), dtype)[off:]
        hw = r.integers(5, 3000, size=nbk).astype(np.float32) if r.random() < 0.7 else None
        w = torch.from_numpy(hw).to(DEV) if hw is not None else None
        print("tv random seed=%d case=%d dtype=%d L=%d nb=%d off=%d weighted=%s"
              % (seed, case, dtype, L, nbk, off, hw is not None), flush=True)
        ws = scar.new_workspace(nbk, DEV)
        close(scar.tv_block_scores(x, c, L, w).cpu().numpy(), oracle.tv_block_scores(dtype, hx, hc, L, hw))
        norm_close(scar.read_norm(scar.tv_perturbation_norm(x, c, L, None, ws, w)),
                   oracle.tv_perturbation_norm(dtype, hx, hc, L, hw))
        S = r.permutation(nbk)[: max(1, nbk // 3)].astype(np.uint32)
        pre = scar.read_norm(scar.tv_perturbation_norm(x, c, L, idx_dev(S), ws, w))
        got = scar.read_norm(scar.tv_partial_recover(x, c, L, idx_dev(S), ws, w))
        norm_close(got, oracle.tv_partial_recover(dtype, hx, hc, L, S, hw))
        assert pre == got
        np.testing.assert_array_equal(to_host(x.contiguous()), hx)


@pytest.mark.parametrize("dtype", [F32, BF16])
@pytest.mark.parametrize("case", ["short_rows", "mixed", "few_giant"])
@pytest.mark.parametrize("weighted", [False, True])
def test_tv_calls_on_rows_of_unequal_length(dtype, case, weighted):
    # the scaled total variation over blocks of unequal length (scar_var_tv_*): scores, the norm
    # of all blocks and of a list, recovery with the fused norm, and the selection on the scores
    r = np.random.default_rng(len(case) + dtype)
    if case == "short_rows":
        sizes = r.integers(0, 60, size=20_000)
    elif case == "mixed":
        sizes = wl.mixed_layer_sizes(300, 3_000_000, seed=31)
    else:
        sizes = np.array([5_000_000, 3, 0, 2_500_000, 700_001])
    off = np.concatenate([[0], np.cumsum(sizes)]).astype(np.uint64)
    nb, n = sizes.size, int(off[-1])
    c = r.random(n, dtype=np.float32)
    x = np.where(r.random(n) < 0.3, c + r.normal(0, 0.01, size=n).astype(np.float32), c).astype(np.float32)
    hx, hc = (wl.f32_to_bf16_bits(x), wl.f32_to_bf16_bits(c)) if dtype == BF16 else (x, c)
    hw = r.integers(5, 3000, size=nb).astype(np.float32) if weighted else None
    w = torch.from_numpy(hw).to(DEV) if weighted else None
    print("var tv dtype=%d case=%s weighted=%s blocks=%d elems=%d" % (dtype, case, weighted, nb, n), flush=True)
    xd, cd = to_dev(hx, dtype), to_dev(hc, dtype)
    d_off = torch.from_numpy(off.astype(np.int64)).to(DEV)
    ws, ws_sel = scar.new_var_workspace(nb, DEV), scar.new_workspace(nb, DEV)

    s = scar.var_tv_block_scores(xd, cd, d_off, ws, w)
    s_ref = oracle.var_tv_block_scores(dtype, hx, hc, off, hw)
    np.testing.assert_allclose(s.cpu().numpy().astype(np.float64), s_ref, rtol=REL_TOL, atol=0)
    k = max(1, nb // 5)
    idx = scar.select_topk(s, k, ws_sel)
    assert_selection_matches(idx_host(idx), s.cpu().numpy(), s_ref, k)

    full = scar.read_norm(scar.var_tv_perturbation_norm(xd, cd, d_off, None, ws, w))
    norm_close(full, oracle.var_tv_perturbation_norm(dtype, hx, hc, off, hw))
    S = np.sort(r.choice(nb, size=max(1, nb // 3), replace=False)).astype(np.uint32)
    pre = scar.read_norm(scar.var_tv_perturbation_norm(xd, cd, d_off, idx_dev(S), ws, w))
    got = scar.read_norm(scar.var_tv_partial_recover(xd, cd, d_off, idx_dev(S), ws, w))
    want = oracle.var_tv_partial_recover(dtype, hx, hc, off, S, hw)
    norm_close(got, want)
    norm_close(pre, want)
    assert got[1] <= full[1] * (1 + REL_TOL)
    np.testing.assert_array_equal(to_host(xd), hx)
    np.testing.assert_array_equal(to_host(cd), hc)
    # without a norm it is the plain recovery
    scar.var_tv_partial_recover(xd, cd, d_off, idx_dev(S), ws, w, want_norm=False)
    np.testing.assert_array_equal(to_host(xd), hx)
    # integer tables are scored by the plain calls (L1 = twice this norm): not built here
    xi = torch.zeros(8, dtype=torch.int32, device=DEV)
    with pytest.raises(scar.ScarError) as e:
        scar.var_tv_block_scores(xi, xi.clone(), torch.tensor([0, 8], device=DEV), ws)
    assert e.value.status == -5
