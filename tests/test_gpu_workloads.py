"""Whole checkpoint / failure / recovery cycles on the synthetic MLR-, MF-, LDA-, CNN-like
stores and the flat store, GPU against the oracle after every call, three cycles with the
store drifting in between (the running checkpoint holds a mix of ages, Section 4.2)."""
import numpy as np
import pytest
import torch

import oracle
from paper_1810_07354_amd import scar
from paper_1810_07354_amd import workloads as wl
from gpu_util import (DEV, REL_TOL, DeviceStore, assert_norm_matches, assert_scores_match,
                      assert_selection_matches, idx_dev, idx_host, to_dev, to_host)

pytestmark = pytest.mark.gpu


def drift(store: DeviceStore, seed: int):
    """Untimed stand-in for training between checkpoints: move a random tenth of the store."""
    r = np.random.default_rng(seed)
    n = store.hx.size
    lo = int(r.integers(0, n - n // 10))
    hi = lo + n // 10
    if store.dtype == wl.I32:
        store.hx[lo:hi] += r.integers(-2, 3, size=hi - lo).astype(np.int32)
    elif store.dtype == wl.BF16:
        f = wl.bf16_bits_to_f32(store.hx[lo:hi]) + r.normal(0, 1e-3, size=hi - lo).astype(np.float32)
        store.hx[lo:hi] = wl.f32_to_bf16_bits(f)
    else:
        store.hx[lo:hi] += r.normal(0, 1e-3, size=hi - lo).astype(np.float32)
    store.x = to_dev(store.hx, store.dtype)


def three_cycles(w: wl.Workload, staging=False):
    s = DeviceStore(w)
    for cyc in range(3):
        print("%s cycle %d" % (w.name, cyc), flush=True)
        lost = w.lost if cyc == 0 else wl.random_lost_blocks(w.n_blocks, w.lost.size, 50 + cyc)
        s.cycle(w.k, lost, staging=staging and cyc == 0)
        drift(s, 900 + cyc)


def test_mlr_like_full_size():
    three_cycles(wl.mlr_like(), staging=True)


def test_mf_like_full_size():
    three_cycles(wl.mf_like())


def test_lda_like_quarter_size():
    three_cycles(wl.lda_like(words=25_000, topics=1000))


def test_lda_like_full_size_one_cycle():
    w = wl.lda_like()
    print("lda full size generated", flush=True)
    oracle.set_num_threads(8)
    try:
        DeviceStore(w).cycle(w.k, w.lost)
    finally:
        oracle.set_num_threads(1)


@pytest.mark.parametrize("fraction", [0.01, 0.10, 0.50])
def test_cnn_like_full_size(fraction):
    three_cycles(wl.cnn_like(fraction=fraction))


@pytest.mark.parametrize("dtype", [wl.F32, wl.BF16])
def test_flat_like_16m(dtype):
    three_cycles(wl.flat_like(n_elems=1 << 24, dtype=dtype))


def test_priority_beats_round_robin_and_random_on_the_norm():
    # Saving the most-changed blocks leaves a smaller full-recovery perturbation than
    # saving the same number of blocks chosen round-robin or at random (Section 5.4).
    w = wl.cnn_like(n_elems=4_000_000)
    nb, k, L = w.n_blocks, w.k, w.block_len
    x = to_dev(w.x, w.dtype)
    ws = scar.new_workspace(nb, DEV)
    res = {}
    picks = {"priority": None,
             "round": np.arange(k, dtype=np.uint32),
             "random": np.sort(np.random.default_rng(1).choice(nb, size=k, replace=False)).astype(np.uint32)}
    for name, idx in picks.items():
        c = to_dev(w.c, w.dtype)
        if idx is None:
            d_idx = scar.select_topk(scar.block_scores(x, c, L), k, ws)
        else:
            d_idx = idx_dev(idx)
        scar.checkpoint_commit(x, c, L, d_idx)
        res[name] = scar.read_norm(scar.perturbation_norm(x, c, L, None, ws))[1]
    assert res["priority"] < res["round"] and res["priority"] < res["random"]


def test_strategy_study_orders_the_strategies_as_the_paper_does():
    # Section 5.4 / Fig. 8: at the same write volume, prioritized partial checkpoints leave a
    # smaller perturbation than round-robin or random ones, and partial recovery a smaller one
    # than full recovery (Theorem 4.1; about sqrt(1/2) of it for half the blocks, Theorem 4.2).
    from paper_1810_07354_amd import strategy_study
    r = strategy_study.run(n_blocks=4096, block_len=256, iters=24, period=8, lost_fraction=0.5)
    m = r["mean_perturbation_norm"]
    print(r, flush=True)
    assert m["priority"] < m["round"] and m["priority"] < m["random"]
    assert m["partial"] < m["traditional"]
    assert 0.6 < m["partial"] / m["traditional"] < 0.8
    assert m["priority"] < m["partial"]


def test_iteration_cost_demo_reproduces_the_papers_ordering():
    # Figs. 7 and 8 on a synthetic contracting job: partial recovery costs fewer iterations
    # than full recovery, prioritized partial checkpoints fewer still, and a full checkpoint
    # every C iterations with full recovery costs about C/2 iterations per failure.
    from paper_1810_07354_amd import iteration_cost_demo
    r = iteration_cost_demo.run(n_blocks=1024, block_len=256, interval=32, fraction=0.125,
                                lost_fraction=0.5, trials=8)
    print(r, flush=True)
    cost = r["mean_iteration_cost"]
    assert all(v >= 0 for v in cost.values())
    assert 4 <= cost["traditional"] <= 32
    assert cost["partial"] <= cost["traditional"]
    assert cost["priority"] < cost["partial"] and cost["priority"] < cost["round"]
    for name, b in r["theorem_3_1_bound_at_mean"].items():
        assert cost[name] <= b + 1, name
