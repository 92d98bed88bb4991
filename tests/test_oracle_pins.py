"""Pins for the CPU oracle: it is checked against things other than itself - closed
forms, the identities the paper proves (Theorems 4.1 and 4.2, Appendix A.3/A.4),
brute force over all subsets on tiny inputs, special cases and a few values worked out
by hand - chosen so that a dropped term, a wrong sign, a shifted block boundary or a
swapped operand fails at least one of them.  CPU only.
"""
import itertools
import math

import numpy as np
import pytest

import oracle
from oracle import F32, BF16, I32


def rng_of(seed):
    return np.random.default_rng(seed)


# --------------------------------------------------------------------------- scores

@pytest.mark.parametrize("n_elems,L", [(40, 8), (45, 8), (7, 1), (5, 64), (1000, 100)])
def test_scores_closed_form_constant_offset_per_block(n_elems, L):
    # x = c + a_b with a_b a power of two: every difference is exact in fp32, so
    # s_b = (elements in block b) * a_b^2 exactly, short tail block included.
    nb = oracle.n_blocks_of(n_elems, L)
    c = rng_of(1).integers(-8, 8, size=n_elems).astype(np.float32)
    a = 2.0 ** rng_of(2).integers(-6, 6, size=nb)
    x = (c + np.repeat(a, L)[:n_elems]).astype(np.float32)
    s = oracle.block_scores(F32, x, c, L)
    lens = np.minimum(L, n_elems - np.arange(nb) * L)
    assert s.dtype == np.float64
    np.testing.assert_array_equal(s, lens * a * a)


def test_scores_zero_when_unchanged_and_symmetric():
    x = rng_of(3).normal(size=300).astype(np.float32)
    c = rng_of(4).normal(size=300).astype(np.float32)
    np.testing.assert_array_equal(oracle.block_scores(F32, x, x.copy(), 7), np.zeros(43))
    np.testing.assert_array_equal(oracle.block_scores(F32, x, c, 7), oracle.block_scores(F32, c, x, 7))


def test_scores_single_changed_element_lands_in_its_block_only():
    L, nb = 5, 9
    for j in (0, 4, 5, 22, 44):
        c = np.zeros(L * nb, dtype=np.float32)
        x = c.copy()
        x[j] = -3.0
        s = oracle.block_scores(F32, x, c, L)
        want = np.zeros(nb)
        want[j // L] = 9.0
        np.testing.assert_array_equal(s, want)


def test_scores_hand_worked_values():
    # blocks of 2: (3,4) -> 25 ; (1,-1) vs (0,1) -> 1+4 = 5 ; tail (0.5) vs (-0.5) -> 1
    x = np.array([3, 4, 1, -1, 0.5], dtype=np.float32)
    c = np.array([0, 0, 0, 1, -0.5], dtype=np.float32)
    np.testing.assert_array_equal(oracle.block_scores(F32, x, c, 2), [25.0, 5.0, 1.0])


def test_scores_accumulate_in_double():
    # 1 + 2^-30 squared differences: a float32 accumulator would lose the small terms.
    L = 1 << 12
    c = np.zeros(L, dtype=np.float32)
    x = np.full(L, 2.0 ** -15, dtype=np.float32)
    x[0] = 1.0
    s = oracle.block_scores(F32, x, c, L)
    assert s[0] == 1.0 + (L - 1) * 2.0 ** -30


def test_scores_sum_equals_flat_squared_distance():
    x = rng_of(5).normal(size=12345).astype(np.float32)
    c = rng_of(6).normal(size=12345).astype(np.float32)
    d = x.astype(np.float64) - c.astype(np.float64)
    s = oracle.block_scores(F32, x, c, 100)
    assert math.isclose(s.sum(), float(d @ d), rel_tol=1e-13)
    ref = np.add.reduceat(d * d, np.arange(0, 12345, 100))
    np.testing.assert_allclose(s, ref, rtol=1e-13)


def test_scores_bf16_bits_decode_exactly():
    # 0x3F80 = 1.0, 0x3F00 = 0.5, 0xC000 = -2.0, 0x0000 = 0, 0x4049 = 3.140625
    x = np.array([0x3F80, 0x3F80, 0xC000, 0x4049], dtype=np.uint16)
    c = np.array([0x3F00, 0x3F00, 0x3F80, 0x0000], dtype=np.uint16)
    s = oracle.block_scores(BF16, x, c, 2)
    np.testing.assert_array_equal(s, [0.5, 9.0 + 3.140625 ** 2])


def test_scores_int_l1_closed_form_and_extremes():
    L, nb = 50, 6
    c = rng_of(7).integers(0, 1000, size=L * nb).astype(np.int32)
    x = c.copy()
    want = np.zeros(nb, dtype=np.int64)
    for b, (m, t) in enumerate([(0, 0), (1, 50), (3, 7), (2, 1), (5, 10), (7, 49)]):
        cols = rng_of(10 + b).choice(L, size=t, replace=False)
        sign = rng_of(20 + b).choice([-1, 1], size=t)
        x[b * L + cols] += (sign * m).astype(np.int32)
        want[b] = m * t
    s = oracle.block_scores(I32, x, c, L)
    assert s.dtype == np.int64
    np.testing.assert_array_equal(s, want)
    # no 32-bit wrap: max - min = 2^32 - 1 per element
    hi = np.full(3, np.iinfo(np.int32).max, dtype=np.int32)
    lo = np.full(3, np.iinfo(np.int32).min, dtype=np.int32)
    np.testing.assert_array_equal(oracle.block_scores(I32, hi, lo, 3), [3 * (2 ** 32 - 1)])
    np.testing.assert_array_equal(oracle.block_scores(I32, lo, hi, 2), [2 * (2 ** 32 - 1), 2 ** 32 - 1])


def test_scores_int_row_moves_are_twice_scaled_total_variation():
    # a row of topic counts with N tokens; moving m tokens between topics changes the
    # length-scaled total variation N * (1/2) sum |x/N - c/N| by m, and L1 by 2m.
    c = np.array([5, 0, 7, 8], dtype=np.int32)
    x = np.array([3, 2, 7, 8], dtype=np.int32)     # 2 tokens moved topic 0 -> 1
    n_tok = c.sum()
    tv_scaled = n_tok * 0.5 * np.abs(x / n_tok - c / n_tok).sum()
    s = oracle.block_scores(I32, x, c, 4)
    assert s[0] == 4 and math.isclose(2 * tv_scaled, 4.0)


# --------------------------------------------------------------------------- top-k

def python_topk(scores, k):
    order = sorted(range(len(scores)), key=lambda b: (-scores[b], b))
    return sorted(order[:k])


@pytest.mark.parametrize("seed", range(6))
def test_topk_maximises_total_score_over_all_subsets(seed):
    r = rng_of(100 + seed)
    n = int(r.integers(1, 12))
    scores = r.integers(0, 5, size=n).astype(np.float64) if seed % 2 else r.random(n)
    for k in range(n + 1):
        idx = oracle.select_topk(scores, k)
        assert len(idx) == k and len(set(idx.tolist())) == k
        best = max((sum(scores[list(sub)]) for sub in itertools.combinations(range(n), k)))
        assert math.isclose(scores[idx].sum(), best, rel_tol=1e-12, abs_tol=0)
        if k:
            assert math.isclose(oracle.brute_force_topk(scores, k), best, rel_tol=1e-12)
        np.testing.assert_array_equal(idx, python_topk(scores.tolist(), k))


def test_topk_int_scores_brute_force_and_ties():
    scores = np.array([4, 9, 4, 4, 0, 9, 1, 4], dtype=np.int64)
    for k in range(9):
        idx = oracle.select_topk(scores, k)
        best = max(sum(int(scores[i]) for i in sub) for sub in itertools.combinations(range(8), k))
        assert int(scores[idx].sum()) == best
        if k:
            assert oracle.brute_force_topk(scores, k) == best
    # k = 4: both 9s, then the two lowest-index 4s
    np.testing.assert_array_equal(oracle.select_topk(scores, 4), [0, 1, 2, 5])
    np.testing.assert_array_equal(oracle.select_topk(scores, 3), [0, 1, 5])


def test_topk_all_equal_takes_lowest_indices_and_edges():
    s = np.full(10, 2.5)
    np.testing.assert_array_equal(oracle.select_topk(s, 4), [0, 1, 2, 3])
    np.testing.assert_array_equal(oracle.select_topk(np.zeros(6, dtype=np.int64), 2), [0, 1])
    assert oracle.select_topk(s, 0).size == 0
    np.testing.assert_array_equal(oracle.select_topk(s, 10), np.arange(10))
    with pytest.raises(oracle.OracleError):
        oracle.select_topk(s, 11)


def test_topk_output_ascending_and_matches_stable_argsort():
    s = rng_of(7).integers(0, 50, size=5000).astype(np.float64)
    for k in (1, 17, 2500, 4999):
        idx = oracle.select_topk(s, k)
        assert np.all(np.diff(idx.astype(np.int64)) > 0)
        ref = np.sort(np.argsort(-s, kind="stable")[:k])
        np.testing.assert_array_equal(idx, ref)


def test_topk_permutation_equivariance_distinct_scores():
    r = rng_of(8)
    s = r.permutation(200).astype(np.float64)
    perm = r.permutation(200)
    a = set(oracle.select_topk(s, 30).tolist())
    b = oracle.select_topk(s[perm], 30)          # block j of the permuted store is block perm[j]
    assert a == set(perm[b].tolist())


def test_topk_nan_and_inf_order():
    s = np.array([1.0, np.inf, np.nan, 5.0, -0.0, 0.0, np.nan])
    np.testing.assert_array_equal(oracle.select_topk(s, 1), [2])
    np.testing.assert_array_equal(oracle.select_topk(s, 2), [2, 6])
    np.testing.assert_array_equal(oracle.select_topk(s, 3), [1, 2, 6])
    np.testing.assert_array_equal(oracle.select_topk(s, 4), [1, 2, 3, 6])
    # -0 and +0 tie: lower index first
    np.testing.assert_array_equal(oracle.select_topk(s, 6), [0, 1, 2, 3, 4, 6])


# --------------------------------------------------------------------------- commit

def small_store(seed, n_elems=203, dtype=F32):
    r = rng_of(seed)
    if dtype == I32:
        c = r.integers(0, 100, size=n_elems).astype(np.int32)
        x = (c + r.integers(-3, 4, size=n_elems)).astype(np.int32)
    elif dtype == BF16:
        c = (r.integers(0, 1 << 15, size=n_elems) & 0x7F7F).astype(np.uint16)
        x = (r.integers(0, 1 << 15, size=n_elems) & 0x7F7F).astype(np.uint16)
    else:
        c = r.normal(size=n_elems).astype(np.float32)
        x = (c + r.normal(size=n_elems) * 0.1).astype(np.float32)
    return x, c


@pytest.mark.parametrize("dtype", [F32, BF16, I32])
def test_commit_all_blocks_makes_checkpoint_equal_x_and_norm_zero(dtype):
    x, c = small_store(11, dtype=dtype)
    L = 10
    nb = oracle.n_blocks_of(x.size, L)
    x0 = x.copy()
    oracle.checkpoint_commit(dtype, x, c, L, np.arange(nb))
    np.testing.assert_array_equal(c, x)
    np.testing.assert_array_equal(x, x0)
    s, nrm, isum = oracle.perturbation_norm(dtype, x, c, L)
    assert s == 0.0 and nrm == 0.0 and isum == 0


@pytest.mark.parametrize("dtype", [F32, I32])
def test_commit_touches_only_chosen_blocks_and_fills_staging(dtype):
    x, c = small_store(12, dtype=dtype)
    L = 10
    nb = oracle.n_blocks_of(x.size, L)           # 21 blocks, tail of 3
    idx = np.array([20, 3, 7], dtype=np.uint32)  # unsorted on purpose, includes the tail
    c0, x0 = c.copy(), x.copy()
    staging = np.full(len(idx) * L, 77, dtype=x.dtype)
    oracle.checkpoint_commit(dtype, x, c, L, idx, staging)
    np.testing.assert_array_equal(x, x0)
    for b in range(nb):
        lo, hi = b * L, min(x.size, (b + 1) * L)
        np.testing.assert_array_equal(c[lo:hi], x0[lo:hi] if b in idx else c0[lo:hi])
    for i, b in enumerate(idx):
        lo, hi = b * L, min(x.size, (b + 1) * L)
        np.testing.assert_array_equal(staging[i * L:i * L + hi - lo], x0[lo:hi])
    np.testing.assert_array_equal(staging[3:L], 77)   # row 0 holds the short tail: rest untouched


def test_commit_subtracts_exactly_the_chosen_scores():
    x, c = small_store(13, n_elems=400)
    L = 16
    s0 = oracle.block_scores(F32, x, c, L)
    idx = oracle.select_topk(s0, 6)
    oracle.checkpoint_commit(F32, x, c, L, idx)
    s1 = oracle.block_scores(F32, x, c, L)
    want = s0.copy()
    want[idx] = 0.0
    np.testing.assert_array_equal(s1, want)


def test_priority_commit_minimises_distance_to_checkpoint_over_all_subsets():
    # Saving the k most-changed blocks leaves the smallest ||x - c|| any k blocks can.
    x, c = small_store(14, n_elems=9 * 4)
    L, nb, k = 4, 9, 3
    s0 = oracle.block_scores(F32, x, c, L)
    idx = oracle.select_topk(s0, k)
    c1 = c.copy()
    oracle.checkpoint_commit(F32, x, c1, L, idx)
    got = oracle.perturbation_norm(F32, x, c1, L)[0]
    best = math.inf
    for sub in itertools.combinations(range(nb), k):
        c2 = c.copy()
        oracle.checkpoint_commit(F32, x, c2, L, np.array(sub, dtype=np.uint32))
        best = min(best, oracle.perturbation_norm(F32, x, c2, L)[0])
    assert math.isclose(got, best, rel_tol=1e-12)


def test_index_lists_are_validated():
    x, c = small_store(15)
    with pytest.raises(oracle.OracleError):
        oracle.checkpoint_commit(F32, x, c, 10, np.array([1, 1], dtype=np.uint32))
    with pytest.raises(oracle.OracleError):
        oracle.checkpoint_commit(F32, x, c, 10, np.array([21], dtype=np.uint32))
    with pytest.raises(oracle.OracleError):
        oracle.partial_recover(F32, x, c, 10, np.array([0, 5, 0], dtype=np.uint32))
    with pytest.raises(oracle.OracleError):
        oracle.perturbation_norm(F32, x, c, 10, np.array([99], dtype=np.uint32))


# --------------------------------------------------------------------------- recovery

@pytest.mark.parametrize("dtype", [F32, BF16, I32])
def test_recover_empty_lost_set_changes_nothing(dtype):
    x, c = small_store(21, dtype=dtype)
    x0, c0 = x.copy(), c.copy()
    s, nrm, isum = oracle.partial_recover(dtype, x, c, 10, np.zeros(0, dtype=np.uint32))
    np.testing.assert_array_equal(x, x0)
    np.testing.assert_array_equal(c, c0)
    assert (s, nrm, isum) == (0.0, 0.0, 0)


@pytest.mark.parametrize("dtype", [F32, BF16, I32])
def test_recover_all_is_full_recovery_and_idempotent(dtype):
    x, c = small_store(22, dtype=dtype)
    L = 10
    nb = oracle.n_blocks_of(x.size, L)
    full = oracle.perturbation_norm(dtype, x, c, L)
    c0 = c.copy()
    got = oracle.partial_recover(dtype, x, c, L, np.arange(nb))
    assert got == full and full[0] > 0
    np.testing.assert_array_equal(x, c)
    np.testing.assert_array_equal(c, c0)
    assert oracle.partial_recover(dtype, x, c, L, np.arange(nb)) == (0.0, 0.0, 0)


def test_recover_touches_only_lost_blocks_and_reads_x_before_overwrite():
    x, c = small_store(23)
    L = 10
    nb = oracle.n_blocks_of(x.size, L)
    lost = np.array([0, 20, 9], dtype=np.uint32)
    x0, c0 = x.copy(), c.copy()
    d = c0.astype(np.float64) - x0.astype(np.float64)
    want = sum(float(d[b * L:(b + 1) * L] @ d[b * L:(b + 1) * L]) for b in lost)
    s, nrm, isum = oracle.partial_recover(F32, x, c, L, lost)
    assert math.isclose(s, want, rel_tol=1e-13) and math.isclose(nrm, math.sqrt(want), rel_tol=1e-13)
    assert isum == 0
    for b in range(nb):
        lo, hi = b * L, min(x.size, (b + 1) * L)
        np.testing.assert_array_equal(x[lo:hi], c0[lo:hi] if b in lost else x0[lo:hi])
    np.testing.assert_array_equal(c, c0)


# --------------------------------------------------------------------------- norm

def test_norm_hand_worked_values():
    # one block (3,4): Euclidean 5.  Two blocks (3,4),(12,0) -> sqrt(169) = 13.
    c = np.array([3, 4, 12, 0], dtype=np.float32)
    x = np.zeros(4, dtype=np.float32)
    assert oracle.perturbation_norm(F32, x, c, 2, [0]) == (25.0, 5.0, 0)
    assert oracle.perturbation_norm(F32, x, c, 2) == (169.0, 13.0, 0)
    assert oracle.perturbation_norm(F32, x, c, 2, []) == (0.0, 0.0, 0)
    # integer table: plain sum of absolute differences, no square root
    ci = np.array([3, -4, 12, 0, 1], dtype=np.int32)
    xi = np.array([0, 0, 10, 5, 1], dtype=np.int32)
    assert oracle.perturbation_norm(I32, xi, ci, 2) == (14.0, 14.0, 14)
    assert oracle.perturbation_norm(I32, xi, ci, 2, [1, 2]) == (7.0, 7.0, 7)


@pytest.mark.parametrize("dtype", [F32, BF16, I32])
def test_partial_perturbation_never_exceeds_full(dtype):
    # Theorem 4.1 (with the <= of its proof).
    x, c = small_store(31, n_elems=997, dtype=dtype)
    L = 13
    nb = oracle.n_blocks_of(x.size, L)
    full = oracle.perturbation_norm(dtype, x, c, L)[1]
    for seed in range(20):
        r = rng_of(seed)
        lost = r.choice(nb, size=int(r.integers(0, nb + 1)), replace=False)
        assert oracle.perturbation_norm(dtype, x, c, L, lost)[1] <= full
    assert oracle.perturbation_norm(dtype, x, c, L, np.arange(nb))[1] == full


@pytest.mark.parametrize("dtype", [F32, I32])
def test_norm_is_additive_over_any_partition_of_blocks(dtype):
    # Appendix A.4: ||d_S||^2 is a sum over the lost coordinates, so over a partition of
    # the blocks the squared (float) or L1 (integer) norms add up to the full one.
    x, c = small_store(32, n_elems=1203, dtype=dtype)
    L = 10
    nb = oracle.n_blocks_of(x.size, L)
    full = oracle.perturbation_norm(dtype, x, c, L)
    parts = np.array_split(rng_of(5).permutation(nb), 7)
    tot = [oracle.perturbation_norm(dtype, x, c, L, p) for p in parts]
    assert math.isclose(sum(t[0] for t in tot), full[0], rel_tol=1e-12)
    assert sum(t[2] for t in tot) == full[2]


def test_expected_partial_perturbation_is_p_times_full_exactly_over_all_subsets():
    # Theorem 4.2: E||d'||^2 = p ||d||^2 when a uniformly random fraction p is lost.
    # Averaging over *all* subsets of size m of n blocks makes the expectation exact.
    x, c = small_store(33, n_elems=8 * 3)
    L, nb = 3, 8
    full = oracle.perturbation_norm(F32, x, c, L)[0]
    for m in (1, 2, 4, 7):
        vals = [oracle.perturbation_norm(F32, x, c, L, np.array(sub, dtype=np.uint32))[0]
                for sub in itertools.combinations(range(nb), m)]
        assert math.isclose(np.mean(vals), (m / nb) * full, rel_tol=1e-12)


def test_expected_partial_perturbation_random_masks():
    x, c = small_store(34, n_elems=4000)
    L = 8
    nb = 500
    full = oracle.perturbation_norm(F32, x, c, L)[0]
    p = 0.25
    r = rng_of(9)
    vals = []
    for _ in range(400):
        lost = oracle.mask_to_indices(r.random(nb) < p)
        vals.append(oracle.perturbation_norm(F32, x, c, L, lost)[0])
    assert abs(np.mean(vals) / (p * full) - 1.0) < 0.02


def test_norm_consistent_with_scores_and_with_commit():
    x, c = small_store(35, n_elems=640)
    L = 16
    s0 = oracle.block_scores(F32, x, c, L)
    lost = np.array([1, 5, 6, 30, 39], dtype=np.uint32)
    assert math.isclose(oracle.perturbation_norm(F32, x, c, L, lost)[0], s0[lost].sum(), rel_tol=1e-13)
    K = oracle.select_topk(s0, 10)
    oracle.checkpoint_commit(F32, x, c, L, K)
    rest = [b for b in lost if b not in set(K.tolist())]
    assert math.isclose(oracle.perturbation_norm(F32, x, c, L, lost)[0], s0[rest].sum(),
                        rel_tol=1e-13, abs_tol=1e-300)


def test_mask_to_indices():
    m = np.array([0, 1, 1, 0, 0, 255, 0, 1], dtype=np.uint8)
    np.testing.assert_array_equal(oracle.mask_to_indices(m), [1, 2, 5, 7])
    assert oracle.mask_to_indices(np.zeros(5, dtype=np.uint8)).size == 0
    assert oracle.mask_to_indices(np.zeros(0, dtype=np.uint8)).size == 0


def test_threads_do_not_change_results():
    x, c = small_store(36, n_elems=50000)
    L = 7
    oracle.set_num_threads(1)
    a = oracle.block_scores(F32, x, c, L)
    na = oracle.perturbation_norm(F32, x, c, L)
    oracle.set_num_threads(4)
    try:
        b = oracle.block_scores(F32, x, c, L)
        nb_ = oracle.perturbation_norm(F32, x, c, L)
    finally:
        oracle.set_num_threads(1)
    np.testing.assert_array_equal(a, b)
    assert na == nb_


def test_three_cycles_keep_the_running_checkpoint_consistent():
    # Running checkpoint starts at x(0) and holds a mix of ages afterwards (Section 4.2).
    r = rng_of(40)
    L, nb = 8, 64
    x = r.normal(size=L * nb).astype(np.float32)
    c = x.copy()
    assert oracle.perturbation_norm(F32, x, c, L)[0] == 0.0
    for cycle in range(3):
        x += (r.normal(size=x.size) * 0.01).astype(np.float32)
        s = oracle.block_scores(F32, x, c, L)
        K = oracle.select_topk(s, 16)
        oracle.checkpoint_commit(F32, x, c, L, K)
        s_after = oracle.block_scores(F32, x, c, L)
        assert np.all(s_after[K] == 0.0)
        others = np.setdiff1d(np.arange(nb), K)
        assert s_after[others].max() <= s[K].min()


# --------------------------------------------------------------------------- comparison strategies

def test_philox_known_answers():
    import os
    path = os.path.join(os.path.dirname(__file__), "golden", "philox4x32_10_kat.txt")
    rows = [l.split() for l in open(path) if l.strip() and not l.startswith("#")]
    assert len(rows) == 3
    for r in rows:
        w = [int(v, 16) for v in r]
        np.testing.assert_array_equal(oracle.philox4x32_10(w[0:4], w[4:6]), w[6:10])


def test_round_robin_covers_every_block_once_per_sweep():
    n, k = 40, 8
    seen = []
    for t in range(5):
        idx = oracle.select_round(n, k, t * k)
        np.testing.assert_array_equal(idx, np.arange(t * k, (t + 1) * k))
        seen.extend(idx.tolist())
    assert sorted(seen) == list(range(n))
    # wrap-around stays ascending and the cursor is taken modulo n
    np.testing.assert_array_equal(oracle.select_round(10, 4, 8), [0, 1, 8, 9])
    np.testing.assert_array_equal(oracle.select_round(10, 4, 28), [0, 1, 8, 9])
    np.testing.assert_array_equal(oracle.select_round(10, 10, 3), np.arange(10))
    assert oracle.select_round(10, 0, 3).size == 0


def test_random_strategy_is_a_seeded_uniform_subset():
    n, k = 200, 50
    a = oracle.select_random(n, k, seed=7, draw=0)
    assert a.size == k and len(set(a.tolist())) == k and a.max() < n
    assert np.all(np.diff(a.astype(np.int64)) > 0)
    np.testing.assert_array_equal(a, oracle.select_random(n, k, seed=7, draw=0))
    assert not np.array_equal(a, oracle.select_random(n, k, seed=7, draw=1))
    assert not np.array_equal(a, oracle.select_random(n, k, seed=8, draw=0))
    # the choice is the top-k of the blocks' Philox numbers
    num = np.array([oracle.philox4x32_10([b, 0, 3, 0], [7, 0])[0] for b in range(n)], dtype=np.int64)
    np.testing.assert_array_equal(oracle.select_random(n, k, seed=7, draw=3), oracle.select_topk(num, k))
    # every block is chosen with probability k/n
    hits = np.zeros(n)
    draws = 2000
    for d in range(draws):
        hits[oracle.select_random(n, k, seed=1, draw=d)] += 1
    p = k / n
    z = (hits - draws * p) / np.sqrt(draws * p * (1 - p))
    assert np.abs(z).max() < 4.5 and abs(z.mean()) < 0.3
    np.testing.assert_array_equal(oracle.select_random(9, 9, 1, 1), np.arange(9))


# --------------------------------------------------------------------------- unequal blocks

def ragged_offsets(seed, n_blocks, max_len, empties=True):
    r = rng_of(seed)
    lens = r.integers(1, max_len + 1, size=n_blocks)
    if empties:
        lens[r.choice(n_blocks, size=max(1, n_blocks // 10), replace=False)] = 0
    return np.concatenate([[0], np.cumsum(lens)]).astype(np.uint64)


@pytest.mark.parametrize("dtype", [F32, BF16, I32])
def test_var_layout_with_equal_blocks_is_the_fixed_layout(dtype):
    x, c = small_store(51, n_elems=230, dtype=dtype)
    L = 10
    off = np.arange(0, 231, L, dtype=np.uint64)
    np.testing.assert_array_equal(oracle.var_block_scores(dtype, x, c, off), oracle.block_scores(dtype, x, c, L))
    idx = np.array([3, 22, 0], dtype=np.uint32)
    assert oracle.var_perturbation_norm(dtype, x, c, off, idx) == oracle.perturbation_norm(dtype, x, c, L, idx)
    assert oracle.var_perturbation_norm(dtype, x, c, off) == oracle.perturbation_norm(dtype, x, c, L)
    c1, c2 = c.copy(), c.copy()
    oracle.var_checkpoint_commit(dtype, x, c1, off, idx)
    oracle.checkpoint_commit(dtype, x, c2, L, idx)
    np.testing.assert_array_equal(c1, c2)
    x1, x2 = x.copy(), x.copy()
    assert oracle.var_partial_recover(dtype, x1, c, off, idx) == oracle.partial_recover(dtype, x2, c, L, idx)
    np.testing.assert_array_equal(x1, x2)


def test_var_scores_closed_form_and_empty_blocks():
    off = np.array([0, 3, 3, 10, 11, 11, 40], dtype=np.uint64)       # lengths 3 0 7 1 0 29
    c = rng_of(52).integers(-4, 4, size=40).astype(np.float32)
    a = np.array([0.5, 9.0, 2.0, -4.0, 7.0, 0.25])
    x = (c + np.repeat(a, np.diff(off.astype(np.int64)))).astype(np.float32)
    np.testing.assert_array_equal(oracle.var_block_scores(F32, x, c, off), np.diff(off.astype(np.int64)) * a * a)
    s, nrm, _ = oracle.var_perturbation_norm(F32, x, c, off, [2, 3, 4])
    assert s == 7 * 4.0 + 16.0 and nrm == math.sqrt(s)
    ci = np.zeros(40, dtype=np.int32)
    xi = np.repeat(np.array([1, 5, -2, 3, 9, 1]), np.diff(off.astype(np.int64))).astype(np.int32)
    np.testing.assert_array_equal(oracle.var_block_scores(I32, xi, ci, off), [3, 0, 14, 3, 0, 29])


def test_var_commit_and_recover_touch_only_their_blocks():
    off = ragged_offsets(53, 30, 17)
    n = int(off[-1])
    x, c = small_store(54, n_elems=n)
    x0, c0 = x.copy(), c.copy()
    K = np.array([29, 4, 11], dtype=np.uint32)
    oracle.var_checkpoint_commit(F32, x, c, off, K)
    np.testing.assert_array_equal(x, x0)
    for b in range(30):
        lo, hi = int(off[b]), int(off[b + 1])
        np.testing.assert_array_equal(c[lo:hi], x0[lo:hi] if b in K else c0[lo:hi])
    S = np.array([0, 4, 17, 28], dtype=np.uint32)
    c1 = c.copy()
    full = oracle.var_perturbation_norm(F32, x, c, off)
    got = oracle.var_partial_recover(F32, x, c, off, S)
    assert got[1] <= full[1]
    np.testing.assert_array_equal(c, c1)
    for b in range(30):
        lo, hi = int(off[b]), int(off[b + 1])
        np.testing.assert_array_equal(x[lo:hi], c1[lo:hi] if b in S else x0[lo:hi])
    assert oracle.var_partial_recover(F32, x, c, off, S) == (0.0, 0.0, 0)
    parts = np.array_split(rng_of(1).permutation(30), 4)
    x2, _ = small_store(55, n_elems=n)
    tot = sum(oracle.var_perturbation_norm(F32, x2, c, off, p)[0] for p in parts)
    assert math.isclose(tot, oracle.var_perturbation_norm(F32, x2, c, off)[0], rel_tol=1e-12)
    with pytest.raises(oracle.OracleError):
        oracle.var_checkpoint_commit(F32, x, c, off, [30])
    with pytest.raises(oracle.OracleError):
        oracle.var_block_scores(F32, x, c, np.array([0, 5, 4], dtype=np.uint64))


def test_var_staging_layout_by_hand():
    # lengths 3 0 5 2 4; listed 2, 0, 3, 1: packed offsets 0 5 8 10 10 (an empty block takes no
    # room), packed content = the blocks of x one after the other in list order
    off = np.array([0, 3, 3, 8, 10, 14], dtype=np.uint64)
    x = np.arange(100, 114, dtype=np.float32)
    c = np.zeros(14, dtype=np.float32)
    st = np.full(12, -1, dtype=np.float32)
    got = oracle.var_checkpoint_commit(F32, x, c, off, [2, 0, 3, 1], st)
    np.testing.assert_array_equal(got, [0, 5, 8, 10, 10])
    np.testing.assert_array_equal(st, [103, 104, 105, 106, 107, 100, 101, 102, 108, 109, -1, -1])
    np.testing.assert_array_equal(c, [100, 101, 102, 103, 104, 105, 106, 107, 108, 109, 0, 0, 0, 0])
    # nothing listed: offsets = [0], nothing written
    st[:] = -1
    np.testing.assert_array_equal(oracle.var_checkpoint_commit(F32, x, c, off, [], st), [0])
    assert (st == -1).all()


@pytest.mark.parametrize("dtype", [F32, BF16, I32])
def test_var_staging_with_equal_blocks_is_the_fixed_layouts_staging(dtype):
    x, c = small_store(56, n_elems=240, dtype=dtype)
    L = 10
    off = np.arange(0, 241, L, dtype=np.uint64)
    idx = np.array([7, 23, 0, 11], dtype=np.uint32)
    c1, c2 = c.copy(), c.copy()
    st1, st2 = np.zeros(idx.size * L, dtype=x.dtype), np.zeros(idx.size * L, dtype=x.dtype)
    st_off = oracle.var_checkpoint_commit(dtype, x, c1, off, idx, st1)
    oracle.checkpoint_commit(dtype, x, c2, L, idx, st2)
    np.testing.assert_array_equal(st_off, np.arange(idx.size + 1) * L)
    np.testing.assert_array_equal(st1, st2)
    np.testing.assert_array_equal(c1, c2)


@pytest.mark.parametrize("dtype", [F32, I32])
def test_var_recovery_from_packed_rows_is_recovery_from_the_checkpoint(dtype):
    # rows packed by a commit hold c's values of those blocks; recovering the same blocks from
    # the rows must equal recovering them from c, norm and bytes, and touch nothing else
    off = ragged_offsets(57, 40, 23)
    n = int(off[-1])
    x, c = small_store(58, n_elems=n, dtype=dtype)
    K = np.array([31, 2, 17, 9, 38], dtype=np.uint32)
    st = np.zeros(n, dtype=x.dtype)
    st_off = oracle.var_checkpoint_commit(dtype, x, c, off, K, st)
    x_new, _ = small_store(59, n_elems=n, dtype=dtype)          # training moved on
    xa, xb = x_new.copy(), x_new.copy()
    want = oracle.var_partial_recover(dtype, xa, c, off, K)
    got = oracle.var_partial_recover_rows(dtype, xb, st, st_off[:-1], off, K)
    assert want[1] > 0 and got[2] == want[2]
    assert math.isclose(got[0], want[0], rel_tol=1e-12) and math.isclose(got[1], want[1], rel_tol=1e-12)
    np.testing.assert_array_equal(xa, xb)
    # by hand on one block: x <- row, norm = |row - x|
    o2 = np.array([0, 2, 5], dtype=np.uint64)
    if dtype == F32:
        xs = np.array([1, 2, 3, 4, 5], dtype=np.float32)
        rows = np.array([9, 9, 9, 6, 8, 5], dtype=np.float32)      # block 1 packed at offset 3
        assert oracle.var_partial_recover_rows(F32, xs, rows, [3], o2, [1]) == (9.0 + 16.0, 5.0, 0)
        np.testing.assert_array_equal(xs, [1, 2, 6, 8, 5])


# --------------------------------------------------------------------------- reduced-precision checkpoint

MIX = oracle.F32_BF16C


def bf16_of(values):
    """bfloat16 bit patterns of values that are exactly representable (top 16 bits of the float32)."""
    bits = np.asarray(values, dtype=np.float32).view(np.uint32)
    assert np.all(bits & 0xFFFF == 0)
    return (bits >> 16).astype(np.uint16)


def test_mixed_scores_and_norm_hand_worked():
    x = np.array([1.5, -2.0, 0.75, 3.0], dtype=np.float32)
    c = bf16_of([1.0, -2.0, 0.25, -1.0])
    np.testing.assert_array_equal(oracle.block_scores(MIX, x, c, 2), [0.25, 0.25 + 16.0])
    assert oracle.perturbation_norm(MIX, x, c, 2) == (16.5, math.sqrt(16.5), 0)
    assert oracle.perturbation_norm(MIX, x, c, 2, [0]) == (0.25, 0.5, 0)


def test_mixed_commit_rounds_to_nearest_even_and_recover_widens():
    # 1 + 2^-8 lies half-way between 1 and 1 + 2^-7: ties go to the even significand (1.0);
    # 1 + 3*2^-8 is half-way between 1 + 2^-7 (odd) and 1 + 2^-6 (even) -> 1 + 2^-6;
    # 1 + 2^-8 + 2^-20 is above the half-way point -> 1 + 2^-7; -0.3 -> nearest bfloat16
    x = np.array([1.0 + 2.0 ** -8, 1.0 + 3 * 2.0 ** -8, 1.0 + 2.0 ** -8 + 2.0 ** -20, -0.3,
                  3.0e38, 1e-40, np.inf, 0.0], dtype=np.float32)
    c = np.zeros(8, dtype=np.uint16)
    st = np.zeros(8, dtype=np.uint16)
    oracle.checkpoint_commit(MIX, x, c, 8, [0], st)
    back = (c.astype(np.uint32) << 16).view(np.float32)
    np.testing.assert_array_equal(back[:3], np.array([1.0, 1.0 + 2.0 ** -6, 1.0 + 2.0 ** -7], dtype=np.float32))
    assert back[3] == np.float32(-0.30078125)
    assert abs(back[4] - 3.0e38) <= 3.0e38 * 2.0 ** -8 and back[6] == np.inf and back[7] == 0.0
    np.testing.assert_array_equal(st, c)
    # second opinion on the rounding from a library conversion
    import torch
    ref = torch.from_numpy(x).to(torch.bfloat16).view(torch.int16).numpy().view(np.uint16)
    np.testing.assert_array_equal(c, ref)
    nan = np.array([np.nan], dtype=np.float32)
    cn = np.zeros(1, dtype=np.uint16)
    oracle.checkpoint_commit(MIX, nan, cn, 1, [0])
    assert np.isnan((cn.astype(np.uint32) << 16).view(np.float32))[0]
    # recovery widens exactly
    x2 = np.zeros(8, dtype=np.float32)
    oracle.partial_recover(MIX, x2, c, 8, [0])
    np.testing.assert_array_equal(x2, back)


def test_mixed_rounding_perturbation_obeys_the_reduced_precision_bound():
    # Example 2.1: storing with a p-bit significand perturbs by less than 2^-(p-1) |y| per
    # element (p = 8 for bfloat16; round-to-nearest achieves half of that), so right after
    # saving everything the distance to the checkpoint is at most 2^-8 ||x||.
    r = rng_of(70)
    x = (r.normal(size=5000) * 10.0 ** r.uniform(-3, 3, size=5000)).astype(np.float32)
    c = np.zeros(5000, dtype=np.uint16)
    oracle.checkpoint_commit(MIX, x, c, 50, np.arange(100))
    back = (c.astype(np.uint32) << 16).view(np.float32).astype(np.float64)
    assert np.all(np.abs(back - x) <= np.abs(x.astype(np.float64)) * 2.0 ** -8)
    s, nrm, _ = oracle.perturbation_norm(MIX, x, c, 50)
    assert 0 < nrm <= 2.0 ** -8 * float(np.linalg.norm(x.astype(np.float64)))
    scores = oracle.block_scores(MIX, x, c, 50)
    assert math.isclose(scores.sum(), s, rel_tol=1e-12)


def test_mixed_equals_float_store_when_values_are_representable():
    r = rng_of(71)
    cf = (r.integers(-64, 64, size=300) / 8.0).astype(np.float32)      # exact in bfloat16
    xf = (cf + r.integers(-8, 8, size=300) / 4.0).astype(np.float32)
    cb = bf16_of(cf)
    np.testing.assert_array_equal(oracle.block_scores(MIX, xf, cb, 7), oracle.block_scores(F32, xf, cf, 7))
    assert oracle.perturbation_norm(MIX, xf, cb, 7, [1, 5]) == oracle.perturbation_norm(F32, xf, cf, 7, [1, 5])
    x1, x2 = xf.copy(), xf.copy()
    assert oracle.partial_recover(MIX, x1, cb, 7, [0, 42]) == oracle.partial_recover(F32, x2, cf, 7, [0, 42])
    np.testing.assert_array_equal(x1, x2)
    one = np.array([0, 300], dtype=np.uint64)                            # the same in one block of unequal-length kind
    np.testing.assert_array_equal(oracle.var_block_scores(MIX, xf, cb, one), oracle.var_block_scores(F32, xf, cf, one))
    with pytest.raises(oracle.OracleError):                               # the total variation has no such store
        oracle.var_tv_block_scores(MIX, xf, cb, one)


# ------------------------------------------- scaled total variation (Section 5.1, Appendix C)

def one_hot(n, i):
    v = np.zeros(n, dtype=np.float32)
    v[i] = 1.0
    return v


def test_tv_of_disjoint_and_equal_distributions():
    # TV of two distributions with disjoint support is 1, of equal ones 0; the score is the
    # document length times that
    x = np.concatenate([one_hot(5, 0), one_hot(5, 2), one_hot(5, 4)])
    c = np.concatenate([one_hot(5, 1), one_hot(5, 2), one_hot(5, 0)])
    np.testing.assert_array_equal(oracle.tv_block_scores(F32, x, c, 5), [1.0, 0.0, 1.0])
    np.testing.assert_array_equal(oracle.tv_block_scores(F32, x, c, 5, [120, 7, 33]), [120.0, 0.0, 33.0])
    np.testing.assert_array_equal(oracle.tv_block_scores(F32, c, x, 5, [120, 7, 33]), [120.0, 0.0, 33.0])


def test_tv_closed_form_and_ragged_tail():
    # x = c + a on t entries of a block  =>  TV = t * a / 2, the short tail block included
    L, n = 8, 8 * 5 + 3
    c = np.full(n, 0.125, dtype=np.float32)
    x = c.copy()
    x[0:3] += 0.25           # block 0: t = 3
    x[17] -= 0.5             # block 2: t = 1
    x[40:43] += 2.0 ** -10   # tail block (3 elements): t = 3
    w = np.array([2, 3, 5, 7, 11, 13], dtype=np.float32)
    want = np.array([3 * 0.25 / 2, 0, 0.5 / 2, 0, 0, 3 * 2.0 ** -10 / 2])
    np.testing.assert_array_equal(oracle.tv_block_scores(F32, x, c, L), want)
    np.testing.assert_array_equal(oracle.tv_block_scores(F32, x, c, L, w), want * w)


def test_tv_on_normalised_counts_is_half_the_l1_of_the_counts():
    # rows of topic counts with N = 1024 tokens each (n / N is exact in float32): the
    # length-scaled TV of the normalised rows is exactly half the L1 distance of the counts,
    # which is what the integer path scores (its reading of the same norm)
    r = np.random.default_rng(5)
    rows, topics, n_tok = 40, 16, 1024
    c = r.multinomial(n_tok, np.full(topics, 1.0 / topics), size=rows).astype(np.int32)
    x = c.copy()
    for d in range(rows):
        for _ in range(int(r.integers(0, 6))):
            src, dst = r.choice(topics, size=2, replace=False)
            m = min(int(x[d, src]), int(r.integers(1, 4)))
            x[d, src] -= m
            x[d, dst] += m
    l1 = oracle.block_scores(I32, x.ravel(), c.ravel(), topics)
    tv = oracle.tv_block_scores(F32, (x / n_tok).astype(np.float32).ravel(), (c / n_tok).astype(np.float32).ravel(),
                                topics, np.full(rows, n_tok, dtype=np.float32))
    np.testing.assert_array_equal(2 * tv, l1.astype(np.float64))


def test_tv_is_a_metric_bounded_by_one_on_distributions():
    r = np.random.default_rng(6)
    L, nb = 20, 50
    p, q, s = (r.dirichlet(np.full(L, 0.3), size=nb).astype(np.float32).ravel() for _ in range(3))
    pq, qs, ps = (oracle.tv_block_scores(F32, a, b, L) for a, b in ((p, q), (q, s), (p, s)))
    assert np.all(pq >= 0) and np.all(pq <= 1 + 1e-6)
    assert np.all(ps <= pq + qs + 1e-12)                                   # triangle inequality
    np.testing.assert_array_equal(pq, oracle.tv_block_scores(F32, q, p, L))
    ref = 0.5 * np.abs(p.astype(np.float64) - q.astype(np.float64)).reshape(nb, L).sum(1)
    np.testing.assert_allclose(pq, ref, rtol=1e-14)
    # bfloat16 rows decode exactly
    pb, qb = (np.frombuffer(a.tobytes(), dtype=np.uint16)[1::2].copy() for a in (p, q))
    pf, qf = ((b.astype(np.uint32) << 16).view(np.float32) for b in (pb, qb))
    np.testing.assert_array_equal(oracle.tv_block_scores(BF16, pb, qb, L), oracle.tv_block_scores(F32, pf, qf, L))


def test_tv_norm_is_the_weighted_sum_of_the_block_distances():
    r = np.random.default_rng(7)
    L, nb = 12, 30
    x = r.dirichlet(np.full(L, 0.5), size=nb).astype(np.float32).ravel()[: L * nb - 5]
    c = r.dirichlet(np.full(L, 0.5), size=nb).astype(np.float32).ravel()[: L * nb - 5]
    w = r.integers(1, 500, size=nb).astype(np.float32)
    s = oracle.tv_block_scores(F32, x, c, L, w)
    full = oracle.tv_perturbation_norm(F32, x, c, L, w)
    assert math.isclose(full[0], s.sum(), rel_tol=1e-13) and full[0] == full[1] and full[2] == 0
    S = np.array([29, 3, 11, 4], dtype=np.uint32)
    part = oracle.tv_perturbation_norm(F32, x, c, L, w, S)
    assert math.isclose(part[0], s[S].sum(), rel_tol=1e-13)
    assert part[1] <= full[1]                                               # Theorem 4.1's analogue
    rest = np.setdiff1d(np.arange(nb), S).astype(np.uint32)
    assert math.isclose(part[0] + oracle.tv_perturbation_norm(F32, x, c, L, w, rest)[0], full[0], rel_tol=1e-13)
    assert oracle.tv_perturbation_norm(F32, x, c, L, w, np.zeros(0, dtype=np.uint32)) == (0.0, 0.0, 0)
    unweighted = oracle.tv_perturbation_norm(F32, x, c, L)
    assert math.isclose(unweighted[0], oracle.tv_block_scores(F32, x, c, L).sum(), rel_tol=1e-13)
    # recovery: the norm is measured before the overwrite, only the lost rows change
    x0 = x.copy()
    got = oracle.tv_partial_recover(F32, x, c, L, S, w)
    assert got == part
    keep = np.ones(x.size, dtype=bool)
    for b in S:
        keep[b * L:(b + 1) * L] = False
        np.testing.assert_array_equal(x[b * L:(b + 1) * L], c[b * L:(b + 1) * L])
    np.testing.assert_array_equal(x[keep], x0[keep])
    assert oracle.tv_partial_recover(F32, x, c, L, S, w) == (0.0, 0.0, 0)
    with pytest.raises(oracle.OracleError):
        oracle.tv_block_scores(I32, x.view(np.int32), c.view(np.int32), L)


# ------------------------------------------------------------- scores of listed blocks only

@pytest.mark.parametrize("dtype", [F32, BF16, I32, oracle.F32_BF16C])
def test_rescoring_listed_blocks_equals_rescoring_everything(dtype):
    r = np.random.default_rng(21 + dtype)
    L, nb = 7, 40
    n = L * nb - 3
    if dtype == I32:
        c = r.integers(-50, 50, size=n).astype(np.int32)
        x = c.copy()
    else:
        c = r.normal(size=n).astype(np.float32)
        x = c.copy()
        if dtype == BF16:
            x, c = (np.frombuffer(a.tobytes(), dtype=np.uint16)[1::2].copy() for a in (x, c))
        elif dtype == oracle.F32_BF16C:                           # c in bfloat16, x its exact widening
            c = np.frombuffer(c.tobytes(), dtype=np.uint16)[1::2].copy()
            x = (c.astype(np.uint32) << 16).view(np.float32)
    s = oracle.block_scores(dtype, x, c, L)
    assert not s.any()
    touched = np.array([39, 0, 17, 5, 16], dtype=np.uint32)      # unsorted, two neighbours, the short tail
    for b in touched:
        lo, hi = b * L, min((b + 1) * L, n)
        if dtype == I32:
            x[lo:hi] += 3
        elif x.dtype == np.float32:
            x[lo:hi] += np.float32(0.5)
        else:
            x[lo:hi] ^= np.uint16(0x0080)                         # flip a mantissa bit
    full = oracle.block_scores(dtype, x, c, L)
    assert full[touched].all() and np.count_nonzero(full) == touched.size
    stale = s.copy()
    stale[1] = 123                                                # an entry that must survive
    got = oracle.block_scores_rows(dtype, x, c, L, touched, stale)
    want = full.copy()
    want[1] = 123
    np.testing.assert_array_equal(got, want)
    np.testing.assert_array_equal(oracle.block_scores_rows(dtype, x, c, L, np.zeros(0, dtype=np.uint32), stale), want)
    with pytest.raises(oracle.OracleError):
        oracle.block_scores_rows(dtype, x, c, L, np.array([40], dtype=np.uint32), stale)
    with pytest.raises(oracle.OracleError):
        oracle.block_scores_rows(dtype, x, c, L, np.array([3, 3], dtype=np.uint32), stale)


def test_var_tv_closed_forms_and_reduction_to_equal_rows():
    # rows of unequal length: disjoint one-hot rows have TV 1, equal rows 0, an empty row 0;
    # x = c + a on t entries => t * a / 2; weights multiply; equal rows reduce to the fixed layout
    off = np.array([0, 3, 3, 8, 10], dtype=np.uint64)                     # lengths 3 0 5 2
    c = np.concatenate([one_hot(3, 0), one_hot(5, 1), np.array([0.5, 0.5], dtype=np.float32)])
    x = np.concatenate([one_hot(3, 2), one_hot(5, 1), np.array([0.75, 0.25], dtype=np.float32)])
    np.testing.assert_array_equal(oracle.var_tv_block_scores(F32, x, c, off), [1.0, 0.0, 0.0, 0.25])
    w = np.array([40, 9, 7, 8], dtype=np.float32)
    np.testing.assert_array_equal(oracle.var_tv_block_scores(F32, x, c, off, w), [40.0, 0.0, 0.0, 2.0])
    assert oracle.var_tv_perturbation_norm(F32, x, c, off, w) == (42.0, 42.0, 0)
    assert oracle.var_tv_perturbation_norm(F32, x, c, off, w, [3, 1]) == (2.0, 2.0, 0)
    assert oracle.var_tv_perturbation_norm(F32, x, c, off, w, []) == (0.0, 0.0, 0)
    x1 = x.copy()
    assert oracle.var_tv_partial_recover(F32, x1, c, off, [0], w) == (40.0, 40.0, 0)
    np.testing.assert_array_equal(x1[:3], c[:3])
    np.testing.assert_array_equal(x1[3:], x[3:])
    r = np.random.default_rng(8)
    L, nb = 12, 25
    xe = r.dirichlet(np.full(L, 0.5), size=nb).astype(np.float32).ravel()
    ce = r.dirichlet(np.full(L, 0.5), size=nb).astype(np.float32).ravel()
    we = r.integers(1, 300, size=nb).astype(np.float32)
    offe = np.arange(0, L * nb + 1, L, dtype=np.uint64)
    np.testing.assert_array_equal(oracle.var_tv_block_scores(F32, xe, ce, offe, we), oracle.tv_block_scores(F32, xe, ce, L, we))
    S = np.array([7, 0, 19], dtype=np.uint32)
    assert oracle.var_tv_perturbation_norm(F32, xe, ce, offe, we, S) == oracle.tv_perturbation_norm(F32, xe, ce, L, we, S)
    xa, xb = xe.copy(), xe.copy()
    assert oracle.var_tv_partial_recover(F32, xa, ce, offe, S, we) == oracle.tv_partial_recover(F32, xb, ce, L, S, we)
    np.testing.assert_array_equal(xa, xb)


def test_var_layout_with_a_bfloat16_checkpoint_reduces_to_the_fixed_layout_and_rounds_by_hand():
    # float32 x against a bfloat16 c in blocks of unequal length: with equal blocks every call
    # equals its fixed-layout twin; by hand: a commit stores x rounded to nearest even, the
    # staging rows hold those rounded values, recovery widens them
    r = rng_of(60)
    L, nb = 10, 24
    x = r.normal(0, 1, size=L * nb).astype(np.float32)
    c = (r.normal(0, 1, size=L * nb).astype(np.float32).view(np.uint32) >> 16).astype(np.uint16)
    off = np.arange(0, L * nb + 1, L, dtype=np.uint64)
    np.testing.assert_array_equal(oracle.var_block_scores(MIX, x, c, off), oracle.block_scores(MIX, x, c, L))
    idx = np.array([5, 23, 0, 11], dtype=np.uint32)
    assert oracle.var_perturbation_norm(MIX, x, c, off, idx) == oracle.perturbation_norm(MIX, x, c, L, idx)
    c1, c2 = c.copy(), c.copy()
    st1, st2 = np.zeros(idx.size * L, dtype=np.uint16), np.zeros(idx.size * L, dtype=np.uint16)
    oracle.var_checkpoint_commit(MIX, x, c1, off, idx, st1)
    oracle.checkpoint_commit(MIX, x, c2, L, idx, st2)
    np.testing.assert_array_equal(c1, c2)
    np.testing.assert_array_equal(st1, st2)
    x1, x2 = x.copy(), x.copy()
    assert oracle.var_partial_recover(MIX, x1, c1, off, idx) == oracle.partial_recover(MIX, x2, c2, L, idx)
    np.testing.assert_array_equal(x1, x2)
    # by hand, lengths 2 and 3: 1 + 2^-8 is a tie and rounds to even (1.0), 1 + 3 * 2^-8 rounds up
    o2 = np.array([0, 2, 5], dtype=np.uint64)
    xs = np.array([9.0, 9.0, 1.0 + 2.0 ** -8, 1.0 + 3 * 2.0 ** -8, -2.5], dtype=np.float32)
    cs = bf16_of([0, 0, 0, 0, 0])
    st = np.zeros(3, dtype=np.uint16)
    np.testing.assert_array_equal(oracle.var_checkpoint_commit(MIX, xs, cs, o2, [1], st), [0, 3])
    want = bf16_of([1.0, 1.0 + 2.0 ** -6, -2.5])
    np.testing.assert_array_equal(st, want)
    np.testing.assert_array_equal(cs, np.concatenate([bf16_of([0, 0]), want]))
    xr = np.zeros(5, dtype=np.float32)
    got = oracle.var_partial_recover_rows(MIX, xr, st, [0], o2, [1])
    np.testing.assert_array_equal(xr, [0, 0, 1.0, 1.0 + 2.0 ** -6, -2.5])
    assert got[0] == 1.0 + (1.0 + 2.0 ** -6) ** 2 + 6.25
