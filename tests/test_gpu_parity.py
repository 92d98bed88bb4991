"""GPU parity: every entry point of libscar.so against the CPU oracle on the same seeded
inputs, element by element.  Integer results and indices are compared bit for bit, float
scores and norms to 1e-5 relative (float32/float64 accumulation against the float64
oracle).  Sizes span several tiles, several group sizes and ragged tails."""
import numpy as np
import pytest
import torch

import oracle
from paper_1810_07354_amd import scar
from paper_1810_07354_amd import workloads as wl
from gpu_util import (DEV, REL_TOL, DeviceStore, assert_norm_matches, assert_scores_match,
                      assert_selection_matches, idx_dev, idx_host, to_dev, to_host)

pytestmark = pytest.mark.gpu

F32, BF16, I32 = wl.F32, wl.BF16, wl.I32


def make_store(dtype, n_elems, seed):
    r = np.random.default_rng(seed)
    if dtype == I32:
        c = r.integers(-1000, 1000, size=n_elems).astype(np.int32)
        x = (c + r.integers(-5, 6, size=n_elems) * (r.random(n_elems) < 0.1)).astype(np.int32)
    else:
        c = r.normal(0, 0.1, size=n_elems).astype(np.float32)
        x = (c + r.normal(0, 0.01, size=n_elems) * (r.random(n_elems) < 0.7)).astype(np.float32)
        if dtype == BF16:
            x, c = wl.f32_to_bf16_bits(x), wl.f32_to_bf16_bits(c)
    return x, c


BLOCK_LENS = [1, 3, 8, 100, 784, 1000, 1024, 4096, 5000, 70000]


@pytest.mark.parametrize("dtype", [F32, BF16, I32])
@pytest.mark.parametrize("L", BLOCK_LENS)
def test_block_scores(dtype, L):
    n_elems = min(max(L * 37 + L // 3, 4099), 3_000_000)     # ragged tail unless L == 1
    x, c = make_store(dtype, n_elems, seed=L)
    print("scores dtype=%d L=%d n=%d" % (dtype, L, n_elems), flush=True)
    got = scar.block_scores(to_dev(x, dtype), to_dev(c, dtype), L)
    assert_scores_match(got, oracle.block_scores(dtype, x, c, L), dtype)


@pytest.mark.parametrize("dtype", [F32, BF16, I32])
@pytest.mark.parametrize("L", [4, 100, 1024])
def test_block_scores_unaligned_base(dtype, L):
    # a view that starts one element into the allocation: no 16-byte alignment
    n_elems = L * 50 + 7
    x, c = make_store(dtype, n_elems + 1, seed=100 + L)
    dx, dc = to_dev(x, dtype)[1:], to_dev(c, dtype)[1:]
    print("scores unaligned dtype=%d L=%d" % (dtype, L), flush=True)
    got = scar.block_scores(dx, dc, L)
    assert_scores_match(got, oracle.block_scores(dtype, x[1:].copy(), c[1:].copy(), L), dtype)


@pytest.mark.parametrize("dtype", [F32, BF16, I32])
@pytest.mark.parametrize("L", [1, 6, 100, 1000, 1024, 5000])
def test_block_scores_of_listed_blocks(dtype, L):
    # scores[b] for b in idx equals the full scan's, every other entry stays as it was; the
    # list is unsorted, holds the short tail block and two entries out of range (skipped)
    nb = 3000 if L <= 1024 else 300
    n = L * nb - L // 2
    x, c = make_store(dtype, n, seed=11 * L + dtype)
    nbk = oracle.n_blocks_of(n, L)
    r = np.random.default_rng(L)
    listed = np.unique(np.append(r.permutation(nbk)[: nbk // 5], nbk - 1)).astype(np.uint32)
    r.shuffle(listed)
    print("listed scores dtype=%d L=%d n_idx=%d" % (dtype, L, listed.size), flush=True)
    dx, dc = to_dev(x, dtype), to_dev(c, dtype)
    stale_h = (np.arange(nbk) * 7).astype(np.int64 if dtype == I32 else np.float32)
    stale = torch.from_numpy(stale_h.copy()).to(DEV)
    with_bad = np.concatenate([listed[:5], [nbk, 0xFFFFFFFF], listed[5:]]).astype(np.uint32)
    scar.block_scores_rows(dx, dc, L, idx_dev(with_bad), stale)
    want = stale_h.astype(np.int64 if dtype == I32 else np.float64)
    oracle.block_scores_rows(dtype, x, c, L, listed, want)
    got = stale.cpu().numpy()
    keep = np.ones(nbk, dtype=bool)
    keep[listed] = False
    np.testing.assert_array_equal(got[keep], stale_h[keep])
    if dtype == I32:
        np.testing.assert_array_equal(got, want)
    else:
        np.testing.assert_allclose(got[listed].astype(np.float64), want[listed], rtol=1e-5, atol=0)
    # the listed scores are bit for bit those of the full scan
    full = scar.block_scores(dx, dc, L)
    assert torch.equal(full[idx_dev(listed).long()], stale[idx_dev(listed).long()])
    # an empty list changes nothing
    before = stale.clone()
    scar.block_scores_rows(dx, dc, L, torch.zeros(0, dtype=torch.int32, device=DEV), stale)
    assert torch.equal(before, stale)


def test_incremental_scores_track_the_full_scan_over_cycles():
    # a trainer that touches a few rows per iteration keeps `scores` current by rescoring the
    # touched rows and the saved ones: after every cycle they equal the full scan's, bit for bit
    L, nb, k = 100, 20_000, 500
    hx, hc = make_store(F32, L * nb, seed=5)
    x, c = to_dev(hx, F32), to_dev(hc, F32)
    ws = scar.new_workspace(nb, DEV)
    scores = scar.block_scores(x, c, L)
    g = torch.Generator(device=DEV)
    g.manual_seed(3)
    for it in range(4):
        touched = torch.randperm(nb, device=DEV, generator=g)[:1500].to(torch.int32)
        rows = x.view(nb, L)
        rows[touched.long()] += 1e-2 * torch.empty(1500, L, device=DEV).normal_(generator=g)
        scar.block_scores_rows(x, c, L, touched, scores)
        idx = scar.select_topk(scores, k, ws)
        scar.checkpoint_commit(x, c, L, idx)
        scar.block_scores_rows(x, c, L, idx, scores)            # saved blocks: distance 0 again
        assert torch.equal(scores, scar.block_scores(x, c, L))
        assert float(scores[idx.long()].abs().max()) == 0.0


SHORT_ROW_BYTES = [16, 32, 48, 80, 112, 128, 208, 400, 496, 512, 528,        # whole 16-byte steps
                   12, 20, 36, 100, 200, 404, 1000, 2004, 4004, 4100,        # whole 4-byte words
                   6, 18, 50, 202, 1002, 2002, 4090]                         # bfloat16 only


@pytest.mark.parametrize("dtype,row_bytes", [(d, rb) for d in (F32, BF16, I32) for rb in SHORT_ROW_BYTES
                                             if d == BF16 or rb % 4 == 0])
def test_block_scores_of_many_short_rows(dtype, row_bytes):
    # many rows of up to 512 bytes (up to 4 KiB when they are not whole 16-byte steps) are read
    # as contiguous runs of whole rows; the scores are the oracle's and, bit for bit, those of
    # the listed walk; last block whole, short by less than a 16-byte step, and short by more
    L = row_bytes // (2 if dtype == BF16 else 4)
    sizes = [(4096, 0), (9001, 1), (20_011, L // 2 + 1), (70_000, L - 1)]
    for nb, cut in sizes if row_bytes <= 1024 else [(4096, 0), (6001, 1), (9011, L // 2 + 1)]:
        n = L * nb - cut
        x, c = make_store(dtype, n, seed=row_bytes + nb)
        dx, dc = to_dev(x, dtype), to_dev(c, dtype)
        print("short rows dtype=%d L=%d nb=%d cut=%d" % (dtype, L, nb, cut), flush=True)
        s = scar.block_scores(dx, dc, L)
        assert s.numel() == nb
        assert_scores_match(s, oracle.block_scores(dtype, x, c, L), dtype)
        listed = torch.full_like(s, -1)
        scar.block_scores_rows(dx, dc, L, torch.randperm(nb, device=DEV).to(torch.int32), listed)
        assert torch.equal(s, listed)


@pytest.mark.parametrize("dtype", [F32, BF16, I32])
@pytest.mark.parametrize("L", [1, 2, 4])
def test_block_scores_of_rows_shorter_than_16_bytes(dtype, L):
    # per-scalar and per-pair selection: a lane scores several rows from one 16-byte step; every
    # remainder of the store after the last whole step (0 ... 7 elements, ragged last row) is tried
    for n in [1, 2, 3, 5, 8, 4096, 100_000, 100_001, 100_002, 100_003, 100_005, 100_007, 1_000_003]:
        x, c = make_store(dtype, n, seed=n + L)
        dx, dc = to_dev(x, dtype), to_dev(c, dtype)
        s = scar.block_scores(dx, dc, L)
        assert s.numel() == oracle.n_blocks_of(n, L)
        assert_scores_match(s, oracle.block_scores(dtype, x, c, L), dtype)
        listed = torch.full_like(s, -1)                      # the listed walk agrees bit for bit
        scar.block_scores_rows(dx, dc, L, torch.arange(s.numel(), dtype=torch.int32, device=DEV), listed)
        assert torch.equal(s, listed)


@pytest.mark.parametrize("dtype", [F32, BF16, I32, wl.F32_BF16C])
@pytest.mark.parametrize("nb,L,off", [(16, 1 << 20, 0), (5, 700_001, 0), (3, 1 << 18, 1), (40, 65_536 + 24, 4),
                                      (2048, 1 << 16, 0), (16_384, 1 << 14, 0), (9000, 16_390, 3),
                                      (2, 5_000_001, 0)])
def test_block_scores_of_a_few_very_long_blocks(dtype, nb, L, off):
    # fewer blocks than the chip has room for workgroups: scored in pieces, many workgroups per
    # block (a ragged last block, bases off the 16-byte grid, rows that are not whole steps),
    # and the listed call must give the same bits
    if dtype == BF16 and L * 2 < 64 * 1024:
        L *= 2
    n = L * nb - L // 3
    xdt = cdt = dtype
    if dtype == wl.F32_BF16C:             # float32 x against a bfloat16 checkpoint
        xdt, cdt = F32, BF16
    hx, hc = make_store(xdt, n, seed=nb + L)
    if dtype == wl.F32_BF16C:
        hc = wl.f32_to_bf16_bits(hc)
    x = to_dev(np.concatenate([np.zeros(off, dtype=hx.dtype), hx]), xdt)[off:]
    c = to_dev(np.concatenate([np.zeros(off, dtype=hc.dtype), hc]), cdt)[off:]
    print("giant blocks dtype=%d nb=%d L=%d off=%d" % (dtype, nb, L, off), flush=True)
    oracle.set_num_threads(8)
    try:
        want = oracle.block_scores(dtype, hx, hc, L)
    finally:
        oracle.set_num_threads(1)
    s = scar.block_scores(x, c, L)
    assert_scores_match(s, want, dtype)
    listed = torch.full_like(s, -1)
    order = torch.randperm(nb, device=DEV).to(torch.int32)
    scar.block_scores_rows(x, c, L, order, listed)
    assert torch.equal(s, listed)
    some = torch.full_like(s, -7)
    scar.block_scores_rows(x, c, L, order[: max(1, nb // 3)], some)
    chosen = order[: max(1, nb // 3)].long()
    assert torch.equal(some[chosen], s[chosen])
    rest = torch.ones(nb, dtype=torch.bool, device=DEV)
    rest[chosen] = False
    assert bool((some[rest] == -7).all())


@pytest.mark.parametrize("dtype", [F32, BF16, wl.F32_BF16C])
@pytest.mark.parametrize("L,nb", [(8, 3000), (100, 2000), (1024, 600), (5000, 40_000 // 100)])
def test_nan_inf_and_negative_zero_in_the_store(dtype, L, nb):
    # NaN, +-Inf and -0 as *elements of x and c*: scores follow IEEE (NaN or Inf), the selection
    # ranks NaN above Inf above every number, commit and recovery move the bit patterns as they
    # are (a bfloat16 checkpoint rounds: NaN stays NaN, Inf stays Inf), norms become NaN or Inf
    r = np.random.default_rng(L + nb + dtype)
    n = L * nb - L // 2
    hx, hc = make_store(F32, n, seed=L)
    specials = np.array([np.nan, np.inf, -np.inf, -0.0, 0.0], dtype=np.float32)
    for arr in (hx, hc):
        where = r.choice(n, size=nb // 4, replace=False)
        arr[where] = r.choice(specials, size=where.size)
    both = r.choice(n, size=nb // 8, replace=False)          # Inf - Inf = NaN, Inf - (-Inf) = Inf
    hx[both], hc[both] = np.inf, r.choice(np.array([np.inf, -np.inf], dtype=np.float32), size=both.size)
    if dtype == BF16:
        hx, hc = wl.f32_to_bf16_bits(hx), wl.f32_to_bf16_bits(hc)
        x, c = to_dev(hx, BF16), to_dev(hc, BF16)
    elif dtype == wl.F32_BF16C:
        hc = wl.f32_to_bf16_bits(hc)
        x, c = to_dev(hx, F32), to_dev(hc, BF16)
    else:
        x, c = to_dev(hx, F32), to_dev(hc, F32)
    nbk = oracle.n_blocks_of(n, L)
    ws = scar.new_workspace(nbk, DEV)
    print("non-finite store dtype=%d L=%d nb=%d" % (dtype, L, nbk), flush=True)

    s = scar.block_scores(x, c, L)
    s_ref = oracle.block_scores(dtype, hx, hc, L)
    s_h = s.cpu().numpy()
    assert np.isnan(s_ref).sum() > 0 and np.isinf(s_ref).sum() > 0
    np.testing.assert_array_equal(np.isnan(s_h), np.isnan(s_ref))
    np.testing.assert_array_equal(np.isposinf(s_h), np.isposinf(s_ref))
    fin = np.isfinite(s_ref)
    np.testing.assert_allclose(s_h[fin].astype(np.float64), s_ref[fin], rtol=REL_TOL, atol=0)

    n_nan, n_big = int(np.isnan(s_ref).sum()), int((~fin).sum())
    for k in sorted({1, n_nan, n_nan + 1, n_big, n_big + 5, nbk // 2}):
        idx = scar.select_topk(s, k, ws)
        np.testing.assert_array_equal(idx_host(idx), oracle.select_topk(s_h.astype(np.float64), k))
        if k in (n_nan, n_big):       # exactly the NaN blocks / the non-finite blocks: the same in float64
            np.testing.assert_array_equal(idx_host(idx), oracle.select_topk(s_ref, k))

    def as_bits(a):
        return a.view(np.uint32) if a.dtype == np.float32 else a

    scar.checkpoint_commit(x, c, L, idx)
    oracle.checkpoint_commit(dtype, hx, hc, L, idx_host(idx))
    np.testing.assert_array_equal(as_bits(to_host(c)), as_bits(hc))
    np.testing.assert_array_equal(as_bits(to_host(x)), as_bits(hx))

    lost = np.sort(r.choice(nbk, size=nbk // 3, replace=False)).astype(np.uint32)
    got = scar.read_norm(scar.partial_recover(x, c, L, idx_dev(lost), ws))
    want = oracle.partial_recover(dtype, hx, hc, L, lost)
    for g, w in zip(got[:2], want[:2]):
        assert (np.isnan(w) and np.isnan(g)) or (np.isinf(w) and g == w) or abs(g - w) <= REL_TOL * abs(w)
    np.testing.assert_array_equal(as_bits(to_host(x)), as_bits(hx))
    # a list without the poisoned blocks gives a finite norm again
    clean = np.nonzero(np.isfinite(oracle.block_scores(dtype, hx, hc, L)))[0].astype(np.uint32)
    got = scar.read_norm(scar.perturbation_norm(x, c, L, idx_dev(clean), ws))
    assert_norm_matches(got, oracle.perturbation_norm(dtype, hx, hc, L, clean), F32)


@pytest.mark.parametrize("dtype", [F32, BF16, I32, wl.F32_BF16C])
@pytest.mark.parametrize("nb,L,n_list", [(16, 1 << 20, 2), (5, 700_001, 1), (9, 300_000, 9), (300, 20_000, 70)])
def test_commit_and_recover_of_a_few_very_long_rows(dtype, nb, L, n_list):
    # a short list of rows that are cut into thousands of 4 KiB pieces: the pieces, not the list,
    # are spread over the chip; every byte against the oracle, norm alone = norm with recovery
    r = np.random.default_rng(nb + L)
    n = L * nb - L // 3
    xdt = F32 if dtype == wl.F32_BF16C else dtype
    hx, hc = make_store(xdt, n, seed=nb + L + 1)
    if dtype == wl.F32_BF16C:
        hc = wl.f32_to_bf16_bits(hc)
    x, c = to_dev(hx, xdt), to_dev(hc, BF16 if dtype == wl.F32_BF16C else dtype)
    ws = scar.new_workspace(nb, DEV)
    norm_kind = I32 if dtype == I32 else F32
    print("long rows dtype=%d nb=%d L=%d list=%d" % (dtype, nb, L, n_list), flush=True)
    K = np.sort(np.unique(np.append(r.choice(nb, size=n_list, replace=False), nb - 1))).astype(np.uint32)
    st = torch.zeros(K.size * L, dtype=c.dtype, device=DEV)
    scar.checkpoint_commit(x, c, L, idx_dev(K), st)
    hst = np.zeros(K.size * L, dtype=hc.dtype)
    oracle.checkpoint_commit(dtype, hx, hc, L, K, hst)
    np.testing.assert_array_equal(to_host(c), hc)
    np.testing.assert_array_equal(to_host(st), hst)
    S = np.sort(np.unique(np.append(r.choice(nb, size=n_list, replace=False), nb - 1))).astype(np.uint32)
    hx2 = hx.copy()
    hx2[: n // 2] += hx2.dtype.type(1)        # move x away from c again, so the lost rows differ
    x = to_dev(hx2, xdt)
    pre = scar.read_norm(scar.perturbation_norm(x, c, L, idx_dev(S), ws))
    got = scar.read_norm(scar.partial_recover(x, c, L, idx_dev(S), ws))
    want = oracle.partial_recover(dtype, hx2, hc, L, S)
    assert_norm_matches(got, want, norm_kind)
    assert pre == got
    np.testing.assert_array_equal(to_host(x), hx2)
    np.testing.assert_array_equal(to_host(c), hc)


def test_block_scores_int_extremes():
    hi = np.full(2048, np.iinfo(np.int32).max, dtype=np.int32)
    lo = np.full(2048, np.iinfo(np.int32).min, dtype=np.int32)
    got = scar.block_scores(to_dev(hi, I32), to_dev(lo, I32), 1024)
    np.testing.assert_array_equal(got.cpu().numpy(), [1024 * (2 ** 32 - 1)] * 2)


@pytest.mark.parametrize("n,kind", [(1, "rand"), (7, "rand"), (2048, "rand"), (2049, "rand"),
                                    (8192, "ties"), (8193, "ties"), (5000, "special"), (8000, "zeros"),
                                    (10_000, "rand"), (16_384, "rand"), (16_384, "ties"), (16_385, "ties"),
                                    (12_000, "special"), (16_384, "zeros"), (32_769, "rand"),
                                    (300_000, "rand"), (300_000, "ties"),
                                    (50_000, "zeros"), (70_000, "special")])
def test_select_topk_float(n, kind):
    r = np.random.default_rng(n)
    if kind == "rand":
        s = (r.lognormal(-3, 2, size=n)).astype(np.float32)
    elif kind == "ties":
        s = r.integers(0, 40, size=n).astype(np.float32) * 0.25
    elif kind == "zeros":
        s = np.zeros(n, dtype=np.float32)
        s[r.choice(n, size=100, replace=False)] = 1.0
    else:
        s = r.normal(size=n).astype(np.float32)          # negative scores are ordered too
        s[r.choice(n, size=50, replace=False)] = np.nan
        s[r.choice(n, size=50, replace=False)] = np.inf
        s[r.choice(n, size=50, replace=False)] = -0.0
        s[r.choice(n, size=50, replace=False)] = 0.0
        s[r.choice(n, size=5, replace=False)] = -np.inf
    d = torch.from_numpy(s).to(DEV)
    ws = scar.new_workspace(n, DEV)
    ks = sorted({0, 1, n // 10, n // 2, n - 1, n, min(n, 137)})
    for k in ks:
        print("select float n=%d kind=%s k=%d" % (n, kind, k), flush=True)
        got = idx_host(scar.select_topk(d, k, ws))
        np.testing.assert_array_equal(got, oracle.select_topk(s.astype(np.float64), k))


@pytest.mark.parametrize("n,hi", [(5, 3), (4097, 4), (8192, 2 ** 40), (100_000, 50), (100_000, 2 ** 40),
                                  (30_000, 1), (16_000, 2 ** 40), (16_384, 2 ** 40), (16_384, 7), (16_385, 2 ** 40)])
def test_select_topk_int(n, hi):
    r = np.random.default_rng(n + 1)
    s = r.integers(0, hi, size=n).astype(np.int64)
    if hi > 2 ** 32:
        s[::7] = -s[::7]                                   # the key order covers negatives too
        s[5] = np.iinfo(np.int64).max
        s[6] = np.iinfo(np.int64).min
    d = torch.from_numpy(s).to(DEV)
    ws = scar.new_workspace(n, DEV)
    for k in sorted({0, 1, n // 20, n // 2, n - 1, n}):
        print("select int n=%d hi=%d k=%d" % (n, hi, k), flush=True)
        got = idx_host(scar.select_topk(d, k, ws))
        np.testing.assert_array_equal(got, oracle.select_topk(s, k))


@pytest.mark.parametrize("n,k", [(5_000_000, 1234), (5_000_000, 2_500_000), (33_554_432 + 5000, 40_000)])
def test_select_topk_many_tiles(n, k):
    # thousands of tiles: long chains of look-back windows in the ordered write
    r = np.random.default_rng(n + k)
    s = r.integers(0, 1 << 20, size=n).astype(np.float32)       # many ties
    d = torch.from_numpy(s).to(DEV)
    ws = scar.new_workspace(n, DEV)
    print("select many tiles n=%d k=%d" % (n, k), flush=True)
    got = idx_host(scar.select_topk(d, k, ws))
    oracle.set_num_threads(1)
    np.testing.assert_array_equal(got, oracle.select_topk(s.astype(np.float64), k))
    m = (s > (1 << 19)).astype(np.uint8)
    out, cnt = scar.mask_to_indices(torch.from_numpy(m).to(DEV), ws)
    want = oracle.mask_to_indices(m)
    assert int(cnt.item()) == want.size
    np.testing.assert_array_equal(idx_host(out)[: want.size], want)


@pytest.mark.parametrize("n,hi,bound", [(100_000, 50, 49), (100_000, 50, 1000 * 2 ** 32), (30_000, 2 ** 21, 2 ** 21),
                                        (30_000, 2 ** 40, 2 ** 33 - 1), (20_000, 2 ** 40, 2 ** 54), (16_000, 300, 10 ** 6),
                                        (250_000, 2 ** 62, 2 ** 62), (1_200_000, 5000, 2 ** 22 - 1), (70_000, 100, 20)])
def test_select_topk_bounded(n, hi, bound):
    # 64-bit integer scores with an upper bound known on the host: fewer digit passes, the same
    # choice as the oracle makes on the scores taken into [0, bound] (a negative score counts
    # as 0 and one above the bound as the bound)
    r = np.random.default_rng(n + 3)
    s = r.integers(0, hi, size=n).astype(np.int64)
    s[::11] = -s[::11]
    d = torch.from_numpy(s).to(DEV)
    ws = scar.new_workspace(n, DEV)
    clamped = np.clip(s, 0, bound)
    for k in sorted({1, n // 20, n // 2, n - 1}):
        print("select bounded n=%d hi=%d bound=%d k=%d" % (n, hi, bound, k), flush=True)
        got = idx_host(scar.select_topk_bounded(d, k, bound, ws))
        np.testing.assert_array_equal(got, oracle.select_topk(clamped, k))
    # float scores ignore the bound
    f = r.random(n).astype(np.float32)
    got = idx_host(scar.select_topk_bounded(torch.from_numpy(f).to(DEV), n // 3, 5, ws))
    np.testing.assert_array_equal(got, oracle.select_topk(f.astype(np.float64), n // 3))


@pytest.mark.parametrize("limit", [0, 1])
def test_ordered_write_when_no_workgroup_waits_for_another(limit):
    # the chained scan's bounded wait, forced from the host to give up at once: every workgroup
    # then counts the tiles before its own itself; results must not change
    r = np.random.default_rng(limit)
    scar.set_lookback_spin_limit(limit)
    try:
        # 4.3 M keys: more tiles than workgroups, so each workgroup owns two tiles and counts them first
        for n, k in ((300_000, 30_000), (1_000_000, 999_999), (20_000, 1), (4_300_000, 500_000)):
            print("forced fallback limit=%d n=%d k=%d" % (limit, n, k), flush=True)
            s = r.integers(0, 30, size=n).astype(np.float32)
            ws = scar.new_workspace(n, DEV)
            got = idx_host(scar.select_topk(torch.from_numpy(s).to(DEV), k, ws))
            np.testing.assert_array_equal(got, oracle.select_topk(s.astype(np.float64), k))
            m = (s > 20).astype(np.uint8)
            out, cnt = scar.mask_to_indices(torch.from_numpy(m).to(DEV), ws)
            want = oracle.mask_to_indices(m)
            assert int(cnt.item()) == want.size
            np.testing.assert_array_equal(idx_host(out)[: want.size], want)
            si = r.integers(0, 5, size=n).astype(np.int64)
            got = idx_host(scar.select_topk(torch.from_numpy(si).to(DEV), k, ws))
            np.testing.assert_array_equal(got, oracle.select_topk(si, k))
    finally:
        scar.set_lookback_spin_limit(1 << 16)


@pytest.mark.parametrize("groups,limit", [(1, 1 << 16), (3, 1 << 16), (7, 1 << 16), (64, 1 << 16), (5, 0)])
def test_ordered_write_over_spans_of_tiles(groups, limit):
    # long key arrays give every workgroup a span of tiles; a small number of workgroups, set
    # from the host, makes short arrays take the same paths: spans of up to 489 tiles, the first
    # 32 of them placed from classes kept while counting, the rest read again; with and without
    # a look-back that gives up at once
    r = np.random.default_rng(groups)
    scar.set_compaction_groups(groups)
    scar.set_lookback_spin_limit(limit)
    try:
        for n, k in ((1_000_000, 100_000), (300_001, 300_000), (70_000, 1)):
            print("spans groups=%d limit=%d n=%d k=%d" % (groups, limit, n, k), flush=True)
            s = r.integers(0, 50, size=n).astype(np.float32)
            ws = scar.new_workspace(n, DEV)
            got = idx_host(scar.select_topk(torch.from_numpy(s).to(DEV), k, ws))
            np.testing.assert_array_equal(got, oracle.select_topk(s.astype(np.float64), k))
            f = r.random(n).astype(np.float32)
            got = idx_host(scar.select_topk(torch.from_numpy(f).to(DEV), k, ws))
            np.testing.assert_array_equal(got, oracle.select_topk(f.astype(np.float64), k))
            m = (s > 30).astype(np.uint8)
            out, cnt = scar.mask_to_indices(torch.from_numpy(m).to(DEV), ws)
            want = oracle.mask_to_indices(m)
            assert int(cnt.item()) == want.size
            np.testing.assert_array_equal(idx_host(out)[: want.size], want)
            si = r.integers(0, 5, size=n).astype(np.int64)
            got = idx_host(scar.select_topk(torch.from_numpy(si).to(DEV), k, ws))
            np.testing.assert_array_equal(got, oracle.select_topk(si, k))
    finally:
        scar.set_compaction_groups(0)
        scar.set_lookback_spin_limit(1 << 16)


@pytest.mark.parametrize("dtype", [F32, BF16, I32])
@pytest.mark.parametrize("L", [1, 6, 100, 1024, 4100, 20000])
def test_commit_and_recover(dtype, L):
    nb = 300 if L < 5000 else 40
    n_elems = L * nb - (L // 2)
    x, c = make_store(dtype, n_elems, seed=7 * L + dtype)
    nbk = oracle.n_blocks_of(n_elems, L)
    r = np.random.default_rng(L)
    K = r.permutation(nbk)[: nbk // 3].astype(np.uint32)            # unsorted, may hold the tail
    K[0] = nbk - 1
    K = np.unique(K)
    r.shuffle(K)
    print("commit/recover dtype=%d L=%d" % (dtype, L), flush=True)
    dx, dc = to_dev(x, dtype), to_dev(c, dtype)
    st = torch.zeros(K.size * L, dtype=dx.dtype, device=DEV)
    scar.checkpoint_commit(dx, dc, L, idx_dev(K), st)
    hst = np.zeros(K.size * L, dtype=x.dtype)
    x0 = x.copy()
    oracle.checkpoint_commit(dtype, x, c, L, K, hst)
    np.testing.assert_array_equal(to_host(dc), c)
    np.testing.assert_array_equal(to_host(dx), x0)
    np.testing.assert_array_equal(to_host(st), hst)

    S = np.sort(r.permutation(nbk)[: nbk // 2]).astype(np.uint32)
    S[-1] = nbk - 1
    S = np.unique(S)
    ws = scar.new_workspace(nbk, DEV)
    pre = scar.read_norm(scar.perturbation_norm(dx, dc, L, idx_dev(S), ws))
    nrm = scar.read_norm(scar.partial_recover(dx, dc, L, idx_dev(S), ws))
    want = oracle.partial_recover(dtype, x, c, L, S)
    assert_norm_matches(nrm, want, dtype)
    assert pre == nrm                                                 # same kernel, same order
    np.testing.assert_array_equal(to_host(dx), x)
    np.testing.assert_array_equal(to_host(dc), c)
    # recovering again changes nothing and measures zero
    again = scar.read_norm(scar.partial_recover(dx, dc, L, idx_dev(S), ws))
    assert again == (0.0, 0.0, 0)
    # without the norm no workspace is needed
    scar.partial_recover(dx, dc, L, idx_dev(S), None, want_norm=False)
    np.testing.assert_array_equal(to_host(dx), x)


@pytest.mark.parametrize("dtype,L,nb", [(F32, 24, 600_000), (BF16, 40, 600_000), (I32, 8, 1_500_000),
                                        (F32, 1024, 40_000), (I32, 7, 300_000)])
def test_recover_and_norm_over_long_index_lists(dtype, L, nb):
    # Long index lists run the recovery kernel with larger workgroups (several groups per
    # workgroup, every group width); results must not depend on that.
    n_elems = L * nb - (L // 2)
    x, c = make_store(dtype, n_elems, seed=3 * L + dtype)
    r = np.random.default_rng(L + nb)
    S = np.unique(np.append(r.permutation(nb)[: (3 * nb) // 4], nb - 1)).astype(np.uint32)
    r.shuffle(S)                                                      # unsorted, holds the tail block
    print("long list dtype=%d L=%d n_idx=%d" % (dtype, L, S.size), flush=True)
    dx, dc = to_dev(x, dtype), to_dev(c, dtype)
    ws = scar.new_workspace(nb, DEV)
    oracle.set_num_threads(8)
    try:
        pre = scar.read_norm(scar.perturbation_norm(dx, dc, L, idx_dev(S), ws))
        full = scar.read_norm(scar.perturbation_norm(dx, dc, L, None, ws))
        assert_norm_matches(full, oracle.perturbation_norm(dtype, x, c, L), dtype)
        nrm = scar.read_norm(scar.partial_recover(dx, dc, L, idx_dev(S), ws))
        want = oracle.partial_recover(dtype, x, c, L, S)
    finally:
        oracle.set_num_threads(1)
    assert_norm_matches(nrm, want, dtype)
    assert pre == nrm
    np.testing.assert_array_equal(to_host(dx), x)
    np.testing.assert_array_equal(to_host(dc), c)


@pytest.mark.parametrize("dtype", [F32, I32])
def test_invariants_on_the_gpu(dtype):
    L = 96
    x, c = make_store(dtype, L * 1000 + 5, seed=3)
    nb = 1001
    dx, dc = to_dev(x, dtype), to_dev(c, dtype)
    ws = scar.new_workspace(nb, DEV)
    everything = idx_dev(np.arange(nb))
    # empty lost set: x untouched, norm zero
    empty = torch.zeros(0, dtype=torch.int32, device=DEV)
    assert scar.read_norm(scar.partial_recover(dx, dc, L, empty, ws)) == (0.0, 0.0, 0)
    assert scar.read_norm(scar.perturbation_norm(dx, dc, L, empty, ws)) == (0.0, 0.0, 0)
    np.testing.assert_array_equal(to_host(dx), x)
    # norms over a partition of the blocks add up to the full norm (Appendix A.4)
    full = scar.read_norm(scar.perturbation_norm(dx, dc, L, None, ws))
    parts = np.array_split(np.random.default_rng(0).permutation(nb), 5)
    tot = [scar.read_norm(scar.perturbation_norm(dx, dc, L, idx_dev(np.sort(p)), ws)) for p in parts]
    if dtype == I32:
        assert sum(t[2] for t in tot) == full[2]
    else:
        assert abs(sum(t[0] for t in tot) - full[0]) <= 1e-12 * full[0]
    # k = all: checkpoint equals x and the perturbation vanishes
    scar.checkpoint_commit(dx, dc, L, everything)
    assert torch.equal(dx, dc)
    assert scar.read_norm(scar.perturbation_norm(dx, dc, L, None, ws)) == (0.0, 0.0, 0)


@pytest.mark.parametrize("n,p", [(0, 0.5), (1, 1.0), (2047, 0.3), (2048, 0.0), (100_001, 0.125), (100_001, 1.0)])
def test_mask_to_indices(n, p):
    m = (np.random.default_rng(n).random(n) < p).astype(np.uint8) * 3
    ws = scar.new_workspace(n, DEV)
    out, cnt = scar.mask_to_indices(torch.from_numpy(m).to(DEV), ws)
    want = oracle.mask_to_indices(m)
    assert int(cnt.item()) == want.size
    np.testing.assert_array_equal(idx_host(out)[: want.size], want)


def test_results_are_reproducible_bit_for_bit():
    w = wl.flat_like(n_elems=1 << 20)
    s = DeviceStore(w)
    a = scar.block_scores(s.x, s.c, s.L)
    b = scar.block_scores(s.x, s.c, s.L)
    assert torch.equal(a, b)
    n1 = scar.read_norm(scar.perturbation_norm(s.x, s.c, s.L, None, s.ws))
    n2 = scar.read_norm(scar.perturbation_norm(s.x, s.c, s.L, None, s.ws))
    assert n1 == n2
    i1 = scar.select_topk(a, w.k, s.ws).clone()
    i2 = scar.select_topk(a, w.k, s.ws)
    assert torch.equal(i1, i2)


def test_argument_errors_are_reported_not_launched():
    x = torch.zeros(1024, dtype=torch.float32, device=DEV)
    c = torch.zeros(1024, dtype=torch.float32, device=DEV)
    ws = scar.new_workspace(8, DEV)
    s = scar.block_scores(x, c, 128)
    with pytest.raises(scar.ScarError):
        scar.block_scores(x, c, 0)
    with pytest.raises(scar.ScarError):
        scar.select_topk(s, 9, ws)
    with pytest.raises(scar.ScarError) as e:
        scar.select_topk(s, 2, ws[:1024])
    assert e.value.status == -2
    with pytest.raises(scar.ScarError):
        scar.select_topk(s, 2, ws[1:])
    # the binding refuses index lists and outputs of the wrong type before calling
    with pytest.raises(TypeError):
        scar.checkpoint_commit(x, c, 128, torch.zeros(2, dtype=torch.int64, device=DEV))
    with pytest.raises(TypeError):
        scar.partial_recover(x, c, 128, torch.zeros(2, dtype=torch.int64, device=DEV), ws)
    with pytest.raises(ValueError):
        scar.block_scores(x, c, 128, out=torch.zeros(3, device=DEV))
    with pytest.raises(ValueError):
        scar.select_topk(s, 4, ws, out=torch.zeros(2, dtype=torch.int32, device=DEV))
    torch.cuda.synchronize()


@pytest.mark.parametrize("n,k", [(1, 1), (10, 4), (8192, 1000), (8193, 8193), (100_000, 12_500),
                                 (1 << 20, 104_858)])
def test_comparison_strategies(n, k):
    # Section 5.4's round-robin and random choices of K, index for index against the oracle
    ws = scar.new_workspace(n, DEV)
    for cursor in (0, n - 1, 3 * n + k // 2, n - k):
        print("round n=%d k=%d cursor=%d" % (n, k, cursor), flush=True)
        got = idx_host(scar.select_round(n, k, cursor, DEV))
        np.testing.assert_array_equal(got, oracle.select_round(n, k, cursor))
    for seed, draw in ((0, 0), (7, 3), (2 ** 40 + 5, 2 ** 33 + 1)):
        print("random n=%d k=%d seed=%d draw=%d" % (n, k, seed, draw), flush=True)
        got = idx_host(scar.select_random(n, k, seed, draw, ws))
        np.testing.assert_array_equal(got, oracle.select_random(n, k, seed, draw))


def test_cycle_replays_correctly_from_a_hip_graph():
    # The library enqueues only kernels (no allocation, no memset, no synchronisation), so a
    # whole cycle can be captured once and replayed.  Every replay - with the program's own
    # eager work and synchronisations in between - must give what the eager calls give.
    # (2^26 elements: large enough for the launches that ask for unused LDS to limit the
    # workgroups per compute unit.)
    w = wl.flat_like(n_elems=1 << 26)
    L, nb, k = w.block_len, w.n_blocks, w.k
    x, c = to_dev(w.x, w.dtype), to_dev(w.c, w.dtype)
    ws = scar.new_workspace(nb, DEV)
    scores = torch.empty(nb, dtype=torch.float32, device=DEV)
    idx = torch.empty(k, dtype=torch.int32, device=DEV)
    norm = torch.zeros(3, dtype=torch.float64, device=DEV)
    lost = idx_dev(w.lost)

    def cycle(x_, c_, scores_, idx_, norm_, ws_):
        scar.block_scores(x_, c_, L, out=scores_)
        scar.select_topk(scores_, k, ws_, out=idx_)
        scar.checkpoint_commit(x_, c_, L, idx_)
        scar.partial_recover(x_, c_, L, lost, ws_, norm_out=norm_)

    x0, c0 = x.clone(), c.clone()
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):                      # warm-up outside the capture
        cycle(x, c, scores, idx, norm, ws)
    torch.cuda.current_stream().wait_stream(side)
    torch.cuda.synchronize()
    graph = torch.cuda.CUDAGraph()
    x.copy_(x0), c.copy_(c0)
    with torch.cuda.graph(graph):
        cycle(x, c, scores, idx, norm, ws)
    torch.cuda.synchronize()

    ws2 = scar.new_workspace(nb, DEV)
    s2, i2, n2 = torch.empty_like(scores), torch.empty_like(idx), torch.zeros_like(norm)
    g = torch.Generator(device=DEV)
    g.manual_seed(1)
    state_x, state_c = x0.clone(), c0.clone()
    for rep in range(4):
        print("graph replay %d" % rep, flush=True)
        x.copy_(state_x), c.copy_(state_c)
        graph.replay()
        torch.cuda.synchronize()
        x2, c2 = state_x.clone(), state_c.clone()
        cycle(x2, c2, s2, i2, n2, ws2)                 # the same cycle, eagerly
        torch.cuda.synchronize()
        assert torch.equal(scores, s2) and torch.equal(idx, i2)
        assert torch.equal(x, x2) and torch.equal(c, c2) and torch.equal(norm, n2)
        # eager work between replays: the next state drifts from this one
        state_x = x2 + 1e-3 * torch.empty_like(x2).normal_(generator=g) * (torch.rand(1, device=DEV) + 0.5)
        state_c = c2
        torch.cuda.synchronize()


def test_sixty_random_stores_incl_bf16_checkpoint():
    # 60 seeded random stores: element type, block length, size (ragged or not), k and lost
    # set all drawn at random; one full cycle each, compared with the oracle call by call
    r = np.random.default_rng(2024)
    for case in range(60):
        dtype = int(r.choice([F32, BF16, I32, wl.F32_BF16C]))
        L = int(r.choice([1, 2, 3, 4, 5, 7, 8, 12, 16, 31, 32, 33, 64, 100, 128, 255, 256, 500, 1000, 1024,
                          2048, 3000, 4096, 9000]))
        nb = int(r.integers(1, 400))
        n = max(1, L * nb - int(r.integers(0, L)))
        nb = oracle.n_blocks_of(n, L)
        k = int(r.integers(0, nb + 1))
        lost = np.sort(r.choice(nb, size=int(r.integers(0, nb + 1)), replace=False)).astype(np.uint32)
        print("case %d dtype=%d L=%d n=%d k=%d lost=%d" % (case, dtype, L, n, k, lost.size), flush=True)
        if dtype == wl.F32_BF16C:
            hx, hc = make_store(F32, n, seed=case)
            hc = wl.f32_to_bf16_bits(hc)
            x, c = to_dev(hx, F32), to_dev(hc, BF16)
        else:
            hx, hc = make_store(dtype, n, seed=case)
            x, c = to_dev(hx, dtype), to_dev(hc, dtype)
        ws = scar.new_workspace(nb, DEV)
        s = scar.block_scores(x, c, L)
        s_ref = oracle.block_scores(dtype, hx, hc, L)
        assert_scores_match(s, s_ref, I32 if dtype == I32 else F32)
        idx = scar.select_topk(s, k, ws)
        assert_selection_matches(idx_host(idx), s.cpu().numpy(), s_ref, k)
        scar.checkpoint_commit(x, c, L, idx)
        oracle.checkpoint_commit(dtype, hx, hc, L, idx_host(idx))
        np.testing.assert_array_equal(to_host(c), hc)
        got = scar.read_norm(scar.partial_recover(x, c, L, idx_dev(lost), ws))
        want = oracle.partial_recover(dtype, hx, hc, L, lost)
        assert_norm_matches(got, want, I32 if dtype == I32 else F32)
        np.testing.assert_array_equal(to_host(x), hx)


@pytest.mark.parametrize("dtype", [F32, BF16, I32])
@pytest.mark.parametrize("off_x,off_c", [(1, 1), (3, 3), (1, 2), (0, 5), (4, 0)])
def test_misaligned_bases_whole_cycles(dtype, off_x, off_c):
    # x and c start off_x / off_c elements into their allocations: with equal offsets rows
    # are walked as head + 16-byte body + tail, with different ones element by element; both
    # must give the oracle's results for every row length, with and without staging rows
    r = np.random.default_rng(100 * off_x + off_c)
    for L in (1, 3, 4, 6, 9, 37, 100, 250, 1000, 1024, 4100):
        nb = 260 if L < 2000 else 40
        n = L * nb - L // 3
        nbk = oracle.n_blocks_of(n, L)
        hx, hc = make_store(dtype, n, seed=L + dtype)
        pad_x, pad_c = np.zeros(off_x, dtype=hx.dtype), np.zeros(off_c, dtype=hc.dtype)
        x = to_dev(np.concatenate([pad_x, hx]), dtype)[off_x:]
        c = to_dev(np.concatenate([pad_c, hc]), dtype)[off_c:]
        print("misaligned dtype=%d L=%d offsets=(%d,%d)" % (dtype, L, off_x, off_c), flush=True)
        ws = scar.new_workspace(nbk, DEV)
        s = scar.block_scores(x, c, L)
        assert_scores_match(s, oracle.block_scores(dtype, hx, hc, L), dtype)
        K = np.unique(np.append(r.permutation(nbk)[: nbk // 3], nbk - 1)).astype(np.uint32)
        r.shuffle(K)
        st = torch.zeros(K.size * L + 1, dtype=x.dtype, device=DEV)[1:]      # staging off the grid too
        scar.checkpoint_commit(x, c, L, idx_dev(K), st)
        hst = np.zeros(K.size * L, dtype=hx.dtype)
        oracle.checkpoint_commit(dtype, hx, hc, L, K, hst)
        np.testing.assert_array_equal(to_host(c.contiguous()), hc)
        np.testing.assert_array_equal(to_host(st.contiguous()), hst)
        S = np.unique(np.append(r.permutation(nbk)[: nbk // 2], nbk - 1)).astype(np.uint32)
        pre = scar.read_norm(scar.perturbation_norm(x, c, L, idx_dev(S), ws))
        got = scar.read_norm(scar.partial_recover(x, c, L, idx_dev(S), ws))
        want = oracle.partial_recover(dtype, hx, hc, L, S)
        assert_norm_matches(got, want, dtype)
        assert pre == got
        np.testing.assert_array_equal(to_host(x.contiguous()), hx)
        np.testing.assert_array_equal(to_host(c.contiguous()), hc)


def test_index_list_checker_counts_repeats_and_entries_out_of_range():
    r = np.random.default_rng(3)
    for nb, n in ((1, 1), (50, 50), (100_000, 60_000), (3_000_000, 1_500_000)):
        good = r.permutation(nb)[:n].astype(np.uint32)
        assert scar.check_indices(idx_dev(good), nb) == (0, 0)
        bad = good.copy()
        n_rep, n_out = min(7, n // 2), min(5, n // 3)
        if n_rep:
            bad[-n_rep:] = bad[:n_rep]                      # repeats of the first entries
        if n_out:
            bad[n_rep:n_rep + n_out] = nb + np.arange(n_out, dtype=np.uint32)
        print("check indices nb=%d n=%d" % (nb, n), flush=True)
        assert scar.check_indices(idx_dev(bad), nb) == (n_out, n_rep)
    assert scar.check_indices(torch.zeros(0, dtype=torch.int32, device=DEV), 10) == (0, 0)
    # the selection's own output always passes
    s = torch.rand(200_000, device=DEV)
    idx = scar.select_topk(s, 77_777, scar.new_workspace(200_000, DEV))
    assert scar.check_indices(idx, 200_000) == (0, 0)


@pytest.mark.parametrize("dtype", [F32, I32])
def test_out_of_range_list_entries_are_skipped(dtype):
    # documented device-side behaviour: an index >= n_blocks in a list is ignored
    L, nb = 64, 50
    hx, hc = make_store(dtype, L * nb, seed=77)
    x, c = to_dev(hx, dtype), to_dev(hc, dtype)
    ws = scar.new_workspace(nb, DEV)
    good = np.array([3, 49, 10], dtype=np.uint32)
    mixed = np.array([3, 50, 49, 0xFFFFFFFF, 10, 1 << 20], dtype=np.uint32)
    scar.checkpoint_commit(x, c, L, idx_dev(mixed))
    oracle.checkpoint_commit(dtype, hx, hc, L, good)
    np.testing.assert_array_equal(to_host(c), hc)
    lost_good = np.array([0, 7, 48], dtype=np.uint32)
    lost_mixed = np.array([0, 99, 7, 48, 50], dtype=np.uint32)
    got = scar.read_norm(scar.partial_recover(x, c, L, idx_dev(lost_mixed), ws))
    assert_norm_matches(got, oracle.partial_recover(dtype, hx, hc, L, lost_good), dtype)
    np.testing.assert_array_equal(to_host(x), hx)


@pytest.mark.parametrize("kind", ["by_layer", "total_variation", "bf16_checkpoint", "few_long_blocks",
                                  "counts_bounded_static"])
def test_other_cycles_replay_correctly_from_a_hip_graph(kind):
    # the by-layer, total-variation and reduced-precision paths are kernels only as well
    r = np.random.default_rng(5)
    if kind == "by_layer":
        w = wl.layers_like(wl.mixed_layer_sizes(120, 5_000_000, seed=3), seed=4, fraction=0.2, n_lost=30)
        x, c = to_dev(w.x, w.dtype), to_dev(w.c, w.dtype)
        off = torch.from_numpy(w.offsets.astype(np.int64)).to(DEV)
        nb, k, lost = w.n_blocks, w.k, idx_dev(w.lost)
        ws, ws_sel = scar.new_var_workspace(nb, DEV), scar.new_workspace(nb, DEV)

        def cycle(x_, c_):
            s = scar.var_block_scores(x_, c_, off, ws)
            idx = scar.select_topk(s, k, ws_sel)
            scar.var_checkpoint_commit(x_, c_, off, idx, ws)
            return s, idx, scar.var_partial_recover(x_, c_, off, lost, ws)
    elif kind == "total_variation":
        L, nb = 100, 30_000
        hx = r.dirichlet(np.full(L, 0.3), size=nb).astype(np.float32).ravel()
        hc = r.dirichlet(np.full(L, 0.3), size=nb).astype(np.float32).ravel()
        x, c = to_dev(hx, F32), to_dev(hc, F32)
        wts = torch.from_numpy(r.integers(5, 2000, size=nb).astype(np.float32)).to(DEV)
        k, lost = nb // 8, idx_dev(wl.random_lost_blocks(nb, nb // 4, 9))
        ws = scar.new_workspace(nb, DEV)

        def cycle(x_, c_):
            s = scar.tv_block_scores(x_, c_, L, wts)
            idx = scar.select_topk(s, k, ws)
            scar.checkpoint_commit(x_, c_, L, idx)
            return s, idx, scar.tv_partial_recover(x_, c_, L, lost, ws, wts)
    elif kind == "few_long_blocks":
        # scored in pieces through the library's fixed array, copied in pieces spread over the XCDs
        L, nb = 1 << 20, 12
        hx, hc = make_store(F32, L * nb - 77, seed=8)
        x, c = to_dev(hx, F32), to_dev(hc, F32)
        k, lost = 3, idx_dev(np.array([1, 7, 11], dtype=np.uint32))
        ws = scar.new_workspace(nb, DEV)

        def cycle(x_, c_):
            s = scar.block_scores(x_, c_, L)
            idx = scar.select_topk(s, k, ws)
            scar.checkpoint_commit(x_, c_, L, idx)
            return s, idx, scar.partial_recover(x_, c_, L, lost, ws)
    elif kind == "counts_bounded_static":
        # an int32 count table: bounded 64-bit selection, and the selection on the library's own scratch
        L, nb = 200, 60_000
        hx, hc = make_store(I32, L * nb, seed=8)
        x, c = to_dev(hx, I32), to_dev(hc, I32)
        k, lost = nb // 10, idx_dev(wl.random_lost_blocks(nb, nb // 8, 9))
        ws = scar.new_workspace(nb, DEV)
        idx_static = torch.empty(k, dtype=torch.int32, device=DEV)

        def cycle(x_, c_):
            s = scar.block_scores(x_, c_, L)
            idx = scar.select_topk_bounded(s, k, L * (2 ** 32 - 1), ws)
            scar.select_topk_static(s, k, out=idx_static)
            scar.checkpoint_commit(x_, c_, L, idx_static)
            return s, idx, scar.partial_recover(x_, c_, L, lost, ws)
    else:
        L, nb = 1024, 4096
        hx, hc = make_store(F32, L * nb, seed=8)
        x, c = to_dev(hx, F32), to_dev(wl.f32_to_bf16_bits(hc), BF16)
        k, lost = nb // 10, idx_dev(wl.random_lost_blocks(nb, nb // 8, 9))
        ws = scar.new_workspace(nb, DEV)

        def cycle(x_, c_):
            s = scar.block_scores(x_, c_, L)
            idx = scar.select_topk(s, k, ws)
            scar.checkpoint_commit(x_, c_, L, idx)
            return s, idx, scar.partial_recover(x_, c_, L, lost, ws)

    x0, c0 = x.clone(), c.clone()
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):                      # warm-up outside the capture
        cycle(x, c)
    torch.cuda.current_stream().wait_stream(side)
    torch.cuda.synchronize()
    x.copy_(x0), c.copy_(c0)
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph):
        s_g, idx_g, norm_g = cycle(x, c)
    torch.cuda.synchronize()
    state_x, state_c = x0.clone(), c0.clone()
    g = torch.Generator(device=DEV)
    g.manual_seed(2)
    for rep in range(3):
        print("%s graph replay %d" % (kind, rep), flush=True)
        x.copy_(state_x), c.copy_(state_c)
        graph.replay()
        torch.cuda.synchronize()
        x2, c2 = state_x.clone(), state_c.clone()
        s2, idx2, norm2 = cycle(x2, c2)
        torch.cuda.synchronize()
        assert torch.equal(s_g, s2) and torch.equal(idx_g, idx2) and torch.equal(norm_g, norm2)
        assert torch.equal(x.view(torch.int32), x2.view(torch.int32))
        assert torch.equal(c.view(torch.int16), c2.view(torch.int16))
        noise = 1e-3 * torch.empty(x2.numel(), device=DEV).normal_(generator=g)
        state_x, state_c = (x2 + noise.to(x2.dtype)).contiguous(), c2
        torch.cuda.synchronize()
        if kind == "counts_bounded_static":
            assert torch.equal(idx_g, idx_static)


@pytest.mark.parametrize("seed", range(6))
def test_random_layouts_whole_cycles(seed):
    # seeded random stores - element type, block length (log-uniform 1 ... 6,000), block count
    # (a few ... tens of thousands, so both the group-per-row and the run-of-rows scans are
    # met), offsets of x and c into their allocations, short last block - each taken through
    # scores (full and listed), selection, commit with staging, norm and recovery
    r = np.random.default_rng(1000 + seed)
    for case in range(10):
        dtype = int(r.choice([F32, BF16, I32]))
        L = int(np.exp(r.uniform(0, np.log(6000))))
        nb = int(np.exp(r.uniform(np.log(3), np.log(60_000))))
        nb = max(2, min(nb, 6_000_000 // L))
        n = L * nb - int(r.integers(0, L))
        nbk = oracle.n_blocks_of(n, L)
        off_x = int(r.choice([0, 0, 0, 1, 4, 5]))
        off_c = off_x if r.random() < 0.8 else int(r.integers(0, 8))
        hx, hc = make_store(dtype, n, seed=seed * 100 + case)
        x = to_dev(np.concatenate([np.zeros(off_x, dtype=hx.dtype), hx]), dtype)[off_x:]
        c = to_dev(np.concatenate([np.zeros(off_c, dtype=hc.dtype), hc]), dtype)[off_c:]
        print("random layout seed=%d case=%d dtype=%d L=%d nb=%d n=%d offsets=(%d,%d)"
              % (seed, case, dtype, L, nbk, n, off_x, off_c), flush=True)
        ws = scar.new_workspace(nbk, DEV)
        s = scar.block_scores(x, c, L)
        s_ref = oracle.block_scores(dtype, hx, hc, L)
        assert_scores_match(s, s_ref, dtype)
        listed = torch.full_like(s, -1)
        scar.block_scores_rows(x, c, L, torch.randperm(nbk, device=DEV).to(torch.int32), listed)
        assert torch.equal(s, listed)
        k = int(r.integers(1, nbk + 1))
        idx = scar.select_topk(s, k, ws)
        assert_selection_matches(idx_host(idx), s.cpu().numpy(), s_ref, k)
        st = torch.zeros(k * L, dtype=x.dtype, device=DEV)
        scar.checkpoint_commit(x, c, L, idx, st)
        hst = np.zeros(k * L, dtype=hx.dtype)
        oracle.checkpoint_commit(dtype, hx, hc, L, idx_host(idx), hst)
        np.testing.assert_array_equal(to_host(c.contiguous()), hc)
        np.testing.assert_array_equal(to_host(st), hst)
        S = r.permutation(nbk)[: max(1, nbk // 3)].astype(np.uint32)
        pre = scar.read_norm(scar.perturbation_norm(x, c, L, idx_dev(S), ws))
        got = scar.read_norm(scar.partial_recover(x, c, L, idx_dev(S), ws))
        assert_norm_matches(got, oracle.partial_recover(dtype, hx, hc, L, S), dtype)
        assert pre == got
        np.testing.assert_array_equal(to_host(x.contiguous()), hx)


@pytest.mark.parametrize("dtype,L,nb", [(F32, 3, 20_000_003), (BF16, 50, 5_000_001), (I32, 25, 6_000_000),
                                        (F32, 100, 2_684_354)])
def test_block_scores_of_very_many_short_rows(dtype, L, nb):
    # tens of thousands of chunks of the run-of-rows scan
    n = L * nb - (L // 2)
    r = np.random.default_rng(L + nb)
    if dtype == I32:
        c = r.integers(-50, 50, size=n, dtype=np.int32)
        x = c + (r.integers(0, 16, size=n, dtype=np.int32) == 0)
        x = x.astype(np.int32)
    else:
        c = r.random(n, dtype=np.float32)
        x = c + np.float32(0.01) * r.random(n, dtype=np.float32)
        if dtype == BF16:
            x, c = wl.f32_to_bf16_bits(x), wl.f32_to_bf16_bits(c)
    print("very many short rows dtype=%d L=%d nb=%d" % (dtype, L, nb), flush=True)
    oracle.set_num_threads(8)
    try:
        want = oracle.block_scores(dtype, x, c, L)
    finally:
        oracle.set_num_threads(1)
    s = scar.block_scores(to_dev(x, dtype), to_dev(c, dtype), L)
    assert_scores_match(s, want, dtype)


def test_two_streams_run_their_cycles_side_by_side():
    # two stores, each with its own workspace, go through three cycles on two streams with no
    # wait between them, so kernels of the two interleave on the device (the ordered write of
    # the selection included, whose workgroups wait for lower-numbered tiles of their own
    # launch only); every result must equal the one the same calls give one after the other
    specs = [(F32, 256, (1 << 25) - 77, 0.10), (I32, 1000, 40_000 * 1000, 0.05)]
    stores = []
    for dtype, L, n, frac in specs:
        hx, hc = make_store(dtype, n, seed=700 + L)
        if dtype == I32:          # few distinct scores: the selection is decided by its tie rule
            hx = (hc + (np.arange(n) % 997 == 0)).astype(np.int32)
        nb = oracle.n_blocks_of(n, L)
        lost = [idx_dev(wl.random_lost_blocks(nb, nb // 8, 900 + cyc)) for cyc in range(3)]
        stores.append(dict(dtype=dtype, L=L, nb=nb, k=wl.k_of_fraction(frac, nb), lost=lost,
                           x0=to_dev(hx, dtype), c0=to_dev(hc, dtype)))

    def run(st, x, c, out):
        ws = st["ws"]
        for cyc in range(3):
            s = scar.block_scores(x, c, st["L"])
            idx = scar.select_topk(s, st["k"], ws)
            scar.checkpoint_commit(x, c, st["L"], idx)
            norm = scar.partial_recover(x, c, st["L"], st["lost"][cyc], ws)
            out.append((s, idx, norm))

    serial = []
    for st in stores:                                  # one after the other on the current stream
        st["ws"] = scar.new_workspace(st["nb"], DEV)
        x, c, out = st["x0"].clone(), st["c0"].clone(), []
        run(st, x, c, out)
        torch.cuda.synchronize()
        serial.append((x, c, out))

    streams = [torch.cuda.Stream(), torch.cuda.Stream()]
    side = []
    for st in stores:
        side.append((st["x0"].clone(), st["c0"].clone(), []))
    torch.cuda.synchronize()
    for st, sm, (x, c, out) in zip(stores, streams, side):
        print("stream for dtype=%d L=%d blocks=%d" % (st["dtype"], st["L"], st["nb"]), flush=True)
        with torch.cuda.stream(sm):                    # enqueued without waiting for the other
            run(st, x, c, out)
    torch.cuda.synchronize()
    for (x1, c1, o1), (x2, c2, o2) in zip(serial, side):
        assert torch.equal(x1, x2) and torch.equal(c1, c2)
        for (s1, i1, n1), (s2, i2, n2) in zip(o1, o2):
            assert torch.equal(s1, s2) and torch.equal(i1, i2) and torch.equal(n1, n2)
