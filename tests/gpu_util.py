"""Helpers shared by the GPU parity tests: host <-> device moves and the comparison rules."""
import numpy as np
import torch

import oracle
from paper_1810_07354_amd import scar
from paper_1810_07354_amd import workloads as wl

DEV = "cuda:0"
REL_TOL = 1e-5        # float scores and norms: float32 path against the float64 oracle
BAND = 1e-6           # blocks whose score is this close (relative) to the k-th key may differ


def to_dev(a: np.ndarray, dtype: int) -> torch.Tensor:
    """numpy host array (uint16 bits for bfloat16) -> device tensor of the store's type."""
    a = np.ascontiguousarray(a)
    if dtype == wl.BF16:
        return torch.from_numpy(a.view(np.int16)).to(DEV).view(torch.bfloat16)
    return torch.from_numpy(a).to(DEV)


def to_host(t: torch.Tensor) -> np.ndarray:
    """device tensor -> numpy (bfloat16 comes back as its uint16 bits)."""
    if t.dtype == torch.bfloat16:
        return t.view(torch.int16).cpu().numpy().view(np.uint16)
    return t.cpu().numpy()


def idx_dev(idx) -> torch.Tensor:
    return torch.from_numpy(np.ascontiguousarray(idx, dtype=np.uint32).view(np.int32).copy()).to(DEV)


def idx_host(t: torch.Tensor) -> np.ndarray:
    return t.cpu().numpy().view(np.uint32)


def assert_scores_match(gpu_scores: torch.Tensor, want: np.ndarray, dtype: int):
    got = gpu_scores.cpu().numpy()
    if dtype == wl.I32:
        assert got.dtype == np.int64
        np.testing.assert_array_equal(got, want)
    else:
        assert got.dtype == np.float32
        np.testing.assert_allclose(got.astype(np.float64), want, rtol=REL_TOL, atol=0.0)


def assert_selection_matches(gpu_idx: np.ndarray, gpu_scores: np.ndarray, oracle_scores: np.ndarray, k: int):
    """The two rules for a top-k result.

    (1) On the scores the GPU itself used, the choice (ties included) must be exactly the
        oracle's, index for index.
    (2) Against the oracle's own float64 scores, every block clearly above the k-th key
        must be chosen and none clearly below it; inside the band either is fine.
    Integer scores have no band: rule (1) on identical scores is the whole story."""
    assert gpu_idx.size == k
    assert np.all(np.diff(gpu_idx.astype(np.int64)) > 0), "indices must be ascending and distinct"
    if gpu_scores.dtype == np.int64:
        np.testing.assert_array_equal(gpu_scores, oracle_scores)
        np.testing.assert_array_equal(gpu_idx, oracle.select_topk(oracle_scores, k))
        return
    np.testing.assert_array_equal(gpu_idx, oracle.select_topk(gpu_scores.astype(np.float64), k))
    if k == 0 or k == oracle_scores.size:
        return
    tau = np.sort(oracle_scores)[::-1][k - 1]
    chosen = np.zeros(oracle_scores.size, dtype=bool)
    chosen[gpu_idx] = True
    must = oracle_scores > tau * (1 + BAND)
    never = oracle_scores < tau * (1 - BAND)
    assert np.all(chosen[must]), "a block clearly above the k-th score was not selected"
    assert not np.any(chosen[never]), "a block clearly below the k-th score was selected"


def assert_norm_matches(got, want, dtype: int):
    gs, gn, gi = got
    ws, wn, wi = want
    if dtype == wl.I32:
        assert gi == wi and gs == float(wi) and gn == float(wi)
    else:
        assert gi == 0
        assert abs(gs - ws) <= REL_TOL * abs(ws), (gs, ws)
        assert abs(gn - wn) <= REL_TOL * abs(wn), (gn, wn)


class DeviceStore:
    """x, c on the device plus host mirrors that the oracle advances in lock step."""

    def __init__(self, w: wl.Workload):
        self.w = w
        self.dtype, self.L = w.dtype, w.block_len
        self.hx, self.hc = w.x.copy(), w.c.copy()
        self.x, self.c = to_dev(self.hx, self.dtype), to_dev(self.hc, self.dtype)
        self.ws = scar.new_workspace(w.n_blocks, DEV)

    def check_state(self):
        np.testing.assert_array_equal(to_host(self.x), self.hx)
        np.testing.assert_array_equal(to_host(self.c), self.hc)

    def cycle(self, k: int, lost: np.ndarray, staging: bool = False):
        """One checkpoint + failure + recovery cycle on both sides, compared call by call."""
        dt, L = self.dtype, self.L
        s_gpu = scar.block_scores(self.x, self.c, L)
        s_ref = oracle.block_scores(dt, self.hx, self.hc, L)
        assert_scores_match(s_gpu, s_ref, dt)

        idx_gpu = scar.select_topk(s_gpu, k, self.ws)
        assert_selection_matches(idx_host(idx_gpu), s_gpu.cpu().numpy(), s_ref, k)

        st = torch.full((k * L,), 0, dtype=self.x.dtype, device=DEV) if staging else None
        scar.checkpoint_commit(self.x, self.c, L, idx_gpu, st)
        hst = np.zeros(k * L, dtype=self.hx.dtype) if staging else None
        oracle.checkpoint_commit(dt, self.hx, self.hc, L, idx_host(idx_gpu), hst)
        self.check_state()
        if staging:
            np.testing.assert_array_equal(to_host(st), hst)

        full_gpu = scar.read_norm(scar.perturbation_norm(self.x, self.c, L, None, self.ws))
        assert_norm_matches(full_gpu, oracle.perturbation_norm(dt, self.hx, self.hc, L), dt)

        lost_d = idx_dev(lost)
        nrm = scar.partial_recover(self.x, self.c, L, lost_d, self.ws)
        want = oracle.partial_recover(dt, self.hx, self.hc, L, lost)
        got = scar.read_norm(nrm)
        assert_norm_matches(got, want, dt)
        self.check_state()
        # Theorem 4.1: the partial perturbation never exceeds the full one
        assert got[1] <= full_gpu[1] * (1 + REL_TOL)
        return s_gpu, idx_gpu, got
