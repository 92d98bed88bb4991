"""ctypes face of the CPU oracle (oracle/scar_oracle.c) on numpy host arrays.

TEST INFRASTRUCTURE: only tests, the smoke check and the benchmark's CPU-baseline leg
may import this package.  It never touches the GPU library, and the GPU library never
touches it.  Float data are scored in double, integer tables in int64.
"""
import ctypes
import os

import numpy as np

from . import build as _build

F32, BF16, I32, F32_BF16C = 0, 1, 2, 3
_NP_OF = {F32: np.float32, BF16: np.uint16, I32: np.int32}
_X_OF = {F32: F32, BF16: BF16, I32: I32, F32_BF16C: F32}      # element type of x per store type
_C_OF = {F32: F32, BF16: BF16, I32: I32, F32_BF16C: BF16}     # element type of c per store type


class Norm(ctypes.Structure):
    _fields_ = [("sum", ctypes.c_double), ("norm", ctypes.c_double), ("isum", ctypes.c_int64)]


class OracleError(RuntimeError):
    pass


_lib = None


def lib():
    global _lib
    if _lib is None:
        path = os.environ.get("SCAR_ORACLE_LIB")      # a test may point at another build of the oracle
        if not path:
            path = _build.LIB
            if not os.path.exists(path) or os.path.getmtime(path) < os.path.getmtime(_build.SRC):
                _build.build(force=True)
        L = ctypes.CDLL(path)
        vp, u64, u32, i32 = ctypes.c_void_p, ctypes.c_uint64, ctypes.c_uint32, ctypes.c_int
        L.oracle_set_num_threads.argtypes = [i32]
        L.oracle_set_num_threads.restype = None
        L.oracle_get_num_threads.restype = i32
        L.oracle_block_scores.argtypes = [i32, vp, vp, u64, u32, vp]
        L.oracle_block_scores_rows.argtypes = [i32, vp, vp, u64, u32, vp, u32, vp]
        L.oracle_select_topk.argtypes = [i32, vp, u32, u32, vp]
        L.oracle_brute_force_topk.argtypes = [i32, vp, u32, u32, vp]
        L.oracle_checkpoint_commit.argtypes = [i32, vp, vp, u64, u32, vp, u32, vp]
        L.oracle_perturbation_norm.argtypes = [i32, vp, vp, u64, u32, vp, u32, ctypes.POINTER(Norm)]
        L.oracle_partial_recover.argtypes = [i32, vp, vp, u64, u32, vp, u32, ctypes.POINTER(Norm)]
        L.oracle_mask_to_indices.argtypes = [vp, u32, vp, ctypes.POINTER(u32)]
        L.oracle_var_block_scores.argtypes = [i32, vp, vp, vp, u32, vp]
        L.oracle_var_checkpoint_commit.argtypes = [i32, vp, vp, vp, u32, vp, u32, vp, vp]
        L.oracle_var_partial_recover_rows.argtypes = [i32, vp, vp, vp, vp, u32, vp, u32, ctypes.POINTER(Norm)]
        L.oracle_var_perturbation_norm.argtypes = [i32, vp, vp, vp, u32, vp, u32, ctypes.POINTER(Norm)]
        L.oracle_var_partial_recover.argtypes = [i32, vp, vp, vp, u32, vp, u32, ctypes.POINTER(Norm)]
        L.oracle_tv_block_scores.argtypes = [i32, vp, vp, u64, u32, vp, vp]
        L.oracle_tv_perturbation_norm.argtypes = [i32, vp, vp, u64, u32, vp, vp, u32, ctypes.POINTER(Norm)]
        L.oracle_tv_partial_recover.argtypes = [i32, vp, vp, u64, u32, vp, vp, u32, ctypes.POINTER(Norm)]
        L.oracle_var_tv_block_scores.argtypes = [i32, vp, vp, vp, u32, vp, vp]
        L.oracle_var_tv_perturbation_norm.argtypes = [i32, vp, vp, vp, u32, vp, vp, u32, ctypes.POINTER(Norm)]
        L.oracle_var_tv_partial_recover.argtypes = [i32, vp, vp, vp, u32, vp, vp, u32, ctypes.POINTER(Norm)]
        L.oracle_select_round.argtypes = [u32, u32, u64, vp]
        L.oracle_select_random.argtypes = [u32, u32, u64, u64, vp]
        L.oracle_philox4x32_10.argtypes = [vp, vp, vp]
        L.oracle_philox4x32_10.restype = None
        _lib = L
    return _lib


def set_num_threads(n: int) -> None:
    lib().oracle_set_num_threads(int(n))


def get_num_threads() -> int:
    return int(lib().oracle_get_num_threads())


def _check(rc, what):
    if rc != 0:
        raise OracleError("%s failed with status %d" % (what, rc))


def _flat_x(a, dtype):
    return _flat(a, _X_OF[dtype])


def _flat_c(a, dtype):
    return _flat(a, _C_OF[dtype])


def _flat(a, dtype):
    a = np.asarray(a)
    if a.dtype != _NP_OF[dtype]:
        raise TypeError("expected %s array, got %s" % (_NP_OF[dtype], a.dtype))
    if not a.flags["C_CONTIGUOUS"]:
        raise ValueError("array must be C-contiguous")
    return a.reshape(-1)


def _ptr(a):
    return ctypes.c_void_p(a.ctypes.data) if a is not None and a.size else ctypes.c_void_p(0)


def _idx(idx):
    if idx is None:
        return None
    idx = np.ascontiguousarray(idx, dtype=np.uint32)
    return idx


def n_blocks_of(n_elems: int, block_len: int) -> int:
    return (n_elems + block_len - 1) // block_len


def block_scores(dtype, x, c, block_len):
    """Distance of every block of x from c: float64 squared-L2 (float data) or int64 L1."""
    x, c = _flat_x(x, dtype), _flat_c(c, dtype)
    assert x.size == c.size
    nb = n_blocks_of(x.size, block_len)
    out = np.zeros(nb, dtype=np.int64 if dtype == I32 else np.float64)
    _check(lib().oracle_block_scores(dtype, _ptr(x), _ptr(c), x.size, block_len, _ptr(out)),
           "oracle_block_scores")
    return out


def block_scores_rows(dtype, x, c, block_len, idx, scores):
    """Recomputes scores[b] for b in idx, in place; other entries stay."""
    x, c, idx = _flat_x(x, dtype), _flat_c(c, dtype), _idx(idx)
    want = np.int64 if dtype == I32 else np.float64
    assert scores.dtype == want and scores.flags.c_contiguous and scores.size == n_blocks_of(x.size, block_len)
    _check(lib().oracle_block_scores_rows(dtype, _ptr(x), _ptr(c), x.size, block_len, _ptr(idx), idx.size,
                                          _ptr(scores)), "oracle_block_scores_rows")
    return scores


def select_topk(scores, k):
    """Ascending indices of the k largest scores; ties go to the lower index."""
    scores = np.ascontiguousarray(scores)
    if scores.dtype == np.int64:
        is_int = 1
    else:
        scores = np.ascontiguousarray(scores, dtype=np.float64)
        is_int = 0
    out = np.zeros(k, dtype=np.uint32)
    _check(lib().oracle_select_topk(is_int, _ptr(scores), scores.size, k, _ptr(out)),
           "oracle_select_topk")
    return out


def brute_force_topk(scores, k):
    """Largest total score over all k-subsets (tiny inputs only)."""
    scores = np.ascontiguousarray(scores)
    if scores.dtype == np.int64:
        res = ctypes.c_int64(0)
        is_int = 1
    else:
        scores = np.ascontiguousarray(scores, dtype=np.float64)
        res = ctypes.c_double(0)
        is_int = 0
    _check(lib().oracle_brute_force_topk(is_int, _ptr(scores), scores.size, k,
                                          ctypes.cast(ctypes.byref(res), ctypes.c_void_p)),
           "oracle_brute_force_topk")
    return res.value


def checkpoint_commit(dtype, x, c, block_len, idx, staging=None):
    """c[b] <- x[b] for b in idx, in place on c; optional packed staging rows."""
    x, c = _flat_x(x, dtype), _flat_c(c, dtype)
    idx = _idx(idx)
    st = _flat_c(staging, dtype) if staging is not None else None
    if st is not None:
        assert st.size >= idx.size * block_len
    _check(lib().oracle_checkpoint_commit(dtype, _ptr(x), _ptr(c), x.size, block_len, _ptr(idx),
                                          idx.size, _ptr(st)), "oracle_checkpoint_commit")


def perturbation_norm(dtype, x, c, block_len, idx=None):
    """(sum, norm, isum) of c - x over the blocks in idx (None = all blocks)."""
    x, c = _flat_x(x, dtype), _flat_c(c, dtype)
    idx = _idx(idx)
    out = Norm()
    if idx is None:
        rc = lib().oracle_perturbation_norm(dtype, _ptr(x), _ptr(c), x.size, block_len,
                                            ctypes.c_void_p(0), 0, ctypes.byref(out))
    else:
        # an empty list is "no blocks", not "all blocks": hand over a real pointer
        keep = idx if idx.size else np.zeros(1, dtype=np.uint32)
        rc = lib().oracle_perturbation_norm(dtype, _ptr(x), _ptr(c), x.size, block_len,
                                            ctypes.c_void_p(keep.ctypes.data), idx.size,
                                            ctypes.byref(out))
    _check(rc, "oracle_perturbation_norm")
    return out.sum, out.norm, out.isum


def partial_recover(dtype, x, c, block_len, lost, want_norm=True):
    """x[b] <- c[b] for b in lost, in place on x; returns (sum, norm, isum) or None."""
    x, c = _flat_x(x, dtype), _flat_c(c, dtype)
    lost = _idx(lost)
    out = Norm()
    _check(lib().oracle_partial_recover(dtype, _ptr(x), _ptr(c), x.size, block_len, _ptr(lost),
                                        lost.size, ctypes.byref(out) if want_norm else None),
           "oracle_partial_recover")
    return (out.sum, out.norm, out.isum) if want_norm else None


def mask_to_indices(mask):
    mask = np.ascontiguousarray(mask, dtype=np.uint8)
    out = np.zeros(mask.size, dtype=np.uint32)
    cnt = ctypes.c_uint32(0)
    _check(lib().oracle_mask_to_indices(_ptr(mask), mask.size, _ptr(out), ctypes.byref(cnt)),
           "oracle_mask_to_indices")
    return out[:cnt.value].copy()


def select_round(n_blocks, k, cursor):
    """Round-robin strategy: the k blocks from `cursor` on (mod n_blocks), ascending."""
    out = np.zeros(k, dtype=np.uint32)
    _check(lib().oracle_select_round(n_blocks, k, cursor, _ptr(out)), "oracle_select_round")
    return out


def select_random(n_blocks, k, seed, draw):
    """Random strategy: a uniformly random k-subset fixed by (seed, draw), ascending."""
    out = np.zeros(k, dtype=np.uint32)
    _check(lib().oracle_select_random(n_blocks, k, seed, draw, _ptr(out)), "oracle_select_random")
    return out


def philox4x32_10(counter, key):
    c = np.ascontiguousarray(counter, dtype=np.uint32)
    k = np.ascontiguousarray(key, dtype=np.uint32)
    out = np.zeros(4, dtype=np.uint32)
    lib().oracle_philox4x32_10(_ptr(c), _ptr(k), _ptr(out))
    return out


# ---- blocks of unequal length: offsets is a uint64 array of n_blocks + 1 element offsets

def _offsets(offsets):
    return np.ascontiguousarray(offsets, dtype=np.uint64)


def var_block_scores(dtype, x, c, offsets):
    x, c, off = _flat_x(x, dtype), _flat_c(c, dtype), _offsets(offsets)
    nb = off.size - 1
    out = np.zeros(nb, dtype=np.int64 if dtype == I32 else np.float64)
    _check(lib().oracle_var_block_scores(dtype, _ptr(x), _ptr(c), _ptr(off), nb, _ptr(out)),
           "oracle_var_block_scores")
    return out


def var_checkpoint_commit(dtype, x, c, offsets, idx, staging=None):
    """c_b <- x_b for the listed blocks of unequal length.  With staging (a flat array of c's
    type with room for the listed blocks) the blocks are also packed into it in list order;
    returns the uint64 element offsets of the packed blocks (n_idx + 1 entries) or None."""
    x, c, off, idx = _flat_x(x, dtype), _flat_c(c, dtype), _offsets(offsets), _idx(idx)
    st_off = None
    if staging is not None:
        staging = _flat_c(staging, dtype)
        need = int(sum(int(off[b + 1] - off[b]) for b in idx))
        if staging.size < need:
            raise ValueError("staging too small")
        st_off = np.zeros(idx.size + 1, dtype=np.uint64)
    _check(lib().oracle_var_checkpoint_commit(dtype, _ptr(x), _ptr(c), _ptr(off), off.size - 1,
                                              _ptr(idx), idx.size, _ptr(staging),
                                              ctypes.c_void_p(st_off.ctypes.data) if st_off is not None
                                              else ctypes.c_void_p(0)), "oracle_var_checkpoint_commit")
    return st_off


def var_partial_recover_rows(dtype, x, rows, row_offsets, offsets, lost):
    """x_b <- the packed row of block b for the lost blocks; (sum, norm, isum) of rows - x_S
    measured before the overwrite."""
    x, rows, off, lost = _flat_x(x, dtype), _flat_c(rows, dtype), _offsets(offsets), _idx(lost)
    row_offsets = np.ascontiguousarray(row_offsets, dtype=np.uint64)
    out = Norm()
    _check(lib().oracle_var_partial_recover_rows(dtype, _ptr(x), _ptr(rows),
                                                 ctypes.c_void_p(row_offsets.ctypes.data), _ptr(off),
                                                 off.size - 1, _ptr(lost), lost.size, ctypes.byref(out)),
           "oracle_var_partial_recover_rows")
    return out.sum, out.norm, out.isum


def var_perturbation_norm(dtype, x, c, offsets, idx=None):
    x, c, off = _flat_x(x, dtype), _flat_c(c, dtype), _offsets(offsets)
    out = Norm()
    if idx is None:
        ptr, n = ctypes.c_void_p(0), 0
    else:
        idx = _idx(idx)
        keep = idx if idx.size else np.zeros(1, dtype=np.uint32)
        ptr, n = ctypes.c_void_p(keep.ctypes.data), idx.size
    _check(lib().oracle_var_perturbation_norm(dtype, _ptr(x), _ptr(c), _ptr(off), off.size - 1, ptr, n,
                                              ctypes.byref(out)), "oracle_var_perturbation_norm")
    return out.sum, out.norm, out.isum


def var_partial_recover(dtype, x, c, offsets, lost):
    x, c, off, lost = _flat_x(x, dtype), _flat_c(c, dtype), _offsets(offsets), _idx(lost)
    out = Norm()
    _check(lib().oracle_var_partial_recover(dtype, _ptr(x), _ptr(c), _ptr(off), off.size - 1,
                                            _ptr(lost), lost.size, ctypes.byref(out)),
           "oracle_var_partial_recover")
    return out.sum, out.norm, out.isum


# ---- document-length-scaled total variation (rows of a float store are distributions) -------

def _weights(w):
    return None if w is None else np.ascontiguousarray(w, dtype=np.float32)


def tv_block_scores(dtype, x, c, block_len, weights=None):
    """w_b * TV(x_b, c_b) per block, TV = half the L1 distance; float64."""
    x, c, w = _flat_x(x, dtype), _flat_c(c, dtype), _weights(weights)
    out = np.zeros(n_blocks_of(x.size, block_len), dtype=np.float64)
    _check(lib().oracle_tv_block_scores(dtype, _ptr(x), _ptr(c), x.size, block_len, _ptr(w), _ptr(out)),
           "oracle_tv_block_scores")
    return out


def tv_perturbation_norm(dtype, x, c, block_len, weights=None, idx=None):
    x, c, w = _flat_x(x, dtype), _flat_c(c, dtype), _weights(weights)
    out = Norm()
    if idx is None:
        ptr, n = ctypes.c_void_p(0), 0
    else:
        idx = _idx(idx)
        keep = idx if idx.size else np.zeros(1, dtype=np.uint32)
        ptr, n = ctypes.c_void_p(keep.ctypes.data), idx.size
    _check(lib().oracle_tv_perturbation_norm(dtype, _ptr(x), _ptr(c), x.size, block_len, _ptr(w), ptr, n,
                                             ctypes.byref(out)), "oracle_tv_perturbation_norm")
    return out.sum, out.norm, out.isum


def tv_partial_recover(dtype, x, c, block_len, lost, weights=None):
    x, c, w, lost = _flat_x(x, dtype), _flat_c(c, dtype), _weights(weights), _idx(lost)
    out = Norm()
    _check(lib().oracle_tv_partial_recover(dtype, _ptr(x), _ptr(c), x.size, block_len, _ptr(w), _ptr(lost),
                                           lost.size, ctypes.byref(out)), "oracle_tv_partial_recover")
    return out.sum, out.norm, out.isum


# ---- scaled total variation over blocks of unequal length -------------------------------------

def var_tv_block_scores(dtype, x, c, offsets, weights=None):
    x, c, off, w = _flat_x(x, dtype), _flat_c(c, dtype), _offsets(offsets), _weights(weights)
    out = np.zeros(off.size - 1, dtype=np.float64)
    _check(lib().oracle_var_tv_block_scores(dtype, _ptr(x), _ptr(c), _ptr(off), off.size - 1, _ptr(w), _ptr(out)),
           "oracle_var_tv_block_scores")
    return out


def var_tv_perturbation_norm(dtype, x, c, offsets, weights=None, idx=None):
    x, c, off, w = _flat_x(x, dtype), _flat_c(c, dtype), _offsets(offsets), _weights(weights)
    out = Norm()
    if idx is None:
        ptr, n = ctypes.c_void_p(0), 0
    else:
        idx = _idx(idx)
        keep = idx if idx.size else np.zeros(1, dtype=np.uint32)
        ptr, n = ctypes.c_void_p(keep.ctypes.data), idx.size
    _check(lib().oracle_var_tv_perturbation_norm(dtype, _ptr(x), _ptr(c), _ptr(off), off.size - 1, _ptr(w), ptr, n,
                                                 ctypes.byref(out)), "oracle_var_tv_perturbation_norm")
    return out.sum, out.norm, out.isum


def var_tv_partial_recover(dtype, x, c, offsets, lost, weights=None):
    x, c, off, w, lost = _flat_x(x, dtype), _flat_c(c, dtype), _offsets(offsets), _weights(weights), _idx(lost)
    out = Norm()
    _check(lib().oracle_var_tv_partial_recover(dtype, _ptr(x), _ptr(c), _ptr(off), off.size - 1, _ptr(w),
                                               _ptr(lost), lost.size, ctypes.byref(out)),
           "oracle_var_tv_partial_recover")
    return out.sum, out.norm, out.isum
