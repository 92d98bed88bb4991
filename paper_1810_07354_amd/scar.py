"""Python face of the C-ABI library libscar.so: same names, argument marshalling only.

Every function takes torch tensors that live on the GPU, hands their device pointers and
torch's current HIP stream to the library and returns (asynchronously) torch tensors.
Nothing is computed here, and there is no fallback: without the built library, or with
tensors that are not on a GPU, these calls raise.
"""
import ctypes
import os

import torch

F32, BF16, I32, F32_BF16C = 0, 1, 2, 3
SCORE_F32, SCORE_I64 = 0, 1
MAX_BLOCKS = 0x7FFFFFFF

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libscar.so")

_TORCH_OF = {F32: torch.float32, BF16: torch.bfloat16, I32: torch.int32}
_DTYPE_OF = {v: k for k, v in _TORCH_OF.items()}


class ScarError(RuntimeError):
    def __init__(self, status, what):
        self.status = status
        super().__init__("%s: %s (status %d)" % (what, strerror(status), status))


class Layout(ctypes.Structure):
    """scar_layout: how x and c are cut into blocks."""
    _fields_ = [("dtype", ctypes.c_int32), ("block_len", ctypes.c_uint32), ("n_elems", ctypes.c_uint64)]


class VarLayout(ctypes.Structure):
    """scar_var_layout: blocks of unequal length given by device-resident offsets."""
    _fields_ = [("dtype", ctypes.c_int32), ("n_blocks", ctypes.c_uint32), ("n_elems", ctypes.c_uint64),
                ("offsets", ctypes.c_void_p)]


class Norm(ctypes.Structure):
    """scar_norm as laid out in device memory."""
    _fields_ = [("sum", ctypes.c_double), ("norm", ctypes.c_double), ("isum", ctypes.c_int64)]


_lib = None


def lib():
    """The loaded library; raises if it has not been built."""
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise RuntimeError("libscar.so is not built: run `python -c 'import __graft_entry__ as g; "
                               "g.build()'` (or paper_1810_07354_amd/build.py) first")
        L = ctypes.CDLL(LIB_PATH)
        vp, u32, u64, i32, sz = (ctypes.c_void_p, ctypes.c_uint32, ctypes.c_uint64, ctypes.c_int32,
                                 ctypes.c_size_t)
        lp = ctypes.POINTER(Layout)
        L.scar_n_blocks.argtypes = [lp]
        L.scar_n_blocks.restype = u64
        L.scar_workspace_bytes.argtypes = [u64]
        L.scar_workspace_bytes.restype = sz
        L.scar_strerror.argtypes = [ctypes.c_int]
        L.scar_strerror.restype = ctypes.c_char_p
        L.scar_block_scores.argtypes = [lp, vp, vp, vp, vp]
        L.scar_block_scores_rows.argtypes = [lp, vp, vp, vp, u32, vp, vp]
        L.scar_block_scores_rows.restype = ctypes.c_int
        L.scar_select_topk.argtypes = [i32, vp, u32, u32, vp, vp, sz, vp]
        L.scar_checkpoint_commit.argtypes = [lp, vp, vp, vp, u32, vp, vp]
        L.scar_check_workspace_bytes.argtypes = [u64]
        L.scar_check_workspace_bytes.restype = sz
        L.scar_check_indices.argtypes = [vp, u32, u32, vp, vp, sz, vp]
        L.scar_check_indices.restype = ctypes.c_int
        L.scar_select_topk_bounded.argtypes = [i32, vp, u32, u32, u64, vp, vp, sz, vp]
        L.scar_select_topk_bounded.restype = ctypes.c_int
        L.scar_set_lookback_spin_limit.argtypes = [u32]
        L.scar_set_lookback_spin_limit.restype = None
        L.scar_set_compaction_groups.argtypes = [u32]
        L.scar_set_compaction_groups.restype = None
        L.scar_select_topk_static.argtypes = [i32, vp, u32, u32, vp, vp]
        L.scar_select_topk_static.restype = ctypes.c_int
        L.scar_partial_recover.argtypes = [lp, vp, vp, vp, u32, vp, vp, sz, vp]
        L.scar_perturbation_norm.argtypes = [lp, vp, vp, vp, u32, vp, vp, sz, vp]
        L.scar_mask_to_indices.argtypes = [vp, u32, vp, vp, vp, sz, vp]
        L.scar_select_round.argtypes = [u32, u32, u64, vp, vp]
        L.scar_select_random.argtypes = [u32, u32, u64, u64, vp, vp, sz, vp]
        vlp = ctypes.POINTER(VarLayout)
        L.scar_var_workspace_bytes.argtypes = [u64]
        L.scar_var_workspace_bytes.restype = sz
        L.scar_var_block_scores.argtypes = [vlp, vp, vp, vp, vp, sz, vp]
        L.scar_var_checkpoint_commit.argtypes = [vlp, vp, vp, vp, u32, vp, sz, vp]
        L.scar_var_partial_recover.argtypes = [vlp, vp, vp, vp, u32, vp, vp, sz, vp]
        L.scar_var_perturbation_norm.argtypes = [vlp, vp, vp, vp, u32, vp, vp, sz, vp]
        L.scar_var_tv_block_scores.argtypes = [vlp, vp, vp, vp, vp, vp, sz, vp]
        L.scar_var_tv_partial_recover.argtypes = [vlp, vp, vp, vp, vp, u32, vp, vp, sz, vp]
        L.scar_var_tv_perturbation_norm.argtypes = [vlp, vp, vp, vp, vp, u32, vp, vp, sz, vp]
        for name in ("scar_var_tv_block_scores", "scar_var_tv_partial_recover", "scar_var_tv_perturbation_norm"):
            getattr(L, name).restype = ctypes.c_int
        L.scar_var_checkpoint_commit_staged.argtypes = [vlp, vp, vp, vp, u32, vp, vp, vp, sz, vp]
        L.scar_var_partial_recover_rows.argtypes = [vlp, vp, vp, vp, vp, u32, vp, vp, sz, vp]
        for name in ("scar_var_block_scores", "scar_var_checkpoint_commit", "scar_var_partial_recover",
                     "scar_var_perturbation_norm", "scar_var_checkpoint_commit_staged",
                     "scar_var_partial_recover_rows"):
            getattr(L, name).restype = ctypes.c_int
        L.scar_tv_block_scores.argtypes = [lp, vp, vp, vp, vp, vp]
        L.scar_tv_partial_recover.argtypes = [lp, vp, vp, vp, vp, u32, vp, vp, sz, vp]
        L.scar_tv_perturbation_norm.argtypes = [lp, vp, vp, vp, vp, u32, vp, vp, sz, vp]
        for name in ("scar_tv_block_scores", "scar_tv_partial_recover", "scar_tv_perturbation_norm"):
            getattr(L, name).restype = ctypes.c_int
        pp = ctypes.POINTER(ctypes.c_void_p)
        L.scar_store_create.argtypes = [ctypes.c_char_p, lp, u32, pp]
        L.scar_store_open.argtypes = [ctypes.c_char_p, u32, lp, pp]
        L.scar_store_save_async.argtypes = [vp, vp, vp, u32, vp]
        L.scar_store_wait.argtypes = [vp]
        L.scar_store_load.argtypes = [vp, vp, u32, vp, vp]
        L.scar_store_close.argtypes = [vp]
        L.scar_partial_recover_rows.argtypes = [lp, vp, vp, vp, u32, vp, vp, sz, vp]
        L.scar_var_store_create.argtypes = [ctypes.c_char_p, i32, u32, vp, u32, u64, pp]
        L.scar_var_store_save_async.argtypes = [vp, vp, u64, vp, u32, vp]
        L.scar_var_store_load.argtypes = [vp, vp, u32, vp, vp, vp]
        for name in ("scar_var_store_create", "scar_var_store_save_async", "scar_var_store_load"):
            getattr(L, name).restype = ctypes.c_int
        for name in ("scar_store_create", "scar_store_open", "scar_store_save_async", "scar_store_wait",
                     "scar_store_load", "scar_store_close", "scar_partial_recover_rows"):
            getattr(L, name).restype = ctypes.c_int
        for name in ("scar_block_scores", "scar_select_topk", "scar_checkpoint_commit",
                     "scar_partial_recover", "scar_perturbation_norm", "scar_mask_to_indices",
                     "scar_select_round", "scar_select_random"):
            getattr(L, name).restype = ctypes.c_int
        L.scar_ceiling_read2.argtypes = [vp, vp, u64, vp, vp]
        L.scar_ceiling_copy.argtypes = [vp, vp, u64, vp]
        L.scar_ceiling_read2_write1.argtypes = [vp, vp, u64, vp, vp]
        for name in ("scar_ceiling_read2", "scar_ceiling_copy", "scar_ceiling_read2_write1"):
            getattr(L, name).restype = ctypes.c_int
        _lib = L
    return _lib


def strerror(status: int) -> str:
    return lib().scar_strerror(int(status)).decode()


def _check(status, what):
    if status != 0:
        raise ScarError(status, what)


def _dev(t, what):
    if not isinstance(t, torch.Tensor) or not t.is_cuda:
        raise TypeError("%s must be a torch tensor on the GPU" % what)
    if not t.is_contiguous():
        raise ValueError("%s must be contiguous" % what)
    return t


def _idx(t, what):
    """An index list: contiguous int32 tensor on the GPU (the library reads uint32)."""
    _dev(t, what)
    if t.dtype != torch.int32:
        raise TypeError("%s must be an int32 tensor" % what)
    return t


def _bytes(t):
    return t.numel() * t.element_size() if t is not None else 0


def _p(t):
    return ctypes.c_void_p(t.data_ptr() if t is not None else 0)


def _stream():
    return ctypes.c_void_p(torch.cuda.current_stream().cuda_stream)


def store_type(x, c=None) -> int:
    """scar_dtype of a store: x's element type, or F32_BF16C for float32 x with a bfloat16
    checkpoint (the reduced-precision checkpoint)."""
    if c is not None and x.dtype == torch.float32 and c.dtype == torch.bfloat16:
        return F32_BF16C
    if x.dtype not in _DTYPE_OF:
        raise TypeError("unsupported element type %s" % x.dtype)
    if c is not None and c.dtype != x.dtype:
        raise ValueError("x and c must have the same element type (or float32 x with bfloat16 c)")
    return _DTYPE_OF[x.dtype]


def layout_of(x, block_len: int, c=None) -> Layout:
    if c is not None and x.numel() != c.numel():
        raise ValueError("x and c must have the same number of elements")
    return Layout(store_type(x, c), int(block_len), x.numel())


def n_blocks(layout: Layout) -> int:
    return int(lib().scar_n_blocks(ctypes.byref(layout)))


def workspace_bytes(n_blocks_: int) -> int:
    return int(lib().scar_workspace_bytes(int(n_blocks_)))


def new_workspace(n_blocks_: int, device) -> torch.Tensor:
    """A device buffer big enough for any call on a store of n_blocks_ blocks."""
    return torch.empty(workspace_bytes(n_blocks_), dtype=torch.uint8, device=device)


def block_scores(x, c, block_len, out=None):
    """scar_block_scores: float32 (F32/BF16 stores) or int64 (I32 stores) score per block."""
    _dev(x, "x"), _dev(c, "c")
    lay = layout_of(x, block_len, c)
    nb = n_blocks(lay)
    if out is None:
        out = torch.empty(nb, dtype=torch.int64 if x.dtype == torch.int32 else torch.float32,
                          device=x.device)
    _dev(out, "out")
    if out.dtype != (torch.int64 if x.dtype == torch.int32 else torch.float32) or out.numel() < nb:
        raise ValueError("out must hold n_blocks scores (int64 for int32 stores, else float32)")
    _check(lib().scar_block_scores(ctypes.byref(lay), _p(x), _p(c), _p(out), _stream()),
           "scar_block_scores")
    return out


def block_scores_rows(x, c, block_len, idx, scores):
    """scar_block_scores_rows: recomputes scores[b] for b in idx, in place."""
    _dev(x, "x"), _dev(c, "c"), _idx(idx, "idx"), _dev(scores, "scores")
    lay = layout_of(x, block_len, c)
    if scores.dtype != (torch.int64 if x.dtype == torch.int32 else torch.float32) or scores.numel() < n_blocks(lay):
        raise ValueError("scores must hold n_blocks scores (int64 for int32 stores, else float32)")
    _check(lib().scar_block_scores_rows(ctypes.byref(lay), _p(x), _p(c), _p(idx), idx.numel(), _p(scores),
                                        _stream()), "scar_block_scores_rows")
    return scores


def select_topk(scores, k, workspace, out=None):
    """scar_select_topk: ascending int32-viewed uint32 indices of the k largest scores."""
    _dev(scores, "scores"), _dev(workspace, "workspace")
    if scores.dtype == torch.float32:
        st = SCORE_F32
    elif scores.dtype == torch.int64:
        st = SCORE_I64
    else:
        raise TypeError("scores must be float32 or int64")
    if out is None:
        out = torch.empty(int(k), dtype=torch.int32, device=scores.device)
    elif _idx(out, "out").numel() < int(k):
        raise ValueError("out must hold k indices")
    _check(lib().scar_select_topk(st, _p(scores), scores.numel(), int(k), _p(out), _p(workspace), _bytes(workspace), _stream()), "scar_select_topk")
    return out


def select_topk_bounded(scores, k, score_max, workspace, out=None):
    """scar_select_topk_bounded: scar_select_topk for int64 scores known to lie in [0, score_max]."""
    _dev(scores, "scores"), _dev(workspace, "workspace")
    if scores.dtype == torch.float32:
        st = SCORE_F32
    elif scores.dtype == torch.int64:
        st = SCORE_I64
    else:
        raise TypeError("scores must be float32 or int64")
    if out is None:
        out = torch.empty(int(k), dtype=torch.int32, device=scores.device)
    elif _idx(out, "out").numel() < int(k):
        raise ValueError("out must hold k indices")
    _check(lib().scar_select_topk_bounded(st, _p(scores), scores.numel(), int(k), int(score_max), _p(out),
                                          _p(workspace), _bytes(workspace), _stream()),
           "scar_select_topk_bounded")
    return out


def check_indices(idx, n_blocks_):
    """scar_check_indices: (entries out of range, repeated entries) of an index list; synchronises."""
    _idx(idx, "idx")
    ws = torch.empty(int(lib().scar_check_workspace_bytes(int(n_blocks_))), dtype=torch.uint8, device=idx.device)
    counts = torch.empty(2, dtype=torch.int32, device=idx.device)
    _check(lib().scar_check_indices(_p(idx), idx.numel(), int(n_blocks_), _p(counts), _p(ws), _bytes(ws),
                                    _stream()), "scar_check_indices")
    host = counts.cpu()
    return int(host[0]), int(host[1])


def set_lookback_spin_limit(polls: int) -> None:
    lib().scar_set_lookback_spin_limit(int(polls))


def set_compaction_groups(groups: int) -> None:
    """scar_set_compaction_groups (testing aid): at most `groups` workgroups in the ordered write."""
    lib().scar_set_compaction_groups(int(groups))


STATIC_MAX_BLOCKS = 1 << 24


def select_topk_static(scores, k, out=None):
    """scar_select_topk_static: scar_select_topk on the library's own fixed scratch (no
    workspace, nothing allocated by the call when `out` is given)."""
    _dev(scores, "scores")
    if scores.dtype == torch.float32:
        st = SCORE_F32
    elif scores.dtype == torch.int64:
        st = SCORE_I64
    else:
        raise TypeError("scores must be float32 or int64")
    if out is None:
        out = torch.empty(int(k), dtype=torch.int32, device=scores.device)
    elif _idx(out, "out").numel() < int(k):
        raise ValueError("out must hold k indices")
    _check(lib().scar_select_topk_static(st, _p(scores), scores.numel(), int(k), _p(out), _stream()),
           "scar_select_topk_static")
    return out


def checkpoint_commit(x, c, block_len, idx, staging=None, n_idx=None):
    """scar_checkpoint_commit: c[b] <- x[b] for b in idx (optionally also packed into staging)."""
    _dev(x, "x"), _dev(c, "c"), _idx(idx, "idx")
    lay = layout_of(x, block_len, c)
    n = idx.numel() if n_idx is None else int(n_idx)
    if n > idx.numel():
        raise ValueError("n_idx exceeds the index list")
    if staging is not None:
        _dev(staging, "staging")
        if staging.dtype != c.dtype or staging.numel() < n * block_len:
            raise ValueError("staging must hold n_idx * block_len elements of c's type")
    _check(lib().scar_checkpoint_commit(ctypes.byref(lay), _p(x), _p(c), _p(idx), n, _p(staging),
                                        _stream()), "scar_checkpoint_commit")


def _norm_buffer(device):
    return torch.empty(3, dtype=torch.float64, device=device)


def read_norm(buf):
    """(sum, norm, isum) from a device scar_norm buffer; synchronises."""
    host = buf.cpu()
    return float(host[0]), float(host[1]), int(host[2:3].view(torch.int64)[0])


def partial_recover(x, c, block_len, lost_idx, workspace=None, want_norm=True, norm_out=None, n_lost=None):
    """scar_partial_recover: x[b] <- c[b] for the lost blocks; returns the device scar_norm
    buffer (read it with read_norm) or None."""
    _dev(x, "x"), _dev(c, "c"), _idx(lost_idx, "lost_idx")
    lay = layout_of(x, block_len, c)
    n = lost_idx.numel() if n_lost is None else int(n_lost)
    if n > lost_idx.numel():
        raise ValueError("n_lost exceeds the index list")
    if want_norm and norm_out is None:
        norm_out = _norm_buffer(x.device)
    if not want_norm:
        norm_out = None
    _check(lib().scar_partial_recover(ctypes.byref(lay), _p(x), _p(c), _p(lost_idx), n, _p(norm_out),
                                      _p(workspace), _bytes(workspace),
                                      _stream()), "scar_partial_recover")
    return norm_out


def perturbation_norm(x, c, block_len, idx, workspace, norm_out=None, n_idx=None):
    """scar_perturbation_norm over the blocks in idx (None = all blocks); returns the device
    scar_norm buffer."""
    _dev(x, "x"), _dev(c, "c"), _dev(workspace, "workspace")
    lay = layout_of(x, block_len, c)
    if norm_out is None:
        norm_out = _norm_buffer(x.device)
    if idx is None:
        ptr, n = ctypes.c_void_p(0), 0
    else:
        _idx(idx, "idx")
        n = idx.numel() if n_idx is None else int(n_idx)
        if n > idx.numel():
            raise ValueError("n_idx exceeds the index list")
        # an empty list means "no blocks", not "all blocks": keep the pointer non-NULL
        ptr = _p(idx) if idx.numel() else _p(norm_out)
    _check(lib().scar_perturbation_norm(ctypes.byref(lay), _p(x), _p(c), ptr, n, _p(norm_out),
                                        _p(workspace), _bytes(workspace), _stream()),
           "scar_perturbation_norm")
    return norm_out


def mask_to_indices(mask, workspace):
    """scar_mask_to_indices: (indices buffer of n_blocks int32, device count tensor)."""
    _dev(mask, "mask"), _dev(workspace, "workspace")
    if mask.dtype not in (torch.uint8, torch.bool):
        raise TypeError("mask must be uint8 or bool")
    out = torch.empty(mask.numel(), dtype=torch.int32, device=mask.device)
    cnt = torch.empty(1, dtype=torch.int32, device=mask.device)
    _check(lib().scar_mask_to_indices(_p(mask), mask.numel(), _p(out), _p(cnt), _p(workspace), _bytes(workspace), _stream()), "scar_mask_to_indices")
    return out, cnt


def select_round(n_blocks_, k, cursor, device, out=None):
    """scar_select_round: the round-robin strategy's k blocks from `cursor` on, ascending."""
    if out is None:
        out = torch.empty(int(k), dtype=torch.int32, device=device)
    _check(lib().scar_select_round(int(n_blocks_), int(k), int(cursor), _p(out), _stream()),
           "scar_select_round")
    return out


def select_random(n_blocks_, k, seed, draw, workspace, out=None):
    """scar_select_random: a seeded uniformly random k-subset of the blocks, ascending."""
    _dev(workspace, "workspace")
    if out is None:
        out = torch.empty(int(k), dtype=torch.int32, device=workspace.device)
    _check(lib().scar_select_random(int(n_blocks_), int(k), int(seed), int(draw), _p(out),
                                    _p(workspace), _bytes(workspace), _stream()), "scar_select_random")
    return out


# ---- blocks of unequal length -------------------------------------------------------------

def var_layout_of(x, offsets, c=None) -> VarLayout:
    """offsets: int64 device tensor of n_blocks + 1 element offsets (offsets[0] = 0).  c (or
    packed rows of c's type) decides between a plain store and float32 x with a bfloat16 c."""
    _dev(offsets, "offsets")
    if offsets.dtype != torch.int64:
        raise TypeError("offsets must be an int64 tensor")
    return VarLayout(store_type(x, c), offsets.numel() - 1, x.numel(), offsets.data_ptr())


def var_workspace_bytes(n_blocks_: int) -> int:
    return int(lib().scar_var_workspace_bytes(int(n_blocks_)))


def new_var_workspace(n_blocks_: int, device) -> torch.Tensor:
    return torch.empty(var_workspace_bytes(n_blocks_), dtype=torch.uint8, device=device)


def var_block_scores(x, c, offsets, workspace, out=None):
    """scar_var_block_scores."""
    _dev(x, "x"), _dev(c, "c"), _dev(workspace, "workspace")
    if x.numel() != c.numel():
        raise ValueError("x and c must have the same size")
    lay = var_layout_of(x, offsets, c)
    if out is None:
        out = torch.empty(lay.n_blocks, dtype=torch.int64 if x.dtype == torch.int32 else torch.float32,
                          device=x.device)
    _check(lib().scar_var_block_scores(ctypes.byref(lay), _p(x), _p(c), _p(out), _p(workspace), _bytes(workspace), _stream()), "scar_var_block_scores")
    return out


def var_checkpoint_commit(x, c, offsets, idx, workspace):
    """scar_var_checkpoint_commit."""
    _dev(x, "x"), _dev(c, "c"), _idx(idx, "idx"), _dev(workspace, "workspace")
    lay = var_layout_of(x, offsets, c)
    _check(lib().scar_var_checkpoint_commit(ctypes.byref(lay), _p(x), _p(c), _p(idx), idx.numel(),
                                            _p(workspace), _bytes(workspace), _stream()),
           "scar_var_checkpoint_commit")


def var_checkpoint_commit_staged(x, c, offsets, idx, workspace, staging):
    """scar_var_checkpoint_commit_staged: also packs the listed blocks into staging; returns the
    device tensor of their n_idx + 1 element offsets (int64)."""
    _dev(x, "x"), _dev(c, "c"), _idx(idx, "idx"), _dev(workspace, "workspace"), _dev(staging, "staging")
    if staging.dtype != c.dtype:
        raise TypeError("staging must have c's element type")
    lay = var_layout_of(x, offsets, c)
    st_off = torch.empty(idx.numel() + 1, dtype=torch.int64, device=x.device)
    _check(lib().scar_var_checkpoint_commit_staged(ctypes.byref(lay), _p(x), _p(c), _p(idx), idx.numel(),
                                                   _p(staging), _p(st_off), _p(workspace), _bytes(workspace),
                                                   _stream()), "scar_var_checkpoint_commit_staged")
    return st_off


def var_partial_recover_rows(x, rows, row_offsets, offsets, lost_idx, workspace, want_norm=True):
    """scar_var_partial_recover_rows: x[b] <- the packed row of block b for the lost blocks;
    returns the device scar_norm buffer or None."""
    _dev(x, "x"), _dev(rows, "rows"), _dev(row_offsets, "row_offsets"), _idx(lost_idx, "lost_idx")
    _dev(workspace, "workspace")
    if row_offsets.dtype != torch.int64 or row_offsets.numel() < lost_idx.numel():
        raise ValueError("row_offsets must be an int64 tensor with an entry per lost block")
    lay = var_layout_of(x, offsets, rows)
    norm_out = _norm_buffer(x.device) if want_norm else None
    _check(lib().scar_var_partial_recover_rows(ctypes.byref(lay), _p(x), _p(rows), _p(row_offsets), _p(lost_idx),
                                               lost_idx.numel(), _p(norm_out), _p(workspace), _bytes(workspace),
                                               _stream()), "scar_var_partial_recover_rows")
    return norm_out


def var_partial_recover(x, c, offsets, lost_idx, workspace, want_norm=True):
    """scar_var_partial_recover; returns the device scar_norm buffer or None."""
    _dev(x, "x"), _dev(c, "c"), _idx(lost_idx, "lost_idx"), _dev(workspace, "workspace")
    lay = var_layout_of(x, offsets, c)
    norm_out = _norm_buffer(x.device) if want_norm else None
    _check(lib().scar_var_partial_recover(ctypes.byref(lay), _p(x), _p(c), _p(lost_idx), lost_idx.numel(),
                                          _p(norm_out), _p(workspace), _bytes(workspace), _stream()),
           "scar_var_partial_recover")
    return norm_out


def var_perturbation_norm(x, c, offsets, idx, workspace):
    """scar_var_perturbation_norm (idx None = every block)."""
    _dev(x, "x"), _dev(c, "c"), _dev(workspace, "workspace")
    lay = var_layout_of(x, offsets, c)
    norm_out = _norm_buffer(x.device)
    if idx is None:
        ptr, n = ctypes.c_void_p(0), 0
    else:
        _idx(idx, "idx")
        n = idx.numel()
        ptr = _p(idx) if n else _p(norm_out)
    _check(lib().scar_var_perturbation_norm(ctypes.byref(lay), _p(x), _p(c), ptr, n, _p(norm_out),
                                            _p(workspace), _bytes(workspace), _stream()),
           "scar_var_perturbation_norm")
    return norm_out


# ---- document-length-scaled total variation (float rows that are distributions) ----------

def _weights(weights, n_blocks_, device):
    if weights is None:
        return None
    _dev(weights, "weights")
    if weights.dtype != torch.float32 or weights.numel() != n_blocks_ or not weights.is_contiguous():
        raise ValueError("weights must be a contiguous float32 tensor with one entry per block")
    return weights


def tv_block_scores(x, c, block_len, weights=None, out=None):
    """scar_tv_block_scores: w_b * TV(x_b, c_b) per block (float32)."""
    _dev(x, "x"), _dev(c, "c")
    lay = layout_of(x, block_len, c)
    nb = n_blocks(lay)
    w = _weights(weights, nb, x.device)
    if out is None:
        out = torch.empty(nb, dtype=torch.float32, device=x.device)
    _check(lib().scar_tv_block_scores(ctypes.byref(lay), _p(x), _p(c), _p(w), _p(out), _stream()),
           "scar_tv_block_scores")
    return out


def tv_partial_recover(x, c, block_len, lost_idx, workspace, weights=None, want_norm=True):
    """scar_tv_partial_recover; returns the device scar_norm buffer or None."""
    _dev(x, "x"), _dev(c, "c"), _idx(lost_idx, "lost_idx")
    lay = layout_of(x, block_len, c)
    w = _weights(weights, n_blocks(lay), x.device)
    norm_out = _norm_buffer(x.device) if want_norm else None
    if want_norm:
        _dev(workspace, "workspace")
    _check(lib().scar_tv_partial_recover(ctypes.byref(lay), _p(x), _p(c), _p(w), _p(lost_idx), lost_idx.numel(),
                                         _p(norm_out), _p(workspace), _bytes(workspace),
                                         _stream()), "scar_tv_partial_recover")
    return norm_out


def tv_perturbation_norm(x, c, block_len, idx, workspace, weights=None):
    """scar_tv_perturbation_norm (idx None = every block)."""
    _dev(x, "x"), _dev(c, "c"), _dev(workspace, "workspace")
    lay = layout_of(x, block_len, c)
    w = _weights(weights, n_blocks(lay), x.device)
    norm_out = _norm_buffer(x.device)
    if idx is None:
        ptr, n = ctypes.c_void_p(0), 0
    else:
        _idx(idx, "idx")
        n = idx.numel()
        ptr = _p(idx) if n else _p(norm_out)
    _check(lib().scar_tv_perturbation_norm(ctypes.byref(lay), _p(x), _p(c), _p(w), ptr, n, _p(norm_out),
                                           _p(workspace), _bytes(workspace), _stream()),
           "scar_tv_perturbation_norm")
    return norm_out


def var_tv_block_scores(x, c, offsets, workspace, weights=None, out=None):
    """scar_var_tv_block_scores: w_b * TV(x_b, c_b) per block of unequal length (float32)."""
    _dev(x, "x"), _dev(c, "c"), _dev(workspace, "workspace")
    lay = var_layout_of(x, offsets)
    w = _weights(weights, lay.n_blocks, x.device)
    if out is None:
        out = torch.empty(lay.n_blocks, dtype=torch.float32, device=x.device)
    _check(lib().scar_var_tv_block_scores(ctypes.byref(lay), _p(x), _p(c), _p(w), _p(out), _p(workspace),
                                          _bytes(workspace), _stream()), "scar_var_tv_block_scores")
    return out


def var_tv_partial_recover(x, c, offsets, lost_idx, workspace, weights=None, want_norm=True):
    """scar_var_tv_partial_recover; returns the device scar_norm buffer or None."""
    _dev(x, "x"), _dev(c, "c"), _idx(lost_idx, "lost_idx"), _dev(workspace, "workspace")
    lay = var_layout_of(x, offsets)
    w = _weights(weights, lay.n_blocks, x.device)
    norm_out = _norm_buffer(x.device) if want_norm else None
    _check(lib().scar_var_tv_partial_recover(ctypes.byref(lay), _p(x), _p(c), _p(w), _p(lost_idx),
                                             lost_idx.numel(), _p(norm_out), _p(workspace), _bytes(workspace),
                                             _stream()), "scar_var_tv_partial_recover")
    return norm_out


def var_tv_perturbation_norm(x, c, offsets, idx, workspace, weights=None):
    """scar_var_tv_perturbation_norm (idx None = every block)."""
    _dev(x, "x"), _dev(c, "c"), _dev(workspace, "workspace")
    lay = var_layout_of(x, offsets)
    w = _weights(weights, lay.n_blocks, x.device)
    norm_out = _norm_buffer(x.device)
    if idx is None:
        ptr, n = ctypes.c_void_p(0), 0
    else:
        _idx(idx, "idx")
        n = idx.numel()
        ptr = _p(idx) if n else _p(norm_out)
    _check(lib().scar_var_tv_perturbation_norm(ctypes.byref(lay), _p(x), _p(c), _p(w), ptr, n, _p(norm_out),
                                               _p(workspace), _bytes(workspace), _stream()),
           "scar_var_tv_perturbation_norm")
    return norm_out


# ---- persistent-storage leg (include/scar_store.h) ----------------------------------------

class Store:
    """scar_store: the running checkpoint in a file, written by a background thread."""

    def __init__(self, path, max_rows, layout=None):
        """layout given: create (truncate) the file for that layout; else open an existing file."""
        self._h = ctypes.c_void_p(0)
        self.layout = Layout()
        if layout is not None:
            self.layout = layout
            _check(lib().scar_store_create(os.fsencode(path), ctypes.byref(layout), int(max_rows),
                                           ctypes.byref(self._h)), "scar_store_create")
        else:
            _check(lib().scar_store_open(os.fsencode(path), int(max_rows), ctypes.byref(self.layout),
                                         ctypes.byref(self._h)), "scar_store_open")

    def save_async(self, staging, idx, n_idx=None):
        _dev(staging, "staging"), _idx(idx, "idx")
        n = idx.numel() if n_idx is None else int(n_idx)
        _check(lib().scar_store_save_async(self._h, _p(staging), _p(idx), n, _stream()),
               "scar_store_save_async")

    def wait(self):
        _check(lib().scar_store_wait(self._h), "scar_store_wait")

    def load(self, idx_host, rows):
        """Reads the blocks idx_host (sequence of ints) into the packed device rows tensor."""
        import numpy as np
        idx_host = np.ascontiguousarray(idx_host, dtype=np.uint32)
        _dev(rows, "rows")
        _check(lib().scar_store_load(self._h, ctypes.c_void_p(idx_host.ctypes.data), idx_host.size,
                                     _p(rows), _stream()), "scar_store_load")
        return rows

    def close(self):
        if self._h:
            h, self._h = self._h, ctypes.c_void_p(0)
            _check(lib().scar_store_close(h), "scar_store_close")


class VarStore:
    """scar_store for blocks of unequal length: the running checkpoint of a by-layer store in a
    file, written by the same background thread."""

    def __init__(self, path, dtype, offsets_host, max_rows, max_elems):
        import numpy as np
        self._h = ctypes.c_void_p(0)
        off = np.ascontiguousarray(offsets_host, dtype=np.uint64)
        _check(lib().scar_var_store_create(os.fsencode(path), int(dtype), off.size - 1,
                                           ctypes.c_void_p(off.ctypes.data), int(max_rows), int(max_elems),
                                           ctypes.byref(self._h)), "scar_var_store_create")

    def save_async(self, staging, staging_elems, idx):
        _dev(staging, "staging"), _idx(idx, "idx")
        if staging_elems > staging.numel():
            raise ValueError("staging_elems exceeds the staging buffer")
        _check(lib().scar_var_store_save_async(self._h, _p(staging), int(staging_elems), _p(idx), idx.numel(),
                                               _stream()), "scar_var_store_save_async")

    def wait(self):
        _check(lib().scar_store_wait(self._h), "scar_store_wait")

    def load(self, idx_host, rows):
        """Reads the blocks idx_host into the packed device tensor rows; returns the device tensor
        of their n_idx + 1 element offsets (int64)."""
        import numpy as np
        idx_host = np.ascontiguousarray(idx_host, dtype=np.uint32)
        _dev(rows, "rows")
        row_off = torch.empty(idx_host.size + 1, dtype=torch.int64, device=rows.device)
        _check(lib().scar_var_store_load(self._h, ctypes.c_void_p(idx_host.ctypes.data), idx_host.size,
                                         _p(rows), _p(row_off), _stream()), "scar_var_store_load")
        return row_off

    def close(self):
        if self._h:
            h, self._h = self._h, ctypes.c_void_p(0)
            _check(lib().scar_store_close(h), "scar_store_close")


def partial_recover_rows(x, rows, block_len, lost_idx, workspace=None, want_norm=True):
    """scar_partial_recover_rows: x[b] <- rows[i] for b = lost_idx[i]; returns the device
    scar_norm buffer or None."""
    _dev(x, "x"), _dev(rows, "rows"), _idx(lost_idx, "lost_idx")
    lay = Layout(store_type(x, rows), int(block_len), x.numel())
    if rows.numel() < lost_idx.numel() * block_len:
        raise ValueError("rows must hold lost_idx.numel() * block_len elements")
    norm_out = _norm_buffer(x.device) if want_norm else None
    _check(lib().scar_partial_recover_rows(ctypes.byref(lay), _p(x), _p(rows), _p(lost_idx),
                                           lost_idx.numel(), _p(norm_out), _p(workspace),
                                           _bytes(workspace), _stream()),
           "scar_partial_recover_rows")
    return norm_out
