"""The C-ABI boundary without a GPU: the library loads, exports every symbol that
include/scar.h declares, and its host-side checks answer with status codes."""
import ctypes
import os
import re

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
HEADER = os.path.join(ROOT, "include", "scar.h")
HEADERS = [os.path.join(ROOT, "include", f) for f in sorted(os.listdir(os.path.join(ROOT, "include")))
           if f.endswith(".h")]


@pytest.fixture(scope="module")
def lib():
    from paper_1810_07354_amd import build, scar
    if build.stale():
        build.build(force=True)
    return scar.lib()


def declared_symbols():
    text = "\n".join(open(h).read() for h in HEADERS)
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(scar_[a-z_0-9]+)\s*\(", text)))


def test_header_declares_the_five_calls_of_the_path():
    names = declared_symbols()
    for want in ("scar_block_scores", "scar_select_topk", "scar_checkpoint_commit",
                 "scar_partial_recover", "scar_perturbation_norm"):
        assert want in names


def test_every_declared_symbol_is_exported(lib):
    for name in declared_symbols():
        assert hasattr(lib, name), name


def test_strerror_and_sizes(lib):
    from paper_1810_07354_amd import scar
    assert scar.strerror(0) == "ok"
    for code in (-1, -2, -3, 17):
        assert scar.strerror(code)
    small, big = scar.workspace_bytes(1), scar.workspace_bytes(1 << 20)
    assert 0 < small <= big and big < 1 << 20 and small % 256 == 0
    assert scar.workspace_bytes(scar.MAX_BLOCKS + 1) == 0
    assert scar.n_blocks(scar.Layout(scar.F32, 4096, 25_000_000)) == 6104
    assert scar.n_blocks(scar.Layout(scar.F32, 1024, 1 << 30)) == 1 << 20
    assert scar.n_blocks(scar.Layout(scar.F32, 0, 10)) == 0
    assert scar.n_blocks(scar.Layout(7, 4, 10)) == 0
    assert scar.n_blocks(scar.Layout(scar.I32, 1, 1 << 32)) == 0        # too many blocks


def test_host_checks_reject_bad_arguments_before_any_gpu_work(lib):
    from paper_1810_07354_amd import scar
    null = ctypes.c_void_p(0)
    fake = ctypes.c_void_p(0x1000)          # never dereferenced: every call below fails first
    lay = scar.Layout(scar.F32, 0, 100)
    assert lib.scar_block_scores(ctypes.byref(lay), fake, fake, fake, null) == -1
    lay = scar.Layout(scar.F32, 10, 100)
    assert lib.scar_block_scores(ctypes.byref(lay), null, fake, fake, null) == -1
    assert lib.scar_block_scores(ctypes.byref(lay), ctypes.c_void_p(0x1002), fake, fake, null) == -1
    assert lib.scar_select_topk(0, fake, 10, 11, fake, fake, 1 << 20, null) == -1
    assert lib.scar_select_topk(5, fake, 10, 1, fake, fake, 1 << 20, null) == -1
    assert lib.scar_select_topk(0, fake, 10, 1, fake, null, 0, null) == -2
    assert lib.scar_select_topk(0, fake, 10, 1, fake, fake, 16, null) == -2
    assert lib.scar_select_topk(0, fake, 10, 0, null, null, 0, null) == 0      # k = 0: nothing to do
    assert lib.scar_checkpoint_commit(ctypes.byref(lay), fake, fake, null, 3, null, null) == -1
    assert lib.scar_checkpoint_commit(ctypes.byref(lay), fake, fake, null, 0, null, null) == 0
    assert lib.scar_partial_recover(ctypes.byref(lay), fake, fake, fake, 3, fake, null, 0, null) == -2
    assert lib.scar_partial_recover(ctypes.byref(lay), fake, fake, null, 0, null, null, 0, null) == 0
    assert lib.scar_perturbation_norm(ctypes.byref(lay), fake, fake, null, 0, null, fake, 1 << 20, null) == -1
    assert lib.scar_mask_to_indices(fake, 10, fake, null, fake, 1 << 20, null) == -1


def test_binding_refuses_cpu_tensors():
    import torch
    from paper_1810_07354_amd import scar
    x = torch.zeros(16)
    with pytest.raises(TypeError):
        scar.block_scores(x, x.clone(), 4)


def test_binding_checks_index_and_output_types_before_calling():
    # wrong tensors are refused in Python, before any pointer reaches the library (CPU tensors
    # are refused first, so these checks are exercised through the helpers)
    import pytest
    import torch
    from paper_1810_07354_amd import scar
    with pytest.raises(TypeError):
        scar._idx(torch.zeros(4, dtype=torch.int64), "idx")         # not on the GPU
    assert scar._bytes(None) == 0
    assert scar._bytes(torch.zeros(6, dtype=torch.float64)) == 48
