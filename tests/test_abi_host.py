"""The C-ABI library loads and exports every symbol the header declares; host-only calls
behave (no GPU needed, no compute is launched)."""
import ctypes as C
import os
import re

import pytest

from paper_2211_10280_amd import binding as B

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def _declared():
    src = open(os.path.join(ROOT, "include", "tensair.h")).read()
    src = re.sub(r"/\*.*?\*/", "", src, flags=re.S)
    return sorted(set(re.findall(r"\b(tensair_[a-z_]+)\s*\(", src)))


def test_every_declared_symbol_is_exported():
    if not os.path.exists(B.LIB_PATH):
        pytest.fail("libtensair.so has not been built (python -m paper_2211_10280_amd.build)")
    L = C.CDLL(B.LIB_PATH)
    names = _declared()
    assert len(names) >= 27
    for n in names:
        assert hasattr(L, n), n
    assert sorted(B.SYMBOLS) == names        # the binding forwards to exactly these


def test_host_side_argument_checks():
    L = B.lib()
    good = B.Config(1000, 32, 32, B.F32, 2, 5, 64, 0, 0, 7)
    assert B.tensair_workspace_bytes(good) > 2 * 1000 * 4
    assert B.tensair_aligned_row_stride(300, B.F32) == 320 and B.tensair_aligned_row_stride(300, B.BF16) == 320
    assert B.tensair_aligned_row_stride(512, B.BF16) == 512 and B.tensair_aligned_row_stride(4, B.F32) == 32
    assert L.tensair_aligned_row_stride(0, B.F32) == -1 and L.tensair_aligned_row_stride(8, 9) == -1
    assert B.tensair_capacity_in(good, 64) == 64
    assert B.tensair_capacity_out(good, 64) == 1000          # min(V, 2*2*64*6 = 1536)
    assert B.tensair_capacity_out(good, 10) == 240
    assert B.tensair_workspace_bytes(B.Config(1000, 32, 32, B.F32, 2, 5, 64, 0, 0, 7, B.RESAMPLE_NEGATIVES)) > 0
    # sizes beyond what one launch of the update kernels covers are refused, the largest allowed ones are not
    assert B.tensair_workspace_bytes(B.Config(B.MAX_VOCAB, 4, 4, B.F32, 1, 0, 1, 0, 0, 7)) > 0
    with pytest.raises(B.TensairError):
        B.tensair_workspace_bytes(B.Config(B.MAX_VOCAB + 1, 4, 4, B.F32, 1, 0, 1, 0, 0, 7))
    for bad in (B.Config(0, 32, 32, B.F32, 2, 5, 64, 0, 0, 7),      # vocab
                B.Config(1000, 30, 32, B.F32, 2, 5, 64, 0, 0, 7),    # dim not a multiple of 4
                B.Config(1000, 32, 28, B.F32, 2, 5, 64, 0, 0, 7),    # stride < dim
                B.Config(1000, 32, 32, 5, 2, 5, 64, 0, 0, 7),        # dtype
                B.Config(1000, 32, 32, B.F32, 0, 5, 64, 0, 0, 7),    # window
                B.Config(1000, 32, 32, B.F32, 2, 5, 64, 32, 0, 7),   # too many peers
                B.Config(1000, 32, 32, B.F32, 2, 5, 64, 0, 70000, 7),   # worker id
                B.Config(1000, 32, 32, B.F32, 2, 5, 64, 0, 0, 7, 4)):   # unknown flag
        with pytest.raises(B.TensairError):
            B.tensair_workspace_bytes(bad)
    assert L.tensair_last_error()                                # a message is left behind
    # NULL handles are rejected, not dereferenced
    assert L.tensair_model_rebind(None, None, None, 0) == B.EINVAL
    assert L.tensair_dasgd_apply(None, None, None, 0, 0.1, None) == B.EINVAL
    assert L.tensair_status(None, None) == B.EINVAL
    assert L.tensair_pair_count(None, 10, 0, 1) == -1
    h = C.c_void_p()
    assert L.tensair_model_init(C.byref(h), C.byref(good), None, None, 1, None, None, 0, None) == B.EINVAL
    assert h.value is None


def test_host_side_argument_checks_of_the_further_entry_points():
    """Everything below is refused on the host, before any GPU call is made."""
    L = B.lib()
    buf = (C.c_float * 64)()
    addr = C.addressof(buf)
    aligned = (addr + 15) & ~15
    ptrs = (C.c_void_p * 40)(*([aligned] * 40))
    # dense apply: NULL theta, unknown dtype, negative n, too many blocks, NaN step, misaligned pointers
    assert L.tensair_dense_apply(None, B.F32, 16, ptrs, 1, 0.1, None) == B.EINVAL
    assert L.tensair_dense_apply(aligned, 7, 16, ptrs, 1, 0.1, None) == B.EINVAL
    assert L.tensair_dense_apply(aligned, B.F32, -1, ptrs, 1, 0.1, None) == B.EINVAL
    assert L.tensair_dense_apply(aligned, B.F32, B.MAX_DENSE + 4, ptrs, 1, 0.1, None) == B.EINVAL
    assert L.tensair_dense_apply(aligned, B.F32, 16, ptrs, B.MAX_PEERS + 2, 0.1, None) == B.ECAPACITY
    assert L.tensair_dense_apply(aligned, B.F32, 16, ptrs, 1, float("nan"), None) == B.EINVAL
    assert L.tensair_dense_apply(aligned + 4, B.F32, 16, ptrs, 1, 0.1, None) == B.EINVAL
    assert L.tensair_dense_apply(aligned, B.F32, 16, None, 1, 0.1, None) == B.EINVAL
    # nothing to do is not an error and launches nothing
    assert L.tensair_dense_apply(aligned, B.F32, 0, ptrs, 1, 0.1, None) == B.OK
    assert L.tensair_dense_apply(aligned, B.F32, 16, ptrs, 0, 0.1, None) == B.OK
    # cosine difference: NULL, dtype, shape
    assert L.tensair_cosine_difference(None, aligned, B.F32, 4, 4, 4, aligned, None) == B.EINVAL
    assert L.tensair_cosine_difference(aligned, aligned, 3, 4, 4, 4, aligned, None) == B.EINVAL
    assert L.tensair_cosine_difference(aligned, aligned, B.F32, 4, 6, 8, aligned, None) == B.EINVAL
    assert L.tensair_cosine_difference(aligned, aligned, B.F32, 4, 8, 4, aligned, None) == B.EINVAL
    assert L.tensair_cosine_difference(aligned, aligned, B.F32, -1, 4, 4, aligned, None) == B.EINVAL
    # the entry point with the fixed scratch: sizes beyond it are refused first, then the usual checks
    assert L.tensair_dasgd_apply_static(aligned, aligned, B.STATIC_MAX_VOCAB + 1, 4, 4, B.F32, None, None, 0, 0.1, None, None) == B.ECAPACITY
    assert L.tensair_dasgd_apply_static(aligned, aligned, 64, 4, 4, B.F32, None, None, B.STATIC_MAX_PEERS + 1, 0.1, None, None) == B.ECAPACITY
    assert L.tensair_dasgd_apply_static(None, aligned, 64, 4, 4, B.F32, None, None, 0, 0.1, None, None) == B.EINVAL
    assert L.tensair_dasgd_apply_static(aligned, aligned, 64, 6, 8, B.F32, None, None, 0, 0.1, None, None) == B.EINVAL
    assert L.tensair_dasgd_apply_static(aligned, aligned, 64, 4, 4, B.F32, None, None, 1, 0.1, None, None) == B.EINVAL
    assert L.tensair_dasgd_apply_static(aligned, aligned, 64, 4, 4, B.F32, None, None, 0, 0.1, None, None) == B.OK   # nothing to apply
    assert L.tensair_stream_probe(aligned, aligned + 4, 64, 0, None) == B.EINVAL
    assert L.tensair_stream_probe(aligned, aligned, 64, 7, None) == B.EINVAL
    # calls that need a model
    assert L.tensair_lookup(None, 0, None, 0, None, None) == B.EINVAL
    assert L.tensair_grad_add(None, None, None, None, None) == B.EINVAL
    assert L.tensair_prefetch(None, None, 1, 0, 0, 0, None) == B.EINVAL
    assert L.tensair_step(None, None, 1, 0, 0, 0, None, 0, 0.1, None, None, None) == B.EINVAL
    assert L.tensair_sgns_grad(None, None, 1, 0, 0, 0, None, None, None, None, None, None) == B.EINVAL
    assert L.tensair_profile(None, 1) == B.EINVAL
    assert L.tensair_model_destroy(None) == B.OK             # destroying nothing is allowed


def test_bench_refuses_more_than_one_gpu():
    """This build is the one-GPU worker step: bench.py says so and exits instead of pretending to scale."""
    import subprocess
    import sys
    r = subprocess.run([sys.executable, os.path.join(ROOT, "bench.py"), "--gpus", "2"], capture_output=True, text=True)
    assert r.returncode != 0 and "one-GPU" in r.stderr and r.stdout.strip() == ""
