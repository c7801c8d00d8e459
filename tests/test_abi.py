"""The C-ABI library loads and exports every symbol include/dq.h declares (no GPU needed),
and its pure host functions agree with the oracle's layout arithmetic."""
import ctypes
import os
import re

import pytest

from oracle import dq_oracle as O
from paper_2602_08923_amd import binding as B

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def declared_functions():
    text = open(os.path.join(ROOT, "include", "dq.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(dq_[a-z0-9_]+)\s*\(", text)))


def test_library_exports_every_declared_symbol():
    if not os.path.exists(B.LIB_PATH):
        import __graft_entry__
        __graft_entry__.build()
    lib = ctypes.CDLL(B.LIB_PATH)
    names = declared_functions()
    assert len(names) >= 20
    for n in names:
        assert hasattr(lib, n), f"libdq.so does not export {n}"
    assert sorted(B.EXPORTS) == names


def test_host_only_functions():
    L = B.lib()
    for n_sg in ([0, 0, 0], [1, 0, 0], [5, 7, 3], [0, 5900, 500], [123456, 7, 99999]):
        assert B.dq_packed_bytes(B.make_chunk(0, n_sg)) == O.Oracle.packed_bytes(O.make_chunk(0, n_sg))
    for fmt in (1, 2, 3):
        for n in (256, 256 * 37, 13_107_200):
            assert B.dq_mx_packed_bytes(fmt, n) == O.mx_packed_bytes(fmt, n)
        assert B.dq_mx_packed_bytes(fmt, 100) == 0      # not a multiple of 256
    assert B.dq_mx_packed_bytes(0, 256) == 0            # not an MX format
    assert L.dq_status_str(0) == b"ok" and L.dq_status_str(2).startswith(b"pointer")
    # bits per entry of the two codecs, from the sizes alone (Section 3.5 accounting)
    assert B.dq_packed_bytes(B.make_chunk(0, [0, 5900, 500])) * 8 / (6400 * 256) == 4.875
    assert B.dq_mx_packed_bytes(1, 256 * 64) * 8 / (256 * 64) == 8.25


def test_null_arguments_are_rejected_without_a_gpu():
    L = B.lib()
    h = ctypes.c_void_p()
    assert L.dq_create(None, ctypes.byref(h)) == B.DQ_EINVAL
    cfg = B.Config(1.3, 1.02, 0, 0, 0, 0, 0)   # zero workers
    assert L.dq_create(ctypes.byref(cfg), ctypes.byref(h)) == B.DQ_EINVAL
    cfg = B.Config(1.0, 1.02, 0, 0, 4, 0, 0)   # degenerate level set
    assert L.dq_create(ctypes.byref(cfg), ctypes.byref(h)) == B.DQ_EINVAL
    assert L.dq_compress(None, None, None, 0, None, None) == B.DQ_EINVAL
    assert L.dq_reorder_mean(None, None, None, 4, 1, None, None, None) == B.DQ_EINVAL
    assert L.dq_mx_compress(1, None, 0, 256, None, None) == B.DQ_EINVAL
    assert L.dq_replay_n_steps(None) == 0


def test_replay_binding_checks_the_worker_count():
    """A context of 8 workers and 3 gradient tensors: refused before anything reads past the list."""
    import torch

    class FakeCtx:
        n_workers = 8
        h = None

    with pytest.raises(B.DqError, match="3 worker gradients for a context of 8"):
        B.Replay(FakeCtx(), B.DQ_RING, B.DQ_DYNAMIQ, [torch.zeros(256 * 8, dtype=torch.bfloat16)] * 3, 8, [[0, 8, 0]])
