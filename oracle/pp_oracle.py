"""ctypes front end of pp_oracle.c: the steps before and after the main all-reduce
(statistics, their combination, bit allocation, reorder, the means of the main stage, restore).

TEST INFRASTRUCTURE, NOT PRODUCT CODE: only tests, the smoke check and the
benchmark's cpu_baseline leg may import this module.
"""
import ctypes as C

import numpy as np

from . import dq_oracle as _O

_ready = False


def _lib():
    global _ready
    L = _O.lib()
    if not _ready:
        L.ppo_bf16_rne.restype = C.c_uint16
        L.ppo_bf16_rne.argtypes = [C.c_float]
        L.ppo_sg_stats.argtypes = [C.c_void_p, C.c_int, C.c_uint64, C.c_void_p, C.c_void_p]
        L.ppo_stats_combine.argtypes = [C.c_void_p, C.c_void_p, C.c_uint32, C.c_uint64, C.c_void_p, C.c_void_p]
        L.ppo_width.restype = C.c_int
        L.ppo_width.argtypes = [C.c_float, C.c_float, C.c_int]
        L.ppo_cost.restype = C.c_uint64
        L.ppo_cost.argtypes = [C.c_void_p, C.c_uint64, C.c_float, C.c_int]
        L.ppo_allocate.restype = C.c_int64
        L.ppo_allocate.argtypes = [C.c_void_p, C.c_uint64, C.c_uint64, C.c_int, C.c_void_p]
        L.ppo_positions.argtypes = [C.c_void_p, C.c_uint64, C.c_void_p, C.c_void_p]
        L.ppo_reorder.argtypes = [C.c_void_p, C.c_int, C.c_void_p, C.c_uint64, C.c_void_p]
        L.ppo_reorder_mean.argtypes = [C.c_void_p, C.c_void_p, C.c_uint64, C.c_uint32, C.c_void_p]
        L.ppo_restore.argtypes = [C.c_void_p, C.c_void_p, C.c_void_p, C.c_uint32, C.c_uint64, C.c_void_p]
        _ready = True
    return L


def _p(a):
    return a.ctypes.data_as(C.c_void_p)


def _dtype_code(a):
    """fp32 arrays are float32; bf16 arrays travel as uint16 bit patterns."""
    if a.dtype == np.float32:
        return 0
    if a.dtype == np.uint16:
        return 1
    raise TypeError("gradients are float32 or uint16 (bf16 patterns)")


def bf16_rne(f):
    return int(_lib().ppo_bf16_rne(np.float32(f)))


def sg_stats(x):
    """(mu, F) per super-group in float64 (Section 3.1)."""
    x = np.ascontiguousarray(x)
    n_sg = x.size // 256
    mu = np.empty(n_sg, np.float64)
    F = np.empty(n_sg, np.float64)
    _lib().ppo_sg_stats(_p(x), _dtype_code(x), n_sg, _p(mu), _p(F))
    return mu, F


def stats_combine(mu_all, F_all):
    """mu_all, F_all: float32 [n, J] per-worker statistics -> (mu, F) float32 [J]."""
    mu_all = np.ascontiguousarray(mu_all, np.float32)
    F_all = np.ascontiguousarray(F_all, np.float32)
    n, J = mu_all.shape
    mu = np.empty(J, np.float32)
    F = np.empty(J, np.float32)
    _lib().ppo_stats_combine(_p(mu_all), _p(F_all), n, J, _p(mu), _p(F))
    return mu, F


def width(F, theta, max_width=8):
    return int(_lib().ppo_width(np.float32(F), np.float32(theta), int(max_width)))


def cost(F, theta, max_width=8):
    F = np.ascontiguousarray(F, np.float32)
    return int(_lib().ppo_cost(_p(F), F.size, np.float32(theta), int(max_width)))


def allocate(F, max_code_bits, max_width=8):
    """-> (widths uint8 [J], threshold bit pattern); raises if even 2 bits everywhere do not fit.
    max_width 8: W = {2,4,8}; 16: W = {2,4,8,16}."""
    F = np.ascontiguousarray(F, np.float32)
    w = np.empty(F.size, np.uint8)
    t = int(_lib().ppo_allocate(_p(F), F.size, int(max_code_bits), int(max_width), _p(w)))
    if t < 0:
        raise ValueError("budget below 2 code bits per coordinate")
    return w, t


def positions(widths):
    widths = np.ascontiguousarray(widths, np.uint8)
    pos = np.empty(widths.size, np.uint32)
    counts = np.zeros(4, np.uint32)      # 2, 4, 8, 16 bits
    _lib().ppo_positions(_p(widths), widths.size, _p(pos), _p(counts))
    return pos, [int(c) for c in counts]


def reorder(x, pos):
    """Whole super-groups of x moved to their places pos (Section 3.5)."""
    x = np.ascontiguousarray(x)
    pos = np.ascontiguousarray(pos, np.uint32)
    out = np.empty_like(x)
    _lib().ppo_reorder(_p(x), _dtype_code(x), _p(pos), pos.size, _p(out))
    return out


def reorder_mean(mu, pos, n16):
    """The means the main stage subtracts, in reordered order: zero for the last n16
    (uncompressed) super-groups."""
    mu = np.ascontiguousarray(mu, np.float32)
    pos = np.ascontiguousarray(pos, np.uint32)
    out = np.empty_like(mu)
    _lib().ppo_reorder_mean(_p(mu), _p(pos), pos.size, int(n16), _p(out))
    return out


def restore(total, pos, mu_main, n_workers):
    """total: the main stage's sums in reordered order; mu_main: what reorder_mean returned, or None."""
    total = np.ascontiguousarray(total, np.float32)
    pos = np.ascontiguousarray(pos, np.uint32)
    out = np.empty_like(total)
    m = None if mu_main is None else np.ascontiguousarray(mu_main, np.float32)
    _lib().ppo_restore(_p(total), _p(pos), None if m is None else _p(m), int(n_workers), pos.size, _p(out))
    return out
