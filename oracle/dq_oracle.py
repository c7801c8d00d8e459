"""ctypes front end of the CPU oracle (dq_oracle.c, mx_oracle.c; pp_oracle.c is wrapped by pp_oracle.py).

TEST INFRASTRUCTURE, NOT PRODUCT CODE: only tests, the smoke check and the
benchmark's cpu_baseline leg may import this module.  It never imports the GPU
package and the GPU package never imports it.

Besides thin wrappers of the C functions it holds the hop schedules of
Section 3.4 ("Reduce-scatter") written out as plain Python loops over
(worker, chunk): the ring path and the recursive-halving butterfly of
Appendix B, with the kernel each node runs chosen as Section 3.4 "Fused
kernels" says (leaf: compress; last parent received: decompress-accumulate-
recompress; other parents and the sink: decompress-accumulate).
"""
import ctypes as C
import os
import subprocess

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_LIB_PATH = os.path.join(_HERE, "liboracle_dq.so")
_SOURCES = ["dq_oracle.c", "mx_oracle.c", "pp_oracle.c"]
CFLAGS = ["-O2", "-ffp-contract=off", "-fno-fast-math", "-std=c11", "-shared", "-fPIC", "-Wall"]


def build(force=False):
    """Compile the oracle with gcc (plain C, no SIMD intrinsics, no FMA contraction)."""
    srcs = [os.path.join(_HERE, s) for s in _SOURCES if os.path.exists(os.path.join(_HERE, s))]
    if not force and os.path.exists(_LIB_PATH):
        if all(os.path.getmtime(_LIB_PATH) >= os.path.getmtime(s) for s in srcs):
            return _LIB_PATH
    subprocess.check_call(["gcc"] + CFLAGS + srcs + ["-o", _LIB_PATH, "-lm"])
    return _LIB_PATH


class Config(C.Structure):
    _fields_ = [("g4", C.c_double), ("g8", C.c_double), ("seed", C.c_uint64),
                ("round", C.c_uint32), ("n_workers", C.c_uint32), ("independent", C.c_uint32), ("reserved", C.c_uint32)]


class Chunk(C.Structure):
    _fields_ = [("first_sg", C.c_uint64), ("n_sg", C.c_uint32 * 4)]  # 2, 4, 8, 16 bits


_lib = None


def lib():
    global _lib
    if _lib is None:
        L = C.CDLL(build())
        L.dqo_create.restype = C.c_void_p
        L.dqo_create.argtypes = [C.POINTER(Config)]
        L.dqo_destroy.argtypes = [C.c_void_p]
        L.dqo_table_T.restype = C.POINTER(C.c_float)
        L.dqo_table_T.argtypes = [C.c_void_p, C.c_int]
        L.dqo_table_D.restype = C.POINTER(C.c_float)
        L.dqo_table_D.argtypes = [C.c_void_p, C.c_int]
        L.dqo_levels.restype = C.c_int
        L.dqo_levels.argtypes = [C.c_int, C.c_double, C.c_void_p, C.c_void_p]
        L.dqo_philox4x32_10.argtypes = [C.c_void_p, C.c_void_p, C.c_void_p]
        L.dqo_perm_slot.restype = C.c_uint32
        L.dqo_perm_slot.argtypes = [C.c_void_p, C.c_uint32, C.c_uint32]
        L.dqo_perm_bits.restype = C.c_uint32
        L.dqo_perm_bits.argtypes = [C.c_uint32]
        L.dqo_draw_sg.argtypes = [C.c_void_p, C.c_uint64, C.c_uint32, C.c_void_p, C.c_void_p, C.c_void_p]
        L.dqo_entry_uniform.restype = C.c_float
        L.dqo_entry_uniform.argtypes = [C.c_void_p, C.c_uint32, C.c_uint8]
        L.dqo_sq_index.restype = C.c_int
        L.dqo_sq_index.argtypes = [C.c_void_p, C.c_void_p, C.c_int, C.c_float, C.c_float]
        L.dqo_bf16_ceil.restype = C.c_uint16
        L.dqo_bf16_ceil.argtypes = [C.c_float]
        L.dqo_encode_sg_core.argtypes = [C.c_void_p, C.c_int, C.c_void_p, C.c_void_p, C.c_void_p, C.c_uint32,
                                         C.c_void_p, C.c_void_p, C.c_void_p]
        L.dqo_decode_sg_core.argtypes = [C.c_void_p, C.c_int, C.c_void_p, C.c_void_p, C.c_uint16, C.c_void_p,
                                         C.c_void_p]
        L.dqo_packed_bytes.restype = C.c_uint64
        L.dqo_packed_bytes.argtypes = [C.POINTER(Chunk)]
        L.dqo_compress.argtypes = [C.c_void_p, C.POINTER(Chunk), C.c_uint32, C.c_void_p, C.c_int, C.c_void_p,
                                   C.c_void_p]
        L.dqo_dar_hop.argtypes = [C.c_void_p, C.POINTER(Chunk), C.c_uint32, C.c_void_p, C.c_void_p, C.c_int,
                                  C.c_void_p, C.c_void_p]
        L.dqo_decompress.argtypes = [C.c_void_p, C.POINTER(Chunk), C.c_void_p, C.c_void_p, C.c_int, C.c_void_p,
                                     C.c_void_p]
        if hasattr(L, "mxo_packed_bytes"):
            L.mxo_packed_bytes.restype = C.c_uint64
            L.mxo_packed_bytes.argtypes = [C.c_int, C.c_uint64]
            L.mxo_compress.argtypes = [C.c_int, C.c_uint64, C.c_void_p, C.c_int, C.c_void_p]
            L.mxo_dar_hop.argtypes = [C.c_int, C.c_uint64, C.c_void_p, C.c_void_p, C.c_int, C.c_void_p]
            L.mxo_decompress.argtypes = [C.c_int, C.c_uint64, C.c_void_p, C.c_void_p, C.c_int, C.c_void_p]
            L.mxo_encode_elem.restype = C.c_uint32
            L.mxo_encode_elem.argtypes = [C.c_int, C.c_float, C.c_int]
            L.mxo_decode_elem.restype = C.c_float
            L.mxo_decode_elem.argtypes = [C.c_int, C.c_uint32, C.c_int]
            L.mxo_block_scale.restype = C.c_int
            L.mxo_block_scale.argtypes = [C.c_int, C.c_float]
        _lib = L
    return _lib


BITS = (2, 4, 8)
RMAX = (1, 7, 127)
F32, BF16 = 0, 1


def _p(a):
    return a.ctypes.data_as(C.c_void_p)


def _dtype_code(a):
    if a.dtype == np.float32:
        return F32
    if a.dtype == np.uint16:
        return BF16  # bf16 bit patterns
    raise TypeError("local must be float32 or uint16 (bf16 bit patterns)")


def _mu_arg(mu, chunk):
    """Per-super-group means of a chunk as a float32 array (kept alive by the caller), or None."""
    if mu is None:
        return None
    mu = np.ascontiguousarray(mu, np.float32)
    assert mu.size == sum(chunk.n_sg), "one mean per super-group of the chunk"
    return mu


def make_chunk(first_sg, n_sg):
    ch = Chunk()
    ch.first_sg = int(first_sg)
    for i in range(len(n_sg)):      # 2, 4, 8 bits and optionally 16
        ch.n_sg[i] = int(n_sg[i])
    return ch


class Oracle:
    """One codec context: level tables + PRNG key (seed, round) + worker count."""

    def __init__(self, n_workers, seed=0, round=0, g4=1.3, g8=1.02, independent=False):
        self.cfg = Config(g4, g8, seed, round, n_workers, 1 if independent else 0, 0)
        self.n_workers = n_workers
        self.h = lib().dqo_create(C.byref(self.cfg))
        if not self.h:
            raise ValueError("oracle: invalid configuration")

    def __del__(self):
        if getattr(self, "h", None):
            lib().dqo_destroy(self.h)
            self.h = None

    # -- tables and pieces ---------------------------------------------------
    def T(self, wi):
        return np.ctypeslib.as_array(lib().dqo_table_T(self.h, wi), shape=(RMAX[wi] + 1,)).copy()

    def D(self, wi):
        return np.ctypeslib.as_array(lib().dqo_table_D(self.h, wi), shape=(RMAX[wi],)).copy()

    def draw_sg(self, sg, rank):
        gamma = np.empty(256, np.uint8)
        sb = np.empty(16, np.uint8)
        slot = C.c_uint32()
        lib().dqo_draw_sg(self.h, sg, rank, _p(gamma), _p(sb), C.byref(slot))
        return gamma, sb, slot.value

    def entry_uniform(self, slot, byte):
        return lib().dqo_entry_uniform(self.h, slot, byte)

    def encode_sg_core(self, wi, v, gamma, scale_byte, slot):
        v = np.ascontiguousarray(v, np.float32)
        gamma = np.ascontiguousarray(gamma, np.uint8)
        scale_byte = np.ascontiguousarray(scale_byte, np.uint8)
        assert v.size == 256 and gamma.size == 256 and scale_byte.size == 16
        code = np.empty(256, np.uint8)
        rG = np.empty(16, np.uint8)
        sf = C.c_uint16()
        lib().dqo_encode_sg_core(self.h, wi, _p(v), _p(gamma), _p(scale_byte), slot, _p(code), _p(rG), C.byref(sf))
        return code, rG, sf.value

    def decode_sg_core(self, wi, code, rG, sf_bits, local=None):
        code = np.ascontiguousarray(code, np.uint8)
        rG = np.ascontiguousarray(rG, np.uint8)
        out = np.empty(256, np.float32)
        loc = None if local is None else np.ascontiguousarray(local, np.float32)
        lib().dqo_decode_sg_core(self.h, wi, _p(code), _p(rG), sf_bits, None if loc is None else _p(loc), _p(out))
        return out

    # -- chunk-level calls (wire format) ---------------------------------------
    @staticmethod
    def packed_bytes(chunk):
        return lib().dqo_packed_bytes(C.byref(chunk))

    def compress(self, chunk, rank, local, mu=None):
        """mu: one mean per super-group of the chunk, subtracted from the local entries in fp32
        (Section 3.1), or None."""
        out = np.zeros(self.packed_bytes(chunk), np.uint8)
        mu = _mu_arg(mu, chunk)
        lib().dqo_compress(self.h, C.byref(chunk), rank, _p(local), _dtype_code(local),
                           None if mu is None else _p(mu), _p(out))
        return out

    def dar_hop(self, chunk, rank, packed_in, local, mu=None):
        out = np.zeros(self.packed_bytes(chunk), np.uint8)
        mu = _mu_arg(mu, chunk)
        lib().dqo_dar_hop(self.h, C.byref(chunk), rank, _p(packed_in), _p(local), _dtype_code(local),
                          None if mu is None else _p(mu), _p(out))
        return out

    def decompress(self, chunk, packed_in, local=None, mu=None):
        n = sum(chunk.n_sg) * 256
        out = np.empty(n, np.float32)
        mu = None if local is None else _mu_arg(mu, chunk)
        lib().dqo_decompress(self.h, C.byref(chunk), _p(packed_in), None if local is None else _p(local),
                             0 if local is None else _dtype_code(local), None if mu is None else _p(mu), _p(out))
        return out


def perm_slot(words, n, rank):
    """pi_rank of the shared permutation of 0..n-1 that the four PERM words define."""
    w = np.asarray(words, np.uint32)
    return int(lib().dqo_perm_slot(_p(w), int(n), int(rank)))


def perm_bits(n):
    return int(lib().dqo_perm_bits(int(n)))


def sq_index(T, D, x, u):
    T = np.ascontiguousarray(T, np.float32)
    D = np.ascontiguousarray(D, np.float32)
    return lib().dqo_sq_index(_p(T), _p(D), len(T) - 1, float(x), float(u))


def levels(wi, g):
    T = np.zeros(128, np.float32)
    D = np.zeros(128, np.float32)
    rc = lib().dqo_levels(wi, g, _p(T), _p(D))
    return rc, T[:RMAX[wi] + 1].copy(), D[:RMAX[wi]].copy()


def philox4x32_10(ctr, key):
    c = np.asarray(ctr, np.uint32)
    k = np.asarray(key, np.uint32)
    o = np.zeros(4, np.uint32)
    lib().dqo_philox4x32_10(_p(c), _p(k), _p(o))
    return o


def bf16_ceil(x):
    return lib().dqo_bf16_ceil(float(x))


# ------------------------------------------------------------------ chunking

def split_bucket(n_sg_by_width, n_chunks, first_sg=0):
    """Cut a reordered bucket (all 2-bit super-groups, then 4-bit, 8-bit and, if a fourth
    count is given, 16-bit; Section 3.5) into n_chunks chunks of equal super-group count."""
    counts = list(n_sg_by_width) + [0] * (4 - len(n_sg_by_width))
    total = sum(counts)
    assert total % n_chunks == 0, "bucket must be padded to a multiple of the worker count"
    m = total // n_chunks
    edges = [0]
    for c in counts:
        edges.append(edges[-1] + c)
    out = []
    for i in range(n_chunks):
        lo, hi = i * m, (i + 1) * m
        n_sg = [max(0, min(hi, edges[w + 1]) - max(lo, edges[w])) for w in range(4)]
        out.append(make_chunk(first_sg + lo, n_sg))
    return out


# ------------------------------------------------------------------ hop schedules

def ring_reduce_scatter(orc, grads, n_sg_by_width, first_sg=0, trace=None, mu=None):
    """Ring reduce-scatter (Section 3.4): chunk c starts at worker c (leaf,
    compress), visits workers c+1 .. c+n-2 (decompress-accumulate-recompress)
    and ends at worker c+n-1 (sink: decompress + add local).  grads[w] is worker
    w's reordered bucket (float32 or bf16 bit patterns).  Returns the list of
    fp32 sums per chunk; trace (a dict) receives every packed message as
    trace[(step, chunk)].  mu: the bucket's per-super-group means in reordered order,
    subtracted from every worker's entries where they enter (Section 3.1), or None."""
    n = orc.n_workers
    chunks = split_bucket(n_sg_by_width, n, first_sg)
    m = sum(n_sg_by_width) // n * 256
    out = []
    for c in range(n):
        ch = chunks[c]
        sl = slice(c * m, (c + 1) * m)
        mc = None if mu is None else mu[c * m // 256:(c + 1) * m // 256]
        if n == 1:
            g = grads[0][sl]
            g = g.astype(np.float32) if g.dtype == np.float32 else (g.astype(np.uint32) << 16).view(np.float32)
            out.append(g if mc is None else g - np.repeat(np.asarray(mc, np.float32), 256))
            continue
        w = c
        msg = orc.compress(ch, w, np.ascontiguousarray(grads[w][sl]), mc)
        if trace is not None:
            trace[(0, c)] = msg
        for t in range(1, n - 1):
            w = (c + t) % n
            msg = orc.dar_hop(ch, w, msg, np.ascontiguousarray(grads[w][sl]), mc)
            if trace is not None:
                trace[(t, c)] = msg
        w = (c + n - 1) % n
        out.append(orc.decompress(ch, msg, np.ascontiguousarray(grads[w][sl]), mc))
    return out


def butterfly_reduce_scatter(orc, grads, n_sg_by_width, first_sg=0, trace=None, mu=None):
    """Recursive-halving reduce-scatter (Appendix B): at step k = 1..log2 n worker
    w exchanges with w XOR (n >> k); it keeps the half of its current range whose
    index bit matches its own and sends the other half.  What it sends at step 1
    is compress(local half); a message received at step k covers the range kept at
    step k: the part sent at step k+1 goes through decompress-accumulate-recompress,
    the part kept through decompress-accumulate into an fp32 buffer that is the
    `local` of later steps.  Worker w ends with the sum of chunk w.  mu (the bucket's means
    in reordered order, or None) is subtracted where a worker's raw gradient enters a kernel,
    never from an fp32 buffer that already holds mean-subtracted sums."""
    n = orc.n_workers
    L = n.bit_length() - 1
    assert n == 1 << L and n >= 2
    chunks = split_bucket(n_sg_by_width, n, first_sg)
    m = sum(n_sg_by_width) // n * 256

    def sl(c):
        return slice(c * m, (c + 1) * m)

    # acc[w][c]: worker w's current accumulation of chunk c (raw gradient slice at the start)
    acc = [{c: np.ascontiguousarray(grads[w][sl(c)]) for c in range(n)} for w in range(n)]
    raw = [{c: True for c in range(n)} for w in range(n)]  # acc[w][c] is still the raw gradient slice

    def mean_of(w, c):
        return mu[c * m // 256:(c + 1) * m // 256] if (mu is not None and raw[w][c]) else None

    lo = [0] * n
    ln = [n] * n
    inbox = [dict() for _ in range(n)]  # chunk -> packed message waiting at the worker
    for k in range(1, L + 1):
        half = n >> k
        sends = []
        for w in range(n):
            keep_lo = lo[w] + half if (w & half) else lo[w]
            send_lo = lo[w] if (w & half) else lo[w] + half
            partner = w ^ half
            for c in range(send_lo, send_lo + half):
                if k == 1:
                    msg = orc.compress(chunks[c], w, acc[w][c], mean_of(w, c))
                else:
                    msg = orc.dar_hop(chunks[c], w, inbox[w].pop(c), acc[w][c], mean_of(w, c))
                sends.append((partner, c, msg))
                if trace is not None:
                    trace[(k, w, c)] = msg
                del acc[w][c]
            if k > 1:
                for c in range(keep_lo, keep_lo + half):
                    acc[w][c] = orc.decompress(chunks[c], inbox[w].pop(c), acc[w][c], mean_of(w, c))
                    raw[w][c] = False
            lo[w], ln[w] = keep_lo, half
        for partner, c, msg in sends:
            inbox[partner][c] = msg
    out = []
    for w in range(n):
        assert lo[w] == w and ln[w] == 1
        out.append(orc.decompress(chunks[w], inbox[w].pop(w), acc[w][w], mean_of(w, w)))
    return out



def all_gather(orc, sums, n_sg_by_width, topology, first_sg=0):
    """All-gather phase (Section 3.4): the sink of chunk c compresses its fp32 sum and
    broadcasts it; whoever receives it decompresses it.  Every worker, the sink included,
    keeps the decompressed message, so all workers end with the same bytes.  The sink is
    worker c-1 mod n on a ring (where the reduce-scatter of chunk c ended) and worker c after
    recursive halving; it compresses with its own rank, for super-groups it has compressed
    nothing of before.  sums: the reduce-scatter's result per chunk."""
    n = orc.n_workers
    chunks = split_bucket(n_sg_by_width, n, first_sg)
    out = []
    for c in range(n):
        sink = (c + n - 1) % n if topology == "ring" else c
        msg = orc.compress(chunks[c], sink, np.ascontiguousarray(sums[c], dtype=np.float32))
        out.append(orc.decompress(chunks[c], msg))
    return out


# ------------------------------------------------------------------ MX comparison codec

MXFP8, MXFP6, MXFP4 = 1, 2, 3
MX_CODE_BITS = {1: 8, 2: 6, 3: 4}


def mx_packed_bytes(fmt, n):
    return lib().mxo_packed_bytes(fmt, n)


def mx_compress(fmt, local):
    n = local.size
    out = np.zeros(mx_packed_bytes(fmt, n), np.uint8)
    lib().mxo_compress(fmt, n, _p(local), _dtype_code(local), _p(out))
    return out


def mx_dar_hop(fmt, packed_in, local):
    n = local.size
    out = np.zeros(mx_packed_bytes(fmt, n), np.uint8)
    lib().mxo_dar_hop(fmt, n, _p(packed_in), _p(local), _dtype_code(local), _p(out))
    return out


def mx_decompress(fmt, packed_in, n, local=None):
    out = np.empty(n, np.float32)
    lib().mxo_decompress(fmt, n, _p(packed_in), None if local is None else _p(local),
                         0 if local is None else _dtype_code(local), _p(out))
    return out


def mx_encode_elem(fmt, v, e):
    return lib().mxo_encode_elem(fmt, float(v), int(e))


def mx_decode_elem(fmt, code, e):
    return lib().mxo_decode_elem(fmt, int(code), int(e))


def mx_block_scale(fmt, m):
    return lib().mxo_block_scale(fmt, float(m))


def mx_ring_reduce_scatter(fmt, grads, trace=None):
    """The ring path of ring_reduce_scatter with the MX codec: n equal chunks."""
    n = len(grads)
    m = grads[0].size // n
    out = []
    for c in range(n):
        sl = slice(c * m, (c + 1) * m)
        msg = mx_compress(fmt, np.ascontiguousarray(grads[c][sl]))
        if trace is not None:
            trace[(0, c)] = msg
        for t in range(1, n - 1):
            msg = mx_dar_hop(fmt, msg, np.ascontiguousarray(grads[(c + t) % n][sl]))
            if trace is not None:
                trace[(t, c)] = msg
        out.append(mx_decompress(fmt, msg, m, np.ascontiguousarray(grads[(c + n - 1) % n][sl])))
    return out


def mx_all_gather(fmt, sums):
    """All-gather phase with the MX codec: compress each chunk's fp32 sum, decompress it."""
    return [mx_decompress(fmt, mx_compress(fmt, np.ascontiguousarray(x, dtype=np.float32)), len(x)) for x in sums]
