"""Thin ctypes binding of libdq.so: same names as include/dq.h, argument marshalling only.

PyTorch is used for device memory and streams; every step of the path runs in the HIP
kernels.  There is no fallback: if the library is not built, or no GPU is present when a
compute call is made, the call raises.
"""
import ctypes as C
import os

import torch

HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(HERE, "libdq.so")

DQ_OK, DQ_EINVAL, DQ_EALIGN, DQ_EUNSUPPORTED, DQ_EHIP = range(5)
DQ_F32, DQ_BF16 = 0, 1
DQ_DYNAMIQ, DQ_MXFP8_E4M3, DQ_MXFP6_E3M2, DQ_MXFP4_E2M1 = 0, 1, 2, 3
DQ_RING, DQ_BUTTERFLY, DQ_CHAIN = 0, 1, 2

EXPORTS = [
    "dq_create", "dq_destroy", "dq_set_round", "dq_packed_bytes", "dq_compress", "dq_dar_hop", "dq_decompress",
    "dq_decompress_restore",
    "dq_mx_packed_bytes", "dq_mx_compress", "dq_mx_dar_hop", "dq_mx_decompress",
    "dq_replay_scratch_bytes", "dq_replay_create", "dq_replay_n_steps", "dq_replay_run", "dq_replay_run_steps",
    "dq_replay_step_info", "dq_replay_message", "dq_replay_run_launch", "dq_stream_probe",
    "dq_replay_destroy", "dq_status_str", "dq_last_hip_error",
    "dq_sg_stats", "dq_stats_combine", "dq_allocate", "dq_reorder", "dq_reorder_mean", "dq_restore",
    "dq_pipelined_wire_bytes", "dq_pipelined_stage_bytes", "dq_dar_hop_pipelined", "dq_dar_hop_pipelined_static",
]
DQ_STATIC_STAGE_BYTES = 8 << 20


class DqError(RuntimeError):
    pass


class Config(C.Structure):
    _fields_ = [("g4", C.c_double), ("g8", C.c_double), ("seed", C.c_uint64), ("round", C.c_uint32),
                ("n_workers", C.c_uint32), ("independent_rounding", C.c_uint32), ("reserved", C.c_uint32)]


class Chunk(C.Structure):
    _fields_ = [("first_sg", C.c_uint64), ("n_sg", C.c_uint32 * 4)]


class ReplayDesc(C.Structure):
    _fields_ = [("topology", C.c_int), ("codec", C.c_int), ("dtype", C.c_int), ("n_buckets", C.c_uint32),
                ("n_sg_bucket", C.c_uint64), ("n_sg_by_width", C.POINTER(C.c_uint32)), ("first_sg", C.c_uint64),
                ("all_gather", C.c_uint32), ("mu", C.c_void_p), ("origin", C.c_void_p),
                ("inputs_in_original_order", C.c_uint32), ("n_grads", C.c_uint32)]


class Local(C.Structure):
    """dq_local: a worker's own entries, their means, and where each super-group of the chunk lives."""
    _fields_ = [("data", C.c_void_p), ("dtype", C.c_int), ("mu", C.c_void_p), ("sg_index", C.c_void_p)]


_lib = None


def lib():
    """Load libdq.so (built in-tree by build.py).  Raises if it is missing."""
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise DqError(f"{LIB_PATH} is not built: run `python -m paper_2602_08923_amd.build` "
                          "(there is no CPU fallback)")
        L = C.CDLL(LIB_PATH)
        vp, u32, u64, i = C.c_void_p, C.c_uint32, C.c_uint64, C.c_int
        L.dq_create.argtypes = [C.POINTER(Config), C.POINTER(vp)]
        L.dq_destroy.argtypes = [vp]
        L.dq_destroy.restype = None
        L.dq_set_round.argtypes = [vp, u32]
        L.dq_packed_bytes.argtypes = [C.POINTER(Chunk)]
        L.dq_packed_bytes.restype = C.c_size_t
        L.dq_compress.argtypes = [vp, C.POINTER(Local), C.POINTER(Chunk), u32, vp, vp]
        L.dq_dar_hop.argtypes = [vp, vp, C.POINTER(Local), C.POINTER(Chunk), u32, vp, vp]
        L.dq_decompress.argtypes = [vp, vp, C.POINTER(Local), C.POINTER(Chunk), vp, vp]
        L.dq_decompress_restore.argtypes = [vp, vp, C.POINTER(Local), C.POINTER(Chunk), vp, vp, vp, vp]
        L.dq_status_str.argtypes = [i]
        L.dq_status_str.restype = C.c_char_p
        L.dq_last_hip_error.restype = C.c_char_p
        L.dq_mx_packed_bytes.argtypes = [i, u64]
        L.dq_mx_packed_bytes.restype = C.c_size_t
        L.dq_mx_compress.argtypes = [i, vp, i, u64, vp, vp]
        L.dq_mx_dar_hop.argtypes = [i, vp, vp, i, u64, vp, vp]
        L.dq_mx_decompress.argtypes = [i, vp, vp, i, u64, vp, vp]
        L.dq_replay_scratch_bytes.argtypes = [vp, C.POINTER(ReplayDesc)]
        L.dq_replay_scratch_bytes.restype = C.c_size_t
        L.dq_replay_create.argtypes = [vp, C.POINTER(ReplayDesc), C.POINTER(vp), vp, C.c_size_t, vp, C.POINTER(vp)]
        L.dq_replay_n_steps.argtypes = [vp]
        L.dq_replay_n_steps.restype = u32
        L.dq_replay_run.argtypes = [vp, C.POINTER(C.c_float), vp]
        L.dq_replay_run_steps.argtypes = [vp, u32, u32, vp]
        L.dq_replay_step_info.argtypes = [vp, u32, C.POINTER(u32), C.POINTER(u64), C.POINTER(u64)]
        L.dq_replay_message.argtypes = [vp, u32, u32, u32, C.POINTER(vp), C.POINTER(C.c_size_t)]
        L.dq_replay_run_launch.argtypes = [vp, u32, u32, vp]
        L.dq_stream_probe.argtypes = [vp, vp, C.c_size_t, vp, C.c_size_t, vp]
        L.dq_replay_destroy.argtypes = [vp]
        L.dq_replay_destroy.restype = None
        L.dq_sg_stats.argtypes = [vp, i, u64, vp, vp, vp]
        L.dq_stats_combine.argtypes = [vp, vp, u32, u64, vp, vp, vp]
        L.dq_allocate.argtypes = [vp, u32, u32, u64, u32, vp, vp, vp, vp]
        L.dq_reorder.argtypes = [vp, i, vp, u32, u32, vp, vp]
        L.dq_reorder_mean.argtypes = [vp, vp, vp, u32, u32, vp, vp, vp]
        L.dq_restore.argtypes = [vp, vp, vp, u32, u32, u32, vp, vp]
        L.dq_pipelined_wire_bytes.argtypes = [C.POINTER(Chunk), u32]
        L.dq_pipelined_wire_bytes.restype = C.c_size_t
        L.dq_pipelined_stage_bytes.argtypes = [C.POINTER(Chunk), u32]
        L.dq_pipelined_stage_bytes.restype = C.c_size_t
        L.dq_dar_hop_pipelined.argtypes = [vp, vp, C.POINTER(Local), C.POINTER(Chunk), u32, u32, vp, vp, vp, vp]
        L.dq_dar_hop_pipelined_static.argtypes = [vp, vp, C.POINTER(Local), C.POINTER(Chunk), u32, u32, vp, vp, vp]
        _lib = L
    return _lib


def _check(st, detail=False):
    if st != DQ_OK:
        L = lib()
        msg = L.dq_status_str(st).decode()
        if st == DQ_EHIP or detail:
            msg += ": " + L.dq_last_hip_error().decode()
        raise DqError(msg)


def _stream():
    return C.c_void_p(torch.cuda.current_stream().cuda_stream)


def _ptr(t):
    if t is None:
        return None
    if not t.is_cuda or not t.is_contiguous():
        raise DqError("tensors must be contiguous CUDA tensors")
    return C.c_void_p(t.data_ptr())


def _dtype(t):
    if t.dtype == torch.float32:
        return DQ_F32
    if t.dtype == torch.bfloat16:
        return DQ_BF16
    raise DqError("local slices must be float32 or bfloat16")


def make_chunk(first_sg, n_sg):
    ch = Chunk()
    ch.first_sg = int(first_sg)
    for k in range(len(n_sg)):      # 2, 4, 8 bits and optionally 16
        ch.n_sg[k] = int(n_sg[k])
    return ch


def dq_packed_bytes(chunk):
    return lib().dq_packed_bytes(C.byref(chunk))


def _entries(chunk):
    return sum(chunk.n_sg) * 256


def _mean(mu, chunk):
    """The chunk's per-super-group means (float32, one each) or None."""
    if mu is not None and (mu.dtype != torch.float32 or mu.numel() != sum(chunk.n_sg)):
        raise DqError("mu is float32, one per super-group of the chunk")
    return mu


def _local(local, chunk, mu=None, sg_index=None):
    """dq_local for a tensor of the chunk's entries (sg_index None) or for the original tensor whose
    super-groups sg_index (int32, one per super-group of the chunk) picks; None stays None."""
    if local is None:
        return None
    if sg_index is None:
        if local.numel() != _entries(chunk):
            raise DqError("local slice does not match the chunk")
    else:
        if sg_index.dtype != torch.int32 or sg_index.numel() != sum(chunk.n_sg) or local.numel() % 256:
            raise DqError("sg_index is int32, one per super-group of the chunk")
        if sg_index.numel() and not 0 <= int(sg_index.min()) <= int(sg_index.max()) < local.numel() // 256:
            raise DqError("sg_index points outside the tensor")
    d, m, x = _ptr(local), _ptr(_mean(mu, chunk)), _ptr(sg_index)
    return C.byref(Local(d, _dtype(local), m, x))


class Context:
    """dq_ctx: level tables on the device + PRNG key (seed, round) + worker count."""

    def __init__(self, n_workers, seed=0, round=0, g4=1.3, g8=1.02, independent_rounding=False):
        self.h = C.c_void_p()
        self.n_workers = n_workers
        cfg = Config(g4, g8, seed, round, n_workers, 1 if independent_rounding else 0, 0)
        _check(lib().dq_create(C.byref(cfg), C.byref(self.h)))

    def close(self):
        # _lib is read directly: at interpreter exit module functions may already be gone
        if getattr(self, "h", None) and _lib is not None:
            _lib.dq_destroy(self.h)
            self.h = None

    __del__ = close

    def set_round(self, r):
        _check(lib().dq_set_round(self.h, r))

    def dq_compress(self, local, chunk, rank, packed_out=None, mu=None, sg_index=None):
        loc = _local(local, chunk, mu, sg_index)
        if packed_out is None:
            packed_out = torch.zeros(dq_packed_bytes(chunk), dtype=torch.uint8, device=local.device)
        if packed_out.numel() < dq_packed_bytes(chunk):
            raise DqError("packed_out too small")
        _check(lib().dq_compress(self.h, loc, C.byref(chunk), rank, _ptr(packed_out), _stream()))
        return packed_out

    def dq_dar_hop(self, packed_in, local, chunk, rank, packed_out=None, mu=None, sg_index=None):
        loc = _local(local, chunk, mu, sg_index)
        if packed_in.numel() < dq_packed_bytes(chunk):
            raise DqError("buffers do not match the chunk")
        if packed_out is None:
            packed_out = torch.zeros(dq_packed_bytes(chunk), dtype=torch.uint8, device=local.device)
        if packed_out.numel() < dq_packed_bytes(chunk):
            raise DqError("packed_out too small")
        _check(lib().dq_dar_hop(self.h, _ptr(packed_in), loc, C.byref(chunk), rank, _ptr(packed_out), _stream()))
        return packed_out

    def dq_decompress(self, packed_in, chunk, local=None, out=None, mu=None, sg_index=None):
        loc = _local(local, chunk, mu, sg_index)
        if packed_in.numel() < dq_packed_bytes(chunk):
            raise DqError("buffers do not match the chunk")
        if out is None:
            out = torch.empty(_entries(chunk), dtype=torch.float32, device=packed_in.device)
        if out.numel() != _entries(chunk) or out.dtype != torch.float32:
            raise DqError("out must be float32 with one element per entry")
        _check(lib().dq_decompress(self.h, _ptr(packed_in), loc, C.byref(chunk), _ptr(out), _stream()))
        return out

    def dq_decompress_restore(self, packed_in, chunk, origin, out_base, local=None, mu=None, mu_back=None, sg_index=None):
        """Decompress (+ local - mu) with every super-group written to out_base[origin[j]] and
        n_workers * mu_back[j] added: the restore fused into the sink's kernel."""
        loc = _local(local, chunk, mu, sg_index)
        if packed_in.numel() < dq_packed_bytes(chunk):
            raise DqError("buffers do not match the chunk")
        if origin.dtype != torch.int32 or origin.numel() != sum(chunk.n_sg):
            raise DqError("origin is int32, one per super-group of the chunk")
        if out_base.dtype != torch.float32 or (origin.numel() and out_base.numel() < (int(origin.max()) + 1) * 256):
            raise DqError("out_base is float32 and holds every destination super-group")
        _check(lib().dq_decompress_restore(self.h, _ptr(packed_in), loc, C.byref(chunk), _ptr(origin),
                                           _ptr(_mean(mu_back, chunk)), _ptr(out_base), _stream()))
        return out_base


# ---- MX comparison codec -------------------------------------------------------------

def dq_mx_packed_bytes(fmt, n_entries):
    return lib().dq_mx_packed_bytes(fmt, n_entries)


def dq_mx_compress(fmt, local, packed_out=None):
    n = local.numel()
    if packed_out is None:
        packed_out = torch.zeros(dq_mx_packed_bytes(fmt, n), dtype=torch.uint8, device=local.device)
    _check(lib().dq_mx_compress(fmt, _ptr(local), _dtype(local), n, _ptr(packed_out), _stream()))
    return packed_out


def dq_mx_dar_hop(fmt, packed_in, local, packed_out=None):
    n = local.numel()
    if packed_in.numel() < dq_mx_packed_bytes(fmt, n):
        raise DqError("packed_in too small")
    if packed_out is None:
        packed_out = torch.zeros(dq_mx_packed_bytes(fmt, n), dtype=torch.uint8, device=local.device)
    _check(lib().dq_mx_dar_hop(fmt, _ptr(packed_in), _ptr(local), _dtype(local), n, _ptr(packed_out), _stream()))
    return packed_out


def dq_mx_decompress(fmt, packed_in, n_entries, local=None, out=None):
    if packed_in.numel() < dq_mx_packed_bytes(fmt, n_entries):
        raise DqError("packed_in too small")
    if out is None:
        out = torch.empty(n_entries, dtype=torch.float32, device=packed_in.device)
    _check(lib().dq_mx_decompress(fmt, _ptr(packed_in), _ptr(local), 0 if local is None else _dtype(local), n_entries,
                                  _ptr(out), _stream()))
    return out


# ---- hop replay ------------------------------------------------------------------------

class Replay:
    """dq_replay: a prepared ring / butterfly / chain schedule over N simulated workers."""

    def __init__(self, ctx, topology, codec, worker_grads, n_sg_bucket, n_sg_by_width=None, n_buckets=1, first_sg=0,
                 all_gather=False, mu=None, origin=None, inputs_in_original_order=False):
        """mu: None, or the float32 means of all n_buckets * n_sg_bucket super-groups in reordered order.
        origin: None, or int32 [n_buckets * n_sg_bucket] (from dq_reorder_mean): the result is then written
        in the original order with the means added back.  inputs_in_original_order (needs origin): the
        worker gradients are the original tensors; the kernels gather their super-groups through origin."""
        self.ctx = ctx
        self.mu = mu
        self.origin = origin
        if origin is not None and (origin.dtype != torch.int32 or origin.numel() != n_buckets * n_sg_bucket):
            raise DqError("origin is int32, one per super-group")
        if mu is not None and (mu.dtype != torch.float32 or mu.numel() != n_buckets * n_sg_bucket):
            raise DqError("mu is float32, one per super-group")
        self.grads = list(worker_grads)
        if len(self.grads) != ctx.n_workers:
            raise DqError(f"{len(self.grads)} worker gradients for a context of {ctx.n_workers} workers")
        dev = self.grads[0].device
        n = len(self.grads)
        flat = (C.c_uint32 * (4 * n_buckets))()
        if n_sg_by_width is not None:
            for b in range(n_buckets):
                for k in range(len(n_sg_by_width[b])):      # 2, 4, 8 bits and optionally 16
                    flat[4 * b + k] = int(n_sg_by_width[b][k])
        self._widths = flat
        desc = ReplayDesc(topology, codec, _dtype(self.grads[0]), n_buckets, n_sg_bucket, flat, first_sg,
                          1 if all_gather else 0, _ptr(mu), _ptr(origin), 1 if inputs_in_original_order else 0, n)
        self.desc = desc
        entries = n_sg_bucket * 256 * n_buckets
        for g in self.grads:
            if g.numel() != entries or _dtype(g) != desc.dtype:
                raise DqError("every worker gradient must hold n_buckets * n_sg_bucket * 256 entries of one dtype")
        nbytes = lib().dq_replay_scratch_bytes(ctx.h, C.byref(desc))
        if nbytes == 0:
            raise DqError("invalid replay description")
        self.scratch = torch.empty(nbytes, dtype=torch.uint8, device=dev)
        self.out = torch.empty(entries, dtype=torch.float32, device=dev)
        ptrs = (C.c_void_p * n)(*[g.data_ptr() for g in self.grads])
        self.h = C.c_void_p()
        _check(lib().dq_replay_create(ctx.h, C.byref(desc), ptrs, _ptr(self.scratch), nbytes, _ptr(self.out),
                                      C.byref(self.h)))
        self.n_steps = lib().dq_replay_n_steps(self.h)

    def run(self, timed=False):
        if timed:
            ms = (C.c_float * self.n_steps)()
            _check(lib().dq_replay_run(self.h, ms, _stream()))
            return list(ms)
        _check(lib().dq_replay_run(self.h, None, _stream()))
        return None

    def run_steps(self, first, count):
        _check(lib().dq_replay_run_steps(self.h, first, count, _stream()))

    def run_launch(self, step, launch):
        _check(lib().dq_replay_run_launch(self.h, step, launch, _stream()))

    def step_info(self, step):
        kind, a, b = C.c_uint32(), C.c_uint64(), C.c_uint64()
        _check(lib().dq_replay_step_info(self.h, step, C.byref(kind), C.byref(a), C.byref(b)))
        return kind.value, a.value, b.value

    def message(self, step, bucket, chunk):
        """The packed message step `step` wrote for (bucket, chunk): a view into the scratch (ring, chain)."""
        ptr, nbytes = C.c_void_p(), C.c_size_t()
        _check(lib().dq_replay_message(self.h, step, bucket, chunk, C.byref(ptr), C.byref(nbytes)))
        off = ptr.value - self.scratch.data_ptr()
        return self.scratch[off:off + nbytes.value]

    def close(self):
        if getattr(self, "h", None) and _lib is not None:
            _lib.dq_replay_destroy(self.h)
            self.h = None

    __del__ = close


# ------------------------------------------------------------------ before and after the main stage
def dq_sg_stats(x, mu_out=None, F_out=None):
    """Per-super-group mean and sum of squares of one worker's tensor -> (mu, F) float32."""
    n_sg = x.numel() // 256
    if x.numel() % 256:
        raise DqError("tensor length must be a multiple of 256")
    if mu_out is None:
        mu_out = torch.empty(n_sg, dtype=torch.float32, device=x.device)
    if F_out is None:
        F_out = torch.empty(n_sg, dtype=torch.float32, device=x.device)
    _check(lib().dq_sg_stats(_ptr(x), _dtype(x), n_sg, _ptr(mu_out), _ptr(F_out), _stream()))
    return mu_out, F_out


def dq_stats_combine(mu_all, F_all):
    """mu_all, F_all: float32 [n_workers, n_sg] -> (mu, F) float32 [n_sg]."""
    n, J = mu_all.shape
    if F_all.shape != mu_all.shape or mu_all.dtype != torch.float32 or F_all.dtype != torch.float32:
        raise DqError("statistics are two float32 tensors of the same [n_workers, n_sg] shape")
    mu = torch.empty(J, dtype=torch.float32, device=mu_all.device)
    F = torch.empty(J, dtype=torch.float32, device=mu_all.device)
    _check(lib().dq_stats_combine(_ptr(mu_all), _ptr(F_all), n, J, _ptr(mu), _ptr(F), _stream()))
    return mu, F


def dq_allocate(F, n_sg_per_bucket, max_code_bits, max_width=8):
    """F: float32 [n_buckets * n_sg_per_bucket] -> (widths uint8, pos int32 (holds uint32),
    counts int32 [n_buckets, 5] = #2-bit, #4-bit, #8-bit, #16-bit, threshold pattern)."""
    if F.dtype != torch.float32 or F.numel() % n_sg_per_bucket:
        raise DqError("F is float32 with a whole number of buckets")
    nb = F.numel() // n_sg_per_bucket
    widths = torch.empty(F.numel(), dtype=torch.uint8, device=F.device)
    pos = torch.empty(F.numel(), dtype=torch.int32, device=F.device)
    counts = torch.empty((nb, 5), dtype=torch.int32, device=F.device)
    _check(lib().dq_allocate(_ptr(F), n_sg_per_bucket, nb, int(max_code_bits), int(max_width), _ptr(widths), _ptr(pos),
                             _ptr(counts), _stream()))
    return widths, pos, counts


def dq_reorder(x, pos, n_sg_per_bucket, out=None):
    nb = pos.numel() // n_sg_per_bucket
    if x.numel() != pos.numel() * 256 or pos.numel() % n_sg_per_bucket or pos.dtype != torch.int32:
        raise DqError("x holds 256 entries per position; positions are int32, a whole number of buckets")
    if out is None:
        out = torch.empty_like(x)
    _check(lib().dq_reorder(_ptr(x), _dtype(x), _ptr(pos), n_sg_per_bucket, nb, _ptr(out), _stream()))
    return out


def dq_reorder_mean(mu, pos, n_sg_per_bucket, counts=None, out=None, with_origin=False):
    """The means the main stage subtracts, in reordered order (zero for 16-bit super-groups).
    counts: what dq_allocate returned (int32 [n_buckets, 5]) or None (no 16-bit class).
    mu None: only the origins.  with_origin: also return origin (int32, origin[pos[j]] = j per bucket)."""
    nb = pos.numel() // n_sg_per_bucket
    if pos.numel() % n_sg_per_bucket or pos.dtype != torch.int32:
        raise DqError("positions are int32, a whole number of buckets")
    if mu is not None and (mu.dtype != torch.float32 or mu.numel() != pos.numel()):
        raise DqError("mu is float32, one per position")
    if counts is not None and (counts.dtype != torch.int32 or counts.numel() != 5 * nb):
        raise DqError("counts is int32 [n_buckets, 5]")
    if mu is None and not with_origin:
        raise DqError("nothing to compute")
    if out is None and mu is not None:
        out = torch.empty_like(mu)
    origin = torch.empty_like(pos) if with_origin else None
    _check(lib().dq_reorder_mean(_ptr(mu), _ptr(pos), _ptr(counts), n_sg_per_bucket, nb,
                                 _ptr(out) if mu is not None else None, _ptr(origin), _stream()))
    return (out, origin) if with_origin else out


def dq_restore(total, pos, n_sg_per_bucket, n_workers, mu_main=None, out=None):
    nb = pos.numel() // n_sg_per_bucket
    if total.dtype != torch.float32 or total.numel() != pos.numel() * 256 or pos.dtype != torch.int32:
        raise DqError("the main stage's result is float32, 256 entries per position")
    if mu_main is not None and (mu_main.dtype != torch.float32 or mu_main.numel() != pos.numel()):
        raise DqError("mu_main is float32, one per super-group")
    if out is None:
        out = torch.empty_like(total)
    _check(lib().dq_restore(_ptr(total), _ptr(pos), _ptr(mu_main), n_workers, n_sg_per_bucket, nb, _ptr(out), _stream()))
    return out


# ------------------------------------------------------------------ block-wise pipelining
def dq_pipelined_wire_bytes(chunk, block_sg):
    return lib().dq_pipelined_wire_bytes(C.byref(chunk), block_sg)


def dq_pipelined_stage_bytes(chunk, block_sg):
    return lib().dq_pipelined_stage_bytes(C.byref(chunk), block_sg)


def dq_dar_hop_pipelined(ctx, wire_in, local, chunk, rank, block_sg, compute_stream, copy_stream, stage=None,
                         wire_out=None, mu=None, sg_index=None):
    """One hop of a chunk in blocks of block_sg super-groups: block i is encoded on compute_stream
    while block i-1 travels (a device copy) on copy_stream.  wire_in None: the first hop."""
    dev = local.device
    if stage is None:
        # zeros: the kernels never write the padding at the end of a packed block
        stage = torch.zeros(dq_pipelined_stage_bytes(chunk, block_sg), dtype=torch.uint8, device=dev)
    if wire_out is None:
        wire_out = torch.zeros(dq_pipelined_wire_bytes(chunk, block_sg), dtype=torch.uint8, device=dev)
    _check(lib().dq_dar_hop_pipelined(ctx.h, _ptr(wire_in), _local(local, chunk, mu, sg_index),
                                      C.byref(chunk), rank, block_sg,
                                      _ptr(stage), _ptr(wire_out), C.c_void_p(compute_stream.cuda_stream),
                                      C.c_void_p(copy_stream.cuda_stream)))
    return wire_out


def dq_dar_hop_pipelined_static(ctx, wire_in, local, chunk, rank, block_sg, compute_stream, copy_stream, wire_out,
                                mu=None, sg_index=None):
    """dq_dar_hop_pipelined with the library's static staging array: allocates nothing, so the
    caller passes wire_out (dq_pipelined_wire_bytes bytes, zero-filled once: the kernels never write
    the padding between blocks)."""
    _check(lib().dq_dar_hop_pipelined_static(ctx.h, _ptr(wire_in), _local(local, chunk, mu, sg_index),
                                             C.byref(chunk), rank, block_sg, _ptr(wire_out),
                                             C.c_void_p(compute_stream.cuda_stream),
                                             C.c_void_p(copy_stream.cuda_stream)), detail=True)
    return wire_out


def dq_stream_probe(ctx, src, dst):
    """Streaming probe: reads all of src, writes all of dst (uint8 tensors, sizes multiples of 16, dst <= src)."""
    _check(lib().dq_stream_probe(ctx.h, _ptr(src), src.numel() * src.element_size(), _ptr(dst),
                                 dst.numel() * dst.element_size(), _stream()))
