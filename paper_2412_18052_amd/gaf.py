"""Thin ctypes binding of libgaf.so (the C ABI in include/gaf.h).

Argument marshalling only: torch tensors supply device pointers and the
current stream; every step of the computation runs inside the HIP library.
There is no CPU fallback: a missing library or a failing call raises.
"""
import ctypes
import os

import torch

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libgaf.so")

GAF_OK, GAF_EINVAL, GAF_EALIGN, GAF_ENOMEM, GAF_EHIP, GAF_EUNSUPPORTED, GAF_EDEVICE, GAF_ELIMIT = range(8)
GAF_STATIC_MAX_N, GAF_STATIC_MAX_P = 64, 1 << 36
GAF_F32, GAF_BF16 = 0, 1

SYMBOLS = ("gaf_create", "gaf_destroy", "gaf_strerror", "gaf_aggregate", "gaf_step", "gaf_pairwise",
           "gaf_profile_begin", "gaf_profile_end", "gaf_set_schedule", "gaf_aggregate_with_gram",
           "gaf_aggregate_best_seed", "gaf_aggregate_sgd", "gaf_aggregate_bucketed",
           "gaf_aggregate_with_matrix", "gaf_fused_mean_record", "gaf_static_init", "gaf_aggregate_static",
           "gaf_step_lookahead", "gaf_flush")
GAF_SCHEDULE_AUTO, GAF_SCHEDULE_SEQUENTIAL, GAF_SCHEDULE_GRAM = 0, 1, 2
SCHEDULES = {"auto": 0, "sequential": 1, "gram": 2}
KERNEL_NAMES = ("init", "seed_reduce", "reduce", "update", "gram", "gram_finalize", "distance", "decide",
                "filter", "mean", "gram_sample")


class LaunchTime(ctypes.Structure):
    _fields_ = [("kernel", ctypes.c_int32), ("ms", ctypes.c_float)]


class GafError(RuntimeError):
    def __init__(self, status, what):
        self.status = int(status)
        super().__init__("%s: %s (status %d)" % (what, strerror(status), status))


_lib = None


def load(path=None):
    """Load libgaf.so. The in-tree library is built first if it is missing or older than any of
    its sources (a stale binary would silently run yesterday's kernels); a failing build raises."""
    global _lib
    if _lib is not None and path is None:
        return _lib
    if path is None:
        from . import build as _build
        _build.build(force=False)
    path = path or LIB_PATH
    lib = ctypes.CDLL(path)
    c = ctypes
    lib.gaf_create.restype = c.c_int
    lib.gaf_create.argtypes = [c.POINTER(c.c_void_p), c.c_int, c.c_size_t, c.c_int]
    lib.gaf_destroy.restype = c.c_int
    lib.gaf_destroy.argtypes = [c.c_void_p]
    lib.gaf_strerror.restype = c.c_char_p
    lib.gaf_strerror.argtypes = [c.c_int]
    lib.gaf_aggregate.restype = c.c_int
    lib.gaf_aggregate.argtypes = [c.c_void_p, c.POINTER(c.c_void_p), c.c_int, c.c_size_t, c.c_int,
                                  c.c_float, c.c_void_p, c.c_void_p, c.c_void_p, c.c_void_p,
                                  c.c_void_p]
    lib.gaf_step.restype = c.c_int
    lib.gaf_step.argtypes = [c.c_void_p, c.c_void_p, c.c_void_p, c.c_void_p, c.c_size_t, c.c_int,
                             c.c_float, c.c_void_p, c.c_void_p, c.c_void_p]
    lib.gaf_step_lookahead.restype = c.c_int
    lib.gaf_step_lookahead.argtypes = lib.gaf_step.argtypes
    lib.gaf_flush.restype = c.c_int
    lib.gaf_flush.argtypes = [c.c_void_p, c.c_void_p]
    lib.gaf_pairwise.restype = c.c_int
    lib.gaf_pairwise.argtypes = [c.c_void_p, c.POINTER(c.c_void_p), c.c_int, c.c_size_t, c.c_int,
                                 c.c_void_p, c.c_void_p, c.c_void_p]
    lib.gaf_aggregate_with_gram.restype = c.c_int
    lib.gaf_aggregate_with_gram.argtypes = [c.c_void_p, c.POINTER(c.c_void_p), c.c_int, c.c_size_t,
                                            c.c_int, c.c_float, c.c_void_p, c.c_void_p, c.c_void_p,
                                            c.c_void_p, c.c_void_p, c.c_void_p]
    lib.gaf_aggregate_with_matrix.restype = c.c_int
    lib.gaf_aggregate_with_matrix.argtypes = [c.c_void_p, c.POINTER(c.c_void_p), c.c_int, c.c_size_t,
                                              c.c_int, c.c_float] + [c.c_void_p] * 7
    lib.gaf_aggregate_best_seed.restype = c.c_int
    lib.gaf_aggregate_best_seed.argtypes = [c.c_void_p, c.POINTER(c.c_void_p), c.c_int, c.c_size_t,
                                            c.c_int, c.c_float] + [c.c_void_p] * 6
    lib.gaf_aggregate_sgd.restype = c.c_int
    lib.gaf_aggregate_sgd.argtypes = [c.c_void_p, c.POINTER(c.c_void_p), c.c_int, c.c_size_t, c.c_int,
                                      c.c_float, c.c_void_p, c.c_void_p, c.c_float, c.c_float,
                                      c.c_float] + [c.c_void_p] * 5
    lib.gaf_aggregate_bucketed.restype = c.c_int
    lib.gaf_aggregate_bucketed.argtypes = [c.c_void_p, c.POINTER(c.c_void_p), c.c_int, c.c_size_t,
                                           c.c_int, c.c_float, c.c_int, c.POINTER(c.c_size_t)] + \
                                          [c.c_void_p] * 5
    lib.gaf_set_schedule.restype = c.c_int
    lib.gaf_set_schedule.argtypes = [c.c_void_p, c.c_int]
    lib.gaf_fused_mean_record.restype = c.c_int
    lib.gaf_fused_mean_record.argtypes = [c.c_void_p, c.POINTER(c.c_int32)]
    lib.gaf_static_init.restype = c.c_int
    lib.gaf_static_init.argtypes = []
    lib.gaf_aggregate_static.restype = c.c_int
    lib.gaf_aggregate_static.argtypes = [c.POINTER(c.c_void_p), c.c_int, c.c_size_t, c.c_int, c.c_float,
                                         c.c_void_p, c.c_void_p, c.c_void_p, c.c_void_p, c.c_void_p]
    lib.gaf_profile_begin.restype = c.c_int
    lib.gaf_profile_begin.argtypes = [c.c_void_p, c.c_int]
    lib.gaf_profile_end.restype = c.c_int
    lib.gaf_profile_end.argtypes = [c.c_void_p, c.POINTER(LaunchTime), c.c_int, c.POINTER(c.c_int)]
    _lib = lib
    return lib


def strerror(status):
    return load().gaf_strerror(int(status)).decode()


def _check(status, what):
    if status != GAF_OK:
        raise GafError(status, what)


def _dtype_code(t):
    if t.dtype == torch.float32:
        return GAF_F32
    if t.dtype == torch.bfloat16:
        return GAF_BF16
    raise TypeError("gradients must be float32 or bfloat16, got %s" % t.dtype)


def _stream_handle(stream):
    if stream is None:
        stream = torch.cuda.current_stream()
    return ctypes.c_void_p(stream.cuda_stream)


def _ptr(t):
    return ctypes.c_void_p(t.data_ptr()) if t is not None else ctypes.c_void_p(0)


def _grad_table(grads):
    if len(grads) < 1:
        raise ValueError("need at least one gradient")
    P, code = grads[0].numel(), _dtype_code(grads[0])
    for g in grads:
        if not g.is_cuda or not g.is_contiguous() or g.dim() != 1 or g.numel() != P \
                or _dtype_code(g) != code:
            raise ValueError("gradients must be contiguous 1-D device tensors of one length and dtype")
    table = (ctypes.c_void_p * len(grads))(*[g.data_ptr() for g in grads])
    return table, P, code


class Context:
    """Owns a gaf_ctx handle (gaf_create / gaf_destroy)."""

    def __init__(self, max_P, max_N, device=None):
        device = torch.cuda.current_device() if device is None else int(device)
        self.device = device
        self._h = ctypes.c_void_p(0)
        _check(load().gaf_create(ctypes.byref(self._h), device, int(max_P), int(max_N)), "gaf_create")

    @property
    def handle(self):
        return self._h

    def close(self):
        if self._h:
            load().gaf_destroy(self._h)
            self._h = ctypes.c_void_p(0)

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass


def gaf_create(max_P, max_N, device=None):
    return Context(max_P, max_N, device)


def gaf_destroy(ctx):
    ctx.close()


def gaf_strerror(status):
    return strerror(status)


def gaf_set_schedule(ctx, schedule):
    """schedule: "auto" | "sequential" | "gram" (or the integer code)."""
    code = SCHEDULES[schedule] if isinstance(schedule, str) else int(schedule)
    _check(load().gaf_set_schedule(ctx.handle, code), "gaf_set_schedule")


def gaf_fused_mean_record(ctx):
    """Returns {write, valid, backoff, penalty} (waits for the device; diagnostics only)."""
    rec = (ctypes.c_int32 * 4)()
    _check(load().gaf_fused_mean_record(ctx.handle, rec), "gaf_fused_mean_record")
    return dict(zip(("write", "valid", "backoff", "penalty"), (int(v) for v in rec)))


def gaf_aggregate(ctx, grads, tau, out=None, accept_mask=None, cos_dist=None, count=None,
                  stream=None):
    """Enqueue the batch aggregation. Returns (out, accept_mask, cos_dist, count) device tensors;
    valid after the stream is synchronised."""
    table, P, code = _grad_table(grads)
    dev = grads[0].device
    N = len(grads)
    out = torch.empty(P, dtype=torch.float32, device=dev) if out is None else out
    accept_mask = torch.empty(N, dtype=torch.uint8, device=dev) if accept_mask is None else accept_mask
    cos_dist = torch.empty(N, dtype=torch.float32, device=dev) if cos_dist is None else cos_dist
    count = torch.empty(1, dtype=torch.int32, device=dev) if count is None else count
    _check(load().gaf_aggregate(ctx.handle, table, N, P, code, float(tau), _ptr(out),
                                _ptr(accept_mask), _ptr(cos_dist), _ptr(count),
                                _stream_handle(stream)), "gaf_aggregate")
    return out, accept_mask, cos_dist, count


def gaf_static_init():
    """Looks up the current device's fixed workspace ahead of the first gaf_aggregate_static."""
    _check(load().gaf_static_init(), "gaf_static_init")


def gaf_aggregate_static(grads, tau, out, accept_mask, cos_dist, count, stream=None):
    """gaf_aggregate without a context and without any allocation: every output is the caller's."""
    table, P, code = _grad_table(grads)
    _check(load().gaf_aggregate_static(table, len(grads), P, code, float(tau), _ptr(out), _ptr(accept_mask),
                                       _ptr(cos_dist), _ptr(count), _stream_handle(stream)),
           "gaf_aggregate_static")
    return out, accept_mask, cos_dist, count


def gaf_aggregate_with_gram(ctx, grads, tau, gram, out=None, accept_mask=None, cos_dist=None,
                            count=None, stream=None):
    """Batch aggregation reusing the Gram matrix gaf_pairwise wrote (N x N float64 device tensor)."""
    table, P, code = _grad_table(grads)
    dev = grads[0].device
    N = len(grads)
    if gram.dtype != torch.float64 or gram.numel() != N * N or not gram.is_contiguous():
        raise ValueError("gram must be a contiguous N x N float64 device tensor")
    out = torch.empty(P, dtype=torch.float32, device=dev) if out is None else out
    accept_mask = torch.empty(N, dtype=torch.uint8, device=dev) if accept_mask is None else accept_mask
    cos_dist = torch.empty(N, dtype=torch.float32, device=dev) if cos_dist is None else cos_dist
    count = torch.empty(1, dtype=torch.int32, device=dev) if count is None else count
    _check(load().gaf_aggregate_with_gram(ctx.handle, table, N, P, code, float(tau), _ptr(gram),
                                          _ptr(out), _ptr(accept_mask), _ptr(cos_dist), _ptr(count),
                                          _stream_handle(stream)), "gaf_aggregate_with_gram")
    return out, accept_mask, cos_dist, count


def _batch_outputs(grads, rows, out, accept_mask, cos_dist, count):
    P, N, dev = grads[0].numel(), len(grads), grads[0].device
    out = torch.empty(P, dtype=torch.float32, device=dev) if out is None else out
    shape = (N,) if rows is None else (rows, N)
    accept_mask = torch.empty(shape, dtype=torch.uint8, device=dev) if accept_mask is None else accept_mask
    cos_dist = torch.empty(shape, dtype=torch.float32, device=dev) if cos_dist is None else cos_dist
    count = torch.empty(1 if rows is None else rows, dtype=torch.int32, device=dev) if count is None else count
    return out, accept_mask, cos_dist, count


def gaf_aggregate_with_matrix(ctx, grads, tau, out=None, accept_mask=None, cos_dist=None, count=None,
                              D=None, gram=None, stream=None):
    """Batch aggregation plus the N x N distance matrix from the same Gram pass.
    Returns (out, accept_mask, cos_dist, count, D)."""
    table, P, code = _grad_table(grads)
    N = len(grads)
    out, accept_mask, cos_dist, count = _batch_outputs(grads, None, out, accept_mask, cos_dist, count)
    D = torch.empty((N, N), dtype=torch.float32, device=grads[0].device) if D is None else D
    _check(load().gaf_aggregate_with_matrix(ctx.handle, table, N, P, code, float(tau), _ptr(out),
                                            _ptr(accept_mask), _ptr(cos_dist), _ptr(count), _ptr(D),
                                            _ptr(gram), _stream_handle(stream)), "gaf_aggregate_with_matrix")
    return out, accept_mask, cos_dist, count, D


def gaf_aggregate_best_seed(ctx, grads, tau, out=None, accept_mask=None, cos_dist=None, count=None,
                            seed=None, stream=None):
    """Order-indifferent variant. Returns (out, accept_mask, cos_dist, count, seed)."""
    table, P, code = _grad_table(grads)
    out, accept_mask, cos_dist, count = _batch_outputs(grads, None, out, accept_mask, cos_dist, count)
    seed = torch.empty(1, dtype=torch.int32, device=grads[0].device) if seed is None else seed
    _check(load().gaf_aggregate_best_seed(ctx.handle, table, len(grads), P, code, float(tau), _ptr(out),
                                          _ptr(accept_mask), _ptr(cos_dist), _ptr(count), _ptr(seed),
                                          _stream_handle(stream)), "gaf_aggregate_best_seed")
    return out, accept_mask, cos_dist, count, seed


def gaf_aggregate_sgd(ctx, grads, tau, params, momentum_buf, lr, momentum, weight_decay, out=None,
                      accept_mask=None, cos_dist=None, count=None, want_out=True, stream=None):
    """Aggregation fused with the GAF-SGD step on (params, momentum_buf), in place.
    Returns (out or None, accept_mask, cos_dist, count)."""
    table, P, code = _grad_table(grads)
    for t in (params, momentum_buf):
        if t.dtype != torch.float32 or t.numel() != P or not t.is_contiguous() or not t.is_cuda:
            raise ValueError("params and momentum_buf must be contiguous float32 device tensors of length P")
    o, accept_mask, cos_dist, count = _batch_outputs(grads, None, out if want_out else params[:0],
                                                     accept_mask, cos_dist, count)
    o = o if want_out else None
    _check(load().gaf_aggregate_sgd(ctx.handle, table, len(grads), P, code, float(tau), _ptr(params),
                                    _ptr(momentum_buf), float(lr), float(momentum), float(weight_decay),
                                    _ptr(o), _ptr(accept_mask), _ptr(cos_dist), _ptr(count),
                                    _stream_handle(stream)), "gaf_aggregate_sgd")
    return o, accept_mask, cos_dist, count


def gaf_aggregate_bucketed(ctx, grads, tau, bucket_offsets, out=None, accept_mask=None, cos_dist=None,
                           count=None, stream=None):
    """Independent filter per bucket. Returns (out[P], accept_mask[B,N], cos_dist[B,N], count[B])."""
    table, P, code = _grad_table(grads)
    B = len(bucket_offsets) - 1
    out, accept_mask, cos_dist, count = _batch_outputs(grads, B, out, accept_mask, cos_dist, count)
    offs = (ctypes.c_size_t * (B + 1))(*[int(x) for x in bucket_offsets])
    _check(load().gaf_aggregate_bucketed(ctx.handle, table, len(grads), P, code, float(tau), B, offs,
                                         _ptr(out), _ptr(accept_mask), _ptr(cos_dist), _ptr(count),
                                         _stream_handle(stream)), "gaf_aggregate_bucketed")
    return out, accept_mask, cos_dist, count


def gaf_step(ctx, accum, count, g_i, tau, cos_dist_out=None, accepted_out=None, stream=None):
    """Enqueue one streaming visit; (accum, count) are updated in place on the device."""
    if not g_i.is_cuda or not g_i.is_contiguous() or g_i.dim() != 1:
        raise ValueError("g_i must be a contiguous 1-D device tensor")
    if accum.dtype != torch.float32 or accum.numel() != g_i.numel() or not accum.is_contiguous():
        raise ValueError("accum must be contiguous float32 of the gradient's length")
    if count.dtype != torch.int32 or count.numel() != 1:
        raise ValueError("count must be a single int32 on the device")
    _check(load().gaf_step(ctx.handle, _ptr(accum), _ptr(count), _ptr(g_i), g_i.numel(),
                           _dtype_code(g_i), float(tau), _ptr(cos_dist_out), _ptr(accepted_out),
                           _stream_handle(stream)), "gaf_step")


def gaf_step_lookahead(ctx, accum, count, g_i, tau, cos_dist_out=None, accepted_out=None, stream=None):
    """One streaming visit whose update of accum stays pending until the next such call or
    gaf_flush; g_i must stay alive until then."""
    if not g_i.is_cuda or not g_i.is_contiguous() or g_i.dim() != 1:
        raise ValueError("g_i must be a contiguous 1-D device tensor")
    if accum.dtype != torch.float32 or accum.numel() != g_i.numel() or not accum.is_contiguous():
        raise ValueError("accum must be contiguous float32 of the gradient's length")
    if count.dtype != torch.int32 or count.numel() != 1:
        raise ValueError("count must be a single int32 on the device")
    _check(load().gaf_step_lookahead(ctx.handle, _ptr(accum), _ptr(count), _ptr(g_i), g_i.numel(),
                                     _dtype_code(g_i), float(tau), _ptr(cos_dist_out), _ptr(accepted_out),
                                     _stream_handle(stream)), "gaf_step_lookahead")


def gaf_flush(ctx, stream=None):
    """Applies the update gaf_step_lookahead left pending, if any."""
    _check(load().gaf_flush(ctx.handle, _stream_handle(stream)), "gaf_flush")


def gaf_pairwise(ctx, grads, D=None, gram=None, stream=None):
    """Enqueue the all-pairs cosine-distance matrix. Returns D (N x N float32 device tensor)."""
    table, P, code = _grad_table(grads)
    N = len(grads)
    D = torch.empty((N, N), dtype=torch.float32, device=grads[0].device) if D is None else D
    _check(load().gaf_pairwise(ctx.handle, table, N, P, code, _ptr(D), _ptr(gram),
                               _stream_handle(stream)), "gaf_pairwise")
    return D


def gaf_profile_begin(ctx, max_launches=4096):
    _check(load().gaf_profile_begin(ctx.handle, int(max_launches)), "gaf_profile_begin")


def gaf_profile_end(ctx, cap=4096):
    """Returns [(kernel_name, milliseconds), ...] in launch order (waits for the launches)."""
    buf = (LaunchTime * cap)()
    n = ctypes.c_int(0)
    _check(load().gaf_profile_end(ctx.handle, buf, cap, ctypes.byref(n)), "gaf_profile_end")
    return [(KERNEL_NAMES[buf[k].kernel], float(buf[k].ms)) for k in range(n.value)]
