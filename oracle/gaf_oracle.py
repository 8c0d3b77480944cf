"""ctypes front end of the CPU oracle (``gaf_oracle.c``).

TEST INFRASTRUCTURE ONLY: imported by the test suite, the smoke check and the
benchmark's CPU-baseline leg. The HIP library and its Python binding never
import this module.

Arrays are numpy: ``float32`` for binary32 inputs, ``uint16`` holding bfloat16
bit patterns for bf16 inputs. All results are fp64.

Functions mirror the passages of the paper they implement:
``cosine_distance`` is Eq. 4; ``aggregate`` is Algorithm 1's aggregation part
followed by Eq. 5; ``step`` is one visit of the algorithm's inner loop;
``plain_average`` is Eq. 2; ``pairwise`` is Eq. 4 over all pairs.
"""
import ctypes
import os
import subprocess

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "gaf_oracle.c")
_LIB = os.path.join(_HERE, "libgaf_oracle.so")
# The mutation test of the pins (tests/test_oracle_mutants.py) loads a private copy of this
# module and points it at a deliberately broken build of the oracle, expecting the pins to
# fail; nothing else sets it.
_OVERRIDE = None

F32, BF16 = 0, 1


def build(force=False):
    """Compile the oracle with gcc (-O2, OpenMP, no fast-math)."""
    if _OVERRIDE:
        return _OVERRIDE
    if (not force and os.path.exists(_LIB)
            and os.path.getmtime(_LIB) >= os.path.getmtime(_SRC)):
        return _LIB
    cmd = ["gcc", "-O2", "-fopenmp", "-fPIC", "-shared", "-std=c11", "-Wall", "-Wextra",
           "-ffp-contract=off", "-o", _LIB, _SRC, "-lm"]
    subprocess.run(cmd, check=True)
    return _LIB


_lib = None


def _load():
    global _lib
    if _lib is not None:
        return _lib
    lib = ctypes.CDLL(build())
    c = ctypes
    lib.oracle_num_threads.restype = c.c_int
    lib.oracle_distance_from_sums.restype = c.c_double
    lib.oracle_distance_from_sums.argtypes = [c.c_double] * 3
    lib.oracle_cosine_distance.restype = c.c_double
    lib.oracle_cosine_distance.argtypes = [c.c_void_p, c.c_void_p, c.c_size_t, c.c_int]
    lib.oracle_gaf_step.restype = c.c_int
    lib.oracle_gaf_step.argtypes = [c.c_void_p, c.c_void_p, c.c_void_p, c.c_size_t, c.c_int,
                                    c.c_double, c.c_void_p, c.c_void_p]
    lib.oracle_gaf_aggregate.restype = c.c_int
    lib.oracle_gaf_aggregate.argtypes = [c.c_void_p, c.c_int, c.c_size_t, c.c_int, c.c_double,
                                         c.c_void_p, c.c_void_p, c.c_void_p, c.c_void_p]
    lib.oracle_plain_average.restype = c.c_int
    lib.oracle_plain_average.argtypes = [c.c_void_p, c.c_int, c.c_size_t, c.c_int, c.c_void_p]
    lib.oracle_gaf_pairwise.restype = c.c_int
    lib.oracle_gaf_pairwise.argtypes = [c.c_void_p, c.c_int, c.c_size_t, c.c_int, c.c_void_p,
                                        c.c_void_p]
    lib.oracle_gaf_best_seed.restype = c.c_int
    lib.oracle_gaf_best_seed.argtypes = [c.c_void_p, c.c_int, c.c_size_t, c.c_int, c.c_double] + [c.c_void_p] * 6
    lib.oracle_sgd_step.restype = c.c_int
    lib.oracle_sgd_step.argtypes = [c.c_void_p, c.c_void_p, c.c_void_p, c.c_int32, c.c_size_t,
                                    c.c_double, c.c_double, c.c_double]
    lib.oracle_gaf_bucketed.restype = c.c_int
    lib.oracle_gaf_bucketed.argtypes = [c.c_void_p, c.c_int, c.c_size_t, c.c_int, c.c_double, c.c_int,
                                        c.c_void_p, c.c_void_p, c.c_void_p, c.c_void_p, c.c_void_p]
    _lib = lib
    return lib


def num_threads():
    return int(_load().oracle_num_threads())


def _dtype_code(a):
    if a.dtype == np.float32:
        return F32
    if a.dtype == np.uint16:
        return BF16
    raise TypeError("oracle inputs must be float32 or uint16 (bf16 bits), got %s" % a.dtype)


def _prep(grads):
    grads = [np.ascontiguousarray(g) for g in grads]
    if not grads:
        raise ValueError("need at least one gradient")
    code = _dtype_code(grads[0])
    P = grads[0].size
    for g in grads:
        if g.ndim != 1 or g.size != P or _dtype_code(g) != code:
            raise ValueError("all gradients must be 1-D, same length, same dtype")
    ptrs = (ctypes.c_void_p * len(grads))(*[g.ctypes.data for g in grads])
    return grads, ptrs, P, code


def distance_from_sums(xy, xx, yy):
    return float(_load().oracle_distance_from_sums(float(xy), float(xx), float(yy)))


def cosine_distance(x, y):
    (x, y), _, P, code = _prep([x, y])
    return float(_load().oracle_cosine_distance(x.ctypes.data, y.ctypes.data, P, code))


def aggregate(grads, tau):
    """Returns (out[P] f64, mask[N] u8, dist[N] f64, count)."""
    grads, ptrs, P, code = _prep(grads)
    N = len(grads)
    out = np.empty(P, dtype=np.float64)
    mask = np.zeros(N, dtype=np.uint8)
    dist = np.zeros(N, dtype=np.float64)
    count = ctypes.c_int32(0)
    rc = _load().oracle_gaf_aggregate(ptrs, N, P, code, float(tau), out.ctypes.data,
                                      mask.ctypes.data, dist.ctypes.data, ctypes.byref(count))
    if rc:
        raise RuntimeError("oracle_gaf_aggregate failed: %d" % rc)
    return out, mask, dist, int(count.value)


def step(g_sum, count, g_i, tau):
    """One visit; g_sum (f64, length P) is updated in place.

    Returns (dist, accepted, new_count). count == 0 makes g_i the seed."""
    g_i = np.ascontiguousarray(g_i)
    code = _dtype_code(g_i)
    if g_sum.dtype != np.float64 or not g_sum.flags.c_contiguous or g_sum.size != g_i.size:
        raise ValueError("g_sum must be contiguous float64 of the gradient's length")
    c = ctypes.c_int32(int(count))
    dist = ctypes.c_double(0.0)
    acc = ctypes.c_uint8(0)
    rc = _load().oracle_gaf_step(g_sum.ctypes.data, ctypes.byref(c), g_i.ctypes.data, g_i.size,
                                 code, float(tau), ctypes.byref(dist), ctypes.byref(acc))
    if rc:
        raise RuntimeError("oracle_gaf_step failed: %d" % rc)
    return float(dist.value), int(acc.value), int(c.value)


def plain_average(grads):
    grads, ptrs, P, code = _prep(grads)
    out = np.empty(P, dtype=np.float64)
    rc = _load().oracle_plain_average(ptrs, len(grads), P, code, out.ctypes.data)
    if rc:
        raise RuntimeError("oracle_plain_average failed: %d" % rc)
    return out


def pairwise(grads):
    """Returns (D[N,N] f64 distances, G[N,N] f64 inner products)."""
    grads, ptrs, P, code = _prep(grads)
    N = len(grads)
    D = np.empty((N, N), dtype=np.float64)
    G = np.empty((N, N), dtype=np.float64)
    rc = _load().oracle_gaf_pairwise(ptrs, N, P, code, D.ctypes.data, G.ctypes.data)
    if rc:
        raise RuntimeError("oracle_gaf_pairwise failed: %d" % rc)
    return D, G


def best_seed(grads, tau):
    """Order-indifferent variant. Returns (out, mask, dist, count, seed, counts_of_all_seeds)."""
    grads, ptrs, P, code = _prep(grads)
    N = len(grads)
    out = np.empty(P, dtype=np.float64)
    mask = np.zeros(N, dtype=np.uint8)
    dist = np.zeros(N, dtype=np.float64)
    counts = np.zeros(N, dtype=np.int32)
    count, seed = ctypes.c_int32(0), ctypes.c_int32(-1)
    rc = _load().oracle_gaf_best_seed(ptrs, N, P, code, float(tau), out.ctypes.data, mask.ctypes.data,
                                      dist.ctypes.data, ctypes.addressof(count), ctypes.addressof(seed),
                                      counts.ctypes.data)
    if rc:
        raise RuntimeError("oracle_gaf_best_seed failed: %d" % rc)
    return out, mask, dist, int(count.value), int(seed.value), counts


def sgd_step(theta, v, g_gaf, count, lr, mu, wd):
    """GAF-SGD step on float64 arrays, in place (skipped when count == 1)."""
    for a in (theta, v, g_gaf):
        if a.dtype != np.float64 or not a.flags.c_contiguous or a.size != theta.size:
            raise ValueError("theta, v, g_gaf must be contiguous float64 of one length")
    rc = _load().oracle_sgd_step(theta.ctypes.data, v.ctypes.data, g_gaf.ctypes.data, int(count),
                                 theta.size, float(lr), float(mu), float(wd))
    if rc:
        raise RuntimeError("oracle_sgd_step failed: %d" % rc)


def bucketed(grads, tau, offsets):
    """Independent filter per bucket. Returns (out[P], mask[B,N], dist[B,N], count[B])."""
    grads, ptrs, P, code = _prep(grads)
    N = len(grads)
    off = np.ascontiguousarray(offsets, dtype=np.uint64)
    B = off.size - 1
    out = np.empty(P, dtype=np.float64)
    mask = np.zeros((B, N), dtype=np.uint8)
    dist = np.zeros((B, N), dtype=np.float64)
    count = np.zeros(B, dtype=np.int32)
    rc = _load().oracle_gaf_bucketed(ptrs, N, P, code, float(tau), B, off.ctypes.data, out.ctypes.data,
                                     mask.ctypes.data, dist.ctypes.data, count.ctypes.data)
    if rc:
        raise RuntimeError("oracle_gaf_bucketed failed: %d" % rc)
    return out, mask, dist, count
