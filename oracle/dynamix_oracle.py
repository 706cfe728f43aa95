"""TEST INFRASTRUCTURE -- ctypes front end of the plain C oracle (dynamix_oracle.c).

Marshals numpy arrays into the C function and compiles it with gcc when the shared object is
missing or older than the source.  Holds none of the method's arithmetic.
"""
import ctypes
import os
import subprocess

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "dynamix_oracle.c")
_LIB = os.path.join(_HERE, "libdynamix_oracle.so")

HEAD = 8
#: positions of the scalars in a statistics record (the per-worker entries follow at HEAD)
IDX = {
    "agg_sqnorm": 0,
    "tr_sigma": 1,
    "agg_sqnorm_unbiased": 2,
    "noise_scale": 3,
    "noise_scale_biased": 4,
    "sigma2_norm": 5,
    "sigma_norm": 6,
    "count": 7,
}

_lib = None


def build(force=False):
    """Compile the C oracle into oracle/libdynamix_oracle.so."""
    stale = (not os.path.exists(_LIB)) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC)
    if force or stale:
        cmd = ["gcc", "-O2", "-fopenmp", "-shared", "-fPIC", "-std=c11", "-Wall", "-Wextra",
               "-o", _LIB, _SRC, "-lm"]
        subprocess.run(cmd, check=True)
    return _LIB


def _load():
    global _lib
    if _lib is None:
        lib = ctypes.CDLL(build())
        lib.dynamix_oracle_aggregate_stats.restype = ctypes.c_int
        lib.dynamix_oracle_aggregate_stats.argtypes = [
            ctypes.POINTER(ctypes.c_void_p), ctypes.POINTER(ctypes.c_int32), ctypes.c_int32,
            ctypes.c_int64, ctypes.c_int32, ctypes.POINTER(ctypes.c_int64), ctypes.c_int64,
            ctypes.POINTER(ctypes.c_double), ctypes.POINTER(ctypes.c_double), ctypes.c_int32]
        lib.dynamix_oracle_sgd_step.restype = ctypes.c_int
        lib.dynamix_oracle_sgd_step.argtypes = [
            ctypes.POINTER(ctypes.c_double), ctypes.POINTER(ctypes.c_float), ctypes.c_int64,
            ctypes.c_double, ctypes.c_double, ctypes.POINTER(ctypes.c_double)]
        dp, fp = ctypes.POINTER(ctypes.c_double), ctypes.POINTER(ctypes.c_float)
        lib.dynamix_oracle_sgd_momentum_step.restype = ctypes.c_int
        lib.dynamix_oracle_sgd_momentum_step.argtypes = [
            dp, fp, fp, ctypes.c_int64, ctypes.c_double, ctypes.c_double, ctypes.c_double,
            ctypes.c_int32, dp, dp]
        lib.dynamix_oracle_adam_step.restype = ctypes.c_int
        lib.dynamix_oracle_adam_step.argtypes = [
            dp, fp, fp, fp, ctypes.c_int64, ctypes.c_double, ctypes.c_double, ctypes.c_double,
            ctypes.c_double, ctypes.c_double, ctypes.c_int32, ctypes.c_int64, dp, dp, dp]
        lib.dynamix_oracle_max_threads.restype = ctypes.c_int
        lib.dynamix_oracle_widen.restype = ctypes.c_int
        lib.dynamix_oracle_widen.argtypes = [ctypes.c_void_p, ctypes.c_int32, ctypes.c_int64,
                                             ctypes.c_void_p]
        _lib = lib
    return _lib


def max_threads():
    return int(_load().dynamix_oracle_max_threads())


def widen(stored):
    """The value the oracle takes each stored element to be, as float64: `stored` is a 1-d array
    of float32, float16, or uint16 holding bf16 bit patterns."""
    a = np.ascontiguousarray(stored)
    code = {np.dtype(np.float32): 0, np.dtype(np.uint16): 1, np.dtype(np.float16): 2}[a.dtype]
    out = np.empty(a.shape[0], dtype=np.float64)
    if _load().dynamix_oracle_widen(a.ctypes.data, code, a.shape[0], out.ctypes.data) != 0:
        raise ValueError("oracle rejected the arguments")
    return out


def stats_count(K, S):
    return (1 + S) * (HEAD + 2 * K)


def aggregate_stats(grads, batch_sizes, segment_offsets=None, want_agg=True, threads=1):
    """Run the oracle.

    grads: K one-dimensional numpy arrays of equal length, dtype float32, float16, or uint16
    holding bf16 bit patterns.  batch_sizes: K positive integers.  segment_offsets: None, or S+1
    increasing offsets from 0 to P.
    Returns (agg, stats): agg is float64[P] (None if not wanted), stats is float64[1+S, 8+2K].
    """
    lib = _load()
    K = len(grads)
    if K < 1:
        raise ValueError("need at least one worker")
    arrs = [np.ascontiguousarray(g) for g in grads]
    dt = arrs[0].dtype
    if dt == np.float32:
        code = 0
    elif dt == np.uint16:
        code = 1
    elif dt == np.float16:
        code = 2
    else:
        raise TypeError("gradients must be float32, float16 or uint16 (bf16 bits), got %s" % dt)
    P = arrs[0].shape[0]
    for a in arrs:
        if a.ndim != 1 or a.shape[0] != P or a.dtype != dt:
            raise ValueError("all worker gradients must be 1-d, same length and dtype")
    ptrs = (ctypes.c_void_p * K)(*[a.ctypes.data for a in arrs])
    b = np.ascontiguousarray(np.asarray(batch_sizes, dtype=np.int32))
    if b.shape != (K,):
        raise ValueError("batch_sizes must have one entry per worker")
    if segment_offsets is None:
        S, off_p, off = 0, None, None
    else:
        off = np.ascontiguousarray(np.asarray(segment_offsets, dtype=np.int64))
        S = off.shape[0] - 1
        off_p = off.ctypes.data_as(ctypes.POINTER(ctypes.c_int64))
    agg = np.empty(P, dtype=np.float64) if want_agg else None
    stats = np.empty((1 + S, HEAD + 2 * K), dtype=np.float64)
    rc = lib.dynamix_oracle_aggregate_stats(
        ptrs, b.ctypes.data_as(ctypes.POINTER(ctypes.c_int32)), K, P, code, off_p, S,
        agg.ctypes.data_as(ctypes.POINTER(ctypes.c_double)) if want_agg else None,
        stats.ctypes.data_as(ctypes.POINTER(ctypes.c_double)), int(threads))
    if rc != 0:
        raise ValueError("oracle rejected its arguments")
    return agg, stats


def sgd_step(agg, params, lr, weight_decay=0.0):
    """p - lr * (G + weight_decay * p) with G = agg (float64[P]) and params float32[P];
    returns float64[P]."""
    lib = _load()
    agg = np.ascontiguousarray(agg, dtype=np.float64)
    params = np.ascontiguousarray(params)
    if params.dtype != np.float32 or params.shape != agg.shape or agg.ndim != 1:
        raise TypeError("params must be float32 and match agg")
    out = np.empty_like(agg)
    rc = lib.dynamix_oracle_sgd_step(
        agg.ctypes.data_as(ctypes.POINTER(ctypes.c_double)),
        params.ctypes.data_as(ctypes.POINTER(ctypes.c_float)), agg.shape[0], float(lr),
        float(weight_decay), out.ctypes.data_as(ctypes.POINTER(ctypes.c_double)))
    if rc != 0:
        raise ValueError("oracle rejected its arguments")
    return out


def _f32(a, shape):
    a = np.ascontiguousarray(a)
    if a.dtype != np.float32 or a.shape != shape:
        raise TypeError("parameters and optimizer state must be float32 and match agg")
    return a


def _dp(a):
    return a.ctypes.data_as(ctypes.POINTER(ctypes.c_double))


def _fp(a):
    return a.ctypes.data_as(ctypes.POINTER(ctypes.c_float))


def sgd_momentum_step(agg, params, buf, lr, weight_decay=0.0, momentum=0.0, nesterov=False):
    """One step of SGD with momentum on G = agg (float64[P]); params and buf float32[P].
    Returns (new params, new momentum buffer) as float64[P]."""
    lib = _load()
    agg = np.ascontiguousarray(agg, dtype=np.float64)
    if agg.ndim != 1:
        raise TypeError("agg must be 1-d")
    params, buf = _f32(params, agg.shape), _f32(buf, agg.shape)
    out_p, out_b = np.empty_like(agg), np.empty_like(agg)
    rc = lib.dynamix_oracle_sgd_momentum_step(_dp(agg), _fp(params), _fp(buf), agg.shape[0],
                                              float(lr), float(weight_decay), float(momentum),
                                              int(bool(nesterov)), _dp(out_p), _dp(out_b))
    if rc != 0:
        raise ValueError("oracle rejected its arguments")
    return out_p, out_b


def adam_step(agg, params, exp_avg, exp_avg_sq, lr, beta1=0.9, beta2=0.999, eps=1e-8,
              weight_decay=0.0, decoupled=False, step=1):
    """One step of Adam (decoupled: AdamW) on G = agg (float64[P]); params and the two moment
    estimates float32[P]; step counts from 1.  Returns (params, exp_avg, exp_avg_sq) as float64[P]."""
    lib = _load()
    agg = np.ascontiguousarray(agg, dtype=np.float64)
    if agg.ndim != 1:
        raise TypeError("agg must be 1-d")
    params, m, v = (_f32(x, agg.shape) for x in (params, exp_avg, exp_avg_sq))
    out_p, out_m, out_v = np.empty_like(agg), np.empty_like(agg), np.empty_like(agg)
    rc = lib.dynamix_oracle_adam_step(_dp(agg), _fp(params), _fp(m), _fp(v), agg.shape[0],
                                      float(lr), float(beta1), float(beta2), float(eps),
                                      float(weight_decay), int(bool(decoupled)), int(step),
                                      _dp(out_p), _dp(out_m), _dp(out_v))
    if rc != 0:
        raise ValueError("oracle rejected its arguments")
    return out_p, out_m, out_v
