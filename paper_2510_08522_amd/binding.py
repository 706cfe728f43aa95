"""ctypes binding of libdynamix.so: argument marshalling only.

Every step of the path (aggregation, statistics, reductions, derived scalars) runs in the HIP
kernels behind the C ABI declared in include/dynamix.h; torch is used for device memory and
streams.  There is no CPU fallback: a missing library raises.
"""
import ctypes
import os

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libdynamix.so")

DYNAMIX_F32, DYNAMIX_BF16, DYNAMIX_F16 = 0, 1, 2
DYNAMIX_OK = 0
DYNAMIX_ERR_NULL, DYNAMIX_ERR_ARG, DYNAMIX_ERR_SEGMENTS = 1, 2, 3
DYNAMIX_ERR_ALIGN, DYNAMIX_ERR_NOMEM, DYNAMIX_ERR_HIP = 4, 5, 6
DYNAMIX_ERR_CAPACITY = 7
DYNAMIX_STATIC_SCRATCH_BYTES = 4 << 20
DYNAMIX_K_MAX = 256
DYNAMIX_K_MAX_ONE_SWEEP = 64
DYNAMIX_K_MAX_STATEFUL = 32
DYNAMIX_STATS_HEAD = 8
STAT = {"agg_sqnorm": 0, "tr_sigma": 1, "agg_sqnorm_unbiased": 2, "noise_scale": 3,
        "noise_scale_biased": 4, "sigma2_norm": 5, "sigma_norm": 6, "count": 7}

_lib = None


class DynamixError(RuntimeError):
    def __init__(self, status):
        self.status = int(status)
        super().__init__("dynamix: %s (status %d)" % (dynamix_status_string(status), status))


def load():
    """Load libdynamix.so from the package directory; raises if it has not been built."""
    global _lib
    if _lib is not None:
        return _lib
    if not os.path.exists(LIB_PATH):
        raise RuntimeError("libdynamix.so is not built: run `python -m paper_2510_08522_amd.build` "
                           "(there is no fallback path)")
    lib = ctypes.CDLL(LIB_PATH)
    vp, i32, i64 = ctypes.c_void_p, ctypes.c_int32, ctypes.c_int64
    lib.dynamix_grad_aggregate_stats.restype = ctypes.c_int
    lib.dynamix_grad_aggregate_stats.argtypes = [vp, vp, i32, i64, i32, vp, vp, vp, vp]
    lib.dynamix_grad_aggregate_stats_ex.restype = ctypes.c_int
    lib.dynamix_grad_aggregate_stats_ex.argtypes = [vp, vp, i32, i64, i32, vp, i64, vp, vp, vp]
    lib.dynamix_grad_aggregate_stats_static.restype = ctypes.c_int
    lib.dynamix_grad_aggregate_stats_static.argtypes = [vp, vp, i32, i64, i32, vp, i64, vp, vp, vp]
    lib.dynamix_grad_aggregate_stats_sgd.restype = ctypes.c_int
    lib.dynamix_grad_aggregate_stats_sgd.argtypes = [vp, vp, i32, i64, i32, vp, i64, vp,
                                                     ctypes.c_float, ctypes.c_float, vp, vp]
    f32 = ctypes.c_float
    lib.dynamix_grad_aggregate_stats_sgd_momentum.restype = ctypes.c_int
    lib.dynamix_grad_aggregate_stats_sgd_momentum.argtypes = [vp, vp, i32, i64, i32, vp, i64, vp, vp,
                                                              f32, f32, f32, i32, vp, vp]
    lib.dynamix_grad_aggregate_stats_adam.restype = ctypes.c_int
    lib.dynamix_grad_aggregate_stats_adam.argtypes = [vp, vp, i32, i64, i32, vp, i64, vp, vp, vp,
                                                      f32, f32, f32, f32, f32, i32, i64, vp, vp]
    lib.dynamix_stats_count.restype = i64
    lib.dynamix_stats_count.argtypes = [i32, i64]
    lib.dynamix_status_string.restype = ctypes.c_char_p
    lib.dynamix_status_string.argtypes = [ctypes.c_int]
    lib.dynamix_plan_describe.restype = i64
    lib.dynamix_plan_describe.argtypes = [i32, i64, i32, vp, i64, i64, vp, i64]
    lib.dynamix_timing_begin.restype = ctypes.c_int
    lib.dynamix_timing_begin.argtypes = [i32]
    lib.dynamix_timing_every.restype = ctypes.c_int
    lib.dynamix_timing_every.argtypes = [i32]
    lib.dynamix_timing_count.restype = i32
    lib.dynamix_timing_count.argtypes = []
    lib.dynamix_timing_read.restype = ctypes.c_int
    lib.dynamix_timing_read.argtypes = [i32, ctypes.POINTER(ctypes.c_float),
                                        ctypes.POINTER(ctypes.c_float)]
    lib.dynamix_cycle_accumulate.restype = ctypes.c_int
    lib.dynamix_cycle_accumulate.argtypes = [vp, i64, vp, i32, vp]
    lib.dynamix_cycle_summary.restype = ctypes.c_int
    lib.dynamix_cycle_summary.argtypes = [vp, i32, i64, vp, ctypes.c_double, ctypes.c_double, vp, vp]
    lib.dynamix_cycle_summary_count.restype = i64
    lib.dynamix_cycle_summary_count.argtypes = [i32, i64]
    lib.dynamix_hbm_probe.restype = ctypes.c_int
    lib.dynamix_hbm_probe.argtypes = [vp, i32, i64, i32, i32, vp]
    f64 = ctypes.c_double
    lib.dynamix_policy_weight_count.restype = i64
    lib.dynamix_policy_weight_count.argtypes = [vp, i32]
    lib.dynamix_policy_forward.restype = ctypes.c_int
    lib.dynamix_policy_forward.argtypes = [vp, vp, i32, vp, i32, vp]
    lib.dynamix_policy_choose.restype = ctypes.c_int
    lib.dynamix_policy_choose.argtypes = [vp, i32, vp, vp]
    lib.dynamix_batch_sizes_step.restype = ctypes.c_int
    lib.dynamix_batch_sizes_step.argtypes = [vp, vp, i32, i32, i32, vp]
    lib.dynamix_cycle_rewards.restype = ctypes.c_int
    lib.dynamix_cycle_rewards.argtypes = [vp, vp, vp, vp, i32, f64, f64, f64, f64, f64, f64, i32, vp]
    lib.dynamix_policy_update.restype = ctypes.c_int
    lib.dynamix_policy_update.argtypes = [vp, vp, i32, vp, vp, vp, vp, i64, i32, f64, f64, vp]
    lib.dynamix_discounted_return.restype = f64
    lib.dynamix_discounted_return.argtypes = [vp, i64, f64]
    lib.dynamix_release_cached.restype = ctypes.c_int
    lib.dynamix_release_cached.argtypes = []
    _lib = lib
    return lib


def dynamix_stats_count(K, num_segments):
    return int(load().dynamix_stats_count(int(K), int(num_segments)))


def dynamix_status_string(status):
    return load().dynamix_status_string(int(status)).decode()


def dynamix_release_cached():
    return int(load().dynamix_release_cached())


DYNAMIX_PROBE_READ, DYNAMIX_PROBE_READ_SPREAD, DYNAMIX_PROBE_WRITE, DYNAMIX_PROBE_COPY = 0, 1, 2, 3
DYNAMIX_PROBE_READ_SPREAD_128B, DYNAMIX_PROBE_READ_SPREAD_512B = 4, 5


def dynamix_hbm_probe(buffers, nbytes, mode, blocks, stream=None):
    """Enqueue one of the plain streaming kernels (measurement aid) over `buffers`, device tensors
    of at least `nbytes` bytes each."""
    import torch
    if stream is None:
        stream = torch.cuda.current_stream(buffers[0].device)
    ptrs = (ctypes.c_void_p * len(buffers))(*[t.data_ptr() for t in buffers])
    rc = int(load().dynamix_hbm_probe(ptrs, len(buffers), int(nbytes), int(mode), int(blocks),
                                      stream.cuda_stream))
    if rc != DYNAMIX_OK:
        raise DynamixError(rc)


def dynamix_plan_describe(K, P, dtype, segment_offsets=None, max_blocks=256):
    """The work decomposition for a shape as an int64 array [pieces, 6]:
    (first vector, end vector, vectors per iteration, first element, end element, block).
    Host only."""
    lib = load()
    off, S = None, 0
    if segment_offsets is not None:
        S = len(segment_offsets) - 1
        off = (ctypes.c_int64 * (S + 1))(*[int(x) for x in segment_offsets])
    n = lib.dynamix_plan_describe(K, P, dtype, off, S, max_blocks, None, 0)
    if n < 0:
        raise DynamixError(-n)
    out = np.zeros((n, 6), dtype=np.int64)
    lib.dynamix_plan_describe(K, P, dtype, off, S, max_blocks,
                              out.ctypes.data_as(ctypes.c_void_p), n)
    return out


def dynamix_timing_begin(capacity):
    rc = int(load().dynamix_timing_begin(int(capacity)))
    if rc != DYNAMIX_OK:
        raise DynamixError(rc)


def dynamix_timing_every(n):
    rc = int(load().dynamix_timing_every(int(n)))
    if rc != DYNAMIX_OK:
        raise DynamixError(rc)


def dynamix_timing_count():
    return int(load().dynamix_timing_count())


def dynamix_timing_read(index):
    """(streaming pass ms, final reduction ms) of the index-th timed call; sync the stream first."""
    a, b = ctypes.c_float(), ctypes.c_float()
    rc = int(load().dynamix_timing_read(int(index), ctypes.byref(a), ctypes.byref(b)))
    if rc != DYNAMIX_OK:
        raise DynamixError(rc)
    return a.value, b.value


def dynamix_cycle_summary_count(K, num_segments):
    return int(load().dynamix_cycle_summary_count(int(K), int(num_segments)))


def dynamix_cycle_accumulate(stats, window=None, first=False, stream=None):
    """window += stats on the device (window := stats when first); returns the window tensor,
    float64[stats.numel() + 1], whose last entry counts the iterations."""
    import torch
    count = stats.numel()
    if window is None:
        if not first:
            raise ValueError("a window must be given unless this call starts a cycle")
        window = torch.empty(count + 1, dtype=torch.float64, device=stats.device)
    if stream is None:
        stream = torch.cuda.current_stream(stats.device)
    rc = int(load().dynamix_cycle_accumulate(stats.data_ptr(), count, window.data_ptr(),
                                             int(bool(first)), stream.cuda_stream))
    if rc != DYNAMIX_OK:
        raise DynamixError(rc)
    return window


def dynamix_cycle_summary(window, K, num_segments, batch_sizes, eta, delta, summary=None,
                          stream=None):
    """Means, pooled ratios and reward terms of the cycle held in `window`; returns the summary
    tensor float64[dynamix_cycle_summary_count(K, S)]."""
    import torch
    if summary is None:
        summary = torch.empty(dynamix_cycle_summary_count(K, num_segments), dtype=torch.float64,
                              device=window.device)
    if stream is None:
        stream = torch.cuda.current_stream(window.device)
    b = (ctypes.c_int32 * K)(*[int(x) for x in batch_sizes])
    rc = int(load().dynamix_cycle_summary(window.data_ptr(), K, num_segments, b, float(eta),
                                          float(delta), summary.data_ptr(), stream.cuda_stream))
    if rc != DYNAMIX_OK:
        raise DynamixError(rc)
    return summary


def call_raw(grad_ptrs, batch_sizes, K, P, dtype, segment_offsets, num_segments, out_agg_ptr,
             out_stats_ptr, stream_ptr, explicit_count=True, static=False):
    """The C entry points on plain integers/sequences; returns the status.  grad_ptrs and
    batch_sizes may be None to pass NULL.  Used directly by the error-path tests."""
    lib = load()
    ptrs = None if grad_ptrs is None else (ctypes.c_void_p * len(grad_ptrs))(*grad_ptrs)
    b = None if batch_sizes is None else (ctypes.c_int32 * len(batch_sizes))(*batch_sizes)
    off = None
    if segment_offsets is not None:
        off = (ctypes.c_int64 * len(segment_offsets))(*segment_offsets)
    if static:
        return int(lib.dynamix_grad_aggregate_stats_static(
            ptrs, b, K, P, dtype, off, num_segments, out_agg_ptr, out_stats_ptr, stream_ptr))
    if explicit_count:
        return int(lib.dynamix_grad_aggregate_stats_ex(
            ptrs, b, K, P, dtype, off, num_segments, out_agg_ptr, out_stats_ptr, stream_ptr))
    return int(lib.dynamix_grad_aggregate_stats(
        ptrs, b, K, P, dtype, off, out_agg_ptr, out_stats_ptr, stream_ptr))


def _marshal(grads, batch_sizes, segment_offsets, out_agg, out_stats, stream, stats_only):
    import torch
    K = len(grads)
    g0 = grads[0]
    if g0.dtype == torch.float32:
        dtype = DYNAMIX_F32
    elif g0.dtype == torch.bfloat16:
        dtype = DYNAMIX_BF16
    elif g0.dtype == torch.float16:
        dtype = DYNAMIX_F16
    else:
        raise TypeError("gradients must be float32, bfloat16 or float16")
    P = g0.numel()
    for g in grads:
        if not (g.is_cuda and g.is_contiguous() and g.dim() == 1 and g.numel() == P
                and g.dtype == g0.dtype and g.device == g0.device):
            raise ValueError("every gradient must be a contiguous 1-d device tensor of equal "
                             "length, dtype and device")
    S = 0 if segment_offsets is None else len(segment_offsets) - 1
    if out_agg is None and not stats_only:
        out_agg = torch.empty(P, dtype=torch.float32, device=g0.device)
    if out_stats is None:
        out_stats = torch.empty((1 + S, DYNAMIX_STATS_HEAD + 2 * K), dtype=torch.float64,
                                device=g0.device)
    if stream is None:
        stream = torch.cuda.current_stream(g0.device)
    off = None if segment_offsets is None else [int(x) for x in segment_offsets]
    return dict(grad_ptrs=[g.data_ptr() for g in grads], batch_sizes=[int(x) for x in batch_sizes],
                K=K, P=P, dtype=dtype, segment_offsets=off, num_segments=S,
                out_agg_ptr=None if out_agg is None else out_agg.data_ptr(),
                out_stats_ptr=out_stats.data_ptr(), stream_ptr=stream.cuda_stream), out_agg, out_stats


def dynamix_grad_aggregate_stats_ex(grads, batch_sizes, segment_offsets=None, out_agg=None,
                                    out_stats=None, stream=None, stats_only=False):
    """Enqueue one aggregate + statistics pass on `stream` (default: torch's current stream).

    grads: K contiguous 1-d device tensors (float32, bfloat16 or float16).  Returns (out_agg, out_stats):
    float32[P] (None when stats_only) and float64[1+S, 8+2K]; valid after the stream is
    synchronised.  Raises DynamixError on a non-zero status.
    """
    kw, out_agg, out_stats = _marshal(grads, batch_sizes, segment_offsets, out_agg, out_stats,
                                      stream, stats_only)
    rc = call_raw(explicit_count=True, **kw)
    if rc != DYNAMIX_OK:
        raise DynamixError(rc)
    return out_agg, out_stats


def dynamix_grad_aggregate_stats_static(grads, batch_sizes, segment_offsets=None, out_agg=None,
                                        out_stats=None, stream=None, stats_only=False):
    """As dynamix_grad_aggregate_stats_ex, through the entry point whose workspace is the
    library's static device array: the library allocates nothing (pass out_agg and out_stats, or
    this wrapper allocates them with torch before the call).  Raises DynamixError with status
    DYNAMIX_ERR_CAPACITY for a shape that needs more than DYNAMIX_STATIC_SCRATCH_BYTES."""
    kw, out_agg, out_stats = _marshal(grads, batch_sizes, segment_offsets, out_agg, out_stats,
                                      stream, stats_only)
    rc = call_raw(static=True, **kw)
    if rc != DYNAMIX_OK:
        raise DynamixError(rc)
    return out_agg, out_stats


def dynamix_grad_aggregate_stats(grads, batch_sizes, segment_offsets=None, out_agg=None,
                                 out_stats=None, stream=None, stats_only=False):
    """As dynamix_grad_aggregate_stats_ex, through the entry point that finds the number of
    segments from the offsets array (it ends at the entry equal to P)."""
    kw, out_agg, out_stats = _marshal(grads, batch_sizes, segment_offsets, out_agg, out_stats,
                                      stream, stats_only)
    rc = call_raw(explicit_count=False, **kw)
    if rc != DYNAMIX_OK:
        raise DynamixError(rc)
    return out_agg, out_stats


def dynamix_grad_aggregate_stats_sgd(grads, batch_sizes, params, lr, weight_decay=0.0,
                                     segment_offsets=None, out_stats=None, stream=None):
    """Aggregate + statistics with the SGD step fused in: params (float32[P] device tensor) is
    updated in place to params - lr * (G + weight_decay * params).  Returns out_stats."""
    import torch
    if not (params.is_cuda and params.is_contiguous() and params.dtype == torch.float32
            and params.numel() == grads[0].numel()):
        raise ValueError("params must be a contiguous float32 device tensor of P elements")
    kw, _, out_stats = _marshal(grads, batch_sizes, segment_offsets, None, out_stats, stream, True)
    lib = load()
    K = kw["K"]
    ptrs = (ctypes.c_void_p * K)(*kw["grad_ptrs"])
    b = (ctypes.c_int32 * K)(*kw["batch_sizes"])
    off = None
    if kw["segment_offsets"] is not None:
        off = (ctypes.c_int64 * len(kw["segment_offsets"]))(*kw["segment_offsets"])
    rc = int(lib.dynamix_grad_aggregate_stats_sgd(
        ptrs, b, K, kw["P"], kw["dtype"], off, kw["num_segments"], params.data_ptr(), float(lr),
        float(weight_decay), kw["out_stats_ptr"], kw["stream_ptr"]))
    if rc != DYNAMIX_OK:
        raise DynamixError(rc)
    return out_stats


def _update_args(grads, batch_sizes, segment_offsets, out_stats, stream, tensors):
    """C arguments shared by the fused-update entry points; `tensors` are the parameter and state
    tensors, checked here."""
    import torch
    for t in tensors:
        if not (t.is_cuda and t.is_contiguous() and t.dtype == torch.float32
                and t.numel() == grads[0].numel()):
            raise ValueError("parameters and optimizer state must be contiguous float32 device "
                             "tensors of P elements")
    kw, _, out_stats = _marshal(grads, batch_sizes, segment_offsets, None, out_stats, stream, True)
    K = kw["K"]
    ptrs = (ctypes.c_void_p * K)(*kw["grad_ptrs"])
    b = (ctypes.c_int32 * K)(*kw["batch_sizes"])
    off = None
    if kw["segment_offsets"] is not None:
        off = (ctypes.c_int64 * len(kw["segment_offsets"]))(*kw["segment_offsets"])
    head = (ptrs, b, K, kw["P"], kw["dtype"], off, kw["num_segments"])
    return head, kw["out_stats_ptr"], kw["stream_ptr"], out_stats


def dynamix_grad_aggregate_stats_sgd_momentum(grads, batch_sizes, params, momentum_buf, lr,
                                              weight_decay=0.0, momentum=0.9, nesterov=False,
                                              segment_offsets=None, out_stats=None, stream=None):
    """Aggregate + statistics with SGD with momentum fused in: params and momentum_buf
    (float32[P] device tensors) are updated in place.  Returns out_stats."""
    head, st_ptr, s_ptr, out_stats = _update_args(grads, batch_sizes, segment_offsets, out_stats,
                                                  stream, (params, momentum_buf))
    rc = int(load().dynamix_grad_aggregate_stats_sgd_momentum(
        *head, params.data_ptr(), momentum_buf.data_ptr(), float(lr), float(weight_decay),
        float(momentum), int(bool(nesterov)), st_ptr, s_ptr))
    if rc != DYNAMIX_OK:
        raise DynamixError(rc)
    return out_stats


def dynamix_grad_aggregate_stats_adam(grads, batch_sizes, params, exp_avg, exp_avg_sq, lr, step,
                                      beta1=0.9, beta2=0.999, eps=1e-8, weight_decay=0.0,
                                      decoupled=False, segment_offsets=None, out_stats=None,
                                      stream=None):
    """Aggregate + statistics with an Adam step (decoupled: AdamW) fused in: params, exp_avg and
    exp_avg_sq (float32[P] device tensors) are updated in place; step counts from 1.  Returns
    out_stats."""
    head, st_ptr, s_ptr, out_stats = _update_args(grads, batch_sizes, segment_offsets, out_stats,
                                                  stream, (params, exp_avg, exp_avg_sq))
    rc = int(load().dynamix_grad_aggregate_stats_adam(
        *head, params.data_ptr(), exp_avg.data_ptr(), exp_avg_sq.data_ptr(), float(lr),
        float(beta1), float(beta2), float(eps), float(weight_decay), int(bool(decoupled)),
        int(step), st_ptr, s_ptr))
    if rc != DYNAMIX_OK:
        raise DynamixError(rc)
    return out_stats


# ---- host side of an adjustment cycle (numpy arrays in, numpy arrays out; no device work)
DYNAMIX_NUM_ACTIONS = 5
DYNAMIX_ACTIONS = (-100, -25, 0, 25, 100)


def _np(a, dtype):
    return np.ascontiguousarray(np.asarray(a, dtype=dtype))


def _check(rc):
    if rc != DYNAMIX_OK:
        raise DynamixError(rc)


def dynamix_policy_weight_count(layer_sizes):
    ls = _np(layer_sizes, np.int32)
    return int(load().dynamix_policy_weight_count(ls.ctypes.data, len(ls)))


def dynamix_policy_forward(weights, layer_sizes, states):
    """Action probabilities float32[K, 5] of the shared policy for K state rows."""
    ls, w = _np(layer_sizes, np.int32), _np(weights, np.float32)
    st = _np(states, np.float32)
    if st.ndim != 2 or st.shape[1] != ls[0] or w.size != dynamix_policy_weight_count(ls):
        raise ValueError("states must be [K, layer_sizes[0]] and weights must match the layer sizes")
    probs = np.empty((st.shape[0], DYNAMIX_NUM_ACTIONS), dtype=np.float32)
    _check(int(load().dynamix_policy_forward(w.ctypes.data, ls.ctypes.data, len(ls), st.ctypes.data,
                                             st.shape[0], probs.ctypes.data)))
    return probs


def dynamix_policy_choose(probs, uniforms=None):
    p = _np(probs, np.float32)
    u = None if uniforms is None else _np(uniforms, np.float32)
    out = np.empty(p.shape[0], dtype=np.int32)
    _check(int(load().dynamix_policy_choose(p.ctypes.data, p.shape[0],
                                            None if u is None else u.ctypes.data, out.ctypes.data)))
    return out


def dynamix_batch_sizes_step(batch_sizes, actions, b_min=32, b_max=1024):
    b, a = _np(batch_sizes, np.int32), _np(actions, np.int32)
    out = np.empty_like(b)
    _check(int(load().dynamix_batch_sizes_step(b.ctypes.data, a.ctypes.data, len(b), int(b_min),
                                               int(b_max), out.ctypes.data)))
    return out


def dynamix_cycle_rewards(mean_accuracy, accuracy_gain, iteration_time, batch_sizes, alpha, beta, delta,
                          eta=0.0, sigma2_norm=0.0, sigma_norm=0.0, adaptive_optimizer=False):
    A, dA, T = (_np(x, np.float64) for x in (mean_accuracy, accuracy_gain, iteration_time))
    b = _np(batch_sizes, np.int32)
    out = np.empty(len(b), dtype=np.float64)
    _check(int(load().dynamix_cycle_rewards(A.ctypes.data, dA.ctypes.data, T.ctypes.data, b.ctypes.data,
                                            len(b), float(alpha), float(beta), float(delta), float(eta),
                                            float(sigma2_norm), float(sigma_norm),
                                            int(bool(adaptive_optimizer)), out.ctypes.data)))
    return out


def dynamix_discounted_return(rewards, gamma):
    r = _np(rewards, np.float64)
    return float(load().dynamix_discounted_return(r.ctypes.data, len(r), float(gamma)))


DYNAMIX_POLICY_RETURN_WEIGHTED, DYNAMIX_POLICY_CLIPPED = 0, 1


def dynamix_policy_update(weights, layer_sizes, states, actions, signal, lr, old_probs=None,
                          clip_eps=0.2):
    """One ascent step on n recorded decisions; returns (new weights float32, objective before the
    step).  With old_probs the clipped surrogate (signal = advantages), else the return-weighted
    log-likelihood (signal = cumulative rewards)."""
    ls = _np(layer_sizes, np.int32)
    w = _np(weights, np.float32).copy()
    st, a, sg = _np(states, np.float32), _np(actions, np.int32), _np(signal, np.float64)
    if st.ndim != 2 or st.shape[1] != ls[0] or len(a) != st.shape[0] or len(sg) != st.shape[0] \
            or w.size != dynamix_policy_weight_count(ls):
        raise ValueError("states [n, layer_sizes[0]], actions [n], signal [n] and matching weights")
    op = None if old_probs is None else _np(old_probs, np.float32)
    obj = ctypes.c_double()
    _check(int(load().dynamix_policy_update(
        w.ctypes.data, ls.ctypes.data, len(ls), st.ctypes.data, a.ctypes.data, sg.ctypes.data,
        None if op is None else op.ctypes.data, st.shape[0],
        DYNAMIX_POLICY_RETURN_WEIGHTED if op is None else DYNAMIX_POLICY_CLIPPED, float(clip_eps),
        float(lr), ctypes.byref(obj))))
    return w, obj.value
