"""Comparison of the HIP path's outputs with the CPU oracle's, to the stated tolerances.

Tolerances (relative): 1e-5 for the aggregate vector and the squared norms with fp32 inputs,
1e-3 with bf16 inputs, 1e-4 for the noise scale whatever the input type.

A vector is compared in the 2-norm and in the max-norm relative to the oracle's largest entry,
because single entries of a weighted mean can cancel to almost nothing.

The sums A, n_k, d_k, T of a record meet the plain relative tolerance whenever the record is
well conditioned: it covers at least 4096 elements (no single cancelling entry can dominate) and
the workers are not identical to within rounding (d_k >= 1e-6 max(n_k, A)).  Otherwise the bound
adds what the fp32 evaluation of G_i = sum_k w_k g_ki (K fused multiply-adds with weights rounded
once) can contribute: |dG_i| <= eps_c sqrt(sum_k w_k g_ki^2) with eps_c = K 2^-23, hence
|dA| <= 2 eps_c sqrt(A N) + eps_c^2 N with N = sum_k w_k n_k, and
|dd_k| <= 2 eps_c sqrt(d_k M) + eps_c^2 M with M = max(n_k, A).  Ratios inherit the relative
bounds of their parts; A - T/B is compared against the size of its two parts.
"""
import numpy as np

HEAD = 8


def tolerances(is_bf16):
    return (1e-3, 1e-4) if is_bf16 else (1e-5, 1e-4)


def compare(agg_gpu, stats_gpu, agg_ref, stats_ref, batch_sizes, is_bf16=False, where=""):
    tol, tol_ns = tolerances(is_bf16)
    K = len(batch_sizes)
    B = float(np.sum(batch_sizes))
    stats_gpu = np.asarray(stats_gpu, dtype=np.float64)
    assert stats_gpu.shape == stats_ref.shape, where
    if agg_gpu is not None:
        a = np.asarray(agg_gpu, dtype=np.float64)
        assert a.shape == agg_ref.shape
        den = float(np.linalg.norm(agg_ref))
        diff = a - agg_ref
        if den > 0:
            assert np.linalg.norm(diff) <= tol * den, (where, "agg 2-norm", np.linalg.norm(diff) / den)
            assert np.abs(diff).max() <= tol * np.abs(agg_ref).max(), (where, "agg max-norm")
        else:
            assert not diff.any()
    for r in range(stats_ref.shape[0]):
        g, o = stats_gpu[r], stats_ref[r]
        tag = "%s record %d" % (where, r)
        A, T = o[0], o[1]
        n, d = o[HEAD:HEAD + K], o[HEAD + K:HEAD + 2 * K]
        assert g[7] == o[7], tag
        if not np.isfinite(o[:7]).all() or not np.isfinite(o[HEAD:]).all():
            # degenerate record (e.g. all-zero gradients): same non-finite pattern, same finite values
            assert (np.isnan(g) == np.isnan(o)).all(), tag
            fin = np.isfinite(o)
            np.testing.assert_allclose(g[fin], o[fin], rtol=tol_ns, atol=0, err_msg=tag)
            continue
        w = np.asarray(batch_sizes, dtype=np.float64) / B
        eps_c = K * 2.0 ** -23
        big = o[7] >= 4096
        N = float(np.dot(w, n))
        bound_A = tol * A + (0.0 if big else 2 * eps_c * np.sqrt(A * N) + eps_c ** 2 * N)
        assert abs(g[0] - A) <= bound_A, (tag, "A", g[0], A)
        gn, gd = g[HEAD:HEAD + K], g[HEAD + K:HEAD + 2 * K]
        assert (np.abs(gn - n) <= tol * n).all(), (tag, "n_k")
        M = np.maximum(n, A)
        well = big & (d >= 1e-6 * M)
        bound_d = tol * d + np.where(well, 0.0, 2 * eps_c * np.sqrt(d * M) + eps_c ** 2 * M)
        assert (np.abs(gd - d) <= bound_d).all(), (tag, "d_k", gd, d)
        bound_T = float(np.dot(batch_sizes, bound_d)) / max(K - 1, 1)
        assert abs(g[1] - T) <= bound_T, (tag, "T", g[1], T)
        part = abs(A) + abs(T) / B
        bound_U = bound_A + bound_T / B
        assert abs(g[2] - o[2]) <= bound_U + tol * part, (tag, "A_unb", g[2], o[2])
        if K > 1:
            # the ratios are checked where they mean something: T is not a rounding residue,
            # and for the unbiased noise scale A - T/B has not cancelled
            if T > 1e-6 * B * A and A > 0:
                slack = (bound_A - tol * A) / A + (bound_T - tol * T) / T
                assert abs(g[4] - o[4]) <= (tol_ns + slack) * abs(o[4]), (tag, "noise_scale_biased", g[4], o[4])
                assert abs(g[5] - o[5]) <= (tol_ns + slack) * abs(o[5]), (tag, "sigma2_norm")
                assert abs(g[6] - o[6]) <= (tol_ns + slack) * abs(o[6]), (tag, "sigma_norm")
                if abs(o[2]) > 0.05 * part:
                    slack_u = (bound_U - tol * part) / abs(o[2]) + (bound_T - tol * T) / T
                    assert abs(g[3] - o[3]) <= (tol_ns + slack_u) * abs(o[3]), (tag, "noise_scale", g[3], o[3])
        else:
            assert g[1] == 0.0 and g[3] == 0.0 and g[4] == 0.0 and g[6] == 0.0, tag


def compare_sgd(got, ref, p0, agg_ref, lr, is_bf16=False, where=""):
    """Updated parameters of the fused SGD step against the oracle's: the fp32 evaluation of
    p - lr (G + wd p) adds two roundings to the aggregate's own error."""
    tol = 1e-3 if is_bf16 else 1e-5
    got = np.asarray(got, dtype=np.float64)
    scale = np.abs(np.asarray(p0, dtype=np.float64)) + abs(lr) * np.abs(agg_ref)
    assert np.linalg.norm(got - ref) <= tol * np.linalg.norm(ref), where
    assert (np.abs(got - ref) <= 4e-7 * scale + tol * abs(lr) * np.abs(agg_ref).max()).all(), where


EPS32 = 2.0 ** -24      # unit roundoff of fp32


def aggregate_error_bound(host_grads, batch_sizes, widen):
    """Element-wise bound on the error of the fp32 aggregate: K fused multiply-adds in worker
    order with weights rounded once give |dG_i| <= (K + 2) 2^-24 sum_k w_k |g_ki|.  host_grads are
    the stored inputs, `widen` turns one of them into float64."""
    K = len(host_grads)
    w = np.asarray(batch_sizes, dtype=np.float64) / float(np.sum(batch_sizes))
    s = np.zeros(len(host_grads[0]), dtype=np.float64)
    for k in range(K):
        s += w[k] * np.abs(widen(host_grads[k]))
    return (K + 2) * EPS32 * s


def compare_momentum(got_p, got_b, ref_p, ref_b, p0, b0, agg_ref, dg, lr, wd, mu, nesterov,
                     is_bf16=False, where=""):
    """Fused SGD-with-momentum step against the oracle's.  dg: element-wise error bound of the
    aggregate.  The buffer is two fp32 fused multiply-adds on top of G, the parameter one or two
    more; each rounds at most half an ulp of its result, bounded here by the sum of the magnitudes
    of its operands."""
    tol = 1e-3 if is_bf16 else 1e-5
    p0, b0 = np.asarray(p0, dtype=np.float64), np.asarray(b0, dtype=np.float64)
    got_p, got_b = np.asarray(got_p, dtype=np.float64), np.asarray(got_b, dtype=np.float64)
    g_mag = np.abs(agg_ref) + abs(wd) * np.abs(p0)
    b_mag = abs(mu) * np.abs(b0) + g_mag
    bound_b = 3 * EPS32 * b_mag + dg
    assert (np.abs(got_b - ref_b) <= bound_b).all(), (where, "momentum buffer")
    assert np.linalg.norm(got_b - ref_b) <= tol * np.linalg.norm(ref_b), (where, "buffer 2-norm")
    step_mag = (g_mag + abs(mu) * b_mag) if nesterov else b_mag
    amp = (1 + abs(mu)) if nesterov else 1.0
    bound_p = 2 * EPS32 * (np.abs(p0) + abs(lr) * step_mag) + abs(lr) * (amp * bound_b + 2 * EPS32 * step_mag)
    assert (np.abs(got_p - ref_p) <= bound_p).all(), (where, "parameters")
    assert np.linalg.norm(got_p - ref_p) <= tol * np.linalg.norm(ref_p), (where, "parameters 2-norm")


def compare_adam(got, ref, p0, m0, v0, agg_ref, dg, lr, beta1, beta2, eps, wd, decoupled, step,
                 is_bf16=False, where=""):
    """Fused Adam step against the oracle's.  got, ref: (params, exp_avg, exp_avg_sq).  With
    g' the gradient after L2 decay, D = sqrt(v' / (1 - beta2^t)) + eps and s = lr / (1 - beta1^t),
    an error dg in g' moves m' by (1 - beta1) dg, v' by at most 2 (1 - beta2) |g'| dg + (1 - beta2) dg^2,
    its root by at most sqrt(1 - beta2) dg, and the update s m' / D by at most
    s dg ((1 - beta1) / D + |m'| sqrt((1 - beta2) / (1 - beta2^t)) / D^2); on top come the roundings
    of the fp32 operations themselves (a handful of half-ulps of each result)."""
    tol = 1e-3 if is_bf16 else 1e-5
    p0, m0, v0 = (np.asarray(x, dtype=np.float64) for x in (p0, m0, v0))
    gp, gm, gv = (np.asarray(x, dtype=np.float64) for x in got)
    rp, rm, rv = ref
    c1, c2 = 1.0 - beta1 ** step, 1.0 - beta2 ** step
    s = lr / c1
    g = agg_ref if decoupled else agg_ref + wd * p0
    dg = dg + 2 * EPS32 * (np.abs(agg_ref) + abs(wd) * np.abs(p0))
    bound_m = 3 * EPS32 * (beta1 * np.abs(m0) + (1 - beta1) * np.abs(g)) + (1 - beta1) * dg
    assert (np.abs(gm - rm) <= bound_m).all(), (where, "exp_avg")
    bound_v = 4 * EPS32 * rv + (1 - beta2) * (2 * np.abs(g) * dg + dg * dg)
    assert (np.abs(gv - rv) <= bound_v).all(), (where, "exp_avg_sq")
    D = np.sqrt(rv / c2) + eps
    upd = s * np.abs(rm) / D
    droot = np.sqrt(1 - beta2) * dg + 3 * EPS32 * np.sqrt(rv)       # error of sqrt(v')
    bound_u = 8 * EPS32 * upd + s * (bound_m / D + np.abs(rm) * droot / np.sqrt(c2) / (D * D))
    bound_p = 3 * EPS32 * (np.abs(p0) + upd) + bound_u
    assert (np.abs(gp - rp) <= bound_p).all(), (where, "parameters",
                                                 float(np.max(np.abs(gp - rp) / bound_p)))
    assert np.linalg.norm(gm - rm) <= tol * np.linalg.norm(rm), (where, "exp_avg 2-norm")
    assert np.linalg.norm(gv - rv) <= tol * np.linalg.norm(rv), (where, "exp_avg_sq 2-norm")
    assert np.linalg.norm(gp - rp) <= tol * np.linalg.norm(rp), (where, "parameters 2-norm")
