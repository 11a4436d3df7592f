"""Parity criteria shared by the GPU tests (kept apart from the oracle: this is the
judging logic, not an implementation of the layer).

Bars (stated in the tests that call these):
  * int32 accumulators: bit-exact on identical codes.
  * activation codes: bit-exact, except elements whose exact rotated value lies
    within one fp32 ulp of the row maximum (in code units: qmax * 2^-23) of a
    rounding boundary -- widened by the row's own scale difference, which is
    itself limited to 2 fp32 ulps -- each off by exactly 1, and at most
    ceil(1e-5 * elements) of them.  Only where a caller asks for it
    (allow_fp32_ties=True: the sweeps over tiny rotation blocks and random shapes,
    never a task workload) values that sit within half an fp32 ulp OF THEMSELVES
    (2^-24 * max(1, |t|) in code units) of the boundary -- ties at the resolution
    of any fp32 evaluation, which bf16 inputs rotated over blocks of 1 to 8
    channels produce in clusters (the same few input values recur along a row)
    -- are checked like every other flip but not counted against the budget.
  * token scales: within 2 fp32 ulps.
  * bf16 outputs on identical accumulators and scales: within 1 bf16 ulp
    everywhere, max relative error <= 1e-2, mean relative error <= 1e-3.  With a
    bias the kernel's fp32 product (three roundings, relative 2^-22 at most) is
    added to a number of similar size; where the two nearly cancel the result's
    own ulp shrinks below that error, so there the bar is absolute:
    |y - y_ref| <= 2^-21 * |bias|.
"""
import math

import numpy as np

import dvdq_inputs as di


def ulp_diff_f32(a, b):
    ia = np.ascontiguousarray(a, dtype=np.float32).view(np.int32).astype(np.int64)
    ib = np.ascontiguousarray(b, dtype=np.float32).view(np.int32).astype(np.int64)
    return np.abs(ia - ib)        # inputs here are non-negative scales: bit patterns are ordered


def check_codes_and_scales(codes_gpu, scale_gpu, codes_ref, scale_ref, xrot_ref, act_bits, label="",
                           allow_fp32_ties=False):
    """Returns a dict of counters; raises AssertionError on any violation."""
    qmax = 2 ** (act_bits - 1) - 1
    d_ulp = ulp_diff_f32(scale_gpu, scale_ref)
    assert d_ulp.max(initial=0) <= 2, f"{label}: token scale off by {d_ulp.max()} fp32 ulps (bar: 2)"
    zero = scale_ref == 0
    assert np.array_equal(scale_gpu[zero], scale_ref[zero]), f"{label}: zero rows must give scale 0"
    mism = codes_gpu != codes_ref
    n_mis = int(mism.sum())
    budget = math.ceil(1e-5 * codes_ref.size)
    out = dict(elements=int(codes_ref.size), mismatches=n_mis, budget=budget,
               max_scale_ulp=int(d_ulp.max(initial=0)), max_boundary_dist_ulps=0.0)
    if n_mis == 0:
        return out
    rows, cols = np.nonzero(mism)
    g = codes_gpu[rows, cols].astype(np.int64)
    r = codes_ref[rows, cols].astype(np.int64)
    assert np.all(np.abs(g - r) == 1), f"{label}: a code differs by more than 1"
    t = xrot_ref[rows, cols] / scale_ref[rows].astype(np.float64)     # exact value in code units
    boundary = np.minimum(g, r) + 0.5
    dist = np.abs(t - boundary)
    unit = qmax * 2.0 ** -23                                          # one fp32 ulp of the row maximum
    tol = unit * (1.0 + d_ulp[rows])
    out["max_boundary_dist_ulps"] = float((dist / unit).max())
    bad = dist > tol
    assert not bad.any(), (f"{label}: {int(bad.sum())} code mismatches are not within one fp32 ulp of a rounding "
                           f"boundary (worst {float((dist / unit).max()):.3f} ulps)")
    fp32_ties = dist <= 2.0 ** -24 * np.maximum(1.0, np.abs(t))
    out["fp32_ties"] = int(fp32_ties.sum())
    counted = n_mis - (out["fp32_ties"] if allow_fp32_ties else 0)
    assert counted <= budget, f"{label}: {counted} boundary flips exceed the budget of {budget}"
    return out


def bf16_ulp_distance(a_bits, b_bits):
    """Distance in bf16 ulps between two arrays of bf16 bit patterns (sign-magnitude aware)."""
    def key(u):
        u = np.ascontiguousarray(u, dtype=np.uint16).astype(np.int32)
        return np.where(u & 0x8000, -(u & 0x7FFF), u & 0x7FFF)
    return np.abs(key(a_bits) - key(b_bits))


def check_y(y_gpu_bits, y_ref_bits, label="", bias_bits=None):
    """bf16 outputs computed from identical accumulators and scales (bias_bits: the layer's bias, if any)."""
    d = bf16_ulp_distance(y_gpu_bits, y_ref_bits)
    yg = di.bf16_bits_to_f32(y_gpu_bits).astype(np.float64)
    yr = di.bf16_bits_to_f32(y_ref_bits).astype(np.float64)
    far = d > 1
    if bias_bits is not None and far.any():
        b = np.abs(di.bf16_bits_to_f32(bias_bits).astype(np.float64))[None, :]
        cancel = np.abs(yg - yr) <= 2.0 ** -21 * np.broadcast_to(b, yr.shape)
        assert int((far & cancel).sum()) <= max(4, int(1e-4 * d.size)), f"{label}: too many cancellation cases"
        far = far & ~cancel
    assert not far.any(), f"{label}: output differs by {d[far].max()} bf16 ulps (bar: 1)"
    rho = np.sqrt((yr ** 2).mean(axis=1, keepdims=True))              # floor for outputs near zero
    rel = np.abs(yg - yr) / np.maximum(np.abs(yr), np.maximum(rho, 1e-30))
    assert rel.max(initial=0) <= 1e-2, f"{label}: max relative error {rel.max():.3e} > 1e-2"
    assert rel.mean() <= 1e-3, f"{label}: mean relative error {rel.mean():.3e} > 1e-3"
    return dict(max_rel=float(rel.max(initial=0)), mean_rel=float(rel.mean()), ulp1=int((d == 1).sum()))


def check_blockwise(values_gpu, scale_gpu, values_ref, scale_ref, exps_ref, xrot_ref, act_bits, group, label="",
                    allow_fp32_ties=False):
    """Block-wise scaled quantizer: stored int8 values against the oracle's.

    Bars: handed-on token scales within 2 fp32 ulps.  A group whose stored values differ from the
    oracle's is either (a) on the oracle's exponent, with code flips judged as in
    check_codes_and_scales -- the tolerance, one fp32 ulp of the ROW maximum, is 2^e times larger in
    the code units of a group that is quantized 2^e times finer -- or (b) one exponent off, which is
    only accepted when the group maximum times a power of two is within 2^-20 of the row maximum
    (the comparison that chooses the exponent is taken on fp32 butterfly sums by the kernel and on
    exact values by the oracle); such a group must still be a valid quantization on its own step.
    Budgets: ceil(1e-5 * elements) code flips (with allow_fp32_ties, as in check_codes_and_scales, values
    within half an fp32 ulp of themselves of a boundary are checked but not counted: unrotated bf16 inputs
    produce such exact ties in clusters), ceil(1e-4 * groups) exponent flips."""
    qmax = 2 ** (act_bits - 1) - 1
    emax = 8 - act_bits
    M, K = values_ref.shape
    G = K // group
    d_ulp = ulp_diff_f32(scale_gpu, scale_ref)
    assert d_ulp.max(initial=0) <= 2, f"{label}: token scale off by {d_ulp.max()} fp32 ulps (bar: 2)"
    vg = values_gpu.astype(np.int64).reshape(M, G, group)
    vr = values_ref.astype(np.int64).reshape(M, G, group)
    xr = xrot_ref.reshape(M, G, group)
    e = exps_ref.astype(np.int64)
    s_tok = scale_ref.astype(np.float64) * 2.0 ** emax                  # s_m
    out = dict(elements=int(values_ref.size), groups=int(M * G), code_flips=0, exp_flips=0, max_boundary_dist_ulps=0.0)
    differing = np.argwhere(np.any(vg != vr, axis=2))
    amax_row = np.abs(xrot_ref).max(axis=1)
    for m, g in differing:
        sh = emax - e[m, g]
        same_exp = np.all(vg[m, g] % (1 << sh) == 0) and np.abs(vg[m, g] >> sh).max() <= qmax
        if same_exp:
            qg, qr = vg[m, g] >> sh, vr[m, g] >> sh
            idx = np.nonzero(qg != qr)[0]
            assert np.all(np.abs(qg[idx] - qr[idx]) == 1), f"{label}: a code differs by more than 1"
            t = xr[m, g, idx] / (s_tok[m] * 2.0 ** -e[m, g])
            dist = np.abs(t - (np.minimum(qg[idx], qr[idx]) + 0.5))
            unit = qmax * 2.0 ** -23 * 2.0 ** e[m, g]
            assert np.all(dist <= unit * (1.0 + d_ulp[m])), f"{label}: code flip {dist.max() / unit:.3f} ulps from its boundary"
            ties = dist <= 2.0 ** -24 * np.maximum(1.0, np.abs(t))      # ties at fp32 resolution: checked, not counted
            out["fp32_ties"] = out.get("fp32_ties", 0) + int(ties.sum())
            out["code_flips"] += int(idx.size - (ties.sum() if allow_fp32_ties else 0))
            out["max_boundary_dist_ulps"] = max(out["max_boundary_dist_ulps"], float(dist.max() / unit))
        else:
            a = np.abs(xr[m, g]).max()
            near = min(abs(a * 2.0 ** t / amax_row[m] - 1.0) for t in (e[m, g], e[m, g] + 1))
            assert near <= 2.0 ** -20, f"{label}: group ({m},{g}) is on another exponent away from a boundary ({near:.3e})"
            ok = False
            for e_alt in (e[m, g] - 1, e[m, g] + 1):
                if 0 <= e_alt <= emax and np.all(vg[m, g] % (1 << (emax - e_alt)) == 0):
                    step = s_tok[m] * 2.0 ** -e_alt
                    q = vg[m, g] >> (emax - e_alt)
                    ok = ok or (np.abs(q).max() <= qmax and np.all(np.abs(xr[m, g] - q * step) <= step / 2 * (1 + 1e-5)))
            assert ok, f"{label}: group ({m},{g}) is not a valid quantization on a neighbouring exponent"
            out["exp_flips"] += 1
    assert out["code_flips"] <= math.ceil(1e-5 * values_ref.size), f"{label}: {out['code_flips']} code flips"
    assert out["exp_flips"] <= math.ceil(1e-4 * M * G), f"{label}: {out['exp_flips']} exponent flips"
    return out
