"""Helpers shared by the GPU parity tests (comparison rules only; no kernel or oracle arithmetic)."""
import numpy as np

REL_TOL = 1e-3  # max relative error of the fp16 outputs


def fp16_rel_err(got_f16, ref_f16, acc, x_scale, w_scale, bias_f16):
    """Relative error of fp16 outputs against the oracle's.

    The denominator is |ref|, floored where the bias cancels the product (1e-3 of the
    magnitudes that were added) and at the smallest normal fp16 (2^-14), so that a
    one-ulp difference of a cancelled or subnormal result does not count as a large error.
    """
    g = got_f16.astype(np.float64)
    r = ref_f16.astype(np.float64)
    p = np.abs(acc.astype(np.float64) * x_scale.astype(np.float64)[:, None] * w_scale.astype(np.float64)[None, :])
    b = 0.0 if bias_f16 is None else np.abs(bias_f16.astype(np.float64))[None, :]
    den = np.maximum(np.maximum(np.abs(r), 1e-3 * (p + b)), 2.0 ** -14)
    return np.abs(g - r) / den


def assert_fp16_close(got_f16, ref_f16, acc, x_scale, w_scale, bias_f16):
    assert got_f16.shape == ref_f16.shape
    fin = np.isfinite(ref_f16.astype(np.float32))
    assert np.array_equal(np.isfinite(got_f16.astype(np.float32)), fin)
    err = fp16_rel_err(got_f16, ref_f16, acc, x_scale, w_scale, bias_f16)
    worst = float(err[fin].max()) if fin.any() else 0.0
    assert worst <= REL_TOL, f"max relative error {worst:.3e} > {REL_TOL}"
    return worst


def freivalds_check(acc_i32, xq, wq, seed, rounds=3):
    """acc == xq @ wq.T checked as acc @ r == xq @ (wq.T @ r) in exact int64 arithmetic.

    A wrong entry survives one round with probability <= 1/15 (r drawn from 15 values),
    so `rounds` rounds miss it with probability <= 15^-rounds.
    """
    g = np.random.default_rng(seed)
    N = wq.shape[0]
    for _ in range(rounds):
        r = g.integers(-7, 8, N).astype(np.int64)
        lhs = acc_i32.astype(np.int64) @ r
        rhs = xq.astype(np.int64) @ (wq.astype(np.int64).T @ r)
        if not np.array_equal(lhs, rhs):
            return False
    return True
