"""Acceptance rule for end-to-end results of DEEP bf16 stages, where element-wise agreement to 2e-2
between two correct implementations is not attainable (a one-ulp difference in a stored activation
flips ReLU gates / pool arg-max choices further down, and flips compound with depth).

Both the oracle in storage="bf16" mode and the implementation under test compute the same exact
function with bf16 rounding at the same points; the oracle in storage="exact" mode computes that
function without rounding.  How far bf16 storage moves a tensor, e_ref = ||oracle_bf16 - exact|| /
||exact||, is the natural unit: a correct implementation lands about as far from the exact result
as the bf16 oracle does, whatever its summation order, and a wrong one (dropped term, wrong sign or
index, stale operand) lands O(1) away.  The rule, per tensor:

    ||impl - exact|| <= FACTOR * ||oracle_bf16 - exact|| + FLOOR * ||exact||        (L2 norms)

and the share of elements whose error exceeds the element-wise tolerance is bounded the same way.
tests/test_flip_bound.py checks the rule on the CPU: a second correct implementation (fp32 PyTorch
ops) passes it, planted mistakes fail it."""
import numpy as np

FACTOR = 1.5
FLOOR = 2e-3          # tensors that bf16 storage hardly moves (fp32 sums of thousands of terms)


def l2(a, ref):
    a, ref = np.asarray(a, np.float64), np.asarray(ref, np.float64)
    return float(np.linalg.norm((a - ref).ravel()) / max(np.linalg.norm(ref.ravel()), 1e-300))


def off_fraction(a, ref, tol):
    """share of elements further than tol * max|ref| from ref"""
    a, ref = np.asarray(a, np.float64), np.asarray(ref, np.float64)
    return float(np.mean(np.abs(a - ref) > tol * max(float(np.max(np.abs(ref))), 1e-300)))


def check(name, impl, oracle_bf16, exact, tol=2e-2):
    """Returns (ok, record); record holds the figures for the log."""
    e_impl, e_ref, e_pair = l2(impl, exact), l2(oracle_bf16, exact), l2(impl, oracle_bf16)
    f_impl, f_ref = off_fraction(impl, exact, tol), off_fraction(oracle_bf16, exact, tol)
    ok = bool(np.all(np.isfinite(np.asarray(impl, np.float64)))) and e_impl <= FACTOR * e_ref + FLOOR and \
        f_impl <= FACTOR * f_ref + 1e-3
    return ok, dict(name=name, e_impl=e_impl, e_ref=e_ref, e_pair=e_pair, f_impl=f_impl, f_ref=f_ref)


def fmt(r):
    return "%-8s |impl-exact| %.3e  |bf16-exact| %.3e  |impl-bf16| %.3e   off>tol: impl %.2e  bf16 %.2e" % (
        r["name"], r["e_impl"], r["e_ref"], r["e_pair"], r["f_impl"], r["f_ref"])
