"""Comparison rule between a GPU result and the oracle (test infrastructure).

Floating point: pass iff for every element |g - r| <= rtol * max(|r|, rho),
rho = RMS of the oracle's output tensor (the floor keeps "relative" error
meaningful for outputs near zero).  rtol = 1e-5 for fp32 operators, 2e-2 for
fp16/bf16 inputs with fp32 accumulation.  Integer: bit-exact.
"""
import numpy as np

RTOL_F32 = 1e-5
RTOL_HALF = 2e-2
# 8-bit float inputs (4 exponent, 3 mantissa bits) with fp32 output.  The products are exact in 8 significant bits; what
# the tolerance has to cover is how one matrix-core instruction adds its n = 16 ... 128 products: the public
# instruction-set text fixes the fp32 result format, not the width of that block adder.  Model: the adder aligns the n
# products to the largest of them and keeps w bits below its leading bit, so a block is off by at most n * 2^-w times
# its largest product.  With N(0, 1) inputs the largest product of a block is about 9 sigma^2, the K / n block errors
# add like a random walk, and the output RMS is sqrt(K) sigma^2: relative error about 9 * sqrt(n) * 2^-w, i.e.
# 4e-4 for w = 18 and n = 128.  1e-3 therefore holds for any adder that keeps at least 18 bits (fp32 itself keeps
# 24) and fails a narrower one (w = 16: 1.6e-3); integer-valued 8-bit floats, whose sums are exact at any such width,
# are compared bit for bit in the same tests.
RTOL_F8 = 1e-3


def float_report(got, ref, rtol):
    g = np.asarray(got, np.float64).reshape(-1)
    r = np.asarray(ref, np.float64).reshape(-1)
    assert g.shape == r.shape, (g.shape, r.shape)
    rho = float(np.sqrt(np.mean(r * r))) if r.size else 0.0
    denom = np.maximum(np.abs(r), rho)
    err = np.abs(g - r)
    with np.errstate(divide="ignore", invalid="ignore"):
        rel = np.where(denom > 0, err / denom, np.where(err == 0, 0.0, np.inf))
    worst = int(np.argmax(rel)) if rel.size else -1
    ok = bool(np.all(np.isfinite(g))) and bool(np.all(rel <= rtol))
    return {"ok": ok, "max_rel": float(rel.max()) if rel.size else 0.0, "rho": rho, "worst": worst,
            "got": float(g[worst]) if rel.size else 0.0, "ref": float(r[worst]) if rel.size else 0.0}


def assert_float_close(got, ref, rtol, what=""):
    rep = float_report(got, ref, rtol)
    assert rep["ok"], "%s: max rel err %.3e > %.1e at flat index %d (got %r, oracle %r, rms %.3e)" % (
        what, rep["max_rel"], rtol, rep["worst"], rep["got"], rep["ref"], rep["rho"])
    return rep


def assert_int_equal(got, ref, what=""):
    g = np.asarray(got)
    r = np.asarray(ref)
    assert g.shape == r.shape and g.dtype == r.dtype, (g.shape, r.shape, g.dtype, r.dtype)
    bad = np.flatnonzero(g.reshape(-1) != r.reshape(-1))
    assert bad.size == 0, "%s: %d mismatches, first at %d (got %d, oracle %d)" % (
        what, bad.size, bad[0], g.reshape(-1)[bad[0]], r.reshape(-1)[bad[0]])
