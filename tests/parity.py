"""Error measures of the GPU parity tests, stated once.

nmax: the bar of the workload description, max|g - r| / max|r| per output tensor (1e-4 fp32,
2e-2 fp16 / bf16 against the fp32 oracle).  That measure alone lets an element far below the
tensor's maximum be wrong by many times its own size, so every check also counts the elements
with |g - r| <= rtol * |r| + rtol * rms(r) (same rtol): all of them must pass in fp32.  In the
16-bit types the roundings of the weights and of every stored activation count as error and a
whole network's logits sit at half the bar already, so there the pass rate must stay above
MIN_RATE and no element may miss by more than WORST_FACTOR times the bound.  Failure messages
carry all figures."""
import numpy as np

RTOL = {0: 1e-4, 1: 2e-2, 2: 2e-2}          # by cprune_dtype: fp32, fp16, bf16
MIN_RATE = {0: 1.0, 1: 0.9, 2: 0.9}
WORST_FACTOR = {0: 1.0, 1: 3.0, 2: 3.0}


def nmax(g, r):
    g = np.asarray(g, dtype=np.float64)
    r = np.asarray(r, dtype=np.float64)
    assert g.shape == r.shape, (g.shape, r.shape)
    return float(np.max(np.abs(g - r)) / max(np.max(np.abs(r)), 1e-30))


def elementwise(g, r, rtol):
    """-> (fraction of elements with |g - r| <= rtol |r| + rtol rms(r), largest |g - r| / (|r| + rms(r)))."""
    g = np.asarray(g, dtype=np.float64)
    r = np.asarray(r, dtype=np.float64)
    rms = float(np.sqrt(np.mean(r * r)))
    d = np.abs(g - r)
    bound = np.abs(r) + max(rms, 1e-30)
    return float(np.mean(d <= rtol * bound)), float(np.max(d / bound))


def check(g, r, dtype, what=""):
    """Asserts both measures; returns (nmax, elementwise pass rate)."""
    e = nmax(g, r)
    rate, worst = elementwise(g, r, RTOL[dtype])
    msg = f"{what}: nmax {e:.3e} (bar {RTOL[dtype]:g}), element-wise pass rate {rate:.6f} " \
          f"(bar {MIN_RATE[dtype]:g}), worst element {worst:.3e} of |r| + rms(r)"
    assert e < RTOL[dtype], msg
    assert rate >= MIN_RATE[dtype], msg
    assert worst <= WORST_FACTOR[dtype] * RTOL[dtype], msg
    return e, rate
