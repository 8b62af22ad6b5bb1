"""Error measures of the GPU-vs-oracle parity tests.

Two forms are computed for every compared tensor and listed at the end of a pytest run:
  max form      max_i |g_i - o_i| / max_j |o_j|                      (the bound the task states: 1e-5 fp32, 2e-2 bf16)
  element form  max_i |g_i - o_i| / max(|o_i|, rms(o))               (element-wise, with an absolute floor of tol * rms(o))
The element form is never smaller than the max form, so a test that asserts it asserts both.
"""
import numpy as np

RECORDS = []          # (test id, max form, element form, elements)
_current = ["?"]


def set_current(nodeid):
    _current[0] = nodeid


def both(got, want):
    got = np.asarray(got, np.float64)
    want = np.asarray(want, np.float64)
    assert got.shape == want.shape, (got.shape, want.shape)
    if want.size == 0:
        return 0.0, 0.0
    d = np.abs(got - want)
    if not np.all(np.isfinite(d)):
        return float("inf"), float("inf")
    top = max(float(np.max(np.abs(want))), 1e-30)
    rms = max(float(np.sqrt(np.mean(want * want))), 1e-30)
    e_max = float(np.max(d)) / top
    e_elem = float(np.max(d / np.maximum(np.abs(want), rms)))
    RECORDS.append((_current[0], e_max, e_elem, int(want.size)))
    return e_max, e_elem


def relerr(got, want):
    """Element form (the stricter of the two); both forms are recorded for the summary."""
    return both(got, want)[1]


def relerr_max(got, want):
    return both(got, want)[0]


def summary_lines():
    worst = {}
    for node, e1, e2, n in RECORDS:
        w = worst.setdefault(node, [0.0, 0.0, 0, 0])
        w[0] = max(w[0], e1)
        w[1] = max(w[1], e2)
        w[2] += 1
        w[3] += n
    lines = ["parity error per test: worst max-form | worst element-form | tensors compared | elements"]
    for node, (e1, e2, k, n) in worst.items():
        lines.append(f"  {e1:9.3e} | {e2:9.3e} | {k:5d} | {n:10d} | {node}")
    return lines
