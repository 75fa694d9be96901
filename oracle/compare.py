"""Acceptance rules used when a GPU result is compared with the CPU checker.
Test infrastructure only.

Two rules, both element by element on |double(gpu) - ref|:

* pointwise (elementwise / reduction outputs): pass iff
      |g - o| <= rtol * max(|o|, floor_frac * rms(o)),   rtol = 1e-4,
  rms taken over the whole reference tensor.  A bare relative error is
  undefined where the true output is ~0 (layernorm at x ~ mu, GELU's negative
  tail), hence the floor at 1e-2 of the tensor's rms.
* contraction (fp32 matmul / conv / attention outputs): with
  o = b0 + sum_t a_t b_t and Dn = |b0| + sum_t |a_t| |b_t|, pass iff
      |g - o| <= tol * Dn,   tol = 2e-3.
  ReLU is 1-Lipschitz, so the same bound holds after it.
"""
from __future__ import annotations

import numpy as np

RTOL_POINTWISE = 1e-4
FLOOR_FRAC = 1e-2
TOL_CONTRACTION = 2e-3


class Verdict:
    def __init__(self, ok, worst, index, bare_rel):
        self.ok = bool(ok)          # every element inside its bound
        self.worst = float(worst)   # max over elements of err / bound  (<= 1 passes)
        self.index = index          # where that maximum is
        self.bare_rel = float(bare_rel)  # information only: max |g-o| / |o|

    def __bool__(self):
        return self.ok

    def __repr__(self):
        return "Verdict(ok=%s, worst err/bound=%.3g at %s, bare max rel=%.3g)" % (
            self.ok, self.worst, self.index, self.bare_rel)


def _finish(err, bound, ref):
    if err.size == 0:
        return Verdict(True, 0.0, None, 0.0)
    finite = np.isfinite(err).all()
    with np.errstate(divide="ignore", invalid="ignore"):
        ratio = np.where(bound > 0, err / bound, np.where(err == 0, 0.0, np.inf))
        bare = np.where(ref != 0, err / np.abs(ref), 0.0)
    k = int(np.argmax(ratio))
    idx = np.unravel_index(k, ratio.shape)
    worst = ratio.flat[k]
    return Verdict(finite and worst <= 1.0, worst, idx, np.max(bare))


def pointwise(gpu, ref, rtol=RTOL_POINTWISE, floor_frac=FLOOR_FRAC) -> Verdict:
    g = np.asarray(gpu, dtype=np.float64)
    o = np.asarray(ref, dtype=np.float64)
    assert g.shape == o.shape, (g.shape, o.shape)
    if o.size == 0:
        return Verdict(True, 0.0, None, 0.0)
    rms = float(np.sqrt(np.mean(o * o)))
    bound = rtol * np.maximum(np.abs(o), floor_frac * rms)
    return _finish(np.abs(g - o), bound, o)


def contraction(gpu, ref, Dn, tol=TOL_CONTRACTION) -> Verdict:
    g = np.asarray(gpu, dtype=np.float64)
    o = np.asarray(ref, dtype=np.float64)
    d = np.asarray(Dn, dtype=np.float64)
    assert g.shape == o.shape == d.shape, (g.shape, o.shape, d.shape)
    return _finish(np.abs(g - o), tol * d, o)
