"""Shared helpers of the GPU parity tests: oracle evaluation (cached) and the error metric."""
import numpy as np

from oracle import lstm_oracle as O
from paper_1604_01946_amd.inputs import make_inputs

FWD_TOL = 1e-4   # max-abs normalised, forward outputs (fp32)
BWD_TOL = 1e-3   # max-abs normalised, gradients

_cache = {}


def oracle_results(cfg, seed, with_states=True, with_dstates=True, backward=True):
    key = (cfg.dims, cfg.state_std, cfg.dstate_std, seed, with_states, with_dstates, backward)
    if key not in _cache:
        d = make_inputs(cfg, seed)
        h0 = d["h0"] if with_states else None
        c0 = d["c0"] if with_states else None
        y, hT, cT, res = O.lstm_forward(*cfg.dims, d["x"], h0, c0, d["W"], d["R"], d["b"])
        out = {"y": y, "hT": hT, "cT": cT}
        if backward:
            g = O.lstm_backward(*cfg.dims, d["x"], h0, c0, d["W"], d["R"], res, d["dy"],
                                d["dhT"] if with_dstates else None, d["dcT"] if with_dstates else None)
            out.update(dict(zip(("dx", "dh0", "dc0", "dW", "dR", "db"), g)))
        if len(_cache) > 6:
            _cache.pop(next(iter(_cache)))
        _cache[key] = (d, out)
    return _cache[key]


def nerr(got, ref):
    """max|got - ref| / max|ref| (absolute if the reference is identically zero)."""
    got = np.asarray(got, np.float64).reshape(-1)
    ref = np.asarray(ref, np.float64).reshape(-1)
    assert got.shape == ref.shape, (got.shape, ref.shape)
    if not np.all(np.isfinite(got)):
        return float("inf")
    den = np.max(np.abs(ref))
    return float(np.max(np.abs(got - ref)) / (den if den > 0 else 1.0))


ATOL_REPORT = 1e-6   # x max|ref|: absolute floor of the reported element-wise relative error
ATOL_ASSERT = 1e-5   # x max|ref|: absolute term of the asserted element-wise bound


def relerr(got, ref, atol=ATOL_REPORT):
    """max_i |got_i - ref_i| / (|ref_i| + atol * max|ref|): the element-wise relative error with an absolute floor.
    Reported beside the normalised error, not bounded: the rounding error of an fp32 sum is proportional to the
    magnitude of its terms, not of its result, so an element that cancels to nearly zero keeps an absolute error of
    a few 1e-6 of the tensor's scale and any relative figure for it is arbitrary."""
    got = np.asarray(got, np.float64).reshape(-1)
    ref = np.asarray(ref, np.float64).reshape(-1)
    if not np.all(np.isfinite(got)):
        return float("inf")
    den = np.max(np.abs(ref))
    den = den if den > 0 else 1.0
    return float(np.max(np.abs(got - ref) / (np.abs(ref) + atol * den)))


def mixed_excess(got, ref, rtol, atol=ATOL_ASSERT):
    """max_i |got_i - ref_i| / (rtol * |ref_i| + atol * max|ref|): at most 1 when every element is within the relative
    tolerance of its own reference value plus an absolute term of 1e-5 of the tensor's scale (ten times the rounding
    of the longest fp32 sums here, K = 6400).  Small elements are thereby held 10 to 100 times tighter than the
    normalised error holds them."""
    got = np.asarray(got, np.float64).reshape(-1)
    ref = np.asarray(ref, np.float64).reshape(-1)
    if not np.all(np.isfinite(got)):
        return float("inf")
    den = np.max(np.abs(ref))
    den = den if den > 0 else 1.0
    return float(np.max(np.abs(got - ref) / (rtol * np.abs(ref) + atol * den)))


last_relerr = {}   # name -> element-wise relative error of the most recent assert_close (printed by the tests)


def assert_close(got, ref, names, tol, tag=""):
    errs = {k: nerr(got[k], ref[k]) for k in names}
    bad = {k: v for k, v in errs.items() if not v <= tol}
    assert not bad, f"{tag} normalised errors above {tol}: {bad} (all: {errs})"
    mixed = {k: mixed_excess(got[k], ref[k], tol) for k in names}
    bad = {k: v for k, v in mixed.items() if not v <= 1.0}
    assert not bad, f"{tag} elements outside {tol} * |ref_i| + {ATOL_ASSERT} * max|ref| (ratio to that bound): {bad}"
    for k in names:
        last_relerr[k] = relerr(got[k], ref[k])
    return errs
