"""Shared pieces of the GPU parity tests: tolerances, oracle/GPU adapters."""
import math

import numpy as np

import oracle
from paper_2602_11812_amd import workloads as wl

# Tolerances of the parity bar: entropy absolute (nats), pooled relative L2, prediction relative
TOL_ENTROPY_ABS = 1e-3
TOL_POOLED_REL_L2 = 2e-3
TOL_PRED_REL = 1e-2
TOL_LSE_ABS = 1e-3


def oracle_head(w: "wl.Workload", b1=None, b2=None, bin_centers=None, w2=None):
    return oracle.Head(w.w1, w.w2 if w2 is None else w2, b1, b2, bin_centers)


def rel_l2(a, b):
    a = np.asarray(a, dtype=np.float64)
    b = np.asarray(b, dtype=np.float64)
    den = np.linalg.norm(b)
    return float(np.linalg.norm(a - b) / den) if den > 0 else float(np.linalg.norm(a - b))


# Predictions of a random zero-mean head can sit arbitrarily close to 0, where a relative error means nothing:
# below this fraction of the batch's root-mean-square prediction the bound stops shrinking.
PRED_FLOOR_FRACTION = 1e-3


def assert_pred_close(got, want, tol=TOL_PRED_REL, strict=False):
    """|got - want| <= tol * |want|, the stated bar; for predictions smaller than PRED_FLOOR_FRACTION of the
    batch's rms the bound is tol * PRED_FLOOR_FRACTION * rms instead.  strict: no floor at all (heads whose
    outputs are bounded away from zero)."""
    got = np.asarray(got, dtype=np.float64)
    want = np.asarray(want, dtype=np.float64)
    floor = 0.0 if strict or not want.size else PRED_FLOOR_FRACTION * math.sqrt(float(np.mean(want ** 2)))
    bound = tol * np.maximum(np.abs(want), floor)
    bad = np.abs(got - want) > bound + 1e-30
    assert not bad.any(), f"pred mismatch at {np.nonzero(bad)[0][:8]}: got {got[bad][:4]} want {want[bad][:4]}"


def assert_egtp_close(got: dict, want: "oracle.EgtpResult", lens=None):
    """got: dict of numpy arrays (entropy, pooled, lse, pred) from the GPU."""
    if want.entropy.size:
        err = np.abs(got["entropy"].astype(np.float64) - want.entropy)
        assert err.max() <= TOL_ENTROPY_ABS, f"entropy max abs err {err.max()} at token {err.argmax()}"
    for b in range(want.pooled.shape[0]):
        r = rel_l2(got["pooled"][b], want.pooled[b])
        assert r <= TOL_POOLED_REL_L2, f"pooled[{b}] rel L2 {r}"
    finite = np.isfinite(want.lse)
    assert np.array_equal(np.isfinite(got["lse"]), finite)
    if finite.any():
        assert np.abs(got["lse"][finite].astype(np.float64) - want.lse[finite]).max() <= TOL_LSE_ABS
    assert np.all(got["lse"][~finite] == -np.inf)
    assert_pred_close(got["pred"], want.pred)
