"""Shared machinery of the GPU parity tests: run the CPU oracle on the same tensors the HIP
library saw, unit by unit, and compare to the bars stated in each test.

Tie protocol.  Slot assignments must agree exactly.  Where they do not, the oracle's own scores
decide: if the library's choice lies within 1e-4 of the oracle's best score (its fp32
matrix-core accumulation rounds differently from the oracle's fp64 sum) the event is counted
as a tie, the oracle is re-run for that unit with that one choice overridden (the oracle checks
the 1e-4 margin itself and refuses anything else), and the comparison goes on.  Any other
disagreement fails.
"""
from __future__ import annotations

import numpy as np
import torch

from oracle import kvm_oracle as ko

F32_EPS = dict(ln_eps=float(np.float32(1e-5)), norm_eps=float(np.float32(1e-12)))
ORACLE_BUDGET = {"none": ko.BUDGET_NONE, "fixed": ko.BUDGET_FIXED, "sqrt": ko.BUDGET_SQRT,
                 "table": ko.BUDGET_TABLE}


def oracle_cfg(w) -> ko.KVMConfig:
    return ko.KVMConfig(head_dim=w.head_dim, rope_dims=w.rope_dims, chunk_len=w.chunk_len,
                        n_bswa_chunks=w.n_bswa_chunks, n_sink=w.n_sink, io=w.io,
                        budget_kind=ORACLE_BUDGET[w.budget_kind], budget_fixed=w.budget_fixed,
                        budget_scale=w.budget_scale,
                        budget_table=list(w.budget_table) if w.budget_kind == "table" else None, **F32_EPS)


def f64(t) -> np.ndarray:
    return t.detach().to("cpu", torch.float64).numpy()


def unit_inputs(w, q, k, v, params, b, h):
    """Slices of one (batch, KV head) unit as fp64 numpy, laid out for the oracle."""
    G = w.n_q_heads // w.n_kv_heads
    qs = f64(q[b, :, h * G:(h + 1) * G]).transpose(1, 0, 2)         # [G, T, d]
    g = params.get("gate")
    return dict(q=qs, k=f64(k[b, :, h]), v=f64(v[b, :, h]), g=None if g is None else f64(g[b, :, h]))


def make_oracle_unit(w, params, h) -> ko.KVMUnit:
    G = w.n_q_heads // w.n_kv_heads
    pick = lambda key, sl: None if params.get(key) is None else f64(params[key][sl])
    return ko.KVMUnit(oracle_cfg(w), G, pick("ln_gamma", h), pick("ln_beta", h),
                      pick("tau_state", slice(h * G, (h + 1) * G)), pick("tau_bswa", slice(h * G, (h + 1) * G)))


class Ties:
    """Counted ties of one run: disagreements with the oracle that the oracle's own scores put
    inside the 1e-4 margin (merge: the library's row scores within 1e-4 of the best row; append:
    the swapped tokens' scores within 1e-4 of the selection boundary)."""

    def __init__(self, merge=0, append=0):
        self.merge, self.append = merge, append

    @property
    def total(self):
        return self.merge + self.append

    def __iadd__(self, other):
        self.merge += other.merge
        self.append += other.append
        return self

    def __repr__(self):
        return f"Ties(merge={self.merge}, append={self.append})"


# Ceiling on counted ties per (batch, KV head) unit and fold.  fp32 I/O: both sides sum the same
# fp32 operands in fp64, so none.  bf16 I/O: the library's scores are fp32 sums of exact products
# on the matrix cores (error up to ~d * 2^-24 * |score| ~ 1e-5 on scores of size 10), the oracle's
# are fp64 sums: two rows (or two tokens at the append boundary) closer than that can swap.  With
# C tokens per fold and continuous random data such near-ties are rare: at most one in four folds
# of a unit is allowed, and never more than one per fold.
def tie_ceiling(w, n_folds):
    return 0 if w.io == "f32" else (n_folds + 3) // 4


# What the parity tests of a session saw, one record per test case: written to a JSON file
# (parity_stats.json in the run's output folder) by tests/conftest.py when the session ends.
PARITY_LOG = []


def record_parity(case, units, ties, max_err, io):
    PARITY_LOG.append(dict(case=case, io=io, units=int(units), ties_merge=int(ties.merge),
                           ties_append=int(ties.append), max_err=float(max_err)))


def run_oracle_following(w, params, h, drive, gpu_assign, n_folds=None):
    """Run `drive(unit)` (which feeds tokens and returns outputs) and compare the fold logs with
    gpu_assign [F, C] (the library's trace for this unit).  Ties are overridden and the run is
    repeated; more of them than tie_ceiling allows fail.  n_folds: folds the run must have (the
    rows of gpu_assign by default).  Returns (outputs of drive, unit, Ties)."""
    overrides, app_overrides, ties = {}, {}, Ties()
    n_folds = gpu_assign.shape[0] if n_folds is None else n_folds
    ceiling = tie_ceiling(w, n_folds)
    while True:
        unit = make_oracle_unit(w, params, h)
        unit.overrides, unit.append_overrides = dict(overrides), dict(app_overrides)
        out = drive(unit)
        assert len(unit.fold_logs) == n_folds, (len(unit.fold_logs), n_folds)
        bad = None
        for f, log in enumerate(unit.fold_logs):
            ga = gpu_assign[f]
            if not np.array_equal(log["assign"], ga):
                bad = (f, log, ga)
                break
        if bad is None:
            return out, unit, ties
        f, log, ga = bad
        m0 = log["m_before"]
        gpu_app = sorted(int(j) for j in np.nonzero(ga >= m0)[0]) if m0 > 0 else None
        ora_app = sorted(int(j) for j in np.nonzero(log["appended"])[0]) if m0 > 0 else None
        if m0 > 0 and gpu_app != ora_app:
            assert f not in app_overrides, f"fold {f}: the append override did not settle the selection"
            ties.append += 1
            app_overrides[f] = gpu_app        # the oracle raises unless it is a boundary tie
        else:
            j = int(np.nonzero(log["assign"] != ga)[0][0])
            assert (f, j) not in overrides, f"fold {f} token {j}: the override did not settle the row"
            ties.merge += 1
            overrides[(f, j)] = int(ga[j])    # the oracle raises unless within the margin
        assert ties.total <= ceiling, f"{ties} over {n_folds} folds of one unit: more than the {ceiling} allowed"


def check_outputs(w, y_gpu: np.ndarray, y_ref: np.ndarray, what=""):
    """fp32: max-abs <= 1e-4.  bf16: per output row, max-abs error <= 2e-2 * max(row max-abs of
    the reference, 1e-3)."""
    err = np.abs(y_gpu - y_ref)
    if w.io == "f32":
        assert err.max() <= 1e-4, f"{what}: fp32 max-abs error {err.max():.3e}"
        return float(err.max())
    row_err = err.max(axis=-1)
    bound = 2e-2 * np.maximum(np.abs(y_ref).max(axis=-1), 1e-3)
    worst = float((row_err / bound).max())
    assert worst <= 1.0, f"{what}: bf16 row error is {worst:.3f} x the 2e-2 relative bound"
    return worst


def check_state(w, exp: dict, unit: ko.KVMUnit, b: int, h: int):
    """Exported library state of unit (b, h) against the oracle's."""
    st = unit.state
    m = st.m
    assert exp["m"] == m
    sK = exp["sK"][b, h].cpu().numpy()
    # both sides add exact products g * k-bar to an fp64 sum in position order
    np.testing.assert_array_equal(sK, st.sK)
    # the value sums are fp32 running sums on the GPU: each of a row's n additions rounds to within
    # 2^-24 of the partial sum, which is of the size of the row's largest element, so an element
    # may be off by n * 2^-24 * max|row| in absolute terms (it shows on elements that cancel to
    # far below the row's scale) on top of the relative bar
    sV_gpu = exp["sV"][b, h].cpu().numpy().astype(np.float64)
    row_abs = np.asarray(st.n, np.float64)[:, None] * 2.0 ** -24 * np.abs(st.sV).max(axis=1, keepdims=True)
    bad = np.abs(sV_gpu - st.sV) > 2e-5 * np.abs(st.sV) + 1e-5 + row_abs
    assert not bad.any(), f"{int(bad.sum())} of {bad.size} value-sum elements outside the fp32 summation bound"
    np.testing.assert_allclose(exp["rho"][b, h].cpu().numpy(), st.rho, rtol=1e-6)
    np.testing.assert_allclose(exp["w"][b, h].cpu().numpy(), st.w, rtol=1e-5)
    np.testing.assert_array_equal(exp["n"][b, h].cpu().numpy(), st.n)
    khat, vhat = ko.readout(st, unit.cfg, unit.gamma, unit.beta)
    kh_gpu, vh_gpu = f64(exp["khat"][b, h]), f64(exp["vhat"][b, h])
    # LN_s is done in fp64 on both sides from bit-equal sums; the last bits of the two fp64
    # evaluations may differ (a reciprocal against a division), so an element flips only when its
    # exact value lies within ~1e-15 of a rounding boundary of the I/O dtype: none is expected
    n_diff = int((kh_gpu != khat).sum())
    assert n_diff == 0, f"{n_diff} of {khat.size} key readout elements differ"
    tol = 2.0 ** -7 if w.io == "bf16" else 1e-5
    np.testing.assert_allclose(vh_gpu, vhat, rtol=tol, atol=tol * 1e-2)
