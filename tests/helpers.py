"""Shared test plumbing: error measures of the parity gates."""
from __future__ import annotations

import numpy as np

from paper_2508_11584_amd.synthetic import KIND, head_cfgs, make_engine  # noqa: F401  (re-exported for the tests)


def relerr(got, ref) -> float:
    """max |got - ref| / max |ref| over one tensor (the gate's error measure)."""
    got, ref = np.asarray(got, dtype=np.float64), np.asarray(ref, dtype=np.float64)
    assert got.shape == ref.shape, (got.shape, ref.shape)
    return float(np.max(np.abs(got - ref)) / max(np.max(np.abs(ref)), 1e-300))


# A depth map whose largest value is below this share of its largest magnitude before the final ReLU is taken
# to be clipped: the ReLU has removed (almost) all of the signal the head computed.
CLIPPED_BELOW = 0.25


def depth_errs(got, ref) -> dict:
    """Both normalisations of the depth error, and how much of the oracle's map survives its final ReLU.

    stated   max |got - depth| / max |depth|: the measure every other tensor uses
    pre_relu max |got - depth| / max |depth before its final ReLU|: ReLU is 1-Lipschitz, so this bounds the
             error of the un-clipped signal relative to that signal's size
    positive fraction of the oracle's pixels above zero;  clipped: max depth < CLIPPED_BELOW max |pre-ReLU|
    """
    got = np.asarray(got, dtype=np.float64)
    assert got.shape == ref["depth"].shape, (got.shape, ref["depth"].shape)
    num = float(np.max(np.abs(got - ref["depth"])))
    top, top_pre = float(np.max(ref["depth"])), float(np.max(np.abs(ref["pre_relu"])))
    return {"stated": num / max(top, 1e-300), "pre_relu": num / max(top_pre, 1e-300),
            "positive": float(np.mean(ref["depth"] > 0.0)), "clipped": bool(top < CLIPPED_BELOW * top_pre)}


def depth_gate(errs: dict, tol: float) -> bool:
    """The stated measure decides wherever the map is not clipped; a clipped map is held to the pre-ReLU form."""
    return errs["pre_relu"] <= tol if errs["clipped"] else errs["stated"] <= tol
