"""Shared pieces of the GPU parity tests: error measures that look inside a
tensor (a whole-tensor norm can hide one wrong pixel per plane), and a log of
every measured error (one line per parity case, for tabulating).

Uses numpy only; the reference values always come from the oracle."""
import json
import os

import numpy as np


def rel_l2(got, ref, axis=None):
    got = np.asarray(got, dtype=np.float64)
    ref = np.asarray(ref, dtype=np.float64)
    num = np.sqrt(((got - ref) ** 2).sum(axis=axis))
    den = np.maximum(np.sqrt((ref ** 2).sum(axis=axis)), 1e-30)
    return num / den


def structure(got, ref):
    """Error measures of an NCHW tensor that a mis-indexed border, plane or
    image cannot hide from:
      per_image / per_channel : largest relative L2 error over images / channels
      border                  : largest relative L2 error of the four border
                                slices (first and last row and column)
      max_abs_over_rms        : largest elementwise error over the RMS of ref
      outliers                : fraction of elements whose error exceeds RMS / 4
    """
    got = np.asarray(got, dtype=np.float64)
    ref = np.asarray(ref, dtype=np.float64)
    err = np.abs(got - ref)
    rms = max(float(np.sqrt((ref ** 2).mean())), 1e-30)
    out = dict(per_image=float(rel_l2(got, ref, axis=(1, 2, 3)).max()),
               per_channel=float(rel_l2(got, ref, axis=(0, 2, 3)).max()),
               max_abs_over_rms=float(err.max() / rms),
               outliers=float((err > 0.25 * rms).mean()))
    slices = [np.s_[:, :, 0, :], np.s_[:, :, -1, :], np.s_[:, :, :, 0], np.s_[:, :, :, -1]]
    out["border"] = float(max(rel_l2(got[s], ref[s]) for s in slices))
    return out


def assert_structure(name, got, ref, bar, smooth):
    """No image, channel or border slice may be further off than 3x the
    whole-tensor bar (their norms hold fewer elements, so they scatter more).
    `smooth` tensors (forward values, reconstructions: no 0/1 decision lies
    between the two computations' roundings and the value) must also be
    close element by element: nothing beyond 40x the bar in units of the
    tensor's RMS.  Gradients pass through ReLU derivatives, where a decision
    taken the other way is an O(1) change of single elements on either side;
    there the fraction of such elements is bounded instead."""
    s = structure(got, ref)
    print("    %-6s per-image %.2e  per-channel %.2e  border %.2e  max|err|/rms %.2e  outliers %.1e" %
          (name, s["per_image"], s["per_channel"], s["border"], s["max_abs_over_rms"], s["outliers"]), flush=True)
    assert s["per_image"] < 3 * bar, (name, "per image", s)
    assert s["per_channel"] < 3 * bar, (name, "per channel", s)
    assert s["border"] < 3 * bar, (name, "border slices", s)
    if smooth:
        assert s["max_abs_over_rms"] < 40 * bar, (name, "max abs", s)
    else:
        assert s["outliers"] < bar, (name, "outlier fraction", s)
    return s


FLOOR_FACTOR = 1.5
# The GPU and the float32 oracle are two independent float32 evaluations, each about one floor away
# from the float64 value, so about sqrt(2) floors from each other; held to the same factor.
PAIR_FACTOR = 1.5 * 2 ** 0.5


def check_with_floors(errs, floors, vs32, bar, pooled=False):
    """errs, floors, vs32: {tensor name: relative error} of the GPU against the
    float64 oracle, of the float32 oracle against the float64 oracle (the
    floor), and of the GPU against the float32 oracle.  A tensor passes below
    the fixed bar, or -- where two correct evaluations are further apart than
    that -- within FLOOR_FACTOR floors of the float64 oracle and PAIR_FACTOR
    floors of the float32 one.

    pooled (fp32 operands): the differences come from a handful of ReLU
    decisions, rare events that land in different tensors in different
    evaluations, so a tensor's own floor is not a stable quantity; every
    tensor is held to FLOOR_FACTOR x the largest floor of the case instead.

    Returns the largest fraction of its allowance that any tensor used."""
    used = 0.0
    top = max(floors.values()) if floors else None
    for key, e in errs.items():
        if e < bar:
            used = max(used, e / bar)
            continue
        fl = top if pooled else floors.get(key)
        assert fl is not None, (key, e, "above the bar", bar)
        print("  %s: %.2e is above the %.0e bar; %s %.2e%s" %
              (key, e, bar, "largest floor of the case" if pooled else "floor of this tensor", fl,
               "" if pooled else ", GPU against the float32 oracle %.2e" % vs32[key]), flush=True)
        assert e < FLOOR_FACTOR * fl, (key, e, "floor", fl)
        if not pooled:
            assert vs32[key] < PAIR_FACTOR * fl, (key, "against the float32 oracle", vs32[key], "floor", fl)
        used = max(used, e / (FLOOR_FACTOR * fl))
    return used


def record(case, **values):
    """Append one line to the file named by RVN_PARITY_LOG (if set): the
    measured errors of a parity case."""
    path = os.environ.get("RVN_PARITY_LOG")
    if not path:
        return
    clean = {k: (float(v) if isinstance(v, (int, float, np.floating)) else v) for k, v in values.items()}
    with open(path, "a") as f:
        f.write(json.dumps(dict(case=case, **clean)) + "\n")
