"""Helpers shared by the CPU and GPU tests (no arithmetic of the method lives here)."""
from __future__ import annotations

import numpy as np
import torch

RTOL = 1e-10      # relative tolerance on values (fp64), per the benchmark spec
AFLOOR = 1e-12    # absolute floor, in units of A = sum |term| of the element (covers cancellation)


def np_(t):
    return None if t is None else t.detach().cpu().numpy()


def assert_values_close(got, ref, absum, what=""):
    """|got - ref| <= RTOL*|ref| + AFLOOR*A element by element."""
    got, ref, absum = np.asarray(got, dtype=np.float64), np.asarray(ref, dtype=np.float64), np.asarray(absum)
    assert got.shape == ref.shape, "%s: shape %s vs %s" % (what, got.shape, ref.shape)
    err = np.abs(got - ref)
    bound = RTOL * np.abs(ref) + AFLOOR * absum
    bad = err > bound
    if bad.any():
        idx = np.argwhere(bad)[0]
        raise AssertionError("%s: %d of %d elements off; first at %s got %.17g ref %.17g A %.3g" % (
            what, int(bad.sum()), bad.size, tuple(idx), got[tuple(idx)], ref[tuple(idx)], absum[tuple(idx)]))


def assert_index_equal(got, ref, what=""):
    got, ref = np.asarray(got), np.asarray(ref)
    assert got.dtype == np.int32, "%s: dtype %s" % (what, got.dtype)
    assert got.shape == ref.shape, "%s: shape %s vs %s" % (what, got.shape, ref.shape)
    assert np.array_equal(got, ref.astype(np.int32)), "%s: index arrays differ" % what


def level_arrays_np(T):
    """(tags, pos list, crd list, vals) of a synth.LevelTensor as numpy arrays."""
    return list(T.tags), [np_(p) for p in T.pos], [np_(c) for c in T.crd], np_(T.vals)
