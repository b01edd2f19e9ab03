"""Comparison helpers shared by the parity tests."""
import numpy as np

REL_TOL = 1e-6      # aggregate and weights: |x - y| <= REL_TOL * max(|x|, |y|) (+ ABS_FLOOR)
ABS_FLOOR = 1e-12


def bits(a):
    a = np.ascontiguousarray(a)
    if a.dtype == np.float32:
        return a.view(np.uint32)
    if a.dtype == np.int32:
        return a.view(np.uint32)
    return a


def assert_bits_equal(got, want, what=""):
    """Bit-for-bit, except that any NaN matches any NaN."""
    got = np.ascontiguousarray(got)
    want = np.ascontiguousarray(want)
    assert got.shape == want.shape, "%s: shape %s vs %s" % (what, got.shape, want.shape)
    gb, wb = bits(got), bits(want)
    neq = gb != wb
    if got.dtype == np.float32:
        neq &= ~(np.isnan(got) & np.isnan(want))
    if neq.any():
        idx = np.flatnonzero(neq)
        i = int(idx[0])
        raise AssertionError("%s: %d of %d differ, first at %d: got %r (0x%08x) want %r (0x%08x)" % (
            what, idx.size, got.size, i, got.reshape(-1)[i], int(gb.reshape(-1)[i]),
            want.reshape(-1)[i], int(wb.reshape(-1)[i])))


def assert_close(got, want, what=""):
    """The floating-point bar: relative 1e-6 with an absolute floor for values at zero."""
    got = np.ascontiguousarray(got).astype(np.float64)
    want = np.ascontiguousarray(want).astype(np.float64)
    assert got.shape == want.shape
    err = np.abs(got - want)
    bound = REL_TOL * np.maximum(np.abs(got), np.abs(want)) + ABS_FLOOR
    bad = ~(err <= bound)
    bad &= ~(np.isnan(got) & np.isnan(want))
    if bad.any():
        i = int(np.flatnonzero(bad)[0])
        raise AssertionError("%s: %d of %d outside 1e-6 relative, first at %d: got %r want %r" % (
            what, int(bad.sum()), got.size, i, got.reshape(-1)[i], want.reshape(-1)[i]))


def count_bit_equal(got, want):
    return int((bits(got) == bits(want)).sum()), int(np.asarray(got).size)
