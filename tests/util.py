"""Shared helpers of the GPU parity tests (no arithmetic of the method lives here)."""
import numpy as np

TOL = 1e-2  # elementwise bound |gpu - oracle| <= TOL * (1 + |oracle|)


def dev(a):
    import torch
    return None if a is None else torch.from_numpy(np.ascontiguousarray(a)).cuda()


def host(t):
    return t.detach().cpu().numpy()


def assert_close(gpu, ref, what=""):
    g = np.asarray(gpu, dtype=np.float64)
    r = np.asarray(ref, dtype=np.float64)
    assert g.shape == r.shape, (what, g.shape, r.shape)
    assert np.all(np.isfinite(g)), what + ": non-finite GPU output"
    err = np.abs(g - r)
    bound = TOL * (1.0 + np.abs(r))
    bad = err > bound
    if bad.any():
        i = np.unravel_index(np.argmax(err - bound), err.shape)
        raise AssertionError("%s: %d of %d outside tolerance; worst at %s gpu=%r oracle=%r" %
                             (what, int(bad.sum()), bad.size, i, g[i], r[i]))


def assert_bit_equal(gpu, ref, what=""):
    g = np.ascontiguousarray(gpu).view(np.uint16)
    r = np.ascontiguousarray(ref).view(np.uint16)
    assert g.shape == r.shape, (what, g.shape, r.shape)
    # +0 and -0 compare equal as values; integer-valued cases never produce -0 after ReLU / sums
    if not np.array_equal(g, r):
        diff = np.argwhere(g != r)
        i = tuple(diff[0])
        raise AssertionError("%s: %d elements differ; first at %s gpu=%r oracle=%r" %
                             (what, len(diff), i, np.asarray(gpu)[i], np.asarray(ref)[i]))
