"""Shared helpers of the GPU parity tests: run a synthetic net through libdlf and through the
oracle on the same seeded tensors and compare with the tolerance the workload states."""
import sys

import numpy as np

# Tolerance of the fp16 path against the fp32 oracle, per output tensor:
#   max |err| <= 1e-2 * max |ref|   and   ||err||_2 / ||ref||_2 <= 5e-3
MAX_ERR_FRAC = 1e-2
REL_L2 = 5e-3


def compare(got, ref, what=""):
    got = np.asarray(got, dtype=np.float32)
    ref = np.asarray(ref, dtype=np.float32)
    assert got.shape == ref.shape, (what, got.shape, ref.shape)
    assert np.all(np.isfinite(got)), what + ": non-finite output"
    err = np.abs(got - ref)
    mref = float(np.abs(ref).max())
    merr = float(err.max())
    rl2 = float(np.linalg.norm(got - ref) / max(np.linalg.norm(ref), 1e-30))
    msg = "%s: max|err|=%.4g (%.3g of max|ref|=%.4g) relL2=%.3g" % (what, merr,
                                                                  merr / max(mref, 1e-30), mref, rl2)
    print(msg)
    sys.stdout.flush()
    if mref == 0.0:
        assert merr == 0.0, msg
        return merr, rl2
    assert merr <= MAX_ERR_FRAC * mref, msg
    assert rl2 <= REL_L2, msg
    return merr, rl2


def announce(*a):
    print("[case]", *a)
    sys.stdout.flush()
