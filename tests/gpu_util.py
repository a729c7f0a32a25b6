"""Shared pieces of the GPU parity tests: device upload of the seeded inputs and the
acceptance bar (bf16 inputs, fp32 accumulation): max-abs <= 2e-3 and relative L2 <= 1e-3
against the fp64 oracle; integer outputs bit-exact."""
import numpy as np

import ts_synth as S
from helpers import err_metrics

MAX_ABS = 2e-3
REL_L2 = 1e-3


def dev(bits, device="cuda"):
    return S.bits_to_torch_bf16(bits, device)


def assert_close(got, ref, what, max_abs=MAX_ABS, rel_l2=REL_L2):
    got = np.asarray(got, dtype=np.float64)
    ref = np.asarray(ref, dtype=np.float64)
    assert got.shape == ref.shape, (what, got.shape, ref.shape)
    assert np.all(np.isfinite(got)), what + ": non-finite output"
    a, r = err_metrics(got, ref)
    assert a <= max_abs and r <= rel_l2, "%s: max-abs %.3e (bar %.1e), rel-L2 %.3e (bar %.1e)" % (
        what, a, max_abs, r, rel_l2)
    return a, r
