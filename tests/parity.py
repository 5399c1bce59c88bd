"""Shared helpers of the GPU parity tests (comparison rule, uploads, oracle graph)."""
import sys

import numpy as np

RTOL_F32 = 1e-4
RTOL_BF16 = 2e-2


def say(msg):
    """Names the case before a GPU step runs, flushed, so a lost box still shows it."""
    print("[case] " + msg, file=sys.stderr, flush=True)


def assert_close(got, ref, rtol, what="", cascade_share=0.0):
    """Per tensor: |got - ref| <= rtol * |ref| + rtol * RMS(ref) for every element.

    cascade_share > 0 (bf16 storage, whole-model comparisons only): that share of the elements
    may lie outside the bound, by at most a factor of two.  Both sides round every stored tensor
    to bf16; where an exact sum falls within accumulation error of a rounding boundary the two
    roundings legitimately differ by one unit (2^-8 relative), and the layers above see that
    unit multiplied by a weight.  An element fed by such a flip of a large input can leave the
    bound although every operation is within it on its own inputs (which the same tests check
    layer by layer without this allowance)."""
    got = np.asarray(got, dtype=np.float64)
    ref = np.asarray(ref, dtype=np.float64)
    assert got.shape == ref.shape, f"{what}: shape {got.shape} vs {ref.shape}"
    assert np.all(np.isfinite(got)), f"{what}: non-finite values"
    rms = float(np.sqrt(np.mean(ref * ref))) if ref.size else 0.0
    err = np.abs(got - ref)
    bound = rtol * np.abs(ref) + rtol * rms
    bad = err > bound
    if cascade_share > 0.0 and bad.any() and bad.mean() <= cascade_share:
        bad = err > 2.0 * bound
    if bad.any():
        i = np.unravel_index(np.argmax(err - bound), err.shape)
        fro = np.linalg.norm(got - ref) / max(np.linalg.norm(ref), 1e-300)
        raise AssertionError(
            f"{what}: {int(bad.sum())} of {bad.size} elements outside tolerance; worst at {i}: "
            f"got {got[i]!r} ref {ref[i]!r} (rms {rms:.3e}, rel fro {fro:.3e})")


def rel_fro(got, ref):
    got = np.asarray(got, dtype=np.float64)
    ref = np.asarray(ref, dtype=np.float64)
    return float(np.linalg.norm(got - ref) / max(np.linalg.norm(ref), 1e-300))
