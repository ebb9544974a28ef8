"""Helpers shared by the GPU parity tests."""
import numpy as np


def rel_err(got, ref):
    """max_ij |got_ij - ref_ij| / max(|ref_ij|, rms(ref_i,:)).

    A relative error that does not blow up on outputs that happen to be near
    zero: an element is measured against its own magnitude or, if it is smaller
    than that, against the root-mean-square of its row.  The row is the right
    scale because every element of a row is a dot product with the same
    activation vector, so rounding errors grow with that row's magnitude, and
    rows of one batch can differ by orders of magnitude.  1-D inputs are one
    row."""
    got = np.atleast_2d(np.asarray(got, dtype=np.float64))
    ref = np.atleast_2d(np.asarray(ref, dtype=np.float64))
    if ref.size == 0:
        return 0.0
    rms = np.sqrt(np.mean(ref * ref, axis=-1, keepdims=True))
    rms = np.where(rms > 0, rms, 1.0)
    return float(np.max(np.abs(got - ref) / np.maximum(np.abs(ref), rms)))


def fro_err(got, ref):
    got = np.asarray(got, dtype=np.float64)
    ref = np.asarray(ref, dtype=np.float64)
    n = float(np.linalg.norm(ref))
    return float(np.linalg.norm(got - ref)) / (n if n > 0 else 1.0)


def bf16_bits_to_f64(b):
    return (np.asarray(b, dtype=np.uint16).astype(np.uint32) << np.uint32(16)).view(np.float32).astype(np.float64)


def as_f64(a):
    a = np.asarray(a)
    return bf16_bits_to_f64(a) if a.dtype == np.uint16 else a.astype(np.float64)


# tolerances of the parity bar: bf16 in / fp32 accumulate, and fp32
TOL_BF16 = 2e-2
TOL_F32 = 1e-4
