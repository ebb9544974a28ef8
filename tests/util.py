"""Helpers shared by the GPU parity tests."""
import numpy as np


def rel_err(got, ref):
    """max_i |got_i - ref_i| / max(|ref_i|, rms(ref)): a relative error that
    does not blow up on outputs that happen to be near zero."""
    got = np.asarray(got, dtype=np.float64)
    ref = np.asarray(ref, dtype=np.float64)
    if ref.size == 0:
        return 0.0
    rms = float(np.sqrt(np.mean(ref * ref)))
    den = np.maximum(np.abs(ref), rms if rms > 0 else 1.0)
    return float(np.max(np.abs(got - ref) / den))


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
