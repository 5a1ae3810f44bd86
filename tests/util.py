"""Helpers shared by the parity tests: error metrics and oracle/device glue (no method arithmetic)."""
import numpy as np


def rel_max_err(y, ref):
    """max |y - ref| / max |ref|."""
    ref = np.asarray(ref, dtype=np.float64)
    y = np.asarray(y, dtype=np.float64)
    return float(np.abs(y - ref).max() / max(np.abs(ref).max(), 1e-30))


def floored_elem_err(y, ref):
    """max over elements of |y - ref| / max(|ref|, tau), tau = 1e-2 * rms(ref)."""
    ref = np.asarray(ref, dtype=np.float64)
    y = np.asarray(y, dtype=np.float64)
    tau = 1e-2 * np.sqrt(np.mean(ref * ref)) + 1e-30
    return float((np.abs(y - ref) / np.maximum(np.abs(ref), tau)).max())


# Output tolerance of the linear layers against the fp32 oracle (both metrics), from the
# benchmark definition: max relative error 1e-2 after bf16 rounding of the inputs. The arithmetic
# predicts far less: identical bf16 operands, exact fp32 products, a different summation order
# (~1e-6) and one bf16 rounding of the stored result (2^-9 = 2e-3 of the element).
Y_TOL = 1e-2
