"""Shared helpers of the GPU parity tests (buffers and error measures only)."""
import numpy as np

TOL = {"f32": 1e-4, "bf16": 2e-2}   # max |y - ref| / max |ref|  (the stated parity bar)


def rel_err(got, ref):
    got = np.asarray(got, np.float64)
    ref = np.asarray(ref, np.float64)
    denom = np.abs(ref).max()
    return float(np.abs(got - ref).max() / (denom if denom > 0 else 1.0))


def host(t):
    """Device tensor -> fp64 numpy."""
    return t.detach().float().cpu().numpy().astype(np.float64)


def draw(shape, seed, dtype, std=1.0):
    """Seeded N(0, std) values rounded once to the storage dtype (fp32 container)."""
    from paper_2401_10652_amd import inputs as I
    n = int(np.prod(shape))
    return I.round_to_storage(I.standard_normal(900000 + seed, n) * std, dtype).reshape(shape)
