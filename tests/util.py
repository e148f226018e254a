"""Shared helpers of the GPU parity tests (buffers and error measures only)."""
import numpy as np

TOL = {"f32": 1e-4, "bf16": 2e-2}   # max |y - ref| / max |ref|  (the stated parity bar)


def rel_err(got, ref):
    got = np.asarray(got, np.float64)
    ref = np.asarray(ref, np.float64)
    denom = np.abs(ref).max()
    return float(np.abs(got - ref).max() / (denom if denom > 0 else 1.0))


def mixed_err(got, ref, rtol):
    """Largest |got - ref| / (rtol |ref| + rtol RMS(ref)) over the elements: <= 1 means every
    element is within rtol of its own magnitude plus rtol of the tensor's typical magnitude.
    (A purely elementwise relative error is meaningless at the zero crossings of an N(0, .)
    output, and a purely global one lets a small element be far off; this gate sits between.)"""
    got = np.asarray(got, np.float64)
    ref = np.asarray(ref, np.float64)
    rms = float(np.sqrt(np.mean(ref * ref))) if ref.size else 0.0
    den = rtol * np.abs(ref) + rtol * (rms if rms > 0 else 1.0)
    return float((np.abs(got - ref) / den).max()) if ref.size else 0.0


def check(got, ref, dtype, what="", depth=1):
    """The parity bar: the global gate at the dtype's tolerance whatever the depth, and the
    mixed gate at the tolerance for one kernel, layer or module.  Behind a chain of ``depth``
    layers (pair-stack modules) the rounding errors of the stages, independent of each other,
    add in quadrature, so the mixed gate is held to sqrt(depth) times the tolerance.
    Returns (global relative error, mixed-gate ratio)."""
    tol = TOL[dtype]
    e, m = rel_err(got, ref), mixed_err(got, ref, tol)
    assert e <= tol, f"{what}: max|d|/max|ref| = {e:.3e} > {tol}"
    assert m <= depth ** 0.5, f"{what}: mixed gate ratio {m:.3f} > sqrt({depth}) (rtol {tol})"
    return e, m


def host(t):
    """Device tensor -> fp64 numpy."""
    return t.detach().float().cpu().numpy().astype(np.float64)


def draw(shape, seed, dtype, std=1.0):
    """Seeded N(0, std) values rounded once to the storage dtype (fp32 container)."""
    from paper_2401_10652_amd import inputs as I
    n = int(np.prod(shape))
    return I.round_to_storage(I.standard_normal(900000 + seed, n) * std, dtype).reshape(shape)
