"""Shared helpers for the GPU parity tests (no arithmetic of the method lives here)."""
import numpy as np

RTOL = 1e-4     # the stated bar: 1e-4 relative (fp32) against the double-accumulated oracle


def assert_close(got, ref, what=""):
    """|got - ref| <= 1e-4 |ref| + 1e-4 rms(ref), element by element.  The rms term covers sums
    that cancel to nearly zero, where a relative bound on the element itself is meaningless."""
    got = np.asarray(got, np.float64)
    ref = np.asarray(ref, np.float64)
    assert got.shape == ref.shape, (what, got.shape, ref.shape)
    assert np.all(np.isfinite(got)), f"{what}: non-finite output"
    rms = float(np.sqrt(np.mean(ref * ref))) if ref.size else 0.0
    err = np.abs(got - ref)
    bound = RTOL * np.abs(ref) + RTOL * rms + 1e-30
    worst = int(np.argmax(err / bound)) if ref.size else 0
    assert np.all(err <= bound), (
        f"{what}: worst at flat index {worst}: got {got.flat[worst]!r} ref {ref.flat[worst]!r} "
        f"err {err.flat[worst]:.3e} bound {bound.flat[worst]:.3e} rms {rms:.3e}")


def rel_fro(got, ref):
    got = np.asarray(got, np.float64)
    ref = np.asarray(ref, np.float64)
    return float(np.linalg.norm(got - ref) / max(np.linalg.norm(ref), 1e-300))


def dev(a):
    import torch
    return torch.from_numpy(np.ascontiguousarray(a)).cuda()


def host(t):
    return t.detach().cpu().numpy()
