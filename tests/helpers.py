"""Shared test plumbing: workloads -> device tensors, and the parity gates."""
import numpy as np
import torch


def to_device(w, names=("q", "k", "v", "dout"), pad_rows=0, pad_value=float("nan")):
    """Device tensors for a Workload.  bf16 workloads are uploaded from their exact bf16 bit patterns.

    pad_rows > 0 appends guard rows filled with pad_value AFTER row sum_B (they must never be read or written).
    """
    out = {}
    for n in names:
        x = getattr(w, n)
        if x is None:
            continue
        if w.dtype == "bf16":
            t = torch.from_numpy(w.bits[n].view(np.int16)).view(torch.bfloat16)
        else:
            t = torch.from_numpy(x)
        if pad_rows:
            pad = torch.full((pad_rows,) + tuple(t.shape[1:]), pad_value, dtype=t.dtype)
            t = torch.cat([t, pad], dim=0)
        out[n] = t.cuda()
    out["offsets"] = torch.from_numpy(w.offsets).cuda()
    return out


def f64(t: torch.Tensor) -> np.ndarray:
    return t.detach().to(torch.float64).cpu().numpy()


def gate_bf16(name, got, ref, abs_tol=2e-2, rel_tol=1e-2):
    """bf16 gate: max |g - r| <= abs_tol AND max |g - r| / max |r| <= rel_tol (error relative to the tensor's scale)."""
    got = np.asarray(got, dtype=np.float64); ref = np.asarray(ref, dtype=np.float64)
    assert got.shape == ref.shape, (name, got.shape, ref.shape)
    if ref.size == 0:
        return 0.0, 0.0
    assert np.isfinite(got).all(), f"{name}: non-finite values in the GPU result"
    err = np.abs(got - ref)
    max_abs = float(err.max())
    scale = float(np.abs(ref).max())
    rel = max_abs / scale if scale > 0 else 0.0
    assert max_abs <= abs_tol, f"{name}: max abs err {max_abs:.3e} > {abs_tol}"
    assert rel <= rel_tol, f"{name}: max err / max|ref| = {rel:.3e} > {rel_tol}"
    return max_abs, rel


def gate_f32(name, got, ref, tol=1e-5, relative_to_one=False):
    got = np.asarray(got, dtype=np.float64); ref = np.asarray(ref, dtype=np.float64)
    assert got.shape == ref.shape
    if ref.size == 0:
        return 0.0
    assert np.isfinite(got).all(), f"{name}: non-finite values in the GPU result"
    err = np.abs(got - ref)
    if relative_to_one:
        err = err / np.maximum(1.0, np.abs(ref))
    m = float(err.max())
    assert m <= tol, f"{name}: max err {m:.3e} > {tol}"
    return m


GUARD = 777.0


def sentinel_like(t: torch.Tensor, n_valid: int) -> torch.Tensor:
    """An output buffer shaped like t: NaN in the first n_valid rows (every one of them has to be written by the
    call under test, so a work item that is never claimed or is decoded to the wrong place shows up in an isfinite
    check over the whole tensor) and GUARD in the rows after them (which must stay untouched)."""
    x = torch.full_like(t, float("nan"))
    x[n_valid:] = GUARD
    return x


def sentinel_stats(shape) -> torch.Tensor:
    return torch.full(shape, float("nan"), dtype=torch.float32, device="cuda")


def assert_guard_rows_untouched(name, t: torch.Tensor, n_valid: int):
    assert (t[n_valid:] == GUARD).all(), f"guard rows of {name} were written"
