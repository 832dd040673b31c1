"""Shared helpers of the GPU parity tests: moving seeded NumPy inputs to the
device in the library's layouts and comparing against the CPU checker."""
import numpy as np
import torch

DEV = "cuda:0"


def tdtype(dtype):
    return torch.bfloat16 if dtype == "bf16" else torch.float32


def to_dev(a, dtype):
    """float32 NumPy array (values exactly representable in `dtype`) -> device tensor."""
    return torch.from_numpy(np.ascontiguousarray(a)).to(DEV).to(tdtype(dtype)).contiguous()


def i32(a):
    return torch.from_numpy(np.ascontiguousarray(a, dtype=np.int32)).to(DEV)


def round_up(x, m):
    return (x + m - 1) // m * m


def pad_rows(a, l_max):
    """Pad a [B, n_kv, L, d] cache with NaN rows up to l_max (rows the step must never use)."""
    B, n, L, d = a.shape
    if L == l_max:
        return a
    out = np.full((B, n, l_max, d), np.nan, dtype=np.float32)
    out[:, :, :L] = a
    return out


def v_blocked_to_rows(vb):
    """Library value-cache layout [B, n_kv, L/32, d, 32] -> [B, n_kv, L, d] (host side, for checks)."""
    B, n, nb, d, kb = vb.shape
    return vb.permute(0, 1, 2, 4, 3).reshape(B, n, nb * kb, d)


def k_cache_to_rows(kc, blocked=None):
    """Library key-cache layout (shape [B, n_kv, L, d]) -> row-major [B, n_kv, L, d] (host side, for checks).
    fp32 caches are row-major already; bf16 caches hold blocks of 32 rows as [half][d/8][slot 16][8] with
    row jj of a block = slot 4*(jj/8) + jj%4 of half (jj/4)%2."""
    if blocked is None:
        blocked = kc.dtype == torch.bfloat16
    if not blocked:
        return kc
    B, n, L, d = kc.shape
    t = kc.reshape(B, n, L // 32, 2, d // 8, 4, 4, 8)          # [.., half, chunk, jj/8, jj%4, e]
    return t.permute(0, 1, 2, 5, 3, 6, 4, 7).reshape(B, n, L, d)


def max_rel_err(got, ref):
    """max |got - ref| / max |ref| over the tensor (tensor-max normalised)."""
    got = np.asarray(got, dtype=np.float64)
    ref = np.asarray(ref, dtype=np.float64)
    return float(np.max(np.abs(got - ref)) / max(np.max(np.abs(ref)), 1e-30))


def assert_close(got, ref, tol, what=""):
    assert np.all(np.isfinite(np.asarray(got, dtype=np.float64))), f"{what}: non-finite output"
    err = max_rel_err(got, ref)
    assert err <= tol, f"{what}: max relative error {err:.3e} > {tol:.1e}"
    return err
