"""Comparator between GPU outputs and the CPU fp64 checker, and GPU upload helpers (test-side only)."""
from __future__ import annotations

import numpy as np

TIE_TOL = 1e-3      # ids may differ only where the checker's logits are within this distance
LOGPROB_TOL = 2e-2  # absolute tolerance on log-probabilities for bf16 weights


def compare_with_oracle(gpu_ids, gpu_lp, ora_ids, ora_lse, z_at, V, tie_tol=TIE_TOL, lp_tol=LOGPROB_TOL):
    """Check GPU top-k against the checker.

    gpu_ids/gpu_lp: [rows, k] numpy; ora_ids: [rows, k]; ora_lse: [rows] fp64;
    z_at(row_idx, col_idx) -> fp64 checker logits at those (row, id) pairs.
    Returns the number of positions that needed the tie exemption.  Raises AssertionError otherwise.
    """
    rows, k = gpu_ids.shape
    assert ora_ids.shape == (rows, k)
    assert gpu_ids.min() >= 0 and gpu_ids.max() < V, "id out of range"
    for i in range(rows):
        assert len(set(gpu_ids[i].tolist())) == k, f"row {i}: duplicate ids {gpu_ids[i]}"
    rr = np.repeat(np.arange(rows, dtype=np.int32), k)
    zg = z_at(rr, gpu_ids.ravel()).reshape(rows, k)
    zo = z_at(rr, ora_ids.ravel()).reshape(rows, k)
    differ = gpu_ids != ora_ids
    bad = differ & (np.abs(zg - zo) > tie_tol)
    if bad.any():
        i, p = np.argwhere(bad)[0]
        raise AssertionError(f"row {i} rank {p}: gpu id {gpu_ids[i, p]} (z={zg[i, p]:.6f}) vs "
                             f"checker id {ora_ids[i, p]} (z={zo[i, p]:.6f}); {bad.sum()} such positions")
    lp_ref = zg - ora_lse[:, None]
    err = np.abs(gpu_lp.astype(np.float64) - lp_ref)
    assert np.all(np.isfinite(gpu_lp)), "non-finite log-probability"
    if err.max() > lp_tol:
        i, p = np.unravel_index(np.argmax(err), err.shape)
        raise AssertionError(f"row {i} rank {p}: logprob {gpu_lp[i, p]} vs {lp_ref[i, p]} (err {err.max():.3e})")
    # descending order of the checker's logits along each row, up to the tie tolerance
    assert np.all(zg[:, :-1] - zg[:, 1:] >= -tie_tol), "output not in descending order"
    return int(differ.sum()), float(err.max())


def to_dev_bf16(bits: np.ndarray):
    """uint16 bf16 bit patterns -> torch.bfloat16 device tensor (bitwise copy)."""
    import torch
    t = torch.from_numpy(np.ascontiguousarray(bits).view(np.int16))
    return t.cuda().view(torch.bfloat16)


def to_dev_f32(x: np.ndarray):
    import torch
    return torch.from_numpy(np.ascontiguousarray(x, dtype=np.float32)).cuda()
