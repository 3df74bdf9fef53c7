"""Helpers shared by the GPU parity tests: host tensor <-> device tensor, tolerance check."""
import numpy as np
import torch

from paper_2106_08301_amd import synth

REL_FRO_TOL = 1e-3      # ||Y - Y_oracle||_F / ||Y_oracle||_F
MAX_ABS_TOL = 1e-2      # max |Y - Y_oracle| / RMS(Y_oracle)


def to_device(t: synth.Tensor):
    if t.dtype == "f32":
        return torch.from_numpy(np.ascontiguousarray(t.data)).cuda()
    return torch.from_numpy(np.ascontiguousarray(t.data).view(np.int16)).view(torch.bfloat16).cuda()


def to_f64(t: torch.Tensor):
    return t.detach().to(torch.float64).cpu().numpy()


def storage_code(dtype, oracle):
    return oracle.STORE_F32 if dtype == "f32" else oracle.STORE_BF16


def check_close(Y, Y_ref, rel=REL_FRO_TOL, mx=MAX_ABS_TOL):
    Y, Y_ref = np.asarray(Y, dtype=np.float64), np.asarray(Y_ref, dtype=np.float64)
    assert Y.shape == Y_ref.shape
    assert np.all(np.isfinite(Y))
    ref_norm = np.sqrt((Y_ref ** 2).sum())
    if ref_norm == 0.0:
        assert not Y.any(), "reference is exactly zero, output is not"
        return 0.0, 0.0
    rel_fro = np.sqrt(((Y - Y_ref) ** 2).sum()) / ref_norm
    rms = ref_norm / np.sqrt(Y_ref.size)
    max_abs = np.abs(Y - Y_ref).max() / rms
    assert rel_fro <= rel, f"relative Frobenius error {rel_fro:.3e} > {rel}"
    assert max_abs <= mx, f"max abs error {max_abs:.3e} x RMS > {mx}"
    return rel_fro, max_abs
