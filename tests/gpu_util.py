"""Helpers shared by the GPU parity tests (data movement and error metrics only)."""
import numpy as np
import torch

# acceptance tolerances: bf16 output against the unrounded fp64 oracle
O_MAX_ABS = 2e-2
O_MEAN_ABS = 2e-3
LSE_MAX_ABS = 1e-3


def to_device(bits: np.ndarray, fmt: str = "bf16") -> torch.Tensor:
    """uint16 bf16 (or binary16) bit patterns -> tensor of that type on cuda:0 (bit-exact)."""
    dtype = torch.bfloat16 if fmt == "bf16" else torch.float16
    return torch.from_numpy(np.ascontiguousarray(bits).view(np.int16)).view(dtype).cuda()


def errors(out_gpu: torch.Tensor, lse_gpu: torch.Tensor, out_ref: np.ndarray, lse_ref: np.ndarray, rows=None):
    """(max abs O, mean abs O, max abs LSE) of GPU results against oracle rows."""
    if rows is not None:
        idx = torch.as_tensor(np.asarray(rows, dtype=np.int64), device=out_gpu.device)
        out_gpu = out_gpu.index_select(2, idx)
        lse_gpu = lse_gpu.index_select(2, idx)
    o = out_gpu.float().cpu().numpy().astype(np.float64)
    l = lse_gpu.cpu().numpy().astype(np.float64)
    assert o.shape == out_ref.shape and l.shape == lse_ref.shape
    assert np.isfinite(o).all() and np.isfinite(l).all()
    d = np.abs(o - out_ref)
    return float(d.max()), float(d.mean()), float(np.abs(l - lse_ref).max())


def assert_parity(out_gpu, lse_gpu, out_ref, lse_ref, rows=None, tag=""):
    mx, mean, lmx = errors(out_gpu, lse_gpu, out_ref, lse_ref, rows)
    print(f"[parity] {tag}: O max-abs {mx:.3e} mean-abs {mean:.3e}; LSE max-abs {lmx:.3e}", flush=True)
    assert mx <= O_MAX_ABS, (tag, mx)
    assert mean <= O_MEAN_ABS, (tag, mean)
    assert lmx <= LSE_MAX_ABS, (tag, lmx)
