"""Helpers for the GPU parity tests: tensors to/from the device, error metrics."""
import numpy as np
import torch

DEV = "cuda:0"


def dev_h(a):
    """numpy float array (binary16-representable) -> device half tensor."""
    return torch.from_numpy(np.ascontiguousarray(a, dtype=np.float32)).to(torch.float16).to(DEV)


def dev_f(a):
    return torch.from_numpy(np.ascontiguousarray(a, dtype=np.float32)).to(DEV)


def dev_i(a):
    return torch.from_numpy(np.ascontiguousarray(a, dtype=np.int32)).to(DEV)


def host(t):
    torch.cuda.synchronize()
    return t.detach().to("cpu").to(torch.float64).numpy()


def rel_err(a, b):
    """max_i |a_i-b_i| / max(|b_i|, 1e-2*max|b|): the relative error used for FP16 tensors."""
    a = np.asarray(a, np.float64).reshape(-1)
    b = np.asarray(b, np.float64).reshape(-1)
    scale = np.maximum(np.abs(b), 1e-2 * np.max(np.abs(b)) + 1e-300)
    return float(np.max(np.abs(a - b) / scale)) if a.size else 0.0


def rel_err_fp32(a, b, floor_frac=0.0):
    """max_i |a_i-b_i| / max(|b_i|, floor_frac*max|b|, tiny): used for FP32 loss and update.

    floor_frac > 0 keeps elements that cancel to almost zero (where FP32 rounding of the
    operands, not of the result, sets the error) from dominating a per-element relative error."""
    a = np.asarray(a, np.float64).reshape(-1)
    b = np.asarray(b, np.float64).reshape(-1)
    if not a.size:
        return 0.0
    floor = max(floor_frac * float(np.max(np.abs(b))), 1e-30)
    return float(np.max(np.abs(a - b) / np.maximum(np.abs(b), floor)))
