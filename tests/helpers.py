"""Host<->device plumbing shared by the GPU tests (no arithmetic of the method)."""
import os
import re

import numpy as np

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def ensure_built():
    """Load the in-tree library; build it only if it is not there."""
    from paper_2412_01034_amd import binding
    if not os.path.exists(binding.LIB_PATH):
        from paper_2412_01034_amd import build
        build.build_library()
    return binding


def header_functions():
    """Names of the functions declared in include/qail.h."""
    text = open(os.path.join(ROOT, "include", "qail.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(qail_[a-z0-9_]+)\s*\(", text)))


def dev(a: np.ndarray):
    """numpy -> device tensor with the same bytes (uint32 -> int32, uint16 -> int16, ...)."""
    import torch
    a = np.ascontiguousarray(a)
    view = {np.dtype(np.uint32): np.int32, np.dtype(np.uint16): np.int16, np.dtype(np.float16): np.float16}
    if a.dtype in view and a.dtype != np.float16:
        a = a.view(view[a.dtype])
    return torch.from_numpy(a).cuda()


def host(t, dtype):
    """device tensor -> numpy array reinterpreted as `dtype`."""
    import torch
    if t.dtype == torch.bfloat16:
        t = t.view(torch.int16)
    return t.cpu().numpy().view(dtype)


def w4a16_norm_err(y_bits: np.ndarray, y_ref: np.ndarray, nx: np.ndarray, nw: np.ndarray) -> float:
    """max |y - y_ref| / (||x_m|| * ||w_hat_n||) with y given as bf16 bit patterns."""
    y = (y_bits.astype(np.uint32) << np.uint32(16)).view(np.float32).astype(np.float64)
    denom = nx[:, None] * nw[None, :]
    denom = np.where(denom == 0, 1.0, denom)
    return float((np.abs(y - y_ref) / denom).max())


def ws_for(B, nbytes):
    """Device workspace of at least nbytes (None when none is needed)."""
    import torch
    if nbytes == 0:
        return None
    return torch.empty(nbytes, dtype=torch.uint8, device="cuda")
