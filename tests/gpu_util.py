"""Helpers for the GPU parity tests: move seeded NumPy inputs to the device,
run the HIP path through the binding, bring results back as float64."""
import numpy as np
import torch

from oracle import transformer as otr
from paper_2408_12596_amd import binding as pb

DEV = "cuda:0"


def tdtype(name):
    return torch.bfloat16 if name == "bf16" else torch.float32


def to_dev(a, dtype="f32"):
    t = torch.from_numpy(np.ascontiguousarray(a))
    if t.dtype in (torch.float32, torch.float64):
        t = t.to(tdtype(dtype))
    return t.to(DEV)


def to_np(t):
    return t.detach().to("cpu").to(torch.float64).numpy() if t.is_floating_point() else t.cpu().numpy()


def rel_l2(a, b):
    a = np.asarray(a, np.float64).ravel()
    b = np.asarray(b, np.float64).ravel()
    n = np.linalg.norm(b)
    return np.linalg.norm(a - b) / (n if n > 0 else 1.0)


def scratch(nbytes):
    """Caller-owned scratch memory, poisoned: every byte 0xFF reads as NaN in fp32 and in bf16, so a kernel that
    reads workspace or stash it has not written shows up in the results."""
    return torch.full((int(nbytes) + 256,), 255, dtype=torch.uint8, device=DEV)


def quantize(a, dtype):
    """Values the device actually receives (bf16 rounding of the inputs), as float64."""
    if dtype == "bf16":
        return torch.from_numpy(np.asarray(a, np.float32)).to(torch.bfloat16).to(torch.float64).numpy()
    return np.asarray(a, np.float32).astype(np.float64)


def oracle_cfg(cfg):
    return {k: cfg[k] for k in ("arch", "L", "H", "nh", "F", "S", "V")}


def sync():
    torch.cuda.synchronize()
