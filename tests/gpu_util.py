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


def blockwise_rel_l2(a, b, block=64, floor=0.25):
    """Largest relative L2 error over the block x block tiles of a matrix (1-D input: runs of `block` elements),
    trailing partial tiles included as tiles of their own.  A whole-tensor rel-L2 of 2e-2 lets a dropped 64 x 64
    tile of a large output through; per tile the same mistake is an error of 1.0.  Tiles whose reference norm is
    far below the tensor's average (`floor` times the root mean square, over the tile's elements) are measured
    against that floor instead, so that a tile of near-zeros does not turn rounding noise into a large ratio."""
    a = np.asarray(a, np.float64)
    b = np.asarray(b, np.float64)
    assert a.shape == b.shape
    if a.ndim == 1:
        a, b = a[None, :], b[None, :]
    a = a.reshape(-1, a.shape[-1])
    b = b.reshape(-1, b.shape[-1])
    R, C = b.shape
    br, bc = min(block, R), min(block, C)
    pr, pc = (-R) % br, (-C) % bc

    def tiles(x):
        x = np.pad(x, ((0, pr), (0, pc)))
        return x.reshape((R + pr) // br, br, (C + pc) // bc, bc).sum(axis=(1, 3))
    err = np.sqrt(tiles((a - b) ** 2))
    ref = np.sqrt(tiles(b ** 2))
    count = tiles(np.ones_like(b))
    rms = np.sqrt((b ** 2).mean()) if b.size else 0.0
    den = np.maximum(ref, floor * rms * np.sqrt(count))
    den[den == 0] = 1.0
    return float((err / den).max())


def assert_close_blockwise(a, b, tol, name="", block=64):
    """Whole-tensor rel-L2 and the same bound on every block x block tile."""
    whole, worst = rel_l2(a, b), blockwise_rel_l2(a, b, block)
    assert whole <= tol, (name, "whole tensor", whole)
    assert worst <= tol, (name, "worst tile", worst)


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
