"""Seeded synthetic gradients with the shapes and value distributions of the five workloads.

This module only draws numbers.  It holds none of the method's arithmetic (no norm, no rounding,
no packing), so the CPU oracle's tests and the HIP library's tests can both take their inputs
from it.  The paper's own workloads are gradients of DeepLight, Wide ResNet-101-2 and
Transformer-XL (its Table 3, 1.3e8 to 6.1e8 parameters); none of those models or datasets are
available, so these synthetic gradients stand in for them.

Every worker's buffer is drawn chunk by chunk (CHUNK coordinates at a time) from one
torch.Generator seeded with DATA_SEED[config] * 1000003 + worker, on the device the buffer lives on.
The values therefore depend on (config, worker, d, device type) only.
"""
import math

import torch

CHUNK = 1 << 24

# name -> workload description.  `norm`, `scheme`, `s`, `pack`, `agg` are the quantiser settings
# the workload is run with; they are read by tests and bench, never used here.
CONFIGS = {
    "c1": dict(d=1_048_576, K=4, dist="normal", norm="l2", scheme="linear", s=127, pack="i8", agg="i32"),
    "c2": dict(d=25_600_000, K=8, dist="layer_blocks", blocks=160, norm="l2", scheme="exp", s=16,
               pack="i8", agg="i32"),
    "c3": dict(d=110_000_000, K=16, dist="normal_outliers", norm="linf", scheme="linear", s=127,
               pack="i8", agg="i32"),
    "c4": dict(d=350_000_000, K=32, dist="student_t3", norm="linf", scheme="exp", s=7, pack="i4", agg="i16"),
    "c5": dict(d=1_500_000_000, K=8, dist="mixture", norm="l2", scheme="linear", s=15, pack="u4s",
               agg="i32", bucket=1 << 26),
}
DATA_SEED = {"c1": 0x5EED0001, "c2": 0x5EED0002, "c3": 0x5EED0003, "c4": 0x5EED0004, "c5": 0x5EED0005}
QUANT_SEED = 0xC0FFEE


def _generator(name, worker, device):
    g = torch.Generator(device=device)
    g.manual_seed(DATA_SEED[name] * 1000003 + int(worker))
    return g


def block_std(name, blocks):
    """Per-layer-block standard deviations for the `layer_blocks` workload: log-uniform in
    [1e-5, 1e-2], one per block, shared by all workers (a layer's scale belongs to the model)."""
    g = torch.Generator(device="cpu")
    g.manual_seed(DATA_SEED[name] * 1000003 + 999_983)
    u = torch.rand(blocks, generator=g, dtype=torch.float64)
    return torch.pow(10.0, -5.0 + 3.0 * u).to(torch.float32)


def fill_worker(out, name, worker):
    """Overwrite the 1-D float32 tensor `out` with worker `worker`'s gradient for workload `name`.
    The length of `out` sets d (any d: reduced sizes keep the distribution)."""
    cfg = CONFIGS[name]
    assert out.dtype == torch.float32 and out.dim() == 1 and out.is_contiguous()
    d = out.numel()
    dev = out.device
    g = _generator(name, worker, dev)
    dist = cfg["dist"]
    if dist == "layer_blocks":
        blocks = cfg["blocks"]
        std = block_std(name, blocks).to(dev)
        per = max(1, -(-d // blocks))           # ceil(d / blocks) coordinates per block
    for lo in range(0, d, CHUNK):
        n = min(CHUNK, d - lo)
        view = out[lo:lo + n]
        if dist == "normal":
            view.normal_(0.0, 1e-3, generator=g)
        elif dist == "layer_blocks":
            view.normal_(0.0, 1.0, generator=g)
            idx = torch.arange(lo, lo + n, device=dev, dtype=torch.int64)
            idx = torch.div(idx, per, rounding_mode="floor").clamp_(max=blocks - 1)
            view.mul_(std[idx])
        elif dist == "normal_outliers":
            view.normal_(0.0, 1e-3, generator=g)
            mask = torch.rand(n, generator=g, device=dev) < 0.01
            view[mask] *= 100.0
        elif dist == "student_t3":
            z = torch.randn(4, n, generator=g, device=dev)
            den = torch.sqrt((z[1] * z[1] + z[2] * z[2] + z[3] * z[3]) / 3.0)
            view.copy_(1e-4 * z[0] / den)
        elif dist == "mixture":
            view.normal_(0.0, 1.0, generator=g)
            wide = torch.rand(n, generator=g, device=dev) < 0.1
            view.mul_(torch.where(wide, torch.tensor(1e-2, device=dev), torch.tensor(1e-4, device=dev)))
        else:
            raise ValueError(dist)
    return out


def make_workers(name, d=None, K=None, device="cpu"):
    """K float32 tensors of d coordinates each (defaults: the workload's own d and K)."""
    cfg = CONFIGS[name]
    d = cfg["d"] if d is None else int(d)
    K = cfg["K"] if K is None else int(K)
    return [fill_worker(torch.empty(d, dtype=torch.float32, device=device), name, w) for w in range(K)]


def num_buckets(d, bucket):
    return int(math.ceil(d / bucket))
