"""Helpers shared by the GPU parity tests (not collected by pytest)."""
import numpy as np
import torch

from oracle.model import Config
from paper_2602_06412_amd import binding as B
from paper_2602_06412_amd import workloads as wl

DEV = "cuda:0"


def oracle_cfg(shape):
    return Config(shape.n_layers, shape.d_model, shape.n_heads, shape.d_head, shape.d_ff,
                  shape.vocab, shape.mask_id, shape.rms_eps, shape.rope_theta, shape.storage)


def dev(a, dtype=None):
    t = torch.as_tensor(np.ascontiguousarray(a))
    if dtype is not None:
        t = t.to(dtype)
    return t.to(DEV).contiguous()


def weights_to_device(w):
    out = {k: v.to(DEV) for k, v in w.items() if k != "layers"}
    out["layers"] = [{k: v.to(DEV) for k, v in l.items()} for l in w["layers"]]
    return out


def bf16_ulp(x):
    """Spacing of bf16 numbers at |x| (fp64 array)."""
    ax = np.maximum(np.abs(x), 2.0 ** -126)
    return 2.0 ** (np.floor(np.log2(ax)) - 7)


def logits_tol(z_oracle, storage):
    """Per-element tolerance on logits.  bf16: 2e-2 absolute, or one bf16 spacing where that
    is larger (|z| >= 4), since two correctly rounded results may land on neighbouring grid
    points.  fp32: 2e-4 absolute (fp32 accumulation over <= 4096-term dot products)."""
    if storage == "bf16":
        return np.maximum(2e-2, bf16_ulp(z_oracle))
    return np.full_like(z_oracle, 2e-4)


def compact(lock_np):
    """Run sl_compact_active on a [B, N] uint8 mask; returns (active_idx, cu_active) as numpy."""
    Bn, N = lock_np.shape
    lock = dev(lock_np.astype(np.uint8))
    idx = torch.full((Bn * N,), -1, dtype=torch.int32, device=DEV)
    cu = torch.full((Bn + 1,), -1, dtype=torch.int32, device=DEV)
    B.sl_compact_active(lock, Bn, N, idx, cu)
    torch.cuda.synchronize()
    cu = cu.cpu().numpy()
    return idx.cpu().numpy()[:cu[-1]], cu
