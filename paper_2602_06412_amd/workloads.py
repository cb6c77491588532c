"""Seeded synthetic inputs shared by the tests, the oracle's callers and bench.py.

This module holds NO arithmetic of the method: it only draws weights, prompts,
active sets and forced-lock priorities from seeds and names the workload shapes.
The shapes stand in for the paper's LLaDA-8B runs on MT-Bench / WikiText-103
(Sec. 3): prompt + generation lengths of a few hundred to ~2k positions, batch
<= 8, S = N_gen steps; no dataset item and no trained weight is used.
"""
from dataclasses import dataclass, asdict

import numpy as np
import torch


@dataclass(frozen=True)
class Shape:
    name: str
    n_layers: int
    d_model: int
    n_heads: int
    d_head: int
    d_ff: int
    vocab: int
    storage: str            # "fp32" | "bf16"
    rms_eps: float = 1e-5
    rope_theta: float = 10000.0

    @property
    def mask_id(self):
        return self.vocab - 1

    def asdict(self):
        d = asdict(self)
        d["mask_id"] = self.mask_id
        return d


# Tiny masked-diffusion LM, fp32: N=128 (32 prompt + 96 [MASK]), T=32, top-3 per step.
C1 = Shape("C1-tiny-fp32", 2, 256, 4, 64, 688, 1024, "fp32")
# One LLaDA-8B-shaped layer, bf16 (LM head at the LLaDA vocabulary so the whole step runs).
C2 = Shape("C2-llada8b-1layer", 1, 4096, 32, 128, 12288, 126464, "bf16")
# Full 32-layer LLaDA-8B shape.
C3 = Shape("C3-llada8b-32layer", 32, 4096, 32, 128, 12288, 126464, "bf16")
# Reduced shapes for parity tests the oracle finishes in seconds (several tiles + ragged tails).
S_BF16 = Shape("small-bf16", 2, 512, 4, 128, 1536, 4160, "bf16")
S_BF16_WIDE = Shape("small-bf16-wide", 1, 1024, 8, 128, 2816, 8256, "bf16")
# a very wide FFN (2 d_ff = 41472 columns): thin gate|up launches take the 256-column form of the weight-stream kernel
S_BF16_FFN = Shape("small-bf16-wide-ffn", 1, 256, 2, 128, 20736, 1056, "bf16")
# bf16 with 64-wide heads: runs on the shape-generic kernels instead of the MFMA ones
S_BF16_H64 = Shape("small-bf16-h64", 2, 256, 4, 64, 688, 1024, "bf16")


def torch_dtype(storage):
    return {"fp32": torch.float32, "bf16": torch.bfloat16}[storage]


def _normal(gen, shape, std, dtype, device):
    t = torch.empty(shape, dtype=torch.float32, device=device)
    t.normal_(0.0, std, generator=gen)
    return t.to(dtype)


def make_weights(shape, seed, device="cpu", std=0.02, norm_gain_jitter=0.0, emb_std=None):
    """Every matrix i.i.d. N(0, std^2) drawn in fp32 from the seed, then rounded
    to the storage type; norm gains are 1 (optionally 1 + jitter*N(0,1), which
    tests use so a dropped gain cannot hide).  emb_std overrides the embedding's std
    (the one-layer microbench feeds block inputs x ~ N(0,1)).
    Layout: [out_features, in_features]."""
    gen = torch.Generator(device=device)
    gen.manual_seed(int(seed))
    dt = torch_dtype(shape.storage)
    d, dff, V = shape.d_model, shape.d_ff, shape.vocab
    hd = shape.n_heads * shape.d_head

    def gain():
        g = torch.ones(d, dtype=torch.float32, device=device)
        if norm_gain_jitter:
            g = g + norm_gain_jitter * torch.empty(d, device=device).normal_(generator=gen)
        return g.to(dt)

    w = {"emb": _normal(gen, (V, d), std if emb_std is None else emb_std, dt, device), "layers": []}
    for _ in range(shape.n_layers):
        w["layers"].append({
            "attn_norm": gain(),
            "wq": _normal(gen, (hd, d), std, dt, device),
            "wk": _normal(gen, (hd, d), std, dt, device),
            "wv": _normal(gen, (hd, d), std, dt, device),
            "wo": _normal(gen, (d, hd), std, dt, device),
            "ffn_norm": gain(),
            "w_gate": _normal(gen, (dff, d), std, dt, device),
            "w_up": _normal(gen, (dff, d), std, dt, device),
            "w_down": _normal(gen, (d, dff), std, dt, device),
        })
    w["final_norm"] = gain()
    w["lm_head"] = _normal(gen, (V, d), std, dt, device)
    return w


def weights_to_numpy64(w):
    """The same stored values as fp64 NumPy arrays (a lossless conversion)."""
    def cv(t):
        return t.detach().to("cpu", torch.float64).numpy()
    out = {k: cv(v) for k, v in w.items() if k != "layers"}
    out["layers"] = [{k: cv(v) for k, v in l.items()} for l in w["layers"]]
    return out


def prompt_uniform(seed, n, vocab, mask_id):
    """n token ids uniform over the vocabulary without the mask id."""
    rng = np.random.default_rng(seed)
    ids = rng.integers(0, vocab - 1, size=n, dtype=np.int64)
    ids[ids >= mask_id] += 1
    return ids


def prompt_zipf(seed, n, vocab, mask_id, a=1.1):
    """n token ids with rank r drawn with probability proportional to r^-a over
    ranks 1..vocab-1 (inverse CDF); rank -> id is the identity skipping mask_id."""
    rng = np.random.default_rng(seed)
    ranks = np.arange(1, vocab, dtype=np.float64)
    cdf = np.cumsum(ranks ** (-a))
    cdf /= cdf[-1]
    r = np.searchsorted(cdf, rng.random(n), side="left")
    ids = r.astype(np.int64)
    ids[ids >= mask_id] += 1
    return ids


def active_positions(seed, N, M):
    """M distinct positions of 0..N-1 drawn uniformly from the seed, ascending."""
    rng = np.random.default_rng(seed)
    return np.sort(rng.permutation(N)[:M]).astype(np.int64)


def lock_mask_from_active(N, active):
    lock = np.ones(N, dtype=np.uint8)
    lock[np.asarray(active)] = 0
    return lock


def linear_m_schedule(M_start, M_end, T):
    """Target number of active rows at the START of step t = 1..T, falling
    linearly from M_start to M_end."""
    if T == 1:
        return [M_start]
    return [int(round(M_start - (M_start - M_end) * t / (T - 1))) for t in range(T)]


def forced_lock_positions(priority, lock, masked, n_lock):
    """The n_lock eligible (unlocked and unmasked) positions of smallest priority.
    Stands in for the convergence a trained model would show: with random weights
    posteriors never settle, so a seeded schedule grows the lock mask instead."""
    elig = [i for i in range(len(lock)) if not lock[i] and not masked[i]]
    elig.sort(key=lambda i: priority[i])
    return elig[:max(0, n_lock)]


def gaussian_rows(seed, rows, cols, storage, std=1.0):
    gen = torch.Generator().manual_seed(int(seed))
    return (torch.empty(rows, cols).normal_(0.0, std, generator=gen)).to(torch_dtype(storage))
