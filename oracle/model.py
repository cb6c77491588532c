"""Transformer-block arithmetic of the oracle (test infrastructure, fp64 NumPy).

The paper treats the network as an L-block bidirectional Transformer whose
per-position work is Q/K/V/Out projections, QK^T and AV, and a three-matrix
FFN (Sec. 2.4, the terms of the baseline FLOP count).  It does not fix the
block's details; the reading taken here is the LLaDA/LLaMA-style block:
pre-RMSNorm, rotary position embedding on q and k (half-split pairing,
position = the row's fixed slot, footnote 1), softmax(QK^T/sqrt(d_h))V with no
mask, SwiGLU FFN, two residual adds, a final RMSNorm and an untied LM head,
no biases.  That reading is pinned structurally (hand-worked two-position
block in scalar arithmetic, zero output projections leave the stream unchanged,
gate/up are not interchangeable, the final gain shows in the logits: the block
tests of the CPU suite); what cannot be pinned is agreement with the authors'
own block, of which the paper prints no value: parity unpinned in that sense.

Weights use the ``[out_features, in_features]`` convention: y = x @ W.T.
"""
from dataclasses import dataclass

import numpy as np

from .rounding import STORAGE


@dataclass(frozen=True)
class Config:
    n_layers: int
    d_model: int
    n_heads: int
    d_head: int
    d_ff: int
    vocab: int
    mask_id: int
    rms_eps: float = 1e-5
    rope_theta: float = 10000.0
    storage: str = "bf16"          # "bf16" | "fp32": type tensors are stored in

    @property
    def rnd(self):
        return STORAGE[self.storage]


def rmsnorm(x, g, eps):
    """x / sqrt(mean(x^2) + eps) * g, row-wise."""
    ms = np.mean(x * x, axis=-1, keepdims=True)
    return x / np.sqrt(ms + eps) * g


def rope(x, pos, theta):
    """Rotate head vectors x[..., H, d_h] at integer slot positions pos[...].

    Half-split pairing: dimension j is paired with j + d_h/2 and the pair is
    rotated by the angle pos * theta**(-2j/d_h), j = 0 .. d_h/2-1.
    """
    dh = x.shape[-1]
    half = dh // 2
    j = np.arange(half, dtype=np.float64)
    inv_freq = theta ** (-2.0 * j / dh)
    ang = np.asarray(pos, dtype=np.float64)[:, None] * inv_freq[None, :]   # [R, half]
    c, s = np.cos(ang)[:, None, :], np.sin(ang)[:, None, :]                # [R,1,half]
    x1, x2 = x[..., :half], x[..., half:]
    return np.concatenate([x1 * c - x2 * s, x2 * c + x1 * s], axis=-1)


def silu(x):
    return x / (1.0 + np.exp(-x))


def attention_rows(q, K, V):
    """Bidirectional softmax attention for a subset of query rows.

    q: [M, H, d_h] queries of the active rows; K, V: [N, H, d_h] keys/values of
    ALL N slots (live and cached alike, Sec. 2.1).  No mask.  Returns [M, H, d_h].
    """
    dh = q.shape[-1]
    s = np.einsum("mhd,nhd->hmn", q, K) / np.sqrt(dh)
    s = s - s.max(axis=-1, keepdims=True)
    p = np.exp(s)
    p = p / p.sum(axis=-1, keepdims=True)
    return np.einsum("hmn,nhd->mhd", p, V)


def layer_active(cfg, w, x, pos, Kc, Vc, write_cache=True):
    """One Transformer block on the active rows only (Alg. 1, the loop body).

    x: [M, d] block input of the active rows; pos: [M] their slot indices;
    Kc, Vc: [N, H, d_h] this layer's key/value table, updated IN PLACE at the
    active slots (the 'assemble' line of Alg. 1: live K/V for active rows,
    cached K/V for locked rows, which this function never touches).
    write_cache=False is the read-only probe of App. 'Optional Unlocking': the
    rows' queries attend to the table as it stands (their own entries included)
    and nothing is written.
    Returns the block output for the active rows.
    """
    rnd = cfg.rnd
    H, dh = cfg.n_heads, cfg.d_head
    M = x.shape[0]
    h = rnd(rmsnorm(x, w["attn_norm"], cfg.rms_eps))
    q = (h @ w["wq"].T).reshape(M, H, dh)
    k = (h @ w["wk"].T).reshape(M, H, dh)
    v = (h @ w["wv"].T).reshape(M, H, dh)
    q = rnd(rope(q, pos, cfg.rope_theta))
    k = rnd(rope(k, pos, cfg.rope_theta))
    v = rnd(v)
    if write_cache:
        Kc[pos] = k
        Vc[pos] = v
    o = rnd(attention_rows(q, Kc, Vc)).reshape(M, H * dh)
    x = rnd(x + o @ w["wo"].T)
    h2 = rnd(rmsnorm(x, w["ffn_norm"], cfg.rms_eps))
    a = rnd(silu(h2 @ w["w_gate"].T) * (h2 @ w["w_up"].T))
    x = rnd(x + a @ w["w_down"].T)
    return x


def lm_head(cfg, weights, x):
    """Final RMSNorm and output projection: logits for the given rows."""
    rnd = cfg.rnd
    hf = rnd(rmsnorm(x, weights["final_norm"], cfg.rms_eps))
    return rnd(hf @ weights["lm_head"].T)


def forward_active(cfg, weights, tokens, active_pos, Kc, Vc, write_cache=True):
    """Restricted forward of Alg. 1: embeddings of the active rows through all
    L blocks and the LM head.  Kc, Vc: lists (one per layer) of [N, H, d_h]
    tables, updated in place at the active slots (left untouched with
    write_cache=False).  Returns logits [M, V].
    """
    x = weights["emb"][np.asarray(tokens)[active_pos]]
    for l in range(cfg.n_layers):
        x = layer_active(cfg, weights["layers"][l], x, active_pos, Kc[l], Vc[l], write_cache)
    return lm_head(cfg, weights, x)


def forward_full(cfg, weights, tokens):
    """The standard sampler's forward: every one of the N positions recomputed,
    no cache, no index sets (Sec. 2, 'each step recomputes self-attention and
    FFN for all tokens').  Written without the cache machinery on purpose so it
    can pin forward_active.  Returns (logits [N, V], K list, V list).
    """
    rnd = cfg.rnd
    N = len(tokens)
    H, dh = cfg.n_heads, cfg.d_head
    pos = np.arange(N)
    x = weights["emb"][np.asarray(tokens)]
    Ks, Vs = [], []
    for l in range(cfg.n_layers):
        w = weights["layers"][l]
        h = rnd(rmsnorm(x, w["attn_norm"], cfg.rms_eps))
        q = rnd(rope((h @ w["wq"].T).reshape(N, H, dh), pos, cfg.rope_theta))
        k = rnd(rope((h @ w["wk"].T).reshape(N, H, dh), pos, cfg.rope_theta))
        v = rnd((h @ w["wv"].T).reshape(N, H, dh))
        Ks.append(k)
        Vs.append(v)
        o = np.empty((N, H, dh))
        for hd in range(H):
            s = q[:, hd, :] @ k[:, hd, :].T / np.sqrt(dh)
            s = s - s.max(axis=1, keepdims=True)
            p = np.exp(s)
            p /= p.sum(axis=1, keepdims=True)
            o[:, hd, :] = p @ v[:, hd, :]
        o = rnd(o).reshape(N, H * dh)
        x = rnd(x + o @ w["wo"].T)
        h2 = rnd(rmsnorm(x, w["ffn_norm"], cfg.rms_eps))
        a = rnd(silu(h2 @ w["w_gate"].T) * (h2 @ w["w_up"].T))
        x = rnd(x + a @ w["w_down"].T)
    return lm_head(cfg, weights, x), Ks, Vs
