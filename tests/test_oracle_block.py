"""Structural pins of the oracle's Transformer block (model.layer_active, model.forward_full,
model.forward_active, model.lm_head) against the mathematics of the block the GEMM terms of
Sec. 2.4 belong to: pre-norm, two residual adds, silu(gate) * up, final norm before the LM head.

The restricted and the full forward repeat the same block formula, so agreeing with each other
says nothing about a mistake both share (a dropped residual, gate and up swapped, a missing
final norm, a norm applied to the residual stream instead of the branch).  Every case here has an
expected value that does not come from either of them: exact identities, and a two-position,
two-dimensional block worked through with scalar arithmetic."""
import math

import numpy as np
import pytest

from oracle import model
from oracle.model import Config


def _cfg(L=1, d=2, H=1, dh=2, dff=2, V=3, eps=0.0, storage="fp64"):
    return Config(L, d, H, dh, dff, V, V - 1, eps, 10000.0, storage)


def _rand_layer(rng, d, hd, dff, scale=0.5):
    return {"attn_norm": 1.0 + 0.3 * rng.standard_normal(d), "ffn_norm": 1.0 + 0.3 * rng.standard_normal(d),
            "wq": scale * rng.standard_normal((hd, d)), "wk": scale * rng.standard_normal((hd, d)),
            "wv": scale * rng.standard_normal((hd, d)), "wo": scale * rng.standard_normal((d, hd)),
            "w_gate": scale * rng.standard_normal((dff, d)), "w_up": scale * rng.standard_normal((dff, d)),
            "w_down": scale * rng.standard_normal((d, dff))}


def _weights(rng, cfg, layers):
    return {"emb": rng.standard_normal((cfg.vocab, cfg.d_model)), "layers": layers,
            "final_norm": 1.0 + 0.3 * rng.standard_normal(cfg.d_model),
            "lm_head": rng.standard_normal((cfg.vocab, cfg.d_model))}


def _tables(cfg, N):
    return (np.zeros((N, cfg.n_heads, cfg.d_head)), np.zeros((N, cfg.n_heads, cfg.d_head)))


# ------------------------------------------------------------------ the worked example
# d = 2, one head of 2 dims, d_ff = 2, two positions (slots 0 and 1), no rounding, rms_eps = 0.
#   x0 = (7, 1), x1 = (1, 7):  mean square 25, rms 5  ->  h0 = (1.4, 0.2), h1 = (0.2, 1.4)  (gain 1)
#   Wq = Wk = I, Wv = [[1, 0], [0, 2]]:  q = k = h,  v0 = (1.4, 0.4), v1 = (0.2, 2.8)
#   RoPE, d_h = 2: one pair (dims 0, 1), angle = slot * theta^0 = slot: slot 0 unrotated, slot 1 by 1 rad
#   scores s_ij = q_i . k_j / sqrt(2), softmax over j in {0, 1}, o_i = sum_j p_ij v_j
#   Wo = [[0, 1], [1, 0]] (swaps the two dims):  x' = x + (o[1], o[0])
#   second branch: h' = x' / rms(x') * (2, 1)   (ffn gain (2, 1))
#   W_gate = [[1, 0], [0, 1]], W_up = [[0, 1], [1, 0]]:  g = h', u = (h'[1], h'[0]),  a = silu(g) * u
#   W_down = [[1, 1], [1, -1]]:  out = x' + (a0 + a1, a0 - a1)
HAND_LAYER = {"attn_norm": np.array([1.0, 1.0]), "ffn_norm": np.array([2.0, 1.0]),
              "wq": np.eye(2), "wk": np.eye(2), "wv": np.array([[1.0, 0.0], [0.0, 2.0]]),
              "wo": np.array([[0.0, 1.0], [1.0, 0.0]]),
              "w_gate": np.eye(2), "w_up": np.array([[0.0, 1.0], [1.0, 0.0]]),
              "w_down": np.array([[1.0, 1.0], [1.0, -1.0]])}
HAND_X = np.array([[7.0, 1.0], [1.0, 7.0]])


def _hand_block(silu_on_gate=True):
    """The example above in scalar arithmetic (math module only).  Returns (out rows, k rows, v rows)."""
    h = [(1.4, 0.2), (0.2, 1.4)]
    for (a, b), (x0, x1) in zip(h, HAND_X):
        r = math.sqrt((x0 * x0 + x1 * x1) / 2.0)
        assert abs(a - x0 / r) < 1e-15 and abs(b - x1 / r) < 1e-15
    c, s = math.cos(1.0), math.sin(1.0)
    q = [h[0], (h[1][0] * c - h[1][1] * s, h[1][1] * c + h[1][0] * s)]
    k = q
    v = [(1.4, 0.4), (0.2, 2.8)]
    out = []
    for i in range(2):
        sc = [(q[i][0] * k[j][0] + q[i][1] * k[j][1]) / math.sqrt(2.0) for j in range(2)]
        e = [math.exp(t - max(sc)) for t in sc]
        p = [t / sum(e) for t in e]
        o = (p[0] * v[0][0] + p[1] * v[1][0], p[0] * v[0][1] + p[1] * v[1][1])
        x1 = (HAND_X[i][0] + o[1], HAND_X[i][1] + o[0])
        r = math.sqrt((x1[0] ** 2 + x1[1] ** 2) / 2.0)
        hp = (x1[0] / r * 2.0, x1[1] / r * 1.0)
        g, u = hp, (hp[1], hp[0])
        if not silu_on_gate:
            g, u = u, g
        a = tuple(gg / (1.0 + math.exp(-gg)) * uu for gg, uu in zip(g, u))
        out.append((x1[0] + a[0] + a[1], x1[1] + a[0] - a[1]))
    return np.array(out), np.array(k), np.array(v)


def test_worked_block_layer_active_and_forward_full():
    cfg = _cfg()
    want, k_want, v_want = _hand_block()
    # anchors of the example that can be checked by eye: attention pulls row 0 towards v0, whose
    # second component lands (through Wo's swap) on the first dim
    assert want[0][0] > 7.0 and not np.allclose(want, _hand_block(silu_on_gate=False)[0])
    Kc, Vc = _tables(cfg, 2)
    got = model.layer_active(cfg, HAND_LAYER, HAND_X.copy(), np.arange(2), Kc, Vc)
    assert np.allclose(got, want, rtol=1e-13, atol=0)
    assert np.allclose(Kc[:, 0, :], k_want, rtol=1e-14) and np.allclose(Vc[:, 0, :], v_want, rtol=1e-14)
    # the same block through forward_full / forward_active: logits = rmsnorm(out) * g_f . W_out^T
    gf, Wl = np.array([0.5, 3.0]), np.array([[1.0, 0.0], [0.0, 1.0], [1.0, 1.0]])
    w = {"emb": HAND_X, "layers": [HAND_LAYER], "final_norm": gf, "lm_head": Wl}
    z_want = []
    for row in want:
        r = math.sqrt((row[0] ** 2 + row[1] ** 2) / 2.0)
        n0, n1 = row[0] / r * 0.5, row[1] / r * 3.0
        z_want.append((n0, n1, n0 + n1))
    z_full, Ks, Vs = model.forward_full(cfg, w, np.array([0, 1]))
    assert np.allclose(z_full, z_want, rtol=1e-13)
    assert np.allclose(Ks[0][:, 0, :], k_want, rtol=1e-14) and np.allclose(Vs[0][:, 0, :], v_want, rtol=1e-14)
    Kc, Vc = _tables(cfg, 2)
    z_act = model.forward_active(cfg, w, np.array([0, 1]), np.arange(2), [Kc], [Vc])
    assert np.allclose(z_act, z_want, rtol=1e-13)


def test_worked_block_one_active_row_reads_the_other_from_the_cache():
    """Row 1 alone, row 0's K/V already in the tables: same value for row 1 as in the two-row example,
    and row 0's table entries stay as they were."""
    cfg = _cfg()
    want, k_want, v_want = _hand_block()
    Kc, Vc = _tables(cfg, 2)
    Kc[0, 0], Vc[0, 0] = k_want[0], v_want[0]
    got = model.layer_active(cfg, HAND_LAYER, HAND_X[1:2].copy(), np.array([1]), Kc, Vc)
    assert np.allclose(got[0], want[1], rtol=1e-13)
    assert np.array_equal(Kc[0, 0], k_want[0]) and np.array_equal(Vc[0, 0], v_want[0])


# ------------------------------------------------------------------ identities (random weights)
@pytest.mark.parametrize("storage", ["fp64", "bf16"])
def test_zero_out_and_down_projections_make_the_block_the_identity(storage):
    rng = np.random.default_rng(0)
    cfg = _cfg(L=3, d=8, H=2, dh=4, dff=6, V=16, eps=1e-5, storage=storage)
    layers = [_rand_layer(rng, 8, 8, 6) for _ in range(3)]
    for l in layers:
        l["wo"][:] = 0.0
        l["w_down"][:] = 0.0
    w = _weights(rng, cfg, layers)
    w["emb"] = cfg.rnd(w["emb"])
    tok = rng.integers(0, 16, 5)
    x = w["emb"][tok]
    Kc, Vc = _tables(cfg, 5)
    assert np.array_equal(model.layer_active(cfg, layers[0], x.copy(), np.arange(5), Kc, Vc), x)
    # all three blocks are the identity, so the logits are the LM head of the embeddings
    want = model.lm_head(cfg, w, x)
    z_full, _, _ = model.forward_full(cfg, w, tok)
    assert np.array_equal(z_full, want)
    tabs = [_tables(cfg, 5) for _ in range(3)]
    z_act = model.forward_active(cfg, w, tok, np.arange(5), [t[0] for t in tabs], [t[1] for t in tabs])
    assert np.array_equal(z_act, want)


def test_each_branch_is_added_to_the_unnormalised_stream():
    """Pre-norm with rms_eps = 0: both branches see only the direction of their input, so scaling the
    block input by c > 0 scales nothing but the residual stream itself when the first branch is off,
    and the first branch's increment does not depend on c either."""
    rng = np.random.default_rng(1)
    cfg = _cfg(d=8, H=2, dh=4, dff=6, V=16)
    lay = _rand_layer(rng, 8, 8, 6)
    x = rng.standard_normal((4, 8))
    pos = np.arange(4)
    only_attn = dict(lay, w_down=np.zeros_like(lay["w_down"]))
    inc1 = model.layer_active(cfg, only_attn, x.copy(), pos, *_tables(cfg, 4)) - x
    inc3 = model.layer_active(cfg, only_attn, 3.0 * x, pos, *_tables(cfg, 4)) - 3.0 * x
    assert np.abs(inc1).max() > 1e-2 and np.allclose(inc1, inc3, rtol=1e-12, atol=1e-13)
    only_ffn = dict(lay, wo=np.zeros_like(lay["wo"]))
    f1 = model.layer_active(cfg, only_ffn, x.copy(), pos, *_tables(cfg, 4)) - x
    f3 = model.layer_active(cfg, only_ffn, 3.0 * x, pos, *_tables(cfg, 4)) - 3.0 * x
    assert np.abs(f1).max() > 1e-2 and np.allclose(f1, f3, rtol=1e-12, atol=1e-13)


def test_ffn_branch_reads_the_stream_after_the_attention_add():
    """out = x' + FFN(norm(x')), x' = x + attention branch: the second increment, recomputed from
    primitives on x', must be what the block adds."""
    rng = np.random.default_rng(2)
    cfg = _cfg(d=8, H=2, dh=4, dff=6, V=16, eps=1e-5)
    lay = _rand_layer(rng, 8, 8, 6)
    x = rng.standard_normal((4, 8))
    pos = np.arange(4)
    x_mid = model.layer_active(cfg, dict(lay, w_down=np.zeros_like(lay["w_down"])), x.copy(), pos, *_tables(cfg, 4))
    out = model.layer_active(cfg, lay, x.copy(), pos, *_tables(cfg, 4))
    ffn = np.zeros_like(x)
    for r in range(4):                                    # scalar loops, no shared helper
        ms = sum(float(t) ** 2 for t in x_mid[r]) / 8.0
        hn = [float(x_mid[r, c]) / math.sqrt(ms + 1e-5) * float(lay["ffn_norm"][c]) for c in range(8)]
        a = []
        for j in range(6):
            g = sum(lay["w_gate"][j, c] * hn[c] for c in range(8))
            u = sum(lay["w_up"][j, c] * hn[c] for c in range(8))
            a.append(g / (1.0 + math.exp(-g)) * u)
        for c in range(8):
            ffn[r, c] = sum(lay["w_down"][c, j] * a[j] for j in range(6))
    assert np.allclose(out - x_mid, ffn, rtol=1e-11, atol=1e-13)
    assert np.abs(x_mid - x).max() > 1e-2                 # the attention branch did contribute


def test_swapping_gate_and_up_changes_the_block():
    rng = np.random.default_rng(3)
    cfg = _cfg(d=8, H=2, dh=4, dff=6, V=16, eps=1e-5)
    lay = _rand_layer(rng, 8, 8, 6)
    x = rng.standard_normal((4, 8))
    a = model.layer_active(cfg, lay, x.copy(), np.arange(4), *_tables(cfg, 4))
    b = model.layer_active(cfg, dict(lay, w_gate=lay["w_up"], w_up=lay["w_gate"]), x.copy(), np.arange(4), *_tables(cfg, 4))
    assert np.abs(a - b).max() > 1e-3


def test_final_norm_and_its_gain_show_in_the_logits():
    rng = np.random.default_rng(4)
    cfg = _cfg(d=8, H=2, dh=4, dff=6, V=16, eps=0.0)
    w = _weights(rng, cfg, [])
    x = rng.standard_normal((3, 8))
    z = model.lm_head(cfg, w, x)
    # the norm: logits do not change with the scale of the final block output
    assert np.allclose(model.lm_head(cfg, w, 5.0 * x), z, rtol=1e-12)
    # the gain: element c of it multiplies column c of the output matrix
    w2 = dict(w, final_norm=w["final_norm"] * np.arange(1, 9), lm_head=w["lm_head"] / np.arange(1, 9))
    assert np.allclose(model.lm_head(cfg, w2, x), z, rtol=1e-12)
    w3 = dict(w, final_norm=2.0 * w["final_norm"])
    assert np.allclose(model.lm_head(cfg, w3, x), 2.0 * z, rtol=1e-12)
    # value: z[r, v] = sum_c x[r, c] / rms_r * g[c] * W[v, c]
    r, v = 1, 5
    rms = math.sqrt(sum(float(t) ** 2 for t in x[r]) / 8.0)
    want = sum(float(x[r, c]) / rms * float(w["final_norm"][c]) * float(w["lm_head"][v, c]) for c in range(8))
    assert abs(z[r, v] - want) <= 1e-12 * abs(want)


def test_layers_are_applied_in_order_with_their_own_weights():
    """Two different blocks do not commute; forward_full over [A, B] equals layer B applied to layer
    A's output (every row live), and differs from [B, A]."""
    rng = np.random.default_rng(5)
    cfg2 = _cfg(L=2, d=8, H=2, dh=4, dff=6, V=16, eps=1e-5)
    A, Bl = _rand_layer(rng, 8, 8, 6), _rand_layer(rng, 8, 8, 6)
    w = _weights(rng, cfg2, [A, Bl])
    tok = rng.integers(0, 16, 4)
    x = w["emb"][tok]
    pos = np.arange(4)
    xa = model.layer_active(cfg2, A, x.copy(), pos, *_tables(cfg2, 4))
    xb = model.layer_active(cfg2, Bl, xa, pos, *_tables(cfg2, 4))
    z, _, _ = model.forward_full(cfg2, w, tok)
    assert np.allclose(z, model.lm_head(cfg2, w, xb), rtol=1e-12)
    z_swapped, _, _ = model.forward_full(cfg2, dict(w, layers=[Bl, A]), tok)
    assert np.abs(z - z_swapped).max() > 1e-3
