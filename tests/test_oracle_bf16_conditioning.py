"""How far apart two correct evaluations of the bf16 model can be: the oracle against itself.

The precision contract rounds every stored tensor to bf16.  A value that lies within the summation
error of a rounding boundary lands on one or the other neighbour depending on how the sum was taken,
a whole spacing (2^-8 .. 2^-7 relative) apart; the next operator sums thousands of such inputs, so
a fraction f of flipped inputs moves its outputs by about sqrt(f) spacings' worth, which flips a
fraction ~sqrt(f) of ITS outputs at the next rounding.  The map f -> ~sqrt(f) has the fixed point
'about half of the values differ by a spacing' and reaches it from any non-zero start within a few
rounding points: the size of the initial difference (fp32 versus fp64 accumulation, about 1e-7, or a
perturbation of 1e-8) only decides how many rounding points it takes.

This is what bounds GPU-versus-oracle logit differences in the multi-layer bf16 configurations, and
the reason their tests state the 2e-2 bound on all but a small tail of the logits.  Shown here on the
CPU with no GPU code involved: the oracle's forward with every rounding preceded by a relative
perturbation of 1e-8, 1e-6 or 1e-4 against the plain forward (a model of this size, 5e4 values per
tensor, needs about 1e-8 for some value to sit close enough to a boundary; the 10^6-value tensors of the
full-size configurations find one at any fp32 summation error)."""
import numpy as np
import pytest

from oracle import model, rounding
from oracle.model import Config


def _perturbed_rounding(rel, seed):
    rng = np.random.default_rng(seed)

    def rnd(x):
        x = np.asarray(x, dtype=np.float64)
        return rounding.round_bf16(x * (1.0 + rel * rng.standard_normal(x.shape)))
    return rnd


def _model(L, seed=0, d=256, H=2, dh=128, dff=768, V=4096):
    rng = np.random.default_rng(seed)
    r = rounding.round_bf16
    layers = [{"attn_norm": np.ones(d), "ffn_norm": np.ones(d),
               "wq": r(0.02 * rng.standard_normal((H * dh, d))), "wk": r(0.02 * rng.standard_normal((H * dh, d))),
               "wv": r(0.02 * rng.standard_normal((H * dh, d))), "wo": r(0.02 * rng.standard_normal((d, H * dh))),
               "w_gate": r(0.02 * rng.standard_normal((dff, d))), "w_up": r(0.02 * rng.standard_normal((dff, d))),
               "w_down": r(0.02 * rng.standard_normal((d, dff)))} for _ in range(L)]
    w = {"emb": r(0.02 * rng.standard_normal((V, d))), "layers": layers, "final_norm": np.ones(d),
         "lm_head": r(0.02 * rng.standard_normal((V, d)))}
    return w, (L, d, H, dh, dff, V)


@pytest.mark.parametrize("L", [6, 12])
def test_two_evaluations_of_the_bf16_model_decorrelate_to_the_rounding_noise(L, monkeypatch):
    w, dims = _model(L, d=512, H=4, dff=1536, V=8192)
    tok = np.random.default_rng(1).integers(0, dims[-1] - 1, 96)
    z0, _, _ = model.forward_full(Config(*dims, dims[-1] - 1, 1e-5, 10000.0, "bf16"), w, tok)
    scale = np.sqrt(np.mean(z0 ** 2))
    level = {}
    for rel in (1e-8, 1e-6, 1e-4):
        monkeypatch.setitem(rounding.STORAGE, "bf16_perturbed", _perturbed_rounding(rel, 7))
        z1, _, _ = model.forward_full(Config(*dims, dims[-1] - 1, 1e-5, 10000.0, "bf16_perturbed"), w, tok)
        e = np.abs(z1 - z0)
        level[rel] = e.mean() / scale
        print(f"L={L}, perturbation {rel:g}: logit rms {scale:.3g}, mean |dz| / rms {level[rel]:.2e}, max |dz| {e.max():.3g} "
              f"over {z0.size} logits, share beyond 2e-2 (at a logit rms of 1.28): {np.mean(e > 2e-2 * scale / 1.28):.2e}")
    # perturbations four orders of magnitude apart end at the same level, that of the bf16 rounding
    # noise (2^-9 .. 2^-8 relative per rounding), i.e. 5 to 6 orders of magnitude above the smallest
    for rel in level:
        assert 2e-3 < level[rel] < 1.2e-2, (rel, level[rel])
    assert level[1e-4] / level[1e-8] < 2.0
