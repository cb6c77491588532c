"""GPU parity at the full size of the 32-layer configurations (LLaDA-8B shape: 32 layers, d = 4096,
32 x 128 heads, FFN 12288, vocabulary 126464; 16 GB of random bf16 weights).

The oracle cannot run 32 full layers on every row in test time, so it checks sampled outputs it CAN
compute one by one, each from the GPU's own inputs to that stage:
  * layers: the GPU runs the stack one layer at a time (sl_forward_layers); for sampled layers and
    sampled rows the oracle recomputes the block from the row's block input and the layer's K/V
    cache (both read back from the GPU) and compares the K/V rows the GPU wrote and the block output;
  * LM head + scoring: the whole step (sl_surelock_step) on the same state; the oracle applies the
    final norm and LM head to the sampled rows' last block output, and log-softmax / KL / confidence
    / argmax to the GPU's logits of those rows;
  * controller: compaction, UpdateMASK and the lock rule are integer work, recomputed in full from the
    GPU's conf / argmax / KL with the oracle's controller functions.
Tolerance on a block output element: one bf16 spacing at its magnitude + 1.5e-2 of the row's rms, and
a mean error below 4e-3 of the rms.  Both sides round the same six tensors per block to bf16, but
accumulate in fp32 / fp64; a value on a rounding boundary lands one spacing (2^-8 relative) apart,
and such differences multiply through the block: ~0.3 % of the attention outputs differ, which moves
~5 % of the (small, early-layer) residual entries by a spacing, which shifts the FFN pre-activations
by ~5e-4 relative and flips ~15 % of the silu(g)*u entries, which ends as a ~1e-3 relative difference
in the block output before its own rounding (measured: mean 0.6e-3 .. 2.1e-3 of the rms, largest
element 8.6e-3 over ~4e5 sampled).  A wrong operand, index or missing term shows as O(0.1 .. 1) of the rms."""
import numpy as np
import pytest
import torch

from oracle import control, model, posterior
from paper_2602_06412_amd import binding as B
from paper_2602_06412_amd import workloads as wl
from tests.gpu_util import DEV, bf16_ulp, check_logits, dev, oracle_cfg

pytestmark = [pytest.mark.gpu, pytest.mark.timeout(900)]

f64 = lambda t: t.detach().to("cpu", torch.float64).numpy()
CHECK_LAYERS = (0, 1, 13, 31)


def _kv_candidates(cfg, w64, x_row, pos):
    """The K/V cache rows the precision contract admits for one block input row.

    The normalised input h = rnd(rmsnorm(x)) is x times ONE factor r per row, and x holds bf16 values (8-bit
    mantissas): for some r a whole group of elements (all with the same mantissa) lands on bf16 rounding
    boundaries at once, and an fp32 evaluation of r (relative error up to ~3e-7) rounds that group the other
    way.  About one row in a thousand is affected (measured on the CPU: fp32 against fp64 RMSNorm of bf16 rows at
    d = 4096, ~45 elements flip together), and then every element of the row's K and V moves by about
    spacing x |w| x sqrt(45) ~ 1e-3, far beyond one spacing of the small ones.  Both roundings are correct
    evaluations of the contract, so for such a row the K/V of either side of the boundary is accepted; for all
    other rows this is the single oracle row."""
    rnd, H, dh = cfg.rnd, cfg.n_heads, cfg.d_head
    hn = model.rmsnorm(x_row[None], w64["attn_norm"], cfg.rms_eps)
    out, seen = [], []
    for f in (1.0, 1.0 - 3e-7, 1.0 + 3e-7):
        h = rnd(hn * f)
        if any(np.array_equal(h, s_) for s_ in seen):
            continue
        seen.append(h)
        k = rnd(model.rope((h @ w64["wk"].T).reshape(1, H, dh), np.array([pos]), cfg.rope_theta))[0]
        v = rnd((h @ w64["wv"].T).reshape(1, H, dh))[0]
        out.append((k, v))
    return out


def _run_case(Bn, N, prompts, n_prompt, eps_list, schedule, block, seed, n_masked=None):
    """schedule: per step a list of per-sequence active counts (nested forced locks; a count below the
    number of lockable, i.e. unmasked, positions is met as far as those go).
    n_masked: generation slots still masked at the first step (default: all); the others already hold
    seeded token ids, the state late in a schedule, where most positions can lock."""
    shape = wl.C3
    cfg = oracle_cfg(shape)
    w = wl.make_weights(shape, seed=seed, device="cuda")
    sess = B.Session(shape, w, Bn, N)
    rng = np.random.default_rng(seed)
    try:
        tokens = np.full((Bn, N), shape.mask_id, dtype=np.int64)
        masked = np.ones((Bn, N), dtype=np.uint8)
        for b in range(Bn):
            tokens[b, :n_prompt] = prompts[b]
            masked[b, :n_prompt] = 0
            if n_masked is not None:
                done = N - n_masked
                tokens[b, n_prompt:done] = wl.prompt_uniform(seed * 10 + b, done - n_prompt, shape.vocab, shape.mask_id)
                masked[b, n_prompt:done] = 0
        lock = np.zeros((Bn, N), dtype=np.uint8)
        pri = [np.random.default_rng(seed * 100 + b).permutation(N) for b in range(Bn)]
        eps_d = dev(np.asarray(eps_list, dtype=np.float32))
        lm64 = fn64 = None
        for t, counts in enumerate(schedule, start=1):
            # forced locks (the seeded stand-in for convergence): shrink each sequence to its count
            for b in range(Bn):
                n_lock = int((lock[b] == 0).sum()) - counts[b]
                for i in wl.forced_lock_positions(pri[b], lock[b], masked[b], n_lock):
                    lock[b, i] = 1
            active, cu = control.compact_active(lock)
            M = len(active)
            print(f"32-layer case B={Bn} N={N} step t={t} M={M} per-seq {np.diff(cu).tolist()}", flush=True)
            tok_d, msk_d, lock_d = dev(tokens.reshape(-1), torch.int32), dev(masked.reshape(-1)), dev(lock.reshape(-1))
            # ---- the stack, one layer at a time, with sampled checks
            idx_d = dev(active, torch.int32)
            m_dev = dev(np.array([M], dtype=np.int32))
            x = w["emb"][tok_d.long()[idx_d.long()]].contiguous()
            sample = np.sort(rng.choice(M, size=min(M, 4), replace=False))
            rows_d = torch.as_tensor(sample, device=DEV, dtype=torch.long)
            for l in range(shape.n_layers):
                x_next = sess.forward_layers(x, idx_d, m_dev, M, l, l + 1)
                if l in CHECK_LAYERS:
                    torch.cuda.synchronize()
                    wl64 = {k: f64(v) for k, v in w["layers"][l].items()}
                    kg, vg = sess.kv_read(l)
                    x_in, x_out = f64(x[rows_d]), f64(x_next[rows_d])
                    for j, r in enumerate(sample):
                        b, i = divmod(int(active[r]), N)
                        Kc, Vc = f64(kg[b]), f64(vg[b])
                        k_gpu, v_gpu = Kc[i].copy(), Vc[i].copy()
                        want = model.layer_active(cfg, wl64, x_in[j:j + 1], np.array([i]), Kc, Vc)[0]
                        cands = _kv_candidates(cfg, wl64, x_in[j], i)
                        if len(cands) > 1:
                            print(f"layer {l} row {r}: normalised input sits on bf16 rounding boundaries, "
                                  f"{len(cands)} admissible K/V rows", flush=True)
                        for got, c, what in ((k_gpu, 0, "K"), (v_gpu, 1, "V")):
                            # one bf16 spacing, plus the fp32 accumulation noise of a 4096-term dot product
                            # that cancels to nearly zero (2^-24 x sum |h w| ~ 3e-6), against any admissible row
                            bad = []
                            for cand in cands:
                                ref = cand[c]
                                e = np.abs(got - ref)
                                bad.append(int((e > bf16_ulp(ref) + 1e-5).sum()))
                            ref = cands[0][c]
                            e = np.abs(got - ref)
                            a = np.unravel_index(int(np.argmax(e / bf16_ulp(ref))), e.shape)
                            assert min(bad) == 0, (
                                f"layer {l} row {r}: cached {what} {a}: got {got[a]!r} want {ref[a]!r}, "
                                f"{bad} of {e.size} beyond one spacing (per admissible row)")
                        err, rms = np.abs(x_out[j] - want), np.sqrt(np.mean(want ** 2))
                        tol = bf16_ulp(want) + 1.5e-2 * rms
                        assert np.all(err <= tol), f"layer {l} row {r}: block output off by {np.max(err / tol):.2f} x tolerance"
                        assert err.mean() <= 4e-3 * rms, f"layer {l} row {r}: mean error {err.mean() / rms:.2e} of the row rms"
                    del wl64
                x = x_next
            # ---- the whole step on the same state
            new_lock = torch.zeros_like(lock_d)
            lo, hi, k = block
            sess.step(tok_d, msk_d, lock_d, eps_d, t, lo, hi, k, m_upper=M, new_lock=new_lock)
            torch.cuda.synchronize()
            assert np.array_equal(sess.cu_active.cpu().numpy(), cu)
            assert np.array_equal(sess.active_idx[:M].cpu().numpy(), active)
            if lm64 is None:
                lm64, fn64 = f64(w["lm_head"]), f64(w["final_norm"])
            hf = cfg.rnd(model.rmsnorm(f64(x[rows_d]), fn64, cfg.rms_eps))
            z = cfg.rnd(hf @ lm64.T)
            flat = torch.as_tensor(active[sample], device=DEV, dtype=torch.long)
            z_gpu = sess.logits_view(t)[flat].double().cpu().numpy()
            check_logits(z_gpu, z, "bf16", f"32-layer t={t}")
            lp = posterior.log_softmax(z_gpu)
            conf_g = sess.conf[:M].cpu().numpy()
            am_g = sess.argmax[:M].cpu().numpy()
            kl_g = sess.kl[:M].cpu().numpy()
            assert np.array_equal(am_g[sample], posterior.argmax_lowest(z_gpu))
            assert np.allclose(conf_g[sample], posterior.max_prob(lp), rtol=2e-6)
            if t > 1:
                prev = sess.logits_view(t - 1)[flat].double().cpu().numpy()
                want = posterior.kl_rows(lp, posterior.log_softmax(prev))
                assert np.all(np.abs(kl_g[sample].astype(np.float64) - want) <= 1e-4 * want + 2e-7)
            else:
                assert np.all(np.isinf(kl_g))
            # ---- controller, in full, from the GPU's scores
            tok_out, msk_out = tok_d.cpu().numpy().reshape(Bn, N), msk_d.cpu().numpy().reshape(Bn, N)
            lock_out = new_lock.cpu().numpy().reshape(Bn, N)
            for b in range(Bn):
                r0, r1 = cu[b], cu[b + 1]
                pos = active[r0:r1] - b * N
                tk, mk = tokens[b].copy(), masked[b].copy()
                control.update_mask(mk, tk, pos, conf_g[r0:r1], am_g[r0:r1], lo, hi, k)
                assert np.array_equal(mk, msk_out[b]) and np.array_equal(tk, tok_out[b])
                F = control.lock_rule(lock[b], mk, pos, kl_g[r0:r1], 1.0 - conf_g[r0:r1], np.float32(eps_list[b]), t == 1)
                want_lock = lock[b].copy()
                want_lock[F] = 1
                near = np.abs(kl_g[r0:r1].astype(np.float64) - eps_list[b]) <= 1e-6
                ok = want_lock == lock_out[b]
                ok[pos[near]] = True
                assert np.all(ok)
                tokens[b], masked[b] = tk, mk
            lock = np.maximum(lock, lock_out)      # the rule's locks join the forced ones
    finally:
        sess.close()
        del w
        torch.cuda.empty_cache()


def test_c3_shape_32_layers_single_sequence():
    """N = 512 (256 uniform prompt tokens + 256 [MASK]), blocks of 32, one token per step."""
    N, n_p = 512, 256
    prompts = [wl.prompt_uniform(11, n_p, wl.C3.vocab, wl.C3.mask_id)]
    _run_case(1, N, prompts, n_p, [1e-3], [[512], [384], [40]], (n_p, n_p + 32, 1), seed=3)


def test_c5_shape_32_layers_ragged_batch():
    """Config 5 at its own batch size: eight sequences of N = 1024 (512 Zipf(1.1) prompt tokens + 512 [MASK]),
    per-sequence thresholds {1e-4, 1e-3, 1e-2}[b mod 3] and different active counts per sequence: packed
    varlen rows (8192, then 4841, then 1328 in total) through all 32 layers.  All but the last 64 slots of
    each sequence are already unmasked, so that the per-sequence counts (down to one row) can be met."""
    N, n_p, Bn = 1024, 512, 8
    prompts = [wl.prompt_zipf(20 + b, n_p, wl.C3.vocab, wl.C3.mask_id) for b in range(Bn)]
    eps = [[1e-4, 1e-3, 1e-2][b % 3] for b in range(Bn)]
    schedule = [[1024] * Bn, [900, 640, 1000, 130, 512, 777, 257, 625], [300, 64, 700, 17, 33, 128, 1, 85]]
    _run_case(Bn, N, prompts, n_p, eps, schedule, (N - 64, N, 1), seed=5, n_masked=64)


def test_c4_shape_32_layers_long_sequence():
    """N = 2048 (1024 prompt + 1024 [MASK]), blocks of 64: 32 key tiles per attention row."""
    N, n_p = 2048, 1024
    prompts = [wl.prompt_uniform(12, n_p, wl.C3.vocab, wl.C3.mask_id)]
    _run_case(1, N, prompts, n_p, [1e-3], [[2048], [1500], [1030]], (n_p, n_p + 64, 1), seed=4)
