#!/usr/bin/env python3
"""Step latency of the 32-layer configurations along their lock schedules, on one GPU.

    python -m paper_2602_06412_amd.run_config --config c3|c4|c5 [--points 6] [--steps 5]

Random-init LLaDA-8B-shaped bf16 weights (32 layers, d = 4096, 32 x 128 heads, FFN 12288, vocabulary
126464) and seeded synthetic prompts.  Random weights never converge, so the lock mask follows the
configuration's linear schedule of active rows M_t (locked positions chosen by a seeded priority
among prompt and already-unmasked slots); the KL rule still runs inside every step.  The schedule is
sampled at `--points` values of M_t; at each, the state of that moment is built and `--steps` steps
are timed (events on the launch stream) after a warm-up, with a per-kernel split from the
library's profiling hooks.  The last line sums the sampled latencies over the whole schedule
(trapezoid rule) next to the same number of full-recompute steps (M = N), which is the
paper's comparison: algorithmic work saved vs time saved.

bench.py imports ScheduleRunner from here for its recorded line."""
import argparse
import json
import sys

import numpy as np
import torch

from . import binding as B
from . import workloads as wl

CONFIGS = {
    # name: (batch, N, prompt, block, T, per-sequence final active counts, prompt kind, eps)
    "c3": (1, 512, 256, 32, 256, [32], "uniform", [1e-3]),
    "c4": (1, 2048, 1024, 64, 1024, [64], "uniform", [1e-3]),
    "c5": (8, 1024, 512, 512, 512, [64 * (b + 1) for b in range(8)], "zipf", [[1e-4, 1e-3, 1e-2][b % 3] for b in range(8)]),
}
DESCRIBE = {
    "c3": "C3: 32-layer LLaDA-8B shape, B=1, N=512 (256 prompt + 256 generated), blocks of 32, T=256, forced linear M_t 512 -> 32",
    "c4": "C4: 32-layer LLaDA-8B shape, B=1, N=2048 (1024 + 1024), blocks of 64, T=1024, forced linear M_t 2048 -> 64",
    "c5": "C5: 32-layer LLaDA-8B shape, B=8 x N=1024 (512 Zipf(1.1) prompt + 512 generated), T=512, per-sequence eps "
          "{1e-4,1e-3,1e-2}, per-sequence forced linear M_t 1024 -> 64(b+1), packed ragged rows",
}
GROUPS = {"gemm": ["gemm_qkv", "gemm_out", "gemm_gate_up", "gemm_down"], "lm_head": ["lm_head"],
          "attention": ["attention"], "score": ["score"],
          "row-wise": ["embed_norm", "rope_kv", "add_norm", "swiglu"], "control": ["compact", "unmask", "lock_rule"]}
MFMA_BF16_PEAK = 2.5e15      # dense bf16 FLOP/s, MI355X
HBM_PEAK = 8.0e12            # B/s


def state_at(step, Bn, N, n_p, block, T, M_end, pri):
    """tokens-independent part of the sampler state at the start of 1-based step `step`:
    one slot unmasked per earlier step (block order), active counts on the linear schedule."""
    masked = np.zeros((Bn, N), dtype=np.uint8)
    masked[:, n_p + min(step - 1, N - n_p):] = 1
    lock = np.zeros((Bn, N), dtype=np.uint8)
    for b in range(Bn):
        target = wl.linear_m_schedule(N, M_end[b], T)[step - 1]
        elig = np.flatnonzero(masked[b] == 0)
        order = elig[np.argsort(pri[b][elig])]
        lock[b, order[:max(0, N - target)]] = 1
    blk = (step - 1) // block if block < N - n_p else 0
    lo = n_p + blk * block
    return masked, lock, (lo, min(N, lo + block))


def slot_work(shape, N, M):
    """Algorithmic work of one launch of each kernel slot at M active rows in total (Sec. 2.4's terms at this
    shape; the LM head and the scoring pass, which the paper's count leaves out, by their definitions):
    flops for the MFMA-bound slots, bytes for the HBM-bound ones (weights once + activations in and out)."""
    d, dff, hd, V = shape.d_model, shape.d_ff, shape.n_heads * shape.d_head, shape.vocab
    return {
        "gemm_qkv": {"flops": 2.0 * M * d * 3 * hd, "bytes": 2.0 * (3 * hd * d) + 2.0 * M * (d + 3 * hd)},
        "gemm_out": {"flops": 2.0 * M * hd * d, "bytes": 2.0 * (hd * d) + 2.0 * M * (hd + d)},
        "gemm_gate_up": {"flops": 2.0 * M * d * 2 * dff, "bytes": 2.0 * (2 * dff * d) + 2.0 * M * (d + dff)},
        "gemm_down": {"flops": 2.0 * M * dff * d, "bytes": 2.0 * (dff * d) + 2.0 * M * (dff + d)},
        "lm_head": {"flops": 2.0 * M * d * V, "bytes": 2.0 * (V * d) + 2.0 * M * (d + V)},
        "attention": {"flops": 4.0 * M * N * hd, "bytes": None},
        "score": {"flops": None, "bytes": 4.0 * M * V},
        # row-wise kernels, lower bounds: token row in, x and h out; x in, h out (the launch that also adds
        # k-split partial planes moves 4 bytes per element and plane more)
        "embed_norm": {"flops": None, "bytes": 6.0 * M * d},
        "add_norm": {"flops": None, "bytes": 4.0 * M * d},
    }


class ScheduleRunner:
    """One configuration's session and seeded state; times steps at chosen points of its schedule."""

    def __init__(self, name, weights, seed=0, packed=None, shape=None):
        self.name = name
        self.Bn, self.N, self.n_p, self.block, self.T, self.M_end, kind, eps = CONFIGS[name]
        self.shape = wl.C3 if shape is None else shape
        shape = self.shape
        self.dev = torch.device("cuda:0")
        self.sess = B.Session(shape, weights, self.Bn, self.N, packed=packed)
        mk = wl.prompt_zipf if kind == "zipf" else wl.prompt_uniform
        Bn, N, n_p = self.Bn, self.N, self.n_p
        self.tokens = np.full((Bn, N), shape.mask_id, dtype=np.int64)
        for b in range(Bn):
            self.tokens[b, :n_p] = mk(seed + 10 + b, n_p, shape.vocab, shape.mask_id)
            self.tokens[b, n_p:] = wl.prompt_uniform(seed + 50 + b, N - n_p, shape.vocab, shape.mask_id)   # ids of unmasked slots
        self.pri = [np.random.default_rng(seed * 100 + b).permutation(N) for b in range(Bn)]
        self.eps_d = torch.as_tensor(np.asarray(eps, dtype=np.float32), device=self.dev)
        self.t = 2

    def close(self):
        self.sess.close()

    def state(self, step, full=False):
        M_end = [self.N] * self.Bn if full else self.M_end
        return state_at(step, self.Bn, self.N, self.n_p, self.block, self.T, M_end, self.pri)

    def timed(self, masked, lock, blk, K, warmup=2, profile=True):
        """K timed steps on the given state (after `warmup` untimed ones; at least two, so that both posterior
        buffers hold these rows).  Returns (M, ms per step, {slot: (ms per launch, launches per step)})."""
        shape, sess = self.shape, self.sess
        tok = self.tokens.copy()
        tok[masked == 1] = shape.mask_id
        tok_d = torch.as_tensor(tok.reshape(-1), dtype=torch.int32, device=self.dev)
        msk_d = torch.as_tensor(masked.reshape(-1), device=self.dev)
        lock_d = torch.as_tensor(lock.reshape(-1), device=self.dev)
        out = torch.empty_like(lock_d)
        M = int((lock == 0).sum())

        def run(n):
            for _ in range(n):
                self.t += 1
                sess.step(tok_d, msk_d, lock_d, self.eps_d, self.t, blk[0], blk[1], 1, m_upper=M, new_lock=out)

        run(max(2, warmup))
        torch.cuda.synchronize()
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record()
        run(K)
        e1.record()
        torch.cuda.synchronize()
        ms = e0.elapsed_time(e1) / K
        assert int(sess.cu_active[-1].item()) == M
        per = {}
        if profile:
            Kp = min(K, 5)
            B.sl_profile_begin(sess.ctx, Kp * (16 + 12 * shape.n_layers))
            run(Kp)
            prof = B.sl_profile_end(sess.ctx)
            per = {s: (v[0] / max(v[1], 1), v[1] / Kp) for s, v in prof.items()}
        return M, ms, per

    def point(self, step, K, warmup=2, full=False):
        masked, lock, blk = self.state(step, full)
        if full:
            lock = np.zeros_like(lock)
        M, ms, per = self.timed(masked, lock, blk, K, warmup)
        row = {"step": step, "M": M, "M_over_N": round(M / (self.Bn * self.N), 4), "ms": round(ms, 4),
               "rows_per_s": round(M / ms * 1e3)}
        if per:
            tot = sum(a * n for a, n in per.values())
            row["percent"] = {g: round(100 * sum(per[s][0] * per[s][1] for s in slots) / tot, 1) for g, slots in GROUPS.items()}
            work = slot_work(self.shape, self.N, M)
            fr = {}
            for s, wk in work.items():
                if per.get(s, (0, 0))[1] == 0:
                    continue
                sec = per[s][0] * 1e-3
                e = {"us": round(per[s][0] * 1e3, 1)}
                if wk["flops"] is not None:
                    e["mfma_frac"] = round(wk["flops"] / sec / MFMA_BF16_PEAK, 4)
                if wk["bytes"] is not None:
                    e["hbm_frac"] = round(wk["bytes"] / sec / HBM_PEAK, 4)
                fr[s] = e
            row["kernels"] = fr
            gsec = sum(per[s][0] for s in GROUPS["gemm"] if per[s][1]) * 1e-3
            row["layer_gemm_mfma_frac"] = round(sum(work[s]["flops"] for s in GROUPS["gemm"]) / gsec / MFMA_BF16_PEAK, 4)
            row["layer_gemm_hbm_frac"] = round(sum(work[s]["bytes"] for s in GROUPS["gemm"]) / gsec / HBM_PEAK, 4)
        return row, per

    def sweep(self, points, K, warmup=2, log=None):
        """The full-recompute step and `points` samples of the schedule; returns (rows, summary)."""
        full, _ = self.point(1, K, warmup, full=True)
        full["note"] = "full recompute (no locks)"
        rows = [full]
        if log:
            log(full)
        for st in sorted({int(round(x)) for x in np.linspace(1, self.T, points)}):
            r, _ = self.point(st, K, warmup)
            rows.append(r)
            if log:
                log(r)
        xs = np.array([r["step"] for r in rows[1:]], dtype=np.float64)
        ys = np.array([r["ms"] for r in rows[1:]])
        total = float(np.trapezoid(ys, xs)) + ys[-1]       # T steps: integral over [1, T] plus the last step itself
        act = float(np.trapezoid([r["M"] for r in rows[1:]], xs) + rows[-1]["M"]) / (self.Bn * self.N * self.T)
        summary = {"config": self.name, "batch": self.Bn, "N": self.N, "T": self.T, "schedule_ms": round(total, 1),
                   "full_recompute_ms": round(full["ms"] * self.T, 1),
                   "time_ratio": round(total / (full["ms"] * self.T), 3), "active_row_ratio": round(act, 3)}
        return rows, summary


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--config", choices=sorted(CONFIGS), default="c3")
    ap.add_argument("--points", type=int, default=6)
    ap.add_argument("--steps", type=int, default=5)
    ap.add_argument("--seed", type=int, default=0)
    args = ap.parse_args()
    assert torch.cuda.is_available(), "run_config needs a GPU"
    w = wl.make_weights(wl.C3, args.seed, device="cuda")
    r = ScheduleRunner(args.config, w, args.seed)
    rows, summary = r.sweep(args.points, args.steps, log=lambda row: print(json.dumps(row), flush=True))
    print(json.dumps(summary))
    r.close()


if __name__ == "__main__":
    main()
    sys.exit(0)
