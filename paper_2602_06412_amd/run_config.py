#!/usr/bin/env python3
"""Step latency of the 32-layer configurations along their lock schedules, on one GPU.

    python -m paper_2602_06412_amd.run_config --config c3|c4|c5 [--points 6] [--steps 5]

Random-init LLaDA-8B-shaped bf16 weights (32 layers, d = 4096, 32 x 128 heads, FFN 12288, vocabulary
126464) and seeded synthetic prompts.  Random weights never converge, so the lock mask follows the
configuration's linear schedule of active rows M_t (locked positions chosen by a seeded priority
among prompt and already-unmasked slots); the KL rule still runs inside every step.  The schedule is
sampled at `--points` values of M_t; at each, the state of that moment is built and `--steps` steps
are timed (events on the launch stream) after one warm-up, with a per-kernel split from the
library's profiling hooks.  The last line sums the sampled latencies over the whole schedule
(trapezoid rule) next to the same number of full-recompute steps (M = N), which is the
paper's comparison: algorithmic work saved vs time saved."""
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
GROUPS = {"gemm": ["gemm_qkv", "gemm_out", "gemm_gate_up", "gemm_down"], "lm_head": ["lm_head"],
          "attention": ["attention"], "score": ["score"],
          "row-wise": ["embed_norm", "rope_kv", "add_norm", "swiglu"], "control": ["compact", "unmask", "lock_rule"]}


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


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--config", choices=sorted(CONFIGS), default="c3")
    ap.add_argument("--points", type=int, default=6)
    ap.add_argument("--steps", type=int, default=5)
    ap.add_argument("--seed", type=int, default=0)
    args = ap.parse_args()
    Bn, N, n_p, block, T, M_end, kind, eps = CONFIGS[args.config]
    assert torch.cuda.is_available(), "run_config needs a GPU"
    dev = torch.device("cuda:0")
    shape = wl.C3
    w = wl.make_weights(shape, args.seed, device="cuda")
    sess = B.Session(shape, w, Bn, N)
    mk = wl.prompt_zipf if kind == "zipf" else wl.prompt_uniform
    tokens = np.full((Bn, N), shape.mask_id, dtype=np.int64)
    for b in range(Bn):
        tokens[b, :n_p] = mk(args.seed + 10 + b, n_p, shape.vocab, shape.mask_id)
        tokens[b, n_p:] = wl.prompt_uniform(args.seed + 50 + b, N - n_p, shape.vocab, shape.mask_id)   # ids of unmasked slots
    pri = [np.random.default_rng(args.seed * 100 + b).permutation(N) for b in range(Bn)]
    eps_d = torch.as_tensor(np.asarray(eps, dtype=np.float32), device=dev)
    K = args.steps

    def timed(masked, lock, blk, t0):
        tok = tokens.copy()
        tok[masked == 1] = shape.mask_id
        tok_d = torch.as_tensor(tok.reshape(-1), dtype=torch.int32, device=dev)
        msk_d = torch.as_tensor(masked.reshape(-1), device=dev)
        lock_d = torch.as_tensor(lock.reshape(-1), device=dev)
        out = torch.empty_like(lock_d)
        M = int((lock == 0).sum())
        run = lambda t: sess.step(tok_d, msk_d, lock_d, eps_d, t, blk[0], blk[1], 1, m_upper=M, new_lock=out)
        run(t0); run(t0 + 1)                       # warm-up; both posterior buffers hold these rows
        torch.cuda.synchronize()
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record()
        for i in range(K):
            run(t0 + 2 + i)
        e1.record()
        torch.cuda.synchronize()
        ms = e0.elapsed_time(e1) / K
        B.sl_profile_begin(sess.ctx, K * (16 + 12 * shape.n_layers))
        for i in range(K):
            run(t0 + 2 + K + i)
        prof = B.sl_profile_end(sess.ctx)
        tot = sum(v[0] for v in prof.values())
        split = {g: round(100 * sum(prof[s][0] for s in slots) / tot, 1) for g, slots in GROUPS.items()}
        return M, ms, split

    # fill the K/V cache and both posterior buffers for every slot
    full_m, full_l, blk0 = state_at(1, Bn, N, n_p, block, T, [N] * Bn, pri)
    M0, ms_full, split_full = timed(full_m, np.zeros_like(full_l), blk0, 2)
    rows = [{"step": 0, "M": M0, "M_over_N": 1.0, "ms": round(ms_full, 3), "rows_per_s": round(M0 / ms_full * 1e3),
             "percent": split_full, "note": "full recompute (no locks)"}]
    print(json.dumps(rows[-1]), flush=True)
    pts = sorted({int(round(x)) for x in np.linspace(1, T, args.points)})
    for st in pts:
        masked, lock, blk = state_at(st, Bn, N, n_p, block, T, M_end, pri)
        M, ms, split = timed(masked, lock, blk, 2)
        rows.append({"step": st, "M": M, "M_over_N": round(M / (Bn * N), 4), "ms": round(ms, 3),
                     "rows_per_s": round(M / ms * 1e3), "percent": split})
        print(json.dumps(rows[-1]), flush=True)
    xs = np.array([r["step"] for r in rows[1:]], dtype=np.float64)
    ys = np.array([r["ms"] for r in rows[1:]])
    total = float(np.trapezoid(ys, xs)) + ys[-1]       # T steps: integral over [1, T] plus the last step itself
    print(json.dumps({"config": args.config, "batch": Bn, "N": N, "T": T, "schedule_ms": round(total, 1),
                      "full_recompute_ms": round(ms_full * T, 1), "time_ratio": round(total / (ms_full * T), 3),
                      "active_row_ratio": round(float(np.trapezoid([r["M"] for r in rows[1:]], xs) + rows[-1]["M"]) / (Bn * N * T), 3)}))
    sess.close()


if __name__ == "__main__":
    main()
    sys.exit(0)
