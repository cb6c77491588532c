#!/usr/bin/env python3
"""SureLock step latency vs unlocked fraction M/N on one MI355X.

Workload (BASELINE config 2): one LLaDA-8B-shaped bf16 layer (d=4096, 32 heads x 128,
SwiGLU FFN 12288) plus the LLaDA LM head (vocab 126464) so that every step of the hot path
runs: compaction, gather+RMSNorm, QKV GEMM, RoPE + K/V cache write, M x N attention over
N=1024 cached slots, Out GEMM, FFN GEMMs, LM head, KL/conf/argmax scoring, UpdateMASK,
lock rule.  Active sets of M in {1024, 512, 256, 64, 16} positions are drawn uniformly
without replacement from a seed.  Inputs are resident in HBM before the timed region.

    python bench.py [--gpus 1] [--steps K] [--warmup W]

Prints one JSON line; `value` is the step latency at M = N, `sweep` the latency at each M.
"""
import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

MFMA_BF16_PEAK = 2.5e15      # dense bf16 FLOP/s, MI355X
HBM_PEAK = 8.0e12            # B/s
# HBM bytes (fetched + written) of one LM-head launch, from the rocprofv3 FETCH_SIZE and
# WRITE_SIZE counter runs summarised in profiles/bench_c2_hbm_traffic.txt (already scaled by
# the copy-kernel calibration given there), keyed by M.
LM_HEAD_TRAFFIC_BYTES = {1024: 1851893935, 16: 1042204494}


def lm_head_clock_probe(B, torch, w_lm, M, V, d, seed, launches=12):
    """Shader clock and matrix-pipe occupancy inside the LM-head GEMM, from the library's in-kernel
    cycle probe (one mid-grid workgroup, last of `launches` back-to-back launches)."""
    dev = w_lm.device
    packed = torch.empty_like(w_lm)
    B.sl_linear_pack(w_lm, packed)
    g = torch.Generator(device="cpu").manual_seed(seed + 7)
    x = B.tile_activations(torch.randn(M, d, generator=g).to(torch.bfloat16).to(dev))
    m_dev = torch.tensor([M], dtype=torch.int32, device=dev)
    y = torch.empty(M, V, dtype=torch.bfloat16, device=dev)
    counters = torch.zeros(8, dtype=torch.int64, device=dev)
    for _ in range(launches):
        B.sl_linear_clock_probe(x, packed, m_dev, M, V, d, y, counters, x_tiled=1)
    torch.cuda.synchronize()
    c = [int(v) for v in counters.cpu()]
    del packed, y
    if c[4] <= 0 or c[1] <= 0:
        return None
    return {"sclk_mhz_in_k_loop": round(c[1] / c[4] * 100.0, 1),
            "matrix_pipe_busy_in_k_loop": round(1024.0 * c[7] / c[1], 4),
            "prologue_us": round(c[3] / 100.0, 2), "k_loop_us": round(c[4] / 100.0, 2),
            "epilogue_us": round(c[5] / 100.0, 2), "workgroups": c[6], "k_tiles": c[7], "nominal_mhz": 2400}


def achievable_peaks(B, torch, dev, seed):
    """What the chip sustains with nothing else in the way (the library's two peak probes): a bare loop of the
    projection kernels' MFMA instruction on N(0,1) bf16 register operands, and one read-only / one copying pass
    over 1 GiB.  Timed with events on the stream the probes are launched on (torch's current one)."""
    g = torch.Generator(device="cpu").manual_seed(seed + 11)
    operands = torch.randn(4096, generator=g).to(torch.bfloat16).to(dev)
    sink = torch.zeros(1 << 19, dtype=torch.float32, device=dev)                  # 2 MiB
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    out = {}
    for wps in (1, 2):
        iters = 16384 // wps
        B.sl_peak_probe_mfma(operands, 1024, wps, sink)
        torch.cuda.synchronize()
        e0.record()
        flops = 0
        for _ in range(4):
            flops += B.sl_peak_probe_mfma(operands, iters, wps, sink)
        e1.record()
        torch.cuda.synchronize()
        out["mfma_bf16_tflops_%d_wave%s_per_simd" % (wps, "" if wps == 1 else "s")] = round(
            flops / (e0.elapsed_time(e1) * 1e-3) / 1e12, 1)
    src = torch.randn(1 << 28, dtype=torch.float32, device=dev)                   # 1 GiB
    dst = torch.empty_like(src)
    for name, d_, factor in (("hbm_read_GBps", None, 1), ("hbm_copy_GBps", dst, 2)):
        B.sl_peak_probe_stream(src, d_, sink)
        torch.cuda.synchronize()
        e0.record()
        for _ in range(10):
            B.sl_peak_probe_stream(src, d_, sink)
        e1.record()
        torch.cuda.synchronize()
        out[name] = round(10 * factor * src.numel() * 4 / (e0.elapsed_time(e1) * 1e-3) / 1e9, 1)
    del src, dst
    out["note"] = ("bare v_mfma_f32_16x16x32_bf16 loop on N(0,1) bf16 register operands (one workgroup per CU); "
                   "one pass of 16-byte loads over 1 GiB, read-only and copied (bytes read + written)")
    return out


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=50)
    ap.add_argument("--warmup", type=int, default=10)
    ap.add_argument("--seed", type=int, default=0)
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--sweep", type=str, default="1024,512,256,64,16")
    ap.add_argument("--calibrate-copy", action="store_true",
                    help="also run one 1 GiB elementwise copy kernel, for scaling rocprofv3 FETCH_SIZE/WRITE_SIZE")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build runs on one GPU only (no collectives, no sharding); use --gpus 1",
              file=sys.stderr)
        sys.exit(2)

    import numpy as np
    import torch
    from paper_2602_06412_amd import binding as B
    from paper_2602_06412_amd import workloads as wl

    assert torch.cuda.is_available(), "bench.py needs a GPU"
    torch.cuda.set_device(0)
    dev = torch.device("cuda:0")
    shape, N, Bn = wl.C2, 1024, 1
    K, W = args.steps, args.warmup
    sweep = [int(x) for x in args.sweep.split(",")]

    w = wl.make_weights(shape, args.seed, device="cuda", emb_std=1.0)
    sess = B.Session(shape, w, Bn, N)
    rng = np.random.default_rng(args.seed)
    tokens0 = torch.as_tensor(wl.prompt_uniform(args.seed + 1, N, shape.vocab, shape.mask_id), dtype=torch.int32,
                              device=dev)
    eps = torch.full((Bn,), 1e-3, dtype=torch.float32, device=dev)
    zero_mask = torch.zeros(N, dtype=torch.uint8, device=dev)
    new_lock = torch.zeros(N, dtype=torch.uint8, device=dev)

    # cache + both posterior buffers filled by two M = N passes
    t = 0
    for _ in range(2):
        t += 1
        sess.step(tokens0.clone(), zero_mask.clone(), zero_mask, eps, t, 0, N, 0, m_upper=N, new_lock=new_lock)
    torch.cuda.synchronize()

    d, dff, hd, V = shape.d_model, shape.d_ff, shape.n_heads * shape.d_head, shape.vocab
    layer_gemm_flops = 2 * d * (3 * hd) + 2 * hd * d + 2 * d * (2 * dff) + 2 * dff * d      # per row
    lm_flops = 2 * d * V
    attn_flops = 4 * N * hd                                                                 # per row
    layer_w_bytes = 2 * (d * 3 * hd + hd * d + d * 2 * dff + dff * d)
    lm_w_bytes = 2 * d * V
    gemm_slots = ["gemm_qkv", "gemm_out", "gemm_gate_up", "gemm_down", "lm_head"]

    results = []
    for M in sweep:
        active = wl.active_positions(args.seed + 100 + M, N, M)
        lock = torch.as_tensor(wl.lock_mask_from_active(N, active), device=dev)
        masked = (1 - lock).clone()                 # every active slot still masked: UpdateMASK has work
        tokens = tokens0.clone()

        def run(n_steps):
            nonlocal t
            for _ in range(n_steps):
                t += 1
                sess.step(tokens, masked, lock, eps, t, 0, N, 1, m_upper=M, new_lock=new_lock)

        run(W)
        torch.cuda.synchronize()
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        t0 = time.perf_counter()
        e0.record()
        run(K)
        e1.record()
        torch.cuda.synchronize()
        wall_ms = (time.perf_counter() - t0) * 1e3 / K
        ms = e0.elapsed_time(e1) / K
        # per-kernel event timing of the same steps (profiling on: separate pass)
        B.sl_profile_begin(sess.ctx, K * 16)
        run(K)
        prof = B.sl_profile_end(sess.ctx)
        per = {k: v[0] / K for k, v in prof.items()}            # ms per step per kernel slot
        gemm_ms = sum(per[s] for s in gemm_slots)
        gemm_flops = M * (layer_gemm_flops + lm_flops)
        gemm_bytes = layer_w_bytes + lm_w_bytes + 2 * M * (d * 6 + hd * 2 + dff * 2) + 2 * M * V
        score_bytes = M * V * 4
        results.append({
            "M": M, "M_over_N": M / N, "ms": round(ms, 4), "wall_ms": round(wall_ms, 4),
            "rows_per_s": round(M / (ms * 1e-3), 1),
            "gemm_ms": round(gemm_ms, 4), "gemm_tflops": round(gemm_flops / (gemm_ms * 1e-3) / 1e12, 2),
            "gemm_mfma_frac": round(gemm_flops / (gemm_ms * 1e-3) / MFMA_BF16_PEAK, 4),
            "gemm_weight_stream_GBps": round(gemm_bytes / (gemm_ms * 1e-3) / 1e9, 1),
            "gemm_hbm_frac": round(gemm_bytes / (gemm_ms * 1e-3) / HBM_PEAK, 4),
            "attention_ms": round(per["attention"], 4),
            "attention_mfma_frac": round(M * attn_flops / (per["attention"] * 1e-3) / MFMA_BF16_PEAK, 4),
            "score_ms": round(per["score"], 4),
            "score_hbm_frac": round(score_bytes / (per["score"] * 1e-3) / HBM_PEAK, 4),
            "kernels_ms": {k: round(v, 4) for k, v in per.items()},
        })

    # Optional unlocking (appendix): cost of one read-only probe + unlock rule over N/2 locked rows, to be
    # amortised over the probe period P.  eps_unlock = +inf: nothing unlocks, the state stays as it is.
    Mp = N // 2
    active = wl.active_positions(args.seed + 100 + Mp, N, N - Mp)
    lock = torch.as_tensor(wl.lock_mask_from_active(N, active), device=dev)
    sess.unlock_state()
    sess.t_lock.copy_(torch.as_tensor(rng.integers(1, 3, N), dtype=torch.int32, device=dev) * lock.to(torch.int32))
    sess.step(tokens0.clone(), (1 - lock).clone(), lock, eps, t + 1, 0, N, 1, m_upper=N - Mp, new_lock=new_lock)
    for _ in range(W):
        sess.unlock_probe(tokens0, lock, t + 1, 20.0, float("inf"), 1, 2, m_upper_probe=Mp, m_upper_active=N - Mp)
    torch.cuda.synchronize()
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    e0.record()
    for _ in range(K):
        sess.unlock_probe(tokens0, lock, t + 1, 20.0, float("inf"), 1, 2, m_upper_probe=Mp, m_upper_active=N - Mp)
    e1.record()
    torch.cuda.synchronize()
    assert int(sess.cu_probe[-1].item()) == Mp and int(lock.sum().item()) == Mp
    probe_ms = e0.elapsed_time(e1) / K
    t += 1

    # Selection hybrid (Exp-5, combined setting): the step that computes ceil(0.8 n) of the n = N non-locked
    # rows, chosen on the device by their last KL; skipped rows have their posterior row carried over.
    k_sel = 0.8
    M_sel = int(np.ceil(float(np.float32(k_sel)) * N))
    sel_masked = zero_mask.clone()
    for i in range(W + K):
        if i == W:
            torch.cuda.synchronize()
            e0.record()
        t += 1
        sess.step_selected(tokens0, sel_masked, zero_mask, eps, t, 0, N, 0, k_sel, m_upper=M_sel, new_lock=new_lock)
    e1.record()
    torch.cuda.synchronize()
    assert int(sess.cu_active[-1].item()) == M_sel
    sel_ms = e0.elapsed_time(e1) / K

    if args.calibrate_copy:
        src = torch.ones(1 << 28, dtype=torch.float32, device=dev)          # 1 GiB read + 1 GiB written
        dst = torch.empty_like(src)
        torch.add(src, 1.0, out=dst)
        torch.cuda.synchronize()
        del src, dst

    head = results[0]
    M0 = head["M"]
    # Dominant kernel of the step: the LM-head GEMM launch (one per step).  Its duration is the
    # HIP-event time of that launch on the step's stream, averaged over the K profiled steps.
    lm_ms = head["kernels_ms"]["lm_head"]
    if M0 >= 512:
        ach = M0 * lm_flops / (lm_ms * 1e-3) / 1e12
        roof = {"kernel": "gemm_mfma256_kernel<1, 256, false> (LM head, M=%d x V=%d x d=%d)" % (M0, V, d), "bound": "mfma",
                "achieved": round(ach, 2), "peak": MFMA_BF16_PEAK / 1e12, "unit": "TFLOP/s",
                "frac": round(ach * 1e12 / MFMA_BF16_PEAK, 4), "traffic": LM_HEAD_TRAFFIC_BYTES.get(M0),
                "launch_ms": round(lm_ms, 4), "algorithmic_flops_per_launch": M0 * lm_flops,
                "gemm_family_tflops": head["gemm_tflops"], "gemm_family_frac": head["gemm_mfma_frac"]}
    else:
        bytes_ = lm_w_bytes + 2 * M0 * d + 2 * M0 * V
        ach = bytes_ / (lm_ms * 1e-3) / 1e9
        roof = {"kernel": "thin-launch GEMM (LM head weight stream, M=%d)" % M0, "bound": "hbm",
                "achieved": round(ach, 1), "peak": HBM_PEAK / 1e9, "unit": "GB/s",
                "frac": round(ach * 1e9 / HBM_PEAK, 4), "traffic": LM_HEAD_TRAFFIC_BYTES.get(M0),
                "launch_ms": round(lm_ms, 4), "algorithmic_bytes_per_launch": bytes_}

    if M0 >= 512:
        roof["clock"] = lm_head_clock_probe(B, torch, w["lm_head"], M0, V, d, args.seed)

    ach_peaks = achievable_peaks(B, torch, dev, args.seed)
    mfma_ach = max(v for k_, v in ach_peaks.items() if k_.startswith("mfma_bf16_tflops"))
    if roof["bound"] == "mfma":
        roof["frac_of_achievable"] = round(roof["achieved"] / mfma_ach, 4)
    else:
        roof["frac_of_achievable"] = round(roof["achieved"] / ach_peaks["hbm_read_GBps"], 4)
    for r_ in results:
        r_["gemm_frac_of_achievable_mfma"] = round(r_["gemm_tflops"] / mfma_ach, 4)
        r_["score_frac_of_achievable_hbm_read"] = round(r_["score_hbm_frac"] * HBM_PEAK / 1e9 / ach_peaks["hbm_read_GBps"], 4)

    cpu = None
    if not args.no_cpu_baseline:
        cpu = cpu_baseline(shape, w, tokens0, N)

    out = {
        "metric": "SureLock step latency (ms) vs unlocked fraction M/N; % bf16 MFMA peak",
        "value": head["ms"], "unit": "ms", "n_gpus": 1, "steps": K, "warmup": W, "ms_per_step": head["ms"],
        "higher_is_better": False, "scaling": "weak", "vs_baseline": None, "dtype": "bf16", "data": "synthetic",
        "config": {"workload": "C2: one LLaDA-8B-shaped bf16 layer + LM head (V=126464), N=1024 cached K/V, "
                               "whole SureLock step at M=%d active rows (value); sweep over M in `sweep`" % M0,
                   "N": N, "batch": Bn, "M": M0, "d_model": d, "n_heads": shape.n_heads, "d_head": shape.d_head,
                   "d_ff": dff, "vocab": V, "n_layers": shape.n_layers},
        "rows_per_s": head["rows_per_s"],
        "roofline": roof,
        "achievable": ach_peaks,
        "cpu_baseline": cpu,
        "sweep": results,
        "selected_step": {"k": k_sel, "non_locked_rows": N, "computed_rows": M_sel, "ms": round(sel_ms, 4),
                          "note": "step with on-device selection of ceil(k n) rows + posterior carry of the skipped ones"},
        "unlock_probe": {"locked_rows": Mp, "ms": round(probe_ms, 4),
                         "note": "read-only probe + unlock rule over the locked rows, once per P steps"},
    }
    print(json.dumps(out))
    sess.close()


def cpu_baseline(shape, w, tokens0, N):
    """The oracle, as it stands, on the host cores: one full C2 step at M = N (restricted
    forward of one layer + LM head + scoring), timed once."""
    import numpy as np
    import torch
    from oracle import model, posterior
    from oracle.model import Config

    cfg = Config(shape.n_layers, shape.d_model, shape.n_heads, shape.d_head, shape.d_ff, shape.vocab, shape.mask_id,
                 shape.rms_eps, shape.rope_theta, shape.storage)
    tok = tokens0.cpu().numpy().astype(np.int64)
    f64 = lambda t_: t_.detach().to("cpu", torch.float64).numpy()
    w64 = {"emb": f64(w["emb"][torch.as_tensor(tok, device=w["emb"].device)]),      # only the rows the tokens use
           "final_norm": f64(w["final_norm"]), "lm_head": f64(w["lm_head"]),
           "layers": [{k: f64(v) for k, v in l.items()} for l in w["layers"]]}
    Kc = [np.zeros((N, cfg.n_heads, cfg.d_head)) for _ in range(cfg.n_layers)]
    Vc = [np.zeros((N, cfg.n_heads, cfg.d_head)) for _ in range(cfg.n_layers)]
    prev = None
    t0 = time.perf_counter()
    z = model.forward_active(cfg, w64, np.arange(N), np.arange(N), Kc, Vc)
    lp = posterior.log_softmax(z)
    conf = posterior.max_prob(lp)
    amax = posterior.argmax_lowest(z)
    D = posterior.kl_rows(lp, lp if prev is None else prev)
    dt = time.perf_counter() - t0
    try:
        cores = len(os.sched_getaffinity(0))
    except Exception:
        cores = os.cpu_count()
    try:
        import threadpoolctl
        nthreads = max((p.get("num_threads", 1) for p in threadpoolctl.threadpool_info()), default=1)
        cores = min(cores, nthreads) if nthreads else cores
    except Exception:
        pass
    return {"value": round(dt * 1e3, 1), "unit": "ms", "cores": int(cores), "kind": "oracle",
            "sample": "one full step of the same workload at M=N=1024 (1 layer + LM head + KL/conf/argmax), "
                      "NumPy fp64, timed once", "rows_per_s": round(N / dt, 1),
            "checksum": float(np.sum(D) + conf[0] + amax[0])}


if __name__ == "__main__":
    main()
