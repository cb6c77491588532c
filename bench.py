#!/usr/bin/env python3
"""SureLock step latency vs unlocked fraction M/N on one MI355X.

Headline workload (BASELINE config 5, the largest that is one GPU's share): the full 32-layer
LLaDA-8B-shaped bf16 model (d=4096, 32 heads x 128, SwiGLU FFN 12288, vocabulary 126464, random-init
N(0, 0.02)), B = 8 sequences of N = 1024 slots (512 Zipf(1.1) prompt tokens + 512 generated), packed
ragged rows.  `value` is the latency of one whole SureLock step (compaction, gather + RMSNorm, 32 x
[Q|K|V projection, RoPE + K/V cache write, M x N attention, Out projection, SwiGLU FFN], LM head,
KL / confidence / argmax scoring, UpdateMASK, lock rule) with every row active (sum M = 8192), timed
over exactly --steps steps; `sweep` samples the configuration's forced linear lock schedule, so that
latency can be read against M/N, and gives the time ratio of the whole schedule against full
recompute beside the active-row ratio (the algorithmic work kept, Sec. 2.4).  The same is done for
configs 4 (B=1, N=2048) and 3 (B=1, N=512) and, on one layer, config 2 (N=1024, M in
{1024,512,256,64,16}).  All inputs are seeded, synthetic and resident in HBM before any timed region.

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--only c5,c4,c3,c2] [--points P]

Prints one JSON line."""
import argparse
import json
import os
import re
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

MFMA_BF16_PEAK = 2.5e15      # dense bf16 FLOP/s, MI355X
HBM_PEAK = 8.0e12            # B/s
TRAFFIC_PROFILE = os.path.join(ROOT, "profiles", "bench_c5_gate_up_hbm_traffic.txt")


def traffic_from_profile():
    """HBM bytes per launch of the dominant kernel, read from the rocprofv3 counter summary that measured
    them (the line 'roofline.traffic = <bytes>' of the profile, which also gives the commands); None when the
    summary is not there.  Counters cannot be collected by this run itself."""
    try:
        m = re.search(r"roofline\.traffic\s*=\s*([0-9][0-9,]*)", open(TRAFFIC_PROFILE).read())
        return int(m.group(1).replace(",", "")) if m else None
    except OSError:
        return None


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


def c2_sweep(B, torch, np, wl, w, K, W, seed, sweep):
    """Config 2: one layer (layer 0 of the model) + LM head, N = 1024, M swept; plus the optional-unlocking probe
    and the selection-hybrid step on the same session."""
    from paper_2602_06412_amd.run_config import slot_work
    shape, N = wl.C2, 1024
    dev = torch.device("cuda:0")
    w1 = {"emb": w["emb"], "final_norm": w["final_norm"], "lm_head": w["lm_head"], "layers": [w["layers"][0]]}
    sess = B.Session(shape, w1, 1, N)
    rng = np.random.default_rng(seed)
    tokens0 = torch.as_tensor(wl.prompt_uniform(seed + 1, N, shape.vocab, shape.mask_id), dtype=torch.int32, device=dev)
    eps = torch.full((1,), 1e-3, dtype=torch.float32, device=dev)
    zero_mask = torch.zeros(N, dtype=torch.uint8, device=dev)
    new_lock = torch.zeros(N, dtype=torch.uint8, device=dev)
    t = 0
    for _ in range(2):                       # cache + both posterior buffers filled by two M = N passes
        t += 1
        sess.step(tokens0.clone(), zero_mask.clone(), zero_mask, eps, t, 0, N, 0, m_upper=N, new_lock=new_lock)
    torch.cuda.synchronize()
    results = []
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    for M in sweep:
        active = wl.active_positions(seed + 100 + M, N, M)
        lock = torch.as_tensor(wl.lock_mask_from_active(N, active), device=dev)
        masked = (1 - lock).clone()                 # every active slot still masked: UpdateMASK has work
        tokens = tokens0.clone()

        def run(n_steps):
            nonlocal t
            for _ in range(n_steps):
                t += 1
                sess.step(tokens, masked, lock, eps, t, 0, N, 1, m_upper=M, new_lock=new_lock)

        run(max(W, 2))
        torch.cuda.synchronize()
        e0.record()
        run(K)
        e1.record()
        torch.cuda.synchronize()
        ms = e0.elapsed_time(e1) / K
        B.sl_profile_begin(sess.ctx, K * 32)
        run(K)
        prof = B.sl_profile_end(sess.ctx)
        per = {k: v[0] / K for k, v in prof.items()}            # ms per step per kernel slot
        work = slot_work(shape, N, M)
        gem = ["gemm_qkv", "gemm_out", "gemm_gate_up", "gemm_down", "lm_head"]
        gsec = sum(per[s] for s in gem) * 1e-3
        results.append({
            "M": M, "M_over_N": M / N, "ms": round(ms, 4), "rows_per_s": round(M / (ms * 1e-3), 1),
            "gemm_mfma_frac": round(sum(work[s]["flops"] for s in gem) / gsec / MFMA_BF16_PEAK, 4),
            "gemm_hbm_frac": round(sum(work[s]["bytes"] for s in gem) / gsec / HBM_PEAK, 4),
            "attention_mfma_frac": round(work["attention"]["flops"] / (per["attention"] * 1e-3) / MFMA_BF16_PEAK, 4),
            "score_hbm_frac": round(work["score"]["bytes"] / (per["score"] * 1e-3) / HBM_PEAK, 4),
            "kernels_ms": {k: round(v, 4) for k, v in per.items()},
        })
    # Optional unlocking (appendix): one read-only probe + unlock rule over N/2 locked rows (eps_unlock = +inf:
    # nothing unlocks, the state stays as it is); amortised over the probe period P.
    Mp = N // 2
    active = wl.active_positions(seed + 100 + Mp, N, N - Mp)
    lock = torch.as_tensor(wl.lock_mask_from_active(N, active), device=dev)
    sess.unlock_state()
    sess.t_lock.copy_(torch.as_tensor(rng.integers(1, 3, N), dtype=torch.int32, device=dev) * lock.to(torch.int32))
    sess.step(tokens0.clone(), (1 - lock).clone(), lock, eps, t + 1, 0, N, 1, m_upper=N - Mp, new_lock=new_lock)
    for i in range(W + K):
        if i == W:
            torch.cuda.synchronize()
            e0.record()
        sess.unlock_probe(tokens0, lock, t + 1, 20.0, float("inf"), 1, 2, m_upper_probe=Mp, m_upper_active=N - Mp)
    e1.record()
    torch.cuda.synchronize()
    probe_ms = e0.elapsed_time(e1) / K
    t += 1
    # Selection hybrid (Exp-5, combined setting): the step that computes ceil(0.8 n) of the n = N non-locked rows.
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
    sel_ms = e0.elapsed_time(e1) / K
    sess.close()
    return {"workload": "C2: one LLaDA-8B-shaped bf16 layer + LM head (V=126464), N=1024 cached K/V, B=1", "sweep": results,
            "unlock_probe": {"locked_rows": Mp, "ms": round(probe_ms, 4),
                             "note": "read-only probe + unlock rule over the locked rows, once per P steps"},
            "selected_step": {"k": k_sel, "non_locked_rows": N, "computed_rows": M_sel, "ms": round(sel_ms, 4),
                              "note": "step with on-device selection of ceil(k n) rows + posterior carry of the skipped ones"}}


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=20)
    ap.add_argument("--warmup", type=int, default=3)
    ap.add_argument("--seed", type=int, default=0)
    ap.add_argument("--points", type=int, default=6, help="samples of each lock schedule")
    ap.add_argument("--only", type=str, default="c5,c4,c3,c2", help="which configurations to run (c5 is always run)")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-probes", action="store_true", help="skip the peak and clock probes")
    ap.add_argument("--c2-sweep", type=str, default="1024,512,256,64,16")
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
    from paper_2602_06412_amd.run_config import DESCRIBE, ScheduleRunner, slot_work

    assert torch.cuda.is_available(), "bench.py needs a GPU"
    torch.cuda.set_device(0)
    dev = torch.device("cuda:0")
    K, W = args.steps, args.warmup
    only = set(args.only.split(",")) | {"c5"}
    shape = wl.C3
    d, V = shape.d_model, shape.vocab

    w = wl.make_weights(shape, args.seed, device="cuda")
    log = lambda row: print(json.dumps(row), file=sys.stderr, flush=True)

    # ---- headline: config 5, every row active, exactly K timed steps after W warm-up steps ----
    r5 = ScheduleRunner("c5", w, args.seed)
    packed = r5.sess.packed
    masked, lock, blk = r5.state(1, full=True)
    lock = np.zeros_like(lock)
    M0, ms0, per0 = r5.timed(masked, lock, blk, K, warmup=W)
    work0 = slot_work(shape, r5.N, M0)
    dom = max((s for s in per0 if per0[s][1] > 0), key=lambda s: per0[s][0] * per0[s][1])      # largest share of the step
    dom_ms = per0[dom][0]
    roof = {"kernel": "%s launch (layer projection d=%d -> 2 x d_ff=%d with SwiGLU epilogue, %d rows)" % (dom, d, shape.d_ff, M0)
            if dom == "gemm_gate_up" else "%s launch at %d rows" % (dom, M0),
            "bound": "mfma", "achieved": round(work0[dom]["flops"] / (dom_ms * 1e-3) / 1e12, 2),
            "peak": MFMA_BF16_PEAK / 1e12, "unit": "TFLOP/s",
            "frac": round(work0[dom]["flops"] / (dom_ms * 1e-3) / MFMA_BF16_PEAK, 4),
            "traffic": traffic_from_profile() if dom == "gemm_gate_up" else None,
            "launch_ms": round(dom_ms, 4), "launches_per_step": per0[dom][1],
            "algorithmic_flops_per_launch": work0[dom]["flops"],
            "share_of_step": round(per0[dom][0] * per0[dom][1] / sum(a * n for a, n in per0.values()), 3)}
    fam = {}
    for s, wk in work0.items():
        if per0.get(s, (0, 0))[1] == 0:
            continue
        sec = per0[s][0] * 1e-3
        fam[s] = {"us": round(per0[s][0] * 1e3, 1), "launches_per_step": per0[s][1]}
        if wk["flops"] is not None:
            fam[s]["mfma_frac"] = round(wk["flops"] / sec / MFMA_BF16_PEAK, 4)
        else:
            fam[s]["hbm_frac"] = round(wk["bytes"] / sec / HBM_PEAK, 4)
    roof["per_kernel"] = fam
    gemm4 = ["gemm_qkv", "gemm_out", "gemm_gate_up", "gemm_down"]
    roof["layer_projections_frac"] = round(sum(work0[s]["flops"] for s in gemm4) /
                                           (sum(per0[s][0] for s in gemm4) * 1e-3) / MFMA_BF16_PEAK, 4)

    sweeps, summaries = {}, {}
    rows, summ = r5.sweep(args.points, max(3, min(K, 10)), log=log)
    sweeps["c5"], summaries["c5"] = rows, summ
    r5.close()
    torch.cuda.empty_cache()
    for name in ("c4", "c3"):
        if name not in only:
            continue
        r = ScheduleRunner(name, w, args.seed, packed=packed)
        rows, summ = r.sweep(args.points, max(3, min(K, 10)), log=log)
        sweeps[name], summaries[name] = rows, summ
        r.close()
        torch.cuda.empty_cache()
    c2 = None
    if "c2" in only:
        c2 = c2_sweep(B, torch, np, wl, w, max(3, min(K, 20)), W, args.seed, [int(x) for x in args.c2_sweep.split(",")])

    if args.calibrate_copy:
        src = torch.ones(1 << 28, dtype=torch.float32, device=dev)          # 1 GiB read + 1 GiB written
        dst = torch.empty_like(src)
        torch.add(src, 1.0, out=dst)
        torch.cuda.synchronize()
        del src, dst

    ach_peaks = None
    if not args.no_probes:
        roof["lm_head_clock"] = lm_head_clock_probe(B, torch, w["lm_head"], 1024, V, d, args.seed)
        ach_peaks = achievable_peaks(B, torch, dev, args.seed)
        mfma_ach = max(v for k_, v in ach_peaks.items() if k_.startswith("mfma_bf16_tflops"))
        roof["frac_of_achievable"] = round(roof["achieved"] / mfma_ach, 4)

    cpu = None
    if not args.no_cpu_baseline:
        cpu = cpu_baseline(shape, w, args.seed)

    out = {
        "metric": "SureLock step latency (ms) vs unlocked fraction M/N; % bf16 MFMA peak",
        "value": round(ms0, 4), "unit": "ms", "n_gpus": 1, "steps": K, "warmup": W, "ms_per_step": round(ms0, 4),
        "higher_is_better": False, "scaling": "weak", "vs_baseline": None, "dtype": "bf16", "data": "synthetic",
        "config": {"workload": DESCRIBE["c5"] + "; value = whole SureLock step with every row active (sum M = %d); "
                               "`sweep` samples the lock schedule" % M0,
                   "N": r5.N, "batch": r5.Bn, "M": M0, "d_model": d, "n_heads": shape.n_heads, "d_head": shape.d_head,
                   "d_ff": shape.d_ff, "vocab": V, "n_layers": shape.n_layers,
                   "arithmetic": "bf16 storage and MFMA operands, fp32 accumulation; attention's P.V product on half-precision "
                                 "operands (V cached as the half image of its bf16 value, probabilities rounded to half: "
                                 "11 significant bits where a bf16 attention keeps 8)"},
        "rows_per_s": round(M0 / ms0 * 1e3),
        "roofline": roof,
        "achievable": ach_peaks,
        "cpu_baseline": cpu,
        "latency_vs_active_fraction": {k: {"workload": DESCRIBE[k], **summaries[k]} for k in summaries},
        "sweep": sweeps,
        "c2": c2,
    }
    print(json.dumps(out))


def cpu_baseline(shape, w, seed):
    """The oracle, as it stands, on the host cores, on a bounded sample of the headline workload: ONE of
    config 5's eight sequences (N = 1024) through ONE of the 32 layers, the LM head and the scoring
    (log-softmax, KL, confidence, argmax), at the sequence's largest, median and smallest active-row counts
    (1024, 544, 64), with all cores; and the smallest once more on a single thread."""
    import numpy as np
    import torch
    from oracle import model, posterior
    from oracle.model import Config
    from paper_2602_06412_amd import workloads as wl
    try:
        import threadpoolctl
    except Exception:
        threadpoolctl = None

    N, n_p = 1024, 512
    cfg = Config(1, shape.d_model, shape.n_heads, shape.d_head, shape.d_ff, shape.vocab, shape.mask_id,
                 shape.rms_eps, shape.rope_theta, shape.storage)
    tok = np.concatenate([wl.prompt_zipf(seed + 10, n_p, shape.vocab, shape.mask_id),
                          wl.prompt_uniform(seed + 50, N - n_p, shape.vocab, shape.mask_id)]).astype(np.int64)
    f64 = lambda t_: t_.detach().to("cpu", torch.float64).numpy()
    w64 = {"emb": f64(w["emb"][torch.as_tensor(tok, device=w["emb"].device)]),      # only the rows the tokens use
           "final_norm": f64(w["final_norm"]), "lm_head": f64(w["lm_head"]),
           "layers": [{k: f64(v) for k, v in w["layers"][0].items()}]}
    Kc = [np.zeros((N, cfg.n_heads, cfg.d_head))]
    Vc = [np.zeros((N, cfg.n_heads, cfg.d_head))]
    try:
        cores = len(os.sched_getaffinity(0))
    except Exception:
        cores = os.cpu_count()
    pools = threadpoolctl.threadpool_info() if threadpoolctl else []
    nthreads = max((p.get("num_threads", 1) for p in pools), default=cores)

    def one(M):
        active = wl.active_positions(seed + 100 + M, N, M) if M < N else np.arange(N)
        t0 = time.perf_counter()
        z = model.forward_active(cfg, w64, np.arange(N), active, Kc, Vc)
        lp = posterior.log_softmax(z)
        conf = posterior.max_prob(lp)
        amax = posterior.argmax_lowest(z)
        D = posterior.kl_rows(lp, lp)
        return time.perf_counter() - t0, float(np.sum(D) + conf[0] + amax[0])

    samples, chk = [], 0.0
    for M in (1024, 544, 64):
        dt, c = one(M)
        chk += c
        samples.append({"M": M, "ms": round(dt * 1e3, 1), "rows_per_s": round(M / dt, 1), "threads": int(min(cores, nthreads))})
    single = None
    if threadpoolctl:
        with threadpoolctl.threadpool_limits(limits=1):
            dt, c = one(64)
        chk += c
        single = {"M": 64, "ms": round(dt * 1e3, 1), "rows_per_s": round(64 / dt, 1), "threads": 1}
    # config 1 (the tiny fp32 model: 2 layers, d = 256, V = 1024, N = 32 + 96, T = 32, three tokens per step): the
    # oracle's whole run, with the lock rule (eps = 1e-3) and without (eps < 0 = the plain sampler), in seconds
    c1 = wl.C1
    cfg1 = Config(c1.n_layers, c1.d_model, c1.n_heads, c1.d_head, c1.d_ff, c1.vocab, c1.mask_id, c1.rms_eps,
                  c1.rope_theta, c1.storage)
    w1 = wl.make_weights(c1, seed)
    w1_64 = {"emb": f64(w1["emb"]), "final_norm": f64(w1["final_norm"]), "lm_head": f64(w1["lm_head"]),
             "layers": [{k_: f64(v) for k_, v in L.items()} for L in w1["layers"]]}
    from oracle import sampler
    prompt1 = wl.prompt_uniform(seed + 1, 32, c1.vocab, c1.mask_id)
    c1_run = {}
    for label, eps1 in (("surelock_eps_1e-3", 1e-3), ("plain_sampler", -1.0)):
        st = sampler.init_state(cfg1, w1_64, prompt1, 96)
        t0 = time.perf_counter()
        rows = 0
        for lo, hi, k_ in sampler.block_schedule(32, 96, 96, 32):
            rows += int((st.lock == 0).sum())
            sampler.surelock_step(cfg1, w1_64, st, eps1, lo, hi, k_)
        c1_run[label] = {"s": round(time.perf_counter() - t0, 3), "active_rows_summed": rows}
        chk += float(st.lock.sum())
    top = samples[0]
    # one layer + LM head of one sequence -> 32 layers + LM head of eight sequences (labelled: an extrapolation)
    layer_share = 436.2 / (436.2 + 1036.0)            # of the sample's matrix work that is the layer (MFLOP per row)
    full_step_ms = top["ms"] * 8 * (32 * layer_share + (1 - layer_share))
    return {"value": top["ms"], "unit": "ms", "cores": int(min(cores, nthreads)), "kind": "oracle",
            "sample": "one of config 5's eight sequences (N=1024) through one of the 32 layers + LM head + KL/conf/argmax "
                      "scoring, NumPy fp64, all host cores, at M=1024 (value), 544 and 64 active rows; M=64 again on one thread",
            "rows_per_s": top["rows_per_s"], "samples": samples, "single_thread": single,
            "config1_full_run": c1_run,
            "extrapolated_full_step_ms": round(full_step_ms, 1),
            "extrapolation": "value x 8 sequences x (32 layers + LM head) / (1 layer + LM head) by matrix work; not measured",
            "host_cores": int(cores), "checksum": chk}


if __name__ == "__main__":
    main()
