"""CPU oracle for the SureLock hot path (TEST INFRASTRUCTURE, not product code).

Everything under ``oracle/`` is a plain, slow, fp64 NumPy statement of what one
SureLock diffusion step computes (Algorithm 1 of the paper and Sec. 2.1-2.2),
written to be checked against the paper by eye.  It shares no code with the HIP
path and must never be imported by the product package: only ``tests/``,
``__graft_entry__.smoke()`` and the ``cpu_baseline`` leg of ``bench.py`` use it.

Modules
-------
rounding   storage-type rounding (fp64 -> bf16 / fp32, round-to-nearest-even)
model      the transformer block arithmetic (RMSNorm, RoPE, attention, SwiGLU)
posterior  log-softmax, step-wise KL, confidence, argmax
control    active-set compaction, UpdateMASK, candidates and the lock rule
sampler    Algorithm 1 end to end, plus the plain full-recompute sampler
flops      the algorithmic-FLOP model of Sec. 2.4

Parity status: the end-to-end sampler trajectory is *parity unpinned* against
the authors' own implementation (the paper prints no logits, KL values, masks
or M_t traces).  Every individual function is pinned by the CPU tests to
closed forms, invariants the paper states, brute force, or library routines.
"""
