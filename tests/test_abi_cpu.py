"""CPU-only checks of the C-ABI library: it loads without a GPU, exports every symbol the
header declares, and rejects bad arguments before anything is launched."""
import ctypes as C
import os
import re

import pytest

from paper_2602_06412_amd import binding as B
from paper_2602_06412_amd import workloads as wl

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def _declared():
    src = open(os.path.join(ROOT, "include", "surelock.h")).read()
    src = re.sub(r"/\*.*?\*/", "", src, flags=re.S)
    return sorted(set(re.findall(r"\b(sl_[a-z_0-9]+)\s*\(", src)))


def test_library_exports_every_declared_symbol():
    names = _declared()
    assert "sl_surelock_step" in names and "sl_lock_test" in names and "sl_init" in names
    lib = B.lib()
    for n in names:
        assert hasattr(lib, n), n
    assert sorted(B.EXPORTS) == names          # the binding covers the whole header


def test_strerror():
    lib = B.lib()
    assert lib.sl_strerror(0) == b"ok"
    for s in (B.SL_EINVAL, B.SL_ENOSPC, B.SL_EHIP, B.SL_ESTATE, -99):
        assert len(lib.sl_strerror(s)) > 3


@pytest.mark.parametrize("field,value", [("n_layers", 0), ("d_head", 48), ("vocab", 1001), ("dtype", 2),
                                         ("mask_id", -1), ("mask_id", 1024), ("rms_eps", 0.0), ("d_model", 4)])
def test_init_rejects_bad_config(field, value):
    cfg = B.make_config(wl.C1)
    setattr(cfg, field, value)
    h = C.c_void_p()
    assert B.lib().sl_init(C.byref(cfg), C.byref(h)) == B.SL_EINVAL
    assert not h.value


def test_size_queries_and_call_order_without_gpu():
    ctx = B.sl_init(B.make_config(wl.C3))
    try:
        s = wl.C3
        kv = B.sl_kv_cache_bytes(ctx, 1, 512)
        assert kv >= 2 * s.n_layers * 512 * s.n_heads * s.d_head * 2          # K and V, bf16
        assert kv <= 2 * s.n_layers * 512 * s.n_heads * s.d_head * 2 + (1 << 20)
        assert B.sl_posterior_bytes(ctx, 1, 512) == 2 * 512 * s.vocab * 2
        assert B.sl_workspace_bytes(ctx, 1, 512) > 512 * s.d_model * 2
        lib = B.lib()
        out = C.c_size_t()
        assert lib.sl_kv_cache_bytes(ctx, 0, 512, C.byref(out)) == B.SL_EINVAL
        assert lib.sl_kv_cache_bytes(ctx, 1, 512, None) == B.SL_EINVAL
        assert lib.sl_kv_cache_bytes(ctx, 255, 64, C.byref(out)) == B.SL_OK              # SL_MAX_BATCH
        assert lib.sl_kv_cache_bytes(ctx, 256, 64, C.byref(out)) == B.SL_EINVAL
        assert lib.sl_kv_cache_bind(ctx, None, 256, 1 << 40, 256, 64) == B.SL_EINVAL
        assert lib.sl_kv_cache_bind(ctx, None, None, 1 << 30, 1, 512) == B.SL_EINVAL
        assert lib.sl_kv_cache_bind(ctx, None, 256, 16, 1, 512) == B.SL_ENOSPC
        assert lib.sl_kv_cache_bind(ctx, None, 257, 1 << 40, 1, 512) == B.SL_EINVAL      # misaligned
        assert lib.sl_posterior_bind(ctx, 256, 1 << 40) == B.SL_ESTATE                   # cache first
        p = C.c_void_p()
        assert lib.sl_logits_ptr(ctx, 1, C.byref(p)) == B.SL_ESTATE
        # the step refuses to run before weights / cache / store are bound
        assert lib.sl_surelock_step(ctx, None, 256, 256, 256, 256, 1, 0, 1, 1, 1, 256, 256, 256, 256, 256, 256, 256,
                                    1 << 40) == B.SL_ESTATE
        assert lib.sl_forward_layers(ctx, None, 256, 256, 256, 256, 1, 0, 1, 256, 1 << 40) == B.SL_ESTATE
        assert lib.sl_bind_weights(ctx, None, None, None, 0) == B.SL_EINVAL
    finally:
        B.sl_destroy(ctx)
    assert B.lib().sl_destroy(None) == B.SL_EINVAL
    assert B.lib().sl_init(None, None) == B.SL_EINVAL


def test_controller_entry_points_reject_null_and_bad_sizes():
    lib = B.lib()
    assert lib.sl_compact_active(None, None, 1, 8, 256, 256) == B.SL_EINVAL
    assert lib.sl_compact_active(None, 256, 0, 8, 256, 256) == B.SL_EINVAL
    assert lib.sl_score_posteriors(None, 256, 0, 256, 1, 1001, 256, 256, 4, 0, 256, 256, 256) == B.SL_EINVAL   # vocab % 8
    assert lib.sl_score_posteriors(None, 256, 0, None, 1, 1024, 256, 256, 4, 0, 256, 256, 256) == B.SL_EINVAL  # prev missing
    assert lib.sl_score_posteriors(None, 260, 0, 256, 1, 1024, 256, 256, 4, 0, 256, 256, 256) == B.SL_EINVAL   # alignment
    assert lib.sl_score_posteriors(None, 256, 0, 256, 5, 1024, 256, 256, 4, 0, 256, 256, 256) == B.SL_EINVAL   # dtype
    assert lib.sl_unmask_topk(None, 256, 256, 256, 256, 256, 256, 1, 64, 10, 65, 1) == B.SL_EINVAL
    assert lib.sl_unmask_topk(None, 256, 256, 256, 256, 256, 256, 1, 64, 10, 5, 1) == B.SL_EINVAL
    assert lib.sl_lock_rule(None, 256, 256, 256, 256, 4, 256, None, 1, 64, 0, 256) == B.SL_EINVAL
    assert lib.sl_lock_test(None, 256, 1, 256, 1, 1024, 256, 256, 256, 256, None, 4, 256, 1, 64, 0, 0, 64, 1,
                            256, 256, 256, 256) == B.SL_EINVAL
    fl = C.c_int64()
    assert lib.sl_peak_probe_mfma(None, 256, 8192, 0, 1, 256, 1 << 20, C.byref(fl)) == B.SL_EINVAL      # iters
    assert lib.sl_peak_probe_mfma(None, 256, 8192, 8, 3, 256, 1 << 20, C.byref(fl)) == B.SL_EINVAL      # waves per SIMD
    assert lib.sl_peak_probe_mfma(None, 256, 8192, 8, 1, 256, 1 << 20, None) == B.SL_EINVAL
    assert lib.sl_peak_probe_mfma(None, 256, 4096, 8, 1, 256, 1 << 20, C.byref(fl)) == B.SL_ENOSPC      # operands
    assert lib.sl_peak_probe_stream(None, 256, None, 40, 256, 1 << 21) == B.SL_EINVAL                   # bytes % 16
    assert lib.sl_peak_probe_stream(None, 256, 512, 1024, 256, 1 << 21) == B.SL_EINVAL                  # overlap
    assert lib.sl_peak_probe_stream(None, 264, None, 1024, 256, 1 << 21) == B.SL_EINVAL                 # alignment


def test_noalloc_draw_rejects_bad_arguments_without_gpu():
    """sl_sample_tokens_noalloc validates on the host before it touches HIP: null pointers and a row bound
    beyond its static buffer (16384 rows) are errors with no GPU present."""
    lib = B.lib()
    buf = (C.c_char * 64)()
    p = C.cast(buf, C.c_void_p)                    # any non-null address: nothing is dereferenced on the host
    ok = [None, p, 1, B.SL_BF16, 64, p, p, 16, p, 32, 0, 32, C.c_float(1.0), C.c_uint64(1), 1, p, p]
    bad = list(ok); bad[7] = 16385
    assert lib.sl_sample_tokens_noalloc(*bad) == B.SL_ENOSPC
    for i in (1, 5, 6, 8, 15, 16):
        bad = list(ok); bad[i] = None
        assert lib.sl_sample_tokens_noalloc(*bad) == B.SL_EINVAL
    bad = list(ok); bad[12] = C.c_float(0.0)
    assert lib.sl_sample_tokens_noalloc(*bad) == B.SL_EINVAL
    bad = list(ok); bad[4] = 63
    assert lib.sl_sample_tokens_noalloc(*bad) == B.SL_EINVAL
