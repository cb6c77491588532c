"""ctypes binding of libsurelock.so: the same entry points as include/surelock.h, taking
torch tensors (device memory) and Python ints.  Argument marshalling only: every step of the
path runs in the HIP kernels.  There is no fallback: a missing library raises."""
import ctypes as C
import os

import torch

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libsurelock.so")

SL_F32, SL_BF16 = 0, 1
SL_OK, SL_EINVAL, SL_ENOSPC, SL_EHIP, SL_ESTATE = 0, -1, -2, -3, -4


class sl_config(C.Structure):
    _fields_ = [("n_layers", C.c_int32), ("d_model", C.c_int32), ("n_heads", C.c_int32),
                ("d_head", C.c_int32), ("d_ff", C.c_int32), ("vocab", C.c_int32),
                ("dtype", C.c_int32), ("mask_id", C.c_int32),
                ("rms_eps", C.c_float), ("rope_theta", C.c_float), ("candidates_pre_update", C.c_int32),
                ("gate_percentile", C.c_float), ("temperature", C.c_float), ("seed", C.c_uint64)]


class sl_layer_weights(C.Structure):
    _fields_ = [(n, C.c_void_p) for n in ("attn_norm", "wq", "wk", "wv", "wo", "ffn_norm",
                                          "w_gate", "w_up", "w_down")]


class sl_weights(C.Structure):
    _fields_ = [("emb", C.c_void_p), ("final_norm", C.c_void_p), ("lm_head", C.c_void_p),
                ("layers", C.POINTER(sl_layer_weights))]


_P, _I, _Z = C.c_void_p, C.c_int32, C.c_size_t
_SIGS = {
    "sl_init": [C.POINTER(sl_config), C.POINTER(_P)],
    "sl_destroy": [_P],
    "sl_last_hip_error": [],
    "sl_packed_weights_bytes": [_P, C.POINTER(_Z)],
    "sl_bind_weights": [_P, _P, C.POINTER(sl_weights), _P, _Z],
    "sl_kv_cache_bytes": [_P, _I, _I, C.POINTER(_Z)],
    "sl_kv_cache_bind": [_P, _P, _P, _Z, _I, _I],
    "sl_kv_cache_read": [_P, _P, _I, _P, _P],
    "sl_posterior_bytes": [_P, _I, _I, C.POINTER(_Z)],
    "sl_posterior_bind": [_P, _P, _Z],
    "sl_logits_ptr": [_P, _I, C.POINTER(_P)],
    "sl_workspace_bytes": [_P, _I, _I, C.POINTER(_Z)],
    "sl_surelock_step": [_P, _P, _P, _P, _P, _P, _I, _I, _I, _I, _I, _P, _P, _P, _P, _P, _P, _P, _Z],
    "sl_surelock_step_selected": [_P, _P, _P, _P, _P, _P, _I, _I, _I, _I, C.c_float, _P, _P, _I, _P, _P, _P, _P, _P, _P,
                                  _P, _Z],
    "sl_forward_layers": [_P, _P, _P, _P, _P, _P, _I, _I, _I, _P, _Z],
    "sl_compact_active": [_P, _P, _I, _I, _P, _P],
    "sl_score_posteriors": [_P, _P, _I, _P, _I, _I, _P, _P, _I, _I, _P, _P, _P],
    "sl_unmask_topk": [_P, _P, _P, _P, _P, _P, _P, _I, _I, _I, _I, _I],
    "sl_lock_rule": [_P, _P, _P, _P, _P, _I, _P, _P, _I, _I, _I, _P],
    "sl_lock_rule_gated": [_P, _P, _P, _P, _P, _I, _P, _P, _P, C.c_float, _I, _I, _I, _P],
    "sl_select_rows": [_P, _P, _P, _P, _I, _I, _I, _I, C.c_float, _P],
    "sl_sample_tokens": [_P, _P, _I, _I, _I, _P, _P, _I, _P, _I, _I, _I, C.c_float, C.c_uint64, _I, _P, _P, _P, _Z],
    "sl_sample_tokens_noalloc": [_P, _P, _I, _I, _I, _P, _P, _I, _P, _I, _I, _I, C.c_float, C.c_uint64, _I, _P, _P],
    "sl_lock_rule_relock": [_P, _P, _P, _P, _P, _I, _P, _P, _P, C.c_float, _P, _P, C.c_float, _I, _I, _I, _P, _P],
    "sl_unlock_probe": [_P, _P, _P, _P, _P, _I, _P, _P, _P, _P, _P, _P, _P, _Z],
    "sl_unlock_rule": [_P, _P, _P, _P, _P, _P, _P, _P, _I, _P, _P, _P, _I, _P, C.c_float, C.c_float, _I, _I, _I, _P],
    "sl_linear_pack": [_P, _P, _I, _I, _P, _Z],
    "sl_linear_splits": [_I, _I, _I],
    "sl_linear_plan": [_I, _I, _I, C.POINTER(_I), C.POINTER(_I), C.POINTER(_I), C.POINTER(_I), C.POINTER(_I)],
    "sl_linear_forward": [_P, _P, _I, _P, _P, _I, _I, _I, _I, _P, _P, _P],
    "sl_linear_clock_probe": [_P, _P, _I, _P, _P, _I, _I, _I, _P, _P, _P],
    "sl_peak_probe_mfma": [_P, _P, _Z, _I, _I, _P, _Z, C.POINTER(C.c_int64)],
    "sl_peak_probe_stream": [_P, _P, _P, _Z, _P, _Z],
    "sl_profile_begin": [_P, _I],
    "sl_profile_end": [_P, C.POINTER(C.c_float), C.POINTER(_I)],
    "sl_lock_test": [_P, _P, _I, _P, _I, _I, _P, _P, _P, _P, _P, _I, _P, _I, _I, _I, _I, _I, _I, _P, _P, _P, _P],
}
EXPORTS = sorted(list(_SIGS) + ["sl_strerror"])

_lib = None


def lib():
    """The loaded C-ABI library (opened on first use)."""
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise RuntimeError(f"{LIB_PATH} is not built: run `python -m paper_2602_06412_amd.build`")
        l = C.CDLL(LIB_PATH)
        for name, args in _SIGS.items():
            fn = getattr(l, name)
            fn.argtypes = args
            fn.restype = C.c_int
        l.sl_strerror.argtypes = [C.c_int]
        l.sl_strerror.restype = C.c_char_p
        _lib = l
    return _lib


class SureLockError(RuntimeError):
    def __init__(self, fn, status):
        self.status = status
        msg = lib().sl_strerror(status).decode()
        if status == SL_EHIP:
            msg += f" [hipError {lib().sl_last_hip_error()}]"
        super().__init__(f"{fn}: {msg} ({status})")


def _check(fn, status):
    if status != SL_OK:
        raise SureLockError(fn, status)


def _ptr(t):
    if t is None:
        return None
    if isinstance(t, int):
        return t
    assert t.is_contiguous()
    return t.data_ptr()


def _stream():
    return torch.cuda.current_stream().cuda_stream


def dtype_code(dt):
    return {torch.float32: SL_F32, torch.bfloat16: SL_BF16}[dt]


def make_config(shape, candidates_pre_update=0, gate_percentile=0.0, temperature=0.0, seed=0):
    return sl_config(shape.n_layers, shape.d_model, shape.n_heads, shape.d_head, shape.d_ff, shape.vocab,
                     {"fp32": SL_F32, "bf16": SL_BF16}[shape.storage], shape.mask_id, shape.rms_eps,
                     shape.rope_theta, int(candidates_pre_update), float(gate_percentile), float(temperature), int(seed))


# ---- entry points, same names as the header -------------------------------------------------
def sl_init(cfg):
    h = _P()
    _check("sl_init", lib().sl_init(C.byref(cfg), C.byref(h)))
    return h


def sl_destroy(ctx):
    _check("sl_destroy", lib().sl_destroy(ctx))


def _size_query(name, ctx, *args):
    out = _Z()
    _check(name, getattr(lib(), name)(ctx, *args, C.byref(out)))
    return out.value


def sl_packed_weights_bytes(ctx):
    return _size_query("sl_packed_weights_bytes", ctx)


def sl_kv_cache_bytes(ctx, batch, n_seq):
    return _size_query("sl_kv_cache_bytes", ctx, batch, n_seq)


def sl_posterior_bytes(ctx, batch, n_seq):
    return _size_query("sl_posterior_bytes", ctx, batch, n_seq)


def sl_workspace_bytes(ctx, batch, n_seq):
    return _size_query("sl_workspace_bytes", ctx, batch, n_seq)


def sl_bind_weights(ctx, weights, packed):
    """weights: dict as made by workloads.make_weights (device tensors); packed: uint8 buffer."""
    n = len(weights["layers"])
    arr = (sl_layer_weights * n)()
    for i, l in enumerate(weights["layers"]):
        for f, _ in sl_layer_weights._fields_:
            setattr(arr[i], f, l[f].data_ptr())
    w = sl_weights(weights["emb"].data_ptr(), weights["final_norm"].data_ptr(), weights["lm_head"].data_ptr(), arr)
    _check("sl_bind_weights", lib().sl_bind_weights(ctx, _stream(), C.byref(w), _ptr(packed),
                                                    packed.numel() if packed is not None else 0))


def sl_kv_cache_bind(ctx, kv, batch, n_seq):
    _check("sl_kv_cache_bind", lib().sl_kv_cache_bind(ctx, _stream(), _ptr(kv), kv.numel(), batch, n_seq))


def sl_kv_cache_read(ctx, layer, k_out, v_out):
    _check("sl_kv_cache_read", lib().sl_kv_cache_read(ctx, _stream(), layer, _ptr(k_out), _ptr(v_out)))


def sl_posterior_bind(ctx, store):
    _check("sl_posterior_bind", lib().sl_posterior_bind(ctx, _ptr(store), store.numel()))


def sl_logits_ptr(ctx, t):
    out = _P()
    _check("sl_logits_ptr", lib().sl_logits_ptr(ctx, t, C.byref(out)))
    return out.value


def sl_surelock_step(ctx, tokens, masked, lock, eps, t, block_lo, block_hi, k, m_upper, active_idx, cu_active,
                     kl, conf, argmax, new_lock, workspace):
    _check("sl_surelock_step", lib().sl_surelock_step(
        ctx, _stream(), _ptr(tokens), _ptr(masked), _ptr(lock), _ptr(eps), t, block_lo, block_hi, k, m_upper,
        _ptr(active_idx), _ptr(cu_active), _ptr(kl), _ptr(conf), _ptr(argmax), _ptr(new_lock), _ptr(workspace),
        workspace.numel()))


def sl_surelock_step_selected(ctx, tokens, masked, lock, eps, t, block_lo, block_hi, k, select_fraction, d_last,
                              compute_mask, m_upper, active_idx, cu_active, kl, conf, argmax, new_lock, workspace):
    _check("sl_surelock_step_selected", lib().sl_surelock_step_selected(
        ctx, _stream(), _ptr(tokens), _ptr(masked), _ptr(lock), _ptr(eps), t, block_lo, block_hi, k,
        C.c_float(select_fraction), _ptr(d_last), _ptr(compute_mask), m_upper, _ptr(active_idx), _ptr(cu_active),
        _ptr(kl), _ptr(conf), _ptr(argmax), _ptr(new_lock), _ptr(workspace), workspace.numel()))


def sl_forward_layers(ctx, x_in, x_out, active_idx, m_dev, m_upper, layer_lo, layer_hi, workspace):
    _check("sl_forward_layers", lib().sl_forward_layers(
        ctx, _stream(), _ptr(x_in), _ptr(x_out), _ptr(active_idx), _ptr(m_dev), m_upper, layer_lo, layer_hi,
        _ptr(workspace), workspace.numel()))


def sl_compact_active(lock, batch, n_seq, active_idx, cu_active):
    _check("sl_compact_active", lib().sl_compact_active(_stream(), _ptr(lock), batch, n_seq, _ptr(active_idx),
                                                        _ptr(cu_active)))


def sl_score_posteriors(logits_cur, cur_packed, logits_prev, dtype, vocab, active_idx, m_dev, m_upper, first_step,
                        kl, conf, argmax):
    _check("sl_score_posteriors", lib().sl_score_posteriors(
        _stream(), _ptr(logits_cur), int(cur_packed), _ptr(logits_prev), dtype, vocab, _ptr(active_idx), _ptr(m_dev),
        m_upper, int(first_step), _ptr(kl), _ptr(conf), _ptr(argmax)))


def sl_unmask_topk(tokens, masked, active_idx, cu_active, conf, argmax, batch, n_seq, block_lo, block_hi, k):
    _check("sl_unmask_topk", lib().sl_unmask_topk(_stream(), _ptr(tokens), _ptr(masked), _ptr(active_idx),
                                                  _ptr(cu_active), _ptr(conf), _ptr(argmax), batch, n_seq, block_lo,
                                                  block_hi, k))


def sl_lock_rule(lock, masked, active_idx, m_dev, m_upper, kl, eps, batch, n_seq, first_step, new_lock):
    _check("sl_lock_rule", lib().sl_lock_rule(_stream(), _ptr(lock), _ptr(masked), _ptr(active_idx), _ptr(m_dev),
                                              m_upper, _ptr(kl), _ptr(eps), batch, n_seq, int(first_step),
                                              _ptr(new_lock)))


def sl_lock_rule_gated(lock, masked, active_idx, cu_active, m_upper, kl, conf, eps, gate_percentile, batch, n_seq,
                       first_step, new_lock):
    _check("sl_lock_rule_gated", lib().sl_lock_rule_gated(
        _stream(), _ptr(lock), _ptr(masked), _ptr(active_idx), _ptr(cu_active), m_upper, _ptr(kl), _ptr(conf), _ptr(eps),
        C.c_float(gate_percentile), batch, n_seq, int(first_step), _ptr(new_lock)))


def sl_sample_tokens(logits_cur, cur_packed, dtype, vocab, active_idx, m_dev, m_upper, masked, n_seq, block_lo, block_hi,
                     temperature, seed, t, argmax, write_id, scratch=None):
    if scratch is None:
        scratch = torch.empty(max(64 * m_upper, 64), dtype=torch.uint8, device=write_id.device)
    _check("sl_sample_tokens", lib().sl_sample_tokens(
        _stream(), _ptr(logits_cur), int(cur_packed), dtype, vocab, _ptr(active_idx), _ptr(m_dev), m_upper, _ptr(masked),
        n_seq, block_lo, block_hi, C.c_float(temperature), C.c_uint64(seed), t, _ptr(argmax), _ptr(write_id),
        _ptr(scratch), scratch.numel()))


def sl_sample_tokens_noalloc(logits_cur, cur_packed, dtype, vocab, active_idx, m_dev, m_upper, masked, n_seq, block_lo,
                             block_hi, temperature, seed, t, argmax, write_id):
    _check("sl_sample_tokens_noalloc", lib().sl_sample_tokens_noalloc(
        _stream(), _ptr(logits_cur), int(cur_packed), dtype, vocab, _ptr(active_idx), _ptr(m_dev), m_upper, _ptr(masked),
        n_seq, block_lo, block_hi, C.c_float(temperature), C.c_uint64(seed), t, _ptr(argmax), _ptr(write_id)))


def sl_select_rows(lock, masked, d_last, batch, n_seq, block_lo, block_hi, select_fraction, compute_mask):
    _check("sl_select_rows", lib().sl_select_rows(_stream(), _ptr(lock), _ptr(masked), _ptr(d_last), batch, n_seq,
                                                  block_lo, block_hi, C.c_float(select_fraction), _ptr(compute_mask)))


def sl_lock_rule_relock(lock, masked, active_idx, cu_active, m_upper, kl, conf, eps, gate_percentile, relocked,
                        cool_until, rho, t, batch, n_seq, new_lock, t_lock):
    _check("sl_lock_rule_relock", lib().sl_lock_rule_relock(
        _stream(), _ptr(lock), _ptr(masked), _ptr(active_idx), _ptr(cu_active), m_upper, _ptr(kl), _ptr(conf), _ptr(eps),
        C.c_float(gate_percentile), _ptr(relocked), _ptr(cool_until), C.c_float(rho), t, batch, n_seq, _ptr(new_lock),
        _ptr(t_lock)))


def sl_unlock_probe(ctx, tokens, lock, t_lock, m_upper, probe_idx, cu_probe, probe_logits, kl, conf, argmax, workspace):
    _check("sl_unlock_probe", lib().sl_unlock_probe(
        ctx, _stream(), _ptr(tokens), _ptr(lock), _ptr(t_lock), m_upper, _ptr(probe_idx), _ptr(cu_probe),
        _ptr(probe_logits), _ptr(kl), _ptr(conf), _ptr(argmax), _ptr(workspace), workspace.numel()))


def sl_unlock_rule(ctx, lock, relocked, cool_until, t_lock, probe_idx, cu_probe, m_upper_probe, kl_probe, conf_probe,
                   cu_active, m_upper_active, conf_active, percentile, eps_unlock, t, d_interval, d_cool, unlocked):
    _check("sl_unlock_rule", lib().sl_unlock_rule(
        ctx, _stream(), _ptr(lock), _ptr(relocked), _ptr(cool_until), _ptr(t_lock), _ptr(probe_idx), _ptr(cu_probe),
        m_upper_probe, _ptr(kl_probe), _ptr(conf_probe), _ptr(cu_active), m_upper_active, _ptr(conf_active),
        C.c_float(percentile), C.c_float(eps_unlock), t, d_interval, d_cool, _ptr(unlocked)))


def sl_lock_test(logits_cur, cur_packed, logits_prev, dtype, vocab, tokens, masked, lock, active_idx, cu_active,
                 m_upper, eps, batch, n_seq, first_step, block_lo, block_hi, k, kl, conf, argmax, new_lock):
    _check("sl_lock_test", lib().sl_lock_test(
        _stream(), _ptr(logits_cur), int(cur_packed), _ptr(logits_prev), dtype, vocab, _ptr(tokens), _ptr(masked),
        _ptr(lock), _ptr(active_idx), _ptr(cu_active), m_upper, _ptr(eps), batch, n_seq, int(first_step), block_lo,
        block_hi, k, _ptr(kl), _ptr(conf), _ptr(argmax), _ptr(new_lock)))


def sl_linear_pack(w, packed):
    n, k = w.shape
    _check("sl_linear_pack", lib().sl_linear_pack(_stream(), _ptr(w), n, k, _ptr(packed),
                                                  packed.numel() * packed.element_size()))


def sl_linear_splits(m_upper, n, k):
    r = lib().sl_linear_splits(m_upper, n, k)
    if r < 0:
        raise SureLockError("sl_linear_splits", r)
    return r


def sl_linear_plan(m_upper, n, k):
    """(kernel, splits, tile_rows, tile_cols, tail_tile) of the launch a row bound gets (host only)."""
    out = [_I() for _ in range(5)]
    _check("sl_linear_plan", lib().sl_linear_plan(m_upper, n, k, *[C.byref(o) for o in out]))
    return tuple(int(o.value) for o in out)


def sl_linear_forward(x, packed, m_dev, m_upper, n, k, splits=0, y_f32=None, y_bf16=None, row_map=None, x_tiled=0):
    _check("sl_linear_forward", lib().sl_linear_forward(_stream(), _ptr(x), int(x_tiled), _ptr(packed), _ptr(m_dev),
                                                        m_upper, n, k, splits, _ptr(y_f32), _ptr(y_bf16),
                                                        _ptr(row_map)))


def sl_linear_clock_probe(x, packed, m_dev, m_upper, n, k, y_bf16, counters, row_map=None, x_tiled=0):
    """counters: 8 x int64 on the device (see the header for their meaning)."""
    _check("sl_linear_clock_probe", lib().sl_linear_clock_probe(_stream(), _ptr(x), int(x_tiled), _ptr(packed), _ptr(m_dev),
                                                                m_upper, n, k, _ptr(y_bf16), _ptr(row_map), _ptr(counters)))


def _nbytes(t):
    return t.numel() * t.element_size()


def sl_peak_probe_mfma(operands, iters, waves_per_simd, sink):
    """Enqueues the bare MFMA loop; returns the floating-point operations of the launch."""
    flops = C.c_int64()
    _check("sl_peak_probe_mfma", lib().sl_peak_probe_mfma(_stream(), _ptr(operands), _nbytes(operands), int(iters),
                                                          int(waves_per_simd), _ptr(sink), _nbytes(sink), C.byref(flops)))
    return flops.value


def sl_peak_probe_stream(src, dst, sink):
    """Enqueues one streaming pass over src (dst None: read only; else copy)."""
    _check("sl_peak_probe_stream", lib().sl_peak_probe_stream(_stream(), _ptr(src), _ptr(dst), _nbytes(src), _ptr(sink),
                                                              _nbytes(sink)))


def tile_activations(x):
    """[rows, k] bf16 row-major -> the fragment-tiled layout sl_linear_forward(x_tiled=1) reads
    (rows padded to a multiple of 32).  A torch permutation, for tests and tuning."""
    rows, k = x.shape
    r32 = (rows + 31) // 32 * 32
    xp = torch.zeros(r32, k, dtype=x.dtype, device=x.device)
    xp[:rows] = x
    # [mb, r, kb, half, e] -> [mb, kb, half, r, e]
    return xp.view(r32 // 32, 32, k // 16, 2, 8).permute(0, 2, 3, 1, 4).contiguous().view(-1)


PROF_SLOTS = ["compact", "embed_norm", "gemm_qkv", "rope_kv", "attention", "gemm_out", "add_norm", "gemm_gate_up",
              "swiglu", "gemm_down", "lm_head", "score", "unmask", "lock_rule"]


def sl_profile_begin(ctx, max_launches):
    _check("sl_profile_begin", lib().sl_profile_begin(ctx, max_launches))


def sl_profile_end(ctx):
    """Returns {slot name: (total ms, launches)}."""
    n = len(PROF_SLOTS)
    ms, cnt = (C.c_float * n)(), (_I * n)()
    _check("sl_profile_end", lib().sl_profile_end(ctx, ms, cnt))
    return {PROF_SLOTS[i]: (float(ms[i]), int(cnt[i])) for i in range(n)}


# ---- device-memory plumbing for one model + one batch geometry ---------------------------------
class Session:
    """Owns the torch buffers a context needs (packed weights, K/V cache, posterior store,
    workspace, per-step outputs) and forwards to the entry points above."""

    def __init__(self, shape, weights, batch, n_seq, device="cuda:0", candidates_pre_update=False,
                 gate_percentile=0.0, temperature=0.0, seed=0, packed=None):
        self.shape, self.B, self.N, self.device = shape, batch, n_seq, torch.device(device)
        self.weights = weights
        self.T = {"fp32": torch.float32, "bf16": torch.bfloat16}[shape.storage]
        self.ctx = sl_init(make_config(shape, candidates_pre_update, gate_percentile, temperature, seed))
        dev = self.device
        u8 = lambda n: torch.empty(max(int(n), 256), dtype=torch.uint8, device=dev)
        # `packed`: a buffer another session of the same model already holds its re-tiled weights in (it is
        # written again with the same bytes); saves a second copy of the weights
        need = sl_packed_weights_bytes(self.ctx)
        self.packed = u8(need) if packed is None else packed
        assert self.packed.numel() >= need
        sl_bind_weights(self.ctx, weights, self.packed)
        self.kv = u8(sl_kv_cache_bytes(self.ctx, batch, n_seq))
        sl_kv_cache_bind(self.ctx, self.kv, batch, n_seq)
        self.post = u8(sl_posterior_bytes(self.ctx, batch, n_seq))
        sl_posterior_bind(self.ctx, self.post)
        self.workspace = u8(sl_workspace_bytes(self.ctx, batch, n_seq))
        R = batch * n_seq
        self.active_idx = torch.zeros(R, dtype=torch.int32, device=dev)
        self.cu_active = torch.zeros(batch + 1, dtype=torch.int32, device=dev)
        self.kl = torch.zeros(R, dtype=torch.float32, device=dev)
        self.conf = torch.zeros(R, dtype=torch.float32, device=dev)
        self.argmax = torch.zeros(R, dtype=torch.int32, device=dev)

    def close(self):
        if self.ctx is not None:
            torch.cuda.synchronize()
            sl_destroy(self.ctx)
            self.ctx = None

    def step(self, tokens, masked, lock, eps, t, block_lo, block_hi, k, m_upper=None, new_lock=None):
        m_upper = self.B * self.N if m_upper is None else m_upper
        new_lock = lock if new_lock is None else new_lock
        sl_surelock_step(self.ctx, tokens, masked, lock, eps, t, block_lo, block_hi, k, m_upper, self.active_idx,
                         self.cu_active, self.kl, self.conf, self.argmax, new_lock, self.workspace)
        return new_lock

    def step_selected(self, tokens, masked, lock, eps, t, block_lo, block_hi, k, select_fraction, m_upper=None,
                      new_lock=None):
        """The step on the fraction of the non-locked rows the selection keeps (d_last and compute_mask
        are owned here; d_last starts at +inf)."""
        if not hasattr(self, "d_last"):
            R = self.B * self.N
            self.d_last = torch.full((R,), float("inf"), dtype=torch.float32, device=self.device)
            self.compute_mask = torch.zeros(R, dtype=torch.uint8, device=self.device)
        m_upper = self.B * self.N if m_upper is None else m_upper
        new_lock = lock if new_lock is None else new_lock
        sl_surelock_step_selected(self.ctx, tokens, masked, lock, eps, t, block_lo, block_hi, k, select_fraction,
                                  self.d_last, self.compute_mask, m_upper, self.active_idx, self.cu_active, self.kl,
                                  self.conf, self.argmax, new_lock, self.workspace)
        return new_lock

    # -- optional unlocking: per-position state and probe outputs, allocated on first use --
    def unlock_state(self):
        if not hasattr(self, "t_lock"):
            dev, R = self.device, self.B * self.N
            self.t_lock = torch.zeros(R, dtype=torch.int32, device=dev)
            self.cool_until = torch.zeros(R, dtype=torch.int32, device=dev)
            self.relocked = torch.zeros(R, dtype=torch.uint8, device=dev)
            self.probe_idx = torch.zeros(R, dtype=torch.int32, device=dev)
            self.cu_probe = torch.zeros(self.B + 1, dtype=torch.int32, device=dev)
            self.probe_logits = torch.zeros(R, self.shape.vocab, dtype=self.T, device=dev)
            self.probe_kl = torch.zeros(R, dtype=torch.float32, device=dev)
            self.probe_conf = torch.zeros(R, dtype=torch.float32, device=dev)
            self.probe_argmax = torch.zeros(R, dtype=torch.int32, device=dev)
            self.unlocked = torch.zeros(R, dtype=torch.uint8, device=dev)
            self.rule_scratch = torch.zeros(R, dtype=torch.uint8, device=dev)
        return self

    def step_unlockable(self, tokens, masked, lock, eps, t, block_lo, block_hi, k, rho, gate_percentile=0.0,
                        m_upper=None):
        """One step whose lock rule obeys the cool-down and the stricter re-lock threshold and
        records the lock time: the step's own rule output is discarded, sl_lock_rule_relock decides
        (on the masked flags UpdateMASK left, the default candidate reading).  lock is updated in place."""
        self.unlock_state()
        m_upper = self.B * self.N if m_upper is None else m_upper
        sl_surelock_step(self.ctx, tokens, masked, lock, eps, t, block_lo, block_hi, k, m_upper, self.active_idx,
                         self.cu_active, self.kl, self.conf, self.argmax, self.rule_scratch, self.workspace)
        sl_lock_rule_relock(lock, masked, self.active_idx, self.cu_active, m_upper, self.kl, self.conf, eps,
                            gate_percentile, self.relocked, self.cool_until, rho, t, self.B, self.N, lock, self.t_lock)
        return lock

    def unlock_probe(self, tokens, lock, t, percentile, eps_unlock, d_interval, d_cool, m_upper_probe=None,
                     m_upper_active=None):
        """The read-only probe on the locked rows followed by the unlock rule, after step t."""
        self.unlock_state()
        R = self.B * self.N
        mp = R if m_upper_probe is None else m_upper_probe
        ma = R if m_upper_active is None else m_upper_active
        sl_unlock_probe(self.ctx, tokens, lock, self.t_lock, mp, self.probe_idx, self.cu_probe, self.probe_logits,
                        self.probe_kl, self.probe_conf, self.probe_argmax, self.workspace)
        sl_unlock_rule(self.ctx, lock, self.relocked, self.cool_until, self.t_lock, self.probe_idx, self.cu_probe, mp,
                       self.probe_kl, self.probe_conf, self.cu_active, ma, self.conf, percentile, eps_unlock, t,
                       d_interval, d_cool, self.unlocked)
        return lock

    def logits_view(self, t):
        """[B*N, V] tensor view of the posterior buffer step t writes (rows by flat id)."""
        buf = self.post.view(self.T)
        per = buf.numel() // 2
        R, V = self.B * self.N, self.shape.vocab
        return buf[(t & 1) * per:(t & 1) * per + R * V].view(R, V)

    def forward_layers(self, x_in, active_idx, m_dev, m_upper, layer_lo=0, layer_hi=None):
        layer_hi = self.shape.n_layers if layer_hi is None else layer_hi
        x_out = torch.empty_like(x_in)
        sl_forward_layers(self.ctx, x_in, x_out, active_idx, m_dev, m_upper, layer_lo, layer_hi, self.workspace)
        return x_out

    def kv_read(self, layer):
        s = self.shape
        k = torch.empty(self.B, self.N, s.n_heads, s.d_head, dtype=self.T, device=self.device)
        v = torch.empty_like(k)
        sl_kv_cache_read(self.ctx, layer, k, v)
        return k, v
