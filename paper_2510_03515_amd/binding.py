"""ctypes binding over librapid_hip.so: argument marshalling only.

Every function mirrors one entry point of include/rapid.h with the same name and takes torch
tensors that live on the GPU (PyTorch supplies device memory and the current stream, nothing
else).  There is no CPU fallback: if the library has not been built, loading raises.
"""
from __future__ import annotations

import ctypes as C
import math
import os

import torch

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "librapid_hip.so")

RAPID_OK = 0
DTYPE_F32, DTYPE_BF16 = 0, 1
W_DV, W_VD = 0, 1
OP_LOGPROB_FWD, OP_GROUP_ADVANTAGE, OP_IW_PG_FWD_BWD, OP_IW_PG_FWD_BWD_CACHED = 0, 1, 2, 3
STATUS_BAD_TOKEN, STATUS_BAD_GROUP, STATUS_NONFINITE_REWARD, STATUS_NONFINITE_LOGP, STATUS_LOGIT_RANGE = 1, 2, 4, 8, 16
STATUS_TOKEN_BOUND = 32
STATUS_GROUP_LAYOUT = 64

EXPORTS = ["rapid_version", "rapid_last_error", "rapid_logits_cache_rows", "rapid_iw_pg_default_opts", "rapid_set_tuning",
           "rapid_workspace_bytes", "rapid_workspace_min_bytes", "rapid_workspace_bytes_max_tokens", "rapid_logprob_fwd", "rapid_logprob_fwd_rmsnorm",
           "rapid_group_advantage", "rapid_iw_pg_loss_fwd_bwd", "rapid_compaction", "rapid_profile_read", "rapid_mfma_probe", "rapid_sgd_step",
           "rapid_logprob_fwd_static", "rapid_clip_pg_default_opts", "rapid_clip_pg_loss_fwd_bwd",
           "rapid_seq_logratio", "rapid_adamw_step"]
STAGES = ["compaction", "pack", "fwd_lse", "merge_lse", "estimator", "zero_rows", "dz", "unused", "dh",
          "dw", "f32_path", "dw_convert"]


class RapidError(RuntimeError):
    def __init__(self, code, msg):
        super().__init__(f"rapid error {code}: {msg}")
        self.code = code


class IwPgOpts(C.Structure):
    _fields_ = [("eta", C.c_float), ("coef_mode", C.c_int), ("baseline_mode", C.c_int),
                ("loss_scale", C.c_float), ("temperature", C.c_float), ("w_layout", C.c_int),
                ("dw_dtype", C.c_int), ("accumulate_dw", C.c_int), ("normalized_grads", C.c_int),
                ("logits_cache", C.c_int), ("ratio_level", C.c_int), ("max_tokens", C.c_int64),
                ("coef_override", C.c_void_p), ("rms_weight", C.c_void_p), ("drms_weight_out", C.c_void_p),
                ("rms_eps", C.c_float)]


class ClipPgOpts(C.Structure):
    _fields_ = [("eps_low", C.c_float), ("eps_high", C.c_float), ("kl_beta", C.c_float), ("norm_mode", C.c_int),
                ("adv_eps", C.c_float), ("std_ddof", C.c_int), ("loss_scale", C.c_float), ("temperature", C.c_float),
                ("w_layout", C.c_int), ("dw_dtype", C.c_int), ("accumulate_dw", C.c_int), ("logits_cache", C.c_int),
                ("max_tokens", C.c_int64)]


class ClipPgDiag(C.Structure):
    _fields_ = [("n_tokens", C.c_int64), ("n_clipped", C.c_int64), ("n_sequences", C.c_int32), ("mean_kl", C.c_float)]


class IwPgDiag(C.Structure):
    _fields_ = [("n_tokens", C.c_int64), ("n_clipped", C.c_int32), ("n_sequences", C.c_int32),
                ("mean_log_w", C.c_float), ("mean_abs_log_w", C.c_float), ("max_abs_s", C.c_float),
                ("grad_log_scale", C.c_float)]


_lib = None


def load():
    """Loads the built library (once).  Raises if it is missing: there is no fallback path."""
    global _lib
    if _lib is not None:
        return _lib
    if not os.path.exists(LIB_PATH):
        raise RuntimeError(f"{LIB_PATH} is not built; run `python -m paper_2510_03515_amd.build`")
    lib = C.CDLL(LIB_PATH)
    i64, vp, f32, sz, ci = C.c_int64, C.c_void_p, C.c_float, C.c_size_t, C.c_int
    lib.rapid_version.restype = ci
    lib.rapid_last_error.restype = C.c_char_p
    lib.rapid_iw_pg_default_opts.argtypes = [C.POINTER(IwPgOpts)]
    lib.rapid_iw_pg_default_opts.restype = None
    lib.rapid_set_tuning.argtypes = [ci, ci]
    lib.rapid_set_tuning.restype = ci
    for fn in (lib.rapid_workspace_bytes, lib.rapid_workspace_min_bytes):
        fn.argtypes = [ci, i64, i64, i64, i64, i64, ci]
        fn.restype = sz
    lib.rapid_workspace_bytes_max_tokens.argtypes = [ci, i64, i64, i64, i64, i64, ci, i64]
    lib.rapid_workspace_bytes_max_tokens.restype = sz
    lib.rapid_logits_cache_rows.argtypes = [i64, i64, i64, i64, i64, i64, sz]
    lib.rapid_logits_cache_rows.restype = i64
    lib.rapid_logprob_fwd.argtypes = [vp, vp, vp, vp, i64, i64, i64, i64, ci, ci, f32, vp, vp, vp, vp, sz, vp]
    lib.rapid_logprob_fwd.restype = ci
    lib.rapid_logprob_fwd_static.argtypes = [vp, vp, vp, vp, i64, i64, i64, i64, ci, ci, f32, vp, vp, vp, vp]
    lib.rapid_logprob_fwd_static.restype = ci
    lib.rapid_logprob_fwd_rmsnorm.argtypes = [vp, vp, vp, vp, i64, i64, i64, i64, ci, ci, f32, vp, f32, vp, vp, vp, vp, sz, vp]
    lib.rapid_logprob_fwd_rmsnorm.restype = ci
    lib.rapid_group_advantage.argtypes = [vp, vp, vp, i64, i64, f32, ci, vp, vp, vp, vp, vp, vp, vp]
    lib.rapid_group_advantage.restype = ci
    lib.rapid_iw_pg_loss_fwd_bwd.argtypes = [vp, vp, vp, vp, vp, vp, vp, i64, i64, i64, i64, i64, ci,
                                             C.POINTER(IwPgOpts), vp, vp, vp, vp, vp, vp, vp, vp, vp, vp, sz, vp]
    lib.rapid_iw_pg_loss_fwd_bwd.restype = ci
    lib.rapid_clip_pg_default_opts.argtypes = [C.POINTER(ClipPgOpts), ci]
    lib.rapid_clip_pg_default_opts.restype = None
    lib.rapid_clip_pg_loss_fwd_bwd.argtypes = [vp, vp, vp, vp, vp, vp, vp, vp, i64, i64, i64, i64, i64, ci,
                                               C.POINTER(ClipPgOpts), vp, vp, vp, vp, vp, vp, vp, vp, sz, vp]
    lib.rapid_clip_pg_loss_fwd_bwd.restype = ci
    lib.rapid_compaction.argtypes = [vp, i64, i64, vp, vp, vp, vp]
    lib.rapid_compaction.restype = ci
    lib.rapid_profile_read.argtypes = [C.POINTER(C.c_double), C.POINTER(C.c_int64), ci]
    lib.rapid_profile_read.restype = ci
    lib.rapid_mfma_probe.argtypes = [ci, ci, C.POINTER(C.c_double), C.POINTER(C.c_double), C.c_void_p]
    lib.rapid_mfma_probe.restype = ci
    lib.rapid_sgd_step.argtypes = [vp, vp, i64, C.c_float, vp, ci, vp]
    lib.rapid_sgd_step.restype = ci
    lib.rapid_adamw_step.argtypes = [vp, vp, vp, vp, i64, f32, f32, f32, f32, f32, i64, vp, ci, vp]
    lib.rapid_adamw_step.restype = ci
    lib.rapid_seq_logratio.argtypes = [vp, vp, vp, i64, i64, vp, vp, vp, vp]
    lib.rapid_seq_logratio.restype = ci
    _lib = lib
    return lib


def _check(rc):
    if rc != RAPID_OK:
        raise RapidError(rc, load().rapid_last_error().decode())


def _ptr(t):
    return None if t is None else C.c_void_p(t.data_ptr())


def _stream():
    return C.c_void_p(torch.cuda.current_stream().cuda_stream)


def _dtype_code(t):
    if t.dtype == torch.bfloat16:
        return DTYPE_BF16
    if t.dtype == torch.float32:
        return DTYPE_F32
    raise TypeError(f"unsupported dtype {t.dtype}")


def _need(t, dtype, name):
    if not t.is_cuda or not t.is_contiguous() or t.dtype != dtype:
        raise TypeError(f"{name}: need a contiguous {dtype} tensor on the GPU")


def rapid_version():
    return load().rapid_version()


def rapid_set_tuning(key, value):
    _check(load().rapid_set_tuning(key, value))


def rapid_mfma_probe(random_operands, iters=100000):
    """Returns (TFLOP/s, milliseconds) of the MFMA-only probe kernel."""
    tf, ms = C.c_double(0.0), C.c_double(0.0)
    _check(load().rapid_mfma_probe(int(bool(random_operands)), int(iters), C.byref(tf), C.byref(ms), _stream()))
    return tf.value, ms.value


def rapid_sgd_step(master, grad, lr, w_out=None):
    """master (fp32) -= lr * grad (fp32), and w_out (bf16 or fp32, optional) = the updated weights."""
    _need(master, torch.float32, "master"); _need(grad, torch.float32, "grad")
    assert master.numel() == grad.numel() and (w_out is None or w_out.numel() == master.numel())
    dt = DTYPE_F32 if w_out is None else _dtype_code(w_out)
    _check(load().rapid_sgd_step(_ptr(master), _ptr(grad), master.numel(), float(lr), _ptr(w_out), dt, _stream()))


def rapid_adamw_step(master, grad, exp_avg, exp_avg_sq, step, lr, beta1=0.9, beta2=0.999, eps=1e-8, weight_decay=0.0,
                     w_out=None):
    """One AdamW step on fp32 master weights (exp_avg / exp_avg_sq: the optimiser state, zero before step 1), and
    w_out (bf16 or fp32, optional) = the updated weights."""
    for t, name in ((master, "master"), (grad, "grad"), (exp_avg, "exp_avg"), (exp_avg_sq, "exp_avg_sq")):
        _need(t, torch.float32, name)
    assert master.numel() == grad.numel() == exp_avg.numel() == exp_avg_sq.numel()
    dt = DTYPE_F32 if w_out is None else _dtype_code(w_out)
    _check(load().rapid_adamw_step(_ptr(master), _ptr(grad), _ptr(exp_avg), _ptr(exp_avg_sq), master.numel(), float(lr),
                                   float(beta1), float(beta2), float(eps), float(weight_decay), int(step), _ptr(w_out), dt,
                                   _stream()))


def rapid_seq_logratio(logp_cur, logp_behav, mask, want_tokens=False, dev_status=None):
    """Returns (seq_logratio [N] f32, tok_logratio [N,T] f32 or None)."""
    N, T = mask.shape
    _need(logp_cur, torch.float32, "logp_cur"); _need(logp_behav, torch.float32, "logp_behav"); _need(mask, torch.uint8, "mask")
    s = torch.empty(N, dtype=torch.float32, device=mask.device)
    tok = torch.empty((N, T), dtype=torch.float32, device=mask.device) if want_tokens else None
    _check(load().rapid_seq_logratio(_ptr(logp_cur), _ptr(logp_behav), _ptr(mask), N, T, _ptr(tok), _ptr(s),
                                     _ptr(dev_status), _stream()))
    return s, tok


def rapid_profile_read():
    """Returns {stage: (milliseconds, spans)} for the calls made since profiling was switched on
    (rapid_set_tuning(1, 1)) or last read."""
    n = len(STAGES)
    ms = (C.c_double * n)()
    cnt = (C.c_int64 * n)()
    _check(load().rapid_profile_read(ms, cnt, n))
    return {STAGES[i]: (ms[i], cnt[i]) for i in range(n)}


def rapid_workspace_bytes(op, N, T, d, V, K, dtype, minimum=False, max_tokens=0):
    lib = load()
    if max_tokens:
        return lib.rapid_workspace_bytes_max_tokens(op, N, T, d, V, K, dtype, int(max_tokens))
    fn = lib.rapid_workspace_min_bytes if minimum else lib.rapid_workspace_bytes
    return fn(op, N, T, d, V, K, dtype)


def rapid_logits_cache_rows(N, T, d, V, K, max_tokens, workspace_bytes):
    return load().rapid_logits_cache_rows(N, T, d, V, K, int(max_tokens), int(workspace_bytes))


def alloc_workspace(nbytes, device="cuda"):
    return torch.empty(int(nbytes), dtype=torch.uint8, device=device)


def rapid_compaction(mask):
    N, T = mask.shape
    _need(mask, torch.uint8, "mask")
    seq_len = torch.empty(N, dtype=torch.int32, device=mask.device)
    cu = torch.empty(N + 1, dtype=torch.int32, device=mask.device)
    row_index = torch.full((N * T,), -1, dtype=torch.int32, device=mask.device)
    _check(load().rapid_compaction(_ptr(mask), N, T, _ptr(seq_len), _ptr(cu), _ptr(row_index), _stream()))
    return seq_len, cu, row_index


def rapid_logprob_fwd(hidden, W, tokens, mask, w_layout=W_DV, temperature=1.0, want_lse=False,
                      workspace=None, dev_status=None, rms_weight=None, rms_eps=1e-6):
    """Returns (logp [N,T] f32, lse [N,T] f32 or None).  With rms_weight [d] (bf16), `hidden` is the
    input of the final RMSNorm, which is applied on the way in."""
    N, T, d = hidden.shape
    V = W.shape[1] if w_layout == W_DV else W.shape[0]
    dt = _dtype_code(hidden)
    _need(hidden, hidden.dtype, "hidden"); _need(W, hidden.dtype, "W")
    _need(tokens, torch.int32, "tokens"); _need(mask, torch.uint8, "mask")
    if workspace is None:
        workspace = alloc_workspace(rapid_workspace_bytes(OP_LOGPROB_FWD, N, T, d, V, 1, dt), hidden.device)
    logp = torch.empty((N, T), dtype=torch.float32, device=hidden.device)
    lse = torch.empty((N, T), dtype=torch.float32, device=hidden.device) if want_lse else None
    if rms_weight is not None:
        _need(rms_weight, hidden.dtype, "rms_weight")
        _check(load().rapid_logprob_fwd_rmsnorm(_ptr(hidden), _ptr(W), _ptr(tokens), _ptr(mask), N, T, d, V, dt,
                                                w_layout, float(temperature), _ptr(rms_weight), float(rms_eps),
                                                _ptr(logp), _ptr(lse), _ptr(dev_status), _ptr(workspace),
                                                workspace.numel(), _stream()))
        return logp, lse
    _check(load().rapid_logprob_fwd(_ptr(hidden), _ptr(W), _ptr(tokens), _ptr(mask), N, T, d, V, dt, w_layout,
                                    float(temperature), _ptr(logp), _ptr(lse), _ptr(dev_status),
                                    _ptr(workspace), workspace.numel(), _stream()))
    return logp, lse


def rapid_logprob_fwd_static(hidden, W, tokens, mask, logp_out, lse_out=None, w_layout=W_DV, temperature=1.0,
                             dev_status=None):
    """rapid_logprob_fwd on the library's static scratch: no workspace, and nothing is allocated here
    either (the caller brings the outputs).  Returns (logp_out, lse_out)."""
    N, T, d = hidden.shape
    V = W.shape[1] if w_layout == W_DV else W.shape[0]
    dt = _dtype_code(hidden)
    _need(hidden, hidden.dtype, "hidden"); _need(W, hidden.dtype, "W")
    _need(tokens, torch.int32, "tokens"); _need(mask, torch.uint8, "mask")
    _need(logp_out, torch.float32, "logp_out")
    if lse_out is not None:
        _need(lse_out, torch.float32, "lse_out")
    _check(load().rapid_logprob_fwd_static(_ptr(hidden), _ptr(W), _ptr(tokens), _ptr(mask), N, T, d, V, dt, w_layout,
                                           float(temperature), _ptr(logp_out), _ptr(lse_out), _ptr(dev_status),
                                           _stream()))
    return logp_out, lse_out


def rapid_group_advantage(rewards, group_ids, K, seq_logratio=None, eta=2.0, baseline_mode=0,
                          dev_status=None):
    """Returns dict(adv, weight, group_mean, group_std, group_size)."""
    N = rewards.shape[0]
    _need(rewards, torch.float32, "rewards"); _need(group_ids, torch.int32, "group_ids")
    if seq_logratio is not None:
        _need(seq_logratio, torch.float32, "seq_logratio")
    dev = rewards.device
    adv = torch.empty(N, dtype=torch.float32, device=dev)
    weight = torch.empty(N, dtype=torch.float32, device=dev)
    gmean = torch.empty(K, dtype=torch.float32, device=dev)
    gstd = torch.empty(K, dtype=torch.float32, device=dev)
    gsize = torch.empty(K, dtype=torch.int32, device=dev)
    _check(load().rapid_group_advantage(_ptr(rewards), _ptr(group_ids), _ptr(seq_logratio), N, K, float(eta),
                                        baseline_mode, _ptr(adv), _ptr(weight), _ptr(gmean), _ptr(gstd),
                                        _ptr(gsize), _ptr(dev_status), _stream()))
    return dict(adv=adv, weight=weight, group_mean=gmean, group_std=gstd, group_size=gsize)


def default_opts():
    o = IwPgOpts()
    load().rapid_iw_pg_default_opts(C.byref(o))
    return o


class IwPgBuffers:
    """Output and workspace tensors of rapid_iw_pg_loss_fwd_bwd, allocated once and reusable."""

    def __init__(self, hidden, W, K, w_layout=W_DV, dw_dtype=torch.float32, workspace_bytes=None,
                 minimum_workspace=False, logits_cache=False, max_tokens=0):
        N, T, d = hidden.shape
        V = W.shape[1] if w_layout == W_DV else W.shape[0]
        dev = hidden.device
        dt = _dtype_code(hidden)
        if workspace_bytes is None:
            op = OP_IW_PG_FWD_BWD_CACHED if logits_cache else OP_IW_PG_FWD_BWD
            workspace_bytes = rapid_workspace_bytes(op, N, T, d, V, K, dt, minimum=minimum_workspace,
                                                    max_tokens=max_tokens if logits_cache else 0)
        self.workspace = alloc_workspace(workspace_bytes, dev)
        self.loss = torch.empty(1, dtype=torch.float32, device=dev)
        self.dhidden = torch.empty_like(hidden)
        self.dW = torch.empty(W.shape, dtype=dw_dtype, device=dev)
        self.logp_cur = torch.empty((N, T), dtype=torch.float32, device=dev)
        self.tok_logratio = torch.empty((N, T), dtype=torch.float32, device=dev)
        self.seq_logratio = torch.empty(N, dtype=torch.float32, device=dev)
        self.adv = torch.empty(N, dtype=torch.float32, device=dev)
        self.diag = torch.zeros(C.sizeof(IwPgDiag), dtype=torch.uint8, device=dev)
        self.dev_status = torch.zeros(1, dtype=torch.int32, device=dev)

    def read_diag(self):
        raw = bytes(self.diag.cpu().numpy().tobytes())
        dg = IwPgDiag.from_buffer_copy(raw)
        return {f: getattr(dg, f) for f, _ in IwPgDiag._fields_}


def rapid_iw_pg_loss_fwd_bwd(hidden, W, tokens, mask, logp_behav, rewards, group_ids, K, buffers=None,
                             eta=2.0, coef_mode=0, baseline_mode=0, loss_scale=1.0, temperature=1.0,
                             w_layout=W_DV, accumulate_dw=False, normalized_grads=False, coef_override=None,
                             optional_outputs=True, logits_cache=False, ratio_level=0, max_tokens=0,
                             rms_weight=None, rms_eps=1e-6):
    """Enqueues the fused forward+backward on the current stream and returns the IwPgBuffers that
    hold the outputs (loss, dhidden, dW, logp_cur, tok_logratio, seq_logratio, adv, diag)."""
    N, T, d = hidden.shape
    V = W.shape[1] if w_layout == W_DV else W.shape[0]
    dt = _dtype_code(hidden)
    _need(hidden, hidden.dtype, "hidden"); _need(W, hidden.dtype, "W")
    _need(tokens, torch.int32, "tokens"); _need(mask, torch.uint8, "mask")
    if logp_behav is not None:          # None: on-policy (Sec. 3.3), all ratios 1
        _need(logp_behav, torch.float32, "logp_behav")
    _need(rewards, torch.float32, "rewards")
    _need(group_ids, torch.int32, "group_ids")
    if buffers is None:
        buffers = IwPgBuffers(hidden, W, K, w_layout, logits_cache=logits_cache, max_tokens=max_tokens)
    b = buffers
    o = default_opts()
    o.eta = float(eta) if math.isfinite(eta) else float("inf")
    o.coef_mode, o.baseline_mode = int(coef_mode), int(baseline_mode)
    o.loss_scale, o.temperature = float(loss_scale), float(temperature)
    o.w_layout = int(w_layout)
    o.dw_dtype = _dtype_code(b.dW)
    o.accumulate_dw = int(bool(accumulate_dw))
    o.normalized_grads = int(bool(normalized_grads))
    o.logits_cache = int(bool(logits_cache))
    o.ratio_level = int(ratio_level)
    o.max_tokens = int(max_tokens)
    if rms_weight is not None:          # hidden is the input of the final RMSNorm; dhidden is dLoss/d(that input)
        _need(rms_weight, hidden.dtype, "rms_weight")
        if getattr(b, "drms_weight", None) is None:
            b.drms_weight = torch.empty(d, dtype=torch.float32, device=hidden.device)
        o.rms_weight, o.rms_eps, o.drms_weight_out = rms_weight.data_ptr(), float(rms_eps), b.drms_weight.data_ptr()
    if coef_override is not None:
        _need(coef_override, torch.float32, "coef_override")
        o.coef_override = coef_override.data_ptr()
    opt = optional_outputs
    _check(load().rapid_iw_pg_loss_fwd_bwd(
        _ptr(hidden), _ptr(W), _ptr(tokens), _ptr(mask), _ptr(logp_behav), _ptr(rewards), _ptr(group_ids),
        N, T, d, V, K, dt, C.byref(o), _ptr(b.loss), _ptr(b.dhidden), _ptr(b.dW),
        _ptr(b.logp_cur) if opt else None, _ptr(b.tok_logratio) if opt else None,
        _ptr(b.seq_logratio) if opt else None, _ptr(b.adv) if opt else None,
        _ptr(b.diag) if opt else None, _ptr(b.dev_status), _ptr(b.workspace), b.workspace.numel(), _stream()))
    return b


def clip_pg_default_opts(variant="grpo"):
    o = ClipPgOpts()
    load().rapid_clip_pg_default_opts(C.byref(o), {"grpo": 0, "dapo": 1}[variant])
    return o


def rapid_clip_pg_loss_fwd_bwd(hidden, W, tokens, mask, logp_old, logp_ref, rewards, group_ids, K, variant="grpo",
                               buffers=None, w_layout=W_DV, accumulate_dw=False, logits_cache=False, max_tokens=0,
                               optional_outputs=True, **overrides):
    """The loss step of the GRPO ("grpo") or DAPO ("dapo") baseline on the current stream; `overrides` replace
    fields of the variant's default options (eps_low, eps_high, kl_beta, norm_mode, adv_eps, std_ddof, loss_scale,
    temperature).  Returns the IwPgBuffers that hold loss, dhidden, dW, logp_cur, adv; the call's diagnostics are in
    buffers.clip_diag (read_clip_diag)."""
    N, T, d = hidden.shape
    V = W.shape[1] if w_layout == W_DV else W.shape[0]
    dt = _dtype_code(hidden)
    _need(hidden, hidden.dtype, "hidden"); _need(W, hidden.dtype, "W")
    _need(tokens, torch.int32, "tokens"); _need(mask, torch.uint8, "mask")
    for t, name in ((logp_old, "logp_old"), (logp_ref, "logp_ref")):
        if t is not None:
            _need(t, torch.float32, name)
    _need(rewards, torch.float32, "rewards"); _need(group_ids, torch.int32, "group_ids")
    if buffers is None:
        buffers = IwPgBuffers(hidden, W, K, w_layout, logits_cache=logits_cache, max_tokens=max_tokens)
    b = buffers
    if getattr(b, "clip_diag", None) is None:
        b.clip_diag = torch.zeros(C.sizeof(ClipPgDiag), dtype=torch.uint8, device=hidden.device)
    o = clip_pg_default_opts(variant)
    for k, v in overrides.items():
        if not hasattr(o, k):
            raise TypeError(f"unknown option {k}")
        setattr(o, k, v)
    o.w_layout, o.dw_dtype = int(w_layout), _dtype_code(b.dW)
    o.accumulate_dw, o.logits_cache, o.max_tokens = int(bool(accumulate_dw)), int(bool(logits_cache)), int(max_tokens)
    opt = optional_outputs
    _check(load().rapid_clip_pg_loss_fwd_bwd(
        _ptr(hidden), _ptr(W), _ptr(tokens), _ptr(mask), _ptr(logp_old), _ptr(logp_ref), _ptr(rewards), _ptr(group_ids),
        N, T, d, V, K, dt, C.byref(o), _ptr(b.loss), _ptr(b.dhidden), _ptr(b.dW), _ptr(b.logp_cur) if opt else None,
        _ptr(b.adv) if opt else None, _ptr(b.clip_diag) if opt else None, _ptr(b.dev_status), _ptr(b.workspace),
        b.workspace.numel(), _stream()))
    return b


def read_clip_diag(buffers):
    dg = ClipPgDiag.from_buffer_copy(bytes(buffers.clip_diag.cpu().numpy().tobytes()))
    return {f: getattr(dg, f) for f, _ in ClipPgDiag._fields_}
