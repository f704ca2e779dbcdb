"""Thin ctypes binding over libfog.so: the same calls as include/fog.h, argument marshalling only.

Tensors are torch CUDA tensors used purely as device buffers (`data_ptr()`); every step of the
path runs in the library's HIP kernels.  There is no CPU fallback: if the library has not been
built, `load()` raises.
"""
import ctypes
import os

import torch

E4M3, E5M2 = 0, 1
NT, NN, TN = 0, 1, 2
CAST_BATCH_MAX = 32          # FOG_CAST_BATCH_MAX of the header

_LIB = None
_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libfog.so")

_c = ctypes
_P, _I64, _I, _F, _SZ = _c.c_void_p, _c.c_int64, _c.c_int, _c.c_float, _c.c_size_t

SIGNATURES = {
    "fog_status_string": (_c.c_char_p, [_I]),
    "fog_version": (_I, []),
    "fog_amax": (_I, [_P, _I64, _P, _P]),
    "fog_scale": (_I, [_P, _I, _I, _P, _P, _P]),
    "fog_scale_delayed": (_I, [_P, _I, _P, _I, _I, _P, _P, _P]),
    "fog_quantize": (_I, [_P, _I64, _I64, _I64, _I, _P, _P, _I64, _P, _I64, _P, _P]),
    "fog_quantize_jit": (_I, [_P, _I64, _I64, _I64, _I, _I, _P, _I64, _P, _I64, _P, _P, _P, _P, _SZ, _P]),
    "fog_quantize_jit_workspace": (_SZ, []),
    "fog_quantize_jit_batch": (_I, [_P, _I, _P, _SZ, _P]),
    "fog_quantize_jit_batch_workspace": (_SZ, [_I]),
    "fog_quantize_delayed": (_I, [_P, _I64, _I64, _I64, _I, _I, _P, _I, _I64, _P, _SZ, _P, _I64, _P, _I64, _P, _P, _P, _P]),
    "fog_quantize_delayed_batch": (_I, [_P, _I, _I64, _P]),
    "fog_quantize_delayed_state": (_SZ, []),
    "fog_delayed_amax": (_I, [_P, _I64, _P, _P]),
    "fog_rmsnorm_quantize": (_I, [_P, _I64, _I64, _I64, _F, _I, _P, _P, _I64, _P, _P]),
    "fog_xielu_quantize": (_I, [_P, _I64, _I64, _I64, _F, _F, _I, _P, _P, _I64, _P, _P]),
    "fog_gelu_quantize": (_I, [_P, _I64, _I64, _I64, _I, _P, _P, _I64, _P, _P]),
    "fog_tanh_quantize": (_I, [_P, _I64, _I64, _I64, _F, _I, _P, _P, _I64, _P, _P]),
    "fog_postnorm_residual_quantize": (_I, [_P, _I64, _P, _I64, _I64, _I64, _P, _I, _P, _P, _I64, _P, _I64, _P, _P]),
    "fog_kurtosis": (_I, [_P, _I64, _I64, _I64, _P, _P, _P]),
    "fog_fp8_gemm": (_I, [_I, _I64, _I64, _I64, _P, _I, _I64, _P, _P, _I, _I64, _P, _P, _I64, _P, _SZ, _P]),
    "fog_fp8_gemm_workspace": (_SZ, [_I, _I64, _I64, _I64]),
    "fog_fp8_attn_fwd": (_I, [_I, _I, _I, _I, _I, _F, _I, _P, _P, _P, _P, _P, _P, _P, _P, _P, _P, _P, _SZ, _P]),
    "fog_fp8_attn_bwd": (_I, [_I, _I, _I, _I, _I, _F, _I, _P, _P, _P, _P, _P, _P, _P, _P, _P, _P, _P, _P, _P,
                              _P, _P, _P, _P, _P, _SZ, _P]),
    "fog_fp8_attn_workspace": (_SZ, [_I, _I, _I, _I, _I, _I]),
    "fog_fp8_attn_bwd_static": (_I, [_I, _I, _I, _I, _I, _F, _I, _P, _P, _P, _P, _P, _P, _P, _P, _P, _P, _P, _P, _P,
                                     _P, _P, _P, _P, _P]),
}
ATTN_BWD_STATIC_MAX_ROWS = 524288      # FOG_ATTN_BWD_STATIC_MAX_ROWS of the header


# measurement helpers of the benchmark (include/fog_probe.h): not part of the hot path
PROBE_SIGNATURES = {
    "fog_probe_mfma_rate": (_I, [_P, _I, _P, _SZ, _c.POINTER(_c.c_double), _c.POINTER(_c.c_double), _P]),
    "fog_probe_attention_loop": (_I, [_I, _I, _I, _P, _SZ, _c.POINTER(_c.c_double), _P]),
    "fog_probe_mfma_coissue": (_I, [_I, _I, _I, _I, _P, _SZ, _c.POINTER(_c.c_double), _P]),
    "fog_probe_mfma_cross_wave": (_I, [_I, _I, _I, _I, _P, _SZ, _c.POINTER(_c.c_double), _c.POINTER(_c.c_double), _P]),
    "fog_probe_gemm_products_only": (_I, [_I64, _I64, _I64, _P, _I64, _P, _I64, _P, _P, _P, _I64, _P]),
}


class FogError(RuntimeError):
    def __init__(self, code, where):
        self.code = code
        msg = load().fog_status_string(code).decode()
        super().__init__("%s failed: %s (status %d)" % (where, msg, code))


def load():
    """Loads libfog.so (built by __graft_entry__.build()); raises if it is missing."""
    global _LIB
    if _LIB is None:
        if not os.path.exists(LIB_PATH):
            raise RuntimeError("libfog.so is not built: run `python __graft_entry__.py` (hipcc, gfx950) first; "
                               "there is no fallback path")
        lib = ctypes.CDLL(LIB_PATH)
        for name, (res, args) in list(SIGNATURES.items()) + list(PROBE_SIGNATURES.items()):
            fn = getattr(lib, name)
            fn.restype, fn.argtypes = res, args
        _LIB = lib
    return _LIB


def _ptr(t):
    return None if t is None else t.data_ptr()


def _stream(stream):
    if stream is None:
        stream = torch.cuda.current_stream()
    return stream.cuda_stream


def _check(code, where):
    if code != 0:
        raise FogError(code, where)


def amax(x, out, stream=None):
    _check(load().fog_amax(_ptr(x), x.numel(), _ptr(out), _stream(stream)), "fog_amax")


def scale(amax_t, fmt, scale_out, scale_inv_out, margin=0, stream=None):
    _check(load().fog_scale(_ptr(amax_t), fmt, margin, _ptr(scale_out), _ptr(scale_inv_out), _stream(stream)), "fog_scale")


def scale_delayed(history, new_amax, fmt, scale_out, scale_inv_out, margin=0, stream=None):
    _check(load().fog_scale_delayed(_ptr(history), history.numel(), _ptr(new_amax), fmt, margin, _ptr(scale_out),
                                    _ptr(scale_inv_out), _stream(stream)), "fog_scale_delayed")


def quantize(x, fmt, scale_t, q=None, qT=None, amax_out=None, stream=None):
    rows, cols = x.shape
    _check(load().fog_quantize(_ptr(x), rows, cols, x.stride(0), fmt, _ptr(scale_t),
                               _ptr(q), q.stride(0) if q is not None else 0,
                               _ptr(qT), qT.stride(0) if qT is not None else 0,
                               _ptr(amax_out), _stream(stream)), "fog_quantize")


def quantize_jit(x, fmt, amax_out, scale_out, scale_inv_out, workspace, q=None, qT=None, margin=0, stream=None):
    rows, cols = x.shape
    _check(load().fog_quantize_jit(_ptr(x), rows, cols, x.stride(0), fmt, margin,
                                   _ptr(q), q.stride(0) if q is not None else 0,
                                   _ptr(qT), qT.stride(0) if qT is not None else 0,
                                   _ptr(amax_out), _ptr(scale_out), _ptr(scale_inv_out),
                                   _ptr(workspace), workspace.numel() * workspace.element_size(), _stream(stream)),
           "fog_quantize_jit")


def quantize_jit_workspace():
    return load().fog_quantize_jit_workspace()


class CastJob(ctypes.Structure):
    """Mirror of fog_cast_job."""
    _fields_ = [("x_bf16", _P), ("rows", _I64), ("cols", _I64), ("fmt", _I), ("margin", _I), ("q", _P), ("amax", _P),
                ("scale", _P), ("scale_inv", _P)]


def make_cast_jobs(items, margin=0):
    """items: (x, fmt, q, amax, scale, scale_inv) tuples of contiguous tensors -> ctypes array for quantize_jit_batch."""
    arr = (CastJob * len(items))()
    for job, (x, fmt, q, amax_t, scale_t, sinv_t) in zip(arr, items):
        rows, cols = x.shape
        job.x_bf16, job.rows, job.cols, job.fmt, job.margin = _ptr(x), rows, cols, fmt, margin
        job.q, job.amax, job.scale, job.scale_inv = _ptr(q), _ptr(amax_t), _ptr(scale_t), _ptr(sinv_t)
    return arr


def quantize_jit_batch(jobs, workspace, stream=None):
    """jobs: the array make_cast_jobs returns (it can be built once and reused while the tensors stay in place)."""
    _check(load().fog_quantize_jit_batch(ctypes.cast(jobs, _P), len(jobs), _ptr(workspace),
                                         workspace.numel() * workspace.element_size(), _stream(stream)), "fog_quantize_jit_batch")


def quantize_jit_batch_workspace(count):
    return load().fog_quantize_jit_batch_workspace(count)


def quantize_delayed(x, fmt, history, step, state, scale_out, scale_inv_out=None, q=None, qT=None, amax_prev=None, margin=0,
                     stream=None):
    rows, cols = x.shape
    _check(load().fog_quantize_delayed(_ptr(x), rows, cols, x.stride(0), fmt, margin, _ptr(history), history.numel(), step,
                                       _ptr(state), state.numel() * state.element_size(),
                                       _ptr(q), q.stride(0) if q is not None else 0,
                                       _ptr(qT), qT.stride(0) if qT is not None else 0,
                                       _ptr(amax_prev), _ptr(scale_out), _ptr(scale_inv_out), _stream(stream)),
           "fog_quantize_delayed")


class DelayedJob(ctypes.Structure):
    """Mirror of fog_delayed_job."""
    _fields_ = [("x_bf16", _P), ("rows", _I64), ("cols", _I64), ("fmt", _I), ("margin", _I), ("history", _P), ("history_len", _I),
                ("state", _P), ("state_bytes", _SZ), ("q", _P), ("amax_prev", _P), ("scale", _P), ("scale_inv", _P)]


def make_delayed_jobs(items, margin=0):
    """items: (x, fmt, q, history, state, amax_prev, scale, scale_inv) tuples of contiguous tensors (amax_prev and
    scale_inv may be None) -> ctypes array for quantize_delayed_batch."""
    arr = (DelayedJob * len(items))()
    for job, (x, fmt, q, history, state, amax_prev, scale_t, sinv_t) in zip(arr, items):
        rows, cols = x.shape
        job.x_bf16, job.rows, job.cols, job.fmt, job.margin = _ptr(x), rows, cols, fmt, margin
        job.history, job.history_len = _ptr(history), history.numel()
        job.state, job.state_bytes = _ptr(state), state.numel() * state.element_size()
        job.q, job.amax_prev, job.scale, job.scale_inv = _ptr(q), _ptr(amax_prev), _ptr(scale_t), _ptr(sinv_t)
    return arr


def quantize_delayed_batch(jobs, step, stream=None):
    """jobs: the array make_delayed_jobs returns (built once, reused while the tensors stay in place); step: the call number."""
    _check(load().fog_quantize_delayed_batch(ctypes.cast(jobs, _P), len(jobs), step, _stream(stream)), "fog_quantize_delayed_batch")


def quantize_delayed_state():
    return load().fog_quantize_delayed_state()


def delayed_amax(state, step, amax_out, stream=None):
    _check(load().fog_delayed_amax(_ptr(state), step, _ptr(amax_out), _stream(stream)), "fog_delayed_amax")


def rmsnorm_quantize(x, fmt, scale_t, q, gain=1.0, amax_out=None, stream=None):
    rows, cols = x.shape
    _check(load().fog_rmsnorm_quantize(_ptr(x), rows, cols, x.stride(0), gain, fmt, _ptr(scale_t), _ptr(q),
                                       q.stride(0) if q is not None else 0, _ptr(amax_out), _stream(stream)),
           "fog_rmsnorm_quantize")


def xielu_quantize(x, alpha_p, alpha_n, fmt, scale_t, q, amax_out=None, stream=None):
    rows, cols = x.shape
    _check(load().fog_xielu_quantize(_ptr(x), rows, cols, x.stride(0), alpha_p, alpha_n, fmt, _ptr(scale_t), _ptr(q),
                                     q.stride(0) if q is not None else 0, _ptr(amax_out), _stream(stream)),
           "fog_xielu_quantize")


def gelu_quantize(x, fmt, scale_t, q, amax_out=None, stream=None):
    rows, cols = x.shape
    _check(load().fog_gelu_quantize(_ptr(x), rows, cols, x.stride(0), fmt, _ptr(scale_t), _ptr(q),
                                    q.stride(0) if q is not None else 0, _ptr(amax_out), _stream(stream)), "fog_gelu_quantize")


def tanh_quantize(x, alpha, fmt, scale_t, q, amax_out=None, stream=None):
    rows, cols = x.shape
    _check(load().fog_tanh_quantize(_ptr(x), rows, cols, x.stride(0), alpha, fmt, _ptr(scale_t), _ptr(q),
                                    q.stride(0) if q is not None else 0, _ptr(amax_out), _stream(stream)), "fog_tanh_quantize")


def postnorm_residual_quantize(x, y, gamma, fmt, scale_t, xnew, q=None, amax_out=None, stream=None):
    rows, cols = y.shape
    _check(load().fog_postnorm_residual_quantize(_ptr(x), x.stride(0), _ptr(y), y.stride(0), rows, cols, _ptr(gamma), fmt,
                                                 _ptr(scale_t), _ptr(xnew), xnew.stride(0), _ptr(q),
                                                 q.stride(0) if q is not None else 0, _ptr(amax_out), _stream(stream)),
           "fog_postnorm_residual_quantize")


def kurtosis(x, out, amax_out=None, stream=None):
    rows, cols = x.shape
    _check(load().fog_kurtosis(_ptr(x), rows, cols, x.stride(0), _ptr(out), _ptr(amax_out), _stream(stream)), "fog_kurtosis")


def fp8_gemm(layout, M, N, K, A, fmt_a, sinv_a, B, fmt_b, sinv_b, C, workspace=None, stream=None):
    ws = workspace.numel() * workspace.element_size() if workspace is not None else 0
    _check(load().fog_fp8_gemm(layout, M, N, K, _ptr(A), fmt_a, A.stride(0), _ptr(sinv_a),
                               _ptr(B), fmt_b, B.stride(0), _ptr(sinv_b), _ptr(C), C.stride(0),
                               _ptr(workspace), ws, _stream(stream)), "fog_fp8_gemm")


def fp8_gemm_workspace(layout, M, N, K):
    return load().fog_fp8_gemm_workspace(layout, M, N, K)


def fp8_attn_fwd(B, H, S, D, softmax_scale, causal, Q, K, V, sinv_q, sinv_k, sinv_v, scale_p, O, lse,
                 amax_p=None, workspace=None, stream=None, H_kv=None):
    """H_kv: key/value heads (grouped-query attention); None means H (multi-head)."""
    ws = workspace.numel() * workspace.element_size() if workspace is not None else 0
    _check(load().fog_fp8_attn_fwd(B, H, H if H_kv is None else H_kv, S, D, softmax_scale, int(causal), _ptr(Q), _ptr(K), _ptr(V),
                                   _ptr(sinv_q), _ptr(sinv_k), _ptr(sinv_v), _ptr(scale_p), _ptr(O), _ptr(lse),
                                   _ptr(amax_p), _ptr(workspace), ws, _stream(stream)), "fog_fp8_attn_fwd")


def fp8_attn_bwd(B, H, S, D, softmax_scale, causal, Q, K, V, sinv_q, sinv_k, sinv_v, O, dO, dO8, sinv_do,
                 lse, scale_p, scale_ds, dQ, dK, dV, amax_ds=None, workspace=None, stream=None, H_kv=None):
    ws = workspace.numel() * workspace.element_size() if workspace is not None else 0
    _check(load().fog_fp8_attn_bwd(B, H, H if H_kv is None else H_kv, S, D, softmax_scale, int(causal), _ptr(Q), _ptr(K), _ptr(V),
                                   _ptr(sinv_q), _ptr(sinv_k), _ptr(sinv_v), _ptr(O), _ptr(dO), _ptr(dO8),
                                   _ptr(sinv_do), _ptr(lse), _ptr(scale_p), _ptr(scale_ds),
                                   _ptr(dQ), _ptr(dK), _ptr(dV), _ptr(amax_ds), _ptr(workspace), ws,
                                   _stream(stream)), "fog_fp8_attn_bwd")


def fp8_attn_bwd_static(B, H, S, D, softmax_scale, causal, Q, K, V, sinv_q, sinv_k, sinv_v, O, dO, dO8, sinv_do,
                        lse, scale_p, scale_ds, dQ, dK, dV, amax_ds=None, stream=None, H_kv=None):
    """fp8_attn_bwd without a workspace: the library's own device array serves (B * H * S <= ATTN_BWD_STATIC_MAX_ROWS)."""
    _check(load().fog_fp8_attn_bwd_static(B, H, H if H_kv is None else H_kv, S, D, softmax_scale, int(causal), _ptr(Q), _ptr(K),
                                          _ptr(V), _ptr(sinv_q), _ptr(sinv_k), _ptr(sinv_v), _ptr(O), _ptr(dO), _ptr(dO8),
                                          _ptr(sinv_do), _ptr(lse), _ptr(scale_p), _ptr(scale_ds),
                                          _ptr(dQ), _ptr(dK), _ptr(dV), _ptr(amax_ds), _stream(stream)), "fog_fp8_attn_bwd_static")


def fp8_attn_workspace(B, H, S, D, is_bwd, H_kv=None):
    return load().fog_fp8_attn_workspace(B, H, H if H_kv is None else H_kv, S, D, int(is_bwd))


def probe_mfma_rate(operand_bytes, iters, sink, stream=None):
    """(TFLOP/s, GHz) of a register-resident FP8 matrix-instruction loop on the given 64 KB of operand codes (fog_probe.h)."""
    tf, ghz = _c.c_double(0.0), _c.c_double(0.0)
    _check(load().fog_probe_mfma_rate(_ptr(operand_bytes), iters, _ptr(sink), sink.numel() * sink.element_size(),
                                      _c.byref(tf), _c.byref(ghz), _stream(stream)), "fog_probe_mfma_rate")
    return tf.value, ghz.value


def probe_attention_loop(what, waves_per_simd, iters, sink, stream=None):
    """ns a SIMD spends per wave and key block in the memory-free attention inner loop (fog_probe.h); what: 0 all, 1 matrix
    instructions only, 2 softmax arithmetic only."""
    ns = _c.c_double(0.0)
    _check(load().fog_probe_attention_loop(what, waves_per_simd, iters, _ptr(sink), sink.numel() * sink.element_size(),
                                           _c.byref(ns), _stream(stream)), "fog_probe_attention_loop")
    return ns.value


def probe_mfma_coissue(op, vector_ops, with_mfma, iters, sink, stream=None):
    """Shader cycles per slot (one matrix instruction + vector_ops vector operations, order pinned), one wave per SIMD."""
    cyc = _c.c_double(0.0)
    _check(load().fog_probe_mfma_coissue(op, vector_ops, int(with_mfma), iters, _ptr(sink), sink.numel() * sink.element_size(),
                                         _c.byref(cyc), _stream(stream)), "fog_probe_mfma_coissue")
    return cyc.value


def probe_mfma_cross_wave(op, vector_ops, iters_matrix, iters_vector, sink, stream=None):
    """(cycles per matrix instruction of the matrix waves, cycles per group of vector_ops operations of the vector waves that
    share their SIMDs); a role with zero trips is absent."""
    cm, cv = _c.c_double(0.0), _c.c_double(0.0)
    _check(load().fog_probe_mfma_cross_wave(op, vector_ops, iters_matrix, iters_vector, _ptr(sink), sink.numel() * sink.element_size(),
                                            _c.byref(cm), _c.byref(cv), _stream(stream)), "fog_probe_mfma_cross_wave")
    return cm.value, cv.value


def probe_gemm_products_only(M, N, K, A, sinv_a, B, sinv_b, C, stream=None):
    """fog_fp8_gemm's NT product of E4M3 operands without any tile's epilogue (fog_probe.h); C is not written."""
    _check(load().fog_probe_gemm_products_only(M, N, K, _ptr(A), A.stride(0), _ptr(B), B.stride(0), _ptr(sinv_a), _ptr(sinv_b),
                                               _ptr(C), C.stride(0), _stream(stream)), "fog_probe_gemm_products_only")
