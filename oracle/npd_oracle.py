"""numpy front-end of the float64 C oracle (``npd_oracle.c``).  Test infrastructure only.

Argument marshalling and nothing else: every number comes out of the C file.
bf16 logits are passed as ``uint16`` arrays holding the raw bit patterns.
"""
import ctypes
import os

import numpy as np

from . import build as _build

ZONE_DEGENERATE, ZONE_PROXIMAL, ZONE_DISCONNECT, ZONE_INVALID = 0, 1, 2, 3
DIVERGENCES = {"forward": 0, "reverse": 1, "skew": 2, "skew_reverse": 3}

_lib = None

_i64, _i32, _u32, _f64 = ctypes.c_int64, ctypes.c_int32, ctypes.c_uint32, ctypes.c_double
_p = ctypes.c_void_p


def lib():
    """Load (building first if missing or stale) the oracle library."""
    global _lib
    if _lib is None:
        # NPD_ORACLE_LIB: a differently built oracle (the pin tests run against copies with planted mistakes)
        path = os.environ.get("NPD_ORACLE_LIB") or _build.build(force=False)
        L = ctypes.CDLL(path)
        L.npd_oracle_threads.restype = ctypes.c_int
        L.npd_oracle_kd_dense_f64.restype = None
        L.npd_oracle_kd_dense_f64.argtypes = [_i64, _i64, _p, _p, _p, _p, _f64, _f64, _f64, _p, _p, _p, _p, _p]
        L.npd_oracle_kd_topk_f64.restype = _i64
        L.npd_oracle_kd_topk_f64.argtypes = [_i64, _i64, _i32, _p, _p, _p, _p, _p, _f64, _f64, _f64, _p, _p, _p, _p]
        L.npd_oracle_nll_f64.restype = None
        L.npd_oracle_nll_f64.argtypes = [_i64, _i64, _p, _p, _p, _p, _p]
        L.npd_oracle_kd_dense_bf16.restype = None
        L.npd_oracle_kd_dense_bf16.argtypes = [_i64, _i64, _p, _i64, _p, _i64, _p, _p, _f64, _f64, _f64,
                                               _p, _p, _p, _p, _p]
        L.npd_oracle_div_dense_f64.restype = None
        L.npd_oracle_div_dense_f64.argtypes = [_i64, _i64, _p, _p, _p, _p, _f64, _f64, _f64, _i32, _f64, _p, _p]
        L.npd_oracle_div_dense_bf16.restype = None
        L.npd_oracle_div_dense_bf16.argtypes = [_i64, _i64, _p, _i64, _p, _i64, _p, _p, _f64, _f64, _f64, _i32, _f64,
                                                _p, _p]
        L.npd_oracle_kd_topk_bf16.restype = _i64
        L.npd_oracle_kd_topk_bf16.argtypes = [_i64, _i64, _i32, _p, _i64, _p, _p, _p, _p, _f64, _f64, _f64,
                                              _p, _p, _p, _p]
        L.npd_oracle_nll_bf16.restype = None
        L.npd_oracle_nll_bf16.argtypes = [_i64, _i64, _p, _i64, _p, _p, _p, _p]
        L.npd_oracle_teacher_topk_bf16.restype = None
        L.npd_oracle_teacher_topk_bf16.argtypes = [_i64, _i64, _i32, _p, _i64, _p, ctypes.c_int, _p, _p]
        L.npd_oracle_segment_reduce.restype = ctypes.c_int
        L.npd_oracle_segment_reduce.argtypes = [_i64, _i32, _p, _p, _p, _p, _p, _p, _p]
        L.npd_oracle_policy_lag.restype = ctypes.c_int
        L.npd_oracle_policy_lag.argtypes = [_i64, _i32, _p, _p, _p, _f64, _p, _p, _p, _p]
        L.npd_oracle_perplexity.restype = None
        L.npd_oracle_perplexity.argtypes = [_i32, _p, _p, _p]
        L.npd_oracle_delta_ifd.restype = _i32
        L.npd_oracle_delta_ifd.argtypes = [_i32, _p, _p, _p, _p, _p, _f64, _f64, _u32, _p, _p, _p, _p, _p]
        _lib = L
    return _lib


def threads() -> int:
    return int(lib().npd_oracle_threads())


def _c(a, dtype):
    a = np.ascontiguousarray(a, dtype=dtype)
    return a


def _ptr(a):
    return None if a is None else a.ctypes.data_as(_p)


def _labels_mask(T, labels, mask):
    mask = np.ones(T, np.uint8) if mask is None else _c(mask, np.uint8)
    assert mask.shape == (T,)
    if labels is not None:
        labels = _c(labels, np.int32)
        assert labels.shape == (T,)
    return labels, mask


def kd_dense(s, t, labels=None, mask=None, tau=1.0, grad_scale=1.0, want_grad=True, ce_grad_scale=0.0):
    """Dense-teacher KD.  ``s``, ``t``: [T, V] float64, or uint16 (bf16 bits; may be strided views).

    ``grad`` is grad_scale * d kd / d s  +  ce_grad_scale * d nll_s / d s  (the composite loss of Eq. 1).
    Returns dict(kd, nll_s, nll_t, lse_s, grad) of float64 arrays (None where not computed).
    """
    assert ce_grad_scale == 0.0 or labels is not None
    T, V = s.shape
    assert t.shape == (T, V)
    labels, mask = _labels_mask(T, labels, mask)
    kd = np.empty(T)
    lse = np.empty(T)
    nll_s = np.empty(T) if labels is not None else None
    nll_t = np.empty(T) if labels is not None else None
    grad = np.empty((T, V)) if want_grad else None
    if s.dtype == np.uint16:
        assert t.dtype == np.uint16 and s.strides[1] == 2 and t.strides[1] == 2
        lib().npd_oracle_kd_dense_bf16(T, V, s.ctypes.data, s.strides[0] // 2, t.ctypes.data, t.strides[0] // 2,
                                       _ptr(labels), _ptr(mask), tau, grad_scale, ce_grad_scale,
                                       _ptr(kd), _ptr(nll_s), _ptr(nll_t), _ptr(lse), _ptr(grad))
    else:
        s = _c(s, np.float64)
        t = _c(t, np.float64)
        lib().npd_oracle_kd_dense_f64(T, V, _ptr(s), _ptr(t), _ptr(labels), _ptr(mask), tau, grad_scale, ce_grad_scale,
                                      _ptr(kd), _ptr(nll_s), _ptr(nll_t), _ptr(lse), _ptr(grad))
    return dict(kd=kd, nll_s=nll_s, nll_t=nll_t, lse_s=lse, grad=grad)


def div_dense(s, t, divergence, alpha=0.1, labels=None, mask=None, tau=1.0, grad_scale=1.0, want_grad=True,
              ce_grad_scale=0.0):
    """Dense-teacher distillation under ``divergence`` in {"forward", "reverse", "skew", "skew_reverse"}
    (``alpha``: skew coefficient).  Inputs as for ``kd_dense``; returns dict(kd, grad)."""
    assert ce_grad_scale == 0.0 or labels is not None
    T, V = s.shape
    assert t.shape == (T, V)
    labels, mask = _labels_mask(T, labels, mask)
    kd = np.empty(T)
    grad = np.empty((T, V)) if want_grad else None
    code = DIVERGENCES[divergence]
    if s.dtype == np.uint16:
        assert t.dtype == np.uint16 and s.strides[1] == 2 and t.strides[1] == 2
        lib().npd_oracle_div_dense_bf16(T, V, s.ctypes.data, s.strides[0] // 2, t.ctypes.data, t.strides[0] // 2,
                                        _ptr(labels), _ptr(mask), tau, grad_scale, ce_grad_scale, code, alpha,
                                        _ptr(kd), _ptr(grad))
    else:
        s = _c(s, np.float64)
        t = _c(t, np.float64)
        lib().npd_oracle_div_dense_f64(T, V, _ptr(s), _ptr(t), _ptr(labels), _ptr(mask), tau, grad_scale,
                                       ce_grad_scale, code, alpha, _ptr(kd), _ptr(grad))
    return dict(kd=kd, grad=grad)


def kd_topk(s, idx, val, labels=None, mask=None, tau=1.0, grad_scale=1.0, want_grad=True, ce_grad_scale=0.0):
    """Top-k-teacher KD.  ``s``: [T, V] float64 or uint16 bf16 bits; ``idx`` int32 [T, k]; ``val`` [T, k]."""
    T, V = s.shape
    idx = _c(idx, np.int32)
    k = idx.shape[1]
    assert idx.shape == (T, k) and val.shape == (T, k)
    labels, mask = _labels_mask(T, labels, mask)
    kd = np.empty(T)
    lse = np.empty(T)
    nll_s = np.empty(T) if labels is not None else None
    grad = np.empty((T, V)) if want_grad else None
    if s.dtype == np.uint16:
        assert s.strides[1] == 2
        val = _c(val, np.float32)
        bad = lib().npd_oracle_kd_topk_bf16(T, V, k, s.ctypes.data, s.strides[0] // 2, _ptr(idx), _ptr(val),
                                            _ptr(labels), _ptr(mask), tau, grad_scale, ce_grad_scale,
                                            _ptr(kd), _ptr(nll_s), _ptr(lse), _ptr(grad))
    else:
        s = _c(s, np.float64)
        val = _c(val, np.float64)
        bad = lib().npd_oracle_kd_topk_f64(T, V, k, _ptr(s), _ptr(idx), _ptr(val), _ptr(labels), _ptr(mask),
                                           tau, grad_scale, ce_grad_scale, _ptr(kd), _ptr(nll_s), _ptr(lse), _ptr(grad))
    return dict(kd=kd, nll_s=nll_s, lse_s=lse, grad=grad, bad_index_rows=int(bad))


def nll(o, labels, mask=None):
    """Forward-only per-position CE loss (and log-sum-exp) of logits ``o`` [T, V]."""
    T, V = o.shape
    labels, mask = _labels_mask(T, labels, mask)
    out = np.empty(T)
    lse = np.empty(T)
    if o.dtype == np.uint16:
        assert o.strides[1] == 2
        lib().npd_oracle_nll_bf16(T, V, o.ctypes.data, o.strides[0] // 2, _ptr(labels), _ptr(mask),
                                  _ptr(out), _ptr(lse))
    else:
        o = _c(o, np.float64)
        lib().npd_oracle_nll_f64(T, V, _ptr(o), _ptr(labels), _ptr(mask), _ptr(out), _ptr(lse))
    return dict(nll=out, lse=lse)


def teacher_topk(t_bits, k, mask=None, log_probs=True):
    """Top-k record of teacher logits ``t_bits`` (uint16 bf16 bits [T, V]): ids int32 [T, k] (largest logit first,
    equal logits by increasing id) and float64 values [T, k] (the logits, or their log-softmax over the k)."""
    T, V = t_bits.shape
    assert t_bits.dtype == np.uint16 and t_bits.strides[1] == 2 and 1 <= k <= V
    if mask is not None:
        mask = _c(mask, np.uint8)
        assert mask.shape == (T,)
    idx = np.empty((T, k), np.int32)
    val = np.empty((T, k))
    lib().npd_oracle_teacher_topk_bf16(T, V, k, t_bits.ctypes.data, t_bits.strides[0] // 2, _ptr(mask),
                                       1 if log_probs else 0, _ptr(idx), _ptr(val))
    return dict(idx=idx, val=val)


def segment_reduce(x, mask, cu_seqlens, want_token_to_sample=True):
    """Per-sample sum / count / mean of ``x`` under ``mask`` over ``cu_seqlens`` (int32 [S+1])."""
    x = _c(x, np.float64)
    T = x.shape[0]
    mask = _c(mask, np.uint8)
    cu = _c(cu_seqlens, np.int32)
    S = cu.shape[0] - 1
    seg_sum = np.empty(S)
    seg_count = np.empty(S, np.int32)
    seg_mean = np.empty(S)
    t2s = np.empty(T, np.int32) if want_token_to_sample else None
    rc = lib().npd_oracle_segment_reduce(T, S, _ptr(x), _ptr(mask), _ptr(cu), _ptr(seg_sum), _ptr(seg_count),
                                         _ptr(seg_mean), _ptr(t2s))
    if rc != 0:
        raise ValueError("cu_seqlens is not a non-decreasing sequence inside [0, T]")
    return dict(sum=seg_sum, count=seg_count, mean=seg_mean, token_to_sample=t2s)


def delta_ifd(mean_nll_student, mean_nll_teacher, seg_count, pair_cond, pair_uncond, lo=0.0, hi=1.0, flags=0):
    """IFD (Eq. 3), Delta-IFD (Eq. 4), zone and keep mask (Sec. 3.2) for P sample pairs."""
    ms = _c(mean_nll_student, np.float64)
    mt = _c(mean_nll_teacher, np.float64)
    cnt = _c(seg_count, np.int32)
    pc = _c(pair_cond, np.int32)
    pu = _c(pair_uncond, np.int32)
    P = pc.shape[0]
    S = ms.shape[0]
    assert mt.shape == (S,) and cnt.shape == (S,) and pu.shape == (P,)
    if P and (pc.min() < 0 or pu.min() < 0 or pc.max() >= S or pu.max() >= S):
        raise ValueError("pair index outside [0, S)")
    ifd_s, ifd_t, delta = np.empty(P), np.empty(P), np.empty(P)
    zone, keep = np.empty(P, np.uint8), np.empty(P, np.uint8)
    kept = lib().npd_oracle_delta_ifd(P, _ptr(ms), _ptr(mt), _ptr(cnt), _ptr(pc), _ptr(pu), lo, hi, flags,
                                      _ptr(ifd_s), _ptr(ifd_t), _ptr(delta), _ptr(zone), _ptr(keep))
    return dict(ifd_student=ifd_s, ifd_teacher=ifd_t, delta=delta, zone=zone, keep=keep, keep_count=int(kept))


def policy_lag(kl_tok, mask, cu_seqlens, epsilon=0.10):
    """Policy-latency monitor: per-sample and per-batch mean of a per-position KL(learner || generator) over the scored
    positions, and whether the batch left the near-policy regime (batch mean > epsilon)."""
    x = _c(kl_tok, np.float64)
    T = x.shape[0]
    mask = _c(mask, np.uint8)
    cu = _c(cu_seqlens, np.int32)
    S = cu.shape[0] - 1
    seg_mean = np.empty(S)
    seg_count = np.empty(S, np.int32)
    batch_mean = np.zeros(1)
    batch_count = np.zeros(1, np.int64)
    rc = lib().npd_oracle_policy_lag(T, S, _ptr(x), _ptr(mask), _ptr(cu), float(epsilon), _ptr(seg_mean),
                                     _ptr(seg_count), _ptr(batch_mean), _ptr(batch_count))
    if rc < 0:
        raise ValueError("cu_seqlens is not a non-decreasing sequence inside [0, T]")
    return dict(seg_mean=seg_mean, seg_count=seg_count, batch_mean=float(batch_mean[0]),
                batch_count=int(batch_count[0]), exceeded=int(rc))


def perplexity(mean_nll, seg_count):
    """PPL = exp(mean CE loss) per sample; 0 for samples without a scored position."""
    m = _c(mean_nll, np.float64)
    c = _c(seg_count, np.int32)
    out = np.empty(m.shape[0])
    lib().npd_oracle_perplexity(m.shape[0], _ptr(m), _ptr(c), _ptr(out))
    return out
