"""ctypes binding of libnpd (C ABI in ``include/npd.h``): argument marshalling only.

Every function takes torch tensors that already live on the GPU, passes their device pointers and
the current HIP stream to the library, and raises ``NpdError`` on a non-zero status.  There is no
fallback: without the built library these calls fail.
"""
import ctypes
import os
from typing import Optional

import torch

HERE = os.path.dirname(os.path.abspath(__file__))
# NPD_LIB_PATH overrides the in-tree library (e.g. to try a differently tuned build)
LIB_PATH = os.environ.get("NPD_LIB_PATH") or os.path.join(HERE, "libnpd.so")

NPD_TEACHER_DENSE_BF16, NPD_TEACHER_TOPK, NPD_TEACHER_NONE = 0, 1, 2
NPD_FLAG_FWD_ONLY, NPD_FLAG_INPLACE_GRAD, NPD_FLAG_NO_WORKSPACE = 1, 2, 4
NPD_DIV_FORWARD_KL, NPD_DIV_REVERSE_KL, NPD_DIV_SKEW_KL, NPD_DIV_SKEW_REVERSE_KL = 0, 1, 2, 3
NPD_DEV_BAD_LABEL, NPD_DEV_BAD_TOPK_INDEX, NPD_DEV_BAD_CU_SEQLENS, NPD_DEV_GANG_TIMEOUT = 1, 2, 4, 8
NPD_ZONE_DEGENERATE, NPD_ZONE_PROXIMAL, NPD_ZONE_DISCONNECT, NPD_ZONE_INVALID = 0, 1, 2, 3
NPD_IFD_REQUIRE_TEACHER_LE_1 = 1
NPD_TOPK_LOG_PROBS = 1
NOALLOC_WORKSPACE_BYTES = 16 << 20   # NPD_NOALLOC_WORKSPACE_BYTES

EXPORTS = ("npd_version", "npd_status_string", "npd_workspace_bytes", "npd_kd_loss_fwd_bwd",
           "npd_segment_reduce", "npd_delta_ifd_score", "npd_teacher_topk", "npd_debug_gang_spin_limit",
           "npd_kd_loss_fwd_bwd_noalloc", "npd_policy_lag", "npd_segment_ppl", "npd_kd_kernel_name")


class NpdError(RuntimeError):
    def __init__(self, status: int, message: str):
        super().__init__(f"libnpd status {status}: {message}")
        self.status = status


class KdDesc(ctypes.Structure):
    """Mirror of ``npd_kd_desc``."""
    _fields_ = [("n_tokens", ctypes.c_int64), ("vocab", ctypes.c_int32), ("teacher_kind", ctypes.c_int32),
                ("student_stride", ctypes.c_int64), ("teacher_stride", ctypes.c_int64),
                ("topk", ctypes.c_int32), ("flags", ctypes.c_uint32),
                ("tau", ctypes.c_float), ("grad_scale", ctypes.c_float), ("ce_grad_scale", ctypes.c_float),
                ("divergence", ctypes.c_int32), ("skew_alpha", ctypes.c_float)]


_lib = None
_vp = ctypes.c_void_p


def load() -> ctypes.CDLL:
    """Load ``libnpd.so`` (built beforehand by ``paper_2605_05940_amd/build.py``); raises if it is missing."""
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise RuntimeError(f"{LIB_PATH} is not built: run `python -m paper_2605_05940_amd.build` "
                               "(or __graft_entry__.build()) first")
        L = ctypes.CDLL(LIB_PATH)
        L.npd_version.restype = ctypes.c_int
        L.npd_status_string.restype = ctypes.c_char_p
        L.npd_status_string.argtypes = [ctypes.c_int]
        L.npd_debug_gang_spin_limit.restype = ctypes.c_int
        L.npd_debug_gang_spin_limit.argtypes = [ctypes.c_int]
        L.npd_kd_kernel_name.restype = ctypes.c_char_p
        L.npd_kd_kernel_name.argtypes = [ctypes.POINTER(KdDesc)]
        L.npd_workspace_bytes.restype = ctypes.c_size_t
        L.npd_workspace_bytes.argtypes = [ctypes.POINTER(KdDesc)]
        L.npd_kd_loss_fwd_bwd.restype = ctypes.c_int
        L.npd_kd_loss_fwd_bwd.argtypes = [ctypes.POINTER(KdDesc)] + [_vp] * 13 + [ctypes.c_size_t, _vp]
        L.npd_kd_loss_fwd_bwd_noalloc.restype = ctypes.c_int
        L.npd_kd_loss_fwd_bwd_noalloc.argtypes = [ctypes.POINTER(KdDesc)] + [_vp] * 13
        L.npd_segment_reduce.restype = ctypes.c_int
        L.npd_segment_reduce.argtypes = [ctypes.c_int64, ctypes.c_int32] + [_vp] * 9
        L.npd_delta_ifd_score.restype = ctypes.c_int
        L.npd_delta_ifd_score.argtypes = ([ctypes.c_int32, ctypes.c_int32] + [_vp] * 5 +
                                          [ctypes.c_float, ctypes.c_float, ctypes.c_uint32] + [_vp] * 7)
        L.npd_policy_lag.restype = ctypes.c_int
        L.npd_policy_lag.argtypes = [ctypes.c_int64, ctypes.c_int32] + [_vp] * 3 + [ctypes.c_float] + [_vp] * 7
        L.npd_segment_ppl.restype = ctypes.c_int
        L.npd_segment_ppl.argtypes = [ctypes.c_int32] + [_vp] * 4
        L.npd_teacher_topk.restype = ctypes.c_int
        L.npd_teacher_topk.argtypes = ([ctypes.c_int64, ctypes.c_int32, ctypes.c_int64, ctypes.c_int32,
                                        ctypes.c_uint32] + [_vp] * 5)
        _lib = L
    return _lib


def _check(status: int) -> None:
    if status != 0:
        raise NpdError(status, load().npd_status_string(status).decode())


def _ptr(t: Optional[torch.Tensor], dtype=None):
    if t is None:
        return None
    if not t.is_cuda:
        raise ValueError("libnpd takes device tensors")
    if dtype is not None and t.dtype != dtype:
        raise ValueError(f"expected {dtype}, got {t.dtype}")
    return t.data_ptr()


def _stream():
    return torch.cuda.current_stream().cuda_stream


def version() -> int:
    return int(load().npd_version())


def _row_stride(x: torch.Tensor) -> int:
    if x.dim() != 2 or x.stride(1) != 1:
        raise ValueError("logits must be 2-D with unit stride along the vocabulary")
    return x.stride(0)


def npd_kd_loss_fwd_bwd(student_logits: torch.Tensor, loss_mask: torch.Tensor, *,
                        teacher_dense: Optional[torch.Tensor] = None,
                        teacher_idx: Optional[torch.Tensor] = None, teacher_val: Optional[torch.Tensor] = None,
                        labels: Optional[torch.Tensor] = None, tau: float = 1.0, grad_scale: float = 1.0,
                        ce_grad_scale: float = 0.0, divergence: int = NPD_DIV_FORWARD_KL, skew_alpha: float = 0.0,
                        grad_out: Optional[torch.Tensor] = None, kd_tok: Optional[torch.Tensor] = None,
                        nll_tok: Optional[torch.Tensor] = None, teacher_nll_tok: Optional[torch.Tensor] = None,
                        lse_tok: Optional[torch.Tensor] = None, dev_status: Optional[torch.Tensor] = None,
                        workspace: Optional[torch.Tensor] = None, no_workspace: bool = False,
                        noalloc: bool = False) -> None:
    """Enqueue the fused KD loss / gradient on the current stream (see ``npd_kd_loss_fwd_bwd`` in npd.h).

    The teacher kind follows from which teacher tensors are given; ``grad_out is None`` means forward
    only; ``grad_out`` sharing storage with ``student_logits`` means the in-place gradient.  ``workspace``:
    a uint8 tensor of at least ``npd_workspace_bytes`` bytes; if it is None one is taken from
    ``workspace_for`` (a per-device tensor that this module keeps and grows).  ``no_workspace`` sets
    ``NPD_FLAG_NO_WORKSPACE``.  ``noalloc`` calls ``npd_kd_loss_fwd_bwd_noalloc`` instead (the library's built-in
    scratch array; no workspace argument).
    """
    T, V = student_logits.shape
    d = KdDesc()
    d.n_tokens, d.vocab = T, V
    d.student_stride = _row_stride(student_logits)
    d.tau, d.grad_scale, d.ce_grad_scale = tau, grad_scale, ce_grad_scale
    d.divergence, d.skew_alpha = divergence, skew_alpha
    if teacher_dense is not None:
        d.teacher_kind, d.teacher_stride = NPD_TEACHER_DENSE_BF16, _row_stride(teacher_dense)
        if teacher_dense.shape != (T, V):
            raise ValueError("teacher_dense must be [T, V]")
    elif teacher_idx is not None:
        d.teacher_kind, d.topk = NPD_TEACHER_TOPK, teacher_idx.shape[1]
        if not (teacher_idx.is_contiguous() and teacher_val.is_contiguous() and teacher_val.shape == teacher_idx.shape
                and teacher_idx.shape[0] == T):
            raise ValueError("teacher_idx / teacher_val must be contiguous [T, k]")
    else:
        d.teacher_kind = NPD_TEACHER_NONE
    flags = 0
    if grad_out is None:
        flags |= NPD_FLAG_FWD_ONLY
    else:
        if grad_out.shape != (T, V) or _row_stride(grad_out) != d.student_stride:
            raise ValueError("grad_out must have the shape and row stride of student_logits")
        if grad_out.data_ptr() == student_logits.data_ptr():
            flags |= NPD_FLAG_INPLACE_GRAD
    if no_workspace:
        flags |= NPD_FLAG_NO_WORKSPACE
    d.flags = flags
    if workspace is None and not no_workspace and not noalloc:
        workspace = workspace_for(int(load().npd_workspace_bytes(ctypes.byref(d))), student_logits.device)
    for name, t, n in (("loss_mask", loss_mask, T), ("labels", labels, T), ("kd_tok", kd_tok, T),
                       ("nll_tok", nll_tok, T), ("teacher_nll_tok", teacher_nll_tok, T), ("lse_tok", lse_tok, T)):
        if t is not None and (t.numel() != n or not t.is_contiguous()):
            raise ValueError(f"{name} must be contiguous with {n} elements")
    if noalloc:
        if workspace is not None:
            raise ValueError("the no-allocation entry point takes no workspace")
        _check(load().npd_kd_loss_fwd_bwd_noalloc(
            ctypes.byref(d), _ptr(student_logits, torch.bfloat16), _ptr(teacher_dense, torch.bfloat16),
            _ptr(teacher_idx, torch.int32), _ptr(teacher_val, torch.float32), _ptr(labels, torch.int32),
            _ptr(loss_mask, torch.uint8), _ptr(grad_out, torch.bfloat16), _ptr(kd_tok, torch.float32),
            _ptr(nll_tok, torch.float32), _ptr(teacher_nll_tok, torch.float32), _ptr(lse_tok, torch.float32),
            _ptr(dev_status, torch.int32), _stream()))
        return
    ws_bytes = 0 if workspace is None else workspace.numel() * workspace.element_size()
    _check(load().npd_kd_loss_fwd_bwd(
        ctypes.byref(d), _ptr(student_logits, torch.bfloat16), _ptr(teacher_dense, torch.bfloat16),
        _ptr(teacher_idx, torch.int32), _ptr(teacher_val, torch.float32), _ptr(labels, torch.int32),
        _ptr(loss_mask, torch.uint8), _ptr(grad_out, torch.bfloat16), _ptr(kd_tok, torch.float32),
        _ptr(nll_tok, torch.float32), _ptr(teacher_nll_tok, torch.float32), _ptr(lse_tok, torch.float32),
        _ptr(dev_status, torch.int32), _ptr(workspace), ws_bytes, _stream()))


_workspaces = {}


def workspace_for(n_bytes: int, device) -> Optional[torch.Tensor]:
    """A device buffer of at least ``n_bytes`` bytes (None for 0), kept per device and grown on demand, for callers
    that do not manage the workspace of ``npd_kd_loss_fwd_bwd`` themselves.  Calls that share it must be ordered on
    one stream."""
    if n_bytes == 0:
        return None
    key = torch.device(device).index or 0
    ws = _workspaces.get(key)
    if ws is None or ws.numel() < n_bytes:
        ws = torch.empty(n_bytes, dtype=torch.uint8, device=device)
        _workspaces[key] = ws
    return ws


def npd_workspace_bytes(n_tokens: int, vocab: int, teacher_kind: int = NPD_TEACHER_DENSE_BF16, topk: int = 0,
                        flags: int = 0, tau: float = 1.0) -> int:
    d = KdDesc()
    d.n_tokens, d.vocab, d.teacher_kind, d.topk, d.flags = n_tokens, vocab, teacher_kind, topk, flags
    d.student_stride = d.teacher_stride = vocab
    d.tau, d.grad_scale, d.ce_grad_scale = tau, 1.0, 0.0
    return int(load().npd_workspace_bytes(ctypes.byref(d)))


def npd_segment_reduce(values: Optional[torch.Tensor], loss_mask: torch.Tensor, cu_seqlens: torch.Tensor, *,
                       seg_sum: Optional[torch.Tensor] = None, seg_count: Optional[torch.Tensor] = None,
                       seg_mean: Optional[torch.Tensor] = None, token_to_sample: Optional[torch.Tensor] = None,
                       dev_status: Optional[torch.Tensor] = None) -> None:
    """Enqueue the per-sample reduction on the current stream (see ``npd_segment_reduce`` in npd.h)."""
    T = loss_mask.numel()
    S = cu_seqlens.numel() - 1
    for name, t, n in (("values", values, T), ("seg_sum", seg_sum, S), ("seg_count", seg_count, S),
                       ("seg_mean", seg_mean, S), ("token_to_sample", token_to_sample, T)):
        if t is not None and (t.numel() != n or not t.is_contiguous()):
            raise ValueError(f"{name} must be contiguous with {n} elements")
    _check(load().npd_segment_reduce(
        T, S, _ptr(values, torch.float32), _ptr(loss_mask, torch.uint8), _ptr(cu_seqlens, torch.int32),
        _ptr(seg_sum, torch.float32), _ptr(seg_count, torch.int32), _ptr(seg_mean, torch.float32),
        _ptr(token_to_sample, torch.int32), _ptr(dev_status, torch.int32), _stream()))


def npd_delta_ifd_score(mean_nll_student: torch.Tensor, mean_nll_teacher: torch.Tensor, seg_count: torch.Tensor,
                        pair_cond: torch.Tensor, pair_uncond: torch.Tensor, lo: float, hi: float, *, flags: int = 0,
                        ifd_student: Optional[torch.Tensor] = None, ifd_teacher: Optional[torch.Tensor] = None,
                        delta: Optional[torch.Tensor] = None, zone: Optional[torch.Tensor] = None,
                        keep: Optional[torch.Tensor] = None, keep_count: Optional[torch.Tensor] = None) -> None:
    """Enqueue the Delta-IFD score on the current stream (see ``npd_delta_ifd_score`` in npd.h)."""
    S = mean_nll_student.numel()
    P = pair_cond.numel()
    if mean_nll_teacher.numel() != S or seg_count.numel() != S or pair_uncond.numel() != P:
        raise ValueError("inconsistent sizes")
    for name, t in (("ifd_student", ifd_student), ("ifd_teacher", ifd_teacher), ("delta", delta), ("zone", zone),
                    ("keep", keep)):
        if t is not None and (t.numel() != P or not t.is_contiguous()):
            raise ValueError(f"{name} must be contiguous with {P} elements")
    _check(load().npd_delta_ifd_score(
        P, S, _ptr(mean_nll_student, torch.float32), _ptr(mean_nll_teacher, torch.float32),
        _ptr(seg_count, torch.int32), _ptr(pair_cond, torch.int32), _ptr(pair_uncond, torch.int32),
        lo, hi, flags, _ptr(ifd_student, torch.float32), _ptr(ifd_teacher, torch.float32),
        _ptr(delta, torch.float32), _ptr(zone, torch.uint8), _ptr(keep, torch.uint8),
        _ptr(keep_count, torch.int32), _stream()))


def npd_teacher_topk(teacher_logits: torch.Tensor, k: int, *, topk_idx: torch.Tensor, topk_val: torch.Tensor,
                     loss_mask: Optional[torch.Tensor] = None, log_probs: bool = True) -> None:
    """Enqueue the teacher-side top-k extraction on the current stream (see ``npd_teacher_topk`` in npd.h)."""
    T, V = teacher_logits.shape
    for name, t in (("topk_idx", topk_idx), ("topk_val", topk_val)):
        if t.shape != (T, k) or not t.is_contiguous():
            raise ValueError(f"{name} must be contiguous [T, k]")
    if loss_mask is not None and (loss_mask.numel() != T or not loss_mask.is_contiguous()):
        raise ValueError("loss_mask must be contiguous with T elements")
    _check(load().npd_teacher_topk(T, V, _row_stride(teacher_logits), k, NPD_TOPK_LOG_PROBS if log_probs else 0,
                                   _ptr(teacher_logits, torch.bfloat16), _ptr(loss_mask, torch.uint8),
                                   _ptr(topk_idx, torch.int32), _ptr(topk_val, torch.float32), _stream()))


def npd_policy_lag(kl_tok: torch.Tensor, loss_mask: torch.Tensor, cu_seqlens: torch.Tensor, epsilon: float = 0.10, *,
                   seg_kl_mean: Optional[torch.Tensor] = None, seg_count: Optional[torch.Tensor] = None,
                   batch_kl_mean: Optional[torch.Tensor] = None, batch_count: Optional[torch.Tensor] = None,
                   lag_exceeded: Optional[torch.Tensor] = None, dev_status: Optional[torch.Tensor] = None) -> None:
    """Enqueue the policy-latency monitor on the current stream (see ``npd_policy_lag`` in npd.h)."""
    T = loss_mask.numel()
    S = cu_seqlens.numel() - 1
    for name, t, n in (("kl_tok", kl_tok, T), ("seg_kl_mean", seg_kl_mean, S), ("seg_count", seg_count, S),
                       ("batch_kl_mean", batch_kl_mean, 1), ("batch_count", batch_count, 1),
                       ("lag_exceeded", lag_exceeded, 1)):
        if t is not None and (t.numel() != n or not t.is_contiguous()):
            raise ValueError(f"{name} must be contiguous with {n} elements")
    _check(load().npd_policy_lag(
        T, S, _ptr(kl_tok, torch.float32), _ptr(loss_mask, torch.uint8), _ptr(cu_seqlens, torch.int32), epsilon,
        _ptr(seg_kl_mean, torch.float32), _ptr(seg_count, torch.int32), _ptr(batch_kl_mean, torch.float32),
        _ptr(batch_count, torch.int32), _ptr(lag_exceeded, torch.int32), _ptr(dev_status, torch.int32), _stream()))


def npd_segment_ppl(seg_mean_nll: torch.Tensor, seg_count: torch.Tensor, seg_ppl: torch.Tensor) -> None:
    """Enqueue PPL = exp(mean NLL) per sample on the current stream (see ``npd_segment_ppl`` in npd.h)."""
    S = seg_mean_nll.numel()
    if seg_count.numel() != S or seg_ppl.numel() != S:
        raise ValueError("inconsistent sizes")
    _check(load().npd_segment_ppl(S, _ptr(seg_mean_nll, torch.float32), _ptr(seg_count, torch.int32),
                                  _ptr(seg_ppl, torch.float32), _stream()))
