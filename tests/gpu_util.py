"""Helpers for the GPU parity tests: run the HIP library through its C ABI and the float64 oracle on
the same bits, and compare to the stated bars."""
import numpy as np
import torch

from paper_2605_05940_amd import binding, synth

# Parity bars (bf16 inputs, fp32 accumulation):
REL_PER_SAMPLE = 1e-3     # per-sample KD loss / mean NLL: |gpu - ref| <= 1e-3 * |ref|
GRAD_MAX_ABS = 2e-3       # gradient, max abs error at grad_scale = 1
TOK_ABS, TOK_REL = 1e-4, 1e-4   # sharper per-position diagnostic for the fp32 scalars
CANARY = 24               # guard elements around every output buffer


def dev():
    return torch.device("cuda:0")


class Guarded:
    """An output buffer with NaN / 0x7f canaries on both sides, to catch out-of-bounds writes."""

    def __init__(self, n, dtype):
        self.dtype = dtype
        self.n = n
        self.full = torch.empty(n + 2 * CANARY, dtype=dtype, device=dev())
        self.poison()

    def poison(self):
        if self.dtype.is_floating_point:
            self.full.fill_(float("nan"))
        else:
            self.full.fill_(0x7f if self.dtype == torch.uint8 else 0x7f7f7f7f)

    @property
    def t(self):
        return self.full[CANARY:CANARY + self.n]

    def check(self):
        edge = torch.cat([self.full[:CANARY], self.full[CANARY + self.n:]])
        if self.dtype.is_floating_point:
            assert torch.isnan(edge).all(), "canary overwritten"
        else:
            want = 0x7f if self.dtype == torch.uint8 else 0x7f7f7f7f
            assert (edge == want).all(), "canary overwritten"
        return self.t


def guarded_rows(T, V, stride):
    """A bf16 [T, V] view with row stride `stride` inside a NaN-poisoned buffer (16-byte aligned start)."""
    pad = 64
    full = torch.full((T * stride + 2 * pad,), float("nan"), dtype=torch.bfloat16, device=dev())
    view = full[pad:pad + T * stride].view(T, stride)[:, :V]
    return full, view


def check_row_canaries(full, T, V, stride):
    pad = 64
    assert torch.isnan(full[:pad]).all() and torch.isnan(full[pad + T * stride:]).all(), "canary overwritten"
    if stride > V:
        gaps = full[pad:pad + T * stride].view(T, stride)[:, V:]
        assert torch.isnan(gaps).all(), "row padding overwritten"


def run_gpu_kd(s, mask, *, t=None, idx=None, val=None, labels=None, tau=1.0, grad_scale=1.0, want_grad=True,
               inplace=False, want_tnll=None, ce_grad_scale=0.0, divergence=0, skew_alpha=0.0, no_workspace=False):
    """Call npd_kd_loss_fwd_bwd with guarded outputs.  Returns a dict of host numpy arrays.  `no_workspace`: set
    NPD_FLAG_NO_WORKSPACE (the kernels that keep a whole row in one workgroup instead of the row-gang kernels)."""
    T, V = s.shape
    stride = s.stride(0)
    status = torch.zeros(1, dtype=torch.int32, device=dev())
    has_teacher = t is not None or idx is not None
    kd = Guarded(T, torch.float32) if has_teacher else None
    nll = Guarded(T, torch.float32) if labels is not None else None
    if want_tnll is None:
        want_tnll = labels is not None and t is not None
    tnll = Guarded(T, torch.float32) if want_tnll else None
    lse = Guarded(T, torch.float32)
    gfull = g = None
    if want_grad:
        if inplace:
            g = s
        else:
            gfull, g = guarded_rows(T, V, stride)
    binding.npd_kd_loss_fwd_bwd(s, mask, teacher_dense=t, teacher_idx=idx, teacher_val=val, labels=labels, tau=tau,
                                grad_scale=grad_scale, ce_grad_scale=ce_grad_scale, divergence=divergence,
                                skew_alpha=skew_alpha, grad_out=g, kd_tok=kd.t if kd else None,
                                nll_tok=nll.t if nll else None, teacher_nll_tok=tnll.t if tnll else None,
                                lse_tok=lse.t, dev_status=status, no_workspace=no_workspace)
    torch.cuda.synchronize()
    out = dict(status=int(status.item()))
    for name, buf in (("kd", kd), ("nll_s", nll), ("nll_t", tnll), ("lse_s", lse)):
        out[name] = buf.check().cpu().numpy().astype(np.float64) if buf is not None else None
    if want_grad:
        if gfull is not None:
            check_row_canaries(gfull, T, V, stride)
        out["grad"] = g.float().cpu().numpy().astype(np.float64)
        out["grad_bits"] = synth.bf16_bits(g.contiguous())
    return out


def bf16_ulp(x):
    """Spacing of bf16 numbers at |x| (8 significand bits), with a floor for tiny values."""
    ax = np.maximum(np.abs(x), 2.0 ** -100)
    return 2.0 ** (np.floor(np.log2(ax)) - 7)


def compare_kd(gpu, ref, mask, cu=None, oracle=None, grad_scale=1.0, tau=1.0, amp_from_ref=False, folded=True):
    """Assert the parity bars between a GPU result dict and an oracle result dict.

    The gradient bar of 2e-3 is stated for |grad_scale| / tau <= 1 (elements of magnitude <= 1, where half a bf16
    step is at most 2^-9); it scales with that factor beyond.  `amp_from_ref`: for divergences whose gradient
    elements exceed 1 in magnitude (a log-ratio multiplies the probability) the bar scales with the largest oracle
    element instead, by the same argument.  `folded=False`: the call runs a kernel that always takes the precise form
    of the gradient (weights outside the exponents: the streaming kernels for short or unaligned rows), whose fp32
    value before rounding is held to a bound 25 times tighter."""
    m = mask.astype(bool)
    for key in ("kd", "nll_s", "nll_t", "lse_s"):
        if gpu.get(key) is None or ref.get(key) is None:
            continue
        g, r = gpu[key], ref[key]
        assert (g[~m] == 0).all(), f"{key}: masked positions must be exactly 0"
        err = np.abs(g[m] - r[m])
        assert (err <= TOK_ABS + TOK_REL * np.abs(r[m])).all(), f"{key}: per-position error {err.max():.3g}"
        if cu is not None:
            sg = oracle.segment_reduce(g, mask, cu)
            sr = oracle.segment_reduce(r, mask, cu)
            nz = sr["count"] > 0
            # the relative bar, with a floor of 1e-5 per scored position for samples whose loss is ~0
            excess = np.abs(sg["sum"][nz] - sr["sum"][nz]) - REL_PER_SAMPLE * np.abs(sr["sum"][nz])
            assert (excess <= 1e-5 * sr["count"][nz]).all(), f"{key}: per-sample error beyond 1e-3 relative"
    if gpu.get("grad") is not None and ref.get("grad") is not None:
        g, r = gpu["grad"], ref["grad"]
        assert (g[~m] == 0).all(), "gradient rows of masked positions must be zero"
        err = np.abs(g - r)
        amp = 2.0 ** np.ceil(np.log2(max(1.0, abs(grad_scale) / tau)))   # bf16 steps double per binade
        if amp_from_ref:
            amp = 2.0 ** np.ceil(np.log2(max(1.0, float(np.abs(r).max()))))
        assert err.max() <= GRAD_MAX_ABS * amp, f"gradient max abs error {err.max():.3g}"
        # sharper: within half a bf16 step of the oracle value, plus the fp32 error of the value before rounding.
        # Folded form (weights inside the exponents, row-resident and row-gang kernels): exponent arguments up to 2^10
        # carry an absolute error of 2^-15, i.e. 2.2e-5 relative on each of the two probabilities that are subtracted
        # (both can be ~1 while their difference is ~0): 5e-5 absolute covers it.  Precise form: exponents are taken
        # against the row's reference only (arguments <= 0 where it matters), a few fp32 roundings in all.
        noise = (5e-5 * amp + 3e-5 * np.abs(r)) if folded else (2e-6 * amp + 1e-5 * np.abs(r))
        tol = 0.5 * bf16_ulp(np.abs(r) + noise) + noise
        bad = err > tol
        assert not bad.any(), f"{bad.sum()} gradient elements off by more than half a bf16 step (+fp32 noise)"
