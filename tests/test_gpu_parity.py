"""GPU parity: the HIP library, called through its C ABI, against the float64 oracle on the same bits.

Bars (bf16 inputs, fp32 accumulation): per-sample KD loss and mean NLL within 1e-3 relative, gradient max abs
error <= 2e-3 at grad_scale = 1, all integer / index / zone bookkeeping bit-exact.
"""
import os

import numpy as np
import pytest
import torch

from paper_2605_05940_amd import binding, synth

from gpu_util import (Guarded, REL_PER_SAMPLE, compare_kd, dev, guarded_rows, run_gpu_kd)

pytestmark = pytest.mark.gpu
HERE = os.path.dirname(os.path.abspath(__file__))


def _say(msg):
    print(f"[gpu-parity] {msg}", flush=True)


def _inputs(w, stride=None, seed=synth.SEED, dense_teacher=True):
    """Layout + bf16 logits of workload `w` on the GPU (row stride `stride` elements, default V)."""
    lay = synth.make_layout(w, seed)
    T, V = w.n_tokens, w.vocab
    stride = stride or V
    s = torch.zeros((T, stride), dtype=torch.bfloat16, device=dev())[:, :V]
    t = torch.zeros((T, stride), dtype=torch.bfloat16, device=dev())[:, :V] if dense_teacher else None
    synth.fill_logits(w, s, t, seed)
    mask = torch.from_numpy(lay.loss_mask).to(dev())
    labels = torch.from_numpy(lay.labels).to(dev())
    return lay, s, t, mask, labels


def _bits(x):
    return synth.bf16_bits(x)


# --------------------------------------------------------------------------- dense teacher

def test_cfg0_tiny_dense_full(oracle):
    w = synth.config(0)
    _say(f"{w.name} T={w.n_tokens} V={w.vocab}")
    lay, s, t, mask, labels = _inputs(w)
    gpu = run_gpu_kd(s, mask, t=t, labels=labels, tau=w.tau)
    ref = oracle.kd_dense(_bits(s), _bits(t), lay.labels, lay.loss_mask, tau=w.tau)
    assert gpu["status"] == 0
    compare_kd(gpu, ref, lay.loss_mask, lay.cu_seqlens, oracle, folded=False)
    # rows of the bf16 gradient sum to ~0 (each element carries up to half a bf16 step)
    assert np.abs(gpu["grad"].sum(1)).max() < 1e-2


@pytest.mark.parametrize("V,stride,tau,scale", [
    (151936, 151936, 1.0, 1.0),      # the 1B-student vocabulary: 1024-thread path, 18.5 groups per thread
    (4099, 4104, 2.0, 1.0),          # 256-thread path, ragged 3-element tail, padded rows
    (4099, 4099, 1.0, -0.5),         # rows not 16-byte aligned: element-wise path; negative scale
    (1000, 1000, 0.5, 3.0),          # 64-thread path
    (7, 7, 1.0, 1.0),                # shorter than one 128-bit group
    (1, 8, 1.0, 1.0),                # single-token vocabulary: KL = 0, grad = 0
    (262144, 262144, 1.0, 1.0),      # largest vocabulary
    (128256, 128256, 1.0, 1.0),      # 16 groups per thread, the last one ragged
    (131072, 131072, 2.0, 1.0),      # exactly 16 full groups per thread
    (102400, 102400, 1.0, 1.0),      # 13 groups per thread
    (124000, 124000, 1.0, 1.0),      # 16 > 15.1 groups: the 13-group variant streams the rest twice
    (81920, 81920, 1.0, 1.0),        # 10 groups per thread of 1024: row-resident with empty trailing groups
    (65536, 65544, 1.0, 1.0),        # 512-thread workgroups, 16 full groups, padded stride
    (50264, 50264, 2.0, 0.5),        # 512 threads, 12.3 groups: ragged last group, tau != 1
    (40000, 40000, 1.0, 1.0),        # 512 threads, 10 groups
    (32000, 32000, 1.0, 1.0),        # 256-thread workgroups, 15.6 groups
    (20488, 20488, 1.0, -1.0),       # 256 threads, 10.004 groups: one vector in the last group
    (8192, 8192, 1.0, 1.0),          # 256 threads, 4 groups: the shortest row-resident shape
    (8184, 8184, 1.0, 1.0),          # just below: streaming kernel
])
@pytest.mark.parametrize("no_workspace", [False, True])
def test_dense_shapes(oracle, V, stride, tau, scale, no_workspace):
    if no_workspace and binding.npd_workspace_bytes(8, V, tau=tau) == 0:
        pytest.skip("this shape needs no workspace: one kernel either way")
    n_rows, row_len = (2, 96) if V > 100000 else (2, 160)
    w = synth.scaled(synth.config(1), n_rows=n_rows, row_len=row_len, vocab=V, length_lo=8, length_hi=64)
    _say(f"dense V={V} stride={stride} tau={tau} scale={scale} T={w.n_tokens} no_workspace={no_workspace}")
    lay, s, t, mask, labels = _inputs(w, stride)
    gpu = run_gpu_kd(s, mask, t=t, labels=labels, tau=tau, grad_scale=scale, no_workspace=no_workspace)
    ref = oracle.kd_dense(_bits(s.contiguous()), _bits(t.contiguous()), lay.labels, lay.loss_mask, tau=tau,
                          grad_scale=scale)
    assert gpu["status"] == 0
    # rows shorter than 8,192 entries or not 16-byte aligned run the streaming kernel: always the precise gradient form
    compare_kd(gpu, ref, lay.loss_mask, lay.cu_seqlens, oracle, grad_scale=scale, tau=tau,
               folded=V >= 8192 and stride % 8 == 0)


def test_dense_forward_only_and_tau_not_one_nll(oracle):
    w = synth.scaled(synth.config(1), n_rows=1, row_len=128, vocab=33000, length_lo=8, length_hi=64)
    lay, s, t, mask, labels = _inputs(w)
    _say("dense forward only, tau=2 with tau=1 NLLs")
    gpu = run_gpu_kd(s, mask, t=t, labels=labels, tau=2.0, want_grad=False)
    ref = oracle.kd_dense(_bits(s), _bits(t), lay.labels, lay.loss_mask, tau=2.0, want_grad=False)
    compare_kd(gpu, ref, lay.loss_mask, lay.cu_seqlens, oracle)
    # forward-only and forward+backward give the same scalars up to the order of summation (the two runs may
    # partition a row differently: other workgroup sizes)
    both = run_gpu_kd(s, mask, t=t, labels=labels, tau=2.0)
    for key in ("kd", "nll_s", "nll_t", "lse_s"):
        np.testing.assert_allclose(gpu[key], both[key], rtol=1e-5, atol=1e-6)


def test_student_equals_teacher_gives_exact_zero(oracle):
    w = synth.scaled(synth.config(1), n_rows=1, row_len=64, vocab=151936, length_lo=8, length_hi=32)
    lay, s, _, mask, labels = _inputs(w, dense_teacher=False)
    t = s.clone()
    _say("student == teacher")
    for tau in (1.0, 2.0):
        gpu = run_gpu_kd(s, mask, t=t, labels=labels, tau=tau)
        assert (gpu["kd"] == 0.0).all()
        assert (gpu["grad_bits"] & 0x7fff == 0).all()       # +0 or -0 everywhere
        np.testing.assert_array_equal(gpu["nll_s"], gpu["nll_t"])


def test_inplace_matches_out_of_place_bitwise(oracle):
    w = synth.scaled(synth.config(4), n_rows=1, row_len=192, vocab=262144, length_lo=16, length_hi=64)
    _say(f"{w.name} reduced: in-place gradient, heavy tails, V={w.vocab}")
    lay, s, t, mask, labels = _inputs(w)
    ref = oracle.kd_dense(_bits(s), _bits(t), lay.labels, lay.loss_mask, tau=1.0)
    out = run_gpu_kd(s, mask, t=t, labels=labels)
    compare_kd(out, ref, lay.loss_mask, lay.cu_seqlens, oracle)
    s2 = s.clone()
    inp = run_gpu_kd(s2, mask, t=t, labels=labels, inplace=True)
    np.testing.assert_array_equal(inp["grad_bits"], out["grad_bits"])
    for key in ("kd", "nll_s", "nll_t", "lse_s"):
        np.testing.assert_array_equal(inp[key], out[key])
    assert np.abs(_bits(s).astype(np.int32)).max() > 0 and np.isfinite(out["kd"]).all()
    # heavy tails really are heavy here: some logit beyond +-100
    assert np.abs(s.float().cpu().numpy()).max() > 100


def test_all_masked_and_single_row(oracle):
    V = 4104
    s = torch.randn((5, V), device=dev()).to(torch.bfloat16)
    t = torch.randn((5, V), device=dev()).to(torch.bfloat16)
    labels = torch.zeros(5, dtype=torch.int32, device=dev())
    mask = torch.zeros(5, dtype=torch.uint8, device=dev())
    gpu = run_gpu_kd(s, mask, t=t, labels=labels)
    assert (gpu["kd"] == 0).all() and (gpu["nll_s"] == 0).all() and (gpu["grad_bits"] == 0).all()
    one = run_gpu_kd(s[:1], torch.ones(1, dtype=torch.uint8, device=dev()), t=t[:1], labels=labels[:1])
    ref = oracle.kd_dense(_bits(s[:1]), _bits(t[:1]), np.zeros(1, np.int32), np.ones(1, np.uint8))
    compare_kd(one, ref, np.ones(1, np.uint8))


def test_zero_scale_and_determinism(oracle):
    w = synth.scaled(synth.config(1), n_rows=1, row_len=64, vocab=40000, length_lo=8, length_hi=32)
    lay, s, t, mask, labels = _inputs(w)
    z = run_gpu_kd(s, mask, t=t, labels=labels, grad_scale=0.0)
    assert (z["grad_bits"] & 0x7fff == 0).all()
    a = run_gpu_kd(s, mask, t=t, labels=labels, tau=2.0)
    b = run_gpu_kd(s, mask, t=t, labels=labels, tau=2.0)
    np.testing.assert_array_equal(a["grad_bits"], b["grad_bits"])
    for key in ("kd", "nll_s", "nll_t", "lse_s"):
        np.testing.assert_array_equal(a[key], b[key])


def test_bad_label_sets_status_and_nan(oracle):
    V = 520
    s = torch.randn((4, V), device=dev()).to(torch.bfloat16)
    t = torch.randn((4, V), device=dev()).to(torch.bfloat16)
    labels = torch.tensor([3, V, -1, 5], dtype=torch.int32, device=dev())
    mask = torch.tensor([1, 1, 0, 1], dtype=torch.uint8, device=dev())
    gpu = run_gpu_kd(s, mask, t=t, labels=labels)
    assert gpu["status"] == binding.NPD_DEV_BAD_LABEL
    assert np.isnan(gpu["nll_s"][1]) and np.isnan(gpu["nll_t"][1]) and np.isfinite(gpu["nll_s"][[0, 3]]).all()
    assert gpu["nll_s"][2] == 0 and np.isfinite(gpu["kd"]).all()     # masked bad label is ignored


# --------------------------------------------------------------------------- top-k teacher

@pytest.mark.parametrize("V,k,tau,scale,inplace", [
    (151936, 64, 2.0, 1.0, False),   # config 2's shape
    (151936, 10, 1.0, 1.0, True),    # the paper's default k, in place
    (128256, 64, 2.0, 1.0, False),   # 16 groups per thread
    (5003, 200, 2.0, -2.0, False),   # k larger than a wave, unaligned rows
    (300, 300, 1.0, 1.0, False),     # k = V
    (40000, 1, 1.0, 1.0, False),     # k = 1; 512-thread row-resident shape
    (32000, 64, 2.0, 1.0, True),     # 256-thread workgroups, in place, tau != 1
    (65536, 16, 1.0, 1.0, False),    # 512 threads, 16 groups
    (90000, 64, 1.0, 1.0, False),    # 512 threads, 22 groups: the last ones streamed twice
    (151936, 4096, 1.0, 1.0, False), # the largest supported k
    (20000, 4096, 2.0, 1.0, True),   # the largest k on a 256-thread shape, in place
])
def test_topk_shapes(oracle, V, k, tau, scale, inplace):
    n_rows, row_len = (2, 96) if V > 100000 else (2, 128)
    w = synth.scaled(synth.config(2), n_rows=n_rows, row_len=row_len, vocab=V, length_lo=8, length_hi=64, topk=k)
    _say(f"top-k V={V} k={k} tau={tau} scale={scale} inplace={inplace}")
    lay, s, _, mask, labels = _inputs(w, dense_teacher=False)
    idx, val = synth.make_topk_teacher(w, s)
    ref = oracle.kd_topk(_bits(s), idx.cpu().numpy(), val.cpu().numpy(), lay.labels, lay.loss_mask, tau=tau,
                         grad_scale=scale)
    assert ref["bad_index_rows"] == 0
    for no_workspace in (False, True):     # row-gang kernel where it applies | one workgroup per row
        gpu = run_gpu_kd(s.clone() if inplace else s, mask, idx=idx, val=val, labels=labels, tau=tau, grad_scale=scale,
                         inplace=inplace, no_workspace=no_workspace)
        assert gpu["status"] == 0
        compare_kd(gpu, ref, lay.loss_mask, lay.cu_seqlens, oracle, grad_scale=scale, tau=tau)


def test_topk_uniform_closed_form_on_gpu():
    # uniform student, k equal teacher entries: KL = ln(V / k)
    V, k = 151936, 64
    s = torch.zeros((2, V), dtype=torch.bfloat16, device=dev())
    idx = (torch.arange(k, device=dev(), dtype=torch.int32) * 997 + 5).repeat(2, 1).contiguous()
    val = torch.full((2, k), -3.0, device=dev())
    gpu = run_gpu_kd(s, torch.ones(2, dtype=torch.uint8, device=dev()), idx=idx, val=val, want_grad=False)
    np.testing.assert_allclose(gpu["kd"], np.log(V / k), rtol=1e-5)


@pytest.mark.parametrize("V", [1000, 151936])
def test_topk_bad_index_is_flagged(V):
    k = 8
    s = torch.randn((3, V), device=dev()).to(torch.bfloat16)
    idx = torch.arange(k, dtype=torch.int32, device=dev()).repeat(3, 1).contiguous()
    idx[1, 3] = V
    val = torch.zeros((3, k), device=dev())
    gpu = run_gpu_kd(s, torch.ones(3, dtype=torch.uint8, device=dev()), idx=idx, val=val)
    assert gpu["status"] == binding.NPD_DEV_BAD_TOPK_INDEX
    assert np.isnan(gpu["kd"][1]) and np.isfinite(gpu["kd"][[0, 2]]).all()
    assert np.isnan(gpu["grad"][1]).all() and np.isfinite(gpu["grad"][[0, 2]]).all()


# --------------------------------------------------------------------------- scoring pass, segment reduce, Delta-IFD

def _segment_gpu(values, mask, cu, want_t2s=True):
    T, S = mask.numel(), cu.numel() - 1
    ssum, scnt, smean = Guarded(S, torch.float32), Guarded(S, torch.int32), Guarded(S, torch.float32)
    t2s = Guarded(T, torch.int32) if want_t2s else None
    status = torch.zeros(1, dtype=torch.int32, device=dev())
    binding.npd_segment_reduce(values, mask, cu, seg_sum=ssum.t, seg_count=scnt.t, seg_mean=smean.t,
                               token_to_sample=t2s.t if t2s else None, dev_status=status)
    torch.cuda.synchronize()
    return dict(sum=ssum.check().cpu().numpy().astype(np.float64), count=scnt.check().cpu().numpy(),
                mean=smean.check().cpu().numpy().astype(np.float64),
                token_to_sample=t2s.check().cpu().numpy() if t2s else None, status=int(status.item()),
                mean_dev=smean.t, count_dev=scnt.t)


def _ifd_gpu(ms, mt, cnt, pc, pu, lo, hi, flags=0):
    P = pc.numel()
    outs = dict(ifd_student=Guarded(P, torch.float32), ifd_teacher=Guarded(P, torch.float32),
                delta=Guarded(P, torch.float32), zone=Guarded(P, torch.uint8), keep=Guarded(P, torch.uint8),
                keep_count=Guarded(1, torch.int32))
    binding.npd_delta_ifd_score(ms, mt, cnt, pc, pu, lo, hi, flags=flags, **{k: v.t for k, v in outs.items()})
    torch.cuda.synchronize()
    return {k: v.check().cpu().numpy() for k, v in outs.items()}


def test_segment_reduce_bookkeeping_bit_exact(oracle):
    rng = np.random.default_rng(7)
    for T, cu in ((1000, [0, 0, 1, 1, 9, 300, 300, 555, 901]),          # empty, length-1, unowned tail
                  (5000, np.concatenate([[3], 3 + np.cumsum(rng.integers(0, 40, 300))])),   # starts at 3
                  (70000, [0, 70000])):                                   # one long sample
        cu = np.asarray(cu, np.int32)
        cu = cu[cu <= T]
        x = rng.normal(size=T).astype(np.float32)
        m = (rng.random(T) < 0.7).astype(np.uint8)
        _say(f"segment reduce T={T} S={len(cu) - 1}")
        gpu = _segment_gpu(torch.from_numpy(x).to(dev()), torch.from_numpy(m).to(dev()), torch.from_numpy(cu).to(dev()))
        ref = oracle.segment_reduce(x.astype(np.float64), m, cu)
        assert gpu["status"] == 0
        np.testing.assert_array_equal(gpu["count"], ref["count"])
        np.testing.assert_array_equal(gpu["token_to_sample"], ref["token_to_sample"])
        np.testing.assert_allclose(gpu["sum"], ref["sum"], rtol=1e-5, atol=1e-4)
        np.testing.assert_allclose(gpu["mean"], ref["mean"], rtol=1e-5, atol=1e-5)
        assert (gpu["mean"][ref["count"] == 0] == 0).all()
    # S = 0 only clears token_to_sample; a decreasing cu_seqlens is flagged
    t2s = torch.zeros(10, dtype=torch.int32, device=dev())
    binding.npd_segment_reduce(None, torch.ones(10, dtype=torch.uint8, device=dev()),
                               torch.zeros(1, dtype=torch.int32, device=dev()), token_to_sample=t2s)
    assert (t2s == -1).all()
    bad = _segment_gpu(torch.ones(10, device=dev()), torch.ones(10, dtype=torch.uint8, device=dev()),
                       torch.tensor([0, 6, 4, 11], dtype=torch.int32, device=dev()))
    assert bad["status"] == binding.NPD_DEV_BAD_CU_SEQLENS
    assert bad["count"].tolist() == [6, 0, 0] and np.isnan(bad["sum"][1:]).all() and bad["sum"][0] == 6


def test_delta_ifd_hand_worked_cases_on_gpu():
    rows = []
    with open(os.path.join(HERE, "golden", "delta_ifd_zones.txt")) as f:
        for line in f:
            line = line.strip()
            if line and not line.startswith("#"):
                lhs, rhs = line.split("|")
                rows.append(([float(v) for v in lhs.split()], [float(v) for v in rhs.split()]))
    for (lsc, lsu, ltc, ltu, nc, nu, lo, hi, flags), (ifs, ift, d, zone, keep) in rows:
        f32 = lambda a: torch.tensor(a, dtype=torch.float32, device=dev())
        i32 = lambda a: torch.tensor(a, dtype=torch.int32, device=dev())
        out = _ifd_gpu(f32([lsc, lsu]), f32([ltc, ltu]), i32([int(nc), int(nu)]), i32([0]), i32([1]), lo, hi, int(flags))
        np.testing.assert_array_equal(out["ifd_student"], np.float32([ifs]))
        np.testing.assert_array_equal(out["ifd_teacher"], np.float32([ift]))
        np.testing.assert_array_equal(out["delta"], np.float32([d]))
        assert out["zone"][0] == int(zone) and out["keep"][0] == int(keep) and out["keep_count"][0] == int(keep)


def test_delta_ifd_invalid_pair_index_and_empty():
    f32 = lambda a: torch.tensor(a, dtype=torch.float32, device=dev())
    i32 = lambda a: torch.tensor(a, dtype=torch.int32, device=dev())
    out = _ifd_gpu(f32([1, 2]), f32([1, 2]), i32([3, 3]), i32([0, 5, -1]), i32([1, 1, 0]), 0.0, 1.0)
    assert out["zone"].tolist() == [1, 3, 3] and out["keep"].tolist() == [1, 0, 0] and out["keep_count"][0] == 1
    kc = torch.full((1,), 99, dtype=torch.int32, device=dev())
    binding.npd_delta_ifd_score(f32([1.0]), f32([1.0]), i32([1]), i32([]), i32([]), 0.0, 1.0, keep_count=kc)
    assert kc.item() == 0


@pytest.mark.parametrize("row_len,vocab,length_lo,length_hi,min_pairs", [
    (1024, 32000, 16, 200, 6),        # a handful of pairs at a real vocabulary
    (32768, 1024, 32, 400, 180),      # about 200 pairs (the sample count the blueprint names for this pass), small V
])
def test_cfg3_scoring_pass_reduced(oracle, row_len, vocab, length_lo, length_hi, min_pairs):
    """The Delta-IFD pass end to end on a reduced config 3: forward-only NLL of student and teacher logits,
    per-sample means, Delta-IFD, zones, and the middle-80 % filter."""
    w = synth.scaled(synth.config(3), n_rows=2, row_len=row_len, vocab=vocab, length_lo=length_lo,
                     length_hi=length_hi)
    w.prefix_lo, w.prefix_hi = 8, 64
    lay = synth.make_layout(w)
    P = len(lay.pair_cond)
    assert P >= min_pairs
    _say(f"{w.name} reduced: T={w.n_tokens} V={w.vocab} pairs={P}")
    T, V = w.n_tokens, w.vocab
    bs, bt = synth.delta_ifd_boosts(w, lay)
    s = torch.zeros((T, V), dtype=torch.bfloat16, device=dev())
    t = torch.zeros((T, V), dtype=torch.bfloat16, device=dev())
    labels = torch.from_numpy(lay.labels).to(dev())
    synth.fill_logits(w, s, t, label_boost=(labels, torch.from_numpy(bs).to(dev()), torch.from_numpy(bt).to(dev())))
    mask = torch.from_numpy(lay.loss_mask).to(dev())
    cu = torch.from_numpy(lay.cu_seqlens).to(dev())

    gs = run_gpu_kd(s, mask, labels=labels, want_grad=False)       # teacher kind NONE: NLL only
    gt = run_gpu_kd(t, mask, labels=labels, want_grad=False)
    rs = oracle.nll(_bits(s), lay.labels, lay.loss_mask)
    rt = oracle.nll(_bits(t), lay.labels, lay.loss_mask)
    compare_kd(dict(nll_s=gs["nll_s"], lse_s=gs["lse_s"]), dict(nll_s=rs["nll"], lse_s=rs["lse"]), lay.loss_mask,
               lay.cu_seqlens, oracle)
    compare_kd(dict(nll_s=gt["nll_s"]), dict(nll_s=rt["nll"]), lay.loss_mask, lay.cu_seqlens, oracle)

    seg_s = _segment_gpu(torch.from_numpy(gs["nll_s"].astype(np.float32)).to(dev()), mask, cu)
    seg_t = _segment_gpu(torch.from_numpy(gt["nll_s"].astype(np.float32)).to(dev()), mask, cu)
    ref_s = oracle.segment_reduce(rs["nll"], lay.loss_mask, lay.cu_seqlens)
    ref_t = oracle.segment_reduce(rt["nll"], lay.loss_mask, lay.cu_seqlens)
    np.testing.assert_array_equal(seg_s["count"], ref_s["count"])
    np.testing.assert_array_equal(seg_s["token_to_sample"], ref_s["token_to_sample"])
    nz = ref_s["count"] > 0
    assert (np.abs(seg_s["mean"][nz] - ref_s["mean"][nz]) <= REL_PER_SAMPLE * np.abs(ref_s["mean"][nz])).all()
    assert (np.abs(seg_t["mean"][nz] - ref_t["mean"][nz]) <= REL_PER_SAMPLE * np.abs(ref_t["mean"][nz])).all()

    # thresholds: the paper's fixed [0, 0.8], and the middle 80 % of the oracle's own Delta values
    ref0 = oracle.delta_ifd(ref_s["mean"], ref_t["mean"], ref_s["count"], lay.pair_cond, lay.pair_uncond, 0.0, 0.8)
    d_sorted = np.sort(ref0["delta"])
    n_cut = max(1, int(round(0.1 * P)))
    lo = float(0.5 * (d_sorted[n_cut - 1] + d_sorted[n_cut]))
    hi = float(0.5 * (d_sorted[P - n_cut - 1] + d_sorted[P - n_cut]))
    pc, pu = torch.from_numpy(lay.pair_cond).to(dev()), torch.from_numpy(lay.pair_uncond).to(dev())
    for (a, b) in ((0.0, 0.8), (lo, hi)):
        ref = oracle.delta_ifd(ref_s["mean"], ref_t["mean"], ref_s["count"], lay.pair_cond, lay.pair_uncond, a, b)
        gpu = _ifd_gpu(seg_s["mean_dev"], seg_t["mean_dev"], seg_s["count_dev"], pc, pu, a, b)
        np.testing.assert_allclose(gpu["delta"], ref["delta"], rtol=0, atol=2e-3)
        np.testing.assert_allclose(gpu["ifd_student"], ref["ifd_student"], rtol=REL_PER_SAMPLE)
        np.testing.assert_allclose(gpu["ifd_teacher"], ref["ifd_teacher"], rtol=REL_PER_SAMPLE)
        # pairs whose Delta sits within 1e-5 of a threshold may legitimately fall on either side
        clear = (np.abs(ref["delta"] - a) > 1e-5) & (np.abs(ref["delta"] - b) > 1e-5)
        np.testing.assert_array_equal(gpu["zone"][clear], ref["zone"][clear])
        np.testing.assert_array_equal(gpu["keep"][clear], ref["keep"][clear])
        assert gpu["keep_count"][0] == int(gpu["keep"].sum())
        if clear.all():
            assert gpu["keep_count"][0] == ref["keep_count"]
    assert ref["keep_count"] == P - 2 * n_cut     # the middle 80 %
    assert len(set(ref0["zone"].tolist())) >= 2   # the synthetic IFDs do spread over more than one zone


def test_cfg4_many_short_samples_inplace(oracle):
    """About 1,500 samples of 16..71 tokens in 65,536 tokens (the sample count the blueprint names for the stress
    configuration), heavy-tailed logits, gradient in place; small vocabulary so that every row is compared."""
    w = synth.scaled(synth.config(4), vocab=2048, length_lo=16, length_hi=71)
    lay, s, t, mask, labels = _inputs(w)
    S = lay.n_segments
    _say(f"{w.name} short samples: T={w.n_tokens} V={w.vocab} segments={S}")
    assert w.n_tokens == 65536 and S >= 1400
    sb = _bits(s)
    ref = oracle.kd_dense(sb, _bits(t), lay.labels, lay.loss_mask)
    gpu = run_gpu_kd(s, mask, t=t, labels=labels, inplace=True)
    assert gpu["status"] == 0
    compare_kd(gpu, ref, lay.loss_mask, lay.cu_seqlens, oracle)
    cu = torch.from_numpy(lay.cu_seqlens).to(dev())
    seg = _segment_gpu(torch.from_numpy(gpu["kd"].astype(np.float32)).to(dev()), mask, cu)
    rseg = oracle.segment_reduce(ref["kd"], lay.loss_mask, lay.cu_seqlens)
    np.testing.assert_array_equal(seg["count"], rseg["count"])
    np.testing.assert_array_equal(seg["token_to_sample"], rseg["token_to_sample"])
    nz = rseg["count"] > 0
    assert (np.abs(seg["mean"][nz] - rseg["mean"][nz]) <= REL_PER_SAMPLE * np.abs(rseg["mean"][nz]) + 1e-5).all()
    assert (seg["mean"][~nz] == 0).all()


# --------------------------------------------------------------------------- full benchmark sizes

def _all_rows_scalars(oracle, fn, lay, s, gpu_cols, chunk=2048):
    """Every row of a full-size batch against the oracle, scalar outputs only: `fn(r0, r1)` returns the oracle's dict
    for rows [r0, r1); `gpu_cols` maps its keys to device tensors [T].  The per-position bars of compare_kd."""
    T = s.shape[0]
    for r0 in range(0, T, chunk):
        r1 = min(T, r0 + chunk)
        ref = fn(r0, r1)
        gpu = {key: col[r0:r1].cpu().numpy().astype(np.float64) for key, col in gpu_cols.items()}
        compare_kd(gpu, {key: ref[key] for key in gpu}, lay.loss_mask[r0:r1])


def _grad_chunks(T, n_chunks=4, rows=512):
    """Starts of `n_chunks` blocks of `rows` consecutive rows spread over [0, T): first, last and evenly between."""
    return [int(round(c * (T - rows) / (n_chunks - 1))) for c in range(n_chunks)]


@pytest.mark.parametrize("div,no_workspace", [("forward", False), ("forward", True), ("reverse", False),
                                              ("skew", False), ("skew_reverse", False)])
def test_cfg1_full_size(oracle, div, no_workspace):
    """Config 1 at its real size (32,768 x 151,936, the launch bench.py times).  Forward KL: the three per-position
    scalars of ALL rows and the gradient of 2,048 rows (four blocks of 512) against the oracle, with the row-gang
    kernels and with the kernels that need no workspace.  The other divergences: a sample of rows element by element.
    Every row, always: properties that hold at any size."""
    w = synth.config(1)
    lay, s, t, mask, labels = _inputs(w)
    T, V = w.n_tokens, w.vocab
    _say(f"{w.name} full size T={T} V={V} div={div} no_workspace={no_workspace}")
    g = torch.empty((T, V), dtype=torch.bfloat16, device=dev())
    kd = torch.empty(T, device=dev())
    nll = torch.empty(T, device=dev())
    tnll = torch.empty(T, device=dev())
    status = torch.zeros(1, dtype=torch.int32, device=dev())
    binding.npd_kd_loss_fwd_bwd(s, mask, teacher_dense=t, labels=labels, grad_out=g, kd_tok=kd, nll_tok=nll,
                                teacher_nll_tok=tnll, dev_status=status, no_workspace=no_workspace,
                                divergence=0 if div == "forward" else DIVS[div], skew_alpha=0.1)
    torch.cuda.synchronize()
    assert status.item() == 0
    m = mask.bool()
    assert (kd[~m] == 0).all() and (kd[m] > 0).all() and torch.isfinite(kd).all()
    assert (nll[~m] == 0).all() and (nll[m] > 0).all()
    # masked rows zero-filled; every gradient row sums to ~0 (bf16 rounding noise only)
    rs = _row_sums(g, 2048)
    assert (rs[~m] == 0).all() and rs.abs().max().item() < (2e-2 if div == "forward" else 0.5)
    if div == "forward":
        _all_rows_scalars(oracle, lambda r0, r1: oracle.kd_dense(_bits(s[r0:r1]), _bits(t[r0:r1]), lay.labels[r0:r1],
                                                                 lay.loss_mask[r0:r1], want_grad=False),
                          lay, s, dict(kd=kd, nll_s=nll, nll_t=tnll))
        for r0 in _grad_chunks(T):
            r1 = r0 + 512
            ref = oracle.kd_dense(_bits(s[r0:r1]), _bits(t[r0:r1]), lay.labels[r0:r1], lay.loss_mask[r0:r1])
            compare_kd(dict(grad=g[r0:r1].float().cpu().numpy().astype(np.float64)), dict(grad=ref["grad"]),
                       lay.loss_mask[r0:r1])
        return
    rng = np.random.default_rng(5)
    scored = np.flatnonzero(lay.loss_mask)
    rows = np.sort(np.concatenate([rng.choice(scored, 44, replace=False), [scored[0], scored[-1]],
                                   np.flatnonzero(lay.loss_mask == 0)[:2]]))
    ridx = torch.from_numpy(rows).to(dev())
    ref = oracle.kd_dense(_bits(s[ridx]), _bits(t[ridx]), lay.labels[rows], lay.loss_mask[rows])
    ref.update(oracle.div_dense(_bits(s[ridx]), _bits(t[ridx]), div, 0.1, mask=lay.loss_mask[rows]))
    gpu = dict(kd=kd[ridx].cpu().numpy().astype(np.float64), nll_s=nll[ridx].cpu().numpy().astype(np.float64),
               nll_t=tnll[ridx].cpu().numpy().astype(np.float64), grad=g[ridx].float().cpu().numpy().astype(np.float64))
    compare_kd(gpu, ref, lay.loss_mask[rows], amp_from_ref=True)


def _row_sums(g, step=1024):
    T = g.shape[0]
    rs = torch.empty(T, device=g.device)
    for r0 in range(0, T, step):
        rs[r0:r0 + step] = g[r0:r0 + step].float().sum(1)
    return rs


def _sample_rows(lay, n, seed):
    rng = np.random.default_rng(seed)
    scored = np.flatnonzero(lay.loss_mask)
    masked = np.flatnonzero(lay.loss_mask == 0)
    return np.sort(np.concatenate([rng.choice(scored, n, replace=False), [scored[0], scored[-1]], masked[:2]]))


def test_cfg2_full_size(oracle):
    """Config 2 at its real size (top-k = 64 teacher, tau = 2): kd_tok and nll_tok of all rows and the gradient of
    1,024 rows against the oracle; all rows by properties that hold at any size."""
    w = synth.config(2)
    lay, s, _, mask, labels = _inputs(w, dense_teacher=False)
    T, V = w.n_tokens, w.vocab
    _say(f"{w.name} full size T={T} V={V} k={w.topk}")
    idx, val = synth.make_topk_teacher(w, s)
    g = torch.empty((T, V), dtype=torch.bfloat16, device=dev())
    kd, nll = torch.empty(T, device=dev()), torch.empty(T, device=dev())
    status = torch.zeros(1, dtype=torch.int32, device=dev())
    binding.npd_kd_loss_fwd_bwd(s, mask, teacher_idx=idx, teacher_val=val, labels=labels, tau=w.tau, grad_out=g,
                                kd_tok=kd, nll_tok=nll, dev_status=status)
    torch.cuda.synchronize()
    assert status.item() == 0
    m = mask.bool()
    assert (kd[~m] == 0).all() and (kd[m] > 0).all() and torch.isfinite(kd).all()
    rs = _row_sums(g)
    assert (rs[~m] == 0).all() and rs.abs().max().item() < 2e-2
    iv, vv = idx.cpu().numpy(), val.cpu().numpy()
    _all_rows_scalars(oracle, lambda r0, r1: oracle.kd_topk(_bits(s[r0:r1]), iv[r0:r1], vv[r0:r1], lay.labels[r0:r1],
                                                            lay.loss_mask[r0:r1], tau=w.tau, want_grad=False),
                      lay, s, dict(kd=kd, nll_s=nll))
    for r0 in _grad_chunks(T, 2):
        r1 = r0 + 512
        ref = oracle.kd_topk(_bits(s[r0:r1]), iv[r0:r1], vv[r0:r1], lay.labels[r0:r1], lay.loss_mask[r0:r1], tau=w.tau)
        compare_kd(dict(grad=g[r0:r1].float().cpu().numpy().astype(np.float64)), dict(grad=ref["grad"]),
                   lay.loss_mask[r0:r1], tau=w.tau)


def test_cfg3_full_size_scoring_pass(oracle):
    """Config 3 at its real size (2 x 32,768 tokens, two logit tensors): every per-token NLL of both models, the
    per-sample means and the Delta-IFD decisions against the oracle."""
    w = synth.config(3)
    lay = synth.make_layout(w)
    T, V, P = w.n_tokens, w.vocab, len(lay.pair_cond)
    _say(f"{w.name} full size T={T} V={V} pairs={P}")
    bs, bt = synth.delta_ifd_boosts(w, lay)
    s = torch.empty((T, V), dtype=torch.bfloat16, device=dev())
    t = torch.empty((T, V), dtype=torch.bfloat16, device=dev())
    labels = torch.from_numpy(lay.labels).to(dev())
    synth.fill_logits(w, s, t, label_boost=(labels, torch.from_numpy(bs).to(dev()), torch.from_numpy(bt).to(dev())))
    mask = torch.from_numpy(lay.loss_mask).to(dev())
    cu = torch.from_numpy(lay.cu_seqlens).to(dev())
    nll_s, nll_t = torch.empty(T, device=dev()), torch.empty(T, device=dev())
    status = torch.zeros(1, dtype=torch.int32, device=dev())
    binding.npd_kd_loss_fwd_bwd(s, mask, labels=labels, nll_tok=nll_s, dev_status=status)
    binding.npd_kd_loss_fwd_bwd(t, mask, labels=labels, nll_tok=nll_t, dev_status=status)
    torch.cuda.synchronize()
    assert status.item() == 0
    ref_s, ref_t = np.zeros(T), np.zeros(T)
    step = 2048
    for r0 in range(0, T, step):          # the oracle sees the same bits, chunk by chunk
        r1 = min(T, r0 + step)
        if lay.loss_mask[r0:r1].any():
            ref_s[r0:r1] = oracle.nll(_bits(s[r0:r1]), lay.labels[r0:r1], lay.loss_mask[r0:r1])["nll"]
            ref_t[r0:r1] = oracle.nll(_bits(t[r0:r1]), lay.labels[r0:r1], lay.loss_mask[r0:r1])["nll"]
        _say(f"  oracle rows {r1}/{T}")
    compare_kd(dict(nll_s=nll_s.cpu().numpy().astype(np.float64), nll_t=nll_t.cpu().numpy().astype(np.float64)),
               dict(nll_s=ref_s, nll_t=ref_t), lay.loss_mask, lay.cu_seqlens, oracle)
    seg_s, seg_t = _segment_gpu(nll_s, mask, cu), _segment_gpu(nll_t, mask, cu, want_t2s=False)
    rseg_s = oracle.segment_reduce(ref_s, lay.loss_mask, lay.cu_seqlens)
    rseg_t = oracle.segment_reduce(ref_t, lay.loss_mask, lay.cu_seqlens)
    np.testing.assert_array_equal(seg_s["count"], rseg_s["count"])
    np.testing.assert_array_equal(seg_s["token_to_sample"], rseg_s["token_to_sample"])
    ref0 = oracle.delta_ifd(rseg_s["mean"], rseg_t["mean"], rseg_s["count"], lay.pair_cond, lay.pair_uncond, 0.0, 0.8)
    d_sorted = np.sort(ref0["delta"])
    n_cut = max(1, int(round(0.1 * P)))
    lo = float(0.5 * (d_sorted[n_cut - 1] + d_sorted[n_cut]))
    hi = float(0.5 * (d_sorted[P - n_cut - 1] + d_sorted[P - n_cut]))
    pc, pu = torch.from_numpy(lay.pair_cond).to(dev()), torch.from_numpy(lay.pair_uncond).to(dev())
    for (a, b) in ((0.0, 0.8), (lo, hi)):
        ref = oracle.delta_ifd(rseg_s["mean"], rseg_t["mean"], rseg_s["count"], lay.pair_cond, lay.pair_uncond, a, b)
        gpu = _ifd_gpu(seg_s["mean_dev"], seg_t["mean_dev"], seg_s["count_dev"], pc, pu, a, b)
        np.testing.assert_allclose(gpu["delta"], ref["delta"], rtol=0, atol=2e-3)
        clear = (np.abs(ref["delta"] - a) > 1e-5) & (np.abs(ref["delta"] - b) > 1e-5)
        np.testing.assert_array_equal(gpu["zone"][clear], ref["zone"][clear])
        np.testing.assert_array_equal(gpu["keep"][clear], ref["keep"][clear])
        assert gpu["keep_count"][0] == int(gpu["keep"].sum())
    assert ref["keep_count"] == P - 2 * n_cut


def test_cfg4_full_size_inplace(oracle):
    """Config 4 at its real size (65,536 x 262,144, heavy tails, ~500 short samples, gradient written over the
    student logits): the three per-position scalars of all rows and the gradient of two blocks of 256 rows against
    the oracle (which sees the student logits before the call destroys them); all rows by properties."""
    w = synth.config(4)
    lay, s, t, mask, labels = _inputs(w)
    T, V = w.n_tokens, w.vocab
    _say(f"{w.name} full size T={T} V={V} segments={lay.n_segments}")
    ref_all = {key: np.empty(T) for key in ("kd", "nll_s", "nll_t")}
    for r0 in range(0, T, 2048):
        r1 = r0 + 2048
        ref = oracle.kd_dense(_bits(s[r0:r1]), _bits(t[r0:r1]), lay.labels[r0:r1], lay.loss_mask[r0:r1], want_grad=False)
        for key in ref_all:
            ref_all[key][r0:r1] = ref[key]
    blocks = _grad_chunks(T, 2, 256)
    ref_grad = [oracle.kd_dense(_bits(s[r0:r0 + 256]), _bits(t[r0:r0 + 256]), lay.labels[r0:r0 + 256],
                                lay.loss_mask[r0:r0 + 256])["grad"] for r0 in blocks]
    kd, nll, tnll = (torch.empty(T, device=dev()) for _ in range(3))
    status = torch.zeros(1, dtype=torch.int32, device=dev())
    binding.npd_kd_loss_fwd_bwd(s, mask, teacher_dense=t, labels=labels, grad_out=s, kd_tok=kd, nll_tok=nll,
                                teacher_nll_tok=tnll, dev_status=status)
    torch.cuda.synchronize()
    assert status.item() == 0
    m = mask.bool()
    assert (kd[~m] == 0).all() and (kd[m] >= 0).all() and torch.isfinite(kd).all() and torch.isfinite(nll).all()
    rs = _row_sums(s, 512)
    assert (rs[~m] == 0).all() and rs.abs().max().item() < 2e-2
    compare_kd(dict(kd=kd.cpu().numpy().astype(np.float64), nll_s=nll.cpu().numpy().astype(np.float64),
                    nll_t=tnll.cpu().numpy().astype(np.float64)), ref_all, lay.loss_mask)
    for r0, rg in zip(blocks, ref_grad):
        compare_kd(dict(grad=s[r0:r0 + 256].float().cpu().numpy().astype(np.float64)), dict(grad=rg),
                   lay.loss_mask[r0:r0 + 256])
    # per-sample bookkeeping of the ~500 short segments
    cu = torch.from_numpy(lay.cu_seqlens).to(dev())
    seg = _segment_gpu(kd, mask, cu)
    rseg = oracle.segment_reduce(kd.cpu().numpy().astype(np.float64), lay.loss_mask, lay.cu_seqlens)
    np.testing.assert_array_equal(seg["count"], rseg["count"])
    np.testing.assert_array_equal(seg["token_to_sample"], rseg["token_to_sample"])
    np.testing.assert_allclose(seg["sum"], rseg["sum"], rtol=1e-5, atol=1e-5)


# --------------------------------------------------------------------------- row-gang kernels: slices and their exchange

@pytest.mark.parametrize("V,stride", [
    (8 * 3828, 8 * 3828),          # the shortest rows that are shared: two slices of 1,920 + 1,908 groups
    (8 * 5104, 8 * 5104),          # two full slices
    (8 * 5105 + 5, 8 * 5106),      # three slices and a 5-element tail; rows that begin 16 bytes off a 128-byte line
    (151936, 151936),              # eight slices of 2,374 groups
    (8 * 2552 * 9 + 8, 8 * 2552 * 9 + 24),   # ten slices; a row pitch that moves the boundaries by 0 .. 7 groups
])
@pytest.mark.parametrize("tau,div", [(1.0, "forward"), (2.0, "forward"), (1.0, "reverse"), (1.0, "skew"),
                                     (2.0, "skew"), (1.0, "skew_reverse"), (2.0, "skew_reverse")])
def test_gang_slices_with_labels_on_their_edges(oracle, V, stride, tau, div):
    """Rows shared by 2 .. 10 workgroups; the labels sit on the first and last element of slices, in the tail and
    next to slice boundaries, so that the label logit, the NLLs and the one-hot term of the composite gradient are
    taken by the right workgroup.  Out of place and in place."""
    assert binding.npd_workspace_bytes(4, V, tau=1.0) > 0
    nvec = V // 8
    width = 1528 if div.startswith("skew") else 2552     # groups a slice is sized to at most (fewer for the skew forms)
    gang = -(-nvec // width)
    per = -(-(-(-nvec // gang)) // 8) * 8      # slices are multiples of 8 groups (128 bytes) long; a boundary sits
    sh = 3 if stride % 64 else 0                # 0 .. 7 groups below a multiple of that (by the row's address)
    edges = sorted({0, 7, 8 * (per - sh) - 1, 8 * (per - sh), 8 * per - 1, 8 * per, 8 * per + 1,
                    8 * (gang - 1) * per - 1, 8 * (gang - 1) * per, 8 * nvec - 1, V - 1, V // 2})
    T = 2 * len(edges)
    w = synth.scaled(synth.config(1), n_rows=1, row_len=T, vocab=V, length_lo=4, length_hi=9)
    lay, s, t, mask, _ = _inputs(w, stride)
    lab = np.array([edges[i % len(edges)] for i in range(T)], np.int32)
    labels = torch.from_numpy(lab).to(dev())
    ce = 0.25 if tau == 1.0 else 0.0       # the composite gradient shares the student's exponentials at tau = 1 only
    _say(f"gang slices V={V} stride={stride} gang={gang} tau={tau} div={div}")
    sb, tb = _bits(s.contiguous()), _bits(t.contiguous())
    if div == "forward":
        ref = oracle.kd_dense(sb, tb, lab, lay.loss_mask, tau=tau, grad_scale=0.75, ce_grad_scale=ce)
    else:
        ref = oracle.div_dense(sb, tb, div, 0.1, labels=lab, mask=lay.loss_mask, tau=tau, grad_scale=0.75,
                               ce_grad_scale=ce)
        nl = oracle.kd_dense(sb, tb, lab, lay.loss_mask, want_grad=False)
        ref.update(nll_s=nl["nll_s"], nll_t=nl["nll_t"], lse_s=nl["lse_s"])
    for inplace in (False, True):
        gpu = run_gpu_kd(s.clone() if inplace else s, mask, t=t, labels=labels, tau=tau, grad_scale=0.75,
                         ce_grad_scale=ce, inplace=inplace, divergence=DIVS.get(div, 0), skew_alpha=0.1)
        assert gpu["status"] == 0
        compare_kd(gpu, ref, lay.loss_mask, lay.cu_seqlens, oracle, grad_scale=0.75 + ce, tau=tau,
                   amp_from_ref=div != "forward")


@pytest.mark.parametrize("V,stride,tau", [(8 * 5105 + 5, 8 * 5106, 1.0), (151936, 151936, 2.0), (151936, 151936, 1.0)])
def test_gang_topk_support_and_labels_on_slice_edges(oracle, V, stride, tau):
    """Top-k teacher on rows shared by several workgroups: support positions and labels on the first and last element
    of slices and in the sub-group tail, labels inside and outside the support; out of place and in place."""
    assert binding.npd_workspace_bytes(4, V, teacher_kind=binding.NPD_TEACHER_TOPK, topk=24) > 0
    nvec = V // 8
    gang = -(-nvec // 2552)
    per = -(-(-(-nvec // gang)) // 8) * 8      # slices are multiples of 8 groups (128 bytes) long; a boundary sits
    sh = 3 if stride % 64 else 0                # 0 .. 7 groups below a multiple of that (by the row's address)
    edges = sorted({0, 7, 8 * (per - sh) - 1, 8 * (per - sh), 8 * per - 1, 8 * per, 8 * per + 1,
                    8 * (gang - 1) * per - 1, 8 * (gang - 1) * per, 8 * nvec - 1, V - 1, V // 2})
    T, k = 2 * len(edges), 24
    w = synth.scaled(synth.config(2), n_rows=1, row_len=T, vocab=V, length_lo=4, length_hi=9, topk=k)
    lay, s, _, mask, _ = _inputs(w, stride, dense_teacher=False)
    idx, val = synth.make_topk_teacher(w, s)
    lab = np.array([edges[i % len(edges)] for i in range(T)], np.int32)
    idx_np = idx.cpu().numpy().copy()
    for r in range(T):
        # the first entries of the support sit on slice edges (kept unique); in even rows the label is one of them
        want = [e for e in edges if r % 2 == 0 or e != lab[r]][:10]
        rest = [int(v) for v in idx_np[r] if int(v) not in want][:k - len(want)]
        idx_np[r] = np.array(want + rest, np.int32)
        assert len(set(idx_np[r].tolist())) == k
    idx = torch.from_numpy(idx_np).to(dev())
    labels = torch.from_numpy(lab).to(dev())
    ce = 0.25 if tau == 1.0 else 0.0
    _say(f"gang top-k V={V} stride={stride} gang={gang} tau={tau}")
    ref = oracle.kd_topk(_bits(s.contiguous()), idx_np, val.cpu().numpy(), lab, lay.loss_mask, tau=tau, grad_scale=0.75,
                         ce_grad_scale=ce)
    assert ref["bad_index_rows"] == 0
    for inplace in (False, True):
        gpu = run_gpu_kd(s.clone() if inplace else s, mask, idx=idx, val=val, labels=labels, tau=tau, grad_scale=0.75,
                         ce_grad_scale=ce, inplace=inplace)
        assert gpu["status"] == 0
        compare_kd(gpu, ref, lay.loss_mask, lay.cu_seqlens, oracle, grad_scale=0.75 + ce, tau=tau)


def test_gang_wait_is_bounded(oracle):
    """A workgroup of a row gang that does not see the rest of its row within its poll limit gives up, marks what it
    writes NaN and sets NPD_DEV_GANG_TIMEOUT: forced here with a limit of one poll (the kernel still ends normally);
    with the default limit restored the same call is exact again."""
    V = 151936
    w = synth.scaled(synth.config(1), n_rows=1, row_len=256, vocab=V, length_lo=8, length_hi=64)
    lay, s, t, mask, labels = _inputs(w)
    good = run_gpu_kd(s, mask, t=t, labels=labels)
    assert good["status"] == 0
    lib = binding.load()
    prev = lib.npd_debug_gang_spin_limit(1)
    try:
        hurried = run_gpu_kd(s, mask, t=t, labels=labels)
    finally:
        lib.npd_debug_gang_spin_limit(prev)
    assert hurried["status"] in (0, binding.NPD_DEV_GANG_TIMEOUT)
    m = lay.loss_mask.astype(bool)
    if hurried["status"]:
        # a row is either what it should be or carries NaN (slices of workgroups that gave up)
        gb, hb = good["grad_bits"], hurried["grad_bits"]
        ok = (gb == hb) | (hb == 0x7fc0)
        assert ok.all() and (hb[m] == 0x7fc0).any()
        assert (hb[~m] == 0).all()
        kd_ok = (hurried["kd"] == good["kd"]) | np.isnan(hurried["kd"])
        assert kd_ok.all()
    again = run_gpu_kd(s, mask, t=t, labels=labels)
    assert again["status"] == 0
    np.testing.assert_array_equal(again["grad_bits"], good["grad_bits"])
    for key in ("kd", "nll_s", "nll_t", "lse_s"):
        np.testing.assert_array_equal(again[key], good[key])
    ref = oracle.kd_dense(_bits(s), _bits(t), lay.labels, lay.loss_mask)
    compare_kd(again, ref, lay.loss_mask, lay.cu_seqlens, oracle)


# --------------------------------------------------------------------------- logits in the thousands

@pytest.mark.parametrize("V", [151936, 262144])
@pytest.mark.parametrize("mode", ["dense", "dense_no_workspace", "dense_inplace", "topk", "skew", "skew_reverse"])
def test_logits_in_the_thousands(oracle, V, mode):
    """Heavy tails by construction: every row carries a cluster of 48 logits around +-800 ... +-3000 in both models
    (same places or not), so the row's log-sum-exp is in the thousands of bits and the gradient sweep takes its
    precise form rather than the one with the weights folded into the exponents.  (The skew forms: sweep 1 of the
    row-gang kernel cannot keep its fixed references on such rows and rebuilds its cached exponentials.)"""
    T = 16
    gen = torch.Generator(device=dev()).manual_seed(77 + V % 1000)
    s = (3.0 * torch.randn((T, V), device=dev(), generator=gen)).to(torch.bfloat16)
    t = (3.0 * torch.randn((T, V), device=dev(), generator=gen)).to(torch.bfloat16)
    levels = [800.0, -800.0, 1200.0, 2000.0, -2000.0, 3000.0, 1000.0, -3000.0]
    idx = torch.empty((T, 64), dtype=torch.int32, device=dev())
    for r in range(T):
        pos = torch.randperm(V, device=dev(), generator=gen)[:64]
        level = levels[r % len(levels)]
        bump = level + 6.0 * torch.randn(48, device=dev(), generator=gen)
        s[r, pos[:48]] = bump.to(torch.bfloat16)
        # the teacher's cluster sits on the same places in even rows, on 48 places shifted by 16 in odd rows
        tp = pos[:48] if r % 2 == 0 else pos[16:64]
        t[r, tp] = (level + 8.0 + 6.0 * torch.randn(48, device=dev(), generator=gen)).to(torch.bfloat16)
        idx[r] = pos.to(torch.int32)
    labels = torch.randint(0, V, (T,), device=dev(), generator=gen, dtype=torch.int32)
    mask_np = np.ones(T, np.uint8)
    mask_np[5] = 0
    mask = torch.from_numpy(mask_np).to(dev())
    sb, tb = _bits(s), _bits(t)
    _say(f"logits in the thousands V={V} mode={mode}")
    if mode == "topk":
        val = torch.gather(t.float(), 1, idx.long()).contiguous()
        ref = oracle.kd_topk(sb, idx.cpu().numpy(), val.cpu().numpy(), labels.cpu().numpy(), mask_np)
        gpu = run_gpu_kd(s, mask, idx=idx, val=val, labels=labels)
    elif mode.startswith("skew"):
        ref = oracle.div_dense(sb, tb, mode, 0.1, labels=labels.cpu().numpy(), mask=mask_np)
        nl = oracle.kd_dense(sb, tb, labels.cpu().numpy(), mask_np, want_grad=False)
        ref.update(nll_s=nl["nll_s"], nll_t=nl["nll_t"], lse_s=nl["lse_s"])
        assert np.isfinite(ref["kd"]).all() and np.isfinite(ref["grad"]).all()
        gpu = run_gpu_kd(s, mask, t=t, labels=labels, divergence=DIVS[mode], skew_alpha=0.1)
    else:
        ref = oracle.kd_dense(sb, tb, labels.cpu().numpy(), mask_np)
        gpu = run_gpu_kd(s.clone() if mode == "dense_inplace" else s, mask, t=t, labels=labels,
                         inplace=mode == "dense_inplace", no_workspace=mode == "dense_no_workspace")
    assert gpu["status"] == 0
    # more than half of the rows have a log-sum-exp of 800 ... 3000 nats (the negative clusters carry no mass)
    assert (np.abs(ref["lse_s"]) > 700).sum() > T // 2
    compare_kd(gpu, ref, mask_np, amp_from_ref=mode.startswith("skew"))
    assert np.abs(gpu["grad"]).max() > 0.02      # the clusters really carry the probability mass


# --------------------------------------------------------------------------- composite loss of Eq. 1 (KD + hard-label CE)

@pytest.mark.parametrize("V,tau,gs,cs,inplace", [
    (151936, 1.0, 0.9, 0.1, False),    # lambda = 0.9 (the paper's default): row-resident kernel, folded weights
    (151936, 1.0, 0.0, 1.0, True),     # CE only, in place
    (151936, 1.0, -0.5, 1.0, False),   # weights of opposite sign: precise form
    (151936, 2.0, 0.9, 0.1, False),    # tau != 1: the CE softmax needs its own exponentials
    (4099, 1.0, 0.9, 0.1, False),      # small vocabulary, ragged tail
    (1000, 2.0, 0.5, 0.5, True),
])
@pytest.mark.parametrize("no_workspace", [False, True])
def test_composite_gradient_dense(oracle, V, tau, gs, cs, inplace, no_workspace):
    if no_workspace and binding.npd_workspace_bytes(8, V, tau=tau) == 0:
        pytest.skip("this shape needs no workspace: one kernel either way")
    n_rows, row_len = (2, 64) if V > 100000 else (2, 160)
    w = synth.scaled(synth.config(1), n_rows=n_rows, row_len=row_len, vocab=V, length_lo=8, length_hi=64)
    _say(f"composite dense V={V} tau={tau} grad_scale={gs} ce_grad_scale={cs} inplace={inplace}")
    lay, s, t, mask, labels = _inputs(w)
    ref = oracle.kd_dense(_bits(s), _bits(t), lay.labels, lay.loss_mask, tau=tau, grad_scale=gs, ce_grad_scale=cs)
    gpu = run_gpu_kd(s.clone() if inplace else s, mask, t=t, labels=labels, tau=tau, grad_scale=gs, ce_grad_scale=cs,
                     inplace=inplace, no_workspace=no_workspace)
    assert gpu["status"] == 0
    compare_kd(gpu, ref, lay.loss_mask, lay.cu_seqlens, oracle, grad_scale=abs(gs) + abs(cs) * tau, tau=tau)
    # the label position carries the -ce_grad_scale of the one-hot target: a sizeable negative entry there
    if cs > 0 and gs >= 0:
        rows = np.flatnonzero(lay.loss_mask)[:8]
        assert (gpu["grad"][rows, lay.labels[rows]] < -0.5 * cs).all()


@pytest.mark.parametrize("V,k,tau,inplace", [(151936, 64, 1.0, False), (151936, 10, 2.0, True), (5003, 20, 1.0, False)])
def test_composite_gradient_topk(oracle, V, k, tau, inplace):
    n_rows, row_len = (2, 64) if V > 100000 else (2, 128)
    w = synth.scaled(synth.config(2), n_rows=n_rows, row_len=row_len, vocab=V, length_lo=8, length_hi=64, topk=k)
    _say(f"composite top-k V={V} k={k} tau={tau} inplace={inplace}")
    lay, s, _, mask, labels = _inputs(w, dense_teacher=False)
    idx, val = synth.make_topk_teacher(w, s)
    # every other row: the label is one of the teacher's support positions (unless it already is)
    for r in range(0, w.n_tokens, 2):
        if not (idx[r] == int(lay.labels[r])).any():
            idx[r, r % k] = int(lay.labels[r])
    ref = oracle.kd_topk(_bits(s), idx.cpu().numpy(), val.cpu().numpy(), lay.labels, lay.loss_mask, tau=tau,
                         grad_scale=0.9, ce_grad_scale=0.1)
    for no_workspace in (False, True):
        gpu = run_gpu_kd(s.clone() if inplace else s, mask, idx=idx, val=val, labels=labels, tau=tau, grad_scale=0.9,
                         ce_grad_scale=0.1, inplace=inplace, no_workspace=no_workspace)
        assert gpu["status"] == 0 and ref["bad_index_rows"] == 0
        compare_kd(gpu, ref, lay.loss_mask, lay.cu_seqlens, oracle, grad_scale=0.9 + 0.1 * tau, tau=tau)


def test_composite_gradient_bad_label_poisons_row():
    V = 151936
    s = torch.randn((3, V), device=dev()).to(torch.bfloat16)
    t = torch.randn((3, V), device=dev()).to(torch.bfloat16)
    labels = torch.tensor([5, V, 7], dtype=torch.int32, device=dev())
    mask = torch.ones(3, dtype=torch.uint8, device=dev())
    gpu = run_gpu_kd(s, mask, t=t, labels=labels, grad_scale=0.9, ce_grad_scale=0.1)
    assert gpu["status"] == binding.NPD_DEV_BAD_LABEL
    assert np.isnan(gpu["grad"][1]).all() and np.isfinite(gpu["grad"][[0, 2]]).all() and np.isfinite(gpu["kd"]).all()


def test_policy_lag_monitor_is_the_same_entry_point_with_roles_swapped(oracle):
    """The paper tracks KL(pi_learner || pi_generator) per step: forward-only npd_kd_loss_fwd_bwd with the learner's
    logits in the teacher slot and the generator's in the student slot, then a per-sample mean."""
    w = synth.scaled(synth.config(1), n_rows=1, row_len=96, vocab=151936, length_lo=8, length_hi=48)
    lay, gen, learner, mask, labels = _inputs(w)
    gpu = run_gpu_kd(gen, mask, t=learner, want_grad=False)
    ref = oracle.kd_dense(_bits(gen), _bits(learner), None, lay.loss_mask, want_grad=False)
    compare_kd(gpu, ref, lay.loss_mask, lay.cu_seqlens, oracle)
    rev = oracle.kd_dense(_bits(learner), _bits(gen), None, lay.loss_mask, want_grad=False)
    assert np.abs(rev["kd"] - ref["kd"]).max() > 1e-3      # the direction matters


def _policy_lag_gpu(kl, mask, cu, eps):
    S = cu.numel() - 1
    seg_mean, seg_cnt = Guarded(S, torch.float32), Guarded(S, torch.int32)
    bmean, bcnt, exc = Guarded(1, torch.float32), Guarded(1, torch.int32), Guarded(1, torch.int32)
    status = torch.zeros(1, dtype=torch.int32, device=dev())
    binding.npd_policy_lag(kl, mask, cu, eps, seg_kl_mean=seg_mean.t, seg_count=seg_cnt.t, batch_kl_mean=bmean.t,
                           batch_count=bcnt.t, lag_exceeded=exc.t, dev_status=status)
    torch.cuda.synchronize()
    return dict(seg_mean=seg_mean.check().cpu().numpy().astype(np.float64), seg_count=seg_cnt.check().cpu().numpy(),
                batch_mean=float(bmean.check().item()), batch_count=int(bcnt.check().item()),
                exceeded=int(exc.check().item()), status=int(status.item()))


def test_policy_lag_and_perplexity_at_full_vocabulary(oracle):
    """The appendix's policy-latency monitor, end to end on the GPU at V = 151,936: per-position KL(learner ||
    generator) from the forward-only KD call with the roles swapped, its per-sample and per-step means, the
    near-policy decision against epsilon, and the perplexity of every sample from the same call's NLLs -- all three
    against the oracle."""
    w = synth.scaled(synth.config(1), n_rows=2, row_len=160, vocab=151936, length_lo=8, length_hi=64)
    lay, gen, _, mask, labels = _inputs(w, dense_teacher=False)
    # a learner a few optimiser steps away from the generator: small logit drift
    g = torch.Generator(device=dev()).manual_seed(41)
    learner = (gen.float() + 0.35 * torch.randn(gen.shape, device=dev(), generator=g)).to(torch.bfloat16)
    cu = torch.from_numpy(lay.cu_seqlens).to(dev())
    T, S = w.n_tokens, lay.n_segments
    kl, nll = torch.empty(T, device=dev()), torch.empty(T, device=dev())
    binding.npd_kd_loss_fwd_bwd(gen, mask, teacher_dense=learner, labels=labels, kd_tok=kl, teacher_nll_tok=nll)
    ref_tok = oracle.kd_dense(_bits(gen), _bits(learner), lay.labels, lay.loss_mask, want_grad=False)
    ref = oracle.policy_lag(ref_tok["kd"], lay.loss_mask, lay.cu_seqlens, 0.10)
    assert 0.01 < ref["batch_mean"] < 1.0
    for eps in (0.10, ref["batch_mean"] * 0.9, ref["batch_mean"] * 1.1, 0.0, 5.0):
        got = _policy_lag_gpu(kl, mask, cu, eps)
        want = oracle.policy_lag(ref_tok["kd"], lay.loss_mask, lay.cu_seqlens, eps)
        assert got["status"] == 0 and got["exceeded"] == want["exceeded"], eps
        assert got["batch_count"] == want["batch_count"] == int(lay.loss_mask.sum())
        np.testing.assert_array_equal(got["seg_count"], want["seg_count"])
        assert abs(got["batch_mean"] - want["batch_mean"]) <= 1e-3 * want["batch_mean"]
        np.testing.assert_allclose(got["seg_mean"], want["seg_mean"], rtol=1e-3, atol=1e-7)
    assert _policy_lag_gpu(kl, mask, cu, ref["batch_mean"] * 0.9)["exceeded"] == 1
    assert _policy_lag_gpu(kl, mask, cu, ref["batch_mean"] * 1.1)["exceeded"] == 0
    # learner == generator: exactly on-policy
    binding.npd_kd_loss_fwd_bwd(gen, mask, teacher_dense=gen.clone(), kd_tok=kl)
    same = _policy_lag_gpu(kl, mask, cu, 0.0)
    assert same["batch_mean"] == 0.0 and same["exceeded"] == 0 and (same["seg_mean"] == 0.0).all()
    # perplexity of the learner on every sample: exp of the per-sample mean NLL
    seg = _segment_gpu(nll, mask, cu, want_t2s=False)
    ppl = Guarded(S, torch.float32)
    binding.npd_segment_ppl(torch.from_numpy(seg["mean"].astype(np.float32)).to(dev()),
                            torch.from_numpy(seg["count"]).to(dev()), ppl.t)
    torch.cuda.synchronize()
    rseg = oracle.segment_reduce(ref_tok["nll_t"], lay.loss_mask, lay.cu_seqlens)
    rppl = oracle.perplexity(rseg["mean"], rseg["count"])
    got = ppl.check().cpu().numpy().astype(np.float64)
    assert (got[rseg["count"] == 0] == 0).all() and (rseg["count"] == 0).any()
    nz = rseg["count"] > 0
    np.testing.assert_allclose(got[nz], rppl[nz], rtol=1e-3)      # exp amplifies the 1e-4 bar of the mean by ~12
    assert rppl[nz].min() > 1e3                                    # random logits: perplexity of the order of V


def test_policy_lag_edge_cases():
    f32 = lambda a: torch.tensor(a, dtype=torch.float32, device=dev())
    u8 = lambda a: torch.tensor(a, dtype=torch.uint8, device=dev())
    i32 = lambda a: torch.tensor(a, dtype=torch.int32, device=dev())
    kl = f32([0.5, 0.25, 9.0, 0.125, 0.125, 7.0, 1.0, 3.0])
    mask = u8([1, 1, 0, 1, 1, 1, 1, 1])
    out = _policy_lag_gpu(kl, mask, i32([1, 3, 3, 5]), 0.10)       # position 0 and 5.. belong to no sample
    assert out["batch_count"] == 3 and out["batch_mean"] == float(np.float32(0.5) / np.float32(3)) and out["exceeded"] == 1
    np.testing.assert_array_equal(out["seg_count"], [1, 0, 2])
    np.testing.assert_array_equal(out["seg_mean"], np.float32([0.25, 0.0, 0.125]))
    assert _policy_lag_gpu(kl, mask, i32([3, 5]), 0.125)["exceeded"] == 0                   # the bound is closed
    assert _policy_lag_gpu(kl, u8([0] * 8), i32([0, 8]), 0.10) == dict(
        seg_mean=pytest.approx(np.zeros(1)), seg_count=pytest.approx(np.zeros(1)), batch_mean=0.0, batch_count=0,
        exceeded=0, status=0)
    bad = _policy_lag_gpu(kl, mask, i32([0, 6, 4, 8]), 0.10)       # decreasing boundaries
    assert bad["status"] == binding.NPD_DEV_BAD_CU_SEQLENS and np.isnan(bad["batch_mean"]) and bad["exceeded"] == 1
    assert bad["batch_count"] == 0
    nan = _policy_lag_gpu(f32([0.1, float("nan"), 0.1]), u8([1, 1, 1]), i32([0, 3]), 0.10)
    assert np.isnan(nan["batch_mean"]) and nan["exceeded"] == 1 and nan["status"] == 0


# --------------------------------------------------------------------------- teacher-side top-k record (Sec. 3.1)

def _topk_gpu(t, k, mask=None, log_probs=True):
    T = t.shape[0]
    idx, val = Guarded(T * k, torch.int32), Guarded(T * k, torch.float32)
    binding.npd_teacher_topk(t, k, topk_idx=idx.t.view(T, k), topk_val=val.t.view(T, k), loss_mask=mask,
                             log_probs=log_probs)
    torch.cuda.synchronize()
    return idx.check().view(T, k), val.check().view(T, k)


@pytest.mark.parametrize("V,stride,k,log_probs", [
    (151936, 151936, 64, True),      # config 2's record
    (151936, 151936, 10, False),     # the paper's default k, raw logits
    (151936, 151936, 1, True),       # arg-max
    (262144, 262144, 64, False),     # 32 groups per thread: the window is refilled twice
    (262144, 262144, 1024, True),    # as many entries as threads
    (40000, 40000, 2000, False),     # k beyond the per-thread-maximum bound: exact slow path
    (151936, 151936, 256, True),     # long candidate list: radix cut before the ordering
    (50001, 50008, 40, False),       # aligned rows with a ragged last group and V mod 8 elements at the end
    (9000, 9000, 7, True),           # two groups per thread only: shorter than the register window
    (5003, 5003, 33, True),          # unaligned rows: element-wise path
    (5003, 5008, 4096, False),       # the largest supported k on unaligned, strided rows
    (300, 300, 300, True),           # k = V: a full ordering of the row
])
def test_teacher_topk_shapes(oracle, V, stride, k, log_probs):
    T = 24 if V > 100000 else 40
    w = synth.scaled(synth.config(1), n_rows=1, row_len=T, vocab=V, length_lo=4, length_hi=16)
    _say(f"teacher top-k V={V} stride={stride} k={k} log_probs={log_probs}")
    lay, _, t, mask, _ = _inputs(w, stride)
    idx, val = _topk_gpu(t, k, mask, log_probs)
    ref = oracle.teacher_topk(_bits(t.contiguous()), k, lay.loss_mask, log_probs)
    np.testing.assert_array_equal(idx.cpu().numpy(), ref["idx"])                 # ids bit-exact, ties included
    np.testing.assert_allclose(val.cpu().numpy(), ref["val"], rtol=0, atol=2e-5 if log_probs else 0)


# k = 64 and 128 run with 512-thread workgroups, 129 and 200 with 1024-thread ones
@pytest.mark.parametrize("k", [64, 128, 129, 200])
def test_teacher_topk_ties_and_degenerate_rows(oracle, k):
    V = 151936
    t = (torch.randn((6, V), device=dev()) * 3).to(torch.bfloat16)
    t[0, :] = 1.5                                    # constant row: ids 0..k-1 (slow path: every element ties)
    t[1, 1000:9000] = 50.0                           # 8000 equal maxima: the 64 lowest ids among them
    t[2, :] = 0.0
    t[2, ::2] = -0.0                                 # +0 and -0 are equal values
    t[3, 7] = 30.0
    t[3, 100000:100000 + k - 1] = 30.0               # exactly k tied maxima, one far from the others
    t[4, -1] = 99.0                                  # the last element of the row
    idx, val = _topk_gpu(t, k, None, False)
    ref = oracle.teacher_topk(_bits(t), k, None, False)
    np.testing.assert_array_equal(idx.cpu().numpy(), ref["idx"])
    np.testing.assert_array_equal(val.cpu().numpy().astype(np.float64), ref["val"])
    assert idx[0].tolist() == list(range(k)) and idx[1].tolist() == list(range(1000, 1000 + k))
    assert idx[2].tolist() == list(range(k)) and idx[4, 0].item() == V - 1
    assert idx[3].tolist() == [7] + list(range(100000, 100000 + k - 1))


@pytest.mark.parametrize("k", [64, 200])
def test_teacher_topk_negative_rows_and_tie_runs(oracle, k):
    """Rows of log-probabilities (all negative), rows whose bound is zero, and tie runs at the cut that are
    longer than the short list but fit the candidate list (3000 ties: within the 4096 of the 1024-thread
    kernel, beyond the 2048 of the 512-thread one, which then takes the exact slow path; 1500 ties fit both)."""
    V = 151936
    g = torch.Generator(device="cpu").manual_seed(synth.SEED + 77)
    base = torch.randn((8, V), generator=g) * 3
    t = base.clone()
    t[0] = torch.log_softmax(base[0], dim=-1)                    # all negative
    t[1] = -torch.abs(base[1]) - 0.5                              # all negative, dense near the top
    t[2] = torch.where(base[2] > 0, torch.zeros(()), base[2])    # half the row is +0: the bound is zero
    t[2, 5::7] = -0.0
    t[3, 20000:23000] = 40.0                                      # 3000 equal maxima: a tie run at the cut
    t[4] = torch.where(base[4] > 6.0, base[4], torch.full((), -3.0e38))   # a handful of finite values
    t[4, :200] = 1.0
    t[6, 70000:71500] = 40.0                                      # 1500 equal maxima
    t[5] = -base[5].abs()
    t[5, 100] = 0.0                                               # a single +0 above negatives
    t = t.to(torch.bfloat16).to(dev())
    for log_probs in (False, True):
        idx, val = _topk_gpu(t, k, None, log_probs)
        ref = oracle.teacher_topk(_bits(t), k, None, log_probs)
        np.testing.assert_array_equal(idx.cpu().numpy(), ref["idx"])
        np.testing.assert_allclose(val.cpu().numpy(), ref["val"], rtol=0, atol=2e-5 if log_probs else 0)
    assert idx[3].tolist() == list(range(20000, 20000 + k)) and idx[6].tolist() == list(range(70000, 70000 + k))


def test_teacher_topk_feeds_the_kd_loss(oracle):
    """Phase 2 then Phase 3 on the device: extract the record, then distil against it."""
    w = synth.scaled(synth.config(2), n_rows=1, row_len=64, vocab=151936, length_lo=8, length_hi=32)
    lay, s, t, mask, labels = _inputs(w)
    k = 64
    idx, val = _topk_gpu(t, k, mask, True)
    gpu = run_gpu_kd(s, mask, idx=idx.contiguous(), val=val.contiguous(), labels=labels, tau=2.0)
    rec = oracle.teacher_topk(_bits(t), k, lay.loss_mask, True)
    ref = oracle.kd_topk(_bits(s), rec["idx"], rec["val"], lay.labels, lay.loss_mask, tau=2.0)
    assert gpu["status"] == 0
    compare_kd(gpu, ref, lay.loss_mask, lay.cu_seqlens, oracle, tau=2.0)


@pytest.mark.parametrize("k", [10, 64])
def test_cfg1_full_size_teacher_topk(oracle, k):
    """The top-k record of config 1's teacher logits at their real size (32,768 x 151,936; the launch that
    `bench.py --op teacher_topk` times): sampled rows bit-exact against the oracle's selection, every row through
    properties that hold at any size (ids in range and distinct, values in decreasing order, the selected values
    equal to the k largest of the row, not-scored rows as documented)."""
    w = synth.config(1)
    lay, _, t, mask, _ = _inputs(w)
    T, V = w.n_tokens, w.vocab
    _say(f"{w.name} full size teacher top-k, k={k}")
    idx, val = _topk_gpu(t, k, mask, log_probs=False)
    m = mask.bool()
    assert ((idx >= 0) & (idx < V)).all()
    assert (idx[~m] == torch.arange(k, device=dev(), dtype=torch.int32)).all() and (val[~m] == 0).all()
    srt = idx[m].sort(dim=1).values
    assert (srt[:, 1:] != srt[:, :-1]).all()                       # distinct ids
    assert (val[m][:, 1:] <= val[m][:, :-1]).all()                 # largest first
    rows_m = torch.nonzero(m).flatten()
    for r0 in range(0, rows_m.numel(), 2048):                      # the k largest values of every scored row
        rr = rows_m[r0:r0 + 2048]
        top = torch.topk(t[rr].float(), k, dim=1).values
        assert torch.equal(top, val[rr])
        assert torch.equal(torch.gather(t[rr].float(), 1, idx[rr].long()), val[rr])   # ids point at those values
    rows = _sample_rows(lay, 60, 17)
    ridx = torch.from_numpy(rows).to(dev())
    ref = oracle.teacher_topk(_bits(t[ridx]), k, lay.loss_mask[rows], False)
    np.testing.assert_array_equal(idx[ridx].cpu().numpy(), ref["idx"])
    np.testing.assert_array_equal(val[ridx].cpu().numpy().astype(np.float64), ref["val"])
    # the log-softmax form of the same record, sampled rows
    idx2, lp = _topk_gpu(t, k, mask, log_probs=True)
    assert torch.equal(idx2, idx)
    ref2 = oracle.teacher_topk(_bits(t[ridx]), k, lay.loss_mask[rows], True)
    np.testing.assert_allclose(lp[ridx].cpu().numpy(), ref2["val"], rtol=0, atol=2e-5)


# --------------------------------------------------------------------------- other divergences (Related Works)

DIVS = {"reverse": binding.NPD_DIV_REVERSE_KL, "skew": binding.NPD_DIV_SKEW_KL,
        "skew_reverse": binding.NPD_DIV_SKEW_REVERSE_KL}


@pytest.mark.parametrize("no_workspace", [False, True])
@pytest.mark.parametrize("div", sorted(DIVS))
@pytest.mark.parametrize("V,stride,tau,alpha,scale,inplace", [
    (1024, 1024, 1.0, 0.1, 1.0, False),        # one wave per row
    (5003, 5003, 2.0, 0.5, 1.0, False),        # unaligned rows: element-wise path
    (50264, 50272, 1.0, 0.1, 0.5, True),       # ragged last group, padded stride, in place
    (151936, 151936, 1.0, 0.1, 1.0, False),    # the headline vocabulary
    (151936, 151936, 3.0, 0.9, -2.0, True),
    (600000, 600000, 1.0, 0.3, 1.0, False),    # 74 groups per thread: most of the row streamed in every sweep
])
def test_divergence_shapes(oracle, div, V, stride, tau, alpha, scale, inplace, no_workspace):
    if no_workspace and V < 8 * 2292:
        pytest.skip("rows of one slice take the same kernel with and without a workspace")
    T = (12 if V > 500000 else 24) if V > 100000 else 64
    w = synth.scaled(synth.config(1), n_rows=1, row_len=T, vocab=V, length_lo=4, length_hi=16)
    _say(f"divergence {div} V={V} stride={stride} tau={tau} alpha={alpha} scale={scale} inplace={inplace}")
    lay, s, t, mask, labels = _inputs(w, stride)
    ref = oracle.div_dense(_bits(s), _bits(t), div, alpha, labels=lay.labels, mask=lay.loss_mask, tau=tau,
                           grad_scale=scale)
    nll = oracle.kd_dense(_bits(s), _bits(t), lay.labels, lay.loss_mask, want_grad=False)
    ref.update(nll_s=nll["nll_s"], nll_t=nll["nll_t"], lse_s=nll["lse_s"])
    gpu = run_gpu_kd(s, mask, t=t, labels=labels, tau=tau, grad_scale=scale, inplace=inplace, divergence=DIVS[div],
                     skew_alpha=alpha, no_workspace=no_workspace)
    assert gpu["status"] == 0
    compare_kd(gpu, ref, lay.loss_mask, lay.cu_seqlens, oracle, grad_scale=scale, tau=tau, amp_from_ref=True)


def test_divergence_forward_only_zero_at_equality_and_limits(oracle):
    w = synth.scaled(synth.config(1), n_rows=1, row_len=32, vocab=40000, length_lo=4, length_hi=16)
    lay, s, t, mask, labels = _inputs(w)
    for div, code in DIVS.items():
        ref = oracle.div_dense(_bits(s), _bits(t), div, 0.25, mask=lay.loss_mask, want_grad=False)
        gpu = run_gpu_kd(s, mask, t=t, want_grad=False, divergence=code, skew_alpha=0.25)
        compare_kd(gpu, ref, lay.loss_mask, lay.cu_seqlens, oracle)
        same = run_gpu_kd(s, mask, t=s.clone(), divergence=code, skew_alpha=0.25)
        assert np.abs(same["kd"]).max() <= 1e-5 and np.abs(same["grad"]).max() <= 1e-5
    # the reverse KL of a distribution with itself is exactly zero, and so is its gradient
    same = run_gpu_kd(s, mask, t=s.clone(), divergence=binding.NPD_DIV_REVERSE_KL)
    assert (same["kd"] == 0).all() and (same["grad_bits"] & 0x7fff == 0).all()
    # alpha = 0 takes the skew out: skew KL = Eq. 2, skew reverse KL = reverse KL
    fwd = oracle.kd_dense(_bits(s), _bits(t), mask=lay.loss_mask)
    gpu = run_gpu_kd(s, mask, t=t, divergence=binding.NPD_DIV_SKEW_KL, skew_alpha=0.0)
    compare_kd(gpu, dict(kd=fwd["kd"], grad=fwd["grad"]), lay.loss_mask, lay.cu_seqlens, oracle)


@pytest.mark.parametrize("div", sorted(DIVS))
@pytest.mark.parametrize("tau", [1.0, 2.0])
def test_divergence_composite_gradient_and_bad_label(oracle, div, tau):
    w = synth.scaled(synth.config(1), n_rows=1, row_len=24, vocab=32000, length_lo=4, length_hi=12)
    lay, s, t, mask, labels = _inputs(w)
    ref = oracle.div_dense(_bits(s), _bits(t), div, 0.1, labels=lay.labels, mask=lay.loss_mask, tau=tau,
                           grad_scale=0.9, ce_grad_scale=0.1)
    gpu = run_gpu_kd(s, mask, t=t, labels=labels, tau=tau, grad_scale=0.9, ce_grad_scale=0.1, divergence=DIVS[div],
                     skew_alpha=0.1)
    assert gpu["status"] == 0
    compare_kd(gpu, ref, lay.loss_mask, lay.cu_seqlens, oracle, grad_scale=0.9, tau=tau, amp_from_ref=True)
    bad = labels.clone()
    r = int(np.flatnonzero(lay.loss_mask)[0])
    bad[r] = w.vocab + 5
    gpu = run_gpu_kd(s, mask, t=t, labels=bad, tau=tau, ce_grad_scale=0.1, divergence=DIVS[div], skew_alpha=0.1)
    assert gpu["status"] == binding.NPD_DEV_BAD_LABEL
    assert np.isnan(gpu["grad"][r]).all() and np.isnan(gpu["nll_s"][r])
    others = lay.loss_mask.astype(bool).copy()
    others[r] = False
    assert np.isfinite(gpu["grad"][others]).all()


# --------------------------------------------------------------------------- stream capture

def test_whole_step_replays_from_a_hip_graph(oracle):
    """The library allocates nothing and never synchronises, so a whole step (fused loss + gradient, top-k record,
    the per-sample reductions, Delta-IFD) can be captured once and replayed: every replay, on new logits in the same
    buffers, must reproduce the eager results bit for bit."""
    w = synth.scaled(synth.config(1), n_rows=2, row_len=96, vocab=50264, length_lo=8, length_hi=48)
    lay, s, t, mask, labels = _inputs(w)
    T, V, S, k = w.n_tokens, w.vocab, lay.n_segments, 16
    cu = torch.from_numpy(lay.cu_seqlens).to(dev())
    real = np.flatnonzero(~lay.is_pad_segment).astype(np.int32)
    pc = torch.from_numpy(real[0::2][:len(real) // 2]).to(dev())
    pu = torch.from_numpy(real[1::2][:len(real) // 2]).to(dev())
    P = pc.numel()

    def buffers():
        return dict(g=torch.zeros_like(s), kd=torch.zeros(T, device=dev()), nll=torch.zeros(T, device=dev()),
                    tnll=torch.zeros(T, device=dev()), idx=torch.zeros((T, k), dtype=torch.int32, device=dev()),
                    val=torch.zeros((T, k), device=dev()), seg=torch.zeros(S, device=dev()),
                    cnt=torch.zeros(S, dtype=torch.int32, device=dev()), ms=torch.zeros(S, device=dev()),
                    mt=torch.zeros(S, device=dev()), delta=torch.zeros(P, device=dev()),
                    zone=torch.zeros(P, dtype=torch.uint8, device=dev()),
                    keep_count=torch.zeros(1, dtype=torch.int32, device=dev()),
                    status=torch.zeros(1, dtype=torch.int32, device=dev()))

    def step(b):
        binding.npd_kd_loss_fwd_bwd(s, mask, teacher_dense=t, labels=labels, grad_scale=0.9, ce_grad_scale=0.1,
                                    grad_out=b["g"], kd_tok=b["kd"], nll_tok=b["nll"], teacher_nll_tok=b["tnll"],
                                    dev_status=b["status"])
        binding.npd_teacher_topk(t, k, topk_idx=b["idx"], topk_val=b["val"], loss_mask=mask, log_probs=True)
        binding.npd_segment_reduce(b["kd"], mask, cu, seg_sum=b["seg"], seg_count=b["cnt"])
        binding.npd_segment_reduce(b["nll"], mask, cu, seg_mean=b["ms"])
        binding.npd_segment_reduce(b["tnll"], mask, cu, seg_mean=b["mt"])
        binding.npd_delta_ifd_score(b["ms"], b["mt"], b["cnt"], pc, pu, 0.0, 0.8, delta=b["delta"], zone=b["zone"],
                                    keep_count=b["keep_count"])

    captured = buffers()
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):
        step(captured)                                   # warm-up outside the capture
    torch.cuda.current_stream().wait_stream(side)
    torch.cuda.synchronize()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph):
        step(captured)
    for trial in range(3):
        synth.fill_logits(w, s, t, synth.SEED + 100 + trial)   # new logits in the same buffers, eager work in between
        eager = buffers()
        step(eager)
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        for name in eager:
            a, b = eager[name], captured[name]
            assert torch.equal(a.view(torch.uint8) if a.dtype != torch.bfloat16 else a.view(torch.int16),
                               b.view(torch.uint8) if b.dtype != torch.bfloat16 else b.view(torch.int16)), \
                f"replay {trial}: {name} differs from the eager run"
        assert int(captured["status"].item()) == 0
    ref = oracle.kd_dense(_bits(s), _bits(t), lay.labels, lay.loss_mask, grad_scale=0.9, ce_grad_scale=0.1)
    gpu = dict(kd=captured["kd"].cpu().numpy().astype(np.float64), nll_s=captured["nll"].cpu().numpy().astype(np.float64),
               grad=captured["g"].float().cpu().numpy().astype(np.float64))
    compare_kd(gpu, ref, lay.loss_mask, lay.cu_seqlens, oracle)


# --------------------------------------------------------------------------- shape-selection boundaries

@pytest.mark.parametrize("V", [
    8 * 1024, 8 * 1025,                 # first row-resident shape (256 threads, 4 groups) and one vector more
    8 * 13 * 256, 8 * 13 * 256 + 8,     # 13 full groups at 256 threads | a 14th group with one vector
    8 * 16 * 256 + 16, 8 * 19 * 256,    # 16 -> 19 unrolled groups | exactly 19
    8 * 5119, 8 * 5120, 8 * 5121,       # 256 -> 512 threads
    8 * 19 * 512, 8 * 19 * 512 + 8,     # exactly 19 groups at 512 threads | one streamed vector beyond
    8 * 13000, 8 * 13001,               # forward-only: 512 -> 1024 threads
    8 * 16384 + 8,                      # 512 -> 1024 threads with gradient (17 groups: 16 unrolled + streamed)
    8 * 18 * 1024 + 24,                 # 19 unrolled groups of 1024 threads, the last one nearly empty
    8 * 19 * 1024 + 8 + 3,              # one streamed vector and a 3-element tail beyond 19 groups
    1 << 20, 1000003,                   # rows of a million entries: 109 of 128 groups per thread streamed twice
])
def test_shape_selection_boundaries(oracle, V):
    w = synth.scaled(synth.config(1), n_rows=1, row_len=20, vocab=V, length_lo=4, length_hi=10)
    _say(f"boundary V={V}")
    lay, s, t, mask, labels = _inputs(w, V + (8 - V % 8) % 8)
    ref = oracle.kd_dense(_bits(s.contiguous()), _bits(t.contiguous()), lay.labels, lay.loss_mask)
    for no_workspace in (False, True):     # row-gang kernels where they apply | one workgroup per row
        gpu = run_gpu_kd(s, mask, t=t, labels=labels, no_workspace=no_workspace)
        assert gpu["status"] == 0
        compare_kd(gpu, ref, lay.loss_mask, lay.cu_seqlens, oracle)
    fwd = run_gpu_kd(s, mask, t=t, labels=labels, want_grad=False)
    compare_kd(fwd, dict(kd=ref["kd"], nll_s=ref["nll_s"], nll_t=ref["nll_t"], lse_s=ref["lse_s"]), lay.loss_mask,
               lay.cu_seqlens, oracle)
    idx, val = _topk_gpu(t, 8, mask, True)
    rk = oracle.teacher_topk(_bits(t.contiguous()), 8, lay.loss_mask, True)
    np.testing.assert_array_equal(idx.cpu().numpy(), rk["idx"])
    tk = run_gpu_kd(s, mask, idx=idx.contiguous(), val=val.contiguous(), labels=labels, tau=2.0)
    rt = oracle.kd_topk(_bits(s.contiguous()), rk["idx"], rk["val"], lay.labels, lay.loss_mask, tau=2.0)
    compare_kd(tk, rt, lay.loss_mask, lay.cu_seqlens, oracle, tau=2.0)


# --------------------------------------------------------------------------- seeded random shapes

def _random_case(i):
    """Case i of a fixed, seeded list: vocabulary, row padding, teacher kind, temperature, weights and modes drawn
    so that every kernel family, thread count and streamed / ragged / tail combination turns up somewhere."""
    rng = np.random.default_rng(9000 + i)
    V = int(np.exp(rng.uniform(np.log(200), np.log(300000))))
    if rng.random() < 0.6:
        V = max(8, V // 8 * 8)                                   # most vocabularies are multiples of 8
    aligned = rng.random() < 0.8
    stride = (V + 7) // 8 * 8 + 8 * int(rng.integers(0, 3)) if aligned else V + int(rng.integers(0, 2)) * 3 + (V % 2 == 0)
    kind = rng.choice(["dense", "dense", "topk", "none"])
    tau = float(rng.choice([0.5, 1.0, 1.0, 2.0, 3.7]))
    scale = float(rng.choice([1.0, 1.0, -0.5, 3.0]))
    fwd_only = kind == "none" or rng.random() < 0.2
    inplace = (not fwd_only) and rng.random() < 0.3
    ce = 0.1 if (not fwd_only and rng.random() < 0.3) else 0.0
    div = rng.choice(["forward", "forward", "reverse", "skew", "skew_reverse"]) if kind == "dense" else "forward"
    k = int(min(V, np.exp(rng.uniform(0, np.log(600))))) if kind == "topk" else 0
    return dict(V=V, stride=int(stride), kind=str(kind), tau=tau, scale=scale, fwd_only=bool(fwd_only),
                inplace=bool(inplace), ce=ce, div=str(div), k=max(1, k), alpha=float(rng.choice([0.1, 0.5, 0.9])))


@pytest.mark.parametrize("i", range(96))
def test_seeded_random_shapes(oracle, i):
    c = _random_case(i)
    V = c["V"]
    T = 10 if V > 100000 else 24
    w = synth.scaled(synth.config(1), n_rows=1, row_len=T, vocab=V, length_lo=3, length_hi=9, topk=c["k"])
    _say(f"random case {i}: {c}")
    lay, s, t, mask, labels = _inputs(w, c["stride"], dense_teacher=c["kind"] == "dense")
    sb = _bits(s.contiguous())
    tol = dict(grad_scale=c["scale"], tau=c["tau"], amp_from_ref=c["div"] != "forward" or c["ce"] != 0.0,
               folded=not (c["div"] == "forward" and (V < 8192 or c["stride"] % 8 != 0)))
    want_grad = not c["fwd_only"]
    if c["kind"] == "dense":
        tb = _bits(t.contiguous())
        if c["div"] == "forward":
            ref = oracle.kd_dense(sb, tb, lay.labels, lay.loss_mask, tau=c["tau"], grad_scale=c["scale"],
                                  ce_grad_scale=c["ce"], want_grad=want_grad)
        else:
            ref = oracle.div_dense(sb, tb, c["div"], c["alpha"], labels=lay.labels, mask=lay.loss_mask, tau=c["tau"],
                                   grad_scale=c["scale"], ce_grad_scale=c["ce"], want_grad=want_grad)
            nl = oracle.kd_dense(sb, tb, lay.labels, lay.loss_mask, want_grad=False)
            ref.update(nll_s=nl["nll_s"], nll_t=nl["nll_t"], lse_s=nl["lse_s"])
        gpu = run_gpu_kd(s.clone() if c["inplace"] else s, mask, t=t, labels=labels, tau=c["tau"],
                         grad_scale=c["scale"], ce_grad_scale=c["ce"], want_grad=want_grad, inplace=c["inplace"],
                         divergence=0 if c["div"] == "forward" else DIVS[c["div"]], skew_alpha=c["alpha"],
                         no_workspace=i % 2 == 1)   # odd cases: the kernels that need no workspace
    elif c["kind"] == "topk":
        idx, val = synth.make_topk_teacher(w, s)
        ref = oracle.kd_topk(sb, idx.cpu().numpy(), val.cpu().numpy(), lay.labels, lay.loss_mask, tau=c["tau"],
                             grad_scale=c["scale"], ce_grad_scale=c["ce"], want_grad=want_grad)
        assert ref["bad_index_rows"] == 0
        gpu = run_gpu_kd(s.clone() if c["inplace"] else s, mask, idx=idx, val=val, labels=labels, tau=c["tau"],
                         grad_scale=c["scale"], ce_grad_scale=c["ce"], want_grad=want_grad, inplace=c["inplace"],
                         no_workspace=i % 2 == 1)
    else:
        nl = oracle.nll(sb, lay.labels, lay.loss_mask)
        ref = dict(nll_s=nl["nll"], lse_s=nl["lse"])
        gpu = run_gpu_kd(s, mask, labels=labels, want_grad=False)
    assert gpu["status"] == 0
    if not want_grad:
        ref = {key: v for key, v in ref.items() if key != "grad"}
    compare_kd(gpu, ref, lay.loss_mask, lay.cu_seqlens, oracle, **tol)
    # the teacher-side record of the same logits (dense cases), k drawn like the top-k cases
    if c["kind"] == "dense":
        kk = int(min(V, 1 + (i * 37) % 300))
        idx, val = _topk_gpu(t, kk, mask, True)
        rk = oracle.teacher_topk(_bits(t.contiguous()), kk, lay.loss_mask, True)
        np.testing.assert_array_equal(idx.cpu().numpy(), rk["idx"])
        np.testing.assert_allclose(val.cpu().numpy(), rk["val"], rtol=0, atol=2e-5)


# --------------------------------------------------------------------------- non-finite inputs stay in their row

@pytest.mark.parametrize("V", [5003, 50264, 151936])
def test_non_finite_logits_poison_only_their_own_row(V):
    """Inputs are required to be finite; if they are not, the damage must stay in the offending position: every
    other row's outputs are bit-identical to a run on clean inputs."""
    w = synth.scaled(synth.config(1), n_rows=1, row_len=24, vocab=V, length_lo=4, length_hi=12)
    lay, s, t, mask, labels = _inputs(w)
    clean = run_gpu_kd(s, mask, t=t, labels=labels)
    scored = np.flatnonzero(lay.loss_mask)
    r_nan, r_inf = int(scored[1]), int(scored[3])
    s2, t2 = s.clone(), t.clone()
    s2[r_nan, V // 2] = float("nan")
    t2[r_inf, 17] = float("inf")
    dirty = run_gpu_kd(s2, mask, t=t2, labels=labels)
    others = np.ones(w.n_tokens, bool)
    others[[r_nan, r_inf]] = False
    for key in ("kd", "nll_s", "nll_t", "lse_s"):
        np.testing.assert_array_equal(dirty[key][others], clean[key][others])
    np.testing.assert_array_equal(dirty["grad_bits"][others], clean["grad_bits"][others])
    assert np.isnan(dirty["kd"][r_nan]) and np.isnan(dirty["nll_s"][r_nan]) and np.isnan(dirty["grad"][r_nan]).all()
    assert not np.isfinite(dirty["kd"][r_inf])
    assert dirty["status"] == 0          # not a bookkeeping error: nothing is flagged


@pytest.mark.parametrize("V", [5003, 50264, 151936])
def test_minus_infinity_marks_a_masked_vocabulary_entry(oracle, V):
    """A logit of -inf is a vocabulary entry of probability 0 (vocabulary padding, banned tokens).  In the teacher it
    contributes nothing to Eq. 2 and the gradient there is p_S; where the student is -inf too, the gradient is 0."""
    w = synth.scaled(synth.config(1), n_rows=1, row_len=24, vocab=V, length_lo=4, length_hi=12)
    lay, s, t, mask, labels = _inputs(w)
    t[:, V - 70:] = float("-inf")                 # padded tail of the teacher's vocabulary
    t[3, 100:200] = float("-inf")
    s[:, V - 6:] = float("-inf")                  # the last entries are masked in both
    labels = torch.clamp(labels, max=V - 100)     # labels stay on real entries
    lab = labels.cpu().numpy()
    ref = oracle.kd_dense(_bits(s), _bits(t), lab, lay.loss_mask)
    assert np.isfinite(ref["kd"]).all() and np.isfinite(ref["grad"]).all()
    gpu = run_gpu_kd(s, mask, t=t, labels=labels)
    assert gpu["status"] == 0
    compare_kd(gpu, ref, lay.loss_mask, lay.cu_seqlens, oracle)
    m = lay.loss_mask.astype(bool)
    assert (gpu["grad"][m][:, V - 6:] == 0).all()
    # top-k record of such a teacher, then the top-k loss against it
    idx, val = _topk_gpu(t, 16, mask, True)
    rk = oracle.teacher_topk(_bits(t), 16, lay.loss_mask, True)
    np.testing.assert_array_equal(idx.cpu().numpy(), rk["idx"])
    tk = run_gpu_kd(s, mask, idx=idx.contiguous(), val=val.contiguous(), labels=labels)
    rt = oracle.kd_topk(_bits(s), rk["idx"], rk["val"], lab, lay.loss_mask)
    compare_kd(tk, rt, lay.loss_mask, lay.cu_seqlens, oracle)
    # the skew forms: p_T = 0 terms vanish there too (the reverse forms are +inf by definition where p_T = 0 < p_S)
    for div in ("skew", "skew_reverse"):
        rd = oracle.div_dense(_bits(s), _bits(t), div, 0.1, mask=lay.loss_mask)
        assert np.isfinite(rd["kd"]).all() and np.isfinite(rd["grad"]).all()
        gd = run_gpu_kd(s, mask, t=t, divergence=DIVS[div], skew_alpha=0.1)
        compare_kd(gd, rd, lay.loss_mask, lay.cu_seqlens, oracle, amp_from_ref=True)
    # a vocabulary padded with -inf in both models: every divergence, the reverse KL included, is the one of the
    # real entries, and the gradient on the padding is 0
    t2 = t.clone()
    t2[3, 100:200] = 1.0
    s2 = s.clone()
    s2[:, V - 70:] = float("-inf")
    for div in ("reverse", "skew", "skew_reverse"):
        rd = oracle.div_dense(_bits(s2), _bits(t2), div, 0.1, mask=lay.loss_mask)
        assert np.isfinite(rd["kd"]).all() and np.isfinite(rd["grad"]).all()
        gd = run_gpu_kd(s2, mask, t=t2, divergence=DIVS[div], skew_alpha=0.1)
        compare_kd(gd, rd, lay.loss_mask, lay.cu_seqlens, oracle, amp_from_ref=True)
        assert (gd["grad"][m][:, V - 70:] == 0).all()
        fo = run_gpu_kd(s2, mask, t=t2, divergence=DIVS[div], skew_alpha=0.1, want_grad=False)
        compare_kd(fo, dict(kd=rd["kd"]), lay.loss_mask, lay.cu_seqlens, oracle)
    # a stored top-k value of -inf is an entry of probability 0 as well
    val2 = val.clone()
    val2[:, -1] = float("-inf")
    tk2 = run_gpu_kd(s, mask, idx=idx.contiguous(), val=val2.contiguous(), labels=labels)
    rt2 = oracle.kd_topk(_bits(s), rk["idx"], val2.cpu().numpy(), lab, lay.loss_mask)
    assert np.isfinite(rt2["kd"]).all()
    compare_kd(tk2, rt2, lay.loss_mask, lay.cu_seqlens, oracle)
