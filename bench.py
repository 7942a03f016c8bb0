"""Benchmark of the NPD packed KD-loss hot path on one MI355X.

A step is one pass of the whole hot path over one packed batch that is already resident in HBM:
the fused KD loss + gradient kernel (log-softmax, KL, NLLs, bf16 gradient), the per-sample reductions of the
KD loss and of the student / teacher NLLs over cu_seqlens, and the Delta-IFD score of the per-sample mean
NLLs.  Prints ONE JSON line.

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--config 1] [--no-cpu-baseline]

`--op teacher_topk [--topk K]` times the teacher-side top-k record of the same batch's teacher logits instead
(Alg. 1 Phase 2: not part of the student step, so not part of the headline line).
"""
import argparse
import ctypes
import json
import os
import sys
import time

import numpy as np
import torch

HBM_PEAK_GBS = 8000.0   # MI355X HBM3E, published peak

# HBM-side bytes per launch of the dominant kernel, counted by rocprofv3 (--pmc FETCH_SIZE, then WRITE_SIZE, each scaled by
# what the same counter reads for a plain copy of known size) in earlier runs of this very command: bench_hbm_traffic.json
# holds one record per workload with the kernel and the library version it was counted on.  `roofline.traffic` is printed
# only when both match what this run launches; otherwise null (the record says what it was measured on).
TRAFFIC_RECORD = os.path.join(os.path.dirname(os.path.abspath(__file__)), "bench_hbm_traffic.json")


def counted_traffic(workload, kernel, version):
    """(bytes per launch or None, provenance string) for `workload` as launched by `kernel` of library `version`."""
    try:
        with open(TRAFFIC_RECORD) as f:
            rec = json.load(f).get(workload)
    except (OSError, ValueError):
        return None, "no traffic record"
    if rec is None:
        return None, "no traffic record for this workload"
    src = f"{rec['profile']} ({rec['kernel']}, libnpd {rec['npd_version']})"
    if rec["kernel"] != kernel or rec["npd_version"] != version:
        return None, f"stale: counted on {src}; this run launches {kernel}, libnpd {version}"
    return int(1024 * (rec["fetch_kib"] * rec["fetch_scale"] + rec["write_kib"] * rec["write_scale"])), src


def algorithmic_bytes(w, lay):
    """Bytes the method must move per launch of the fused kernel: every scored row's logits once in and its
    gradient once out; a masked row only has its gradient row zero-filled."""
    V = w.vocab
    n_scored = int(lay.loss_mask.sum())
    n_masked = w.n_tokens - n_scored
    if w.paired:                       # scoring pass: student and teacher rows read once, nothing written
        return n_scored * 2 * (2 * V)
    if w.teacher == "topk":
        per_scored = 2 * V + 2 * V + w.topk * 8
    else:
        per_scored = 2 * (2 * V) + 2 * V
    return n_scored * per_scored + n_masked * 2 * V


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=50)
    ap.add_argument("--warmup", type=int, default=5)
    ap.add_argument("--config", type=int, default=1, help="workload index (1 = the 32,768 x 151,936 headline)")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--divergence", choices=("forward", "reverse", "skew", "skew_reverse"), default="forward",
                    help="divergence of the dense-teacher configurations (forward = Eq. 2, the headline)")
    ap.add_argument("--skew-alpha", type=float, default=0.1)
    ap.add_argument("--op", choices=("kd", "teacher_topk", "membench"), default="kd",
                    help="kd: the fused loss step (default); teacher_topk: the teacher-side top-k record; membench: "
                         "arithmetic-free streaming kernels over arrays of the workload's size (practical ceilings)")
    ap.add_argument("--topk", type=int, default=64, help="k of --op teacher_topk")
    ap.add_argument("--no-workspace", action="store_true",
                    help="set NPD_FLAG_NO_WORKSPACE: time the kernels that keep a whole row in one workgroup")
    ap.add_argument("--skip-all-scored", action="store_true",
                    help="do not add the few extra launches with every position scored (roofline.all_scored)")
    ap.add_argument("--all-scored", action="store_true",
                    help="score every position (no prompt or padding rows): the rate of a batch without write-only rows")
    ap.add_argument("--traffic-calibration", action="store_true",
                    help="also run a plain 2 GiB device-to-device copy (untimed), so that a rocprofv3 --pmc "
                         "FETCH_SIZE / WRITE_SIZE run holds a kernel of known traffic to scale the counters by")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build runs on exactly one GPU (the loss shards trivially by token rows; "
              "no multi-GPU path is part of it). Use --gpus 1.", file=sys.stderr)
        sys.exit(2)

    from paper_2605_05940_amd import binding, synth
    binding.load()
    dev = torch.device("cuda:0")
    torch.cuda.set_device(dev)
    if args.op == "teacher_topk":
        return bench_teacher_topk(args, binding, synth, dev)
    if args.op == "membench":
        return bench_memory_system(args, synth, dev)
    w = synth.config(args.config)
    lay = synth.make_layout(w)
    if args.all_scored:
        lay.loss_mask[:] = 1
    T, V, S = w.n_tokens, w.vocab, lay.n_segments

    s = torch.empty((T, V), dtype=torch.bfloat16, device=dev)
    dense = w.teacher == "dense"
    t = torch.empty((T, V), dtype=torch.bfloat16, device=dev) if dense else None
    labels = torch.from_numpy(lay.labels).to(dev)
    if w.paired:
        bs, bt = synth.delta_ifd_boosts(w, lay)
        synth.fill_logits(w, s, t, label_boost=(labels, torch.from_numpy(bs).to(dev), torch.from_numpy(bt).to(dev)))
    else:
        synth.fill_logits(w, s, t)
    idx = val = None
    if w.teacher == "topk":
        idx, val = synth.make_topk_teacher(w, s)
    mask = torch.from_numpy(lay.loss_mask).to(dev)
    cu = torch.from_numpy(lay.cu_seqlens).to(dev)
    if w.paired:
        pc, pu = torch.from_numpy(lay.pair_cond).to(dev), torch.from_numpy(lay.pair_uncond).to(dev)
    else:   # no instruction/response pairs in a training batch: score consecutive samples against each other
        real = np.flatnonzero(~lay.is_pad_segment).astype(np.int32)
        pc, pu = torch.from_numpy(real[0::2][:len(real) // 2]).to(dev), torch.from_numpy(real[1::2]).to(dev)
    P = pc.numel()

    pristine = s.clone() if w.inplace else None
    g = None if w.paired else (s if w.inplace else torch.empty_like(s))
    kd, nll, tnll = (torch.empty(T, device=dev) for _ in range(3))
    seg_sum, seg_mean, mean_s, mean_t = (torch.empty(S, device=dev) for _ in range(4))
    seg_cnt = torch.empty(S, dtype=torch.int32, device=dev)
    ifd_s, ifd_t, delta = (torch.empty(P, device=dev) for _ in range(3))
    zone, keep = (torch.empty(P, dtype=torch.uint8, device=dev) for _ in range(2))
    keep_count = torch.zeros(1, dtype=torch.int32, device=dev)
    status = torch.zeros(1, dtype=torch.int32, device=dev)

    kernel_events = []
    all_scored_events = []
    div_code = ("forward", "reverse", "skew", "skew_reverse").index(args.divergence)
    if div_code and not (dense and not w.paired):
        print("bench.py: --divergence applies to the dense-teacher training configurations", file=sys.stderr)
        sys.exit(2)

    def fused(record):
        if record:
            e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            e0.record()
        if w.paired:       # scoring pass: forward-only NLL of the student logits, then of the teacher logits
            binding.npd_kd_loss_fwd_bwd(s, mask, labels=labels, nll_tok=nll, dev_status=status,
                                        no_workspace=args.no_workspace)
            binding.npd_kd_loss_fwd_bwd(t, mask, labels=labels, nll_tok=tnll, dev_status=status,
                                        no_workspace=args.no_workspace)
        elif dense:
            binding.npd_kd_loss_fwd_bwd(s, mask, teacher_dense=t, labels=labels, tau=w.tau, grad_scale=1.0,
                                        divergence=div_code, skew_alpha=args.skew_alpha, no_workspace=args.no_workspace,
                                        grad_out=g, kd_tok=kd, nll_tok=nll, teacher_nll_tok=tnll, dev_status=status)
        else:
            binding.npd_kd_loss_fwd_bwd(s, mask, teacher_idx=idx, teacher_val=val, labels=labels, tau=w.tau,
                                        grad_scale=1.0, no_workspace=args.no_workspace, grad_out=g, kd_tok=kd,
                                        nll_tok=nll, dev_status=status)
        if record:
            e1.record()
            kernel_events.append((e0, e1))

    def step(record=False):
        if w.inplace:
            s.copy_(pristine)          # the in-place gradient destroys its input; restored outside the kernel timing
        fused(record)
        if not w.paired:
            binding.npd_segment_reduce(kd, mask, cu, seg_sum=seg_sum, seg_count=seg_cnt, seg_mean=seg_mean)
        binding.npd_segment_reduce(nll, mask, cu, seg_count=seg_cnt, seg_mean=mean_s)
        if dense:
            binding.npd_segment_reduce(tnll, mask, cu, seg_mean=mean_t)
            binding.npd_delta_ifd_score(mean_s, mean_t, seg_cnt, pc, pu, 0.0, 0.8, ifd_student=ifd_s,
                                        ifd_teacher=ifd_t, delta=delta, zone=zone, keep=keep, keep_count=keep_count)

    if args.traffic_calibration:
        src = torch.empty(2 << 30, dtype=torch.uint8, device=dev).fill_(1)
        dst = torch.empty_like(src)
        for _ in range(3):
            dst.copy_(src)         # reads 2 GiB, writes 2 GiB
        torch.cuda.synchronize()
        del src, dst

    for _ in range(args.warmup):
        step()
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(args.steps):
        step(record=True)
    torch.cuda.synchronize()
    elapsed = time.perf_counter() - t0
    assert status.item() == 0, f"device status {status.item()}"

    ms_per_step = 1e3 * elapsed / args.steps
    kernel_all = np.array([a.elapsed_time(b) for a, b in kernel_events])
    kernel_ms = float(kernel_all.mean())
    alg_bytes = algorithmic_bytes(w, lay)
    achieved = alg_bytes / (kernel_ms * 1e-3) / 1e9
    n_scored = int(lay.loss_mask.sum())
    version = binding.version()
    kernel_name = kd_kernel_name(binding, w, T, V, div_code, args.no_workspace)
    traffic, traffic_source = counted_traffic(w.name if div_code == 0 else f"{w.name}/{args.divergence}", kernel_name,
                                              version)
    # v_exp_f32 per student logit: one per tensor in the loss sweep, one per tensor in the gradient sweep
    exps_per_logit = 2 if w.paired else (4 if dense else 2)
    # keep the last timed step's outputs for the check against the oracle (the extra timing below overwrites them)
    last = dict(kd=kd.clone(), nll=nll.clone(), tnll=tnll.clone(), seg_sum=seg_sum.clone(), mean_s=mean_s.clone(),
                mean_t=mean_t.clone(), seg_cnt=seg_cnt.clone(), delta=delta.clone(), zone=zone.clone(),
                grad=None if g is None else g)

    # The same launch with every position scored (no prompt or padding rows, whose gradient rows are only zero-filled):
    # the rate of a batch that is all responses.  A few launches, outside the headline timing.
    all_scored = None
    if not w.paired and not args.all_scored and not args.skip_all_scored:
        keep_mask = mask.clone()
        mask.fill_(1)
        for i in range(2 + max(3, args.steps // 4)):
            if w.inplace:
                s.copy_(pristine)
            if i >= 2:
                e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
                e0.record()
            if dense:
                binding.npd_kd_loss_fwd_bwd(s, mask, teacher_dense=t, labels=labels, tau=w.tau, divergence=div_code,
                                            skew_alpha=args.skew_alpha, no_workspace=args.no_workspace, grad_out=g,
                                            kd_tok=kd, nll_tok=nll,
                                            teacher_nll_tok=tnll, dev_status=status)
            else:
                binding.npd_kd_loss_fwd_bwd(s, mask, teacher_idx=idx, teacher_val=val, labels=labels, tau=w.tau,
                                            no_workspace=args.no_workspace, grad_out=g, kd_tok=kd, nll_tok=nll,
                                            dev_status=status)
            if i >= 2:
                e1.record()
                all_scored_events.append((e0, e1))
        torch.cuda.synchronize()
        ms = float(np.mean([a.elapsed_time(b) for a, b in all_scored_events]))
        per_row = (2 * (2 * V) + 2 * V) if dense else (2 * V + 2 * V + w.topk * 8)
        all_scored = {"kernel_ms": ms, "achieved": T * per_row / (ms * 1e-3) / 1e9,
                      "frac": T * per_row / (ms * 1e-3) / 1e9 / HBM_PEAK_GBS,
                      "note": "same batch with every position scored (no write-only rows)"}
        mask.copy_(keep_mask)    # and the gradient of the timed workload again, for the check below
        if w.inplace:
            s.copy_(pristine)
        fused(False)
        torch.cuda.synchronize()

    out = {
        "metric": "kd_fwd_bwd_logit_tokens_per_sec", "value": T * args.steps / elapsed, "unit": "tokens/s",
        "n_gpus": 1, "steps": args.steps, "warmup": args.warmup, "ms_per_step": ms_per_step,
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None, "dtype": "f32",
        "data": "synthetic",
        "config": {"workload": f"{w.name}: {w.n_rows}x{w.row_len} tokens x vocab {V}, teacher {w.teacher}"
                               f"{'' if dense else ' k=' + str(w.topk)}, tau {w.tau}, "
                               f"{'in-place' if w.inplace else 'out-of-place'} bf16 grad"
                               f"{'' if div_code == 0 else ', divergence ' + args.divergence}",
                   "tokens": T, "scored_tokens": n_scored, "segments": S, "pairs": P,
                   "io_dtype": "bf16 logits and gradient, fp32 accumulation"},
        "roofline": {"bound": "hbm", "achieved": achieved, "peak": HBM_PEAK_GBS, "unit": "GB/s",
                     "frac": achieved / HBM_PEAK_GBS, "traffic": traffic, "traffic_source": traffic_source,
                     "kernel": f"npd::{kernel_name}", "npd_version": version,
                     "kernel_ms": kernel_ms,
                     "kernel_ms_median": float(np.median(kernel_all)), "kernel_ms_min": float(kernel_all.min()),
                     "algorithmic_bytes_per_launch": alg_bytes,
                     "counter_gbs": (traffic / (kernel_ms * 1e-3) / 1e9) if traffic else None,
                     "scored_tokens_per_sec": n_scored / (kernel_ms * 1e-3),
                     "exp_per_sec": n_scored * V * exps_per_logit / (kernel_ms * 1e-3),
                     "all_scored": all_scored},
        "context": "paper reports only a pipeline-level 8.1x train-time speed-up of NPD over DistiLLM-2 on "
                   "unnamed NPUs; not comparable to this kernel",
    }

    if not args.no_cpu_baseline:
        base, check = cpu_baseline_and_check(w, lay, s if pristine is None else pristine, t, idx, val, last,
                                             lay.cu_seqlens, args.divergence, args.skew_alpha)
        out["cpu_baseline"] = base
        out["verification"] = check
    print(json.dumps(out))


def bench_memory_system(args, synth, dev):
    """What the memory system gives each access mix of the KD kernels: arithmetic-free row-streaming kernels
    (``bench_membench/``) over three arrays the size of the workload's logits, every workgroup size
    with and without the non-temporal hint, plus the runtime's own fill and copy.  Context for `roofline.frac`."""
    import bench_membench as membench
    membench.load()
    w = synth.config(args.config)
    rows, groups = w.n_tokens, w.vocab // 8
    nbytes = rows * groups * 16
    a, b, o = (torch.empty(nbytes, dtype=torch.uint8, device=dev) for _ in range(3))
    a.fill_(1), b.fill_(2), o.zero_()

    def rate(fn, moved):
        for _ in range(max(1, min(args.warmup, 3))):
            fn()
        times = []
        for _ in range(args.steps):
            e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            e0.record()
            fn()
            e1.record()
            times.append((e0, e1))
        torch.cuda.synchronize()
        ms = float(np.mean([x.elapsed_time(y) for x, y in times]))
        return moved * nbytes / (ms * 1e-3) / 1e9

    patterns = {}
    for order in membench.ORDERS:
        for name in membench.PATTERNS:
            if name == "row_read_2_then_write_1" and order != "rows":
                continue
            moved = sum(membench.MOVES[name])
            variants = {}
            for threads in (256, 512, 1024):
                if name == "row_read_2_then_write_1" and groups > membench.ROW_GROUPS_PER_THREAD * threads:
                    continue           # the row does not fit this workgroup's registers
                for nt in (False, True):
                    key = f"{threads}{'_nt' if nt else ''}"
                    variants[key] = rate(lambda: membench.run(name, threads, nt, a, b, o, rows, groups, order=order),
                                         moved)
            if not variants:
                continue
            best = max(variants, key=variants.get)
            patterns[f"{name}/{order}"] = {"best_gbs": variants[best], "best_variant": best,
                                           "frac_of_peak": variants[best] / HBM_PEAK_GBS, "variants_gbs": variants}
    need = membench.gang_scratch_bytes(rows, groups)
    if need:
        scratch = torch.empty(need, dtype=torch.uint8, device=dev)
        gbs = rate(lambda: membench.run_gang(a, b, o, scratch, rows, groups), 3)
        patterns["gang_read_2_then_write_1/rows"] = {"best_gbs": gbs, "best_variant": "256_nt", "frac_of_peak": gbs / HBM_PEAK_GBS,
                                                     "variants_gbs": {"256_nt": gbs}}
        gbs = rate(lambda: membench.run_gang(a, b, o, scratch, rows, groups, reads=1), 2)
        patterns["gang_read_1_then_write_1/rows"] = {"best_gbs": gbs, "best_variant": "256_nt", "frac_of_peak": gbs / HBM_PEAK_GBS,
                                                     "variants_gbs": {"256_nt": gbs}}
    runtime = {"fill_gbs": rate(lambda: o.zero_(), 1), "copy_gbs": rate(lambda: o.copy_(a), 2)}
    print(json.dumps({
        "metric": "memory_system_stream_rate_2_reads_1_write",
        "value": max(patterns[p]["best_gbs"] for p in ("read_2_write_1/rows", "row_read_2_then_write_1/rows",
                                                       "gang_read_2_then_write_1/rows") if p in patterns),
        "unit": "GB/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup, "higher_is_better": True,
        "data": "synthetic", "dtype": "u8",
        "config": {"workload": f"three arrays of {rows} rows x {groups * 16} bytes ({w.name}'s logit tensors), 128-bit "
                               f"accesses; order rows = one workgroup per row (4 requests in flight per thread), "
                               f"address = one short-lived workgroup per consecutive run of groups; gang = a row shared by "
                               f"short-lived workgroups that exchange before they write; value = best 2-reads-1-write "
                               f"rate among the orders a row-reduction kernel can produce"},
        "peak_gbs": HBM_PEAK_GBS, "patterns": patterns, "runtime": runtime}))


def bench_teacher_topk(args, binding, synth, dev):
    """Top-k record (ids + log-softmax over the k) of every scored row of the workload's teacher logits."""
    from dataclasses import replace
    w = replace(synth.config(args.config), teacher="dense")
    lay = synth.make_layout(w)
    T, V, k = w.n_tokens, w.vocab, args.topk
    s = torch.empty((T, V), dtype=torch.bfloat16, device=dev)
    t = torch.empty((T, V), dtype=torch.bfloat16, device=dev)
    synth.fill_logits(w, s, t)
    del s
    mask = torch.from_numpy(lay.loss_mask).to(dev)
    idx = torch.empty((T, k), dtype=torch.int32, device=dev)
    val = torch.empty((T, k), dtype=torch.float32, device=dev)
    for _ in range(args.warmup):
        binding.npd_teacher_topk(t, k, topk_idx=idx, topk_val=val, loss_mask=mask, log_probs=True)
    torch.cuda.synchronize()
    events = []
    t0 = time.perf_counter()
    for _ in range(args.steps):
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record()
        binding.npd_teacher_topk(t, k, topk_idx=idx, topk_val=val, loss_mask=mask, log_probs=True)
        e1.record()
        events.append((e0, e1))
    torch.cuda.synchronize()
    elapsed = time.perf_counter() - t0
    kernel_ms = float(np.mean([a.elapsed_time(b) for a, b in events]))
    n_scored = int(lay.loss_mask.sum())
    alg_bytes = n_scored * (2 * V) + T * k * 8          # scored rows read once; every row's record written
    achieved = alg_bytes / (kernel_ms * 1e-3) / 1e9
    topk_traffic, topk_traffic_source = counted_traffic(f"{w.name}/teacher_topk_k{k}", "teacher_topk_stream_kernel",
                                                        binding.version())
    out = {
        "metric": "teacher_topk_tokens_per_sec", "value": T * args.steps / elapsed, "unit": "tokens/s",
        "n_gpus": 1, "steps": args.steps, "warmup": args.warmup, "ms_per_step": 1e3 * elapsed / args.steps,
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None, "dtype": "u16", "data": "synthetic",
        "config": {"workload": f"{w.name}: teacher logits {T} x {V} bf16, top-{k} ids + log-probs",
                   "tokens": T, "scored_tokens": n_scored},
        "roofline": {"bound": "hbm", "achieved": achieved, "peak": HBM_PEAK_GBS, "unit": "GB/s",
                     "frac": achieved / HBM_PEAK_GBS,
                     "traffic": topk_traffic, "traffic_source": topk_traffic_source,
                     "kernel": "npd::teacher_topk_stream_kernel", "npd_version": binding.version(),
                     "kernel_ms": kernel_ms,
                     "algorithmic_bytes_per_launch": alg_bytes},
    }
    if not args.no_cpu_baseline:
        from oracle import npd_oracle
        rows, spent = 0, 0.0
        while rows < T and spent < 10.0:
            r1 = min(rows + 256, T)
            tb = synth.bf16_bits(t[rows:r1])
            c0 = time.perf_counter()
            npd_oracle.teacher_topk(tb, k, lay.loss_mask[rows:r1], True)
            spent += time.perf_counter() - c0
            rows = r1
        out["cpu_baseline"] = {"value": rows / spent, "unit": "tokens/s", "cores": npd_oracle.threads(),
                               "kind": "oracle", "sample": f"first {rows} of {T} token rows, {spent:.1f} s"}
    print(json.dumps(out))


def kd_kernel_name(binding, w, T, V, div_code, no_workspace=False):
    """The kernel family a call of this workload takes (aligned, contiguous rows), as the library reports it."""
    d = binding.KdDesc()
    d.n_tokens, d.vocab, d.student_stride, d.teacher_stride = T, V, V, V
    d.teacher_kind = (binding.NPD_TEACHER_NONE if w.paired else
                      binding.NPD_TEACHER_DENSE_BF16 if w.teacher == "dense" else binding.NPD_TEACHER_TOPK)
    d.topk = w.topk if w.teacher == "topk" else 0
    d.flags = binding.NPD_FLAG_FWD_ONLY if w.paired else (binding.NPD_FLAG_INPLACE_GRAD if w.inplace else 0)
    if no_workspace:
        d.flags |= binding.NPD_FLAG_NO_WORKSPACE
    d.tau, d.grad_scale, d.divergence, d.skew_alpha = w.tau, 1.0, div_code, 0.1
    return binding.load().npd_kd_kernel_name(ctypes.byref(d)).decode()


def cpu_baseline_and_check(w, lay, s, t, idx, val, last, cu_host, divergence="forward", alpha=0.1, budget_s=15.0,
                           chunk=512, grad_chunks=4):
    """The float64 oracle, as it stands, on the first rows of the same batch, on this machine's host cores -- timed (the
    `cpu_baseline` object) and, since it computes them anyway, compared with what the last timed step left on the GPU
    (the `verification` object): per-sample sums of the per-position losses for every sample the oracle covered within
    its time budget, sample counts, and every gradient element of the first `grad_chunks` blocks of rows."""
    from paper_2605_05940_amd import synth
    from oracle import npd_oracle
    T = w.n_tokens
    rows, spent = 0, 0.0
    ref = {key: np.zeros(T) for key in ("kd", "nll_s", "nll_t")}
    grad_err, grad_rows = 0.0, 0
    while rows < T and spent < budget_s:
        r0, r1 = rows, min(rows + chunk, T)
        sb = synth.bf16_bits(s[r0:r1])
        lab, m = lay.labels[r0:r1], lay.loss_mask[r0:r1]
        if w.paired:
            tb = synth.bf16_bits(t[r0:r1])
            t0 = time.perf_counter()
            a = npd_oracle.nll(sb, lab, m)
            b = npd_oracle.nll(tb, lab, m)
            spent += time.perf_counter() - t0
            ref["nll_s"][r0:r1], ref["nll_t"][r0:r1] = a["nll"], b["nll"]
            o = None
        elif w.teacher == "dense":
            tb = synth.bf16_bits(t[r0:r1])
            t0 = time.perf_counter()
            if divergence == "forward":
                o = npd_oracle.kd_dense(sb, tb, lab, m, tau=w.tau)
            else:
                o = npd_oracle.kd_dense(sb, tb, lab, m, tau=w.tau, want_grad=False)
                o.update(npd_oracle.div_dense(sb, tb, divergence, alpha, mask=m, tau=w.tau))
            spent += time.perf_counter() - t0
            ref["kd"][r0:r1], ref["nll_s"][r0:r1], ref["nll_t"][r0:r1] = o["kd"], o["nll_s"], o["nll_t"]
        else:
            ib, vb = idx[r0:r1].cpu().numpy(), val[r0:r1].cpu().numpy()
            t0 = time.perf_counter()
            o = npd_oracle.kd_topk(sb, ib, vb, lab, m, tau=w.tau)
            spent += time.perf_counter() - t0
            ref["kd"][r0:r1], ref["nll_s"][r0:r1] = o["kd"], o["nll_s"]
        if o is not None and last["grad"] is not None and grad_rows < grad_chunks * chunk:
            got = last["grad"][r0:r1].float().cpu().numpy()
            grad_err = max(grad_err, float(np.abs(got - o["grad"]).max()))
            grad_rows += r1 - r0
        rows = r1
    base = {"value": rows / spent, "unit": "tokens/s", "cores": npd_oracle.threads(), "kind": "oracle",
            "sample": f"first {rows} of {T} token rows of the same batch (masked rows included), "
                      f"float64 C oracle with OpenMP, {spent:.1f} s of wall time"}

    # per-sample comparison over the samples that lie inside the rows the oracle covered
    cu = np.asarray(cu_host)
    covered = np.flatnonzero(cu[1:] <= rows)
    cu_cov = cu[:len(covered) + 1] if len(covered) else cu[:1]

    def rel_err(gpu_per_sample, key, mean):
        if len(covered) == 0:
            return None
        seg = npd_oracle.segment_reduce(ref[key][:rows], lay.loss_mask[:rows], cu_cov, want_token_to_sample=False)
        want = seg["mean"] if mean else seg["sum"]
        got = gpu_per_sample.cpu().numpy().astype(np.float64)[:len(covered)]
        nz = seg["count"] > 0
        return float((np.abs(got[nz] - want[nz]) / np.maximum(np.abs(want[nz]), 1e-30)).max()) if nz.any() else 0.0

    check = {"rows_checked": rows, "samples_checked": int(len(covered)),
             "max_rel_err_per_sample_kd": None if w.paired else rel_err(last["seg_sum"], "kd", False),
             "max_rel_err_per_sample_nll": rel_err(last["mean_s"], "nll_s", True),
             "max_rel_err_per_sample_teacher_nll": rel_err(last["mean_t"], "nll_t", True) if w.teacher == "dense" else None,
             "max_abs_err_grad": grad_err if grad_rows else None, "grad_rows_checked": grad_rows,
             "seg_count_mismatches": None, "tolerance": {"per_sample_rel": 1e-3, "grad_max_abs": 2e-3}}
    if len(covered):
        seg = npd_oracle.segment_reduce(ref["nll_s"][:rows], lay.loss_mask[:rows], cu_cov, want_token_to_sample=False)
        check["seg_count_mismatches"] = int((last["seg_cnt"].cpu().numpy()[:len(covered)] != seg["count"]).sum())
    errs = [check[k] for k in ("max_rel_err_per_sample_kd", "max_rel_err_per_sample_nll",
                               "max_rel_err_per_sample_teacher_nll") if check[k] is not None]
    check["ok"] = bool(all(e <= 1e-3 for e in errs) and (check["max_abs_err_grad"] is None or
                                                          check["max_abs_err_grad"] <= 2e-3)
                       and not check["seg_count_mismatches"])
    return base, check


if __name__ == "__main__":
    main()
