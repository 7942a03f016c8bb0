"""Seeded synthetic inputs shaped like the paper's workloads.

This module serves both the GPU library's tests/benchmark and the CPU oracle's
tests.  It holds none of the method's arithmetic: it only lays samples out in
packed rows (Alg. 1, "Sequence Packing", pack length L) and draws random logits,
labels and top-k teacher records.  The paper's models and datasets are not
available; these inputs stand in for the logits of a ~1B student and a larger
teacher over packed rows of student-generated responses.

Packed layout produced here (the paper does not fix a representation):
  * the batch is ``n_rows`` rows of ``row_len`` positions, flattened to T positions;
  * ``cu_seqlens`` (int32 [S+1], cu[0] = 0, non-decreasing, cu[S] = T) delimits the
    samples; the unused tail of a row is a segment of its own whose mask is all 0;
  * ``loss_mask`` (uint8 [T]) is 1 on the response positions that are scored;
  * ``labels`` (int32 [T]) is the token each position predicts (already shifted).
"""
from dataclasses import dataclass, field
from typing import List, Optional, Tuple

import numpy as np
import torch

SEED = 26050594
GEN_CHUNK_ROWS = 256  # logits are drawn per chunk of this many rows, each chunk from its own seed


@dataclass
class Workload:
    """One named configuration: sizes, value distributions and loss settings."""
    name: str
    n_rows: int
    row_len: int
    vocab: int
    tau: float = 1.0
    teacher: str = "dense"            # "dense" | "topk" | "none"
    topk: int = 0
    length_dist: str = "loguniform"   # "fixed" | "loguniform" | "uniform"
    length_lo: int = 64
    length_hi: int = 4096
    fixed_lengths: Tuple[int, ...] = ()
    prompt_frac: Tuple[float, float] = (0.10, 0.30)
    value_dist: str = "normal"        # "normal" | "student_t3"
    student_scale: float = 3.0
    teacher_mix: float = 0.8          # teacher = teacher_mix * student + teacher_noise * noise
    teacher_noise: float = 1.5
    paired: bool = False              # Delta-IFD layout: every sample twice (with / without instruction)
    prefix_lo: int = 64
    prefix_hi: int = 512
    inplace: bool = False
    seed_offset: int = 0

    @property
    def n_tokens(self) -> int:
        return self.n_rows * self.row_len


def config(i: int) -> Workload:
    """The five benchmark configurations, by index."""
    if i == 0:   # Tiny
        return Workload("cfg0_tiny", 1, 512, 1024, fixed_lengths=(37, 64, 90, 121), length_dist="fixed",
                        prompt_frac=(0.25, 0.25), student_scale=2.0, teacher_mix=1.0, teacher_noise=0.5,
                        seed_offset=0)
    if i == 1:   # 1B-student shape
        return Workload("cfg1_1b_dense", 4, 8192, 151936, seed_offset=1)
    if i == 2:   # sparse (top-k) teacher, same token layout as config 1
        return Workload("cfg2_topk64", 4, 8192, 151936, tau=2.0, teacher="topk", topk=64, seed_offset=1)
    if i == 3:   # Delta-IFD scoring pass
        return Workload("cfg3_delta_ifd", 2, 32768, 151936, teacher="dense", length_lo=128, length_hi=8192,
                        paired=True, seed_offset=3)
    if i == 4:   # many short segments, heavy tails, in-place gradient
        return Workload("cfg4_stress", 8, 8192, 262144, length_dist="uniform", length_lo=16, length_hi=256,
                        value_dist="student_t3", student_scale=4.0, teacher_mix=0.8, teacher_noise=2.0,
                        inplace=True, seed_offset=4)
    raise ValueError(f"no config {i}")


def scaled(w: Workload, *, n_rows=None, row_len=None, vocab=None, length_lo=None, length_hi=None,
           topk=None, name=None) -> Workload:
    """A reduced copy of a workload (same distributions, smaller sizes) for oracle-speed parity tests."""
    import dataclasses
    kw = {}
    for k, v in dict(n_rows=n_rows, row_len=row_len, vocab=vocab, length_lo=length_lo, length_hi=length_hi,
                     topk=topk, name=name).items():
        if v is not None:
            kw[k] = v
    return dataclasses.replace(w, **kw)


@dataclass
class Layout:
    n_tokens: int
    cu_seqlens: np.ndarray          # int32 [S+1]
    loss_mask: np.ndarray           # uint8 [T]
    labels: np.ndarray              # int32 [T]
    is_pad_segment: np.ndarray      # bool [S]
    pair_cond: np.ndarray = field(default_factory=lambda: np.zeros(0, np.int32))    # int32 [P]
    pair_uncond: np.ndarray = field(default_factory=lambda: np.zeros(0, np.int32))  # int32 [P]

    @property
    def n_segments(self) -> int:
        return int(self.cu_seqlens.shape[0] - 1)


def _draw_length(w: Workload, rng) -> int:
    if w.length_dist == "loguniform":
        return int(np.floor(np.exp(rng.uniform(np.log(w.length_lo), np.log(w.length_hi + 1)))))
    if w.length_dist == "uniform":
        return int(rng.integers(w.length_lo, w.length_hi + 1))
    raise ValueError(w.length_dist)


def make_layout(w: Workload, seed: int = SEED) -> Layout:
    """Greedy sequential packing: samples are drawn one by one and appended to the current row;
    the first one that does not fit closes the row (its tail becomes a masked pad segment) and is
    dropped, and drawing continues with the next row."""
    rng = np.random.default_rng(seed + w.seed_offset)
    T, L = w.n_tokens, w.row_len
    cu = [0]
    pad = []
    mask = np.zeros(T, np.uint8)
    labels = rng.integers(0, w.vocab, size=T, dtype=np.int64).astype(np.int32)
    pair_cond, pair_uncond = [], []

    def add_segment(start, length, n_masked_lead, is_pad=False):
        cu.append(start + length)
        pad.append(is_pad)
        if not is_pad:
            mask[start + n_masked_lead:start + length] = 1

    fixed = list(w.fixed_lengths)
    for row in range(w.n_rows):
        pos, end = row * L, (row + 1) * L
        while True:
            if w.length_dist == "fixed":
                if not fixed:
                    break
                n = fixed.pop(0)
            else:
                n = _draw_length(w, rng)
            frac = rng.uniform(w.prompt_frac[0], w.prompt_frac[1]) if w.prompt_frac[0] != w.prompt_frac[1] \
                else w.prompt_frac[0]
            if w.paired:
                # copy 1: instruction prefix + response (prefix masked); copy 2: the response alone
                q = int(rng.integers(w.prefix_lo, w.prefix_hi + 1))
                if pos + q + n + n > end:
                    break
                add_segment(pos, q + n, q)
                add_segment(pos + q + n, n, 0)
                # both copies predict the same response tokens
                labels[pos + q + n:pos + q + 2 * n] = labels[pos + q:pos + q + n]
                pair_cond.append(len(cu) - 3)
                pair_uncond.append(len(cu) - 2)
                pos += q + 2 * n
            else:
                if pos + n > end:
                    break
                add_segment(pos, n, int(np.floor(frac * n)))
                pos += n
        if pos < end:
            add_segment(pos, end - pos, 0, is_pad=True)
    return Layout(T, np.asarray(cu, np.int32), mask, labels, np.asarray(pad, bool),
                  np.asarray(pair_cond, np.int32), np.asarray(pair_uncond, np.int32))


def _chunk_generator(device, seed: int, tensor_id: int, chunk: int) -> torch.Generator:
    g = torch.Generator(device=device)
    g.manual_seed((seed * 1000003 + tensor_id * 7919 + chunk) % (2 ** 62))
    return g


def _draw(shape, dist: str, g: torch.Generator, device) -> torch.Tensor:
    z = torch.randn(shape, generator=g, device=device, dtype=torch.float32)
    if dist == "normal":
        return z
    if dist == "student_t3":   # N(0,1) / sqrt(chi2_3 / 3)
        chi2 = torch.zeros(shape, device=device, dtype=torch.float32)
        for _ in range(3):
            chi2 += torch.randn(shape, generator=g, device=device, dtype=torch.float32) ** 2
        return z / torch.sqrt(chi2 / 3.0)
    raise ValueError(dist)


def fill_logits(w: Workload, student: torch.Tensor, teacher: Optional[torch.Tensor], seed: int = SEED,
                label_boost: Optional[Tuple[torch.Tensor, torch.Tensor, torch.Tensor]] = None) -> None:
    """Fill bf16 ``student`` (and dense ``teacher``) [T, >=V] in place, chunk by chunk, on their device.

    student = student_scale * X;  teacher = teacher_mix * student(fp32) + teacher_noise * Y,  X, Y drawn from
    ``value_dist``; both rounded once to bf16.  ``label_boost`` = (labels, boost_student, boost_teacher),
    each [T] on the same device: adds the boost to the logit of the label token (used by the Delta-IFD
    layout so that the with-instruction copy predicts the response better than the response-only copy).
    """
    T, V = w.n_tokens, w.vocab
    dev = student.device
    for ci, r0 in enumerate(range(0, T, GEN_CHUNK_ROWS)):
        r1 = min(T, r0 + GEN_CHUNK_ROWS)
        g = _chunk_generator(dev, seed + w.seed_offset, 1, ci)
        s32 = w.student_scale * _draw((r1 - r0, V), w.value_dist, g, dev)
        t32 = None
        if teacher is not None:
            t32 = w.teacher_mix * s32 + w.teacher_noise * _draw((r1 - r0, V), w.value_dist, g, dev)
        if label_boost is not None:
            lab, bs, bt = label_boost
            rows = torch.arange(r1 - r0, device=dev)
            s32[rows, lab[r0:r1].long()] += bs[r0:r1]
            if t32 is not None:
                t32[rows, lab[r0:r1].long()] += bt[r0:r1]
        student[r0:r1, :V] = s32.to(torch.bfloat16)
        if teacher is not None:
            teacher[r0:r1, :V] = t32.to(torch.bfloat16)


def make_topk_teacher(w: Workload, student: torch.Tensor, seed: int = SEED,
                      zipf_a: float = 1.1) -> Tuple[torch.Tensor, torch.Tensor]:
    """Top-k teacher record: int32 indices [T, k] (unique per row) and fp32 log-probabilities [T, k].

    Values: p_j proportional to rank^-a (a Zipf-shaped head), normalised over the k entries, stored as
    log p_j in rank order.  Placement: for about half of the rows the student's own k largest logits in
    random order (teacher and student agree on the support), otherwise k distinct random tokens.
    """
    T, V, k = w.n_tokens, w.vocab, w.topk
    dev = student.device
    ranks = torch.arange(1, k + 1, device=dev, dtype=torch.float64)
    p = ranks ** (-zipf_a)
    logp = torch.log(p / p.sum()).to(torch.float32)
    idx = torch.empty((T, k), device=dev, dtype=torch.int32)
    for ci, r0 in enumerate(range(0, T, GEN_CHUNK_ROWS)):
        r1 = min(T, r0 + GEN_CHUNK_ROWS)
        n = r1 - r0
        g = _chunk_generator(dev, seed + w.seed_offset, 2, ci)
        top = torch.topk(student[r0:r1, :V].float(), k, dim=1).indices
        perm = torch.argsort(torch.rand((n, k), generator=g, device=dev), dim=1)
        agree = torch.gather(top, 1, perm)
        # k distinct random tokens: positions of the k smallest of V random keys would cost O(V); instead
        # draw with a stride trick: start + j * step (mod V) with step coprime to V is a set of k distinct ids
        start = torch.randint(0, V, (n, 1), generator=g, device=dev)
        step = 2 * torch.randint(0, max(1, (V - 1) // (2 * k)), (n, 1), generator=g, device=dev) + 1
        j = torch.arange(k, device=dev).unsqueeze(0)
        rand_ids = (start + j * step) % V          # distinct because j*step < V for all j < k
        use_agree = torch.rand((n, 1), generator=g, device=dev) < 0.5
        idx[r0:r1] = torch.where(use_agree, agree, rand_ids).to(torch.int32)
    return idx, logp.unsqueeze(0).expand(T, k).contiguous()


def delta_ifd_boosts(w: Workload, lay: Layout, seed: int = SEED) -> Tuple[np.ndarray, np.ndarray]:
    """Per-position label-logit boosts for the paired (Delta-IFD) layout: one level per sample copy and
    model, larger with the instruction than without, so that IFD values spread below and around 1."""
    rng = np.random.default_rng(seed + w.seed_offset + 17)
    bs = np.zeros(lay.n_tokens, np.float32)
    bt = np.zeros(lay.n_tokens, np.float32)
    cu = lay.cu_seqlens
    for pc, pu in zip(lay.pair_cond, lay.pair_uncond):
        base_s, base_t = rng.uniform(4.0, 10.0), rng.uniform(4.0, 10.0)
        gain_s, gain_t = rng.uniform(-1.0, 4.0), rng.uniform(-1.0, 6.0)
        bs[cu[pu]:cu[pu + 1]] = base_s
        bt[cu[pu]:cu[pu + 1]] = base_t
        bs[cu[pc]:cu[pc + 1]] = base_s + gain_s
        bt[cu[pc]:cu[pc + 1]] = base_t + gain_t
    return bs, bt


def bf16_bits(x: torch.Tensor) -> np.ndarray:
    """Raw bit patterns (uint16 numpy, host) of a bf16 tensor; this is what the oracle consumes."""
    assert x.dtype == torch.bfloat16
    return x.detach().cpu().contiguous().view(torch.int16).numpy().view(np.uint16)
