"""Pins for the float64 oracle: each check ties it to something other than itself --
closed forms, float64 library routines, finite differences, brute force, hand-worked cases.
No GPU is needed (run with -m "not gpu")."""
import math
import os

import numpy as np
import pytest
import torch
import torch.nn.functional as F

HERE = os.path.dirname(os.path.abspath(__file__))
RNG = np.random.default_rng(1234)


def _rand(T, V, scale=2.0, rng=RNG):
    return rng.normal(0.0, scale, size=(T, V))


# --------------------------------------------------------------------------- log-sum-exp / NLL

def test_lse_uniform_row_is_logit_plus_ln_V(oracle):
    for V in (1024, 151936, 262144):
        s = np.full((1, V), 0.75)
        out = oracle.nll(s, labels=np.array([V - 1]))
        assert out["lse"][0] == pytest.approx(0.75 + math.log(V), rel=0, abs=1e-12)
        assert out["nll"][0] == pytest.approx(math.log(V), rel=0, abs=1e-12)
    # the three printed constants
    assert math.log(151936) == pytest.approx(11.931214658, abs=1e-8)


def test_lse_shift_invariance_and_library(oracle):
    s = _rand(7, 333, 5.0)
    lab = RNG.integers(0, 333, 7)
    a = oracle.nll(s, lab)
    b = oracle.nll(s + 123.5, lab)
    np.testing.assert_allclose(a["nll"], b["nll"], atol=1e-11)
    np.testing.assert_allclose(a["lse"] + 123.5, b["lse"], atol=1e-11)
    ts = torch.from_numpy(s)
    np.testing.assert_allclose(a["lse"], torch.logsumexp(ts, 1).numpy(), atol=1e-12)
    np.testing.assert_allclose(a["nll"], F.cross_entropy(ts, torch.from_numpy(lab), reduction="none").numpy(),
                               atol=1e-12)


def test_lse_survives_huge_logits(oracle):
    s = np.array([[5000.0, 4999.0, -5000.0]])
    out = oracle.nll(s, np.array([1]))
    assert out["lse"][0] == pytest.approx(5000.0 + math.log1p(math.exp(-1.0)), abs=1e-9)
    assert out["nll"][0] == pytest.approx(1.0 + math.log1p(math.exp(-1.0)), abs=1e-9)


def test_nll_uses_label_and_tau_free(oracle):
    # NLL is the tau = 1 cross-entropy whatever the KD temperature
    s, t = _rand(5, 50), _rand(5, 50)
    lab = RNG.integers(0, 50, 5)
    o1 = oracle.kd_dense(s, t, lab, tau=1.0)
    o2 = oracle.kd_dense(s, t, lab, tau=3.0)
    np.testing.assert_array_equal(o1["nll_s"], o2["nll_s"])
    np.testing.assert_array_equal(o1["nll_t"], o2["nll_t"])
    ref_s = -torch.log_softmax(torch.from_numpy(s), 1)[torch.arange(5), torch.from_numpy(lab)]
    ref_t = -torch.log_softmax(torch.from_numpy(t), 1)[torch.arange(5), torch.from_numpy(lab)]
    np.testing.assert_allclose(o1["nll_s"], ref_s.numpy(), atol=1e-12)
    np.testing.assert_allclose(o1["nll_t"], ref_t.numpy(), atol=1e-12)
    np.testing.assert_allclose(o1["lse_s"], torch.logsumexp(torch.from_numpy(s), 1).numpy(), atol=1e-12)


def test_nll_bad_label_is_nan(oracle):
    s = _rand(2, 10)
    out = oracle.nll(s, np.array([10, -1]))
    assert np.isnan(out["nll"]).all()


# --------------------------------------------------------------------------- dense KL (Eq. 2 with support = V)

def test_kl_nonnegative_and_zero_iff_equal(oracle):
    s, t = _rand(64, 257, 3.0), _rand(64, 257, 3.0)
    for tau in (1.0, 2.0, 0.5):
        out = oracle.kd_dense(s, t, tau=tau)
        assert (out["kd"] > 0).all()
        same = oracle.kd_dense(s, s.copy(), tau=tau)
        assert (same["kd"] == 0.0).all()          # exactly zero
        assert (same["grad"] == 0.0).all()


def test_kl_two_level_closed_form(oracle):
    # student logits (beta, 0, ..., 0), teacher (alpha, 0, ..., 0): KL collapses to a binary KL
    V, alpha, beta = 1000, 3.0, 1.0
    s = np.zeros((1, V)); s[0, 0] = beta
    t = np.zeros((1, V)); t[0, 0] = alpha
    pt = math.exp(alpha) / (math.exp(alpha) + V - 1)
    ps = math.exp(beta) / (math.exp(beta) + V - 1)
    want = pt * math.log(pt / ps) + (1 - pt) * math.log((1 - pt) / (1 - ps))
    got = oracle.kd_dense(s, t)["kd"][0]
    assert got == pytest.approx(want, rel=1e-12)
    # the direction is KL(teacher || student): swapping the roles gives the other binary KL
    want_rev = ps * math.log(ps / pt) + (1 - ps) * math.log((1 - ps) / (1 - pt))
    assert oracle.kd_dense(t, s)["kd"][0] == pytest.approx(want_rev, rel=1e-12)
    assert abs(want - want_rev) > 1e-3


def test_kl_temperature_identity_and_no_tau_squared(oracle):
    s, t = _rand(9, 120, 4.0), _rand(9, 120, 4.0)
    tau = 2.5
    a = oracle.kd_dense(s, t, tau=tau)
    b = oracle.kd_dense(s / tau, t / tau, tau=1.0)
    np.testing.assert_allclose(a["kd"], b["kd"], rtol=1e-12)
    # d/ds at temperature tau = (1/tau) * d/d(s/tau) at temperature 1
    np.testing.assert_allclose(a["grad"], b["grad"] / tau, rtol=1e-10, atol=1e-15)


def test_kl_matches_library_kl_div(oracle):
    s, t = _rand(11, 77, 3.0), _rand(11, 77, 3.0)
    for tau in (1.0, 2.0):
        ls = torch.log_softmax(torch.from_numpy(s) / tau, 1)
        lt = torch.log_softmax(torch.from_numpy(t) / tau, 1)
        ref = F.kl_div(ls, lt, reduction="none", log_target=True).sum(1)
        np.testing.assert_allclose(oracle.kd_dense(s, t, tau=tau)["kd"], ref.numpy(), rtol=1e-11)


# --------------------------------------------------------------------------- top-k KL (Eq. 2)

def test_topk_uniform_closed_form(oracle):
    # uniform student, k equal teacher entries: KL = ln(V / k)
    for V, k in ((151936, 64), (1024, 10)):
        s = np.zeros((1, V))
        idx = (np.arange(k, dtype=np.int32) * 7 + 3).reshape(1, k)
        val = np.full((1, k), -2.0)
        out = oracle.kd_topk(s, idx, val, want_grad=False)
        assert out["kd"][0] == pytest.approx(math.log(V / k), rel=1e-12)
    assert math.log(151936 / 64) == pytest.approx(7.772331575, abs=1e-8)


def test_topk_with_k_equal_V_is_dense(oracle):
    V = 40
    s, t = _rand(6, V), _rand(6, V)
    idx = np.tile(np.arange(V, dtype=np.int32), (6, 1))
    for tau in (1.0, 2.0):
        d = oracle.kd_dense(s, t, tau=tau, grad_scale=0.7)
        k = oracle.kd_topk(s, idx, t, tau=tau, grad_scale=0.7)
        np.testing.assert_allclose(k["kd"], d["kd"], rtol=1e-12)
        np.testing.assert_allclose(k["grad"], d["grad"], rtol=1e-10, atol=1e-15)


def test_topk_permutation_and_shift_invariance(oracle):
    T, V, k = 5, 300, 16
    s = _rand(T, V, 3.0)
    idx = np.stack([RNG.choice(V, k, replace=False) for _ in range(T)]).astype(np.int32)
    val = _rand(T, k, 2.0)
    base = oracle.kd_topk(s, idx, val, tau=2.0)
    perm = RNG.permutation(k)
    p = oracle.kd_topk(s, idx[:, perm], val[:, perm], tau=2.0)
    np.testing.assert_allclose(p["kd"], base["kd"], rtol=1e-12)
    np.testing.assert_allclose(p["grad"], base["grad"], rtol=1e-10, atol=1e-15)
    sh = oracle.kd_topk(s, idx, val + 11.0, tau=2.0)      # stored logits vs stored log-probabilities
    np.testing.assert_allclose(sh["kd"], base["kd"], rtol=1e-11)


def test_topk_brute_force_tiny(oracle):
    # Eq. 2 written out with python floats: p_T renormalised over the k entries, p_S over the full vocabulary
    V, k, tau = 12, 3, 2.0
    s = _rand(1, V, 2.0)
    idx = np.array([[7, 2, 9]], np.int32)
    val = np.array([[0.3, -1.2, 0.9]])
    zs = sum(math.exp(x / tau) for x in s[0])
    zt = sum(math.exp(v / tau) for v in val[0])
    kl = 0.0
    for j in range(k):
        pt = math.exp(val[0, j] / tau) / zt
        ps = math.exp(s[0, idx[0, j]] / tau) / zs
        kl += pt * math.log(pt / ps)
    out = oracle.kd_topk(s, idx, val, tau=tau, grad_scale=1.0)
    assert out["kd"][0] == pytest.approx(kl, rel=1e-12)
    g = np.array([math.exp(x / tau) / zs for x in s[0]]) / tau
    for j in range(k):
        g[idx[0, j]] -= math.exp(val[0, j] / tau) / zt / tau
    np.testing.assert_allclose(out["grad"][0], g, rtol=1e-11, atol=1e-15)
    # support smaller than V: KL stays >= 0 and is > KL of the renormalised student on the support
    assert out["kd"][0] > 0


def test_topk_bad_index_flagged(oracle):
    s = _rand(2, 10)
    idx = np.array([[1, 2], [3, 10]], np.int32)
    out = oracle.kd_topk(s, idx, np.zeros((2, 2)))
    assert out["bad_index_rows"] == 1 and np.isnan(out["kd"][1]) and np.isfinite(out["kd"][0])


# --------------------------------------------------------------------------- gradient

@pytest.mark.parametrize("tau", [1.0, 2.0])
def test_grad_dense_finite_differences(oracle, tau):
    T, V, h = 3, 48, 1e-6
    s, t = _rand(T, V), _rand(T, V)
    g = oracle.kd_dense(s, t, tau=tau, grad_scale=1.0)["grad"]
    for r in range(T):
        for c in range(V):
            sp, sm = s.copy(), s.copy()
            sp[r, c] += h
            sm[r, c] -= h
            fd = (oracle.kd_dense(sp, t, tau=tau, want_grad=False)["kd"][r]
                  - oracle.kd_dense(sm, t, tau=tau, want_grad=False)["kd"][r]) / (2 * h)
            assert g[r, c] == pytest.approx(fd, rel=2e-6, abs=1e-9)


@pytest.mark.parametrize("tau", [1.0, 2.0])
def test_grad_topk_finite_differences(oracle, tau):
    T, V, k, h = 2, 40, 5, 1e-6
    s = _rand(T, V)
    idx = np.stack([RNG.choice(V, k, replace=False) for _ in range(T)]).astype(np.int32)
    val = _rand(T, k)
    g = oracle.kd_topk(s, idx, val, tau=tau)["grad"]
    for r in range(T):
        for c in range(V):
            sp, sm = s.copy(), s.copy()
            sp[r, c] += h
            sm[r, c] -= h
            fd = (oracle.kd_topk(sp, idx, val, tau=tau, want_grad=False)["kd"][r]
                  - oracle.kd_topk(sm, idx, val, tau=tau, want_grad=False)["kd"][r]) / (2 * h)
            assert g[r, c] == pytest.approx(fd, rel=2e-6, abs=1e-9)


def test_grad_rows_sum_to_zero_and_match_softmax_difference(oracle):
    T, V = 8, 2000
    s, t = _rand(T, V, 3.0), _rand(T, V, 3.0)
    for tau, scale in ((1.0, 1.0), (2.0, -0.3)):
        g = oracle.kd_dense(s, t, tau=tau, grad_scale=scale)["grad"]
        assert np.abs(g.sum(1)).max() < 1e-12 * V
        ref = scale / tau * (torch.softmax(torch.from_numpy(s) / tau, 1) - torch.softmax(torch.from_numpy(t) / tau, 1))
        np.testing.assert_allclose(g, ref.numpy(), rtol=1e-10, atol=1e-16)
    idx = np.stack([RNG.choice(V, 64, replace=False) for _ in range(T)]).astype(np.int32)
    g = oracle.kd_topk(s, idx, _rand(T, 64), tau=2.0)["grad"]
    assert np.abs(g.sum(1)).max() < 1e-12 * V


def test_masked_rows_are_zero(oracle):
    T, V = 6, 30
    s, t = _rand(T, V), _rand(T, V)
    mask = np.array([1, 0, 1, 0, 0, 1], np.uint8)
    lab = RNG.integers(0, V, T)
    out = oracle.kd_dense(s, t, lab, mask)
    for key in ("kd", "nll_s", "nll_t", "lse_s"):
        assert (out[key][mask == 0] == 0).all() and (out[key][mask == 1] != 0).all()
    assert (out["grad"][mask == 0] == 0).all()
    full = oracle.kd_dense(s, t, lab)
    np.testing.assert_array_equal(out["kd"][mask == 1], full["kd"][mask == 1])


# --------------------------------------------------------------------------- bf16 front-ends

def test_bf16_entry_points_equal_f64_entry_points_on_converted_values(oracle):
    T, V, k = 5, 130, 8
    sb = torch.from_numpy(_rand(T, V + 6, 3.0)).to(torch.bfloat16)     # row stride V + 6
    tb = torch.from_numpy(_rand(T, V, 3.0)).to(torch.bfloat16)
    s_bits = sb.view(torch.int16).numpy().view(np.uint16)[:, :V]
    t_bits = tb.view(torch.int16).numpy().view(np.uint16)
    s64, t64 = sb[:, :V].double().numpy(), tb.double().numpy()         # library conversion bf16 -> f64
    lab = RNG.integers(0, V, T)
    mask = np.array([1, 1, 0, 1, 1], np.uint8)
    a = oracle.kd_dense(s_bits, t_bits, lab, mask, tau=2.0, grad_scale=0.5)
    b = oracle.kd_dense(s64, t64, lab, mask, tau=2.0, grad_scale=0.5)
    for key in a:
        np.testing.assert_array_equal(a[key], b[key])
    idx = np.stack([RNG.choice(V, k, replace=False) for _ in range(T)]).astype(np.int32)
    val = _rand(T, k).astype(np.float32)
    a = oracle.kd_topk(s_bits, idx, val, lab, mask, tau=2.0)
    b = oracle.kd_topk(s64, idx, val.astype(np.float64), lab, mask, tau=2.0)
    for key in ("kd", "nll_s", "lse_s", "grad"):
        np.testing.assert_array_equal(a[key], b[key])
    a = oracle.nll(t_bits, lab, mask)
    b = oracle.nll(t64, lab, mask)
    np.testing.assert_array_equal(a["nll"], b["nll"])


# --------------------------------------------------------------------------- segment reduce / packing invariance

def _brute_segments(x, mask, cu):
    S = len(cu) - 1
    sums, counts, t2s = [0.0] * S, [0] * S, [-1] * len(x)
    for i in range(S):
        for p in range(cu[i], cu[i + 1]):
            t2s[p] = i
            if mask[p]:
                sums[i] += float(x[p])
                counts[i] += 1
    return sums, counts, t2s


def test_segment_reduce_brute_force_and_edge_cases(oracle):
    T = 100
    x = RNG.normal(size=T)
    mask = (RNG.random(T) < 0.6).astype(np.uint8)
    cu = np.array([0, 0, 1, 1, 8, 9, 40, 40, 77, 93], np.int32)   # empty, length-1, tokens 93.. unowned
    mask[9:40] = 0                                                # an all-masked sample
    out = oracle.segment_reduce(x, mask, cu)
    sums, counts, t2s = _brute_segments(x, mask, cu)
    np.testing.assert_array_equal(out["count"], counts)
    np.testing.assert_array_equal(out["token_to_sample"], t2s)
    np.testing.assert_allclose(out["sum"], sums, rtol=0, atol=1e-13)
    for i in range(len(cu) - 1):
        want = sums[i] / counts[i] if counts[i] else 0.0
        assert out["mean"][i] == pytest.approx(want, abs=1e-13)
    assert out["count"][5] == 0 and out["mean"][5] == 0.0 and out["sum"][5] == 0.0
    assert (out["token_to_sample"][93:] == -1).all()
    with pytest.raises(ValueError):
        oracle.segment_reduce(x, mask, np.array([0, 5, 3], np.int32))
    with pytest.raises(ValueError):
        oracle.segment_reduce(x, mask, np.array([0, 5, 101], np.int32))
    # every start alignment 0..7, S = 1
    for a in range(8):
        o = oracle.segment_reduce(x, np.ones(T, np.uint8), np.array([a, a + 13], np.int32))
        assert o["sum"][0] == pytest.approx(float(np.sum(x[a:a + 13])), abs=1e-13) and o["count"][0] == 13


def test_packing_invariance(oracle):
    # a packed batch gives, position by position, what each sample gives on its own
    from paper_2605_05940_amd import synth
    w = synth.config(0)
    lay = synth.make_layout(w)
    assert lay.cu_seqlens.tolist() == [0, 37, 101, 191, 312, 512]
    assert int(lay.loss_mask.sum()) == 28 + 48 + 68 + 91
    V = 96
    s, t = _rand(512, V), _rand(512, V)
    lab = lay.labels % V
    packed = oracle.kd_dense(s, t, lab, lay.loss_mask, tau=2.0)
    seg = oracle.segment_reduce(packed["kd"], lay.loss_mask, lay.cu_seqlens)
    for i in range(lay.n_segments):
        a, b = lay.cu_seqlens[i], lay.cu_seqlens[i + 1]
        alone = oracle.kd_dense(s[a:b], t[a:b], lab[a:b], lay.loss_mask[a:b], tau=2.0)
        for key in ("kd", "nll_s", "nll_t", "grad"):
            np.testing.assert_array_equal(alone[key], packed[key][a:b])
        one = oracle.segment_reduce(alone["kd"], lay.loss_mask[a:b], np.array([0, b - a], np.int32))
        assert one["sum"][0] == seg["sum"][i] and one["count"][0] == seg["count"][i]
        assert one["mean"][0] == seg["mean"][i]
    assert seg["count"].tolist() == [28, 48, 68, 91, 0]


# --------------------------------------------------------------------------- policy latency, perplexity (appendix)

def test_perplexity_of_a_uniform_model_is_the_vocabulary_size(oracle):
    # uniform next-token distribution over V entries: CE loss ln V at every position, so PPL = V exactly
    for V in (2, 1024, 151936):
        s = np.full((9, V), -3.25)
        lab = RNG.integers(0, V, 9)
        mask = np.array([1, 1, 0, 1, 1, 1, 0, 0, 1], np.uint8)
        cu = np.array([0, 4, 4, 9], np.int32)                       # a sample of 3 scored, an empty one, one of 3
        nl = oracle.nll(s, lab, mask)
        seg = oracle.segment_reduce(nl["nll"], mask, cu)
        ppl = oracle.perplexity(seg["mean"], seg["count"])
        assert ppl[0] == pytest.approx(V, rel=1e-12) and ppl[2] == pytest.approx(V, rel=1e-12)
        assert ppl[1] == 0.0 and seg["count"].tolist() == [3, 0, 3]


def test_perplexity_is_the_geometric_mean_of_inverse_token_probabilities(oracle):
    # PPL = (prod_t 1 / p(y_t))^(1/n), written with the library softmax and python floats
    V, T = 37, 11
    s = _rand(T, V, 3.0)
    lab = RNG.integers(0, V, T)
    mask = np.ones(T, np.uint8)
    mask[[2, 7]] = 0
    p = torch.softmax(torch.from_numpy(s), 1).numpy()
    prod, n = 1.0, 0
    for t in range(T):
        if mask[t]:
            prod *= 1.0 / p[t, lab[t]]
            n += 1
    nl = oracle.nll(s, lab, mask)
    seg = oracle.segment_reduce(nl["nll"], mask, np.array([0, T], np.int32))
    assert oracle.perplexity(seg["mean"], seg["count"])[0] == pytest.approx(prod ** (1.0 / n), rel=1e-12)


def test_policy_lag_is_zero_when_learner_and_generator_coincide(oracle):
    V, T = 53, 40
    gen = _rand(T, V)
    mask = (RNG.random(T) < 0.7).astype(np.uint8)
    cu = np.array([0, 13, 13, 31, 40], np.int32)
    kl = oracle.kd_dense(gen, gen.copy(), None, mask, want_grad=False)["kd"]      # KL(learner || generator), learner == generator
    out = oracle.policy_lag(kl, mask, cu, 0.10)
    assert out["batch_mean"] == 0.0 and out["exceeded"] == 0 and (out["seg_mean"] == 0.0).all()
    assert out["batch_count"] == int(mask.sum())
    assert oracle.policy_lag(kl, mask, cu, 0.0)["exceeded"] == 0                  # on-policy: D_KL <= 0 holds at 0


def test_policy_lag_brute_force_and_threshold(oracle):
    V, T = 41, 64
    gen, learner = _rand(T, V), None
    learner = gen + RNG.normal(0.0, 0.6, size=(T, V))
    mask = (RNG.random(T) < 0.75).astype(np.uint8)
    cu = np.array([3, 20, 21, 21, 50, 60], np.int32)               # positions 0..2 and 60.. belong to no sample
    mask[20] = 1
    # KL(learner || generator): the learner's distribution leads, so it sits in the teacher slot of Eq. 2's form
    kl = oracle.kd_dense(gen, learner, None, mask, want_grad=False)["kd"]
    pl = torch.log_softmax(torch.from_numpy(learner), 1)
    pg = torch.log_softmax(torch.from_numpy(gen), 1)
    ref_tok = (pl.exp() * (pl - pg)).sum(1).numpy()
    np.testing.assert_allclose(kl[mask == 1], ref_tok[mask == 1], rtol=0, atol=1e-12)
    out = oracle.policy_lag(kl, mask, cu, 0.10)
    total, n = 0.0, 0
    for i in range(len(cu) - 1):
        acc, k = 0.0, 0
        for p in range(cu[i], cu[i + 1]):
            if mask[p]:
                acc += ref_tok[p]
                k += 1
        assert out["seg_count"][i] == k
        assert out["seg_mean"][i] == pytest.approx(acc / k if k else 0.0, abs=1e-12)
        total, n = total + acc, n + k
    assert out["batch_count"] == n and n < int(mask.sum())          # unowned positions are not counted
    assert out["batch_mean"] == pytest.approx(total / n, abs=1e-12)
    # the step mean weighs every scored token the same: the count-weighted mean of the sample means
    w = out["seg_count"].astype(np.float64)
    assert out["batch_mean"] == pytest.approx(float((out["seg_mean"] * w).sum() / w.sum()), abs=1e-12)
    assert abs(out["batch_mean"] - out["seg_mean"][out["seg_count"] > 0].mean()) > 1e-4   # ... not the mean of means
    # near-policy regime: D_KL <= epsilon (closed); beyond it the batch is flagged
    m = out["batch_mean"]
    assert oracle.policy_lag(kl, mask, cu, m * 1.01)["exceeded"] == 0
    assert oracle.policy_lag(kl, mask, cu, m * 0.99)["exceeded"] == 1
    assert oracle.policy_lag(kl, mask, cu, float(np.float32(m)))["exceeded"] == 0     # equality is inside
    assert oracle.policy_lag(np.full(T, 0.10), mask, cu, 0.10)["exceeded"] == 0
    kl_nan = kl.copy()
    kl_nan[cu[0]] = np.nan
    mask[cu[0]] = 1
    assert oracle.policy_lag(kl_nan, mask, cu, 0.10)["exceeded"] == 1                 # a broken monitor is not "near"
    assert oracle.policy_lag(kl, np.zeros(T, np.uint8), cu, 0.10) == dict(
        seg_mean=pytest.approx(np.zeros(5)), seg_count=pytest.approx(np.zeros(5)), batch_mean=0.0, batch_count=0,
        exceeded=0)
    with pytest.raises(ValueError):
        oracle.policy_lag(kl, mask, np.array([0, 9, 4], np.int32), 0.10)


# --------------------------------------------------------------------------- Delta-IFD (Eq. 3, Eq. 4, zones)

def _golden_rows():
    rows = []
    with open(os.path.join(HERE, "golden", "delta_ifd_zones.txt")) as f:
        for line in f:
            line = line.strip()
            if not line or line.startswith("#"):
                continue
            lhs, rhs = line.split("|")
            rows.append(([float(v) for v in lhs.split()], [float(v) for v in rhs.split()]))
    return rows


def test_delta_ifd_hand_worked_cases(oracle):
    rows = _golden_rows()
    assert len(rows) >= 10
    for (lsc, lsu, ltc, ltu, nc, nu, lo, hi, flags), (ifs, ift, d, zone, keep) in rows:
        out = oracle.delta_ifd([lsc, lsu], [ltc, ltu], [int(nc), int(nu)], [0], [1], lo, hi, int(flags))
        np.testing.assert_array_equal(out["ifd_student"], [ifs])
        np.testing.assert_array_equal(out["ifd_teacher"], [ift])
        np.testing.assert_array_equal(out["delta"], [d])
        assert out["zone"][0] == int(zone) and out["keep"][0] == int(keep) and out["keep_count"] == int(keep)


def test_delta_ifd_brute_force_from_token_losses(oracle):
    # 6 pairs; per-position CE losses -> per-sample means -> ratios, written with python loops
    P = 6
    lens_c = RNG.integers(3, 30, P)
    lens_u = RNG.integers(3, 30, P)
    cu = np.concatenate([[0], np.cumsum(np.stack([lens_c, lens_u], 1).reshape(-1))]).astype(np.int32)
    T = int(cu[-1])
    nll_s, nll_t = RNG.uniform(0.1, 5, T), RNG.uniform(0.1, 5, T)
    mask = (RNG.random(T) < 0.8).astype(np.uint8)
    mask[cu[:-1]] = 1
    ms = oracle.segment_reduce(nll_s, mask, cu)
    mt = oracle.segment_reduce(nll_t, mask, cu)
    pc, pu = np.arange(0, 2 * P, 2), np.arange(1, 2 * P, 2)
    out = oracle.delta_ifd(ms["mean"], mt["mean"], ms["count"], pc, pu, 0.0, 0.8)
    kept = 0
    for j in range(P):
        def mean(x, i):
            vals = [x[p] for p in range(cu[i], cu[i + 1]) if mask[p]]
            return sum(vals) / len(vals)
        ifs = mean(nll_s, pc[j]) / mean(nll_s, pu[j])
        ift = mean(nll_t, pc[j]) / mean(nll_t, pu[j])
        d = ift - ifs
        assert out["ifd_student"][j] == pytest.approx(ifs, rel=1e-12)
        assert out["ifd_teacher"][j] == pytest.approx(ift, rel=1e-12)
        assert out["delta"][j] == pytest.approx(d, rel=1e-10, abs=1e-13)
        zone = 0 if d < 0 else (2 if d > 0.8 else 1)
        assert out["zone"][j] == zone
        kept += zone == 1
    assert out["keep_count"] == kept == int(out["keep"].sum())


def test_delta_ifd_symmetries(oracle):
    S = 10
    ms, mt = RNG.uniform(0.5, 3, S), RNG.uniform(0.5, 3, S)
    cnt = np.full(S, 4, np.int32)
    pc, pu = np.arange(0, S, 2), np.arange(1, S, 2)
    a = oracle.delta_ifd(ms, mt, cnt, pc, pu, 0.0, 1.0)
    b = oracle.delta_ifd(mt, ms, cnt, pc, pu, 0.0, 1.0)        # swap teacher and student
    np.testing.assert_array_equal(a["delta"], -b["delta"])
    same = oracle.delta_ifd(ms, ms, cnt, pc, pu, 0.0, 0.8)      # teacher == student: delta 0, proximal (closed)
    assert (same["delta"] == 0).all() and (same["zone"] == 1).all() and same["keep_count"] == len(pc)
    # IFD > 1 exactly when the instruction makes the response harder to predict
    assert ((a["ifd_student"] > 1) == (ms[pc] > ms[pu])).all()


# --------------------------------------------------------------------------- composite loss (Eq. 1)

@pytest.mark.parametrize("tau", [1.0, 2.0])
def test_composite_gradient_finite_differences(oracle, tau):
    # L_total = (1 - lambda) L_CE + lambda L_KD (Eq. 1): its gradient from the oracle vs central differences of
    # the oracle's own per-position kd and nll outputs (which are pinned separately above)
    T, V, h, lam, w = 2, 40, 1e-6, 0.9, 0.7
    s, t = _rand(T, V), _rand(T, V)
    lab = RNG.integers(0, V, T)
    g = oracle.kd_dense(s, t, lab, tau=tau, grad_scale=lam * w, ce_grad_scale=(1 - lam) * w)["grad"]

    def total(x, r):
        o = oracle.kd_dense(x, t, lab, tau=tau, want_grad=False)
        return w * (lam * o["kd"][r] + (1 - lam) * o["nll_s"][r])
    for r in range(T):
        for c in range(V):
            sp, sm = s.copy(), s.copy()
            sp[r, c] += h
            sm[r, c] -= h
            assert g[r, c] == pytest.approx((total(sp, r) - total(sm, r)) / (2 * h), rel=2e-6, abs=1e-9)


def test_composite_gradient_matches_autograd_and_sums_to_zero(oracle):
    T, V, k = 6, 300, 12
    s, t = _rand(T, V, 3.0), _rand(T, V, 3.0)
    lab = RNG.integers(0, V, T)
    mask = np.array([1, 1, 0, 1, 1, 1], np.uint8)
    ts = torch.from_numpy(s).requires_grad_(True)
    F.cross_entropy(ts, torch.from_numpy(lab), reduction="sum").backward()     # library CE gradient, float64
    ce = ts.grad.numpy()
    kd_only = oracle.kd_dense(s, t, lab, mask, tau=2.0, grad_scale=0.4)["grad"]
    both = oracle.kd_dense(s, t, lab, mask, tau=2.0, grad_scale=0.4, ce_grad_scale=0.25)["grad"]
    m = mask.astype(bool)
    np.testing.assert_allclose((both - kd_only)[m], 0.25 * ce[m], rtol=1e-10, atol=1e-15)
    assert (both[~m] == 0).all()
    assert np.abs(both.sum(1)).max() < 1e-12 * V
    # CE only (lambda = 0): the gradient is softmax - onehot whatever the teacher is
    ce_only = oracle.kd_dense(s, t, lab, tau=1.0, grad_scale=0.0, ce_grad_scale=1.0)["grad"]
    np.testing.assert_allclose(ce_only, ce, rtol=1e-10, atol=1e-15)
    # top-k teacher: same CE term
    idx = np.stack([RNG.choice(V, k, replace=False) for _ in range(T)]).astype(np.int32)
    idx[0, 0] = lab[0]                                   # the label inside the teacher's support
    val = _rand(T, k)
    a = oracle.kd_topk(s, idx, val, lab, mask, tau=2.0, grad_scale=0.4)["grad"]
    b = oracle.kd_topk(s, idx, val, lab, mask, tau=2.0, grad_scale=0.4, ce_grad_scale=0.25)["grad"]
    np.testing.assert_allclose((b - a)[m], 0.25 * ce[m], rtol=1e-10, atol=1e-15)
    # an out-of-range label poisons that row's gradient only
    bad = lab.copy()
    bad[1] = V
    g = oracle.kd_dense(s, t, bad, tau=1.0, ce_grad_scale=1.0)["grad"]
    assert np.isnan(g[1]).all() and np.isfinite(g[[0, 2, 3]]).all()


# --------------------------------------------------------------------------- teacher-side top-k record (Sec. 3.1)

def _bf16_bits(x):
    return torch.from_numpy(np.asarray(x, np.float32)).to(torch.bfloat16).view(torch.int16).numpy().view(np.uint16)


def test_teacher_topk_against_library_sort_and_ties(oracle):
    T, V, k = 6, 3000, 17
    x = RNG.normal(0, 3, size=(T, V))
    x[1, :] = 0.5                                  # a constant row: the k lowest ids
    x[2, 100:140] = x[2].max() + 1.0               # forty equal maxima: ids 100..116
    bits = _bf16_bits(x)
    vals = torch.from_numpy(bits.view(np.int16)).view(torch.bfloat16).double().numpy()   # what bf16 really holds
    out = oracle.teacher_topk(bits, k, log_probs=False)
    for r in range(T):
        order = np.lexsort((np.arange(V), -vals[r]))[:k]         # library: value descending, then id ascending
        np.testing.assert_array_equal(out["idx"][r], order)
        np.testing.assert_array_equal(out["val"][r], vals[r][order])
    assert out["idx"][1].tolist() == list(range(k)) and out["idx"][2].tolist() == list(range(100, 117))
    tv = torch.topk(torch.from_numpy(vals), k, dim=1).values.numpy()             # values agree with torch.topk
    np.testing.assert_array_equal(out["val"], tv)
    # k = 1 is the arg-max (first of equals); k = V is a full stable sort
    np.testing.assert_array_equal(oracle.teacher_topk(bits, 1, log_probs=False)["idx"][:, 0], vals.argmax(1))
    full = oracle.teacher_topk(bits[:2, :50].copy(), 50, log_probs=False)
    assert sorted(full["idx"][0].tolist()) == list(range(50))


def test_teacher_topk_log_probs_and_consistency_with_eq2(oracle):
    T, V, k = 4, 500, 9
    s, t = _rand(T, V, 3.0), _rand(T, V, 3.0)
    sb, tb = _bf16_bits(s), _bf16_bits(t)
    raw = oracle.teacher_topk(tb, k, log_probs=False)
    lp = oracle.teacher_topk(tb, k, log_probs=True)
    np.testing.assert_array_equal(raw["idx"], lp["idx"])
    np.testing.assert_allclose(np.exp(lp["val"]).sum(1), 1.0, atol=1e-12)
    np.testing.assert_allclose(lp["val"], torch.log_softmax(torch.from_numpy(raw["val"]), 1).numpy(), atol=1e-12)
    # Eq. 2 does not care whether the record holds logits or renormalised log-probabilities
    a = oracle.kd_topk(sb, raw["idx"], raw["val"].astype(np.float32), tau=2.0)
    b = oracle.kd_topk(sb, lp["idx"], lp["val"].astype(np.float32), tau=2.0)
    np.testing.assert_allclose(a["kd"], b["kd"], rtol=1e-6)
    # with k = V the record reproduces the dense-teacher loss
    full = oracle.teacher_topk(tb, V, log_probs=False)
    np.testing.assert_allclose(oracle.kd_topk(sb, full["idx"], full["val"].astype(np.float32))["kd"],
                               oracle.kd_dense(sb, tb)["kd"], rtol=1e-9)
    # unscored positions: ids 0..k-1, values 0
    m = oracle.teacher_topk(tb, k, mask=np.array([1, 0, 1, 1], np.uint8))
    assert m["idx"][1].tolist() == list(range(k)) and (m["val"][1] == 0).all()
    np.testing.assert_array_equal(m["idx"][[0, 2, 3]], lp["idx"][[0, 2, 3]])


# --------------------------------------------------------------------------- other divergences (Related Works)

DIVS = ("reverse", "skew", "skew_reverse")


def test_divergence_values_through_the_pinned_forward_kl(oracle):
    """Each divergence is a forward KL between other distributions, and the forward KL is pinned above:
    reverse = KL(p_S || p_T) = forward with the roles swapped; skew = KL(p_T || m) and skew reverse = KL(p_S || m),
    i.e. the forward KL against a 'student' whose logits are log m."""
    s, t = _rand(7, 90, 3.0), _rand(7, 90, 3.0)
    for tau in (1.0, 2.0):
        ps = torch.softmax(torch.from_numpy(s) / tau, 1).numpy()
        pt = torch.softmax(torch.from_numpy(t) / tau, 1).numpy()
        np.testing.assert_allclose(oracle.div_dense(s, t, "reverse", tau=tau, want_grad=False)["kd"],
                                   oracle.kd_dense(t, s, tau=tau, want_grad=False)["kd"], rtol=1e-12)
        for alpha in (0.1, 0.5):
            m = alpha * pt + (1 - alpha) * ps
            np.testing.assert_allclose(oracle.div_dense(s, t, "skew", alpha, tau=tau, want_grad=False)["kd"],
                                       oracle.kd_dense(np.log(m), t / tau, want_grad=False)["kd"], rtol=1e-11)
            m = (1 - alpha) * pt + alpha * ps
            np.testing.assert_allclose(oracle.div_dense(s, t, "skew_reverse", alpha, tau=tau, want_grad=False)["kd"],
                                       oracle.kd_dense(np.log(m), s / tau, want_grad=False)["kd"], rtol=1e-11)


def test_divergence_library_values_and_two_level_closed_form(oracle):
    s, t = _rand(5, 64, 2.5), _rand(5, 64, 2.5)
    ls, lt = torch.log_softmax(torch.from_numpy(s), 1), torch.log_softmax(torch.from_numpy(t), 1)
    # F.kl_div(input, target) = sum target * (log target - input)
    ref = F.kl_div(lt, ls, reduction="none", log_target=True).sum(1)
    np.testing.assert_allclose(oracle.div_dense(s, t, "reverse")["kd"], ref.numpy(), rtol=1e-11)
    lm = torch.log(0.1 * lt.exp() + 0.9 * ls.exp())
    ref = F.kl_div(lm, lt, reduction="none", log_target=True).sum(1)
    np.testing.assert_allclose(oracle.div_dense(s, t, "skew", 0.1)["kd"], ref.numpy(), rtol=1e-11)
    lm = torch.log(0.9 * lt.exp() + 0.1 * ls.exp())
    ref = F.kl_div(lm, ls, reduction="none", log_target=True).sum(1)
    np.testing.assert_allclose(oracle.div_dense(s, t, "skew_reverse", 0.1)["kd"], ref.numpy(), rtol=1e-11)
    # two-level rows: reverse KL is the binary KL with the student in front
    V, a, b = 500, 2.0, 0.5
    s1 = np.zeros((1, V)); s1[0, 0] = b
    t1 = np.zeros((1, V)); t1[0, 0] = a
    pt = math.exp(a) / (math.exp(a) + V - 1)
    ps = math.exp(b) / (math.exp(b) + V - 1)
    want = ps * math.log(ps / pt) + (1 - ps) * math.log((1 - ps) / (1 - pt))
    assert oracle.div_dense(s1, t1, "reverse")["kd"][0] == pytest.approx(want, rel=1e-12)


def test_divergence_limits_and_zero_at_equality(oracle):
    s, t = _rand(6, 50, 3.0), _rand(6, 50, 3.0)
    fwd = oracle.kd_dense(s, t, tau=1.5)
    rev = oracle.div_dense(s, t, "reverse", tau=1.5)
    # alpha = 0 removes the skew
    a0 = oracle.div_dense(s, t, "skew", 0.0, tau=1.5)
    np.testing.assert_allclose(a0["kd"], fwd["kd"], rtol=1e-12)
    np.testing.assert_allclose(a0["grad"], fwd["grad"], rtol=1e-9, atol=1e-15)
    b0 = oracle.div_dense(s, t, "skew_reverse", 0.0, tau=1.5)
    np.testing.assert_allclose(b0["kd"], rev["kd"], rtol=1e-12)
    np.testing.assert_allclose(b0["grad"], rev["grad"], rtol=1e-9, atol=1e-15)
    # "forward" is Eq. 2 itself
    f = oracle.div_dense(s, t, "forward", tau=1.5)
    assert (f["kd"] == fwd["kd"]).all() and (f["grad"] == fwd["grad"]).all()
    for d in DIVS:
        out = oracle.div_dense(s, t, d, 0.3)
        assert (out["kd"] > 0).all()
        np.testing.assert_allclose(out["grad"].sum(1), 0.0, atol=1e-13)      # softmax Jacobian: rows sum to zero
        same = oracle.div_dense(s, s.copy(), d, 0.3)
        np.testing.assert_allclose(same["kd"], 0.0, atol=1e-15)
        np.testing.assert_allclose(same["grad"], 0.0, atol=1e-15)
    # skewing towards the other distribution can only shrink the divergence (convexity of KL)
    assert (oracle.div_dense(s, t, "skew", 0.3)["kd"] < oracle.kd_dense(s, t)["kd"]).all()
    assert (oracle.div_dense(s, t, "skew_reverse", 0.3)["kd"] < oracle.div_dense(s, t, "reverse")["kd"]).all()


@pytest.mark.parametrize("div", DIVS)
@pytest.mark.parametrize("tau", [1.0, 2.0])
def test_divergence_gradient_finite_differences(oracle, div, tau):
    T, V, h, alpha = 2, 40, 1e-6, 0.2
    s, t = _rand(T, V), _rand(T, V)
    g = oracle.div_dense(s, t, div, alpha, tau=tau, grad_scale=1.0)["grad"]
    for r in range(T):
        for c in range(V):
            sp, sm = s.copy(), s.copy()
            sp[r, c] += h
            sm[r, c] -= h
            fd = (oracle.div_dense(sp, t, div, alpha, tau=tau, want_grad=False)["kd"][r]
                  - oracle.div_dense(sm, t, div, alpha, tau=tau, want_grad=False)["kd"][r]) / (2 * h)
            assert g[r, c] == pytest.approx(fd, rel=5e-6, abs=2e-9)


def test_divergence_gradient_matches_autograd_with_composite_term_and_bf16_front_end(oracle):
    T, V, tau, alpha, gs, cs = 4, 33, 2.0, 0.1, 0.9, 0.1
    s, t = _rand(T, V), _rand(T, V)
    labels = RNG.integers(0, V, T).astype(np.int32)
    for div in DIVS:
        st = torch.from_numpy(s).requires_grad_(True)
        ps, pt = torch.softmax(st / tau, 1), torch.softmax(torch.from_numpy(t) / tau, 1)
        if div == "reverse":
            d = (ps * (ps.log() - pt.log())).sum(1)
        elif div == "skew":
            d = (pt * (pt.log() - (alpha * pt + (1 - alpha) * ps).log())).sum(1)
        else:
            d = (ps * (ps.log() - ((1 - alpha) * pt + alpha * ps).log())).sum(1)
        loss = gs * d.sum() + cs * F.cross_entropy(st, torch.from_numpy(labels).long(), reduction="sum")
        loss.backward()
        out = oracle.div_dense(s, t, div, alpha, labels=labels, tau=tau, grad_scale=gs, ce_grad_scale=cs)
        np.testing.assert_allclose(out["kd"], d.detach().numpy(), rtol=1e-11)
        np.testing.assert_allclose(out["grad"], st.grad.numpy(), rtol=1e-9, atol=1e-13)
    # the bf16 front-end converts exactly and masks rows
    sb = torch.from_numpy(s).to(torch.bfloat16)
    tb = torch.from_numpy(t).to(torch.bfloat16)
    mask = np.array([1, 0, 1, 1], np.uint8)
    a = oracle.div_dense(sb.view(torch.int16).numpy().view(np.uint16), tb.view(torch.int16).numpy().view(np.uint16),
                         "skew_reverse", alpha, mask=mask)
    b = oracle.div_dense(sb.double().numpy(), tb.double().numpy(), "skew_reverse", alpha, mask=mask)
    assert (a["kd"] == b["kd"]).all() and (a["grad"] == b["grad"]).all()
    assert a["kd"][1] == 0 and (a["grad"][1] == 0).all()


# --------------------------------------------------------------------------- entries of probability 0 (-inf logits)

def test_minus_infinity_logits_are_entries_of_probability_zero(oracle):
    """A logit of -inf marks a vocabulary entry of probability 0 (a padded or banned token).  Pins: the library
    softmax (which gives such entries exactly 0), the same problem on the reduced vocabulary, and the definition of
    Eq. 2 with its p_T = 0 terms left out."""
    rng = np.random.default_rng(77)
    T, V, tau = 5, 40, 2.0
    s, t = _rand(T, V, 2.0, rng), _rand(T, V, 2.0, rng)
    banned = np.zeros(V, bool)
    banned[[3, 11, 12, 39]] = True
    labels = rng.choice(np.flatnonzero(~banned), T).astype(np.int32)

    # (1) both models padded on the same entries: the problem on the reduced vocabulary, gradient 0 on the padding
    s1, t1 = s.copy(), t.copy()
    s1[:, banned] = -np.inf
    t1[:, banned] = -np.inf
    full = oracle.kd_dense(s1, t1, labels, tau=tau, grad_scale=0.7)
    keep = np.flatnonzero(~banned)
    relabel = np.searchsorted(keep, labels).astype(np.int32)
    red = oracle.kd_dense(s[:, keep], t[:, keep], relabel, tau=tau, grad_scale=0.7)
    np.testing.assert_allclose(full["kd"], red["kd"], rtol=1e-13)
    np.testing.assert_allclose(full["nll_s"], red["nll_s"], rtol=1e-13)
    np.testing.assert_allclose(full["nll_t"], red["nll_t"], rtol=1e-13)
    np.testing.assert_allclose(full["grad"][:, keep], red["grad"], rtol=1e-12, atol=1e-15)
    assert (full["grad"][:, banned] == 0).all()

    # (2) only the teacher bans entries: Eq. 2 without the p_T = 0 terms, p_S still over the full vocabulary
    out = oracle.kd_dense(s, t1, labels, tau=tau, grad_scale=1.0)
    lps = torch.log_softmax(torch.from_numpy(s) / tau, -1)
    pt = torch.softmax(torch.from_numpy(t1) / tau, -1)                     # exactly 0 on the banned entries
    assert (pt[:, banned] == 0).all()
    lpt = torch.log_softmax(torch.from_numpy(t[:, keep]) / tau, -1)
    kl = (pt[:, keep] * (lpt - lps[:, keep])).sum(-1)
    np.testing.assert_allclose(out["kd"], kl.numpy(), rtol=1e-12)
    np.testing.assert_allclose(out["grad"], ((lps.exp() - pt) / tau).numpy(), rtol=1e-12, atol=1e-16)
    assert np.isfinite(out["kd"]).all() and np.isfinite(out["grad"]).all()

    # (3) the student gives probability 0 where the teacher does not: the divergence is infinite
    s3 = s.copy()
    s3[0, 5] = -np.inf
    assert np.isposinf(oracle.kd_dense(s3, t, want_grad=False)["kd"][0])
    # ... and its own label there has an infinite loss
    lab = labels.copy()
    lab[0] = 5
    assert np.isposinf(oracle.kd_dense(s3, t, lab, want_grad=False)["nll_s"][0])

    # (4) a top-k value of -inf is an entry the record does not have
    k = 6
    idx = np.stack([rng.choice(V, k, replace=False) for _ in range(T)]).astype(np.int32)
    val = rng.normal(0, 1, (T, k))
    val_inf = val.copy()
    val_inf[:, 2] = -np.inf
    a = oracle.kd_topk(s, idx, val_inf, tau=tau)
    b = oracle.kd_topk(s, np.delete(idx, 2, axis=1), np.delete(val, 2, axis=1), tau=tau)
    np.testing.assert_allclose(a["kd"], b["kd"], rtol=1e-13)
    np.testing.assert_allclose(a["grad"], b["grad"], rtol=1e-12, atol=1e-16)

    # (5) the other divergences: entries of probability 0 in both models contribute no term and no gradient
    for div in ("reverse", "skew", "skew_reverse"):
        fa = oracle.div_dense(s1, t1, div, 0.3, tau=tau)
        re = oracle.div_dense(s[:, keep], t[:, keep], div, 0.3, tau=tau)
        np.testing.assert_allclose(fa["kd"], re["kd"], rtol=1e-12)
        np.testing.assert_allclose(fa["grad"][:, keep], re["grad"], rtol=1e-11, atol=1e-15)
        assert (fa["grad"][:, banned] == 0).all()
