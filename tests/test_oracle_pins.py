"""Pins for the CPU oracle: closed forms, hand-worked fixtures, invariants, brute force and
library routines.  No GPU.  A plausible slip in the oracle (inclusive instead of exclusive
anchor, dropped 1/t, population/sample variance mix-up in alpha, wrong tie-break, K/V swapped
in attention, wrong GQA head map, missing causal mask) fails at least one test here."""
import math
import os
from fractions import Fraction

import numpy as np
import pytest
import torch

import oracle
from paper_2512_07090_amd import synth


def _load_table(path):
    rows = []
    with open(path) as f:
        for line in f:
            line = line.strip()
            if line and not line.startswith("#"):
                rows.append([float(x) for x in line.split()])
    return np.array(rows)


# ------------------------------------------------------------------ anchor / prefix mean

def test_anchor_golden_closed_form(golden_dir):
    tab = _load_table(os.path.join(golden_dir, "cosine_closed_forms.txt"))
    x = tab[:, 1:3].astype(np.float32).reshape(1, 1, 4, 2)
    cosv, anchors = oracle.anchor_cosine(x, return_anchors=True)
    np.testing.assert_allclose(anchors[0, 0], tab[:, 3:5], rtol=0, atol=1e-15)
    np.testing.assert_allclose(cosv[0, 0], tab[:, 5], rtol=0, atol=1e-15)


def test_anchor_brute_force_prefix_mean():
    rng = np.random.default_rng(1)
    x = rng.standard_normal((2, 3, 9, 5)).astype(np.float32)
    cosv, anchors = oracle.anchor_cosine(x, return_anchors=True)
    xd = x.astype(np.float64)
    for b in range(2):
        for h in range(3):
            for t in range(9):
                ref = xd[b, h, :t].mean(axis=0) if t else np.zeros(5)   # O(n^2) recomputation
                np.testing.assert_allclose(anchors[b, h, t], ref, rtol=0, atol=1e-14)
                if t:
                    c = np.dot(ref, xd[b, h, t]) / (np.linalg.norm(ref) * np.linalg.norm(xd[b, h, t]))
                    assert abs(cosv[b, h, t] - c) < 1e-13
                else:
                    assert cosv[b, h, t] == 0.0


def test_anchor_two_tokens():
    x = np.array([[3.0, 4.0], [4.0, 3.0]], dtype=np.float32).reshape(1, 1, 2, 2)
    cosv, anchors = oracle.anchor_cosine(x, return_anchors=True)
    np.testing.assert_array_equal(anchors[0, 0, 1], [3.0, 4.0])      # anchor at t=1 is x_0
    assert abs(cosv[0, 0, 1] - 24.0 / 25.0) < 1e-15


def test_cosine_range_and_identical_tokens():
    q, k, v, _ = synth.make_random_qkv(2, 4, 4, 64, 16, seed=3)
    for x in (k, v):
        c = oracle.anchor_cosine(x)
        assert np.all(c <= 1.0) and np.all(c >= -1.0)
        assert np.all(c[:, :, 0] == 0.0)
    row = np.random.default_rng(0).standard_normal(16).astype(np.float32)
    same = np.broadcast_to(row, (1, 2, 10, 16)).copy()
    c = oracle.anchor_cosine(same)
    assert np.all(c[:, :, 0] == 0.0)
    np.testing.assert_allclose(c[:, :, 1:], 1.0, rtol=0, atol=1e-15)   # scores 1 after the first


def test_cosine_opposite_orthogonal_and_zero_rows():
    # x_t = -(mean of previous) gives -1
    x = np.zeros((1, 1, 3, 4), dtype=np.float32)
    x[0, 0, 0] = [1, 2, 0, 0]
    x[0, 0, 1] = [3, 0, 0, 0]
    x[0, 0, 2] = [-2, -1, 0, 0]       # -(x0 + x1)/2
    c = oracle.anchor_cosine(x)
    assert abs(c[0, 0, 2] + 1.0) < 1e-15
    # orthogonal basis vectors give 0; an all-zero row gives 0 through the guard
    e = np.zeros((1, 1, 4, 4), dtype=np.float32)
    e[0, 0, 0, 0] = e[0, 0, 1, 1] = e[0, 0, 2, 2] = 1.0
    c = oracle.anchor_cosine(e)
    np.testing.assert_array_equal(c[0, 0], [0, 0, 0, 0])


def test_cosine_scale_invariance_and_mean_vs_sum():
    rng = np.random.default_rng(5)
    x = rng.standard_normal((1, 2, 33, 8)).astype(np.float32)
    c1 = oracle.anchor_cosine(x)
    c2 = oracle.anchor_cosine(x * np.float32(4.0))          # power of two: exact rescale
    np.testing.assert_allclose(c1, c2, rtol=0, atol=1e-14)
    xd = x.astype(np.float64)
    sums = np.cumsum(xd, axis=2) - xd                        # exclusive prefix SUM
    num = (sums * xd).sum(-1)
    den = np.linalg.norm(sums, axis=-1) * np.linalg.norm(xd, axis=-1)
    ref = np.where(den > 0, num / np.where(den > 0, den, 1), 0.0)
    np.testing.assert_allclose(c1, ref, rtol=0, atol=1e-13)  # cos(mean, x) == cos(sum, x)



# ------------------------------------------------------------------ incremental (EMA) anchor

def test_ema_anchor_golden_worked_example(golden_dir):
    tab = _load_table(os.path.join(golden_dir, "ema_anchor_worked_example.txt"))
    x = tab[:, 1:3].astype(np.float32).reshape(1, 1, 4, 2)
    cosv, anchors = oracle.anchor_cosine_ema(x, 0.5, return_anchors=True)
    np.testing.assert_allclose(anchors[0, 0], tab[:, 3:5], rtol=0, atol=1e-15)
    np.testing.assert_allclose(cosv[0, 0], tab[:, 5], rtol=0, atol=1e-15)


def test_ema_anchor_brute_force_weights_and_special_cases():
    rng = np.random.default_rng(11)
    x = rng.normal(size=(2, 3, 40, 8)).astype(np.float32)
    for gamma in (0.9, 0.5, 0.99):
        cosv, anchors = oracle.anchor_cosine_ema(x, gamma, return_anchors=True)
        # closed form of the recurrence: A_t = (1 - gamma) * sum_{j<t} gamma^(t-1-j) x_j
        xd = x.astype(np.float64)
        for t in (0, 1, 2, 7, 39):
            w = (1 - gamma) * gamma ** (t - 1 - np.arange(t))
            ref = np.einsum("j,bhjd->bhd", w, xd[:, :, :t]) if t else np.zeros((2, 3, 8))
            np.testing.assert_allclose(anchors[:, :, t], ref, rtol=1e-12, atol=1e-15)
            if t:
                num = np.einsum("bhd,bhd->bh", ref, xd[:, :, t])
                den = np.linalg.norm(ref, axis=-1) * np.linalg.norm(xd[:, :, t], axis=-1)
                np.testing.assert_allclose(cosv[:, :, t], num / den, rtol=1e-12, atol=1e-15)
        assert np.all(cosv[:, :, 0] == 0)                      # empty anchor
        assert np.all(np.abs(cosv) <= 1)
    # identical tokens: anchor = (1 - gamma^t) x, cosine 1 after the first
    row = rng.normal(size=8).astype(np.float32)
    same = np.broadcast_to(row, (1, 1, 30, 8)).copy()
    c = oracle.anchor_cosine_ema(same, 0.9)
    assert c[0, 0, 0] == 0 and np.all(np.abs(c[0, 0, 1:] - 1) <= 1e-12)
    # gamma = 0: the anchor is the previous row alone
    c0 = oracle.anchor_cosine_ema(x, 0.0)
    xd = x.astype(np.float64)
    prev, cur = xd[:, :, :-1], xd[:, :, 1:]
    ref = np.einsum("bhtd,bhtd->bht", prev, cur) / (np.linalg.norm(prev, axis=-1) * np.linalg.norm(cur, axis=-1))
    np.testing.assert_allclose(c0[:, :, 1:], ref, rtol=1e-12, atol=1e-15)
    # the cosine does not see a power-of-two rescaling of the input
    np.testing.assert_allclose(oracle.anchor_cosine_ema(x * 4, 0.9), oracle.anchor_cosine_ema(x, 0.9),
                               rtol=1e-13, atol=1e-15)
    # and differs from the exact-mean anchor (a different weighting, not a renaming)
    assert np.abs(oracle.anchor_cosine_ema(x, 0.9) - oracle.anchor_cosine(x)).max() > 1e-3


# ------------------------------------------------------------------ head statistics / fusion

def test_fusion_golden_worked_example(golden_dir):
    tab = _load_table(os.path.join(golden_dir, "fusion_worked_example.txt"))
    ck = np.array([0.2, 0.6]).reshape(1, 2, 1)
    cv = np.array([0.5, 0.7]).reshape(1, 2, 1)
    for mode, alpha, s in tab:
        S, st = oracle.fuse(ck, cv, int(mode), return_stats=True)
        assert abs(st[0, 0, 4] - alpha) < 1e-9
        assert abs(S[0, 0] - s) < 1e-9
        np.testing.assert_allclose(st[0, 0, :4], [0.4, 0.6, 0.04, 0.01], rtol=0, atol=1e-15)


def test_fusion_stats_vs_numpy_and_properties():
    rng = np.random.default_rng(7)
    ck = rng.uniform(-1, 1, (3, 6, 50))
    cv = rng.uniform(-1, 1, (3, 6, 50))
    S0, st = oracle.fuse(ck, cv, oracle.FUSE_EQ2, return_stats=True)
    S1, st1 = oracle.fuse(ck, cv, oracle.FUSE_INVVAR, return_stats=True)
    np.testing.assert_allclose(st[..., 0], ck.mean(1), atol=1e-15)
    np.testing.assert_allclose(st[..., 1], cv.mean(1), atol=1e-15)
    np.testing.assert_allclose(st[..., 2], ck.var(1), atol=1e-15)        # ddof = 0
    np.testing.assert_allclose(st[..., 3], cv.var(1), atol=1e-15)
    np.testing.assert_allclose(st[..., 4] + st1[..., 4], 1.0, atol=1e-12)  # the two readings mirror
    # alpha depends only on the variance ratio, so ddof cannot matter
    a_ddof1 = ck.var(1, ddof=1) / (ck.var(1, ddof=1) + cv.var(1, ddof=1))
    np.testing.assert_allclose(st[..., 4], a_ddof1, atol=1e-9)
    # printed formula: the higher-variance side gets the larger weight
    hi_k = st[..., 2] > st[..., 3]
    assert np.all(st[..., 4][hi_k] > 0.5) and np.all(st1[..., 4][hi_k] < 0.5)
    lo, hi = np.minimum(st[..., 0], st[..., 1]), np.maximum(st[..., 0], st[..., 1])
    for S in (S0, S1):
        assert np.all(S >= lo - 1e-15) and np.all(S <= hi + 1e-15)
    np.testing.assert_allclose(oracle.fuse(ck, cv, oracle.FUSE_KEY_ONLY), ck.mean(1), atol=1e-15)
    np.testing.assert_allclose(oracle.fuse(ck, cv, oracle.FUSE_VALUE_ONLY), cv.mean(1), atol=1e-15)
    # head permutation leaves S unchanged
    perm = rng.permutation(6)
    np.testing.assert_allclose(oracle.fuse(ck[:, perm], cv[:, perm]), S0, atol=1e-14)
    # K == V: S = s_k whatever alpha is
    np.testing.assert_allclose(oracle.fuse(ck, ck), ck.mean(1), atol=1e-15)
    # equal variances: plain average.  cv = const - ck has the same variance
    np.testing.assert_allclose(oracle.fuse(ck, 0.25 - ck), np.full((3, 50), 0.125), atol=1e-12)


def test_fusion_degenerate_variances():
    ck = np.full((1, 4, 3), 0.3)
    cv = np.full((1, 4, 3), 0.9)
    S, st = oracle.fuse(ck, cv, return_stats=True)          # both variances zero: alpha = 1/2
    np.testing.assert_allclose(st[..., 4], 0.5, atol=1e-12)
    np.testing.assert_allclose(S, 0.6, atol=1e-12)
    one = np.array([0.1]).reshape(1, 1, 1)                   # a single head
    assert abs(oracle.fuse(one, one * 5)[0, 0] - 0.3) < 1e-12


def test_gqa_scoring_equals_repeated_heads():
    _, k, v, _ = synth.make_random_qkv(1, 8, 2, 40, 16, seed=11)
    S = oracle.fuse(oracle.anchor_cosine(k), oracle.anchor_cosine(v))
    kr, vr = k.repeat_interleave(4, dim=1), v.repeat_interleave(4, dim=1)
    Sr = oracle.fuse(oracle.anchor_cosine(kr), oracle.anchor_cosine(vr))
    np.testing.assert_allclose(S, Sr, rtol=0, atol=1e-13)



# ------------------------------------------------------------------ tail-focused schedule

def test_tail_schedule_paper_examples_and_budget():
    # Section 3.3's own example: a 25 % global budget on the last half of the layers is 50 % there
    r, n_tail = oracle.tail_schedule(32, 0.25, 0.5)
    assert n_tail == 16 and np.all(r[:16] == 0) and np.all(r[16:] == 0.5)
    # the hyper-parameter table of the appendix: 33 % on LLaMA-2-13B (40 layers), Y in 0.4 .. 0.6
    for y, count, ratio in ((0.4, 16, 0.825), (0.5, 20, 0.66), (0.6, 24, 0.55)):
        r, n_tail = oracle.tail_schedule(40, 0.33, y)
        assert n_tail == count
        np.testing.assert_allclose(r[40 - count:], ratio, rtol=1e-15)
        assert np.all(r[:40 - count] == 0)
        np.testing.assert_allclose(r.mean(), 0.33, rtol=1e-12)      # the budget is met exactly
    # Eq. 3 in exact rationals whenever y * L is whole; the tail is never pruned above 1
    for L in (1, 7, 32, 40, 80):
        for num, den in ((1, 1), (1, 2), (1, 4), (3, 4)):
            if (L * num) % den:
                continue
            for pg in (Fraction(0), Fraction(1, 10), Fraction(1, 4), Fraction(1, 2)):
                r, n_tail = oracle.tail_schedule(L, float(pg), num / den)
                assert n_tail == L * num // den
                want = min(pg * den / num, Fraction(1))
                np.testing.assert_allclose(r[L - n_tail:], float(want), rtol=1e-15, atol=0)
                assert np.all(r[:L - n_tail] == 0)
    r, n_tail = oracle.tail_schedule(10, 0.9, 0.5)
    assert np.all(r[5:] == 1.0)
    r, n_tail = oracle.tail_schedule(10, 0.3, 0.25)                   # 2.5 layers -> 3
    assert n_tail == 3
    for bad in ((0, 0.2, 0.5), (4, -0.1, 0.5), (4, 0.2, 0.0), (4, 0.2, 1.5)):
        with pytest.raises(ValueError):
            oracle.tail_schedule(*bad)


# ------------------------------------------------------------------ count / selection

def test_keep_count_golden(golden_dir):
    tab = _load_table(os.path.join(golden_dir, "keep_count_table.txt"))
    for n, r, m in tab:
        assert oracle.keep_count(int(n), r) == int(m)


def test_keep_count_is_ceil_exact_rational():
    for n in (1, 2, 3, 10, 127, 512, 4096, 32768):
        for num in range(0, 100):
            r = Fraction(num, 100)
            want = math.ceil((1 - r) * n)
            assert oracle.keep_count(n, num / 100.0) == want, (n, num)


def _brute_select(s32, m, W):
    n = s32.shape[0]
    forced = min(W, m)
    keep = np.zeros(n, dtype=np.uint8)
    keep[:forced] = 1
    rest = np.arange(forced, n)
    order = rest[np.lexsort((rest, s32[rest]))]             # by score, then by index
    keep[order[:m - forced]] = 1
    return keep


def test_select_vs_brute_force_and_invariants():
    rng = np.random.default_rng(13)
    for n, r, W in [(50, 0.5, 1), (64, 0.25, 4), (33, 0.9, 1), (17, 0.0, 1), (40, 0.5, 0),
                    (12, 0.8, 5)]:
        S = rng.uniform(-1, 1, (3, n))
        S[1] = np.round(S[1] * 4) / 4                        # many exact ties
        keep, idx, tau = oracle.select(S, r, W)
        m = oracle.keep_count(n, r)
        s32 = S.astype(np.float32)
        for b in range(3):
            assert keep[b].sum() == m
            np.testing.assert_array_equal(keep[b], _brute_select(s32[b], m, W))
            np.testing.assert_array_equal(idx[b], np.nonzero(keep[b])[0])
            assert np.all(np.diff(idx[b]) > 0)
            forced = min(W, m)
            kept_nf = [t for t in idx[b] if t >= forced]
            filt = np.nonzero(keep[b] == 0)[0]
            if m == n:
                assert tau[b] == np.inf
            elif not kept_nf:
                assert tau[b] == -np.inf
            else:
                assert tau[b] == s32[b, kept_nf].max()
            if len(filt):
                assert np.all(s32[b, filt] >= tau[b])        # skip iff S >= tau (ties by index)


def test_select_tie_break_and_nesting():
    S = np.array([[0.5, 0.1, 0.1, 0.1, 0.1, 0.9]])
    keep, idx, tau = oracle.select(S, 0.5, 1)                # m = 3: forced 0, then ties 1, 2
    np.testing.assert_array_equal(keep[0], [1, 1, 1, 0, 0, 0])
    assert tau[0] == np.float32(0.1)
    rng = np.random.default_rng(17)
    S = rng.uniform(-1, 1, (2, 200))
    prev = None
    for r in (0.0, 0.1, 0.25, 0.5, 0.75, 0.9):
        keep, _, _ = oracle.select(S, r, 1)
        if prev is not None:
            assert np.all(keep <= prev)                       # kept sets shrink monotonically
        prev = keep
    assert np.all(oracle.select(S, 0.0, 1)[0] == 1)



# ------------------------------------------------------------------ online adaptive threshold

def test_online_threshold_golden_worked_example(golden_dir):
    tab = _load_table(os.path.join(golden_dir, "online_threshold_worked_example.txt"))
    S = tab[:, 1][None]
    keep, idx, count, tau = oracle.select_online(S, 0.5, 0.1, 0.5, 1)
    np.testing.assert_array_equal(keep[0], tab[:, 2].astype(np.uint8))
    assert count[0] == 2 and list(idx[0]) == [0, 2, -1, -1, -1]
    assert abs(float(tau[0]) - 23.0 / 60.0) <= 1e-6
    # the prefix of the run gives the intermediate thresholds
    for t in range(5):
        _, _, _, tau_t = oracle.select_online(S[:, :t + 1], 0.5, 0.1, 0.5, 1)
        assert abs(float(tau_t[0]) - tab[t, 3]) <= 1e-6
    # the per-token trace is the same list: the threshold each token was judged with
    _, _, _, _, trace = oracle.select_online(S, 0.5, 0.1, 0.5, 1, return_trace=True)
    assert np.all(np.abs(trace[0] - tab[:, 3]) <= 1e-6)
    assert np.array_equal(keep[0] == 0, (S[0].astype(np.float32) > trace[0]) & (np.arange(5) >= 1))


def test_online_threshold_closed_forms_and_feedback():
    rng = np.random.default_rng(21)
    S = rng.uniform(0, 1, (3, 5000)).astype(np.float32)
    n = S.shape[1]
    # eta = 0: a fixed threshold, plain comparison after the warm-up
    for W in (0, 1, 64):
        keep, idx, count, tau = oracle.select_online(S, 0.3, 0.0, 0.6, W)
        ref = (S <= np.float32(0.6)) | (np.arange(n) < W)
        np.testing.assert_array_equal(keep.astype(bool), ref)
        assert np.all(tau == np.float32(0.6))
        for b in range(3):
            assert count[b] == ref[b].sum()
            np.testing.assert_array_equal(idx[b, :count[b]], np.nonzero(ref[b])[0])
            assert np.all(idx[b, count[b]:] == -1)
    # warm-up covering the row: nothing skipped, the threshold still moves: tau0 - eta * r * n
    keep, _, count, tau = oracle.select_online(S, 0.25, 1e-3, 0.5, n)
    assert keep.all() and np.all(count == n)
    np.testing.assert_allclose(tau, 0.5 - 1e-3 * 0.25 * n, rtol=1e-4)
    # scores that never exceed the threshold: same trajectory, nothing skipped
    keep, _, _, tau2 = oracle.select_online(np.full((1, n), -5.0), 0.25, 1e-3, 0.5, 1)
    assert keep.all()
    np.testing.assert_array_equal(tau2[0], tau[0])
    # scores that always exceed it (no warm-up): P_current is 1 from the second token on, so
    # tau = tau0 - eta r + (n - 1) eta (1 - r)
    keep, _, count, tau3 = oracle.select_online(np.full((1, 2000), 50.0), 0.25, 1e-3, 0.5, 0)
    assert not keep.any() and count[0] == 0
    np.testing.assert_allclose(tau3[0], 0.5 - 1e-3 * 0.25 + 1999 * 1e-3 * 0.75, rtol=1e-4)
    # negative feedback: on exchangeable scores the achieved skip fraction settles at the target
    for target in (0.25, 0.5, 0.75):
        keep, _, count, _ = oracle.select_online(S, target, 0.05, 0.5, 16)
        frac = 1.0 - count / n
        assert np.all(np.abs(frac - target) <= 0.02), frac
    # rows are independent
    k1, i1, c1, t1 = oracle.select_online(S[1:2], 0.5, 0.05, 0.5, 16)
    kk, ii, cc, tt = oracle.select_online(S, 0.5, 0.05, 0.5, 16)
    np.testing.assert_array_equal(k1[0], kk[1])
    assert c1[0] == cc[1] and t1[0] == tt[1]


# ------------------------------------------------------------------ attention

def _sdpa(q, k, v, **kw):
    return torch.nn.functional.scaled_dot_product_attention(q.double(), k.double(), v.double(), **kw)


def test_attention_ratio_zero_is_dense_causal_sdpa():
    q, k, v, _ = synth.make_random_qkv(2, 4, 4, 24, 16, seed=19)
    idx = np.tile(np.arange(24, dtype=np.int32), (2, 1))
    O = oracle.attend(q, k, v, idx)
    ref = _sdpa(q, k, v, is_causal=True).numpy()
    np.testing.assert_allclose(O, ref, rtol=0, atol=1e-12)


def test_attention_gqa_head_map_vs_sdpa():
    q, k, v, _ = synth.make_random_qkv(1, 6, 2, 20, 8, seed=23)
    idx = np.arange(20, dtype=np.int32)[None]
    O = oracle.attend(q, k, v, idx)
    ref = _sdpa(q, k.repeat_interleave(3, 1), v.repeat_interleave(3, 1), is_causal=True).numpy()
    np.testing.assert_allclose(O, ref, rtol=0, atol=1e-12)


def test_filtered_attention_equals_compacted_dense_and_masked_dense():
    q, k, v, _ = synth.make_random_qkv(2, 4, 2, 30, 8, seed=29)
    res = oracle.filtered_attention(q, k, v, 0.4, warmup=1)
    O, idx, keep = res["O"], res["kept_idx"], res["keep"]
    n = 30
    for b in range(2):
        ii = torch.from_numpy(idx[b].astype(np.int64))
        kr, vr = k.repeat_interleave(2, 1), v.repeat_interleave(2, 1)
        # (i) dense causal attention on the physically compacted tensors
        ref = _sdpa(q[b:b + 1, :, ii], kr[b:b + 1, :, ii], vr[b:b + 1, :, ii], is_causal=True)[0].numpy()
        np.testing.assert_allclose(O[b][:, idx[b]], ref, rtol=0, atol=1e-12)
        # (ii) dense attention with filtered key columns masked out
        mask = torch.tril(torch.ones(n, n, dtype=torch.bool)) & torch.from_numpy(keep[b].astype(bool))[None, :]
        mask[:, 0] |= ~mask.any(1)                            # keep fully-masked rows finite
        ref2 = _sdpa(q[b:b + 1], kr[b:b + 1], vr[b:b + 1], attn_mask=mask)[0].numpy()
        np.testing.assert_allclose(O[b][:, idx[b]], ref2[:, idx[b]], rtol=0, atol=1e-12)
        filt = np.nonzero(keep[b] == 0)[0]
        assert len(filt) and np.all(O[b][:, filt] == 0.0)     # filtered rows exactly zero
        # first kept row attends only itself: output is its own V row
        np.testing.assert_allclose(O[b][:, idx[b][0]], vr[b, :, idx[b][0]].double().numpy(), atol=1e-15)
        # every output row is a convex combination of kept V rows
        vk = vr[b][:, ii].double().numpy()
        assert np.all(O[b][:, idx[b]] <= vk.max(1, keepdims=True) + 1e-12)
        assert np.all(O[b][:, idx[b]] >= vk.min(1, keepdims=True) - 1e-12)


def test_attention_softmax_scale_and_rows_entry():
    q, k, v, _ = synth.make_random_qkv(1, 2, 2, 16, 8, seed=31)
    idx = np.array([[0, 2, 3, 7, 8, 12, 15]], dtype=np.int32)
    O = oracle.attend(q, k, v, idx, scale=0.7)
    ii = torch.from_numpy(idx[0].astype(np.int64))
    ref = _sdpa(q[:, :, ii], k[:, :, ii], v[:, :, ii], is_causal=True, scale=0.7)[0].numpy()
    np.testing.assert_allclose(O[0][:, idx[0]], ref, rtol=0, atol=1e-12)
    rows = np.array([[0, 0, 0], [0, 1, 6], [0, 0, 3]], dtype=np.int32)
    got = oracle.attend_rows(q, k, v, idx, rows, scale=0.7)
    for r, (b, h, i) in enumerate(rows):
        np.testing.assert_array_equal(got[r], O[b, h, idx[b, i]])


def test_uniform_attention_closed_form():
    # all-zero queries: softmax is uniform, so row i is the running mean of the kept V rows
    q, k, v, _ = synth.make_random_qkv(1, 1, 1, 12, 4, seed=37)
    idx = np.array([[1, 4, 5, 9]], dtype=np.int32)
    O = oracle.attend(torch.zeros_like(q), k, v, idx)
    vk = v[0, 0, idx[0].astype(np.int64)].double().numpy()
    for i in range(4):
        np.testing.assert_allclose(O[0, 0, idx[0, i]], vk[:i + 1].mean(0), atol=1e-15)


# ------------------------------------------------------------------ whole path on workload 1

def test_whole_path_on_first_workload():
    w = synth.workload(0)
    q, k, v, z = synth.make_qkv(w)
    res = oracle.filtered_attention(q, k, v, 0.5, with_attention=False)
    m = oracle.keep_count(w.seq, 0.5)
    assert m == math.ceil(0.5 * w.seq) == res["kept_idx"].shape[1]
    assert res["keep"].sum() == m * w.batch
    assert res["keep"][0, 0] == 1                             # warm-up token
    assert np.all(np.abs(res["fused"]) <= 1.0)
    # the recipe's point: a token whose identity was seen often scores higher (is more
    # redundant) on average than one seen for the first time
    S = res["fused"][0]
    zz = z[0].numpy()
    first = np.zeros(w.seq, dtype=bool)
    seen = set()
    for t, i in enumerate(zz):
        first[t] = i not in seen
        seen.add(i)
    assert S[~first][10:].mean() > S[first][1:].mean()


# ------------------------------------------------------------------ per-token (decoding) form

def _run_decode(q, k, v, **kw):
    B, Hq, n, d = q.shape
    st = oracle.DecodeState(B, Hq, k.shape[1], d, kw.pop("capacity", n), **kw)
    F, S, O = [], [], []
    for t in range(n):
        o, s, f = st.step(q[:, :, t], k[:, :, t], v[:, :, t])
        F.append(f), S.append(s), O.append(o)
    return st, np.stack(F, 1), np.stack(S, 1), np.stack(O, 2)


def test_decode_step_hand_worked_three_tokens():
    # one head, d = 2, K = V: the scores are plain cosines with the mean of the rows before
    # (one head: both variances are zero, alpha = 1/2, S = (s_k + s_v) / 2 = the cosine).
    # Fixed threshold 0.5 (eta = 0), warm-up 1: token 0 kept; token 1 repeats token 0 (S = 1):
    # skipped, zero output, not cached; token 2 is orthogonal to the mean (S = 0): kept, and it
    # sees a cache of tokens 0 and 2 only.
    x = np.array([[1, 0], [1, 0], [0, 1]], dtype=np.float32).reshape(1, 1, 3, 2)
    L = 3.0
    q = np.array([[0, 0], [5, 5], [0, L]], dtype=np.float32).reshape(1, 1, 3, 2)
    st, F, S, O = _run_decode(q, x, x, target=0.5, eta=0.0, tau0=0.5, warmup=1)
    np.testing.assert_allclose(F[0], [0, 1, 0], atol=1e-15)
    assert list(S[0]) == [0, 1, 0]
    assert st.seen[0] == 3 and st.skipped[0] == 1 and st.cache_len[0] == 2 and st.tau[0] == np.float32(0.5)
    np.testing.assert_array_equal(st.k_cache[0, 0, :2], [[1, 0], [0, 1]])
    np.testing.assert_allclose(st.anchor_k[0, 0], [2, 1])           # sums of ALL rows seen
    np.testing.assert_allclose(O[0, 0, 0], [1, 0], atol=1e-15)      # alone in the cache
    np.testing.assert_array_equal(O[0, 0, 1], [0, 0])
    w2 = math.exp(L / math.sqrt(2)) / (1 + math.exp(L / math.sqrt(2)))
    np.testing.assert_allclose(O[0, 0, 2], [1 - w2, w2], rtol=1e-14)


@pytest.mark.parametrize("gamma,mode,hq,hkv", [(None, oracle.FUSE_EQ2, 4, 4), (0.9, oracle.FUSE_INVVAR, 6, 2),
                                               (None, oracle.FUSE_KEY_ONLY, 2, 1), (0.5, oracle.FUSE_EQ2, 8, 4)])
def test_decode_steps_reduce_to_the_batched_path(gamma, mode, hq, hkv):
    # token by token = the batched definitions on the whole sequence: anchor cosines + fusion,
    # the online decision on those scores, attention among the kept tokens
    rng = np.random.default_rng(31)
    B, n, d = 3, 90, 16
    proto = rng.normal(size=(5, d))
    z = rng.integers(0, 5, size=(B, 1, n))
    k = (proto[z] + 0.4 * rng.normal(size=(B, hkv, n, d))).astype(np.float32)
    v = (proto[z][..., ::-1] + 0.4 * rng.normal(size=(B, hkv, n, d))).astype(np.float32)
    q = rng.normal(size=(B, hq, n, d)).astype(np.float32)
    W, target, eta, tau0 = 3, 0.4, 0.05, 0.2
    st, F, S, O = _run_decode(q, k, v, target=target, eta=eta, tau0=tau0, warmup=W, mode=mode,
                              ema_gamma=gamma, scale=0.3)
    cos = (lambda x: oracle.anchor_cosine(x)) if gamma is None else (lambda x: oracle.anchor_cosine_ema(x, gamma))
    fb = oracle.fuse(cos(k), cos(v), mode)
    np.testing.assert_allclose(F, fb, rtol=1e-12, atol=1e-14)
    keep, idx, cnt, tau = oracle.select_online(fb, target, eta, tau0, W)
    np.testing.assert_array_equal(S, 1 - keep)
    assert 0 < (keep == 0).sum() < keep.size                 # both branches taken
    np.testing.assert_array_equal(st.cache_len, cnt)
    np.testing.assert_array_equal(st.seen, n)
    np.testing.assert_array_equal(st.skipped, n - cnt)
    np.testing.assert_array_equal(st.tau, tau)
    for b in range(B):
        np.testing.assert_array_equal(st.k_cache[b, :, :cnt[b]], k[b][:, idx[b, :cnt[b]]])
        np.testing.assert_array_equal(st.v_cache[b, :, :cnt[b]], v[b][:, idx[b, :cnt[b]]])
    rows = np.array([(b, h, i) for b in range(B) for h in range(hq) for i in range(cnt[b])], dtype=np.int32)
    ref = oracle.attend_rows(q, k, v, idx, rows, scale=0.3)
    got = np.stack([O[b, h, idx[b, i]] for b, h, i in rows])
    np.testing.assert_allclose(got, ref, rtol=1e-12, atol=1e-14)
    assert np.all(O[np.broadcast_to((keep == 0)[:, None, :, None], O.shape)] == 0)


def test_decode_step_forced_decisions_and_full_cache():
    rng = np.random.default_rng(32)
    B, H, d = 2, 2, 8
    st = oracle.DecodeState(B, H, H, d, 2, target=0.5, eta=0.0, tau0=0.0, warmup=0)
    x = lambda: rng.normal(size=(B, H, d)).astype(np.float32)
    # the decision follows the scores handed in, not the ones computed: row 0 kept, row 1 skipped
    o, skip, fused = st.step(x(), x(), x(), decide_on=np.array([-1.0, 1.0], dtype=np.float32))
    assert list(skip) == [0, 1] and list(st.cache_len) == [1, 0] and np.all(o[1] == 0) and np.any(o[0] != 0)
    st.step(x(), x(), x(), decide_on=np.array([-1.0, 1.0], dtype=np.float32))
    before = (st.anchor_k.copy(), st.seen.copy(), st.tau.copy(), st.cache_len.copy(), st.k_cache.copy())
    with pytest.raises(OverflowError):                       # row 0's cache holds 2 rows already
        st.step(x(), x(), x(), decide_on=np.array([-1.0, 1.0], dtype=np.float32))
    for a, b in zip(before, (st.anchor_k, st.seen, st.tau, st.cache_len, st.k_cache)):
        np.testing.assert_array_equal(a, b)
    # a skipped token leaves no trace in what later tokens attend to: the output of a kept
    # token is the softmax average of the cached values only
    st2 = oracle.DecodeState(1, 1, 1, 2, 4, target=0.5, eta=0.0, tau0=0.0, warmup=0, scale=1.0)
    one = lambda a, b: np.array([[[a, b]]], dtype=np.float32)
    st2.step(one(0, 0), one(1, 0), one(10, 0), decide_on=np.array([-1.0], dtype=np.float32))
    st2.step(one(0, 0), one(0, 9), one(0, 99), decide_on=np.array([1.0], dtype=np.float32))
    o, _, _ = st2.step(one(0, 0), one(0, 1), one(0, 20), decide_on=np.array([-1.0], dtype=np.float32))
    np.testing.assert_allclose(o[0, 0], [5, 10], rtol=1e-14)   # zero query: uniform over 2 rows


# ------------------------------------------------------------------ anchor that includes the token

def test_inclusive_anchor_closed_forms_and_brute_force():
    # x0 = (3, 4), x1 = (4, 3): the mean of both is (3.5, 3.5); cos with x1 = 24.5 / (sqrt(24.5) * 5)
    x = np.array([[3.0, 4.0], [4.0, 3.0]], dtype=np.float32).reshape(1, 1, 2, 2)
    c, a = oracle.anchor_cosine(x, return_anchors=True, inclusive=True)
    np.testing.assert_array_equal(a[0, 0], [[3, 4], [3.5, 3.5]])
    assert c[0, 0, 0] == 1.0                                   # a token against itself
    assert abs(c[0, 0, 1] - math.sqrt(24.5) / 5) < 1e-15
    # incremental anchor, gamma = 1/2, from zero: A0 = x0 / 2 (cos 1), A1 = x0 / 4 + x1 / 2 = (2.75, 2.5)
    c, a = oracle.anchor_cosine_ema(x, 0.5, return_anchors=True, inclusive=True)
    np.testing.assert_array_equal(a[0, 0], [[1.5, 2.0], [2.75, 2.5]])
    assert abs(c[0, 0, 0] - 1.0) < 1e-15
    assert abs(c[0, 0, 1] - 18.5 / (math.sqrt(2.75 ** 2 + 2.5 ** 2) * 5)) < 1e-15
    # brute force on random rows, both kinds
    rng = np.random.default_rng(41)
    xr = rng.normal(size=(2, 3, 25, 6)).astype(np.float32)
    xd = xr.astype(np.float64)
    c, a = oracle.anchor_cosine(xr, return_anchors=True, inclusive=True)
    ce, ae = oracle.anchor_cosine_ema(xr, 0.8, return_anchors=True, inclusive=True)
    for t in range(25):
        ref = xd[:, :, :t + 1].mean(axis=2)
        np.testing.assert_allclose(a[:, :, t], ref, rtol=1e-13, atol=1e-15)
        cs = (ref * xd[:, :, t]).sum(-1) / (np.linalg.norm(ref, axis=-1) * np.linalg.norm(xd[:, :, t], axis=-1))
        np.testing.assert_allclose(c[:, :, t], cs, rtol=1e-12)
        w = 0.2 * 0.8 ** (t - np.arange(t + 1))
        refe = np.einsum("j,bhjd->bhd", w, xd[:, :, :t + 1])
        np.testing.assert_allclose(ae[:, :, t], refe, rtol=1e-12, atol=1e-15)
        cse = (refe * xd[:, :, t]).sum(-1) / (np.linalg.norm(refe, axis=-1) * np.linalg.norm(xd[:, :, t], axis=-1))
        np.testing.assert_allclose(ce[:, :, t], cse, rtol=1e-12)
    # the inclusive anchor of token t is the exclusive anchor of token t + 1
    _, ax = oracle.anchor_cosine(xr, return_anchors=True)
    np.testing.assert_allclose(a[:, :, :-1], ax[:, :, 1:], rtol=1e-14, atol=1e-16)
    _, axe = oracle.anchor_cosine_ema(xr, 0.8, return_anchors=True)
    np.testing.assert_allclose(ae[:, :, :-1], axe[:, :, 1:], rtol=1e-14, atol=1e-16)
    # a zero row still scores 0 through the guard; including the token raises the score of a
    # token that differs from its past
    z = np.zeros((1, 1, 3, 4), dtype=np.float32)
    z[0, 0, 0] = [1, 0, 0, 0]
    assert oracle.anchor_cosine(z, inclusive=True)[0, 0, 1] == 0
    assert np.all(c[:, :, 1:] > oracle.anchor_cosine(xr)[:, :, 1:])


def test_inclusive_decode_steps_reduce_to_the_batched_scores():
    rng = np.random.default_rng(42)
    B, H, n, d = 2, 3, 40, 8
    k = rng.normal(size=(B, H, n, d)).astype(np.float32) + 0.5
    v = rng.normal(size=(B, H, n, d)).astype(np.float32) - 0.5
    q = rng.normal(size=(B, H, n, d)).astype(np.float32)
    for gamma in (None, 0.7):
        st = oracle.DecodeState(B, H, H, d, n, 0.5, 0.05, 0.9, 2, ema_gamma=gamma, inclusive=True)
        F = np.stack([st.step(q[:, :, t], k[:, :, t], v[:, :, t])[2] for t in range(n)], 1)
        cos = (lambda x: oracle.anchor_cosine(x, inclusive=True)) if gamma is None else \
              (lambda x: oracle.anchor_cosine_ema(x, gamma, inclusive=True))
        np.testing.assert_allclose(F, oracle.fuse(cos(k), cos(v)), rtol=1e-12, atol=1e-14)
        # the state itself does not depend on the flag
        st0 = oracle.DecodeState(B, H, H, d, n, 0.5, 0.0, 9.0, 2, ema_gamma=gamma)
        st1 = oracle.DecodeState(B, H, H, d, n, 0.5, 0.0, 9.0, 2, ema_gamma=gamma, inclusive=True)
        for t in range(5):
            st0.step(q[:, :, t], k[:, :, t], v[:, :, t])
            st1.step(q[:, :, t], k[:, :, t], v[:, :, t])
        np.testing.assert_array_equal(st0.anchor_k, st1.anchor_k)


def test_anchor_state_footprint_matches_the_papers_figure():
    # Section 3.2: one anchor key and one anchor value per layer, one vector per head, about
    # 800 KB in total.  LLaMA-2-13B (40 layers, 40 heads of 128) in 16-bit storage:
    assert 2 * 40 * 40 * 128 * 2 == 800 * 1024
    # the per-layer state of the per-token form has exactly that structure (per batch row)
    st = oracle.DecodeState(1, 40, 40, 128, 4, 0.5, 0.02, 0.5)
    assert st.anchor_k.shape == st.anchor_v.shape == (1, 40, 128)
    assert 40 * (st.anchor_k.size + st.anchor_v.size) * 2 == 800 * 1024
