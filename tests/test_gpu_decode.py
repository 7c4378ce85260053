"""Parity of the per-token (decoding) entry points with the CPU oracle, through the C ABI.

The GPU runs a whole sequence token by token; the oracle then replays it step by step.  The
oracle takes each decision on the GPU's score of that step (the threshold recurrence feeds its
own decisions back, so a last-bit difference in a score that sits on the threshold would
otherwise change everything after it); scores themselves are compared to the usual bound
|gpu - oracle| <= 1e-5 |oracle| + 1e-6, decisions, counters, thresholds and cache contents bit
for bit, attention outputs to 1e-4 (fp32) / 2e-2 (bf16).
"""
import numpy as np
import pytest
import torch

import oracle
from paper_2512_07090_amd import binding as B
from paper_2512_07090_amd import synth

pytestmark = pytest.mark.gpu

ATTN_TOL = {torch.float32: 1e-4, torch.bfloat16: 2e-2}


@pytest.fixture(scope="module")
def ctx():
    assert torch.cuda.is_available(), "these tests need the MI355X"
    c = B.Context(0)
    yield c
    c.close()


def _say(msg):
    print("[case] " + msg, flush=True)


def gpu_decode(ctx, q, k, v, target, eta, tau0, W, capacity, fusion=B.TF_FUSE_EQ2, scale=0.0,
               ema_gamma=None, alloc_capacity=None, inclusive=False):
    """All n tokens through tf_decode_step.  Returns (buffers, O [n,B,Hq,d], skip [n,B], fused [n,B])."""
    Bn, Hq, n, d = q.shape
    p = B.make_params(tuple(q.shape), tuple(k.shape), q.dtype, target, W, fusion, scale,
                      ema_gamma=ema_gamma, anchor_inclusive=inclusive)
    buf = B.DecodeBuffers(p, alloc_capacity or capacity)
    buf.state.capacity = capacity
    buf.k_cache.fill_(-77.0)
    buf.v_cache.fill_(-77.0)
    qs = q.permute(2, 0, 1, 3).contiguous().cuda()        # [n][B][H][d]: one contiguous slice per step
    ks = k.permute(2, 0, 1, 3).contiguous().cuda()
    vs = v.permute(2, 0, 1, 3).contiguous().cuda()
    O = torch.full((n, Bn, Hq, d), float("nan"), dtype=q.dtype, device="cuda:0")
    skip = torch.full((n, Bn), 9, dtype=torch.uint8, device="cuda:0")
    fused = torch.full((n, Bn), float("nan"), dtype=torch.float32, device="cuda:0")
    ctx.tf_decode_init(p, buf.state, tau0)
    for t in range(n):
        ctx.tf_decode_step(p, eta, buf.state, qs[t], ks[t], vs[t], O[t], skip[t], fused[t], buf.ws)
    torch.cuda.synchronize()
    return buf, O.float().cpu().numpy().astype(np.float64), skip.cpu().numpy(), fused.cpu().numpy()


def check_decode(ctx, q, k, v, target, eta, tau0, W, fusion=B.TF_FUSE_EQ2, scale=0.0,
                 ema_gamma=None, capacity=None, inclusive=False):
    Bn, Hq, n, d = q.shape
    Hkv = k.shape[1]
    capacity = capacity or n
    g32 = None if ema_gamma is None else float(np.float32(ema_gamma))   # the value the library sees
    buf, O_g, skip_g, fused_g = gpu_decode(ctx, q, k, v, target, eta, tau0, W, capacity, fusion,
                                           scale, ema_gamma, inclusive=inclusive)
    assert not np.isnan(O_g).any() and not np.isnan(fused_g).any() and skip_g.max() <= 1
    st = oracle.DecodeState(Bn, Hq, Hkv, d, capacity, target, eta, tau0, W, fusion, scale, g32,
                            inclusive=inclusive)
    qf, kf, vf = q.float().numpy(), k.float().numpy(), v.float().numpy()
    worst = 0.0
    for t in range(n):
        o_r, skip_r, fused_r = st.step(qf[:, :, t], kf[:, :, t], vf[:, :, t], decide_on=fused_g[t])
        assert np.all(np.abs(fused_g[t] - fused_r) <= 1e-5 * np.abs(fused_r) + 1e-6), "score, token %d" % t
        np.testing.assert_array_equal(skip_g[t], skip_r, err_msg="decision, token %d" % t)
        worst = max(worst, np.abs(O_g[t] - o_r).max())
        assert np.all(O_g[t][skip_r == 1] == 0)
    assert worst <= ATTN_TOL[q.dtype], "attention output, worst %.3e" % worst
    for name in ("seen", "skipped", "cache_len", "tau"):
        np.testing.assert_array_equal(getattr(buf, name).cpu().numpy(), getattr(st, name), err_msg=name)
    assert np.all(buf.overflow.cpu().numpy() == 0)
    kc, vc = buf.k_cache.float().cpu().numpy(), buf.v_cache.float().cpu().numpy()
    for b in range(Bn):
        c = int(st.cache_len[b])
        np.testing.assert_array_equal(kc[b, :, :c], st.k_cache[b, :, :c])
        np.testing.assert_array_equal(vc[b, :, :c], st.v_cache[b, :, :c])
        assert np.all(kc[b, :, c:] == -77.0) and np.all(vc[b, :, c:] == -77.0)   # nothing past the end
    np.testing.assert_allclose(buf.anchor_k.cpu().numpy(), st.anchor_k, rtol=1e-12, atol=1e-13)
    np.testing.assert_allclose(buf.anchor_v.cpu().numpy(), st.anchor_v, rtol=1e-12, atol=1e-13)
    return skip_g


@pytest.mark.parametrize("case", [
    # (dtype, B, Hq, Hkv, n, target, eta, tau0, W, fusion, gamma, scale)
    ("f32", 2, 4, 4, 300, 0.5, 0.05, 0.5, 4, B.TF_FUSE_EQ2, None, 0.0),
    ("bf16", 3, 8, 2, 700, 0.5, 0.02, 0.5, 8, B.TF_FUSE_INVVAR, 0.9, 0.0),
    ("bf16", 2, 6, 2, 200, 0.3, 0.05, 0.4, 1, B.TF_FUSE_EQ2, None, 0.11),     # 3 query heads per KV head
    ("bf16", 1, 8, 1, 150, 0.6, 0.1, 0.3, 0, B.TF_FUSE_KEY_ONLY, None, 0.0),  # 8 per KV head
    ("f32", 1, 4, 2, 130, 0.5, 0.05, 0.5, 2, B.TF_FUSE_VALUE_ONLY, 0.5, 0.0),
    ("bf16", 5, 2, 2, 40, 0.5, 0.0, 0.2, 3, B.TF_FUSE_EQ2, None, 0.0),        # fixed threshold, short
])
def test_decode_steps_match_oracle(ctx, case):
    dt, Bn, Hq, Hkv, n, target, eta, tau0, W, fusion, gamma, scale = case
    _say("decode %s" % (case,))
    w = synth.scaled(synth.workload(0), batch=Bn, seq=n, n_q_heads=Hq, n_kv_heads=Hkv, dtype=dt)
    q, k, v, _ = synth.make_qkv(w)
    skip = check_decode(ctx, q, k, v, target, eta, tau0, W, fusion, scale, gamma)
    if eta > 0:
        assert 0 < skip.sum() < skip.size                 # both branches were exercised


@pytest.mark.parametrize("gamma", [None, 0.9])
def test_decode_steps_anchor_including_the_token(ctx, gamma):
    _say("decode inclusive %s" % gamma)
    w = synth.scaled(synth.workload(0), batch=2, seq=250, n_q_heads=4, n_kv_heads=2, dtype="bf16")
    q, k, v, _ = synth.make_qkv(w)
    # scores are higher when the token is part of its own anchor: a higher starting threshold
    check_decode(ctx, q, k, v, 0.5, 0.05, 0.9, 4, ema_gamma=gamma, inclusive=True)


def test_decode_first_token_and_all_skipped_after_warmup(ctx):
    """Token 0 has no anchor (score 0); a threshold far below every score skips everything after
    the warm-up, so each row's cache holds exactly the warm-up tokens."""
    _say("decode warm-up only")
    q, k, v, _ = synth.make_random_qkv(2, 4, 4, 30, 128, dtype="bf16", seed=5)
    buf, O_g, skip_g, fused_g = gpu_decode(ctx, q, k, v, 0.5, 0.0, -5.0, 3, capacity=30)
    assert np.all(fused_g[0] == 0)
    assert np.all(skip_g[:3] == 0) and np.all(skip_g[3:] == 1)
    assert np.all(buf.cache_len.cpu().numpy() == 3) and np.all(buf.skipped.cpu().numpy() == 27)
    assert np.all(O_g[3:] == 0)
    # the first token attends to itself alone: its output is its value row
    np.testing.assert_array_equal(O_g[0], v[:, :, 0].float().numpy().astype(np.float64))


def test_decode_full_cache_sets_overflow_and_writes_nothing_past_it(ctx):
    _say("decode overflow")
    q, k, v, _ = synth.make_random_qkv(2, 2, 2, 12, 128, dtype="bf16", seed=6)
    # nothing is ever skipped by the rule (threshold far above); the cache takes 5 tokens
    buf, O_g, skip_g, fused_g = gpu_decode(ctx, q, k, v, 0.5, 0.0, 50.0, 1, capacity=5, alloc_capacity=9)
    assert np.all(skip_g[:5] == 0) and np.all(skip_g[5:] == 1)
    assert np.all(buf.overflow.cpu().numpy() == 1)
    assert np.all(buf.cache_len.cpu().numpy() == 5) and np.all(buf.seen.cpu().numpy() == 12)
    assert np.all(O_g[5:] == 0) and np.all(np.abs(O_g[:5]).max(axis=(1, 2, 3)) > 0)
    # the tensors were allocated with 9 rows per head and declared with 5: with that declared
    # row stride the first 2 * 2 * 5 rows may be written, nothing after them
    kc = buf.k_cache.float().cpu().numpy().reshape(-1, 128)
    assert np.all(kc[2 * 2 * 5:] == -77.0)


def test_decode_argument_errors(ctx):
    q, k, v, _ = synth.make_random_qkv(1, 2, 2, 4, 128, dtype="bf16", seed=7)
    p = B.make_params(tuple(q.shape), tuple(k.shape), q.dtype, 0.5)
    buf = B.DecodeBuffers(p, 4)
    ctx.tf_decode_init(p, buf.state, 0.5)
    qd = q[:, :, 0].contiguous().cuda()
    kd = k[:, :, 0].contiguous().cuda()
    with pytest.raises(B.TokfiltError):                   # workspace too small
        ctx.tf_decode_step(p, 0.1, buf.state, qd, kd, kd, buf.o, buf.skip, buf.fused, buf.ws[:16])
    with pytest.raises(B.TokfiltError):                   # negative step size
        ctx.tf_decode_step(p, -0.1, buf.state, qd, kd, kd, buf.o, buf.skip, buf.fused, buf.ws)
    bad = B.tf_decode_state.from_buffer_copy(buf.state)
    bad.capacity = 0
    with pytest.raises(B.TokfiltError):
        ctx.tf_decode_step(p, 0.1, bad, qd, kd, kd, buf.o, buf.skip, buf.fused, buf.ws)
    bad = B.tf_decode_state.from_buffer_copy(buf.state)
    bad.tau = None
    with pytest.raises(B.TokfiltError):
        ctx.tf_decode_init(p, bad, 0.5)
    torch.cuda.synchronize()
    assert np.all(buf.seen.cpu().numpy() == 0)            # nothing was enqueued by the failed calls


def test_decode_agrees_with_batched_online_path(ctx):
    """Token by token and all at once are the same computation: scores agree to the bound, and
    where the two masks coincide the outputs agree to twice the attention tolerance."""
    _say("decode vs batched online")
    w = synth.scaled(synth.workload(1), batch=2, seq=900, n_q_heads=8, n_kv_heads=8)
    q, k, v, _ = synth.make_qkv(w)
    target, eta, tau0, W = 0.5, 0.02, 0.5, 8
    buf, O_d, skip_d, fused_d = gpu_decode(ctx, q, k, v, target, eta, tau0, W, capacity=900)
    p = B.make_params(tuple(q.shape), tuple(k.shape), q.dtype, target, W)
    bb = B.Buffers(p, "cuda:0")
    idx = torch.empty((2, 900), dtype=torch.int32, device="cuda:0")
    cnt = torch.empty((2,), dtype=torch.int32, device="cuda:0")
    ctx.tf_filtered_attention_online(p, eta, tau0, q.cuda(), k.cuda(), v.cuda(), bb.keep, idx, cnt,
                                     bb.fused, bb.tau, bb.O, bb.ws)
    torch.cuda.synchronize()
    fused_b = bb.fused.cpu().numpy()
    assert np.all(np.abs(fused_d.T - fused_b) <= 2e-5 * np.abs(fused_b) + 2e-6)
    keep_b = bb.keep.cpu().numpy()
    O_b = bb.O.float().cpu().numpy()
    for b in range(2):
        if np.array_equal(keep_b[b], 1 - skip_d[:, b]):
            assert np.abs(O_d[:, b].transpose(1, 0, 2) - O_b[b]).max() <= 2 * ATTN_TOL[q.dtype]
            assert buf.tau.cpu().numpy()[b] == bb.tau.cpu().numpy()[b]


def test_decode_full_size_bench_shape(ctx):
    """The benchmark's shape (8 rows, 32 heads, bf16, 4096 tokens): every decision against the
    oracle's controller on the GPU's scores, the scores against the oracle's batched scoring,
    and sampled output rows against the oracle's attention over the kept set."""
    _say("decode full size")
    w = synth.workload(1)
    q, k, v, _ = synth.make_qkv(w)
    Bn, Hq, n, d = q.shape
    target, eta, tau0, W = 0.5, 0.02, 0.5, 8
    buf, O_g, skip_g, fused_g = gpu_decode(ctx, q, k, v, target, eta, tau0, W, capacity=n)
    ref = oracle.filtered_attention(q, k, v, target, W, with_attention=False)
    assert np.all(np.abs(fused_g.T - ref["fused"]) <= 1e-5 * np.abs(ref["fused"]) + 1e-6)
    keep_r, idx_r, cnt_r, tau_r = oracle.select_online(fused_g.T, target, eta, tau0, W)
    np.testing.assert_array_equal(1 - skip_g.T, keep_r)
    np.testing.assert_array_equal(buf.cache_len.cpu().numpy(), cnt_r)
    np.testing.assert_array_equal(buf.tau.cpu().numpy(), tau_r)
    assert np.all(buf.overflow.cpu().numpy() == 0)
    assert np.all(O_g[skip_g == 1] == 0)
    # end to end: against the oracle's decisions on the oracle's own scores, a row's masks are
    # equal or first part at a token whose oracle score sits on its threshold
    keep_o, _, _, _, trace = oracle.select_online(ref["fused"], target, eta, tau0, W, return_trace=True)
    s32 = ref["fused"].astype(np.float32).astype(np.float64)
    for b in range(Bn):
        diff = np.nonzero((1 - skip_g.T)[b] != keep_o[b])[0]
        if len(diff):
            t = int(diff[0])
            gap = abs(s32[b, t] - float(trace[b, t]))
            _say("  row %d parts from the oracle's own mask at token %d, |score - threshold| %.2e" % (b, t, gap))
            assert gap <= 1e-5, "row %d: first differing token %d is %.3e from its threshold" % (b, t, gap)
    rng = np.random.default_rng(3)
    rows = []
    for b in range(Bn):
        c = int(cnt_r[b])
        for i in (0, 1, 63, 64, c // 2, c - 2, c - 1):
            rows.append((b, int(rng.integers(Hq)), i))
        rows += [(b, int(rng.integers(Hq)), int(rng.integers(c))) for _ in range(9)]
    rows = np.array(rows, dtype=np.int32)
    want = oracle.attend_rows(q, k, v, idx_r, rows)
    got = np.stack([O_g[idx_r[b, i], b, h] for b, h, i in rows])
    assert np.abs(got - want).max() <= ATTN_TOL[q.dtype]
    # the cache of row 0, head 5 is the kept keys in order
    c0 = int(cnt_r[0])
    assert torch.equal(buf.k_cache[0, 5, :c0].cpu(), k[0, 5][torch.from_numpy(idx_r[0, :c0]).long()])


@pytest.mark.parametrize("case", [
    # (dtype, B, Hq, Hkv, prompt, decoded, gamma, fusion)
    ("bf16", 2, 8, 4, 600, 150, None, B.TF_FUSE_EQ2),
    ("f32", 1, 4, 4, 300, 60, 0.9, B.TF_FUSE_INVVAR),
    ("bf16", 3, 4, 2, 70, 30, 0.0, B.TF_FUSE_EQ2),          # gamma 0: the anchor is the previous row
    ("bf16", 1, 2, 2, 1, 40, None, B.TF_FUSE_EQ2),          # a prompt of one token
])
def test_prefill_then_decode_matches_oracle(ctx, case):
    """A prompt through the batched online path with the hand-off to the decoding state, then
    single steps: the oracle goes through all tokens one by one."""
    dt, Bn, Hq, Hkv, n1, n2, gamma, fusion = case
    _say("prefill + decode %s" % (case,))
    w = synth.scaled(synth.workload(0), batch=Bn, seq=n1 + n2, n_q_heads=Hq, n_kv_heads=Hkv, dtype=dt)
    q, k, v, _ = synth.make_qkv(w)
    target, eta, tau0, W = 0.5, 0.03, 0.5, 4
    d = q.shape[3]
    qp, kp, vp = (x[:, :, :n1].contiguous() for x in (q, k, v))
    p = B.make_params(tuple(qp.shape), tuple(kp.shape), q.dtype, target, W, fusion, ema_gamma=gamma)
    cap = n1 + n2
    buf = B.DecodeBuffers(p, cap)
    buf.k_cache.fill_(-77.0)
    buf.v_cache.fill_(-77.0)
    for t_ in (buf.seen, buf.skipped, buf.cache_len, buf.overflow):
        t_.fill_(-5)
    buf.anchor_k.fill_(float("nan"))
    buf.anchor_v.fill_(float("nan"))
    bb = B.Buffers(p, "cuda:0")
    bb.O.fill_(float("nan"))
    idx = torch.full((Bn, n1), -7, dtype=torch.int32, device="cuda:0")
    cnt = torch.zeros((Bn,), dtype=torch.int32, device="cuda:0")
    ctx.tf_decode_prefill(p, eta, tau0, buf.state, qp.cuda(), kp.cuda(), vp.cuda(), bb.keep, idx, cnt,
                          bb.fused, bb.O, bb.ws)
    torch.cuda.synchronize()
    after_prefill = {name: getattr(buf, name).cpu().numpy().copy()
                     for name in ("seen", "skipped", "cache_len", "tau", "overflow", "anchor_k", "anchor_v")}
    qs = q[:, :, n1:].permute(2, 0, 1, 3).contiguous().cuda()
    ks = k[:, :, n1:].permute(2, 0, 1, 3).contiguous().cuda()
    vs = v[:, :, n1:].permute(2, 0, 1, 3).contiguous().cuda()
    O2 = torch.full((n2, Bn, Hq, d), float("nan"), dtype=q.dtype, device="cuda:0")
    skip2 = torch.full((n2, Bn), 9, dtype=torch.uint8, device="cuda:0")
    fused2 = torch.full((n2, Bn), float("nan"), dtype=torch.float32, device="cuda:0")
    for t in range(n2):
        ctx.tf_decode_step(p, eta, buf.state, qs[t], ks[t], vs[t], O2[t], skip2[t], fused2[t], buf.ws)
    torch.cuda.synchronize()

    fused1 = bb.fused.cpu().numpy()
    keep1 = bb.keep.cpu().numpy()
    O1 = bb.O.float().cpu().numpy().astype(np.float64)
    O2n, skip2n, fused2n = O2.float().cpu().numpy().astype(np.float64), skip2.cpu().numpy(), fused2.cpu().numpy()
    g32 = None if gamma is None else float(np.float32(gamma))
    st = oracle.DecodeState(Bn, Hq, Hkv, d, cap, target, eta, tau0, W, fusion, 0.0, g32)
    qf, kf, vf = q.float().numpy(), k.float().numpy(), v.float().numpy()
    tol = ATTN_TOL[q.dtype]
    for t in range(n1 + n2):
        gpu_fused = fused1[:, t] if t < n1 else fused2n[t - n1]
        o_r, skip_r, fused_r = st.step(qf[:, :, t], kf[:, :, t], vf[:, :, t], decide_on=gpu_fused)
        assert np.all(np.abs(gpu_fused - fused_r) <= 1e-5 * np.abs(fused_r) + 1e-6), "score, token %d" % t
        if t < n1:
            np.testing.assert_array_equal(1 - keep1[:, t], skip_r, err_msg="prompt decision, token %d" % t)
            assert np.abs(O1[:, :, t] - o_r).max() <= tol, "prompt output, token %d" % t
        else:
            np.testing.assert_array_equal(skip2n[t - n1], skip_r, err_msg="decision, token %d" % t)
            assert np.abs(O2n[t - n1] - o_r).max() <= tol, "output, token %d" % t
        if t == n1 - 1:                                    # the state the hand-off must have produced
            for name in ("seen", "skipped", "cache_len", "tau"):
                np.testing.assert_array_equal(after_prefill[name], getattr(st, name), err_msg=name)
            assert np.all(after_prefill["overflow"] == 0)
            np.testing.assert_allclose(after_prefill["anchor_k"], st.anchor_k, rtol=1e-11, atol=1e-12)
            np.testing.assert_allclose(after_prefill["anchor_v"], st.anchor_v, rtol=1e-11, atol=1e-12)
    for name in ("seen", "skipped", "cache_len", "tau"):
        np.testing.assert_array_equal(getattr(buf, name).cpu().numpy(), getattr(st, name), err_msg=name)
    kc, vc = buf.k_cache.float().cpu().numpy(), buf.v_cache.float().cpu().numpy()
    for b in range(Bn):
        c = int(st.cache_len[b])
        np.testing.assert_array_equal(kc[b, :, :c], st.k_cache[b, :, :c])
        np.testing.assert_array_equal(vc[b, :, :c], st.v_cache[b, :, :c])
        assert np.all(kc[b, :, c:] == -77.0) and np.all(vc[b, :, c:] == -77.0)


def test_prefill_rejects_caches_shorter_than_the_prompt(ctx):
    q, k, v, _ = synth.make_random_qkv(1, 2, 2, 64, 128, dtype="bf16", seed=8)
    p = B.make_params(tuple(q.shape), tuple(k.shape), q.dtype, 0.5)
    buf = B.DecodeBuffers(p, 63)
    bb = B.Buffers(p, "cuda:0")
    idx = torch.empty((1, 64), dtype=torch.int32, device="cuda:0")
    cnt = torch.empty((1,), dtype=torch.int32, device="cuda:0")
    with pytest.raises(B.TokfiltError):
        ctx.tf_decode_prefill(p, 0.02, 0.5, buf.state, q.cuda(), k.cuda(), v.cuda(), bb.keep, idx, cnt,
                              bb.fused, bb.O, bb.ws)


@pytest.mark.parametrize("dt", ["bf16", "f32"])
def test_prefill_strided_layout_equals_contiguous(ctx, dt):
    """[B, n, H, d] storage of the prompt through the stride arguments: identical outputs, the
    same decoding state, and the same next decoding step as with [B, H, n, d] storage."""
    _say("prefill strided %s" % dt)
    Bn, Hq, Hkv, n, d = 2, 4, 2, 333, 128
    q, k, v, _ = synth.make_random_qkv(Bn, Hq, Hkv, n + 1, d, dtype=dt, seed=77)
    eta, tau0 = 0.05, 0.1
    results = []
    for strided in (False, True):
        qp, kp, vp = (x[:, :, :n].contiguous() for x in (q, k, v))
        if strided:
            qd, kd, vd = (x.permute(0, 2, 1, 3).contiguous().cuda() for x in (qp, kp, vp))
            p = B.make_params(tuple(qp.shape), tuple(kp.shape), q.dtype, 0.5, 2, ema_gamma=0.9,
                              q_stride=(n * Hq * d, d, Hq * d), kv_stride=(n * Hkv * d, d, Hkv * d),
                              o_stride=(n * Hq * d, d, Hq * d))
            O = torch.empty((Bn, n, Hq, d), dtype=q.dtype, device="cuda:0")
        else:
            qd, kd, vd = qp.cuda(), kp.cuda(), vp.cuda()
            p = B.make_params(tuple(qp.shape), tuple(kp.shape), q.dtype, 0.5, 2, ema_gamma=0.9)
            O = torch.empty((Bn, Hq, n, d), dtype=q.dtype, device="cuda:0")
        buf = B.DecodeBuffers(p, n + 1)
        bb = B.Buffers(p, "cuda:0")
        idx = torch.full((Bn, n), -7, dtype=torch.int32, device="cuda:0")
        cnt = torch.zeros((Bn,), dtype=torch.int32, device="cuda:0")
        ctx.tf_decode_prefill(p, eta, tau0, buf.state, qd, kd, vd, bb.keep, idx, cnt, bb.fused, O, bb.ws)
        ctx.tf_decode_step(p, eta, buf.state, q[:, :, n].contiguous().cuda(), k[:, :, n].contiguous().cuda(),
                           v[:, :, n].contiguous().cuda(), buf.o, buf.skip, buf.fused, buf.ws)
        torch.cuda.synchronize()
        c = cnt.cpu()
        clen = buf.cache_len.cpu()                         # after the decoded token
        results.append(dict(
            O=(O.permute(0, 2, 1, 3) if strided else O).cpu(), keep=bb.keep.cpu(), fused=bb.fused.cpu(),
            cnt=c, tau=buf.tau.cpu(), anchor_k=buf.anchor_k.cpu(), anchor_v=buf.anchor_v.cpu(),
            clen=clen,
            kc=[buf.k_cache[b, :, :int(clen[b])].cpu() for b in range(Bn)],
            vc=[buf.v_cache[b, :, :int(clen[b])].cpu() for b in range(Bn)],
            o=buf.o.cpu(), skip=buf.skip.cpu(), f1=buf.fused.cpu(), seen=buf.seen.cpu()))
    a, b_ = results
    for name in ("O", "keep", "fused", "cnt", "clen", "tau", "anchor_k", "anchor_v", "o", "skip", "f1", "seen"):
        assert torch.equal(a[name], b_[name]), name
    for x, y in zip(a["kc"] + a["vc"], b_["kc"] + b_["vc"]):
        assert torch.equal(x, y)
    assert 0 < int(a["cnt"].sum()) < Bn * n


def test_decode_step_replays_from_a_captured_graph(ctx):
    """tf_decode_step allocates nothing and never synchronises: one captured step, replayed once
    per token with the token copied into fixed input buffers, must give what the eager loop
    gives, bit for bit (the serving pattern: one graph launch per token)."""
    _say("decode graph replay")
    w = synth.scaled(synth.workload(0), batch=2, seq=120, n_q_heads=8, n_kv_heads=4, dtype="bf16")
    q, k, v, _ = synth.make_qkv(w)
    Bn, Hq, n, d = q.shape
    target, eta, tau0, W = 0.5, 0.05, 0.5, 4
    buf_e, O_e, skip_e, fused_e = gpu_decode(ctx, q, k, v, target, eta, tau0, W, capacity=n)

    p = B.make_params(tuple(q.shape), tuple(k.shape), q.dtype, target, W)
    buf = B.DecodeBuffers(p, n)
    qs = q.permute(2, 0, 1, 3).contiguous().cuda()
    ks = k.permute(2, 0, 1, 3).contiguous().cuda()
    vs = v.permute(2, 0, 1, 3).contiguous().cuda()
    q_in, k_in, v_in = torch.empty_like(qs[0]), torch.empty_like(ks[0]), torch.empty_like(vs[0])

    def step():
        ctx.tf_decode_step(p, eta, buf.state, q_in, k_in, v_in, buf.o, buf.skip, buf.fused, buf.ws)
    # warm the call on a side stream (as capture requires), then start the sequence afresh
    ctx.tf_decode_init(p, buf.state, tau0)
    q_in.copy_(qs[0]); k_in.copy_(ks[0]); v_in.copy_(vs[0])
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):
        step()
    torch.cuda.current_stream().wait_stream(side)
    g = torch.cuda.CUDAGraph()
    with torch.cuda.graph(g):
        step()
    ctx.tf_decode_init(p, buf.state, tau0)
    torch.cuda.synchronize()
    for t in range(n):
        q_in.copy_(qs[t]); k_in.copy_(ks[t]); v_in.copy_(vs[t])
        buf.ws.fill_(0xFF)                                   # stale partial results
        g.replay()
        torch.cuda.synchronize()
        assert np.array_equal(buf.skip.cpu().numpy(), skip_e[t]), "decision, token %d" % t
        assert np.array_equal(buf.fused.cpu().numpy(), fused_e[t]), "score, token %d" % t
        assert np.array_equal(buf.o.float().cpu().numpy().astype(np.float64), O_e[t]), "output, token %d" % t
    for name in ("seen", "skipped", "cache_len", "tau", "anchor_k", "anchor_v"):
        assert torch.equal(getattr(buf, name), getattr(buf_e, name)), name
    for b in range(Bn):
        c = int(buf.cache_len[b])
        assert torch.equal(buf.k_cache[b, :, :c], buf_e.k_cache[b, :, :c])
        assert torch.equal(buf.v_cache[b, :, :c], buf_e.v_cache[b, :, :c])
