"""Pins for the float64 oracle (CPU only).

The mounted paper prints nothing about this path, so the oracle is pinned to what the
mathematics fixes: a hand-worked example with rational probabilities, closed forms,
invariants, independent library routines (scipy log_softmax, torch cross-entropy autograd)
and brute-force central finite differences.  Each pin is chosen so that a plausible slip
(dropped term, wrong sign, transposed operand, wrong normaliser) fails at least one."""
import math

import numpy as np
import pytest
import scipy.special
import torch

from oracle import policy_oracle as orc

LN2, LN3, LN4 = math.log(2), math.log(3), math.log(4)


# ---------------------------------------------------------------------------
# hand-worked example: V=3, H=2, three rows, two sequences of one prompt
#   W = [[1,0],[0,1],[0,0]]
#   t0: x=[ln2, ln3] -> logits [ln2, ln3, 0] -> p = [1/3, 1/2, 1/6]
#   t1: x=[0,  ln4] -> logits [0,  ln4, 0] -> p = [1/6, 2/3, 1/6]
#   t2: x=[ln2, ln3] -> p = [1/3, 1/2, 1/6]
#   targets y = [0, 1, 2]  ->  logp = [ln 1/3, ln 2/3, ln 1/6],  lse = ln 6 everywhere
# ---------------------------------------------------------------------------
def _worked():
    W = np.array([[1.0, 0.0], [0.0, 1.0], [0.0, 0.0]])
    X = np.array([[LN2, LN3], [0.0, LN4], [LN2, LN3]])
    ids = np.array([0, 1, 2])
    mask = np.array([1, 1, 1], dtype=np.uint8)
    cu = np.array([0, 2, 3])
    logp = np.array([math.log(1 / 3), math.log(2 / 3), math.log(1 / 6)])
    return W, X, ids, mask, cu, logp


def test_worked_logprob():
    W, X, ids, mask, cu, logp = _worked()
    lp, lse = orc.token_logprob(X, W, ids, mask)
    np.testing.assert_allclose(lp, logp, rtol=0, atol=1e-14)
    np.testing.assert_allclose(lse, math.log(6.0), rtol=0, atol=1e-14)


def test_worked_grpo():
    # rewards [1,0], adv_eps=0 -> A = [+1,-1].
    # rho = [2 (clipped high, A>0), 1, 0.5 (clipped low, A<0)], d = ref-logp = [0, ln2, -ln2], kl_coef=0.5
    # token terms: t0 -1.2 + 0 ; t1 -1 + 0.5(1-ln2) ; t2 +0.8 + 0.5(ln2-0.5)
    W, X, ids, mask, cu, logp = _worked()
    old = logp - np.array([LN2, 0.0, -LN2])
    ref = logp + np.array([0.0, LN2, -LN2])
    adv = orc.group_advantage([1.0, 0.0], [0, 0], 1, adv_eps=0.0)
    np.testing.assert_allclose(adv, [1.0, -1.0], atol=1e-15)
    out = orc.grpo_loss(logp, old, ref, mask, cu, adv, clip_eps=0.2, kl_coef=0.5)
    np.testing.assert_allclose(out["seq_loss"], [-0.85 - 0.25 * LN2, 0.55 + 0.5 * LN2], atol=1e-14)
    assert out["loss"] == pytest.approx(-0.15 + 0.125 * LN2, abs=1e-14)
    np.testing.assert_allclose(out["c"], [0.0, -0.375, 0.125], atol=1e-14)
    assert (out["n_clip_hi"], out["n_clip_lo"]) == (1, 1)
    lse = np.full(3, math.log(6.0))
    dX, dW = orc.lm_head_backward(X, W, ids, mask, lse, out["c"])
    np.testing.assert_allclose(dX, [[0, 0], [0.0625, -0.125], [-1 / 24, -1 / 16]], atol=1e-14)
    x1, x2 = np.array([0.0, LN4]), np.array([LN2, LN3])
    exp_dW = np.stack([0.0625 * x1 - x2 / 24, -0.125 * x1 - x2 / 16, 0.0625 * x1 + 5 * x2 / 48])
    np.testing.assert_allclose(dW, exp_dW, atol=1e-14)


def test_worked_flow():
    # logZ=0.3, beta=2, A=[+1,-1]
    # seq0: mean(logp-ref) = -ln2/2, sum(logp-old) = ln2 -> w = 1.2, delta0 = 0.3 - ln2/2 - 2
    # seq1: mean(logp-ref) = +ln2,   sum(logp-old) = -ln2 -> w = 0.8, delta1 = 0.3 + ln2 + 2
    W, X, ids, mask, cu, logp = _worked()
    old = logp - np.array([LN2, 0.0, -LN2])
    ref = logp + np.array([0.0, LN2, -LN2])
    adv = np.array([1.0, -1.0])
    out = orc.flow_loss(logp, old, ref, mask, cu, adv, [0, 0], [0.3], clip_eps=0.2, beta=2.0)
    d0, d1 = 0.3 - LN2 / 2 - 2, 0.3 + LN2 + 2
    np.testing.assert_allclose(out["w"], [1.2, 0.8], atol=1e-14)
    np.testing.assert_allclose(out["delta"], [d0, d1], atol=1e-14)
    assert out["loss"] == pytest.approx(0.5 * (1.2 * d0 ** 2 + 0.8 * d1 ** 2), abs=1e-13)
    np.testing.assert_allclose(out["c"], [0.6 * d0, 0.6 * d0, 0.8 * d1], atol=1e-14)
    np.testing.assert_allclose(out["d_log_z"], [1.2 * d0 + 0.8 * d1], atol=1e-14)
    assert (out["n_clip_hi"], out["n_clip_lo"]) == (1, 1)


# ---------------------------------------------------------------------------
# log-prob
# ---------------------------------------------------------------------------
def _rand_problem(rng, R=11, H=5, V=7, scale=1.0):
    X = rng.normal(size=(R, H))
    W = rng.normal(size=(V, H)) * scale
    ids = rng.integers(0, V, size=R)
    return X, W, ids


def test_logprob_matches_library_log_softmax():
    rng = np.random.default_rng(0)
    X, W, ids = _rand_problem(rng, R=37, H=9, V=23)
    mask = np.ones(37, dtype=np.uint8)
    lp, lse = orc.token_logprob(X, W, ids, mask)
    Z = np.einsum("th,vh->tv", X, W)
    ls = scipy.special.log_softmax(Z, axis=1)
    np.testing.assert_allclose(lp, ls[np.arange(37), ids], atol=1e-13)
    np.testing.assert_allclose(lse, scipy.special.logsumexp(Z, axis=1), atol=1e-13)
    ce = torch.nn.functional.cross_entropy(torch.from_numpy(Z), torch.from_numpy(ids), reduction="none")
    np.testing.assert_allclose(lp, -ce.numpy(), atol=1e-13)


def test_logprob_brute_force_loops():
    """Direct exp/sum without max-subtraction, scalar python loops (catches transposition)."""
    rng = np.random.default_rng(1)
    X, W, ids = _rand_problem(rng, R=6, H=4, V=9, scale=0.5)
    mask = np.ones(6, dtype=np.uint8)
    lp, lse = orc.token_logprob(X, W, ids, mask)
    for t in range(6):
        z = [sum(W[v][h] * X[t][h] for h in range(4)) for v in range(9)]
        s = sum(math.exp(zv) for zv in z)
        assert lse[t] == pytest.approx(math.log(s), abs=1e-13)
        assert lp[t] == pytest.approx(z[ids[t]] - math.log(s), abs=1e-13)


def test_logprob_closed_forms_and_invariants():
    rng = np.random.default_rng(2)
    X, W, ids = _rand_problem(rng, R=8, H=6, V=50)
    mask = np.ones(8, dtype=np.uint8)
    lp, _ = orc.token_logprob(X, np.zeros_like(W), ids, mask)
    np.testing.assert_allclose(lp, -math.log(50), atol=1e-14)          # uniform distribution
    lp, _ = orc.token_logprob(np.zeros_like(X), W, ids, mask)
    np.testing.assert_allclose(lp, -math.log(50), atol=1e-14)
    # one dominant logit: z_y = 40, others 0  ->  logp = -log1p((V-1) e^-40)
    Wd = np.zeros((50, 6)); Wd[3, 0] = 40.0
    Xd = np.zeros((1, 6)); Xd[0, 0] = 1.0
    lp, _ = orc.token_logprob(Xd, Wd, [3], [1])
    assert lp[0] == pytest.approx(-math.log1p(49 * math.exp(-40.0)), rel=1e-12)
    # rows sum to 1 in probability space, logp <= 0, large logits do not overflow
    Xb = X * 300.0
    lp, lse = orc.token_logprob(Xb, W, ids, mask)
    Z = Xb @ W.T
    np.testing.assert_allclose(np.exp(Z - lse[:, None]).sum(1), 1.0, atol=1e-12)
    assert np.all(lp <= 0) and np.all(np.isfinite(lp))
    # shift invariance: a constant feature times a constant weight column shifts every logit
    X1 = np.concatenate([X, np.ones((8, 1))], 1)
    W1 = np.concatenate([W, np.full((50, 1), 7.5)], 1)
    a, la = orc.token_logprob(X, W, ids, mask)
    b, lb = orc.token_logprob(X1, W1, ids, mask)
    np.testing.assert_allclose(a, b, atol=1e-12)
    np.testing.assert_allclose(lb - la, 7.5, atol=1e-12)


def test_entropy_pins():
    import scipy.stats
    rng = np.random.default_rng(31)
    X, W, ids = _rand_problem(rng, R=9, H=5, V=13)
    mask = np.array([1, 1, 1, 0, 1, 1, 0, 1, 1], dtype=np.uint8)
    ent = orc.token_entropy(X, W, mask)
    P = scipy.special.softmax(X @ W.T, axis=1)
    ref = scipy.stats.entropy(P, axis=1)                       # independent library routine
    np.testing.assert_allclose(ent[mask.astype(bool)], ref[mask.astype(bool)], atol=1e-13)
    assert np.all(ent[~mask.astype(bool)] == 0)
    # H = lse - sum_v p_v z_v (the identity the online version uses)
    lp, lse = orc.token_logprob(X, W, ids, np.ones(9, np.uint8))
    np.testing.assert_allclose(orc.token_entropy(X, W, np.ones(9, np.uint8)), lse - (P * (X @ W.T)).sum(1), atol=1e-12)
    # closed forms: uniform -> ln V; one dominant logit a, V-1 zeros -> lse - a p_y
    np.testing.assert_allclose(orc.token_entropy(X, np.zeros_like(W), np.ones(9, np.uint8)), math.log(13), atol=1e-14)
    Wd = np.zeros((13, 5)); Wd[4, 0] = 3.0
    Xd = np.zeros((1, 5)); Xd[0, 0] = 1.0
    lse_d = math.log(math.exp(3.0) + 12)
    assert orc.token_entropy(Xd, Wd, [1])[0] == pytest.approx(lse_d - 3.0 * math.exp(3.0 - lse_d), rel=1e-13)
    # bounds and invariance to a shift of every logit; an extreme logit gives exactly 0 without NaN
    assert np.all(ent >= 0) and np.all(ent <= math.log(13) + 1e-12)
    X1 = np.concatenate([X, np.ones((9, 1))], 1); W1 = np.concatenate([W, np.full((13, 1), -4.0)], 1)
    np.testing.assert_allclose(orc.token_entropy(X1, W1, mask), ent, atol=1e-12)
    Wd[4, 0] = 2000.0
    assert orc.token_entropy(Xd, Wd, [1])[0] == 0.0


def test_masked_rows_are_ignored():
    rng = np.random.default_rng(3)
    X, W, ids = _rand_problem(rng, R=12, H=5, V=7)
    mask = np.array([1, 1, 0, 0, 1, 0, 1, 1, 1, 0, 0, 0], dtype=np.uint8)
    cu = np.array([0, 4, 6, 12])
    keep = mask.astype(bool)
    cu_packed = np.array([0, 2, 3, 6])
    kw = dict(group_idx=[0, 0, 0], rewards=[1.0, 0.0, 1.0], P=1)
    old = rng.normal(size=12) * 0.1 - 2; ref = rng.normal(size=12) * 0.1 - 2
    for obj in (orc.GRPO, orc.FLOW):
        a = orc.policy_loss_fwd_bwd(obj, X, W, ids, mask, cu, old_logprob=old, ref_logprob=ref,
                                    log_z=[0.2], **kw)
        Xg = X.copy(); Xg[~keep] = 1e3          # garbage in masked rows must not matter
        idg = ids.copy(); idg[~keep] = 0
        g = orc.policy_loss_fwd_bwd(obj, Xg, W, idg, mask, cu, old_logprob=old, ref_logprob=ref,
                                    log_z=[0.2], **kw)
        b = orc.policy_loss_fwd_bwd(obj, X[keep], W, ids[keep], np.ones(6, np.uint8), cu_packed,
                                    old_logprob=old[keep], ref_logprob=ref[keep], log_z=[0.2], **kw)
        for o in (g, b):
            assert a["loss"] == pytest.approx(o["loss"], abs=1e-14)
            np.testing.assert_allclose(a["d_weight"], o["d_weight"], atol=1e-14)
        np.testing.assert_array_equal(a["seq_len"], [2, 1, 3])
        np.testing.assert_allclose(a["d_hidden"][keep], b["d_hidden"], atol=1e-14)
        assert np.all(a["d_hidden"][~keep] == 0) and np.all(a["logprob"][~keep] == 0)
        assert np.all(g["d_hidden"][~keep] == 0)


def test_bf16_widening_is_exact():
    t = torch.randn(1000, dtype=torch.float32).to(torch.bfloat16)
    bits = t.view(torch.int16).numpy()
    np.testing.assert_array_equal(orc.widen(bits), t.to(torch.float64).numpy())
    np.testing.assert_array_equal(orc.widen(bits.view(np.uint16)), t.to(torch.float64).numpy())


# ---------------------------------------------------------------------------
# advantage
# ---------------------------------------------------------------------------
def test_advantage_invariants_and_closed_form():
    rng = np.random.default_rng(4)
    P, G = 5, 8
    r = rng.normal(size=P * G)
    g = np.repeat(np.arange(P), G)
    perm = rng.permutation(P * G)               # membership is by index, not by position
    adv = orc.group_advantage(r[perm], g[perm], P, adv_eps=0.0)
    for p in range(P):
        a = adv[g[perm] == p]
        assert a.sum() == pytest.approx(0.0, abs=1e-13)
        assert (a ** 2).mean() == pytest.approx(1.0, abs=1e-12)
    adv1 = orc.group_advantage(r, g, P, adv_eps=0.0, ddof=1)
    for p in range(P):
        assert (adv1[g == p] ** 2).sum() / (G - 1) == pytest.approx(1.0, abs=1e-12)
    # Bernoulli group with k ones out of G: A = (1-k/G)/sqrt(k/G (1-k/G)) for the ones
    for k in range(1, G):
        rr = np.array([1.0] * k + [0.0] * (G - k))
        a = orc.group_advantage(rr, np.zeros(G, int), 1, adv_eps=0.0)
        q = k / G
        assert a[0] == pytest.approx((1 - q) / math.sqrt(q * (1 - q)), rel=1e-12)
        assert a[-1] == pytest.approx(-q / math.sqrt(q * (1 - q)), rel=1e-12)
    # eps is added to the std, outside the root
    a = orc.group_advantage([1.0, 0.0], [0, 0], 1, adv_eps=0.5)
    np.testing.assert_allclose(a, [0.5, -0.5], atol=1e-15)
    # zero-variance group: exactly zero, no NaN
    a = orc.group_advantage([1.0, 1.0, 1.0, 0.0, 1.0], [0, 0, 0, 1, 1], 2)
    assert np.all(a[:3] == 0.0) and np.all(np.isfinite(a))


# ---------------------------------------------------------------------------
# GRPO / FLOW closed forms
# ---------------------------------------------------------------------------
def _seqs(rng, lens):
    cu = np.concatenate([[0], np.cumsum(lens)])
    R = int(cu[-1])
    return cu, R, np.ones(R, np.uint8), rng.normal(size=R) * 0.3 - 3.0


def test_grpo_closed_forms():
    rng = np.random.default_rng(5)
    lens = [3, 1, 4, 2]
    cu, R, mask, lp = _seqs(rng, lens)
    adv = np.array([0.7, -1.3, 0.0, 2.0])
    B = 4
    # old = ref = current: rho = 1, KL = 0 -> loss = -(1/B) sum A_i ; c_t = -A_i/(B |y_i|)
    out = orc.grpo_loss(lp, lp, lp, mask, cu, adv, 0.2, 1e-3)
    assert out["loss"] == pytest.approx(-adv.mean(), abs=1e-15)
    np.testing.assert_allclose(out["c"], np.repeat(-adv / (B * np.array(lens)), lens), atol=1e-15)
    # forced clipping on both sides with both signs
    for rho, A, term, act in [(2.0, 1.5, -1.2 * 1.5, 0), (0.5, 1.5, -0.5 * 1.5, 1),
                              (2.0, -1.5, 2.0 * 1.5, 1), (0.5, -1.5, 0.8 * 1.5, 0)]:
        o = orc.grpo_loss(lp, lp - math.log(rho), lp, mask, cu, np.full(4, A), 0.2, 0.0)
        assert o["loss"] == pytest.approx(term, rel=1e-13)
        np.testing.assert_allclose(o["c"], np.repeat(-A * rho * act / (B * np.array(lens)), lens), atol=1e-14)
    # KL term: >= 0, zero iff ref == current, value e^d - d - 1
    o = orc.grpo_loss(lp, lp, lp + 0.4, mask, cu, np.zeros(4), 0.2, 2.0)
    assert o["loss"] == pytest.approx(2.0 * (math.exp(0.4) - 0.4 - 1), rel=1e-13)
    o = orc.grpo_loss(lp, lp, lp - 0.4, mask, cu, np.zeros(4), 0.2, 2.0)
    assert o["loss"] == pytest.approx(2.0 * (math.exp(-0.4) + 0.4 - 1), rel=1e-13)
    # empty sequence: contributes zero, still counted in B
    cu2 = np.array([0, 3, 3, 5]); m2 = np.ones(5, np.uint8)
    o = orc.grpo_loss(lp[:5], lp[:5], lp[:5], m2, cu2, np.array([1.0, 5.0, 1.0]), 0.2, 0.0)
    assert o["loss"] == pytest.approx(-2.0 / 3.0, abs=1e-15)


def test_flow_closed_forms():
    rng = np.random.default_rng(6)
    lens = [3, 1, 4, 2]
    cu, R, mask, lp = _seqs(rng, lens)
    ref = lp + rng.normal(size=R) * 0.1
    old = lp + rng.normal(size=R) * 0.05
    adv = np.array([0.7, -1.3, 0.0, 2.0])
    beta = 15.0
    a = np.array([(lp - ref)[cu[i]:cu[i + 1]].mean() for i in range(4)])
    # one prompt per sequence and logZ chosen to balance: delta = 0 -> loss 0, all gradients 0
    lz = beta * adv - a
    o = orc.flow_loss(lp, old, ref, mask, cu, adv, np.arange(4), lz, 0.2, beta)
    assert abs(o["loss"]) < 1e-25 and np.all(np.abs(o["c"]) < 1e-13) and np.all(np.abs(o["d_log_z"]) < 1e-13)
    # old = current -> w = 1; then loss = mean delta^2
    g = np.array([0, 0, 1, 1]); lz2 = np.array([0.4, -0.9])
    o = orc.flow_loss(lp, lp, ref, mask, cu, adv, g, lz2, 0.2, beta)
    np.testing.assert_allclose(o["w"], 1.0, atol=1e-15)
    delta = lz2[g] + a - beta * adv
    assert o["loss"] == pytest.approx((delta ** 2).mean(), rel=1e-13)
    # weight always inside the clip range, even for huge log-ratios
    o = orc.flow_loss(lp, lp - 1000.0, ref, mask, cu, adv, g, lz2, 0.2, beta)
    np.testing.assert_allclose(o["w"], 1.2, atol=1e-15)
    o = orc.flow_loss(lp, lp + 1000.0, ref, mask, cu, adv, g, lz2, 0.2, beta)
    np.testing.assert_allclose(o["w"], 0.8, atol=1e-15)
    # c is constant inside a sequence and d_logZ_p = sum over members of |y_i| c_i
    o = orc.flow_loss(lp, old, ref, mask, cu, adv, g, lz2, 0.2, beta)
    for i in range(4):
        ci = o["c"][cu[i]:cu[i + 1]]
        assert np.all(ci == ci[0])
    per_seq = np.array([o["c"][cu[i]] * lens[i] for i in range(4)])
    np.testing.assert_allclose(o["d_log_z"], [per_seq[:2].sum(), per_seq[2:].sum()], atol=1e-14)


# ---------------------------------------------------------------------------
# backward: invariants, textbook special case, brute-force finite differences
# ---------------------------------------------------------------------------
def test_backward_is_mean_cross_entropy_gradient_when_c_is_minus_one_over_T():
    rng = np.random.default_rng(7)
    X, W, ids = _rand_problem(rng, R=13, H=6, V=10)
    mask = np.ones(13, np.uint8)
    _, lse = orc.token_logprob(X, W, ids, mask)
    dX, dW = orc.lm_head_backward(X, W, ids, mask, lse, np.full(13, -1.0 / 13))
    Xt = torch.tensor(X, requires_grad=True); Wt = torch.tensor(W, requires_grad=True)
    torch.nn.functional.cross_entropy(Xt @ Wt.T, torch.from_numpy(ids)).backward()
    np.testing.assert_allclose(dX, Xt.grad.numpy(), atol=1e-13)
    np.testing.assert_allclose(dW, Wt.grad.numpy(), atol=1e-13)
    np.testing.assert_allclose(dW.sum(0), 0.0, atol=1e-13)     # sum_v (onehot - p) = 0
    # <dX, X> = <dW, W> (both are sum dS * Z)
    assert (dX * X).sum() == pytest.approx((dW * W).sum(), abs=1e-12)


def _fd_problem(seed):
    rng = np.random.default_rng(seed)
    lens = [2, 1, 2, 1]
    cu = np.concatenate([[0], np.cumsum(lens)]); R = 6; H = 4; V = 7
    X = rng.normal(size=(R, H)); W = rng.normal(size=(V, H)) * 0.5
    ids = rng.integers(0, V, size=R)
    mask = np.ones(R, np.uint8)
    g = np.array([0, 0, 1, 1]); rew = np.array([1.0, 0.0, 0.3, 0.9])
    lp, _ = orc.token_logprob(X, W, ids, mask)
    old = lp + rng.choice([-0.1, 0.05, 0.12], size=R)          # rho well away from 1 +- eps
    old[0] = lp[0] - 0.5; old[3] = lp[3] + 0.5                 # two tokens outside the clip range
    ref = lp + rng.normal(size=R) * 0.2
    lz = rng.normal(size=2)
    return dict(hidden=X, weight=W, token_ids=ids, mask=mask, cu_seqlens=cu, group_idx=g,
                rewards=rew, old_logprob=old, ref_logprob=ref, log_z=lz, P=2,
                clip_eps=0.2, kl_coef=0.3, beta=1.5)


@pytest.mark.parametrize("objective", [orc.GRPO, orc.FLOW])
def test_gradients_match_central_finite_differences(objective):
    pb = _fd_problem(11 + objective)
    base = orc.policy_loss_fwd_bwd(objective, **pb)
    assert base["n_clip_hi"] + base["n_clip_lo"] >= 1 or objective == orc.FLOW
    w0 = base.get("w")

    def loss_of(**over):
        q = dict(pb); q.update(over)
        o = orc.policy_loss_fwd_bwd(objective, want_grads=False, **q)
        if objective == orc.FLOW:           # importance weight is a constant of the objective
            return float((w0 * o["delta"] ** 2).sum() / w0.size)
        return float(o["loss"])

    h = 1e-6
    for name, grad in (("hidden", base["d_hidden"]), ("weight", base["d_weight"])):
        A = pb[name]
        fd = np.zeros_like(A)
        for idx in np.ndindex(*A.shape):
            Ap = A.copy(); Ap[idx] += h
            Am = A.copy(); Am[idx] -= h
            fd[idx] = (loss_of(**{name: Ap}) - loss_of(**{name: Am})) / (2 * h)
        scale = np.abs(grad).max()
        assert scale > 1e-3
        np.testing.assert_allclose(grad, fd, atol=2e-7 * max(scale, 1.0))
    if objective == orc.FLOW:
        fd = np.zeros(2)
        for p in range(2):
            zp = pb["log_z"].copy(); zp[p] += h
            zm = pb["log_z"].copy(); zm[p] -= h
            fd[p] = (loss_of(log_z=zp) - loss_of(log_z=zm)) / (2 * h)
        np.testing.assert_allclose(base["d_log_z"], fd, atol=1e-7)


def test_c_is_the_derivative_of_the_loss_in_logp():
    """dloss/dlogp_t by finite differences on the loss functions alone (both objectives)."""
    rng = np.random.default_rng(21)
    lens = [3, 2, 4, 1]
    cu, R, mask, lp = _seqs(rng, lens)
    old = lp + rng.choice([-0.4, -0.1, 0.08, 0.45], size=R)
    ref = lp + rng.normal(size=R) * 0.3
    adv = np.array([1.1, -0.6, -1.4, 0.8]); g = np.array([0, 1, 0, 1]); lz = np.array([0.2, -0.5])
    h = 1e-6
    o = orc.grpo_loss(lp, old, ref, mask, cu, adv, 0.2, 0.25)
    assert o["n_clip_hi"] > 0 and o["n_clip_lo"] > 0
    f = orc.flow_loss(lp, old, ref, mask, cu, adv, g, lz, 0.2, 3.0)
    for t in range(R):
        e = np.zeros(R); e[t] = h
        gp = orc.grpo_loss(lp + e, old, ref, mask, cu, adv, 0.2, 0.25)["loss"]
        gm = orc.grpo_loss(lp - e, old, ref, mask, cu, adv, 0.2, 0.25)["loss"]
        assert o["c"][t] == pytest.approx((gp - gm) / (2 * h), abs=1e-8)
        fp = orc.flow_loss(lp + e, old, ref, mask, cu, adv, g, lz, 0.2, 3.0)["delta"]
        fm = orc.flow_loss(lp - e, old, ref, mask, cu, adv, g, lz, 0.2, 3.0)["delta"]
        num = ((f["w"] * fp ** 2).mean() - (f["w"] * fm ** 2).mean()) / (2 * h)
        assert f["c"][t] == pytest.approx(num, abs=1e-8)


# ---------------------------------------------------------------------------
# objective variants: reduce to the base objectives, closed forms per option, finite differences
# ---------------------------------------------------------------------------
def _variant_case(seed=10):
    rng = np.random.default_rng(seed)
    lens = [3, 1, 5, 2, 0, 4]
    cu, R, mask, lp = _seqs(rng, lens)
    old = lp + rng.normal(size=R) * 0.25            # wide enough that both clip branches occur
    ref = lp + rng.normal(size=R) * 0.1
    adv = np.array([0.7, -1.3, 0.4, 2.0, 1.0, -0.6])
    g = np.array([0, 0, 1, 1, 2, 2]); lz = np.array([0.4, -0.9, 0.1])
    return lens, cu, R, mask, lp, old, ref, adv, g, lz


def test_variants_reduce_to_the_base_objectives():
    lens, cu, R, mask, lp, old, ref, adv, g, lz = _variant_case()
    a = orc.grpo_loss(lp, old, ref, mask, cu, adv, 0.2, 0.3)
    b = orc.grpo_loss_variant(lp, old, ref, mask, cu, adv, 0.2, 0.3)
    b2 = orc.grpo_loss_variant(lp, old, ref, mask, cu, adv, 0.2, 0.3, clip_eps_high=0.2)
    for k in ("loss", "seq_loss", "c", "n_clip_hi", "n_clip_lo"):
        np.testing.assert_allclose(a[k], b[k], rtol=0, atol=1e-15)
        np.testing.assert_allclose(a[k], b2[k], rtol=0, atol=1e-15)
    assert a["n_clip_hi"] > 0 and a["n_clip_lo"] > 0
    f = orc.flow_loss(lp, old, ref, mask, cu, adv, g, lz, 0.2, 3.0)
    fv = orc.flow_loss_variant(lp, old, ref, mask, cu, adv, g, lz, 0.2, 3.0)
    for k in ("loss", "seq_loss", "c", "d_log_z", "w", "delta"):
        np.testing.assert_allclose(f[k], fv[k], rtol=0, atol=1e-15)


def test_asymmetric_clip_closed_forms():
    lens, cu, R, mask, lp, old, ref, adv, g, lz = _variant_case()
    B = len(lens); n = np.array(lens)
    # rho = 1.25 everywhere, A > 0: clipped with eps_high = 0.2 (term -1.2 A, no gradient), not with 0.28 (term -1.25 A)
    A = np.full(B, 1.5)
    o = orc.grpo_loss_variant(lp, lp - math.log(1.25), lp, mask, cu, A, 0.2, 0.0, clip_eps_high=0.2)
    assert o["loss"] == pytest.approx(-1.2 * 1.5 * 5 / 6, rel=1e-13) and np.all(o["c"] == 0)        # 5 of 6 sequences non-empty
    o = orc.grpo_loss_variant(lp, lp - math.log(1.25), lp, mask, cu, A, 0.2, 0.0, clip_eps_high=0.28)
    assert o["loss"] == pytest.approx(-1.25 * 1.5 * 5 / 6, rel=1e-13)
    want = np.repeat(np.where(n > 0, -1.5 * 1.25 / (B * np.maximum(n, 1)), 0.0), lens)
    np.testing.assert_allclose(o["c"], want, atol=1e-15)
    # the lower bound is unaffected by eps_high: rho = 0.7, A < 0 -> term +0.8 |A|... (-min(0.7A, 0.8A) = -0.8A for A<0)
    o = orc.grpo_loss_variant(lp, lp - math.log(0.7), lp, mask, cu, -A, 0.2, 0.0, clip_eps_high=0.5)
    assert o["loss"] == pytest.approx(0.8 * 1.5 * 5 / 6, rel=1e-13) and np.all(o["c"] == 0)
    # flow: the weight's upper bound moves, the lower does not
    f = orc.flow_loss_variant(lp, lp - 1000.0, ref, mask, cu, adv, g, lz, 0.2, 3.0, clip_eps_high=0.5)
    np.testing.assert_allclose(f["w"][n > 0], 1.5, atol=1e-15)
    f = orc.flow_loss_variant(lp, lp + 1000.0, ref, mask, cu, adv, g, lz, 0.2, 3.0, clip_eps_high=0.5)
    np.testing.assert_allclose(f["w"][n > 0], 0.8, atol=1e-15)


def test_token_mean_aggregation():
    lens, cu, R, mask, lp, old, ref, adv, g, lz = _variant_case()
    B = len(lens); T = sum(lens)
    seq = orc.grpo_loss_variant(lp, old, ref, mask, cu, adv, 0.2, 0.3)
    tok = orc.grpo_loss_variant(lp, old, ref, mask, cu, adv, 0.2, 0.3, aggregation="token")
    # same per-token terms, different weights: sequence mode weighs token t of sequence i by 1/(B n_i), token mode by 1/T
    per_tok_seq = np.concatenate([seq["seq_loss"][i] * np.ones(lens[i]) for i in range(B)])      # mean l over the sequence
    sums = np.array([seq["seq_loss"][i] * lens[i] for i in range(B)])                            # sum_t l_t per sequence
    assert tok["loss"] == pytest.approx(sums.sum() / T, rel=1e-13)
    np.testing.assert_allclose(tok["seq_loss"], sums * B / T, rtol=1e-13)
    assert tok["loss"] == pytest.approx(tok["seq_loss"].mean(), rel=1e-13)
    nrep = np.repeat(np.array(lens), lens)
    np.testing.assert_allclose(tok["c"], seq["c"] * (B * nrep) / T, rtol=1e-13)
    # equal lengths: both aggregations coincide
    cu2 = np.array([0, 4, 8, 12]); m2 = np.ones(12, np.uint8)
    a = orc.grpo_loss_variant(lp[:12], old[:12], ref[:12], m2, cu2, adv[:3], 0.2, 0.3)
    b = orc.grpo_loss_variant(lp[:12], old[:12], ref[:12], m2, cu2, adv[:3], 0.2, 0.3, aggregation="token")
    assert a["loss"] == pytest.approx(b["loss"], rel=1e-13)
    np.testing.assert_allclose(a["c"], b["c"], rtol=1e-13)


def test_sequence_level_ratio_closed_forms():
    lens, cu, R, mask, lp, old, ref, adv, g, lz = _variant_case()
    B = len(lens); n = np.array(lens)
    # a constant per-token log-ratio makes the sequence ratio equal to the token ratio: same loss as the token-level form
    for r in (1.1, 0.9, 1.5, 0.6):
        a = orc.grpo_loss_variant(lp, lp - math.log(r), ref, mask, cu, adv, 0.2, 0.3)
        b = orc.grpo_loss_variant(lp, lp - math.log(r), ref, mask, cu, adv, 0.2, 0.3, ratio_level="sequence")
        assert a["loss"] == pytest.approx(b["loss"], rel=1e-13)
        np.testing.assert_allclose(a["seq_loss"], b["seq_loss"], rtol=1e-12, atol=1e-15)
        np.testing.assert_allclose(a["c"], b["c"], rtol=1e-12, atol=1e-16)
    # geometric mean: log-ratios that cancel inside every sequence give s_i = 1 -> loss = -mean(A) over all B (+0 KL)
    d = np.concatenate([x - x.mean() if x.size else x for x in np.split(np.resize([0.3, -0.1, 0.2], R).astype(float), cu[1:-1])])
    o = orc.grpo_loss_variant(lp, lp - d, lp, mask, cu, adv, 0.2, 0.0, ratio_level="sequence")
    assert o["loss"] == pytest.approx(-(adv[n > 0]).sum() / B, rel=1e-12)
    np.testing.assert_allclose(o["c"], np.repeat(np.where(n > 0, -adv / (B * np.maximum(n, 1)), 0.0), lens), atol=1e-14)
    # counts are per sequence
    o = orc.grpo_loss_variant(lp, lp - math.log(2.0), lp, mask, cu, np.abs(adv), 0.2, 0.0, ratio_level="sequence")
    assert o["n_clip_hi"] == 5 and o["n_clip_lo"] == 0 and np.all(o["c"] == 0)


def test_flow_length_normalised_weight():
    lens, cu, R, mask, lp, old, ref, adv, g, lz = _variant_case()
    n = np.array(lens)
    o = orc.flow_loss_variant(lp, old, ref, mask, cu, adv, g, lz, 0.2, 3.0, weight_norm="mean")
    base = orc.flow_loss_variant(lp, old, ref, mask, cu, adv, g, lz, 0.2, 3.0)
    np.testing.assert_allclose(o["delta"], base["delta"], atol=0)                  # only w changes
    want = np.array([math.exp(min(max((lp - old)[cu[i]:cu[i + 1]].mean(), math.log(0.8)), math.log(1.2))) if lens[i] else 0.0 for i in range(len(lens))])
    np.testing.assert_allclose(o["w"], want, rtol=1e-14)
    np.testing.assert_allclose(o["seq_loss"], want * base["delta"] ** 2, rtol=1e-13)
    # single-token sequences: sum and mean coincide
    assert o["w"][1] == base["w"][1]
    # a constant log-ratio r per token: mean gives exp(r) whatever the length, sum gives exp(n r)
    o = orc.flow_loss_variant(lp, lp - 0.05, ref, mask, cu, adv, g, lz, 0.2, 3.0, weight_norm="mean")
    np.testing.assert_allclose(o["w"][n > 0], math.exp(0.05), rtol=1e-14)


@pytest.mark.parametrize("opts", [dict(clip_eps_high=0.35), dict(aggregation="token"), dict(ratio_level="sequence"),
                                  dict(clip_eps_high=0.3, aggregation="token"), dict(clip_eps_high=0.1, ratio_level="sequence")])
def test_variant_gradients_by_finite_differences(opts):
    lens, cu, R, mask, lp, old, ref, adv, g, lz = _variant_case(seed=10)
    o = orc.grpo_loss_variant(lp, old, ref, mask, cu, adv, 0.2, 0.25, **opts)
    h = 1e-6
    num = np.zeros(R)
    for t in range(R):
        e = np.zeros(R); e[t] = h
        num[t] = (orc.grpo_loss_variant(lp + e, old, ref, mask, cu, adv, 0.2, 0.25, **opts)["loss"]
                  - orc.grpo_loss_variant(lp - e, old, ref, mask, cu, adv, 0.2, 0.25, **opts)["loss"]) / (2 * h)
    np.testing.assert_allclose(o["c"], num, rtol=2e-7, atol=1e-9)
    assert o["n_clip_hi"] + o["n_clip_lo"] > 0                     # the case does exercise a switched-off branch


def test_flow_variant_gradient_with_frozen_weight():
    lens, cu, R, mask, lp, old, ref, adv, g, lz = _variant_case(seed=29)
    for opts in (dict(weight_norm="mean"), dict(weight_norm="mean", clip_eps_high=0.4)):
        o = orc.flow_loss_variant(lp, old, ref, mask, cu, adv, g, lz, 0.2, 3.0, **opts)
        B = len(lens)
        h = 1e-6
        for t in range(R):
            e = np.zeros(R); e[t] = h
            dp = orc.flow_loss_variant(lp + e, old, ref, mask, cu, adv, g, lz, 0.2, 3.0, **opts)["delta"]
            dm = orc.flow_loss_variant(lp - e, old, ref, mask, cu, adv, g, lz, 0.2, 3.0, **opts)["delta"]
            num = (o["w"] * (dp ** 2 - dm ** 2)).sum() / B / (2 * h)          # w held at the base point
            assert o["c"][t] == pytest.approx(num, rel=2e-7, abs=1e-9)



# ---------------------------------------------------------------------------
# temperature: the policy is softmax(W x / tau)
# ---------------------------------------------------------------------------
def test_temperature_logprob_entropy_against_library_and_closed_forms():
    rng = np.random.default_rng(31)
    X, W, ids = _rand_problem(rng, R=9, H=5, V=8)
    mask = np.ones(9, np.uint8)
    for tau in (0.5, 1.0, 1.7):
        lp, lse = orc.token_logprob(X, W, ids, mask, temperature=tau)
        ref = scipy.special.log_softmax((X @ W.T) / tau, axis=1)
        np.testing.assert_allclose(lp, ref[np.arange(9), ids], atol=1e-13)
        np.testing.assert_allclose(lse, scipy.special.logsumexp((X @ W.T) / tau, axis=1), atol=1e-13)
        ent = orc.token_entropy(X, W, mask, temperature=tau)
        p = np.exp(ref)
        np.testing.assert_allclose(ent, -(p * ref).sum(1), atol=1e-13)
    # the temperature only rescales the head: (W, tau) and (W / tau, 1) are the same policy
    a, _ = orc.token_logprob(X, W, ids, mask, temperature=0.8)
    b, _ = orc.token_logprob(X, W / 0.8, ids, mask)
    np.testing.assert_allclose(a, b, atol=1e-13)
    # worked example: x = [ln 2, ln 3], W = I2 + zero row, tau = 1/2 squares the odds: p ~ [4, 9, 1] / 14
    Ww, Xw, idw, mw, _, _ = _worked()
    lp, lse = orc.token_logprob(Xw[:1], Ww, idw[:1], mw[:1], temperature=0.5)
    assert lp[0] == pytest.approx(math.log(4 / 14), abs=1e-14) and lse[0] == pytest.approx(math.log(14.0), abs=1e-14)
    # a hot distribution tends to the uniform one
    lp, _ = orc.token_logprob(X, W, ids, mask, temperature=1e9)
    np.testing.assert_allclose(lp, -math.log(8), atol=1e-7)
    ent = orc.token_entropy(X, W, mask, temperature=1e9)
    np.testing.assert_allclose(ent, math.log(8), atol=1e-7)


def test_temperature_backward_is_the_autograd_gradient_of_tempered_cross_entropy():
    rng = np.random.default_rng(32)
    X, W, ids = _rand_problem(rng, R=12, H=6, V=9)
    mask = np.ones(12, np.uint8)
    tau = 0.6
    c = rng.normal(size=12)
    _, lse = orc.token_logprob(X, W, ids, mask, temperature=tau)
    dX, dW = orc.lm_head_backward(X, W, ids, mask, lse, c, temperature=tau)
    Xt = torch.tensor(X, requires_grad=True); Wt = torch.tensor(W, requires_grad=True)
    lsm = torch.log_softmax(Xt @ Wt.T / tau, dim=1)
    (torch.tensor(c) * lsm[torch.arange(12), torch.from_numpy(ids)]).sum().backward()
    np.testing.assert_allclose(dX, Xt.grad.numpy(), atol=1e-13)
    np.testing.assert_allclose(dW, Wt.grad.numpy(), atol=1e-13)
    np.testing.assert_allclose(dW.sum(0), 0.0, atol=1e-13)


@pytest.mark.parametrize("objective", [orc.GRPO, orc.FLOW])
def test_temperature_whole_path_by_finite_differences(objective):
    tau = 0.7
    pb = _fd_problem(41 + objective)
    rng = np.random.default_rng(43)
    lp, _ = orc.token_logprob(pb["hidden"], pb["weight"], pb["token_ids"], pb["mask"], temperature=tau)
    old = lp + rng.choice([-0.1, 0.05, 0.12], size=lp.size)
    old[0] = lp[0] - 0.5; old[3] = lp[3] + 0.5
    pb["old_logprob"] = old
    pb["ref_logprob"] = lp + rng.normal(size=lp.size) * 0.2
    base = orc.policy_loss_fwd_bwd(objective, temperature=tau, **pb)
    np.testing.assert_allclose(base["logprob"], lp, atol=0)
    w0 = base.get("w")

    def loss_of(**over):
        q = dict(pb); q.update(over)
        o = orc.policy_loss_fwd_bwd(objective, want_grads=False, temperature=tau, **q)
        if objective == orc.FLOW:
            return float((w0 * o["delta"] ** 2).sum() / w0.size)
        return float(o["loss"])

    h = 1e-6
    for name, grad in (("hidden", base["d_hidden"]), ("weight", base["d_weight"])):
        A = pb[name]
        fd = np.zeros_like(A)
        for idx in np.ndindex(*A.shape):
            Ap = A.copy(); Ap[idx] += h
            Am = A.copy(); Am[idx] -= h
            fd[idx] = (loss_of(**{name: Ap}) - loss_of(**{name: Am})) / (2 * h)
        scale = np.abs(grad).max()
        assert scale > 1e-3
        np.testing.assert_allclose(grad, fd, atol=2e-7 * max(scale, 1.0))
    # same policy written with the temperature folded into the head: dX equal, dW scaled by the chain rule
    q = dict(pb); q["weight"] = pb["weight"] / tau
    fold = orc.policy_loss_fwd_bwd(objective, **q)
    assert fold["loss"] == pytest.approx(base["loss"], abs=1e-13)
    np.testing.assert_allclose(fold["d_hidden"], base["d_hidden"], atol=1e-13)
    np.testing.assert_allclose(fold["d_weight"] / tau, base["d_weight"], atol=1e-13)


# ---------------------------------------------------------------------------
# integer work: usable sequences, row compaction, group sizes
# ---------------------------------------------------------------------------
def test_valid_sequences_hand_cases():
    # well-formed offsets: every sequence usable (empty ones included)
    assert orc.valid_sequences([0, 3, 3, 7, 10], 10).tolist() == [True, True, True, True]
    # the range of the last sequence runs past the rows
    assert orc.valid_sequences([0, 3, 12], 10).tolist() == [True, False]
    # a negative start
    assert orc.valid_sequences([-2, 3, 10], 10).tolist() == [False, True]
    # alternating {0, R, 0, R}: only the first range may be kept, or rows would count twice
    assert orc.valid_sequences([0, 10, 0, 10], 10).tolist() == [True, False, False]
    # decreasing, then increasing again below an earlier offset: [5, 20) overlaps [0, 10)
    assert orc.valid_sequences([0, 10, 5, 20], 20).tolist() == [True, False, False]
    # decreasing, then increasing from above every earlier offset: usable again
    assert orc.valid_sequences([0, 10, 5, 12, 20], 20).tolist() == [True, False, False, True]


def test_valid_sequences_kept_ranges_never_overlap():
    rng = np.random.default_rng(50)
    for _ in range(200):
        R = int(rng.integers(1, 30))
        cu = rng.integers(-3, R + 4, size=int(rng.integers(2, 9)))
        ok = orc.valid_sequences(cu, R)
        hits = np.zeros(R, dtype=np.int64)
        for i in np.nonzero(ok)[0]:
            assert 0 <= cu[i] <= cu[i + 1] <= R
            hits[cu[i]:cu[i + 1]] += 1
        assert hits.max(initial=0) <= 1
        # a sorted chain inside [0, R] keeps everything
        s = np.sort(np.clip(cu, 0, R))
        assert orc.valid_sequences(s, R).all()


def test_compact_rows_hand_worked():
    #        row: 0  1  2  3  4  5  6  7  8  9
    mask = np.array([1, 0, 1, 1, 1, 1, 0, 1, 1, 1], dtype=np.uint8)
    ids = np.array([4, 9, 7, -1, 0, 2, 2, 8, 3, 1])          # V = 8: rows 3 (id -1) and 7 (id 8) are out of range
    cu = np.array([0, 3, 3, 8, 10])
    out = orc.compact_rows(mask, ids, cu, V=8)
    assert out["row_map"].tolist() == [0, 2, 4, 5, 8, 9]
    assert out["seq_len"].tolist() == [2, 0, 2, 2]
    assert (out["n_bad_token"], out["n_bad_seq"], out["n_bad_group"]) == (2, 0, 0)
    # a prompt index out of range empties its sequence (and its out-of-range ids are no longer looked at)
    out = orc.compact_rows(mask, ids, cu, V=8, group_idx=[0, 1, 2, 1], P=2)
    assert out["row_map"].tolist() == [0, 2, 8, 9]
    assert out["seq_len"].tolist() == [2, 0, 0, 2]
    assert (out["n_bad_token"], out["n_bad_seq"], out["n_bad_group"]) == (0, 0, 1)
    # broken offsets: [0,3) kept, [3,2) decreasing, [2,8) starts below the earlier offset 3, [8,10) kept
    out = orc.compact_rows(mask, ids, np.array([0, 3, 2, 8, 10]), V=8)
    assert out["row_map"].tolist() == [0, 2, 8, 9]
    assert out["seq_len"].tolist() == [2, 0, 0, 2] and out["n_bad_seq"] == 2 and out["n_bad_token"] == 0


def test_compact_rows_against_library_routines():
    rng = np.random.default_rng(51)
    R, V = 200, 50
    mask = (rng.random(R) < 0.6).astype(np.uint8)
    ids = rng.integers(-3, V + 3, size=R)
    cuts = np.sort(rng.integers(0, R + 1, size=7))
    cu = np.concatenate([[0], cuts, [R]])
    out = orc.compact_rows(mask, ids, cu, V)
    keep = (mask != 0) & (ids >= 0) & (ids < V)
    np.testing.assert_array_equal(out["row_map"], np.flatnonzero(keep))     # clean offsets: plain stream compaction
    np.testing.assert_array_equal(out["seq_len"], np.add.reduceat(np.append(keep, 0).astype(np.int64), cu[:-1]) * (np.diff(cu) > 0))
    assert out["n_bad_token"] == int(((mask != 0) & ~keep).sum())
    np.testing.assert_array_equal(orc.compact_rows(mask, np.clip(ids, 0, V - 1), cu, V)["seq_len"], orc.segment_lengths(mask, cu))
    g = rng.integers(-1, 6, size=40)
    np.testing.assert_array_equal(orc.group_count(g, 5), np.bincount(g[(g >= 0) & (g < 5)], minlength=5))


def test_target_logit_is_the_gathered_entry_of_the_logits():
    rng = np.random.default_rng(52)
    X, W, ids = _rand_problem(rng, R=13, H=6, V=10)
    mask = (rng.random(13) < 0.8).astype(np.uint8); mask[0] = 1
    for tau in (1.0, 0.6):
        zy = orc.target_logit(X, W, ids, mask, temperature=tau)
        Z = np.einsum("th,vh->tv", X, W) / tau
        np.testing.assert_allclose(zy, np.take_along_axis(Z, ids[:, None], 1)[:, 0] * (mask != 0), atol=1e-14)
        lp, lse = orc.token_logprob(X, W, ids, mask, temperature=tau)
        np.testing.assert_allclose(zy, lp + lse, atol=1e-13)
    # hand value: row 0 of the worked example reads logit ln 2 for target 0
    Ww, Xw, idw, mw, _, _ = _worked()
    np.testing.assert_allclose(orc.target_logit(Xw, Ww, idw, mw), [LN2, LN4, 0.0], atol=1e-15)


def test_weight_grad_rows_are_rows_of_the_autograd_gradient():
    rng = np.random.default_rng(53)
    R, H, V = 14, 5, 9
    X, W, ids = _rand_problem(rng, R=R, H=H, V=V)
    mask = (rng.random(R) < 0.8).astype(np.uint8)
    c = rng.normal(size=R)
    for tau in (1.0, 0.7):
        _, lse = orc.token_logprob(X, W, ids, np.ones(R, np.uint8), temperature=tau)
        Xt = torch.tensor(X); Wt = torch.tensor(W, requires_grad=True)
        lsm = torch.log_softmax(Xt @ Wt.T / tau, dim=1)
        (torch.tensor(c * (mask != 0)) * lsm[torch.arange(R), torch.from_numpy(ids)]).sum().backward()
        vs = np.array([0, V - 1, 4, int(ids[np.flatnonzero(mask)[0]])])
        got = orc.weight_grad_rows(X, W[vs], vs, ids, mask, lse, c, temperature=tau)
        np.testing.assert_allclose(got, Wt.grad.numpy()[vs], atol=1e-13)
        # a plain sum over rows: two row blocks add up to the whole
        a = orc.weight_grad_rows(X[:6], W[vs], vs, ids[:6], mask[:6], lse[:6], c[:6], temperature=tau)
        b = orc.weight_grad_rows(X[6:], W[vs], vs, ids[6:], mask[6:], lse[6:], c[6:], temperature=tau)
        np.testing.assert_allclose(a + b, got, atol=1e-13)
    # worked example (the GRPO coefficients [0, -0.375, 0.125], lse = ln 6): same rows as the full backward
    Ww, Xw, idw, mw, _, _ = _worked()
    cw = np.array([0.0, -0.375, 0.125])
    x1, x2 = np.array([0.0, LN4]), np.array([LN2, LN3])
    exp_dW = np.stack([0.0625 * x1 - x2 / 24, -0.125 * x1 - x2 / 16, 0.0625 * x1 + 5 * x2 / 48])
    np.testing.assert_allclose(orc.weight_grad_rows(Xw, Ww[[2, 0]], [2, 0], idw, mw, np.full(3, math.log(6.0)), cw), exp_dW[[2, 0]], atol=1e-14)
