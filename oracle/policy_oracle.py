"""Float64 CPU oracle for the fused LM-head log-prob + policy-loss path.

TEST INFRASTRUCTURE ONLY.  This file is the slow, plain definition of what the
HIP library computes.  It may be imported by the tests, by the smoke check and
by the benchmark's CPU-baseline leg, never by the product path, and it shares
no code with the HIP sources (its bf16 widening, its reductions and its
formulas are its own).

The mounted paper has no passage on this path; every function below follows
the problem statement of the benchmark contract (fused LM-head projection,
per-token log-probability, group-relative advantage, GRPO clipped-ratio loss
or flow-balance / trajectory-balance loss, and the backward pass through the
LM head) under the readings listed with each function.  Because nothing here
can be checked against a printed value of the paper, each function is pinned
in tests/test_oracle_pins.py by closed forms, invariants, independent library
routines and brute-force finite differences.

Notation: R rows (tokens incl. masked), H hidden, V vocab, B sequences,
P prompts; sequence i owns rows [cu[i], cu[i+1]); m_t is the response mask;
|y_i| = sum of m_t over the sequence; g(i) is the prompt (group) index.

All arithmetic is float64.  Matrix products use numpy's matmul (a library
primitive used as a step); the row-block loop only bounds memory: rows are
independent and dW is a plain sum over rows.
"""
from __future__ import annotations

import numpy as np

ROW_BLOCK = 256


def widen(a) -> np.ndarray:
    """Exact widening of stored inputs to float64.

    Accepts float64/float32 arrays, or uint16/int16 arrays holding bfloat16 bit
    patterns (a bfloat16 is the upper half of a float32)."""
    a = np.asarray(a)
    if a.dtype == np.float64:
        return a
    if a.dtype == np.float32:
        return a.astype(np.float64)
    if a.dtype in (np.uint16, np.int16):
        bits = a.view(np.uint16).astype(np.uint32) << np.uint32(16)
        return bits.view(np.float32).astype(np.float64)
    raise TypeError(f"unsupported input dtype {a.dtype}")


# --------------------------------------------------------------------------
# log-prob:  z = W x_t,  lse_t = log sum_v exp z_v,  logp_t = z[y_t] - lse_t
# --------------------------------------------------------------------------
def token_logprob(hidden, weight, token_ids, mask, temperature=1.0):
    """Per-token log-probability of the sampled token under softmax(W x_t / temperature).

    Returns (logp[R], lse[R]) of the tempered logits; masked rows give 0 in both.  lse is
    computed with the row maximum subtracted (same value, no overflow)."""
    X = widen(hidden)
    W = widen(weight)
    ids = np.asarray(token_ids).astype(np.int64)
    m = np.asarray(mask).astype(bool)
    R = X.shape[0]
    logp = np.zeros(R)
    lse = np.zeros(R)
    for s in range(0, R, ROW_BLOCK):
        e = min(R, s + ROW_BLOCK)
        rows = np.nonzero(m[s:e])[0] + s
        if rows.size == 0:
            continue
        Z = X[rows] @ W.T                       # [n, V] logits
        Z = Z / temperature
        M = Z.max(axis=1)
        l = M + np.log(np.exp(Z - M[:, None]).sum(axis=1))
        zy = Z[np.arange(rows.size), ids[rows]]
        lse[rows] = l
        logp[rows] = zy - l
    return logp, lse


def token_entropy(hidden, weight, mask, temperature=1.0):
    """Entropy of the full next-token distribution, H_t = -sum_v p_v log p_v with
    p = softmax(W x_t / temperature) (0 log 0 = 0), written out from the definition.  Masked rows give 0."""
    X = widen(hidden)
    W = widen(weight)
    m = np.asarray(mask).astype(bool)
    R = X.shape[0]
    ent = np.zeros(R)
    for s in range(0, R, ROW_BLOCK):
        e = min(R, s + ROW_BLOCK)
        rows = np.nonzero(m[s:e])[0] + s
        if rows.size == 0:
            continue
        Z = X[rows] @ W.T / temperature
        Z = Z - Z.max(axis=1, keepdims=True)
        P = np.exp(Z)
        P /= P.sum(axis=1, keepdims=True)
        with np.errstate(divide="ignore", invalid="ignore"):
            term = np.where(P > 0, P * np.log(P), 0.0)
        ent[rows] = -term.sum(axis=1)
    return ent


def segment_lengths(mask, cu_seqlens):
    """|y_i|: number of mask=1 rows of each sequence (integer, exact)."""
    m = np.asarray(mask).astype(np.int64)
    cu = np.asarray(cu_seqlens).astype(np.int64)
    return np.array([m[cu[i]:cu[i + 1]].sum() for i in range(cu.size - 1)], dtype=np.int64)


# --------------------------------------------------------------------------
# integer work: which rows count, in which order, and how the groups are filled
# --------------------------------------------------------------------------
def valid_sequences(cu_seqlens, R):
    """Which sequences have a usable row range (boolean [B]).

    The problem statement takes well-formed offsets as given (cu[0] = 0, non-decreasing, cu[B] = R).
    Reading for offsets that are not: sequence i keeps its rows iff 0 <= cu[i] <= cu[i+1] <= R and
    cu[i] is not below any earlier offset cu[0..i]; otherwise it is treated as empty.  Kept ranges are
    then pairwise disjoint and in increasing order, whatever the offsets were."""
    cu = np.asarray(cu_seqlens).astype(np.int64)
    B = cu.size - 1
    ok = np.zeros(B, dtype=bool)
    highest = None
    for i in range(B):
        highest = cu[i] if highest is None else max(highest, cu[i])
        ok[i] = (0 <= cu[i] <= cu[i + 1] <= R) and cu[i] >= highest
    return ok


def compact_rows(mask, token_ids, cu_seqlens, V, group_idx=None, P=None):
    """The rows that count, in the order the path walks them.

    A row counts iff it lies in the range of a usable sequence (valid_sequences; with group_idx given the
    sequence's prompt index must also lie in [0, P)), its mask is non-zero and its token id lies in [0, V).
    Returns dict(row_map[T] = original row of the k-th counting row (sequence by sequence, rows ascending),
    seq_len[B], n_bad_token, n_bad_seq, n_bad_group); rows outside every sequence never count."""
    m = np.asarray(mask)
    ids = np.asarray(token_ids).astype(np.int64)
    cu = np.asarray(cu_seqlens).astype(np.int64)
    R = m.shape[0]
    B = cu.size - 1
    ok = valid_sequences(cu, R)
    grp_ok = np.ones(B, dtype=bool)
    if group_idx is not None:
        g = np.asarray(group_idx).astype(np.int64)
        grp_ok = (g >= 0) & (g < P)
    row_map = []
    seq_len = np.zeros(B, dtype=np.int64)
    n_bad_token = 0
    for i in range(B):
        if not (ok[i] and grp_ok[i]):
            continue
        for r in range(cu[i], cu[i + 1]):
            if m[r] == 0:
                continue
            if 0 <= ids[r] < V:
                row_map.append(r)
                seq_len[i] += 1
            else:
                n_bad_token += 1
    return dict(row_map=np.array(row_map, dtype=np.int64), seq_len=seq_len, n_bad_token=n_bad_token,
                n_bad_seq=int((~ok).sum()), n_bad_group=int((~grp_ok).sum()))


def group_count(group_idx, P):
    """Number of sequences that name each prompt (indices outside [0, P) belong to none)."""
    g = np.asarray(group_idx).astype(np.int64)
    return np.array([int((g == p).sum()) for p in range(P)], dtype=np.int64)


def target_logit(hidden, weight, token_ids, mask, temperature=1.0):
    """z_t[y_t] = W[y_t] . x_t / temperature for every counting row (0 on masked rows): the gather written
    as the one dot product it is, without forming the other logits."""
    X = widen(hidden); W = widen(weight)
    ids = np.asarray(token_ids).astype(np.int64)
    m = np.asarray(mask).astype(bool)
    zy = np.zeros(X.shape[0])
    for t in np.nonzero(m)[0]:
        zy[t] = float(np.dot(W[ids[t]], X[t])) / temperature
    return zy


def weight_grad_rows(hidden, weight_rows, vocab_rows, token_ids, mask, lse, c, temperature=1.0):
    """Rows `vocab_rows` of dW = dS^T X, straight from the definition, for the given rows of the batch:
         dS[t, v] = c_t (1[v = y_t] - exp(W[v] . x_t / temperature - lse_t)) / temperature,
         dW[v, :] = sum_t m_t dS[t, v] x_t.
    weight_rows = W[vocab_rows] ([n, H]).  dW is a plain sum over rows, so a large batch may be fed in
    row blocks and the results added.  lse is taken as given (it is an input here, like c)."""
    X = widen(hidden); Wr = widen(weight_rows)
    vs = np.asarray(vocab_rows).astype(np.int64)
    ids = np.asarray(token_ids).astype(np.int64)
    m = np.asarray(mask).astype(bool)
    lse = np.asarray(lse, dtype=np.float64); c = np.asarray(c, dtype=np.float64)
    rows = np.nonzero(m)[0]
    Xr = X if rows.size == m.size else X[rows]             # (no copy of a block in which every row counts)
    Z = Xr @ Wr.T / temperature                            # [n_rows, n] logits of the sampled vocabulary entries
    dS = -np.exp(Z - lse[rows][:, None])
    dS += (ids[rows][:, None] == vs[None, :])
    dS *= (c[rows] / temperature)[:, None]
    return dS.T @ Xr


# --------------------------------------------------------------------------
# group-relative advantage
# --------------------------------------------------------------------------
def group_advantage(rewards, group_idx, P, adv_eps=1e-6, ddof=0):
    """A_i = (r_i - mean_p) / (std_p + adv_eps) over the rollouts of prompt p = g(i).

    Readings: std is the population std (ddof=0) unless ddof=1 is asked for;
    adv_eps is added to the std (outside the square root), so an all-equal
    group gives exactly 0.  A group with n <= ddof members gives 0."""
    r = widen(np.asarray(rewards))
    g = np.asarray(group_idx).astype(np.int64)
    adv = np.zeros_like(r)
    for p in range(P):
        members = np.nonzero(g == p)[0]
        n = members.size
        if n == 0:
            continue
        mu = r[members].sum() / n
        if n - ddof <= 0:
            continue
        var = ((r[members] - mu) ** 2).sum() / (n - ddof)
        adv[members] = (r[members] - mu) / (np.sqrt(var) + adv_eps)
    return adv


# --------------------------------------------------------------------------
# GRPO clipped-ratio loss with the k3 KL estimator to the reference policy
# --------------------------------------------------------------------------
def grpo_loss(logp, old_logprob, ref_logprob, mask, cu_seqlens, adv, clip_eps, kl_coef):
    """loss = (1/B) sum_i (1/|y_i|) sum_t m_t l_t with
         rho_t = exp(logp_t - old_t)
         l_t   = -min(rho_t A_i, clip(rho_t, 1-eps, 1+eps) A_i) + kl_coef (e^d - d - 1),
         d     = ref_t - logp_t.
    Returns dict(loss, seq_loss[B], c[R] = dloss/dlogp_t, n_clip_hi, n_clip_lo).
    A sequence with |y_i| = 0 contributes 0 and is still counted in B.
    The gradient passes at ties (rho exactly on a clip bound, or A = 0)."""
    lp = widen(np.asarray(logp)); old = widen(np.asarray(old_logprob)); ref = widen(np.asarray(ref_logprob))
    m = np.asarray(mask).astype(bool)
    cu = np.asarray(cu_seqlens).astype(np.int64)
    B = cu.size - 1
    seq_loss = np.zeros(B)
    c = np.zeros(lp.shape[0])
    n_hi = n_lo = 0
    for i in range(B):
        rows = np.arange(cu[i], cu[i + 1])[m[cu[i]:cu[i + 1]]]
        n = rows.size
        if n == 0:
            continue
        A = adv[i]
        rho = np.exp(lp[rows] - old[rows])
        unclipped = rho * A
        clipped = np.clip(rho, 1.0 - clip_eps, 1.0 + clip_eps) * A
        d = ref[rows] - lp[rows]
        kl = np.exp(d) - d - 1.0
        l = -np.minimum(unclipped, clipped) + kl_coef * kl
        seq_loss[i] = l.sum() / n
        hi = (A > 0) & (rho > 1.0 + clip_eps)
        lo = (A < 0) & (rho < 1.0 - clip_eps)
        act = ~(hi | lo)
        n_hi += int(hi.sum()); n_lo += int(lo.sum())
        c[rows] = (-A * rho * act + kl_coef * (1.0 - np.exp(d))) / (B * n)
    return dict(loss=seq_loss.sum() / B, seq_loss=seq_loss, c=c, n_clip_hi=n_hi, n_clip_lo=n_lo)


# --------------------------------------------------------------------------
# flow-balance (trajectory-balance) loss
# --------------------------------------------------------------------------
def flow_loss(logp, old_logprob, ref_logprob, mask, cu_seqlens, adv, group_idx, log_z,
              clip_eps, beta):
    """loss = (1/B) sum_i w_i delta_i^2 with
         delta_i = logZ_{g(i)} + (1/|y_i|) sum_t m_t (logp_t - ref_t) - beta A_i
         w_i     = clip(exp(sum_t m_t (logp_t - old_t)), 1-eps, 1+eps), held constant
                   (no gradient flows through it).
    Returns dict(loss, seq_loss[B], c[R], d_log_z[P], w[B], delta[B], n_clip_hi, n_clip_lo);
    n_clip_* count sequences whose weight sits on the upper / lower bound."""
    lp = widen(np.asarray(logp)); old = widen(np.asarray(old_logprob)); ref = widen(np.asarray(ref_logprob))
    lz = widen(np.asarray(log_z))
    g = np.asarray(group_idx).astype(np.int64)
    m = np.asarray(mask).astype(bool)
    cu = np.asarray(cu_seqlens).astype(np.int64)
    B = cu.size - 1
    seq_loss = np.zeros(B); w = np.zeros(B); delta = np.zeros(B)
    c = np.zeros(lp.shape[0])
    dz = np.zeros(lz.shape[0])
    n_hi = n_lo = 0
    lo_b, hi_b = np.log(1.0 - clip_eps), np.log(1.0 + clip_eps)
    for i in range(B):
        rows = np.arange(cu[i], cu[i + 1])[m[cu[i]:cu[i + 1]]]
        n = rows.size
        if n == 0:
            continue
        log_ratio = (lp[rows] - old[rows]).sum()
        w[i] = np.exp(min(max(log_ratio, lo_b), hi_b))     # = clip(exp(.)), overflow-free
        n_hi += int(log_ratio > hi_b); n_lo += int(log_ratio < lo_b)
        delta[i] = lz[g[i]] + (lp[rows] - ref[rows]).sum() / n - beta * adv[i]
        seq_loss[i] = w[i] * delta[i] ** 2
        c[rows] = 2.0 * w[i] * delta[i] / (B * n)
        dz[g[i]] += 2.0 * w[i] * delta[i] / B
    return dict(loss=seq_loss.sum() / B, seq_loss=seq_loss, c=c, d_log_z=dz, w=w, delta=delta,
                n_clip_hi=n_hi, n_clip_lo=n_lo)


# --------------------------------------------------------------------------
# objective variants (asymmetric clip, batch token-mean aggregation, sequence-level ratio,
# length-normalised flow weight).  Written out separately from the base objectives above so that each
# can be read against its own definition; with every option at its default they reduce to them.
# --------------------------------------------------------------------------
def grpo_loss_variant(logp, old_logprob, ref_logprob, mask, cu_seqlens, adv, clip_eps, kl_coef,
                      clip_eps_high=None, aggregation="sequence", ratio_level="token"):
    """Clipped-ratio objective with the options
      clip_eps_high   upper clip bound 1 + clip_eps_high (lower stays 1 - clip_eps); None = symmetric
      aggregation     "sequence": loss = (1/B) sum_i (1/|y_i|) sum_t l_t
                      "token":    loss = (1/T) sum_i sum_t l_t, T = all counting tokens of the batch;
                                  reported seq_loss_i = (B/T) sum_t l_t, so loss = mean_i seq_loss_i either way
      ratio_level     "token":    rho_t = exp(logp_t - old_t) per token
                      "sequence": one ratio per sequence, s_i = exp((1/|y_i|) sum_t (logp_t - old_t)), used for
                                  every token of it: l_i = -min(s_i A_i, clip(s_i) A_i) + (kl_coef/|y_i|) sum_t k3_t
                                  (sequence aggregation only).
    The KL term is the per-token k3 estimator in every case.  Same return dict as grpo_loss; n_clip_* count
    tokens (token level) or sequences (sequence level)."""
    lp = widen(np.asarray(logp)); old = widen(np.asarray(old_logprob)); ref = widen(np.asarray(ref_logprob))
    m = np.asarray(mask).astype(bool)
    cu = np.asarray(cu_seqlens).astype(np.int64)
    B = cu.size - 1
    lo_c = 1.0 - clip_eps
    hi_c = 1.0 + (clip_eps if clip_eps_high is None else clip_eps_high)
    if aggregation not in ("sequence", "token") or ratio_level not in ("token", "sequence"):
        raise ValueError("option")
    if ratio_level == "sequence" and aggregation != "sequence":
        raise ValueError("sequence-level ratio goes with sequence aggregation")
    seg = [np.arange(cu[i], cu[i + 1])[m[cu[i]:cu[i + 1]]] for i in range(B)]
    T = sum(r.size for r in seg)
    seq_loss = np.zeros(B)
    c = np.zeros(lp.shape[0])
    n_hi = n_lo = 0
    for i, rows in enumerate(seg):
        n = rows.size
        if n == 0:
            continue
        A = adv[i]
        d = ref[rows] - lp[rows]
        k3 = np.exp(d) - d - 1.0
        dk3 = 1.0 - np.exp(d)                                  # d k3 / d logp
        if ratio_level == "token":
            rho = np.exp(lp[rows] - old[rows])
            surr = np.minimum(rho * A, np.clip(rho, lo_c, hi_c) * A)
            hi = (A > 0) & (rho > hi_c)
            lo = (A < 0) & (rho < lo_c)
            n_hi += int(hi.sum()); n_lo += int(lo.sum())
            l = -surr + kl_coef * k3
            g = -A * rho * ~(hi | lo) + kl_coef * dk3           # d l_t / d logp_t
            if aggregation == "sequence":
                seq_loss[i] = l.sum() / n
                c[rows] = g / (B * n)
            else:
                seq_loss[i] = l.sum() * B / T
                c[rows] = g / T
        else:
            s = np.exp((lp[rows] - old[rows]).sum() / n)
            surr = min(s * A, min(max(s, lo_c), hi_c) * A)
            hi = bool(A > 0 and s > hi_c)
            lo = bool(A < 0 and s < lo_c)
            n_hi += int(hi); n_lo += int(lo)
            seq_loss[i] = -surr + kl_coef * k3.sum() / n
            ds = 0.0 if (hi or lo) else -A * s / n               # d(-surr)/d logp_t: s depends on every token equally
            c[rows] = (ds + kl_coef * dk3 / n) / B
    return dict(loss=seq_loss.sum() / B, seq_loss=seq_loss, c=c, n_clip_hi=n_hi, n_clip_lo=n_lo)


def flow_loss_variant(logp, old_logprob, ref_logprob, mask, cu_seqlens, adv, group_idx, log_z,
                      clip_eps, beta, clip_eps_high=None, weight_norm="sum"):
    """Flow-balance objective with the options
      clip_eps_high   upper bound of the importance weight, 1 + clip_eps_high; None = symmetric
      weight_norm     "sum":  w_i = clip(exp(sum_t (logp_t - old_t)))       (the base objective)
                      "mean": w_i = clip(exp((1/|y_i|) sum_t (logp_t - old_t)))  (geometric-mean ratio)
    w stays a constant (no gradient).  Same return dict as flow_loss."""
    lp = widen(np.asarray(logp)); old = widen(np.asarray(old_logprob)); ref = widen(np.asarray(ref_logprob))
    lz = widen(np.asarray(log_z))
    g = np.asarray(group_idx).astype(np.int64)
    m = np.asarray(mask).astype(bool)
    cu = np.asarray(cu_seqlens).astype(np.int64)
    B = cu.size - 1
    if weight_norm not in ("sum", "mean"):
        raise ValueError("option")
    lo_b = np.log(1.0 - clip_eps)
    hi_b = np.log(1.0 + (clip_eps if clip_eps_high is None else clip_eps_high))
    seq_loss = np.zeros(B); w = np.zeros(B); delta = np.zeros(B)
    c = np.zeros(lp.shape[0])
    dz = np.zeros(lz.shape[0])
    n_hi = n_lo = 0
    for i in range(B):
        rows = np.arange(cu[i], cu[i + 1])[m[cu[i]:cu[i + 1]]]
        n = rows.size
        if n == 0:
            continue
        log_ratio = (lp[rows] - old[rows]).sum()
        if weight_norm == "mean":
            log_ratio = log_ratio / n
        w[i] = np.exp(min(max(log_ratio, lo_b), hi_b))
        n_hi += int(log_ratio > hi_b); n_lo += int(log_ratio < lo_b)
        delta[i] = lz[g[i]] + (lp[rows] - ref[rows]).sum() / n - beta * adv[i]
        seq_loss[i] = w[i] * delta[i] ** 2
        c[rows] = 2.0 * w[i] * delta[i] / (B * n)
        dz[g[i]] += 2.0 * w[i] * delta[i] / B
    return dict(loss=seq_loss.sum() / B, seq_loss=seq_loss, c=c, d_log_z=dz, w=w, delta=delta,
                n_clip_hi=n_hi, n_clip_lo=n_lo)


# --------------------------------------------------------------------------
# backward through log-softmax and the LM head
# --------------------------------------------------------------------------
def lm_head_backward(hidden, weight, token_ids, mask, lse, c, want_dw=True, temperature=1.0):
    """Given c_t = dloss/dlogp_t:  dS[t,v] = c_t (1[v = y_t] - p[t,v]) / temperature,
    p = exp(z - lse_t) with z = W x_t / temperature (dS is the gradient with respect to W x_t),
    dX = dS W,  dW = dS^T X.  Masked rows: dX row = 0, no contribution to dW."""
    X = widen(hidden); W = widen(weight)
    ids = np.asarray(token_ids).astype(np.int64)
    m = np.asarray(mask).astype(bool)
    R, H = X.shape
    dX = np.zeros((R, H))
    dW = np.zeros(W.shape) if want_dw else None
    for s in range(0, R, ROW_BLOCK):
        e = min(R, s + ROW_BLOCK)
        rows = np.nonzero(m[s:e])[0] + s
        if rows.size == 0:
            continue
        Z = X[rows] @ W.T
        dS = -np.exp(Z / temperature - lse[rows][:, None])
        dS[np.arange(rows.size), ids[rows]] += 1.0
        dS *= c[rows][:, None] / temperature
        dX[rows] = dS @ W
        if want_dw:
            dW += dS.T @ X[rows]
    return dX, dW


GRPO, FLOW = 0, 1


def policy_loss_fwd_bwd(objective, hidden, weight, token_ids, mask, cu_seqlens, group_idx,
                        rewards, old_logprob, ref_logprob, log_z, P,
                        clip_eps=0.2, kl_coef=1e-3, beta=15.0, adv_eps=1e-6, adv_std_ddof=0,
                        want_dw=True, want_grads=True, want_entropy=False, variant=None, temperature=1.0):
    """The whole path in the order of the problem statement: log-prob, per-sequence lengths,
    group-relative advantage, loss + per-token coefficient, backward through the LM head.
    variant: optional dict of the keyword options of grpo_loss_variant / flow_loss_variant.
    temperature: the policy is softmax(W x_t / temperature)."""
    logp, lse = token_logprob(hidden, weight, token_ids, mask, temperature)
    seq_len = segment_lengths(mask, cu_seqlens)
    adv = group_advantage(rewards, group_idx, P, adv_eps, adv_std_ddof)
    if objective == GRPO and variant:
        out = grpo_loss_variant(logp, old_logprob, ref_logprob, mask, cu_seqlens, adv, clip_eps, kl_coef, **variant)
        out["d_log_z"] = np.zeros(P)
    elif objective == FLOW and variant:
        out = flow_loss_variant(logp, old_logprob, ref_logprob, mask, cu_seqlens, adv, group_idx, log_z,
                                clip_eps, beta, **variant)
    elif objective == GRPO:
        out = grpo_loss(logp, old_logprob, ref_logprob, mask, cu_seqlens, adv, clip_eps, kl_coef)
        out["d_log_z"] = np.zeros(P)
    elif objective == FLOW:
        out = flow_loss(logp, old_logprob, ref_logprob, mask, cu_seqlens, adv, group_idx, log_z,
                        clip_eps, beta)
    else:
        raise ValueError("objective")
    out.update(logprob=logp, lse=lse, seq_len=seq_len, advantages=adv)
    if want_entropy:
        out["entropy"] = token_entropy(hidden, weight, mask, temperature)
    if want_grads:
        dX, dW = lm_head_backward(hidden, weight, token_ids, mask, lse, out["c"], want_dw, temperature)
        out["d_hidden"] = dX
        out["d_weight"] = dW
    return out
