"""Float64 CPU oracle for the log-Z head (the step just upstream of the policy-loss path).

TEST INFRASTRUCTURE ONLY: imported by the tests (and the smoke check), never by the product path; shares
no code with the HIP sources.

The benchmark contract takes "per-prompt log Z" as an input of the flow-balance objective and says nothing
about where it comes from; the mounted paper has no passage on it either.  Reading taken (stated in the
design notes as well): log Z of a prompt is a small MLP over the mean of the prompt's hidden states,

    pooled_p = mean_{t in prompt p} h_t                      (f64 mean over the prompt's rows; 0 for an empty prompt)
    a_p      = W1 pooled_p + b1                              W1 [M, H], b1 [M]
    g_p      = gelu(a_p) = a_p Phi(a_p)                      exact (erf) GELU
    logZ_p   = w2 . g_p + b2                                 w2 [M], b2 scalar

and the hidden states are treated as constants (no gradient flows into the language model through this head).
Given d_logZ (the flow objective's gradient with respect to log Z), the parameter gradients are the textbook ones:

    db2 = sum_p d_p,  dw2 = sum_p d_p g_p,  da_p = d_p w2 * gelu'(a_p),  gelu'(a) = Phi(a) + a phi(a),
    db1 = sum_p da_p, dW1 = sum_p da_p pooled_p^T.

Pinned in tests/test_logz_head_pins.py: closed forms, central finite differences, and the same network evaluated
by an independent library (torch float64 with autograd).
"""
from __future__ import annotations

import math

import numpy as np

from oracle.policy_oracle import widen

_SQRT2 = math.sqrt(2.0)
_erf = np.vectorize(math.erf, otypes=[np.float64])


def gelu(a):
    return 0.5 * a * (1.0 + _erf(a / _SQRT2))


def gelu_grad(a):
    return 0.5 * (1.0 + _erf(a / _SQRT2)) + a * np.exp(-0.5 * a * a) / math.sqrt(2.0 * math.pi)


def prompt_pool(prompt_hidden, cu_prompt):
    """pooled[p] = mean of the rows [cu[p], cu[p+1]) of prompt_hidden; an empty prompt pools to 0."""
    X = widen(prompt_hidden)
    cu = np.asarray(cu_prompt).astype(np.int64)
    P = cu.size - 1
    pooled = np.zeros((P, X.shape[1]))
    for p in range(P):
        if cu[p + 1] > cu[p]:
            pooled[p] = X[cu[p]:cu[p + 1]].sum(axis=0) / (cu[p + 1] - cu[p])
    return pooled


def logz_head_forward(prompt_hidden, cu_prompt, W1, b1, w2, b2):
    """Returns dict(log_z[P], pooled[P,H], a[P,M], g[P,M])."""
    pooled = prompt_pool(prompt_hidden, cu_prompt)
    W1 = widen(W1); b1 = widen(b1); w2 = widen(w2)
    a = pooled @ W1.T + b1
    g = gelu(a)
    return dict(log_z=g @ w2 + float(b2), pooled=pooled, a=a, g=g)


def logz_head_backward(fwd, W1, w2, d_log_z):
    """Parameter gradients from the forward's intermediates and d_logZ[P]: dict(dW1, db1, dw2, db2)."""
    d = widen(np.asarray(d_log_z))
    w2 = widen(w2)
    da = d[:, None] * w2[None, :] * gelu_grad(fwd["a"])
    return dict(dW1=da.T @ fwd["pooled"], db1=da.sum(axis=0), dw2=fwd["g"].T @ d, db2=float(d.sum()))
