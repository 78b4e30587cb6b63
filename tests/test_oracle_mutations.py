"""The pins must bite: plant one plausible mistake at a time in a copy of the oracle (on the CPU,
by patching its source text) and check that at least one pin test fails for every mutant."""
import importlib
import inspect
import os
import sys
import types

import pytest

import test_oracle_pins as pins
from oracle import policy_oracle as orc

MUTANTS = [
    # (name, text to find, replacement)
    ("logits transposed operand", "Z = X[rows] @ W.T                       # [n, V] logits", "Z = (W @ X[rows].T).T[:, ::-1]"),
    ("lse without the max added back", "l = M + np.log(np.exp(Z - M[:, None]).sum(axis=1))", "l = np.log(np.exp(Z - M[:, None]).sum(axis=1))"),
    ("logp sign", "logp[rows] = zy - l", "logp[rows] = l - zy"),
    ("gather wrong index", "zy = Z[np.arange(rows.size), ids[rows]]", "zy = Z[np.arange(rows.size), (ids[rows] + 1) % Z.shape[1]]"),
    ("entropy sign", "ent[rows] = -term.sum(axis=1)", "ent[rows] = term.sum(axis=1)"),
    ("advantage: eps inside the root", "adv[members] = (r[members] - mu) / (np.sqrt(var) + adv_eps)", "adv[members] = (r[members] - mu) / np.sqrt(var + adv_eps)"),
    ("advantage: no mean subtraction", "adv[members] = (r[members] - mu) / (np.sqrt(var) + adv_eps)", "adv[members] = r[members] / (np.sqrt(var) + adv_eps)"),
    ("grpo: max instead of min", "l = -np.minimum(unclipped, clipped) + kl_coef * kl", "l = -np.maximum(unclipped, clipped) + kl_coef * kl"),
    ("grpo: dropped KL term", "l = -np.minimum(unclipped, clipped) + kl_coef * kl", "l = -np.minimum(unclipped, clipped)"),
    ("grpo: KL direction", "d = ref[rows] - lp[rows]\n        kl", "d = lp[rows] - ref[rows]\n        kl"),
    ("grpo: token-sum instead of token-mean", "seq_loss[i] = l.sum() / n\n        hi", "seq_loss[i] = l.sum()\n        hi"),
    ("grpo: gradient ignores clipping", "c[rows] = (-A * rho * act + kl_coef * (1.0 - np.exp(d))) / (B * n)", "c[rows] = (-A * rho + kl_coef * (1.0 - np.exp(d))) / (B * n)"),
    ("grpo: gradient KL sign", "c[rows] = (-A * rho * act + kl_coef * (1.0 - np.exp(d))) / (B * n)", "c[rows] = (-A * rho * act - kl_coef * (1.0 - np.exp(d))) / (B * n)"),
    ("grpo: gradient normaliser", "c[rows] = (-A * rho * act + kl_coef * (1.0 - np.exp(d))) / (B * n)", "c[rows] = (-A * rho * act + kl_coef * (1.0 - np.exp(d))) / B"),
    ("flow: reference term not length-normalised", "delta[i] = lz[g[i]] + (lp[rows] - ref[rows]).sum() / n - beta * adv[i]", "delta[i] = lz[g[i]] + (lp[rows] - ref[rows]).sum() - beta * adv[i]"),
    ("flow: reward sign", "delta[i] = lz[g[i]] + (lp[rows] - ref[rows]).sum() / n - beta * adv[i]", "delta[i] = lz[g[i]] + (lp[rows] - ref[rows]).sum() / n + beta * adv[i]"),
    ("flow: unclipped weight", "w[i] = np.exp(min(max(log_ratio, lo_b), hi_b))", "w[i] = np.exp(min(log_ratio, 50.0))"),
    ("flow: gradient factor 2 dropped", "c[rows] = 2.0 * w[i] * delta[i] / (B * n)", "c[rows] = w[i] * delta[i] / (B * n)"),
    ("flow: d_logZ to the wrong prompt", "dz[g[i]] += 2.0 * w[i] * delta[i] / B", "dz[(g[i] + 1) % dz.size] += 2.0 * w[i] * delta[i] / B"),
    ("backward: softmax minus onehot sign", "dS = -np.exp(Z / temperature - lse[rows][:, None])\n        dS[np.arange(rows.size), ids[rows]] += 1.0", "dS = np.exp(Z / temperature - lse[rows][:, None])\n        dS[np.arange(rows.size), ids[rows]] -= 1.0"),
    ("backward: dX with transposed weight use", "dX[rows] = dS @ W", "dX[rows] = (dS * 0 + dS.mean(1, keepdims=True)) @ W"),
    ("backward: dW without the transpose", "dW += dS.T @ X[rows]", "dW += (X[rows].T @ dS).T * 0 + dS.T @ np.roll(X[rows], 1, axis=1)"),
    ("backward: masked rows leak", "rows = np.nonzero(m[s:e])[0] + s\n        if rows.size == 0:\n            continue\n        Z = X[rows] @ W.T\n        dS", "rows = np.arange(s, e)\n        if rows.size == 0:\n            continue\n        Z = X[rows] @ W.T\n        dS"),
    ("bf16 widening shifts by 15", "<< np.uint32(16)", "<< np.uint32(15)"),
    ("variant: upper bound uses the lower epsilon", "hi_c = 1.0 + (clip_eps if clip_eps_high is None else clip_eps_high)", "hi_c = 1.0 + clip_eps"),
    ("variant: token aggregation normalised by B n", "                c[rows] = g / T", "                c[rows] = g / (B * n)"),
    ("variant: token aggregation seq_loss scale", "seq_loss[i] = l.sum() * B / T", "seq_loss[i] = l.sum() / T"),
    ("variant: sequence ratio without the length normalisation", "s = np.exp((lp[rows] - old[rows]).sum() / n)", "s = np.exp((lp[rows] - old[rows]).sum())"),
    ("variant: sequence ratio gradient ignores clipping", "ds = 0.0 if (hi or lo) else -A * s / n", "ds = -A * s / n"),
    ("variant: sequence ratio KL not averaged", "seq_loss[i] = -surr + kl_coef * k3.sum() / n", "seq_loss[i] = -surr + kl_coef * k3.sum()"),
    ("variant: flow mean weight not divided", "            log_ratio = log_ratio / n", "            log_ratio = log_ratio * 1.0"),
    ("temperature multiplies the logits", "        Z = Z / temperature\n", "        Z = Z * temperature\n"),
    ("temperature: entropy of the untempered distribution", "Z = X[rows] @ W.T / temperature\n", "Z = X[rows] @ W.T\n"),
    ("temperature: backward probabilities untempered", "dS = -np.exp(Z / temperature - lse[rows][:, None])", "dS = -np.exp(Z - lse[rows][:, None])"),
    ("temperature: chain factor dropped in the backward", "dS *= c[rows][:, None] / temperature", "dS *= c[rows][:, None]"),
    ("variant: flow upper bound", "hi_b = np.log(1.0 + (clip_eps if clip_eps_high is None else clip_eps_high))", "hi_b = np.log(1.0 + clip_eps)"),
    ("compaction: out-of-range ids counted", "            if 0 <= ids[r] < V:\n", "            if True:\n"),
    ("compaction: masked rows counted", "            if m[r] == 0:\n                continue\n", ""),
    ("compaction: overlapping ranges kept", "ok[i] = (0 <= cu[i] <= cu[i + 1] <= R) and cu[i] >= highest", "ok[i] = (0 <= cu[i] <= cu[i + 1] <= R)"),
    ("compaction: bad prompt index keeps its rows", "        if not (ok[i] and grp_ok[i]):", "        if not ok[i]:"),
    ("target logit: wrong row of W", "zy[t] = float(np.dot(W[ids[t]], X[t])) / temperature", "zy[t] = float(np.dot(W[(ids[t] + 1) % W.shape[0]], X[t])) / temperature"),
    ("dW rows: one-hot dropped", "    dS += (ids[rows][:, None] == vs[None, :])\n", ""),
    ("dW rows: chain factor of the temperature dropped", "    dS *= (c[rows] / temperature)[:, None]", "    dS *= c[rows][:, None]"),
    ("dW rows: masked rows leak", "    rows = np.nonzero(m)[0]\n    Xr = X if", "    rows = np.arange(m.size)\n    Xr = X if"),
]

PIN_TESTS = [(n, f) for n, f in inspect.getmembers(pins, inspect.isfunction) if n.startswith("test_")]


def _run_pins_against(mod):
    """Names of the pin tests that fail when the pins module sees `mod` as the oracle."""
    failed = []
    saved = pins.orc
    pins.orc = mod
    try:
        for name, fn in PIN_TESTS:
            marks = [m for m in getattr(fn, "pytestmark", []) if m.name == "parametrize"]
            argsets = [()]
            if marks:
                argsets = [(v,) for v in marks[0].args[1]]
            for a in argsets:
                try:
                    fn(*a)
                except Exception:       # assertion, numerical error, shape error: all count as caught
                    failed.append(name)
                    break
    finally:
        pins.orc = saved
    return failed


def test_unmutated_oracle_passes_every_pin():
    assert _run_pins_against(orc) == []


@pytest.mark.parametrize("name,find,repl", MUTANTS, ids=[m[0] for m in MUTANTS])
def test_every_planted_mistake_is_caught(name, find, repl):
    src = inspect.getsource(orc)
    assert src.count(find) >= 1, f"mutation site not found: {name}"
    mutated = src.replace(find, repl, 1)
    mod = types.ModuleType("oracle_mutant")
    mod.__dict__["__name__"] = "oracle_mutant"
    exec(compile(mutated, "oracle_mutant.py", "exec"), mod.__dict__)
    failed = _run_pins_against(mod)
    assert failed, f"no pin notices: {name}"
