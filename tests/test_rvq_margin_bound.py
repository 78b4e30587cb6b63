"""The rounding bound that the GPU residual-VQ kernel's exactness rests on, checked on the CPU.

The kernel scores entries in float32, s = r.c - |c|^2/2 over D = 128 bf16 components, and takes a decision from those
scores only when the winner leads by more than 2 g (|r| c_max + c_max^2 / 2), g = 2^-16; everything closer is settled in
float64.  That is exact provided a float32 score is within g (|r||c| + |c|^2/2) of its exact value, however the 128 exact
products are summed.  This file checks that premise by emulation: several summation orders (in sequence, reversed,
pairwise, four chained blocks of 32 started from -|c|^2/2 as on the matrix cores), with every addition rounded to nearest
or truncated towards zero, on data chosen to be hard (cancellation, wide dynamic range, one dominant term), and the
consequence: a lead of more than the margin in float32 is a lead in exact arithmetic."""
import numpy as np
import torch

G = 2.0 ** -16


def _bf16(a):
    return torch.from_numpy(np.asarray(a, dtype=np.float32)).to(torch.bfloat16).float().numpy()


def _rn(x):                      # float64 -> float32, round to nearest even
    return np.float32(x)


def _rz(x):                      # float64 -> float32, truncated towards zero
    y = np.float32(x)
    if abs(np.float64(y)) > abs(x):
        y = np.nextafter(y, np.float32(0.0))
    return y


def _add(a, b, rnd):
    return rnd(np.float64(a) + np.float64(b))


def _sum_orders(prod, start, rnd):
    """float32 sums of `start` and the (exact, float32-representable) products under different orders"""
    out = []
    acc = start
    for p in prod: acc = _add(acc, p, rnd)
    out.append(acc)
    acc = start
    for p in prod[::-1]: acc = _add(acc, p, rnd)
    out.append(acc)
    level = [np.float32(p) for p in prod]            # pairwise tree, the start value added last
    while len(level) > 1:
        level = [_add(level[i], level[i + 1], rnd) for i in range(0, len(level), 2)]
    out.append(_add(level[0], start, rnd))
    acc = start                                        # four chained blocks of 32, each block summed as a tree first
    for b in range(4):
        level = [np.float32(p) for p in prod[32 * b:32 * b + 32]]
        while len(level) > 1:
            level = [_add(level[i], level[i + 1], rnd) for i in range(0, len(level), 2)]
        acc = _add(acc, level[0], rnd)
    out.append(acc)
    acc = start                                        # the same, each block summed in sequence
    for b in range(4):
        for p in prod[32 * b:32 * b + 32]: acc = _add(acc, p, rnd)
    out.append(acc)
    return out


def _cases(rng):
    D = 128
    for kind in range(6):
        for _ in range(12):
            r = rng.standard_normal(D); c = rng.standard_normal(D)
            if kind == 1: c = r + 1e-2 * rng.standard_normal(D)                     # nearly parallel: large score
            if kind == 2: c = -r + 1e-2 * rng.standard_normal(D)                    # nearly opposite
            if kind == 3: r *= 10.0 ** rng.uniform(-6, 6, D)                         # wide dynamic range
            if kind == 4: r[::2] = 1.0; r[1::2] = -1.0; c[:] = 1.0 + 2 ** -7 * rng.integers(0, 2, D)   # total cancellation
            if kind == 5: r[7] = 3e4; c[7] = 2e4                                     # one dominant term
            yield _bf16(r).astype(np.float64), _bf16(c).astype(np.float64)


def test_a_float32_score_is_within_the_bound_whatever_the_order_and_the_rounding():
    rng = np.random.default_rng(20260316)
    worst = 0.0
    for r, c in _cases(rng):
        prod = (r * c).astype(np.float64)                                           # exact: 8-bit x 8-bit significands
        assert np.all(prod == np.float32(prod).astype(np.float64))
        n2 = np.float32(0.0)
        for x in c: n2 = np.float32(np.float32(x) * np.float32(x) + n2)             # the norm as the norms kernel sums it (float32, in index order)
        exact = float(np.sum(prod) - 0.5 * np.sum(c * c))
        bound = G * (np.linalg.norm(r) * np.linalg.norm(c) + 0.5 * np.sum(c * c))
        for rnd in (_rn, _rz):
            start = rnd(np.float64(-0.5) * np.float64(n2))
            for s in _sum_orders(prod, start, rnd):
                err = abs(float(s) - exact)
                assert err <= bound, (err, bound)
                worst = max(worst, err / bound)
    assert worst > 1e-4          # the check is not vacuous: errors of a visible fraction of the bound occur (truncation, cancellation)


def test_a_lead_beyond_the_margin_in_float32_is_a_lead_in_exact_arithmetic():
    rng = np.random.default_rng(7)
    D, S = 128, 64
    n_decided = n_close = 0
    for trial in range(40):
        r = _bf16(rng.standard_normal(D)).astype(np.float64)
        base = rng.standard_normal((S, D))
        C = _bf16(base).astype(np.float64)
        if trial % 2:                                                                # near-duplicates: pairs that differ by 2^-8 of one small component
            C[1::2] = C[0::2]
            C[1::2, 0] = _bf16(C[0::2, 0] * (1.0 + 2.0 ** -7) * 2.0 ** -6)
            C[0::2, 0] = _bf16(C[0::2, 0] * 2.0 ** -6)
        exact = C @ r - 0.5 * np.sum(C * C, axis=1)
        s32 = np.empty(S, dtype=np.float32)
        for j in range(S):
            n2 = np.float32(0.0)
            for x in C[j]: n2 = np.float32(np.float32(x) * np.float32(x) + n2)
            s32[j] = _sum_orders(r * C[j], _rz(np.float64(-0.5) * np.float64(n2)), _rz)[3]
        cmax2 = float(np.max(np.sum(C * C, axis=1)))
        margin = 2 * G * (np.linalg.norm(r) * np.sqrt(cmax2) + 0.5 * cmax2)
        order = np.argsort(-s32.astype(np.float64), kind="stable")
        w, ru = order[0], order[1]
        if float(s32[w]) - float(s32[ru]) > margin:
            n_decided += 1
            assert int(np.argmax(exact)) == int(w)
        else:
            n_close += 1
            near = [j for j in range(S) if not (float(s32[w]) - float(s32[j]) > margin)]
            assert int(np.argmax(exact)) in near                                     # the exact winner is among the entries within the margin
    assert n_decided >= 10 and n_close >= 5
