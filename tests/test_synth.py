"""Seeded synthetic rollout generator: determinism, shapes, distributions (CPU)."""
import math

import numpy as np
import torch

from paper_2603_16435_amd import synth


def test_counter_based_streams_are_chunk_independent():
    a = synth.normal(7, 3, 0, 1000, "cpu")
    b = torch.cat([synth.normal(7, 3, 0, 333, "cpu"), synth.normal(7, 3, 333, 667, "cpu")])
    assert torch.equal(a, b)
    assert not torch.equal(a, synth.normal(8, 3, 0, 1000, "cpu"))
    assert not torch.equal(a, synth.normal(7, 4, 0, 1000, "cpu"))
    z = synth.normal(1, 1, 0, 200000, "cpu").double()
    assert abs(z.mean()) < 0.01 and abs(z.std() - 1) < 0.01
    u = synth.uniform01(1, 2, 0, 200000, "cpu").double()
    assert 0 < u.min() and u.max() < 1 and abs(u.mean() - 0.5) < 0.005


def test_tiny_batch_layouts():
    for layout in ("padded", "packed"):
        b = synth.make_rollouts("tiny", "cpu", layout)
        c = b.cfg
        assert b.B == 8 and b.hidden.shape == (b.R, c.H) and b.weight.shape == (c.V, c.H)
        assert b.hidden.dtype == torch.float32
        ln = b.lengths.long()
        assert ln.min() >= 16 and ln.max() <= 64 and int(ln.sum()) == b.T
        cu = b.cu_seqlens.long()
        assert cu[0] == 0 and cu[-1] == b.R
        for i in range(b.B):
            assert int(b.mask[cu[i]:cu[i + 1]].sum()) == int(ln[i])
        assert b.token_ids.min() >= 0 and b.token_ids.max() < c.V
        assert set(b.rewards.tolist()) <= {0.0, 1.0}
        assert torch.equal(b.group_idx.long(), torch.arange(8) // 4)
    again = synth.make_rollouts("tiny", "cpu", "packed")
    assert torch.equal(again.hidden, b.hidden) and torch.equal(again.old_logprob, b.old_logprob)


def test_value_distributions_and_closed_form_current():
    b = synth.make_rollouts("tiny", "cpu", "packed")
    assert abs(float(b.hidden.std()) - 1.0) < 0.02
    assert abs(float(b.weight.std()) - 0.02) < 0.001
    # old/ref sit close to the true log-prob (closed-form stand-in + N(0,0.05))
    z = b.hidden.double() @ b.weight.double().T
    lp = torch.log_softmax(z, 1)[torch.arange(b.R), b.token_ids.long()]
    assert float((b.old_logprob.double() - lp).std()) < 0.08
    assert float((b.old_logprob.double() - lp).abs().max()) < 0.4


def test_sub_sampled_and_equal_groups():
    b = synth.make_rollouts(synth.CONFIGS["32b"].__class__(
        "mini32", 32, 8, 1024, 8192, 16, 64, "bf16", 0.5, equal_group_frac=0.1, seed=5), "cpu",
        "packed", len_div=512)
    assert b.hidden.dtype == torch.bfloat16
    full = synth.sequence_lengths(b.cfg)
    assert torch.equal(b.lengths.long(), (full + 511) // 512)
    r = b.rewards.view(32, 8)
    n_equal = int(((r.max(1).values - r.min(1).values) == 0).sum())
    assert n_equal >= 3
    b2 = synth.make_rollouts("tiny", "cpu", "padded", lengths=[0, 1, 5, 64, 3, 0, 2, 1])
    assert b2.T == 76 and b2.R == 8 * 64
