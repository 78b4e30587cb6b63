"""GPU parity: the HIP path through the C ABI against the float64 oracle, same seeded inputs.

Tolerances (written here, from the benchmark contract): loss relative error <= 1e-5 for f32
inputs and <= 1e-2 for bf16 inputs (relative to max(|loss|, mean|seq_loss|), since the GRPO
loss is ~0 by construction); gradient max-abs error <= 2e-2 x max|grad| for bf16 and
<= 1e-4 x max|grad| for f32; masks, lengths, gathers and the set of rows carrying gradient
are exact.  Integer outputs are compared bit for bit."""
import dataclasses

import numpy as np
import pytest
import torch

from oracle import policy_oracle as orc
from paper_2603_16435_amd import binding, synth
from parity_util import (OBJ, compare_all, f64, np_bits, oracle_inputs, run_gpu, run_oracle)

pytestmark = pytest.mark.gpu

F32_TOL = dict(loss_tol=1e-5, logp_atol=2e-5, grad_tol=1e-4)
BF16_TOL = dict(loss_tol=1e-2, logp_atol=2e-3, grad_tol=2e-2)


def _say(*a):
    print(*a, flush=True)


# --------------------------------------------------------------------------- config 1 (f32), whole instance
@pytest.mark.parametrize("objective", ["grpo", "flow"])
@pytest.mark.parametrize("layout", ["padded", "packed"])
def test_tiny_f32_full(objective, layout):
    b = synth.make_rollouts("tiny", "cuda", layout)
    _say("tiny", layout, objective, "R", b.R, "T", b.T)
    ref = run_oracle(b, objective)
    for chunk in (0, 256):                      # one chunk, and several chunks with a ragged last one
        res = run_gpu(b, objective, chunk_rows=chunk)
        err = compare_all(b, res, ref, **F32_TOL)
        _say("  chunk", chunk, err)


@pytest.mark.parametrize("objective", ["grpo", "flow"])
def test_tiny_f32_heavy_clipping(objective):
    """Off-policy noise 0.3 so that both clip branches and both advantage signs occur."""
    b = synth.make_rollouts("tiny", "cuda", "packed", noise=0.3)
    ref = run_oracle(b, objective)
    if objective == "grpo":
        assert ref["n_clip_hi"] > 0 and ref["n_clip_lo"] > 0
    res = run_gpu(b, objective)
    compare_all(b, res, ref, **F32_TOL)
    st = res.stats_dict()
    assert abs(st["n_clip_hi"] - ref["n_clip_hi"]) <= 1 and abs(st["n_clip_lo"] - ref["n_clip_lo"]) <= 1


# --------------------------------------------------------------------------- configs 2-5 (bf16), token-sub-sampled instance
# every sequence cut to ceil(len/len_div) tokens at the true H, V, P, G: the oracle finishes in
# seconds to tens of seconds while the GPU run still spans several 256-row tiles, several
# vocab tiles and ragged tails; the whole pipeline is compared in full.
SUB = {"small": 16, "7b": 256, "long": 512, "32b": 1024}


@pytest.mark.parametrize("name", ["small", "7b", "long", "32b"])
def test_bf16_sub_sampled(name):
    b = synth.make_rollouts(name, "cuda", "padded", len_div=SUB[name])
    _say(name, "sub-sampled: R", b.R, "T", b.T, "H", b.cfg.H, "V", b.cfg.V)
    for objective in ("grpo", "flow"):
        ref = run_oracle(b, objective)
        for mode in ("recompute", "stash"):          # both backward modes against the same oracle result
            res = run_gpu(b, objective, chunk_rows=1024 if name == "small" else 0, mode=mode)
            err = compare_all(b, res, ref, **BF16_TOL)
            _say("  ", objective, mode, err)
        # properties that hold at any size
        dW = f64(res.d_weight)
        assert np.abs(dW.sum(0)).max() <= 1e-3 * np.abs(dW).max() * np.sqrt(dW.shape[0])
    if name == "32b":      # the configuration with all-equal reward groups: advantage exactly zero
        adv = f64(res.advantages).reshape(b.cfg.P, b.cfg.G)
        r = f64(b.rewards).reshape(b.cfg.P, b.cfg.G)
        eq = (r.max(1) == r.min(1))
        assert eq.sum() >= 3 and np.all(adv[eq] == 0.0)


# --------------------------------------------------------------------------- directed edge cases
def _edge_batch(dtype, H, V, lengths, P, G, ids=None, seed=77, layout="padded"):
    cfg = synth.RolloutConfig("edge", P, G, 1, 64, H, V, dtype, 0.5, seed=seed)
    b = synth.make_rollouts(cfg, "cuda", layout, lengths=lengths)
    if ids is not None:
        n = min(len(ids), b.R)
        b.token_ids[:n] = torch.tensor(ids[:n], dtype=torch.int32, device="cuda")
    return b


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
def test_edge_empty_and_single_token_sequences(dtype):
    # empty sequences, length-1 sequences, one group entirely empty, ragged vocab (V % 256 != 0),
    # K tail (H % 64 != 0), target ids on tile borders
    V, H = 1000, 136
    lengths = [0, 1, 5, 37, 0, 0, 0, 0, 3, 1, 64, 2]
    ids = [0, 255, 256, 511, 512, V - 1, 127, 128, 999, 1, 254, 257]
    b = _edge_batch(dtype, H, V, lengths, P=3, G=4, ids=ids)
    tol = F32_TOL if dtype == "f32" else BF16_TOL
    for objective in ("grpo", "flow"):
        ref = run_oracle(b, objective)
        res = run_gpu(b, objective)
        compare_all(b, res, ref, **tol)


def test_edge_no_tokens_at_all():
    b = _edge_batch("bf16", 64, 512, [0, 0, 0, 0], P=2, G=2)
    for objective in ("grpo", "flow"):
        res = run_gpu(b, objective)
        assert float(res.loss.item()) == 0.0
        assert torch.count_nonzero(res.d_weight) == 0 and torch.count_nonzero(res.d_hidden) == 0
        assert res.stats_dict()["n_tokens"] == 0


def test_edge_single_sequence_single_token():
    b = _edge_batch("f32", 32, 300, [1], P=1, G=1)
    for objective in ("grpo", "flow"):
        ref = run_oracle(b, objective)
        res = run_gpu(b, objective)
        compare_all(b, res, ref, **F32_TOL)


def test_zero_variance_groups_and_ddof():
    b = _edge_batch("f32", 64, 512, [8] * 8, P=2, G=4, layout="packed")
    b.rewards[:4] = 1.0                                   # group 0 all equal
    b.rewards[4:] = torch.tensor([1.0, 0.0, 0.0, 1.0], device="cuda")
    for ddof in (0, 1):
        for objective in ("grpo", "flow"):
            ref = run_oracle(b, objective, adv_std_ddof=ddof)
            res = run_gpu(b, objective, adv_std_ddof=ddof)
            compare_all(b, res, ref, **F32_TOL)
            assert torch.all(res.advantages[:4] == 0)


@pytest.mark.parametrize("layout", ["padded", "packed"])
def test_stash_mode_edges(layout):
    # single-pass backward: sequence-aligned chunks of 256 rows (empty, single-token and chunk-filling sequences,
    # several sequences per chunk, a chunk boundary after every kind), ragged vocabulary, targets on tile borders
    V, H = 1000, 128
    lengths = [0, 1, 5, 37, 0, 200, 256, 56, 3, 1, 64, 2, 190, 66, 0, 255]
    ids = [0, 255, 256, 511, 512, V - 1, 127, 128, 999, 1, 254, 257]
    b = _edge_batch("bf16", H, V, lengths, P=4, G=4, ids=ids, layout=layout)
    for objective in ("grpo", "flow"):
        ref = run_oracle(b, objective)
        res = run_gpu(b, objective, chunk_rows=256, mode="stash")
        compare_all(b, res, ref, **BF16_TOL)
        res2 = run_gpu(b, objective, chunk_rows=256, mode="stash")
        assert torch.equal(res.d_weight, res2.d_weight) and torch.equal(res.d_hidden, res2.d_hidden) and torch.equal(res.loss, res2.loss)


@pytest.mark.parametrize("mode", ["recompute", "stash"])
def test_ragged_tiles_in_every_dimension(mode):
    # H = 384: one full and one half N-tile in dX / dW; V = 1300: five full vocabulary tiles and a ragged sixth
    # (zero padding of the K-major operand of dW); 700 tokens in chunks of 512 rows: a full and a partly filled
    # chunk, i.e. XCD shares of one M-tile for some dies and none for others
    V, H = 1300, 384
    lengths = [130, 70, 100, 50, 90, 60, 120, 80]
    b = _edge_batch("bf16", H, V, lengths, P=2, G=4, layout="packed", seed=78)
    for objective in ("grpo", "flow"):
        ref = run_oracle(b, objective)
        res = run_gpu(b, objective, chunk_rows=512, mode=mode)
        compare_all(b, res, ref, **BF16_TOL)


def test_stash_mode_no_tokens_and_broken_promise():
    b = _edge_batch("bf16", 128, 512, [0, 0, 0, 0], P=2, G=2)
    res = run_gpu(b, "flow", mode="stash")
    assert float(res.loss.item()) == 0.0
    assert torch.count_nonzero(res.d_weight) == 0 and torch.count_nonzero(res.d_hidden) == 0
    # a sequence longer than promised: counted, and the loss comes back NaN instead of a silently wrong number
    b = _edge_batch("bf16", 128, 512, [6, 40, 7, 3], P=2, G=2)
    res = run_gpu(b, "grpo", mode="stash", max_seq_len=8)
    assert res.stats_dict()["n_seq_too_long"] == 1
    assert np.isnan(float(res.loss.item()))
    # the same batch with an honest promise is fine again (the flag does not stick)
    ref = run_oracle(b, "grpo")
    res = run_gpu(b, "grpo", mode="stash")
    compare_all(b, res, ref, **BF16_TOL)
    assert res.stats_dict()["n_seq_too_long"] == 0


# --------------------------------------------------------------------------- objective variants
# (oracle option dict, library keyword arguments) per objective
VARIANTS = {
    "grpo": [(dict(clip_eps_high=0.35), dict(clip_eps_high=0.35)),
             (dict(aggregation="token"), dict(aggregation="token")),
             (dict(ratio_level="sequence"), dict(ratio_level="sequence")),
             (dict(clip_eps_high=0.1, aggregation="token"), dict(clip_eps_high=0.1, aggregation="token")),
             (dict(clip_eps_high=0.3, ratio_level="sequence"), dict(clip_eps_high=0.3, ratio_level="sequence"))],
    "flow": [(dict(clip_eps_high=0.5), dict(clip_eps_high=0.5)),
             (dict(weight_norm="mean"), dict(flow_weight_norm="mean")),
             (dict(weight_norm="mean", clip_eps_high=0.05), dict(flow_weight_norm="mean", clip_eps_high=0.05))],
}


@pytest.mark.parametrize("objective", ["grpo", "flow"])
def test_objective_variants_f32(objective):
    # wide old/current noise so that both clip branches, both advantage signs and both weight bounds occur
    b = synth.make_rollouts("tiny", "cuda", "padded", noise=0.3)
    for o_opts, g_opts in VARIANTS[objective]:
        ref = run_oracle(b, objective, variant=o_opts)
        res = run_gpu(b, objective, **g_opts)
        err = compare_all(b, res, ref, **F32_TOL)
        st = res.stats_dict()
        assert abs(st["n_clip_hi"] - ref["n_clip_hi"]) <= 1 and abs(st["n_clip_lo"] - ref["n_clip_lo"]) <= 1
        _say("  variant", objective, o_opts, err, "clipped", st["n_clip_hi"], st["n_clip_lo"])


def test_sequence_level_variants_with_clipped_sequences():
    # per-sequence shifts of the old log-probs push whole sequences over either clip bound, which the per-token
    # noise alone never does for a geometric-mean ratio
    b = synth.make_rollouts("tiny", "cuda", "packed", noise=0.3)
    cu = b.cu_seqlens.cpu().numpy()
    for i, sh in enumerate([0.5, -0.5, 0.3, -0.3, 0.0, 0.25, -0.25, 0.1]):
        b.old_logprob[int(cu[i]):int(cu[i + 1])] += sh
    ref = run_oracle(b, "grpo", variant=dict(ratio_level="sequence"))
    res = run_gpu(b, "grpo", ratio_level="sequence")
    compare_all(b, res, ref, **F32_TOL)
    st = res.stats_dict()
    assert (st["n_clip_hi"], st["n_clip_lo"]) == (ref["n_clip_hi"], ref["n_clip_lo"]) and st["n_clip_hi"] + st["n_clip_lo"] >= 2
    ref = run_oracle(b, "flow", variant=dict(weight_norm="mean", clip_eps_high=0.4))
    res = run_gpu(b, "flow", flow_weight_norm="mean", clip_eps_high=0.4)
    compare_all(b, res, ref, **F32_TOL)
    st = res.stats_dict()
    assert (st["n_clip_hi"], st["n_clip_lo"]) == (ref["n_clip_hi"], ref["n_clip_lo"]) and st["n_clip_hi"] >= 1 and st["n_clip_lo"] >= 1


@pytest.mark.parametrize("mode", ["recompute", "stash"])
def test_objective_variants_bf16_both_backward_modes(mode):
    b = synth.make_rollouts("small", "cuda", "padded", len_div=16, noise=0.3)
    for objective in ("grpo", "flow"):
        for o_opts, g_opts in VARIANTS[objective][:3]:
            ref = run_oracle(b, objective, variant=o_opts)
            res = run_gpu(b, objective, chunk_rows=1024, mode=mode, **g_opts)
            err = compare_all(b, res, ref, **BF16_TOL)
            _say("  variant", objective, mode, o_opts, err)


# --------------------------------------------------------------------------- temperature
@pytest.mark.parametrize("tau", [0.7, 1.6])
def test_temperature_f32(tau):
    b = synth.make_rollouts("tiny", "cuda", "padded", noise=0.3, temperature=tau)
    for objective in ("grpo", "flow"):
        ref = run_oracle(b, objective, temperature=tau)
        res = run_gpu(b, objective, temperature=tau)
        err = compare_all(b, res, ref, **F32_TOL)
        st = res.stats_dict()
        assert abs(st["n_clip_hi"] - ref["n_clip_hi"]) <= 1 and abs(st["n_clip_lo"] - ref["n_clip_lo"]) <= 1
        _say("  temperature", tau, objective, err)
    # the scoring call under the same temperature
    lp, lse = binding.rl_token_logprob_tempered(b.hidden, b.weight, b.token_ids, b.mask, tau, b.cu_seqlens)
    torch.cuda.synchronize()
    inp = oracle_inputs(b)
    rlp, rlse = orc.token_logprob(inp["hidden"], inp["weight"], inp["token_ids"], inp["mask"], temperature=tau)
    assert np.abs(f64(lp) - rlp).max() <= 2e-5 and np.abs(f64(lse) - rlse).max() <= 2e-5


@pytest.mark.parametrize("mode", ["recompute", "stash"])
def test_temperature_bf16_both_backward_modes(mode):
    tau = 0.8
    b = synth.make_rollouts("small", "cuda", "padded", len_div=16, noise=0.3, temperature=tau)
    for objective in ("grpo", "flow"):
        ref = run_oracle(b, objective, temperature=tau)
        res = run_gpu(b, objective, chunk_rows=1024, mode=mode, temperature=tau)
        err = compare_all(b, res, ref, **BF16_TOL)
        _say("  temperature", tau, objective, mode, err)
    # temperature 1 given explicitly is the default path, bit for bit
    b1 = synth.make_rollouts("small", "cuda", "padded", len_div=16)
    a = run_gpu(b1, "grpo", chunk_rows=1024, mode=mode)
    c = run_gpu(b1, "grpo", chunk_rows=1024, mode=mode, temperature=1.0)
    for x, y in ((a.loss, c.loss), (a.logprob, c.logprob), (a.d_hidden, c.d_hidden), (a.d_weight, c.d_weight)):
        assert torch.equal(x, y)


def test_stash_mode_with_wild_old_logprobs():
    # the single-pass backward takes its reference from the old log-probs: values far from the current policy
    # (here -70 .. +5 nats) must cost range only, never correctness
    b = _edge_batch("bf16", 128, 1000, [30, 64, 17, 50], P=2, G=2, layout="packed")
    g = torch.Generator().manual_seed(9)
    b.old_logprob = (b.old_logprob.cpu() + torch.empty(b.R).uniform_(-60.0, 10.0, generator=g)).cuda()
    for objective in ("grpo", "flow"):
        ref = run_oracle(b, objective)
        res = run_gpu(b, objective, mode="stash")
        assert np.isfinite(float(res.loss.item()))
        compare_all(b, res, ref, **BF16_TOL)


def test_out_of_range_token_ids_are_masked_and_counted():
    b = _edge_batch("bf16", 64, 512, [6, 4, 7, 3], P=2, G=2, layout="packed")
    bad_rows = [1, 9, 19]
    b.token_ids[bad_rows] = torch.tensor([512, -1, 100000], dtype=torch.int32, device="cuda")
    res = run_gpu(b, "grpo")
    st = res.stats_dict()
    assert st["n_bad_token"] == 3 and st["n_tokens"] == 17
    b2 = dataclasses.replace(b, mask=b.mask.clone(), token_ids=b.token_ids.clone())
    b2.mask[bad_rows] = 0
    b2.token_ids[bad_rows] = 0
    ref = run_oracle(b2, "grpo")
    assert float(np.abs(f64(res.logprob) - ref["logprob"]).max()) < 2e-3
    assert abs(float(res.loss.item()) - ref["loss"]) <= 1e-2 * max(abs(ref["loss"]), np.abs(ref["seq_loss"]).mean())
    assert torch.count_nonzero(res.d_hidden[bad_rows]) == 0


def test_token_logprob_entry_point():
    for name, tol in (("tiny", 2e-5),):
        b = synth.make_rollouts(name, "cuda", "padded")
        lp, lse = binding.rl_token_logprob(b.hidden, b.weight, b.token_ids, b.mask, b.cu_seqlens)
        torch.cuda.synchronize()
        inp = oracle_inputs(b)
        rlp, rlse = orc.token_logprob(inp["hidden"], inp["weight"], inp["token_ids"], inp["mask"])
        assert np.abs(f64(lp) - rlp).max() <= tol and np.abs(f64(lse) - rlse).max() <= tol
        m = np_bits(b.mask).astype(bool)
        assert np.all(f64(lp)[~m] == 0)
        # without cu_seqlens: one sequence covering all rows
        lp2, _ = binding.rl_token_logprob(b.hidden, b.weight, b.token_ids, b.mask)
        assert torch.equal(lp, lp2)


def test_results_are_bit_reproducible():
    b = synth.make_rollouts("small", "cuda", "padded", len_div=16)
    a = run_gpu(b, "grpo", chunk_rows=1024)
    c = run_gpu(b, "grpo", chunk_rows=1024)
    for x, y in ((a.loss, c.loss), (a.logprob, c.logprob), (a.d_hidden, c.d_hidden), (a.d_weight, c.d_weight)):
        assert torch.equal(x, y)


# --------------------------------------------------------------------------- full size, bench launch configuration
@pytest.mark.timeout(900)
@pytest.mark.parametrize("mode", ["recompute", "stash"])
def test_7b_full_size_sampled_sequences(mode):
    """The 7B-shaped configuration at full size, padded layout, default chunking (what bench.py
    times).  The oracle cannot do 1.6e14 MACs per pass, so it computes, one by one, everything that
    belongs to the two shortest sequences (log-probs, lse, sequence loss, per-token coefficient, dX
    rows - each exact for those rows, given the whole-batch constants B and the advantages, which
    it also computes) and the rest is checked through exact integer outputs and properties that hold
    at any size: sum_v dW[v,:] = 0, <dX,X> = <dW,W>, loss = mean(seq_loss), masked rows zero."""
    b = synth.make_rollouts("7b", "cuda", "padded")
    c = b.cfg
    B = b.B
    lengths = b.lengths.numpy().astype(np.int64)
    cu = np_bits(b.cu_seqlens).astype(np.int64)
    pick = np.argsort(lengths, kind="stable")[:2]
    rows = np.concatenate([np.arange(cu[i], cu[i] + lengths[i]) for i in pick])
    rows_t = torch.from_numpy(rows).cuda()
    _say("7b full: R", b.R, "T", b.T, "oracle rows", rows.size, "sequences", pick.tolist())
    W = np_bits(b.weight)
    Xs = np_bits(b.hidden[rows_t]); ids_s = np_bits(b.token_ids[rows_t])
    old_s = np_bits(b.old_logprob[rows_t]); ref_s = np_bits(b.ref_logprob[rows_t])
    ones = np.ones(rows.size, np.uint8)
    cu_s = np.concatenate([[0], np.cumsum(lengths[pick])])
    lp_ref, lse_ref = orc.token_logprob(Xs, W, ids_s, ones)
    ent_ref = orc.token_entropy(Xs, W, ones)
    adv_ref = orc.group_advantage(np_bits(b.rewards), np_bits(b.group_idx), c.P, c.adv_eps, c.adv_std_ddof)
    gidx = np_bits(b.group_idx).astype(np.int64)
    X64 = None
    for objective in ("grpo", "flow"):
        res = run_gpu(b, objective, mode=mode)
        # exact integer work at full size
        np.testing.assert_array_equal(res.seq_len.cpu().numpy(), lengths)
        st = res.stats_dict()
        assert st["n_tokens"] == b.T and st["n_bad_token"] == 0 and st["n_bad_seq"] == 0
        np.testing.assert_allclose(f64(res.advantages), adv_ref, atol=2e-6, rtol=1e-6)
        # the sampled sequences, element by element
        assert np.abs(f64(res.logprob[rows_t]) - lp_ref).max() <= BF16_TOL["logp_atol"]
        assert np.abs(f64(res.lse[rows_t]) - lse_ref).max() <= BF16_TOL["logp_atol"]
        assert np.abs(f64(res.entropy[rows_t]) - ent_ref).max() <= BF16_TOL["logp_atol"]
        if objective == "grpo":
            o = orc.grpo_loss(lp_ref, old_s, ref_s, ones, cu_s, adv_ref[pick], c.clip_eps, c.kl_coef)
        else:
            o = orc.flow_loss(lp_ref, old_s, ref_s, ones, cu_s, adv_ref[pick], np.arange(2),
                              np_bits(b.log_z)[gidx[pick]], c.clip_eps, c.beta)
        c_ref = o["c"] * (2.0 / B)                      # the oracle normalised by its own B = 2
        sl = f64(res.seq_loss)[pick]
        assert np.abs(sl - o["seq_loss"]).max() <= BF16_TOL["loss_tol"] * max(np.abs(o["seq_loss"]).max(), 1e-30) + 1e-6
        assert np.abs(f64(res.coeff[rows_t]) - c_ref).max() <= 1e-2 * np.abs(c_ref).max()
        dX_ref, _ = orc.lm_head_backward(Xs, W, ids_s, ones, lse_ref, c_ref, want_dw=False)
        dX = f64(res.d_hidden[rows_t])
        err = np.abs(dX - dX_ref).max() / np.abs(dX_ref).max()
        _say("  ", objective, "sampled dX err", err)
        assert err <= BF16_TOL["grad_tol"]
        # properties at full size
        assert abs(float(res.loss.item()) - f64(res.seq_loss).mean()) <= 1e-5 * max(np.abs(f64(res.seq_loss)).mean(), 1e-30)
        m = b.mask.bool()
        assert int((res.d_hidden[~m] != 0).sum().item()) == 0
        assert int((res.logprob[~m] != 0).sum().item()) == 0
        assert int((res.d_hidden[m].abs().amax(1) > 0).sum().item()) == b.T
        dW = res.d_weight
        col = dW.double().sum(0).abs().max().item()
        assert col <= 1e-3 * dW.abs().max().item() * np.sqrt(dW.shape[0])
        ip_x = 0.0
        for s in range(0, b.R, 65536):
            ip_x += float((res.d_hidden[s:s + 65536].double() * b.hidden[s:s + 65536].double()).sum().item())
        ip_w = 0.0
        for s in range(0, c.V, 16384):
            ip_w += float((dW[s:s + 16384].double() * b.weight[s:s + 16384].double()).sum().item())
        scale = float(dW.double().abs().sum().item()) * 0.02 * 1e-3 + 1e-30
        _say("  ", objective, "<dX,X>", ip_x, "<dW,W>", ip_w)
        assert abs(ip_x - ip_w) <= 2e-2 * max(abs(ip_x), abs(ip_w)) + scale
        del res
    del X64
