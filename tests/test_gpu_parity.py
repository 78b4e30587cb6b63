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
from parity_util import (OBJ, check_index_work, cleaned_packed, compare_all, f64, np_bits, oracle_inputs, run_gpu, run_oracle)

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
        err = compare_all(b, res, ref, temperature=tau, **F32_TOL)
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
        err = compare_all(b, res, ref, temperature=tau, **BF16_TOL)
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



# --------------------------------------------------------------------------- data errors found on the device
def _compare_with_cleaned(b, res, objective, tol, **kw):
    """Outputs of a batch with broken offsets / prompt indices / token ids against the oracle on the cleaned batch
    (only the rows that count, packed): per-row outputs are gathered through the oracle's own row map."""
    inp, cr = cleaned_packed(b)
    c = b.cfg
    ref = orc.policy_loss_fwd_bwd(OBJ[objective][0], clip_eps=c.clip_eps, kl_coef=c.kl_coef, beta=c.beta, adv_eps=c.adv_eps,
                                  adv_std_ddof=c.adv_std_ddof, want_entropy=True, **inp, **kw)
    rows = cr["row_map"]
    st = res.stats_dict()
    assert (st["n_tokens"], st["n_bad_token"], st["n_bad_seq"], st["n_bad_group"]) == (rows.size, cr["n_bad_token"], cr["n_bad_seq"], cr["n_bad_group"])
    check_index_work(b, res, clean=cr)
    other = np.ones(b.R, dtype=bool); other[rows] = False
    lp = f64(res.logprob); dX = f64(res.d_hidden)
    assert np.all(lp[other] == 0) and np.all(f64(res.lse)[other] == 0) and np.all(f64(res.coeff)[other] == 0) and np.all(dX[other] == 0)
    assert np.all(np.isfinite(dX)) and np.all(np.isfinite(f64(res.d_weight)))
    assert np.abs(lp[rows] - ref["logprob"]).max() <= tol["logp_atol"]
    assert np.abs(f64(res.entropy)[rows] - ref["entropy"]).max() <= tol["logp_atol"]
    scale = max(abs(ref["loss"]), float(np.abs(ref["seq_loss"]).mean()), 1e-30)
    assert abs(float(res.loss.item()) - ref["loss"]) <= tol["loss_tol"] * scale
    assert np.abs(f64(res.seq_loss) - ref["seq_loss"]).max() <= tol["loss_tol"] * max(np.abs(ref["seq_loss"]).max(), 1e-30)
    np.testing.assert_allclose(f64(res.advantages), ref["advantages"], atol=2e-6, rtol=1e-6)
    assert np.abs(f64(res.coeff)[rows] - ref["c"]).max() <= max(tol["loss_tol"], 1e-4) * np.abs(ref["c"]).max()
    assert np.abs(dX[rows] - ref["d_hidden"]).max() <= tol["grad_tol"] * np.abs(ref["d_hidden"]).max()
    assert np.abs(f64(res.d_weight) - ref["d_weight"]).max() <= tol["grad_tol"] * np.abs(ref["d_weight"]).max()
    np.testing.assert_allclose(f64(res.d_log_z), ref["d_log_z"], atol=tol["loss_tol"] * max(1.0, float(np.abs(ref["d_log_z"]).max())))


@pytest.mark.parametrize("mode", ["recompute", "stash"])
def test_broken_offsets_and_prompt_indices_are_counted_and_harmless(mode):
    """Offsets that decrease and rise again (ranges that would overlap), a last offset beyond the rows, prompt indices
    outside [0, P) and token ids outside [0, V): the offending sequences / rows count as empty / masked, the counters
    say so, nothing beyond the R rows is touched and everything else equals the oracle on the cleaned batch."""
    b = _edge_batch("bf16", 128, 1000, [20, 30, 25, 40, 35, 10, 15, 45], P=2, G=4, layout="packed", seed=80)
    R = b.R                                                    # 220 rows; well-formed offsets 0 20 50 75 115 150 160 175 220
    cases = {
        "alternating": [0, R, 0, R, 0, R, 0, R, 0],            # every second range is the whole batch: one may be kept
        "dip": [0, 20, 50, 30, 115, 150, 160, 175, R],         # decreasing, then rising again from below an earlier offset
        "beyond": [0, 20, 50, 75, 115, 150, 160, 175, R + 40], # the last sequence runs past the rows
        "negative": [-5, 20, 50, 75, 115, 150, 160, 175, R],
    }
    guard = torch.full((64,), 12345, dtype=torch.int32, device="cuda")
    for name, cu in cases.items():
        bb = dataclasses.replace(b, cu_seqlens=torch.tensor(cu, dtype=torch.int32, device="cuda"))
        for objective in ("grpo", "flow"):
            res = run_gpu(bb, objective, mode=mode, max_seq_len=R) if mode == "stash" else run_gpu(bb, objective, mode=mode)
            _say("  offsets", name, objective, mode, res.stats_dict())
            assert res.stats_dict()["n_bad_seq"] >= 1
            _compare_with_cleaned(bb, res, objective, BF16_TOL)
    # prompt indices out of range (and a few token ids as well)
    bb = dataclasses.replace(b, group_idx=b.group_idx.clone(), token_ids=b.token_ids.clone())
    bb.group_idx[2] = 2; bb.group_idx[5] = -1
    bb.token_ids[[3, 60, 219]] = torch.tensor([1000, -7, 1 << 30], dtype=torch.int32, device="cuda")
    for objective in ("grpo", "flow"):
        res = run_gpu(bb, objective, mode=mode)
        st = res.stats_dict()
        # row 60 lies in sequence 2, which is dropped for its prompt index: its bad id is not looked at any more
        assert st["n_bad_group"] == 2 and st["n_bad_token"] == 2 and st["n_bad_seq"] == 0
        assert res.group_count.cpu().tolist() == [3, 3]
        _compare_with_cleaned(bb, res, objective, BF16_TOL)
    assert torch.all(guard == 12345)


def test_index_work_is_exact_on_both_layouts_f32():
    # the order of the counting rows, group sizes and the vocabulary entry every target logit was read from, with
    # out-of-range ids among the rows (f32 inputs: the generic kernel's gather)
    for layout in ("padded", "packed"):
        b = synth.make_rollouts("tiny", "cuda", layout)
        b.token_ids[[0, 7]] = torch.tensor([-1, 1024], dtype=torch.int32, device="cuda")
        res = run_gpu(b, "grpo")
        _compare_with_cleaned(b, res, "grpo", F32_TOL)
        assert res.stats_dict()["n_bad_token"] == int(b.mask[[0, 7]].sum().item())


def test_single_pass_mode_reports_rows_beyond_its_range():
    """One token whose current log-prob lies some 250 nats below its old one: the single-pass backward cannot hold
    its probabilities in range.  It must say so (counter, NaN loss) instead of returning a finite loss next to
    gradients that are not numbers; the mode that recomputes the logits handles the same batch and matches the oracle."""
    b = _edge_batch("bf16", 128, 1000, [30, 64, 17, 50], P=2, G=2, layout="packed", seed=81)
    t = 40
    y = int(b.token_ids[t].item())
    b.hidden[t] = (-4000.0 * b.weight[y].float()).to(torch.bfloat16)
    for objective in ("grpo", "flow"):
        kw = dict(kl_coef=0.0)                                 # the KL term alone would overflow f32 here
        ref = run_oracle(b, objective, **kw)
        assert ref["logprob"][t] < -150
        res = run_gpu(b, objective, mode="recompute", **kw)
        compare_all(b, res, ref, **BF16_TOL)
        res = run_gpu(b, objective, mode="stash", **kw)
        st = res.stats_dict()
        _say("  out of range row:", objective, st)
        assert st["n_overflow_rows"] == 1 and np.isnan(float(res.loss.item()))
        # the flag does not stick
        b2 = _edge_batch("bf16", 128, 1000, [30, 64, 17, 50], P=2, G=2, layout="packed", seed=81)
        res = run_gpu(b2, objective, mode="stash")
        assert res.stats_dict()["n_overflow_rows"] == 0 and np.isfinite(float(res.loss.item()))


# --------------------------------------------------------------------------- full size, bench launch configuration
N_SAMPLE_ROWS = 320
N_SAMPLE_VOCAB = 16


def _wide(t):
    """Exact float64 copy of a stored tensor (every bf16 / f32 value is a float64 value): the same numbers the oracle's own
    widening of the bit patterns gives, produced on the device because the host pass over 1e10 elements takes minutes."""
    return t.detach().to(torch.float64).cpu().numpy()


@pytest.mark.timeout(1100)
@pytest.mark.parametrize("name", ["7b", "long", "32b"])
def test_full_size_sampled(name):
    """The three large configurations at full size, padded layout, default chunking (the launch configuration
    bench.py times), both objectives under both backward modes.  The oracle cannot do 1e14-1e15 multiply-adds per
    pass, so:

      (a) exact integer work at full size: sequence lengths, the order of the counting rows, group sizes, the
          vocabulary entry every target logit was read from, zeros on masked rows;
      (b) element by element, computed by the oracle from the inputs alone: log-prob, lse, entropy and the target
          logit of about N_SAMPLE_ROWS seeded rows spread over EVERY chunk of compacted rows (first and last row of
          each chunk of either mode and of the partly filled last chunk included), the group advantages;
      (c) the O(T) stages re-run by the oracle in full from the GPU's log-probs (which (b) spot-checks): loss, every
          sequence loss, every per-token coefficient, d_logZ - CONDITIONAL on the spot-checked log-probs;
      (d) the dX rows of the sampled rows, from the oracle's own lse and the coefficients of (c);
      (e) N_SAMPLE_VOCAB rows of dW element by element (vocabulary entries 0 and V-1, one in the ragged last tile, a
          sampled target id, the rest seeded), the sum over ALL T rows taken by the oracle from the GPU's lse and
          coefficients - CONDITIONAL on the spot-checked lse and on (c);
      (f) properties that hold at any size: sum_v dW[v,:] = 0, <dX,X> = <dW,W>, loss = mean(seq_loss)."""
    b = synth.make_rollouts(name, "cuda", "padded")
    c = b.cfg
    B, V, H = b.B, c.V, c.H
    cr_len = b.lengths.numpy().astype(np.int64)
    T = int(cr_len.sum())
    rng = np.random.default_rng(c.seed)
    # compacted positions to sample: the borders of the fixed chunks of both modes, sequence starts (where the
    # sequence-aligned chunks of the single-pass mode begin) and seeded positions inside every chunk
    pos = {0, T - 1}
    chunkings = {"recompute": binding.lib().rl_default_chunk_rows(), "stash": binding.lib().rl_default_chunk_rows_single_pass()}
    for tc in chunkings.values():
        n_chunks = -(-T // tc)
        for k in range(n_chunks):
            lo, hi = k * tc, min(T, (k + 1) * tc)
            pos.update({lo, hi - 1})
            pos.update(int(x) for x in rng.integers(lo, hi, size=max(2, (N_SAMPLE_ROWS // 2 - 2 * n_chunks - 8) // n_chunks)))
    starts = np.concatenate([[0], np.cumsum(cr_len)])
    pos.update(int(x) for x in starts[rng.integers(0, B, size=8)] if x < T)
    pos = np.array(sorted(pos))
    # padded layout: compacted position k of sequence i is original row i*Lmax + (k - starts[i])
    Lmax = b.R // B
    seq_of = np.searchsorted(starts, pos, side="right") - 1
    rows = seq_of * Lmax + (pos - starts[seq_of])
    rows_t = torch.from_numpy(rows).cuda()
    assert rows.size >= 256
    _say(name, "full: R", b.R, "T", T, "chunk rows", chunkings, "sampled rows", rows.size)
    W64 = _wide(b.weight)
    np.testing.assert_array_equal(W64[:64], orc.widen(np_bits(b.weight[:64])))          # the same numbers as the oracle's widening
    Xs = np_bits(b.hidden[rows_t]); ids_s = np_bits(b.token_ids[rows_t])
    ones = np.ones(rows.size, np.uint8)
    lp_ref, lse_ref = orc.token_logprob(Xs, W64, ids_s, ones)
    ent_ref = orc.token_entropy(Xs, W64, ones)
    zy_ref = orc.target_logit(Xs, W64, ids_s, ones)
    adv_ref = orc.group_advantage(np_bits(b.rewards), np_bits(b.group_idx), c.P, c.adv_eps, c.adv_std_ddof)
    _say("   oracle: sampled rows done")
    mask_np = np_bits(b.mask); cu_np = np_bits(b.cu_seqlens); gidx = np_bits(b.group_idx)
    old_np = np_bits(b.old_logprob); refp_np = np_bits(b.ref_logprob)
    ids_np = np_bits(b.token_ids)
    m_t = b.mask.bool()
    # vocabulary rows for the dW check
    vs = {0, V - 1, (V // 256) * 256 + 1 if V % 256 else V - 2, int(ids_s[len(ids_s) // 2])}
    while len(vs) < N_SAMPLE_VOCAB:
        vs.add(int(rng.integers(0, V)))
    vs = np.array(sorted(vs))
    Wv = W64[vs]
    vs_t = torch.from_numpy(vs).cuda()
    runs = {}
    for mode in ("recompute", "stash"):
      for objective in ("grpo", "flow"):
        res = run_gpu(b, objective, mode=mode)
        st = res.stats_dict()
        tag = f"{mode}/{objective}"
        # (a)
        np.testing.assert_array_equal(res.seq_len.cpu().numpy(), cr_len)
        assert st["n_tokens"] == T and st["n_bad_token"] == 0 and st["n_bad_seq"] == 0 and st["n_bad_group"] == 0 and st["n_overflow_rows"] == 0
        rm = res.row_map.cpu().numpy()
        np.testing.assert_array_equal(rm[:T], np.flatnonzero(mask_np))
        assert np.all(rm[T:] == -1)
        np.testing.assert_array_equal(res.group_count.cpu().numpy(), orc.group_count(gidx, c.P))
        assert bool(torch.all(torch.where(m_t, res.target_col == b.token_ids, res.target_col == -1)).item())
        for t_ in (res.logprob, res.lse, res.coeff, res.entropy, res.target_logit):
            assert int((t_[~m_t] != 0).sum().item()) == 0
        # exactly the counting rows carry gradient - save a row whose coefficient is exactly zero, which happens: in a group
        # with equal rewards only the KL term is left, and that vanishes when the log-prob equals the reference bit for bit
        nz = res.d_hidden.abs().amax(1) > 0
        want_nz = m_t & (res.coeff != 0)
        if not bool(torch.equal(nz, want_nz)):
            extra = torch.nonzero(nz & ~want_nz).flatten(); missing = torch.nonzero(~nz & want_nz).flatten()
            _say("  ", tag, "rows with gradient that should have none:", extra.numel(), extra[:8].tolist(),
                 "rows without that should have:", missing.numel(), missing[:8].tolist())
            assert False, "set of rows carrying gradient differs from the counting rows with a non-zero coefficient"
        assert int((m_t & ~want_nz).sum().item()) <= 8
        del want_nz
        del nz
        # (b)
        e_lp = np.abs(f64(res.logprob[rows_t]) - lp_ref).max(); e_lse = np.abs(f64(res.lse[rows_t]) - lse_ref).max()
        e_ent = np.abs(f64(res.entropy[rows_t]) - ent_ref).max(); e_zy = np.abs(f64(res.target_logit[rows_t]) - zy_ref).max()
        _say("  ", tag, "sampled rows: logp", e_lp, "lse", e_lse, "entropy", e_ent, "target logit", e_zy)
        assert max(e_lp, e_lse, e_ent, e_zy) <= BF16_TOL["logp_atol"]
        np.testing.assert_allclose(f64(res.advantages), adv_ref, atol=2e-6, rtol=1e-6)
        # (c) conditional on the spot-checked log-probs
        lp_gpu = f64(res.logprob)
        if objective == "grpo":
            o = orc.grpo_loss(lp_gpu, old_np, refp_np, mask_np, cu_np, adv_ref, c.clip_eps, c.kl_coef)
            o["d_log_z"] = np.zeros(c.P)
        else:
            o = orc.flow_loss(lp_gpu, old_np, refp_np, mask_np, cu_np, adv_ref, gidx, np_bits(b.log_z), c.clip_eps, c.beta)
        scale = max(abs(o["loss"]), float(np.abs(o["seq_loss"]).mean()), 1e-30)
        e_loss = abs(float(res.loss.item()) - o["loss"]) / scale
        e_sl = np.abs(f64(res.seq_loss) - o["seq_loss"]).max() / max(np.abs(o["seq_loss"]).max(), 1e-30)
        e_c = np.abs(f64(res.coeff) - o["c"]).max() / np.abs(o["c"]).max()
        _say("  ", tag, "O(T) stages from GPU log-probs: loss", e_loss, "seq_loss", e_sl, "coeff", e_c)
        assert e_loss <= 1e-5 and e_sl <= 1e-5 and e_c <= 1e-4
        np.testing.assert_allclose(f64(res.d_log_z), o["d_log_z"], atol=1e-5 * max(1.0, float(np.abs(o["d_log_z"]).max())))
        assert abs(st["n_clip_hi"] - o["n_clip_hi"]) <= 1 and abs(st["n_clip_lo"] - o["n_clip_lo"]) <= 1
        # (d)
        dX_ref, _ = orc.lm_head_backward(Xs, W64, ids_s, ones, lse_ref, o["c"][rows], want_dw=False)
        e_dx = np.abs(f64(res.d_hidden[rows_t]) - dX_ref).max() / np.abs(dX_ref).max()
        _say("  ", tag, "sampled dX rows", e_dx)
        assert e_dx <= BF16_TOL["grad_tol"]
        # (f)
        assert abs(float(res.loss.item()) - f64(res.seq_loss).mean()) <= 1e-5 * max(np.abs(f64(res.seq_loss)).mean(), 1e-30)
        dW = res.d_weight
        assert dW.double().sum(0).abs().max().item() <= 1e-3 * dW.abs().max().item() * np.sqrt(V)
        ip_x = sum(float((res.d_hidden[s:s + 65536].double() * b.hidden[s:s + 65536].double()).sum().item()) for s in range(0, b.R, 65536))
        ip_w = sum(float((dW[s:s + 16384].double() * b.weight[s:s + 16384].double()).sum().item()) for s in range(0, V, 16384))
        slack = float(dW.double().abs().sum().item()) * 0.02 * 1e-3 + 1e-30
        assert abs(ip_x - ip_w) <= 2e-2 * max(abs(ip_x), abs(ip_w)) + slack, (ip_x, ip_w)
        # keep what (e) needs; free the big outputs before the next call
        runs[tag] = dict(lse=f64(res.lse), c=f64(res.coeff), dW_rows=f64(dW[vs_t]), acc=np.zeros((vs.size, H)))
        del res, dW
        torch.cuda.empty_cache()
    # (e) sampled rows of dW: the oracle adds up all T rows, block by block, from each run's lse and coefficients
    all_rows = np.flatnonzero(mask_np)
    blk = 32768
    for s0 in range(0, T, blk):
        rr = all_rows[s0:s0 + blk]
        Xb = _wide(b.hidden[torch.from_numpy(rr).cuda()])
        on = np.ones(rr.size, np.uint8)
        for r in runs.values():
            r["acc"] += orc.weight_grad_rows(Xb, Wv, vs, ids_np[rr], on, r["lse"][rr], r["c"][rr])
        if (s0 // blk) % 8 == 0:
            _say("   oracle: dW rows, block", s0 // blk, "of", -(-T // blk))
    for tag, r in runs.items():
        gw = np.abs(r["acc"]).max()
        per_row = np.abs(r["dW_rows"] - r["acc"]).max(1) / gw
        _say("  ", tag, "sampled dW rows", vs.tolist(), "max err / max|dW rows|", per_row.max(), "worst row", int(vs[per_row.argmax()]))
        assert per_row.max() <= BF16_TOL["grad_tol"]
