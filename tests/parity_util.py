"""Shared helpers of the GPU parity tests: move one seeded batch to both sides and compare.

The HIP path and the oracle read the same stored bits (bf16 tensors are handed to the oracle
as their 16-bit patterns, which it widens exactly)."""
from __future__ import annotations

import numpy as np
import torch

from oracle import policy_oracle as orc
from paper_2603_16435_amd import binding

OBJ = {"grpo": (orc.GRPO, binding.RL_OBJ_GRPO), "flow": (orc.FLOW, binding.RL_OBJ_FLOW)}


def np_bits(t: torch.Tensor) -> np.ndarray:
    t = t.detach().cpu().contiguous()
    if t.dtype == torch.bfloat16:
        return t.view(torch.int16).numpy()
    return t.numpy()


def oracle_inputs(b, rows=None):
    """numpy views of a RolloutBatch for the oracle (optionally only the given rows of the row tensors)."""
    sel = (lambda t: t) if rows is None else (lambda t: t[rows])
    return dict(hidden=np_bits(sel(b.hidden)), weight=np_bits(b.weight), token_ids=np_bits(sel(b.token_ids)),
                mask=np_bits(sel(b.mask)), old_logprob=np_bits(sel(b.old_logprob)),
                ref_logprob=np_bits(sel(b.ref_logprob)))


def run_oracle(b, objective: str, want_dw=True, **over):
    c = b.cfg
    kw = dict(clip_eps=c.clip_eps, kl_coef=c.kl_coef, beta=c.beta, adv_eps=c.adv_eps, adv_std_ddof=c.adv_std_ddof)
    kw.update(over)
    inp = oracle_inputs(b)
    return orc.policy_loss_fwd_bwd(OBJ[objective][0], cu_seqlens=np_bits(b.cu_seqlens), group_idx=np_bits(b.group_idx),
                                   rewards=np_bits(b.rewards), log_z=np_bits(b.log_z), P=c.P, want_dw=want_dw,
                                   want_entropy=True,
                                   **inp, **kw)


def run_gpu(b, objective: str, chunk_rows=0, backward=True, mode=None, **over):
    """mode: None (library default without a length promise = recompute), "recompute", or "stash" (the
    single-pass backward, with max_seq_len promised as the batch's longest sequence)."""
    c = b.cfg
    kw = dict(clip_eps=c.clip_eps, kl_coef=c.kl_coef, beta=c.beta, adv_eps=c.adv_eps, adv_std_ddof=c.adv_std_ddof)
    if mode == "stash":
        kw.update(backward_mode="stash", max_seq_len=max(int(b.lengths.max()), 1))
    elif mode == "recompute":
        kw.update(backward_mode="recompute")
    kw.update(over)
    res = binding.rl_policy_loss_fwd_bwd(OBJ[objective][1], b.hidden, b.weight, b.token_ids, b.mask, b.cu_seqlens,
                                         b.group_idx, b.rewards, b.old_logprob, b.ref_logprob, b.log_z, P=c.P,
                                         chunk_rows=chunk_rows, backward=backward, index_outputs=True, **kw)
    torch.cuda.synchronize()
    return res


def f64(t):
    return t.detach().to(torch.float64).cpu().numpy()


def loss_rel_err(gpu_loss: float, ref: dict) -> float:
    """|L_gpu - L_ref| / max(|L_ref|, mean_i |seq_loss_i|): the GRPO loss is ~0 by construction
    (zero-mean advantages), so the error is measured against the scale of its terms."""
    scale = max(abs(ref["loss"]), float(np.abs(ref["seq_loss"]).mean()), 1e-30)
    return abs(gpu_loss - ref["loss"]) / scale


def compare_all(b, res, ref, *, loss_tol, logp_atol, grad_tol, check_dw=True, temperature=1.0):
    """Element-by-element comparison of every output; returns a dict of the error figures."""
    m = np_bits(b.mask).astype(bool)
    err = {}
    # integer / index work: exact
    np.testing.assert_array_equal(res.seq_len.cpu().numpy(), ref["seq_len"])
    st = res.stats_dict()
    assert st["n_tokens"] == int(ref["seq_len"].sum())
    assert st["n_bad_token"] == 0 and st["n_bad_group"] == 0 and st["n_bad_seq"] == 0 and st["n_overflow_rows"] == 0
    check_index_work(b, res, temperature=temperature)
    lp = f64(res.logprob); lse = f64(res.lse); coeff = f64(res.coeff)
    assert np.all(lp[~m] == 0) and np.all(lse[~m] == 0) and np.all(coeff[~m] == 0)
    # floats
    err["logp"] = float(np.abs(lp - ref["logprob"]).max())
    err["lse"] = float(np.abs(lse - ref["lse"]).max())
    assert err["logp"] <= logp_atol and err["lse"] <= logp_atol, err
    if "entropy" in ref:
        ent = f64(res.entropy)
        assert np.all(ent[~m] == 0)
        err["entropy"] = float(np.abs(ent - ref["entropy"]).max())
        assert err["entropy"] <= logp_atol, err
    np.testing.assert_allclose(f64(res.advantages), ref["advantages"], atol=2e-6, rtol=1e-6)
    err["loss"] = loss_rel_err(float(res.loss.item()), ref)
    sl_scale = max(float(np.abs(ref["seq_loss"]).max()), 1e-30)
    err["seq_loss"] = float(np.abs(f64(res.seq_loss) - ref["seq_loss"]).max()) / sl_scale
    # The stated relative tolerance.  One exception: logp is computed and returned in f32, so the loss carries at least the
    # first-order effect of a 1e-6 error in logp, sum_t |c_t| 1e-6.  Where the loss is so small against its own sensitivity
    # that the relative bound is tighter than that (a lone KL term ~ d^2/2, say), the bound is ill-conditioned and that
    # effect is allowed on top; everywhere else the plain relative bound must hold.
    c_sum = float(np.abs(ref["c"]).sum())
    scale = max(abs(ref["loss"]), float(np.abs(ref["seq_loss"]).mean()), 1e-30)
    slack = c_sum * 1e-6 if loss_tol * scale < c_sum * 1e-6 else 0.0
    err["loss_slack_used"] = slack > 0.0
    if slack > 0.0:
        print("    (ill-conditioned loss: tol x scale = %.3e < 1e-6 x sum|c| = %.3e; the rounding of logp is allowed on top)" % (loss_tol * scale, 1e-6 * c_sum), flush=True)
    assert abs(float(res.loss.item()) - ref["loss"]) <= loss_tol * scale + slack, err
    assert float(np.abs(f64(res.seq_loss) - ref["seq_loss"]).max()) <= loss_tol * sl_scale + slack * len(ref["seq_loss"]), err
    c_scale = max(float(np.abs(ref["c"]).max()), 1e-30)
    err["coeff"] = float(np.abs(coeff - ref["c"]).max()) / c_scale
    assert err["coeff"] <= max(loss_tol, 1e-4), err
    np.testing.assert_allclose(f64(res.d_log_z), ref["d_log_z"], atol=loss_tol * max(1.0, float(np.abs(ref["d_log_z"]).max())))
    if res.d_hidden is not None:
        dX = f64(res.d_hidden)
        assert np.all(dX[~m] == 0)                      # masked rows: exactly zero
        nz_rows = np.abs(ref["d_hidden"]).max(1) > 0
        assert np.all(np.abs(dX).max(1)[nz_rows] > 0)   # same set of rows carries gradient
        gx = max(float(np.abs(ref["d_hidden"]).max()), 1e-30)
        err["dX"] = float(np.abs(dX - ref["d_hidden"]).max()) / gx
        assert err["dX"] <= grad_tol, err
        if check_dw:
            gw = max(float(np.abs(ref["d_weight"]).max()), 1e-30)
            err["dW"] = float(np.abs(f64(res.d_weight) - ref["d_weight"]).max()) / gw
            assert err["dW"] <= grad_tol, err
    return err


def check_index_work(b, res, clean=None, temperature=1.0):
    """Masks, group indexing and gathers, bit for bit: the order of the counting rows, the group sizes and the
    vocabulary entry each target logit was read from; the target logit itself against the one dot product it is."""
    if res.row_map is None:
        return
    cr = clean if clean is not None else orc.compact_rows(np_bits(b.mask), np_bits(b.token_ids), np_bits(b.cu_seqlens), b.cfg.V,
                                                          np_bits(b.group_idx), b.cfg.P)
    T = cr["row_map"].size
    rm = res.row_map.cpu().numpy()
    np.testing.assert_array_equal(rm[:T], cr["row_map"])
    assert np.all(rm[T:] == -1)
    np.testing.assert_array_equal(res.seq_len.cpu().numpy(), cr["seq_len"])
    np.testing.assert_array_equal(res.group_count.cpu().numpy(), orc.group_count(np_bits(b.group_idx), b.cfg.P))
    counts = np.zeros(b.R, dtype=bool); counts[cr["row_map"]] = True
    col = res.target_col.cpu().numpy()
    ids = np_bits(b.token_ids)
    np.testing.assert_array_equal(col[counts], ids[counts])
    assert np.all(col[~counts] == -1)
    zy = f64(res.target_logit)
    assert np.all(zy[~counts] == 0)
    if b.R * b.cfg.H <= (1 << 24):          # the dot products themselves, where the instance is small enough
        inp = oracle_inputs(b)
        ref = orc.target_logit(inp["hidden"], inp["weight"], np.clip(ids, 0, b.cfg.V - 1), counts.astype(np.uint8), temperature=temperature)
        tol = 2e-5 if b.hidden.dtype == torch.float32 else 2e-3
        assert np.abs(zy - ref).max() <= tol * max(1.0, np.abs(ref).max())


def cleaned_packed(b):
    """The batch as the path must read it when offsets, prompt indices or token ids are broken: only the rows that
    count (oracle's compact_rows), packed, every row unmasked, with the sequence lengths that remain.  Returns
    (oracle keyword inputs, compact_rows result)."""
    cr = orc.compact_rows(np_bits(b.mask), np_bits(b.token_ids), np_bits(b.cu_seqlens), b.cfg.V, np_bits(b.group_idx), b.cfg.P)
    rows = torch.from_numpy(cr["row_map"]).to(b.hidden.device)
    inp = oracle_inputs(b, rows)
    inp["mask"] = np.ones(rows.numel(), np.uint8)
    cu = np.concatenate([[0], np.cumsum(cr["seq_len"])])
    inp.update(cu_seqlens=cu, group_idx=np_bits(b.group_idx), rewards=np_bits(b.rewards), log_z=np_bits(b.log_z), P=b.cfg.P)
    return inp, cr
