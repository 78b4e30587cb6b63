"""The scoring call that allocates nothing (rl_token_logprob_static: workspace in a static device array of the
library) against the existing entry point that takes a caller's workspace, through the C ABI.  Two calls in a row,
the second with a smaller input: the array keeps the first call's contents, which the second must not see."""
import numpy as np
import pytest
import torch

from paper_2603_16435_amd import binding, synth

pytestmark = pytest.mark.gpu


def _case(P, G, lo, hi, H, V, dtype, seed, layout):
    cfg = synth.RolloutConfig("static", P, G, lo, hi, H, V, dtype, 0.5, seed=seed)
    return synth.make_rollouts(cfg, "cuda", layout)


def _both(b, temperature=1.0):
    logp = torch.full((b.R,), 7.0, dtype=torch.float32, device="cuda")
    lse = torch.full((b.R,), 7.0, dtype=torch.float32, device="cuda")
    binding.rl_token_logprob_static(b.hidden, b.weight, b.token_ids, b.mask, b.cu_seqlens, logp, lse, temperature)
    torch.cuda.synchronize()
    if temperature == 1.0:
        ref_lp, ref_lse = binding.rl_token_logprob(b.hidden, b.weight, b.token_ids, b.mask, b.cu_seqlens)
    else:
        ref_lp, ref_lse = binding.rl_token_logprob_tempered(b.hidden, b.weight, b.token_ids, b.mask, temperature, b.cu_seqlens)
    torch.cuda.synchronize()
    return logp, lse, ref_lp, ref_lse


def test_static_scratch_scoring_call_matches_the_workspace_call():
    # first call: 40 k rows x 32000 vocabulary entries; the plan only fits the array with 8192-row chunks, while the
    # workspace call uses one 32768-row chunk and a ragged second one: the results must still agree bit for bit
    big = _case(8, 8, 400, 900, 256, 32000, "bf16", 901, "padded")
    print("first call: R", big.R, "T", big.T, flush=True)
    logp, lse, ref_lp, ref_lse = _both(big)
    assert torch.equal(logp, ref_lp) and torch.equal(lse, ref_lse)
    m = big.mask.bool()
    assert int((logp[~m] != 0).sum().item()) == 0 and bool(torch.all(logp[m] < 0).item())
    # second call, smaller input (f32, ragged vocabulary, packed rows): nothing of the first call may leak in
    small = _case(2, 3, 5, 40, 72, 1000, "f32", 902, "packed")
    print("second call: R", small.R, "T", small.T, flush=True)
    logp, lse, ref_lp, ref_lse = _both(small, temperature=0.8)
    assert torch.equal(logp, ref_lp) and torch.equal(lse, ref_lse)
    # and the first input again: same bits as before
    logp2, lse2, ref_lp2, ref_lse2 = _both(big)
    assert torch.equal(logp2, ref_lp2) and torch.equal(lse2, ref_lse2)


def test_static_scratch_call_refuses_batches_beyond_the_array():
    b = _case(2, 2, 5, 9, 64, 512, "bf16", 903, "packed")
    fake_rows = 4 << 20                                            # 32 bytes a row: far beyond 32 MiB
    bb = binding.make_batch(b.hidden, b.weight, b.token_ids, b.mask, b.cu_seqlens)
    bb.R = fake_rows
    out = torch.zeros(8, dtype=torch.float32, device="cuda")
    import ctypes as C
    st = binding.lib().rl_token_logprob_static(C.byref(bb), 1.0, out.data_ptr(), out.data_ptr(), None)
    assert st == 5                                                 # RL_ERR_WORKSPACE, before anything is launched
    torch.cuda.synchronize()
    assert float(out.abs().sum().item()) == 0.0
