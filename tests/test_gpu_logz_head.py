"""GPU parity of the log-Z head against its float64 oracle, through the C ABI, and the head feeding the
flow-balance objective end to end (log_z in, d_log_z back)."""
import numpy as np
import pytest
import torch

from oracle import logz_head_oracle as lzo
from paper_2603_16435_amd import binding
from parity_util import np_bits, run_gpu, run_oracle
from paper_2603_16435_amd import synth

pytestmark = pytest.mark.gpu


def _head(seed, P, H, M, lens, dtype):
    g = torch.Generator().manual_seed(seed)
    cu = torch.tensor(np.concatenate([[0], np.cumsum(lens)]), dtype=torch.int32)
    X = torch.randn(int(cu[-1]), H, generator=g).to(dtype)
    W1 = torch.randn(M, H, generator=g) * (1.0 / np.sqrt(H))
    b1 = torch.randn(M, generator=g) * 0.1
    w2 = torch.randn(M, generator=g) * (1.0 / np.sqrt(M))
    b2 = torch.tensor([0.25])
    d = torch.randn(P, generator=g)
    return X, cu, W1, b1, w2, b2, d


@pytest.mark.parametrize("dtype,P,H,M,lens", [
    (torch.float32, 5, 37, 50, (4, 1, 0, 7, 3)),                        # ragged everything (odd H, M % 16 != 0), an empty prompt
    (torch.bfloat16, 16, 3584, 3584, tuple(range(100, 900, 50))),       # the 7B-shaped head: 16 prompts, H = M = 3584
    (torch.bfloat16, 300, 256, 520, tuple(3 + (i % 11) for i in range(300))),   # many prompts (several groups of 16), ragged M
])
def test_logz_head_matches_the_oracle(dtype, P, H, M, lens):
    X, cu, W1, b1, w2, b2, d = _head(11, P, H, M, lens, dtype)
    dev = "cuda"
    log_z, ws = binding.rl_logz_head_forward(X.to(dev), cu.to(dev), W1.to(dev), b1.to(dev), w2.to(dev), b2.to(dev))
    dW1, db1, dw2, db2 = binding.rl_logz_head_backward(d.to(dev), w2.to(dev), H, ws)
    torch.cuda.synchronize()
    f = lzo.logz_head_forward(np_bits(X), cu.numpy(), W1.numpy(), b1.numpy(), w2.numpy(), float(b2))
    g = lzo.logz_head_backward(f, W1.numpy(), w2.numpy(), d.numpy())
    # f32 arithmetic with f32 accumulation over H (pooling over <= 850 rows, dot products over H, M <= 3584 terms)
    assert np.abs(log_z.double().cpu().numpy() - f["log_z"]).max() <= 2e-5 * max(1.0, np.abs(f["log_z"]).max())
    for got, want in ((dW1, g["dW1"]), (db1, g["db1"]), (dw2, g["dw2"])):
        assert np.abs(got.double().cpu().numpy() - want).max() <= 2e-5 * np.abs(want).max()
    assert abs(float(db2.item()) - g["db2"]) <= 1e-5 * max(1.0, abs(g["db2"]))
    if 0 in lens:                                                    # the empty prompt sees only the biases
        p = lens.index(0)
        assert abs(float(log_z[p].item()) - (float(lzo.gelu(b1.double().numpy()) @ w2.double().numpy()) + 0.25)) <= 1e-5


def test_head_feeds_the_flow_objective_end_to_end():
    # log Z from the head goes into the flow-balance loss, d_log_z comes back and drives the head's backward:
    # the chain equals the oracle's chain (head oracle -> policy oracle -> head oracle backward)
    b = synth.make_rollouts("small", "cuda", "padded", len_div=16)
    c = b.cfg
    X, cu, W1, b1, w2, b2, _ = _head(5, c.P, 256, 192, tuple(20 + 3 * i for i in range(c.P)), torch.bfloat16)
    dev = "cuda"
    log_z, ws = binding.rl_logz_head_forward(X.to(dev), cu.to(dev), W1.to(dev), b1.to(dev), w2.to(dev), b2.to(dev))
    b.log_z = log_z
    res = run_gpu(b, "flow", chunk_rows=1024, mode="stash")
    dW1, db1, dw2, db2 = binding.rl_logz_head_backward(res.d_log_z, w2.to(dev), 256, ws)
    torch.cuda.synchronize()
    f = lzo.logz_head_forward(np_bits(X), cu.numpy(), W1.numpy(), b1.numpy(), w2.numpy(), float(b2))
    b.log_z = torch.from_numpy(f["log_z"].astype(np.float32)).cuda()          # the oracle chain uses its own log Z
    ref = run_oracle(b, "flow", want_dw=False)
    g = lzo.logz_head_backward(f, W1.numpy(), w2.numpy(), ref["d_log_z"])
    assert abs(float(res.loss.item()) - ref["loss"]) <= 1e-2 * abs(ref["loss"])
    assert np.abs(res.d_log_z.double().cpu().numpy() - ref["d_log_z"]).max() <= 1e-3 * np.abs(ref["d_log_z"]).max()
    for got, want in ((dW1, g["dW1"]), (db1, g["db1"]), (dw2, g["dw2"])):
        assert np.abs(got.double().cpu().numpy() - want).max() <= 2e-3 * np.abs(want).max()
