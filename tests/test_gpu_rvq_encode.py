"""GPU parity of the residual-VQ encode against its float64 oracle, through the C ABI.

Codes are integers, so the bar is exact equality: every code and every residual bit equals the float64 oracle's (no
decision differs).  The kernel scores in float32 on the matrix cores and settles every decision whose lead is inside
the rounding margin from the stored bf16 values in float64, so this holds on any input, near-ties included (there is a
test of entry pairs that float32 cannot tell apart).  Independently of the exact comparison, the oracle also walks the
kernel's own path decision by decision: each chosen entry must be a nearest entry to within 2e-6 of the distance scale,
and the residual must follow from the kernel's own codes bit for bit."""
import numpy as np
import pytest
import torch

from oracle import rvq_oracle as rvq
from paper_2603_16435_amd import binding, synth

pytestmark = pytest.mark.gpu


def _bits(t):
    return t.detach().cpu().contiguous().view(torch.int16).numpy().view(np.uint16)


def _compare(x, cb, codes, res):
    G = x.shape[0]
    n_rows = n_same = n_diff_dec = 0
    for g in range(G):
        xb, cbb = _bits(x[g]), _bits(cb[g])
        want_codes, want_res = rvq.rvq_encode(xb, cbb)
        got = codes[g].cpu().numpy().astype(np.int64)
        same = np.all(got == want_codes, axis=1)
        n_rows += same.size; n_same += int(same.sum())
        # rows on which both agree: the residual must agree bit for bit
        np.testing.assert_array_equal(_bits(res[g])[same], want_res[same])
        # every decision of the kernel is a nearest entry up to float32 rounding; residual consistent with its own codes
        nd, worst = rvq.check_codes_follow_the_definition(xb, cbb, got, 2e-6)
        n_diff_dec += nd
        r = rvq.widen(xb.view(np.int16))
        C = rvq.widen(cbb.view(np.int16))
        rb = xb.copy()
        for i in range(C.shape[0]):
            rb = rvq.bf16_round_bits(rvq.widen(rb.view(np.int16)) - C[i, got[:, i]])
        np.testing.assert_array_equal(_bits(res[g]), rb)
    # pinned on these seeds: every row equal, no decision other than the float64 argmin
    assert n_same == n_rows and n_diff_dec == 0, (n_same, n_rows, n_diff_dec)
    return n_same, n_rows, n_diff_dec


@pytest.mark.parametrize("G,L,N,S", [(2, 300, 6, 128),      # ragged tail (L % 256 != 0), two groups
                                      (1, 1, 3, 64),         # a single vector, a single chunk per stage
                                      (3, 513, 16, 512),     # the value-cache shape of the paper's 8B setting (N=16, S=512)
                                      (9, 256, 4, 192),      # a full workgroup of four wavefronts; 9 groups (the grid covers 16); S not a power of two
                                      (1, 257, 2, 64),       # one vector beyond 256: eight wavefronts, more wavefronts than 16-entry blocks
                                      (1, 130, 2, 4096)])    # a large codebook: 256 blocks per stage, 8-bit block numbers in the block maxima
def test_rvq_encode_matches_the_oracle(G, L, N, S):
    x, cb = synth.make_rvq_case(G, L, N, S, device="cuda")
    codes, res = binding.rl_rvq_encode(x, cb)
    torch.cuda.synchronize()
    assert int(codes.min()) >= 0 and int(codes.max()) < S
    print(_compare(x, cb, codes, res))


def test_rvq_encode_key_cache_shape_sampled():
    # the key-cache shape of the paper's 8B setting, N = 56 stages of S = 1024 entries, L = 1024 vectors (one local window):
    # the oracle checks a seeded sample of 96 vectors in full (rows are independent)
    x, cb = synth.make_rvq_case(2, 1024, 56, 1024, device="cuda")
    codes, res = binding.rl_rvq_encode(x, cb)
    torch.cuda.synchronize()
    pick = torch.from_numpy(np.random.default_rng(1).choice(1024, 96, replace=False)).cuda()
    for g in range(2):
        n_same, n_rows, nd = _compare(x[g:g + 1, pick], cb[g:g + 1], codes[g:g + 1, pick], res[g:g + 1, pick])
        print("group", g, "rows equal", n_same, "of", n_rows, "decisions differing from the float64 argmin", nd)
    # properties at full size: the residual norm shrinks (random codebooks at matched scale), codes in range
    r0 = x.float().pow(2).sum(-1).mean().item(); r1 = res.float().pow(2).sum(-1).mean().item()
    assert r1 < 0.05 * r0
    assert int(codes.min()) >= 0 and int(codes.max()) < 1024


def test_rvq_encode_ties_and_exact_recovery():
    # duplicated entries: the lower index wins; hierarchy of exactly representable entries: codes recovered, residual zero
    D, S, N, L = 128, 64, 3, 200
    g = torch.Generator().manual_seed(3)
    base = torch.randint(-1, 2, (N, S, D), generator=g).float()
    base[:, 0] = 0.0
    base[:, 40] = base[:, 7]                                   # duplicate of entry 7
    cb = (base * (4.0 ** -torch.arange(N).float()).view(N, 1, 1)).to(torch.bfloat16).unsqueeze(0)
    picks = torch.randint(0, S, (L, N), generator=g)
    picks[picks == 40] = 7
    xx = sum(cb[0, i, picks[:, i]].float() for i in range(N)).to(torch.bfloat16).unsqueeze(0)
    codes, res = binding.rl_rvq_encode(xx.cuda(), cb.cuda())
    torch.cuda.synchronize()
    want, want_res = rvq.rvq_encode(_bits(xx[0]), _bits(cb[0]))
    np.testing.assert_array_equal(codes[0].cpu().numpy(), want)
    assert not bool((codes == 40).any())
    assert float(res.float().abs().max()) == 0.0


def test_rvq_encode_near_ties_are_decided_exactly():
    """Entries in near-duplicate pairs: entry 2s+1 equals entry 2s except for 2^-20 in a component where 2s holds zero.
    The two scores differ by about 1e-6 of their size - below what float32 accumulation resolves, so which one wins
    depends on exact arithmetic.  Every decision must still equal the float64 oracle's, and the counter of decisions
    re-evaluated exactly must show that this path did the work."""
    G, L, N, S, D = 1, 300, 4, 128, 128
    x, cb = synth.make_rvq_case(G, L, N, S, D, seed=0x5EED0200, device="cuda")
    cb = cb.clone()
    sign = torch.where(torch.arange(S // 2, device="cuda") % 2 == 0, 1.0, -1.0).to(torch.bfloat16)
    cb[:, :, 0::2, 0] = 0
    cb[:, :, 1::2, :] = cb[:, :, 0::2, :]
    cb[:, :, 1::2, 0] = (sign * 2.0 ** -20).view(1, 1, -1)
    n_exact = torch.zeros(1, dtype=torch.int32, device="cuda")
    codes, res = binding.rl_rvq_encode(x, cb, count_exact=n_exact)
    torch.cuda.synchronize()
    want, want_res = rvq.rvq_encode(_bits(x[0]), _bits(cb[0]))
    got = codes[0].cpu().numpy()
    assert (got % 2 == 1).any() and (got % 2 == 0).any()            # both members of pairs win somewhere
    np.testing.assert_array_equal(got, want)
    np.testing.assert_array_equal(_bits(res[0]), want_res)
    n = int(n_exact.item())
    print("decisions re-evaluated exactly:", n, "of", L * N)
    assert n >= L * N


def test_rvq_encode_exact_path_is_rare_on_ordinary_inputs():
    G, L, N, S = 2, 1024, 16, 1024
    x, cb = synth.make_rvq_case(G, L, N, S, device="cuda")
    n_exact = torch.zeros(1, dtype=torch.int32, device="cuda")
    binding.rl_rvq_encode(x, cb, count_exact=n_exact)
    torch.cuda.synchronize()
    n = int(n_exact.item())
    print("decisions re-evaluated exactly:", n, "of", G * L * N)
    assert n <= 0.01 * G * L * N
