"""Pins of the residual-VQ encode oracle: the ratios the paper prints, brute force, a library nearest-neighbour
routine, exact recovery on a constructed hierarchy, tie rule, monotone error, residual bookkeeping."""
import os

import numpy as np
import pytest
import torch
from scipy.cluster.vq import vq as scipy_vq

from oracle import rvq_oracle as rvq

GOLD = os.path.join(os.path.dirname(__file__), "golden", "vqkv_compression_ratio.txt")


def _bf16_bits(a):
    return torch.from_numpy(np.asarray(a, dtype=np.float32)).to(torch.bfloat16).view(torch.int16).numpy().view(np.uint16)


def _val(bits):
    return rvq.widen(np.asarray(bits).view(np.int16))


def test_compression_ratio_matches_the_values_the_paper_prints():
    for line in open(GOLD):
        if line.startswith("#") or not line.strip():
            continue
        name, nk, nv, sk, sv, d, want = line.split()
        got = rvq.compression_ratio(int(nk), int(sk), int(nv), int(sv), int(d), int(d))
        # printed to one decimal; the table rounds the exact tie 81.25 up to 81.3, so compare within half a unit of that decimal
        assert abs(got - float(want)) <= 0.05 + 1e-9, (name, got)
    assert rvq.compression_ratio(16, 2 ** 16, 16, 2 ** 16, 16, 16) == 0.0          # 16 codes of 16 bits for 16 values: nothing saved


def test_bf16_rounding_is_round_to_nearest_even():
    x = np.array([1.0, 1.0 + 2 ** -8, 1.0 + 3 * 2 ** -8, 1.0 + 2 ** -7, -(1.0 + 2 ** -8), 3.0e-5, 65280.0 + 128.0])
    want = torch.from_numpy(x.astype(np.float32)).to(torch.bfloat16).view(torch.int16).numpy().view(np.uint16)
    np.testing.assert_array_equal(rvq.bf16_round_bits(x), want)
    assert _val(rvq.bf16_round_bits([1.0 + 2 ** -8]))[0] == 1.0 and _val(rvq.bf16_round_bits([1.0 + 3 * 2 ** -8]))[0] == 1.0 + 2 ** -6


def test_brute_force_on_tiny_inputs():
    rng = np.random.default_rng(2)
    L, N, S, D = 7, 3, 5, 4
    xb = _bf16_bits(rng.normal(size=(L, D)))
    cb = _bf16_bits(rng.normal(size=(N, S, D)) * np.array([1.0, 0.5, 0.25])[:, None, None])
    codes, rbits = rvq.rvq_encode(xb, cb)
    C = _val(cb)
    for l in range(L):
        r = [float(v) for v in _val(xb[l])]
        for i in range(N):
            best, bd = -1, None
            for s in range(S):
                dist = 0.0
                for k in range(D):
                    dist += (r[k] - float(C[i, s, k])) ** 2
                if bd is None or dist < bd:
                    best, bd = s, dist
            assert codes[l, i] == best
            r = [float(v) for v in _val(rvq.bf16_round_bits(np.array(r) - C[i, best]))]
        np.testing.assert_array_equal(_val(rbits[l]), np.array(r))


def test_single_stage_equals_a_library_nearest_neighbour_search():
    rng = np.random.default_rng(3)
    xb = _bf16_bits(rng.normal(size=(200, 16)))
    cb = _bf16_bits(rng.normal(size=(1, 64, 16)))
    codes, _ = rvq.rvq_encode(xb, cb)
    want, _ = scipy_vq(_val(xb), _val(cb)[0])
    np.testing.assert_array_equal(codes[:, 0], want)


def test_exact_recovery_on_a_scale_hierarchy():
    # stage i holds small-integer entries scaled by 16^-i: every partial sum is exactly representable in bf16's 8 bits
    # only if few bits are used, so use entries in {-1,0,1}^D at stage scales 1, 1/4, 1/16 (3 stages: 6 bits span)
    rng = np.random.default_rng(4)
    N, S, D, L = 3, 27, 3, 50
    base = np.array([[a, b, c] for a in (-1, 0, 1) for b in (-1, 0, 1) for c in (-1, 0, 1)], dtype=np.float64)
    cb = np.stack([base[rng.permutation(S)] * 4.0 ** -i for i in range(N)])
    picks = rng.integers(0, S, size=(L, N))
    x = sum(cb[i, picks[:, i]] for i in range(N))
    codes, rbits = rvq.rvq_encode(_bf16_bits(x), _bf16_bits(cb))
    np.testing.assert_array_equal(codes, picks)                      # greedy search recovers every stage
    assert np.all(_val(rbits) == 0)
    np.testing.assert_array_equal(rvq.rvq_decode(codes, _bf16_bits(cb)), x)


def test_ties_go_to_the_lowest_index_and_zero_entry_never_increases_the_error():
    rng = np.random.default_rng(5)
    D, S = 8, 16
    cb = rng.normal(size=(4, S, D)) * np.array([1.0, 0.6, 0.4, 0.3])[:, None, None]
    cb[:, 5] = cb[:, 11]                                             # duplicated entries: 5 must win over 11
    cb[:, 0] = 0.0                                                   # every stage can choose "no change"
    xb = _bf16_bits(rng.normal(size=(300, D)))
    codes, rbits, trace = rvq.rvq_encode(xb, _bf16_bits(cb), return_trace=True)
    assert not np.any(codes == 11) and np.any(codes == 5)
    assert np.all(np.diff(trace, axis=1) <= 1e-12)                   # squared residual norm never grows
    # the residual is what is left after subtracting the chosen entries, up to the bf16 rounding of each stage
    recon = rvq.rvq_decode(codes, _bf16_bits(cb))
    err = np.abs(_val(xb) - recon - _val(rbits)).max()
    assert err <= 4 * 2.0 ** -8 * np.abs(_val(xb)).max()


def test_checker_accepts_the_oracle_and_rejects_a_wrong_code():
    rng = np.random.default_rng(6)
    xb = _bf16_bits(rng.normal(size=(40, 8)))
    cb = _bf16_bits(rng.normal(size=(3, 16, 8)) * np.array([1.0, 0.5, 0.25])[:, None, None])
    codes, _ = rvq.rvq_encode(xb, cb)
    n_diff, worst = rvq.check_codes_follow_the_definition(xb, cb, codes, 1e-6)
    assert n_diff == 0 and worst == 0.0
    bad = codes.copy(); bad[3, 1] = (bad[3, 1] + 1) % 16
    with pytest.raises(AssertionError):
        rvq.check_codes_follow_the_definition(xb, cb, bad, 1e-6)
