"""The C-ABI library: loads, exports every symbol the header declares, and rejects bad host
arguments before anything is launched (no GPU needed: none of these calls reaches a kernel)."""
import ctypes as C
import os
import re

import pytest

from paper_2603_16435_amd import binding

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def _declared_functions():
    names = []
    inc = os.path.join(ROOT, "include")
    for fn in sorted(os.listdir(inc)):
        if not fn.endswith(".h"):
            continue
        text = open(os.path.join(inc, fn)).read()
        text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
        names += re.findall(r"\b(rl_[a-z_0-9]+)\s*\(", text)
    return sorted(set(names))


@pytest.fixture(scope="module")
def lib():
    if not os.path.exists(binding.LIB_PATH):
        from paper_2603_16435_amd import build
        build.build(verbose=False)
    return binding.lib()


def test_every_declared_symbol_is_exported(lib):
    names = _declared_functions()
    assert {"rl_workspace_bytes", "rl_token_logprob", "rl_policy_loss_fwd_bwd", "rl_status_string"} <= set(names)
    for n in names:
        assert hasattr(lib, n), n
    assert lib.rl_version() >= 100
    assert lib.rl_default_chunk_rows() % 256 == 0 and lib.rl_default_chunk_rows_single_pass() % 256 == 0


def _batch(**over):
    b = binding.rl_batch()
    b.R, b.H, b.V, b.B, b.P, b.dtype = 1000, 64, 512, 4, 2, binding.RL_BF16
    for k, v in over.items():
        setattr(b, k, v)
    return b


def test_workspace_query_and_shape_errors(lib):
    n = C.c_size_t(0)
    assert lib.rl_workspace_bytes(C.byref(_batch()), None, 1, C.byref(n)) == 0
    fwd = C.c_size_t(0)
    assert lib.rl_workspace_bytes(C.byref(_batch()), None, 0, C.byref(fwd)) == 0
    assert 0 < fwd.value < n.value and n.value % 256 == 0
    # chunk_rows grows the staged dS buffers
    small, big = C.c_size_t(0), C.c_size_t(0)
    b = _batch(R=100000)
    lib.rl_workspace_bytes(C.byref(b), C.byref(binding.make_params(chunk_rows=256)), 1, C.byref(small))
    lib.rl_workspace_bytes(C.byref(b), C.byref(binding.make_params(chunk_rows=4096)), 1, C.byref(big))
    assert small.value < big.value
    for bad in (dict(R=0), dict(H=0), dict(V=0), dict(B=0), dict(P=0), dict(H=60), dict(R=1 << 31)):
        assert lib.rl_workspace_bytes(C.byref(_batch(**bad)), None, 1, C.byref(n)) == 2, bad
    assert lib.rl_workspace_bytes(C.byref(_batch(dtype=7)), None, 1, C.byref(n)) == 3
    assert lib.rl_workspace_bytes(None, None, 1, C.byref(n)) == 1
    assert lib.rl_workspace_bytes(C.byref(_batch()), None, 1, None) == 1
    assert lib.rl_workspace_bytes(C.byref(_batch(dtype=binding.RL_F32, H=60)), None, 1, C.byref(n)) == 0


def test_backward_mode_is_validated_on_the_host(lib):
    n, m = C.c_size_t(0), C.c_size_t(0)
    ok = _batch(R=100000, H=128)
    mk = binding.make_params
    # the single-pass backward needs bf16, H % 128 == 0 and a length promise that fits a chunk
    assert lib.rl_workspace_bytes(C.byref(ok), C.byref(mk(backward_mode="stash", max_seq_len=512)), 1, C.byref(n)) == 0
    assert lib.rl_workspace_bytes(C.byref(ok), C.byref(mk(backward_mode="recompute", max_seq_len=512)), 1, C.byref(m)) == 0
    assert n.value > m.value                                                     # chunk records, references, factors
    assert lib.rl_workspace_bytes(C.byref(ok), C.byref(mk(backward_mode="auto", max_seq_len=512)), 1, C.byref(m)) == 0
    assert m.value == n.value                                                    # auto picks it when it can
    assert lib.rl_workspace_bytes(C.byref(ok), C.byref(mk(backward_mode="stash")), 1, C.byref(n)) == 4            # no promise
    assert lib.rl_workspace_bytes(C.byref(ok), C.byref(mk(backward_mode="stash", max_seq_len=512, chunk_rows=256)), 1, C.byref(n)) == 4
    # ... and where no kernel exists for the shape or dtype, the request is valid but unimplemented
    assert lib.rl_workspace_bytes(C.byref(_batch(H=64)), C.byref(mk(backward_mode="stash", max_seq_len=8)), 1, C.byref(n)) == 7
    assert lib.rl_workspace_bytes(C.byref(_batch(H=128, dtype=binding.RL_F32)), C.byref(mk(backward_mode="stash", max_seq_len=8)), 1, C.byref(n)) == 7
    assert b"no kernel" in lib.rl_status_string(7)
    assert lib.rl_workspace_bytes(C.byref(_batch(H=64)), C.byref(mk(backward_mode="auto", max_seq_len=8)), 1, C.byref(n)) == 0   # falls back
    assert lib.rl_workspace_bytes(C.byref(ok), C.byref(mk(backward_mode=7)), 1, C.byref(n)) == 4
    assert lib.rl_workspace_bytes(C.byref(ok), C.byref(mk(max_seq_len=-1)), 1, C.byref(n)) == 4


def test_null_and_range_errors_are_rejected_on_the_host(lib):
    b = _batch()
    prm = binding.make_params()
    out = binding.rl_outputs()
    # required pointers missing
    assert lib.rl_policy_loss_fwd_bwd(C.byref(b), C.byref(prm), 0, C.byref(out), None, 0, None) == 1
    assert lib.rl_token_logprob(C.byref(b), None, None, None, 0, None) == 1
    # fake non-null pointers: validation still stops before any launch
    fake = 0x1000
    for f in ("hidden", "weight", "token_ids", "mask", "cu_seqlens", "group_idx", "rewards", "old_logprob", "ref_logprob"):
        setattr(b, f, fake)
    out.loss = fake
    assert lib.rl_policy_loss_fwd_bwd(C.byref(b), C.byref(prm), 5, C.byref(out), None, 0, None) == 4      # objective
    assert lib.rl_policy_loss_fwd_bwd(C.byref(b), C.byref(prm), 1, C.byref(out), None, 0, None) == 1      # FLOW needs log_z
    assert lib.rl_policy_loss_fwd_bwd(C.byref(b), C.byref(binding.make_params(clip_eps=1.5)), 0, C.byref(out), None, 0, None) == 4
    assert lib.rl_policy_loss_fwd_bwd(C.byref(b), C.byref(binding.make_params(adv_std_ddof=2)), 0, C.byref(out), None, 0, None) == 4
    for bad in (dict(clip_eps_high=-0.1), dict(aggregation=2), dict(ratio_level=3), dict(flow_weight_norm=-1),
                dict(ratio_level="sequence", aggregation="token"), dict(temperature=-1.0), dict(temperature=float("inf")),
                dict(temperature=float("nan"))):
        assert lib.rl_policy_loss_fwd_bwd(C.byref(b), C.byref(binding.make_params(**bad)), 0, C.byref(out), None, 0, None) == 4, bad
    out.d_hidden = fake                                                                                   # d_weight missing
    assert lib.rl_policy_loss_fwd_bwd(C.byref(b), C.byref(prm), 0, C.byref(out), None, 0, None) == 1
    out.d_weight = fake
    assert lib.rl_policy_loss_fwd_bwd(C.byref(b), C.byref(prm), 0, C.byref(out), None, 0, None) == 5      # no workspace
    assert lib.rl_policy_loss_fwd_bwd(C.byref(b), C.byref(prm), 0, C.byref(out), 0x1001, 1 << 40, None) == 5  # misaligned
    assert lib.rl_policy_loss_fwd_bwd(C.byref(b), C.byref(prm), 0, C.byref(out), 0x1000, 16, None) == 5   # too small
    assert lib.rl_token_logprob(C.byref(b), fake, None, 0x1000, 16, None) == 5
    for bad_t in (0.0, -2.0, float("inf"), float("nan")):
        assert lib.rl_token_logprob_tempered(C.byref(b), bad_t, fake, None, 0x1000, 1 << 40, None) == 4, bad_t
    assert lib.rl_token_logprob_tempered(C.byref(b), 0.7, fake, None, 0x1000, 16, None) == 5
    assert b"workspace" in lib.rl_status_string(5)


def test_logz_head_arguments_are_validated_on_the_host(lib):
    n = C.c_size_t(0)
    assert lib.rl_logz_head_workspace_bytes(16, 3584, 3584, C.byref(n)) == 0
    assert n.value >= 4 * 16 * (3584 + 3 * 3584) and n.value % 256 == 0
    assert lib.rl_logz_head_workspace_bytes(16, 3584, 3584, None) == 1
    for bad in ((0, 64, 64), (4, 0, 64), (4, 64, 0), (4, 64, 1 << 20)):
        assert lib.rl_logz_head_workspace_bytes(*bad, C.byref(n)) == 2, bad
    fake = 0x1000
    f = lib.rl_logz_head_forward
    assert f(None, 1, 10, 64, fake, 2, fake, fake, fake, fake, 8, fake, fake, 1 << 30, None) == 1
    assert f(fake, 5, 10, 64, fake, 2, fake, fake, fake, fake, 8, fake, fake, 1 << 30, None) == 3
    assert f(fake, 1, -1, 64, fake, 2, fake, fake, fake, fake, 8, fake, fake, 1 << 30, None) == 2
    assert f(fake, 1, 10, 64, fake, 2, fake, fake, fake, fake, 8, fake, None, 0, None) == 5
    assert f(fake, 1, 10, 64, fake, 2, fake, fake, fake, fake, 8, fake, fake, 16, None) == 5
    bw = lib.rl_logz_head_backward
    assert bw(None, 2, 64, 8, fake, fake, fake, fake, fake, fake, 1 << 30, None) == 1
    assert bw(fake, 2, 64, 8, fake, fake, fake, fake, fake, 0x1001, 1 << 30, None) == 5


def test_product_path_has_no_oracle_dependency():
    """The package must not import the oracle (it is test infrastructure)."""
    pkg = os.path.join(ROOT, "paper_2603_16435_amd")
    for dirpath, _, files in os.walk(pkg):
        for fn in files:
            if fn.endswith((".py", ".hip", ".h")):
                text = open(os.path.join(dirpath, fn)).read()
                assert "oracle" not in text.replace("CPU oracle", "").lower() or fn == "synth.py", (dirpath, fn)


@pytest.mark.parametrize("by_share", [0, 1])
def test_tile_order_visits_every_tile_once_and_keeps_dies_balanced(lib, by_share):
    """Host logic of the workgroup -> tile map: a bijection onto the tile grid for any grid and band height,
    every accelerator die (workgroup id % 8) gets an equal part, and with shares all dies sweep N in step."""
    for tiles_m, tiles_n, group_m in [(1, 1, 8), (3, 5, 8), (7, 14, 1), (8, 14, 8), (20, 14, 8), (23, 3, 4), (188, 14, 8),
                                      (594, 14, 1), (594, 160, 8), (125, 19, 16), (9, 1, 2)]:
        n = C.c_int32(0)
        assert lib.rl_debug_tile_order(tiles_m, tiles_n, group_m, by_share, C.byref(n), None) == 0
        assert n.value >= tiles_m * tiles_n and n.value % 8 == 0
        buf = (C.c_int32 * (2 * n.value))()
        assert lib.rl_debug_tile_order(tiles_m, tiles_n, group_m, by_share, C.byref(n), buf) == 0
        seen, per_die, seq = set(), [0] * 8, [[] for _ in range(8)]
        for w in range(n.value):
            tm, tn = buf[2 * w], buf[2 * w + 1]
            if tm < 0:
                assert tn < 0
                continue
            assert 0 <= tm < tiles_m and 0 <= tn < tiles_n and (tm, tn) not in seen, (tiles_m, tiles_n, group_m, w)
            seen.add((tm, tn)); per_die[w % 8] += 1; seq[w % 8].append((tm, tn))
        assert len(seen) == tiles_m * tiles_n
        if by_share:
            assert max(per_die) - min(per_die) <= tiles_n          # shares differ by at most one M-tile
            # in step: the q-th tile of every die with a full-height share sits in the same N-tile
            full = [s for s in seq if len(s) == max(per_die)]
            for q in range(0, max(per_die), 7):
                assert len({s[q][1] for s in full}) == 1
            # an M-tile belongs to one die only
            owner = {}
            for die, s in enumerate(seq):
                for tm, _ in s:
                    assert owner.setdefault(tm, die) == die
        else:
            assert max(per_die) - min(per_die) <= 1
    assert lib.rl_debug_tile_order(0, 4, 8, 0, C.byref(n), None) == 2
    assert lib.rl_debug_tile_order(4, 4, 8, 0, None, None) == 1


def test_rvq_encode_rejects_shapes_it_is_not_written_for(lib):
    # host checks only: the pointers are never dereferenced (any non-null value will do), nothing is launched
    p = C.c_void_p(4096)
    args = lambda D, S, N=4, G=1, L=10: (p, p, p, C.c_int32(G), C.c_int64(L), C.c_int32(D), C.c_int32(N), C.c_int32(S), p, None, None)
    lib.rl_rvq_encode.argtypes = [C.c_void_p, C.c_void_p, C.c_void_p, C.c_int32, C.c_int64, C.c_int32, C.c_int32, C.c_int32,
                                  C.c_void_p, C.c_void_p, C.c_void_p]
    lib.rl_rvq_encode.restype = C.c_int
    assert lib.rl_rvq_encode(*args(64, 1024)) == 2           # head dimension other than 128
    assert lib.rl_rvq_encode(*args(128, 100)) == 2           # S not a multiple of 64
    assert lib.rl_rvq_encode(*args(128, 131072, N=1)) == 2   # more entries than block numbers of 12 bits can name
    assert lib.rl_rvq_encode(*args(128, 1024, G=0)) == 2
    assert lib.rl_rvq_encode(None, p, p, 1, 10, 128, 4, 1024, p, None, None) == 1
