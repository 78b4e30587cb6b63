"""Thin ctypes binding over the C ABI declared in include/rl_policy.h.

Argument marshalling only: torch tensors supply device memory and the current stream, every
step of the path runs in the HIP library.  There is no fallback: if the library has not been
built (`python -m paper_2603_16435_amd.build`) loading fails with an error."""
from __future__ import annotations

import ctypes as C
import os
from dataclasses import dataclass
from typing import Optional

import torch

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "librl_policy.so")

RL_OBJ_GRPO, RL_OBJ_FLOW = 0, 1
RL_F32, RL_BF16 = 0, 1
OBJECTIVES = {"grpo": RL_OBJ_GRPO, "flow": RL_OBJ_FLOW}


class rl_batch(C.Structure):
    _fields_ = [("R", C.c_int64), ("H", C.c_int32), ("V", C.c_int32), ("B", C.c_int32), ("P", C.c_int32),
                ("dtype", C.c_int32), ("reserved", C.c_int32),
                ("hidden", C.c_void_p), ("weight", C.c_void_p), ("token_ids", C.c_void_p), ("mask", C.c_void_p),
                ("cu_seqlens", C.c_void_p), ("group_idx", C.c_void_p), ("rewards", C.c_void_p),
                ("old_logprob", C.c_void_p), ("ref_logprob", C.c_void_p), ("log_z", C.c_void_p)]


class rl_params(C.Structure):
    _fields_ = [("clip_eps", C.c_float), ("kl_coef", C.c_float), ("beta", C.c_float), ("adv_eps", C.c_float),
                ("adv_std_ddof", C.c_int32), ("chunk_rows", C.c_int32),
                ("clip_eps_high", C.c_float), ("aggregation", C.c_int32), ("ratio_level", C.c_int32),
                ("flow_weight_norm", C.c_int32),
                ("backward_mode", C.c_int32), ("max_seq_len", C.c_int32), ("temperature", C.c_float)]


class rl_stats(C.Structure):
    _fields_ = [("n_tokens", C.c_int32), ("n_clip_hi", C.c_int32), ("n_clip_lo", C.c_int32),
                ("n_bad_token", C.c_int32), ("n_bad_group", C.c_int32), ("n_bad_seq", C.c_int32),
                ("n_seq_too_long", C.c_int32), ("n_overflow_rows", C.c_int32)]


class rl_outputs(C.Structure):
    _fields_ = [("loss", C.c_void_p), ("seq_loss", C.c_void_p), ("logprob", C.c_void_p), ("lse", C.c_void_p),
                ("advantages", C.c_void_p), ("seq_len", C.c_void_p), ("coeff", C.c_void_p),
                ("d_hidden", C.c_void_p), ("d_weight", C.c_void_p), ("d_log_z", C.c_void_p), ("stats", C.c_void_p),
                ("entropy", C.c_void_p), ("row_map", C.c_void_p), ("group_count", C.c_void_p), ("target_col", C.c_void_p),
                ("target_logit", C.c_void_p)]


PROF_CLASSES = ("prep", "gemm_fwd", "combine", "loss", "transpose", "gemm_ds", "gemm_dx", "gemm_dw", "gemm_bwd")


class rl_profile(C.Structure):
    _fields_ = [("ms", C.c_double * 9), ("launches", C.c_int64 * 9)]


STATS_FIELDS = ("n_tokens", "n_clip_hi", "n_clip_lo", "n_bad_token", "n_bad_group", "n_bad_seq", "n_seq_too_long", "n_overflow_rows")
BACKWARD_MODES = {"auto": 0, "recompute": 1, "stash": 2}

_lib = None


class RlError(RuntimeError):
    def __init__(self, status: int, msg: str):
        super().__init__(f"rl_policy: status {status}: {msg}")
        self.status = status


def lib() -> C.CDLL:
    """Load the in-tree library (once).  Raises if it has not been built."""
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise RuntimeError(f"{LIB_PATH} is missing: build it with `python -m paper_2603_16435_amd.build` "
                               "(there is no fallback path)")
        L = C.CDLL(LIB_PATH)
        L.rl_workspace_bytes.argtypes = [C.POINTER(rl_batch), C.POINTER(rl_params), C.c_int32, C.POINTER(C.c_size_t)]
        L.rl_workspace_bytes.restype = C.c_int
        L.rl_token_logprob.argtypes = [C.POINTER(rl_batch), C.c_void_p, C.c_void_p, C.c_void_p, C.c_size_t, C.c_void_p]
        L.rl_token_logprob.restype = C.c_int
        L.rl_token_logprob_tempered.argtypes = [C.POINTER(rl_batch), C.c_float, C.c_void_p, C.c_void_p, C.c_void_p, C.c_size_t, C.c_void_p]
        L.rl_token_logprob_tempered.restype = C.c_int
        L.rl_token_logprob_static.argtypes = [C.POINTER(rl_batch), C.c_float, C.c_void_p, C.c_void_p, C.c_void_p]
        L.rl_token_logprob_static.restype = C.c_int
        L.rl_policy_loss_fwd_bwd.argtypes = [C.POINTER(rl_batch), C.POINTER(rl_params), C.c_int32,
                                             C.POINTER(rl_outputs), C.c_void_p, C.c_size_t, C.c_void_p]
        L.rl_policy_loss_fwd_bwd.restype = C.c_int
        L.rl_status_string.argtypes = [C.c_int32]
        L.rl_status_string.restype = C.c_char_p
        L.rl_profile_enable.argtypes = [C.c_int32]
        L.rl_profile_enable.restype = None
        L.rl_profile_read.argtypes = [C.POINTER(rl_profile)]
        L.rl_profile_read.restype = C.c_int
        L.rl_measure_mfma_peak.argtypes = [C.c_int32, C.c_void_p, C.c_size_t, C.c_void_p, C.POINTER(C.c_double), C.POINTER(C.c_double)]
        L.rl_measure_mfma_peak.restype = C.c_int
        L.rl_logz_head_workspace_bytes.argtypes = [C.c_int32, C.c_int32, C.c_int32, C.POINTER(C.c_size_t)]
        L.rl_logz_head_workspace_bytes.restype = C.c_int
        L.rl_logz_head_forward.argtypes = [C.c_void_p, C.c_int32, C.c_int64, C.c_int32, C.c_void_p, C.c_int32, C.c_void_p, C.c_void_p,
                                           C.c_void_p, C.c_void_p, C.c_int32, C.c_void_p, C.c_void_p, C.c_size_t, C.c_void_p]
        L.rl_logz_head_forward.restype = C.c_int
        L.rl_logz_head_backward.argtypes = [C.c_void_p, C.c_int32, C.c_int32, C.c_int32, C.c_void_p, C.c_void_p, C.c_void_p,
                                            C.c_void_p, C.c_void_p, C.c_void_p, C.c_size_t, C.c_void_p]
        L.rl_logz_head_backward.restype = C.c_int
        L.rl_rvq_codebook_norms.argtypes = [C.c_void_p, C.c_int32, C.c_int32, C.c_int32, C.c_int32, C.c_void_p, C.c_void_p]
        L.rl_rvq_codebook_norms.restype = C.c_int
        L.rl_rvq_encode.argtypes = [C.c_void_p, C.c_void_p, C.c_void_p, C.c_int32, C.c_int64, C.c_int32, C.c_int32, C.c_int32,
                                    C.c_void_p, C.c_void_p, C.c_void_p]
        L.rl_rvq_encode.restype = C.c_int
        L.rl_rvq_encode_counted.argtypes = [C.c_void_p, C.c_void_p, C.c_void_p, C.c_int32, C.c_int64, C.c_int32, C.c_int32, C.c_int32,
                                            C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p]
        L.rl_rvq_encode_counted.restype = C.c_int
        L.rl_version.restype = C.c_int32
        L.rl_default_chunk_rows.restype = C.c_int32
        L.rl_default_chunk_rows_single_pass.restype = C.c_int32
        L.rl_debug_tile_order.argtypes = [C.c_int32, C.c_int32, C.c_int32, C.c_int32, C.POINTER(C.c_int32), C.POINTER(C.c_int32)]
        L.rl_debug_tile_order.restype = C.c_int
        _lib = L
    return _lib


def _check(st: int):
    if st != 0:
        raise RlError(st, lib().rl_status_string(st).decode())


def _ptr(t: Optional[torch.Tensor], dtype=None, numel=None, name="tensor"):
    if t is None:
        return None
    if not t.is_cuda:
        raise ValueError(f"{name} must live on the GPU")
    if not t.is_contiguous():
        raise ValueError(f"{name} must be contiguous")
    if dtype is not None and t.dtype != dtype:
        raise ValueError(f"{name} must be {dtype}, got {t.dtype}")
    if numel is not None and t.numel() != numel:
        raise ValueError(f"{name} must have {numel} elements, got {t.numel()}")
    return t.data_ptr()


def _dtype_code(t: torch.Tensor) -> int:
    if t.dtype == torch.float32:
        return RL_F32
    if t.dtype == torch.bfloat16:
        return RL_BF16
    raise ValueError(f"hidden/weight must be float32 or bfloat16, got {t.dtype}")


def make_batch(hidden, weight, token_ids, mask, cu_seqlens, group_idx=None, rewards=None,
               old_logprob=None, ref_logprob=None, log_z=None, P: Optional[int] = None) -> rl_batch:
    R, H = hidden.shape
    V = weight.shape[0]
    if weight.shape[1] != H or weight.dtype != hidden.dtype:
        raise ValueError("weight must be [V,H] with the dtype of hidden")
    B = cu_seqlens.numel() - 1
    if P is None:
        P = log_z.numel() if log_z is not None else 1
    b = rl_batch()
    b.R, b.H, b.V, b.B, b.P = R, H, V, B, P
    b.dtype = _dtype_code(hidden)
    b.hidden = _ptr(hidden, name="hidden")
    b.weight = _ptr(weight, name="weight")
    b.token_ids = _ptr(token_ids, torch.int32, R, "token_ids")
    b.mask = _ptr(mask, torch.uint8, R, "mask")
    b.cu_seqlens = _ptr(cu_seqlens, torch.int32, B + 1, "cu_seqlens")
    b.group_idx = _ptr(group_idx, torch.int32, B, "group_idx")
    b.rewards = _ptr(rewards, torch.float32, B, "rewards")
    b.old_logprob = _ptr(old_logprob, torch.float32, R, "old_logprob")
    b.ref_logprob = _ptr(ref_logprob, torch.float32, R, "ref_logprob")
    b.log_z = _ptr(log_z, torch.float32, P, "log_z")
    return b


def rl_workspace_bytes(batch: rl_batch, params: Optional[rl_params], want_backward: bool) -> int:
    n = C.c_size_t(0)
    _check(lib().rl_workspace_bytes(C.byref(batch), C.byref(params) if params is not None else None,
                                    1 if want_backward else 0, C.byref(n)))
    return n.value


def _workspace(nbytes: int, device) -> torch.Tensor:
    ws = torch.empty(nbytes + 256, dtype=torch.uint8, device=device)
    off = (-ws.data_ptr()) % 256
    return ws[off:off + nbytes]


def _stream_handle() -> int:
    return torch.cuda.current_stream().cuda_stream


def rl_token_logprob(hidden, weight, token_ids, mask, cu_seqlens=None, workspace=None):
    """Forward only: (logprob[R], lse[R]) float32; masked rows read 0."""
    return _token_logprob(hidden, weight, token_ids, mask, cu_seqlens, workspace, None)


def rl_token_logprob_tempered(hidden, weight, token_ids, mask, temperature, cu_seqlens=None, workspace=None):
    """The same under softmax(W x / temperature)."""
    return _token_logprob(hidden, weight, token_ids, mask, cu_seqlens, workspace, float(temperature))


def rl_token_logprob_static(hidden, weight, token_ids, mask, cu_seqlens, logprob, lse, temperature=1.0):
    """The scoring call that allocates nothing: its workspace is a static device array of the library (batches beyond
    its size are refused).  The caller passes everything, outputs logprob[R] / lse[R] (float32) included."""
    b = make_batch(hidden, weight, token_ids, mask, cu_seqlens)
    _check(lib().rl_token_logprob_static(C.byref(b), float(temperature), _ptr(logprob, torch.float32, b.R, "logprob"),
                                         _ptr(lse, torch.float32, b.R, "lse"), _stream_handle()))


def _token_logprob(hidden, weight, token_ids, mask, cu_seqlens, workspace, temperature):
    R = hidden.shape[0]
    dev = hidden.device
    if cu_seqlens is None:
        cu_seqlens = torch.tensor([0, R], dtype=torch.int32, device=dev)
    b = make_batch(hidden, weight, token_ids, mask, cu_seqlens)
    need = rl_workspace_bytes(b, None, False)
    ws = workspace if workspace is not None else _workspace(need, dev)
    logp = torch.empty(R, dtype=torch.float32, device=dev)
    lse = torch.empty(R, dtype=torch.float32, device=dev)
    if temperature is None:
        _check(lib().rl_token_logprob(C.byref(b), logp.data_ptr(), lse.data_ptr(), ws.data_ptr(), ws.numel(),
                                      _stream_handle()))
    else:
        _check(lib().rl_token_logprob_tempered(C.byref(b), temperature, logp.data_ptr(), lse.data_ptr(), ws.data_ptr(),
                                               ws.numel(), _stream_handle()))
    return logp, lse


@dataclass
class LossResult:
    loss: torch.Tensor
    seq_loss: torch.Tensor
    logprob: torch.Tensor
    lse: torch.Tensor
    advantages: torch.Tensor
    seq_len: torch.Tensor
    coeff: torch.Tensor
    d_hidden: Optional[torch.Tensor]
    d_weight: Optional[torch.Tensor]
    d_log_z: torch.Tensor
    stats: torch.Tensor          # int32[8]: see STATS_FIELDS
    entropy: Optional[torch.Tensor] = None
    row_map: Optional[torch.Tensor] = None       # int32[R]: first T entries = original rows of the counting rows, rest -1
    group_count: Optional[torch.Tensor] = None   # int32[P]
    target_col: Optional[torch.Tensor] = None    # int32[R]: vocabulary entry the target logit was read from, -1 on other rows
    target_logit: Optional[torch.Tensor] = None  # float32[R]

    def stats_dict(self):
        v = self.stats.cpu().tolist()
        return dict(zip(STATS_FIELDS, v))


class PolicyLossPlan:
    """Pre-allocated outputs + workspace for repeated calls on one batch shape (timing loops)."""

    def __init__(self, batch: rl_batch, params: rl_params, device, hidden_dtype, backward=True, index_outputs=False):
        R, H, V, B, P = batch.R, batch.H, batch.V, batch.B, batch.P
        f32 = dict(dtype=torch.float32, device=device)
        self.res = LossResult(
            loss=torch.empty(1, **f32), seq_loss=torch.empty(B, **f32), logprob=torch.empty(R, **f32),
            lse=torch.empty(R, **f32), advantages=torch.empty(B, **f32),
            seq_len=torch.empty(B, dtype=torch.int32, device=device), coeff=torch.empty(R, **f32),
            d_hidden=torch.empty((R, H), dtype=hidden_dtype, device=device) if backward else None,
            d_weight=torch.empty((V, H), **f32) if backward else None,
            d_log_z=torch.empty(P, **f32), stats=torch.zeros(8, dtype=torch.int32, device=device),
            entropy=torch.empty(R, **f32))
        if index_outputs:
            i32 = dict(dtype=torch.int32, device=device)
            self.res.row_map, self.res.group_count = torch.empty(R, **i32), torch.empty(P, **i32)
            self.res.target_col, self.res.target_logit = torch.empty(R, **i32), torch.empty(R, **f32)
        self.ws = _workspace(rl_workspace_bytes(batch, params, backward), device)
        o = rl_outputs()
        r = self.res
        o.loss, o.seq_loss, o.logprob, o.lse = r.loss.data_ptr(), r.seq_loss.data_ptr(), r.logprob.data_ptr(), r.lse.data_ptr()
        o.advantages, o.seq_len, o.coeff = r.advantages.data_ptr(), r.seq_len.data_ptr(), r.coeff.data_ptr()
        o.d_hidden = r.d_hidden.data_ptr() if backward else None
        o.d_weight = r.d_weight.data_ptr() if backward else None
        o.d_log_z, o.stats = r.d_log_z.data_ptr(), r.stats.data_ptr()
        o.entropy = r.entropy.data_ptr()
        if index_outputs:
            o.row_map, o.group_count = r.row_map.data_ptr(), r.group_count.data_ptr()
            o.target_col, o.target_logit = r.target_col.data_ptr(), r.target_logit.data_ptr()
        self.out = o
        self.batch, self.params = batch, params

    def run(self, objective: int, stream: Optional[int] = None) -> LossResult:
        _check(lib().rl_policy_loss_fwd_bwd(C.byref(self.batch), C.byref(self.params), objective, C.byref(self.out),
                                            self.ws.data_ptr(), self.ws.numel(),
                                            _stream_handle() if stream is None else stream))
        return self.res


AGGREGATIONS = {"sequence": 0, "token": 1}
RATIO_LEVELS = {"token": 0, "sequence": 1}
WEIGHT_NORMS = {"sum": 0, "mean": 1}


def _enum(table, v):
    return table[v] if isinstance(v, str) else int(v)


def make_params(clip_eps=0.2, kl_coef=1e-3, beta=15.0, adv_eps=1e-6, adv_std_ddof=0, chunk_rows=0,
                backward_mode="auto", max_seq_len=0, clip_eps_high=0.0, aggregation="sequence",
                ratio_level="token", flow_weight_norm="sum", temperature=0.0) -> rl_params:
    return rl_params(clip_eps, kl_coef, beta, adv_eps, adv_std_ddof, chunk_rows,
                     float(clip_eps_high or 0.0), _enum(AGGREGATIONS, aggregation), _enum(RATIO_LEVELS, ratio_level),
                     _enum(WEIGHT_NORMS, flow_weight_norm), _enum(BACKWARD_MODES, backward_mode), int(max_seq_len),
                     float(temperature or 0.0))


def rl_policy_loss_fwd_bwd(objective, hidden, weight, token_ids, mask, cu_seqlens, group_idx, rewards,
                           old_logprob, ref_logprob, log_z=None, P: Optional[int] = None,
                           clip_eps=0.2, kl_coef=1e-3, beta=15.0, adv_eps=1e-6, adv_std_ddof=0,
                           chunk_rows=0, backward=True, backward_mode="auto", max_seq_len=0, clip_eps_high=0.0,
                           aggregation="sequence", ratio_level="token", flow_weight_norm="sum",
                           temperature=0.0, index_outputs=False) -> LossResult:
    """One pass of the whole path.  `objective` is "grpo" | "flow" (or the enum value)."""
    obj = OBJECTIVES[objective] if isinstance(objective, str) else int(objective)
    b = make_batch(hidden, weight, token_ids, mask, cu_seqlens, group_idx, rewards, old_logprob, ref_logprob, log_z, P)
    prm = make_params(clip_eps, kl_coef, beta, adv_eps, adv_std_ddof, chunk_rows, backward_mode, max_seq_len,
                      clip_eps_high, aggregation, ratio_level, flow_weight_norm, temperature)
    plan = PolicyLossPlan(b, prm, hidden.device, hidden.dtype, backward, index_outputs)
    return plan.run(obj)


def rl_profile_enable(on: bool) -> None:
    lib().rl_profile_enable(1 if on else 0)


def rl_profile_read() -> dict:
    """{class: (ms, brackets)} accumulated since the last read (waits for the recorded events)."""
    pr = rl_profile()
    _check(lib().rl_profile_read(C.byref(pr)))
    return {name: (pr.ms[i], pr.launches[i]) for i, name in enumerate(PROF_CLASSES)}


def rl_measure_mfma_peak(millis: int = 200, device="cuda:0"):
    """(TFLOP/s, shader MHz) of a pure bf16 MFMA issue loop run for about `millis` ms (synchronises)."""
    buf = torch.empty(2 << 20, dtype=torch.uint8, device=device)
    t, m = C.c_double(0), C.c_double(0)
    _check(lib().rl_measure_mfma_peak(millis, buf.data_ptr(), buf.numel(), _stream_handle(), C.byref(t), C.byref(m)))
    return t.value, m.value


# ------------------------------------------------------------------ log-Z head
def rl_logz_head_forward(prompt_hidden, cu_prompt, W1, b1, w2, b2, workspace=None):
    """log_z[P] = w2 . gelu(W1 mean(prompt rows) + b1) + b2.  Returns (log_z, workspace); hand the workspace to
    rl_logz_head_backward unchanged."""
    dev = prompt_hidden.device
    rows, H = prompt_hidden.shape
    P = cu_prompt.numel() - 1
    M = W1.shape[0]
    assert prompt_hidden.is_contiguous() and W1.is_contiguous() and W1.dtype == torch.float32 and W1.shape[1] == H
    assert cu_prompt.dtype == torch.int32 and b1.dtype == w2.dtype == b2.dtype == torch.float32
    need = C.c_size_t(0)
    _check(lib().rl_logz_head_workspace_bytes(P, H, M, C.byref(need)))
    ws = workspace if workspace is not None else _workspace(need.value, dev)
    log_z = torch.empty(P, dtype=torch.float32, device=dev)
    _check(lib().rl_logz_head_forward(prompt_hidden.data_ptr(), _dtype_code(prompt_hidden), rows, H, cu_prompt.data_ptr(), P,
                                      W1.data_ptr(), b1.data_ptr(), w2.data_ptr(), b2.data_ptr(), M, log_z.data_ptr(),
                                      ws.data_ptr(), ws.numel(), _stream_handle()))
    return log_z, ws


def rl_logz_head_backward(d_log_z, w2, H, workspace):
    """Parameter gradients (dW1[M,H], db1[M], dw2[M], db2[1]) from d_log_z[P] and the forward's workspace."""
    dev = d_log_z.device
    P, M = d_log_z.numel(), w2.numel()
    assert d_log_z.dtype == torch.float32 and w2.dtype == torch.float32
    dW1 = torch.empty(M, H, dtype=torch.float32, device=dev)
    db1 = torch.empty(M, dtype=torch.float32, device=dev)
    dw2 = torch.empty(M, dtype=torch.float32, device=dev)
    db2 = torch.empty(1, dtype=torch.float32, device=dev)
    _check(lib().rl_logz_head_backward(d_log_z.data_ptr(), P, H, M, w2.data_ptr(), dW1.data_ptr(), db1.data_ptr(), dw2.data_ptr(),
                                       db2.data_ptr(), workspace.data_ptr(), workspace.numel(), _stream_handle()))
    return dW1, db1, dw2, db2


# ------------------------------------------------------------------ residual-VQ encode
def rl_rvq_codebook_norms(codebooks):
    """Squared norms [G, N, S] (float32) of the codebook entries [G, N, S, D] (bfloat16): computed once per codebook set."""
    G, N, S, D = codebooks.shape
    assert codebooks.dtype == torch.bfloat16 and codebooks.is_contiguous()
    norms = torch.empty(G, N, S, dtype=torch.float32, device=codebooks.device)
    _check(lib().rl_rvq_codebook_norms(codebooks.data_ptr(), G, N, S, D, norms.data_ptr(), _stream_handle()))
    return norms


def rl_rvq_encode(vectors, codebooks, norms=None, want_residual=True, count_exact=None):
    """codes [G, L, N] int32 (and the residual [G, L, D] bfloat16) of vectors [G, L, D] under codebooks [G, N, S, D].
    count_exact: optional int32[1] device tensor that the diagnostic entry point adds the number of decisions to that
    were re-evaluated exactly in float64."""
    G, L, D = vectors.shape
    _, N, S, _ = codebooks.shape
    assert vectors.dtype == torch.bfloat16 and vectors.is_contiguous() and codebooks.shape[0] == G and codebooks.shape[3] == D
    if norms is None:
        norms = rl_rvq_codebook_norms(codebooks)
    codes = torch.empty(G, L, N, dtype=torch.int32, device=vectors.device)
    res = torch.empty_like(vectors) if want_residual else None
    if count_exact is not None:
        _check(lib().rl_rvq_encode_counted(vectors.data_ptr(), codebooks.data_ptr(), norms.data_ptr(), G, L, D, N, S, codes.data_ptr(),
                                           res.data_ptr() if want_residual else None, _ptr(count_exact, torch.int32, 1, "count_exact"),
                                           _stream_handle()))
        return codes, res
    _check(lib().rl_rvq_encode(vectors.data_ptr(), codebooks.data_ptr(), norms.data_ptr(), G, L, D, N, S, codes.data_ptr(),
                               res.data_ptr() if want_residual else None, _stream_handle()))
    return codes, res

