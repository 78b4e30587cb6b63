"""Seeded synthetic rollout batches (inputs only; none of the method's arithmetic).

This module serves both the HIP path and the CPU oracle with the same stored
bits.  It draws every tensor from one counter-based generator (a 64-bit integer
mixer keyed by (seed, tensor tag, element index)), so any slice of any tensor
can be produced without producing the rest, in any chunking, on any device.
Integer outputs (lengths, ids, rewards, masks, offsets) are identical across
devices; floating outputs go through the device's own log/cos, so a batch is
generated ONCE on one device and both sides then read those bits.

The five workload shapes are the ones the benchmark contract names: a group of
G sampled responses for each of P prompts, response lengths uniform in a
range, hidden ~ N(0,1), LM-head weight ~ N(0, 0.02), token ids uniform in
[0,V), binary rewards, old / reference log-probs = "current" + N(0, 0.05),
log Z ~ N(0,1).

"current" here is a closed-form stand-in, not a call into either
implementation: for Gaussian weights the logits of row t are ~N(0, s^2) with
s = 0.02*|x_t|, hence logsumexp ~= ln V + s^2/2, and the target logit is one
H-long dot product.  old/ref therefore sit within a few 1e-2 of the true
log-prob plus the stated noise, which is what the objectives need (ratios near
1, rare clipping), and no input ever depends on the code under test.
"""
from __future__ import annotations

import math
from dataclasses import dataclass, field

import torch

_MASK63 = (1 << 63) - 1


def _s64(u: int) -> int:
    """Reinterpret an unsigned 64-bit constant as a signed python int."""
    u &= (1 << 64) - 1
    return u - (1 << 64) if u >= (1 << 63) else u


_GOLD = _s64(0x9E3779B97F4A7C15)
_M1 = _s64(0xBF58476D1CE4E5B9)
_M2 = _s64(0x94D049BB133111EB)


def _lsr(x: torch.Tensor, s: int) -> torch.Tensor:
    """Logical right shift on int64 (torch's >> is arithmetic)."""
    return (x >> s) & ((1 << (64 - s)) - 1)


def _mix(x: torch.Tensor) -> torch.Tensor:
    """splitmix64 finaliser on int64 tensors (two's-complement wrap-around)."""
    x = x ^ _lsr(x, 30)
    x = x * _M1
    x = x ^ _lsr(x, 27)
    x = x * _M2
    x = x ^ _lsr(x, 31)
    return x


def _key(seed: int, tag: int) -> int:
    """Scalar stream key from (seed, tensor tag), mixed on the host."""
    def mix_int(v: int) -> int:
        v &= (1 << 64) - 1
        v ^= v >> 30
        v = (v * 0xBF58476D1CE4E5B9) & ((1 << 64) - 1)
        v ^= v >> 27
        v = (v * 0x94D049BB133111EB) & ((1 << 64) - 1)
        v ^= v >> 31
        return v
    return _s64(mix_int(mix_int(seed) ^ (tag * 0x9E3779B97F4A7C15)))


def hash_u64(seed: int, tag: int, start: int, count: int, device) -> torch.Tensor:
    """int64 tensor of `count` hashed words for element indices start..start+count."""
    idx = torch.arange(start, start + count, dtype=torch.int64, device=device)
    return _mix(idx * _GOLD + _key(seed, tag))


def uniform01(seed, tag, start, count, device) -> torch.Tensor:
    """float32 uniforms in (0,1): the top 24 bits of the hash, centred in their cell."""
    h = hash_u64(seed, tag, start, count, device)
    return (_lsr(h, 40).to(torch.float32) + 0.5) * (1.0 / 16777216.0)


def normal(seed, tag, start, count, device) -> torch.Tensor:
    """float32 standard normals by Box-Muller from two 24-bit uniforms per word."""
    h = hash_u64(seed, tag, start, count, device)
    u1 = ((_lsr(h, 40) & 0xFFFFFF).to(torch.float32) + 0.5) * (1.0 / 16777216.0)
    u2 = ((h & 0xFFFFFF).to(torch.float32) + 0.5) * (1.0 / 16777216.0)
    return torch.sqrt(-2.0 * torch.log(u1)) * torch.cos((2.0 * math.pi) * u2)


def randint(seed, tag, start, count, lo: int, hi: int, device) -> torch.Tensor:
    """int64 integers uniform in [lo, hi] (inclusive)."""
    h = hash_u64(seed, tag, start, count, device) & _MASK63
    return lo + h % (hi - lo + 1)


# tensor tags
_T_LEN, _T_HID, _T_W, _T_IDS, _T_REW, _T_OLD, _T_REF, _T_LOGZ, _T_EQ, _T_EQV = range(1, 11)


@dataclass(frozen=True)
class RolloutConfig:
    name: str
    P: int                 # prompts
    G: int                 # rollouts per prompt
    len_lo: int
    len_hi: int
    H: int
    V: int
    dtype: str             # "f32" | "bf16"
    reward_p: float
    equal_group_frac: float = 0.0   # share of groups forced to one common reward
    seed: int = 0
    clip_eps: float = 0.2
    kl_coef: float = 1e-3
    beta: float = 15.0
    adv_eps: float = 1e-6
    adv_std_ddof: int = 0


CONFIGS = {
    "tiny": RolloutConfig("tiny", 2, 4, 16, 64, 128, 1024, "f32", 0.5, seed=0x5EED0000),
    "small": RolloutConfig("small", 8, 8, 128, 1024, 2048, 32000, "bf16", 0.3, seed=0x5EED0001),
    "7b": RolloutConfig("7b", 16, 8, 512, 4096, 3584, 152064, "bf16", 0.4, seed=0x5EED0002),
    "long": RolloutConfig("long", 4, 16, 4096, 16384, 4096, 151936, "bf16", 0.2, seed=0x5EED0003),
    "32b": RolloutConfig("32b", 32, 8, 1024, 8192, 5120, 152064, "bf16", 0.5,
                         equal_group_frac=0.1, seed=0x5EED0004),
}


@dataclass
class RolloutBatch:
    cfg: RolloutConfig
    layout: str
    R: int
    T: int
    B: int
    hidden: torch.Tensor        # [R,H] f32 | bf16
    weight: torch.Tensor        # [V,H] same dtype
    token_ids: torch.Tensor     # [R] int32
    mask: torch.Tensor          # [R] uint8
    cu_seqlens: torch.Tensor    # [B+1] int32
    group_idx: torch.Tensor     # [B] int32
    rewards: torch.Tensor       # [B] f32
    old_logprob: torch.Tensor   # [R] f32
    ref_logprob: torch.Tensor   # [R] f32
    log_z: torch.Tensor         # [P] f32
    lengths: torch.Tensor       # [B] int32 (host-side convenience, = per-sequence mask sums)
    extra: dict = field(default_factory=dict)


def _fill_normal(out: torch.Tensor, seed: int, tag: int, scale: float, chunk: int = 1 << 24):
    flat = out.view(-1)
    n = flat.numel()
    for s in range(0, n, chunk):
        c = min(chunk, n - s)
        z = normal(seed, tag, s, c, out.device)
        if scale != 1.0:
            z = z * scale
        flat[s:s + c] = z.to(out.dtype)


def sequence_lengths(cfg: RolloutConfig, len_div: int = 1) -> torch.Tensor:
    """Per-sequence response lengths (CPU int64), optionally each cut to ceil(len/len_div)."""
    B = cfg.P * cfg.G
    ln = randint(cfg.seed, _T_LEN, 0, B, cfg.len_lo, cfg.len_hi, "cpu")
    if len_div > 1:
        ln = (ln + len_div - 1) // len_div
    return ln


def make_rollouts(cfg: RolloutConfig | str, device="cpu", layout: str = "padded",
                  len_div: int = 1, noise: float = 0.05, weight_std: float = 0.02,
                  lengths=None, temperature: float = 1.0) -> RolloutBatch:
    """Build one batch.

    layout "padded": R = B*Lmax rows, sequence i owns rows [i*Lmax, (i+1)*Lmax), its first
    len_i rows have mask 1, the rest are masked and hold ordinary random values (so that
    ignoring them is tested).  layout "packed": R = T, all rows real.
    len_div > 1 shortens every sequence to ceil(len/len_div) tokens (the token-sub-sampled
    instance of a big configuration: same H, V, P, G, same distributions).
    `lengths` (list of B ints) overrides the drawn lengths (directed edge cases).
    `temperature`: the old / reference log-probs are centred on the policy softmax(W x / temperature).
    """
    if isinstance(cfg, str):
        cfg = CONFIGS[cfg]
    dev = torch.device(device)
    P, G, H, V = cfg.P, cfg.G, cfg.H, cfg.V
    B = P * G
    if lengths is None:
        ln = sequence_lengths(cfg, len_div)
    else:
        ln = torch.as_tensor(list(lengths), dtype=torch.int64)
        assert ln.numel() == B
    T = int(ln.sum())
    if layout == "padded":
        Lmax = max(int(ln.max()), 1)
        R = B * Lmax
        cu = torch.arange(B + 1, dtype=torch.int64) * Lmax
        pos = torch.arange(R, dtype=torch.int64) % Lmax
        mask = (pos < ln.repeat_interleave(Lmax)).to(torch.uint8)
    elif layout == "packed":
        R = T
        cu = torch.zeros(B + 1, dtype=torch.int64)
        cu[1:] = torch.cumsum(ln, 0)
        mask = torch.ones(R, dtype=torch.uint8)
    else:
        raise ValueError(layout)
    tdt = torch.float32 if cfg.dtype == "f32" else torch.bfloat16
    hidden = torch.empty((R, H), dtype=tdt, device=dev)
    weight = torch.empty((V, H), dtype=tdt, device=dev)
    _fill_normal(hidden, cfg.seed, _T_HID, 1.0)
    _fill_normal(weight, cfg.seed, _T_W, weight_std)
    ids = randint(cfg.seed, _T_IDS, 0, R, 0, V - 1, dev).to(torch.int32)
    # rewards: Bernoulli(reward_p); optionally a share of the groups made all-equal
    rew = (uniform01(cfg.seed, _T_REW, 0, B, "cpu") < cfg.reward_p).to(torch.float32)
    gidx = torch.arange(B, dtype=torch.int64) // G
    if cfg.equal_group_frac > 0:
        n_eq = int(round(cfg.equal_group_frac * P))
        order = torch.argsort(hash_u64(cfg.seed, _T_EQ, 0, P, "cpu") & _MASK63)
        val = (uniform01(cfg.seed, _T_EQV, 0, P, "cpu") < 0.5).to(torch.float32)
        for p in order[:n_eq].tolist():
            rew[gidx == p] = val[p]
    # closed-form stand-in for the current log-prob (see module docstring)
    approx = torch.empty(R, dtype=torch.float32, device=dev)
    rows_per = max(1, (1 << 24) // H)
    for s in range(0, R, rows_per):
        e = min(R, s + rows_per)
        x = hidden[s:e].to(torch.float32)
        w = weight[ids[s:e].long()].to(torch.float32)
        zy = (x * w).sum(1)
        s2 = (weight_std ** 2) * (x * x).sum(1)
        approx[s:e] = zy / temperature - math.log(V) - 0.5 * s2 / temperature ** 2
    old = approx + noise * normal(cfg.seed, _T_OLD, 0, R, dev)
    ref = approx + noise * normal(cfg.seed, _T_REF, 0, R, dev)
    log_z = normal(cfg.seed, _T_LOGZ, 0, P, "cpu")
    return RolloutBatch(
        cfg=cfg, layout=layout, R=R, T=T, B=B,
        hidden=hidden, weight=weight, token_ids=ids,
        mask=mask.to(dev), cu_seqlens=cu.to(torch.int32).to(dev),
        group_idx=gidx.to(torch.int32).to(dev), rewards=rew.to(dev),
        old_logprob=old, ref_logprob=ref, log_z=log_z.to(dev),
        lengths=ln.to(torch.int32),
    )


# --------------------------------------------------------------------------- residual-VQ encode inputs
_T_RVQ_X, _T_RVQ_CB = 21, 22


def make_rvq_case(G: int, L: int, N: int, S: int, D: int = 128, seed: int = 0x5EED0100, device="cpu",
                  sigma0: float = 0.33, decay: float = 0.945):
    """Seeded stand-in for a KV-cache segment and its residual codebooks (no trained codebooks exist here):
    vectors ~ N(0,1) [G, L, D] and codebook stage i ~ N(0, (sigma0 decay^i)^2) [G, N, S, D], both rounded to bf16 once.
    The stage scales follow the shrinking residual of a greedy search over S random entries (about 10 % of the
    squared norm per stage at S = 1024, D = 128), so every stage has work to do."""
    x = normal(seed, _T_RVQ_X, 0, G * L * D, device).view(G, L, D).to(torch.bfloat16)
    scale = sigma0 * decay ** torch.arange(N, dtype=torch.float32, device=device)
    cb = normal(seed, _T_RVQ_CB, 0, G * N * S * D, device).view(G, N, S, D)
    cb = (cb * scale.view(1, N, 1, 1)).to(torch.bfloat16)
    return x, cb

