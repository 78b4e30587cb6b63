"""Float64 CPU oracle for the residual vector-quantisation encode of the paper (RSimVQ compression of a KV vector).

TEST INFRASTRUCTURE ONLY: imported by the tests (and the benchmark's CPU-baseline leg), never by the product path; it
shares no code with the HIP sources.

What the paper defines (method section, "Learning High-fidelity VQ Codebooks", Eq. 1-2, and the prefill stage,
Eq. 5-8): a vector x is mapped to N integer codes by N residually connected codebooks,

    for i = 1..N:   z_i = argmin_s || x_i - c_{i,s} ||,     x_{i+1} = x_i - c_{i,z_i},     x_1 = x,

each code indexing one of the S entries of codebook i, and it is reconstructed as the sum of the selected entries
(Eq. 3).  The compression ratio of storing N codes of log2 S bits instead of D 16-bit values is Eq. 13.

Readings where the paper is silent or at odds with itself (listed in the design notes as well):
  * the nearest-entry search of Eq. 1 runs over the projected entries W_i q_s while the reconstruction (Eq. 3, 10)
    sums Q_i[z_i] without W: at inference the stored codebook already holds the projected entries; `codebooks` here are
    those effective entries c_{i,s};
  * Eq. 6-7 subtract the index from the vector: the selected entry is meant;
  * ties: the lowest index wins (argmin of a library, first occurrence);
  * the running residual is held in the cache's own 16-bit storage precision between stages (here bf16, round to
    nearest even after the subtraction): the subtraction itself is exact in float64, so given the same codes both
    implementations hold bit-identical residuals;
  * the distance is the squared Euclidean distance evaluated exactly from the stored bf16 values (float64);
  * log in Eq. 13 is base 2 (the only reading that reproduces the two ratios the paper prints).
"""
from __future__ import annotations

import numpy as np

from oracle.policy_oracle import widen


def bf16_round_bits(a) -> np.ndarray:
    """float64/float32 array -> uint16 bf16 bit patterns, round to nearest even (finite inputs)."""
    f = np.asarray(a, dtype=np.float64).astype(np.float32)          # exact here: callers pass differences of bf16 values
    u = f.view(np.uint32).astype(np.uint64)
    u = (u + 0x7FFF + ((u >> 16) & 1)) >> 16
    return u.astype(np.uint16)


def rvq_encode(x_bits, codebook_bits, return_trace=False):
    """x_bits [L, D] bf16 bit patterns, codebook_bits [N, S, D] bf16 bit patterns.
    Returns codes [L, N] int64 and the final residual [L, D] as bf16 bit patterns (uint16);
    with return_trace also the per-stage squared residual norms [L, N+1] (float64)."""
    r_bits = np.asarray(x_bits).astype(np.uint16).copy()
    C = widen(np.asarray(codebook_bits).view(np.int16) if np.asarray(codebook_bits).dtype == np.uint16 else codebook_bits)
    N, S, D = C.shape
    L = r_bits.shape[0]
    codes = np.zeros((L, N), dtype=np.int64)
    trace = np.zeros((L, N + 1))
    for i in range(N):
        r = widen(r_bits.view(np.int16))
        trace[:, i] = (r * r).sum(axis=1)
        # squared distances to every entry, straight from the definition: sum_d (r_d - c_d)^2
        d = np.empty((L, S))
        for s0 in range(0, S, 256):
            blk = C[i, s0:s0 + 256]
            d[:, s0:s0 + 256] = ((r[:, None, :] - blk[None, :, :]) ** 2).sum(axis=2)
        z = d.argmin(axis=1)                                         # first occurrence on ties
        codes[:, i] = z
        r_bits = bf16_round_bits(r - C[i, z])
    r = widen(r_bits.view(np.int16))
    trace[:, N] = (r * r).sum(axis=1)
    return (codes, r_bits, trace) if return_trace else (codes, r_bits)


def rvq_decode(codes, codebook_bits):
    """Reconstruction of Eq. 3: the sum of the selected entries (float64, no intermediate rounding)."""
    C = widen(np.asarray(codebook_bits).view(np.int16) if np.asarray(codebook_bits).dtype == np.uint16 else codebook_bits)
    codes = np.asarray(codes)
    out = np.zeros((codes.shape[0], C.shape[2]))
    for i in range(C.shape[0]):
        out += C[i, codes[:, i]]
    return out


def check_codes_follow_the_definition(x_bits, codebook_bits, codes, rel_tol):
    """Validity of a given code table, decision by decision: walking the residual along the GIVEN codes, every chosen
    entry must be a nearest entry up to rel_tol of the squared distance scale, and exactly the first minimiser when the
    runner-up is further away than that.  Returns (number of decisions that differ from the exact argmin, worst excess)."""
    r_bits = np.asarray(x_bits).astype(np.uint16).copy()
    C = widen(np.asarray(codebook_bits).view(np.int16) if np.asarray(codebook_bits).dtype == np.uint16 else codebook_bits)
    N, S, D = C.shape
    codes = np.asarray(codes).astype(np.int64)
    L = r_bits.shape[0]
    n_diff = 0
    worst = 0.0
    rows = np.arange(L)
    for i in range(N):
        r = widen(r_bits.view(np.int16))
        d = np.empty((L, S))
        for s0 in range(0, S, 256):
            blk = C[i, s0:s0 + 256]
            d[:, s0:s0 + 256] = ((r[:, None, :] - blk[None, :, :]) ** 2).sum(axis=2)
        best = d.argmin(axis=1)
        z = codes[:, i]
        if np.any((z < 0) | (z >= S)):
            raise AssertionError("code out of range")
        excess = d[rows, z] - d[rows, best]
        scale = (r * r).sum(axis=1) + (C[i, best] ** 2).sum(axis=1) + 1e-300
        worst = max(worst, float((excess / scale).max()))
        if np.any(excess > rel_tol * scale):
            raise AssertionError(f"stage {i}: a chosen entry is not a nearest entry (excess/scale {float((excess / scale).max()):.3e})")
        n_diff += int((z != best).sum())
        r_bits = bf16_round_bits(r - C[i, z])
    return n_diff, worst


def compression_ratio(Nk, Sk, Nv, Sv, Dk, Dv):
    """Eq. 13, in percent: 1 - (N^k log2 S^k + N^v log2 S^v) / (16 (D^k + D^v))."""
    return (1.0 - (Nk * np.log2(Sk) + Nv * np.log2(Sv)) / (16.0 * (Dk + Dv))) * 100.0
