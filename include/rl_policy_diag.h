/*
 * rl_policy_diag.h - benchmark and diagnostic aids of the fused LM-head log-prob + policy-loss library.
 *
 * NOT part of the product surface declared in rl_policy.h, whose calls allocate nothing and never
 * synchronise.  The calls below are for benchmarks and tests only and are the exceptions to those rules:
 * rl_profile_* creates (and keeps) HIP events, rl_profile_read and rl_measure_mfma_peak wait for the
 * stream, rl_measure_mfma_peak copies two words back to the host.  None of them is thread-safe.
 * No passage of the paper defines them; they exist so that the roofline figures of the benchmark are
 * measured inside the library, on the stream its kernels run on.
 */
#ifndef RL_POLICY_DIAG_H
#define RL_POLICY_DIAG_H

#include "rl_policy.h"

#ifdef __cplusplus
extern "C" {
#endif

/* Optional timing of the library's own launches, for benchmarks (not thread-safe; the only
 * place the library creates objects of its own: HIP events, kept for reuse).  While enabled,
 * every group of launches of rl_token_logprob / rl_policy_loss_fwd_bwd is bracketed by a pair of events recorded on
 * the caller's stream.  rl_profile_read waits for the recorded events, adds up elapsed
 * milliseconds and bracket counts per class since the previous read, and clears the list. */
enum { RL_PROF_PREP = 0,       /* counts, scan, compaction, output zero-fill            */
       RL_PROF_GEMM_FWD = 1,   /* forward logits contraction + online partial softmax   */
       RL_PROF_COMBINE = 2,    /* partials -> lse, logp                                 */
       RL_PROF_LOSS = 3,       /* advantage, per-sequence loss, final reduce            */
       RL_PROF_TRANSPOSE = 4,  /* W^T, X^T chunks, zeroing masked dX rows               */
       RL_PROF_GEMM_DS = 5,    /* recomputed logits -> dS                               */
       RL_PROF_GEMM_DX = 6,    /* dX = dS W                                             */
       RL_PROF_GEMM_DW = 7,    /* dW += dS^T X                                          */
       RL_PROF_GEMM_BWD = 8,   /* single-pass backward: dX and dW of a chunk in one launch */
       RL_PROF_CLASSES = 9 };
typedef struct rl_profile {     /* host struct */
  double  ms[RL_PROF_CLASSES];
  int64_t launches[RL_PROF_CLASSES];
} rl_profile;
void rl_profile_enable(int32_t on);
rl_status rl_profile_read(rl_profile* out);

/* Benchmark aid: runs a pure bf16 MFMA issue loop (v_mfma_f32_16x16x32_bf16 in the hot kernel's 8 x 8 register
 * blocking, pseudo-random operands, four wavefronts per CU, no memory traffic) for about `millis` ms on
 * `stream`, SYNCHRONISES on it, and returns the rate it reached and the shader clock it ran at.  This is
 * the ceiling any MFMA-bound kernel can approach on this part at this moment (clock throttling included).
 * scratch: device buffer of at least 1 MiB owned by the caller. */
rl_status rl_measure_mfma_peak(int32_t millis, void* scratch, size_t scratch_bytes, void* stream,
                               double* tflops, double* shader_mhz);

/* Diagnostic (host only, nothing is launched): the workgroup -> tile map of the contraction kernels, for tests.
 * tiles_m x tiles_n tiles, bands of group_m M-tiles, by_share = 0 (eight equal runs of the band sequence) or 1
 * (each of the eight accelerator dies owns a share of the M-tiles).  *workgroups receives the launch size;
 * tile[2 w] / tile[2 w + 1] (caller's array of 2 * launch size ints, or NULL to query the size only) receive
 * the (m, n) tile of workgroup w, or (-1, -1) if it has none. */
rl_status rl_debug_tile_order(int32_t tiles_m, int32_t tiles_n, int32_t group_m, int32_t by_share,
                              int32_t* workgroups, int32_t* tile);

/* rl_rvq_encode that also counts, in the device word *n_exact (added to, not cleared; may be NULL), the decisions whose
 * float32 lead was within the rounding margin and that were therefore settled in float64 among the entries that came
 * within that margin (counted once per decision; the last workgroup of a group counts its padding lanes too).
 * For tests of that path and for its cost in profiles. */
rl_status rl_rvq_encode_counted(const void* vectors, const void* codebooks, const float* norms, int32_t G, int64_t L, int32_t D,
                                int32_t N, int32_t S, int32_t* codes, void* residual, int32_t* n_exact, void* stream);

#ifdef __cplusplus
}
#endif
#endif /* RL_POLICY_DIAG_H */
