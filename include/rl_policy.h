/*
 * rl_policy.h - C ABI of the fused LM-head log-prob + policy-loss library (MI355X / gfx950).
 *
 * What it computes (problem statement of the benchmark contract; the mounted paper has
 * no passage on it): for every response token t of a group of sampled responses,
 *     z_t   = W x_t                      (never stored)
 *     lse_t = log sum_v exp z_t[v],      logp_t = z_t[y_t] - lse_t
 * then the group-relative advantage A_i = (r_i - mean_g)/(std_g + adv_eps) over the G
 * rollouts of a prompt, then one of two objectives
 *     GRPO:  loss = (1/B) sum_i (1/|y_i|) sum_t [ -min(rho_t A_i, clip(rho_t,1-e,1+e) A_i)
 *                                                 + kl_coef (exp(d_t) - d_t - 1) ],
 *            rho_t = exp(logp_t - old_t),  d_t = ref_t - logp_t
 *     FLOW:  loss = (1/B) sum_i w_i delta_i^2,
 *            delta_i = logZ_g(i) + (1/|y_i|) sum_t (logp_t - ref_t) - beta A_i,
 *            w_i = clip(exp(sum_t (logp_t - old_t)), 1-e, 1+e) held constant
 * and the backward pass  c_t = dloss/dlogp_t,  dS[t,v] = c_t (1[v=y_t] - softmax(z_t)[v]),
 * dX = dS W, dW = dS^T X.  T x V is never stored: either the logits are recomputed tile by
 * tile and a chunk of dS in the input precision is staged between the contractions, or the
 * forward keeps a chunk's unnormalised probabilities and the backward is contracted from
 * those (rl_backward_mode).  Optionally the policy is softmax(W x_t / temperature).
 *
 * Conventions
 *  - Every pointer in rl_batch / rl_outputs and the workspace is a DEVICE pointer owned by
 *    the caller; rl_batch / rl_params / rl_outputs structs themselves live on the HOST.
 *  - The library allocates nothing, keeps no pointer after return, and never synchronises:
 *    all work is enqueued on `stream` (a hipStream_t passed as void*; NULL = default
 *    stream); outputs are valid once the stream reaches that point.
 *  - Row-major everywhere.  hidden is [R,H], weight is [V,H] (LM head, no bias); row t of
 *    hidden is the state that predicts token_ids[t] (the caller did the shift).
 *  - Sequence i owns rows [cu_seqlens[i], cu_seqlens[i+1]); cu_seqlens[0]=0, cu_seqlens[B]=R,
 *    non-decreasing.  A row counts iff mask[t] != 0.  Padded layouts simply mask the tail.
 *  - Masked rows: logprob = lse = 0, d_hidden row = 0, no contribution anywhere.
 *  - Host-checkable errors (null pointers, sizes, dtype, objective, clip range, workspace
 *    size) are returned before anything is launched.  Data errors found on the device
 *    (token id outside [0,V), group index outside [0,P), broken cu_seqlens) never
 *    cause an out-of-bounds access: the offending row / sequence is treated as masked /
 *    empty and counted in rl_stats.  A sequence keeps its rows iff 0 <= cu[i] <= cu[i+1] <= R
 *    and cu[i] is not below any earlier offset, so kept ranges never overlap.
 *  - Results are bit-reproducible run to run: no floating-point atomics are used.
 *  - bf16 inputs need H % 8 == 0 (16-byte rows); f32 inputs need H % 4 == 0.
 */
#ifndef RL_POLICY_H
#define RL_POLICY_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum rl_status {
  RL_OK = 0,
  RL_ERR_NULL = 1,        /* a required pointer is NULL                         */
  RL_ERR_SHAPE = 2,       /* a size is non-positive, too large or misaligned    */
  RL_ERR_DTYPE = 3,       /* unknown rl_dtype                                   */
  RL_ERR_RANGE = 4,       /* objective / clip_eps / ddof / backward mode out of range */
  RL_ERR_WORKSPACE = 5,   /* workspace NULL, misaligned or smaller than needed  */
  RL_ERR_HIP = 6,         /* a HIP launch failed (see hipGetLastError)          */
  RL_ERR_UNIMPLEMENTED = 7 /* a valid request this build has no kernel for (RL_BWD_STASH with f32 inputs or H % 128 != 0) */
} rl_status;

typedef enum rl_objective { RL_OBJ_GRPO = 0, RL_OBJ_FLOW = 1 } rl_objective;
typedef enum rl_dtype { RL_F32 = 0, RL_BF16 = 1 } rl_dtype;

/* How the backward pass gets the probabilities of a chunk of rows.
 *  RL_BWD_RECOMPUTE  recompute the logits tile by tile from X and W (four contractions per chunk:
 *                    forward, recompute + dS, dX, dW).  Always available.
 *  RL_BWD_STASH      single pass: chunks are made of whole sequences, the forward contraction also
 *                    stores the chunk's unnormalised probabilities exp(z - ref_t) in the input
 *                    precision (ref_t = target logit - old log-prob, i.e. the row's logsumexp up to
 *                    the drift between old and current policy), and dX / dW are contracted from
 *                    that store (three contractions per chunk, the 6 T H V flops the path needs).
 *                    Needs bf16 inputs, H a multiple of 128 and 16-byte aligned hidden / weight (otherwise
 *                    RL_ERR_UNIMPLEMENTED) and 0 < params->max_seq_len <= chunk rows (otherwise RL_ERR_RANGE).
 *                    old_logprob only steers the reference (clamped to [-40, 0]): the stored probabilities stay
 *                    representable while the current log-prob of the sampled token is above about
 *                    -100 nats.  A row beyond that is counted in rl_stats.n_overflow_rows and the loss of the
 *                    call comes back NaN (its gradient rows are not numbers): the caller re-runs the batch with
 *                    RL_BWD_RECOMPUTE, which has no such limit.
 *  RL_BWD_AUTO       RL_BWD_STASH when its conditions hold, else RL_BWD_RECOMPUTE.
 * Either way at most chunk_rows x V values are held at a time, never T x V. */
typedef enum rl_aggregation { RL_AGG_SEQUENCE = 0, RL_AGG_TOKEN = 1 } rl_aggregation;
typedef enum rl_ratio_level { RL_RATIO_TOKEN = 0, RL_RATIO_SEQUENCE = 1 } rl_ratio_level;
typedef enum rl_weight_norm { RL_WNORM_SUM = 0, RL_WNORM_MEAN = 1 } rl_weight_norm;
typedef enum rl_backward_mode { RL_BWD_AUTO = 0, RL_BWD_RECOMPUTE = 1, RL_BWD_STASH = 2 } rl_backward_mode;

typedef struct rl_batch {
  int64_t R;                    /* rows (tokens incl. masked ones), 1 <= R < 2^31 - 2^16 */
  int32_t H, V, B, P;           /* hidden, vocab, sequences, prompts                     */
  int32_t dtype;                /* rl_dtype of hidden, weight, d_hidden                  */
  int32_t reserved;
  const void*    hidden;        /* [R,H]                                                 */
  const void*    weight;        /* [V,H]                                                 */
  const int32_t* token_ids;     /* [R]   sampled token y_t in [0,V)                      */
  const uint8_t* mask;          /* [R]   1 = response token                              */
  const int32_t* cu_seqlens;    /* [B+1]                                                 */
  const int32_t* group_idx;     /* [B]   prompt index g(i) in [0,P)   (loss call only)   */
  const float*   rewards;       /* [B]                                (loss call only)   */
  const float*   old_logprob;   /* [R]   log-prob under the sampling policy  (loss only) */
  const float*   ref_logprob;   /* [R]   log-prob under the reference policy (loss only) */
  const float*   log_z;         /* [P]   per-prompt log partition; FLOW only, else NULL  */
} rl_batch;

typedef struct rl_params {
  float   clip_eps;             /* in (0,1)                                              */
  float   kl_coef;              /* GRPO only                                             */
  float   beta;                 /* FLOW only: reward scale                               */
  float   adv_eps;              /* added to the group std                                */
  int32_t adv_std_ddof;         /* 0 (population std) or 1                               */
  int32_t chunk_rows;           /* rows staged at once; 0 = library default (rl_default_chunk_rows / _single_pass) */
                                /* rounded up to a multiple of 256; sizes the workspace  */
  float   clip_eps_high;        /* upper bound of the ratio / weight is 1 + clip_eps_high; 0 = clip_eps (symmetric) */
  int32_t aggregation;          /* GRPO: RL_AGG_SEQUENCE (mean over sequences of the token mean) or         */
                                /* RL_AGG_TOKEN (mean over all counting tokens of the batch; seq_loss[i]    */
                                /* is then (B/T) sum_t l_t, so loss = mean_i seq_loss_i still holds)        */
  int32_t ratio_level;          /* GRPO: RL_RATIO_TOKEN, or RL_RATIO_SEQUENCE = one ratio per sequence,     */
                                /* exp(mean_t(logp_t - old_t)), clipped as a whole (sequence aggregation)   */
  int32_t flow_weight_norm;     /* FLOW: weight from the RL_WNORM_SUM or RL_WNORM_MEAN of token log-ratios  */
  int32_t backward_mode;        /* rl_backward_mode; 0 = RL_BWD_AUTO                     */
  int32_t max_seq_len;          /* promise: no sequence has more counting rows than this; */
                                /* 0 = no promise.  Needed by the single-pass backward.   */
  float   temperature;          /* the policy is softmax(W x_t / temperature): logprob, lse, entropy refer to the */
                                /* tempered logits and d_hidden / d_weight carry the 1/temperature chain factor;  */
                                /* 0 = 1.0 (logits used as they are); otherwise finite and > 0                    */
} rl_params;

typedef struct rl_stats {       /* device struct written by the loss call                */
  int32_t n_tokens;             /* number of rows that counted (T)                       */
  int32_t n_clip_hi;            /* GRPO: tokens with A>0, rho>1+e; FLOW: sequences with the weight on the upper bound */
  int32_t n_clip_lo;            /* GRPO: tokens with A<0, rho<1-e; FLOW: ... lower bound */
  int32_t n_bad_token;          /* mask=1 rows dropped because token id was out of range */
  int32_t n_bad_group;          /* sequences dropped because group_idx was out of range  */
  int32_t n_bad_seq;            /* sequences treated as empty (cu_seqlens decreasing / out of [0,R]) */
  int32_t n_seq_too_long;       /* sequences longer than params->max_seq_len (single-pass backward): loss is then NaN */
  int32_t n_overflow_rows;      /* single-pass backward: rows whose stored probabilities left the representable range  */
                                /* (sum outside [1e-30, 1e30] or not a number): loss is then NaN                       */
} rl_stats;

typedef struct rl_outputs {     /* NULL = not wanted, except loss                        */
  float*    loss;               /* [1]                                                   */
  float*    seq_loss;           /* [B]                                                   */
  float*    logprob;            /* [R]                                                   */
  float*    lse;                /* [R]                                                   */
  float*    advantages;         /* [B]                                                   */
  int32_t*  seq_len;            /* [B]   |y_i|                                           */
  float*    coeff;              /* [R]   c_t = dloss/dlogp_t                             */
  void*     d_hidden;           /* [R,H] input dtype; d_hidden and d_weight NULL together skips the backward */
  float*    d_weight;           /* [V,H] f32, overwritten                                */
  float*    d_log_z;            /* [P]   zero for GRPO                                   */
  rl_stats* stats;              /* [1]                                                   */
  float*    entropy;            /* [R]   entropy of softmax(W x_t), from the forward pass' online sums */
  /* Index work of the path, for callers that want to check it bit for bit: */
  int32_t*  row_map;            /* [R]   entry k < T: original row of the k-th counting row (sequence by sequence, rows  */
                                /*       ascending); entries T..R-1 are -1                                               */
  int32_t*  group_count;        /* [P]   sequences naming each prompt                                                    */
  int32_t*  target_col;         /* [R]   vocabulary entry the target logit of the row was read from (the accumulator's   */
                                /*       own position in the logits tile, or the row of W in single-pass mode): equals   */
                                /*       token_ids on counting rows, -1 elsewhere                                        */
  float*    target_logit;       /* [R]   z_t[y_t] (tempered), 0 on rows that do not count                                */
} rl_outputs;

/* Bytes of device workspace the two calls below need for this batch shape (host only; reads
 * R, H, V, B, P, dtype, the alignment of hidden / weight, and params->chunk_rows, backward_mode,
 * max_seq_len; params may be NULL = defaults; want_backward
 * = 0 sizes it for rl_token_logprob / loss-only calls).  The workspace must be 256-byte
 * aligned.  Its contents on entry are irrelevant and on return unspecified. */
rl_status rl_workspace_bytes(const rl_batch* batch, const rl_params* params,
                             int32_t want_backward, size_t* bytes);

/* Forward only: logprob[R] and lse[R] (either may be NULL, not both) for the rows with
 * mask != 0; reads hidden, weight, token_ids, mask, cu_seqlens (B may be 1 with
 * cu_seqlens = {0,R}).  Used to score rollouts under the old / reference policies. */
rl_status rl_token_logprob(const rl_batch* batch, float* logprob, float* lse,
                           void* workspace, size_t workspace_bytes, void* stream);

/* The same under softmax(W x_t / temperature), temperature finite and > 0 (else RL_ERR_RANGE): the
 * scoring call that matches rl_params.temperature of the loss call.  Same workspace size. */
rl_status rl_token_logprob_tempered(const rl_batch* batch, float temperature, float* logprob, float* lse,
                                    void* workspace, size_t workspace_bytes, void* stream);

/* For callers that cannot allocate or hand over a workspace (code under HIP graph capture, tight serving loops,
 * harnesses that forbid hipMalloc): rl_token_logprob_tempered with its workspace in a static device array of
 * RL_STATIC_SCRATCH_BYTES that every GPU the library runs on holds until the process ends.  The call itself allocates
 * nothing (no hipMalloc / hipFree, no allocating library routine) and clears what it needs itself; the caller still
 * passes inputs and outputs.  The chunk size is chosen so that the plan fits the array; a batch whose plan does not
 * fit even with 256-row chunks (about 32 bytes per row plus 16 bytes x ceil(V / 256) x 256) is rejected with
 * RL_ERR_WORKSPACE before anything is launched.  All calls on one GPU share that GPU's array: calls that overlap on one
 * GPU (two streams, two threads) race; serialise them.  The first call on a device looks the array's address up
 * (not capturable: make one call before capturing a graph).  Results are bit-identical to rl_token_logprob_tempered. */
#define RL_STATIC_SCRATCH_BYTES (32u << 20)
rl_status rl_token_logprob_static(const rl_batch* batch, float temperature, float* logprob, float* lse, void* stream);

/* The whole path: log-prob, per-sequence length-normalised sums, group advantage, loss and
 * per-token coefficient, and (if d_hidden and d_weight are given) the backward pass. */
rl_status rl_policy_loss_fwd_bwd(const rl_batch* batch, const rl_params* params,
                                 int32_t objective, const rl_outputs* outputs,
                                 void* workspace, size_t workspace_bytes, void* stream);

const char* rl_status_string(int32_t status);

/* Library version (major*100 + minor) and the chunk sizes used when chunk_rows = 0 (recompute mode; single-pass mode). */
int32_t rl_version(void);
int32_t rl_default_chunk_rows(void);
int32_t rl_default_chunk_rows_single_pass(void);

/* The log-Z head: the step that produces rl_batch.log_z for the flow-balance objective (the problem
 * statement takes "per-prompt log Z" as given; reading: a two-layer MLP over the mean of the prompt's
 * hidden states, log_z[p] = w2 . gelu(W1 mean_t(h_t) + b1) + b2 with the exact (erf) GELU; the hidden
 * states are constants).  All pointers are device pointers.
 *   prompt_hidden [rows, H] in `dtype` (rl_dtype), row-major; prompt p owns rows [cu_prompt[p], cu_prompt[p+1])
 *                 (cu_prompt: P+1 int32; an empty prompt pools to zero; ranges are clamped to [0, rows]);
 *   W1 [M, H] f32 row-major, b1 [M], w2 [M], b2 [1] f32 (M at most 524280);
 *   log_z [P] f32, overwritten.
 * The workspace (rl_logz_head_workspace_bytes, 256-byte aligned, caller-owned) keeps the pooled states and
 * the hidden-layer activations between the two calls: rl_logz_head_backward must be given the workspace of
 * the matching forward call, unmodified.  Backward: from d_log_z [P] (rl_outputs.d_log_z) it overwrites
 * dW1 [M, H], db1 [M], dw2 [M], db2 [1] (f32).  Neither call allocates or synchronises; both enqueue on
 * `stream`.  Errors as for the other entry points (RL_ERR_NULL / SHAPE / DTYPE / WORKSPACE / HIP). */
rl_status rl_logz_head_workspace_bytes(int32_t P, int32_t H, int32_t M, size_t* bytes);
rl_status rl_logz_head_forward(const void* prompt_hidden, int32_t dtype, int64_t rows, int32_t H,
                               const int32_t* cu_prompt, int32_t P, const float* W1, const float* b1,
                               const float* w2, const float* b2, int32_t M, float* log_z,
                               void* workspace, size_t workspace_bytes, void* stream);
rl_status rl_logz_head_backward(const float* d_log_z, int32_t P, int32_t H, int32_t M, const float* w2,
                                float* dW1, float* db1, float* dw2, float* db2,
                                void* workspace, size_t workspace_bytes, void* stream);

/* Residual vector-quantisation encode of KV-cache vectors: the compression step of the paper (method section,
 * "Learning High-fidelity VQ Codebooks", Eq. 1-2, and the prefill stage, Eq. 5-8).  For each of G independent
 * codebook groups (one per layer / head / cache type) and each of its L vectors x (D = 128 values, bf16):
 *     for i = 0..N-1:   codes[i] = argmin_s || r - c[i][s] ||^2  (lowest index on ties),   r <- bf16(r - c[i][codes[i]]),
 * starting from r = x, where c[i][s] are the effective entries of codebook i (the paper's W_i q_s, stored already
 * projected) and the running residual is kept in the 16-bit storage precision between stages.  The arg-min is the one
 * exact arithmetic gives on the stored values: scores are computed in float32 on the matrix cores, and every decision
 * whose lead is within the rounding bound of those scores is settled from the bf16 values in float64.
 *   vectors   [G][L][D] bf16, 16-byte aligned;       codebooks [G][N][S][D] bf16, 16-byte aligned;
 *   norms     [G][N][S] f32: squared norms of the entries, as written by rl_rvq_codebook_norms (once per codebook set);
 *   codes     [G][L][N] int32, overwritten (each in [0, S));
 *   residual  [G][L][D] bf16 or NULL: what is left of each vector after the N stages.
 * D must be 128 and S a multiple of 64, at most 65536 (else RL_ERR_SHAPE).  All pointers are device pointers; the calls allocate
 * nothing, do not synchronise, and enqueue on `stream`. */
rl_status rl_rvq_codebook_norms(const void* codebooks, int32_t G, int32_t N, int32_t S, int32_t D, float* norms, void* stream);
rl_status rl_rvq_encode(const void* vectors, const void* codebooks, const float* norms, int32_t G, int64_t L, int32_t D,
                        int32_t N, int32_t S, int32_t* codes, void* residual, void* stream);

#ifdef __cplusplus
}
#endif
#endif /* RL_POLICY_H */
