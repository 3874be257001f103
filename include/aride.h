/*
 * aride.h -- C ABI of the MI355X (gfx950) scoring pass of A-RIDE, the learner-side
 * algorithm of DistRL (arXiv 2410.14803): policy logits -> per-action log-probability
 * and entropy -> Retrace(lambda) targets -> replay priorities -> prioritized
 * sampling / priority update.
 *
 * Conventions shared by every entry point
 *  - Every pointer is a DEVICE pointer unless its comment says "host".
 *  - The caller owns every buffer.  The library never allocates, frees or
 *    synchronises (aride_status_read is the one documented exception: it copies a
 *    few words to the host and waits for the stream).
 *  - All work is enqueued on `stream` (a hipStream_t passed as void*; NULL is the
 *    default stream) and is asynchronous with respect to the host.
 *  - Return value: ARIDE_OK or a negative ARIDE_E_* code.  Argument errors are
 *    detected on the host before anything is launched; nothing is enqueued then.
 *  - Conditions only the device can see (a token outside the vocabulary, a weight that
 *    is NaN/negative/infinite, a replay buffer with no mass, an index outside the
 *    buffer) set a bit in the status word of the workspace; read it with
 *    aride_status_read after the work has finished.
 *  - Shapes: B trajectories, N steps flattened trajectory after trajectory with CSR
 *    offsets traj_offsets[B+1] (traj_offsets[0] = 0, traj_offsets[B] = N), A action
 *    tokens per step, R = N*A logit rows, vocabulary V, replay capacity M, batch K.
 *  - Output pointers documented "nullable" may be NULL; that output is then skipped.
 *  - Calls that share a workspace must be ordered on one stream (or otherwise
 *    serialised); concurrent calls on one workspace race.
 */
#ifndef ARIDE_H
#define ARIDE_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

#define ARIDE_OK            0
#define ARIDE_E_NULL       -1   /* a required pointer is NULL */
#define ARIDE_E_SHAPE      -2   /* negative size, R not a multiple of A, stride < V, ... */
#define ARIDE_E_ALIGN      -3   /* a pointer or stride violates the stated alignment */
#define ARIDE_E_RANGE      -4   /* a scalar or size is outside the supported range */
#define ARIDE_E_ZERO_MASS  -5   /* reported by aride_status_read: the buffer has no mass */
#define ARIDE_E_WORKSPACE  -6   /* workspace NULL, misaligned or smaller than required */
#define ARIDE_E_HIP        -7   /* a HIP runtime call failed (launch, copy) */

/* Bits of the workspace status word (aride_status_read). */
#define ARIDE_ST_BAD_TOKEN   0x1u  /* a token >= V was seen; that row was masked */
#define ARIDE_ST_BAD_WEIGHT  0x2u  /* a NaN/negative/infinite weight was read as 0 */
#define ARIDE_ST_ZERO_MASS   0x4u  /* rebuild found Total == 0 */
#define ARIDE_ST_BAD_INDEX   0x8u  /* update_priorities skipped an index outside [0,M) */
#define ARIDE_ST_BAD_UNIFORM 0x10u /* a uniform < 0 or NaN was read as 0 */

#define ARIDE_MAX_REPLAY (1 << 24) /* largest M: keeps the integer CDF below 2^63 */
#define ARIDE_MAX_ROWS 8589934528LL       /* largest R of the logit sweeps: 2^33 - 64 (more rows than one launch covers go out as several) */
#define ARIDE_MAX_STEPS 2147475455LL      /* largest N of the scan calls: 2^31 - 1 - 8192 (a chunk of steps past N still indexes as int32) */
#define ARIDE_MAX_TRAJECTORIES 33554431LL /* largest B of the scan calls: 2^25 - 1 */

#define ARIDE_TRACE_RETRACE 0  /* Section 5.2: c_i = lambda * min(1, rho_i), product from i = t+1 */
#define ARIDE_TRACE_VTRACE  1  /* the V-trace targets the paper contrasts Retrace with */

typedef struct {
    float gamma;   /* discount */
    float lambda;  /* trace decay, in [0,1] */
    int32_t mode;  /* ARIDE_TRACE_RETRACE (the paper's method) or ARIDE_TRACE_VTRACE */
    float rho_bar; /* V-trace only: clip of the ratio that weights the TD error */
    float c_bar;   /* V-trace only: clip of the ratio in the trace coefficient */
} aride_retrace_cfg;

typedef struct {
    float w_td, w_rho, w_ent;  /* w1, w2, w3 of Section 5.3 */
    float td_scale, ent_scale; /* normalisers of Appendix A.4.3 (max |delta|, max H); nonzero */
    float eps;                 /* additive floor, 0 for the paper's formula */
    int32_t truncate_rho;      /* nonzero: use min(1, rho) (the appendix's [0,1] range) */
} aride_prio_cfg;

typedef struct {
    float beta;        /* entropy weight of eq. (1) */
    float lambda_pen;  /* weight of the invalid-action penalty of eq. (1) */
    float scale;       /* multiplies loss and gradient; 1/N for the batch mean */
    int32_t grad_f32;  /* 0: gradient stored as bf16 (round to nearest even); nonzero: fp32 */
} aride_actor_cfg;

typedef struct {
    uint32_t flags;     /* OR of ARIDE_ST_* since the last aride_workspace_init */
    uint32_t reserved;
    uint64_t total;     /* integer mass of the replay CDF after the last rebuild */
    float wmax;         /* largest valid weight seen by the last rebuild */
    int32_t exponent;   /* e = ilogb(wmax) + 1 used by the quantisation */
} aride_status;

/*
 * Bytes of device workspace needed for a replay buffer of capacity M (pass M = 0 when
 * only the scoring calls are used: the workspace then holds just the status block).
 * With a replay index it is about 190 KB plus 0.53 * M bytes (an integer sum per 16 weights
 * and per 256 weights): 8.6 MB beside the 64 MB of weights at M = 2^24.
 * Host-only; *out_bytes is a host pointer.  The workspace must be 256-byte aligned.
 */
int aride_workspace_bytes(int64_t M, size_t* out_bytes);

/* Zeroes the whole workspace (status word, replay index).  Must run once before first use. */
int aride_workspace_init(void* ws, size_t ws_bytes, void* stream);

/*
 * Copies the status block to host memory `out` and waits for `stream`.  Returns
 * ARIDE_E_ZERO_MASS when the index as last rebuilt has no mass (total == 0), else ARIDE_OK.
 * The bits of `flags` are sticky: they accumulate until aride_workspace_init.
 */
int aride_status_read(const void* ws, aride_status* out /* host */, void* stream);

/*
 * score_logits -- Section 5.1, eq. (1): log pi(a_t|s_t) and the entropy regulariser
 * H(pi(.|s_t)) of a token-level policy.  For every row r of logits (one vocabulary
 * distribution per action token):
 *     logp_v   = x_v - log sum_u exp(x_u)
 *     tok_logp = logp_{tokens[r]},   tok_ent = - sum_v exp(logp_v) logp_v
 * and per step n the sums over its A rows: step_logp[n] = log pi(a_n|s_n) (the
 * numerator of the ratio rho of Section 5.1), step_ent[n] = entropy along the realised
 * token path.  Each logit is read from memory exactly once; accumulation is fp32 per row
 * (fp64 for the A-term per-step sums, rounded once).
 *
 *  logits  bf16 [R, row_stride] row-major, device; the first V columns of a row are
 *          used.  Base pointer 16-byte aligned; row_stride >= V.  Rows whose byte
 *          offset is not 16-byte aligned are handled (slower head/tail path).
 *  tokens  int32 [R]; a negative token marks a padding row (contributes 0 to every
 *          output); a token >= V is masked the same way and sets ARIDE_ST_BAD_TOKEN.
 *  tok_logp, tok_ent   fp32 [R], nullable -- except that step_logp needs tok_logp and
 *                      step_ent needs tok_ent: the per-step sums are formed from them by a
 *                      second, small kernel (fp64 running sums, rounded to fp32 once).
 *  step_logp, step_ent fp32 [R/A], nullable.
 *  ws      workspace (only its status word is used).
 * Errors: E_NULL (logits/tokens, or a per-step output without its per-token array), E_SHAPE
 *         (R<0, V<=0, A<=0, R%A!=0, stride<V),
 *         E_ALIGN, E_RANGE (V > 2^31-1, R > ARIDE_MAX_ROWS, R/A > 2^25-1), E_WORKSPACE.  R == 0 is a no-op.
 */
int aride_score_logits(const void* logits_bf16, int64_t R, int64_t V, int64_t row_stride,
                       const int32_t* tokens, int32_t A,
                       float* tok_logp, float* tok_ent, float* step_logp, float* step_ent,
                       void* ws, size_t ws_bytes, void* stream);

/*
 * score_logits_timed -- a measurement aid, the same call as aride_score_logits with two HIP
 * events (hipEvent_t, created by the caller with timing enabled) attached to the dispatch of
 * the row-sweep kernel itself: once the stream has drained, hipEventElapsedTime(sweep_start,
 * sweep_stop) is that kernel's execution time, without the marker packets that recording
 * events around the call would put on the stream.  Both events are required (E_NULL); when
 * R == 0 nothing is launched and the events are left as they were.
 */
int aride_score_logits_timed(const void* logits_bf16, int64_t R, int64_t V, int64_t row_stride,
                             const int32_t* tokens, int32_t A, float* tok_logp, float* tok_ent,
                             float* step_logp, float* step_ent, void* ws, size_t ws_bytes,
                             void* stream, void* sweep_start /* hipEvent_t */,
                             void* sweep_stop /* hipEvent_t */);

/*
 * retrace_targets -- Section 5.2 (Retrace(lambda) applied to the value estimate) with
 * the TD error of Section 5.3 / Appendix A.4.2.  Per trajectory, for t = T-1 .. 0:
 *     rho_t   = exp(logp_pi[t] - logp_mu[t])
 *     delta_t = reward[t] + gamma * V_next(t) - Q_t      V_next = value[t+1], or boot[b]
 *                                                        past the trajectory's last step
 *     Delta_t = delta_t + gamma * lambda * min(1, rho_{t+1}) * Delta_{t+1}   (Delta_T = 0)
 *     target[t] = Q_t + Delta_t,  td[t] = delta_t,  rho[t] = rho_t
 * which is the closed form  Delta_t = sum_k gamma^(k-t) (prod_{i=t+1..k} c_i) delta_k,
 * c_i = lambda min(1, rho_i).  Q == value when q is NULL (the paper's form).  The
 * corrected advantage of Section 5.1 is target - Q.
 *
 * With cfg.mode = ARIDE_TRACE_VTRACE the same scan produces the V-trace targets (Section 2 and
 * Appendix A.4.1 name them as the alternative A-RIDE is set against):
 *     Delta_t = min(rho_bar, rho_t) delta_t + gamma * lambda * min(c_bar, rho_t) * Delta_{t+1}
 * i.e. the step's own ratio weights its TD error and its own trace coefficient; td and rho are
 * unchanged.
 *
 *  logp_pi, logp_mu, reward, value  fp32 [N];  q fp32 [N] nullable;  boot fp32 [B]
 *  nullable (0);  traj_offsets int32 [B+1] non-decreasing;  target, td, rho fp32 [N]
 *  nullable.  Empty trajectories are allowed.
 * Errors: E_NULL, E_SHAPE (B<0, N<0), E_RANGE (N > ARIDE_MAX_STEPS, B > ARIDE_MAX_TRAJECTORIES, unknown mode).
 *         B == 0 is a no-op.
 */
int aride_retrace_targets(const float* logp_pi, const float* logp_mu, const float* reward,
                          const float* value, const float* q, const float* boot,
                          const int32_t* traj_offsets, int64_t B, int64_t N,
                          aride_retrace_cfg cfg, float* target, float* td, float* rho,
                          void* stream);

/*
 * mc_returns -- Section 5.1 (state-value function estimation): the Monte-Carlo return
 *     ret[t] = sum_{k >= t, same trajectory} gamma^(k-t) reward[k]
 * and the classification label the value network is trained on, label[t] = 1 if ret[t] > 0
 * else 0.  Same reverse affine scan as retrace_targets (map X -> reward[t] + gamma X).
 *
 *  reward fp32 [N]; traj_offsets int32 [B+1]; ret, label fp32 [N], each nullable.
 * Errors: E_NULL, E_SHAPE, E_RANGE.  B == 0 is a no-op.
 */
int aride_mc_returns(const float* reward, const int32_t* traj_offsets, int64_t B, int64_t N,
                     float gamma, float* ret, float* label, void* stream);

/*
 * compute_priorities -- Section 5.3 (DPER) with Appendix A.4.3's normalisation:
 *     step_prio[t] = w_td*|td[t]|/td_scale + w_rho*rho~[t] + w_ent*ent[t]/ent_scale + eps
 *     traj_prio[b] = mean of step_prio over trajectory b  (= w1*mean|delta| + w2*mean rho
 *                    + w3*mean H, the paper's p(tau)); 0 for an empty trajectory
 * rho~ = min(1, rho) when cfg.truncate_rho, else rho.  `ent` is whichever entropy the
 * caller uses: step_ent from aride_score_logits (Shannon entropy, eq. (1)) or the
 * negated step_logp (the surprisal printed in Section 5.3).
 *
 *  td, rho, ent fp32 [N]; traj_offsets int32 [B+1]; step_prio fp32 [N] nullable;
 *  traj_prio fp32 [B] nullable.
 * Errors: E_NULL, E_SHAPE, E_RANGE (td_scale or ent_scale == 0, N or B as above).
 */
int aride_compute_priorities(const float* td, const float* rho, const float* ent,
                             const int32_t* traj_offsets, int64_t B, int64_t N,
                             aride_prio_cfg cfg, float* step_prio, float* traj_prio,
                             void* stream);

/*
 * retrace_priorities -- aride_retrace_targets and aride_compute_priorities (Sections 5.2 and
 * 5.3) in one pass over the trajectories: the TD error and the ratio of a step go into its
 * priority while the scan still holds them, so they are not read back (36 bytes of traffic per
 * step instead of 48) and the two steps cost one launch.  target, td, rho and step_prio are
 * exactly what the two calls give one after the other; traj_prio is the same mean summed in
 * another order (fp32, fixed order, so repeated calls agree bit for bit).
 *
 *  Arguments as in the two calls; ent fp32 [N] is compute_priorities' entropy input.  All five
 *  outputs are nullable.
 * Errors: those of the two calls.  B == 0 is a no-op.
 */
int aride_retrace_priorities(const float* logp_pi, const float* logp_mu, const float* reward,
                             const float* value, const float* q, const float* boot, const float* ent,
                             const int32_t* traj_offsets, int64_t B, int64_t N,
                             aride_retrace_cfg cfg, aride_prio_cfg pcfg, float* target, float* td,
                             float* rho, float* step_prio, float* traj_prio, void* stream);

/*
 * update_priorities -- Section 5.3, last sentence (priorities are recomputed under the
 * latest policy and overwritten) and Appendix A.4.2 (the buffer stores p^alpha):
 *     for k = 0..K-1 in order:  weights[idx[k]] = (float) pow(max(prio[k], 0), alpha)
 * so a repeated index keeps its LAST occurrence; NaN priorities store 0; indices
 * outside [0, M) are skipped and set ARIDE_ST_BAD_INDEX.  The sampling index in the
 * workspace (integer sums of the quantised weights per 16 and per 256 weights, and the
 * prefixes of the latter) is then rebuilt from the whole buffer.  K == 0 rebuilds only: call it that way after
 * writing `weights` directly.
 *
 *  weights fp32 [M] in/out, 16-byte aligned, 1 <= M <= ARIDE_MAX_REPLAY;
 *  idx int64 [K]; prio fp32 [K]; alpha >= 0.
 * Errors: E_NULL, E_SHAPE, E_ALIGN, E_RANGE (M, K >= 2^23, alpha < 0 or NaN), E_WORKSPACE.
 */
int aride_update_priorities(float* weights, int64_t M, const int64_t* idx, const float* prio,
                            int64_t K, float alpha, void* ws, size_t ws_bytes, void* stream);

/*
 * replay_insert -- Appendix A.4.2 (circular replay buffer of fixed capacity M): append K new
 * entries; entry k is written at slot (cursor + k) mod M, overwriting the oldest entries, and
 * the buffer index advances as i <- (i + 1) mod M per entry.  The stored value is the entry's
 * sampling weight pow(max(prio[k], 0), alpha); the entry's payload belongs in the caller's own
 * arrays at the same slot, reported through slots_out.  When K > M only the last M entries
 * survive and the earlier ones report slot -1.  The sampling index is current afterwards, as
 * after aride_update_priorities with K = 0: on large buffers (M > 63 * 65536, K <= M/8) only the
 * blocks the new entries fall into are summed again, which requires that the index in the
 * workspace was current for these weights before the call (a workspace that never held one is
 * recognised and built in full); otherwise the index is rebuilt.
 *
 *  weights fp32 [M] in/out (16-byte aligned); cursor in [0, M); prio fp32 [K];
 *  slots_out int64 [K] nullable; cursor_out host pointer, nullable: receives (cursor + K) mod M.
 * Errors: E_NULL, E_SHAPE, E_ALIGN, E_RANGE (cursor outside [0,M), alpha < 0, K > 2^31 - 256), E_WORKSPACE.
 */
int aride_replay_insert(float* weights, int64_t M, int64_t cursor, const float* prio, int64_t K,
                        float alpha, int64_t* slots_out, void* ws, size_t ws_bytes,
                        int64_t* cursor_out /* host */, void* stream);

/*
 * sample_prioritized -- Appendix A.4.2: draw index i with probability
 * P(i) = w_i / sum_j w_j  (w = p^alpha), realised on exact integers so the result is a
 * function of the stored weight bits and the uniform alone:
 *     e = ilogb(max_i w_i) + 1;  q_i = floor(w_i * 2^(39-e));  C_i = q_0 + .. + q_i
 *     t_k = min(floor(u_k * (double)Total), Total-1);  idx_out[k] = min{ i : C_i > t_k }
 *     prob_out[k] = (float)(q_idx / Total)
 * NaN/negative/infinite weights carry no mass.  Zero-weight entries are never drawn.
 * Sampling is with replacement; u < 0 or NaN is read as 0 (ARIDE_ST_BAD_UNIFORM).
 * Requires the index left by the last aride_update_priorities or aride_replay_insert on the same
 * `weights` and workspace (only the status word of the workspace is written).  If the
 * buffer has no mass every idx_out[k] = -1.
 *
 *  weights fp32 [M] (16-byte aligned); uniforms fp64 [K] in [0,1); idx_out int64 [K];
 *  prob_out fp32 [K] nullable.
 * Errors: E_NULL, E_SHAPE, E_ALIGN, E_RANGE, E_WORKSPACE.  K == 0 is a no-op.
 */
int aride_sample_prioritized(const float* weights, int64_t M, void* ws, size_t ws_bytes,
                             const double* uniforms, int64_t K, int64_t* idx_out,
                             float* prob_out, void* stream);

/*
 * sample_prioritized_static -- aride_sample_prioritized for callers that cannot allocate device
 * memory and so have no workspace to pass: code under HIP graph capture, tight serving loops,
 * harnesses that forbid hipMalloc.  The sampling index is built and read in a fixed array that is
 * part of the library's device code (ARIDE_STATIC_MAX_REPLAY sizes it: about 0.75 MB, held on
 * every GPU the library runs on until the process ends), so the call needs only the inputs and
 * outputs.  It allocates and frees nothing, and it does not synchronise.
 *
 * One call = the index of `weights` built as aride_update_priorities with K = 0 builds it (no
 * weight is written), then the draws of aride_sample_prioritized: idx_out and prob_out are
 * exactly what those two calls give with a workspace of the caller's.  The status block starts
 * from zero on every call; status_out, when given, receives it (flags, total, wmax, exponent of
 * this call alone).  A buffer with no mass gives idx_out[k] = -1 and ARIDE_ST_ZERO_MASS.
 *
 * Every call on a GPU uses that GPU's one array: calls that overlap on one GPU (two streams, two
 * threads) race and must be serialised by the caller.  The array's address is looked up on the
 * first call on each device (hipGetSymbolAddress, under a lock).
 *
 *  weights fp32 [M], 16-byte aligned, 1 <= M <= ARIDE_STATIC_MAX_REPLAY; uniforms fp64 [K];
 *  idx_out int64 [K]; prob_out fp32 [K] nullable; status_out device aride_status [1], 8-byte
 *  aligned, nullable.
 * Errors: E_SHAPE (M <= 0, K < 0), E_RANGE (M > ARIDE_STATIC_MAX_REPLAY, K >= 2^25), E_NULL, E_ALIGN,
 *         E_HIP (the array's address could not be obtained, or a launch failed).  K == 0 is a no-op.
 */
#define ARIDE_STATIC_MAX_REPLAY (1 << 20)
int aride_sample_prioritized_static(const float* weights, int64_t M, const double* uniforms, int64_t K,
                                    int64_t* idx_out, float* prob_out, aride_status* status_out /* device */,
                                    void* stream);

/*
 * actor_loss_grad -- Section 5.1, eq. (1) and the policy update of Appendix A.4.2: the actor
 * loss of a batch and its gradient with respect to the logits, as a second sweep over the
 * logits that aride_score_logits reduced.  With A_t = target[t] - baseline[t] (the
 * Retrace-corrected advantage of Sections 5.1/5.2), rho_t and A_t held constant, and
 * p = softmax of row r of step t:
 *     loss = scale * sum_t [ -rho_t A_t step_logp[t] - beta step_ent[t] + lambda_pen penalty[t] ]
 *     grad[r, v] = scale * [ -rho_t A_t (1[v = tokens[r]] - p_v) + beta p_v (log p_v + H_r) ]
 * Masked rows (token < 0 or >= V) get zeros; columns >= V of a row are left untouched.
 *
 *  logits, tokens, R, V, row_stride, A   as for aride_score_logits (same buffers).
 *  tok_logp, tok_ent    fp32 [R]: the per-token outputs of aride_score_logits on these logits
 *                       (they supply each row's log-partition function and entropy).
 *  step_logp, step_ent  fp32 [R/A]: its per-step outputs (needed only for `loss`).
 *  rho, target, baseline fp32 [R/A]; penalty fp32 [R/A] nullable (invalid-action indicator).
 *  grad    [R, row_stride] in the logits' layout, bf16 or fp32 per cfg.grad_f32, 16-byte
 *          aligned, nullable.   loss  fp32 [1] device, nullable.
 * Errors: E_NULL, E_SHAPE, E_ALIGN, E_RANGE as for aride_score_logits.  R == 0 writes loss = 0.
 */
int aride_actor_loss_grad(const void* logits_bf16, int64_t R, int64_t V, int64_t row_stride,
                          const int32_t* tokens, int32_t A, const float* tok_logp,
                          const float* tok_ent, const float* step_logp, const float* step_ent,
                          const float* rho, const float* target, const float* baseline,
                          const float* penalty, aride_actor_cfg cfg, void* grad, float* loss,
                          void* stream);

#ifdef __cplusplus
}
#endif
#endif /* ARIDE_H */
