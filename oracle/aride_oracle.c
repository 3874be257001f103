/*
 * CPU oracle for the A-RIDE learner-side scoring pass (DistRL, arXiv 2410.14803).
 *
 * THIS IS TEST INFRASTRUCTURE, NOT THE PRODUCT.  It is a plain, slow, scalar fp64
 * restatement of what the scoring path computes, written from the paper's formulas
 * so that a reader can check it against the paper by eye.  Only the test-suite, the
 * smoke check and the benchmark's "cpu_baseline" leg may call it.  It shares no code,
 * header, table or constant with the HIP library and neither includes the other.
 *
 * Every function is pinned by CPU tests against closed forms, brute-force
 * expansions and library routines (tests/test_oracle_*.py).  The one exception:
 * the last-ulp value of pow() in oracle_update_priorities depends on the host libm
 * ("parity unpinned" at the final ulp; it is pinned to 1e-12 relative against
 * closed forms, and the sampler is bit-exact as a function of the stored weights).
 *
 * Conventions: B trajectories, N steps flattened trajectory after trajectory,
 * traj_offsets[B+1] (CSR), A action tokens per step, R = N*A logit rows, vocabulary V.
 * All outputs are fp64 unless they are indices.  Output pointers may be NULL.
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>

/* A bf16 is the upper 16 bits of an IEEE-754 binary32; widening is exact. */
static double bf16_to_double(uint16_t h) {
    uint32_t bits = ((uint32_t)h) << 16;
    float f;
    memcpy(&f, &bits, sizeof f);
    return (double)f;
}

/*
 * Section 5.1, eq. (1) and the importance ratio below it: the policy is a token-level
 * language model, so log pi(a_t|s_t) is the sum over the action's A tokens of the
 * log-softmax of that token's logit row, and the entropy regulariser H(pi(.|s_t)) is
 * the Shannon entropy of each row's softmax, summed along the realised token path.
 *
 * Per row:  L = m + log sum_v exp(x_v - m)   (m = max_v x_v, only to keep exp finite)
 *           logp_v = x_v - L
 *           tok_logp = logp_{token},  tok_ent = - sum_v exp(logp_v) * logp_v
 * Rows whose token is negative or >= V are masked: they contribute 0 everywhere.
 * Step values are plain sums over the step's A rows in row order.
 */
int oracle_score_logits(const uint16_t* logits_bf16, int64_t R, int64_t V,
                        int64_t row_stride, const int32_t* tokens, int32_t A,
                        double* tok_logp, double* tok_ent,
                        double* step_logp, double* step_ent, int nthreads) {
    if (R < 0 || V <= 0 || A <= 0 || R % A != 0 || row_stride < V) return -2;
    int64_t N = R / A;
    double* lp = tok_logp ? tok_logp : (double*)malloc(sizeof(double) * (size_t)(R ? R : 1));
    double* en = tok_ent ? tok_ent : (double*)malloc(sizeof(double) * (size_t)(R ? R : 1));
    (void)nthreads;
#ifdef _OPENMP
#pragma omp parallel for schedule(static) num_threads(nthreads > 0 ? nthreads : 1)
#endif
    for (int64_t r = 0; r < R; ++r) {
        const uint16_t* row = logits_bf16 + r * row_stride;
        int32_t tok = tokens[r];
        if (tok < 0 || tok >= V) { lp[r] = 0.0; en[r] = 0.0; continue; }
        double m = -INFINITY;
        for (int64_t v = 0; v < V; ++v) {
            double x = bf16_to_double(row[v]);
            if (x > m) m = x;
        }
        double sum = 0.0;
        for (int64_t v = 0; v < V; ++v) sum += exp(bf16_to_double(row[v]) - m);
        double L = m + log(sum);
        double ent = 0.0;
        for (int64_t v = 0; v < V; ++v) {
            double logp = bf16_to_double(row[v]) - L;
            double p = exp(logp);
            if (p > 0.0) ent -= p * logp;
        }
        lp[r] = bf16_to_double(row[tok]) - L;
        en[r] = ent;
    }
    for (int64_t n = 0; n < N; ++n) {
        double sl = 0.0, se = 0.0;
        for (int32_t j = 0; j < A; ++j) { sl += lp[n * A + j]; se += en[n * A + j]; }
        if (step_logp) step_logp[n] = sl;
        if (step_ent) step_ent[n] = se;
    }
    if (!tok_logp) free(lp);
    if (!tok_ent) free(en);
    return 0;
}

/*
 * Section 5.2 (Retrace) with the TD error of Section 5.3 / Appendix A.4.2:
 *   rho_t   = pi(a_t|s_t) / mu(a_t|s_t) = exp(logpi_t - logmu_t)
 *   c_t     = lambda * min(1, rho_t)
 *   delta_t = r_t + gamma * V(s_{t+1}) - Q_t          (Q == V when q is NULL)
 *   Delta_t = sum_{k=t}^{T-1} gamma^{k-t} (prod_{i=t+1}^{k} c_i) delta_k
 * The product starts at i = t+1, so a step's own ratio never enters its own
 * correction.  Peeling off the k = t term gives the backward recursion used here:
 *   Delta_{T-1} = delta_{T-1},   Delta_t = delta_t + gamma * c_{t+1} * Delta_{t+1}.
 * V(s_T) past the last step is boot[b] (0 when boot is NULL).  target_t = Q_t + Delta_t.
 */
int oracle_retrace_targets(const double* logp_pi, const double* logp_mu,
                           const double* reward, const double* value, const double* q,
                           const double* boot, const int32_t* traj_offsets, int64_t B,
                           int64_t N, double gamma, double lambda,
                           double* target, double* td, double* rho) {
    if (B < 0 || N < 0) return -2;
    if (B > 0 && (traj_offsets[0] != 0 || traj_offsets[B] != N)) return -2;
    for (int64_t b = 0; b < B; ++b) {
        int64_t lo = traj_offsets[b], hi = traj_offsets[b + 1];
        if (hi < lo) return -2;
        double Delta_next = 0.0, c_next = 0.0;
        for (int64_t t = hi - 1; t >= lo; --t) {
            double v_next = (t == hi - 1) ? (boot ? boot[b] : 0.0) : value[t + 1];
            double q_t = q ? q[t] : value[t];
            double delta = reward[t] + gamma * v_next - q_t;
            double rho_t = exp(logp_pi[t] - logp_mu[t]);
            double Delta = (t == hi - 1) ? delta : delta + gamma * c_next * Delta_next;
            if (target) target[t] = q_t + Delta;
            if (td) td[t] = delta;
            if (rho) rho[t] = rho_t;
            Delta_next = Delta;
            c_next = lambda * (rho_t < 1.0 ? rho_t : 1.0);
        }
    }
    return 0;
}

/*
 * Section 5.3 (DPER) with the normalisation of Appendix A.4.3:
 *   p_t = w1 * |delta_t| / s_delta + w2 * rho~_t + w3 * H_t / s_H + eps
 * rho~ = min(1, rho) when truncate_rho is set (the appendix states the ratio term lies
 * in [0,1]), else rho.  The trajectory priority p(tau) is the mean of p_t over the
 * trajectory, which by linearity equals w1*mean|delta| + w2*mean rho + w3*mean H.
 * An empty trajectory has priority 0.
 */
int oracle_compute_priorities(const double* td, const double* rho, const double* ent,
                              const int32_t* traj_offsets, int64_t B, int64_t N,
                              double w_td, double w_rho, double w_ent, double td_scale,
                              double ent_scale, double eps, int truncate_rho,
                              double* step_prio, double* traj_prio) {
    if (B < 0 || N < 0 || td_scale == 0.0 || ent_scale == 0.0) return -2;
    for (int64_t b = 0; b < B; ++b) {
        int64_t lo = traj_offsets[b], hi = traj_offsets[b + 1];
        double acc = 0.0;
        for (int64_t t = lo; t < hi; ++t) {
            double r = rho[t];
            if (truncate_rho && r > 1.0) r = 1.0;
            double p = w_td * fabs(td[t]) / td_scale + w_rho * r + w_ent * ent[t] / ent_scale + eps;
            if (step_prio) step_prio[t] = p;
            acc += p;
        }
        if (traj_prio) traj_prio[b] = (hi > lo) ? acc / (double)(hi - lo) : 0.0;
    }
    return 0;
}

/*
 * Appendix A.4.2 (priority-based sampling) stores p^alpha; Section 5.3's last
 * sentence has priorities recomputed and overwritten.  Sequential order defines
 * "the last occurrence of a repeated index wins".  The stored weight is fp32.
 * Returns the number of indices outside [0, M) (those entries are skipped).
 */
int64_t oracle_update_priorities(float* weights, int64_t M, const int64_t* idx,
                                 const float* prio, int64_t K, float alpha) {
    int64_t bad = 0;
    for (int64_t k = 0; k < K; ++k) {
        if (idx[k] < 0 || idx[k] >= M) { ++bad; continue; }
        double p = (double)prio[k];
        if (!(p > 0.0)) p = 0.0; /* negative and NaN priorities carry no mass */
        weights[idx[k]] = (float)pow(p, (double)alpha);
    }
    return bad;
}

/*
 * Exact-integer form of P(i) = w_i / sum_j w_j (Appendix A.4.2), so that the drawn
 * index is a function of the stored weight bits and the uniform alone:
 *   w_i   stored fp32 weight; NaN, infinite or negative weights carry no mass
 *   wmax  = max_i w_i;  e = ilogb(wmax) + 1  (so w_i * 2^-e < 1)
 *   q_i   = floor(w_i * 2^(39-e))            (< 2^39; exact: power-of-two scaling)
 *   C_i   = q_0 + ... + q_i  (uint64),  Total = C_{M-1}  (< 2^63 for M <= 2^24)
 * quant[] receives q_i; returns Total (0 when there is no mass).
 */
uint64_t oracle_quantise_weights(const float* weights, int64_t M, uint64_t* quant) {
    double wmax = 0.0;
    for (int64_t i = 0; i < M; ++i) {
        double w = (double)weights[i];
        if (isfinite(w) && w > wmax) wmax = w;
    }
    uint64_t total = 0;
    if (wmax == 0.0) { for (int64_t i = 0; i < M; ++i) quant[i] = 0; return 0; }
    int e = ilogb(wmax) + 1;
    for (int64_t i = 0; i < M; ++i) {
        double w = (double)weights[i];
        uint64_t qi = 0;
        if (isfinite(w) && w > 0.0) qi = (uint64_t)floor(ldexp(w, 39 - e));
        quant[i] = qi;
        total += qi;
    }
    return total;
}

/*
 * For each uniform u_k in [0,1):  t_k = min(floor(u_k * (double)Total), Total-1),
 * idx_k = min{ i : C_i > t_k }.  The strict inequality means zero-weight entries are
 * never drawn.  prob_k = q_idx / Total.  u < 0 or NaN is read as 0.  Returns 0, or
 * -5 when Total == 0 (then every idx_k = -1 and prob_k = 0).
 */
int oracle_sample_prioritized(const float* weights, int64_t M, const double* uniforms,
                              int64_t K, int64_t* idx_out, double* prob_out) {
    if (M <= 0 || M > (1 << 24) || K < 0) return -4;
    uint64_t* C = (uint64_t*)malloc(sizeof(uint64_t) * (size_t)M);
    uint64_t total = oracle_quantise_weights(weights, M, C);
    if (total == 0) {
        for (int64_t k = 0; k < K; ++k) { idx_out[k] = -1; if (prob_out) prob_out[k] = 0.0; }
        free(C);
        return -5;
    }
    uint64_t* qv = prob_out ? (uint64_t*)malloc(sizeof(uint64_t) * (size_t)M) : NULL;
    if (qv) memcpy(qv, C, sizeof(uint64_t) * (size_t)M);
    for (int64_t i = 1; i < M; ++i) C[i] += C[i - 1]; /* inclusive prefix, in place */
    for (int64_t k = 0; k < K; ++k) {
        double u = uniforms[k];
        if (!(u > 0.0)) u = 0.0;
        volatile double prod = u * (double)total; /* one rounding, never fused */
        uint64_t t = (prod >= 18446744073709551616.0) ? (total - 1) : (uint64_t)floor(prod);
        if (t > total - 1) t = total - 1;
        /* first i with C_i > t.  C is non-decreasing and C[M-1] = Total > t, so bisect:
         * everything left of lo has C <= t, and C[hi] > t throughout. */
        int64_t lo = 0, hi = M - 1;
        while (lo < hi) {
            int64_t mid = lo + (hi - lo) / 2;
            if (C[mid] > t) hi = mid; else lo = mid + 1;
        }
        int64_t i = lo;
        idx_out[k] = i;
        if (prob_out) prob_out[k] = (double)qv[i] / (double)total;
    }
    free(qv);
    free(C);
    return 0;
}

/*
 * Actor loss of Section 5.1, eq. (1), and its gradient with respect to the logits
 * (Appendix A.4.2, "Policy Update Mechanism"), for a token-level policy:
 *   L = scale * sum_t [ - rho_t * A_t * log pi(a_t|s_t) - beta * H_t + lambda_pen * P_t ]
 * with log pi(a_t|s_t) and H_t the per-step sums of oracle_score_logits, A_t = target_t -
 * baseline_t the Retrace-corrected advantage (Section 5.2), rho_t and A_t constants of the
 * differentiation (importance weight and advantage estimate), and P_t the invalid-action
 * indicator supplied from outside (it does not depend on the logits).  `scale` is 1/N for the
 * batch mean that stands for the expectation over mu.  For row r of step t, with
 * p = softmax(x_r):
 *   dL/dx_{r,v} = scale * [ - rho_t A_t (1[v = tok_r] - p_v) + beta * p_v (log p_v + H_r) ]
 * (the second term is -beta * dH_r/dx_v).  Masked rows (token < 0 or >= V) get a zero
 * gradient.  grad is dense [R, V] fp64.
 */
int oracle_actor_loss_grad(const uint16_t* logits_bf16, int64_t R, int64_t V, int64_t row_stride,
                           const int32_t* tokens, int32_t A, const double* rho,
                           const double* target, const double* baseline, const double* penalty,
                           double beta, double lambda_pen, double scale, double* grad,
                           double* loss_out) {
    if (R < 0 || V <= 0 || A <= 0 || R % A != 0 || row_stride < V) return -2;
    int64_t N = R / A;
    double loss = 0.0;
    double* logp = (double*)malloc(sizeof(double) * (size_t)V);
    for (int64_t t = 0; t < N; ++t) {
        double coef = rho[t] * (target[t] - baseline[t]);
        double step_logp = 0.0, step_ent = 0.0;
        for (int32_t j = 0; j < A; ++j) {
            int64_t r = t * A + j;
            const uint16_t* row = logits_bf16 + r * row_stride;
            int32_t tok = tokens[r];
            if (tok < 0 || tok >= V) {
                if (grad) for (int64_t v = 0; v < V; ++v) grad[r * V + v] = 0.0;
                continue;
            }
            double m = -INFINITY;
            for (int64_t v = 0; v < V; ++v) { double x = bf16_to_double(row[v]); if (x > m) m = x; }
            double sum = 0.0;
            for (int64_t v = 0; v < V; ++v) sum += exp(bf16_to_double(row[v]) - m);
            double L = m + log(sum);
            double ent = 0.0;
            for (int64_t v = 0; v < V; ++v) {
                logp[v] = bf16_to_double(row[v]) - L;
                double p = exp(logp[v]);
                if (p > 0.0) ent -= p * logp[v];
            }
            step_logp += logp[tok];
            step_ent += ent;
            if (grad) {
                for (int64_t v = 0; v < V; ++v) {
                    double p = exp(logp[v]);
                    double onehot = (v == tok) ? 1.0 : 0.0;
                    double ent_term = (p > 0.0) ? p * (logp[v] + ent) : 0.0;
                    grad[r * V + v] = scale * (-coef * (onehot - p) + beta * ent_term);
                }
            }
        }
        loss += -coef * step_logp - beta * step_ent + (penalty ? lambda_pen * penalty[t] : 0.0);
    }
    free(logp);
    if (loss_out) *loss_out = scale * loss;
    return 0;
}

/*
 * V-trace targets (Espeholt et al. 2018, the IMPALA paper), which the DistRL paper names as
 * the standard alternative it sets Retrace against (Section 2; Appendix A.4.1):
 *   v_s = V(x_s) + sum_{t=s}^{T-1} gamma^(t-s) (prod_{i=s}^{t-1} c_i) rho~_t delta_t,
 *   rho~_t = min(rho_bar, rho_t),  c_i = lambda * min(c_bar, rho_i),
 *   delta_t = r_t + gamma V(x_{t+1}) - Q_t   (Q == V when q is NULL).
 * Peeling off the t = s term:  Delta_s = rho~_s delta_s + gamma c_s Delta_{s+1}; the step's OWN
 * ratio enters both factors.  target = Q + Delta; td and rho as in oracle_retrace_targets.
 */
int oracle_vtrace_targets(const double* logp_pi, const double* logp_mu, const double* reward,
                          const double* value, const double* q, const double* boot,
                          const int32_t* traj_offsets, int64_t B, int64_t N, double gamma,
                          double lambda, double rho_bar, double c_bar, double* target, double* td,
                          double* rho) {
    if (B < 0 || N < 0) return -2;
    for (int64_t b = 0; b < B; ++b) {
        int64_t lo = traj_offsets[b], hi = traj_offsets[b + 1];
        double Delta_next = 0.0;
        for (int64_t t = hi - 1; t >= lo; --t) {
            double v_next = (t == hi - 1) ? (boot ? boot[b] : 0.0) : value[t + 1];
            double q_t = q ? q[t] : value[t];
            double delta = reward[t] + gamma * v_next - q_t;
            double rho_t = exp(logp_pi[t] - logp_mu[t]);
            double rho_clip = rho_t < rho_bar ? rho_t : rho_bar;
            double c_t = lambda * (rho_t < c_bar ? rho_t : c_bar);
            double Delta = rho_clip * delta + ((t == hi - 1) ? 0.0 : gamma * c_t * Delta_next);
            if (target) target[t] = q_t + Delta;
            if (td) td[t] = delta;
            if (rho) rho[t] = rho_t;
            Delta_next = Delta;
        }
    }
    return 0;
}

/*
 * Section 5.1, state-value function estimation: Monte-Carlo return G_t = sum_{k=t}^{T-1}
 * gamma^(k-t) r_k within each trajectory, and the label 1[G_t > 0] of the value network's
 * classification loss.
 */
int oracle_mc_returns(const double* reward, const int32_t* traj_offsets, int64_t B, int64_t N,
                      double gamma, double* ret, double* label) {
    if (B < 0 || N < 0) return -2;
    for (int64_t b = 0; b < B; ++b) {
        double G = 0.0;
        for (int64_t t = traj_offsets[b + 1] - 1; t >= traj_offsets[b]; --t) {
            G = reward[t] + gamma * G;
            if (ret) ret[t] = G;
            if (label) label[t] = G > 0.0 ? 1.0 : 0.0;
        }
    }
    return 0;
}

/*
 * Appendix A.4.2, circular replay buffer of fixed capacity M: each new entry is written at the
 * buffer index i, which then advances as i <- (i + 1) mod M, so that new experiences overwrite
 * the oldest ones.  Here the stored value is the entry's sampling weight prio^alpha (the payload
 * lives in the caller's arrays at the same slot).  slots_out[k] receives the slot entry k was
 * written to, or -1 if a later entry of the same batch overwrote it (only possible when K > M).
 * Returns the advanced index.
 */
int64_t oracle_replay_insert(float* weights, int64_t M, int64_t cursor, const float* prio, int64_t K,
                             float alpha, int64_t* slots_out) {
    int64_t i = cursor;
    for (int64_t k = 0; k < K; ++k) {
        double p = (double)prio[k];
        if (!(p > 0.0)) p = 0.0;
        weights[i] = (float)pow(p, (double)alpha);
        if (slots_out) slots_out[k] = i;
        i = (i + 1) % M;
    }
    if (slots_out)
        for (int64_t k = 0; k + M < K; ++k) slots_out[k] = -1; /* overwritten by entry k + M */
    return i;
}
