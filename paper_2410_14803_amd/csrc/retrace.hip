// retrace_targets and compute_priorities (Sections 5.2 and 5.3 of the DistRL paper).
//
// Retrace(lambda): Delta_t = delta_t + gamma*lambda*min(1, rho_{t+1}) * Delta_{t+1} is an
// affine recurrence X -> b + a*X running backwards through each trajectory.  Affine maps
// compose associatively, so a trajectory is scanned 64 steps at a time: lane j of a wave
// owns step (end-1-j), the 64 maps are combined with a 6-round shuffle scan, and the
// value entering the chunk is carried in a register to the next (earlier) chunk.
// The coefficient of a trajectory's last step is 0, which is what isolates trajectories
// from each other.  One wave per trajectory; loads and stores are contiguous 256-byte
// runs.  HBM-bound (about 36 bytes per step); no contraction, no MFMA.
#include "aride_device.h"

namespace aride {

__global__ __launch_bounds__(256) void k_retrace(
    const float* __restrict__ logp_pi, const float* __restrict__ logp_mu,
    const float* __restrict__ reward, const float* __restrict__ value,
    const float* __restrict__ q, const float* __restrict__ boot,
    const int* __restrict__ offsets, int B, int N, float gamma, float lambda,
    float* __restrict__ target, float* __restrict__ td, float* __restrict__ rho_out) {
    const int lane = threadIdx.x & 63;
    const int b = (int)(((long long)blockIdx.x * blockDim.x + threadIdx.x) >> 6);
    if (b >= B) return;   // whole waves leave together
    // offsets outside [0, N] are clamped so a malformed CSR array cannot reach past the inputs
    const int lo = max(offsets[b], 0), hi = min(offsets[b + 1], N);
    const float boot_b = boot ? boot[b] : 0.f;

    float carry_delta = 0.f;  // Delta of the step just after this chunk
    float carry_c = 0.f;      // lambda*min(1,rho) of the step just after this chunk
    for (int end = hi; end > lo; end -= kWave) {
        const int t = end - 1 - lane;
        const bool valid = t >= lo;
        float a = 0.f, bterm = 0.f, qt = 0.f, rho = 0.f, c = 0.f;
        if (valid) {
            const float vt = value[t];
            qt = q ? q[t] : vt;
            const float vnext = (t == hi - 1) ? boot_b : value[t + 1];
            bterm = reward[t] + gamma * vnext - qt;       // delta_t
            rho = expf(logp_pi[t] - logp_mu[t]);
            c = lambda * fminf(1.f, rho);
        }
        // coefficient on Delta_{t+1}: gamma * c_{t+1}; the neighbour lane-1 holds step t+1
        float c_next = __shfl_up(c, 1, kWave);
        if (lane == 0) c_next = carry_c;
        if (valid && t != hi - 1) a = gamma * c_next;

        // inclusive scan of map composition along increasing lane (decreasing t)
        float A = a, Bv = bterm;
#pragma unroll
        for (int d = 1; d < kWave; d <<= 1) {
            float pa = __shfl_up(A, d, kWave);
            float pb = __shfl_up(Bv, d, kWave);
            if (lane >= d) { Bv = fmaf(A, pb, Bv); A = A * pa; }
        }
        const float Delta = fmaf(A, carry_delta, Bv);
        if (valid) {
            if (target) target[t] = qt + Delta;
            if (td) td[t] = bterm;
            if (rho_out) rho_out[t] = rho;
        }
        carry_delta = __shfl(Delta, kWave - 1, kWave);
        carry_c = __shfl(c, kWave - 1, kWave);
    }
}

// Section 5.3 / Appendix A.4.3: p_t = w1*|delta_t|/s_delta + w2*rho~_t + w3*H_t/s_H + eps and
// the per-trajectory mean.  One wave per trajectory, 64 steps per round, fixed-order
// butterfly sum so results are reproducible.
__global__ __launch_bounds__(256) void k_priorities(
    const float* __restrict__ td, const float* __restrict__ rho, const float* __restrict__ ent,
    const int* __restrict__ offsets, int B, int N, float w_td, float w_rho, float w_ent,
    float inv_td_scale, float inv_ent_scale, float eps, int truncate,
    float* __restrict__ step_prio, float* __restrict__ traj_prio) {
    const int lane = threadIdx.x & 63;
    const int b = (int)(((long long)blockIdx.x * blockDim.x + threadIdx.x) >> 6);
    if (b >= B) return;
    const int lo = max(offsets[b], 0), hi = min(offsets[b + 1], N);
    float acc = 0.f;
    for (int t = lo + lane; t < hi; t += kWave) {
        float r = rho[t];
        if (truncate) r = fminf(1.f, r);
        float p = w_td * fabsf(td[t]) * inv_td_scale + w_rho * r + w_ent * ent[t] * inv_ent_scale + eps;
        if (step_prio) step_prio[t] = p;
        acc += p;
    }
    acc = wave_sum(acc);
    if (traj_prio && lane == 0) traj_prio[b] = hi > lo ? acc / (float)(hi - lo) : 0.f;
}

hipError_t retrace_launch(const float* lp, const float* lm, const float* r, const float* v,
                          const float* q, const float* boot, const int* off, int B, int N, float gamma,
                          float lambda, float* target, float* td, float* rho, hipStream_t st) {
    const unsigned blocks = (unsigned)(((long long)B * kWave + 255) / 256);
    hipLaunchKernelGGL(k_retrace, dim3(blocks), dim3(256), 0, st, lp, lm, r, v, q, boot, off, B,
                       N, gamma, lambda, target, td, rho);
    return hipGetLastError();
}

hipError_t priorities_launch(const float* td, const float* rho, const float* ent, const int* off,
                             int B, int N, float w_td, float w_rho, float w_ent, float td_scale,
                             float ent_scale, float eps, int truncate, float* step_prio,
                             float* traj_prio, hipStream_t st) {
    const unsigned blocks = (unsigned)(((long long)B * kWave + 255) / 256);
    hipLaunchKernelGGL(k_priorities, dim3(blocks), dim3(256), 0, st, td, rho, ent, off, B, N, w_td,
                       w_rho, w_ent, 1.f / td_scale, 1.f / ent_scale, eps, truncate, step_prio,
                       traj_prio);
    return hipGetLastError();
}

}  // namespace aride
