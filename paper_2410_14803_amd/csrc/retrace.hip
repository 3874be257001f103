// retrace_targets and compute_priorities (Sections 5.2 and 5.3 of the DistRL paper).
//
// Retrace(lambda): Delta_t = delta_t + gamma*lambda*min(1, rho_{t+1}) * Delta_{t+1} is an
// affine recurrence X -> b + a*X running backwards through each trajectory, and affine maps
// compose associatively.  One wave owns one trajectory and walks it from its end in tiles of
// 256 steps, staged in LDS:
//   1. coalesced: lane l loads steps end-1-(64i+l), i = 0..3 (all loads of a tile in flight
//      together), forms delta, rho, c = lambda*min(1,rho) and parks delta and c in LDS in
//      reverse-time order;
//   2. transposed: lane j takes the four consecutive maps 4j..4j+3 out of LDS, composes them
//      serially, a 6-round shuffle scan combines the 64 lane aggregates, and the lane then
//      replays its four maps from the value entering it; the four Delta go back to LDS;
//   3. coalesced again: target = Q + Delta, delta and rho are stored as contiguous runs.
// Delta and c of the tile's earliest step are carried in registers to the next tile.  The
// coefficient in front of the trajectory's last step is 0 (nothing follows it), which is
// what keeps trajectories apart.  HBM-bound (32 bytes per step); no contraction, no MFMA.
#include "aride_device.h"

namespace aride {

constexpr int kTile = 256;          // steps per wave and tile
constexpr int kPerLane = kTile / kWave;

// Orders this wave's LDS writes before its later LDS reads by other lanes (LDS operations of
// one wave execute in order; this only stops the compiler from moving them).
__device__ __forceinline__ void wave_lds_sync() {
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
    __builtin_amdgcn_wave_barrier();
    __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
}

__global__ __launch_bounds__(256) void k_retrace(
    const float* __restrict__ logp_pi, const float* __restrict__ logp_mu,
    const float* __restrict__ reward, const float* __restrict__ value,
    const float* __restrict__ q, const float* __restrict__ boot,
    const int* __restrict__ offsets, int B, int N, float gamma, float lambda,
    float* __restrict__ target, float* __restrict__ td, float* __restrict__ rho_out) {
    __shared__ __attribute__((aligned(16))) float lds_b[4][kTile];   // delta, later Delta
    __shared__ __attribute__((aligned(16))) float lds_c[4][kTile];   // lambda*min(1,rho)
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int b = (int)(((long long)blockIdx.x * blockDim.x + threadIdx.x) >> 6);
    if (b >= B) return;   // whole waves leave together; there is no workgroup barrier below
    // offsets outside [0, N] are clamped so a malformed CSR array cannot reach past the inputs
    const int lo = max(offsets[b], 0), hi = min(offsets[b + 1], N);
    const float boot_b = boot ? boot[b] : 0.f;
    float* sb = lds_b[wave];
    float* sc = lds_c[wave];

    float carry_delta = 0.f;  // Delta of the step just after this tile (0 past the end)
    float carry_c = 0.f;      // c of that step (0 past the end: nothing follows the last step)
    for (int end = hi; end > lo; end -= kTile) {
        // 1. coalesced loads; position p = 64*i + lane holds step t = end-1-p
        float dlt[kPerLane], rho[kPerLane], qv[kPerLane];
#pragma unroll
        for (int i = 0; i < kPerLane; ++i) {
            const int t = end - 1 - (i * kWave + lane);
            float d = 0.f, r = 0.f, c = 0.f, qt = 0.f;
            if (t >= lo) {
                const float vt = value[t];
                qt = q ? q[t] : vt;
                const float vnext = (t == hi - 1) ? boot_b : value[t + 1];
                d = reward[t] + gamma * vnext - qt;
                r = expf(logp_pi[t] - logp_mu[t]);
                c = lambda * fminf(1.f, r);
            }
            dlt[i] = d; rho[i] = r; qv[i] = qt;
            sb[i * kWave + lane] = d;
            sc[i * kWave + lane] = c;
        }
        wave_lds_sync();
        // 2. lane j owns positions 4j .. 4j+3; the map at position p is X -> b_p + gamma*c_{p-1}*X
        const float4 b4 = *reinterpret_cast<const float4*>(sb + 4 * lane);
        const float4 c4 = *reinterpret_cast<const float4*>(sc + 4 * lane);
        const float c_before = lane ? sc[4 * lane - 1] : carry_c;
        const float a0 = gamma * c_before, a1 = gamma * c4.x, a2 = gamma * c4.y, a3 = gamma * c4.z;
        float A = a0, Bv = b4.x;
        Bv = fmaf(a1, Bv, b4.y); A *= a1;
        Bv = fmaf(a2, Bv, b4.z); A *= a2;
        Bv = fmaf(a3, Bv, b4.w); A *= a3;
#pragma unroll
        for (int d = 1; d < kWave; d <<= 1) {      // inclusive scan of map composition over lanes
            const float pa = __shfl_up(A, d, kWave);
            const float pb = __shfl_up(Bv, d, kWave);
            if (lane >= d) { Bv = fmaf(A, pb, Bv); A = A * pa; }
        }
        // value entering this lane: the composition of all earlier lanes applied to the carry
        const float ea = __shfl_up(A, 1, kWave), eb = __shfl_up(Bv, 1, kWave);
        const float x_in = lane ? fmaf(ea, carry_delta, eb) : carry_delta;
        float4 D;
        D.x = fmaf(a0, x_in, b4.x);
        D.y = fmaf(a1, D.x, b4.y);
        D.z = fmaf(a2, D.y, b4.z);
        D.w = fmaf(a3, D.z, b4.w);
        *reinterpret_cast<float4*>(sb + 4 * lane) = D;
        carry_delta = __shfl(D.w, kWave - 1, kWave);
        carry_c = __shfl(c4.w, kWave - 1, kWave);
        wave_lds_sync();
        // 3. coalesced stores
#pragma unroll
        for (int i = 0; i < kPerLane; ++i) {
            const int t = end - 1 - (i * kWave + lane);
            if (t >= lo) {
                if (target) target[t] = qv[i] + sb[i * kWave + lane];
                if (td) td[t] = dlt[i];
                if (rho_out) rho_out[t] = rho[i];
            }
        }
        wave_lds_sync();   // the next tile overwrites the staging area
    }
}

// Section 5.3 / Appendix A.4.3: p_t = w1*|delta_t|/s_delta + w2*rho~_t + w3*H_t/s_H + eps and
// the per-trajectory mean.  One wave per trajectory, 256 steps per round with all loads of a
// round in flight together, fixed-order butterfly sum so results are reproducible.
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
    for (int t0 = lo; t0 < hi; t0 += kTile) {
        float p[kPerLane];
#pragma unroll
        for (int i = 0; i < kPerLane; ++i) {
            const int t = t0 + i * kWave + lane;
            p[i] = 0.f;
            if (t < hi) {
                float r = rho[t];
                if (truncate) r = fminf(1.f, r);
                p[i] = w_td * fabsf(td[t]) * inv_td_scale + w_rho * r + w_ent * ent[t] * inv_ent_scale + eps;
            }
        }
#pragma unroll
        for (int i = 0; i < kPerLane; ++i) {
            const int t = t0 + i * kWave + lane;
            if (t < hi) { if (step_prio) step_prio[t] = p[i]; acc += p[i]; }
        }
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
