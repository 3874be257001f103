// retrace_targets and compute_priorities (Sections 5.2 and 5.3 of the DistRL paper).
//
// Retrace(lambda): Delta_t = delta_t + gamma*lambda*min(1, rho_{t+1}) * Delta_{t+1} is an
// affine recurrence X -> b + a*X running backwards through each trajectory, and affine maps
// compose associatively.  One wave owns one trajectory and walks it from its end in tiles of
// 256 steps, staged in LDS:
//   1. coalesced: lane l loads steps end-1-(64i+l), i = 0..3 (all loads of a tile in flight
//      together), forms delta and rho, and parks each step's map X -> b + a*X (a = gamma *
//      lambda * min(1, rho of the NEXT step), b = delta) in LDS in reverse-time order;
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

// Steps 2 of the tile: the maps X -> b_p + a_p X of the 256 positions are in LDS (sa, sb) in
// reverse-time order; on return sb holds Delta_p = (f_p o ... o f_0)(carry) and the function
// value is Delta_255.
__device__ __forceinline__ float tile_scan(float* sa, float* sb, int lane, float carry) {
    const float4 a4 = *reinterpret_cast<const float4*>(sa + 4 * lane);
    const float4 b4 = *reinterpret_cast<const float4*>(sb + 4 * lane);
    float A = a4.x, Bv = b4.x;
    Bv = fmaf(a4.y, Bv, b4.y); A *= a4.y;
    Bv = fmaf(a4.z, Bv, b4.z); A *= a4.z;
    Bv = fmaf(a4.w, Bv, b4.w); A *= a4.w;
#pragma unroll
    for (int d = 1; d < kWave; d <<= 1) {      // inclusive scan of map composition over lanes
        const float pa = __shfl_up(A, d, kWave);
        const float pb = __shfl_up(Bv, d, kWave);
        if (lane >= d) { Bv = fmaf(A, pb, Bv); A = A * pa; }
    }
    // value entering this lane: the composition of all earlier lanes applied to the carry
    const float ea = __shfl_up(A, 1, kWave), eb = __shfl_up(Bv, 1, kWave);
    const float x_in = lane ? fmaf(ea, carry, eb) : carry;
    float4 D;
    D.x = fmaf(a4.x, x_in, b4.x);
    D.y = fmaf(a4.y, D.x, b4.y);
    D.z = fmaf(a4.z, D.y, b4.z);
    D.w = fmaf(a4.w, D.z, b4.w);
    *reinterpret_cast<float4*>(sb + 4 * lane) = D;
    return __shfl(D.w, kWave - 1, kWave);
}

// Section 5.3 / Appendix A.4.3: p_t = w1*|delta_t|/s_delta + w2*rho~_t + w3*H_t/s_H + eps.
__device__ __forceinline__ float step_priority(float td, float rho, float ent, float w_td, float w_rho,
                                               float w_ent, float inv_td_scale, float inv_ent_scale,
                                               float eps, int truncate) {
    const float r = truncate ? fminf(1.f, rho) : rho;
    return w_td * fabsf(td) * inv_td_scale + w_rho * r + w_ent * ent * inv_ent_scale + eps;
}

// VTRACE = false: Retrace(lambda) as in Section 5.2 -- the coefficient in front of Delta_{t+1}
// is gamma*lambda*min(1, rho_{t+1}) and the additive term is delta_t.
// VTRACE = true: the V-trace targets of IMPALA, which the paper contrasts Retrace with
// (Section 2, Appendix A.4.1): additive term min(rho_bar, rho_t)*delta_t, coefficient
// gamma*lambda*min(c_bar, rho_t) -- the step's OWN ratio, not its successor's.
// PRIO = true: the priorities of Section 5.3 are formed in the same pass from the TD error and
// the ratio the wave already holds (plus one more load per step, the entropy), and the
// trajectory's mean priority from a wave sum: 36 bytes per step instead of the 48 the two
// kernels move between them, and one launch instead of two.
template <bool VTRACE, bool PRIO>
__global__ __launch_bounds__(256) void k_retrace(
    const float* __restrict__ logp_pi, const float* __restrict__ logp_mu,
    const float* __restrict__ reward, const float* __restrict__ value,
    const float* __restrict__ q, const float* __restrict__ boot,
    const int* __restrict__ offsets, int B, int N, float gamma, float lambda, float rho_bar, float c_bar,
    float* __restrict__ target, float* __restrict__ td, float* __restrict__ rho_out, PrioArgs pa) {
    __shared__ __attribute__((aligned(16))) float lds_a[4][kTile];   // coefficient on Delta_{t+1}
    __shared__ __attribute__((aligned(16))) float lds_b[4][kTile];   // additive term, later Delta
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int b = (int)(((long long)blockIdx.x * blockDim.x + threadIdx.x) >> 6);
    if (b >= B) return;   // whole waves leave together; there is no workgroup barrier below
    // offsets outside [0, N] are clamped so a malformed CSR array cannot reach past the inputs
    const int lo = max(offsets[b], 0), hi = min(offsets[b + 1], N);
    const float boot_b = boot ? boot[b] : 0.f;
    float* sa = lds_a[wave];
    float* sb = lds_b[wave];

    float carry_delta = 0.f;  // Delta of the step just after this tile (0 past the end)
    float carry_c = 0.f;      // Retrace: c of that step (0 past the end: nothing follows the last step)
    float prio_sum = 0.f;     // PRIO: this lane's share of the trajectory's priorities
    for (int end = hi; end > lo; end -= kTile) {
        // 1. coalesced loads; position p = 64*i + lane holds step t = end-1-p
        float dlt[kPerLane], rho[kPerLane], qv[kPerLane], ev[kPerLane];
#pragma unroll
        for (int i = 0; i < kPerLane; ++i) {
            const int t = end - 1 - (i * kWave + lane);
            float d = 0.f, r = 0.f, qt = 0.f, e = 0.f;
            if (t >= lo) {
                const float vt = value[t];
                qt = q ? q[t] : vt;
                const float vnext = (t == hi - 1) ? boot_b : value[t + 1];
                d = reward[t] + gamma * vnext - qt;
                r = expf(logp_pi[t] - logp_mu[t]);
                if constexpr (PRIO) e = pa.ent[t];
            }
            dlt[i] = d; rho[i] = r; qv[i] = qt; ev[i] = e;
        }
#pragma unroll
        for (int i = 0; i < kPerLane; ++i) {
            const int t = end - 1 - (i * kWave + lane);
            float a, bterm;
            if constexpr (VTRACE) {
                a = (t >= lo && t != hi - 1) ? gamma * lambda * fminf(c_bar, rho[i]) : 0.f;
                bterm = fminf(rho_bar, rho[i]) * dlt[i];
            } else {
                const float c = (t >= lo) ? lambda * fminf(1.f, rho[i]) : 0.f;
                float c_next = __shfl_up(c, 1, kWave);      // position p-1 holds step t+1
                if (lane == 0) c_next = carry_c;
                carry_c = __shfl(c, kWave - 1, kWave);
                a = gamma * c_next;
                bterm = dlt[i];
            }
            sa[i * kWave + lane] = a;
            sb[i * kWave + lane] = bterm;
        }
        wave_lds_sync();
        // 2. lane j composes positions 4j .. 4j+3, the wave scans, Delta goes back to LDS
        carry_delta = tile_scan(sa, sb, lane, carry_delta);
        wave_lds_sync();
        // 3. coalesced stores
#pragma unroll
        for (int i = 0; i < kPerLane; ++i) {
            const int t = end - 1 - (i * kWave + lane);
            if (t >= lo) {
                if (target) target[t] = qv[i] + sb[i * kWave + lane];
                if (td) td[t] = dlt[i];
                if (rho_out) rho_out[t] = rho[i];
                if constexpr (PRIO) {
                    const float p = step_priority(dlt[i], rho[i], ev[i], pa.w_td, pa.w_rho, pa.w_ent,
                                                  pa.inv_td_scale, pa.inv_ent_scale, pa.eps, pa.truncate);
                    if (pa.step_prio) pa.step_prio[t] = p;
                    prio_sum += p;
                }
            }
        }
        wave_lds_sync();   // the next tile overwrites the staging area
    }
    if constexpr (PRIO) {
        prio_sum = wave_sum(prio_sum);   // fixed order: reproducible
        if (pa.traj_prio && lane == 0) pa.traj_prio[b] = hi > lo ? prio_sum / (float)(hi - lo) : 0.f;
    }
}

// Section 5.1 (state-value estimation): the Monte-Carlo return G_t = sum_{k>=t} gamma^(k-t) r_k
// of each trajectory and the label 1[G_t > 0] the value network is trained on.  The same
// tile scan with the map X -> r_t + gamma X (coefficient 0 in front of the last step).
__global__ __launch_bounds__(256) void k_mc_returns(
    const float* __restrict__ reward, const int* __restrict__ offsets, int B, int N, float gamma,
    float* __restrict__ ret, float* __restrict__ label) {
    __shared__ __attribute__((aligned(16))) float lds_a[4][kTile];
    __shared__ __attribute__((aligned(16))) float lds_b[4][kTile];
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int b = (int)(((long long)blockIdx.x * blockDim.x + threadIdx.x) >> 6);
    if (b >= B) return;
    const int lo = max(offsets[b], 0), hi = min(offsets[b + 1], N);
    float* sa = lds_a[wave];
    float* sb = lds_b[wave];
    float carry = 0.f;
    for (int end = hi; end > lo; end -= kTile) {
#pragma unroll
        for (int i = 0; i < kPerLane; ++i) {
            const int t = end - 1 - (i * kWave + lane);
            sa[i * kWave + lane] = (t >= lo && t != hi - 1) ? gamma : 0.f;
            sb[i * kWave + lane] = (t >= lo) ? reward[t] : 0.f;
        }
        wave_lds_sync();
        carry = tile_scan(sa, sb, lane, carry);
        wave_lds_sync();
#pragma unroll
        for (int i = 0; i < kPerLane; ++i) {
            const int t = end - 1 - (i * kWave + lane);
            if (t >= lo) {
                const float g = sb[i * kWave + lane];
                if (ret) ret[t] = g;
                if (label) label[t] = g > 0.f ? 1.f : 0.f;
            }
        }
        wave_lds_sync();
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
            if (t < hi)
                p[i] = step_priority(td[t], rho[t], ent[t], w_td, w_rho, w_ent, inv_td_scale, inv_ent_scale, eps,
                                     truncate);
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

// pa == nullptr: targets only; otherwise the priorities are formed in the same pass.
hipError_t retrace_launch(const float* lp, const float* lm, const float* r, const float* v,
                          const float* q, const float* boot, const int* off, int B, int N, float gamma,
                          float lambda, int vtrace, float rho_bar, float c_bar, float* target, float* td,
                          float* rho, const PrioArgs* pa, hipStream_t st) {
    const unsigned blocks = (unsigned)(((long long)B * kWave + 255) / 256);
    const PrioArgs none = {nullptr, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0, nullptr, nullptr};
    auto go = [&](auto kernel) {
        hipLaunchKernelGGL(kernel, dim3(blocks), dim3(256), 0, st, lp, lm, r, v, q, boot, off, B, N, gamma, lambda,
                           rho_bar, c_bar, target, td, rho, pa ? *pa : none);
    };
    if (pa) { if (vtrace) go(k_retrace<true, true>); else go(k_retrace<false, true>); }
    else    { if (vtrace) go(k_retrace<true, false>); else go(k_retrace<false, false>); }
    return hipGetLastError();
}

hipError_t mc_returns_launch(const float* reward, const int* off, int B, int N, float gamma, float* ret,
                             float* label, hipStream_t st) {
    const unsigned blocks = (unsigned)(((long long)B * kWave + 255) / 256);
    hipLaunchKernelGGL(k_mc_returns, dim3(blocks), dim3(256), 0, st, reward, off, B, N, gamma, ret, label);
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
