// retrace_targets, compute_priorities, the two in one pass, and mc_returns (Sections 5.1, 5.2 and
// 5.3 of the DistRL paper) as ONE flat segmented scan over the flattened steps.
//
// Retrace(lambda): Delta_t = delta_t + gamma*lambda*min(1, rho_{t+1}) * Delta_{t+1} is an affine
// recurrence X -> b + a*X running backwards through each trajectory, and affine maps compose
// associatively.  A trajectory's last step takes nothing from the step after it: its map is a
// reset, and that is all that keeps trajectories apart.  So the scan does not follow trajectories.
// The N steps are cut into chunks of 256 regardless of where trajectories begin and end:
//   * a wave owns a span of consecutive chunks and walks it from the last chunk to the first.
//     In a chunk lane l holds four consecutive steps: with 16-byte aligned arrays every load and
//     store is one contiguous 16-byte access per lane, every lane is busy whatever the mix of
//     lengths, no address depends on the offsets array, and all loads of a chunk go out back to
//     back.  The scan's values at a chunk's first step stay in registers for the chunk below, and
//     so do the value estimate and ratio of that step, which the chunk below needs as "the step
//     after".  While a chunk is scanned the loads of the chunk below are already in flight.
//   * where trajectories begin and end inside a chunk is marked in the wave's own 2 KB of LDS:
//     lane i looks at trajectory top - i, walking down from the trajectory `top` that holds the
//     chunk's last step; the trajectory that holds the step before the chunk is the next `top`.
//     Only a span's first `top` is searched for: one probe around the place an even spread of
//     lengths would put it (what it reads also serves the first walk), else a 64-ary search
//     through the offsets.
//   * the value entering a span from the right is whatever the trajectory crossing its right end
//     contributes: the wave scans that trajectory's remainder first (for trajectories of up to 256
//     steps that is one chunk, whose loads go out with the span's first).  No wave ever waits for
//     another -- there is no barrier, no atomic, nothing exchanged -- and every result is a
//     fixed function of the inputs (the same bits on every run).
//   * inside a chunk: each lane composes its four maps, a 6-round shuffle scan runs down the
//     lanes, and each lane replays its four maps from the value entering it.  A reset is carried
//     as a flag and selected, never multiplied by zero, so that an infinity or NaN in one
//     trajectory cannot leak into its neighbour.
// The priorities of Section 5.3 ride along (PRIO): the per-trajectory mean is a second channel of
// the same scan, the segmented sum S_t = p_t + S_{t+1}, read off at each trajectory's first step
// by the wave that owns that step.  The Monte-Carlo return of Section 5.1 is the map
// X -> r_t + gamma*X; compute_priorities alone is the sum channel by itself.
// HBM-bound (12 to 40 bytes per step); no contraction, no MFMA.
#include "aride_device.h"

namespace aride {

constexpr int kChunk = 4 * kWave;          // steps a wave scans at a time: four per lane
constexpr int kWavesPerBlock = 4;          // independent waves in a workgroup of 256 threads
enum { kModeRetrace = 0, kModeVtrace = 1, kModeReturns = 2, kModePriorities = 3 };

struct FlatArgs {
    const float* logp_pi; const float* logp_mu; const float* reward; const float* value;
    const float* q; const float* boot;
    const float* td_in; const float* rho_in;      // kModePriorities: the stored TD errors and ratios
    const int* offsets; int B; int N;
    float gamma, lambda, rho_bar, c_bar;
    float* target; float* td; float* rho_out;     // Retrace / V-trace outputs (nullable)
    float* ret; float* label;                     // Monte-Carlo outputs (nullable)
    PrioArgs pa;
    int vec;                                      // every array is 16-byte aligned: the 16-byte-access kernels serve
};

// Section 5.3 / Appendix A.4.3: p_t = w1*|delta_t|/s_delta + w2*rho~_t + w3*H_t/s_H + eps.
__device__ __forceinline__ float step_priority(float td, float rho, float ent, const PrioArgs& pa) {
    const float r = pa.truncate ? fminf(1.f, rho) : rho;
    return pa.w_td * fabsf(td) * pa.inv_td_scale + pa.w_rho * r + pa.w_ent * ent * pa.inv_ent_scale + pa.eps;
}

// Orders this wave's LDS writes before its later LDS reads by other lanes (LDS operations of one
// wave execute in order; this only stops the compiler from moving them).
__device__ __forceinline__ void wave_lds_sync() {
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront", "local");
    __builtin_amdgcn_wave_barrier();
    __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront", "local");
}

// Steps t0 .. t0+3 of one array (t0 a multiple of 4, last = the array's last index >= 0).  No
// branch and nothing that waits, so that a chunk's loads all go out back to back:
//  VEC   (16-byte aligned arrays) one 16-byte load from the lane's own block of four or, for lanes
//        past it, from the block that holds the last step -- an aligned block with at least one
//        step in it, so the access stays inside memory the array's last page maps;
//  !VEC  four 4-byte loads from indices clamped into the array.
// Values at steps that do not exist are whatever was there; the scan never uses them.
template <bool VEC>
__device__ __forceinline__ float4 load4(const float* __restrict__ p, int t0, int last) {
    if constexpr (VEC) return *reinterpret_cast<const float4*>(p + min(t0, last & ~3));
    return make_float4(p[min(t0, last)], p[min(t0 + 1, last)], p[min(t0 + 2, last)], p[min(t0 + 3, last)]);
}
template <bool VEC>
__device__ __forceinline__ void store4(float* __restrict__ p, int t0, int limit, const float (&x)[4]) {
    if (p == nullptr) return;
    if (VEC && t0 + 3 < limit) {                     // written once, not read again by this kernel
        typedef float f32x4 __attribute__((ext_vector_type(4)));
        const f32x4 o = {x[0], x[1], x[2], x[3]};
        __builtin_nontemporal_store(o, reinterpret_cast<f32x4*>(p + t0));
        return;
    }
#pragma unroll
    for (int j = 0; j < 4; ++j) if (t0 + j < limit) p[t0 + j] = x[j];
}

// What a lane reads for its four steps.
struct LaneIn {
    float4 lp, lm, r, v, q, ent, td, rho;
};

// The chunk that starts at step c0; steps at or past `limit` (at least 1) do not exist.  Only the
// members the mode reads are set.  Nothing here branches or writes a register that is not a load's
// destination: a wave can then have several chunks' loads in flight and wait for each by itself.
template <int MODE, bool PRIO, bool VEC>
__device__ __forceinline__ LaneIn load_lane(const FlatArgs& g, int c0, int limit) {
    const int lane = threadIdx.x & 63, t0 = c0 + 4 * lane;
    LaneIn in;
    const int last = limit - 1;
    if constexpr (MODE == kModeRetrace || MODE == kModeVtrace) {
        in.lp = load4<VEC>(g.logp_pi, t0, last);
        in.lm = load4<VEC>(g.logp_mu, t0, last);
        in.r = load4<VEC>(g.reward, t0, last);
        in.v = load4<VEC>(g.value, t0, last);
        in.q = load4<VEC>(g.q ? g.q : g.value, t0, last);
    }
    if constexpr (MODE == kModeReturns) in.r = load4<VEC>(g.reward, t0, last);
    if constexpr (MODE == kModePriorities) {
        in.td = load4<VEC>(g.td_in, t0, last);
        in.rho = load4<VEC>(g.rho_in, t0, last);
    }
    if constexpr (PRIO) in.ent = load4<VEC>(g.pa.ent, t0, last);
    return in;
}

__device__ __forceinline__ float f4(const float4& v, int j) { return j == 0 ? v.x : j == 1 ? v.y : j == 2 ? v.z : v.w; }

__device__ __forceinline__ float first_lane(float x) {
    return __int_as_float(__builtin_amdgcn_readfirstlane(__float_as_int(x)));
}

__device__ __forceinline__ int wave_max_i32(int v) {
#pragma unroll
    for (int d = 32; d >= 1; d >>= 1) v = max(v, __shfl_xor(v, d, kWave));
    return v;
}

// One chunk of 256 steps starting at step c0, scanned backwards by the wave.
//  MAIN   a chunk of the wave's span: trajectory begins and ends come from the LDS marks, results
//         are stored, trajectory means are written at the begins;
//  !MAIN  a chunk of the one trajectory that runs on past the span: it ends at step `limit`-1
//         with bootstrap value `boot_end`; nothing is stored.
// carry[c]: value of channel c entering the chunk from the right; on return, its value at the
// chunk's first step (the same in every lane).
// nxt: value estimate and importance ratio at the first step of the chunk above, which this wave
// scanned just before (the step after this chunk's last); on return, those of this chunk's first step.
template <int MODE, bool PRIO, bool VEC, bool MAIN>
__device__ __forceinline__ void scan_chunk(const FlatArgs& g, const LaneIn& in, int c0, int limit,
                                           float boot_end, int* tags, const float* aux, float (&carry)[2],
                                           float (&nxt)[2]) {
    constexpr int NC = (MODE == kModePriorities ? 0 : 1) + (PRIO ? 1 : 0);
    constexpr int CS = NC - 1;                      // the sum channel, when there is one
    static_assert(NC >= 1 && NC <= 2, "one or two channels");
    const int lane = threadIdx.x & 63;
    const int t0 = c0 + 4 * lane;

    int tag[4];
    float extra[4];
    if constexpr (MAIN) {
        const int4 tg = *reinterpret_cast<const int4*>(tags + 4 * lane);
        const float4 ax = *reinterpret_cast<const float4*>(aux + 4 * lane);
        tag[0] = tg.x; tag[1] = tg.y; tag[2] = tg.z; tag[3] = tg.w;
        extra[0] = ax.x; extra[1] = ax.y; extra[2] = ax.z; extra[3] = ax.w;
        // cleared for the next chunk's marks (written later by this same wave: LDS keeps the order)
        *reinterpret_cast<int4*>(tags + 4 * lane) = make_int4(0, 0, 0, 0);
    } else {
#pragma unroll
        for (int j = 0; j < 4; ++j) { tag[j] = (t0 + j == limit - 1) ? 2 : 0; extra[j] = boot_end; }
    }
    bool valid[4], reset[4];
#pragma unroll
    for (int j = 0; j < 4; ++j) {
        valid[j] = t0 + j < limit;
        reset[j] = !valid[j] || (tag[j] & 2);      // a trajectory's last step, or no step at all
    }

    // ---- the maps X -> b + a*X of this lane's four steps, per channel
    float a[NC][4], b[NC][4];
    float rho[4], dlt[4], qv[4], prio[4];
    if constexpr (MODE == kModeRetrace || MODE == kModeVtrace) {
#pragma unroll
        for (int j = 0; j < 4; ++j) rho[j] = valid[j] ? expf(f4(in.lp, j) - f4(in.lm, j)) : 0.f;
        // the step after each of the four: the next element, the next lane's first, or the chunk above's first
        float rho_n = __shfl_down(rho[0], 1, kWave), v_n = __shfl_down(in.v.x, 1, kWave);
        if (lane == kWave - 1) {
            v_n = nxt[0];
            rho_n = (t0 + 4 < limit) ? nxt[1] : 0.f;
        }
        nxt[0] = first_lane(in.v.x);
        nxt[1] = first_lane(rho[0]);
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            qv[j] = f4(in.q, j);                    // Q, or the value again when there is no Q
            const float v_next = (tag[j] & 2) ? extra[j] : (j < 3 ? f4(in.v, j + 1) : v_n);
            dlt[j] = valid[j] ? f4(in.r, j) + g.gamma * v_next - qv[j] : 0.f;
            if constexpr (MODE == kModeVtrace) {
                a[0][j] = g.gamma * g.lambda * fminf(g.c_bar, rho[j]);
                b[0][j] = fminf(g.rho_bar, rho[j]) * dlt[j];
            } else {
                const float c_next = g.lambda * fminf(1.f, j < 3 ? rho[j + 1] : rho_n);
                a[0][j] = g.gamma * c_next;
                b[0][j] = dlt[j];
            }
            if (reset[j]) a[0][j] = 0.f;
        }
    }
    if constexpr (MODE == kModeReturns) {
#pragma unroll
        for (int j = 0; j < 4; ++j) { a[0][j] = reset[j] ? 0.f : g.gamma; b[0][j] = valid[j] ? f4(in.r, j) : 0.f; }
    }
    if constexpr (MODE == kModePriorities) {
#pragma unroll
        for (int j = 0; j < 4; ++j) { dlt[j] = f4(in.td, j); rho[j] = f4(in.rho, j); }
    }
    if constexpr (PRIO) {
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            prio[j] = valid[j] ? step_priority(dlt[j], rho[j], f4(in.ent, j), g.pa) : 0.f;
            a[CS][j] = reset[j] ? 0.f : 1.f;
            b[CS][j] = prio[j];
        }
    }

    // what does not depend on the scan goes out before it (and frees its registers)
    if constexpr (MAIN) {
        if constexpr (MODE == kModeRetrace || MODE == kModeVtrace) {
            store4<VEC>(g.td, t0, limit, dlt);
            store4<VEC>(g.rho_out, t0, limit, rho);
        }
        if constexpr (PRIO) store4<VEC>(g.pa.step_prio, t0, limit, prio);
    }

    // ---- this lane's four maps composed: X entering at step 3 -> value at step 0
    float A[NC], Bv[NC];
    bool F = reset[3];
#pragma unroll
    for (int c = 0; c < NC; ++c) { A[c] = a[c][3]; Bv[c] = b[c][3]; }
#pragma unroll
    for (int j = 2; j >= 0; --j) {
#pragma unroll
        for (int c = 0; c < NC; ++c) {
            Bv[c] = reset[j] ? b[c][j] : fmaf(a[c][j], Bv[c], b[c][j]);
            A[c] = reset[j] ? 0.f : a[c][j] * A[c];
        }
        F = F || reset[j];
    }
    // ---- suffix scan down the lanes: lane l ends with the composition of lanes l .. 63
#pragma unroll
    for (int d = 1; d < kWave; d <<= 1) {
        float pa[NC], pb[NC];
#pragma unroll
        for (int c = 0; c < NC; ++c) { pa[c] = __shfl_down(A[c], d, kWave); pb[c] = __shfl_down(Bv[c], d, kWave); }
        const int pf = __shfl_down((int)F, d, kWave);
        if (lane + d < kWave && !F) {
#pragma unroll
            for (int c = 0; c < NC; ++c) { Bv[c] = fmaf(A[c], pb[c], Bv[c]); A[c] = A[c] * pa[c]; }
            F = pf != 0;
        }
    }
    // what lanes l+1 .. 63 make of the value entering the chunk; lane 0 holds the whole chunk's composition
    const int gf = __shfl_down((int)F, 1, kWave);
    const bool f0 = __shfl((int)F, 0, kWave) != 0;
    float val[NC][4];
#pragma unroll
    for (int c = 0; c < NC; ++c) {
        const float ga = __shfl_down(A[c], 1, kWave), gb = __shfl_down(Bv[c], 1, kWave);
        const float a0 = __shfl(A[c], 0, kWave), b0 = __shfl(Bv[c], 0, kWave);
        // ---- replay the four maps from the value entering this lane
        float x = (lane == kWave - 1) ? carry[c] : (gf ? gb : fmaf(ga, carry[c], gb));
#pragma unroll
        for (int j = 3; j >= 0; --j) {
            x = reset[j] ? b[c][j] : fmaf(a[c][j], x, b[c][j]);
            val[c][j] = x;
        }
        carry[c] = f0 ? b0 : fmaf(a0, carry[c], b0);
    }

    if constexpr (MAIN) {
        if constexpr (MODE == kModeRetrace || MODE == kModeVtrace) {
            float tg[4];
#pragma unroll
            for (int j = 0; j < 4; ++j) tg[j] = qv[j] + val[0][j];
            store4<VEC>(g.target, t0, limit, tg);
        }
        if constexpr (MODE == kModeReturns) {
            float lb[4];
#pragma unroll
            for (int j = 0; j < 4; ++j) lb[j] = val[0][j] > 0.f ? 1.f : 0.f;
            store4<VEC>(g.ret, t0, limit, val[0]);
            store4<VEC>(g.label, t0, limit, lb);
        }
        if constexpr (PRIO) {
            if (g.pa.traj_prio) {
#pragma unroll
                for (int j = 0; j < 4; ++j) {
                    if ((tag[j] & 1) && valid[j]) {    // a trajectory begins here: its mean
                        const int len = (tag[j] & 2) ? 1 : __float_as_int(extra[j]);
                        g.pa.traj_prio[tag[j] >> 2] = val[CS][j] / (float)len;
                    }
                }
            }
        }
    }
}

// Each wave owns `span` consecutive chunks and walks them from the last to the first.  The loads of
// the chunk below are in flight while a chunk is scanned (two sets of registers that swap roles),
// and its marks are set while the scanned chunk's stores drain: what the wave waits for are loads
// it asked for a whole chunk earlier.
template <int MODE, bool PRIO, bool VEC>
__global__ __launch_bounds__(kWave * kWavesPerBlock) void k_flat_scan(const FlatArgs g, const int span) {
    __shared__ __attribute__((aligned(16))) int tags_all[kWavesPerBlock * kChunk];
    __shared__ __attribute__((aligned(16))) float aux_all[kWavesPerBlock * kChunk];
    const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
    const int N = g.N, B = g.B;
    // the grid is the number of spans rounded up to whole workgroups and to a multiple of 8
    // workgroups; XCD x takes the x-th eighth.  What is the same in every lane of the wave is
    // kept where the compiler can see that it is.
    const int nchunks = N > 0 ? (int)(((long long)N + kChunk - 1) / kChunk) : 1;
    const long long first_ll = (xcd_contiguous_block() * kWavesPerBlock + wave) * span;
    if (first_ll >= nchunks) return;                  // whole waves leave; there is no workgroup barrier below
    if (N <= 0) {                                     // no steps (and maybe no arrays): every trajectory is empty
        if constexpr (PRIO) {
            if (g.pa.traj_prio) for (int b = lane; b < B; b += kWave) g.pa.traj_prio[b] = 0.f;
        }
        return;
    }
    const int c_first = __builtin_amdgcn_readfirstlane((int)first_ll);
    const int c_last = min(c_first + span, nchunks) - 1;
    int* tags = tags_all + wave * kChunk;
    float* aux = aux_all + wave * kChunk;
    const int span_end = (int)min((long long)(c_last + 1) * kChunk, (long long)N);     // the span's steps end here

    // The span's last chunk, and the chunk after the span in case a trajectory runs on into it, are
    // asked for before anything else: none of their addresses depends on the offsets.
    const bool at_end = span_end >= N;
    LaneIn even = load_lane<MODE, PRIO, VEC>(g, c_last * kChunk, N), odd;
    LaneIn far;
    if (!at_end) far = load_lane<MODE, PRIO, VEC>(g, span_end, N);
    *reinterpret_cast<int4*>(tags + 4 * lane) = make_int4(0, 0, 0, 0);

    // ---- the trajectory that holds the span's last step.  The span that reaches N starts its walk
    // at the last trajectory (so that it meets the empty ones recorded at N); any other looks for
    // the smallest b with offsets[b+1] >= span_end.  offsets[B] = N >= span_end, so there is one.
    // What a lane reads of "its" trajectory in the first round of a walk down from `top`: trajectory
    // top - lane (clamped to 0 when there is none, and then not used).  Lane 0's is `top` itself.
    struct Walk { int o0, o1; float bt; };
    auto walk_loads = [&](int from) {
        const int bc = max(from - lane, 0);
        Walk w;
        w.o0 = g.offsets[bc]; w.o1 = g.offsets[bc + 1]; w.bt = g.boot ? g.boot[bc] : 0.f;
        return w;
    };
    int top = B - 1;
    Walk wk;
    bool have_wk = false;
    if (!at_end) {
        int lo = 0, n = B;
        // First a guess: were all trajectories equally long, step span_end would lie in trajectory
        // span_end * B / N.  One probe of the 64 trajectories around it settles the search whenever
        // the lengths are not too unevenly spread (one round trip to memory instead of two or three).
        {
            const int guess = (int)((long long)span_end * B / N);
            const int w0 = max(min(guess - 32, B - kWave), 0);          // window [w0, w0 + 64) inside [0, B)
            const int p = min(w0 + lane, B - 1);
            const int po0 = g.offsets[p], po1 = g.offsets[p + 1];
            const float pbt = g.boot ? g.boot[p] : 0.f;
            const unsigned long long m = __ballot(po1 >= span_end);
            // the answer is inside the window when its first trajectory fails the test (or is
            // trajectory 0) and some later one passes
            if (m != 0ull && (!(m & 1ull) || w0 == 0)) {
                lo = w0 + __ffsll((long long)m) - 1; n = 1;
                // The probe has then read what the walk over the span's last chunk wants of the
                // trajectories lo, lo - 1, .. down to w0 (a second round trip saved), and whatever
                // lies below the window lies wholly below that chunk if the window's lowest
                // trajectory ends before the chunk starts: offsets[w0 + 1] < the chunk's first step.
                const int o1_w0 = __builtin_amdgcn_readfirstlane(po1);
                if (w0 == 0 || o1_w0 < c_last * kChunk) {
                    const int j = lo - lane - w0;                   // the lane that read trajectory lo - lane
                    const int src = max(j, 0);
                    wk.o0 = __shfl(po0, src, kWave); wk.o1 = __shfl(po1, src, kWave); wk.bt = __shfl(pbt, src, kWave);
                    if (j < 0) { wk.o0 = -1; wk.o1 = -1; }          // reads as: empty, and below every chunk
                    have_wk = true;
                }
            }
        }
        // Else a 64-ary search: each round keeps the sixty-fourth of the candidates [lo, lo+n) that holds it.
        while (n > 1) {
            const int stride = (n + kWave - 1) >> 6;
            const int p = (int)min((long long)lo + (long long)(lane + 1) * stride - 1, (long long)lo + n - 1);
            const unsigned long long m = __ballot(g.offsets[p + 1] >= span_end);
            const int f = m ? __ffsll((long long)m) - 1 : kWave - 1;   // non-decreasing offsets: false .. false true .. true
            const int nlo = (int)min((long long)lo + (long long)f * stride, (long long)lo + n - 1);
            const int nhi = (int)min((long long)lo + (long long)(f + 1) * stride, (long long)lo + n);
            n = max(nhi - nlo, 1);
            lo = nlo;
        }
        top = __builtin_amdgcn_readfirstlane(lo);
    }
    // Marks the begins and ends of the trajectories that touch chunk c, walking down from the
    // trajectory `from` that holds the chunk's last step: lane i takes trajectory from - i,
    // from - i - 64, .. until one lies wholly below the chunk (wk: what walk_loads(from) read).
    // A mark is (trajectory << 2) | 1 at a first step | 2 at a last step; beside it the bootstrap
    // value (at an end) or the length (at a begin that is not also the end).  Returns the
    // trajectory that holds the step before the chunk (-1: none).
    auto mark_chunk = [&](int c, int from, Walk wk) {
        const int c0 = c * kChunk;
        const int c_end = (int)min((long long)c0 + kChunk, (long long)N);
        int below = -1;
        bool first = true;
        for (int b = from - lane; b >= 0; b -= kWave) {
            if (!first) wk = walk_loads(b + lane);    // (b + lane) - lane = b
            first = false;
            const int o0 = wk.o0, o1 = wk.o1;
            const bool empty = o1 <= o0;
            if (!empty && o0 < c0 && c0 <= o1) below = b;
            if (o1 < c0 || (o1 == c0 && !empty)) break;        // wholly below the chunk, and so are all before it
            if (empty) {                              // mean priority 0, written by the chunk that owns position o0
                if constexpr (PRIO) {
                    if (g.pa.traj_prio && ((o0 >= c0 && o0 < c_end) || (o0 >= N && c_end >= N))) g.pa.traj_prio[b] = 0.f;
                }
            } else {
                const int ps = o0 - c0, pe = o1 - 1 - c0;
                if (ps == pe) {
                    if (ps >= 0 && ps < kChunk) { tags[ps] = (b << 2) | 3; aux[ps] = wk.bt; }
                } else {
                    if (ps >= 0 && ps < kChunk) { tags[ps] = (b << 2) | 1; aux[ps] = __int_as_float(o1 - o0); }
                    if (pe >= 0 && pe < kChunk) { tags[pe] = (b << 2) | 2; aux[pe] = wk.bt; }
                }
            }
        }
        below = __builtin_amdgcn_readfirstlane(wave_max_i32(below));
        wave_lds_sync();
        return below;
    };
    if (!have_wk) wk = walk_loads(top);
    wave_lds_sync();
    float carry[2] = {0.f, 0.f};
    // the step after the span's last: the first of the chunk asked for above (a far chunk scanned
    // below leaves the same two values)
    float nxt[2] = {0.f, 0.f};
    if constexpr (MODE == kModeRetrace || MODE == kModeVtrace) {
        if (!at_end) { nxt[0] = first_lane(far.v.x); nxt[1] = expf(first_lane(far.lp.x) - first_lane(far.lm.x)); }
    }
    // ---- a trajectory that runs on past the span is scanned first, from its end down to the span
    if (!at_end) {
        const int o0 = __shfl(wk.o0, 0, kWave), o1 = min(__shfl(wk.o1, 0, kWave), N);
        if (o0 < span_end && o1 > span_end) {
            const float boot_end = __shfl(wk.bt, 0, kWave);
            const int nfar = (int)(((long long)o1 - span_end + kChunk - 1) / kChunk);
            for (int m = nfar - 1; m >= 0; --m) {
                const int c0 = (int)((long long)span_end + (long long)m * kChunk);   // span_end is a multiple of 256 here
                if (nfar > 1) far = load_lane<MODE, PRIO, VEC>(g, c0, o1);           // else: loaded above already
                scan_chunk<MODE, PRIO, VEC, false>(g, far, c0, o1, boot_end, tags, aux, carry, nxt);
            }
        }
    }
    // ---- the span.  Before a chunk is scanned its marks are set and `top` is the trajectory that
    // holds the step before it.  One turn: ask for the next chunk's offsets and data (the span's
    // first chunk once more when there is no next: loads that are not used, and no branch), scan
    // this chunk, then set the next chunk's marks.  (A last turn of its own, with nothing asked
    // for, costs 40 more registers and gains nothing.)
    int c = c_last;
    top = mark_chunk(c, top, wk);
    // false once the span's first chunk has been scanned
    auto turn = [&](const LaneIn& cur, LaneIn& next) {
        wk = walk_loads(top);
        next = load_lane<MODE, PRIO, VEC>(g, max(c - 1, c_first) * kChunk, N);
        scan_chunk<MODE, PRIO, VEC, true>(g, cur, c * kChunk, N, 0.f, tags, aux, carry, nxt);
        if (--c < c_first) return false;
        top = mark_chunk(c, top, wk);
        return true;
    };
    // (the first turn stands outside the loop so that the loop is entered, like it is repeated,
    // with a turn's loads and stores in flight and nothing else)
    if (!turn(even, odd)) return;
    for (;;) {
        if (!turn(odd, even)) return;
        if (!turn(even, odd)) return;
    }
}

// compute_priorities without a per-trajectory output: the step priorities alone, no trajectory
// structure is looked at; a chunk per wave.
template <bool VEC>
__global__ __launch_bounds__(kWave * kWavesPerBlock) void k_step_priorities(const FlatArgs g) {
    const int N = g.N;
    const long long chunk = xcd_contiguous_block() * kWavesPerBlock + (threadIdx.x >> 6);
    if (chunk * kChunk >= N) return;
    const int c0 = (int)(chunk * kChunk), t0 = c0 + 4 * (int)(threadIdx.x & 63);
    const LaneIn in = load_lane<kModePriorities, true, VEC>(g, c0, N);
    float prio[4];
#pragma unroll
    for (int j = 0; j < 4; ++j) prio[j] = step_priority(f4(in.td, j), f4(in.rho, j), f4(in.ent, j), g.pa);
    store4<VEC>(g.pa.step_prio, t0, N, prio);
}

// Chunks per wave: a fixed number of waves whatever the batch, a chunk per wave for small batches.
// With fewer waves the chip is not full, with many more the spans get short and a wave's search and
// its look past its span's end stop being a small part of its work.  Measured on 0.66 M to 84 M
// steps: about 3000 waves for the Retrace and V-trace scans (4 to 5 waves fit a SIMD at their
// register count), about 6000 for the lighter Monte-Carlo and priority scans (6 to 8 fit).
constexpr long long kTargetWavesRetrace = 3072, kTargetWavesLight = 6144, kMaxSpan = 256;

template <int MODE, bool PRIO>
static hipError_t flat_launch(const FlatArgs& g, hipStream_t st) {
    const long long nchunks = g.N > 0 ? ((long long)g.N + kChunk - 1) / kChunk : 1;
    constexpr long long kTargetWaves = (MODE == kModeReturns || MODE == kModePriorities) ? kTargetWavesLight : kTargetWavesRetrace;
    long long span = (nchunks + kTargetWaves - 1) / kTargetWaves;
    if (span > kMaxSpan) span = kMaxSpan;
    const long long nwaves = (nchunks + span - 1) / span;
    const dim3 grid(round_up_8((unsigned)((nwaves + kWavesPerBlock - 1) / kWavesPerBlock)));
    const dim3 block(kWave * kWavesPerBlock);
    if (g.vec) hipLaunchKernelGGL((k_flat_scan<MODE, PRIO, true>), grid, block, 0, st, g, (int)span);
    else hipLaunchKernelGGL((k_flat_scan<MODE, PRIO, false>), grid, block, 0, st, g, (int)span);
    return hipGetLastError();
}

static int all_aligned16(std::initializer_list<const void*> ps) {
    for (const void* p : ps) if (p && ((uintptr_t)p & 15)) return 0;
    return 1;
}

// pa == nullptr: targets only; otherwise the priorities are formed in the same pass.
hipError_t retrace_launch(const float* lp, const float* lm, const float* r, const float* v,
                          const float* q, const float* boot, const int* off, int B, int N, float gamma,
                          float lambda, int vtrace, float rho_bar, float c_bar, float* target, float* td,
                          float* rho, const PrioArgs* pa, hipStream_t st) {
    FlatArgs g = {};
    g.logp_pi = lp; g.logp_mu = lm; g.reward = r; g.value = v; g.q = q; g.boot = boot;
    g.offsets = off; g.B = B; g.N = N;
    g.gamma = gamma; g.lambda = lambda; g.rho_bar = rho_bar; g.c_bar = c_bar;
    g.target = target; g.td = td; g.rho_out = rho;
    if (pa) g.pa = *pa;
    g.vec = all_aligned16({lp, lm, r, v, q, target, td, rho, pa ? pa->ent : nullptr, pa ? pa->step_prio : nullptr});
    if (pa) return vtrace ? flat_launch<kModeVtrace, true>(g, st) : flat_launch<kModeRetrace, true>(g, st);
    return vtrace ? flat_launch<kModeVtrace, false>(g, st) : flat_launch<kModeRetrace, false>(g, st);
}

hipError_t mc_returns_launch(const float* reward, const int* off, int B, int N, float gamma, float* ret,
                             float* label, hipStream_t st) {
    FlatArgs g = {};
    g.reward = reward; g.offsets = off; g.B = B; g.N = N; g.gamma = gamma; g.ret = ret; g.label = label;
    g.vec = all_aligned16({reward, ret, label});
    return flat_launch<kModeReturns, false>(g, st);
}

hipError_t priorities_launch(const float* td, const float* rho, const float* ent, const int* off,
                             int B, int N, float w_td, float w_rho, float w_ent, float td_scale,
                             float ent_scale, float eps, int truncate, float* step_prio,
                             float* traj_prio, hipStream_t st) {
    FlatArgs g = {};
    g.td_in = td; g.rho_in = rho; g.offsets = off; g.B = B; g.N = N;
    g.pa = PrioArgs{ent, w_td, w_rho, w_ent, 1.f / td_scale, 1.f / ent_scale, eps, truncate, step_prio, traj_prio};
    g.vec = all_aligned16({td, rho, ent, step_prio});
    if (traj_prio) return flat_launch<kModePriorities, true>(g, st);
    if (!step_prio || N == 0) return hipSuccess;
    const long long nchunks = ((long long)N + kChunk - 1) / kChunk;
    const dim3 grid(round_up_8((unsigned)((nchunks + kWavesPerBlock - 1) / kWavesPerBlock)));
    if (g.vec) hipLaunchKernelGGL(k_step_priorities<true>, grid, dim3(kWave * kWavesPerBlock), 0, st, g);
    else hipLaunchKernelGGL(k_step_priorities<false>, grid, dim3(kWave * kWavesPerBlock), 0, st, g);
    return hipGetLastError();
}

}  // namespace aride
