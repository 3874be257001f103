// score_logits: per logit row, one pass over bf16 data producing the chosen token's
// log-probability and the row's Shannon entropy (Section 5.1, eq. (1) of the DistRL
// paper: log pi(a_t|s_t) and the regulariser H(pi(.|s_t)) of a token-level policy).
//
// Design for gfx950:
//  * HBM-bound streaming reduction; nothing here is a contraction, so no MFMA.
//  * Who reads what: rows of 16 KB and more belong to one workgroup of 4, 8 or 16 waves
//    (k_score_rows_split; rows from 16, 48, 192 KB), each wave reducing a contiguous share of 6
//    to 16 KB of the row; shorter rows take one wave each, four rows to a workgroup
//    (k_score_rows).  Both map blockIdx to rows so that each of the chip's 8 XCDs streams one
//    contiguous eighth of the rows.  Each lane issues 16-byte non-temporal loads (8 bf16), four of
//    them back to back, so 4 KB per wave are in flight.  On 64 KB rows: one wave per row and a
//    plain mapping 84 % of the HBM peak, XCD-contiguous rows 86 %, 8 waves per row 87-90 %.
//  * Every logit is read once.  Each lane keeps an online log-sum-exp state in base-2
//    units against a lazily updated reference k (k = ref*log2e):
//        s = sum 2^(x*log2e - k),   t = sum 2^(x*log2e - k) * (x*log2e - k)
//    The reference only moves when a group's maximum exceeds it by more than kWindow,
//    so the rescale branch is rarely taken; the exact running maximum is kept
//    separately and all lanes, then all waves of a row, are brought to the common reference
//    once at the end.
//    Terms above the reference are rounded at ulp(x*log2e - k), so the window also bounds
//    the relative error of the largest terms: 1.7e-7 at 4 nats (6.6e-7 at 16, at equal speed).
//  * logp = ln2*(x_tok*log2e - K) - ln S  and  H = ln S - ln2*T/S  hold for any common
//    reference K, so rounding in K cancels; and because x*log2e - k is one fused
//    multiply-add (exact product, one rounding of the small result) the accuracy does not
//    depend on how large the logits themselves are.
//  * Per element: 1 unpack, 1/2 max3, 1/2 min3, 1 fma, 1 exp2, 1 add, 1 fma: the vector ALUs
//    are busy 98 % of the kernel's time, close behind memory -- which is why a sweep takes up to
//    40 % longer while the chip's power management holds the shader clock down at the start of
//    a sustained load.
#include "aride_device.h"
#include <hip/hip_ext.h>

namespace aride {

constexpr int kScoreUnroll = 4;     // 16-byte loads in flight per lane and batch
constexpr int kScoreWaves = 4;      // waves (= rows) per workgroup of the one-wave-per-row kernel

// 16-byte vectors per row from which a row is shared by 4, 8, 16 waves (16 KB, 48 KB, 192 KB rows)
constexpr int kSplit4MinVec = 1024, kSplit8MinVec = 3072, kSplit16MinVec = 12288;

constexpr float kLog2e = 1.4426950408889634f;
constexpr float kLn2 = 0.6931471805599453f;
constexpr float kWindow = 4.0f;      // natural-log units a group max may exceed the reference
constexpr float kHugeNeg = -1.0e30f; // below this x*log2e may overflow: take the guarded path

struct LaneState {
    float ref;   // reference logit (a value seen in this lane, or -inf before the first)
    float negk;  // -(ref * log2e)
    float s0, s1, t0, t1;
    float mx;    // exact running maximum
};

__device__ __forceinline__ void lane_init(LaneState& a) {
    a.ref = -INFINITY; a.negk = INFINITY; a.s0 = a.s1 = a.t0 = a.t1 = 0.f; a.mx = -INFINITY;
}

__device__ __forceinline__ void lane_rebase(LaneState& a, float gm) {
    float knew = gm * kLog2e;
    float d = -a.negk - knew;   // old k - new k  (<= 0, or -inf on first use)
    float r = fast_exp2(d);
    float s = a.s0 + a.s1, t = a.t0 + a.t1;
    a.t0 = (s != 0.f) ? r * fmaf(d, s, t) : 0.f;
    a.s0 = (s != 0.f) ? s * r : 0.f;
    a.s1 = 0.f; a.t1 = 0.f;
    a.ref = gm; a.negk = -knew;
}

template <int NE>
__device__ __forceinline__ void lane_accumulate(LaneState& a, const float (&x)[NE]) {
    float gm = x[0], gn = x[0];
    if constexpr (NE > 1) {
#pragma unroll
        for (int j = 1; j + 1 < NE; j += 2) {
            gm = __builtin_fmaxf(__builtin_fmaxf(gm, x[j]), x[j + 1]);   // v_max3_f32
            gn = __builtin_fminf(__builtin_fminf(gn, x[j]), x[j + 1]);   // v_min3_f32
        }
        if constexpr ((NE & 1) == 0) { gm = fmaxf(gm, x[NE - 1]); gn = fminf(gn, x[NE - 1]); }
    }
    a.mx = fmaxf(a.mx, gm);
    // a reference below kHugeNeg would overflow k = ref*log2e; such logits count as -inf
    if (gm > a.ref + kWindow) lane_rebase(a, fmaxf(gm, kHugeNeg));
    if (gn > kHugeNeg) {
#pragma unroll
        for (int j = 0; j < NE; ++j) {
            float y = fmaf(x[j], kLog2e, a.negk);
            float e = fast_exp2(y);
            if (j & 1) { a.s1 += e; a.t1 = fmaf(e, y, a.t1); }
            else       { a.s0 += e; a.t0 = fmaf(e, y, a.t0); }
        }
    } else {
        // -inf (masked vocabulary entries) or huge negative logits: their probability
        // is exactly 0 and they add nothing to the entropy sum.
        if (gm == -INFINITY) return;   // nothing but -inf here, and maybe no reference yet
#pragma unroll
        for (int j = 0; j < NE; ++j) {
            float y = fmaf(x[j], kLog2e, a.negk);
            float e = fast_exp2(y);
            a.s0 += e;
            a.t0 += (e > 0.f) ? e * y : 0.f;
        }
    }
}

typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));

__device__ __forceinline__ void unpack8(const u32x4& v, float* x) {
    x[0] = bits_to_float(v.x << 16); x[1] = bits_to_float(v.x & 0xffff0000u);
    x[2] = bits_to_float(v.y << 16); x[3] = bits_to_float(v.y & 0xffff0000u);
    x[4] = bits_to_float(v.z << 16); x[5] = bits_to_float(v.z & 0xffff0000u);
    x[6] = bits_to_float(v.w << 16); x[7] = bits_to_float(v.w & 0xffff0000u);
}

__device__ __forceinline__ u32x4 load16(const u32x4* p) {
    return __builtin_nontemporal_load(p);   // streamed once: keep it out of the caches' way (10 points of peak)
}

template <int NV>
__device__ __forceinline__ void accumulate_batch(LaneState& a, const u32x4 (&v)[NV]) {
    float x[8 * NV];
#pragma unroll
    for (int u = 0; u < NV; ++u) unpack8(v[u], x + 8 * u);
    lane_accumulate<8 * NV>(a, x);
}

// Brings a lane's (s, t) from its own reference to the common one: K = kc (log2 units).
__device__ __forceinline__ void to_common(float negk, float s, float t, float kc, float& so, float& to) {
    float d = -negk - kc;
    float r = fast_exp2(d);
    so = (s != 0.f) ? s * r : 0.f;
    to = (s != 0.f) ? r * fmaf(d, s, t) : 0.f;
}

template <int UNROLL>
__global__ __launch_bounds__(64 * kScoreWaves) void k_score_rows(
    const uint16_t* __restrict__ logits, long long row0, long long R, int V, long long row_stride,
    const int* __restrict__ tokens, float* __restrict__ tok_logp, float* __restrict__ tok_ent,
    uint32_t* __restrict__ status) {
    const int lane = threadIdx.x & 63;
    // the grid is a multiple of 8 and XCD x takes the x-th eighth of the rows: each XCD, with its own
    // L2 and its own paths to memory, streams one contiguous region instead of every eighth 256 KB
    const long long row = row0 + xcd_contiguous_block() * kScoreWaves + (threadIdx.x >> 6);   // this launch: rows row0 ..
    if (row >= R) return;   // whole waves leave together; the kernel has no workgroup barrier

    const int tok = tokens[row];
    const bool live = tok >= 0 && tok < V;
    if (tok >= V && lane == 0) atomicOr(status, 0x1u);

    LaneState a;
    lane_init(a);
    float xtok = 0.f;
    if (live) {
        const uint16_t* p = logits + row * row_stride;
        if (lane == 0) xtok = bits_to_float(((uint32_t)p[tok]) << 16);
        // Elements before the first 16-byte boundary, the aligned 8-element vectors, the rest.
        int head = (int)(((16u - (uint32_t)((uintptr_t)p & 15u)) & 15u) >> 1);
        if (head > V) head = V;
        const int nvec = (V - head) >> 3;
        const int tail0 = head + (nvec << 3);
        const u32x4* pv = reinterpret_cast<const u32x4*>(p + head);

        int i = lane;
        for (; i + (UNROLL - 1) * kWave < nvec; i += UNROLL * kWave) {
            u32x4 v[UNROLL];
#pragma unroll
            for (int u = 0; u < UNROLL; ++u) v[u] = load16(pv + i + u * kWave);
            accumulate_batch<UNROLL>(a, v);
        }
        for (; i < nvec; i += kWave) {
            u32x4 v[1] = {load16(pv + i)};
            accumulate_batch<1>(a, v);
        }
        if (lane < head) {
            float x[1] = {bits_to_float(((uint32_t)p[lane]) << 16)};
            lane_accumulate<1>(a, x);
        }
        if (lane < V - tail0) {   // fewer than 8 elements remain (not tail0 + lane < V: that sum can pass 2^31)
            float x[1] = {bits_to_float(((uint32_t)p[tail0 + lane]) << 16)};
            lane_accumulate<1>(a, x);
        }
    }

    // Merge the 64 lane states: common reference = exact row maximum (in log2 units).
    const float M = wave_max(a.mx);
    const float kc = M * kLog2e;
    float s, t;
    to_common(a.negk, a.s0 + a.s1, a.t0 + a.t1, kc, s, t);
    s = wave_sum(s);
    t = wave_sum(t);

    if (lane == 0) {
        float lp = 0.f, en = 0.f;
        if (live) {
            const float logS = logf(s);
            lp = kLn2 * fmaf(xtok, kLog2e, -kc) - logS;
            en = logS - kLn2 * t / s;
        }
        if (tok_logp) tok_logp[row] = lp;
        if (tok_ent) tok_ent[row] = en;
    }
}

// The sweep for long rows: one workgroup of WPR waves per row, each wave reducing a contiguous
// share of the row's 16-byte vectors (wave 0 also takes the unaligned head and tail); the WPR
// (max, s, t) states meet in LDS and are merged exactly as the 64 lane states are.  Fewer rows
// are open at a time on each XCD than with one wave per row (2.5 % faster on 64 KB rows, 4 % on
// 304 KB rows), and a batch of few rows still fills the chip (2560 rows would otherwise be 2.5
// waves per SIMD).
template <int UNROLL, int WPR>
__global__ __launch_bounds__(64 * WPR) void k_score_rows_split(
    const uint16_t* __restrict__ logits, long long row0, long long R, int V, long long row_stride,
    const int* __restrict__ tokens, float* __restrict__ tok_logp, float* __restrict__ tok_ent,
    uint32_t* __restrict__ status) {
    __shared__ float part[WPR][3];
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const long long row = row0 + xcd_contiguous_block();   // the grid is this launch's rows rounded up to a multiple of 8
    if (row >= R) return;                           // the whole workgroup leaves

    const int tok = tokens[row];
    const bool live = tok >= 0 && tok < V;
    if (tok >= V && threadIdx.x == 0) atomicOr(status, 0x1u);

    LaneState a;
    lane_init(a);
    float xtok = 0.f;
    if (live) {
        const uint16_t* p = logits + row * row_stride;
        int head = (int)(((16u - (uint32_t)((uintptr_t)p & 15u)) & 15u) >> 1);
        if (head > V) head = V;
        const int nvec = (V - head) >> 3;
        const int tail0 = head + (nvec << 3);
        const u32x4* pv = reinterpret_cast<const u32x4*>(p + head);
        const int share = (((nvec + WPR - 1) / WPR) + kWave - 1) & ~(kWave - 1);   // whole 1 KB pieces per wave
        const int end = min(nvec, (wave + 1) * share);

        int i = wave * share + lane;
        for (; i + (UNROLL - 1) * kWave < end; i += UNROLL * kWave) {
            u32x4 v[UNROLL];
#pragma unroll
            for (int u = 0; u < UNROLL; ++u) v[u] = load16(pv + i + u * kWave);
            accumulate_batch<UNROLL>(a, v);
        }
        for (; i < end; i += kWave) {
            u32x4 v[1] = {load16(pv + i)};
            accumulate_batch<1>(a, v);
        }
        if (wave == 0) {
            if (lane == 0) xtok = bits_to_float(((uint32_t)p[tok]) << 16);
            if (lane < head) {
                float x[1] = {bits_to_float(((uint32_t)p[lane]) << 16)};
                lane_accumulate<1>(a, x);
            }
            if (lane < V - tail0) {   // (not tail0 + lane < V: that sum can pass 2^31)
                float x[1] = {bits_to_float(((uint32_t)p[tail0 + lane]) << 16)};
                lane_accumulate<1>(a, x);
            }
        }
    }
    // this wave's share: common reference = its exact maximum
    const float Mw = wave_max(a.mx);
    float s, t;
    to_common(a.negk, a.s0 + a.s1, a.t0 + a.t1, Mw * kLog2e, s, t);
    s = wave_sum(s);
    t = wave_sum(t);
    if (lane == 0) { part[wave][0] = Mw; part[wave][1] = s; part[wave][2] = t; }
    __syncthreads();             // every wave of the workgroup gets here: nothing above returns

    // lane w of wave 0 brings wave w's state to the row's reference; the row of 16 lanes sums them
    if (wave == 0) {
        float M = part[0][0];
#pragma unroll
        for (int w = 1; w < WPR; ++w) M = fmaxf(M, part[w][0]);
        const float kc = M * kLog2e;
        float S = 0.f, T = 0.f;
        if (lane < WPR) to_common(-(part[lane][0] * kLog2e), part[lane][1], part[lane][2], kc, S, T);
        S = row_sum_f32(S);
        T = row_sum_f32(T);
        if (lane == 0) {
            float lp = 0.f, en = 0.f;
            if (live) {
                const float logS = logf(S);
                lp = kLn2 * fmaf(xtok, kLog2e, -kc) - logS;
                en = logS - kLn2 * T / S;
            }
            if (tok_logp) tok_logp[row] = lp;
            if (tok_ent) tok_ent[row] = en;
        }
    }
}

// Per-step sums of the A per-token values: one wave per step, lanes stride over the step's
// rows (contiguous 4-byte loads), fp64 running sums combined in a fixed butterfly order and
// rounded to fp32 once.  log pi(a|s) of a long action is a large number whose absolute error
// passes one-to-one into the relative error of rho, hence the fp64 accumulation.
__global__ __launch_bounds__(256) void k_step_sums(
    const float* __restrict__ tok_logp, const float* __restrict__ tok_ent, long long N, int A,
    float* __restrict__ step_logp, float* __restrict__ step_ent) {
    const int lane = threadIdx.x & 63;
    const long long n = ((long long)blockIdx.x * blockDim.x + threadIdx.x) >> 6;
    if (n >= N) return;   // whole waves leave together
    double sl = 0.0, se = 0.0;
    const long long base = n * A;
    for (int j = lane; j < A; j += kWave) {
        if (step_logp) sl += (double)tok_logp[base + j];
        if (step_ent) se += (double)tok_ent[base + j];
    }
#pragma unroll
    for (int d = 32; d >= 1; d >>= 1) {
        sl += __shfl_xor(sl, d, kWave);
        se += __shfl_xor(se, d, kWave);
    }
    if (lane == 0) {
        if (step_logp) step_logp[n] = (float)sl;
        if (step_ent) step_ent[n] = (float)se;
    }
}

// A sweep kernel goes out with the two events attached to its own dispatch, or plainly.
template <typename... Args, typename F = void (*)(Args...)>
static void launch_sweep(F kernel, dim3 grid, dim3 block, hipStream_t st, hipEvent_t start, hipEvent_t stop,
                         Args... args) {
    if (start || stop) hipExtLaunchKernelGGL(kernel, grid, block, 0, st, start, stop, 0, args...);
    else hipLaunchKernelGGL(kernel, grid, block, 0, st, args...);
}

// Row sweep, then (when a per-step output is wanted) the per-step sums of the per-token arrays.
// With events, they are attached to the dispatch of the row sweep itself: the time between
// them is that kernel's execution time, with no marker packets on the stream around it.
// Long rows are shared by 4, 8 or 16 waves so that each wave gets 6 to 16 KB of the row
// (measured on 64 KB and 304 KB rows: 8 and 16 waves are the fastest there; a wave left with
// 4 KB is much slower); rows below 16 KB take the one-wave-per-row kernel.
hipError_t score_logits_launch(const uint16_t* logits, long long R, int V, long long stride,
                               const int* tokens, int A, float* tok_logp, float* tok_ent,
                               float* step_logp, float* step_ent, uint32_t* status, hipStream_t st,
                               hipEvent_t sweep_start, hipEvent_t sweep_stop) {
    constexpr int U = kScoreUnroll;
    const int nvec = V >> 3;                                  // 16-byte vectors per row
    const int wpr = nvec >= kSplit16MinVec ? 16 : nvec >= kSplit8MinVec ? 8 : nvec >= kSplit4MinVec ? 4 : 1;
    // rows one launch may cover (64 work-items per row and wave); more rows go out slice by slice,
    // the events, when given, on the first and the last slice
    const long long slice = kMaxLaunchThreads / (64 * wpr);
    for (long long row0 = 0; row0 < R; row0 += slice) {
        const long long rows = R - row0 < slice ? R - row0 : slice;
        hipEvent_t ev0 = row0 == 0 ? sweep_start : nullptr, ev1 = row0 + rows >= R ? sweep_stop : nullptr;
        const dim3 rows8(round_up_8((unsigned)rows));
        if (wpr == 16)
            launch_sweep(k_score_rows_split<U, 16>, rows8, dim3(1024), st, ev0, ev1, logits, row0, R, V, stride, tokens,
                         tok_logp, tok_ent, status);
        else if (wpr == 8)
            launch_sweep(k_score_rows_split<U, 8>, rows8, dim3(512), st, ev0, ev1, logits, row0, R, V, stride, tokens,
                         tok_logp, tok_ent, status);
        else if (wpr == 4)
            launch_sweep(k_score_rows_split<U, 4>, rows8, dim3(256), st, ev0, ev1, logits, row0, R, V, stride, tokens,
                         tok_logp, tok_ent, status);
        else
            launch_sweep(k_score_rows<U>, dim3(round_up_8((unsigned)((rows + kScoreWaves - 1) / kScoreWaves))),
                         dim3(64 * kScoreWaves), st, ev0, ev1, logits, row0, R, V, stride, tokens, tok_logp, tok_ent, status);
    }
    hipError_t err = hipGetLastError();
    if (err != hipSuccess || (!step_logp && !step_ent)) return err;
    const long long N = R / A;
    hipLaunchKernelGGL(k_step_sums, dim3((unsigned)((N * kWave + 255) / 256)), dim3(256), 0, st,
                       tok_logp, tok_ent, N, A, step_logp, step_ent);
    return hipGetLastError();
}

}  // namespace aride
