// score_logits: per logit row, one pass over bf16 data producing the chosen token's
// log-probability and the row's Shannon entropy (Section 5.1, eq. (1) of the DistRL
// paper: log pi(a_t|s_t) and the regulariser H(pi(.|s_t)) of a token-level policy).
//
// Design for gfx950:
//  * HBM-bound streaming reduction; nothing here is a contraction, so no MFMA.
//  * One row is swept by WPR waves (1, 2 or 4); each lane issues 16-byte loads
//    (8 bf16), UNROLL of them back to back so several KB per wave are in flight.
//  * Every logit is read once.  Each lane keeps an online log-sum-exp state in base-2
//    units against a lazily updated reference k (k = ref*log2e):
//        s = sum 2^(x*log2e - k),   t = sum 2^(x*log2e - k) * (x*log2e - k)
//    The reference only moves when a group's maximum exceeds it by more than kWindow,
//    so the rescale branch is almost never taken; the exact running maximum is kept
//    separately and all lanes are brought to the common reference once at the end.
//  * logp = ln2*(x_tok*log2e - K) - ln S  and  H = ln S - ln2*T/S  hold for any common
//    reference K, so rounding in K cancels.
//  * Per element: 1 unpack, 1/2 max3, 1/2 min3, 1 fma, 1 exp2, 1 add, 1 fma.
#include "aride_device.h"

namespace aride {

#ifndef ARIDE_SCORE_WPR
#define ARIDE_SCORE_WPR 1   // waves per logit row (1, 2 or 4)
#endif

constexpr float kLog2e = 1.4426950408889634f;
constexpr float kLn2 = 0.6931471805599453f;
constexpr float kWindow = 16.0f;     // natural-log units a group max may exceed the reference
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
    a.t0 = (s > 0.f) ? r * fmaf(d, s, t) : 0.f;
    a.s0 = (s > 0.f) ? s * r : 0.f;
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
    if (gm > a.ref + kWindow) lane_rebase(a, gm);
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

// Brings a lane's (s, t) from its own reference to the common one: K = kc (log2 units).
__device__ __forceinline__ void to_common(float negk, float s, float t, float kc, float& so, float& to) {
    float d = -negk - kc;
    float r = fast_exp2(d);
    so = (s > 0.f) ? s * r : 0.f;
    to = (s > 0.f) ? r * fmaf(d, s, t) : 0.f;
}

template <int WPR, int UNROLL>
__global__ __launch_bounds__(256) void k_score_rows(
    const uint16_t* __restrict__ logits, long long R, int V, long long row_stride,
    const int* __restrict__ tokens, float* __restrict__ tok_logp, float* __restrict__ tok_ent,
    uint32_t* __restrict__ status) {
    constexpr int kRowsPerBlock = 4 / WPR;
    constexpr int kTPR = kWave * WPR;  // threads per row
    __shared__ float sh[WPR > 1 ? 4 * 3 : 1];

    const int wave = threadIdx.x >> 6;
    const int lane = threadIdx.x & 63;
    const long long row = (long long)blockIdx.x * kRowsPerBlock + wave / WPR;
    const int sub = wave % WPR;         // which wave of the row
    const int l = sub * kWave + lane;   // thread index within the row
    const bool row_ok = row < R;

    int tok = row_ok ? tokens[row] : -1;
    const bool live = row_ok && tok >= 0 && tok < V;
    if (row_ok && tok >= V && l == 0) atomicOr(status, 0x1u);

    LaneState a;
    lane_init(a);
    float xtok = 0.f;
    if (live) {
        const uint16_t* p = logits + row * row_stride;
        if (l == 0) xtok = bits_to_float(((uint32_t)p[tok]) << 16);
        // Elements before the first 16-byte boundary, the aligned 8-element vectors, the rest.
        int head = (int)(((16u - (uint32_t)((uintptr_t)p & 15u)) & 15u) >> 1);
        if (head > V) head = V;
        const int nvec = (V - head) >> 3;
        const int tail0 = head + (nvec << 3);
        const u32x4* pv = reinterpret_cast<const u32x4*>(p + head);

        int i = l;
        for (; i + (UNROLL - 1) * kTPR < nvec; i += UNROLL * kTPR) {
            u32x4 v[UNROLL];
#pragma unroll
            for (int u = 0; u < UNROLL; ++u) v[u] = __builtin_nontemporal_load(pv + i + u * kTPR);
            float x[8 * UNROLL];
#pragma unroll
            for (int u = 0; u < UNROLL; ++u) unpack8(v[u], x + 8 * u);
            lane_accumulate<8 * UNROLL>(a, x);
        }
        for (; i < nvec; i += kTPR) {
            u32x4 v = __builtin_nontemporal_load(pv + i);
            float x[8];
            unpack8(v, x);
            lane_accumulate<8>(a, x);
        }
        if (l < head) {
            float x[1] = {bits_to_float(((uint32_t)p[l]) << 16)};
            lane_accumulate<1>(a, x);
        }
        if (tail0 + l < V) {   // fewer than 8 elements remain
            float x[1] = {bits_to_float(((uint32_t)p[tail0 + l]) << 16)};
            lane_accumulate<1>(a, x);
        }
    }

    // Wave-level merge: common reference = exact wave maximum.
    float M = wave_max(a.mx);
    float kc = M * kLog2e;
    float s, t;
    to_common(a.negk, a.s0 + a.s1, a.t0 + a.t1, kc, s, t);
    s = wave_sum(s);
    t = wave_sum(t);

    if constexpr (WPR > 1) {
        if (lane == 0) { sh[wave * 3 + 0] = M; sh[wave * 3 + 1] = s; sh[wave * 3 + 2] = t; }
        __syncthreads();
        const int w0 = (wave / WPR) * WPR;
        float Mb = sh[w0 * 3];
#pragma unroll
        for (int w = 1; w < WPR; ++w) Mb = fmaxf(Mb, sh[(w0 + w) * 3]);
        float kb = Mb * kLog2e;
        float S = 0.f, T = 0.f;
#pragma unroll
        for (int w = 0; w < WPR; ++w) {
            float so, to;
            to_common(-(sh[(w0 + w) * 3] * kLog2e), sh[(w0 + w) * 3 + 1], sh[(w0 + w) * 3 + 2], kb, so, to);
            S += so; T += to;
        }
        s = S; t = T; kc = kb;
    }

    if (row_ok && l == 0) {
        float lp = 0.f, en = 0.f;
        if (live) {
            float logS = logf(s);
            lp = kLn2 * fmaf(xtok, kLog2e, -kc) - logS;
            en = logS - kLn2 * t / s;
        }
        if (tok_logp) tok_logp[row] = lp;
        if (tok_ent) tok_ent[row] = en;
    }
}

// Per step: plain sums, in row order, of the step's A per-token values.
__global__ __launch_bounds__(256) void k_step_sums(
    const float* __restrict__ tok_logp, const float* __restrict__ tok_ent, long long N, int A,
    float* __restrict__ step_logp, float* __restrict__ step_ent) {
    long long n = (long long)blockIdx.x * blockDim.x + threadIdx.x;
    if (n >= N) return;
    float sl = 0.f, se = 0.f;
    const float* pl = tok_logp + n * A;
    const float* pe = tok_ent + n * A;
    for (int j = 0; j < A; ++j) { sl += pl[j]; se += pe[j]; }
    if (step_logp) step_logp[n] = sl;
    if (step_ent) step_ent[n] = se;
}

template <int WPR, int UNROLL>
static hipError_t launch_rows(const uint16_t* logits, long long R, int V, long long stride,
                              const int* tokens, float* tl, float* te, uint32_t* status,
                              hipStream_t st) {
    constexpr int rpb = 4 / WPR;
    long long blocks = (R + rpb - 1) / rpb;
    hipLaunchKernelGGL((k_score_rows<WPR, UNROLL>), dim3((unsigned)blocks), dim3(256), 0, st,
                       logits, R, V, stride, tokens, tl, te, status);
    return hipGetLastError();
}

// wpr: waves per row (1, 2, 4); 0 picks the default.
hipError_t score_logits_launch(const uint16_t* logits, long long R, int V, long long stride,
                               const int* tokens, int A, float* tok_logp, float* tok_ent,
                               float* step_logp, float* step_ent, uint32_t* status,
                               int wpr, hipStream_t st) {
    hipError_t err;
    if (wpr == 0) wpr = ARIDE_SCORE_WPR;
    switch (wpr) {
        case 4: err = launch_rows<4, 4>(logits, R, V, stride, tokens, tok_logp, tok_ent, status, st); break;
        case 2: err = launch_rows<2, 4>(logits, R, V, stride, tokens, tok_logp, tok_ent, status, st); break;
        default: err = launch_rows<1, 4>(logits, R, V, stride, tokens, tok_logp, tok_ent, status, st); break;
    }
    if (err != hipSuccess) return err;
    if (step_logp || step_ent) {
        long long N = R / A;
        hipLaunchKernelGGL(k_step_sums, dim3((unsigned)((N + 255) / 256)), dim3(256), 0, st,
                           tok_logp, tok_ent, N, A, step_logp, step_ent);
        err = hipGetLastError();
    }
    return err;
}

}  // namespace aride
