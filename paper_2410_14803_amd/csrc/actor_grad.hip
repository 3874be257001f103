// actor_loss_grad: the actor loss of Section 5.1, eq. (1) of the DistRL paper and its gradient
// with respect to the logits (Appendix A.4.2, policy update), as a second sweep over the
// same bf16 logits that score_logits reduced:
//   dL/dx_{r,v} = scale * [ -rho_t A_t (1[v = tok_r] - p_v) + beta * p_v (log p_v + H_r) ]
// The row's log-partition function and entropy are not recomputed: log Z_r = x_tok - tok_logp[r]
// and H_r = tok_ent[r] come from the first sweep, so each logit is read once and each
// gradient element written once (4 bytes of HBM traffic per element for bf16 output).
// log Z is carried as a two-float value, so p_v = exp(x_v - log Z) is accurate to a few fp32
// ulps whatever the magnitude of the logits, and the chosen token's element, where 1 - p
// cancels when the token dominates its row, is formed from expm1(tok_logp) instead.
// Non-temporal loads and 16-byte non-temporal stores; HBM-bound, no MFMA.
#include "aride_device.h"

namespace aride {

constexpr int kActorUnroll = 4;      // 16-byte loads in flight per lane (bf16 output)
constexpr int kActorUnrollF32 = 8;   // 8-byte loads in flight per lane (fp32 output)

constexpr float kLog2eA = 1.4426950408889634f;
constexpr float kLn2A = 0.6931471805599453f;
constexpr int kSplit8MinV = 8192, kSplit16MinV = 12288;   // row lengths from which a row gets 8 and 16 waves

typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
typedef float f32x4 __attribute__((ext_vector_type(4)));
typedef float f32x2 __attribute__((ext_vector_type(2)));
typedef __bf16 bf16x2 __attribute__((ext_vector_type(2)));

struct RowCoef {
    float negkz;  // -(log Z) * log2e, leading part
    float negkz_lo;  // and the rest of it
    float cbl;    // scale * beta * ln2
    float k1;     // coef + scale * beta * H
    float coef;   // scale * rho * A
};

__device__ __forceinline__ float grad_of(float x, const RowCoef& c) {
    // y = log2 p; clamped so that p = 0 multiplies a finite factor (x may be -inf)
    const float y = fmaxf(fmaf(x, kLog2eA, c.negkz) + c.negkz_lo, -200.f);
    const float p = fast_exp2(y);
    return p * fmaf(c.cbl, y, c.k1);
}

__device__ __forceinline__ uint32_t pack_bf16(float lo, float hi) {
    f32x2 v = {lo, hi};
    bf16x2 b = __builtin_convertvector(v, bf16x2);   // round to nearest even
    return __builtin_bit_cast(uint32_t, b);
}

__device__ __forceinline__ uint16_t pack_bf16_one(float v) {
    return (uint16_t)(pack_bf16(v, 0.f) & 0xffffu);
}

// WPR = 1: one wave per row, four rows per workgroup.  WPR = 8, 16: a workgroup of that many
// waves per row, the rows dealt to the chip's 8 XCDs in contiguous eighths (see
// xcd_contiguous_block); the waves move along the row side by side, the workgroup covering
// WPR KB of it per load instruction, so that a row is read and its gradient written as one
// moving front.  Measured on 64 KB rows: 16 waves 1.71 ms per 5.3 GB batch, 8 waves 1.81, 4 waves
// 1.93, one wave per row 2.02.
// A lane's unit is 8 elements (16 bytes in, 16 out) for bf16 output and 4 elements (8 bytes in,
// 16 out) for fp32 output, so that every store instruction of a wave writes 1 KB without gaps.
template <bool OUT_F32, int WPR>
__global__ __launch_bounds__(WPR == 1 ? 256 : 64 * WPR) void k_actor_grad(
    const uint16_t* __restrict__ logits, long long row0, long long R, int V, long long row_stride,
    const int* __restrict__ tokens, int A, const float* __restrict__ tok_logp,
    const float* __restrict__ tok_ent, const float* __restrict__ rho, const float* __restrict__ target,
    const float* __restrict__ baseline, float beta, float scale, void* __restrict__ grad_out) {
    constexpr int kVec = OUT_F32 ? 4 : 8;            // elements per lane and load
    constexpr int kWords = kVec / 2;
    constexpr uint32_t kVecBytes = 2 * kVec;
    typedef uint32_t vec_t __attribute__((ext_vector_type(kWords)));
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const long long row = row0 + (WPR == 1 ? (((long long)blockIdx.x * blockDim.x + threadIdx.x) >> 6)
                                           : xcd_contiguous_block());   // the grid: this launch's rows, rounded up to a multiple of 8
    if (row >= R) return;   // whole waves (WPR = 1) or the whole workgroup leave; there is no barrier below
    const int tok = tokens[row];
    const bool live = tok >= 0 && tok < V;
    const uint16_t* p = logits + row * row_stride;
    uint16_t* gb = reinterpret_cast<uint16_t*>(grad_out) + row * row_stride;
    float* gf = reinterpret_cast<float*>(grad_out) + row * row_stride;

    // elements before the first aligned load; both bases are 16-byte aligned, so the stores of
    // the vectors that follow are 16-byte aligned as well
    int head = (int)(((kVecBytes - (uint32_t)((uintptr_t)p & (kVecBytes - 1))) & (kVecBytes - 1)) >> 1);
    if (head > V) head = V;
    const int nvec = (V - head) / kVec;
    const int tail0 = head + nvec * kVec;

    RowCoef c;
    c.negkz = 0.f; c.negkz_lo = 0.f; c.cbl = 0.f; c.k1 = 0.f; c.coef = 0.f;
    float gtok = 0.f;   // the chosen token's element
    if (live) {
        const long long t = row / A;
        const float xtok = bits_to_float(((uint32_t)p[tok]) << 16);
        const float lp = tok_logp[row], h = tok_ent[row];
        // (x - log Z) * log2e with the same fp32 log2e on both sides: once per row in fp64
        const double negkz = -((double)xtok - (double)lp) * (double)kLog2eA;
        c.negkz = (float)negkz;
        c.negkz_lo = (float)(negkz - (double)c.negkz);
        c.coef = scale * rho[t] * (target[t] - baseline[t]);
        const float cb = scale * beta;
        c.cbl = cb * kLn2A;
        c.k1 = fmaf(cb, h, c.coef);
        // coef * (p - 1) + cb * p * (log p + H) at the chosen token, without forming p - 1
        const float pm1 = expm1f(lp);
        gtok = fmaf(c.coef, pm1, cb * (1.f + pm1) * (lp + h));
    }
    const int tvec = (live && tok >= head && tok < tail0) ? ((tok - head) / kVec) : -1;
    const int tsub = (tok - head) & (kVec - 1);

    const vec_t* pv = reinterpret_cast<const vec_t*>(p + head);
    auto emit = [&](int i, const vec_t& v) {
        float g[kVec];
        if (live) {
#pragma unroll
            for (int w = 0; w < kWords; ++w) {
                g[2 * w] = grad_of(bits_to_float(v[w] << 16), c);
                g[2 * w + 1] = grad_of(bits_to_float(v[w] & 0xffff0000u), c);
            }
            if (i == tvec) {
#pragma unroll
                for (int j = 0; j < kVec; ++j) g[j] = (j == tsub) ? gtok : g[j];
            }
        } else {
#pragma unroll
            for (int j = 0; j < kVec; ++j) g[j] = 0.f;
        }
        if constexpr (OUT_F32) {
            f32x4 o = {g[0], g[1], g[2], g[3]};
            __builtin_nontemporal_store(o, reinterpret_cast<f32x4*>(gf + head) + i);
        } else {
            u32x4 o = {pack_bf16(g[0], g[1]), pack_bf16(g[2], g[3]), pack_bf16(g[4], g[5]), pack_bf16(g[6], g[7])};
            __builtin_nontemporal_store(o, reinterpret_cast<u32x4*>(gb + head) + i);
        }
    };
    constexpr int kU = OUT_F32 ? kActorUnrollF32 : kActorUnroll;
    constexpr int kStep = WPR * kWave;               // vectors the row's waves cover per load
    int i = (WPR == 1 ? 0 : wave * kWave) + lane;
    if (live) {
        for (; i + (kU - 1) * kStep < nvec; i += kU * kStep) {
            vec_t v[kU];
#pragma unroll
            for (int u = 0; u < kU; ++u) v[u] = __builtin_nontemporal_load(pv + i + u * kStep);
#pragma unroll
            for (int u = 0; u < kU; ++u) emit(i + u * kStep, v[u]);
        }
        for (; i < nvec; i += kStep) emit(i, __builtin_nontemporal_load(pv + i));
    } else {
        vec_t zero;
#pragma unroll
        for (int w = 0; w < kWords; ++w) zero[w] = 0u;
        for (; i < nvec; i += kStep) emit(i, zero);
    }
    // elements before the first aligned vector and after the last full one
    if (WPR > 1 && wave != 0) return;
    for (int k = lane; k < head + (V - tail0); k += kWave) {
        const int v = k < head ? k : tail0 + (k - head);
        float g = 0.f;
        if (live) {
            g = grad_of(bits_to_float(((uint32_t)p[v]) << 16), c);
            if (v == tok) g = gtok;
        }
        if constexpr (OUT_F32) gf[v] = g; else gb[v] = pack_bf16_one(g);
    }
}

// L = scale * sum_t [ -rho_t A_t log pi(a_t|s_t) - beta H_t + lambda_pen P_t ]: one workgroup,
// fp64 partial sums combined in a fixed order, one rounding to fp32.
__global__ __launch_bounds__(1024) void k_actor_loss(
    const float* __restrict__ step_logp, const float* __restrict__ step_ent, const float* __restrict__ rho,
    const float* __restrict__ target, const float* __restrict__ baseline, const float* __restrict__ penalty,
    int N, float beta, float lambda_pen, float scale, float* __restrict__ loss) {
    __shared__ double wave_part[16];
    double acc = 0.0;
    for (int t = threadIdx.x; t < N; t += 1024) {
        const double coef = (double)rho[t] * ((double)target[t] - (double)baseline[t]);
        acc += -coef * (double)step_logp[t] - (double)beta * (double)step_ent[t] +
               (penalty ? (double)lambda_pen * (double)penalty[t] : 0.0);
    }
#pragma unroll
    for (int d = 32; d >= 1; d >>= 1) acc += __shfl_xor(acc, d, kWave);
    if ((threadIdx.x & 63) == 0) wave_part[threadIdx.x >> 6] = acc;
    __syncthreads();
    if (threadIdx.x == 0) {
        double tot = 0.0;
        for (int w = 0; w < 16; ++w) tot += wave_part[w];
        *loss = (float)((double)scale * tot);
    }
}

hipError_t actor_launch(const uint16_t* logits, long long R, int V, long long stride, const int* tokens,
                        int A, const float* tok_logp, const float* tok_ent, const float* step_logp,
                        const float* step_ent, const float* rho, const float* target,
                        const float* baseline, const float* penalty, float beta, float lambda_pen,
                        float scale, int grad_f32, void* grad, float* loss, hipStream_t st) {
    if (grad && R > 0) {
        // rows of 16 KB and more: a workgroup of 8 waves per row, of 24 KB and more: of 16 waves.
        // A launch covers at most kMaxLaunchThreads work-items; more rows go out slice by slice.
        const int wpr = V < kSplit8MinV ? 1 : V < kSplit16MinV ? 8 : 16;
        const long long slice = kMaxLaunchThreads / (64 * wpr);
        for (long long row0 = 0; row0 < R; row0 += slice) {
            const long long rows = R - row0 < slice ? R - row0 : slice;
            const dim3 grid(wpr > 1 ? round_up_8((unsigned)rows) : (unsigned)((rows + 3) / 4));
            auto go = [&](auto kernel) {
                hipLaunchKernelGGL(kernel, grid, dim3(wpr > 1 ? 64 * wpr : 256), 0, st, logits, row0, R, V, stride, tokens,
                                   A, tok_logp, tok_ent, rho, target, baseline, beta, scale, grad);
            };
            if (grad_f32) { if (wpr == 16) go(k_actor_grad<true, 16>); else if (wpr == 8) go(k_actor_grad<true, 8>); else go(k_actor_grad<true, 1>); }
            else          { if (wpr == 16) go(k_actor_grad<false, 16>); else if (wpr == 8) go(k_actor_grad<false, 8>); else go(k_actor_grad<false, 1>); }
        }
    }
    if (loss)
        hipLaunchKernelGGL(k_actor_loss, dim3(1), dim3(1024), 0, st, step_logp, step_ent, rho, target, baseline,
                           penalty, (int)(R / A), beta, lambda_pen, scale, loss);
    return hipGetLastError();
}

}  // namespace aride
