// Prioritized replay (Appendix A.4.2 of the DistRL paper: P(i) = p_i^alpha / sum_j p_j^alpha;
// Section 5.3: priorities are recomputed and overwritten).
//
// The buffer stores w_i = p_i^alpha as fp32.  Sampling is defined on integers so that any
// summation order gives the same answer:
//     e = ilogb(max w) + 1,  q_i = floor(w_i * 2^(39-e)) < 2^39,  C_i = q_0 + ... + q_i (u64)
//     t = min(floor(u * (double)Total), Total - 1),  idx = min{ i : C_i > t }
// The index kept in the workspace is the inclusive prefix of the per-block sums of q
// (blocks of 256 weights = one wave x float4); a draw bisects that prefix and then scans
// one 1 KB block with a wave-wide integer prefix sum.
//
// update_priorities resolves repeated indices without a serial loop: pass 1 writes the
// tag (0xFF800000 | k) with an unsigned atomic max into the weight slot itself -- every
// tag is larger than the bit pattern of any non-negative finite float, and the largest k
// (the last occurrence) wins -- and pass 2 lets exactly the winning k store its weight.
#include "aride_device.h"

namespace aride {

constexpr uint32_t kTagBase = 0xFF800000u;

// q = floor(w * 2^(39-e)) computed on the bit pattern; negative, NaN and infinite
// weights (and -0) carry no mass.
__device__ __forceinline__ unsigned long long quantise(float w, int e) {
    const uint32_t b = float_to_bits(w);
    if (b >= 0x7F800000u) return 0ull;
    uint32_t E = b >> 23;
    uint32_t mant = b & 0x7FFFFFu;
    if (E == 0) E = 1; else mant |= 0x800000u;   // subnormal: no implicit bit, exponent of 1
    // w = mant * 2^(E-150)  =>  q = floor(mant * 2^(E - 111 - e))
    int sh = (int)E - 111 - e;
    if (sh >= 0) return (unsigned long long)mant << (sh > 39 ? 39 : sh);
    sh = -sh;
    return sh >= 24 ? 0ull : (unsigned long long)(mant >> sh);
}

// e = ilogb(wmax) + 1 from the bit pattern of a positive finite float.
__device__ __forceinline__ int exponent_of(uint32_t wmax_bits) {
    const uint32_t E = wmax_bits >> 23;
    if (E != 0) return (int)E - 127 + 1;
    const uint32_t mant = wmax_bits & 0x7FFFFFu;   // subnormal: value = mant * 2^-149
    return (31 - __clz(mant)) - 149 + 1;
}

__global__ void k_reset_index(WsHeader* hdr) {
    if (blockIdx.x == 0 && threadIdx.x == 0) { hdr->wmax_bits = 0u; hdr->total = 0ull; hdr->exponent = 0; }
}

__global__ __launch_bounds__(256) void k_update_tag(
    float* __restrict__ weights, long long M, const long long* __restrict__ idx, int K, WsHeader* hdr) {
    const int k = blockIdx.x * blockDim.x + threadIdx.x;
    if (k == 0) { hdr->wmax_bits = 0u; hdr->total = 0ull; hdr->exponent = 0; }
    if (k >= K) return;
    const long long i = idx[k];
    if (i < 0 || i >= M) { atomicOr(&hdr->flags, 0x8u); return; }
    atomicMax(reinterpret_cast<uint32_t*>(weights) + i, kTagBase | (uint32_t)k);
}

__global__ __launch_bounds__(256) void k_update_commit(
    float* __restrict__ weights, long long M, const long long* __restrict__ idx,
    const float* __restrict__ prio, int K, float alpha) {
    const int k = blockIdx.x * blockDim.x + threadIdx.x;
    if (k >= K) return;
    const long long i = idx[k];
    if (i < 0 || i >= M) return;
    volatile uint32_t* slot = reinterpret_cast<volatile uint32_t*>(weights) + i;
    if (*slot != (kTagBase | (uint32_t)k)) return;   // an occurrence later in the batch owns the slot
    double p = (double)prio[k];
    if (!(p > 0.0)) p = 0.0;
    weights[i] = (float)pow(p, (double)alpha);
}

// Pass A of the rebuild: largest valid weight (order-free, exact).
__global__ __launch_bounds__(256) void k_weight_max(const float* __restrict__ weights, long long M, WsHeader* hdr) {
    const long long nvec = M >> 2;
    const float4* wv = reinterpret_cast<const float4*>(weights);
    uint32_t best = 0u;
    bool bad = false;
    auto see = [&](float w) {
        const uint32_t b = float_to_bits(w);
        if (b < 0x7F800000u) best = max(best, b);          // non-negative finite: bit order = value order
        else if (b != 0x80000000u) bad = true;              // negative, inf or NaN (-0 is fine)
    };
    for (long long i = (long long)blockIdx.x * blockDim.x + threadIdx.x; i < nvec; i += (long long)gridDim.x * blockDim.x) {
        const float4 v = wv[i];
        see(v.x); see(v.y); see(v.z); see(v.w);
    }
    if (blockIdx.x == 0 && threadIdx.x < (M & 3)) see(weights[(nvec << 2) + threadIdx.x]);
#pragma unroll
    for (int d = 32; d >= 1; d >>= 1) best = max(best, (uint32_t)__shfl_xor((int)best, d, kWave));
    const bool any_bad = __any(bad);
    if ((threadIdx.x & 63) == 0) {
        if (best) atomicMax(&hdr->wmax_bits, best);
        if (any_bad) atomicOr(&hdr->flags, 0x2u);
    }
}

// Pass B: integer sum of each block of 256 weights (one wave per block).
__global__ __launch_bounds__(256) void k_block_sums(const float* __restrict__ weights, long long M,
                                                    const WsHeader* __restrict__ hdr,
                                                    unsigned long long* __restrict__ block_sum, int nblk) {
    const int lane = threadIdx.x & 63;
    const int blk = (int)(((long long)blockIdx.x * blockDim.x + threadIdx.x) >> 6);
    if (blk >= nblk) return;
    const uint32_t wb = hdr->wmax_bits;
    unsigned long long s = 0ull;
    if (wb != 0u) {
        const int e = exponent_of(wb);
        const long long base = (long long)blk * kReplayBlock + lane * 4;
        if (base + 3 < M) {
            const float4 v = *reinterpret_cast<const float4*>(weights + base);
            s = quantise(v.x, e) + quantise(v.y, e) + quantise(v.z, e) + quantise(v.w, e);
        } else {
            for (int j = 0; j < 4; ++j) if (base + j < M) s += quantise(weights[base + j], e);
        }
    }
    s = wave_sum_u64(s);
    if (lane == 0) block_sum[blk] = s;
}

// Pass C: in-place inclusive prefix over the block sums; one workgroup of 1024 threads,
// each owning a contiguous run.  Also publishes Total, the exponent and the no-mass flag.
__global__ __launch_bounds__(1024) void k_prefix_blocks(unsigned long long* __restrict__ block_sum, int nblk, WsHeader* hdr) {
    __shared__ unsigned long long wave_tot[16];
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int per = (nblk + 1023) / 1024;
    const int lo = min(tid * per, nblk), hi = min(lo + per, nblk);
    unsigned long long mine = 0ull;
    for (int i = lo; i < hi; ++i) mine += block_sum[i];
    unsigned long long incl = mine;
#pragma unroll
    for (int d = 1; d < kWave; d <<= 1) {
        unsigned long long up = __shfl_up(incl, d, kWave);
        if (lane >= d) incl += up;
    }
    if (lane == 63) wave_tot[wave] = incl;
    __syncthreads();
    unsigned long long before = 0ull, total = 0ull;
    for (int w = 0; w < 16; ++w) { if (w < wave) before += wave_tot[w]; total += wave_tot[w]; }
    unsigned long long run = before + incl - mine;
    for (int i = lo; i < hi; ++i) { run += block_sum[i]; block_sum[i] = run; }
    if (tid == 0) {
        hdr->total = total;
        hdr->exponent = hdr->wmax_bits ? exponent_of(hdr->wmax_bits) : 0;
        if (total == 0ull) atomicOr(&hdr->flags, 0x4u);
    }
}

// One wave per draw.
__global__ __launch_bounds__(256) void k_sample(
    const float* __restrict__ weights, long long M, const WsHeader* __restrict__ hdr,
    const unsigned long long* __restrict__ block_cum, int nblk, const double* __restrict__ uniforms,
    int K, long long* __restrict__ idx_out, float* __restrict__ prob_out, uint32_t* __restrict__ flags) {
    const int lane = threadIdx.x & 63;
    const int k = (int)(((long long)blockIdx.x * blockDim.x + threadIdx.x) >> 6);
    if (k >= K) return;
    const unsigned long long total = hdr->total;
    if (total == 0ull) {
        if (lane == 0) { idx_out[k] = -1; if (prob_out) prob_out[k] = 0.f; }
        return;
    }
    double u = uniforms[k];
    if (!(u >= 0.0)) { u = 0.0; if (lane == 0) atomicOr(flags, 0x10u); }
    // one rounding for the conversion, one for the product, then truncation
    const double prod = __dmul_rn(u, __ull2double_rn(total));
    unsigned long long t = (prod >= 18446744073709551616.0) ? total - 1 : (unsigned long long)prod;
    if (t > total - 1) t = total - 1;

    // first block whose inclusive prefix exceeds t (block_cum[nblk-1] = Total > t)
    int lo = 0, hi = nblk - 1;
    while (lo < hi) {
        const int mid = lo + ((hi - lo) >> 1);
        if (block_cum[mid] > t) hi = mid; else lo = mid + 1;
    }
    const int blk = lo;
    const unsigned long long rem = t - (blk ? block_cum[blk - 1] : 0ull);

    const int e = exponent_of(hdr->wmax_bits);
    const long long base = (long long)blk * kReplayBlock + lane * 4;
    unsigned long long qv[4] = {0ull, 0ull, 0ull, 0ull};
    if (base + 3 < M) {
        const float4 v = *reinterpret_cast<const float4*>(weights + base);
        qv[0] = quantise(v.x, e); qv[1] = quantise(v.y, e); qv[2] = quantise(v.z, e); qv[3] = quantise(v.w, e);
    } else {
        for (int j = 0; j < 4; ++j) if (base + j < M) qv[j] = quantise(weights[base + j], e);
    }
    const unsigned long long mine = qv[0] + qv[1] + qv[2] + qv[3];
    unsigned long long incl = mine;
#pragma unroll
    for (int d = 1; d < kWave; d <<= 1) {
        unsigned long long up = __shfl_up(incl, d, kWave);
        if (lane >= d) incl += up;
    }
    const unsigned long long hit = __ballot(incl > rem);
    // hit is non-zero when the index matches the weights; a stale index yields -1
    if (hit == 0ull) {
        if (lane == 0) { idx_out[k] = -1; if (prob_out) prob_out[k] = 0.f; }
        return;
    }
    const int owner = __ffsll((long long)hit) - 1;
    if (lane == owner) {
        unsigned long long c = incl - mine;
        int j = 0;
        for (; j < 3; ++j) { if (c + qv[j] > rem) break; c += qv[j]; }
        idx_out[k] = base + j;
        if (prob_out) prob_out[k] = (float)((double)qv[j] / (double)total);
    }
}

hipError_t update_launch(float* weights, long long M, const long long* idx, const float* prio, int K,
                         float alpha, WsHeader* hdr, unsigned long long* block_cum, hipStream_t st) {
    const int nblk = (int)((M + kReplayBlock - 1) / kReplayBlock);
    if (K > 0) {
        const unsigned g = (unsigned)((K + 255) / 256);
        hipLaunchKernelGGL(k_update_tag, dim3(g), dim3(256), 0, st, weights, M, idx, K, hdr);
        hipLaunchKernelGGL(k_update_commit, dim3(g), dim3(256), 0, st, weights, M, idx, prio, K, alpha);
    } else {
        hipLaunchKernelGGL(k_reset_index, dim3(1), dim3(64), 0, st, hdr);
    }
    long long want = ((M >> 2) + 255) / 256;
    unsigned gmax = (unsigned)(want < 1 ? 1 : (want > 4096 ? 4096 : want));
    hipLaunchKernelGGL(k_weight_max, dim3(gmax), dim3(256), 0, st, weights, M, hdr);
    hipLaunchKernelGGL(k_block_sums, dim3((unsigned)((nblk + 3) / 4)), dim3(256), 0, st, weights, M, hdr, block_cum, nblk);
    hipLaunchKernelGGL(k_prefix_blocks, dim3(1), dim3(1024), 0, st, block_cum, nblk, hdr);
    return hipGetLastError();
}

hipError_t sample_launch(const float* weights, long long M, const WsHeader* hdr,
                         const unsigned long long* block_cum, const double* uniforms, int K,
                         long long* idx_out, float* prob_out, uint32_t* flags, hipStream_t st) {
    const int nblk = (int)((M + kReplayBlock - 1) / kReplayBlock);
    const unsigned g = (unsigned)(((long long)K * kWave + 255) / 256);
    hipLaunchKernelGGL(k_sample, dim3(g), dim3(256), 0, st, weights, M, hdr, block_cum, nblk,
                       uniforms, K, idx_out, prob_out, flags);
    return hipGetLastError();
}

}  // namespace aride
