// Prioritized replay (Appendix A.4.2 of the DistRL paper: P(i) = p_i^alpha / sum_j p_j^alpha;
// Section 5.3: priorities are recomputed and overwritten).
//
// The buffer stores w_i = p_i^alpha as fp32.  Sampling is defined on integers so that any
// summation order gives the same answer:
//     e = ilogb(max w) + 1,  q_i = floor(w_i * 2^(39-e)) < 2^39,  C_i = q_0 + ... + q_i (u64)
//     t = min(floor(u * (double)Total), Total - 1),  idx = min{ i : C_i > t }
// The index kept in the workspace has three levels of integer sums -- sub-blocks of 16 weights
// (sub_sum), blocks of 256 weights (one wave x float4) and super-blocks of 256 blocks -- plus a
// contiguous copy of every 16th block prefix (coarse_cum).  block_cum holds, per super-block, the
// inclusive prefix of its block sums; super_cum the inclusive prefix of the super-block totals
// (padded to 256 entries with Total).  A draw is served by 16 lanes: the 256 super-block prefixes
// (staged in LDS) and the 256 block prefixes of the chosen super-block are each searched 16-ary in
// two probes (the first probe of the latter reads coarse_cum, one line), then each lane reads one
// of the block's 16 sub-block sums, and last the lanes quantise the chosen sub-block's 16 weights.
//
// Keeping the index current:
//  * a rebuild of a large buffer is ONE sweep (k_super_sums<true>): it finds the maxima and
//    sums under the exponent of the index as it stands; k_super_sums<false> sweeps again only
//    if the maximum's exponent has moved.  Smaller buffers take a maximum pass, a block-sum
//    pass and a scan; the smallest do everything in one workgroup.
//  * alongside, the largest valid weight of every chunk of 16 blocks (chunk_max) and of every
//    four chunks (partial_max) is kept, so that after a contiguous insert the new maximum of the
//    whole buffer follows from the touched chunks alone and the index can be patched
//    (k_insert_patch, k_patch_supers, k_patch_finish) instead of rebuilt.
//
// update_priorities resolves repeated indices without a serial loop: pass 1 puts the tag
// (0xFF800000 | k) into the weight slot itself with an unsigned atomic max -- every tag is larger
// than the bit pattern of any float that is not -inf or a negative NaN, and the largest k (the
// last occurrence) wins -- and pass 2 lets exactly the winning k store its weight.  A slot that
// holds -inf or a negative NaN when the update starts (bits at or above the tag range) would beat
// the tags; claim_slot recognises such a value by its not being a tag any occurrence of this batch
// writes for this slot, and replaces it with a compare-and-swap.
#include "aride_device.h"

namespace aride {

constexpr uint32_t kTagBase = 0xFF800000u;

// q = floor(w * 2^(39-e)); negative, NaN and infinite weights (and -0) carry no mass.
// Exact in fp32: scaling by a power of two (v_ldexp_f32) does not touch the 24-bit mantissa,
// x < 2^39 splits into hi = floor(x / 2^32) and lo = x - hi * 2^32, both exact, and
// v_cvt_u32_f32 truncates.  A result below the normal range floors to 0 either way.
__device__ __forceinline__ unsigned long long quantise(float w, int e) {
    const uint32_t b = float_to_bits(w);
    const float wc = b < 0x7F800000u ? w : 0.f;
    const float x = ldexpf(wc, 39 - e);
    const uint32_t hi = (uint32_t)(x * 2.3283064365386963e-10f);             // 2^-32
    const uint32_t lo = (uint32_t)fmaf(-(float)hi, 4294967296.f, x);
    return ((unsigned long long)hi << 32) | lo;
}

// e = ilogb(wmax) + 1 from the bit pattern of a positive finite float.
__device__ __forceinline__ int exponent_of(uint32_t wmax_bits) {
    const uint32_t E = wmax_bits >> 23;
    if (E != 0) return (int)E - 127 + 1;
    const uint32_t mant = wmax_bits & 0x7FFFFFu;   // subnormal: value = mant * 2^-149
    return (31 - __clz(mant)) - 149 + 1;
}

// Pass 1 for occurrence k of slot i (slot = the weight's word).  Afterwards the slot holds the
// largest tag among the occurrences of i that have run so far, whatever bits it held before.
//  * old value below the tag range: an ordinary weight, the atomic max has replaced it.
//  * old value in the tag range whose low bits name an occurrence j < K with idx[j] == i: a tag of
//    this batch for this slot (or a stored value with the very bits occurrence j writes, which
//    changes nothing): the atomic max has merged mine with it.
//  * otherwise a stored -inf or negative NaN.  If it is below my tag the atomic max has replaced
//    it; if not, swap my tag in for exactly that value.  When the swap fails another occurrence
//    has replaced it meanwhile and the next round finds that occurrence's tag.  The slot only ever
//    moves from a stored value to a tag and from a tag to a larger tag, so at most one retry.
__device__ __forceinline__ void claim_slot(uint32_t* slot, uint32_t k, const long long* __restrict__ idx, int K,
                                           long long i) {
    const uint32_t mine = kTagBase | k;
    for (;;) {
        const uint32_t old = atomicMax(slot, mine);
        if (old < mine) return;
        const uint32_t j = old & 0x7FFFFFu;
        if (j < (uint32_t)K && idx[j] == i) return;
        if (atomicCAS(slot, old, mine) == old) return;
    }
}

__global__ __launch_bounds__(256) void k_update_tag(
    float* __restrict__ weights, long long M, const long long* __restrict__ idx, int K, WsHeader* hdr) {
    const int k = blockIdx.x * blockDim.x + threadIdx.x;
    if (k >= K) return;
    const long long i = idx[k];
    if (i < 0 || i >= M) { atomicOr(&hdr->flags, 0x8u); return; }
    claim_slot(reinterpret_cast<uint32_t*>(weights) + i, (uint32_t)k, idx, K, i);
}

__global__ __launch_bounds__(256) void k_update_commit(
    float* __restrict__ weights, long long M, const long long* __restrict__ idx,
    const float* __restrict__ prio, int K, float alpha) {
    const int k = blockIdx.x * blockDim.x + threadIdx.x;
    if (k >= K) return;
    const long long i = idx[k];
    if (i < 0 || i >= M) return;
    const uint32_t seen = __hip_atomic_load(reinterpret_cast<uint32_t*>(weights) + i, __ATOMIC_RELAXED,
                                            __HIP_MEMORY_SCOPE_AGENT);
    if (seen != (kTagBase | (uint32_t)k)) return;    // an occurrence later in the batch owns the slot
    double p = (double)prio[k];
    if (!(p > 0.0)) p = 0.0;
    weights[i] = (float)pow(p, (double)alpha);
}

// Both passes in one workgroup for batches of up to kSmallBatch entries: a workgroup barrier
// separates them, the tags are written and read with device-scope atomics.
__global__ __launch_bounds__(1024) void k_update_scatter_small(
    float* __restrict__ weights, long long M, const long long* __restrict__ idx, const float* __restrict__ prio,
    int K, float alpha, WsHeader* hdr) {
    uint32_t* wbits = reinterpret_cast<uint32_t*>(weights);
    for (int k = threadIdx.x; k < K; k += 1024) {
        const long long i = idx[k];
        if (i < 0 || i >= M) { atomicOr(&hdr->flags, 0x8u); continue; }
        claim_slot(wbits + i, (uint32_t)k, idx, K, i);
    }
    __syncthreads();
    for (int k = threadIdx.x; k < K; k += 1024) {
        const long long i = idx[k];
        if (i < 0 || i >= M) continue;
        const uint32_t seen = __hip_atomic_load(wbits + i, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        if (seen != (kTagBase | (uint32_t)k)) continue;
        double p = (double)prio[k];
        if (!(p > 0.0)) p = 0.0;
        __hip_atomic_store(weights + i, (float)pow(p, (double)alpha), __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    }
}

// Appendix A.4.2, circular buffer: entry k of the batch goes to slot (cursor + k) mod M.  When
// the batch is longer than the buffer only its last M entries survive (what inserting one at a
// time would leave); the others report slot -1.  Surviving slots are distinct, so no tag pass.
__global__ __launch_bounds__(256) void k_insert(float* __restrict__ weights, long long M, long long cursor,
                                                const float* __restrict__ prio, long long K, float alpha,
                                                long long* __restrict__ slots_out) {
    const long long k = (long long)blockIdx.x * blockDim.x + threadIdx.x;
    if (k >= K) return;
    if (k + M < K) { if (slots_out) slots_out[k] = -1; return; }
    const long long slot = (cursor + k) % M;
    double p = (double)prio[k];
    if (!(p > 0.0)) p = 0.0;
    weights[slot] = (float)pow(p, (double)alpha);
    if (slots_out) slots_out[k] = slot;
}

// This lane's four weights (lane * 4 ..) of block `blk`; entries past the end of the buffer read 0.
__device__ __forceinline__ float4 load_block_quad(const float* __restrict__ weights, long long M, int blk, int lane) {
    const long long base = (long long)blk * kReplayBlock + lane * 4;
    float4 v = make_float4(0.f, 0.f, 0.f, 0.f);
    if (base + 3 < M) v = *reinterpret_cast<const float4*>(weights + base);
    else if (base < M) {
        v.x = weights[base];
        if (base + 1 < M) v.y = weights[base + 1];
        if (base + 2 < M) v.z = weights[base + 2];
    }
    return v;
}
// Largest valid weight among four (bit pattern; 0 when there is none); `bad` collects negative,
// infinite or NaN entries (-0 is fine).
__device__ __forceinline__ uint32_t quad_max_bits(const float4& v, bool& bad) {
    uint32_t best = 0u;
    auto see = [&](float w) {
        const uint32_t b = float_to_bits(w);
        if (b < 0x7F800000u) best = max(best, b);          // non-negative finite: bit order = value order
        else if (b != 0x80000000u) bad = true;
    };
    see(v.x); see(v.y); see(v.z); see(v.w);
    return best;
}
__device__ __forceinline__ uint32_t wave_max_u32(uint32_t v) {
#pragma unroll
    for (int d = 32; d >= 1; d >>= 1) v = max(v, (uint32_t)__shfl_xor((int)v, d, kWave));
    return v;
}

// Pass A of the rebuild: largest valid weight (order-free, exact).  A chunk is 16 consecutive
// blocks (4096 weights); wave w of workgroup g reduces chunk 4g + w -- 16 loads in flight,
// one wave reduction -- and stores its maximum to chunk_max; the maximum of the workgroup's four
// chunks goes to partial_max[g], and the consumers reduce those 1024 words themselves.  (One
// atomic per wave onto a single header word was measured at ~160 us for M = 2^24: same-address
// atomics serialise.)  Used for buffers below 64 super-blocks; larger ones find their maxima
// in the sweep that sums them (k_super_sums).
static_assert(kMaxChunks == 4 * kMaxParts, "one chunk per wave of the maximum pass");
static_assert((long long)kMaxChunks * kChunkBlocks * kReplayBlock >= (1 << 24), "chunks cover the largest buffer");

__global__ __launch_bounds__(256) void k_weight_max(const float* __restrict__ weights, long long M, int nblk,
                                                    WsHeader* hdr, uint32_t* __restrict__ partial_max,
                                                    uint32_t* __restrict__ chunk_max) {
    __shared__ uint32_t wave_best[4];
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int chunk = 4 * blockIdx.x + wave;
    const int first = chunk * kChunkBlocks;
    uint32_t best = 0u;
    bool bad = false;
    if (first < nblk) {
        const int count = min(kChunkBlocks, nblk - first);    // wave-uniform
        float4 v[kChunkBlocks];
        if (count == kChunkBlocks && (long long)(first + kChunkBlocks) * kReplayBlock <= M) {
            const float4* src = reinterpret_cast<const float4*>(weights + (long long)first * kReplayBlock) + lane;
#pragma unroll
            for (int j = 0; j < kChunkBlocks; ++j) v[j] = src[j * kWave];
        } else {                                               // the chunk that holds the end of the buffer
#pragma unroll
            for (int j = 0; j < kChunkBlocks; ++j) {
                v[j] = make_float4(0.f, 0.f, 0.f, 0.f);
                if (j < count) v[j] = load_block_quad(weights, M, first + j, lane);
            }
        }
        // Non-negative finite floats order like their bit patterns and lie below 0x7F800000: when the
        // plain unsigned maximum of this lane's bit patterns is below that, every entry was valid.
        uint32_t raw = 0u;
#pragma unroll
        for (int j = 0; j < kChunkBlocks; ++j) {
            raw = max(max(raw, float_to_bits(v[j].x)), float_to_bits(v[j].y));
            raw = max(max(raw, float_to_bits(v[j].z)), float_to_bits(v[j].w));
        }
        if (raw < 0x7F800000u) {
            best = raw;
        } else {                                               // -0, negative, infinite or NaN among them
#pragma unroll
            for (int j = 0; j < kChunkBlocks; ++j) best = max(best, quad_max_bits(v[j], bad));
        }
    }
    best = wave_max_u32(best);
    const bool any_bad = __any(bad);
    if (lane == 0) {
        chunk_max[chunk] = best;
        wave_best[wave] = best;
        if (any_bad) atomicOr(&hdr->flags, 0x2u);
    }
    __syncthreads();
    if (threadIdx.x == 0)
        partial_max[blockIdx.x] = max(max(wave_best[0], wave_best[1]), max(wave_best[2], wave_best[3]));
}

// Maximum of the kMaxParts partial maxima; every thread of a workgroup of NT threads calls it.
template <int NT>
__device__ __forceinline__ uint32_t reduce_partial_max(const uint32_t* __restrict__ partial_max, uint32_t* lds_waves) {
    uint32_t best = 0u;
    for (int i = threadIdx.x; i < kMaxParts; i += NT) best = max(best, partial_max[i]);
#pragma unroll
    for (int d = 32; d >= 1; d >>= 1) best = max(best, (uint32_t)__shfl_xor((int)best, d, kWave));
    if ((threadIdx.x & 63) == 0) lds_waves[threadIdx.x >> 6] = best;
    __syncthreads();
    uint32_t wb = 0u;
#pragma unroll
    for (int w = 0; w < NT / kWave; ++w) wb = max(wb, lds_waves[w]);
    return wb;
}

// Inclusive scan over the first 256 threads (4 waves) of a workgroup.  EVERY thread of the
// workgroup must call it (it contains a barrier); the result is meaningful for threads < 256.
__device__ __forceinline__ unsigned long long scan256(unsigned long long v, unsigned long long* wave_tot4,
                                                      unsigned long long& total) {
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    unsigned long long incl = v;
#pragma unroll
    for (int d = 1; d < kWave; d <<= 1) {
        unsigned long long up = __shfl_up(incl, d, kWave);
        if (lane >= d) incl += up;
    }
    if (lane == 63 && wave < 4) wave_tot4[wave] = incl;
    __syncthreads();
    unsigned long long before = 0ull;
    total = 0ull;
#pragma unroll
    for (int w = 0; w < 4; ++w) { if (w < wave) before += wave_tot4[w]; total += wave_tot4[w]; }
    return before + incl;
}

// Cross-lane moves inside a row of 16 lanes as DPP operands of ordinary vector instructions
// (no trip through the LDS crossbar, which is what __shfl costs).  CTRL: 0x110 | n shifts the
// row right by n lanes (lanes without a source read 0), 0x120 | n rotates it, 0x00..0xFF permute
// each quad of lanes.
template <int CTRL>
__device__ __forceinline__ unsigned long long dpp_u64(unsigned long long v) {
    const int lo = __builtin_amdgcn_update_dpp(0, (int)(uint32_t)v, CTRL, 0xF, 0xF, true);
    const int hi = __builtin_amdgcn_update_dpp(0, (int)(uint32_t)(v >> 32), CTRL, 0xF, 0xF, true);
    return ((unsigned long long)(uint32_t)hi << 32) | (uint32_t)lo;
}
constexpr int kDppQuadXor1 = 0xB1, kDppQuadXor2 = 0x4E;   // quad_perm [1,0,3,2] and [2,3,0,1]

// Sum over each quad of lanes -- 16 consecutive weights, a sub-block, when every lane holds four
// -- left in all four lanes; the quad's first lane stores it as the sub-block's entry.
__device__ __forceinline__ unsigned long long quad_sum_u64(unsigned long long v) {
    v += dpp_u64<kDppQuadXor1>(v);
    v += dpp_u64<kDppQuadXor2>(v);
    return v;
}
// Sum over a row of 16 lanes, left in all of them: rotations by 8, 4, 2, 1 (by 8 and 4 only when
// the four lanes of every quad already hold the same value, which is then counted once).
template <bool QUADS>
__device__ __forceinline__ unsigned long long row_sum_u64(unsigned long long v) {
    v += dpp_u64<0x128>(v);
    v += dpp_u64<0x124>(v);
    if constexpr (!QUADS) {
        v += dpp_u64<0x122>(v);
        v += dpp_u64<0x121>(v);
    }
    return v;
}
// Inclusive scan along a row of 16 lanes.
__device__ __forceinline__ unsigned long long row_scan_u64(unsigned long long v) {
    v += dpp_u64<0x111>(v);
    v += dpp_u64<0x112>(v);
    v += dpp_u64<0x114>(v);
    v += dpp_u64<0x118>(v);
    return v;
}
// Every 16th entry of a super-block's prefix is kept a second time, contiguously: a draw's first
// probe then reads one 128-byte line instead of 16 lines 128 bytes apart.
__device__ __forceinline__ void store_coarse(unsigned long long* __restrict__ coarse_cum, int sblk, int pos,
                                             unsigned long long incl) {
    if ((pos & 15) == 15) coarse_cum[sblk * 16 + (pos >> 4)] = incl;
}
__device__ __forceinline__ void store_sub_sum(unsigned long long* __restrict__ sub_sum, int blk, int lane,
                                              unsigned long long quad) {
    if ((lane & 3) == 0) sub_sum[(long long)blk * kSubsPerBlock + (lane >> 2)] = quad;
}

// Four wave-wide sums at once: in each of two exchange rounds a lane hands half of its partial
// sums to the partner lane and keeps the other half (the number of live values halves, the
// number of lanes sharing each doubles); more rounds finish the one value left -- four, or
// two when the inputs are quad sums already (QUADS: each value counted once per quad).
// Returns, in lane L, the wave-wide sum of part[L >> 4] (7 shuffles instead of 24).
template <bool QUADS = false>
__device__ __forceinline__ unsigned long long transposed_sum4(unsigned long long (&part)[4], int lane) {
#pragma unroll
    for (int s = 0; s < 2; ++s) {
        const int half = 2 >> s, mask = 32 >> s;
        const bool upper = (lane & mask) != 0;
#pragma unroll
        for (int i = 0; i < half; ++i) {
            const unsigned long long keep = upper ? part[i + half] : part[i];
            const unsigned long long send = upper ? part[i] : part[i + half];
            part[i] = keep + __shfl_xor(send, mask, kWave);
        }
    }
    return row_sum_u64<QUADS>(part[0]);
}

// quantise for a guessed exponent: a weight above 2^e would leave the range the conversions
// are defined on, so the scaled value is capped (such a sum is thrown away afterwards).
__device__ __forceinline__ unsigned long long quantise_capped(float w, int e) {
    const uint32_t b = float_to_bits(w);
    const float wc = b < 0x7F800000u ? w : 0.f;
    const float x = fminf(ldexpf(wc, 39 - e), 1099511627776.f);               // 2^40
    const uint32_t hi = (uint32_t)(x * 2.3283064365386963e-10f);
    const uint32_t lo = (uint32_t)fmaf(-(float)hi, 4294967296.f, x);
    return ((unsigned long long)hi << 32) | lo;
}

// ... and for a weight known to be valid and below 2^e (see k_super_sums): nothing to test or cap.
__device__ __forceinline__ unsigned long long quantise_plain(float w, int e) {
    const float x = ldexpf(w, 39 - e);
    const uint32_t hi = (uint32_t)(x * 2.3283064365386963e-10f);
    const uint32_t lo = (uint32_t)fmaf(-(float)hi, 4294967296.f, x);
    return ((unsigned long long)hi << 32) | lo;
}
// Bit pattern of the float 2^e (0 when 2^e is below the smallest subnormal, +inf's when above the largest).
__device__ __forceinline__ uint32_t pow2_bits(int e) {
    if (e > 127) return 0x7F800000u;
    if (e >= -126) return (uint32_t)(e + 127) << 23;
    if (e >= -149) return 1u << (e + 149);
    return 0u;
}

// The sweep of large buffers: one workgroup of 1024 threads per super-block (65536 weights);
// each wave sums 16 blocks of 256 weights as integers, then the 256 block sums are scanned in
// LDS.  Writes the within-super-block inclusive prefixes and the super-block's total.
//
// The exponent e = ilogb(max w) + 1 is only known once every weight has been seen, which
// would make a rebuild two sweeps.  Between rebuilds it hardly ever changes, so:
//   SPEC = true   one sweep that finds the maxima (chunk_max, partial_max, the bad-weight flag)
//                 AND sums with the exponent of the index as it stands, a guess;
//   SPEC = false  reduces partial_max to the true exponent and returns at once when the guess
//                 was right (or the buffer has no mass: all sums are zero for any exponent);
//                 otherwise it is the second sweep, with the true exponent.
// With a gate, either runs only when *gate is nonzero.
template <bool SPEC>
__global__ __launch_bounds__(1024) void k_super_sums(const float* __restrict__ weights, long long M, WsHeader* hdr,
                                                     uint32_t* __restrict__ partial_max,
                                                     uint32_t* __restrict__ chunk_max,
                                                     unsigned long long* __restrict__ block_cum, int nblk,
                                                     unsigned long long* __restrict__ super_raw,
                                                     unsigned long long* __restrict__ sub_sum,
                                                     unsigned long long* __restrict__ coarse_cum,
                                                     const uint32_t* __restrict__ gate) {
    __shared__ unsigned long long sums[kSuperBlocks];
    __shared__ unsigned long long wave_tot4[4];
    __shared__ uint32_t wave_best[16];
    if (gate && *gate == 0u) return;
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    // the grid is the number of super-blocks rounded up to a multiple of 8: workgroups go to the
    // chip's 8 XCDs in turn, and XCD x takes the x-th eighth of the super-blocks, one contiguous region
    const int nsuper = (nblk + kSuperBlocks - 1) / kSuperBlocks;
    const int sblk = (int)xcd_contiguous_block();
    if (sblk >= nsuper) return;                    // the whole workgroup leaves
    int e = 0;
    if constexpr (!SPEC) {   // decided before any weight is read: this is usually all the kernel does
        const uint32_t wb = reduce_partial_max<1024>(partial_max, wave_best);
        if (wb == 0u) return;                          // the same for every thread of every workgroup
        e = exponent_of(wb);
        if (e == hdr->exponent) return;
    }
    float4 v[16];
    const int blk_first = sblk * kSuperBlocks + wave * 16;
    if ((long long)(blk_first + 16) * kReplayBlock <= M) {     // wave-uniform: all 16 blocks inside the buffer
        const float4* src = reinterpret_cast<const float4*>(weights + (long long)blk_first * kReplayBlock) + lane;
#pragma unroll
        for (int j = 0; j < 16; ++j) v[j] = src[j * kWave];
    } else {
#pragma unroll
        for (int j = 0; j < 16; ++j) v[j] = load_block_quad(weights, M, blk_first + j, lane);
    }
    // SPEC: a weight whose bit pattern is below `safe` is valid (non-negative, finite) and below
    // 2^e, so it needs neither the validity test nor the cap; whole batches of such weights --
    // practically all of them -- are quantised by the short form.  The maxima are taken batch by
    // batch as well, so that nothing waits for the last load before the first is used.
    uint32_t raw = 0u, safe = 0u;
    if constexpr (SPEC) {
        e = hdr->exponent;
        safe = min(0x7F800000u, pow2_bits(e));
        // partial_max entries past the last super-block must not keep an older, larger buffer's maxima
        if (sblk == 0) for (int i = 4 * nsuper + tid; i < kMaxParts; i += 1024) partial_max[i] = 0u;
    }
    // Four blocks at a time, so that a wave starts reducing as soon as its first four loads are
    // back while the rest are still in flight; lane L ends up with the sum of block 4g + (L >> 4).
#pragma unroll
    for (int g = 0; g < 4; ++g) {
        unsigned long long part[4];
        bool plain = false;
        if constexpr (SPEC) {
            uint32_t rb = 0u;
#pragma unroll
            for (int j = 0; j < 4; ++j) {
                const float4 w = v[4 * g + j];
                rb = max(max(rb, float_to_bits(w.x)), float_to_bits(w.y));
                rb = max(max(rb, float_to_bits(w.z)), float_to_bits(w.w));
            }
            raw = max(raw, rb);
            plain = __all(rb < safe);                      // wave-uniform
        }
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            const float4 w = v[4 * g + j];
            if constexpr (SPEC) {
                if (plain)
                    part[j] = quantise_plain(w.x, e) + quantise_plain(w.y, e) + quantise_plain(w.z, e) +
                              quantise_plain(w.w, e);
                else
                    part[j] = quantise_capped(w.x, e) + quantise_capped(w.y, e) + quantise_capped(w.z, e) +
                              quantise_capped(w.w, e);
            } else {
                part[j] = quantise(w.x, e) + quantise(w.y, e) + quantise(w.z, e) + quantise(w.w, e);
            }
            part[j] = quad_sum_u64(part[j]);
        }
        {   // one store for the four blocks: lane 4i + r writes sub-block i of block 4g + r
            const int r = lane & 3;
            const unsigned long long mine = r == 0 ? part[0] : r == 1 ? part[1] : r == 2 ? part[2] : part[3];
            const int blk = blk_first + 4 * g + r;
            if (blk < nblk) sub_sum[(long long)blk * kSubsPerBlock + (lane >> 2)] = mine;
        }
        const unsigned long long sum = transposed_sum4<true>(part, lane);
        if ((lane & 15) == 0) sums[wave * 16 + 4 * g + (lane >> 4)] = sum;
    }
    if constexpr (SPEC) {
        // this wave's 16 blocks are chunk 16*sblk + wave (see k_weight_max for the two paths)
        uint32_t best = 0u;
        bool bad = false;
        if (raw < 0x7F800000u) {
            best = raw;
        } else {
#pragma unroll
            for (int j = 0; j < 16; ++j) best = max(best, quad_max_bits(v[j], bad));
        }
        best = wave_max_u32(best);
        const bool any_bad = __any(bad);
        if (lane == 0) {
            chunk_max[sblk * 16 + wave] = best;
            wave_best[wave] = best;
            if (any_bad) atomicOr(&hdr->flags, 0x2u);
        }
    }
    __syncthreads();
    if constexpr (SPEC) {
        if (tid < 4)
            partial_max[4 * sblk + tid] = max(max(wave_best[4 * tid], wave_best[4 * tid + 1]),
                                              max(wave_best[4 * tid + 2], wave_best[4 * tid + 3]));
    }
    unsigned long long total = 0ull;
    const unsigned long long incl = scan256(tid < kSuperBlocks ? sums[tid] : 0ull, wave_tot4, total);
    if (tid < kSuperBlocks) {
        const int blk = sblk * kSuperBlocks + tid;
        if (blk < nblk) { block_cum[blk] = incl; store_coarse(coarse_cum, sblk, tid, incl); }
        if (tid == 0) super_raw[sblk] = total;
    }
}

// Pass B for buffers of few super-blocks, where one workgroup per super-block would leave the
// chip idle: integer sum of each block of 256 weights, one wave per block, raw sums to block_cum.
__global__ __launch_bounds__(256) void k_block_sums(const float* __restrict__ weights, long long M,
                                                    const uint32_t* __restrict__ partial_max,
                                                    unsigned long long* __restrict__ block_cum, int nblk,
                                                    unsigned long long* __restrict__ sub_sum) {
    __shared__ uint32_t wave_best[4];
    const int lane = threadIdx.x & 63;
    const int blk = (int)(((long long)blockIdx.x * blockDim.x + threadIdx.x) >> 6);
    const uint32_t wb = reduce_partial_max<256>(partial_max, wave_best);
    if (blk >= nblk) return;
    unsigned long long q = 0ull;
    if (wb != 0u) {
        const int e = exponent_of(wb);
        const long long base = (long long)blk * kReplayBlock + lane * 4;
        if (base + 3 < M) {
            const float4 v = *reinterpret_cast<const float4*>(weights + base);
            q = quantise(v.x, e) + quantise(v.y, e) + quantise(v.z, e) + quantise(v.w, e);
        } else {
            for (int j = 0; j < 4; ++j) if (base + j < M) q += quantise(weights[base + j], e);
        }
    }
    store_sub_sum(sub_sum, blk, lane, quad_sum_u64(q));
    q = wave_sum_u64(q);
    if (lane == 0) block_cum[blk] = q;
}

// ... followed by the in-place inclusive scan of each super-block's 256 raw block sums.
// With a single super-block (gridDim.x == 1) it also does the work of k_prefix_super.
__global__ __launch_bounds__(256) void k_scan_supers(unsigned long long* __restrict__ block_cum, int nblk,
                                                     unsigned long long* __restrict__ super_raw,
                                                     const uint32_t* __restrict__ partial_max, WsHeader* hdr,
                                                     WsIndexState* ist, long long M,
                                                     unsigned long long* __restrict__ coarse_cum) {
    __shared__ unsigned long long wave_tot4[4];
    __shared__ uint32_t wave_best[4];
    const int blk = blockIdx.x * kSuperBlocks + threadIdx.x;
    unsigned long long total = 0ull;
    const unsigned long long incl = scan256(blk < nblk ? block_cum[blk] : 0ull, wave_tot4, total);
    if (blk < nblk) { block_cum[blk] = incl; store_coarse(coarse_cum, blockIdx.x, threadIdx.x, incl); }
    if (gridDim.x > 1) {
        if (threadIdx.x == 0) super_raw[blockIdx.x] = total;
        return;
    }
    const uint32_t wb = reduce_partial_max<256>(partial_max, wave_best);
    super_raw[threadIdx.x] = total;            // all 256 entries: the only super-block, then padding
    if (threadIdx.x == 0) {
        hdr->wmax_bits = wb;
        hdr->total = total;
        hdr->exponent = wb ? exponent_of(wb) : 0;
        if (total == 0ull) atomicOr(&hdr->flags, 0x4u);
        ist->index_M = M;
        ist->rebuild = 0u;
    }
}

// Pass C: inclusive prefix of the (at most 256) super-block totals, padded with Total; also
// publishes Total, the exponent and the no-mass flag.
__global__ __launch_bounds__(256) void k_prefix_super(unsigned long long* __restrict__ super_cum, int nsuper,
                                                      const uint32_t* __restrict__ partial_max, WsHeader* hdr,
                                                      WsIndexState* ist, long long M) {
    __shared__ unsigned long long wave_tot4[4];
    __shared__ uint32_t wave_best[4];
    const int tid = threadIdx.x;
    const uint32_t wb = reduce_partial_max<256>(partial_max, wave_best);
    unsigned long long total = 0ull;
    const unsigned long long incl = scan256(tid < nsuper ? super_cum[tid] : 0ull, wave_tot4, total);
    super_cum[tid] = incl;    // entries past nsuper repeat Total
    if (tid == 0) {
        hdr->wmax_bits = wb;
        hdr->total = total;
        hdr->exponent = wb ? exponent_of(wb) : 0;
        if (total == 0ull) atomicOr(&hdr->flags, 0x4u);
        ist->index_M = M;     // chunk_max, partial_max and the prefixes describe these M weights
        ist->rebuild = 0u;
    }
}

// ---- Patching the index after a contiguous insert (Appendix A.4.2, circular buffer) ----------
// Inserting K entries at the cursor changes the blocks b0, b0+1, ... (nt of them, circularly);
// everything else in the index stays valid as long as the exponent e = ilogb(max w) + 1 does.
//   1. k_insert_patch   four workgroups per touched chunk of 16 blocks, one wave per block: store
//                       the new weights, leave the maximum of each quarter chunk in quarter_max
//                       and each block's integer sum under the standing exponent in touched_sum
//   2. k_patch_supers   one workgroup per touched super-block: new maximum of the buffer from
//                       partial_max / chunk_max / quarter_max; same exponent -> put the touched
//                       blocks' new sums in, rescan the super-block; otherwise raise the rebuild gate
//   3. k_super_sums<true>, <false> with the gate: the ordinary rebuild, which runs only then
//   4. k_patch_finish   prefix over the super-block totals, header
// No step waits for the host, so the choice between patch and rebuild is taken on the device.

// A block is touched when its circular distance from b0 is below nt.
__device__ __forceinline__ bool in_circular(int x, int start, int count, int modulus) {
    int d = x - start;
    if (d < 0) d += modulus;
    return d < count;
}

__global__ __launch_bounds__(256) void k_insert_patch(float* __restrict__ weights, long long M, int nblk, int nchunk,
                                                      long long cursor, const float* __restrict__ prio, long long K,
                                                      float alpha, long long* __restrict__ slots_out, int c0,
                                                      WsHeader* hdr, uint32_t* __restrict__ quarter_max,
                                                      unsigned long long* __restrict__ touched_sum,
                                                      unsigned long long* __restrict__ sub_sum) {
    __shared__ uint32_t wave_best[4];
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    int chunk = c0 + (int)(blockIdx.x >> 2);     // the touched chunks c0, c0+1, ... (circular)
    if (chunk >= nchunk) chunk -= nchunk;
    const int quarter = 4 * chunk + (int)(blockIdx.x & 3);
    const int blk = 4 * quarter + wave;
    uint32_t best = 0u;
    bool bad = false;
    if (blk < nblk) {                            // wave-uniform
        const long long base = (long long)blk * kReplayBlock + lane * 4;
        float w[4] = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
        for (int c = 0; c < 4; ++c) {
            const long long i = base + c;
            if (i >= M) continue;
            long long k = i - cursor;
            if (k < 0) k += M;
            if (k < K) {                         // K <= M here: every slot receives at most one entry
                double p = (double)prio[k];
                if (!(p > 0.0)) p = 0.0;
                w[c] = (float)pow(p, (double)alpha);
                weights[i] = w[c];
                if (slots_out) slots_out[k] = i;
            } else {
                w[c] = weights[i];
            }
        }
        best = wave_max_u32(quad_max_bits(make_float4(w[0], w[1], w[2], w[3]), bad));
        // the block's integer sum under the standing exponent, a guess that k_patch_supers checks
        const int e = hdr->exponent;
        const unsigned long long mine = quantise_capped(w[0], e) + quantise_capped(w[1], e) +
                                        quantise_capped(w[2], e) + quantise_capped(w[3], e);
        store_sub_sum(sub_sum, blk, lane, quad_sum_u64(mine));    // stands if the guess does; else all are rewritten
        const unsigned long long q = wave_sum_u64(mine);
        if (lane == 0) touched_sum[4 * blockIdx.x + wave] = q;    // by position: block 16*c0 is entry 0
    }
    const bool any_bad = __any(bad);
    if (lane == 0) {
        wave_best[wave] = best;
        if (any_bad) atomicOr(&hdr->flags, 0x2u);
    }
    __syncthreads();
    if (threadIdx.x == 0)
        quarter_max[quarter] = max(max(wave_best[0], wave_best[1]), max(wave_best[2], wave_best[3]));
}

__global__ __launch_bounds__(1024) void k_patch_supers(long long M, int nblk, int b0, int nt, int c0, int nc,
                                                       int nchunk, int s0, int nsuper,
                                                       const WsHeader* __restrict__ hdr, WsIndexState* ist,
                                                       uint32_t* __restrict__ partial_max,
                                                       uint32_t* __restrict__ chunk_max,
                                                       const uint32_t* __restrict__ quarter_max,
                                                       const unsigned long long* __restrict__ touched_sum,
                                                       unsigned long long* __restrict__ block_cum,
                                                       unsigned long long* __restrict__ super_new,
                                                       unsigned long long* __restrict__ coarse_cum) {
    __shared__ unsigned long long wave_tot4[4];
    __shared__ uint32_t wave_best[16];
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    int s = s0 + blockIdx.x;
    if (s >= nsuper) s -= nsuper;
    const int blk0 = s * kSuperBlocks;

    // Everything the kernel reads is asked for up front: the standing exponent, the capacity the
    // index was built for, and this super-block's block sums -- a touched block's from
    // k_insert_patch, the others' from the differences of the old prefix.
    const int e = hdr->exponent;
    const long long index_M = ist->index_M;
    unsigned long long sum = 0ull;
    if (tid < kSuperBlocks && blk0 + tid < nblk) {
        const int blk = blk0 + tid;
        if (in_circular(blk, b0, nt, nblk)) {
            int cpos = blk / kChunkBlocks - c0;
            if (cpos < 0) cpos += nchunk;
            sum = touched_sum[cpos * kChunkBlocks + (blk & (kChunkBlocks - 1))];
        } else {
            sum = block_cum[blk] - (tid > 0 ? block_cum[blk - 1] : 0ull);
        }
    }

    // New maximum of the whole buffer: thread g answers for the four chunks 4g .. 4g+3 that
    // partial_max[g] covers.  A touched chunk has its new maximum in the four quarter maxima
    // k_insert_patch left (workgroup 0 stores it to chunk_max, and the group's to partial_max);
    // the others still have theirs in chunk_max / partial_max, which nobody writes here.
    uint32_t best = 0u;
    {
        const int first = 4 * tid, last = min(first + 4, nchunk);
        if (first < last) {
            const bool touched = in_circular(first, c0, nc, nchunk) || (c0 >= first && c0 < last);
            if (touched) {
                for (int c = first; c < last; ++c) {
                    uint32_t m;
                    if (in_circular(c, c0, nc, nchunk)) {
                        m = max(max(quarter_max[4 * c], quarter_max[4 * c + 1]),
                                max(quarter_max[4 * c + 2], quarter_max[4 * c + 3]));
                        if (blockIdx.x == 0) chunk_max[c] = m;
                    } else {
                        m = chunk_max[c];
                    }
                    best = max(best, m);
                }
                if (blockIdx.x == 0) partial_max[tid] = best;
            } else {
                best = partial_max[tid];
            }
        }
    }
    best = wave_max_u32(best);
    if (lane == 0) wave_best[wave] = best;
    __syncthreads();
    uint32_t wb = 0u;
#pragma unroll
    for (int w = 0; w < 16; ++w) wb = max(wb, wave_best[w]);

    const bool rebuild = index_M != M || wb == 0u || exponent_of(wb) != e;
    if (rebuild) {           // the same for every thread of every workgroup
        if (blockIdx.x == 0 && tid == 0) ist->rebuild = 1u;
        return;
    }
    unsigned long long total = 0ull;
    const unsigned long long incl = scan256(sum, wave_tot4, total);   // sum is 0 for tid >= 256
    if (tid < kSuperBlocks) {
        const int blk = blk0 + tid;
        if (blk < nblk) { block_cum[blk] = incl; store_coarse(coarse_cum, s, tid, incl); }
        if (tid == 0) super_new[s] = total;
    }
}

// Last step of a patch: raw super-block totals are the new ones (super_new) for the touched
// super-blocks -- for all of them after a gated rebuild -- and the differences of the old
// prefix for the rest; then as k_prefix_super.
__global__ __launch_bounds__(256) void k_patch_finish(unsigned long long* __restrict__ super_cum,
                                                      const unsigned long long* __restrict__ super_new, int nsuper,
                                                      int s0, int ns, const uint32_t* __restrict__ partial_max,
                                                      WsHeader* hdr, WsIndexState* ist, long long M) {
    __shared__ unsigned long long wave_tot4[4];
    __shared__ uint32_t wave_best[4];
    const int tid = threadIdx.x;
    const bool rebuilt = ist->rebuild != 0u;
    const uint32_t wb = reduce_partial_max<256>(partial_max, wave_best);   // barrier: every thread has read the gate
    unsigned long long raw = 0ull;
    if (tid < nsuper) {
        if (rebuilt || in_circular(tid, s0, ns, nsuper)) raw = super_new[tid];
        else raw = super_cum[tid] - (tid > 0 ? super_cum[tid - 1] : 0ull);
    }
    unsigned long long total = 0ull;
    const unsigned long long incl = scan256(raw, wave_tot4, total);        // barrier before the stores below
    super_cum[tid] = incl;    // entries past nsuper repeat Total
    if (tid == 0) {
        hdr->wmax_bits = wb;
        hdr->total = total;
        hdr->exponent = wb ? exponent_of(wb) : 0;
        if (total == 0ull) atomicOr(&hdr->flags, 0x4u);
        ist->index_M = M;
        ist->rebuild = 0u;
    }
}

// Small buffers (M <= kSmallReplay): the whole update -- tag, commit, maximum, block sums, prefix --
// in ONE workgroup of 1024 threads, phases separated by workgroup barriers.  Five dependent
// launches cost more than the work itself at this size; one compute unit stops paying off
// beyond a few thousand weights (measured: 50 us at M = 65536 against 22 us for five launches).
constexpr int kSmallReplay = 1 << 13;   // 32 indexed blocks (the scan phase handles up to 1024)
constexpr int kSmallBatch = 1 << 13;
constexpr int kFusedSuperMin = 64;      // from this many super-blocks on, one workgroup per super-block

__global__ __launch_bounds__(1024) void k_update_small(
    float* __restrict__ weights, int M, const long long* __restrict__ idx, const float* __restrict__ prio,
    int K, float alpha, WsHeader* hdr, WsIndexState* ist, unsigned long long* __restrict__ block_cum, int nblk,
    unsigned long long* __restrict__ super_cum, unsigned long long* __restrict__ sub_sum,
    unsigned long long* __restrict__ coarse_cum) {
    __shared__ unsigned long long sums[1024];
    __shared__ unsigned long long wave_tot[16];
    __shared__ uint32_t wave_max_bits[16];
    __shared__ int any_bad;
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    uint32_t* wbits = reinterpret_cast<uint32_t*>(weights);
    if (tid == 0) any_bad = 0;

    // 1. tag: the last occurrence of an index carries the largest tag
    for (int k = tid; k < K; k += 1024) {
        const long long i = idx[k];
        if (i < 0 || i >= M) { atomicOr(&hdr->flags, 0x8u); continue; }
        claim_slot(wbits + i, (uint32_t)k, idx, K, i);
    }
    __syncthreads();
    // 2. commit: exactly the winning k stores its weight
    for (int k = tid; k < K; k += 1024) {
        const long long i = idx[k];
        if (i < 0 || i >= M) continue;
        const uint32_t seen = __hip_atomic_load(wbits + i, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        if (seen != (kTagBase | (uint32_t)k)) continue;
        double p = (double)prio[k];
        if (!(p > 0.0)) p = 0.0;
        __hip_atomic_store(weights + i, (float)pow(p, (double)alpha), __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    }
    __syncthreads();
    // 3. largest valid weight
    uint32_t best = 0u;
    bool bad = false;
#pragma unroll 8
    for (int i = tid; i < M; i += 1024) {
        const uint32_t b = __hip_atomic_load(wbits + i, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        if (b < 0x7F800000u) best = max(best, b);
        else if (b != 0x80000000u) bad = true;
    }
#pragma unroll
    for (int d = 32; d >= 1; d >>= 1) best = max(best, (uint32_t)__shfl_xor((int)best, d, kWave));
    if (__any(bad) && lane == 0) any_bad = 1;
    if (lane == 0) wave_max_bits[wave] = best;
    __syncthreads();
    uint32_t wb = 0u;
    for (int w = 0; w < 16; ++w) wb = max(wb, wave_max_bits[w]);
    const int e = wb ? exponent_of(wb) : 0;
    // 4. integer sum of each block of 256 weights, one wave per block
    for (int blk = wave; blk < nblk; blk += 16) {
        unsigned long long q = 0ull;
        if (wb != 0u) {
            const int base = blk * kReplayBlock + lane * 4;
            for (int j = 0; j < 4; ++j)
                if (base + j < M)
                    q += quantise(bits_to_float(__hip_atomic_load(wbits + base + j, __ATOMIC_RELAXED,
                                                                  __HIP_MEMORY_SCOPE_AGENT)), e);
        }
        store_sub_sum(sub_sum, blk, lane, quad_sum_u64(q));
        q = wave_sum_u64(q);
        if (lane == 0) sums[blk] = q;
    }
    __syncthreads();
    // 5. inclusive prefix over the (at most 1024) block sums
    const unsigned long long mine = tid < nblk ? sums[tid] : 0ull;
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
    if (tid < nblk) { block_cum[tid] = before + incl; store_coarse(coarse_cum, 0, tid, before + incl); }
    if (tid < kSuperBlocks) super_cum[tid] = total;   // a single super-block
    if (tid == 0) {
        hdr->wmax_bits = wb;
        hdr->total = total;
        hdr->exponent = e;
        uint32_t f = (any_bad ? 0x2u : 0u) | (total == 0ull ? 0x4u : 0u);
        if (f) atomicOr(&hdr->flags, f);
        ist->index_M = 0;     // this path keeps no per-block maxima
        ist->rebuild = 0u;
    }
}

// Sampling: a draw is served by a group of 16 lanes; a wave's four groups take two draws each,
// level by level side by side (eight draws per wave).  Each level of the
// index is a non-decreasing run of 256 u64 values searched 16-ary in two probes: lane g of the
// group first reads the last entry of the g-th run of 16 and the group counts (ballot +
// popcount) how many are <= t, which selects a run; then the lanes read that run's 16 entries
// and count again.  The entry just before the hit -- the mass to subtract -- is already in a
// register of some lane of the group and is fetched with a shuffle.
__device__ __forceinline__ int group_count(bool pred, int group) {
    return __popc((uint32_t)((__ballot(pred) >> (16 * group)) & 0xFFFFull));
}

// Rank of t in the 256-entry run `run` (entries at index >= limit count as +inf), and the entry
// just before that rank (0 for rank 0).  All 16 lanes of a group pass the same t.
// `coarse` holds run[15], run[31], .. contiguously.
__device__ __forceinline__ int search256(const unsigned long long* __restrict__ run,
                                         const unsigned long long* __restrict__ coarse, int limit,
                                         unsigned long long t, int group, int gl, unsigned long long& before) {
    const int ia = 16 * gl + 15;
    const unsigned long long va = ia < limit ? coarse[gl] : ~0ull;
    const int chunk = group_count(va <= t, group);                 // 0..16
    const int ib = 16 * min(chunk, 15) + gl;
    const unsigned long long vb = (chunk < 16 && ib < limit) ? run[ib] : ~0ull;
    const int within = group_count(vb <= t, group);                // 0..15 when chunk < 16
    const unsigned long long prev_b = __shfl(vb, 16 * group + max(within - 1, 0), kWave);
    const unsigned long long prev_a = __shfl(va, 16 * group + max(chunk - 1, 0), kWave);
    before = within > 0 ? prev_b : (chunk > 0 ? prev_a : 0ull);
    return chunk < 16 ? 16 * chunk + within : 256;
}

// D searches of the same kind side by side: the first probes of all of them go out together, then
// the second probes.  run/coarse/limit of search d: base + first[d], coarse_base + crs[d], nblk - first[d].
template <int D>
__device__ __forceinline__ void search256_many(const unsigned long long* __restrict__ base,
                                               const unsigned long long* __restrict__ coarse_base,
                                               const int (&first)[D], const int (&crs)[D], int nblk,
                                               const unsigned long long (&t)[D], int group, int gl,
                                               int (&rank)[D], unsigned long long (&before)[D]) {
    unsigned long long va[D], vb[D];
    int chunk[D];
    const int ia = 16 * gl + 15;
#pragma unroll
    for (int d = 0; d < D; ++d) va[d] = ia < nblk - first[d] ? coarse_base[crs[d] + gl] : ~0ull;
#pragma unroll
    for (int d = 0; d < D; ++d) chunk[d] = group_count(va[d] <= t[d], group);          // 0..16
#pragma unroll
    for (int d = 0; d < D; ++d) {
        const int ib = 16 * min(chunk[d], 15) + gl;
        vb[d] = (chunk[d] < 16 && ib < nblk - first[d]) ? base[first[d] + ib] : ~0ull;
    }
#pragma unroll
    for (int d = 0; d < D; ++d) {
        const int within = group_count(vb[d] <= t[d], group);                            // 0..15 when chunk < 16
        const unsigned long long prev_b = __shfl(vb[d], 16 * group + max(within - 1, 0), kWave);
        const unsigned long long prev_a = __shfl(va[d], 16 * group + max(chunk[d] - 1, 0), kWave);
        before[d] = within > 0 ? prev_b : (chunk[d] > 0 ? prev_a : 0ull);
        rank[d] = chunk[d] < 16 ? 16 * chunk[d] + within : 256;
    }
}

constexpr int kDrawsPerGroup = 2;   // draws a group of 16 lanes works on at a time

__global__ __launch_bounds__(256) void k_sample(
    const float* __restrict__ weights, long long M, const WsHeader* __restrict__ hdr,
    const unsigned long long* __restrict__ block_cum, int nblk,
    const unsigned long long* __restrict__ super_cum, const unsigned long long* __restrict__ sub_sum,
    const unsigned long long* __restrict__ coarse_cum, const double* __restrict__ uniforms, int K, long long* __restrict__ idx_out, float* __restrict__ prob_out,
    uint32_t* __restrict__ flags) {
    // The 256 super-block prefixes are the same for every draw: one load per thread brings them
    // into LDS, which takes the first level's two dependent probes off the global-memory path.
    __shared__ unsigned long long super_lds[kSuperBlocks];
    __shared__ unsigned long long super_coarse[16];  // entries 15, 31, .. again, side by side (no bank conflicts)
    {
        const unsigned long long sc = super_cum[threadIdx.x];
        super_lds[threadIdx.x] = sc;
        if ((threadIdx.x & 15) == 15) super_coarse[threadIdx.x >> 4] = sc;
    }
    __syncthreads();                                 // before any wave may leave
    constexpr int D = kDrawsPerGroup;
    const int lane = threadIdx.x & 63, group = lane >> 4, gl = lane & 15;
    const int wave_id = (int)(((long long)blockIdx.x * blockDim.x + threadIdx.x) >> 6);
    if ((long long)wave_id * (4 * D) >= K) return;   // whole waves leave together
    // A draw is a chain of five dependent reads; a group walks D chains side by side, level by
    // level, so that the reads of one level are in flight together.
    int k[D]; bool live[D];
#pragma unroll
    for (int d = 0; d < D; ++d) {
        k[d] = (wave_id * 4 + group) * D + d;
        live[d] = k[d] < K;                          // dead draws run along on draw K-1 and store nothing
    }
    const unsigned long long total = hdr->total;
    if (total == 0ull) {
#pragma unroll
        for (int d = 0; d < D; ++d)
            if (live[d] && gl == 0) { idx_out[k[d]] = -1; if (prob_out) prob_out[k[d]] = 0.f; }
        return;
    }
    unsigned long long rem[D];
#pragma unroll
    for (int d = 0; d < D; ++d) {
        double u = uniforms[live[d] ? k[d] : K - 1];
        if (!(u >= 0.0)) { u = 0.0; if (live[d] && gl == 0) atomicOr(flags, 0x10u); }
        // one rounding for the conversion, one for the product, then truncation
        const double prod = __dmul_rn(u, __ull2double_rn(total));
        unsigned long long t = (prod >= 18446744073709551616.0) ? total - 1 : (unsigned long long)prod;
        if (t > total - 1) t = total - 1;
        rem[d] = t;
    }
    // level 1: first super-block whose inclusive prefix exceeds t (the padding equals Total > t)
    bool stale[D]; int first[D], crs[D];
#pragma unroll
    for (int d = 0; d < D; ++d) {
        unsigned long long before;
        const int sblk = search256(super_lds, super_coarse, kSuperBlocks, rem[d], group, gl, before);
        stale[d] = sblk >= kSuperBlocks;             // cannot happen with a current index
        rem[d] -= stale[d] ? 0ull : before;
        first[d] = (stale[d] ? 0 : sblk) * kSuperBlocks;
        crs[d] = (stale[d] ? 0 : sblk) * 16;
    }
    // level 2: first block of that super-block whose inclusive prefix exceeds the remainder
    int blk[D];
    {
        int within[D]; unsigned long long before[D];
        search256_many<D>(block_cum, coarse_cum, first, crs, nblk, rem, group, gl, within, before);
#pragma unroll
        for (int d = 0; d < D; ++d) {
            stale[d] = stale[d] || within[d] >= kSuperBlocks || first[d] + within[d] >= nblk;
            blk[d] = stale[d] ? 0 : first[d] + within[d];
            rem[d] -= stale[d] ? 0ull : before[d];
        }
    }
    // level 3: the block's 16 sub-block sums, one per lane; the sub-block whose running total
    // first passes the remainder is the one hit
    unsigned long long sub[D];
#pragma unroll
    for (int d = 0; d < D; ++d) sub[d] = sub_sum[(long long)blk[d] * kSubsPerBlock + gl];
    int hit[D];
#pragma unroll
    for (int d = 0; d < D; ++d) {
        const unsigned long long sub_incl = row_scan_u64(sub[d]);       // the 16 lanes of a draw are one DPP row
        const int owner_sub = group_count(sub_incl <= rem[d], group);   // lanes whose running total has not passed rem yet
        // a stale index (weights changed without a rebuild) can run past the end: report -1
        stale[d] = stale[d] || owner_sub >= kSubsPerBlock;
        hit[d] = stale[d] ? 0 : owner_sub;
        rem[d] -= stale[d] ? 0ull : __shfl(sub_incl - sub[d], 16 * group + hit[d], kWave);
    }
    // level 4: the sub-block's 16 weights, one per lane
    const int e = exponent_of(hdr->wmax_bits);
    long long slot[D]; float wv[D];
#pragma unroll
    for (int d = 0; d < D; ++d) {
        slot[d] = (long long)blk[d] * kReplayBlock + hit[d] * kSubBlock + gl;
        wv[d] = slot[d] < M ? weights[slot[d]] : 0.f;
    }
#pragma unroll
    for (int d = 0; d < D; ++d) {
        const unsigned long long q = quantise(wv[d], e);
        const unsigned long long q_incl = row_scan_u64(q);
        const int owner = group_count(q_incl <= rem[d], group);
        if (stale[d] || owner >= kSubBlock) {
            if (live[d] && gl == 0) { idx_out[k[d]] = -1; if (prob_out) prob_out[k[d]] = 0.f; }
        } else if (live[d] && gl == owner) {
            idx_out[k[d]] = slot[d];
            if (prob_out) prob_out[k[d]] = (float)((double)q / (double)total);
        }
    }
}

hipError_t update_launch(float* weights, long long M, const long long* idx, const float* prio, int K,
                         float alpha, const ReplayWs& w, hipStream_t st) {
    const int nblk = (int)((M + kReplayBlock - 1) / kReplayBlock);
    const int nsuper = (nblk + kSuperBlocks - 1) / kSuperBlocks;
    if (M <= kSmallReplay && K <= kSmallBatch) {
        hipLaunchKernelGGL(k_update_small, dim3(1), dim3(1024), 0, st, weights, (int)M, idx, prio, K, alpha,
                           w.hdr, w.ist, w.block_cum, nblk, w.super_cum, w.sub_sum, w.coarse_cum);
        return hipGetLastError();
    }
    if (K > 0 && K <= kSmallBatch) {
        hipLaunchKernelGGL(k_update_scatter_small, dim3(1), dim3(1024), 0, st, weights, M, idx, prio, K, alpha, w.hdr);
    } else if (K > 0) {
        const unsigned g = (unsigned)((K + 255) / 256);
        hipLaunchKernelGGL(k_update_tag, dim3(g), dim3(256), 0, st, weights, M, idx, K, w.hdr);
        hipLaunchKernelGGL(k_update_commit, dim3(g), dim3(256), 0, st, weights, M, idx, prio, K, alpha);
    }
    if (nsuper >= kFusedSuperMin) {
        const uint32_t* always = nullptr;
        hipLaunchKernelGGL((k_super_sums<true>), dim3(round_up_8((unsigned)nsuper)), dim3(1024), 0, st, weights, M, w.hdr,
                           w.partial_max, w.chunk_max, w.block_cum, nblk, w.super_cum, w.sub_sum, w.coarse_cum, always);
        hipLaunchKernelGGL((k_super_sums<false>), dim3(round_up_8((unsigned)nsuper)), dim3(1024), 0, st, weights, M, w.hdr,
                           w.partial_max, w.chunk_max, w.block_cum, nblk, w.super_cum, w.sub_sum, w.coarse_cum, always);
    } else {
        hipLaunchKernelGGL(k_weight_max, dim3(kMaxParts), dim3(256), 0, st, weights, M, nblk, w.hdr, w.partial_max,
                           w.chunk_max);
        hipLaunchKernelGGL(k_block_sums, dim3((unsigned)((nblk + 3) / 4)), dim3(256), 0, st, weights, M,
                           w.partial_max, w.block_cum, nblk, w.sub_sum);
        hipLaunchKernelGGL(k_scan_supers, dim3((unsigned)nsuper), dim3(256), 0, st, w.block_cum, nblk, w.super_cum,
                           w.partial_max, w.hdr, w.ist, M, w.coarse_cum);
        if (nsuper == 1) return hipGetLastError();   // the scan kernel finalised the index itself
    }
    hipLaunchKernelGGL(k_prefix_super, dim3(1), dim3(256), 0, st, w.super_cum, nsuper, w.partial_max, w.hdr, w.ist, M);
    return hipGetLastError();
}

// Large buffers and short batches are patched; everything else is inserted and rebuilt.
constexpr int kPatchFraction = 8;   // patch when K <= M / kPatchFraction
static_assert((kMaxChunks / kPatchFraction + 2) * kChunkBlocks <= kMaxTouched, "touched_sum holds a patch's blocks");

hipError_t insert_launch(float* weights, long long M, long long cursor, const float* prio, long long K,
                         float alpha, long long* slots_out, const ReplayWs& w, hipStream_t st) {
    const int nblk = (int)((M + kReplayBlock - 1) / kReplayBlock);
    const int nsuper = (nblk + kSuperBlocks - 1) / kSuperBlocks;
    // (K <= M/8 keeps the touched chunks, at most K/4096 + 2 of them, within touched_sum)
    if (K > 0 && nsuper >= kFusedSuperMin && K <= M / kPatchFraction && K / (kChunkBlocks * kReplayBlock) + 2 <= kMaxTouched / kChunkBlocks) {
        const int nchunk = (nblk + kChunkBlocks - 1) / kChunkBlocks;
        const int b0 = (int)(cursor / kReplayBlock);
        const int b1 = (int)(((cursor + K - 1) % M) / kReplayBlock);
        const int nt = (b1 - b0 + nblk) % nblk + 1;              // touched blocks b0, b0+1, ... (circular)
        const int c0 = b0 / kChunkBlocks, c1 = b1 / kChunkBlocks;
        const int nc = (c1 - c0 + nchunk) % nchunk + 1;          // touched chunks c0, c0+1, ...
        const int s0 = b0 / kSuperBlocks, s1 = b1 / kSuperBlocks;
        const int ns = (s1 - s0 + nsuper) % nsuper + 1;          // touched super-blocks s0, s0+1, ...
        const uint32_t* gate = &w.ist->rebuild;
        hipLaunchKernelGGL(k_insert_patch, dim3((unsigned)(4 * nc)), dim3(256), 0, st, weights, M, nblk, nchunk, cursor,
                           prio, K, alpha, slots_out, c0, w.hdr, w.quarter_max, w.touched_sum, w.sub_sum);
        hipLaunchKernelGGL(k_patch_supers, dim3((unsigned)ns), dim3(1024), 0, st, M, nblk, b0, nt, c0, nc, nchunk, s0,
                           nsuper, w.hdr, w.ist, w.partial_max, w.chunk_max, w.quarter_max, w.touched_sum,
                           w.block_cum, w.super_new, w.coarse_cum);
        hipLaunchKernelGGL((k_super_sums<true>), dim3(round_up_8((unsigned)nsuper)), dim3(1024), 0, st, weights, M, w.hdr,
                           w.partial_max, w.chunk_max, w.block_cum, nblk, w.super_new, w.sub_sum, w.coarse_cum, gate);
        hipLaunchKernelGGL((k_super_sums<false>), dim3(round_up_8((unsigned)nsuper)), dim3(1024), 0, st, weights, M, w.hdr,
                           w.partial_max, w.chunk_max, w.block_cum, nblk, w.super_new, w.sub_sum, w.coarse_cum, gate);
        hipLaunchKernelGGL(k_patch_finish, dim3(1), dim3(256), 0, st, w.super_cum, w.super_new, nsuper, s0, ns,
                           w.partial_max, w.hdr, w.ist, M);
        return hipGetLastError();
    }
    if (K > 0)
        hipLaunchKernelGGL(k_insert, dim3((unsigned)((K + 255) / 256)), dim3(256), 0, st, weights, M, cursor, prio,
                           K, alpha, slots_out);
    return update_launch(weights, M, nullptr, nullptr, 0, alpha, w, st);
}

hipError_t sample_launch(const float* weights, long long M, const ReplayWs& w, const double* uniforms, int K,
                         long long* idx_out, float* prob_out, hipStream_t st) {
    const int nblk = (int)((M + kReplayBlock - 1) / kReplayBlock);
    const long long waves = ((long long)K + 4 * kDrawsPerGroup - 1) / (4 * kDrawsPerGroup);   // four groups per wave
    const unsigned g = (unsigned)((waves * kWave + 255) / 256);
    hipLaunchKernelGGL(k_sample, dim3(g), dim3(256), 0, st, weights, M, w.hdr, w.block_cum, nblk, w.super_cum,
                       w.sub_sum, w.coarse_cum, uniforms, K, idx_out, prob_out, &w.hdr->flags);
    return hipGetLastError();
}

}  // namespace aride
