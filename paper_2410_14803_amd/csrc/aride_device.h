// Device-side helpers shared by the HIP kernels of the A-RIDE scoring library (gfx950).
// Wave size is 64 throughout.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace aride {

constexpr int kWave = 64;

// Workspace layout (device memory, 256-byte aligned):
//   [0, 256)                  header: the first 24 bytes mirror the public status struct
//   [256, 256 + 2048)         super_cum: inclusive prefix of the super-block totals (256 x u64)
//   [2304, 2304 + 4096)       partial_max: per-workgroup maxima of the last rebuild (1024 x u32)
//   [6400, 6400 + 8*nblk)     block_cum: per super-block, inclusive prefix of its block sums
struct WsHeader {
    uint32_t flags;      // OR of status bits
    uint32_t reserved;
    unsigned long long total;  // integer mass of the replay CDF
    uint32_t wmax_bits;  // bit pattern of the largest valid weight (non-negative float)
    int32_t exponent;    // e = ilogb(wmax) + 1
};
constexpr size_t kHeaderBytes = 256;
constexpr int kReplayBlock = 256;  // weights per indexed block: one wave reads one as 64 x float4
constexpr int kSuperBlocks = 256;  // blocks per super-block (65536 weights); at most 256 super-blocks
constexpr size_t kSuperBytes = kSuperBlocks * 8;
constexpr int kMaxParts = 1024;    // workgroups of the maximum pass, one partial maximum each
constexpr size_t kPartBytes = kMaxParts * 4;

__device__ __forceinline__ float bits_to_float(uint32_t b) { return __uint_as_float(b); }
__device__ __forceinline__ uint32_t float_to_bits(float f) { return __float_as_uint(f); }

__device__ __forceinline__ float fast_exp2(float x) { return __builtin_amdgcn_exp2f(x); }

__device__ __forceinline__ float wave_max(float v) {
#pragma unroll
    for (int d = 32; d >= 1; d >>= 1) v = fmaxf(v, __shfl_xor(v, d, kWave));
    return v;
}
__device__ __forceinline__ float wave_sum(float v) {
#pragma unroll
    for (int d = 32; d >= 1; d >>= 1) v += __shfl_xor(v, d, kWave);
    return v;
}
__device__ __forceinline__ unsigned long long wave_sum_u64(unsigned long long v) {
#pragma unroll
    for (int d = 32; d >= 1; d >>= 1) v += __shfl_xor(v, d, kWave);
    return v;
}

}  // namespace aride
