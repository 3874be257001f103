// Device-side helpers shared by the HIP kernels of the A-RIDE scoring library (gfx950).
// Wave size is 64 throughout.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace aride {

constexpr int kWave = 64;

// Workspace layout (device memory, 256-byte aligned):
//   [0, 256)                  header: the first 24 bytes mirror the public status struct
//   [256, 256 + 8*nblk)       inclusive prefix of the per-block integer sums (replay index)
struct WsHeader {
    uint32_t flags;      // OR of status bits
    uint32_t reserved;
    unsigned long long total;  // integer mass of the replay CDF
    uint32_t wmax_bits;  // bit pattern of the largest valid weight (non-negative float)
    int32_t exponent;    // e = ilogb(wmax) + 1
};
constexpr size_t kHeaderBytes = 256;
constexpr int kReplayBlock = 256;  // weights per indexed block: one wave reads one as 64 x float4

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
