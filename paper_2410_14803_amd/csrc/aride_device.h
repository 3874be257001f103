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
//   then (256-byte aligned)   super_new: super-block totals handed from a patch pass to its last step (256 x u64)
//   then                      chunk_max: bit pattern of the largest valid weight of each chunk of 16
//                             blocks (4096 x u32); partial_max[g] covers the chunks 4g .. 4g+3
//   then                      quarter_max: maxima of the quarter chunks (4 blocks) an insert has just
//                             touched, handed from its first step to its second (16384 x u32)
//   then                      touched_sum: integer sums of the blocks of those chunks, by position (8448 x u64)
//   then                      coarse_cum: every 16th entry of block_cum (entries 15, 31, .. of each super-block's
//                             run), 16 per super-block, contiguous: the first probe of a draw (256 x 16 x u64)
//   then                      sub_sum: integer sum of every sub-block of 16 weights (16*nblk x u64), the
//                             third level of the index
struct WsHeader {
    uint32_t flags;      // OR of status bits
    uint32_t reserved;
    unsigned long long total;  // integer mass of the replay CDF
    uint32_t wmax_bits;  // bit pattern of the largest valid weight (non-negative float)
    int32_t exponent;    // e = ilogb(wmax) + 1
};
constexpr size_t kHeaderBytes = 256;

// Private state of the replay index, at byte kIndexStateOffset of the header block.
struct WsIndexState {
    long long index_M;   // capacity for which chunk_max, partial_max and the prefixes are current (0: none)
    uint32_t rebuild;    // set by a patch pass that found it cannot patch; read by the gated rebuild kernels
};
constexpr size_t kIndexStateOffset = 64;
constexpr int kReplayBlock = 256;  // weights per indexed block: one wave reads one as 64 x float4
constexpr int kSuperBlocks = 256;  // blocks per super-block (65536 weights); at most 256 super-blocks
constexpr size_t kSuperBytes = kSuperBlocks * 8;
constexpr int kMaxParts = 1024;    // workgroups of the maximum pass, one partial maximum each
constexpr size_t kPartBytes = kMaxParts * 4;
constexpr int kChunkBlocks = 16;   // blocks per chunk (4096 weights), the unit of the per-chunk maxima
constexpr int kMaxChunks = 4096;   // chunks of the largest buffer
constexpr size_t kChunkBytes = kMaxChunks * 4;
constexpr size_t kQuarterBytes = 4 * kChunkBytes;
constexpr int kMaxTouched = 8448;  // blocks of the chunks one patched insert may touch
constexpr size_t kTouchedBytes = kMaxTouched * 8;
constexpr int kSubBlock = 16;      // weights per sub-block: what the 16 lanes serving a draw quantise
constexpr int kSubsPerBlock = kReplayBlock / kSubBlock;
constexpr size_t kCoarseBytes = kSuperBlocks * 16 * 8;

// The arrays of the replay index inside a workspace sized for capacity M.
struct ReplayWs {
    WsHeader* hdr;
    WsIndexState* ist;
    unsigned long long* super_cum;
    uint32_t* partial_max;
    unsigned long long* block_cum;
    unsigned long long* super_new;
    uint32_t* chunk_max;
    uint32_t* quarter_max;
    unsigned long long* touched_sum;
    unsigned long long* sub_sum;
    unsigned long long* coarse_cum;
};
constexpr size_t round_up_256(size_t x) { return (x + 255) / 256 * 256; }
constexpr size_t replay_blocks(long long M) { return (size_t)((M + kReplayBlock - 1) / kReplayBlock); }
constexpr size_t replay_index_bytes(long long M) {
    if (M <= 0) return 0;
    const size_t nblk = replay_blocks(M);
    return kSuperBytes + kPartBytes + round_up_256(nblk * 8) + kSuperBytes + kChunkBytes + kQuarterBytes + kTouchedBytes + kCoarseBytes +
           round_up_256(nblk * kSubsPerBlock * 8);
}
inline ReplayWs replay_ws(void* ws, long long M) {
    char* p = static_cast<char*>(ws);
    const size_t nblk = replay_blocks(M);
    ReplayWs w;
    w.hdr = reinterpret_cast<WsHeader*>(p);
    w.ist = reinterpret_cast<WsIndexState*>(p + kIndexStateOffset);
    w.super_cum = reinterpret_cast<unsigned long long*>(p + kHeaderBytes);
    w.partial_max = reinterpret_cast<uint32_t*>(p + kHeaderBytes + kSuperBytes);
    w.block_cum = reinterpret_cast<unsigned long long*>(p + kHeaderBytes + kSuperBytes + kPartBytes);
    char* after = p + kHeaderBytes + kSuperBytes + kPartBytes + round_up_256(nblk * 8);
    w.super_new = reinterpret_cast<unsigned long long*>(after);
    w.chunk_max = reinterpret_cast<uint32_t*>(after + kSuperBytes);
    w.quarter_max = reinterpret_cast<uint32_t*>(after + kSuperBytes + kChunkBytes);
    w.touched_sum = reinterpret_cast<unsigned long long*>(after + kSuperBytes + kChunkBytes + kQuarterBytes);
    w.coarse_cum = reinterpret_cast<unsigned long long*>(after + kSuperBytes + kChunkBytes + kQuarterBytes + kTouchedBytes);
    w.sub_sum = reinterpret_cast<unsigned long long*>(after + kSuperBytes + kChunkBytes + kQuarterBytes + kTouchedBytes +
                                                      kCoarseBytes);
    return w;
}

__device__ __forceinline__ float bits_to_float(uint32_t b) { return __uint_as_float(b); }
__device__ __forceinline__ uint32_t float_to_bits(float f) { return __float_as_uint(f); }

__device__ __forceinline__ float fast_exp2(float x) { return __builtin_amdgcn_exp2f(x); }

// Workgroups are handed to the chip's 8 XCDs in turn (blockIdx mod 8).  For a grid that is a
// multiple of 8 this is the workgroup number under which XCD x works through the x-th eighth
// of the grid, so that each XCD -- its own L2, its own paths to memory -- streams one contiguous
// region of a tensor that the grid walks front to back.
__device__ __forceinline__ long long xcd_contiguous_block() {
    return (long long)(blockIdx.x & 7) * (gridDim.x >> 3) + (blockIdx.x >> 3);
}
inline unsigned round_up_8(unsigned blocks) { return (blocks + 7u) / 8u * 8u; }

// A dispatch counts its work-items per dimension in 32 bits (more wrap around without an error):
// a launch is given at most 2^31 of them, and work beyond that goes out as several launches.
constexpr long long kMaxLaunchThreads = 1ll << 31;

// Cross-lane moves inside a row of 16 lanes as DPP operands of ordinary vector instructions (no
// trip through the LDS crossbar, which is what __shfl costs).  CTRL: 0x120 | n rotates the row
// by n lanes, 0x110 | n shifts it right by n (lanes without a source read 0), 0x00..0xFF permute
// each quad of lanes.
template <int CTRL>
__device__ __forceinline__ float dpp_f32(float v) {
    return __int_as_float(__builtin_amdgcn_update_dpp(0, __float_as_int(v), CTRL, 0xF, 0xF, true));
}
// Wave-wide maximum / sum, left in every lane: rotations by 8, 4, 2, 1 inside each row of 16
// lanes (both operands of every step are the same pair in all lanes that share them, so all
// lanes end with the same bits), then the four rows are combined with two shuffles.
__device__ __forceinline__ float wave_max(float v) {
    v = fmaxf(v, dpp_f32<0x128>(v));
    v = fmaxf(v, dpp_f32<0x124>(v));
    v = fmaxf(v, dpp_f32<0x122>(v));
    v = fmaxf(v, dpp_f32<0x121>(v));
    v = fmaxf(v, __shfl_xor(v, 16, kWave));
    v = fmaxf(v, __shfl_xor(v, 32, kWave));
    return v;
}
// Sum over a row of 16 lanes, left in all of them.
__device__ __forceinline__ float row_sum_f32(float v) {
    v += dpp_f32<0x128>(v);
    v += dpp_f32<0x124>(v);
    v += dpp_f32<0x122>(v);
    v += dpp_f32<0x121>(v);
    return v;
}
__device__ __forceinline__ float wave_sum(float v) {
    v += dpp_f32<0x128>(v);
    v += dpp_f32<0x124>(v);
    v += dpp_f32<0x122>(v);
    v += dpp_f32<0x121>(v);
    v += __shfl_xor(v, 16, kWave);
    v += __shfl_xor(v, 32, kWave);
    return v;
}
__device__ __forceinline__ unsigned long long wave_sum_u64(unsigned long long v) {
#pragma unroll
    for (int d = 32; d >= 1; d >>= 1) v += __shfl_xor(v, d, kWave);
    return v;
}

// What compute_priorities needs when it rides along with the Retrace scan (k_flat_scan, PRIO).
struct PrioArgs {
    const float* ent;
    float w_td, w_rho, w_ent, inv_td_scale, inv_ent_scale, eps;
    int truncate;
    float* step_prio;
    float* traj_prio;
};

}  // namespace aride
