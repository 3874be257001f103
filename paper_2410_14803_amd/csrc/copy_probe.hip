// Calibration aids for the measurements: kernels whose HBM traffic is known exactly and that do
// nothing else.  Built into their own small library (libaride_probe.so); they are not part of the
// scoring library or of its C ABI.
#include <hip/hip_runtime.h>
#include <stdint.h>

typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
typedef float f32x4 __attribute__((ext_vector_type(4)));

// A plain device-to-device copy (bytes read = bytes written = n): what a hardware counter reads
// for it gives the factor by which that counter's readings are scaled.
__global__ __launch_bounds__(256) void k_copy_probe(const u32x4* __restrict__ src, u32x4* __restrict__ dst, size_t nvec) {
    for (size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x; i < nvec; i += (size_t)gridDim.x * blockDim.x)
        dst[i] = src[i];
}

// Copies nbytes (a multiple of 16; both pointers 16-byte aligned) on `stream`. Returns 0 on success.
extern "C" int aride_probe_copy(void* dst, const void* src, size_t nbytes, void* stream) {
    if (!dst || !src || (nbytes & 15) || ((uintptr_t)dst & 15) || ((uintptr_t)src & 15)) return -1;
    const size_t nvec = nbytes / 16;
    size_t blocks = (nvec + 255) / 256;
    if (blocks > 256 * 32) blocks = 256 * 32;
    if (blocks == 0) return 0;
    hipLaunchKernelGGL(k_copy_probe, dim3((unsigned)blocks), dim3(256), 0, (hipStream_t)stream,
                       (const u32x4*)src, (u32x4*)dst, nvec);
    return hipGetLastError() == hipSuccess ? 0 : -7;
}

// The access pattern of the Retrace + priority scan with the scan taken out: NIN fp32 arrays
// read and NOUT written, 16 bytes per lane and array, one pass, a trivial combination in between.
// What this reaches is what the memory system allows that mix of read and write streams:
//   SPANS = false  a workgroup per 4 KB of each array, in the order the workgroups are dispatched:
//                  at any time the chip works on one compact window of every array;
//   SPANS = true   the scan's own shape: about 3000 waves, each walking its own contiguous span
//                  of every array from the end to the start, 1 KB per array at a time;
//   NTL            non-temporal loads (stores are non-temporal throughout, as in the scan).
template <int NIN, int NOUT, bool SPANS, bool NTL>
__global__ __launch_bounds__(256) void k_mix_probe(const f32x4* const* __restrict__ in, f32x4* const* __restrict__ out,
                                                   size_t nvec, size_t span) {
    // the grid is a multiple of 8; XCD x takes the x-th eighth
    const size_t blk = (size_t)(blockIdx.x & 7) * (gridDim.x >> 3) + (blockIdx.x >> 3);
    size_t first, last;                      // 16-byte units [first, last) in steps of 64 per wave
    if (SPANS) {
        const size_t wave = blk * 4 + (threadIdx.x >> 6);
        first = wave * span * 64; last = first + span * 64;
    } else {
        first = blk * 256 + (threadIdx.x & ~(size_t)63); last = first + 64;
    }
    if (last > nvec) last = nvec;
    for (size_t c = last; c > first;) {
        c = c >= first + 64 ? c - 64 : first;
        const size_t i = c + (threadIdx.x & 63);
        if (i >= last) continue;
        f32x4 acc = {1.f, 2.f, 3.f, 4.f};
        if constexpr (NIN > 0) {
            f32x4 v[NIN];
#pragma unroll
            for (int k = 0; k < NIN; ++k) v[k] = NTL ? __builtin_nontemporal_load(in[k] + i) : in[k][i];
            acc = v[0];
#pragma unroll
            for (int k = 1; k < NIN; ++k) acc = acc * 0.5f + v[k];
        }
        if constexpr (NOUT == 0) {
            if (acc.x == 1.2345678f) __builtin_nontemporal_store(acc, out[0] + i);    // keeps the loads alive
        }
#pragma unroll
        for (int k = 0; k < NOUT; ++k) __builtin_nontemporal_store(acc + (float)k, out[k] + i);
    }
}

template <int NIN, int NOUT>
static void mix_launch(const f32x4* const* ins, f32x4* const* outs, size_t nvec, int pattern, hipStream_t st) {
    const bool spans = pattern & 2, ntl = pattern & 1;
    size_t span = 0, blocks;
    if (spans) {
        const size_t chunks = (nvec + 63) / 64;
        span = (chunks + 3071) / 3072;
        blocks = ((chunks + span - 1) / span + 3) / 4;
    } else {
        blocks = (nvec + 255) / 256;
    }
    const dim3 grid((unsigned)((blocks + 7) / 8 * 8)), block(256);
    if (spans && ntl) hipLaunchKernelGGL((k_mix_probe<NIN, NOUT, true, true>), grid, block, 0, st, ins, outs, nvec, span);
    else if (spans) hipLaunchKernelGGL((k_mix_probe<NIN, NOUT, true, false>), grid, block, 0, st, ins, outs, nvec, span);
    else if (ntl) hipLaunchKernelGGL((k_mix_probe<NIN, NOUT, false, true>), grid, block, 0, st, ins, outs, nvec, span);
    else hipLaunchKernelGGL((k_mix_probe<NIN, NOUT, false, false>), grid, block, 0, st, ins, outs, nvec, span);
}

// in / out: DEVICE arrays of 6 and 4 device pointers to fp32 arrays of n elements each (n a
// multiple of 4, every array 16-byte aligned; out[0] must be valid even when nout is 0);
// (nin, nout) in {(6,4), (5,3), (3,1), (6,0), (0,4)}; pattern: bit 0 = non-temporal loads,
// bit 1 = a contiguous span per wave instead of a workgroup per 4 KB.
extern "C" int aride_probe_mix(const void* in, void* out, int nin, int nout, size_t n, int pattern, void* stream) {
    if (!in || !out || (n & 3) || pattern < 0 || pattern > 3 || n > ((size_t)1 << 33)) return -1;   // a work-item per 16 bytes, at most 2^31 a launch
    const size_t nvec = n / 4;
    if (nvec == 0) return 0;
    auto ins = (const f32x4* const*)in;
    auto outs = (f32x4* const*)out;
    auto st = (hipStream_t)stream;
    if (nin == 6 && nout == 4) mix_launch<6, 4>(ins, outs, nvec, pattern, st);
    else if (nin == 5 && nout == 3) mix_launch<5, 3>(ins, outs, nvec, pattern, st);
    else if (nin == 3 && nout == 1) mix_launch<3, 1>(ins, outs, nvec, pattern, st);
    else if (nin == 6 && nout == 0) mix_launch<6, 0>(ins, outs, nvec, pattern, st);
    else if (nin == 0 && nout == 4) mix_launch<0, 4>(ins, outs, nvec, pattern, st);
    else return -1;
    return hipGetLastError() == hipSuccess ? 0 : -7;
}

// The shader clock right now: cycles of the shader clock (clock64) per tick of the constant 100 MHz
// counter (wall_clock64) over a spin of `wall_ticks` ticks.  out[0] = cycles, out[1] = ticks.
// The spin ends after `wall_ticks` ticks or 2^22 polls, whichever comes first.
__global__ void k_clock_probe(unsigned long long* __restrict__ out, unsigned long long wall_ticks) {
    const unsigned long long c0 = clock64(), w0 = wall_clock64();
    unsigned long long w1 = w0;
    for (int polls = 0; polls < (1 << 22) && w1 - w0 < wall_ticks; ++polls) w1 = wall_clock64();
    const unsigned long long c1 = clock64();
    if (threadIdx.x == 0) { out[0] = c1 - c0; out[1] = w1 - w0; }
}

// out: device, two u64.  wall_ticks: length of the spin in 10 ns ticks (at most 100 000 = 1 ms).
extern "C" int aride_probe_clock(void* out, unsigned long long wall_ticks, void* stream) {
    if (!out || ((uintptr_t)out & 7) || wall_ticks == 0 || wall_ticks > 100000ull) return -1;
    hipLaunchKernelGGL(k_clock_probe, dim3(1), dim3(64), 0, (hipStream_t)stream, (unsigned long long*)out, wall_ticks);
    return hipGetLastError() == hipSuccess ? 0 : -7;
}
