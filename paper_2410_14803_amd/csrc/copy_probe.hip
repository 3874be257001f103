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
// What this reaches is the ceiling the memory system sets for that mix of read and write streams
// (a read-only sweep reaches 90 % of the HBM peak on this part, a mix of six read and four write
// streams about 70 %).  Loads are plain, stores non-temporal, as in the scan.
template <int NIN, int NOUT>
__global__ __launch_bounds__(256) void k_mix_probe(const f32x4* const* __restrict__ in, f32x4* const* __restrict__ out,
                                                   size_t nvec) {
    // the grid is a multiple of 8; XCD x takes the x-th eighth
    const size_t blk = (size_t)(blockIdx.x & 7) * (gridDim.x >> 3) + (blockIdx.x >> 3);
    const size_t i = blk * 256 + threadIdx.x;
    if (i >= nvec) return;
    f32x4 v[NIN];
#pragma unroll
    for (int k = 0; k < NIN; ++k) v[k] = in[k][i];
    f32x4 acc = v[0];
#pragma unroll
    for (int k = 1; k < NIN; ++k) acc = acc * 0.5f + v[k];
#pragma unroll
    for (int k = 0; k < NOUT; ++k) __builtin_nontemporal_store(acc + (float)k, out[k] + i);
}

// in / out: DEVICE arrays of 6 and 4 device pointers to fp32 arrays of n elements each (n a
// multiple of 4, every array 16-byte aligned); nin in {3, 5, 6}, nout in {1, 3, 4}.
extern "C" int aride_probe_mix(const void* in, void* out, int nin, int nout, size_t n, void* stream) {
    if (!in || !out || (n & 3)) return -1;
    const size_t nvec = n / 4;
    if (nvec == 0) return 0;
    const unsigned grid = (unsigned)(((nvec + 255) / 256 + 7) / 8 * 8);
    auto ins = (const f32x4* const*)in;
    auto outs = (f32x4* const*)out;
    if (nin == 6 && nout == 4) hipLaunchKernelGGL((k_mix_probe<6, 4>), dim3(grid), dim3(256), 0, (hipStream_t)stream, ins, outs, nvec);
    else if (nin == 5 && nout == 3) hipLaunchKernelGGL((k_mix_probe<5, 3>), dim3(grid), dim3(256), 0, (hipStream_t)stream, ins, outs, nvec);
    else if (nin == 3 && nout == 1) hipLaunchKernelGGL((k_mix_probe<3, 1>), dim3(grid), dim3(256), 0, (hipStream_t)stream, ins, outs, nvec);
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
