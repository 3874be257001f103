// Calibration aid for hardware-counter readings: a plain device-to-device copy whose HBM
// traffic is known exactly (bytes read = bytes written = n).  Built into its own small
// library (libaride_probe.so); it is not part of the scoring library or of its C ABI.
#include <hip/hip_runtime.h>
#include <stdint.h>

typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));

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

// Read-only companion: streams nbytes with non-temporal 16-byte loads and XORs them into one
// word per workgroup (so the loads cannot be dropped).  Measures the read bandwidth a kernel
// with no arithmetic to speak of reaches on this part.
__global__ __launch_bounds__(256) void k_read_probe(const u32x4* __restrict__ src, size_t nvec, uint32_t* __restrict__ sink) {
    uint32_t acc = 0;
    const size_t stride = (size_t)gridDim.x * blockDim.x;
    size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
    for (; i + 3 * stride < nvec; i += 4 * stride) {
        u32x4 a = __builtin_nontemporal_load(src + i), b = __builtin_nontemporal_load(src + i + stride);
        u32x4 c = __builtin_nontemporal_load(src + i + 2 * stride), d = __builtin_nontemporal_load(src + i + 3 * stride);
        acc ^= a.x ^ a.y ^ a.z ^ a.w ^ b.x ^ b.y ^ b.z ^ b.w ^ c.x ^ c.y ^ c.z ^ c.w ^ d.x ^ d.y ^ d.z ^ d.w;
    }
    for (; i < nvec; i += stride) { u32x4 a = __builtin_nontemporal_load(src + i); acc ^= a.x ^ a.y ^ a.z ^ a.w; }
    if (acc == 0x9e3779b9u) sink[blockIdx.x & 255] = acc;   // practically never taken
}

extern "C" int aride_probe_read(const void* src, size_t nbytes, void* sink256, int blocks, void* stream) {
    if (!src || !sink256 || (nbytes & 15) || ((uintptr_t)src & 15) || blocks <= 0) return -1;
    hipLaunchKernelGGL(k_read_probe, dim3((unsigned)blocks), dim3(256), 0, (hipStream_t)stream,
                       (const u32x4*)src, nbytes / 16, (uint32_t*)sink256);
    return hipGetLastError() == hipSuccess ? 0 : -7;
}
