// Measurement probes, built into their own small library (libseedprobe.so) and used by bench.py only:
// what this GPU actually sustains on the two rooflines the step is priced against.
//   seed_probe_mfma_bf16  a loop of nothing but v_mfma_f32_16x16x32_bf16 on register operands: the matrix
//                         pipe's rate at the clock the chip holds under that load
//   seed_probe_copy       a streaming copy of `bytes` bytes (read + write through HBM): four 16-byte loads in
//                         flight per lane before the first store, non-temporal accesses, one pass per workgroup
//                         with the grid capped at 256 workgroups per compute unit (measured best of 1/4/8 loads
//                         per lane x temporal / non-temporal x 4..256 workgroups per unit: 6.2-6.4 TB/s against
//                         4.6-5.7 TB/s for one load per lane and 5.0 TB/s for the runtime's own device copy)
// Both enqueue on the given stream and return the HIP error code; the caller times them with events.
#include <hip/hip_runtime.h>

#include <cstddef>
#include <cstdint>

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef float floatx4 __attribute__((ext_vector_type(4)));

namespace {

constexpr int PROBE_THREADS = 512;       // 8 wavefronts: two per SIMD
constexpr int PROBE_UNROLL = 64;         // MFMAs per loop iteration, over four independent accumulators

__global__ __launch_bounds__(PROBE_THREADS) void mfma_loop_kernel(float* sink, int iters)
{
    const int lane = threadIdx.x & 63;
    bf16x8 a, b;
#pragma unroll
    for (int e = 0; e < 8; ++e) {
        a[e] = (__bf16)(float)((lane + e) & 7);
        b[e] = (__bf16)(float)((lane * 3 + e) & 3);
    }
    floatx4 acc[4];
#pragma unroll
    for (int i = 0; i < 4; ++i) acc[i] = floatx4{0.f, 0.f, 0.f, 0.f};
    for (int it = 0; it < iters; ++it) {
#pragma unroll
        for (int i = 0; i < PROBE_UNROLL; ++i) acc[i & 3] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(a, b, acc[i & 3], 0, 0, 0);
    }
    const floatx4 s = acc[0] + acc[1] + acc[2] + acc[3];
    if (s[0] + s[1] + s[2] + s[3] == -1.0f) sink[blockIdx.x] = s[0];    // never true: the sums are non-negative
}

typedef unsigned int u32x4 __attribute__((ext_vector_type(4)));
constexpr int COPY_UNROLL = 4;

__global__ __launch_bounds__(256) void copy_kernel(const u32x4* __restrict__ src, u32x4* __restrict__ dst, size_t n)
{
    const size_t stride = (size_t)gridDim.x * 256 * COPY_UNROLL;
    for (size_t base = (size_t)blockIdx.x * 256 * COPY_UNROLL + threadIdx.x; base < n; base += stride) {
        u32x4 v[COPY_UNROLL];
#pragma unroll
        for (int u = 0; u < COPY_UNROLL; ++u) {
            const size_t i = base + (size_t)u * 256;
            if (i < n) v[u] = __builtin_nontemporal_load(src + i);
        }
#pragma unroll
        for (int u = 0; u < COPY_UNROLL; ++u) {
            const size_t i = base + (size_t)u * 256;
            if (i < n) __builtin_nontemporal_store(v[u], dst + i);
        }
    }
}

}  // namespace

extern "C" int seed_probe_mfma_bf16(int blocks, int iters, float* sink_dev, void* hip_stream)
{
    if (blocks <= 0 || iters <= 0 || !sink_dev) return (int)hipErrorInvalidValue;
    hipLaunchKernelGGL(mfma_loop_kernel, dim3(blocks), dim3(PROBE_THREADS), 0, (hipStream_t)hip_stream, sink_dev, iters);
    return (int)hipGetLastError();
}

// floating-point operations one seed_probe_mfma_bf16 launch performs
extern "C" double seed_probe_mfma_flops(int blocks, int iters)
{
    return (double)blocks * (PROBE_THREADS / 64) * (double)iters * PROBE_UNROLL * (2.0 * 16 * 16 * 32);
}

extern "C" int seed_probe_copy(const void* src_dev, void* dst_dev, size_t bytes, void* hip_stream)
{
    if (!src_dev || !dst_dev || bytes % 16 != 0) return (int)hipErrorInvalidValue;
    const size_t n = bytes / 16;
    if (n == 0) return 0;
    int dev = 0, n_cu = 256;
    if (hipGetDevice(&dev) == hipSuccess) {
        int v = 0;
        if (hipDeviceGetAttribute(&v, hipDeviceAttributeMultiprocessorCount, dev) == hipSuccess && v > 0) n_cu = v;
    }
    const size_t want = (n + 256 * COPY_UNROLL - 1) / (256 * COPY_UNROLL), cap = (size_t)n_cu * 256;
    hipLaunchKernelGGL(copy_kernel, dim3((unsigned)(want < cap ? want : cap)), dim3(256), 0, (hipStream_t)hip_stream,
                       (const u32x4*)src_dev, (u32x4*)dst_dev, n);
    return (int)hipGetLastError();
}
