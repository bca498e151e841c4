// Measured ceilings of the machine the library runs on, for the roofline figures a benchmark prints next to the
// nominal peaks: (a) the rate of a plain streaming read of a large buffer (every workgroup reads a private 256 KiB
// region, 16 bytes per lane, four loads in flight per lane, nontemporal), (b) the rate of back-to-back independent bf16 16x16x32 MFMAs, two waves
// per SIMD, at the clock that load sustains.  Neither touches the model.
#include <algorithm>

#include "../../include/exe.h"
#include "common.h"

namespace exe {
int set_error(int code, const char* msg);

typedef unsigned probe_v4u __attribute__((ext_vector_type(4)));

// every workgroup streams a private contiguous region of region_v4 16-byte elements (a multiple of 256 * 4)
__global__ __launch_bounds__(256) void probe_read_kernel(const probe_v4u* __restrict__ src, size_t region_v4, unsigned* __restrict__ sink)
{
    constexpr int U = 4;
    const probe_v4u* p = src + (size_t)blockIdx.x * region_v4;
    probe_v4u acc = {0, 0, 0, 0};
    for (size_t i = threadIdx.x; i < region_v4; i += (size_t)256 * U) {
        probe_v4u v[U];
#pragma unroll
        for (int u = 0; u < U; ++u) v[u] = __builtin_nontemporal_load(p + i + u * 256);
#pragma unroll
        for (int u = 0; u < U; ++u) acc ^= v[u];
    }
    if ((acc.x ^ acc.y ^ acc.z ^ acc.w) == 0x12345u) sink[0] = acc.x;      // keeps the loads alive
}

__global__ __launch_bounds__(512) void probe_mfma_kernel(int iters, float* __restrict__ sink)
{
    int lane = threadIdx.x & 63;
    bf16x8 a, b;
#pragma unroll
    for (int i = 0; i < 8; ++i) {
        a[i] = (bf16_t)(0.001f * (lane + i));
        b[i] = (bf16_t)(0.002f * (lane - i));
    }
    f32x4 acc[8];
#pragma unroll
    for (int j = 0; j < 8; ++j) acc[j] = f32x4{0.f, 0.f, 0.f, 0.f};
    for (int it = 0; it < iters; ++it) {
#pragma unroll
        for (int j = 0; j < 16; ++j) acc[j & 7] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(a, b, acc[j & 7], 0, 0, 0);
    }
    float s = 0.f;
#pragma unroll
    for (int j = 0; j < 8; ++j) s += acc[j][0] + acc[j][1] + acc[j][2] + acc[j][3];
    if (s == 12345.678f) sink[0] = s;
}

}  // namespace exe

extern "C" int exe_probe_peaks(void* hip_stream, uint64_t read_bytes, double* hbm_read_bytes_per_s, double* mfma_bf16_flops_per_s)
{
    using namespace exe;
    hipStream_t s = (hipStream_t)hip_stream;
    if (!hbm_read_bytes_per_s && !mfma_bf16_flops_per_s) return set_error(EXE_ERR_ARG, "nothing to measure");
    int dev = 0, cus = 0;
    if (hipGetDevice(&dev) != hipSuccess || hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess || cus < 1)
        return set_error(EXE_ERR_HIP, "cannot query the device");
    hipEvent_t e0 = nullptr, e1 = nullptr;
    void* buf = nullptr;
    unsigned* sink = nullptr;
    int rc = EXE_OK;
    auto done = [&](int code, const char* msg) {
        if (e0) (void)hipEventDestroy(e0);
        if (e1) (void)hipEventDestroy(e1);
        if (buf) (void)hipFree(buf);
        if (sink) (void)hipFree(sink);
        return code == EXE_OK ? EXE_OK : set_error(code, msg);
    };
    if (hipEventCreate(&e0) != hipSuccess || hipEventCreate(&e1) != hipSuccess || hipMalloc((void**)&sink, 256) != hipSuccess)
        return done(EXE_ERR_HIP, "probe set-up failed");
    if (hbm_read_bytes_per_s) {
        if (read_bytes < ((uint64_t)64 << 20)) read_bytes = (uint64_t)4 << 30;
        const size_t region_v4 = ((size_t)256 << 10) / 16;      // 256 KiB per workgroup
        const int grid = (int)std::min<uint64_t>(read_bytes / ((uint64_t)256 << 10), 1u << 20);
        size_t n = (size_t)grid * region_v4;
        if (n == 0 || hipMalloc(&buf, n * 16) != hipSuccess) return done(EXE_ERR_HIP, "probe buffer allocation failed");
        if (hipMemsetAsync(buf, 1, n * 16, s) != hipSuccess) return done(EXE_ERR_HIP, "probe memset failed");
        const int reps = 10;
        for (int i = 0; i < 3; ++i) probe_read_kernel<<<grid, 256, 0, s>>>((const probe_v4u*)buf, region_v4, sink);
        (void)hipEventRecord(e0, s);
        for (int i = 0; i < reps; ++i) probe_read_kernel<<<grid, 256, 0, s>>>((const probe_v4u*)buf, region_v4, sink);
        (void)hipEventRecord(e1, s);
        float ms = 0.f;
        if (hipEventSynchronize(e1) != hipSuccess || hipEventElapsedTime(&ms, e0, e1) != hipSuccess || ms <= 0.f)
            return done(EXE_ERR_HIP, "read probe failed");
        *hbm_read_bytes_per_s = (double)n * 16.0 * reps / (ms * 1e-3);
    }
    if (mfma_bf16_flops_per_s) {
        const int grid = cus * 2, block = 512, iters = 200000, reps = 3;      // about 70 ms: long enough for the clock to settle
        probe_mfma_kernel<<<grid, block, 0, s>>>(iters, (float*)sink);
        (void)hipEventRecord(e0, s);
        for (int i = 0; i < reps; ++i) probe_mfma_kernel<<<grid, block, 0, s>>>(iters, (float*)sink);
        (void)hipEventRecord(e1, s);
        float ms = 0.f;
        if (hipEventSynchronize(e1) != hipSuccess || hipEventElapsedTime(&ms, e0, e1) != hipSuccess || ms <= 0.f)
            return done(EXE_ERR_HIP, "MFMA probe failed");
        double flops = (double)grid * (block / 64) * (double)iters * 16.0 * (2.0 * 16 * 16 * 32) * reps;
        *mfma_bf16_flops_per_s = flops / (ms * 1e-3);
    }
    return done(rc, "");
}
