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

// ---- ingest probe: one workgroup per compute unit reads a private region `passes` times, U 1 KB wave-loads per
// wave in a batch with the previous batch still in flight.  To registers (16 bytes per lane) or straight into LDS
// (the GEMM's and the prefill kernel's tile loader); ordinary or nontemporal.
template <int U, bool NT>
__global__ void probe_ingest_vgpr_kernel(const probe_v4u* __restrict__ base, size_t region_v4, int passes, unsigned* __restrict__ sink)
{
    const probe_v4u* p = base + (size_t)blockIdx.x * region_v4;
    probe_v4u acc = {0, 0, 0, 0};
    const int stride = blockDim.x;
    const int steps = (int)(region_v4 / ((size_t)stride * U));
    for (int it = 0; it < passes; ++it)
        for (int s = 0; s < steps; ++s) {
            probe_v4u v[U];
#pragma unroll
            for (int u = 0; u < U; ++u) {
                const probe_v4u* q = p + (size_t)(s * U + u) * stride + threadIdx.x;
                v[u] = NT ? __builtin_nontemporal_load(q) : *q;
            }
#pragma unroll
            for (int u = 0; u < U; ++u) acc ^= v[u];
        }
    if ((acc.x ^ acc.y ^ acc.z ^ acc.w) == 0x12345u) sink[0] = acc.x;
}

// row_bytes = 0: the region is read front to back, 1 KB per wave-load.  row_bytes > 0: the region is a panel of 128
// rows of row_bytes bytes and a wave-load takes 128 bytes of 8 rows, the panel being walked 128 bytes at a time (what
// the loader of a 128-row operand tile of a row-major matrix does); the workgroup's waves x U must cover the 16
// wave-loads of a step.
template <int U, bool NT>
__global__ void probe_ingest_lds_kernel(const char* __restrict__ base, size_t region_bytes, int passes, int row_bytes,
                                        unsigned* __restrict__ sink)
{
    extern __shared__ __align__(16) unsigned char probe_smem[];      // waves * U KB
    const char* p = base + (size_t)blockIdx.x * region_bytes;
    const int lane = threadIdx.x & 63, nw = blockDim.x >> 6;
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const unsigned lds0 = (unsigned)(size_t)(__attribute__((address_space(3))) unsigned char*)probe_smem + wave * U * 1024;
    unsigned voff[U];
    size_t step_bytes;
    int steps;
    if (row_bytes == 0) {
#pragma unroll
        for (int u = 0; u < U; ++u) voff[u] = (unsigned)((wave * U + u) * 1024 + lane * 16);
        step_bytes = (size_t)nw * U * 1024;
        steps = (int)(region_bytes / step_bytes);
    } else {
#pragma unroll
        for (int u = 0; u < U; ++u) voff[u] = (unsigned)(((u * nw + wave) * 8 + (lane >> 3)) * row_bytes + ((lane & 7) << 4));
        step_bytes = 128;
        steps = row_bytes / 128;
    }
#pragma clang diagnostic push
#pragma clang diagnostic ignored "-Winline-asm"
    for (int it = 0; it < passes; ++it)
        for (int s = 0; s < steps; ++s) {
            const char* src = p + (size_t)s * step_bytes;
#pragma unroll
            for (int u = 0; u < U; ++u) {
                unsigned dst = lds0 + u * 1024;
                if (NT) asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %1, %2 nt" ::"s"(dst), "v"(voff[u]), "s"(src) : "memory", "m0");
                else asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %1, %2" ::"s"(dst), "v"(voff[u]), "s"(src) : "memory", "m0");
            }
            asm volatile("s_waitcnt vmcnt(%0)" ::"n"(U) : "memory");       // the batch before this one has landed
        }
    asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
#pragma clang diagnostic pop
    if (probe_smem[threadIdx.x] == 0x5a && sink[1] == 77u) sink[0] = 1;
}

template <int U>
static hipError_t launch_ingest(int mode, int grid, int waves, const char* buf, size_t region, int passes, int row_bytes,
                                unsigned* sink, hipStream_t s)
{
    int threads = waves * 64;
    if (mode == 0) probe_ingest_vgpr_kernel<U, false><<<grid, threads, 0, s>>>((const probe_v4u*)buf, region / 16, passes, sink);
    else if (mode == 1) probe_ingest_vgpr_kernel<U, true><<<grid, threads, 0, s>>>((const probe_v4u*)buf, region / 16, passes, sink);
    else if (mode == 2) probe_ingest_lds_kernel<U, false><<<grid, threads, (size_t)waves * U * 1024, s>>>(buf, region, passes, row_bytes, sink);
    else probe_ingest_lds_kernel<U, true><<<grid, threads, (size_t)waves * U * 1024, s>>>(buf, region, passes, row_bytes, sink);
    return hipGetLastError();
}

}  // namespace exe

extern "C" int exe_probe_ingest(void* hip_stream, int32_t mode, uint64_t region_bytes, int32_t passes, int32_t waves,
                                int32_t loads_per_batch, int32_t row_bytes, double* bytes_per_s)
{
    using namespace exe;
    hipStream_t s = (hipStream_t)hip_stream;
    if (!bytes_per_s || mode < 0 || mode > 3 || passes < 1) return set_error(EXE_ERR_ARG, "bad mode, passes or null result");
    if (!(waves == 1 || waves == 2 || waves == 4 || waves == 8 || waves == 16) ||
        !(loads_per_batch == 2 || loads_per_batch == 4 || loads_per_batch == 8 || loads_per_batch == 16))
        return set_error(EXE_ERR_ARG, "waves must be 1, 2, 4, 8 or 16 and loads_per_batch 2, 4, 8 or 16");
    if (waves * loads_per_batch > 64) return set_error(EXE_ERR_ARG, "waves x loads_per_batch above 64 (64 KB of LDS)");
    if (row_bytes != 0) {
        if (mode < 2 || row_bytes < 128 || row_bytes % 128 != 0 || row_bytes > (1 << 20) || waves * loads_per_batch != 16)
            return set_error(EXE_ERR_ARG, "row_bytes needs an LDS mode, a multiple of 128 and waves x loads_per_batch = 16");
        region_bytes = (uint64_t)128 * row_bytes;
    }
    uint64_t batch = (uint64_t)waves * loads_per_batch * 1024;
    if (region_bytes < batch || region_bytes % batch != 0) return set_error(EXE_ERR_ARG, "region_bytes must be a multiple of waves x loads_per_batch KB");
    int dev = 0, cus = 0;
    if (hipGetDevice(&dev) != hipSuccess || hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess || cus < 1)
        return set_error(EXE_ERR_HIP, "cannot query the device");
    if (region_bytes * (uint64_t)cus > ((uint64_t)16 << 30)) return set_error(EXE_ERR_ARG, "region_bytes x compute units above 16 GiB");
    hipEvent_t e0 = nullptr, e1 = nullptr;
    char* buf = nullptr;
    unsigned* sink = nullptr;
    auto done = [&](int code, const char* msg) {
        if (e0) (void)hipEventDestroy(e0);
        if (e1) (void)hipEventDestroy(e1);
        if (buf) (void)hipFree(buf);
        if (sink) (void)hipFree(sink);
        return code == EXE_OK ? EXE_OK : set_error(code, msg);
    };
    size_t total = (size_t)region_bytes * cus;
    if (hipEventCreate(&e0) != hipSuccess || hipEventCreate(&e1) != hipSuccess || hipMalloc((void**)&sink, 256) != hipSuccess ||
        hipMalloc((void**)&buf, total) != hipSuccess)
        return done(EXE_ERR_HIP, "probe set-up failed");
    if (hipMemsetAsync(buf, 1, total, s) != hipSuccess || hipMemsetAsync(sink, 0, 256, s) != hipSuccess) return done(EXE_ERR_HIP, "probe memset failed");
    auto launch = [&]() {
        switch (loads_per_batch) {
            case 2: return launch_ingest<2>(mode, cus, waves, buf, (size_t)region_bytes, passes, row_bytes, sink, s);
            case 4: return launch_ingest<4>(mode, cus, waves, buf, (size_t)region_bytes, passes, row_bytes, sink, s);
            case 8: return launch_ingest<8>(mode, cus, waves, buf, (size_t)region_bytes, passes, row_bytes, sink, s);
            default: return launch_ingest<16>(mode, cus, waves, buf, (size_t)region_bytes, passes, row_bytes, sink, s);
        }
    };
    if (launch() != hipSuccess) return done(EXE_ERR_HIP, "ingest probe launch failed");
    (void)hipEventRecord(e0, s);
    if (launch() != hipSuccess) return done(EXE_ERR_HIP, "ingest probe launch failed");
    (void)hipEventRecord(e1, s);
    float ms = 0.f;
    if (hipEventSynchronize(e1) != hipSuccess || hipEventElapsedTime(&ms, e0, e1) != hipSuccess || ms <= 0.f)
        return done(EXE_ERR_HIP, "ingest probe failed");
    *bytes_per_s = (double)total * passes / (ms * 1e-3);
    return done(EXE_OK, "");
}

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
