// Measured denominators for the roofline: what this machine delivers on the primitive streams
// the lmKAN kernels are made of (HBM copy and read, float32 multiply-adds on the vector and on
// the matrix pipe, LDS reads and writes, 256-byte row gathers from an L2-resident table).
// Not part of the paper's method; lmkan_microbench exists so that a benchmark can print these
// next to the published peaks in the same run.
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "lmkan.h"

namespace {

typedef float f4v __attribute__((ext_vector_type(4)));
constexpr int kThreads = 256;

__global__ __launch_bounds__(kThreads) void mb_copy_kernel(const f4v *__restrict__ src, f4v *__restrict__ dst, size_t n)
{
    const size_t stride = (size_t)gridDim.x * kThreads;
    for (size_t i = (size_t)blockIdx.x * kThreads + threadIdx.x; i < n; i += stride) dst[i] = src[i];
}

__global__ __launch_bounds__(kThreads) void mb_read_kernel(const f4v *__restrict__ src, float *__restrict__ sink, size_t n)
{
    const size_t stride = (size_t)gridDim.x * kThreads;
    f4v acc = {0.f, 0.f, 0.f, 0.f};
    for (size_t i = (size_t)blockIdx.x * kThreads + threadIdx.x; i < n; i += stride) acc += src[i];
    if (acc.x + acc.y + acc.z + acc.w == 1234.5f) sink[0] = acc.x;
}

// independent multiply-adds on 16 registers per lane
__global__ __launch_bounds__(kThreads) void mb_fma_kernel(float *sink, int iters, float seed)
{
    float v[16];
#pragma unroll
    for (int i = 0; i < 16; ++i) v[i] = seed + i + (threadIdx.x & 63);
    const float a = seed, b = seed * 0.5f;
    for (int it = 0; it < iters; ++it) {
#pragma unroll
        for (int i = 0; i < 16; ++i) asm volatile("v_fmac_f32_e32 %0, %1, %2" : "+v"(v[i]) : "v"(a), "v"(b));
    }
    float s = 0.f;
#pragma unroll
    for (int i = 0; i < 16; ++i) s += v[i];
    if (s == 1234.5f) sink[0] = s;
}

// independent 4x4x1 float32 MFMAs (16 blocks: 256 multiply-adds each) on 8 accumulators
__global__ __launch_bounds__(kThreads) void mb_mfma_kernel(float *sink, int iters, float seed)
{
    f4v acc[8];
#pragma unroll
    for (int i = 0; i < 8; ++i) acc[i] = f4v{seed, seed, seed, seed};
    const float a = seed + (threadIdx.x & 63), b = seed * 2.f;
    for (int it = 0; it < iters; ++it) {
#pragma unroll
        for (int i = 0; i < 8; ++i) acc[i] = __builtin_amdgcn_mfma_f32_4x4x1f32(a, b, acc[i], 0, 0, 0);
    }
    float s = 0.f;
#pragma unroll
    for (int i = 0; i < 8; ++i) s += acc[i].x + acc[i].y + acc[i].z + acc[i].w;
    if (s == 1234.5f) sink[0] = s;
}

// 16 bytes per lane, the 16 lanes of a row on one 256-byte LDS row (how the kernels read table rows)
template <bool WRITE>
__global__ __launch_bounds__(kThreads) void mb_lds_kernel(float *sink, int iters, float seed)
{
    __shared__ __align__(16) float lds[8192];
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    for (int i = threadIdx.x; i < 8192; i += kThreads) lds[i] = (float)i;
    __syncthreads();
    const unsigned addr = (unsigned)(size_t)(__attribute__((address_space(3))) float *)lds + wave * 8192 + lane * 16;
    f4v v = {seed, seed + lane, seed, seed}, r = v;
    for (int it = 0; it < iters; ++it) {
#pragma unroll
        for (int u = 0; u < 4; ++u) {
            if (WRITE)
                asm volatile("ds_write_b128 %0, %1 offset:%2" ::"v"(addr), "v"(v), "n"(u * 1024) : "memory");
            else
                asm volatile("ds_read_b128 %0, %1 offset:%2" : "=v"(r) : "v"(addr), "n"(u * 1024) : "memory");
        }
        asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");
    }
    if (r.x + r.y == 1234.5f) sink[0] = r.x;
}

// one wave per workgroup gathers pseudo-random 256-byte rows, four rows per load instruction
// (16 lanes x 16 bytes each), eight loads in flight: the access pattern of the gy gathers
__global__ __launch_bounds__(64) void mb_gather_kernel(const float *__restrict__ tab, int rows, float *sink, int iters)
{
    const int lane = threadIdx.x;
    unsigned h = blockIdx.x * 2654435761u + 12345u;
    f4v acc = {0.f, 0.f, 0.f, 0.f};
    const int sel = lane >> 4, col = (lane & 15) * 4;
    for (int it = 0; it < iters; it += 8) {
        f4v v[8];
#pragma unroll
        for (int u = 0; u < 8; ++u) {
            h = h * 1664525u + 1013904223u;
            unsigned hh = h + sel * 0x9E3779B9u;
            hh ^= hh >> 15;
            hh *= 2246822519u;
            hh ^= hh >> 13;
            v[u] = *reinterpret_cast<const f4v *>(tab + (size_t)(hh % (unsigned)rows) * 64 + col);
        }
#pragma unroll
        for (int u = 0; u < 8; ++u) acc += v[u];
    }
    if (acc.x + acc.y + acc.z + acc.w == 1234.5f) sink[0] = acc.x;
}

template <typename F>
bool time_ms(F launch, hipStream_t stream, float *ms)
{
    hipEvent_t a, b;
    if (hipEventCreate(&a) != hipSuccess) return false;
    if (hipEventCreate(&b) != hipSuccess) {
        (void)hipEventDestroy(a);
        return false;
    }
    launch();  // warm-up
    float best = 1e30f;
    bool ok = true;
    for (int r = 0; r < 3 && ok; ++r) {
        ok = hipEventRecord(a, stream) == hipSuccess;
        launch();
        ok = ok && hipEventRecord(b, stream) == hipSuccess && hipEventSynchronize(b) == hipSuccess;
        float t = 0.f;
        ok = ok && hipEventElapsedTime(&t, a, b) == hipSuccess;
        if (ok && t < best) best = t;
    }
    (void)hipEventDestroy(a);
    (void)hipEventDestroy(b);
    *ms = best;
    return ok && hipGetLastError() == hipSuccess;
}

}  // namespace

extern "C" lmkan_status lmkan_microbench(int32_t which, void *scratch_dev, size_t scratch_bytes, double *result_host,
                                         void *stream)
{
    if (!result_host) return LMKAN_ERR_NULL;
    if (which < 0 || which >= LMKAN_MICROBENCH_COUNT) return LMKAN_ERR_UNSUPPORTED;
    if (!scratch_dev) return LMKAN_ERR_NULL;
    if (scratch_bytes < ((size_t)64 << 20)) return LMKAN_ERR_WORKSPACE;
    if (reinterpret_cast<uintptr_t>(scratch_dev) % 256 != 0) return LMKAN_ERR_ALIGN;
    hipStream_t hs = static_cast<hipStream_t>(stream);
    int dev = 0, cus = 0, khz = 0;
    if (hipGetDevice(&dev) != hipSuccess ||
        hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess ||
        hipDeviceGetAttribute(&khz, hipDeviceAttributeClockRate, dev) != hipSuccess || cus <= 0 || khz <= 0)
        return LMKAN_ERR_HIP;
    (void)hipGetLastError();
    const double clk = (double)khz * 1e3;
    if (which == LMKAN_MICROBENCH_NOMINAL_CLOCK_GHZ) {
        *result_host = clk / 1e9;
        return LMKAN_OK;
    }
    float *sink = static_cast<float *>(scratch_dev);
    float ms = 0.f;
    bool ok = false;
    double value = 0.0;
    if (which == LMKAN_MICROBENCH_COPY_GBPS || which == LMKAN_MICROBENCH_READ_GBPS) {
        // the first 4 KiB stay free for the sink; copy: first half -> second half
        const size_t usable = (scratch_bytes - 4096) / 32 * 32;
        const size_t half = usable / 2;
        const f4v *src = reinterpret_cast<const f4v *>(static_cast<char *>(scratch_dev) + 4096);
        if (which == LMKAN_MICROBENCH_COPY_GBPS) {
            f4v *dst = reinterpret_cast<f4v *>(static_cast<char *>(scratch_dev) + 4096 + half);
            ok = time_ms([&] { mb_copy_kernel<<<cus * 16, kThreads, 0, hs>>>(src, dst, half / 16); }, hs, &ms);
            value = 2.0 * (double)half / (ms * 1e-3) / 1e9;  // bytes read + bytes written
        } else {
            ok = time_ms([&] { mb_read_kernel<<<cus * 16, kThreads, 0, hs>>>(src, sink, usable / 16); }, hs, &ms);
            value = (double)usable / (ms * 1e-3) / 1e9;
        }
    } else if (which == LMKAN_MICROBENCH_FMA_PER_CLK_CU || which == LMKAN_MICROBENCH_MFMA_FMA_PER_CLK_CU) {
        const int iters = 4096, waves = 4;  // four waves per SIMD
        if (which == LMKAN_MICROBENCH_FMA_PER_CLK_CU) {
            ok = time_ms([&] { mb_fma_kernel<<<cus * waves, kThreads, 0, hs>>>(sink, iters, 0.5f); }, hs, &ms);
            value = (double)cus * waves * kThreads * iters * 16.0 / (ms * 1e-3) / clk / cus;
        } else {
            ok = time_ms([&] { mb_mfma_kernel<<<cus * waves, kThreads, 0, hs>>>(sink, iters, 0.5f); }, hs, &ms);
            value = (double)cus * waves * (kThreads / 64) * iters * 8.0 * 256.0 / (ms * 1e-3) / clk / cus;
        }
    } else if (which == LMKAN_MICROBENCH_LDS_READ_B_PER_CLK_CU || which == LMKAN_MICROBENCH_LDS_WRITE_B_PER_CLK_CU) {
        const int iters = 4096, waves = 2;
        if (which == LMKAN_MICROBENCH_LDS_READ_B_PER_CLK_CU)
            ok = time_ms([&] { mb_lds_kernel<false><<<cus * waves, kThreads, 0, hs>>>(sink, iters, 0.5f); }, hs, &ms);
        else
            ok = time_ms([&] { mb_lds_kernel<true><<<cus * waves, kThreads, 0, hs>>>(sink, iters, 0.5f); }, hs, &ms);
        value = (double)cus * waves * (kThreads / 64) * iters * 4.0 * 1024.0 / (ms * 1e-3) / clk / cus;
    } else {
        const int rows = 8192, iters = 2048, waves = 32;  // 2 MiB table: resident in the L2 of an XCD
        const float *tab = reinterpret_cast<const float *>(static_cast<char *>(scratch_dev) + 4096);
        ok = time_ms([&] { mb_gather_kernel<<<cus * waves, 64, 0, hs>>>(tab, rows, sink, iters); }, hs, &ms);
        value = (double)cus * waves * iters * 1024.0 / (ms * 1e-3) / clk / cus;
    }
    if (!ok) return LMKAN_ERR_HIP;
    *result_host = value;
    return LMKAN_OK;
}
