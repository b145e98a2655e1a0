// Benchmark aids (not part of the paper's method): what this GPU itself sustains for the two
// resources the path is priced against, measured with kernels of the same build as the path's.
//   halo_peak_read_stream  a read-only stream organised like the one-token gate/up kernel: 256
//                          workgroups of four waves, a wave takes whole 16 KiB runs (a gate row and an
//                          up row at d = 4096) in 16-byte non-temporal loads per lane, the next run
//                          requested before the current one is consumed.
//   halo_peak_mfma_bf16    v_mfma_f32_16x16x32_bf16 issued back to back on 16 independent accumulator
//                          tiles per wave, two waves per SIMD, operands with ordinary non-zero values
//                          (the rate depends on the data: power).
// Both time their own launches with a HIP event pair on `stream` and wait for the result.
#include "../../include/halo.h"

#include "kernels.hpp"

namespace halo {
namespace {

constexpr int kRunPieces = 16;                       // 16 x 64 lanes x 16 B = 16 KiB per wave and run

struct Run {
    u32x4 v[kRunPieces];
};

__device__ __forceinline__ void load_run(Run &r, const u32x4 *__restrict__ p, int lane)
{
#pragma unroll
    for (int k = 0; k < kRunPieces; ++k) r.v[k] = __builtin_nontemporal_load(p + k * kWave + lane);
}

__device__ __forceinline__ uint32_t fold_run(const Run &r, uint32_t acc)
{
#pragma unroll
    for (int k = 0; k < kRunPieces; ++k) acc ^= r.v[k].x ^ r.v[k].y ^ r.v[k].z ^ r.v[k].w;
    return acc;
}

// n_runs runs of 16 KiB; wave w takes the contiguous range [n_runs*w/nw, n_runs*(w+1)/nw)
__global__ __launch_bounds__(256) void read_stream_kernel(const u32x4 *__restrict__ p, long long n_runs,
                                                          uint32_t *__restrict__ sink)
{
    const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
    const long long nw = (long long)gridDim.x * 4, w = (long long)blockIdx.x * 4 + wave;
    const long long r0 = n_runs * w / nw, r1 = n_runs * (w + 1) / nw;
    if (r0 >= r1) return;
    constexpr size_t kStride = (size_t)kRunPieces * kWave;      // 16-byte pieces per run
    Run a, b;
    uint32_t acc = 0;
    load_run(a, p + (size_t)r0 * kStride, lane);
    long long r = r0;
    while (r + 2 < r1) {
        load_run(b, p + (size_t)(r + 1) * kStride, lane);
        __builtin_amdgcn_sched_barrier(0);
        acc = fold_run(a, acc);
        load_run(a, p + (size_t)(r + 2) * kStride, lane);
        __builtin_amdgcn_sched_barrier(0);
        acc = fold_run(b, acc);
        r += 2;
    }
    if (r + 1 < r1) {
        load_run(b, p + (size_t)(r + 1) * kStride, lane);
        acc = fold_run(a, acc);
        acc = fold_run(b, acc);
    } else {
        acc = fold_run(a, acc);
    }
    if (acc == 0x9e3779b9u) sink[0] = acc;           // keeps the loads alive; practically never taken
}

typedef float f32x4_t __attribute__((ext_vector_type(4)));
typedef __bf16 bf16x8_t __attribute__((ext_vector_type(8)));

constexpr int kMfmaTiles = 16;

__global__ __launch_bounds__(512) void mfma_rate_kernel(int iters, float *__restrict__ sink)
{
    const int lane = threadIdx.x & 63;
    // operands: bf16 values of ordinary size that differ by lane and element (no zeros, no repeats);
    // a 4 x 4 grid of accumulator tiles fed by four row operands and four column operands, as in a
    // register-tiled matrix product
    uint32_t h = (uint32_t)(blockIdx.x * 512 + threadIdx.x) * 2654435761u + 12345u;
    auto next_pair = [&]() -> uint32_t {
        h = h * 1664525u + 1013904223u;
        const uint32_t lo = 0x3c00u + ((h >> 8) & 0x3ffu);          // bf16 in [2^-7, 2^-3)
        const uint32_t hi = 0xbc00u + ((h >> 20) & 0x3ffu);         // and its negative range
        return lo | (hi << 16);
    };
    u32x4 a[4], b[4];
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        a[i] = u32x4{next_pair(), next_pair(), next_pair(), next_pair()};
        b[i] = u32x4{next_pair(), next_pair(), next_pair(), next_pair()};
    }
    f32x4_t acc[kMfmaTiles];
#pragma unroll
    for (int t = 0; t < kMfmaTiles; ++t) acc[t] = f32x4_t{0.0f, 0.0f, 0.0f, 0.0f};
    for (int it = 0; it < iters; ++it) {
#pragma unroll
        for (int t = 0; t < kMfmaTiles; ++t)
            acc[t] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8_t, a[t >> 2]),
                                                             __builtin_bit_cast(bf16x8_t, b[t & 3]), acc[t], 0, 0, 0);
    }
    float s = 0.0f;
#pragma unroll
    for (int t = 0; t < kMfmaTiles; ++t) s += acc[t].x + acc[t].y + acc[t].z + acc[t].w;
    if (s == 12345.678f) sink[lane] = s;
}

struct EventPair {
    hipEvent_t e0 = nullptr, e1 = nullptr;
    bool ok = false;
    EventPair() { ok = hipEventCreate(&e0) == hipSuccess && hipEventCreate(&e1) == hipSuccess; }
    ~EventPair()
    {
        if (e0) (void)hipEventDestroy(e0);
        if (e1) (void)hipEventDestroy(e1);
    }
};

}  // namespace
}  // namespace halo

extern "C" {

int halo_peak_read_stream(const void *buf, size_t buf_bytes, size_t window_bytes, int32_t launches,
                          void *sink, void *stream, double *gbps, double *us_per_launch)
{
    using namespace halo;
    constexpr size_t kRunBytes = (size_t)kRunPieces * kWave * 16;
    if (!buf || !sink) return HALO_ERR_NULL;
    if ((reinterpret_cast<uintptr_t>(buf) & 15u) || launches < 1 || launches > 65536 || window_bytes < kRunBytes ||
        window_bytes > buf_bytes)
        return HALO_ERR_ARG;
    const long long n_runs = (long long)(window_bytes / kRunBytes);
    const size_t win = (size_t)n_runs * kRunBytes;
    const size_t n_windows = buf_bytes / win;               // consecutive launches read different memory
    hipStream_t s = static_cast<hipStream_t>(stream);
    EventPair ev;
    if (!ev.ok) return HALO_ERR_HIP;
    auto launch = [&](int i) {
        const char *p = static_cast<const char *>(buf) + (size_t)(i % (int)n_windows) * win;
        read_stream_kernel<<<dim3(256), dim3(256), 0, s>>>(reinterpret_cast<const u32x4 *>(p), n_runs,
                                                           static_cast<uint32_t *>(sink));
    };
    launch(launches);                                       // untimed: code object upload, clocks
    if (hipEventRecord(ev.e0, s) != hipSuccess) return HALO_ERR_HIP;
    for (int i = 0; i < launches; ++i) launch(i);
    if (hipEventRecord(ev.e1, s) != hipSuccess || hipGetLastError() != hipSuccess) return HALO_ERR_HIP;
    float ms = 0.0f;
    if (hipEventSynchronize(ev.e1) != hipSuccess || hipEventElapsedTime(&ms, ev.e0, ev.e1) != hipSuccess)
        return HALO_ERR_HIP;
    if (gbps) *gbps = (double)win * launches / (ms * 1e-3) / 1e9;
    if (us_per_launch) *us_per_launch = ms * 1e3 / launches;
    return HALO_OK;
}

int halo_peak_mfma_bf16(int32_t iters, int32_t launches, void *sink, void *stream, double *tflops)
{
    using namespace halo;
    if (!sink) return HALO_ERR_NULL;
    if (iters < 1 || iters > (1 << 20) || launches < 1 || launches > 1024) return HALO_ERR_ARG;
    hipStream_t s = static_cast<hipStream_t>(stream);
    EventPair ev;
    if (!ev.ok) return HALO_ERR_HIP;
    constexpr int kBlocks = 256;                            // one workgroup of eight waves per compute unit
    mfma_rate_kernel<<<dim3(kBlocks), dim3(512), 0, s>>>(iters, static_cast<float *>(sink));
    if (hipEventRecord(ev.e0, s) != hipSuccess) return HALO_ERR_HIP;
    for (int i = 0; i < launches; ++i)
        mfma_rate_kernel<<<dim3(kBlocks), dim3(512), 0, s>>>(iters, static_cast<float *>(sink));
    if (hipEventRecord(ev.e1, s) != hipSuccess || hipGetLastError() != hipSuccess) return HALO_ERR_HIP;
    float ms = 0.0f;
    if (hipEventSynchronize(ev.e1) != hipSuccess || hipEventElapsedTime(&ms, ev.e0, ev.e1) != hipSuccess)
        return HALO_ERR_HIP;
    const double flops = (double)launches * kBlocks * 8 * iters * kMfmaTiles * (16.0 * 16.0 * 32.0 * 2.0);
    if (tflops) *tflops = flops / (ms * 1e-3) / 1e12;
    return HALO_OK;
}

}  // extern "C"
