// Measurement aid, not part of the method: plain streaming-read kernels of given sizes, back to back on one
// stream, to establish what the chip gives a kernel chain that does nothing but read -- the ceiling the
// projection kernels of a verify step are compared with.
#include <hip/hip_runtime.h>

#include <vector>

#include "../../include/spd.h"
#include "gemm_core.h"
#include "launch.h"

namespace spd {

// Every wave reads a contiguous run of 1 KiB blocks with non-temporal 16-byte loads, 16 blocks in flight.
__global__ __launch_bounds__(512) void read_probe_kernel(const uint4 *__restrict__ p, size_t n_blocks, unsigned *__restrict__ sink) {
    const int lane = threadIdx.x & 63;
    const size_t wave = ((size_t)blockIdx.x * blockDim.x + threadIdx.x) >> 6;
    const size_t n_waves = ((size_t)gridDim.x * blockDim.x) >> 6;
    const size_t b0 = n_blocks * wave / n_waves, b1 = n_blocks * (wave + 1) / n_waves;
    uint4 acc = {0u, 0u, 0u, 0u};
    size_t b = b0;
    for (; b + 16 <= b1; b += 16) {
        uint4 v[16];
#pragma unroll
        for (int u = 0; u < 16; ++u) v[u] = load_stream(p + (b + u) * 64 + lane);
#pragma unroll
        for (int u = 0; u < 16; ++u) { acc.x ^= v[u].x; acc.y ^= v[u].y; acc.z ^= v[u].z; acc.w ^= v[u].w; }
    }
    for (; b < b1; ++b) {
        const uint4 v = load_stream(p + b * 64 + lane);
        acc.x ^= v.x; acc.y ^= v.y; acc.z ^= v.z; acc.w ^= v.w;
    }
    if ((acc.x ^ acc.y ^ acc.z ^ acc.w) == 0x9e3779b9u) sink[wave & 1023] = 1;     // keeps the loads alive; practically never true
}

}  // namespace spd

extern "C" int32_t spd_probe_read_chain(const void *buffer, size_t buffer_bytes, const size_t *h_stage_bytes, int32_t n_stages,
                                        int32_t reps, void *sink, double *h_kernel_us, double *h_chain_us_per_rep, void *stream) {
    using namespace spd;
    if (!buffer || !h_stage_bytes || !sink || !h_kernel_us || !h_chain_us_per_rep || n_stages < 1 || n_stages > 64 || reps < 1)
        return SPD_ERR_INVALID_ARG;
    size_t total = 0;
    for (int i = 0; i < n_stages; ++i) {
        if (h_stage_bytes[i] < 1024 || (h_stage_bytes[i] & 1023)) return SPD_ERR_INVALID_ARG;
        total += h_stage_bytes[i];
    }
    if (total > buffer_bytes || ((uintptr_t)buffer & 15)) return SPD_ERR_CAPACITY;
    hipStream_t st = (hipStream_t)stream;
    int dev = 0, cus = 0;
    if (hipGetDevice(&dev) != hipSuccess || hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess) return SPD_ERR_HIP;
    std::vector<hipEvent_t> ev(2 * (size_t)n_stages + 2);
    for (auto &e : ev)
        if (hipEventCreate(&e) != hipSuccess) return SPD_ERR_HIP;
    hipEvent_t c0 = ev[2 * n_stages], c1 = ev[2 * n_stages + 1];
    int32_t rc = SPD_OK;
    for (int i = 0; i < n_stages; ++i) h_kernel_us[i] = 0.0;
    // different windows of the buffer in consecutive repetitions, so that nothing is served from a cache
    const size_t n_windows = buffer_bytes / total;
    size_t window = 0;
    auto run_chain = [&](bool timed) {
        const char *base = (const char *)buffer + (window++ % n_windows) * total;
        for (int i = 0; i < n_stages; ++i) {
            LaunchTiming lt{ev[2 * i], ev[2 * i + 1], false};
            if (timed) launch_timing() = &lt;
            launch_kernel(read_probe_kernel, dim3(cus), dim3(512), st, (const uint4 *)base, h_stage_bytes[i] / 1024, (unsigned *)sink);
            launch_timing() = nullptr;
            base += h_stage_bytes[i];
        }
    };
    run_chain(false);
    run_chain(false);
    // (a) the chain as a whole, untimed launches
    if (hipEventRecord(c0, st) != hipSuccess) rc = SPD_ERR_HIP;
    for (int r = 0; r < reps; ++r) run_chain(false);
    if (hipEventRecord(c1, st) != hipSuccess || hipEventSynchronize(c1) != hipSuccess) rc = SPD_ERR_HIP;
    float ms = 0.f;
    if (rc == SPD_OK && hipEventElapsedTime(&ms, c0, c1) != hipSuccess) rc = SPD_ERR_HIP;
    *h_chain_us_per_rep = (double)ms * 1e3 / reps;
    // (b) every kernel's own execution time (start / stop events handed to the launch)
    for (int r = 0; r < reps && rc == SPD_OK; ++r) {
        run_chain(true);
        if (hipStreamSynchronize(st) != hipSuccess) { rc = SPD_ERR_HIP; break; }
        for (int i = 0; i < n_stages; ++i) {
            float k = 0.f;
            if (hipEventElapsedTime(&k, ev[2 * i], ev[2 * i + 1]) != hipSuccess) { rc = SPD_ERR_HIP; break; }
            h_kernel_us[i] += (double)k * 1e3 / reps;
        }
    }
    for (auto &e : ev) (void)hipEventDestroy(e);
    return rc;
}
