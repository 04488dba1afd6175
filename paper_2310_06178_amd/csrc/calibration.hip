// A plain streaming-read kernel with the launch shape of the fused kernel's
// code stream.  It is the yardstick for "how fast can one launch pull this
// many cold bytes through the memory system", nothing more.
#include "msgemm_internal.h"

namespace msgemm {
namespace {

constexpr int kCalibWaves = 8;   // wavefronts per workgroup
constexpr int kCalibDepth = 8;   // loads a wavefront keeps in flight

// Load t of all wavefronts is contiguous (the fused kernel's load-major order);
// every lane takes 16 bytes per load.
__global__ void __launch_bounds__(kCalibWaves * 64)
stream_read_kernel(const uint4* __restrict__ src, uint32_t* sink, int64_t waves_total, int loads)
{
    const int lane = threadIdx.x & 63;
    const int64_t w = (int64_t)blockIdx.x * kCalibWaves + (threadIdx.x >> 6);
    uint4 v[kCalibDepth];
    uint32_t acc = 0;
    auto at = [&](int t) { return src + ((int64_t)t * waves_total + w) * 64 + lane; };
#pragma unroll
    for (int t = 0; t < kCalibDepth; ++t) v[t] = *at(t < loads ? t : 0);
    auto take = [&](int u) {
        const uint4 x = v[u];
        acc += x.x ^ x.y ^ x.z ^ x.w;
        asm volatile("" : "+v"(acc));
    };
    int t0 = 0;
    for (; t0 + 2 * kCalibDepth <= loads; t0 += kCalibDepth) {  // steady state: every slot is refilled
#pragma unroll
        for (int u = 0; u < kCalibDepth; ++u) {
            take(u);
            v[u] = *at(t0 + u + kCalibDepth);
            __builtin_amdgcn_sched_barrier(0);
        }
    }
    for (; t0 < loads; t0 += kCalibDepth) {  // tail: refill only what is left
#pragma unroll
        for (int u = 0; u < kCalibDepth; ++u) {
            if (t0 + u < loads) take(u);
            if (t0 + u + kCalibDepth < loads) v[u] = *at(t0 + u + kCalibDepth);
        }
    }
    if (acc == 0x12345678u) *sink = acc;
}

}  // namespace

int launch_calib_stream_read(const void* src, size_t bytes, void* sink, hipStream_t s)
{
    int cus = 256, dev = 0;
    hipDeviceProp_t prop;
    if (hipGetDevice(&dev) == hipSuccess && hipGetDeviceProperties(&prop, dev) == hipSuccess &&
        prop.multiProcessorCount > 0)
        cus = prop.multiProcessorCount;
    const size_t per_load = (size_t)cus * kCalibWaves * 1024;  // bytes one load of every wavefront covers
    if (bytes == 0 || bytes % per_load != 0 || bytes / per_load > 4096) return MSGEMM_ERR_INVALID_ARG;
    hipLaunchKernelGGL(stream_read_kernel, dim3((unsigned)cus), dim3(kCalibWaves * 64), 0, s, (const uint4*)src,
                       (uint32_t*)sink, (int64_t)cus * kCalibWaves, (int)(bytes / per_load));
    MSGEMM_HIP_TRY(hipGetLastError());
    return MSGEMM_OK;
}

}  // namespace msgemm
