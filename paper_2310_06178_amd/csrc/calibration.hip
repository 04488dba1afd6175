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

// The same read with the launch shape, the loads in flight and the cache policy as parameters: the sweep behind
// the statement of what one launch that only reads can reach.  kDepth loads of 16 bytes per lane in flight per
// wavefront; kNonTemporal marks the loads as streaming (they are not kept in the caches).
template <int kDepth, bool kNonTemporal>
__global__ void __launch_bounds__(1024)
stream_read_shape_kernel(const void* src, uint32_t bytes, uint32_t* sink, int waves_total, int loads)
{
    const int lane = threadIdx.x & 63;
    const int w = blockIdx.x * (blockDim.x >> 6) + (threadIdx.x >> 6);
    __amdgpu_buffer_rsrc_t rsrc = __builtin_amdgcn_make_buffer_rsrc((void*)src, 0, (int)bytes, 0x00020000);
    constexpr int kAux = kNonTemporal ? 2 : 0;
    const uint32_t stride = (uint32_t)waves_total * 1024u;   // load t of all wavefronts is contiguous
    const uint32_t base = (uint32_t)w * 1024u + (uint32_t)lane * 16u;
    typedef unsigned v4 __attribute__((ext_vector_type(4)));
    v4 v[kDepth];
    uint32_t acc = 0;
#pragma unroll
    for (int t = 0; t < kDepth; ++t) v[t] = __builtin_amdgcn_raw_buffer_load_b128(rsrc, (int)(base + (uint32_t)t * stride), 0, kAux);
    for (int t0 = 0; t0 < loads; t0 += kDepth) {   // (loads is a multiple of kDepth)
#pragma unroll
        for (int u = 0; u < kDepth; ++u) {
            const v4 x = v[u];
            acc += x.x ^ x.y ^ x.z ^ x.w;
            asm volatile("" : "+v"(acc));
            // past the end the offset is out of the buffer's range: no memory access
            v[u] = __builtin_amdgcn_raw_buffer_load_b128(
                rsrc, t0 + u + kDepth < loads ? (int)(base + (uint32_t)(t0 + u + kDepth) * stride) : 0x7ffffff0, 0, kAux);
            __builtin_amdgcn_sched_barrier(0);
        }
    }
    if (acc == 0x12345678u) *sink = acc;
}

// Conflict-free LDS reads and nothing else: every lane reads `reads` times W bytes, consecutive lanes
// consecutive W-byte slots (so the lanes served together cover all banks), eight reads in flight.
constexpr int kLdsCalibWaves = 16;
constexpr int kLdsCalibBytes = 65536;

template <typename T>
__global__ void __launch_bounds__(kLdsCalibWaves * 64)
lds_read_kernel(uint32_t* sink, int reads)
{
    __shared__ __align__(16) unsigned char lds[kLdsCalibBytes];
    constexpr int kSlots = kLdsCalibBytes / (int)sizeof(T);
    for (int i = threadIdx.x; i < kLdsCalibBytes / 4; i += blockDim.x) ((uint32_t*)lds)[i] = (uint32_t)i * 2654435761u;
    __syncthreads();
    // eight reads per round at fixed distances from the lane's own slot (immediate offsets: no
    // address arithmetic competes with the reads); consecutive lanes read consecutive slots
    uint32_t base = (uint32_t)(threadIdx.x * sizeof(T));  // byte offset of the lane's slot
    constexpr int kStride = 1024 * (kSlots / 1024 >= 8 ? kSlots / 1024 / 8 : 1);  // slots between the eight reads
    for (int it = 0; it < reads; it += 8) {
        // opaque copies of the offset: the reads are neither hoisted out of the loop nor merged into
        // two-address forms (a gather cannot use those)
        uint32_t at[8];
#pragma unroll
        for (int u = 0; u < 8; ++u) at[u] = base;
        asm volatile("" : "+v"(at[0]), "+v"(at[1]), "+v"(at[2]), "+v"(at[3]), "+v"(at[4]), "+v"(at[5]), "+v"(at[6]), "+v"(at[7]));
        T v[8];
#pragma unroll
        for (int u = 0; u < 8; ++u) v[u] = ((const T*)(lds + at[u]))[(u * kStride) % kSlots];
        // every byte read is demanded in a register, by no instruction: nothing but the reads is timed
#pragma unroll
        for (int u = 0; u < 8; ++u) {
            if constexpr (sizeof(T) == 16) asm volatile("" ::"v"(v[u].x), "v"(v[u].y), "v"(v[u].z), "v"(v[u].w));
            else if constexpr (sizeof(T) == 8) asm volatile("" ::"v"(v[u].x), "v"(v[u].y));
            else asm volatile("" ::"v"(v[u]));
        }
    }
    const uint32_t all = base;
    if (all == 0x12345678u) *sink = all;
}

// The batched kernels' inner loop and nothing else: a 16-byte table look-up at an address a v_perm_b32 makes from a
// code byte, and the two matrix-core adds (v_mfma_f32_4x4x4_16b_f16 against the identity) that put its eight fp16
// columns into fp32 sums; eight wavefronts per compute unit over a 128 KiB table, the look-ups one chunk of eight
// ahead of the adds, the order left to the compiler.  No code stream, no table build, no barriers: the rate at which
// this device sustains the instruction mix, which is what bounds those kernels (LDS and matrix cores are both near
// their limit at 256 bytes per clock per compute unit).
constexpr int kMixWaves = 8;
typedef _Float16 mix_h4 __attribute__((ext_vector_type(4)));
typedef float mix_f4 __attribute__((ext_vector_type(4)));

__global__ void __launch_bounds__(kMixWaves * 64)
lookup_add_kernel(uint32_t* sink, int tiles)
{
    __shared__ __align__(16) unsigned char lds[2 * 65536];
    for (int i = threadIdx.x; i < 2 * 65536 / 4; i += blockDim.x) ((uint32_t*)lds)[i] = 0x3c003800u;  // (1.0, 0.5)
    __syncthreads();
    const int lane = threadIdx.x & 63;
    const int j = lane & 15, half = (lane >> 4) & 1;
    // sixteen "code loads" of eight code bytes each, as a wavefront holds them for one k-tile
    uint32_t codes[16][2];
    uint32_t h = (uint32_t)threadIdx.x * 2654435761u + 12345u;
    for (int t = 0; t < 16; ++t)
        for (int w = 0; w < 2; ++w) {
            h = h * 1664525u + 1013904223u;
            codes[t][w] = h;
        }
    mix_h4 onehot;
    for (int e = 0; e < 4; ++e) onehot[e] = (_Float16)((lane & 3) == e ? 1.0f : 0.0f);
    mix_f4 dlo[8], dhi[8];
    for (int s = 0; s < 8; ++s) {
        dlo[s] = mix_f4{0, 0, 0, 0};
        dhi[s] = mix_f4{0, 0, 0, 0};
    }
    uint4 ent[2][8];
    auto look = [&](int t, uint4 (&e)[8]) {
        const uint32_t lane_off = (uint32_t)((j + t) & 15) * 16u | ((uint32_t)half << 16);
#pragma unroll
        for (int s = 0; s < 8; ++s) {
            const uint32_t addr = __builtin_amdgcn_perm(codes[t][s >> 2], lane_off, 0x0c020000u | ((4u + (s & 3)) << 8));
            e[s] = *(const uint4*)(lds + addr);
        }
    };
    auto add = [&](const uint4 (&e)[8]) {
#pragma unroll
        for (int s = 0; s < 8; ++s) {
            mix_h4 lo, up;
            __builtin_memcpy(&lo, &e[s].x, 8);
            __builtin_memcpy(&up, &e[s].z, 8);
            dlo[s] = __builtin_amdgcn_mfma_f32_4x4x4f16(lo, onehot, dlo[s], 0, 0, 0);
            dhi[s] = __builtin_amdgcn_mfma_f32_4x4x4f16(up, onehot, dhi[s], 0, 0, 0);
        }
    };
    for (int it = 0; it < tiles; ++it) {
        look(0, ent[0]);
#pragma unroll
        for (int t = 0; t < 16; ++t) {
            if (t + 1 < 16) look(t + 1, ent[(t + 1) & 1]);
            add(ent[t & 1]);
        }
        // the codes are opaque again: nothing of a k-tile is hoisted out of the loop
#pragma unroll
        for (int t = 0; t < 16; ++t) asm volatile("" : "+v"(codes[t][0]), "+v"(codes[t][1]));
    }
    float total = 0.0f;
    for (int s = 0; s < 8; ++s) total += dlo[s][0] + dhi[s][3];
    if (total == -1.0f) *sink = 1u;  // (the sums are positive)
}

}  // namespace

int launch_calib_lookup_add(int tiles, void* sink, size_t* lookups_out, hipStream_t s)
{
    int cus = 256, dev = 0;
    hipDeviceProp_t prop;
    if (hipGetDevice(&dev) == hipSuccess && hipGetDeviceProperties(&prop, dev) == hipSuccess &&
        prop.multiProcessorCount > 0)
        cus = prop.multiProcessorCount;
    if (!sink || tiles < 1 || tiles > (1 << 16)) return MSGEMM_ERR_INVALID_ARG;
    hipLaunchKernelGGL(lookup_add_kernel, dim3((unsigned)cus), dim3(kMixWaves * 64), 0, s, (uint32_t*)sink, tiles);
    MSGEMM_HIP_TRY(hipGetLastError());
    if (lookups_out) *lookups_out = (size_t)cus * kMixWaves * 64 * 128 * (size_t)tiles;
    return MSGEMM_OK;
}

int launch_calib_lds_read(int width_bytes, int reads, void* sink, size_t* bytes_out, hipStream_t s)
{
    int cus = 256, dev = 0;
    hipDeviceProp_t prop;
    if (hipGetDevice(&dev) == hipSuccess && hipGetDeviceProperties(&prop, dev) == hipSuccess &&
        prop.multiProcessorCount > 0)
        cus = prop.multiProcessorCount;
    if (!sink || reads < 8 || reads % 8 != 0 || reads > (1 << 20)) return MSGEMM_ERR_INVALID_ARG;
    const dim3 grid((unsigned)cus), blk(kLdsCalibWaves * 64);
    if (width_bytes == 16) hipLaunchKernelGGL(lds_read_kernel<uint4>, grid, blk, 0, s, (uint32_t*)sink, reads);
    else if (width_bytes == 8) hipLaunchKernelGGL(lds_read_kernel<uint2>, grid, blk, 0, s, (uint32_t*)sink, reads);
    else if (width_bytes == 4) hipLaunchKernelGGL(lds_read_kernel<uint32_t>, grid, blk, 0, s, (uint32_t*)sink, reads);
    else return MSGEMM_ERR_INVALID_ARG;
    MSGEMM_HIP_TRY(hipGetLastError());
    if (bytes_out) *bytes_out = (size_t)cus * kLdsCalibWaves * 64 * (size_t)reads * (size_t)width_bytes;
    return MSGEMM_OK;
}

int launch_calib_stream_read_shape(const void* src, size_t bytes, void* sink, int waves_per_workgroup,
                                   int workgroups_per_cu, int depth, int non_temporal, hipStream_t s)
{
    int cus = 256, dev = 0;
    hipDeviceProp_t prop;
    if (hipGetDevice(&dev) == hipSuccess && hipGetDeviceProperties(&prop, dev) == hipSuccess &&
        prop.multiProcessorCount > 0)
        cus = prop.multiProcessorCount;
    if (waves_per_workgroup < 1 || waves_per_workgroup > 16 || workgroups_per_cu < 1 || workgroups_per_cu > 16)
        return MSGEMM_ERR_INVALID_ARG;
    const int64_t waves = (int64_t)cus * workgroups_per_cu * waves_per_workgroup;
    if (bytes == 0 || bytes >= ((size_t)1 << 31) || bytes % ((size_t)waves * 1024) != 0) return MSGEMM_ERR_INVALID_ARG;
    const int64_t loads = (int64_t)(bytes / ((size_t)waves * 1024));
    if (loads % depth != 0) return MSGEMM_ERR_INVALID_ARG;
    const dim3 grid((unsigned)(cus * workgroups_per_cu)), blk((unsigned)(waves_per_workgroup * 64));
#define MSGEMM_SHAPE(D)                                                                                              \
    if (depth == D) {                                                                                                \
        if (non_temporal)                                                                                            \
            hipLaunchKernelGGL((stream_read_shape_kernel<D, true>), grid, blk, 0, s, src, (uint32_t)bytes,           \
                               (uint32_t*)sink, (int)waves, (int)loads);                                             \
        else                                                                                                         \
            hipLaunchKernelGGL((stream_read_shape_kernel<D, false>), grid, blk, 0, s, src, (uint32_t)bytes,          \
                               (uint32_t*)sink, (int)waves, (int)loads);                                             \
        MSGEMM_HIP_TRY(hipGetLastError());                                                                           \
        return MSGEMM_OK;                                                                                            \
    }
    MSGEMM_SHAPE(1) MSGEMM_SHAPE(2) MSGEMM_SHAPE(4) MSGEMM_SHAPE(8) MSGEMM_SHAPE(16)
#undef MSGEMM_SHAPE
    return MSGEMM_ERR_INVALID_ARG;
}

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
