// Two-launch msGeMM: the table L lives in device memory and is shared by all
// rows (Section 4: "L computed in phase 1 is kept in cache").  Works for every
// d in 1..4, every dtype pair and every scale block size; it is the reference
// schedule on the GPU, not the fast one.
#include "device_types.h"
#include "msgemm_internal.h"

namespace msgemm {

namespace {

struct GroupGeom {
    int64_t k, block, gpb;
    int d;
};

__device__ __forceinline__ void group_span(const GroupGeom& g, int64_t jg, int64_t& first, int& len)
{
    int64_t blk = jg / g.gpb, t = jg - blk * g.gpb;
    first = blk * g.block + t * g.d;
    int64_t end = (blk + 1) * g.block;
    len = (int)((first + g.d <= end) ? g.d : (end - first));
}

// Phase 1 (Section 3.1): one thread per (group, code combination, column).
template <typename XT, typename LT>
__global__ void __launch_bounds__(256)
build_lut_kernel(GroupGeom g, int64_t groups, int64_t b, const XT* __restrict__ X, int64_t ldx,
                 ValueMap values, LT* __restrict__ L)
{
    const int64_t E = (int64_t)1 << (4 * g.d);
    const int64_t total = groups * E * b;
    for (int64_t t = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; t < total;
         t += (int64_t)gridDim.x * blockDim.x) {
        int64_t c = t % b;
        int64_t rest = t / b;
        int64_t idx = rest & (E - 1);
        int64_t jg = rest >> (4 * g.d);
        int64_t first;
        int len;
        group_span(g, jg, first, len);
        LT s = 0;
        for (int r = 0; r < len; ++r) {
            LT w = code_value(values, (unsigned)(idx >> (4 * r)) & 15u, LT());
            s += w * (LT)XTraits<XT>::load(X + c * ldx + first + r);
        }
        L[t] = s;
    }
}

__device__ __forceinline__ unsigned code_at(const uint8_t* __restrict__ row, int64_t j)
{
    unsigned byte = row[j >> 1];
    return (j & 1) ? (byte >> 4) : (byte & 15u);
}

// y += q * s for a finished scale block (q = 1 without scales).
__device__ __forceinline__ float add_block(const __half* __restrict__ scales, int64_t at, float s, float y)
{
    return scales ? fmaf(__half2float(scales[at]), s, y) : y + s;
}
__device__ __forceinline__ int add_block(const __half* __restrict__, int64_t, int s, int y) { return y + s; }

// Phase 2 (Section 3.2) with the block scale applied after the block's groups
// have been consumed (Section 3.3): one thread per output element.
template <typename LT, typename YT>
__global__ void __launch_bounds__(256)
consume_lut_kernel(GroupGeom g, int64_t m, int64_t b, int64_t nblocks,
                   const uint8_t* __restrict__ codes, const __half* __restrict__ scales,
                   const LT* __restrict__ L, YT* __restrict__ Y, int64_t ldy)
{
    const int64_t E = (int64_t)1 << (4 * g.d);
    const int64_t total = m * b;
    for (int64_t t = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; t < total;
         t += (int64_t)gridDim.x * blockDim.x) {
        int64_t c = t % b, i = t / b;
        const uint8_t* row = codes + i * (g.k / 2);
        LT y = 0;
        for (int64_t blk = 0; blk < nblocks; ++blk) {
            LT s = 0;
            for (int64_t tg = 0; tg < g.gpb; ++tg) {
                int64_t jg = blk * g.gpb + tg, first;
                int len;
                group_span(g, jg, first, len);
                int64_t idx = 0;
                for (int r = 0; r < len; ++r) idx |= (int64_t)code_at(row, first + r) << (4 * r);
                s += L[(jg * E + idx) * b + c];
            }
            y = add_block(scales, i * nblocks + blk, s, y);
        }
        Y[c * ldy + i] = to_output<YT, LT>(y);
    }
}

inline unsigned grid_for(int64_t total, int threads)
{
    int64_t blocks = (total + threads - 1) / threads;
    const int64_t cap = 256 * 64;
    return (unsigned)(blocks < 1 ? 1 : (blocks > cap ? cap : blocks));
}

}  // namespace

int launch_build_lut(const Plan& p, const void* X, int64_t ldx, void* L, hipStream_t s)
{
    GroupGeom g{p.k, p.block, p.gpb, p.d};
    ValueMap vm;
    for (int i = 0; i < 16; ++i) vm.v[i] = p.values[i];
    const int64_t total = p.lut_groups * ((int64_t)1 << (4 * p.d)) * p.b;
    dim3 grid(grid_for(total, 256)), blk(256);
    switch (p.x_dtype) {
    case MSGEMM_F32:
        hipLaunchKernelGGL((build_lut_kernel<float, float>), grid, blk, 0, s, g, p.lut_groups, p.b,
                           (const float*)X, ldx, vm, (float*)L);
        break;
    case MSGEMM_F16:
        hipLaunchKernelGGL((build_lut_kernel<__half, float>), grid, blk, 0, s, g, p.lut_groups, p.b,
                           (const __half*)X, ldx, vm, (float*)L);
        break;
    case MSGEMM_BF16:
        hipLaunchKernelGGL((build_lut_kernel<bf16_t, float>), grid, blk, 0, s, g, p.lut_groups, p.b,
                           (const bf16_t*)X, ldx, vm, (float*)L);
        break;
    case MSGEMM_I8:
        hipLaunchKernelGGL((build_lut_kernel<int8_t, int>), grid, blk, 0, s, g, p.lut_groups, p.b,
                           (const int8_t*)X, ldx, vm, (int*)L);
        break;
    default:
        return MSGEMM_ERR_INVALID_ARG;
    }
    MSGEMM_HIP_TRY(hipGetLastError());
    return MSGEMM_OK;
}

int launch_consume_lut(const Plan& p, const void* L, void* Y, int64_t ldy, hipStream_t s)
{
    GroupGeom g{p.k, p.block, p.gpb, p.d};
    dim3 grid(grid_for(p.m * p.b, 256)), blk(256);
    const __half* sc = (const __half*)p.scales;
    switch (p.y_dtype) {
    case MSGEMM_F32:
        hipLaunchKernelGGL((consume_lut_kernel<float, float>), grid, blk, 0, s, g, p.m, p.b, p.nblocks,
                           p.codes, sc, (const float*)L, (float*)Y, ldy);
        break;
    case MSGEMM_F16:
        hipLaunchKernelGGL((consume_lut_kernel<float, __half>), grid, blk, 0, s, g, p.m, p.b, p.nblocks,
                           p.codes, sc, (const float*)L, (__half*)Y, ldy);
        break;
    case MSGEMM_BF16:
        hipLaunchKernelGGL((consume_lut_kernel<float, bf16_t>), grid, blk, 0, s, g, p.m, p.b, p.nblocks,
                           p.codes, sc, (const float*)L, (bf16_t*)Y, ldy);
        break;
    case MSGEMM_I32:
        hipLaunchKernelGGL((consume_lut_kernel<int, int>), grid, blk, 0, s, g, p.m, p.b, p.nblocks,
                           p.codes, (const __half*)nullptr, (const int*)L, (int*)Y, ldy);
        break;
    default:
        return MSGEMM_ERR_INVALID_ARG;
    }
    MSGEMM_HIP_TRY(hipGetLastError());
    return MSGEMM_OK;
}

}  // namespace msgemm
