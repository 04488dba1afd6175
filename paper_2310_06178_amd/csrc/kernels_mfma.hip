// Comparison point, not msGeMM: the same Y = M x X as a dense contraction on the
// matrix cores.  The 4-bit codes are expanded to fp16 / bf16 in registers (exact:
// the values are the integers -8..7), multiplied with X by 32x32x8 MFMA
// instructions with fp32 accumulation, and each scale block's partial product is
// multiplied by its scale in fp32 (the same factoring-out as Section 3.3).
// It exists so that the table-lookup path can be timed against the unit the
// paper says it has to compete with (Section 6); nothing in msgemm_run uses it.
//
// Tiling: a workgroup of 4 wavefronts owns 128 rows x 64 (or 32) batch columns;
// each wavefront owns 32 rows (the MFMA M dimension).  The k loop advances 128
// columns at a time: the X slab is staged in LDS once per workgroup (double
// buffered, fetched one chunk ahead), each lane loads 32 bytes of codes of its
// row from the row-major matrix and feeds 16 MFMA steps from them.
#include "device_types.h"
#include "msgemm_internal.h"

namespace msgemm {
namespace {

typedef _Float16 half4 __attribute__((ext_vector_type(4)));
typedef short short4v __attribute__((ext_vector_type(4)));
typedef float float16v __attribute__((ext_vector_type(16)));

constexpr int kChunk = 128;            // k advanced per iteration
constexpr int kPitch = kChunk + 4;     // LDS row pitch in elements (keeps 8-byte alignment, spreads banks)
constexpr int kWavesM = 4;             // wavefronts (32 rows each) per workgroup
constexpr int kRowsPerWg = kWavesM * 32;

struct Pack4 { uint32_t lo, hi; };      // four 16-bit operands of one MFMA lane

// four consecutive codes (16 bits, lowest k in bits 3:0) -> four fp16 values
__device__ __forceinline__ Pack4 expand4(uint32_t h, __half)
{
    const uint32_t t = h ^ 0x8888u;     // code + 8 as an unsigned nibble
    Pack4 r;
    // fp16 0x6400 = 1024: OR-ing a nibble into the mantissa gives 1024 + u exactly
    r.lo = ((t | (t << 12)) & 0x000f000fu) | 0x64006400u;
    r.hi = (((t >> 8) | (t << 4)) & 0x000f000fu) | 0x64006400u;
    const __half2 off = __halves2half2(__ushort_as_half(0xe408), __ushort_as_half(0xe408));  // -1032
    __half2 a = __hadd2(*(const __half2*)&r.lo, off);
    __half2 b = __hadd2(*(const __half2*)&r.hi, off);
    r.lo = *(const uint32_t*)&a;
    r.hi = *(const uint32_t*)&b;
    return r;
}

// ... -> four bf16 values (small integers: the top half of their fp32 form is exact)
__device__ __forceinline__ Pack4 expand4(uint32_t h, bf16_t)
{
    const int s = (int)(h << 16);
    const float f0 = (float)((s << 12) >> 28), f1 = (float)((s << 8) >> 28);
    const float f2 = (float)((s << 4) >> 28), f3 = (float)(s >> 28);
    Pack4 r;
    r.lo = (__float_as_uint(f0) >> 16) | (__float_as_uint(f1) & 0xffff0000u);
    r.hi = (__float_as_uint(f2) >> 16) | (__float_as_uint(f3) & 0xffff0000u);
    return r;
}

__device__ __forceinline__ float16v mfma(Pack4 a, Pack4 b, float16v c, __half)
{
    return __builtin_amdgcn_mfma_f32_32x32x8f16(*(const half4*)&a, *(const half4*)&b, c, 0, 0, 0);
}
__device__ __forceinline__ float16v mfma(Pack4 a, Pack4 b, float16v c, bf16_t)
{
    return __builtin_amdgcn_mfma_f32_32x32x8bf16_1k(*(const short4v*)&a, *(const short4v*)&b, c, 0, 0, 0);
}

// NT = 32-column halves per workgroup (1 for b <= 32); VEC = X rows are 16-byte aligned
template <typename XT, typename YT, int NT, bool VEC>
__global__ void __launch_bounds__(kWavesM * 64)
dequant_mfma_kernel(const uint8_t* __restrict__ codes, const __half* __restrict__ scales,
                    const XT* __restrict__ X, int64_t ldx, YT* __restrict__ Y, int64_t ldy,
                    int64_t m, int64_t k, int64_t b, int64_t nblocks, int chunks_per_block)
{
    constexpr int kCols = NT * 32;
    constexpr int kThreads = kWavesM * 64;
    constexpr int kStageElems = kCols * kChunk / kThreads;  // X elements a thread stages per chunk
    static_assert(kStageElems % 8 == 0, "whole 16-byte pieces per thread");
    __shared__ __align__(16) uint16_t xs[2][kCols * kPitch];

    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int li = lane & 31, kq = lane >> 5;
    const int64_t row_base = (int64_t)blockIdx.x * kRowsPerWg + wave * 32;
    const int64_t row = row_base + li;  // this lane's A row
    const int64_t col0 = (int64_t)blockIdx.y * kCols;
    const int64_t kbytes = k / 2;
    const bool row_ok = row < m;
    const uint8_t* crow = codes + (row_ok ? row : 0) * kbytes;

    // staging assignment: a thread owns kStageElems consecutive k of one column
    constexpr int kPartsPerCol = kChunk / kStageElems;
    const int sc = tid / kPartsPerCol, spart = tid % kPartsPerCol;
    const int64_t scol = col0 + sc;

    float16v total[NT], acc[NT];
#pragma unroll
    for (int nt = 0; nt < NT; ++nt)
#pragma unroll
        for (int v = 0; v < 16; ++v) { total[nt][v] = 0.0f; acc[nt][v] = 0.0f; }

    uint4 xreg[kStageElems / 8], creg[2];
    auto fetch = [&](int kc) {
        const int64_t k0 = (int64_t)kc * kChunk;
        const int64_t kk0 = k0 + spart * kStageElems;
#pragma unroll
        for (int e = 0; e < kStageElems / 8; ++e) {
            uint4 v = make_uint4(0, 0, 0, 0);
            const int64_t kk = kk0 + 8 * e;
            if (scol < b) {
                if (VEC && kk + 8 <= k) {
                    v = *(const uint4*)(X + scol * ldx + kk);
                } else {
                    uint16_t t[8];
#pragma unroll
                    for (int i = 0; i < 8; ++i) t[i] = (kk + i < k) ? *(const uint16_t*)(X + scol * ldx + kk + i) : (uint16_t)0;
                    v.x = t[0] | ((uint32_t)t[1] << 16); v.y = t[2] | ((uint32_t)t[3] << 16);
                    v.z = t[4] | ((uint32_t)t[5] << 16); v.w = t[6] | ((uint32_t)t[7] << 16);
                }
            }
            xreg[e] = v;
        }
        // this lane's 64 codes of the chunk: bytes [k0/2 + 32 kq, +32)
        const int64_t byte0 = k0 / 2 + 32 * kq;
        const uint4* src = (const uint4*)(crow + byte0);
        creg[0] = (row_ok && byte0 + 16 <= kbytes) ? src[0] : make_uint4(0, 0, 0, 0);
        creg[1] = (row_ok && byte0 + 32 <= kbytes) ? src[1] : make_uint4(0, 0, 0, 0);
    };
    auto stage = [&](int buf) {
#pragma unroll
        for (int e = 0; e < kStageElems / 8; ++e) {
            uint2* dst = (uint2*)&xs[buf][sc * kPitch + spart * kStageElems + 8 * e];  // 8-byte aligned (pitch)
            dst[0] = make_uint2(xreg[e].x, xreg[e].y);
            dst[1] = make_uint2(xreg[e].z, xreg[e].w);
        }
    };

    const int nchunks = (int)((k + kChunk - 1) / kChunk);
    fetch(0);
    stage(0);
    __syncthreads();
    for (int kc = 0; kc < nchunks; ++kc) {
        const int cur = kc & 1;
        uint32_t w[8] = {creg[0].x, creg[0].y, creg[0].z, creg[0].w, creg[1].x, creg[1].y, creg[1].z, creg[1].w};
        if (kc + 1 < nchunks) fetch(kc + 1);  // next chunk's X and codes travel during the MFMAs
#pragma unroll
        for (int s = 0; s < 16; ++s) {
            const Pack4 a = expand4((w[s >> 1] >> (16 * (s & 1))) & 0xffffu, XT{});
#pragma unroll
            for (int nt = 0; nt < NT; ++nt) {
                const Pack4 bv = *(const Pack4*)&xs[cur][(nt * 32 + li) * kPitch + 64 * kq + 4 * s];
                acc[nt] = mfma(a, bv, acc[nt], XT{});
            }
        }
        if (kc + 1 < nchunks) stage(cur ^ 1);
        __syncthreads();
        // ---- end of a scale block: total += q(row, block) * acc
        if ((kc + 1) % chunks_per_block == 0 || kc + 1 == nchunks) {
            const int64_t blk = kc / chunks_per_block;
#pragma unroll
            for (int v = 0; v < 16; ++v) {
                const int64_t r = row_base + 8 * (v / 4) + 4 * kq + (v % 4);
                float q = 1.0f;
                if (scales && r < m) q = __half2float(scales[r * nblocks + blk]);
#pragma unroll
                for (int nt = 0; nt < NT; ++nt) {
                    total[nt][v] = fmaf(q, acc[nt][v], total[nt][v]);
                    acc[nt][v] = 0.0f;
                }
            }
        }
    }
#pragma unroll
    for (int nt = 0; nt < NT; ++nt)
#pragma unroll
        for (int v = 0; v < 16; ++v) {
            const int64_t r = row_base + 8 * (v / 4) + 4 * kq + (v % 4);
            const int64_t c = col0 + nt * 32 + li;
            if (r < m && c < b) Y[c * ldy + r] = to_output<YT, float>(total[nt][v]);
        }
}

template <typename XT, typename YT>
void launch_typed(const Plan& p, const void* X, int64_t ldx, void* Y, int64_t ldy, int chunks_per_block,
                  hipStream_t s)
{
    const bool vec = (ldx % 8 == 0) && (((uintptr_t)X & 15) == 0);
    const int nt = p.b <= 32 ? 1 : 2;
    dim3 grid((unsigned)((p.m + kRowsPerWg - 1) / kRowsPerWg), (unsigned)((p.b + nt * 32 - 1) / (nt * 32)));
    const __half* sc = (const __half*)p.scales;
#define MSGEMM_MFMA_LAUNCH(NTV, VECV)                                                                     \
    hipLaunchKernelGGL((dequant_mfma_kernel<XT, YT, NTV, VECV>), grid, dim3(kWavesM * 64), 0, s, p.codes, \
                       sc, (const XT*)X, ldx, (YT*)Y, ldy, p.m, p.k, p.b, p.nblocks, chunks_per_block)
    if (nt == 1 && vec) MSGEMM_MFMA_LAUNCH(1, true);
    else if (nt == 1) MSGEMM_MFMA_LAUNCH(1, false);
    else if (vec) MSGEMM_MFMA_LAUNCH(2, true);
    else MSGEMM_MFMA_LAUNCH(2, false);
#undef MSGEMM_MFMA_LAUNCH
}

}  // namespace

int launch_dequant_mfma(const Plan& p, const void* X, int64_t ldx, void* Y, int64_t ldy, hipStream_t s)
{
    if (p.x_dtype != MSGEMM_F16 && p.x_dtype != MSGEMM_BF16) return MSGEMM_ERR_UNSUPPORTED;
    // 16-byte code loads per row segment and whole 128-column chunks per scale block
    if (p.k % 64 != 0) return MSGEMM_ERR_UNSUPPORTED;
    if (p.scale_group > 0 && p.scale_group % kChunk != 0) return MSGEMM_ERR_UNSUPPORTED;
    const int chunks_per_block = p.scale_group > 0 ? p.scale_group / kChunk : (int)((p.k + kChunk - 1) / kChunk);
    if (p.x_dtype == MSGEMM_F16) launch_typed<__half, __half>(p, X, ldx, Y, ldy, chunks_per_block, s);
    else launch_typed<bf16_t, bf16_t>(p, X, ldx, Y, ldy, chunks_per_block, s);
    MSGEMM_HIP_TRY(hipGetLastError());
    return MSGEMM_OK;
}

}  // namespace msgemm
