// Fused msGeMM with tables of depth d = 3 in LDS (single column, b <= 2; no scale blocks).
//
// Section 5 of the paper finds d = 3 the best depth by operation count: a third fewer look-ups than
// d = 2 at sixteen times the entries per group.  This kernel is the measured point behind the
// choice of depth on this device: a group's table has 16^3 entries of 4 bytes = 16 KiB, so LDS
// holds the tables of 8 groups (24 columns of k) where it holds 64 groups (128 columns) at d = 2.
// With half tables (Section 4.1: only the combinations whose last code has its top bit clear are
// kept, the others follow from L(~idx, j) = c S(j) - L(idx, j), c = value(i) + value(~i), S(j) the
// sum of the group's activations) a group takes 8 KiB and a k-tile holds 16 groups (48 columns).
//
// Work decomposition
//   A k-tile is kGroups consecutive groups; a workgroup of 8 wavefronts runs through a segment of
//   consecutive k-tiles for its rows: build the k-tile's tables (all wavefronts), meet, gather,
//   meet.  A lane owns one row of each of its wavefront's sub-panels of 64 rows; its sums stay in
//   registers over the segment.  One partial sum per (segment, row) leaves the workgroup; a second
//   launch adds the segments (a single segment writes Y itself).
//
// Codes
//   The plan stores, per (k-tile, row, run of 8 groups), the row's 96 code bits rotated by 12 bits
//   per lane (lane l gets them rotated right by 12 (l % 8)): the index a lane extracts at position s
//   belongs to group (s + l) % 8, so the 64 lanes of a look-up spread over the groups.  An entry
//   (idx, g) sits at word idx * kGroups + g: which bank a look-up hits depends on the low bits of
//   idx as well as on the group -- with 8 or 16 groups resident the gather cannot be made free of
//   bank conflicts the way the d = 2 layout (64 groups, bank = group) is.
//
// The index of a group is sum_r code_r << 4r (first code least significant); codes and activations
// past the end of k read as zero, which makes a short last group index the entry it needs.
#include <type_traits>

#include "device_types.h"
#include "fused_common.h"
#include "msgemm_internal.h"

namespace msgemm {
namespace {

constexpr int kD3Waves = 8;

struct Depth3Args {
    const uint32_t* codes3;  // [k-tile][run][row (m_pad)][3] words, rotated per lane
    const void* X;
    int64_t ldx;
    void* Y;
    int64_t ldy;
    float* partials;         // [segment][column][m_pad]
    int64_t m, k, m_pad;
    int b, ktiles, segments, tiles_per_segment, row_blocks, subpanels;  // subpanels of 64 rows per wavefront
    float half_c;            // value(i) + value(~i) (half tables)
};

__device__ __forceinline__ float d3_mul_add(float w, float x, float acc) { return fmaf(w, x, acc); }
__device__ __forceinline__ int d3_mul_add(int w, int x, int acc) { return w * x + acc; }

// index at position s (0..7) of the 96 bits (w0, w1, w2)
template <int S> __device__ __forceinline__ uint32_t index12(uint32_t w0, uint32_t w1, uint32_t w2)
{
    constexpr int bit = 12 * S;
    if constexpr (bit + 12 <= 32) return (w0 >> bit) & 0xfffu;
    else if constexpr (bit < 32) return __builtin_amdgcn_alignbit(w1, w0, bit) & 0xfffu;
    else if constexpr (bit + 12 <= 64) return (w1 >> (bit - 32)) & 0xfffu;
    else if constexpr (bit < 64) return __builtin_amdgcn_alignbit(w2, w1, bit - 32) & 0xfffu;
    else return (w2 >> (bit - 64)) & 0xfffu;
}

template <typename XT, typename YT, typename ET, bool kHalf, int kSub>
__global__ void __launch_bounds__(kD3Waves * 64)
depth3_kernel(Depth3Args a)
{
    using AT = ET;
    constexpr int kGroups = kHalf ? 16 : 8;   // groups of a k-tile
    constexpr int kRuns = kGroups / 8;        // runs of 8 groups = 12 code bytes per row
    constexpr int kEntries = kHalf ? 2048 : 4096;
    __shared__ __align__(16) ET table[kEntries * kGroups];
    __shared__ AT group_sum[16];              // S(j) of the k-tile's groups (half tables)

    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int rb = blockIdx.x / a.segments, seg = blockIdx.x % a.segments;
    const int cp = blockIdx.y;  // column
    const int kt_begin = seg * a.tiles_per_segment;
    const int kt_end = min(kt_begin + a.tiles_per_segment, a.ktiles);
    const XT* __restrict__ X = (const XT*)a.X + (int64_t)cp * a.ldx;
    const int64_t row_first = ((int64_t)rb * kD3Waves + wave) * (kSub * 64) + lane;  // this lane's row of sub-panel 0

    // ---- table build: thread (g, t) makes the entries (i0 = 0..15, i1 in its four, i2 = t / 4) of group g
    const int bg = tid & (kGroups - 1), bt = tid / kGroups;
    const int bi2 = bt >> 2, bi1_first = (bt & 3) * 4;
    auto x_of = [&](int kt, int r) -> XT {
        const int64_t kk = ((int64_t)kt * kGroups + bg) * 3 + r;
        XT zero{};
        return kk < a.k ? X[kk] : zero;
    };
    auto build = [&](XT r0, XT r1, XT r2) {
        const AT x0 = (AT)XTraits<XT>::load(&r0), x1 = (AT)XTraits<XT>::load(&r1), x2 = (AT)XTraits<XT>::load(&r2);
        if (kHalf && bt == 0) group_sum[bg] = x0 + x1 + x2;
        const AT top = (AT)decode4((unsigned)bi2) * x2;
#pragma unroll
        for (int u = 0; u < 4; ++u) {
            const int i1 = bi1_first + u;
            const AT hi = d3_mul_add((AT)decode4((unsigned)i1), x1, top);
#pragma unroll
            for (int v = 0; v < 16; ++v) {
                const int i0 = (v + bt) & 15;  // (threads that write together differ in the low index bits: banks spread)
                const int idx = i0 | (i1 << 4) | (bi2 << 8);
                table[idx * kGroups + bg] = d3_mul_add((AT)decode4((unsigned)i0), x0, hi);
            }
        }
    };

    // ---- this lane's codes of a k-tile: kSub sub-panels x kRuns runs x 3 words
    auto load_codes3 = [&](int kt, uint32_t (&w)[kSub][kRuns][3]) {
#pragma unroll
        for (int sp = 0; sp < kSub; ++sp)
#pragma unroll
            for (int r = 0; r < kRuns; ++r) {
                const uint32_t* p = a.codes3 + (((int64_t)kt * kRuns + r) * a.m_pad + row_first + sp * 64) * 3;
                w[sp][r][0] = load_codes(p);
                w[sp][r][1] = load_codes(p + 1);
                w[sp][r][2] = load_codes(p + 2);
            }
    };

    AT acc[kSub], neg_sums[kSub];
#pragma unroll
    for (int sp = 0; sp < kSub; ++sp) {
        acc[sp] = 0;
        neg_sums[sp] = 0;
    }
    uint32_t cur[kSub][kRuns][3], nxt[kSub][kRuns][3];
    XT xr0 = x_of(kt_begin, 0), xr1 = x_of(kt_begin, 1), xr2 = x_of(kt_begin, 2);
    load_codes3(kt_begin, cur);

    for (int kt = kt_begin; kt < kt_end; ++kt) {
        const bool more = kt + 1 < kt_end;
        __syncthreads();  // every wavefront is done with the old tables
        build(xr0, xr1, xr2);
        if (more) {
            xr0 = x_of(kt + 1, 0); xr1 = x_of(kt + 1, 1); xr2 = x_of(kt + 1, 2);
            load_codes3(kt + 1, nxt);
        }
        __syncthreads();
#pragma unroll
        for (int r = 0; r < kRuns; ++r) {
            // the group behind position s of this lane: 8 r + (s + lane) % 8
            auto gather = [&](auto S) {
                constexpr int s = decltype(S)::value;
                const int g = 8 * r + ((s + lane) & 7);
#pragma unroll
                for (int sp = 0; sp < kSub; ++sp) {
                    const uint32_t idx = index12<s>(cur[sp][r][0], cur[sp][r][1], cur[sp][r][2]);
                    if constexpr (kHalf) {
                        // top bit of the last code set: the entry of the complemented index, negated, and c S(j)
                        const bool flip = (idx & 0x800u) != 0;
                        const uint32_t kept = flip ? (~idx & 0x7ffu) : idx;
                        const AT e = table[kept * kGroups + g];
                        acc[sp] += flip ? -e : e;
                        neg_sums[sp] += flip ? group_sum[g] : (AT)0;
                    } else {
                        acc[sp] += table[idx * kGroups + g];
                    }
                }
            };
            gather(std::integral_constant<int, 0>()); gather(std::integral_constant<int, 1>());
            gather(std::integral_constant<int, 2>()); gather(std::integral_constant<int, 3>());
            gather(std::integral_constant<int, 4>()); gather(std::integral_constant<int, 5>());
            gather(std::integral_constant<int, 6>()); gather(std::integral_constant<int, 7>());
        }
        if (more) {
#pragma unroll
            for (int sp = 0; sp < kSub; ++sp)
#pragma unroll
                for (int r = 0; r < kRuns; ++r)
#pragma unroll
                    for (int i = 0; i < 3; ++i) cur[sp][r][i] = nxt[sp][r][i];
        }
    }

    // ---- one sum per (segment, row): Y, or a partial
    YT* __restrict__ Y = (YT*)a.Y;
#pragma unroll
    for (int sp = 0; sp < kSub; ++sp) {
        AT total = acc[sp];
        if constexpr (kHalf) {
            if constexpr (std::is_same<AT, float>::value) total = fmaf(a.half_c, neg_sums[sp], total);
            else total += (AT)a.half_c * neg_sums[sp];
        }
        const int64_t row = row_first + sp * 64;
        if (a.segments == 1) {
            if (row < a.m) Y[(int64_t)cp * a.ldy + row] = to_output<YT, AT>(total);
        } else {
            unsigned bits = bits_of(total);
            ((unsigned*)a.partials)[((int64_t)seg * a.b + cp) * a.m_pad + row] = bits;
        }
    }
}

// adds the segments in order and writes Y
template <typename YT, typename AT>
__global__ void __launch_bounds__(256)
depth3_reduce_kernel(const float* __restrict__ partials, YT* __restrict__ Y, int64_t ldy, int64_t m, int64_t m_pad, int b,
                     int segments)
{
    const int64_t row = (int64_t)blockIdx.x * 64 + threadIdx.x;  // one wavefront per workgroup: m / 64 workgroups
    const int cp = blockIdx.y;
    if (row >= m) return;
    AT sum = 0;
    const unsigned* src = (const unsigned*)partials + (int64_t)cp * m_pad + row;
    const int64_t step = (int64_t)b * m_pad;
    for (int s0 = 0; s0 < segments; s0 += 8) {  // eight loads in flight, added in segment order
        unsigned w[8];
#pragma unroll
        for (int i = 0; i < 8; ++i) w[i] = s0 + i < segments ? src[(s0 + i) * step] : 0u;
#pragma unroll
        for (int i = 0; i < 8; ++i) {
            AT x;
            set_bits(x, w[i]);
            sum += x;
        }
    }
    Y[(int64_t)cp * ldy + row] = to_output<YT, AT>(sum);
}

// [m][k/2] row-major code bytes -> [k-tile][run][row][3 words], each row's 96 bits of a run rotated right by
// 12 (row % 64 % 8) bits; rows past m and bytes past k/2 are zero.  kInverse: back to row-major.
template <bool kInverse>
__global__ void __launch_bounds__(256)
repack3_kernel(uint8_t* __restrict__ codes, uint32_t* __restrict__ out, int64_t m, int64_t m_pad, int64_t kbytes,
               int64_t runs_total)
{
    const int64_t total = runs_total * m_pad;
    for (int64_t o = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; o < total; o += (int64_t)gridDim.x * blockDim.x) {
        const int64_t run = o / m_pad, row = o % m_pad;
        if constexpr (kInverse) {
            if (row >= m) continue;
            const uint32_t r[3] = {out[o * 3], out[o * 3 + 1], out[o * 3 + 2]};
            const int rot = 12 * (int)(row & 7);
            for (int bt = 0; bt < 12; ++bt) {
                const int64_t byte = run * 12 + bt;
                if (byte >= kbytes) break;
                uint32_t v = 0;
                for (int bit = 0; bit < 8; ++bit) {
                    // source bit j sits at result bit (j - rot) mod 96
                    const int dst = (bt * 8 + bit - rot + 96) % 96;
                    v |= ((r[dst >> 5] >> (dst & 31)) & 1u) << bit;
                }
                codes[row * kbytes + byte] = (uint8_t)v;
            }
            continue;
        }
        uint32_t w[3] = {0, 0, 0};
        if (row < m) {
            for (int bt = 0; bt < 12; ++bt) {
                const int64_t byte = run * 12 + bt;
                const uint32_t v = byte < kbytes ? codes[row * kbytes + byte] : 0u;
                w[bt >> 2] |= v << (8 * (bt & 3));
            }
        }
        // rotate the 96 bits right by 12 * (lane % 8): position s then holds group (s + lane) % 8
        const int rot = 12 * (int)(row & 7);
        uint32_t r[3];
        for (int i = 0; i < 3; ++i) {
            // bit j of the result = bit (j + rot) % 96 of the source
            uint32_t word = 0;
            for (int bit = 0; bit < 32; ++bit) {
                const int src = (i * 32 + bit + rot) % 96;
                word |= ((w[src >> 5] >> (src & 31)) & 1u) << bit;
            }
            r[i] = word;
        }
        out[o * 3 + 0] = r[0];
        out[o * 3 + 1] = r[1];
        out[o * 3 + 2] = r[2];
    }
}

}  // namespace

// Fills the plan for the depth-3 LDS kernel; MSGEMM_ERR_UNSUPPORTED where it does not apply.
int depth3_choose_shape(Plan& p)
{
    if (p.d != 3 || p.b > 2 || p.scale_group != 0 || p.codes8) return MSGEMM_ERR_UNSUPPORTED;
    hipDeviceProp_t prop;
    p.cus = 256;
    if (hipGetDeviceProperties(&prop, p.device) == hipSuccess && prop.multiProcessorCount > 0) p.cus = prop.multiProcessorCount;
    const bool half = p.opt.half_tables_in_lds != 0;
    const int groups = half ? 16 : 8;
    p.d3_half = half;
    p.d3_sub = p.m > 8 * 64 * 2 ? 4 : (p.m > 8 * 64 ? 2 : 1);   // sub-panels of 64 rows per wavefront
    const int64_t tile_rows = (int64_t)kD3Waves * 64 * p.d3_sub;
    p.row_blocks = (p.m + tile_rows - 1) / tile_rows;
    p.m_pad = p.row_blocks * tile_rows;
    p.ktiles = (p.lut_groups + groups - 1) / groups;
    // segments: enough workgroups for every compute unit, whole k-tiles each
    int64_t segs = (p.cus + p.row_blocks * p.b - 1) / (p.row_blocks * p.b);
    if (segs > p.ktiles) segs = p.ktiles;
    if (segs < 1) segs = 1;
    if (p.opt.batched_segments >= 1 && p.opt.batched_segments <= p.ktiles) segs = p.opt.batched_segments;
    p.tiles_per_segment = (int)((p.ktiles + segs - 1) / segs);
    p.segments = (int)((p.ktiles + p.tiles_per_segment - 1) / p.tiles_per_segment);
    if (p.ktiles * (groups / 8) * p.m_pad * 3 >= ((int64_t)1 << 40)) return MSGEMM_ERR_UNSUPPORTED;
    p.fs = FusedShape{};
    p.fs.groups = groups;
    p.fs.cols = 1;
    p.fs.entry_bytes = 4;
    p.fs.waves = kD3Waves;
    p.fs.panels = 1;
    p.fs.panel_rows = (int)tile_rows;
    p.fs.tile_rows = (int)tile_rows;
    p.col_passes = (int)p.b;
    return MSGEMM_OK;
}

int launch_repack3(const Plan& p, uint8_t* row_major, bool inverse, hipStream_t s)
{
    const int64_t runs = p.ktiles * (p.fs.groups / 8);
    int64_t blocks = (runs * p.m_pad + 255) / 256;
    if (blocks > 65536) blocks = 65536;
    if (inverse)
        hipLaunchKernelGGL(repack3_kernel<true>, dim3((unsigned)blocks), dim3(256), 0, s, row_major, (uint32_t*)p.codes_tiled,
                           p.m, p.m_pad, p.k / 2, runs);
    else
        hipLaunchKernelGGL(repack3_kernel<false>, dim3((unsigned)blocks), dim3(256), 0, s, row_major, (uint32_t*)p.codes_tiled,
                           p.m, p.m_pad, p.k / 2, runs);
    MSGEMM_HIP_TRY(hipGetLastError());
    return MSGEMM_OK;
}

template <typename XT, typename YT, typename ET>
static int launch_depth3_typed(const Plan& p, Depth3Args& a, hipStream_t s)
{
    const dim3 grid((unsigned)(p.row_blocks * p.segments), (unsigned)p.b), blk(kD3Waves * 64);
#define MSGEMM_D3(HALF, SUB) hipLaunchKernelGGL((depth3_kernel<XT, YT, ET, HALF, SUB>), grid, blk, 0, s, a)
    if (p.d3_half) {
        if (p.d3_sub == 4) MSGEMM_D3(true, 4); else if (p.d3_sub == 2) MSGEMM_D3(true, 2); else MSGEMM_D3(true, 1);
    } else {
        if (p.d3_sub == 4) MSGEMM_D3(false, 4); else if (p.d3_sub == 2) MSGEMM_D3(false, 2); else MSGEMM_D3(false, 1);
    }
#undef MSGEMM_D3
    MSGEMM_HIP_TRY(hipGetLastError());
    if (p.segments > 1) {
        hipLaunchKernelGGL((depth3_reduce_kernel<YT, ET>), dim3((unsigned)((p.m + 63) / 64), (unsigned)p.b), dim3(64), 0, s,
                           a.partials, (YT*)a.Y, a.ldy, a.m, a.m_pad, a.b, a.segments);
        MSGEMM_HIP_TRY(hipGetLastError());
    }
    return MSGEMM_OK;
}

int launch_depth3(const Plan& p, const void* X, int64_t ldx, void* Y, int64_t ldy, hipStream_t s)
{
    Depth3Args a;
    a.codes3 = (const uint32_t*)p.codes_tiled;
    a.X = X; a.ldx = ldx; a.Y = Y; a.ldy = ldy;
    a.partials = p.partials;
    a.m = p.m; a.k = p.k; a.m_pad = p.m_pad;
    a.b = (int)p.b; a.ktiles = (int)p.ktiles; a.segments = p.segments; a.tiles_per_segment = p.tiles_per_segment;
    a.row_blocks = (int)p.row_blocks; a.subpanels = p.d3_sub;
    a.half_c = p.half_c;
    switch (p.x_dtype) {
    case MSGEMM_F32: return launch_depth3_typed<float, float, float>(p, a, s);
    case MSGEMM_F16: return launch_depth3_typed<__half, __half, float>(p, a, s);
    case MSGEMM_BF16: return launch_depth3_typed<bf16_t, bf16_t, float>(p, a, s);
    case MSGEMM_I8: return launch_depth3_typed<int8_t, int, int>(p, a, s);
    default: return MSGEMM_ERR_INVALID_ARG;
    }
}

}  // namespace msgemm
