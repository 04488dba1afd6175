// Two-launch msGeMM: the table L lives in device memory and is shared by all
// rows (Section 4: the table of phase 1 stays in cache for phase 2).  Works for
// every d in 1..4, every dtype pair and every scale block size.
//
// Two consumers.  The plain one takes one thread per output and reads the
// row-major codes nibble by nibble: any shape.  The tiled one needs scale blocks
// that are whole 32-bit words of codes (block % 8 == 0) and a plan of this
// variant (it reads a transposed copy of the codes made at plan time):
//   * codes as [64-row tile][word of the row][lane]: the w-th words of 64 rows
//     are one contiguous 256-byte load;
//   * a thread owns one row and walks its code words three at a time (96 bits =
//     24 nibbles hold a whole number of groups for every d), pulling the 4d-bit
//     indices out with shifts whose amounts are compile-time constants;
//   * the k dimension is cut into chunks of groups whose tables are about one
//     MiB; a segment is a run of chunks, and the workgroups of one segment run
//     on one XCD (ids congruent modulo 8), so the tables a workgroup gathers
//     from are in that XCD's L2 after the first touch;
//   * per-segment partial sums, then a reduction in segment order.
#include "device_types.h"
#include "fused_common.h"
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

// Phase 1 (Section 3.1).  A workgroup writes kBuildPerWg consecutive entries of
// one group: [code combination][column], the column fastest.
constexpr int kBuildThreads = 256;
constexpr int kBuildItems = 8;
constexpr int kBuildPerWg = kBuildThreads * kBuildItems;

template <typename XT, typename LT>
__global__ void __launch_bounds__(kBuildThreads)
build_lut_kernel(GroupGeom g, int parts, int b, int half, const XT* __restrict__ X, int64_t ldx,
                 ValueMap values, LT* __restrict__ L)
{
    const int64_t jg = blockIdx.x / (unsigned)parts;
    const int part = (int)(blockIdx.x - (unsigned)jg * (unsigned)parts);
    // half tables: the combinations with the top bit of the last code clear are the first half of the index range
    const unsigned per_group = ((1u << (4 * g.d)) >> half) * (unsigned)b;
    int64_t first;
    int len;
    group_span(g, jg, first, len);
    LT* Lg = L + jg * (int64_t)per_group;
#pragma unroll
    for (int i = 0; i < kBuildItems; ++i) {
        const unsigned t = (unsigned)part * kBuildPerWg + (unsigned)i * kBuildThreads + threadIdx.x;
        if (t >= per_group) break;
        const unsigned idx = b == 1 ? t : t / (unsigned)b;
        const unsigned c = b == 1 ? 0u : t - idx * (unsigned)b;
        const XT* xc = X + (int64_t)c * ldx + first;
        LT s = 0;
        for (int r = 0; r < len; ++r)
            s += code_value(values, (idx >> (4 * r)) & 15u, LT()) * (LT)XTraits<XT>::load(xc + r);
        Lg[t] = s;
    }
}

// Phase 1 on the matrix cores, for batches.  The table of a group is the product
// of the [16^d x d] matrix of code values with the group's [d x b] activations
// (Section 6 points out that phase 1 can use the matrix units).  One
// v_mfma_f32_16x16x4_f32 makes 16 combinations x 16 columns: operand A holds, for
// lane l, the value of nibble l / 16 of combination 16 rt + l % 16 (zero for
// positions the group does not have), operand B the activation X(first + l / 16,
// column l % 16); fp32 throughout, so an entry is the same sum of d products as in
// build_lut_kernel.  A wavefront owns one tile of 16 columns of one group and
// walks down the combinations; the four wavefronts of a workgroup take
// neighbouring column tiles, so a row of the table is written by one workgroup.
typedef float f4_t __attribute__((ext_vector_type(4)));
constexpr unsigned kBuildTilesPerWg = 16;

template <typename XT>
__global__ void __launch_bounds__(256)
build_lut_mfma_kernel(GroupGeom g, unsigned chunks, int col_tiles, int b, int half, const XT* __restrict__ X, int64_t ldx,
                      ValueMap values, float* __restrict__ L)
{
    const int64_t jg = blockIdx.x / chunks;
    const unsigned chunk = blockIdx.x % chunks;
    const int ct = (int)blockIdx.y * 4 + (int)(threadIdx.x >> 6);
    if (ct >= col_tiles) return;
    const int lane = threadIdx.x & 63;
    const int i = lane & 15, kq = lane >> 4;
    int64_t first;
    int len;
    group_span(g, jg, first, len);
    const int col = ct * 16 + i;
    const float bval = (kq < len && col < b) ? (float)XTraits<XT>::load(X + (int64_t)col * ldx + first + kq) : 0.0f;
    const float vals = values.v[i];  // lane l keeps the value of pattern l % 16
    const float v_low = kq < len ? vals : 0.0f;  // nibble 0 of a combination is l % 16 itself
    const unsigned stored = (1u << (4 * g.d)) >> half;
    float* Lg = L + jg * (int64_t)stored * b;
    // A workgroup makes kBuildTilesPerWg tiles of 16 combinations, so that the
    // workgroups running at any moment write one compact stretch of the table.
    const unsigned tiles = (stored + 15) / 16;
    const unsigned rt0 = chunk * kBuildTilesPerWg;
    const unsigned rt1 = rt0 + kBuildTilesPerWg < tiles ? rt0 + kBuildTilesPerWg : tiles;
    for (unsigned rt = rt0; rt < rt1; ++rt) {
        // nibbles 1..3 of the combinations of this tile are the same for all 16 of them
        const float u1 = __builtin_bit_cast(float, __builtin_amdgcn_readlane(__builtin_bit_cast(int, vals), (int)(rt & 15)));
        const float u2 = __builtin_bit_cast(float, __builtin_amdgcn_readlane(__builtin_bit_cast(int, vals), (int)((rt >> 4) & 15)));
        const float u3 = __builtin_bit_cast(float, __builtin_amdgcn_readlane(__builtin_bit_cast(int, vals), (int)((rt >> 8) & 15)));
        float aval = kq == 0 ? v_low : (kq == 1 ? u1 : (kq == 2 ? u2 : u3));
        if (kq >= len) aval = 0.0f;
        f4_t acc = {0.0f, 0.0f, 0.0f, 0.0f};
        acc = __builtin_amdgcn_mfma_f32_16x16x4f32(aval, bval, acc, 0, 0, 0);
#pragma unroll
        for (int v = 0; v < 4; ++v) {
            const unsigned row = rt * 16 + 4 * kq + v;  // register v of lane l: combination 4 (l / 16) + v of the tile, column l % 16
            if (row < stored && col < b) Lg[(int64_t)row * b + col] = acc[v];
        }
    }
}

// S(j, c): the sum of a group's activations (half tables: L(~idx) = c * S - L(idx), Section 4.1)
template <typename XT, typename LT>
__global__ void __launch_bounds__(256)
group_sums_kernel(GroupGeom g, int64_t groups, int b, const XT* __restrict__ X, int64_t ldx, LT* __restrict__ S)
{
    const int64_t t = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (t >= groups * b) return;
    const int64_t jg = t / b;
    const int c = (int)(t - jg * b);
    int64_t first;
    int len;
    group_span(g, jg, first, len);
    LT sum = 0;
    for (int r = 0; r < len; ++r) sum += (LT)XTraits<XT>::load(X + (int64_t)c * ldx + first + r);
    S[t] = sum;
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
consume_lut_kernel(GroupGeom g, int64_t m, int64_t b, int64_t nblocks, int half, LT half_c,
                   const uint8_t* __restrict__ codes, const __half* __restrict__ scales,
                   const LT* __restrict__ L, const LT* __restrict__ S, YT* __restrict__ Y, int64_t ldy)
{
    const int64_t E = (int64_t)1 << (4 * g.d);
    const int64_t stored = E >> half;  // entries per group in memory
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
                if (half && idx >= stored) {  // the stored entry is that of the complemented codes
                    idx = ~idx & (E - 1);
                    s += half_c * S[jg * b + c] - L[(jg * stored + idx) * b + c];
                } else {
                    s += L[(jg * stored + idx) * b + c];
                }
            }
            y = add_block(scales, i * nblocks + blk, s, y);
        }
        Y[c * ldy + i] = to_output<YT, LT>(y);
    }
}

// ---------------------------------------------------------------------------
// tiled consumer

constexpr int kUnitWords = 3;       // code words a thread takes per step: 24 nibbles
constexpr int kTiledThreads = 256;  // one row per thread

struct TiledGeom {
    int d;
    int block_words;      // code words per scale block and row
    int row_words;        // code words per row
    int gpb;              // groups per block
    int units_per_block;  // ceil(block_words / kUnitWords)
    int chunk_units;      // units per chunk
    int chunks_per_block;
    int chunks;           // nblocks * chunks_per_block
    int chunks_per_segment;
    int segments;
    int row_tiles;        // 64-row tiles that hold rows
    int wg_rows;          // workgroups along m
    int col_passes;
    int xcd_map;          // 1: segment = id % 8 + 8 * ...
};

// Transposed copy of the codes: T[tile][word][lane] = word `word` of row tile*64+lane (zero beyond m, k).
__global__ void __launch_bounds__(256)
transpose_codes_kernel(const uint8_t* __restrict__ codes, uint32_t* __restrict__ T, int64_t m, int64_t row_bytes,
                       int row_words, int64_t total)
{
    for (int64_t t = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; t < total; t += (int64_t)gridDim.x * blockDim.x) {
        const int lane = (int)(t & 63);
        const int64_t rest = t >> 6;
        const int w = (int)(rest % row_words);
        const int64_t row = (rest / row_words) * 64 + lane;
        uint32_t v = 0;
        if (row < m) {
            for (int i = 0; i < 4; ++i) {
                const int64_t at = (int64_t)w * 4 + i;
                if (at < row_bytes) v |= (uint32_t)codes[row * row_bytes + at] << (8 * i);
            }
        }
        T[t] = v;
    }
}

template <typename T> __device__ __forceinline__ T bits_to(unsigned u);
template <> __device__ __forceinline__ float bits_to<float>(unsigned u) { return __uint_as_float(u); }
template <> __device__ __forceinline__ int bits_to<int>(unsigned u) { return (int)u; }

// the 4*D-bit field number f of a 96-bit window (f is a constant once the caller's loop is unrolled)
template <int D>
__device__ __forceinline__ unsigned window_field(const uint32_t (&w)[kUnitWords], int f)
{
    constexpr int kBits = 4 * D;
    constexpr unsigned mask = (1u << kBits) - 1u;
    const int at = kBits * f;
    const int word = at >> 5, shift = at & 31;
    unsigned v = w[word] >> shift;
    if (shift + kBits > 32) v |= w[word + 1 < kUnitWords ? word + 1 : word] << ((32 - shift) & 31);
    return v & mask;
}

// kVec (CB = 4 only): the four columns of a pass are one aligned 16-byte load.
// kHalf: half tables (see build_lut_kernel): a look-up whose index has its top
// bit set reads the entry of the complemented index and takes c * S - entry.
template <int D, typename LT, typename YT, int CB, bool kVec, bool kHalf>
__global__ void __launch_bounds__(kTiledThreads)
consume_tiled_kernel(TiledGeom g, int64_t m, int b, int64_t nblocks, const uint32_t* __restrict__ T,
                     const __half* __restrict__ scales, const LT* __restrict__ L, const LT* __restrict__ S, LT half_c,
                     LT* __restrict__ partials, YT* __restrict__ Y, int64_t ldy)
{
    constexpr int kFields = 24 / D;  // groups per unit
    constexpr unsigned kAll = 1u << (4 * D);   // index range
    constexpr unsigned E = kHalf ? kAll / 2 : kAll;  // entries per group in memory
    // which (segment, column pass, rows) this workgroup takes
    int seg, rest;
    const int per_seg = g.wg_rows * g.col_passes;
    if (g.xcd_map) {
        const int x = blockIdx.x % kXcds, j = blockIdx.x / kXcds;
        seg = x + kXcds * (j / per_seg);
        rest = j % per_seg;
    } else {
        seg = blockIdx.x / per_seg;
        rest = blockIdx.x % per_seg;
    }
    const int cp = rest / g.wg_rows;
    const int wr = rest - cp * g.wg_rows;
    const int tile = wr * (kTiledThreads / 64) + (int)(threadIdx.x >> 6);
    if (tile >= g.row_tiles) return;  // whole wavefront beyond m
    const int lane = threadIdx.x & 63;
    const int64_t row = (int64_t)tile * 64 + lane;
    const bool live = row < m;
    const int c0 = cp * CB;
    const uint32_t* Trow = T + (int64_t)tile * g.row_words * 64 + lane;

    LT y[CB];
#pragma unroll
    for (int c = 0; c < CB; ++c) y[c] = 0;

    const int q_begin = seg * g.chunks_per_segment;
    const int q_end = min(g.chunks, q_begin + g.chunks_per_segment);
    for (int q = q_begin; q < q_end; ++q) {
        const int blk = q / g.chunks_per_block;
        const int u_begin = (q - blk * g.chunks_per_block) * g.chunk_units;
        const int u_end = min(g.units_per_block, u_begin + g.chunk_units);
        const uint32_t* Tblk = Trow + (int64_t)blk * g.block_words * 64;
        // words past the end of the block read as zero: a short last group then
        // indexes its table with zeros in the positions it does not have
        auto load_unit = [&](int u, uint32_t (&w)[kUnitWords]) {
#pragma unroll
            for (int i = 0; i < kUnitWords; ++i) {
                const int at = u * kUnitWords + i;
                const uint32_t v = Tblk[(int64_t)min(at, g.block_words - 1) * 64];
                w[i] = at < g.block_words ? v : 0u;
            }
        };
        LT s[CB];
#pragma unroll
        for (int c = 0; c < CB; ++c) s[c] = 0;
        uint32_t cur[kUnitWords], nxt[kUnitWords];
        load_unit(u_begin, cur);
        for (int u = u_begin; u < u_end; ++u) {
            if (u + 1 < u_end) load_unit(u + 1, nxt);
            const int t0 = u * kFields;
            const LT* Lu = L + ((int64_t)blk * g.gpb + t0) * (int64_t)E * b + c0;
            const LT* Su = S + ((int64_t)blk * g.gpb + t0) * (int64_t)b + c0;  // group sums (half tables only)
            if (t0 + kFields <= g.gpb) {
                // a whole unit: every look-up is requested before the first is added
                LT got[kFields][CB];
                unsigned flipped = 0;  // bit f: look-up f read the complemented entry
#pragma unroll
                for (int f = 0; f < kFields; ++f) {
                    unsigned idx = window_field<D>(cur, f);
                    if constexpr (kHalf) {
                        const unsigned top = idx >> (4 * D - 1);
                        idx ^= (0u - top) & (kAll - 1u);
                        flipped |= top << f;  // per lane
                    }
                    const LT* e = Lu + (int64_t)f * E * b + (int64_t)idx * b;
                    if constexpr (kVec) {
                        const v4u raw = *(const v4u*)e;
#pragma unroll
                        for (int c = 0; c < CB; ++c) got[f][c] = bits_to<LT>(raw[c]);
                    } else {
#pragma unroll
                        for (int c = 0; c < CB; ++c) got[f][c] = (c0 + c < b) ? e[c] : (LT)0;
                    }
                }
#pragma unroll
                for (int f = 0; f < kFields; ++f) {
#pragma unroll
                    for (int c = 0; c < CB; ++c) {
                        if constexpr (kHalf) {
                            const LT sj = (c0 + c < b) ? Su[(int64_t)f * b + c] : (LT)0;  // uniform
                            s[c] += ((flipped >> f) & 1u) ? half_c * sj - got[f][c] : got[f][c];
                        } else {
                            s[c] += got[f][c];
                        }
                    }
                }
            } else {
                // the last unit of a block: only the groups the block has
#pragma unroll
                for (int f = 0; f < kFields; ++f) {
                    if (t0 + f < g.gpb) {  // uniform
                        unsigned idx = window_field<D>(cur, f);
                        unsigned top = 0;
                        if constexpr (kHalf) {
                            top = idx >> (4 * D - 1);
                            idx ^= (0u - top) & (kAll - 1u);
                        }
                        const LT* e = Lu + (int64_t)f * E * b + (int64_t)idx * b;
#pragma unroll
                        for (int c = 0; c < CB; ++c) {
                            if (c0 + c >= b) continue;
                            if constexpr (kHalf) s[c] += top ? half_c * Su[(int64_t)f * b + c] - e[c] : e[c];
                            else s[c] += e[c];
                        }
                    }
                }
            }
#pragma unroll
            for (int i = 0; i < kUnitWords; ++i) cur[i] = nxt[i];
        }
        const int64_t at = live ? row * nblocks + blk : 0;
#pragma unroll
        for (int c = 0; c < CB; ++c) y[c] = add_block(scales, at, s[c], y[c]);
    }
    if (!live) return;
#pragma unroll
    for (int c = 0; c < CB; ++c) {
        if (c0 + c >= b) break;
        if (g.segments == 1) Y[(int64_t)(c0 + c) * ldy + row] = to_output<YT, LT>(y[c]);
        else partials[((int64_t)seg * b + c0 + c) * m + row] = y[c];
    }
}

// Y(i, c) = sum over segments, in segment order
template <typename LT, typename YT>
__global__ void __launch_bounds__(256)
sum_segments_kernel(const LT* __restrict__ partials, YT* __restrict__ Y, int64_t ldy, int64_t m, int64_t b, int segments)
{
    const int64_t t = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (t >= m * b) return;
    const int64_t c = t / m, row = t - c * m;
    LT y = 0;
    for (int sgm = 0; sgm < segments; ++sgm) y += partials[((int64_t)sgm * b + c) * m + row];
    Y[c * ldy + row] = to_output<YT, LT>(y);
}

// where the group sums start in a half-table L (in table elements)
int64_t half_sums_offset(const Plan& p)
{
    return p.half_table ? p.lut_groups * (((int64_t)1 << (4 * p.d)) / 2) * p.b : 0;
}

bool tiled_applies(const Plan& p)
{
    return p.variant == MSGEMM_VARIANT_GLOBAL_LUT && p.codes_words && (p.block % 8) == 0 &&
           p.global_plain == 0;
}

TiledGeom tiled_geometry(const Plan& p, int cb)
{
    TiledGeom g{};
    g.d = p.d;
    g.block_words = (int)(p.block / 8);
    g.row_words = (int)(p.k / 8);
    g.gpb = (int)p.gpb;
    g.units_per_block = (g.block_words + kUnitWords - 1) / kUnitWords;
    // chunks of about one MiB of tables (plan option global_chunk_kib)
    const int64_t unit_bytes = (int64_t)(24 / p.d) * (((int64_t)1 << (4 * p.d)) >> (p.half_table ? 1 : 0)) * p.b * 4;
    const int64_t want = (int64_t)(p.global_chunk_kib > 0 ? p.global_chunk_kib : 1024) * 1024;
    int64_t cu = want / unit_bytes;
    if (cu < 1) cu = 1;
    if (cu > g.units_per_block) cu = g.units_per_block;
    g.chunk_units = (int)cu;
    g.chunks_per_block = (g.units_per_block + g.chunk_units - 1) / g.chunk_units;
    g.chunks = (int)(p.nblocks * g.chunks_per_block);
    g.row_tiles = (int)((p.m + 63) / 64);
    g.wg_rows = (g.row_tiles + kTiledThreads / 64 - 1) / (kTiledThreads / 64);
    g.col_passes = (int)((p.b + cb - 1) / cb);
    g.segments = p.global_segments;
    g.chunks_per_segment = (g.chunks + g.segments - 1) / g.segments;
    g.xcd_map = (g.segments % kXcds) == 0;
    return g;
}

template <int D, typename LT, typename YT>
int launch_tiled(const Plan& p, const void* L, void* Y, int64_t ldy, hipStream_t s)
{
    const int cb = p.b >= 4 ? 4 : (p.b >= 2 ? 2 : 1);
    const TiledGeom g = tiled_geometry(p, cb);
    const unsigned grid = (unsigned)g.segments * (unsigned)g.wg_rows * (unsigned)g.col_passes;
    const __half* sc = (const __half*)p.scales;
    const bool vec = cb == 4 && (p.b % 4) == 0 && ((uintptr_t)L & 15u) == 0;
    const LT* S = (const LT*)L + half_sums_offset(p);
    const LT half_c = (LT)p.half_c;
#define MSGEMM_TILED(CB, VEC, HALF)                                                                                  \
    hipLaunchKernelGGL((consume_tiled_kernel<D, LT, YT, CB, VEC, HALF>), dim3(grid), dim3(kTiledThreads), 0, s, g,    \
                       p.m, (int)p.b, p.nblocks, p.codes_words, sc, (const LT*)L, S, half_c, (LT*)p.global_partials, \
                       (YT*)Y, ldy)
#define MSGEMM_TILED_CB(HALF)                     \
    if (vec) MSGEMM_TILED(4, true, HALF);         \
    else if (cb == 4) MSGEMM_TILED(4, false, HALF); \
    else if (cb == 2) MSGEMM_TILED(2, false, HALF); \
    else MSGEMM_TILED(1, false, HALF)
    if (p.half_table) { MSGEMM_TILED_CB(true); } else { MSGEMM_TILED_CB(false); }
#undef MSGEMM_TILED_CB
#undef MSGEMM_TILED
    MSGEMM_HIP_TRY(hipGetLastError());
    if (g.segments > 1) {
        const int64_t total = p.m * p.b;
        hipLaunchKernelGGL((sum_segments_kernel<LT, YT>), dim3((unsigned)((total + 255) / 256)), dim3(256), 0, s,
                           (const LT*)p.global_partials, (YT*)Y, ldy, p.m, p.b, g.segments);
        MSGEMM_HIP_TRY(hipGetLastError());
    }
    return MSGEMM_OK;
}

template <typename LT, typename YT>
int launch_tiled_d(const Plan& p, const void* L, void* Y, int64_t ldy, hipStream_t s)
{
    switch (p.d) {
    case 1: return launch_tiled<1, LT, YT>(p, L, Y, ldy, s);
    case 2: return launch_tiled<2, LT, YT>(p, L, Y, ldy, s);
    case 3: return launch_tiled<3, LT, YT>(p, L, Y, ldy, s);
    case 4: return launch_tiled<4, LT, YT>(p, L, Y, ldy, s);
    }
    return MSGEMM_ERR_INVALID_ARG;
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
    const int half = p.half_table ? 1 : 0;
    const int64_t per_group = (((int64_t)1 << (4 * p.d)) >> half) * p.b;
    const int64_t parts = (per_group + kBuildPerWg - 1) / kBuildPerWg;
    if (per_group >= ((int64_t)1 << 31) || p.lut_groups * parts >= ((int64_t)1 << 31)) return MSGEMM_ERR_UNSUPPORTED;
    // batches of floating-point activations: the product on the matrix cores
    const int use_mfma = p.build_mfma;
    const unsigned tiles = (unsigned)((((int64_t)1 << (4 * p.d)) >> half) + 15) / 16;
    const unsigned chunks = (tiles + kBuildTilesPerWg - 1) / kBuildTilesPerWg;
    if (use_mfma && p.x_dtype != MSGEMM_I8 && p.lut_groups * chunks < ((int64_t)1 << 31)) {
        const int col_tiles = (int)((p.b + 15) / 16);
        dim3 mgrid((unsigned)(p.lut_groups * chunks), (unsigned)((col_tiles + 3) / 4)), mblk(256);
        if (p.x_dtype == MSGEMM_F32)
            hipLaunchKernelGGL((build_lut_mfma_kernel<float>), mgrid, mblk, 0, s, g, chunks, col_tiles, (int)p.b, half,
                               (const float*)X, ldx, vm, (float*)L);
        else if (p.x_dtype == MSGEMM_F16)
            hipLaunchKernelGGL((build_lut_mfma_kernel<__half>), mgrid, mblk, 0, s, g, chunks, col_tiles, (int)p.b, half,
                               (const __half*)X, ldx, vm, (float*)L);
        else
            hipLaunchKernelGGL((build_lut_mfma_kernel<bf16_t>), mgrid, mblk, 0, s, g, chunks, col_tiles, (int)p.b, half,
                               (const bf16_t*)X, ldx, vm, (float*)L);
        MSGEMM_HIP_TRY(hipGetLastError());
    } else {
    dim3 grid((unsigned)(p.lut_groups * parts)), blk(kBuildThreads);
    switch (p.x_dtype) {
    case MSGEMM_F32:
        hipLaunchKernelGGL((build_lut_kernel<float, float>), grid, blk, 0, s, g, (int)parts, (int)p.b, half,
                           (const float*)X, ldx, vm, (float*)L);
        break;
    case MSGEMM_F16:
        hipLaunchKernelGGL((build_lut_kernel<__half, float>), grid, blk, 0, s, g, (int)parts, (int)p.b, half,
                           (const __half*)X, ldx, vm, (float*)L);
        break;
    case MSGEMM_BF16:
        hipLaunchKernelGGL((build_lut_kernel<bf16_t, float>), grid, blk, 0, s, g, (int)parts, (int)p.b, half,
                           (const bf16_t*)X, ldx, vm, (float*)L);
        break;
    case MSGEMM_I8:
        hipLaunchKernelGGL((build_lut_kernel<int8_t, int>), grid, blk, 0, s, g, (int)parts, (int)p.b, half,
                           (const int8_t*)X, ldx, vm, (int*)L);
        break;
    default:
        return MSGEMM_ERR_INVALID_ARG;
    }
    MSGEMM_HIP_TRY(hipGetLastError());
    }
    if (p.half_table) {
        const int64_t total = p.lut_groups * p.b;
        dim3 sgrid((unsigned)((total + 255) / 256));
        const int64_t at = half_sums_offset(p);
        switch (p.x_dtype) {
        case MSGEMM_F32:
            hipLaunchKernelGGL((group_sums_kernel<float, float>), sgrid, dim3(256), 0, s, g, p.lut_groups, (int)p.b,
                               (const float*)X, ldx, (float*)L + at);
            break;
        case MSGEMM_F16:
            hipLaunchKernelGGL((group_sums_kernel<__half, float>), sgrid, dim3(256), 0, s, g, p.lut_groups, (int)p.b,
                               (const __half*)X, ldx, (float*)L + at);
            break;
        case MSGEMM_BF16:
            hipLaunchKernelGGL((group_sums_kernel<bf16_t, float>), sgrid, dim3(256), 0, s, g, p.lut_groups, (int)p.b,
                               (const bf16_t*)X, ldx, (float*)L + at);
            break;
        default:
            hipLaunchKernelGGL((group_sums_kernel<int8_t, int>), sgrid, dim3(256), 0, s, g, p.lut_groups, (int)p.b,
                               (const int8_t*)X, ldx, (int*)L + at);
            break;
        }
        MSGEMM_HIP_TRY(hipGetLastError());
    }
    return MSGEMM_OK;
}

int launch_consume_lut(const Plan& p, const void* L, void* Y, int64_t ldy, hipStream_t s)
{
    if (tiled_applies(p)) {
        switch (p.y_dtype) {
        case MSGEMM_F32: return launch_tiled_d<float, float>(p, L, Y, ldy, s);
        case MSGEMM_F16: return launch_tiled_d<float, __half>(p, L, Y, ldy, s);
        case MSGEMM_BF16: return launch_tiled_d<float, bf16_t>(p, L, Y, ldy, s);
        case MSGEMM_I32: return launch_tiled_d<int, int>(p, L, Y, ldy, s);
        default: return MSGEMM_ERR_INVALID_ARG;
        }
    }
    GroupGeom g{p.k, p.block, p.gpb, p.d};
    dim3 grid(grid_for(p.m * p.b, 256)), blk(256);
    const __half* sc = (const __half*)p.scales;
    const int half = p.half_table ? 1 : 0;
    switch (p.y_dtype) {
    case MSGEMM_F32:
        hipLaunchKernelGGL((consume_lut_kernel<float, float>), grid, blk, 0, s, g, p.m, p.b, p.nblocks, half, (float)p.half_c,
                           p.codes, sc, (const float*)L, (const float*)L + half_sums_offset(p), (float*)Y, ldy);
        break;
    case MSGEMM_F16:
        hipLaunchKernelGGL((consume_lut_kernel<float, __half>), grid, blk, 0, s, g, p.m, p.b, p.nblocks, half, (float)p.half_c,
                           p.codes, sc, (const float*)L, (const float*)L + half_sums_offset(p), (__half*)Y, ldy);
        break;
    case MSGEMM_BF16:
        hipLaunchKernelGGL((consume_lut_kernel<float, bf16_t>), grid, blk, 0, s, g, p.m, p.b, p.nblocks, half, (float)p.half_c,
                           p.codes, sc, (const float*)L, (const float*)L + half_sums_offset(p), (bf16_t*)Y, ldy);
        break;
    case MSGEMM_I32:
        hipLaunchKernelGGL((consume_lut_kernel<int, int>), grid, blk, 0, s, g, p.m, p.b, p.nblocks, half, (int)p.half_c,
                           p.codes, (const __half*)nullptr, (const int*)L, (const int*)L + half_sums_offset(p), (int*)Y, ldy);
        break;
    default:
        return MSGEMM_ERR_INVALID_ARG;
    }
    MSGEMM_HIP_TRY(hipGetLastError());
    return MSGEMM_OK;
}

// Plan-time part of the tiled consumer: how many segments, the transposed codes,
// the partial sums.  Leaves the plan on the plain consumer when the shape does
// not fit (p.codes_words stays null).
int global_plan_setup(Plan& p, hipStream_t s)
{
    p.codes_words = nullptr;
    p.global_partials = nullptr;
    p.global_segments = 1;
    p.global_plain = p.opt.global_plain_consumer ? 1 : 0;
    p.global_chunk_kib = p.opt.global_chunk_kib > 0 ? p.opt.global_chunk_kib : 1024;
    if ((p.block % 8) != 0) return MSGEMM_OK;
    if (p.k / 8 > 0x3fffffff || (p.m + 63) / 64 > 0x3fffffff || p.gpb > 0x3fffffff) return MSGEMM_OK;
    // one table entry offset fits 32 bits with room to spare
    if ((((int64_t)1 << (4 * p.d)) * p.b * 24) >= ((int64_t)1 << 31)) return MSGEMM_OK;
    int cus = 256;
    hipDeviceProp_t prop;
    if (hipGetDeviceProperties(&prop, p.device) == hipSuccess && prop.multiProcessorCount > 0)
        cus = prop.multiProcessorCount;
    p.cus = cus;
    const int cb = p.b >= 4 ? 4 : (p.b >= 2 ? 2 : 1);
    p.global_segments = 1;
    TiledGeom g = tiled_geometry(p, cb);
    if ((int64_t)g.chunks > 0x3fffffff) return MSGEMM_OK;
    // enough workgroups for four per compute unit, in multiples of the XCD count
    const int64_t per_seg = (int64_t)g.wg_rows * g.col_passes;
    int seg = g.chunks < kXcds ? g.chunks : kXcds;
    while (g.chunks >= kXcds && seg * per_seg < 4 * (int64_t)cus && 2 * seg <= g.chunks) seg *= 2;
    const int forced = p.opt.global_segments;
    if (forced >= 1 && forced <= g.chunks) seg = forced;
    int cps = (g.chunks + seg - 1) / seg;
    // Workgroups of one segment that run side by side walk its chunks together,
    // and the L2 then holds one chunk at a time.  Once a segment has more
    // workgroups than an XCD runs at once they start at different times and are
    // spread over all of its chunks: then keep a segment's tables within half an
    // L2 (4 MiB per XCD).
    const int64_t chunk_bytes =
        (int64_t)g.chunk_units * (24 / p.d) * (((int64_t)1 << (4 * p.d)) >> (p.half_table ? 1 : 0)) * p.b * 4;
    const int64_t fit = ((int64_t)2 << 20) / chunk_bytes;
    const bool staggered = per_seg > 4 * (int64_t)(cus / kXcds);
    if (forced == 0 && staggered && cps > (fit < 1 ? 1 : fit)) cps = (int)(fit < 1 ? 1 : fit);
    seg = (g.chunks + cps - 1) / cps;
    if (seg * per_seg >= ((int64_t)1 << 31)) return MSGEMM_OK;
    p.global_segments = seg;

    const int64_t words = (int64_t)g.row_tiles * g.row_words * 64;
    MSGEMM_HIP_TRY(hipMalloc((void**)&p.codes_words, (size_t)words * 4u));
    p.workspace_bytes += (size_t)words * 4u;
    if (seg > 1) {
        const size_t pb = (size_t)seg * (size_t)p.b * (size_t)p.m * 4u;
        MSGEMM_HIP_TRY(hipMalloc((void**)&p.global_partials, pb));
        p.workspace_bytes += pb;
    }
    int64_t blocks = (words + 255) / 256;
    if (blocks > 65536) blocks = 65536;
    hipLaunchKernelGGL(transpose_codes_kernel, dim3((unsigned)blocks), dim3(256), 0, s, p.codes, p.codes_words, p.m,
                       p.k / 2, g.row_words, words);
    MSGEMM_HIP_TRY(hipGetLastError());
    return MSGEMM_OK;
}

}  // namespace msgemm
