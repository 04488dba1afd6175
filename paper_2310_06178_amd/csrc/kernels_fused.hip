// Fused msGeMM for d = 2 on gfx950: phase 1 and phase 2 in one launch.
//
// Work decomposition
//   A k-tile is G consecutive table groups (a group = one pair of k-indices =
//   one packed code byte per row); its tables -- 256 entries per group, C batch
//   columns per entry -- are built in LDS by the workgroup that consumes them:
//   the table is produced piecewise along its last dimension and consumed at
//   once (Section 4, "pipeline phase 1 and 2 by partially computing L").
//   A workgroup owns one k-tile and `panels` row panels; each wavefront
//   streams whole panels.  Outputs are reduced over k-tiles through a
//   partial-sum buffer: the wavefront that delivers the last partial of a
//   panel adds them up in k-tile order and writes Y.
//
// LDS layout and the gather
//   entry(code, g) sits at byte (code*G + g) * C * sizeof(ET).  Lane l = 16q+j
//   of a wavefront looks up group 16*(q % NQ) + (j + t) % 16 in its t-th load
//   (NQ = G/16), so the G/NQ... lanes that are served together always address
//   different groups, hence different banks, whatever the codes are: the
//   gather is bank-conflict free by construction.  A lane keeps the same rows
//   for all 16 loads of a panel, so its accumulators never move between lanes;
//   only the NQ lanes that share rows are added at the end of the panel.
//
// Code stream
//   The plan stores the codes in the order the lanes consume them
//   ([k-tile][panel][load][lane][byte]), so every load instruction of a
//   wavefront reads one contiguous 64*LB-byte segment with full-width
//   per-lane loads.
#include "device_types.h"
#include "msgemm_internal.h"

namespace msgemm {
namespace {

constexpr int kWaves = 8;           // wavefronts per workgroup
constexpr int kLoadsPerPanel = 16;  // one load per group of a 16-group class
constexpr int kAuxSc1 = 16;         // buffer-load cache policy: coherent at agent scope

struct FusedArgs {
    const uint8_t* tiled;
    const void* X;
    int64_t ldx;
    void* Y;
    int64_t ldy;
    const __half* scales;   // [m][nblocks] or nullptr
    float* partials;        // [ktiles][b_pad][m_pad]
    unsigned* counters;     // [panels_total][col_passes]
    int64_t m, k, b, m_pad, b_pad;
    int ktiles, panels_total, panels_per_wg, row_blocks, col_passes;
    int64_t nblocks;        // scale blocks per row
    int64_t partial_span;   // bytes of the partial buffer addressable from any panel base (< 2^31)
    int tiles_per_block;    // k-tiles per scale block
};

template <int LB> struct LaneLoad;
template <> struct LaneLoad<16> { using type = uint4; };
template <> struct LaneLoad<8> { using type = uint2; };
template <> struct LaneLoad<4> { using type = uint32_t; };

template <int LB>
__device__ __forceinline__ uint32_t load_word(const typename LaneLoad<LB>::type& v, int w)
{
    if constexpr (LB == 16) return w == 0 ? v.x : w == 1 ? v.y : w == 2 ? v.z : v.w;
    else if constexpr (LB == 8) return w == 0 ? v.x : v.y;
    else return v;
}

template <typename ET> __device__ __forceinline__ ET make_entry(float v);
template <> __device__ __forceinline__ float make_entry<float>(float v) { return v; }
template <> __device__ __forceinline__ __half make_entry<__half>(float v) { return __float2half_rn(v); }
template <typename ET> __device__ __forceinline__ ET make_entry_i(int v) { return (ET)v; }

template <typename ET> struct EntryAcc;
template <> struct EntryAcc<float> { using type = float; static __device__ __forceinline__ float widen(float e) { return e; } };
template <> struct EntryAcc<__half> { using type = float; static __device__ __forceinline__ float widen(__half e) { return __half2float(e); } };
template <> struct EntryAcc<int> { using type = int; static __device__ __forceinline__ int widen(int e) { return e; } };
template <> struct EntryAcc<short> { using type = int; static __device__ __forceinline__ int widen(short e) { return (int)e; } };

typedef unsigned v2u __attribute__((ext_vector_type(2)));

__device__ __forceinline__ unsigned bits_of(float v) { return __float_as_uint(v); }
__device__ __forceinline__ unsigned bits_of(int v) { return (unsigned)v; }
__device__ __forceinline__ void set_bits(float& d, unsigned u) { d = __uint_as_float(u); }
__device__ __forceinline__ void set_bits(int& d, unsigned u) { d = (int)u; }

// a <- a + (a moved across the wave halves), two registers at a time: after the
// call lanes 0..31 hold the full sum of `a` and lanes 32..63 the full sum of `b`.
template <typename AT> __device__ __forceinline__ AT fold32(AT a, AT b)
{
    v2u r = __builtin_amdgcn_permlane32_swap(bits_of(a), bits_of(b), false, false);
    AT x, y;
    set_bits(x, r.x);
    set_bits(y, r.y);
    return x + y;
}
// Same across the two 16-lane rows of each half: even rows end up with `a`, odd rows with `b`.
template <typename AT> __device__ __forceinline__ AT fold16(AT a, AT b)
{
    v2u r = __builtin_amdgcn_permlane16_swap(bits_of(a), bits_of(b), false, false);
    AT x, y;
    set_bits(x, r.x);
    set_bits(y, r.y);
    return x + y;
}

// The partial sums of one output come from workgroups on different XCDs, whose
// L2 slices are not coherent with each other: partials and counters are only
// touched with agent-scope atomic accesses (they go to the coherence point), and
// ordered by waiting for the stores to be acknowledged before the counter is
// bumped.  No cache-wide write-back / invalidate is needed that way.
__device__ __forceinline__ void store_agent(float* p, float v)
{
    __hip_atomic_store(p, v, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}
__device__ __forceinline__ void wait_vmem()
{
    asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
}

template <typename AT> __device__ __forceinline__ float as_stored(AT v);
template <> __device__ __forceinline__ float as_stored<float>(float v) { return v; }
template <> __device__ __forceinline__ float as_stored<int>(int v) { return __int_as_float(v); }
template <typename AT> __device__ __forceinline__ AT from_stored(float v);
template <> __device__ __forceinline__ float from_stored<float>(float v) { return v; }
template <> __device__ __forceinline__ int from_stored<int>(float v) { return __float_as_int(v); }

template <typename ET, int C> struct alignas(C * sizeof(ET) >= 16 ? 16 : C * sizeof(ET)) EntryVec { ET v[C]; };

// Row of a panel that lane (q, j) keeps in accumulator slot s.  Chosen so that
// after the cross-lane fold lane l holds the rows base + 64*i + l, i.e. the
// epilogue's stores are contiguous across the wavefront.
template <int NQ, int LB>
__host__ __device__ __forceinline__ int panel_row(int q, int j, int s)
{
    constexpr int nfinal = LB / NQ;
    const int qr = q / NQ;
    return (s % nfinal) * 64 + (qr * NQ + s / nfinal) * 16 + j;
}

template <typename XT, typename YT, typename ET, int C, int G, int LB>
__global__ void __launch_bounds__(kWaves * 64)
fused_kernel(FusedArgs a)
{
    using AT = typename EntryAcc<ET>::type;
    using LoadT = typename LaneLoad<LB>::type;
    using Entry = EntryVec<ET, C>;
    constexpr int NQ = G / 16;                    // lanes sharing a row (one per 16-group class)
    constexpr int kEntryBytes = C * (int)sizeof(ET);
    constexpr int kCodeStride = G * kEntryBytes;  // bytes between consecutive codes
    constexpr int kFinal = LB / NQ;               // outputs per lane and column after the fold
    constexpr int kPanelRows = kFinal * 64;
    constexpr int kThreads = kWaves * 64;
    static_assert(G == 16 || G == 32 || G == 64, "G");
    static_assert(kThreads % G == 0, "threads per group");
    static_assert(LB % NQ == 0, "rows per lane must split over the lanes sharing them");

    __shared__ __align__(16) unsigned char lds[256 * kCodeStride];

    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int wave = tid >> 6;
    const int q = lane >> 4, j = lane & 15;
    const int qg = q % NQ;

    int bid = blockIdx.x;
    const int kt = bid % a.ktiles; bid /= a.ktiles;
    const int rb = bid % a.row_blocks;
    const int cp = bid / a.row_blocks;
    const int64_t col0 = (int64_t)cp * C;

    const XT* __restrict__ X = (const XT*)a.X;
    YT* __restrict__ Y = (YT*)a.Y;

    // ---- activations of this k-tile (fetched first: the wait for them must not
    // also wait for the code loads issued next)
    const int g = tid % G;
    AT x0[C], x1[C];
    {
        const int64_t kk = ((int64_t)kt * G + g) * 2;
#pragma unroll
        for (int c = 0; c < C; ++c) {
            const bool live = (col0 + c < a.b) && (kk < a.k);
            x0[c] = live ? (AT)XTraits<XT>::load(X + (col0 + c) * a.ldx + kk) : (AT)0;
            x1[c] = live ? (AT)XTraits<XT>::load(X + (col0 + c) * a.ldx + kk + 1) : (AT)0;
        }
    }

    // ---- first panel's codes: in flight while the tables are built
    const int panel_first = rb * a.panels_per_wg;
    int panels_here = a.panels_total - panel_first;
    if (panels_here > a.panels_per_wg) panels_here = a.panels_per_wg;
    const LoadT* __restrict__ tiled =
        (const LoadT*)a.tiled + ((int64_t)kt * a.panels_total + panel_first) * (kLoadsPerPanel * 64) + lane;
    LoadT data[kLoadsPerPanel];
    int p = wave;
    if (p < panels_here) {
        const LoadT* src = tiled + (int64_t)p * (kLoadsPerPanel * 64);
#pragma unroll
        for (int t = 0; t < kLoadsPerPanel; ++t) data[t] = src[t * 64];
    }

    // ---- phase 1: L(code, g, c) = b(code & 15) X(2g', c) + b(code >> 4) X(2g'+1, c)
    for (int code = tid / G; code < 256; code += kThreads / G) {
        const AT w0 = (AT)decode4(code & 15), w1 = (AT)decode4(code >> 4);
        Entry e;
#pragma unroll
        for (int c = 0; c < C; ++c) {
            if constexpr (__is_same(AT, float))
                e.v[c] = make_entry<ET>(fmaf(w0, x0[c], w1 * x1[c]));
            else
                e.v[c] = make_entry_i<ET>(w0 * x0[c] + w1 * x1[c]);
        }
        *(Entry*)(lds + (size_t)code * kCodeStride + g * kEntryBytes) = e;
    }
    __syncthreads();

    // ---- phase 2: stream panels, gather, accumulate
    const uint32_t class_base = (uint32_t)(16 * qg) * kEntryBytes;
    for (; p < panels_here; p += kWaves) {
        AT acc[LB][C];
#pragma unroll
        for (int s = 0; s < LB; ++s)
#pragma unroll
            for (int c = 0; c < C; ++c) acc[s][c] = 0;

        // One load's worth of look-ups is issued while the previous one's
        // entries are being added: the LDS latency hides behind the adds
        // without the scheduler hoisting all 16*LB reads at once.
        auto issue = [&](int t, Entry (&dst)[LB]) {
            const uint32_t lane_off = class_base + (uint32_t)((j + t) & 15) * kEntryBytes;
#pragma unroll
            for (int s = 0; s < LB; ++s) {
                const uint32_t w = load_word<LB>(data[t], s >> 2);
                uint32_t addr;
                if constexpr (kCodeStride == 256)  // code byte drops straight into address bits 15:8
                    addr = __builtin_amdgcn_perm(w, lane_off, 0x0c0c0000u | ((4u + (s & 3)) << 8));
                else
                    addr = ((w >> (8 * (s & 3))) & 0xffu) * kCodeStride + lane_off;
                dst[s] = *(const Entry*)(lds + addr);
            }
        };
        auto consume = [&](const Entry (&src)[LB]) {
#pragma unroll
            for (int s = 0; s < LB; ++s)
#pragma unroll
                for (int c = 0; c < C; ++c) {
                    acc[s][c] += EntryAcc<ET>::widen(src[s].v[c]);
                    // pin the add to this stage: otherwise the compiler sinks all
                    // adds below the gather and keeps every table entry live
                    asm volatile("" : "+v"(acc[s][c]));
                }
        };
        Entry e0[LB], e1[LB];
        issue(0, e0);
#pragma unroll
        for (int t = 0; t < kLoadsPerPanel; t += 2) {
            issue(t + 1, e1);
            consume(e0);
            __builtin_amdgcn_sched_barrier(0);
            if (t + 2 < kLoadsPerPanel) issue(t + 2, e0);
            consume(e1);
            __builtin_amdgcn_sched_barrier(0);
        }
        // next panel's codes (if any) while this panel is being finished
        const int pn = p + kWaves;
        if (pn < panels_here) {
            const LoadT* src = tiled + (int64_t)pn * (kLoadsPerPanel * 64);
#pragma unroll
            for (int t = 0; t < kLoadsPerPanel; ++t) data[t] = src[t * 64];
        }

        // lanes that share rows: fold the NQ group classes; each lane ends up
        // with kFinal distinct rows (base + 64*i + lane)
        AT fin[kFinal][C];
#pragma unroll
        for (int c = 0; c < C; ++c) {
            if constexpr (NQ == 4) {
                AT half[LB / 2];
#pragma unroll
                for (int s = 0; s < LB / 2; ++s) half[s] = fold32(acc[s][c], acc[s + LB / 2][c]);
#pragma unroll
                for (int s = 0; s < kFinal; ++s) fin[s][c] = fold16(half[s], half[s + kFinal]);
            } else if constexpr (NQ == 2) {
#pragma unroll
                for (int s = 0; s < kFinal; ++s) fin[s][c] = fold16(acc[s][c], acc[s + kFinal][c]);
            } else {
#pragma unroll
                for (int s = 0; s < kFinal; ++s) fin[s][c] = acc[s][c];
            }
        }

        // scale of this k-tile's block (Section 3.3), then hand the partial over
        const int panel_g = panel_first + p;
        const int64_t row0 = (int64_t)panel_g * kPanelRows + lane;
        float* part = a.partials + ((int64_t)kt * a.b_pad + col0) * a.m_pad + row0;
#pragma unroll
        for (int i = 0; i < kFinal; ++i) {
            float qv = 1.0f;
            if constexpr (__is_same(AT, float)) {
                const int64_t row = row0 + 64 * i;
                if (a.scales && row < a.m) qv = __half2float(a.scales[row * a.nblocks + kt / a.tiles_per_block]);
            }
#pragma unroll
            for (int c = 0; c < C; ++c) {
                AT v = fin[i][c];
                if constexpr (__is_same(AT, float)) v = v * qv;
                store_agent(part + (int64_t)c * a.m_pad + 64 * i, as_stored<AT>(v));
            }
        }
        wait_vmem();  // partials acknowledged before the counter moves
        unsigned prev = 0;
        unsigned* counter = a.counters + (int64_t)panel_g * a.col_passes + cp;
        if (lane == 0)
            prev = __hip_atomic_fetch_add(counter, 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        prev = __builtin_amdgcn_readfirstlane(prev);
        if (prev == (unsigned)a.ktiles - 1u) {
            // every k-tile's partial for this panel has been published: add them
            // in k-tile order.  Buffer loads with the agent-coherent policy bit:
            // independent loads stay in flight together.
            // (the descriptor is wave-uniform; the lane's rows go into the offset)
            __amdgpu_buffer_rsrc_t rsrc =
                __builtin_amdgcn_make_buffer_rsrc((void*)a.partials, 0, (int)a.partial_span, 0x00020000);
            const uint32_t lane_base = (uint32_t)(col0 * a.m_pad + row0) * 4u;
            const uint32_t tile_stride = (uint32_t)(a.b_pad * a.m_pad * 4);
            AT sum[kFinal][C];
#pragma unroll
            for (int i = 0; i < kFinal; ++i)
#pragma unroll
                for (int c = 0; c < C; ++c) sum[i][c] = 0;
#pragma unroll 4
            for (int t = 0; t < a.ktiles; ++t) {
#pragma unroll
                for (int i = 0; i < kFinal; ++i)
#pragma unroll
                    for (int c = 0; c < C; ++c) {
                        const uint32_t off = lane_base + (uint32_t)t * tile_stride + (uint32_t)(c * (uint32_t)a.m_pad + 64 * i) * 4u;
                        const unsigned u = __builtin_amdgcn_raw_buffer_load_b32(rsrc, (int)off, 0, kAuxSc1);
                        AT v;
                        set_bits(v, u);
                        sum[i][c] += v;
                    }
            }
#pragma unroll
            for (int i = 0; i < kFinal; ++i) {
                const int64_t row = row0 + 64 * i;
#pragma unroll
                for (int c = 0; c < C; ++c)
                    if (row < a.m && col0 + c < a.b) Y[(col0 + c) * a.ldy + row] = to_output<YT, AT>(sum[i][c]);
            }
            if (lane == 0) __hip_atomic_store(counter, 0u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        }
    }
}

// One-off reorder of the row-major code bytes into streaming order.
template <int G, int LB>
__global__ void __launch_bounds__(256)
repack_kernel(const uint8_t* __restrict__ codes, uint8_t* __restrict__ tiled, int64_t m, int64_t kbytes,
              int ktiles, int panels_total)
{
    constexpr int NQ = G / 16;
    constexpr int kPanelRows = (4 / NQ) * LB * 16;
    const int64_t total = (int64_t)ktiles * panels_total * kLoadsPerPanel * 64 * LB;
    for (int64_t o = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; o < total;
         o += (int64_t)gridDim.x * blockDim.x) {
        int64_t r = o;
        const int s = (int)(r % LB); r /= LB;
        const int lane = (int)(r % 64); r /= 64;
        const int t = (int)(r % kLoadsPerPanel); r /= kLoadsPerPanel;
        const int64_t panel = r % panels_total;
        const int64_t kt = r / panels_total;
        const int q = lane >> 4, j = lane & 15;
        const int qg = q % NQ;
        const int64_t row = panel * kPanelRows + panel_row<NQ, LB>(q, j, s);
        const int64_t byte = kt * G + 16 * qg + ((j + t) & 15);
        tiled[o] = (row < m && byte < kbytes) ? codes[row * kbytes + byte] : (uint8_t)0;
    }
}

struct ShapeChoice { int C, G, LB, entry_bytes; };

ShapeChoice pick_shape(const Plan& p)
{
    (void)p;
    return ShapeChoice{1, 64, 16, 4};
}

template <typename XT, typename YT, typename ET, int C, int G, int LB>
int launch_one(const Plan& p, const FusedArgs& a, hipStream_t s)
{
    auto kern = fused_kernel<XT, YT, ET, C, G, LB>;
    const unsigned grid = (unsigned)((int64_t)p.ktiles * p.row_blocks * p.col_passes);
    hipLaunchKernelGGL(kern, dim3(grid), dim3(kWaves * 64), 0, s, a);
    MSGEMM_HIP_TRY(hipGetLastError());
    return MSGEMM_OK;
}

}  // namespace

int fused_choose_shape(Plan& p)
{
    if (p.d != 2) return MSGEMM_ERR_UNSUPPORTED;
    const ShapeChoice sc = pick_shape(p);
    const int cols_per_tile = 2 * sc.G;
    if (p.scale_group > 0 && (p.scale_group % cols_per_tile) != 0) return MSGEMM_ERR_UNSUPPORTED;
    FusedShape& fs = p.fs;
    fs.groups = sc.G;
    fs.lane_bytes = sc.LB;
    fs.cols = sc.C;
    fs.entry_bytes = sc.entry_bytes;
    fs.waves = kWaves;
    fs.panel_rows = (4 / (sc.G / 16)) * sc.LB * 16;
    fs.lds_bytes = (size_t)256 * sc.G * sc.C * sc.entry_bytes;
    p.ktiles = (p.k / 2 + sc.G - 1) / sc.G;
    p.col_passes = (int)((p.b + sc.C - 1) / sc.C);
    const int64_t panels = (p.m + fs.panel_rows - 1) / fs.panel_rows;
    if (panels > (1 << 30) || p.ktiles > (1 << 20)) return MSGEMM_ERR_UNSUPPORTED;

    int cus = 256;
    hipDeviceProp_t prop;
    if (hipGetDeviceProperties(&prop, p.device) == hipSuccess && prop.multiProcessorCount > 0)
        cus = prop.multiProcessorCount;
    // Rows per table build: as many panels per workgroup as still leave one
    // workgroup per compute unit (each build costs 256 entries per group).
    int ppw = 16;
    while (ppw > 1 && (int64_t)p.ktiles * p.col_passes * ((panels + ppw - 1) / ppw) < cus) ppw >>= 1;
    fs.panels = ppw;
    fs.tile_rows = ppw * fs.panel_rows;
    p.row_blocks = (panels + ppw - 1) / ppw;
    p.m_pad = panels * fs.panel_rows;
    if ((int64_t)p.ktiles * p.row_blocks * p.col_passes > 0x7fffffffLL) return MSGEMM_ERR_UNSUPPORTED;
    // the k-tile reduction addresses the partial buffer with 32-bit byte offsets
    if ((int64_t)p.ktiles * p.col_passes * sc.C * p.m_pad * 4 >= 0x7fffffffLL) return MSGEMM_ERR_UNSUPPORTED;
    return MSGEMM_OK;
}

int launch_repack(const Plan& p, hipStream_t s)
{
    const int64_t panels = p.m_pad / p.fs.panel_rows;
    const int64_t total = (int64_t)p.ktiles * p.m_pad * p.fs.groups;
    int64_t blocks = (total + 255) / 256;
    if (blocks > 65536) blocks = 65536;
    if (p.fs.groups == 64 && p.fs.lane_bytes == 16) {
        hipLaunchKernelGGL((repack_kernel<64, 16>), dim3((unsigned)blocks), dim3(256), 0, s, p.codes,
                           p.codes_tiled, p.m, p.k / 2, (int)p.ktiles, (int)panels);
    } else {
        return MSGEMM_ERR_UNSUPPORTED;
    }
    MSGEMM_HIP_TRY(hipGetLastError());
    return MSGEMM_OK;
}

int launch_fused(const Plan& p, const void* X, int64_t ldx, void* Y, int64_t ldy, hipStream_t s)
{
    FusedArgs a;
    a.tiled = p.codes_tiled;
    a.X = X; a.ldx = ldx; a.Y = Y; a.ldy = ldy;
    a.scales = (const __half*)p.scales;
    a.partials = p.partials;
    a.counters = p.counters;
    a.m = p.m; a.k = p.k; a.b = p.b; a.m_pad = p.m_pad;
    a.b_pad = (int64_t)p.col_passes * p.fs.cols;
    a.ktiles = (int)p.ktiles;
    a.panels_total = (int)(p.m_pad / p.fs.panel_rows);
    a.panels_per_wg = p.fs.panels;
    a.row_blocks = (int)p.row_blocks;
    a.col_passes = p.col_passes;
    a.nblocks = p.nblocks;
    a.partial_span = (int64_t)p.ktiles * a.b_pad * p.m_pad * 4;
    a.tiles_per_block = p.scale_group > 0 ? (int)(p.scale_group / (2 * p.fs.groups)) : 1;

    if (p.fs.cols == 1 && p.fs.groups == 64 && p.fs.lane_bytes == 16) {
        switch (p.x_dtype) {
        case MSGEMM_F32: return launch_one<float, float, float, 1, 64, 16>(p, a, s);
        case MSGEMM_F16: return launch_one<__half, __half, float, 1, 64, 16>(p, a, s);
        case MSGEMM_BF16: return launch_one<bf16_t, bf16_t, float, 1, 64, 16>(p, a, s);
        case MSGEMM_I8: return launch_one<int8_t, int, int, 1, 64, 16>(p, a, s);
        default: break;
        }
    }
    return MSGEMM_ERR_UNSUPPORTED;
}

}  // namespace msgemm
