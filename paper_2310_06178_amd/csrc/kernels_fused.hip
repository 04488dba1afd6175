// Fused msGeMM for d = 2 on gfx950: phase 1 and phase 2 in one launch, with
// full-width (fp32 / int32) table entries: the single-column kernels (b <= 2,
// every dtype) and the 4-column kernel for fp32 activations.  Batches of 16-bit
// activations run through kernels_batched.hip.
//
// Work decomposition
//   A k-tile is G consecutive table groups (a group = one pair of k-indices =
//   one packed code byte per row); its tables -- 256 entries per group, C batch
//   columns per entry -- are built in LDS by the workgroup that consumes them:
//   the table is produced piecewise along its last dimension and consumed at
//   once (Section 4, "pipeline phase 1 and 2 by partially computing L").
//   A workgroup owns one k-tile and `panels` row panels; each wavefront
//   streams whole panels.  Outputs are reduced over k-tiles through a
//   partial-sum buffer, in k-tile order (a fixed order: results are
//   reproducible): by trailing workgroups of the same launch that wait for the
//   partials of their panels (single-column kernels), or by a second small
//   launch (4-column kernel).
//
// LDS layout and the gather
//   entry(code, g) sits at byte (code*G + g) * C * sizeof(ET).  Lane l = 16q+j
//   of a wavefront looks up group 16*(q % NQ) + (j + t) % 16 in its t-th load
//   (NQ = G/16): lanes that are served together always address different
//   groups, hence different banks, whatever the codes are -- the gather is
//   bank-conflict free by construction.  A lane keeps the same rows for all 16
//   loads of a panel, so its accumulators never move between lanes; only the
//   NQ lanes that share rows are folded together at the end of the panel.
//
// Code stream
//   The plan stores the codes in the order the lanes consume them
//   ([load][k-tile][panel][lane][byte]), so every load instruction of a
//   wavefront reads one contiguous 64*LB-byte segment with full-width per-lane
//   loads, and the t-th loads of all wavefronts are neighbours in memory.  A
//   wavefront keeps a ring of kRing loads in flight and refills a slot as soon
//   as its bytes have been turned into LDS addresses.
#include <stdlib.h>
#include <type_traits>

#include "device_types.h"
#include "fused_common.h"
#include "msgemm_internal.h"

// Optional phase timestamps for kernel tuning (compiled out unless requested).
#ifdef MSGEMM_PHASE_TRACE
__device__ unsigned long long* g_msgemm_trace = nullptr;
__device__ unsigned long long g_msgemm_trace_slots = 0;  // capacity of the buffer in 64-bit slots
extern "C" int msgemm_debug_set_trace(unsigned long long* buf, unsigned long long slots)
{
    hipError_t e = hipMemcpyToSymbol(HIP_SYMBOL(g_msgemm_trace_slots), &slots, sizeof(slots));
    if (e != hipSuccess) return (int)e;
    return (int)hipMemcpyToSymbol(HIP_SYMBOL(g_msgemm_trace), &buf, sizeof(buf));
}
// slot (workgroup, wavefront, id); writes past the capacity are dropped
__device__ __forceinline__ void msgemm_trace_put(int id, unsigned long long v)
{
    const unsigned long long slot = ((unsigned long long)blockIdx.x * 16 + (threadIdx.x >> 6)) * 16 + (unsigned)id;
    if (g_msgemm_trace && (threadIdx.x & 63) == 0 && (threadIdx.x >> 6) < 16 && slot < g_msgemm_trace_slots)
        g_msgemm_trace[slot] = v;
}
#define MSGEMM_TRACE(id) msgemm_trace_put((id), wall_clock64())
#else
#define MSGEMM_TRACE(id) do { } while (0)
#endif

namespace msgemm {
namespace {

#ifndef MSGEMM_BUILDERS_1COL
#define MSGEMM_BUILDERS_1COL(waves) ((waves) / 2)
#endif
#ifndef MSGEMM_EARLY_BUILDER
#define MSGEMM_EARLY_BUILDER 0
#endif
#ifndef MSGEMM_DEDICATED_1COL
#define MSGEMM_DEDICATED_1COL 4
#endif
#ifndef MSGEMM_RING_BYTES
#define MSGEMM_RING_BYTES 128
#endif
constexpr int kRingBytes = MSGEMM_RING_BYTES;  // code bytes per lane a wavefront keeps in flight (x64 lanes)

struct FusedArgs {
    const uint8_t* tiled;
    const void* X;
    int64_t ldx;
    void* Y;
    int64_t ldy;
    const __half* scales;   // in output order, [nblocks][panels_total][64][outputs per lane], or nullptr
    float* partials;        // [ktiles][b_pad][panels_total][64][outputs per lane]
    unsigned* flags;        // [panels_total][col_passes][ktiles], zero between launches
    int64_t m, k, b, m_pad, b_pad;
    int ktiles, panels_total, panels_per_wg, row_blocks, col_passes;
    int row_groups;         // row_blocks * col_passes
    int xcd_map;            // 1: workgroups that share outputs get ids congruent modulo kXcds; 2: see column_pass_order
    int64_t nblocks;        // scale blocks per row
    int64_t partial_span;   // bytes of the partial buffer (< 2^31)
    int64_t scale_span;     // bytes of the ordered scales (< 2^31)
    int tiles_per_block;    // k-tiles per scale block
    int reduce_mode;        // how partial sums over k-tiles become Y, see ReduceMode
    FastDiv div_ktiles, div_col_passes, div_tiles_per_block;
    int fused_wgs;          // workgroups of the grid that do the fused work; the rest reduce (in-launch mode)
    int red_units;          // (panel, column pass) pairs to reduce, one trailing workgroup each
    int slices;             // partial sums per output: k-tiles, or k-segments in the long-k form
    int tiles_per_segment;  // long-k form: k-tiles a workgroup runs through
    FastDiv div_slices;
    const float* values256; // 8-bit codes: the value of each of the 256 bit patterns (device), else nullptr
    unsigned* epochs;       // wide form, resident reduction: launch count of every workgroup (each bumps its own)
    unsigned* error;        // sticky word: set when a wavefront gave up waiting for partial sums (see msgemm_plan_check)
    unsigned poll_limit;    // polls before a waiting wavefront gives up
    int publish;            // 0 (test aid): producers never announce their partial sums
    int red_chunk;          // resident reduction: partial sums (floats, a multiple of 4) each workgroup of a row group adds up
    ValueMap values;        // value of each 4-bit pattern; last, read only by the forms built for a custom map
};

// Order of the workgroup ids when a plan has several column passes (b = 2; fp32 activations with b > 4): the passes
// of one (row block, k-slice) unit stream the same codes, so they get ids that are congruent modulo the XCD count and
// follow each other there -- they start together on one XCD and the second finds in that L2 what the first has
// fetched (in any other order every pass streams its codes from memory again: 2.0x the bytes on a 300 MB GeMV).
// Units are dealt over the XCDs; ids past the last unit do nothing.  Returns false for such an id.
constexpr int kXcdMapColumnPasses = 2;
__device__ __forceinline__ bool column_pass_order(const FusedArgs& a, uint32_t bid, FastDiv div_slices, int slices,
                                                  int& slice, int& rg)
{
    const uint32_t n = bid / kXcds;
    const uint32_t hi = fast_div(n, a.div_col_passes);
    const uint32_t cp = n - hi * (uint32_t)a.col_passes;
    const uint32_t unit = (bid % kXcds) + kXcds * hi;
    if (unit >= (uint32_t)(slices * a.row_blocks)) return false;
    const uint32_t rb = fast_div(unit, div_slices);
    slice = (int)(unit - rb * (uint32_t)slices);
    rg = (int)(rb * (uint32_t)a.col_passes + cp);
    return true;
}

enum ReduceMode {
    kReduceDirect = 0,    // a single k-tile: the fused kernel writes Y itself
    kReduceSecondPass = 1,  // partials to memory, a second small kernel adds them
    kReduceInLaunch = 2,  // partials to memory, trailing workgroups of the same launch add them
    kReduceResident = 3   // partials to memory, the workgroups that wrote them add them (the whole grid is resident)
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

template <typename ET> struct EntryAcc;
template <> struct EntryAcc<float> {
    using type = float;
    static __device__ __forceinline__ float widen(float e) { return e; }
    static __device__ __forceinline__ float make(float v) { return v; }
};
template <> struct EntryAcc<int> {
    using type = int;
    static __device__ __forceinline__ int widen(int e) { return e; }
    static __device__ __forceinline__ int make(int v) { return v; }
};

__device__ __forceinline__ float mul_add(float w, float x, float acc) { return fmaf(w, x, acc); }
__device__ __forceinline__ int mul_add(int w, int x, int acc) { return w * x + acc; }

template <typename ET, int C> struct alignas(C * sizeof(ET) >= 16 ? 16 : C * sizeof(ET)) EntryVec { ET v[C]; };

// The single-column kernels can reduce inside the launch; the batched ones are
// bound by the gather, not by launches, and have no registers to spare for it.
template <int C> constexpr bool kInLaunchReduce = C == 1;

// Reduction over the k-tiles inside the launch.  Each workgroup that follows
// the fused ones in the grid takes one (panel, column pass) unit.  Its first
// kRedSplit wavefronts share the k-tiles (wavefront w takes w, w + kRedSplit,
// ...): each waits for the flags of its k-tiles, adds their partial sums in
// increasing order and leaves its sum in LDS; wavefront 0 then adds the
// wavefront sums in wavefront order and writes Y.  The association is fixed:
// results are reproducible.  Workgroups are dispatched in id order, so everything
// a reducer waits for is already resident and runs to its flag without waiting
// on anyone: the wait ends (it is bounded all the same).
constexpr int kRedSplit = 8;

template <typename YT, typename AT, int kFinal>
__device__ __forceinline__ void reduce_in_launch(const FusedArgs& a, int unit, int w, int lane, unsigned char* lds)
{
    constexpr int kPanelRows = kFinal * 64;
    const int panel_g = (int)fast_div((uint32_t)unit, a.div_col_passes);
    const int col = unit - panel_g * a.col_passes;  // single-column kernels: a column pass is a column
    AT sum[kFinal];
#pragma unroll
    for (int i = 0; i < kFinal; ++i) sum[i] = 0;
    AT* wave_sums = (AT*)lds;  // [kRedSplit][kFinal][64]: consecutive lanes, consecutive banks
    if (w < kRedSplit) {
        const int mine = w < a.slices ? (a.slices - w + kRedSplit - 1) / kRedSplit : 0;  // slices of this wavefront
        unsigned* flags = a.flags + (int64_t)unit * a.slices;
        for (int base = 0; base < mine; base += 64) {
            const int idx = base + lane;
            const bool need = idx < mine;
            unsigned* flag = flags + w + (int64_t)idx * kRedSplit;
            bool seen = false;
            for (unsigned spins = 0; spins < a.poll_limit; ++spins) {
                asm volatile("" ::: "memory");
                const unsigned f = need ? __hip_atomic_load(flag, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) : 1u;
                if (__builtin_amdgcn_ballot_w64(f != 1u) == 0) {
                    seen = true;
                    break;
                }
                __builtin_amdgcn_s_sleep(2);
            }
            if (!seen) {
                // gave up: the sums below are not the result.  The plan's error word says so (msgemm_plan_check);
                // the flags stay as they are, that call clears them.
                if (lane == 0) __hip_atomic_store(a.error, 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
                continue;
            }
            // lowered again for the next launch (kernel boundaries order launches)
            if (need) __hip_atomic_store(flag, 0u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        }
        asm volatile("" ::: "memory");
        MSGEMM_TRACE(7);
        __amdgpu_buffer_rsrc_t part_rsrc =
            __builtin_amdgcn_make_buffer_rsrc((void*)a.partials, 0, (int)a.partial_span, 0x00020000);
        const uint32_t col_stride = (uint32_t)(a.m_pad * 4);
        const uint32_t tile_stride = (uint32_t)(a.b_pad * a.m_pad * 4);
        const uint32_t off0 = (uint32_t)col * col_stride + (uint32_t)(panel_g * kPanelRows + lane * kFinal) * 4u;
        // kBatch k-tiles' partials are requested together, then added in order;
        // k-tiles past the end get an out-of-range offset, which reads as zero
        constexpr int kBatch = 8;
        for (int t0 = 0; t0 < mine; t0 += kBatch) {
            unsigned v[kBatch][kFinal];
#pragma unroll
            for (int u = 0; u < kBatch; ++u) {
                const uint32_t off =
                    (t0 + u < mine) ? off0 + (uint32_t)(w + (t0 + u) * kRedSplit) * tile_stride : 0x7ffffff0u;
                load_partials<kFinal, kAuxSc1>(part_rsrc, off, v[u]);
            }
            __builtin_amdgcn_sched_barrier(0);
#pragma unroll
            for (int u = 0; u < kBatch; ++u)
#pragma unroll
                for (int i = 0; i < kFinal; ++i) {
                    AT x;
                    set_bits(x, v[u][i]);
                    sum[i] += x;
                }
        }
#pragma unroll
        for (int i = 0; i < kFinal; ++i) wave_sums[(w * kFinal + i) * 64 + lane] = sum[i];
    }
    __syncthreads();  // every wavefront of the workgroup gets here
    if (w != 0) return;
#pragma unroll
    for (int j = 1; j < kRedSplit; ++j)
#pragma unroll
        for (int i = 0; i < kFinal; ++i) sum[i] += wave_sums[(j * kFinal + i) * 64 + lane];
    YT* __restrict__ Y = (YT*)a.Y;
    const int64_t row0 = (int64_t)panel_g * kPanelRows + lane;
#pragma unroll
    for (int i = 0; i < kFinal; ++i) {
        const int64_t row = row0 + 64 * i;
        if (row < a.m && col < a.b) Y[(int64_t)col * a.ldy + row] = to_output<YT, AT>(sum[i]);
    }
    MSGEMM_TRACE(8);
}

// Wavefronts that only build the tables and then retire.  The single-column
// kernel with 8 streaming wavefronts has them: a wavefront that both builds and
// streams requests its codes late, after the activations have arrived.  (The
// 16-wavefront form has no room for more wavefronts in a workgroup.)
template <int C, int kWaves> constexpr int dedicated_builders() { return (C == 1 && kWaves <= 8) ? MSGEMM_DEDICATED_1COL : 0; }

// kValueMode: what the tables are built from.  kValuesDefault: b(.) of Section
// 3.1 as compile-time constants.  kValuesMap16: the plan's 16-value map (a form
// of its own, so that the default never touches that part of the argument
// buffer).  kValuesMap256: 8-bit weights -- a code byte is one element, a group
// is one k-column and an entry is values256[code] * x; everything after the
// table build is the same kernel.
enum { kValuesDefault = 0, kValuesMap16 = 1, kValuesMap256 = 2 };

template <typename XT, typename YT, typename ET, int C, int G, int LB, int kWaves, int kValueMode>
__global__ void __launch_bounds__((kWaves + dedicated_builders<C, kWaves>()) * 64)
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
    // wavefronts that build the tables (phase 1): half of them when one column
    // is built (the others start the code stream at once), all of them for the
    // wide tables of a batch
    constexpr int kDedicated = dedicated_builders<C, kWaves>();
    constexpr int kBuilders = kDedicated ? kDedicated : (C == 1 ? MSGEMM_BUILDERS_1COL(kWaves) : kWaves);
    // loads in flight: the batched kernels are bound by VALU work, half the depth is enough there
    constexpr int kRingWant = (C == 1 ? kRingBytes : kRingBytes / 2) / LB;
    constexpr int kRing = kRingWant < kLoadsPerPanel ? kRingWant : kLoadsPerPanel;
    constexpr int kEarlyBuilder = C == 1 ? MSGEMM_EARLY_BUILDER : 2;  // code loads a builder requests before it waits for the activations
    constexpr int kBuildParts = kBuilders * 64 / G;  // builder threads per group
    static_assert(kBuildParts >= 1 && kBuilders * 64 % G == 0, "builders must cover whole groups");
    static_assert(G == 16 || G == 32 || G == 64, "G");
    static_assert(LB % NQ == 0, "rows per lane must split over the lanes sharing them");
    static_assert(kLoadsPerPanel % kRing == 0, "ring slots are reused with a period dividing the panel");

    __shared__ __align__(16) unsigned char lds[256 * kCodeStride];
    __shared__ unsigned tables_built;  // builder wavefronts that have finished phase 1

    // Fetch every launch argument in one batch of scalar loads.  Left alone the
    // compiler loads each where it is first used, and the kernel then starts with
    // a chain of dependent round trips to the argument buffer -- each a cache miss.
#define MSGEMM_ARG_NOW(x) asm volatile("" ::"s"(x))
    MSGEMM_ARG_NOW((uint64_t)a.tiled); MSGEMM_ARG_NOW((uint64_t)a.X); MSGEMM_ARG_NOW(a.ldx);
    MSGEMM_ARG_NOW((uint64_t)a.Y); MSGEMM_ARG_NOW(a.ldy); MSGEMM_ARG_NOW((uint64_t)a.scales);
    if constexpr (kValueMode == kValuesMap16) {
#pragma unroll
        for (int i = 0; i < 16; ++i) MSGEMM_ARG_NOW(a.values.v[i]);
    }
    if constexpr (kValueMode == kValuesMap256) MSGEMM_ARG_NOW((uint64_t)a.values256);
    MSGEMM_ARG_NOW((uint64_t)a.partials); MSGEMM_ARG_NOW(a.m); MSGEMM_ARG_NOW(a.k); MSGEMM_ARG_NOW(a.b);
    MSGEMM_ARG_NOW(a.m_pad); MSGEMM_ARG_NOW(a.b_pad); MSGEMM_ARG_NOW(a.ktiles); MSGEMM_ARG_NOW(a.panels_total);
    MSGEMM_ARG_NOW(a.panels_per_wg); MSGEMM_ARG_NOW(a.col_passes); MSGEMM_ARG_NOW(a.row_groups);
    MSGEMM_ARG_NOW(a.xcd_map); MSGEMM_ARG_NOW(a.partial_span); MSGEMM_ARG_NOW(a.reduce_mode);
    MSGEMM_ARG_NOW(a.div_ktiles.magic); MSGEMM_ARG_NOW(a.div_ktiles.s1); MSGEMM_ARG_NOW(a.div_ktiles.s2);
    MSGEMM_ARG_NOW(a.div_col_passes.magic); MSGEMM_ARG_NOW(a.div_col_passes.s1); MSGEMM_ARG_NOW(a.div_col_passes.s2);
    MSGEMM_ARG_NOW(a.div_tiles_per_block.magic); MSGEMM_ARG_NOW(a.div_tiles_per_block.s1);
    MSGEMM_ARG_NOW(a.div_tiles_per_block.s2); MSGEMM_ARG_NOW(a.fused_wgs);
#undef MSGEMM_ARG_NOW

    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int wave = (tid >> 6) - kDedicated;  // streaming wavefront index; negative: dedicated builder
    const int q = lane >> 4, j = lane & 15;
    const int qg = q % NQ;

    // ---- which k-tile / row block / column pass
    if ((int)blockIdx.x >= a.fused_wgs) {  // trailing workgroups: the k-tile reduction (in-launch mode only)
        if constexpr (kInLaunchReduce<C>)
            reduce_in_launch<YT, AT, kFinal>(a, (int)blockIdx.x - a.fused_wgs, tid >> 6, lane, lds);
        return;
    }
    int kt, rg;
    {
        const uint32_t bid = blockIdx.x;
        if (a.xcd_map == kXcdMapColumnPasses) {
            if (!column_pass_order(a, bid, a.div_ktiles, a.ktiles, kt, rg)) return;
        } else {
            const uint32_t n = a.xcd_map ? bid / kXcds : bid;
            const uint32_t nq = fast_div(n, a.div_ktiles);
            kt = (int)(n - nq * (uint32_t)a.ktiles);
            rg = a.xcd_map ? (int)((bid % kXcds) + kXcds * nq) : (int)nq;
            if (rg >= a.row_groups) return;
        }
    }
    const int rb = (int)fast_div((uint32_t)rg, a.div_col_passes);
    const int cp = rg - rb * a.col_passes;  // column passes of one row block are neighbours: the codes stay cached
    const int scale_block = (int)fast_div((uint32_t)kt, a.div_tiles_per_block);
    const int64_t col0 = (int64_t)cp * C;

    const XT* __restrict__ X = (const XT*)a.X;
    YT* __restrict__ Y = (YT*)a.Y;
    if (tid == 0) tables_built = 0;
    __syncthreads();  // nothing is in flight yet: this costs a few cycles
    MSGEMM_TRACE(0);
#ifdef MSGEMM_PHASE_TRACE
    msgemm_trace_put(9, 1 + __builtin_amdgcn_s_getreg((3 << 11) | 20));  // hardware XCC_ID register, bits 3:0
#endif

    // ---- this wavefront's stream of panels: wave, wave + kWaves, ...
    const int panel_first = rb * a.panels_per_wg;
    int panels_here = a.panels_total - panel_first;
    if (panels_here > a.panels_per_wg) panels_here = a.panels_per_wg;
    const int npan = (wave >= 0 && wave < panels_here) ? (panels_here - wave + kWaves - 1) / kWaves : 0;
    // load t of every panel of every k-tile is stored together ([load][k-tile][panel][lane]):
    // wavefronts advance through their panels roughly in step, so what the chip has
    // in flight at any time falls into a narrow address window (DRAM page locality)
    const int64_t step_stride = (int64_t)a.ktiles * a.panels_total * 64;  // LoadT elements between loads
    const LoadT* __restrict__ stream =
        (const LoadT*)a.tiled + ((int64_t)kt * a.panels_total + panel_first + wave) * 64 + lane;
    // (idle wavefronts re-read the tile's first panel, which keeps the code below branch-free)
    const LoadT* first = npan > 0 ? stream : (const LoadT*)a.tiled + lane;
    LoadT ring[kRing];
    auto fill_ring = [&](int from, int to) {
#pragma unroll
        for (int u = from; u < to; ++u) {
            ring[u] = load_codes(first + u * step_stride);
            __builtin_amdgcn_sched_barrier(0);  // loads return in issue order: keep slot 0 first
        }
    };

    // ---- phase 1: L(code, g, c) = b(code & 15) X(2g', c) + b(code >> 4) X(2g'+1, c)
    // The first kBuilders wavefronts fetch the activations of the k-tile and
    // build the tables before they join the code stream; the others request
    // their codes at once.  (Were every wavefront to queue its code loads first,
    // the activation fetch would sit behind them in the memory pipeline.)
    // Readiness of the tables is a counter in LDS rather than a barrier: a load
    // instruction stalls its wavefront while the memory queue is full, and a
    // barrier would make the builders -- and so the tables -- wait for that.
    if (kDedicated ? wave < 0 : wave < kBuilders) {
        const int g = tid % G;
        const int64_t kk = ((int64_t)kt * G + g) * 2;
        // raw values from clamped (always valid) addresses first, conversion after
        // the early code loads: nothing waits for the activations before those are out
        constexpr int kC1PerThread = (16 + kBuildParts - 1) / kBuildParts;
        auto value_of = [&](unsigned nibble) -> AT {
            if constexpr (kValueMode == kValuesMap16) return code_value(a.values, nibble, AT());
            else return (AT)decode4(nibble);
        };
        // 8-bit codes: the 16 values behind each of this thread's high nibbles, requested before anything else
        float v256[kValueMode == kValuesMap256 ? kC1PerThread : 1][16];
        if constexpr (kValueMode == kValuesMap256) {
#pragma unroll
            for (int u = 0; u < kC1PerThread; ++u) {
                const int c1 = (tid / G + u * kBuildParts) & 15;
#pragma unroll
                for (int v4 = 0; v4 < 4; ++v4) {
                    const float4 q = *(const float4*)(a.values256 + c1 * 16 + v4 * 4);
                    v256[u][v4 * 4 + 0] = q.x; v256[u][v4 * 4 + 1] = q.y;
                    v256[u][v4 * 4 + 2] = q.z; v256[u][v4 * 4 + 3] = q.w;
                }
            }
        }
        XT xr0[C], xr1[C];
        bool live[C];
#pragma unroll
        for (int c = 0; c < C; ++c) {
            live[c] = (col0 + c < a.b) && (kk < a.k);
            if constexpr (kValueMode == kValuesMap256) {
                // a group is one k-column (a.k counts two per code byte)
                const XT* px = X + (live[c] ? (col0 + c) * a.ldx + (kk >> 1) : 0);
                xr0[c] = px[0];
                xr1[c] = px[0];
            } else {
                const XT* px = X + (live[c] ? (col0 + c) * a.ldx + kk : 0);
                xr0[c] = px[0];
                xr1[c] = px[1];
            }
        }
        if constexpr (!kDedicated) fill_ring(0, kEarlyBuilder);
        MSGEMM_TRACE(1);
        AT x0[C], x1[C];
#pragma unroll
        for (int c = 0; c < C; ++c) {
            x0[c] = live[c] ? (AT)XTraits<XT>::load(&xr0[c]) : (AT)0;
            x1[c] = live[c] ? (AT)XTraits<XT>::load(&xr1[c]) : (AT)0;
        }
#pragma unroll
        for (int u = 0; u < kC1PerThread; ++u) {
            const int c1 = tid / G + u * kBuildParts;
            if (c1 >= 16) break;
            unsigned char* dst = lds + (size_t)(c1 * 16) * kCodeStride + g * kEntryBytes;
            if constexpr (kValueMode == kValuesMap256) {
#pragma unroll
                for (int c0 = 0; c0 < 16; ++c0) {
                    Entry e;
#pragma unroll
                    for (int c = 0; c < C; ++c) e.v[c] = EntryAcc<ET>::make((AT)v256[u][c0] * x0[c]);
                    *(Entry*)(dst + c0 * kCodeStride) = e;
                }
            } else {
                AT hi[C];
                const AT w1 = value_of((unsigned)c1);
#pragma unroll
                for (int c = 0; c < C; ++c) hi[c] = w1 * x1[c];
#pragma unroll
                for (int c0 = 0; c0 < 16; ++c0) {
                    Entry e;
#pragma unroll
                    for (int c = 0; c < C; ++c) e.v[c] = EntryAcc<ET>::make(mul_add(value_of((unsigned)c0), x0[c], hi[c]));
                    *(Entry*)(dst + c0 * kCodeStride) = e;
                }
            }
        }
        // this wavefront's LDS writes have landed; then count it
        __builtin_amdgcn_fence(__ATOMIC_RELEASE, "workgroup");
        if (lane == 0) __hip_atomic_fetch_add(&tables_built, 1u, __ATOMIC_RELEASE, __HIP_MEMORY_SCOPE_WORKGROUP);
        MSGEMM_TRACE(2);
        if constexpr (kDedicated) return;
        fill_ring(kEarlyBuilder, kRing);
    } else {
        fill_ring(0, kRing);
        MSGEMM_TRACE(1);
        MSGEMM_TRACE(2);
    }
    // every builder runs to its increment without waiting on anyone, so this ends
    while (__hip_atomic_load(&tables_built, __ATOMIC_ACQUIRE, __HIP_MEMORY_SCOPE_WORKGROUP) != (unsigned)kBuilders)
        __builtin_amdgcn_s_sleep(1);
    __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "workgroup");
    MSGEMM_TRACE(3);

    // ---- phase 2: stream panels, gather, accumulate
    const uint32_t class_base = (uint32_t)(16 * qg) * kEntryBytes;
    __amdgpu_buffer_rsrc_t part_rsrc =
        __builtin_amdgcn_make_buffer_rsrc((void*)a.partials, 0, (int)a.partial_span, 0x00020000);
    __amdgpu_buffer_rsrc_t scale_rsrc = __builtin_amdgcn_make_buffer_rsrc(
        (void*)(a.scales ? (const void*)a.scales : (const void*)a.tiled), 0, a.scales ? (int)a.scale_span : 0, 0x00020000);
    const uint32_t col_stride = (uint32_t)(a.m_pad * 4);            // bytes between columns of the partials
    const uint32_t tile_stride = (uint32_t)(a.b_pad * a.m_pad * 4); // bytes between k-tiles

    for (int pi = 0; pi < npan; ++pi) {
        const int panel_g = panel_first + wave + pi * kWaves;
        const int64_t row0 = (int64_t)panel_g * kPanelRows + lane;

        // scales of this k-tile's block for the rows this lane will own after the fold
        // (one contiguous load per wavefront: the plan keeps them in the order of the
        // outputs).  In the single-column kernels the load is an unconditional,
        // bounds-checked buffer load -- without scales the buffer is empty and it
        // returns at once, without a memory access -- and its value is first looked
        // at after the gather, so no wait for it sits in front of the code stream.
        struct alignas(2 * kFinal) PackedScales { __half h[kFinal]; };
        PackedScales qraw;
        if constexpr (__is_same(AT, float)) {
            const int64_t qat = (int64_t)scale_block * a.m_pad + (int64_t)panel_g * kPanelRows + lane * kFinal;
            const PackedScales* qp = (const PackedScales*)(a.scales + qat);
            if constexpr (C == 1) {
                static_assert(kFinal == 2 || kFinal == 4, "scales of a lane fit one 4- or 8-byte load");
                if constexpr (kFinal == 4) {
                    const v2u q = __builtin_amdgcn_raw_buffer_load_b64(scale_rsrc, (int)(qat * 2), 0, 0);
                    __builtin_memcpy(&qraw, &q, sizeof(qraw));
                } else {
                    const unsigned q = __builtin_amdgcn_raw_buffer_load_b32(scale_rsrc, (int)(qat * 2), 0, 0);
                    __builtin_memcpy(&qraw, &q, sizeof(qraw));
                }
            } else {
                // (the batched kernels have no registers to spare: a conditional load, waited for at once)
#pragma unroll
                for (int i = 0; i < kFinal; ++i) qraw.h[i] = __float2half(1.0f);
                if (a.scales) qraw = *qp;
            }
        }

        AT acc[LB][C];
#pragma unroll
        for (int s = 0; s < LB; ++s)
#pragma unroll
            for (int c = 0; c < C; ++c) acc[s][c] = 0;

        // One load's worth of look-ups is issued while the previous one's entries
        // are being added, so the LDS latency hides behind the adds without the
        // scheduler hoisting all 16*LB reads at once.
        const bool more = pi + 1 < npan;
        const LoadT* cur = stream + (int64_t)pi * kWaves * 64;
        auto issue = [&](int t, Entry (&dst)[LB]) {
            const uint32_t lane_off = class_base + (uint32_t)((j + t) & 15) * kEntryBytes;
            const LoadT d = ring[t % kRing];
#pragma unroll
            for (int s = 0; s < LB; ++s) {
                const uint32_t w = load_word<LB>(d, s >> 2);
                uint32_t addr;
                if constexpr (kCodeStride == 256)  // code byte drops straight into address bits 15:8
                    addr = __builtin_amdgcn_perm(w, lane_off, 0x0c0c0000u | ((4u + (s & 3)) << 8));
                else
                    addr = ((w >> (8 * (s & 3))) & 0xffu) * kCodeStride + lane_off;
                dst[s] = *(const Entry*)(lds + addr);
            }
            // the slot's bytes are now addresses: refill it with the load kRing ahead
            if (t + kRing < kLoadsPerPanel) {
                ring[t % kRing] = load_codes(cur + (t + kRing) * step_stride);
            } else if (more) {
                ring[t % kRing] = load_codes(cur + kWaves * 64 + (t + kRing - kLoadsPerPanel) * step_stride);
            }
        };
        auto consume = [&](int t, const Entry (&src)[LB]) {
#pragma unroll
            for (int s = 0; s < LB; ++s) {
#pragma unroll
                for (int c = 0; c < C; ++c) {
                    acc[s][c] += EntryAcc<ET>::widen(src[s].v[c]);
                    // pin the add to this stage: otherwise the compiler sinks all
                    // adds below the gather and keeps every table entry live
                    asm volatile("" : "+v"(acc[s][c]));
                }
            }
        };
        Entry e0[LB], e1[LB];
        issue(0, e0);
#pragma unroll
        for (int t = 0; t < kLoadsPerPanel; t += 2) {
            issue(t + 1, e1);
            consume(t, e0);
            __builtin_amdgcn_sched_barrier(0);
            if (t + 2 < kLoadsPerPanel) issue(t + 2, e0);
            consume(t + 1, e1);
            __builtin_amdgcn_sched_barrier(0);
        }
        MSGEMM_TRACE(4);

        // ---- lanes that share rows: fold the NQ group classes; each lane ends
        // up with kFinal distinct rows (64*i + lane); then the block scale (Section 3.3)
        const uint32_t part_off = (uint32_t)col0 * col_stride + (uint32_t)(panel_g * kPanelRows + lane * kFinal) * 4u;
        const bool in_launch = kInLaunchReduce<C> && a.reduce_mode == kReduceInLaunch;
#pragma unroll
        for (int c = 0; c < C; ++c) {
            AT fin[kFinal];
            if constexpr (NQ == 4) {
                AT half[LB / 2];
#pragma unroll
                for (int s = 0; s < LB / 2; ++s) half[s] = fold32(acc[s][c], acc[s + LB / 2][c]);
#pragma unroll
                for (int s = 0; s < kFinal; ++s) fin[s] = fold16(half[s], half[s + kFinal]);
            } else if constexpr (NQ == 2) {
#pragma unroll
                for (int s = 0; s < kFinal; ++s) fin[s] = fold16(acc[s][c], acc[s + kFinal][c]);
            } else {
#pragma unroll
                for (int s = 0; s < kFinal; ++s) fin[s] = acc[s][c];
            }
            unsigned out[kFinal];
#pragma unroll
            for (int i = 0; i < kFinal; ++i) {
                if constexpr (__is_same(AT, float)) fin[i] *= (a.scales ? __half2float(qraw.h[i]) : 1.0f);
                out[i] = bits_of(fin[i]);
            }
            if (a.reduce_mode == kReduceDirect) {
#pragma unroll
                for (int i = 0; i < kFinal; ++i) {
                    const int64_t row = row0 + 64 * i;
                    if (row < a.m && col0 + c < a.b) Y[(col0 + c) * a.ldy + row] = to_output<YT, AT>(fin[i]);
                }
            } else {
                const uint32_t off = (uint32_t)kt * tile_stride + part_off + (uint32_t)c * col_stride;
                if (in_launch) store_partials<kFinal, kAuxSc1>(part_rsrc, off, out);
                else store_partials<kFinal, 0>(part_rsrc, off, out);
            }
        }
        MSGEMM_TRACE(5);
        if (!in_launch) continue;
        // publish: partials acknowledged at the point of coherence, then the flag goes up
        wait_vmem();
        if (lane == 0 && a.publish)
            __hip_atomic_store(a.flags + ((int64_t)panel_g * a.col_passes + cp) * a.ktiles + kt, 1u, __ATOMIC_RELAXED,
                               __HIP_MEMORY_SCOPE_AGENT);
        MSGEMM_TRACE(6);
    }
}

// ---------------------------------------------------------------------------
// Long-k form of the single-column kernel.  When there are more (k-tile, row
// group) pairs than compute units, a workgroup takes a *segment* of consecutive
// k-tiles for its rows instead of one:
//   * two table buffers (2 x 64 KiB): the four builder wavefronts build the
//     tables of k-tile i + 1 while the eight streaming wavefronts gather from
//     those of k-tile i, so the activations -> table start-up is paid once per
//     workgroup and not once per k-tile;
//   * a streaming wavefront keeps the scaled sums of its (at most two) panels in
//     registers across the k-tiles: one partial sum per segment instead of one
//     per k-tile, and its ring of code loads runs on across k-tile boundaries;
//   * hand-over by counters in LDS, one pair per buffer: `built` (builder
//     wavefronts that have finished a generation) and `done` (streaming
//     wavefronts that have).  A builder waits for generation i - 2 to be consumed
//     before it overwrites its buffer; a streamer waits for generation i to be
//     built.  Each wait is for work that does not wait for the waiter: no cycle.
// Same code layout, look-up, fold, scale and reduction as fused_kernel with
// C = 1, G = 64, LB = 16.
constexpr int kLongWaves = 8, kLongBuilders = 4, kLongTableBytes = 65536;

// rounds of 16 slices that a reader of the resident reduction requests at once
#ifndef MSGEMM_WIDE_READ_ROUNDS
#define MSGEMM_WIDE_READ_ROUNDS 4
#endif
constexpr int kReadRounds = MSGEMM_WIDE_READ_ROUNDS;

// The resident reduction's reader (see fused_wide_kernel): this workgroup's share -- 1 / slices -- of its row group's
// outputs, read from all slices until every sum shows the launch's parity, added in slice order, written to Y.
// `reader` of `readers` wavefronts of the workgroup share the share, 64 outputs at a time.  Waits first until the
// workgroup's own streaming wavefronts have stored (`*stored` reaches `stored_target`).
template <typename YT, typename AT>
__device__ __forceinline__ void resident_reader(const FusedArgs& a, __amdgpu_buffer_rsrc_t part_rsrc, int sgm, int panel_first,
                                                int panels_here, int64_t col0, unsigned parity, int lane, unsigned* stored,
                                                unsigned stored_target, uint32_t col_stride, uint32_t tile_stride,
                                                int reader, int readers)
{
    constexpr int kPanelRows = 256;
    const int S = a.slices;
    const uint32_t rg_floats = (uint32_t)panels_here * kPanelRows;
    const uint32_t f0 = (uint32_t)sgm * (uint32_t)a.red_chunk;
    if (f0 >= rg_floats) return;
    const uint32_t f1 = min(f0 + (uint32_t)a.red_chunk, rg_floats);
    // this workgroup's own partial sums are on their way: the others' are about as far (polling from the start
    // would only add traffic)
    while (__hip_atomic_load(stored, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_WORKGROUP) < stored_target)
        __builtin_amdgcn_s_sleep(2);
    YT* __restrict__ Y = (YT*)a.Y;
    const uint32_t base = (uint32_t)col0 * col_stride + ((uint32_t)panel_first * kPanelRows + f0) * 4u;
    // lane (grp, pc): the 16-byte piece pc of a run of 16 pieces, the slices grp, grp + 4, grp + 8, ...
    const int grp = lane >> 4, pc = lane & 15;
    unsigned polls = 0;
    bool gave_up = false;
#pragma unroll 1
    for (uint32_t p0 = 64u * (uint32_t)reader; f0 + p0 < f1 && !gave_up; p0 += 64u * (uint32_t)readers) {
        const uint32_t p = p0 + (uint32_t)pc * 4u;
        const bool have = f0 + p < f1;
        AT sum[4] = {0, 0, 0, 0};
        // kRounds x 16 slices are requested at once (a sum over 56 slices is one trip through memory, not four
        // in a row); a round that has arrived is not requested again.  The sums are added in slice order whatever
        // order they arrive in.  Up to 16 slices take the single-round instance: code that a wavefront runs
        // through once is fetched from memory as it goes, and the longer instance costs a short launch 0.3 us.
        auto add_slices = [&](auto rounds_c) {
        constexpr int kRounds = decltype(rounds_c)::value;
#pragma unroll 1
        for (int sb = 0; sb < S; sb += 16 * kRounds) {
            v4u v[kRounds][4];
            uint32_t off[kRounds][4];
            bool live[kRounds][4];
            bool done[kRounds];  // (the same in all lanes)
#pragma unroll
            for (int r = 0; r < kRounds; ++r) {
                done[r] = sb + 16 * r >= S;  // nothing to read: no slice of this round exists
#pragma unroll
                for (int u = 0; u < 4; ++u) {
                    const int sl = sb + 16 * r + grp + 4 * u;
                    live[r][u] = have && sl < S;
                    off[r][u] = live[r][u] ? base + p * 4u + (uint32_t)sl * tile_stride : 0x7ffffff0u;  // (out of range: reads zero)
                    v[r][u] = v4u{0u, 0u, 0u, 0u};
                }
            }
#pragma unroll 1
            for (;;) {
                asm volatile("" ::: "memory");
#pragma unroll
                for (int r = 0; r < kRounds; ++r) {
                    if (done[r]) continue;
#pragma unroll
                    for (int u = 0; u < 4; ++u) v[r][u] = __builtin_amdgcn_raw_buffer_load_b128(part_rsrc, (int)off[r][u], 0, kAuxSc1);
                }
                bool all = true;
#pragma unroll
                for (int r = 0; r < kRounds; ++r) {
                    if (done[r]) continue;
                    bool arrived = true;
#pragma unroll
                    for (int u = 0; u < 4; ++u)
                        arrived &= !live[r][u] || ((v[r][u].x & v[r][u].y & v[r][u].z & v[r][u].w & 1u) == parity &&
                                                   ((v[r][u].x | v[r][u].y | v[r][u].z | v[r][u].w) & 1u) == parity);
                    done[r] = __builtin_amdgcn_ballot_w64(!arrived) == 0;
                    all &= done[r];
                }
                if (all) break;
                if (++polls >= a.poll_limit) {
                    gave_up = true;
                    break;
                }
                __builtin_amdgcn_s_sleep(1);
            }
            if (gave_up) break;
#pragma unroll
            for (int r = 0; r < kRounds; ++r) {
#pragma unroll
                for (int u = 0; u < 4; ++u) {  // (what is not live read as zero and adds nothing)
                    AT x;
                    untag_partial(x, live[r][u] ? v[r][u].x : 0u); sum[0] += x;
                    untag_partial(x, live[r][u] ? v[r][u].y : 0u); sum[1] += x;
                    untag_partial(x, live[r][u] ? v[r][u].z : 0u); sum[2] += x;
                    untag_partial(x, live[r][u] ? v[r][u].w : 0u); sum[3] += x;
                }
            }
        }
        };
        if (S <= 16) add_slices(std::integral_constant<int, 1>());
        else add_slices(std::integral_constant<int, kReadRounds>());
        if (gave_up) break;
        // the four slice classes, in a fixed order; 16-lane row r ends with output ((r & 1) << 1) | (r >> 1) of its pieces
        const AT total = fold16(fold32(sum[0], sum[1]), fold32(sum[2], sum[3]));
        const int e = ((grp & 1) << 1) | (grp >> 1);
        // partial sum f of a panel belongs to lane f / 4, output f % 4 of the producing wavefront: row 64 (f % 4) + f / 4
        const uint32_t f = f0 + p;
        const int64_t row = ((int64_t)panel_first + f / kPanelRows) * kPanelRows + (f % kPanelRows) / 4 + 64 * e;
        if (have && row < a.m && col0 < a.b) Y[col0 * a.ldy + row] = to_output<YT, AT>(total);
    }
    // gave up: some partial sum never arrived.  The plan's error word says so (msgemm_plan_check).
    if (gave_up && lane == 0) __hip_atomic_store(a.error, 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}

template <typename XT, typename YT, typename ET, int kValueMode>
__global__ void __launch_bounds__((kLongWaves + kLongBuilders) * 64)
fused_long_kernel(FusedArgs a)
{
    using AT = typename EntryAcc<ET>::type;
    constexpr int G = 64, LB = 16, NQ = 4, kFinal = 4, kPanelRows = 256;
    constexpr int kRing = kRingBytes / LB < kLoadsPerPanel ? kRingBytes / LB : kLoadsPerPanel;
    static_assert(sizeof(ET) == 4 && kLoadsPerPanel % kRing == 0, "entries are 4 bytes; ring period divides the panel");
    using LoadT = uint4;

    __shared__ __align__(16) unsigned char lds[2 * kLongTableBytes];
    __shared__ unsigned built[2], done[2];  // per table buffer: generations i with i & 1 == index
    __shared__ unsigned stored;         // resident reduction: streaming wavefronts whose partial sums are on their way
    __shared__ unsigned launch_parity;  // resident reduction: 2 | parity of this workgroup's launch count, once known

#define MSGEMM_ARG_NOW(x) asm volatile("" ::"s"(x))
    MSGEMM_ARG_NOW((uint64_t)a.tiled); MSGEMM_ARG_NOW((uint64_t)a.X); MSGEMM_ARG_NOW(a.ldx);
    MSGEMM_ARG_NOW((uint64_t)a.Y); MSGEMM_ARG_NOW(a.ldy); MSGEMM_ARG_NOW((uint64_t)a.scales);
    MSGEMM_ARG_NOW((uint64_t)a.partials); MSGEMM_ARG_NOW(a.m); MSGEMM_ARG_NOW(a.k); MSGEMM_ARG_NOW(a.b);
    MSGEMM_ARG_NOW(a.m_pad); MSGEMM_ARG_NOW(a.b_pad); MSGEMM_ARG_NOW(a.ktiles); MSGEMM_ARG_NOW(a.panels_total);
    MSGEMM_ARG_NOW(a.panels_per_wg); MSGEMM_ARG_NOW(a.col_passes); MSGEMM_ARG_NOW(a.row_groups);
    MSGEMM_ARG_NOW(a.xcd_map); MSGEMM_ARG_NOW(a.partial_span); MSGEMM_ARG_NOW(a.reduce_mode);
    MSGEMM_ARG_NOW(a.slices); MSGEMM_ARG_NOW(a.tiles_per_segment); MSGEMM_ARG_NOW(a.fused_wgs);
#undef MSGEMM_ARG_NOW

    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int wave = (tid >> 6) - kLongBuilders;  // streaming wavefront index; negative: builder
    const int q = lane >> 4, j = lane & 15;

    if ((int)blockIdx.x >= a.fused_wgs) {  // trailing workgroups: the reduction over the segments
        reduce_in_launch<YT, AT, kFinal>(a, (int)blockIdx.x - a.fused_wgs, tid >> 6, lane, lds);
        return;
    }
    int sgm, rg;
    {
        const uint32_t bid = blockIdx.x;
        if (a.xcd_map == kXcdMapColumnPasses) {
            if (!column_pass_order(a, bid, a.div_slices, a.slices, sgm, rg)) return;
        } else {
            const uint32_t n = a.xcd_map ? bid / kXcds : bid;
            const uint32_t nq = fast_div(n, a.div_slices);
            sgm = (int)(n - nq * (uint32_t)a.slices);
            rg = a.xcd_map ? (int)((bid % kXcds) + kXcds * nq) : (int)nq;
            if (rg >= a.row_groups) return;
        }
    }
    const int rb = (int)fast_div((uint32_t)rg, a.div_col_passes);
    const int cp = rg - rb * a.col_passes;
    const int64_t col0 = cp;
    const int kt0 = sgm * a.tiles_per_segment;
    const int ngen = min(a.ktiles - kt0, a.tiles_per_segment);  // >= 1: the host makes no empty segment

    const int panel_first = rb * a.panels_per_wg;
    int panels_here = a.panels_total - panel_first;
    if (panels_here > a.panels_per_wg) panels_here = a.panels_per_wg;
    const int active = panels_here < kLongWaves ? panels_here : kLongWaves;  // streaming wavefronts with work

    if (tid < 2) {
        built[tid] = 0;
        done[tid] = 0;
    }
    if (tid == 0) {
        stored = 0;
        launch_parity = 0;
    }
    __syncthreads();

    const uint32_t col_stride = (uint32_t)(a.m_pad * 4);
    const uint32_t tile_stride = (uint32_t)(a.b_pad * a.m_pad * 4);
    __amdgpu_buffer_rsrc_t part_rsrc =
        __builtin_amdgcn_make_buffer_rsrc((void*)a.partials, 0, (int)a.partial_span, 0x00020000);
    // the sums over the segments added by the workgroups of this launch (fused_wide_kernel describes the scheme)
    const bool resident = a.reduce_mode == kReduceResident;

    if (wave < 0) {
        // ---- builders: the tables of k-tile kt0 + i into buffer i & 1
        const XT* __restrict__ X = (const XT*)a.X;
        const int g = tid % G;
        const int part = tid / G;  // 0..3: this thread's high codes are part, part + 4, ...
        auto value_of = [&](unsigned nibble) -> AT {
            if constexpr (kValueMode == kValuesMap16) return code_value(a.values, nibble, AT());
            else return (AT)decode4(nibble);
        };
        // 8-bit codes: the 16 values behind each of this thread's high nibbles (see fused_kernel)
        float v256[kValueMode == kValuesMap256 ? 16 / kLongBuilders : 1][16];
        if constexpr (kValueMode == kValuesMap256) {
#pragma unroll
            for (int u = 0; u < 16 / kLongBuilders; ++u) {
#pragma unroll
                for (int v4 = 0; v4 < 4; ++v4) {
                    const float4 q = *(const float4*)(a.values256 + (part + u * kLongBuilders) * 16 + v4 * 4);
                    v256[u][v4 * 4 + 0] = q.x; v256[u][v4 * 4 + 1] = q.y;
                    v256[u][v4 * 4 + 2] = q.z; v256[u][v4 * 4 + 3] = q.w;
                }
            }
        }
        // resident reduction: this workgroup's launch count (the first builder wavefront alone reads and bumps it)
        const bool counts = resident && wave == -kLongBuilders;
        unsigned launches = 0;
        if (counts) launches = __hip_atomic_load(a.epochs + blockIdx.x, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        for (int i = 0; i < ngen; ++i) {
            const int64_t kk = ((int64_t)(kt0 + i) * G + g) * 2;
            const bool live = (col0 < a.b) && (kk < a.k);
            const XT* px = X + (live ? col0 * a.ldx + (kValueMode == kValuesMap256 ? (kk >> 1) : kk) : 0);
            const XT xr0 = px[0], xr1 = px[kValueMode == kValuesMap256 ? 0 : 1];  // requested before the wait below
            if (i >= 2) {
                // generation i - 2, the last to use this buffer, consumed by every streaming wavefront.
                // (One counter per buffer: a wavefront that runs ahead can only add to the other one.)
                const unsigned need = (unsigned)(i / 2) * (unsigned)active;
                while (__hip_atomic_load(&done[i & 1], __ATOMIC_ACQUIRE, __HIP_MEMORY_SCOPE_WORKGROUP) < need)
                    __builtin_amdgcn_s_sleep(1);
                __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "workgroup");
            }
            const AT x0 = live ? (AT)XTraits<XT>::load(&xr0) : (AT)0;
            const AT x1 = live ? (AT)XTraits<XT>::load(&xr1) : (AT)0;
            unsigned char* buf = lds + (i & 1) * kLongTableBytes;
#pragma unroll
            for (int u = 0; u < 16 / kLongBuilders; ++u) {
                const int c1 = part + u * kLongBuilders;
                unsigned char* dst = buf + (size_t)(c1 * 16) * 256 + g * 4;
                if constexpr (kValueMode == kValuesMap256) {
#pragma unroll
                    for (int c0 = 0; c0 < 16; ++c0) *(ET*)(dst + c0 * 256) = EntryAcc<ET>::make((AT)v256[u][c0] * x0);
                } else {
                    const AT hi = value_of((unsigned)c1) * x1;
#pragma unroll
                    for (int c0 = 0; c0 < 16; ++c0)
                        *(ET*)(dst + c0 * 256) = EntryAcc<ET>::make(mul_add(value_of((unsigned)c0), x0, hi));
                }
            }
            __builtin_amdgcn_fence(__ATOMIC_RELEASE, "workgroup");
            if (lane == 0) __hip_atomic_fetch_add(&built[i & 1], 1u, __ATOMIC_RELEASE, __HIP_MEMORY_SCOPE_WORKGROUP);
        }
        if (!resident) return;
        // ---- the builders turn readers: together 1 / slices of the row group's outputs
        unsigned par;
        if (counts) {
            launches += 1;
            par = 2u | (launches & 1u);
            if (lane == 0) {
                __hip_atomic_store(a.epochs + blockIdx.x, launches, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
                __hip_atomic_store(&launch_parity, par, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_WORKGROUP);
            }
        } else {
            // (the first builder publishes it without waiting on anyone)
            while ((par = __hip_atomic_load(&launch_parity, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_WORKGROUP)) == 0)
                __builtin_amdgcn_s_sleep(1);
        }
        resident_reader<YT, AT>(a, part_rsrc, sgm, panel_first, panels_here, col0, par & 1u, lane, &stored, (unsigned)active,
                                col_stride, tile_stride, wave + kLongBuilders, kLongBuilders);
        return;
    }
    if (wave >= active) return;  // nothing to stream; `done` and `stored` do not count this wavefront

    // ---- streamers
    YT* __restrict__ Y = (YT*)a.Y;
    const int npan = (panels_here - wave + kLongWaves - 1) / kLongWaves;  // 1 or 2
    const int64_t step_stride = (int64_t)a.ktiles * a.panels_total * 64;  // LoadT elements between loads
    auto unit_base = [&](int kt, int panel) {
        return (const LoadT*)a.tiled + ((int64_t)kt * a.panels_total + panel) * 64 + lane;
    };
    const LoadT* cur = unit_base(kt0, panel_first + wave);
    LoadT ring[kRing];
#pragma unroll
    for (int u = 0; u < kRing; ++u) {
        ring[u] = load_codes(cur + u * step_stride);
        __builtin_amdgcn_sched_barrier(0);  // loads return in issue order: keep slot 0 first
    }

    __amdgpu_buffer_rsrc_t scale_rsrc = __builtin_amdgcn_make_buffer_rsrc(
        (void*)(a.scales ? (const void*)a.scales : (const void*)a.tiled), 0, a.scales ? (int)a.scale_span : 0, 0x00020000);
    const uint32_t class_base = (uint32_t)(16 * (q % NQ)) * 4u;

    AT y_run[2][kFinal];
#pragma unroll
    for (int pi = 0; pi < 2; ++pi)
#pragma unroll
        for (int i = 0; i < kFinal; ++i) y_run[pi][i] = 0;

    for (int gen = 0; gen < ngen; ++gen) {
        const int kt = kt0 + gen;
        const int scale_block = kt / a.tiles_per_block;
        {
            const unsigned need = (unsigned)(gen / 2 + 1) * kLongBuilders;  // this buffer's generations so far, all builders
            while (__hip_atomic_load(&built[gen & 1], __ATOMIC_ACQUIRE, __HIP_MEMORY_SCOPE_WORKGROUP) < need)
                __builtin_amdgcn_s_sleep(1);
            __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "workgroup");
        }
        const uint32_t table_bit = (uint32_t)(gen & 1) << 16;  // which buffer: bit 16 of every LDS address
#pragma unroll
        for (int pi = 0; pi < 2; ++pi) {
            if (pi >= npan) break;
            const int panel_g = panel_first + wave + pi * kLongWaves;
            // where the ring continues after this panel
            const bool more = (pi + 1 < npan) || (gen + 1 < ngen);
            const LoadT* nxt = (pi + 1 < npan) ? cur + kLongWaves * 64
                             : (gen + 1 < ngen) ? unit_base(kt + 1, panel_first + wave) : cur;

            struct alignas(8) PackedScales { __half h[kFinal]; };
            PackedScales qraw;
            if constexpr (__is_same(AT, float)) {
                const int64_t qat = (int64_t)scale_block * a.m_pad + (int64_t)panel_g * kPanelRows + lane * kFinal;
                const v2u qv = __builtin_amdgcn_raw_buffer_load_b64(scale_rsrc, (int)(qat * 2), 0, 0);
                __builtin_memcpy(&qraw, &qv, sizeof(qraw));
            }

            AT acc[LB];
#pragma unroll
            for (int s = 0; s < LB; ++s) acc[s] = 0;
            auto issue = [&](int t, ET (&dst)[LB]) {
                const uint32_t lane_off = (class_base + (uint32_t)((j + t) & 15) * 4u) | table_bit;
                const LoadT d = ring[t % kRing];
#pragma unroll
                for (int s = 0; s < LB; ++s) {
                    const uint32_t w = load_word<LB>(d, s >> 2);
                    // code byte into address bits 15:8, the lane's group offset in bits 7:0, the buffer in bit 16
                    const uint32_t addr = __builtin_amdgcn_perm(w, lane_off, 0x0c020000u | ((4u + (s & 3)) << 8));
                    dst[s] = *(const ET*)(lds + addr);
                }
                if (t + kRing < kLoadsPerPanel) {
                    ring[t % kRing] = load_codes(cur + (t + kRing) * step_stride);
                } else if (more) {
                    ring[t % kRing] = load_codes(nxt + (t + kRing - kLoadsPerPanel) * step_stride);
                }
            };
            auto consume = [&](const ET (&src)[LB]) {
#pragma unroll
                for (int s = 0; s < LB; ++s) {
                    acc[s] += EntryAcc<ET>::widen(src[s]);
                    asm volatile("" : "+v"(acc[s]));  // keep the adds in their stage
                }
            };
            ET e0[LB], e1[LB];
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
            // fold the four group classes: each lane ends with rows 64 * i + lane; then the block scale (Section 3.3)
            AT half[LB / 2];
#pragma unroll
            for (int s = 0; s < LB / 2; ++s) half[s] = fold32(acc[s], acc[s + LB / 2]);
#pragma unroll
            for (int i = 0; i < kFinal; ++i) {
                AT fin = fold16(half[i], half[i + kFinal]);
                if constexpr (__is_same(AT, float)) fin *= (a.scales ? __half2float(qraw.h[i]) : 1.0f);
                y_run[pi][i] += fin;
            }
            cur = nxt;
        }
        // every look-up of this generation has returned (its value has been added)
        if (lane == 0) __hip_atomic_fetch_add(&done[gen & 1], 1u, __ATOMIC_RELEASE, __HIP_MEMORY_SCOPE_WORKGROUP);
    }

    // ---- one sum per (segment, row): Y, or a partial (with its flag, or tagged with the launch's parity)
    const bool in_launch = a.reduce_mode == kReduceInLaunch;
    unsigned par = 0;
    if (resident) {
        // (the first builder wavefront sets it when its last table is built: long before this point)
        while ((par = __hip_atomic_load(&launch_parity, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_WORKGROUP)) == 0)
            __builtin_amdgcn_s_sleep(1);
    }
#pragma unroll
    for (int pi = 0; pi < 2; ++pi) {
        if (pi >= npan) break;
        const int panel_g = panel_first + wave + pi * kLongWaves;
        if (a.reduce_mode == kReduceDirect) {
#pragma unroll
            for (int i = 0; i < kFinal; ++i) {
                const int64_t row = (int64_t)panel_g * kPanelRows + lane + 64 * i;
                if (row < a.m && col0 < a.b) Y[col0 * a.ldy + row] = to_output<YT, AT>(y_run[pi][i]);
            }
            continue;
        }
        unsigned out[kFinal];
#pragma unroll
        for (int i = 0; i < kFinal; ++i) out[i] = resident ? tag_partial(y_run[pi][i], par & 1u) : bits_of(y_run[pi][i]);
        const uint32_t off = (uint32_t)sgm * tile_stride + (uint32_t)col0 * col_stride +
                             (uint32_t)(panel_g * kPanelRows + lane * kFinal) * 4u;
        if (resident) {
            if (a.publish) store_partials<kFinal, kAuxSc1>(part_rsrc, off, out);  // (publish = 0, a test aid: the readers give up)
            continue;
        }
        if (in_launch) store_partials<kFinal, kAuxSc1>(part_rsrc, off, out);
        else store_partials<kFinal, 0>(part_rsrc, off, out);
        if (!in_launch) continue;
        wait_vmem();
        if (lane == 0 && a.publish)
            __hip_atomic_store(a.flags + ((int64_t)panel_g * a.col_passes + cp) * a.slices + sgm, 1u, __ATOMIC_RELAXED,
                               __HIP_MEMORY_SCOPE_AGENT);
    }
    // tell the workgroup's readers that this wavefront's sums are on their way
    if (resident && lane == 0) __hip_atomic_fetch_add(&stored, 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_WORKGROUP);
}

// ---------------------------------------------------------------------------
// Wide form of the single-column kernel, for problems whose (k-tile, panel)
// units are about as many as the device has streaming wavefronts (the 32 MiB
// GEMV: 2048 units on 256 compute units x 8 wavefronts).  There one launch is a
// single chain of latencies -- arguments, instructions, activations, tables,
// codes, partial sums, reduction -- and the chain is what this form shortens:
//   * every loop is kept rolled.  A wavefront runs through its part of the
//     kernel once, so straight-line code is fetched from memory line by line
//     behind the code stream (measured: about 0.2 us per KiB of code executed
//     once); the look-ups of a unit are a loop of four passes over a body of
//     kRing loads, the table build a loop over the high codes;
//   * a workgroup holds the tables of kTables (1 or 2) consecutive k-tiles at
//     once, 64 KiB each, nothing is reused: its streaming wavefronts are dealt
//     over the tables (wavefront w gathers from table w / (8 / kTables)), a
//     wavefront's work is one (k-tile, panel) unit, and with two tables half as
//     many partial sums per output leave the workgroup;
//   * the builders request the activations before any code load of the
//     workgroup is issued (the streaming wavefronts wait for that request, not
//     for its data), so the activations do not queue behind the codes;
//   * a streaming wavefront keeps kRing loads in flight: eight wavefronts times
//     four loads of 1 KiB is what a compute unit's memory pipeline holds; more
//     only blocks the wavefront at the issue of a load while look-ups wait.  A
//     workgroup with at most four streaming wavefronts (small problems: a 4096 x
//     4096 GEMV has two) keeps eight loads in flight per wavefront instead
//     (measured: 1024 x 1024 6.27 -> 5.76 us, 4096 x 4096 7.31 -> 6.89, 8192 x 2048
//     6.80 -> 6.41; with eight wavefronts 9.6 -> 10.0);
//   * the wavefronts of the two tables that share rows are added through LDS;
//   * the sums over the slices are added by the workgroups that produced them
//     (kReduceResident): each workgroup of a row group adds 1/slices of the row
//     group's outputs.  There are no flags, no acknowledgements and nothing to
//     clear: every 32-bit partial sum carries, in its lowest bit, the parity of
//     the launch that wrote it.  A workgroup keeps its own launch count in the
//     plan's memory (it alone reads and bumps it, so the counts of all
//     workgroups move in step and no count is shared), every slot is written in
//     every launch, so a slot shows the current parity exactly when this
//     launch's sum has arrived.  A workgroup writes its partial sums through to
//     memory and is done; a reader -- the first builder wavefront, which has
//     nothing else left to do -- reads its slots of all slices until all show
//     the parity, adds them in a fixed order (reproducible) and writes Y: one
//     trip through memory between the last partial sum and Y.  The bit costs a
//     floating-point partial sum its last mantissa bit (cleared before the add:
//     at most one unit in the last place of a partial sum, exact for sums that
//     do not need the bit) and an integer one a bit of range (a slice of 256
//     columns stays far inside).  A reader waits for workgroups of its own
//     launch, so the host takes this mode only when the whole grid is resident
//     at once; the wait is bounded all the same, and a wavefront that gives up
//     sets the plan's error word.  Otherwise a second launch adds the slices.
// Same code layout, look-up, fold and scale as fused_kernel with C = 1, G = 64,
// LB = 16.
constexpr int kWideWaves = 8, kWideBuilders = 4, kWideTableBytes = 65536;
#ifndef MSGEMM_WIDE_RING
#define MSGEMM_WIDE_RING 4
#endif
#ifndef MSGEMM_WIDE_RING_SPARSE
#define MSGEMM_WIDE_RING_SPARSE 8
#endif
// code loads in flight per streaming wavefront: of a workgroup with more than four of them, and of one with fewer
constexpr int kWideRing = MSGEMM_WIDE_RING, kWideRingSparse = MSGEMM_WIDE_RING_SPARSE;
// Measurement builds only (never the product): -DMSGEMM_WIDE_LEAVE_OUT=<bits> leaves parts of the wide form out, so that
// the time each part adds to a launch can be read off as a difference (the results are then wrong, of course):
// 1 the readers (nobody adds the partial sums), 2 the partial sums' stores, 4 the look-ups (their addresses are
// still formed and added), 8 the wait for the tables, 16 the wait for the activations' request.
#ifndef MSGEMM_WIDE_LEAVE_OUT
#define MSGEMM_WIDE_LEAVE_OUT 0
#endif
template <typename XT, typename YT, typename ET, int kValueMode, int kTables, int kRing>
__global__ void __launch_bounds__((kWideWaves + kWideBuilders) * 64)
fused_wide_kernel(FusedArgs a)
{
    using AT = typename EntryAcc<ET>::type;
    constexpr int G = 64, LB = 16, NQ = 4, kFinal = 4, kPanelRows = 256;
    // (kRing: code loads a wavefront keeps in flight)
    constexpr int kSlots = kWideWaves / kTables;  // streaming wavefronts per table = panels per workgroup at most
    static_assert(sizeof(ET) == 4 && (kTables == 1 || kTables == 2), "entries are 4 bytes; one or two tables");
    static_assert(kLoadsPerPanel % kRing == 0 && kRing % 2 == 0, "whole passes over the ring; entries alternate between two sets");
    using LoadT = uint4;

    __shared__ __align__(16) unsigned char lds[kTables * kWideTableBytes];
    __shared__ AT stage[kTables == 2 ? kSlots * kFinal * 64 : 1];  // sums of the second table's wavefronts
    __shared__ unsigned x_requested, built[kTables], staged[kSlots], stored;
    __shared__ unsigned launch_parity;  // 2 | parity of this workgroup's launch count, once known

#define MSGEMM_ARG_NOW(x) asm volatile("" ::"s"(x))
    MSGEMM_ARG_NOW((uint64_t)a.tiled); MSGEMM_ARG_NOW((uint64_t)a.X); MSGEMM_ARG_NOW(a.ldx);
    MSGEMM_ARG_NOW((uint64_t)a.Y); MSGEMM_ARG_NOW(a.ldy); MSGEMM_ARG_NOW((uint64_t)a.scales);
    MSGEMM_ARG_NOW((uint64_t)a.partials); MSGEMM_ARG_NOW((uint64_t)a.flags); MSGEMM_ARG_NOW(a.m); MSGEMM_ARG_NOW(a.k);
    MSGEMM_ARG_NOW(a.b); MSGEMM_ARG_NOW(a.m_pad); MSGEMM_ARG_NOW(a.b_pad); MSGEMM_ARG_NOW(a.ktiles);
    MSGEMM_ARG_NOW(a.panels_total); MSGEMM_ARG_NOW(a.panels_per_wg); MSGEMM_ARG_NOW(a.col_passes);
    MSGEMM_ARG_NOW(a.row_groups); MSGEMM_ARG_NOW(a.xcd_map); MSGEMM_ARG_NOW(a.partial_span);
    MSGEMM_ARG_NOW(a.reduce_mode); MSGEMM_ARG_NOW(a.slices); MSGEMM_ARG_NOW(a.red_chunk);
    MSGEMM_ARG_NOW(a.poll_limit); MSGEMM_ARG_NOW(a.publish);
#undef MSGEMM_ARG_NOW

    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int wave = (tid >> 6) - kWideBuilders;  // streaming wavefront index; negative: builder
    const int q = lane >> 4, j = lane & 15;

    int sgm, rg;
    {
        const uint32_t bid = blockIdx.x;
        if (a.xcd_map == kXcdMapColumnPasses) {
            if (!column_pass_order(a, bid, a.div_slices, a.slices, sgm, rg)) return;
        } else {
            const uint32_t n = a.xcd_map ? bid / kXcds : bid;
            const uint32_t nq = fast_div(n, a.div_slices);
            sgm = (int)(n - nq * (uint32_t)a.slices);
            rg = a.xcd_map ? (int)((bid % kXcds) + kXcds * nq) : (int)nq;
            if (rg >= a.row_groups) return;
        }
    }
    const int rb = (int)fast_div((uint32_t)rg, a.div_col_passes);
    const int cp = rg - rb * a.col_passes;
    const int64_t col0 = cp;
    const int kt0 = sgm * kTables;
    const int ntab = min(a.ktiles - kt0, kTables);  // >= 1: the host makes no empty slice

    const int panel_first = rb * a.panels_per_wg;   // (the host keeps panels_per_wg <= kSlots)
    int panels_here = a.panels_total - panel_first;
    if (panels_here > a.panels_per_wg) panels_here = a.panels_per_wg;

    if (tid < kTables) built[tid] = 0;
    if (tid < kSlots) staged[tid] = 0;
    if (tid == 0) {
        x_requested = 0;
        stored = 0;
        launch_parity = 0;
    }
    __syncthreads();  // nothing is in flight yet

    const uint32_t col_stride = (uint32_t)(a.m_pad * 4);            // bytes between columns of the partials
    const uint32_t tile_stride = (uint32_t)(a.b_pad * a.m_pad * 4); // bytes between slices
    __amdgpu_buffer_rsrc_t part_rsrc =
        __builtin_amdgcn_make_buffer_rsrc((void*)a.partials, 0, (int)a.partial_span, 0x00020000);

    if (wave < 0) {
        // ---- builders: activations first, then the tables of k-tiles kt0 .. kt0 + ntab - 1
        const XT* __restrict__ X = (const XT*)a.X;
        const int g = tid % G;
        const int part = __builtin_amdgcn_readfirstlane(tid / G);  // 0..3: this wavefront's high codes are part, part + 4, ...
        XT xr0[kTables], xr1[kTables];
        bool live[kTables];
#pragma unroll
        for (int tb = 0; tb < kTables; ++tb) {
            const int64_t kk = ((int64_t)(kt0 + tb) * G + g) * 2;
            live[tb] = (col0 < a.b) && (kk < a.k) && tb < ntab;
            const XT* px = X + (live[tb] ? col0 * a.ldx + (kValueMode == kValuesMap256 ? (kk >> 1) : kk) : 0);
            xr0[tb] = px[0];
            xr1[tb] = px[kValueMode == kValuesMap256 ? 0 : 1];
        }
        // this workgroup's launch count (resident reduction; the first builder wavefront alone reads and bumps it)
        const bool counts = wave == -kWideBuilders && a.reduce_mode == kReduceResident;
        unsigned launches = 0;
        if (counts) launches = __hip_atomic_load(a.epochs + blockIdx.x, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        // the requests are out (their data is not): now the streaming wavefronts may queue their codes
        __builtin_amdgcn_sched_barrier(0);
        if (lane == 0) __hip_atomic_fetch_add(&x_requested, 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_WORKGROUP);
        __builtin_amdgcn_sched_barrier(0);
        // a custom value map: lane i of the wavefront holds the value of pattern i, so that the value of a code
        // known only at run time is one cross-lane read (the map itself sits in scalar registers)
        float map_lane = 0.0f;
        if constexpr (kValueMode == kValuesMap16) {
#pragma unroll
            for (int i = 0; i < 16; ++i) map_lane = (lane == i) ? a.values.v[i] : map_lane;
        }
        auto value_const = [&](unsigned nibble) -> AT {  // nibble known at compile time
            if constexpr (kValueMode == kValuesMap16) return code_value(a.values, nibble, AT());
            else return (AT)decode4(nibble);
        };
        auto value_uniform = [&](int nibble) -> AT {     // nibble the same in all lanes
            if constexpr (kValueMode == kValuesMap16)
                return (AT)__uint_as_float(__builtin_amdgcn_readlane((int)__float_as_uint(map_lane), nibble));
            else
                return (AT)decode4((unsigned)nibble);
        };
        // 8-bit codes: the 16 values behind each of this thread's high nibbles, requested before the activations are
        // waited for (this form keeps the loop over the high nibbles unrolled: 64 values in registers)
        float v256[kValueMode == kValuesMap256 ? 16 / kWideBuilders : 1][16];
        if constexpr (kValueMode == kValuesMap256) {
#pragma unroll
            for (int u = 0; u < 16 / kWideBuilders; ++u) {
#pragma unroll
                for (int v4 = 0; v4 < 4; ++v4) {
                    const float4 qv = *(const float4*)(a.values256 + (part + u * kWideBuilders) * 16 + v4 * 4);
                    v256[u][v4 * 4 + 0] = qv.x; v256[u][v4 * 4 + 1] = qv.y;
                    v256[u][v4 * 4 + 2] = qv.z; v256[u][v4 * 4 + 3] = qv.w;
                }
            }
        }
#pragma unroll 1
        for (int tb = 0; tb < ntab; ++tb) {
            AT x0, x1;
            if constexpr (kTables == 2) {
                const bool lv = tb ? live[1] : live[0];
                const XT r0 = tb ? xr0[1] : xr0[0], r1 = tb ? xr1[1] : xr1[0];
                x0 = lv ? (AT)XTraits<XT>::load(&r0) : (AT)0;
                x1 = lv ? (AT)XTraits<XT>::load(&r1) : (AT)0;
            } else {
                x0 = live[0] ? (AT)XTraits<XT>::load(&xr0[0]) : (AT)0;
                x1 = live[0] ? (AT)XTraits<XT>::load(&xr1[0]) : (AT)0;
            }
            unsigned char* dst = lds + tb * kWideTableBytes + (size_t)(part * 16) * 256 + g * 4;
            if constexpr (kValueMode == kValuesMap256) {
#pragma unroll
                for (int u = 0; u < 16 / kWideBuilders; ++u)
#pragma unroll
                    for (int c0 = 0; c0 < 16; ++c0)
                        *(ET*)(dst + (size_t)(u * kWideBuilders * 16 + c0) * 256) = EntryAcc<ET>::make((AT)v256[u][c0] * x0);
            } else {
#pragma unroll 1
                for (int c1 = part; c1 < 16; c1 += kWideBuilders) {
                    const AT hi = value_uniform(c1) * x1;
#pragma unroll
                    for (int c0 = 0; c0 < 16; ++c0)
                        *(ET*)(dst + c0 * 256) = EntryAcc<ET>::make(mul_add(value_const((unsigned)c0), x0, hi));
                    dst += (size_t)(kWideBuilders * 16) * 256;
                }
            }
            __builtin_amdgcn_fence(__ATOMIC_RELEASE, "workgroup");
            if (lane == 0) __hip_atomic_fetch_add(&built[tb], 1u, __ATOMIC_RELEASE, __HIP_MEMORY_SCOPE_WORKGROUP);
        }
        if (!counts) return;

        // ---- the first builder wavefront turns reader: 1/slices of the row group's outputs
        launches += 1;
        const unsigned parity = launches & 1u;
        if (lane == 0) {
            __hip_atomic_store(a.epochs + blockIdx.x, launches, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
            // (the streaming wavefronts wait for this word before they store: nothing may come between the tables and it)
            __hip_atomic_store(&launch_parity, 2u | parity, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_WORKGROUP);
        }
        if (MSGEMM_WIDE_LEAVE_OUT & 1) return;
        resident_reader<YT, AT>(a, part_rsrc, sgm, panel_first, panels_here, col0, parity, lane, &stored,
                                (unsigned)panels_here, col_stride, tile_stride, 0, 1);
        return;
    }

    // ---- streamers: wavefront `slot` of table `tb` takes panel `slot` of the row group at k-tile kt0 + tb
    const int tb = wave / kSlots, slot = wave % kSlots;
    if (tb >= ntab || slot >= panels_here) return;  // nothing to stream
    const int kt = kt0 + tb;
    const int panel_g = panel_first + slot;
    const int64_t step_stride = (int64_t)a.ktiles * a.panels_total * 64;  // LoadT elements between loads
    const LoadT* nxt = (const LoadT*)a.tiled + ((int64_t)kt * a.panels_total + panel_g) * 64 + lane;
    // the activations are requested first (a handful of cycles: the builders do nothing before it)
    while (!(MSGEMM_WIDE_LEAVE_OUT & 16) &&
           __hip_atomic_load(&x_requested, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_WORKGROUP) < (unsigned)kWideBuilders)
        __builtin_amdgcn_s_sleep(0);
    LoadT ring[kRing];
#pragma unroll
    for (int u = 0; u < kRing; ++u) {
        ring[u] = load_codes(nxt);
        nxt += step_stride;
        __builtin_amdgcn_sched_barrier(0);  // loads return in issue order: keep slot 0 first
    }
    __amdgpu_buffer_rsrc_t scale_rsrc = __builtin_amdgcn_make_buffer_rsrc(
        (void*)(a.scales ? (const void*)a.scales : (const void*)a.tiled), 0, a.scales ? (int)a.scale_span : 0, 0x00020000);
    struct alignas(8) PackedScales { __half h[kFinal]; };
    PackedScales qraw;
    if constexpr (__is_same(AT, float)) {
        const int scale_block = (int)fast_div((uint32_t)kt, a.div_tiles_per_block);
        const int64_t qat = (int64_t)scale_block * a.m_pad + (int64_t)panel_g * kPanelRows + lane * kFinal;
        const v2u qv = __builtin_amdgcn_raw_buffer_load_b64(scale_rsrc, (int)(qat * 2), 0, 0);
        __builtin_memcpy(&qraw, &qv, sizeof(qraw));
    }
    // LDS address of a look-up: code byte in bits 15:8, the lane's group (16 (q % 4) + (j + t) % 16) in bits 7:2,
    // the table in bit 16
    const uint32_t addr_fixed = ((uint32_t)(16 * (q % NQ)) * 4u) | ((uint32_t)tb << 16);

    while (!(MSGEMM_WIDE_LEAVE_OUT & 8) &&
           __hip_atomic_load(&built[tb], __ATOMIC_ACQUIRE, __HIP_MEMORY_SCOPE_WORKGROUP) < (unsigned)kWideBuilders)
        __builtin_amdgcn_s_sleep(1);
    __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "workgroup");

    AT acc[LB];
    ET ent[2][LB];  // entries of the load being looked up and of the one before it, which is being added
#pragma unroll
    for (int s = 0; s < LB; ++s) {
        acc[s] = 0;
        ent[1][s] = 0;
    }
    // One pass over the ring: the look-ups of kRing loads.  The passes that refill the ring are a rolled loop in
    // which every step issues its load unconditionally (a branch around a load makes the compiler lose count of
    // the loads in flight and wait for all of them); the last pass, which has nothing left to request, is a
    // second copy of the body.
    auto ring_pass = [&](int t0, auto refill) {
#pragma unroll
        for (int u = 0; u < kRing; ++u) {
            // look-ups of load t0 + u ...
            const uint32_t lane_off = addr_fixed | ((uint32_t)((j + t0 + u) & 15) * 4u);
            const LoadT d = ring[u];
#pragma unroll
            for (int s = 0; s < LB; ++s) {
                const uint32_t w = load_word<LB>(d, s >> 2);
                const uint32_t addr = __builtin_amdgcn_perm(w, lane_off, 0x0c020000u | ((4u + (s & 3)) << 8));
                if (MSGEMM_WIDE_LEAVE_OUT & 4) set_bits(ent[u & 1][s], addr);
                else ent[u & 1][s] = *(const ET*)(lds + addr);
            }
            // ... its slot refilled with the load kRing ahead ...
            if constexpr (decltype(refill)::value) {
                ring[u] = load_codes(nxt);
                nxt += step_stride;
            }
            // ... while the entries of the load before it are added (the first time round: zeros)
#pragma unroll
            for (int s = 0; s < LB; ++s) {
                acc[s] += EntryAcc<ET>::widen(ent[(u & 1) ^ 1][s]);
                asm volatile("" : "+v"(acc[s]));  // keep the adds in their stage
            }
            __builtin_amdgcn_sched_barrier(0);
        }
    };
#pragma unroll 1
    for (int t0 = 0; t0 < kLoadsPerPanel - kRing; t0 += kRing) ring_pass(t0, std::true_type());
    ring_pass(kLoadsPerPanel - kRing, std::false_type());
#pragma unroll
    for (int s = 0; s < LB; ++s) acc[s] += EntryAcc<ET>::widen(ent[(kRing - 1) & 1][s]);

    // fold the four group classes: each lane ends with rows 64 * i + lane; then the block scale (Section 3.3)
    AT y_run[kFinal];
    {
        AT half[LB / 2];
#pragma unroll
        for (int s = 0; s < LB / 2; ++s) half[s] = fold32(acc[s], acc[s + LB / 2]);
#pragma unroll
        for (int i = 0; i < kFinal; ++i) {
            AT fin = fold16(half[i], half[i + kFinal]);
            if constexpr (__is_same(AT, float)) fin *= (a.scales ? __half2float(qraw.h[i]) : 1.0f);
            y_run[i] = fin;
        }
    }

    // ---- the two tables' wavefronts of a slot hold sums of the same rows: the second hands its to the first
    if constexpr (kTables == 2) {
        AT* mine = stage + slot * (kFinal * 64) + lane;
        if (tb == 1) {
#pragma unroll
            for (int i = 0; i < kFinal; ++i) mine[i * 64] = y_run[i];
            __builtin_amdgcn_fence(__ATOMIC_RELEASE, "workgroup");
            if (lane == 0) __hip_atomic_fetch_add(&staged[slot], 1u, __ATOMIC_RELEASE, __HIP_MEMORY_SCOPE_WORKGROUP);
            return;
        }
        if (ntab == 2) {
            // (that wavefront runs to its increment without waiting on this one)
            while (__hip_atomic_load(&staged[slot], __ATOMIC_ACQUIRE, __HIP_MEMORY_SCOPE_WORKGROUP) == 0)
                __builtin_amdgcn_s_sleep(1);
            __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "workgroup");
#pragma unroll
            for (int i = 0; i < kFinal; ++i) y_run[i] += mine[i * 64];
        }
    }

    // ---- one sum per (slice, row): Y, or a partial
    if (a.reduce_mode == kReduceDirect) {
        YT* __restrict__ Y = (YT*)a.Y;
#pragma unroll
        for (int i = 0; i < kFinal; ++i) {
            const int64_t row = (int64_t)panel_g * kPanelRows + lane + 64 * i;
            if (row < a.m && col0 < a.b) Y[col0 * a.ldy + row] = to_output<YT, AT>(y_run[i]);
        }
        return;
    }
    const bool resident = a.reduce_mode == kReduceResident;
    if ((!resident || a.publish) && !(MSGEMM_WIDE_LEAVE_OUT & 2)) {  // (publish = 0, a test aid: the readers find nothing and give up)
        unsigned out[kFinal];
        if (resident) {
            // (the launch count was read at the start of the kernel: long known by now)
            unsigned par;
            while ((par = __hip_atomic_load(&launch_parity, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_WORKGROUP)) == 0)
                __builtin_amdgcn_s_sleep(1);
#pragma unroll
            for (int i = 0; i < kFinal; ++i) out[i] = tag_partial(y_run[i], par & 1u);
        } else {
#pragma unroll
            for (int i = 0; i < kFinal; ++i) out[i] = bits_of(y_run[i]);
        }
        const uint32_t off = (uint32_t)sgm * tile_stride + (uint32_t)col0 * col_stride +
                             (uint32_t)(panel_g * kPanelRows + lane * kFinal) * 4u;
        if (resident) store_partials<kFinal, kAuxSc1>(part_rsrc, off, out);
        else store_partials<kFinal, 0>(part_rsrc, off, out);
    }
    // tell the workgroup's reader that these sums are on their way
    if (resident && lane == 0) __hip_atomic_fetch_add(&stored, 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_WORKGROUP);
}

// Second pass of the k-tile reduction.  A workgroup of kReduceWaves wavefronts
// owns 64 consecutive partial sums of one column; wavefront w adds the k-tiles
// t = w, w + kReduceWaves, ... in increasing order, the wavefront sums are then
// added in wavefront order: a fixed order, so the result is reproducible.
// Many small workgroups keep the loads of the whole pass in flight at once.
constexpr int kReduceWaves = 4;

// Slices a row has when the k-tiles were dealt evenly (batched pipelined form): row block r = row / rows was cut into
// the shares floor(r blocks / share) .. floor(((r + 1) blocks - 1) / share), and only that many of the `slices` slots
// were written.  rows = 0: every row has all slices.
struct DealtSlices {
    int rows, blocks, share;
};
__device__ __forceinline__ int slices_of_row(const DealtSlices& d, int64_t row, int slices)
{
    if (d.rows == 0) return slices;
    const int r = (int)(row / d.rows);
    return ((r + 1) * d.blocks - 1) / d.share - (r * d.blocks) / d.share + 1;
}

template <typename YT, typename AT, int F>
__global__ void __launch_bounds__(kReduceWaves * 64)
reduce_kernel(const float* __restrict__ partials, YT* __restrict__ Y, int64_t ldy, int64_t m, int64_t b,
              int64_t m_pad, int64_t b_pad, int ktiles, int64_t span, int quad_major, DealtSlices dealt)
{
    __shared__ AT wave_sum[kReduceWaves][64];
    const int lane = threadIdx.x & 63;
    const int w = threadIdx.x >> 6;
    const int64_t chunks_per_col = m_pad / 64;
    const int64_t chunk = blockIdx.x % chunks_per_col;  // 64 consecutive floats of the column
    const int64_t col = blockIdx.x / chunks_per_col;
    __amdgpu_buffer_rsrc_t rsrc = __builtin_amdgcn_make_buffer_rsrc((void*)partials, 0, (int)span, 0x00020000);
    const uint32_t tile_stride = (uint32_t)(b_pad * m_pad * 4);
    const uint32_t off0 = (uint32_t)(col * m_pad + chunk * 64 + lane) * 4u;
    ktiles = slices_of_row(dealt, chunk * 64, ktiles);  // (the 64 sums of a chunk belong to one panel, hence one row block)
    AT sum = 0;
    constexpr int kBatch = 8;
    for (int t0 = w; t0 < ktiles; t0 += kBatch * kReduceWaves) {
        unsigned v[kBatch];
#pragma unroll
        for (int u = 0; u < kBatch; ++u) {
            const int t = t0 + u * kReduceWaves;
            v[u] = __builtin_amdgcn_raw_buffer_load_b32(rsrc, t < ktiles ? (int)(off0 + (uint32_t)t * tile_stride) : 0x7ffffff0, 0, 0);
        }
        __builtin_amdgcn_sched_barrier(0);
#pragma unroll
        for (int u = 0; u < kBatch; ++u) {
            AT x;
            set_bits(x, v[u]);
            sum += x;
        }
    }
    wave_sum[w][lane] = sum;
    __syncthreads();
    if (w == 0) {
        AT total = wave_sum[0][lane];
#pragma unroll
        for (int i = 1; i < kReduceWaves; ++i) total += wave_sum[i][lane];
        // float f of a panel belongs to lane f / F, output i = f % F, i.e. row 64*i + lane
        const int64_t f = chunk * 64 + lane;
        const int64_t panel = f / (64 * F);
        const int in_panel = (int)(f % (64 * F));
        const int64_t row = panel * (64 * F) + 64 * (in_panel % F) + slot_owner(in_panel / F, quad_major);
        if (row < m) Y[col * ldy + row] = to_output<YT, AT>(total);
    }
}

// The same pass for few partial sums per output (at most kFewSlices): the kernel above would then be a
// great many workgroups with one load each.  Here a lane owns four consecutive partial sums of a column
// and requests all k-segments at once (16-byte loads); added in segment order.
constexpr int kFewSlices = 16;

template <typename YT, typename AT, int F, int kMax>
__global__ void __launch_bounds__(64)
reduce_few_kernel(const float* __restrict__ partials, YT* __restrict__ Y, int64_t ldy, int64_t m, int64_t b,
                  int64_t m_pad, int64_t b_pad, int slices, int64_t span, int quad_major, DealtSlices dealt)
{
    const int lane = threadIdx.x;
    const int64_t chunks_per_col = m_pad / 256;
    const int64_t chunk = blockIdx.x % chunks_per_col;  // 256 consecutive partial sums of the column
    const int64_t col = blockIdx.x / chunks_per_col;
    __amdgpu_buffer_rsrc_t rsrc = __builtin_amdgcn_make_buffer_rsrc((void*)partials, 0, (int)span, 0x00020000);
    const uint32_t tile_stride = (uint32_t)(b_pad * m_pad * 4);
    const uint32_t off0 = (uint32_t)(col * m_pad + chunk * 256 + lane * 4) * 4u;
    slices = slices_of_row(dealt, chunk * 256, slices);  // (256 consecutive sums belong to one row block)
    v4u v[kMax];  // kMax = 4, 8 or 16: the smallest that holds the segments
#pragma unroll
    for (int t = 0; t < kMax; ++t)
        v[t] = __builtin_amdgcn_raw_buffer_load_b128(rsrc, t < slices ? (int)(off0 + (uint32_t)t * tile_stride) : 0x7ffffff0, 0, 0);
    AT sum[4] = {0, 0, 0, 0};
#pragma unroll
    for (int t = 0; t < kMax; ++t) {  // (segments past the last read as zero: the load is out of the buffer's range)
        AT x;
        set_bits(x, v[t].x); sum[0] += x;
        set_bits(x, v[t].y); sum[1] += x;
        set_bits(x, v[t].z); sum[2] += x;
        set_bits(x, v[t].w); sum[3] += x;
    }
#pragma unroll
    for (int e = 0; e < 4; ++e) {
        // partial sum f of a panel belongs to lane f / F, output i = f % F, i.e. row 64*i + lane
        const int64_t f = chunk * 256 + lane * 4 + e;
        const int64_t panel = f / (64 * F);
        const int in_panel = (int)(f % (64 * F));
        const int64_t row = panel * (64 * F) + 64 * (in_panel % F) + slot_owner(in_panel / F, quad_major);
        if (row < m) Y[col * ldy + row] = to_output<YT, AT>(sum[e]);
    }
}

// One-off reorder of the row-major code bytes into streaming order:
// [load t][k-tile][panel][lane][LB], or, kPanelMajor, [panel][k-tile][load t][lane][LB]
// (a wavefront that runs through the k-tiles of its panel then reads one
// sequential stream; with LB = 8 the loads t and t + 1 of a lane sit side by side).
// kInverse: the other way round, streaming order back to row-major (for the entry points that read the
// weights row by row: the plan keeps no row-major copy of its own until one of them is called).
template <int G, int LB, bool kPanelMajor = false, bool kInverse = false>
__global__ void __launch_bounds__(256)
repack_kernel(uint8_t* __restrict__ codes, uint8_t* __restrict__ tiled, int64_t m, int64_t kbytes,
              int ktiles, int panels_total)
{
    constexpr int NQ = G / 16;
    constexpr int kPanelRows = (LB / NQ) * 64;
    const int64_t total = (int64_t)ktiles * panels_total * kLoadsPerPanel * 64 * LB;
    for (int64_t o = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; o < total;
         o += (int64_t)gridDim.x * blockDim.x) {
        int64_t r = o;
        const int s = (int)(r % LB); r /= LB;
        int64_t panel, kt;
        int t, lane;
        if constexpr (kPanelMajor && LB == 8) {
            // (the pipelined batched form with 8 rows per lane fetches two loads of a lane at once:
            // [panel][k-tile][load / 2][lane][load % 2][8])
            const int tp = (int)(r % 2); r /= 2;
            lane = (int)(r % 64); r /= 64;
            t = 2 * (int)(r % (kLoadsPerPanel / 2)) + tp; r /= kLoadsPerPanel / 2;
            kt = r % ktiles;
            panel = r / ktiles;
        } else if constexpr (kPanelMajor) {
            lane = (int)(r % 64); r /= 64;
            t = (int)(r % kLoadsPerPanel); r /= kLoadsPerPanel;
            kt = r % ktiles;
            panel = r / ktiles;
        } else {
            lane = (int)(r % 64); r /= 64;
            panel = r % panels_total; r /= panels_total;
            kt = r % ktiles;
            t = (int)(r / ktiles);
        }
        const int q = lane >> 4, j = lane & 15;
        const int qg = q % NQ;
        const int64_t row = panel * kPanelRows + panel_row<NQ, LB>(q, j, s);
        const int64_t byte = kt * G + 16 * qg + ((j + t) & 15);
        if constexpr (kInverse) {
            if (row < m && byte < kbytes) codes[row * kbytes + byte] = tiled[o];
        } else {
            tiled[o] = (row < m && byte < kbytes) ? codes[row * kbytes + byte] : (uint8_t)0;
        }
    }
}

// One-off reorder of the block scales ([m][nblocks]) into the order in which the
// lanes of the fused kernel hold their outputs: [block][panel][lane][output i],
// output i of lane l being row 64*i + l of the panel.  Rows past m get 1.
__global__ void __launch_bounds__(256)
repack_scales_kernel(const __half* __restrict__ scales, __half* __restrict__ ordered, int64_t m, int64_t m_pad,
                     int64_t nblocks, int panel_rows)
{
    const int64_t total = nblocks * m_pad;
    const int nfinal = panel_rows / 64;
    for (int64_t o = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; o < total;
         o += (int64_t)gridDim.x * blockDim.x) {
        const int64_t blk = o / m_pad;
        const int64_t f = o % m_pad;
        const int64_t panel = f / panel_rows;
        const int in_panel = (int)(f % panel_rows);
        const int64_t row = panel * panel_rows + 64 * (in_panel % nfinal) + in_panel / nfinal;
        ordered[o] = row < m ? scales[row * nblocks + blk] : __float2half(1.0f);
    }
}

struct ShapeChoice { int C, G, LB, entry_bytes, waves; };

// Which instantiation serves a problem.  Entries are full width (fp32 / int32)
// for one or two columns (the b = 1 GEMV streams from HBM and the table traffic
// is small) and 16 bits wide (fp16 / int16) with 8 columns per entry for wider
// batches, where the gather is bound by LDS bytes and VALU adds.  int16 holds
// the int8 table values exactly (|entry| <= 2048); fp16 entries round.
constexpr int64_t kColumnPassBytes = 64ll << 20;  // AUTO: up to this many code bytes x columns, one pass per column

ShapeChoice pick_shape(const Plan& p, int requested_variant)
{
    // rows_per_lane = 8 selects the 16-wavefront, 128-row-panel form of the single-column kernel (an option of the
    // plan; measured within 3 % of the default on the b = 1 GEMV)
    const int lb1 = p.opt.rows_per_lane == 8 ? 8 : 16;
    const bool narrow_ok = p.x_dtype != MSGEMM_F32;
    // A small batch on a small matrix runs the single-column kernels once per column (the passes of a unit side by
    // side on one XCD, full-width entries): the batched kernels cost two launches and a start-up that such a problem
    // never earns back.  Measured cross-over (fp16, scale blocks of 128; 3 to 8 columns on 1024 x 1024 to 16384 x
    // 4096): the passes win while columns x code bytes stay below some 70 MB -- 4096 x 4096 x 4 takes 8.3 us against
    // 14.2, 8192 x 4096 x 4 12.8 against 17.1, 8192 x 4096 x 6 20.0 against 17.4.
    const bool by_passes = requested_variant == MSGEMM_VARIANT_AUTO && p.b > 2 &&
                           (p.scale_group == 0 || p.scale_group % 128 == 0) &&
                           p.b * p.m * (p.k / 2) <= kColumnPassBytes;
    const bool narrow = requested_variant == MSGEMM_VARIANT_FUSED_LDS16 ||
                        (requested_variant == MSGEMM_VARIANT_AUTO && p.b > 2 && !by_passes);
    // (plan options: rows_per_lane = 4, the 12- resp. 16-wavefront form of the batched kernel; batched_form = 1, its
    // form with one 32-group table and a build phase per k-tile, 2 the pipelined one)
    if (narrow && narrow_ok) {
        // The batched kernel has two forms: 16-group k-tiles with the next table built under the
        // look-ups (pipelined), or 32-group k-tiles with a build phase.  Time models of both decide unless
        // the plan's options name one.
        const int pipe_default = batched_pipelined_is_faster(p.m, p.k, p.b, p.scale_group, p.cus) ? 1 : 0;
        const int lb = p.opt.rows_per_lane == 4 ? 4 : 8;
        if (p.opt.batched_form == 2 || (p.opt.batched_form != 1 && pipe_default))
            return lb == 4 ? ShapeChoice{8, 16, 4, 2, 16} : ShapeChoice{8, 16, 8, 2, 8};
        return lb == 4 ? ShapeChoice{8, 32, 4, 2, 12} : ShapeChoice{8, 32, 8, 2, 8};
    }
    if (p.b > 2 && p.x_dtype == MSGEMM_F32 && !by_passes) return ShapeChoice{4, 32, 8, 4, 8};
    return lb1 == 8 ? ShapeChoice{1, 64, 8, 4, 16} : ShapeChoice{1, 64, 16, 4, 8};
}

// Workgroups of `kern` (block threads, static LDS only) that one compute unit holds at once.
template <typename K> int resident_blocks_per_cu(K kern, int threads)
{
    int n = 0;
    if (hipOccupancyMaxActiveBlocksPerMultiprocessor(&n, kern, threads, 0) != hipSuccess) return 0;
    return n;
}

// Workgroups that do the fused work, by the order of their ids (ids past the last unit return at once).
static int fused_workgroups(const FusedArgs& a, int64_t slices)
{
    if (a.xcd_map == kXcdMapColumnPasses)
        return (int)(kXcds * a.col_passes * ((slices * a.row_blocks + kXcds - 1) / kXcds));
    if (a.xcd_map) return (int)(slices * kXcds * ((a.row_groups + kXcds - 1) / kXcds));
    return (int)(slices * a.row_groups);
}

template <typename XT, typename YT, typename ET, int C, int G, int LB, int kWaves, int kValueMode>
int launch_one(const Plan& p, FusedArgs& a, hipStream_t s)
{
    using AT = typename EntryAcc<ET>::type;
    constexpr int kFinal = LB / (G / 16);
    auto kern = fused_kernel<XT, YT, ET, C, G, LB, kWaves, kValueMode>;
    a.fused_wgs = fused_workgroups(a, (int64_t)p.ktiles);
    a.red_units = a.panels_total * a.col_passes;
    int64_t grid = a.fused_wgs;
    if (a.reduce_mode == kReduceInLaunch) grid += a.red_units;
    hipLaunchKernelGGL(kern, dim3((unsigned)grid), dim3((kWaves + dedicated_builders<C, kWaves>()) * 64), 0, s, a);
    MSGEMM_HIP_TRY(hipGetLastError());
    if (a.reduce_mode == kReduceSecondPass) {
        const int64_t blocks = (a.m_pad / 64) * a.b;
        hipLaunchKernelGGL((reduce_kernel<YT, AT, kFinal>), dim3((unsigned)blocks), dim3(kReduceWaves * 64), 0, s,
                           a.partials, (YT*)a.Y, a.ldy, a.m, a.b, a.m_pad, a.b_pad, a.slices, a.partial_span, 0, DealtSlices{0, 0, 0});
        MSGEMM_HIP_TRY(hipGetLastError());
    }
    return MSGEMM_OK;
}

template <typename XT, typename YT, typename ET, int kValueMode>
int launch_long(const Plan& p, FusedArgs& a, hipStream_t s)
{
    using AT = typename EntryAcc<ET>::type;
    auto kern = fused_long_kernel<XT, YT, ET, kValueMode>;
    a.fused_wgs = fused_workgroups(a, (int64_t)a.slices);
    if (a.reduce_mode == kReduceResident) {
        // the readers wait for workgroups of their own launch: only when all of them run at once; else trailing ones
        static const int per_cu = resident_blocks_per_cu(kern, (kLongWaves + kLongBuilders) * 64);  // once per instantiation
        if ((int64_t)a.fused_wgs > (int64_t)per_cu * p.cus) a.reduce_mode = kReduceInLaunch;
    }
    a.red_units = a.panels_total * a.col_passes;
    int64_t grid = a.fused_wgs;
    if (a.reduce_mode == kReduceInLaunch) grid += a.red_units;
    hipLaunchKernelGGL(kern, dim3((unsigned)grid), dim3((kLongWaves + kLongBuilders) * 64), 0, s, a);
    MSGEMM_HIP_TRY(hipGetLastError());
    if (a.reduce_mode == kReduceSecondPass) {
        const int64_t blocks = (a.m_pad / 64) * a.b;
        hipLaunchKernelGGL((reduce_kernel<YT, AT, 4>), dim3((unsigned)blocks), dim3(kReduceWaves * 64), 0, s,
                           a.partials, (YT*)a.Y, a.ldy, a.m, a.b, a.m_pad, a.b_pad, a.slices, a.partial_span, 0, DealtSlices{0, 0, 0});
        MSGEMM_HIP_TRY(hipGetLastError());
    }
    return MSGEMM_OK;
}

template <typename XT, typename YT, typename ET, int kValueMode, int kTables, int kRing>
int launch_wide(const Plan& p, FusedArgs& a, hipStream_t s)
{
    using AT = typename EntryAcc<ET>::type;
    auto kern = fused_wide_kernel<XT, YT, ET, kValueMode, kTables, kRing>;
    constexpr int kThreads = (kWideWaves + kWideBuilders) * 64;
    a.fused_wgs = fused_workgroups(a, (int64_t)a.slices);
    if (a.reduce_mode == kReduceResident) {
        // the readers wait for workgroups of their own launch: only when all of them run at once
        static const int per_cu = resident_blocks_per_cu(kern, kThreads);  // once per instantiation
        if ((int64_t)a.fused_wgs > (int64_t)per_cu * p.cus) a.reduce_mode = kReduceSecondPass;
    }
    hipLaunchKernelGGL(kern, dim3((unsigned)a.fused_wgs), dim3(kThreads), 0, s, a);
    MSGEMM_HIP_TRY(hipGetLastError());
    if (a.reduce_mode == kReduceSecondPass) {
        const int64_t blocks = (a.m_pad / 64) * a.b;
        hipLaunchKernelGGL((reduce_kernel<YT, AT, 4>), dim3((unsigned)blocks), dim3(kReduceWaves * 64), 0, s,
                           a.partials, (YT*)a.Y, a.ldy, a.m, a.b, a.m_pad, a.b_pad, a.slices, a.partial_span, 0, DealtSlices{0, 0, 0});
        MSGEMM_HIP_TRY(hipGetLastError());
    }
    return MSGEMM_OK;
}

template <typename XT, typename YT, typename ET, int kValueMode>
int launch_wide_tables(const Plan& p, FusedArgs& a, hipStream_t s)
{
    // streaming wavefronts of a workgroup that have a unit: panels x tables
    const int tables = p.wide_tables == 2 ? 2 : 1;
    const bool sparse = p.fs.panels * tables <= kWideWaves / 2;
    if (p.wide_tables == 2) {
        if (sparse) return launch_wide<XT, YT, ET, kValueMode, 2, kWideRingSparse>(p, a, s);
        return launch_wide<XT, YT, ET, kValueMode, 2, kWideRing>(p, a, s);
    }
    if (sparse) return launch_wide<XT, YT, ET, kValueMode, 1, kWideRingSparse>(p, a, s);
    return launch_wide<XT, YT, ET, kValueMode, 1, kWideRing>(p, a, s);
}

// integer tables have the one encoding; floating-point ones also a form that reads the plan's map
template <typename XT, typename YT, typename ET, int C, int G, int LB, int kWaves>
int launch_for_values(const Plan& p, FusedArgs& a, hipStream_t s)
{
    constexpr bool kFloatTables = !std::is_same<ET, int>::value;
    if (p.codes8) {  // 8-bit weights: the single-column kernels with 16 rows per lane, and the four-column fp32 one
        if constexpr (C == 1 && LB == 16 && kFloatTables) {
            if (p.wide_tables > 0) return launch_wide_tables<XT, YT, ET, kValuesMap256>(p, a, s);
            if (p.segments > 0) return launch_long<XT, YT, ET, kValuesMap256>(p, a, s);
            return launch_one<XT, YT, ET, C, G, LB, kWaves, kValuesMap256>(p, a, s);
        }
        if constexpr (C == 4 && kFloatTables) return launch_one<XT, YT, ET, C, G, LB, kWaves, kValuesMap256>(p, a, s);
        return MSGEMM_ERR_UNSUPPORTED;
    }
    if constexpr (C == 1 && LB == 16) {
        if (p.wide_tables > 0) {  // wide form: one or two tables per workgroup, a whole unit in flight per wavefront
            if constexpr (kFloatTables) {
                if (p.custom_values) return launch_wide_tables<XT, YT, ET, kValuesMap16>(p, a, s);
            }
            return launch_wide_tables<XT, YT, ET, kValuesDefault>(p, a, s);
        }
        if (p.segments > 0) {  // long-k form
            if constexpr (kFloatTables) {
                if (p.custom_values) return launch_long<XT, YT, ET, kValuesMap16>(p, a, s);
            }
            return launch_long<XT, YT, ET, kValuesDefault>(p, a, s);
        }
    }
    if constexpr (kFloatTables) {
        if (p.custom_values) return launch_one<XT, YT, ET, C, G, LB, kWaves, kValuesMap16>(p, a, s);
    }
    return launch_one<XT, YT, ET, C, G, LB, kWaves, kValuesDefault>(p, a, s);
}

}  // namespace

namespace {
// Panels per workgroup and k-tiles per workgroup of the single-column kernel.
// A workgroup's time is counted in units of one panel per streaming wavefront
// (8 panels of 16 KiB: about 5 us of a compute unit's share of the stream) plus
// half a unit for the activations -> table start-up, which the long-k form pays
// once per workgroup; the workgroups run in rounds over the compute units; a
// reduction over several slices costs a little at the end.  The cheapest of the
// candidates wins, the first of equals (more panels, shorter runs).
void choose_rows_and_segments(int64_t panels, int64_t ktiles, int col_passes, int cus, int& ppw_out, int64_t& tps_out)
{
    double best = 1e300;
    for (int ppw = 2 * kLongWaves; ppw >= 1; ppw >>= 1) {
        const int64_t row_groups = ((panels + ppw - 1) / ppw) * col_passes;
        const int64_t here = panels < ppw ? panels : ppw;
        // (up to four panels: as many wavefronts stream, and what they keep in flight bounds the compute unit's rate)
        const double per_tile = here > 4 ? (double)here / kLongWaves : 0.57;
        int64_t last_tps = 0;
        for (int64_t segs = ktiles; segs >= 1; segs = segs > 4 * (int64_t)cus ? 4 * (int64_t)cus : segs - 1) {
            const int64_t tps = (ktiles + segs - 1) / segs;
            if (tps == last_tps) continue;
            last_tps = tps;
            if (tps > 1 && ppw < kLongWaves) break;  // runs of k-tiles only with every streaming wavefront at work
            const int64_t n_seg = (ktiles + tps - 1) / tps;
            const int64_t wgs = row_groups * n_seg;
            const double rounds = wgs <= 4 * (int64_t)cus ? (double)((wgs + cus - 1) / cus) : (double)wgs / cus + 0.5;
            const double idle = wgs < cus ? 0.2 * (double)(cus - wgs) / cus : 0.0;  // equal otherwise: the wider spread wins
            // (rounds do not line up as neatly as counted.  Sixteen panels over one or two k-tiles lose a tie against
            // eight panels over twice the k-tiles -- the same work with half the partial sums per output: 1 - 7 % faster
            // on 28672 x 4096, 16384 x 8192, 8192 x 28672, 17 % on 6144 x 16384 -- while runs of four k-tiles and more keep
            // sixteen: 49152 x 12288 is 7 % slower with eight.)
            const double cost = rounds * ((double)tps * per_tile + 0.5) + (n_seg > 1 ? 0.3 : 0.0) + idle + 0.1 * (rounds - 1.0) +
                                ((ppw > kLongWaves && tps <= 2) ? 0.1 : 0.0);
            if (cost < best - 1e-9) {
                best = cost;
                ppw_out = ppw;
                tps_out = tps;
            }
        }
    }
}
}  // namespace

int fused_choose_shape(Plan& p, int requested_variant)
{
    p.d3 = false;
    if (p.d == 3 && requested_variant == MSGEMM_VARIANT_FUSED_LDS) {
        // depth 3 with the tables in LDS: on request only (the measured point beside d = 2; never the faster one)
        const int rc = depth3_choose_shape(p);
        if (rc == MSGEMM_OK) p.d3 = true;
        return rc;
    }
    if (p.d != 2) return MSGEMM_ERR_UNSUPPORTED;
    if (requested_variant == MSGEMM_VARIANT_FUSED_LDS16 && p.x_dtype == MSGEMM_F32) return MSGEMM_ERR_UNSUPPORTED;
    p.xcd_map_allowed = p.opt.no_xcd_map ? 0 : 1;
    p.forced_reduce = p.opt.reduce_mode;
    {
        int cus = 256;
        hipDeviceProp_t prop;
        if (hipGetDeviceProperties(&prop, p.device) == hipSuccess && prop.multiProcessorCount > 0)
            cus = prop.multiProcessorCount;
        p.cus = cus;
    }
    const ShapeChoice sc = pick_shape(p, requested_variant);
    const int cols_per_tile = 2 * sc.G;
    if (p.scale_group > 0 && (p.scale_group % cols_per_tile) != 0) return MSGEMM_ERR_UNSUPPORTED;
    FusedShape& fs = p.fs;
    fs.groups = sc.G;
    fs.lane_bytes = sc.LB;
    fs.cols = sc.C;
    fs.entry_bytes = sc.entry_bytes;
    fs.waves = sc.waves;
    fs.panel_rows = (sc.LB / (sc.G / 16)) * 64;
    fs.lds_bytes = (size_t)256 * sc.G * sc.C * sc.entry_bytes;
    p.ktiles = (p.k / 2 + sc.G - 1) / sc.G;
    p.col_passes = (int)((p.b + sc.C - 1) / sc.C);
    const int64_t panels = (p.m + fs.panel_rows - 1) / fs.panel_rows;
    if (panels > (1 << 30) || p.ktiles > (1 << 20)) return MSGEMM_ERR_UNSUPPORTED;

    const int cus = p.cus;
    // Rows per table build: as many panels per workgroup as still leave one
    // workgroup per compute unit (each build costs 256 entries per group).
    // The plan's option panels_per_workgroup overrides the choice.
    // (The batched 16-bit kernel keeps one panel per wavefront and runs through
    // several k-tiles instead; its split over k is chosen below.)
    const bool batched16 = sc.entry_bytes == 2;
    const bool can_run_long = !batched16 && sc.C == 1 && sc.LB == 16;  // the long-k form exists for this kernel
    int ppw = batched16 ? sc.waves : 2 * sc.waves;
    while (ppw > 1 && (int64_t)p.ktiles * p.col_passes * ((panels + ppw - 1) / ppw) < cus) ppw >>= 1;
    int64_t tps = 1;
    if (can_run_long) choose_rows_and_segments(panels, p.ktiles, p.col_passes, cus, ppw, tps);
    const bool batched_pipe = batched16 && sc.G == 16;
    p.segments = 0;
    p.tiles_per_segment = 0;
    if (batched_pipe) batched_choose_rows_and_segments(p, panels, ppw);
    // (the batched form with a build phase, 8 rows per lane: the count between two halvings that its time model prefers)
    if (batched16 && !batched_pipe && sc.LB == 8)
        ppw = batched_phase_form_panels(panels, p.ktiles, p.scale_group, p.col_passes, cus);
    // Eight panels of one k-tile per workgroup and four panels of two are the same workgroups with the same
    // work; the second form halves the partial sums per output (measured on the 32 MiB GEMV: 10.8 -> 10.55 us).
    // The same for four panels (8192 x 4096: 7.73 -> 7.50 us); for two only when the sum runs over many k-tiles
    // (2048 x 8192, 64 k-tiles: 8.27 -> 7.6; 4096 x 4096, 32 k-tiles: 6.89 -> 7.1, so not there): a table built
    // for a single panel is on the critical path of a short launch.
    if (can_run_long && tps == 1 && ppw <= kWideWaves && ppw % 2 == 0 && (ppw >= 4 || p.ktiles >= 64) && p.ktiles >= 2 &&
        p.opt.k_tiles_per_workgroup == 0 && p.opt.panels_per_workgroup == 0) {
        ppw /= 2;
        tps = 2;
    }
    const int forced = p.opt.panels_per_workgroup;
    if (forced >= 1 && forced <= 64 && !batched_pipe) ppw = forced;
    // k_tiles_per_workgroup = 1 keeps one k-tile per workgroup, n > 1 forces runs of n.
    const int forced_tps = p.opt.k_tiles_per_workgroup;
    if (forced_tps >= 1) tps = forced_tps < p.ktiles ? forced_tps : p.ktiles;
    fs.panels = ppw;
    fs.tile_rows = ppw * fs.panel_rows;
    p.row_blocks = (panels + ppw - 1) / ppw;
    p.m_pad = panels * fs.panel_rows;
    const int64_t row_groups = p.row_blocks * p.col_passes;
    if ((int64_t)p.ktiles * (row_groups + kXcds) + (panels + kXcds) * p.col_passes > 0x7fffffffLL) return MSGEMM_ERR_UNSUPPORTED;
    // the k-tile reduction addresses the partial buffer with 32-bit byte offsets
    if (batched16 && !batched_pipe) batched_choose_segments(p);
    // The single-column kernel's forms: wide with one table (one k-tile, up to eight panels per workgroup), wide
    // with two (two k-tiles, up to four panels), long-k (runs of k-tiles through two table buffers; a streaming
    // wavefront holds the sums of at most two panels), and the plain one (one k-tile, up to sixteen panels).
    p.wide_tables = 0;
    if (can_run_long && tps == 1 && ppw <= kWideWaves) {
        p.wide_tables = 1;
    } else if (can_run_long && tps == 2 && ppw <= kWideWaves / 2 && p.ktiles >= 2) {
        p.wide_tables = 2;
        p.tiles_per_segment = 2;
        p.segments = (int)((p.ktiles + 1) / 2);
    } else if (can_run_long && ppw <= 2 * kLongWaves && tps >= 2) {
        p.tiles_per_segment = (int)tps;
        p.segments = (int)((p.ktiles + tps - 1) / tps);
    }
    const int64_t slices = p.segments > 0 ? p.segments : p.ktiles;
    if (slices * p.col_passes * sc.C * p.m_pad * 4 >= 0x7fffffffLL) return MSGEMM_ERR_UNSUPPORTED;
    if (p.nblocks * p.m_pad * 4 >= 0x7fffffffLL) return MSGEMM_ERR_UNSUPPORTED;
    return MSGEMM_OK;
}

// Row-major code bytes -> the plan's streaming order (inverse: back again, without touching scales).
static int repack_codes(const Plan& p, uint8_t* row_major, bool inverse, hipStream_t s)
{
    const int64_t panels = p.m_pad / p.fs.panel_rows;
    const int64_t total = (int64_t)p.ktiles * p.m_pad * p.fs.groups;
    int64_t blocks = (total + 255) / 256;
    if (blocks > 65536) blocks = 65536;
#define MSGEMM_REPACK(GG, LL, PM)                                                                                  \
    if (p.fs.groups == GG && p.fs.lane_bytes == LL) {                                                              \
        if (inverse)                                                                                               \
            hipLaunchKernelGGL((repack_kernel<GG, LL, PM, true>), dim3((unsigned)blocks), dim3(256), 0, s, row_major, \
                               p.codes_tiled, p.m, p.k / 2, (int)p.ktiles, (int)panels);                           \
        else                                                                                                       \
            hipLaunchKernelGGL((repack_kernel<GG, LL, PM, false>), dim3((unsigned)blocks), dim3(256), 0, s, row_major, \
                               p.codes_tiled, p.m, p.k / 2, (int)p.ktiles, (int)panels);                           \
        MSGEMM_HIP_TRY(hipGetLastError());                                                                         \
        return MSGEMM_OK;                                                                                          \
    }
    MSGEMM_REPACK(64, 16, false)
    MSGEMM_REPACK(64, 8, false)
    MSGEMM_REPACK(32, 8, false)
    MSGEMM_REPACK(32, 4, false)
    MSGEMM_REPACK(16, 8, true)
    MSGEMM_REPACK(16, 4, true)
#undef MSGEMM_REPACK
    return MSGEMM_ERR_UNSUPPORTED;
}

int launch_repack(const Plan& p, const void* W_codes, hipStream_t s)
{
    if (p.scales && p.fs.entry_bytes == 2) {
        const int rc = launch_repack_scales_batched(p, s);
        if (rc != MSGEMM_OK) return rc;
    } else if (p.scales) {
        int64_t sblocks = (p.nblocks * p.m_pad + 255) / 256;
        if (sblocks > 65536) sblocks = 65536;
        hipLaunchKernelGGL(repack_scales_kernel, dim3((unsigned)sblocks), dim3(256), 0, s, (const __half*)p.scales,
                           (__half*)p.scales_ordered, p.m, p.m_pad, p.nblocks, p.fs.panel_rows);
        MSGEMM_HIP_TRY(hipGetLastError());
    }
    return repack_codes(p, (uint8_t*)W_codes, false, s);  // (read only in this direction)
}

int launch_unpack(const Plan& p, uint8_t* row_major, hipStream_t s) { return repack_codes(p, row_major, true, s); }

int launch_reduce_second_pass(const Plan& p, const float* partials, void* Y, int64_t ldy, int slices,
                              int64_t span, hipStream_t s)
{
    DealtSlices dealt{0, 0, 0};
    if (p.deal_blocks > 0) {
        const int tpb = p.scale_group > 0 ? (int)(p.scale_group / (2 * p.fs.groups)) : 1;
        dealt = DealtSlices{p.fs.tile_rows, (int)((p.ktiles + tpb - 1) / tpb), p.deal_blocks};
    }
    const int64_t b_pad = (int64_t)p.col_passes * p.fs.cols;
    const dim3 grid((unsigned)((p.m_pad / 64) * p.b)), blk(kReduceWaves * 64);
    const int f = p.fs.panel_rows / 64;  // outputs per lane of the producing kernel: 8, 4 or 2
    const int qm = p.fs.entry_bytes == 2;  // the batched kernels store their sums quad-major (slot_owner)
    const bool few = slices <= kFewSlices && p.m_pad % 256 == 0;
    const dim3 fgrid((unsigned)((p.m_pad / 256) * p.b)), fblk(64);
#define MSGEMM_REDUCE_FEW(YT, AT, FF)                                                                           \
    do {                                                                                                        \
        if (slices <= 4)                                                                                        \
            hipLaunchKernelGGL((reduce_few_kernel<YT, AT, FF, 4>), fgrid, fblk, 0, s, partials, (YT*)Y, ldy, p.m, p.b,  \
                               p.m_pad, b_pad, slices, span, qm, dealt);                                               \
        else if (slices <= 8)                                                                                   \
            hipLaunchKernelGGL((reduce_few_kernel<YT, AT, FF, 8>), fgrid, fblk, 0, s, partials, (YT*)Y, ldy, p.m, p.b,  \
                               p.m_pad, b_pad, slices, span, qm, dealt);                                               \
        else                                                                                                    \
            hipLaunchKernelGGL((reduce_few_kernel<YT, AT, FF, 16>), fgrid, fblk, 0, s, partials, (YT*)Y, ldy, p.m, p.b, \
                               p.m_pad, b_pad, slices, span, qm, dealt);                                               \
    } while (0)
#define MSGEMM_REDUCE(YT, AT)                                                                                   \
    if (few && f == 8) MSGEMM_REDUCE_FEW(YT, AT, 8);                                                            \
    else if (few && f == 4) MSGEMM_REDUCE_FEW(YT, AT, 4);                                                       \
    else if (few) MSGEMM_REDUCE_FEW(YT, AT, 2);                                                                 \
    else if (f == 8)                                                                                            \
        hipLaunchKernelGGL((reduce_kernel<YT, AT, 8>), grid, blk, 0, s, partials, (YT*)Y, ldy, p.m, p.b, p.m_pad, \
                           b_pad, slices, span, qm, dealt);                                                      \
    else if (f == 4)                                                                                            \
        hipLaunchKernelGGL((reduce_kernel<YT, AT, 4>), grid, blk, 0, s, partials, (YT*)Y, ldy, p.m, p.b, p.m_pad, \
                           b_pad, slices, span, qm, dealt);                                                      \
    else                                                                                                        \
        hipLaunchKernelGGL((reduce_kernel<YT, AT, 2>), grid, blk, 0, s, partials, (YT*)Y, ldy, p.m, p.b, p.m_pad, \
                           b_pad, slices, span, qm, dealt);
    switch (p.y_dtype) {
    case MSGEMM_F32: MSGEMM_REDUCE(float, float) break;
    case MSGEMM_F16: MSGEMM_REDUCE(__half, float) break;
    case MSGEMM_BF16: MSGEMM_REDUCE(bf16_t, float) break;
    case MSGEMM_I32: MSGEMM_REDUCE(int, int) break;
    default:
        return MSGEMM_ERR_INVALID_ARG;
    }
#undef MSGEMM_REDUCE
#undef MSGEMM_REDUCE_FEW
    MSGEMM_HIP_TRY(hipGetLastError());
    return MSGEMM_OK;
}

int launch_fused(const Plan& p, const void* X, int64_t ldx, void* Y, int64_t ldy, hipStream_t s)
{
    if (p.d3) return launch_depth3(p, X, ldx, Y, ldy, s);
    if (p.fs.entry_bytes == 2) return launch_batched(p, X, ldx, Y, ldy, s);
    FusedArgs a;
    a.tiled = p.codes_tiled;
    a.X = X; a.ldx = ldx; a.Y = Y; a.ldy = ldy;
    for (int i = 0; i < 16; ++i) a.values.v[i] = p.values[i];
    a.values256 = p.values256;
    a.scales = (const __half*)p.scales_ordered;
    a.partials = p.partials;
    a.flags = p.flags;
    a.error = p.error_word;
    a.epochs = p.epochs;
    a.poll_limit = p.opt.poll_limit > 0 ? (unsigned)p.opt.poll_limit : kMaxFlagPolls;
    a.publish = p.opt.skip_publish ? 0 : 1;
    a.m = p.m; a.k = p.k; a.b = p.b; a.m_pad = p.m_pad;
    a.b_pad = (int64_t)p.col_passes * p.fs.cols;
    a.ktiles = (int)p.ktiles;
    a.panels_total = (int)(p.m_pad / p.fs.panel_rows);
    a.panels_per_wg = p.fs.panels;
    a.row_blocks = (int)p.row_blocks;
    a.col_passes = p.col_passes;
    a.row_groups = (int)(p.row_blocks * p.col_passes);
    // Workgroups are dealt to the XCDs round-robin by id.  Giving the k-tiles of
    // one row block ids that are congruent modulo the XCD count keeps the traffic
    // on their shared counter and partials on one L2 slice.  Purely a locality
    // choice: the accesses are agent-coherent wherever the workgroups land.
    // (Only when the row groups divide evenly over the XCDs: otherwise some XCDs
    // would get twice the workgroups of others.)
    a.xcd_map = (a.row_groups % kXcds == 0 && p.xcd_map_allowed) ? 1 : 0;
    if (a.col_passes > 1 && p.xcd_map_allowed) a.xcd_map = kXcdMapColumnPasses;  // (any shape: units, not row groups, are dealt)
    a.nblocks = p.nblocks;
    a.slices = p.segments > 0 ? p.segments : (int)p.ktiles;
    a.tiles_per_segment = p.segments > 0 ? p.tiles_per_segment : 1;
    a.div_slices = make_fastdiv((uint32_t)a.slices);
    a.partial_span = (int64_t)a.slices * a.b_pad * p.m_pad * 4;
    a.scale_span = p.nblocks * p.m_pad * 2;  // nblocks <= ktiles: within the bound checked for the partials
    a.tiles_per_block = p.scale_group > 0 ? (int)(p.scale_group / (2 * p.fs.groups)) : 1;
    a.div_ktiles = make_fastdiv((uint32_t)a.ktiles);
    a.div_col_passes = make_fastdiv((uint32_t)a.col_passes);
    a.div_tiles_per_block = make_fastdiv((uint32_t)a.tiles_per_block);
    // Several k-tiles: the single-column kernels reduce inside the launch (a second
    // launch costs more than the reduction itself), the batched ones in a second
    // pass.  The plan's option reduce_mode = 1 (second pass) or 2 (in launch) overrides the
    // choice for the single-column kernels.
    a.reduce_mode = kReduceDirect;
    a.red_chunk = 0;
    if (a.slices > 1) {
        // (the wide form adds in its own workgroups, the others in trailing ones: requests for either in-launch
        // mode get the one the kernel has)
        // (the long-k form has both in-launch modes.  Its own workgroups add sums of up to 24 slices -- measured:
        // 28672 x 4096, 16 slices, 15.2 -> 14.6 us, 22016 x 4096 14.3 -> 13.2, 24576 x 6144 18.8 -> 17.9, 13824 x 5120,
        // 20 slices, 14.1 -> 13.4 -- and trailing workgroups longer ones: 8192 x 16384, 64 slices, 16.3 against 17.0,
        // 16384 x 16384, 32 slices, 26.2 against 26.7.  reduce_mode = 2 or 3 asks for one of them.)
        const bool long_form = p.wide_tables == 0 && p.segments > 0 && p.fs.cols == 1 && p.fs.lane_bytes == 16;
        int in_launch = p.wide_tables > 0 ? kReduceResident : kReduceInLaunch;
        if (long_form && p.epochs && p.forced_reduce != kReduceInLaunch &&
            (p.forced_reduce == kReduceResident || a.slices <= 24))
            in_launch = kReduceResident;
        a.reduce_mode = p.fs.cols == 1 ? in_launch : kReduceSecondPass;
        if (p.fs.cols == 1 && p.forced_reduce == kReduceSecondPass) a.reduce_mode = kReduceSecondPass;
        // outputs per reader of the resident reduction: the row group's, dealt evenly in whole 16-byte pieces
        const int64_t rg_floats = (int64_t)p.fs.panels * p.fs.panel_rows;
        a.red_chunk = (int)(((rg_floats + a.slices - 1) / a.slices + 3) / 4 * 4);
    }

    const int C = p.fs.cols, G = p.fs.groups, LB = p.fs.lane_bytes, EB = p.fs.entry_bytes;
#define MSGEMM_CASE(CC, GG, LL, EE, XD, XT, YT, ET)                                   \
    if (C == CC && G == GG && LB == LL && EB == EE && p.x_dtype == XD)               \
        return launch_for_values<XT, YT, ET, CC, GG, LL, (CC == 1 && LL == 8) ? 16 : 8>(p, a, s);
    // single column, full-width entries
    MSGEMM_CASE(1, 64, 16, 4, MSGEMM_F32, float, float, float)
    MSGEMM_CASE(1, 64, 16, 4, MSGEMM_F16, __half, __half, float)
    MSGEMM_CASE(1, 64, 16, 4, MSGEMM_BF16, bf16_t, bf16_t, float)
    MSGEMM_CASE(1, 64, 16, 4, MSGEMM_I8, int8_t, int, int)
    MSGEMM_CASE(1, 64, 8, 4, MSGEMM_F32, float, float, float)
    MSGEMM_CASE(1, 64, 8, 4, MSGEMM_F16, __half, __half, float)
    MSGEMM_CASE(1, 64, 8, 4, MSGEMM_BF16, bf16_t, bf16_t, float)
    MSGEMM_CASE(1, 64, 8, 4, MSGEMM_I8, int8_t, int, int)
    // batched fp32 activations: 4 columns of fp32 entries (16-bit entries: the batched kernel)
    MSGEMM_CASE(4, 32, 8, 4, MSGEMM_F32, float, float, float)
#undef MSGEMM_CASE
    return MSGEMM_ERR_UNSUPPORTED;
}

}  // namespace msgemm
