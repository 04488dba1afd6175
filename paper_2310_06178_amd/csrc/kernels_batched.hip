// Fused msGeMM for batches (b > 2, d = 2) on gfx950: tables of 8 batch columns
// per entry in LDS, the table-adds of phase 2 done by the matrix cores.
// Two kernels: batched_kernel (one table of 32 groups, rebuilt in a phase of
// its own for every k-tile; described first) and batched_pipe_kernel (two
// tables of 16 groups, the next one built while the current one is gathered
// from; chosen for large problems, described where it is defined).
//
// Work decomposition
//   A k-tile is 32 table groups (64 k-columns); its table -- 256 entries per
//   group, 8 fp16 batch columns (16 bytes) per entry, 128 KiB -- is built in LDS
//   by the workgroup that consumes it (Section 4: the table is produced
//   piecewise along its last dimension and consumed at once).  A workgroup owns
//   up to 8 row panels of 256 rows (one per wavefront), one pass of 8 batch
//   columns and a *segment* of consecutive k-tiles: it rebuilds the table for
//   every k-tile of the segment and keeps the outputs in registers across
//   them, so one partial sum per segment -- not per k-tile -- leaves the
//   workgroup.  Segments are as long as the problem allows while every
//   compute unit still gets a workgroup.
//
// Phase 2 on the matrix cores
//   A look-up returns the 8 columns of one row as two 4 x fp16 operands.
//   v_mfma_f32_4x4x4_16B_f16 computes, for each group of four lanes,
//   D[i][j] += sum_k A[i][k] B[k][j] with lane (quad, i) supplying row i of A
//   and lane (quad, j) column j of B and receiving column j of D.  With B the
//   identity this is D[i][j] += A[i][j]: the instruction adds a fp16 entry to
//   an fp32 accumulator, four columns at a time, without using the vector ALU
//   -- which is what bounds a gather that adds with v_pk_add_f16 / v_fma_mix.
//   The accumulators come out transposed within each quad of lanes: lane
//   (quad, j), register i holds column j of the row that lane (quad, i) looked
//   up.  Everything downstream (block scales, fold, stores) works on that
//   layout directly.  Accumulation is in fp32 throughout; int8 activations use
//   the same path (their table entries, |entry| <= 2048, are exact in fp16 and
//   a segment is kept short enough for every sum to stay within 2^24, so the
//   fp32 sums are exact integers; the segments are then added in int32).
//
// Shared scales (Section 3.3) are applied when a scale block of k-columns has
// been consumed: y += q(row, block) * (sum over the block's tables).
#include <type_traits>

#include "device_types.h"
#include "fused_common.h"
#include "msgemm_internal.h"

namespace msgemm {
namespace {

constexpr int kBC = 8;                   // batch columns per table entry and per pass
constexpr int kBG = 32;                  // table groups per k-tile
// LB = rows (code bytes) a lane takes per load: 8 (8 wavefronts of 256-row panels)
// or 4 (12 wavefronts of 128-row panels: half the registers per wavefront, three
// wavefronts per SIMD to hide the LDS latency behind).
template <int LB> constexpr int batched_waves() { return LB == 8 ? 8 : 12; }
// LDS layout of the table: two halves of 16 groups; entry (code, g) at
// (g / 16) * 64 KiB + code * 256 + (g % 16) * 16.  The code byte is then byte 1
// of the address and the half byte 2: one v_perm_b32 turns a packed code into
// an address.  Lanes served together hold different g % 16, i.e. different banks.
constexpr int kBCodeStride = 256;        // bytes between the entries of consecutive codes within a half
constexpr int kBHalfBytes = 256 * kBCodeStride;
#ifndef MSGEMM_BATCHED_RING
#define MSGEMM_BATCHED_RING 8
#endif
constexpr int kBRing = MSGEMM_BATCHED_RING;  // code loads a wavefront keeps in flight (4 and 16 measure the same on every configuration)
// table look-ups issued ahead of the adds that use them (a power of two, at most the rows per load)
#ifndef MSGEMM_BATCHED_LOOKAHEAD
#define MSGEMM_BATCHED_LOOKAHEAD 8
#endif
// Measurement builds only (the result is then wrong): parts of batched_kernel left out, to time what remains.
// Bits: 1 the matrix-core adds (an xor consumes the entries), 2 the table look-ups, 4 the table build (the barriers
// stay), 8 the code loads after the first ring, 16 the partial-sum / output stores, 32 the table builds after a
// workgroup's first.
// schedule of the pipelined form's look-ups: 0 every look-up fenced off, 1 the order given as groups, 2 the compiler's
#ifndef MSGEMM_PIPE_SCHED
#define MSGEMM_PIPE_SCHED 1
#endif
#ifndef MSGEMM_BATCHED_LEAVE_OUT
#define MSGEMM_BATCHED_LEAVE_OUT 0
#endif
// The same for batched_pipe_kernel.  Bits: 1 the matrix-core adds, 2 the table look-ups (addresses are still formed),
// 4 the entries of the next table, 8 the barrier between k-tiles (every address stays inside LDS whatever the tables
// hold, and no wait depends on the barrier), 32 the code loads after the first ring, 64 the code stream (the loads
// stay, but every k-tile reads the segment's first k-tile again: cache hits), 128 the activations after the first two
// k-tiles.
#ifndef MSGEMM_PIPE_LEAVE_OUT
#define MSGEMM_PIPE_LEAVE_OUT 0
#endif
// The sums over the k-segments handed over inside an XCD: on request only (reduce_mode 4).  Measured slower than the
// second launch on every mid-size configuration (14336 x 4096 x 8: 29.6 against 22.3 us; 8192 x 8192 x 16: 39.8 against
// 29.8; level at 28672 x 8192 x 64): the partial sums just written do not come back from the L2 any faster than
// from memory, and a workgroup that waits keeps its compute unit.
constexpr bool kLocalByDefault = false;
// Measurement builds only (the result is then wrong): parts of the XCD-local reduction left out.  Bits: 1 all of it
// (the workgroups keep its order of ids), 2 the wait for the other workgroups, 4 the reads and adds.
#ifndef MSGEMM_LOCAL_LEAVE_OUT
#define MSGEMM_LOCAL_LEAVE_OUT 0
#endif
static_assert(kLoadsPerPanel % kBRing == 0, "ring slots are reused with a period dividing the panel");

template <int LB> struct LaneLoad;
template <> struct LaneLoad<8> { using type = uint2; };
template <> struct LaneLoad<4> { using type = uint32_t; };
template <int LB> __device__ __forceinline__ uint32_t load_word(const typename LaneLoad<LB>::type& v, int w)
{
    if constexpr (LB == 8) return w == 0 ? v.x : v.y;
    else return v;
}

typedef _Float16 h2 __attribute__((ext_vector_type(2)));
typedef _Float16 h4 __attribute__((ext_vector_type(4)));
typedef float f4 __attribute__((ext_vector_type(4)));

struct BatchedArgs {
    const uint8_t* tiled;    // codes in streaming order [load][k-tile][panel][lane][8] (pipelined form: [panel][k-tile][load][lane][8],
                             // with 8 rows per lane [panel][k-tile][load / 2][lane][load % 2][8])
    const void* X;
    int64_t ldx;
    void* Y;
    int64_t ldy;
    ValueMap values;         // value of each 4-bit pattern
    const float* values256;  // 8-bit weights: the value of each of the 256 bit patterns (device), else nullptr
    const __half* scales;    // [block][panel][lane][LB]: scale of the row behind each of a lane's look-ups; or nullptr
    float* partials;         // [segment][column][panel][lane][LB / 2]
    int64_t m, k, b, m_pad, b_pad;
    int ktiles, panels_total, panels_per_wg, row_blocks, col_passes;
    int segments;            // k-segments (partial sums per output)
    int tiles_per_segment;
    int tiles_per_block;     // k-tiles per scale block
    int units;               // segments * row_blocks
    int direct;              // 1: a single segment, the kernel writes Y itself
    int64_t partial_span;    // bytes of the partial buffer (< 2^31)
    FastDiv div_col_passes, div_segments, div_tiles_per_block;
    float x_limit;           // floating-point activations beyond this magnitude can take a table entry out of the fp16 range
    unsigned* error;         // the plan's sticky error word (bit 0: a reduction gave up; bit 1: such an activation was seen), or nullptr
    // the segments' sums added by the workgroups of this launch (every workgroup resident at once), not by a second one
    int resident;            // 1: on
    int publish;             // 0 (a test aid): the partial sums are not stored, the readers find nothing and give up
    unsigned* epochs;        // launch count of every workgroup (each bumps its own)
    unsigned poll_limit;     // polls before a waiting lane gives up
    int red_pieces;          // 16-byte pieces of the outputs one workgroup adds
    int red_groups;          // lanes that share a piece, each taking every red_groups-th segment
    // resident = 2: the workgroups of one (row block, column pass) run on one XCD and hand their sums over through its L2
    int local_inner;         // column passes of a row block that share an XCD (col_passes, or 1: pairs are dealt instead)
    unsigned* arrivals;      // per (row block, column pass): workgroups that have stored their sums, all launches together
    FastDiv div_local_inner;
    // pipelined form, k-tiles dealt evenly (dealt = 1): for one column pass the scale blocks of all row blocks form one
    // sequence, row block after row block; workgroup `unit` takes deal_blocks consecutive ones, which may run from the
    // end of one row block into the start of the next (two runs, a partial sum each)
    int dealt;
    int deal_blocks;         // scale blocks (tiles_per_block k-tiles each) per workgroup
    int blocks_per_rb;       // scale blocks of one row block (all of k)
    int deal_total;          // row_blocks * blocks_per_rb
    FastDiv div_blocks_per_rb, div_deal_blocks;
};

template <typename XT> __device__ __forceinline__ _Float16 to_half(XT v);
template <> __device__ __forceinline__ _Float16 to_half<__half>(__half v) { return (_Float16)__half2float(v); }
template <> __device__ __forceinline__ _Float16 to_half<bf16_t>(bf16_t v) { return (_Float16)XTraits<bf16_t>::load(&v); }
template <> __device__ __forceinline__ _Float16 to_half<int8_t>(int8_t v) { return (_Float16)(float)v; }

// 16-bit table entries hold value(c0) x0 + value(c1) x1 in fp16: an activation larger than x_limit (65504 over twice
// the largest value of a code; int8 activations never are) can push an entry to infinity.  The result then holds
// infinities or NaN where a full-width table would not; the kernel cannot fail the call, so it raises bit 1 of the
// plan's error word (msgemm_plan_check reports MSGEMM_ERR_RANGE).  One comparison per staged activation.
template <typename XT>
__device__ __forceinline__ void flag_range(const BatchedArgs& a, bool live, XT raw)
{
    if constexpr (!__is_same(XT, int8_t)) {
        const float x = fabsf(XTraits<XT>::load(&raw));
        if (live && !(x <= a.x_limit) && a.error) __hip_atomic_fetch_or(a.error, 2u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    }
}

// all of this wavefront's LDS traffic has landed / returned, then the workgroup meets.
// (Not __syncthreads(): its fence would also wait for the code loads in flight.)
__device__ __forceinline__ void lds_barrier()
{
    asm volatile("s_waitcnt lgkmcnt(0)\n\ts_barrier" ::: "memory");
}

// value of `v` in lane i of the caller's quad
template <int I> __device__ __forceinline__ float quad_broadcast(float v)
{
    return __uint_as_float((unsigned)__builtin_amdgcn_mov_dpp((int)__float_as_uint(v), I * 0x55, 0xf, 0xf, true));
}

// The sums over the k-segments, inside the launch that made them.  Every partial sum carries the parity of the launch
// in its last bit (tag_partial), so a reader knows a word of this launch from one of the launch before without flags:
// every launch rewrites every word, and the parity alternates.  When a workgroup has stored its own sums it turns
// reader of 1 / readers of the outputs: lane (piece, g) loads the 16-byte piece of the segments g, g + groups, ...,
// eight loads at a time, again until all carry this launch's parity (at most poll_limit times: then bit 0 of the
// plan's error word is set and msgemm_plan_check reports it), adds them in segment order; the groups' sums meet in
// LDS and are added in group order: a fixed order.  Needs every workgroup of the grid resident at the same time
// (one per compute unit: the host checks) -- a reader waits for sums of workgroups that must be running.
// Called by every thread of the workgroup (it holds workgroup barriers); `scratch` is LDS nobody reads any more once
// all have arrived here, 16 bytes per thread.
template <typename YT, typename AT, int kFinal>
__device__ __forceinline__ void reduce_segments_resident(const BatchedArgs& a, unsigned parity, int reader, unsigned char* scratch)
{
    constexpr int kPanelRowsR = 64 * kFinal;
    const int tid = threadIdx.x;
    const int G = a.red_groups;
    const int per_round = (int)blockDim.x / G;   // pieces a round of the workgroup covers
    const int pl = tid % per_round, g = tid / per_round;
    const uint32_t seg_bytes = (uint32_t)(a.b_pad * a.m_pad * 4);
    const int64_t p0 = (int64_t)reader * a.red_pieces;
    const int64_t p_end = min(p0 + a.red_pieces, a.b_pad * a.m_pad / 4);
    __amdgpu_buffer_rsrc_t rsrc = __builtin_amdgcn_make_buffer_rsrc((void*)a.partials, 0, (int)a.partial_span, 0x00020000);
    YT* __restrict__ Y = (YT*)a.Y;
    unsigned polls = 0;
    bool gave_up = false;
    // One wavefront watches a single piece of every segment (the first of this workgroup's share) until it carries
    // this launch's parity, at a leisurely pace; the others sleep at the barrier.  Workgroups finish at different
    // times: were every lane to poll all of its pieces, the early ones would take memory bandwidth from the late.
    if (tid < 64) {
        const int64_t piece = min(p0, p_end - 1);
#pragma unroll 1
        for (int s0 = 0; s0 < a.segments && !gave_up; s0 += 64) {
            const bool live = s0 + tid < a.segments && p0 < p_end;
            const uint32_t off = live ? (uint32_t)(s0 + tid) * seg_bytes + (uint32_t)piece * 16u : 0x7ffffff0u;
#pragma unroll 1
            for (;;) {
                asm volatile("" ::: "memory");
                const v4u v = __builtin_amdgcn_raw_buffer_load_b128(rsrc, (int)off, 0, kAuxSc1);
                const bool here = !live || ((v.x & v.y & v.z & v.w & 1u) == parity && ((v.x | v.y | v.z | v.w) & 1u) == parity);
                if (__builtin_amdgcn_ballot_w64(!here) == 0) break;
                if (++polls >= a.poll_limit) {
                    gave_up = true;
                    break;
                }
                __builtin_amdgcn_s_sleep(32);
            }
        }
    }
    lds_barrier();  // every wavefront has left the tables (their memory is scratch now), and the sums are about there
#pragma unroll 1
    for (int r0 = 0; r0 < a.red_pieces; r0 += per_round) {
        const int64_t piece = p0 + r0 + pl;
        const bool have = g < G && r0 + pl < a.red_pieces && piece < p_end;
        AT sum[4] = {0, 0, 0, 0};
#pragma unroll 1
        for (int s0 = g; s0 < a.segments && have && !gave_up; s0 += 8 * G) {
            v4u v[8];
            uint32_t off[8];
            bool live[8];
#pragma unroll
            for (int u = 0; u < 8; ++u) {
                const int sl = s0 + u * G;
                live[u] = sl < a.segments;
                off[u] = live[u] ? (uint32_t)sl * seg_bytes + (uint32_t)piece * 16u : 0x7ffffff0u;  // (out of range: reads zero)
            }
#pragma unroll 1
            for (;;) {
                asm volatile("" ::: "memory");
#pragma unroll
                for (int u = 0; u < 8; ++u) v[u] = __builtin_amdgcn_raw_buffer_load_b128(rsrc, (int)off[u], 0, kAuxSc1);
                bool arrived = true;
#pragma unroll
                for (int u = 0; u < 8; ++u)
                    arrived &= !live[u] || ((v[u].x & v[u].y & v[u].z & v[u].w & 1u) == parity &&
                                            ((v[u].x | v[u].y | v[u].z | v[u].w) & 1u) == parity);
                if (arrived) break;
                if (++polls >= a.poll_limit) {
                    gave_up = true;
                    break;
                }
                __builtin_amdgcn_s_sleep(16);
            }
            if (gave_up) break;
#pragma unroll
            for (int u = 0; u < 8; ++u) {  // (what is not live read as zero and adds nothing)
                AT x;
                untag_partial(x, live[u] ? v[u].x : 0u); sum[0] += x;
                untag_partial(x, live[u] ? v[u].y : 0u); sum[1] += x;
                untag_partial(x, live[u] ? v[u].z : 0u); sum[2] += x;
                untag_partial(x, live[u] ? v[u].w : 0u); sum[3] += x;
            }
        }
        // the groups' sums of a piece meet in LDS
        AT* mine = (AT*)(scratch + (size_t)tid * 16);
        if (G > 1) {
#pragma unroll
            for (int e = 0; e < 4; ++e) mine[e] = sum[e];
            lds_barrier();
        }
        if (have && g == 0 && !gave_up) {
            for (int og = 1; og < G; ++og) {
                const AT* other = (const AT*)(scratch + (size_t)(og * per_round + pl) * 16);
#pragma unroll
                for (int e = 0; e < 4; ++e) sum[e] += other[e];
            }
            // piece -> (column, partial-sum slots of a panel); slot f of a panel belongs to lane slot_owner(f / kFinal)
            // of the wavefront that made it, output f % kFinal: row 64 (f % kFinal) + that lane
            const int64_t f = piece * 4;
            const int64_t col = f / a.m_pad, rr = f % a.m_pad;
            const int64_t panel = rr / kPanelRowsR;
            const int q0 = (int)(rr % kPanelRowsR);
#pragma unroll
            for (int e = 0; e < 4; ++e) {
                const int qe = q0 + e;
                const int64_t row = panel * kPanelRowsR + 64 * (qe % kFinal) + slot_owner(qe / kFinal, 1);
                if (row < a.m && col < a.b) Y[col * a.ldy + row] = to_output<YT, AT>(sum[e]);
            }
        }
        if (G > 1) lds_barrier();  // the scratch is read: the next round may write it
    }
    // gave up: some partial sum never arrived.  The plan's error word says so (msgemm_plan_check).
    if (gave_up && a.error) __hip_atomic_fetch_or(a.error, 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}

template <typename AT> __device__ __forceinline__ AT partial_of(unsigned u);
template <> __device__ __forceinline__ float partial_of<float>(unsigned u) { return __uint_as_float(u); }
template <> __device__ __forceinline__ int partial_of<int>(unsigned u) { return (int)u; }

// Id of the XCD (one of the device's eight dies, each with an L2 of its own) that this wavefront runs on.
__device__ __forceinline__ unsigned xcc_id()
{
    unsigned x;
    asm volatile("s_getreg_b32 %0, hwreg(HW_REG_XCC_ID)" : "=s"(x));
    return x & 15u;
}

// *p as the L2 of this XCD holds it: a read-modify-write that changes nothing is carried out in the L2 itself, where a
// load may be answered by the compute unit's own cache (and the compiler turns an atomic add of a constant 0 into one).
__device__ __forceinline__ unsigned l2_read(unsigned* p)
{
    unsigned v;
    asm volatile("global_atomic_or %0, %1, %2, off sc0\n\ts_waitcnt vmcnt(0)" : "=&v"(v) : "v"(p), "v"(0u) : "memory");
    return v;
}

// all of this wavefront's stores have been taken by the L2, its LDS traffic has landed, then the workgroup meets
__device__ __forceinline__ void store_barrier()
{
    asm volatile("s_waitcnt vmcnt(0) lgkmcnt(0)\n\ts_barrier" ::: "memory");
}

// block id -> (row block, k-segment, column pass) when the sums are handed over inside an XCD (resident = 2).
// Workgroup ids are dealt over the XCDs in turn, so id % 8 is the XCD.  XCD x takes the row blocks x, x + 8, ... with
// all their column passes (local_inner = col_passes; the passes of a segment follow each other and share the codes in
// the L2), or, when the row blocks do not divide by eight, the (row block, column pass) pairs x, x + 8, ...
__device__ __forceinline__ void local_block(const BatchedArgs& a, uint32_t bid, int& rb, int& seg, int& cp)
{
    const uint32_t x = bid % kXcds, n = bid / kXcds;
    const uint32_t t = fast_div(n, a.div_local_inner);
    const int li = (int)(n - t * (uint32_t)a.local_inner);
    const uint32_t lp = fast_div(t, a.div_segments);
    seg = (int)(t - lp * (uint32_t)a.segments);
    const uint32_t pr = x + kXcds * lp;
    if (a.local_inner > 1 || a.col_passes == 1) {
        rb = (int)pr;
        cp = li;
    } else {
        rb = (int)fast_div(pr, a.div_col_passes);
        cp = (int)(pr - (uint32_t)rb * (uint32_t)a.col_passes);
    }
}

// The sums over the k-segments inside the launch, handed over through one L2 (resident = 2).  All workgroups of a
// (row block, column pass) run on one XCD at the same time (the host checks the grid against the compute units and,
// once per device, that ids are dealt over the XCDs in turn; every workgroup checks its own XCD id again).  Their
// partial sums are ordinary stores: they go through the compute unit's cache into that L2.  When a wavefront's stores
// have been taken and the workgroup has met, one lane counts the workgroup in (an atomic add in the L2) and waits
// until the count has grown by one for every segment -- the count runs on over the launches, `target` is this launch's
// -- then everybody reads: workgroup `seg` adds share `seg` of the pair's outputs in segment order, from lines this
// compute unit has not touched since the launch began, which therefore come from the L2.  A wait that runs out
// (poll_limit) or a workgroup on an unexpected XCD sets bit 0 of the plan's error word, and nothing is written.
template <typename YT, typename AT, int kFinal>
__device__ __forceinline__ void reduce_segments_local(const BatchedArgs& a, int rb, int cp, int seg, unsigned target,
                                                      bool xcd_as_expected, unsigned char* scratch)
{
    constexpr int kPanelRowsR = 64 * kFinal;
    const int tid = threadIdx.x;
    if constexpr (MSGEMM_LOCAL_LEAVE_OUT & 1) return;
    store_barrier();  // this workgroup's sums are in the L2, and nobody gathers from the tables any more
    if (tid == 0) {
        unsigned* cnt = a.arrivals + ((int64_t)rb * a.col_passes + cp);
        if (a.publish) __hip_atomic_fetch_add(cnt, 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_WORKGROUP);
        unsigned polls = 0;
        bool ok = xcd_as_expected;
        while (!(MSGEMM_LOCAL_LEAVE_OUT & 2) && ok && (int)(l2_read(cnt) - target) < 0) {
            if (++polls >= a.poll_limit) ok = false;
            else __builtin_amdgcn_s_sleep(8);
        }
        *(volatile unsigned*)scratch = ok ? 1u : 0u;
    }
    lds_barrier();
    const bool gave_up = *(volatile unsigned*)scratch == 0u;
    lds_barrier();  // (the word is read: the scratch is free for the sums below)
    if (gave_up) {
        if (tid == 0 && a.error) __hip_atomic_fetch_or(a.error, 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        return;
    }
    if constexpr (MSGEMM_LOCAL_LEAVE_OUT & 4) return;
    const int panels_here = min(a.panels_per_wg, a.panels_total - rb * a.panels_per_wg);
    const int per_col = panels_here * (kPanelRowsR / 4);  // 16-byte pieces of one column of this row block
    const int total = kBC * per_col;
    const int q_begin = seg * a.red_pieces, q_end = min(q_begin + a.red_pieces, total);
    const int64_t f_rb = (int64_t)rb * a.panels_per_wg * kPanelRowsR;  // first partial-sum slot of the row block within a column
    const int G = a.red_groups;
    const int per_round = (int)blockDim.x / G;
    const int pl = tid % per_round, g = tid / per_round;
    const uint32_t seg_bytes = (uint32_t)(a.b_pad * a.m_pad * 4);
    __amdgpu_buffer_rsrc_t rsrc = __builtin_amdgcn_make_buffer_rsrc((void*)a.partials, 0, (int)a.partial_span, 0x00020000);
    YT* __restrict__ Y = (YT*)a.Y;
#pragma unroll 1
    for (int r0 = q_begin; r0 < q_end; r0 += per_round) {
        const int qi = r0 + pl;
        const bool have = g < G && qi < q_end;
        const int c = have ? qi / per_col : 0;
        const int64_t f = ((int64_t)cp * kBC + c) * a.m_pad + f_rb + (int64_t)(have ? qi - c * per_col : 0) * 4;  // slot within a segment
        AT sum[4] = {0, 0, 0, 0};
#pragma unroll 1
        for (int s0 = g; s0 < a.segments && have; s0 += 8 * G) {
            v4u v[8];
#pragma unroll
            for (int u = 0; u < 8; ++u) {
                const int sl = s0 + u * G;
                const uint32_t off = sl < a.segments ? (uint32_t)sl * seg_bytes + (uint32_t)f * 4u : 0x7ffffff0u;  // (out of range: reads zero)
                v[u] = __builtin_amdgcn_raw_buffer_load_b128(rsrc, (int)off, 0, 0);
            }
#pragma unroll
            for (int u = 0; u < 8; ++u) {
                sum[0] += partial_of<AT>(v[u].x); sum[1] += partial_of<AT>(v[u].y);
                sum[2] += partial_of<AT>(v[u].z); sum[3] += partial_of<AT>(v[u].w);
            }
        }
        AT* mine = (AT*)(scratch + (size_t)tid * 16);
        if (G > 1) {
#pragma unroll
            for (int e = 0; e < 4; ++e) mine[e] = sum[e];
            lds_barrier();
        }
        if (have && g == 0) {
            for (int og = 1; og < G; ++og) {
                const AT* other = (const AT*)(scratch + (size_t)(og * per_round + pl) * 16);
#pragma unroll
                for (int e = 0; e < 4; ++e) sum[e] += other[e];
            }
            // slot f of a column belongs to lane slot_owner(f / kFinal) of the wavefront that made it, output f % kFinal
            const int64_t col = (int64_t)cp * kBC + c, rr = f - col * a.m_pad;
            const int64_t panel = rr / kPanelRowsR;
            const int q0 = (int)(rr % kPanelRowsR);
#pragma unroll
            for (int e = 0; e < 4; ++e) {
                const int qe = q0 + e;
                const int64_t row = panel * kPanelRowsR + 64 * (qe % kFinal) + slot_owner(qe / kFinal, 1);
                if (row < a.m && col < a.b) Y[col * a.ldy + row] = to_output<YT, AT>(sum[e]);
            }
        }
        if (G > 1) lds_barrier();  // the scratch is read: the next round may write it
    }
}

// This workgroup's launch count goes up by one (one lane); its parity tags the partial sums of this launch (the count
// itself, times the segments, is what the arrival count of an XCD-local reduction has to reach).
// The caller's next workgroup barrier makes `*slot` (LDS) visible to the other lanes.
__device__ __forceinline__ void count_launch(const BatchedArgs& a, unsigned* slot)
{
    if (a.resident && threadIdx.x == 0) {
        const unsigned n = __hip_atomic_load(a.epochs + blockIdx.x, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) + 1u;
        __hip_atomic_store(a.epochs + blockIdx.x, n, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        *slot = n;
    }
}

// kCodes8: 8-bit weights.  A code byte is one element, a table group one k-column
// (a.k counts two per byte), an entry values256[code] * x; only the table build
// and the activations it reads differ.
template <typename XT, typename YT, typename AT, bool kScaled, int kBLB, bool kCodes8>
__global__ void __launch_bounds__(batched_waves<kBLB>() * 64)
batched_kernel(BatchedArgs a)
{
    constexpr int kBWaves = batched_waves<kBLB>();  // wavefronts per workgroup, one row panel each
    constexpr int kBPanelRows = 32 * kBLB;          // 64 lanes x LB rows / 2 lanes per row
    constexpr int kBFinal = kBLB / 2;               // rows a lane owns after the fold
    // look-ups per chunk (with scales the second set of accumulators leaves registers for half as many)
    constexpr int kLook = (MSGEMM_BATCHED_LOOKAHEAD < kBLB ? MSGEMM_BATCHED_LOOKAHEAD : kBLB) / (kScaled ? 2 : 1);
    constexpr int kThreads = kBWaves * 64;
    using LoadT = typename LaneLoad<kBLB>::type;
    __shared__ __align__(16) unsigned char lds[2 * kBHalfBytes];
    __shared__ __align__(16) _Float16 xs[2][2 * kBG][kBC];            // activations of a k-tile: [k-column][batch column]
    __shared__ unsigned launch_count;

    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int wave = tid >> 6;
    const int q = lane >> 4, j = lane & 15, qg = q & 1;

    // ---- block id -> (k-segment, row block, column pass).  The column passes of a
    // unit (same codes) get ids that are congruent modulo the XCD count and close
    // together: they run on one XCD around the same time and share its L2.
    const uint32_t bid = blockIdx.x;
    int rb, seg, cp, unit;
    if (a.resident == 2) {
        local_block(a, bid, rb, seg, cp);  // (the grid is exactly the workgroups there are)
        unit = rb * a.segments + seg;
    } else {
        const uint32_t n = bid / kXcds;
        const uint32_t hi = fast_div(n, a.div_col_passes);
        cp = (int)(n - hi * (uint32_t)a.col_passes);
        unit = (int)((bid % kXcds) + kXcds * hi);
        if (unit >= a.units) return;
        rb = (int)fast_div((uint32_t)unit, a.div_segments);
        seg = unit - rb * a.segments;
    }
    const bool xcd_as_expected = a.resident != 2 || xcc_id() == bid % kXcds;
    const int kt_begin = seg * a.tiles_per_segment;
    const int kt_end = min(kt_begin + a.tiles_per_segment, a.ktiles);
    const int64_t col0 = (int64_t)cp * kBC;
    const int panel = rb * a.panels_per_wg + wave;
    const bool active = wave < a.panels_per_wg && panel < a.panels_total;

    const XT* __restrict__ X = (const XT*)a.X;

    // ---- activations of a k-tile: thread (c, kc) of the first 512 fetches X(64 kt + kc, col0 + c)
    const int xc = (tid >> 6) & (kBC - 1), xkc = tid & 63;
    auto x_fetch = [&](int kt) -> XT {
        const int64_t kk = (int64_t)kt * (2 * kBG) + xkc;
        const bool live = (col0 + xc < a.b) && (kk < a.k);
        // (8-bit weights: slots 2g and 2g + 1 both hold the column of group g)
        return X[live ? (col0 + xc) * a.ldx + (kCodes8 ? (kk >> 1) : kk) : 0];  // (a clamped, always valid address; masked below)
    };
    auto x_store = [&](int buf, int kt, XT raw) {
        const int64_t kk = (int64_t)kt * (2 * kBG) + xkc;
        const bool live = (col0 + xc < a.b) && (kk < a.k);
        if (tid < 2 * kBG * kBC) xs[buf][xkc][xc] = live ? to_half<XT>(raw) : (_Float16)0.0f;
        flag_range<XT>(a, live, raw);
    };

    // ---- phase 1: L(c0 | c1 << 4, g, c) = b(c0) X(2g, c) + b(c1) X(2g + 1, c), in packed fp16
    // values of this thread's high code and of its low codes (fetched once, ahead of
    // the first table build; exact in fp16 for the paper's b(.))
    const _Float16 w1_mine = (_Float16)a.values.v[(tid >> 5) & 15];
    _Float16 w0_mine[16 / (kThreads % (kBG * 16) == 0 ? kThreads / (kBG * 16) : 1)];
    {
        constexpr int kParts = kThreads % (kBG * 16) == 0 ? kThreads / (kBG * 16) : 1;
        const int first = kParts == 1 ? 0 : (tid >> 9) * (16 / kParts);
#pragma unroll
        for (int cc = 0; cc < 16 / kParts; ++cc) w0_mine[cc] = (_Float16)a.values.v[(first + cc) & 15];
    }
    // thread (g, c1, part) writes 16 / parts entries of its c1 for group g
    constexpr int kBuildParts = kThreads % (kBG * 16) == 0 ? kThreads / (kBG * 16) : 1;
    constexpr int kBuildEach = 16 / kBuildParts;
    auto build_tables = [&](int buf) {
        const int g = tid & (kBG - 1), c1 = (tid >> 5) & 15, part = tid >> 9;
        if (part >= kBuildParts) return;  // (a thread count that is no multiple of 512: the rest sits the build out)
        if constexpr (MSGEMM_BATCHED_LEAVE_OUT & 4) return;
        h2 x0[4], x1[4], top[4];
        __builtin_memcpy(x0, &xs[buf][2 * g][0], 16);
        __builtin_memcpy(x1, &xs[buf][2 * g + 1][0], 16);
        const _Float16 w1 = w1_mine;
#pragma unroll
        for (int p = 0; p < 4; ++p) top[p] = x1[p] * h2{w1, w1};
        unsigned char* dst = lds + (g >> 4) * kBHalfBytes + (size_t)(c1 * 16) * kBCodeStride + (g & 15) * 16;
        if constexpr (kCodes8) {
            // the 16 values behind this thread's high nibble, fetched at every build (no registers to keep them in)
            float v[16];
#pragma unroll
            for (int v4 = 0; v4 < 4; ++v4) {
                const float4 q4 = *(const float4*)(a.values256 + c1 * 16 + v4 * 4);
                v[v4 * 4 + 0] = q4.x; v[v4 * 4 + 1] = q4.y; v[v4 * 4 + 2] = q4.z; v[v4 * 4 + 3] = q4.w;
            }
#pragma unroll
            for (int c0 = 0; c0 < 16; ++c0) {
                const _Float16 w = (_Float16)v[c0];
                h2 e[4];
#pragma unroll
                for (int p = 0; p < 4; ++p) e[p] = x0[p] * h2{w, w};
                __builtin_memcpy(dst + c0 * kBCodeStride, e, 16);
            }
            return;
        }
#pragma unroll
        for (int cc = 0; cc < kBuildEach; ++cc) {
            const int c0 = part * kBuildEach + cc;
            const _Float16 w0 = w0_mine[cc];
            h2 e[4];
#pragma unroll
            for (int p = 0; p < 4; ++p) e[p] = __builtin_elementwise_fma(h2{w0, w0}, x0[p], top[p]);
            __builtin_memcpy(dst + c0 * kBCodeStride, e, 16);
        }
    };

    // ---- the code stream of this wavefront: load t of k-tile kt
    const LoadT* __restrict__ tiled = (const LoadT*)a.tiled;
    auto code_at = [&](int kt, int t) -> const LoadT* {
        return tiled + (((int64_t)t * a.ktiles + kt) * a.panels_total + panel) * 64 + lane;
    };
    LoadT ring[kBRing];

    XT xraw = x_fetch(kt_begin);
    if (active) {
#pragma unroll
        for (int u = 0; u < kBRing; ++u) {
            ring[u] = load_codes(code_at(kt_begin, u));
            __builtin_amdgcn_sched_barrier(0);  // loads return in issue order: keep slot 0 first
        }
    }
    count_launch(a, &launch_count);
    x_store(0, kt_begin, xraw);
    lds_barrier();
    build_tables(0);
    lds_barrier();

    h4 onehot;  // column (lane % 4) of the 4 x 4 identity
#pragma unroll
    for (int e = 0; e < 4; ++e) onehot[e] = (_Float16)((lane & 3) == e ? 1.0f : 0.0f);
    f4 dlo[kBLB], dhi[kBLB];  // sums of the current scale block (of everything, without scales)
    f4 ylo[kScaled ? kBLB : 1], yhi[kScaled ? kBLB : 1];
#pragma unroll
    for (int s = 0; s < kBLB; ++s) {
        dlo[s] = f4{0, 0, 0, 0};
        dhi[s] = f4{0, 0, 0, 0};
        if constexpr (kScaled) {
            ylo[s] = f4{0, 0, 0, 0};
            yhi[s] = f4{0, 0, 0, 0};
        }
    }

    for (int kt = kt_begin; kt < kt_end; ++kt) {
        const bool more = kt + 1 < kt_end;
        if (more) xraw = x_fetch(kt + 1);
        if (active) {
            // scales of the rows behind this lane's 8 look-ups, for the block this k-tile belongs to
            struct alignas(2 * kBLB) LaneScales { __half h[kBLB]; };
            LaneScales qraw;
            if constexpr (kScaled) {
                const int blk = (int)fast_div((uint32_t)kt, a.div_tiles_per_block);
                qraw = *(const LaneScales*)(a.scales + (((int64_t)blk * a.panels_total + panel) * 64 + lane) * kBLB);
            }
            const int kt_next = more ? kt + 1 : kt;  // (the last tile re-requests its own tail: harmless, and branch-free)
            // The look-ups run one chunk ahead of the table-adds: the reads of chunk c + 1 are issued between the
            // matrix-core adds of chunk c, so a read has a whole chunk's adds to land in and the LDS and the matrix
            // cores work at the same time (left to itself the compiler keeps two reads in flight and waits for each).
            constexpr int kChunks = kLoadsPerPanel * kBLB / kLook;
            uint4 ent[2][kLook];
            auto look = [&](int c, uint4 (&e)[kLook]) {
                const int t = c * kLook / kBLB, s0 = c * kLook % kBLB;
                // byte 0: the slot of this lane's group within a code's 256 bytes; byte 2: the half
                const uint32_t lane_off = (uint32_t)((j + t) & 15) * 16u | ((uint32_t)qg << 16);
                const LoadT d = ring[t % kBRing];
#pragma unroll
                for (int i = 0; i < kLook; ++i) {
                    const int s = s0 + i;
                    const uint32_t w = load_word<kBLB>(d, s >> 2);
                    // address bytes (3..0) = (0, half, code, slot)
                    const uint32_t addr = __builtin_amdgcn_perm(w, lane_off, 0x0c020000u | ((4u + (s & 3)) << 8));
                    if constexpr (MSGEMM_BATCHED_LEAVE_OUT & 2) e[i] = uint4{addr, addr, addr, addr};
                    else e[i] = *(const uint4*)(lds + addr);
                }
            };
            auto add = [&](int c, const uint4 (&e)[kLook]) {
                const int s0 = c * kLook % kBLB;
#pragma unroll
                for (int i = 0; i < kLook; ++i) {
                    const int s = s0 + i;
                    if constexpr (MSGEMM_BATCHED_LEAVE_OUT & 1) {
                        asm volatile("" ::"v"(e[i].x), "v"(e[i].y), "v"(e[i].z), "v"(e[i].w));  // demanded, by no instruction
                        continue;
                    }
                    h4 lo, up;
                    __builtin_memcpy(&lo, &e[i].x, 8);
                    __builtin_memcpy(&up, &e[i].z, 8);
                    dlo[s] = __builtin_amdgcn_mfma_f32_4x4x4f16(lo, onehot, dlo[s], 0, 0, 0);
                    dhi[s] = __builtin_amdgcn_mfma_f32_4x4x4f16(up, onehot, dhi[s], 0, 0, 0);
                }
            };
            look(0, ent[0]);
            __builtin_amdgcn_sched_barrier(0);
#pragma unroll
            for (int c = 0; c < kChunks; ++c) {
                if (c + 1 < kChunks) look(c + 1, ent[(c + 1) & 1]);
                add(c, ent[c & 1]);
                if ((c + 1) * kLook % kBLB == 0) {
                    // load t is all addresses now: refill its slot with the load kBRing ahead
                    const int t = c * kLook / kBLB;
                    if constexpr (!(MSGEMM_BATCHED_LEAVE_OUT & 8))
                    ring[t % kBRing] = load_codes((t + kBRing < kLoadsPerPanel) ? code_at(kt, t + kBRing)
                                                                                  : code_at(kt_next, t + kBRing - kLoadsPerPanel));
                }
                if (c + 1 < kChunks) {
#pragma unroll
                    for (int i = 0; i < kLook; ++i) {  // one look-up, then two adds, kLook times
                        __builtin_amdgcn_sched_group_barrier(0x100, 1, 0);
                        __builtin_amdgcn_sched_group_barrier(0x008, 2, 0);
                    }
                }
                __builtin_amdgcn_sched_barrier(0);
            }
            if constexpr (kScaled) {
                // a scale block ends with this k-tile: y += q(row) * block sum (Section 3.3).
                // Register i of the accumulators belongs to the row of quad lane i.
                const int blk = (int)fast_div((uint32_t)kt, a.div_tiles_per_block);
                if (kt + 1 == kt_end || (kt + 1) == (blk + 1) * a.tiles_per_block) {
#pragma unroll
                    for (int s = 0; s < kBLB; ++s) {
                        const float qf = __half2float(qraw.h[s]);
                        const float q0 = quad_broadcast<0>(qf), q1 = quad_broadcast<1>(qf);
                        const float q2 = quad_broadcast<2>(qf), q3 = quad_broadcast<3>(qf);
                        ylo[s][0] = fmaf(q0, dlo[s][0], ylo[s][0]); yhi[s][0] = fmaf(q0, dhi[s][0], yhi[s][0]);
                        ylo[s][1] = fmaf(q1, dlo[s][1], ylo[s][1]); yhi[s][1] = fmaf(q1, dhi[s][1], yhi[s][1]);
                        ylo[s][2] = fmaf(q2, dlo[s][2], ylo[s][2]); yhi[s][2] = fmaf(q2, dhi[s][2], yhi[s][2]);
                        ylo[s][3] = fmaf(q3, dlo[s][3], ylo[s][3]); yhi[s][3] = fmaf(q3, dhi[s][3], yhi[s][3]);
                        dlo[s] = f4{0, 0, 0, 0};
                        dhi[s] = f4{0, 0, 0, 0};
                    }
                }
            }
        }
        if (more) {
            const int buf = (kt + 1 - kt_begin) & 1;
            x_store(buf, kt + 1, xraw);
            lds_barrier();  // every wavefront is done with the old tables; the new activations are in place
            if constexpr (!(MSGEMM_BATCHED_LEAVE_OUT & 32)) build_tables(buf);
            lds_barrier();
        }
    }
    const unsigned launches = a.resident ? launch_count : 0u, parity = launches & 1u;
    if (active && !((MSGEMM_BATCHED_LEAVE_OUT & 16) && dlo[0][0] != 1234.5f)) {

    // ---- lanes 16 apart looked up the same rows (in different groups): fold them.
    // Afterwards lane (quad b, j'), register (s, i) holds row 64 s + 4 b + i of the
    // panel, column 4 h + j' of the pass.
    const int quad = lane >> 2, jq = lane & 3;
    YT* __restrict__ Y = (YT*)a.Y;
    __amdgpu_buffer_rsrc_t part_rsrc =
        __builtin_amdgcn_make_buffer_rsrc((void*)a.partials, 0, (int)a.partial_span, 0x00020000);
#pragma unroll
    for (int h = 0; h < 2; ++h) {
        const int64_t col = col0 + 4 * h + jq;
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            float fin[kBFinal];
#pragma unroll
            for (int s = 0; s < kBFinal; ++s) {
                float lo_s, hi_s;
                if constexpr (kScaled) {
                    lo_s = h ? yhi[s][i] : ylo[s][i];
                    hi_s = h ? yhi[s + kBFinal][i] : ylo[s + kBFinal][i];
                } else {
                    lo_s = h ? dhi[s][i] : dlo[s][i];
                    hi_s = h ? dhi[s + kBFinal][i] : dlo[s + kBFinal][i];
                }
                fin[s] = fold16(lo_s, hi_s);
            }
            const int owner = 4 * quad + i;  // the lane whose look-ups these sums come from
            if (a.direct) {
#pragma unroll
                for (int s = 0; s < kBFinal; ++s) {
                    const int64_t row = (int64_t)panel * kBPanelRows + 64 * s + owner;
                    if (row < a.m && col < a.b) {
                        if constexpr (__is_same(AT, int)) Y[col * a.ldy + row] = (YT)__float2int_rn(fin[s]);
                        else Y[col * a.ldy + row] = to_output<YT, float>(fin[s]);
                    }
                }
            } else {
                unsigned out[kBFinal];
#pragma unroll
                for (int s = 0; s < kBFinal; ++s) {
                    AT v;
                    if constexpr (__is_same(AT, int)) v = __float2int_rn(fin[s]);
                    else v = fin[s];
                    out[s] = a.resident == 1 ? tag_partial(v, parity) : bits_of(v);
                }
                // (slot group 16 i + quad: the quads of this store are neighbours in memory, see slot_owner)
                const uint32_t off =
                    (uint32_t)((((int64_t)seg * a.b_pad + col) * a.m_pad + (int64_t)panel * kBPanelRows + (16 * i + quad) * kBFinal) * 4);
                if (a.resident != 1) store_partials<kBFinal, 0>(part_rsrc, off, out);
                else if (a.publish) store_partials<kBFinal, kAuxSc1>(part_rsrc, off, out);
            }
        }
    }
    }
    if (a.resident == 2) reduce_segments_local<YT, AT, kBFinal>(a, rb, cp, seg, launches * (unsigned)a.segments, xcd_as_expected, lds);
    else if (a.resident) reduce_segments_resident<YT, AT, kBFinal>(a, parity, unit * a.col_passes + cp, lds);
}

// Pipelined form: the table of the next k-tile is built while the current one is
// gathered from.
//   A k-tile is 16 table groups (32 k-columns, 64 KiB of table); LDS holds two
//   tables.  All 64 lanes of a wavefront look up the same 16 groups (lane j of
//   each 16-lane row starts at group j and rotates), each for rows of its own:
//   a panel is 512 rows (8 rows per lane), a lane owns rows 64 s + lane, no
//   fold across lanes.  While the wavefronts gather from table `gen & 1` every
//   thread writes its 8 entries of table `(gen + 1) & 1`, one after every
//   second code load (with 4 rows per lane: 4 entries, every fourth), so the
//   build costs its LDS writes and nothing else: no build phase, and one
//   barrier per k-tile (everyone has finished reading the old table and
//   writing the new one).  The activations of k-tile gen + 2 are fetched during
//   k-tile gen and handed over through `xs` at that barrier.
//   A workgroup runs through a segment of its row block's k-tiles, or -- with the
//   k-tiles dealt evenly (BatchedArgs::dealt, chosen by pipe_form_dealt) -- through
//   an equal share of the k-tiles of all row blocks of its column pass, which may
//   end one row block and begin the next: the loop below then goes on with
//   k-tile 0 of the panels 8 further on, storing and clearing its sums at the
//   border.
constexpr int kPG = 16;                   // table groups per k-tile
constexpr int kPTableBytes = 256 * kPG * 16;
// kPLB = rows (code bytes) a lane takes per load: 8 (8 wavefronts, 512-row panels) or 4
// (16 wavefronts, 256-row panels, four wavefronts per SIMD; measured no faster, and its
// variant with scales spills registers: kept as a tuning aid).
template <int LB> constexpr int pipe_waves() { return 64 / LB; }

template <typename XT, typename YT, typename AT, bool kScaled, bool kCodes8, int kPLB>
__global__ void __launch_bounds__(pipe_waves<kPLB>() * 64)
batched_pipe_kernel(BatchedArgs a)
{
    constexpr int kPWaves = pipe_waves<kPLB>();
    constexpr int kPEach = 256 * kPG / (kPWaves * 64);      // entries a thread writes per table: 8 or 4
    constexpr int kBuildEvery = kLoadsPerPanel / kPEach;    // one entry after every second / fourth code load
    constexpr int kPanelRows = 64 * kPLB;
    using LoadT = typename LaneLoad<kPLB>::type;
    __shared__ __align__(16) unsigned char lds[2 * kPTableBytes];
    __shared__ __align__(16) _Float16 xs[2][2 * kPG][kBC];  // activations of a k-tile: [k-column][batch column]
    __shared__ unsigned launch_count;

    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int wave = tid >> 6;
    const int j = lane & 15;

    // block id -> (k-segment, row block, column pass), as in batched_kernel
    const uint32_t bid = blockIdx.x;
    int rb, seg, cp, unit;
    if (a.resident == 2) {
        local_block(a, bid, rb, seg, cp);  // (the grid is exactly the workgroups there are)
        unit = rb * a.segments + seg;
    } else {
        const uint32_t n = bid / kXcds;
        const uint32_t hi = fast_div(n, a.div_col_passes);
        cp = (int)(n - hi * (uint32_t)a.col_passes);
        unit = (int)((bid % kXcds) + kXcds * hi);
        if (unit >= a.units) return;
        rb = (int)fast_div((uint32_t)unit, a.div_segments);
        seg = unit - rb * a.segments;
    }
    const bool xcd_as_expected = a.resident != 2 || xcc_id() == bid % kXcds;
    const int64_t col0 = (int64_t)cp * kBC;
    // The k-tiles this workgroup runs through: a segment of its row block -- or, with the k-tiles dealt evenly, a run
    // of scale blocks of the row-block-major sequence of its column pass, which may go from the end of one row block
    // (its last k-tiles) into the start of the next (k-tile 0 of the panels 8 further on): the tables depend on the
    // column pass and the k-tile alone, so the pipeline of activations, table builds and code loads runs across that
    // border like across any other k-tile border; only the sums are stored and cleared there.  (Row blocks are cut
    // into different numbers of shares: the second launch works out how many sums each row block has.)
    int kt_begin = seg * a.tiles_per_segment;
    int ngen = min(a.tiles_per_segment, a.ktiles - kt_begin);  // >= 1: the host makes no empty segment
    if (a.dealt) {
        // scale block B of the sequence -> its first k-tile, counted through the row blocks
        auto first_tile = [&](int B) -> int {
            const int r = (int)fast_div((uint32_t)B, a.div_blocks_per_rb);
            return r * a.ktiles + min((B - r * a.blocks_per_rb) * a.tiles_per_block, a.ktiles);
        };
        const int b0 = unit * a.deal_blocks, b1 = min(b0 + a.deal_blocks, a.deal_total);
        rb = (int)fast_div((uint32_t)b0, a.div_blocks_per_rb);
        seg = unit - (int)fast_div((uint32_t)(rb * a.blocks_per_rb), a.div_deal_blocks);
        const int t0 = first_tile(b0);
        kt_begin = t0 - rb * a.ktiles;
        ngen = first_tile(b1) - t0;
    }
    const int panel_first = rb * a.panels_per_wg + wave;
    const bool active_first = wave < a.panels_per_wg && panel_first < a.panels_total;

    const XT* __restrict__ X = (const XT*)a.X;

    // ---- activations of a k-tile: thread (c, kc) of the first 256 fetches X(32 kt + kc, col0 + c)
    const int xc = (tid >> 5) & (kBC - 1), xkc = tid & 31;
    auto x_fetch = [&](int kt) -> XT {
        const int64_t kk = (int64_t)kt * (2 * kPG) + xkc;
        const bool live = (col0 + xc < a.b) && (kk < a.k);
        // (8-bit weights: slots 2g and 2g + 1 both hold the column of group g)
        return X[live ? (col0 + xc) * a.ldx + (kCodes8 ? (kk >> 1) : kk) : 0];  // (a clamped, always valid address; masked below)
    };
    auto x_store = [&](int buf, int kt, XT raw) {
        const int64_t kk = (int64_t)kt * (2 * kPG) + xkc;
        const bool live = (col0 + xc < a.b) && (kk < a.k);
        if (tid < 2 * kPG * kBC) xs[buf][xkc][xc] = live ? to_half<XT>(raw) : (_Float16)0.0f;
        flag_range<XT>(a, live, raw);
    };

    // ---- phase 1: thread (g, c1, part) writes the entries c0 = kPEach part .. kPEach part + kPEach - 1 of its (g, c1):
    // L(c0 | c1 << 4, g, c) = b(c0) X(2g, c) + b(c1) X(2g + 1, c) in packed fp16
    const int bg = tid & (kPG - 1), bc1 = (tid >> 4) & 15, bpart = tid >> 8;
    _Float16 w_mine[kPEach];  // the values of this thread's low codes (8-bit weights: of its 8 code bytes)
    _Float16 w1_mine = (_Float16)0.0f;
    if constexpr (kCodes8) {
#pragma unroll
        for (int v4 = 0; v4 < kPEach / 4; ++v4) {
            const float4 q4 = *(const float4*)(a.values256 + bc1 * 16 + bpart * kPEach + v4 * 4);
            w_mine[v4 * 4 + 0] = (_Float16)q4.x; w_mine[v4 * 4 + 1] = (_Float16)q4.y;
            w_mine[v4 * 4 + 2] = (_Float16)q4.z; w_mine[v4 * 4 + 3] = (_Float16)q4.w;
        }
    } else {
        w1_mine = (_Float16)a.values.v[bc1];
#pragma unroll
        for (int cc = 0; cc < kPEach; ++cc) w_mine[cc] = (_Float16)a.values.v[(bpart * kPEach + cc) & 15];
    }
    const uint32_t build_off = (uint32_t)((bc1 * 16 + bpart * kPEach) * kBCodeStride + bg * 16);
    h2 bx0[4], btop[4];  // this thread's group of the table being built: X(2g, .) and b(c1) X(2g + 1, .)
    auto build_operands = [&](int xbuf) {
        h2 x1[4];
        __builtin_memcpy(bx0, &xs[xbuf][2 * bg][0], 16);
        __builtin_memcpy(x1, &xs[xbuf][2 * bg + 1][0], 16);
#pragma unroll
        for (int p = 0; p < 4; ++p) btop[p] = kCodes8 ? h2{(_Float16)0.0f, (_Float16)0.0f} : x1[p] * h2{w1_mine, w1_mine};
    };
    auto build_entry = [&](unsigned char* table, int cc) {
        const _Float16 w = w_mine[cc];
        h2 e[4];
#pragma unroll
        for (int p = 0; p < 4; ++p) e[p] = __builtin_elementwise_fma(h2{w, w}, bx0[p], btop[p]);
        __builtin_memcpy(table + build_off + cc * kBCodeStride, e, 16);
    };

    // ---- the code stream of this wavefront: the k-tiles of a panel follow each other in memory.  With 8 rows per
    // lane two consecutive loads of a lane (8 bytes each) are stored side by side and fetched as one 16-byte load:
    // half as many memory instructions for the same bytes (with the codes cache-resident the step takes as long as
    // from memory, without the load instructions a twelfth less: it is their issue that costs, not their data).
    constexpr bool kPair = kPLB == 8;
    using RingT = typename std::conditional<kPair, uint4, LoadT>::type;
    constexpr int kSlots = kPair ? kBRing / 2 : kBRing;                     // ring slots (the same bytes in flight)
    constexpr int kSlotsPerTile = kPair ? kLoadsPerPanel / 2 : kLoadsPerPanel;
    // (k-tile kt of the panel 8 r further on is k-tile kt + 8 r ktiles of this one)
    const RingT* __restrict__ tiled = (const RingT*)a.tiled + (int64_t)panel_first * a.ktiles * (kSlotsPerTile * 64) + lane;
    auto code_at = [&](int kt, int u) -> const RingT* {
        if constexpr (MSGEMM_PIPE_LEAVE_OUT & 64) kt = kt_begin;  // (every k-tile re-reads the first one's codes: cache hits)
        return tiled + ((int64_t)kt * kSlotsPerTile + u) * 64;
    };
    RingT ring[kSlots];

    // k-tile that follows kt in the sequence (the next row block starts at its k-tile 0 again)
    auto tile_after = [&](int kt) -> int { return kt + 1 == a.ktiles ? 0 : kt + 1; };
    XT xraw = x_fetch(kt_begin);
    XT xraw1 = x_fetch(ngen > 1 ? tile_after(kt_begin) : kt_begin);
    if (active_first) {
#pragma unroll
        for (int u = 0; u < kSlots; ++u) {
            ring[u] = load_codes(code_at(kt_begin, u));
            __builtin_amdgcn_sched_barrier(0);  // loads return in issue order: keep slot 0 first
        }
    }
    count_launch(a, &launch_count);
    x_store(0, kt_begin, xraw);
    if (ngen > 1) x_store(1, tile_after(kt_begin), xraw1);
    lds_barrier();
    build_operands(0);
#pragma unroll
    for (int cc = 0; cc < kPEach; ++cc) build_entry(lds, cc);
    lds_barrier();

    h4 onehot;  // column (lane % 4) of the 4 x 4 identity
#pragma unroll
    for (int e = 0; e < 4; ++e) onehot[e] = (_Float16)((lane & 3) == e ? 1.0f : 0.0f);
    f4 dlo[kPLB], dhi[kPLB];  // sums of the current scale block (of everything, without scales)
    f4 ylo[kScaled ? kPLB : 1], yhi[kScaled ? kPLB : 1];
#pragma unroll
    for (int s = 0; s < kPLB; ++s) {
        dlo[s] = f4{0, 0, 0, 0};
        dhi[s] = f4{0, 0, 0, 0};
        if constexpr (kScaled) {
            ylo[s] = f4{0, 0, 0, 0};
            yhi[s] = f4{0, 0, 0, 0};
        }
    }

    const unsigned launches = a.resident ? launch_count : 0u, parity = launches & 1u;
    int kt = kt_begin;     // k-tile within the row block
    int rb_now = rb, seg_now = seg;
    int kt_code = kt_begin;  // the same k-tile as the code stream counts it (from the first row block's panel on)
    for (int gen = 0; gen < ngen; ++gen) {
        const bool more = gen + 1 < ngen;   // a table to build during this k-tile
        const bool more2 = gen + 2 < ngen;  // activations to fetch for the one after it
        const bool last_of_row_block = kt + 1 == a.ktiles;
        const int panel = rb_now * a.panels_per_wg + wave;
        const bool active = wave < a.panels_per_wg && panel < a.panels_total;
        // (a wavefront without a panel in the next row block stays with its own codes: every address it forms is valid)
        const bool active_next = !last_of_row_block || panel + a.panels_per_wg < a.panels_total;
        if (more2 && !(MSGEMM_PIPE_LEAVE_OUT & 128)) xraw = x_fetch(tile_after(tile_after(kt)));
        if (more) build_operands((gen + 1) & 1);
        unsigned char* next_table = lds + ((gen + 1) & 1) * kPTableBytes;
        const uint32_t table_bit = (uint32_t)(gen & 1) << 16;
        struct alignas(2 * kPLB) LaneScales { __half h[kPLB]; };
        LaneScales qraw;
        if constexpr (kScaled) {
            if (active) {
                const int blk = (int)fast_div((uint32_t)kt, a.div_tiles_per_block);
                qraw = *(const LaneScales*)(a.scales + (((int64_t)blk * a.panels_total + panel) * 64 + lane) * kPLB);
            }
        }
        // (the last tile re-requests its own tail: harmless, and branch-free)
        const int kt_here = kt_code;
        const int kt_next = (more && active_next) ? (last_of_row_block ? kt_code + (a.panels_per_wg - 1) * a.ktiles + 1 : kt_code + 1) : kt_code;
        // One k-tile as straight-line code (no branch inside, so the counters of the
        // code loads in flight stay known to the compiler): look-ups if this
        // wavefront has a panel, an entry of the next table after every second load
        // if there is a next table.
        auto tile = [&](auto gather_c, auto build_c) {
            constexpr bool kGather = decltype(gather_c)::value, kBuild = decltype(build_c)::value;
            // Look-up s of load t.  byte 0 of the address: the slot of this lane's group within a
            // code's 256 bytes; byte 1: the code; byte 2: the table.
            uint4 e[kPLB];
            // (the slot advances by one group per load; kept in one register that is updated,
            // not in sixteen precomputed ones)
            uint32_t lane_off = (uint32_t)j * 16u | table_bit;
            auto next_slot = [&]() {
                lane_off = ((lane_off + 16u) & 0xf0u) | table_bit;
                asm volatile("" : "+v"(lane_off));
            };
            // the word with code byte s of load t
            auto code_word = [&](int t, int s) -> uint32_t {
                if constexpr (kPair) {
                    const uint4 d = ring[(t / 2) % kSlots];
                    return (t & 1) ? ((s >> 2) ? d.w : d.z) : ((s >> 2) ? d.y : d.x);
                } else {
                    return load_word<kPLB>(ring[t % kSlots], s >> 2);
                }
            };
            auto look_up = [&](int t, int s) {
                const uint32_t addr =
                    __builtin_amdgcn_perm(code_word(t, s), lane_off, 0x0c020000u | ((4u + (s & 3)) << 8));
                if constexpr (MSGEMM_PIPE_LEAVE_OUT & 2) e[s] = uint4{addr, addr, addr, addr};
                else e[s] = *(const uint4*)(lds + addr);
            };
            // once the addresses of load t are out, its ring slot (with pairs: after the second load of the slot)
            // takes the slot kSlots ahead
            auto refill = [&](int t) {
                if constexpr (MSGEMM_PIPE_LEAVE_OUT & 32) return;
                if (kPair && (t & 1) == 0) return;
                const int u = kPair ? t / 2 : t;
                ring[u % kSlots] = load_codes((u + kSlots < kSlotsPerTile) ? code_at(kt_here, u + kSlots)
                                                                           : code_at(kt_next, u + kSlots - kSlotsPerTile));
            };
            if constexpr (kGather) {
#pragma unroll
                for (int s = 0; s < kPLB; ++s) look_up(0, s);
                refill(0);
                next_slot();
                __builtin_amdgcn_sched_barrier(0);
            }
#pragma unroll
            for (int t = 0; t < kLoadsPerPanel; ++t) {
                if constexpr (kGather) {
                    // the entry of look-up s is added, then its register takes look-up s of the next
                    // load: kPLB look-ups stay in flight
#pragma unroll
                    for (int s = 0; s < kPLB; ++s) {
                        if constexpr (MSGEMM_PIPE_LEAVE_OUT & 1) {
                            asm volatile("" ::"v"(e[s].x), "v"(e[s].y), "v"(e[s].z), "v"(e[s].w));  // demanded, by no instruction
                        } else {
                            h4 lo, up;
                            __builtin_memcpy(&lo, &e[s].x, 8);
                            __builtin_memcpy(&up, &e[s].z, 8);
                            dlo[s] = __builtin_amdgcn_mfma_f32_4x4x4f16(lo, onehot, dlo[s], 0, 0, 0);
                            dhi[s] = __builtin_amdgcn_mfma_f32_4x4x4f16(up, onehot, dhi[s], 0, 0, 0);
                        }
                        if (t + 1 < kLoadsPerPanel) look_up(t + 1, s);
                        if constexpr (MSGEMM_PIPE_SCHED == 0) __builtin_amdgcn_sched_barrier(0);
                    }
                    if constexpr (MSGEMM_PIPE_SCHED == 1) {
                        if (t + 1 < kLoadsPerPanel) {
#pragma unroll
                            for (int s = 0; s < kPLB; ++s) {  // two adds, then the look-up that takes their register
                                __builtin_amdgcn_sched_group_barrier(0x008, 2, 0);
                                __builtin_amdgcn_sched_group_barrier(0x100, 1, 0);
                            }
                        }
                    }
                    if (t + 1 < kLoadsPerPanel) refill(t + 1);
                    next_slot();
                }
                if constexpr (kBuild) {
                    if constexpr (!(MSGEMM_PIPE_LEAVE_OUT & 4))
                    if (t % kBuildEvery == 0) build_entry(next_table, t / kBuildEvery);
                }
                __builtin_amdgcn_sched_barrier(0);
            }
        };
        using yes = std::true_type;
        using no = std::false_type;
        if (active && more) tile(yes{}, yes{});
        else if (active) tile(yes{}, no{});
        else if (more) tile(no{}, yes{});
        if constexpr (kScaled) {
            // a scale block ends with this k-tile: y += q(row) * block sum (Section 3.3).
            // Register i of the accumulators belongs to the row of quad lane i.
            const int blk = (int)fast_div((uint32_t)kt, a.div_tiles_per_block);
            if (active && (!more || last_of_row_block || (kt + 1) == (blk + 1) * a.tiles_per_block)) {
#pragma unroll
                for (int s = 0; s < kPLB; ++s) {
                    const float qf = __half2float(qraw.h[s]);
                    const float q0 = quad_broadcast<0>(qf), q1 = quad_broadcast<1>(qf);
                    const float q2 = quad_broadcast<2>(qf), q3 = quad_broadcast<3>(qf);
                    ylo[s][0] = fmaf(q0, dlo[s][0], ylo[s][0]); yhi[s][0] = fmaf(q0, dhi[s][0], yhi[s][0]);
                    ylo[s][1] = fmaf(q1, dlo[s][1], ylo[s][1]); yhi[s][1] = fmaf(q1, dhi[s][1], yhi[s][1]);
                    ylo[s][2] = fmaf(q2, dlo[s][2], ylo[s][2]); yhi[s][2] = fmaf(q2, dhi[s][2], yhi[s][2]);
                    ylo[s][3] = fmaf(q3, dlo[s][3], ylo[s][3]); yhi[s][3] = fmaf(q3, dhi[s][3], yhi[s][3]);
                    dlo[s] = f4{0, 0, 0, 0};
                    dhi[s] = f4{0, 0, 0, 0};
                }
            }
        }
        // ---- the last k-tile of the share, or of a row block: the sums leave
        if (!more || last_of_row_block) {
        const int seg = seg_now;
        if (active) {
    // ---- lane (quad b, j'), register (s, i) holds row 64 s + 4 b + i of the panel,
    // column 4 h + j' of the pass (the matrix cores hand the sums back transposed within a quad)
    // (computed here, from a lane id the compiler cannot see through: hoisted out of the k-tile loop, the addresses of
    // these stores would occupy registers that the look-ups need)
    int lane_here = lane;
    asm volatile("" : "+v"(lane_here));
    const int quad = lane_here >> 2, jq = lane_here & 3;
    YT* __restrict__ Y = (YT*)a.Y;
    __amdgpu_buffer_rsrc_t part_rsrc =
        __builtin_amdgcn_make_buffer_rsrc((void*)a.partials, 0, (int)a.partial_span, 0x00020000);
#pragma unroll
    for (int h = 0; h < 2; ++h) {
        const int64_t col = col0 + 4 * h + jq;
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            float fin[kPLB];
#pragma unroll
            for (int s = 0; s < kPLB; ++s) {
                if constexpr (kScaled) fin[s] = h ? yhi[s][i] : ylo[s][i];
                else fin[s] = h ? dhi[s][i] : dlo[s][i];
            }
            const int owner = 4 * quad + i;  // the lane whose look-ups these sums come from
            if (a.direct) {
#pragma unroll
                for (int s = 0; s < kPLB; ++s) {
                    const int64_t row = (int64_t)panel * kPanelRows + 64 * s + owner;
                    if (row < a.m && col < a.b) {
                        if constexpr (__is_same(AT, int)) Y[col * a.ldy + row] = (YT)__float2int_rn(fin[s]);
                        else Y[col * a.ldy + row] = to_output<YT, float>(fin[s]);
                    }
                }
            } else {
                unsigned out[kPLB];
#pragma unroll
                for (int s = 0; s < kPLB; ++s) {
                    AT v;
                    if constexpr (__is_same(AT, int)) v = __float2int_rn(fin[s]);
                    else v = fin[s];
                    out[s] = a.resident == 1 ? tag_partial(v, parity) : bits_of(v);
                }
                // (slot group 16 i + quad: the quads of this store are neighbours in memory, see slot_owner)
                const uint32_t off =
                    (uint32_t)((((int64_t)seg * a.b_pad + col) * a.m_pad + (int64_t)panel * kPanelRows + (16 * i + quad) * kPLB) * 4);
                if (a.resident != 1) store_partials<kPLB, 0>(part_rsrc, off, out);
                else if (a.publish) store_partials<kPLB, kAuxSc1>(part_rsrc, off, out);
            }
        }
    }
        // the sums of the next row block start at zero
#pragma unroll
        for (int s = 0; s < kPLB; ++s) {
            dlo[s] = f4{0, 0, 0, 0};
            dhi[s] = f4{0, 0, 0, 0};
            if constexpr (kScaled) {
                ylo[s] = f4{0, 0, 0, 0};
                yhi[s] = f4{0, 0, 0, 0};
            }
        }
        }
        }
        if (more2 && !(MSGEMM_PIPE_LEAVE_OUT & 128)) x_store(gen & 1, tile_after(tile_after(kt)), xraw);
        // everyone has finished reading table gen & 1 and writing the other one (and the activations)
        if (more && !(MSGEMM_PIPE_LEAVE_OUT & 8)) lds_barrier();
        if (last_of_row_block) {
            kt = 0;
            rb_now += 1;
            seg_now = 0;  // (this workgroup is the first to touch the next row block)
            kt_code += (a.panels_per_wg - 1) * a.ktiles + 1;
        } else {
            kt += 1;
            kt_code += 1;
        }
    }
    // (the sums are added inside the launch only when the k-tiles are not dealt)
    if (a.resident == 2) reduce_segments_local<YT, AT, kPLB>(a, rb, cp, seg, launches * (unsigned)a.segments, xcd_as_expected, lds);
    else if (a.resident) reduce_segments_resident<YT, AT, kPLB>(a, parity, unit * a.col_passes + cp, lds);
}

// One-off reorder of the block scales ([m][nblocks]) for the batched kernel:
// [block][panel][lane][s] = scale of the row behind look-up s of that lane.
template <int NQ, int kBLB>
__global__ void __launch_bounds__(256)
repack_scales_batched_kernel(const __half* __restrict__ scales, __half* __restrict__ ordered, int64_t m,
                             int64_t nblocks, int64_t panels)
{
    constexpr int kBPanelRows = 64 * kBLB / NQ;
    const int64_t total = nblocks * panels * 64 * kBLB;
    for (int64_t o = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; o < total;
         o += (int64_t)gridDim.x * blockDim.x) {
        int64_t r = o;
        const int s = (int)(r % kBLB); r /= kBLB;
        const int lane = (int)(r % 64); r /= 64;
        const int64_t panel = r % panels;
        const int64_t blk = r / panels;
        const int64_t row = panel * kBPanelRows + panel_row<NQ, kBLB>(lane >> 4, lane & 15, s);
        ordered[o] = row < m ? scales[row * nblocks + blk] : __float2half(1.0f);
    }
}

}  // namespace

// int8 activations: a segment's sums are kept in fp32 and must stay exact integers.  An entry is
// at most 8 * 128 * 2 = 2^11 in magnitude, so a sum over 2^13 groups stays within 2^24: a segment
// is at most 8192 groups (16384 k-columns) long, whatever was chosen or forced.  (int8 plans have
// no scale blocks, so any number of k-tiles is a valid segment.)
static void cap_exact_segment(Plan& p)
{
    if (p.x_dtype != MSGEMM_I8) return;
    const int max_tiles = 8192 / p.fs.groups;
    if (p.tiles_per_segment > max_tiles) p.tiles_per_segment = max_tiles;
}

// Segment length: the longest (a multiple of the scale block) that still gives
// every compute unit a workgroup, preferring grids that fill whole rounds.
static int64_t phase_form_segments(int64_t blocks, int64_t units_per_seg, int64_t cus)
{
    int64_t best_s = blocks;
    double best_eff = -1.0;
    for (int64_t per = blocks; per >= 1; --per) {  // scale blocks per segment, longest first
        const int64_t segs = (blocks + per - 1) / per;
        const int64_t wgs = segs * units_per_seg;
        if (4 * wgs < 3 * cus && per > 1) continue;  // too few workgroups: shorter segments
        const double eff = (double)wgs / (double)(((wgs + cus - 1) / cus) * cus);
        if (eff > best_eff + 0.05) { best_eff = eff; best_s = segs; }  // shorter only if clearly better balanced
        if (wgs >= 8 * cus) break;  // enough rounds to balance: stop shortening
    }
    return best_s;
}

void batched_choose_segments(Plan& p)
{
    const int tpb = p.scale_group > 0 ? (int)(p.scale_group / (2 * p.fs.groups)) : 1;
    const int64_t blocks = (p.ktiles + tpb - 1) / tpb;  // indivisible runs of k-tiles
    int64_t best_s = phase_form_segments(blocks, p.row_blocks * p.col_passes, p.cus);
    const int forced = p.opt.batched_segments;
    if (forced >= 1 && forced <= blocks) best_s = forced;
    const int64_t per = (blocks + best_s - 1) / best_s;
    p.tiles_per_segment = (int)(per * tpb);
    cap_exact_segment(p);
    p.segments = (int)((p.ktiles + p.tiles_per_segment - 1) / p.tiles_per_segment);
}

// Pipelined form: panels per workgroup and segment length together, by a model
// of the time (microseconds).  A workgroup costs a start-up (activations, first
// table, first codes) and a time per k-tile; workgroups run in rounds of one
// per compute unit; the second pass reads one partial sum per segment and
// output.
static double pipe_form_choice(int64_t panels, int64_t ktiles, int tpb, int col_passes, int64_t cus, int lane_bytes,
                               int waves, int& best_ppw, int64_t& best_per)
{
    const int64_t blocks = (ktiles + tpb - 1) / tpb;  // indivisible runs of k-tiles
    const double outputs = (double)panels * (64 * lane_bytes) * col_passes * kBC;
    double best = 1e300;
    best_ppw = waves;
    best_per = blocks;
    // Measured: a k-tile takes a workgroup 2.75 us + 0.12 us per active wavefront (8 rows per
    // lane; 1.9 + 0.085 with 4): what bounds it is the rate at which a wavefront issues its
    // look-ups, and wavefronts that share a SIMD overlap almost completely.  Start-up, launch
    // and tail of a workgroup: 6.5 us.  Every panel count is tried: one wavefront less per
    // workgroup can turn a grid that leaves compute units idle into one that fills them.
    const double tile_base_us = lane_bytes == 8 ? 2.75 : 1.9, tile_wave_us = lane_bytes == 8 ? 0.12 : 0.085;
    for (int ppw = waves; ppw >= 1; --ppw) {
        const int64_t row_blocks = (panels + ppw - 1) / ppw;
        const double tile_us = tile_base_us + tile_wave_us * ppw;
        for (int64_t per = blocks; per >= 1; --per) {
            const int64_t segs = (blocks + per - 1) / per;
            if ((blocks + segs - 1) / segs != per) continue;  // the same split again
            const int64_t wgs = segs * row_blocks * col_passes;
            const int64_t rounds = (wgs + cus - 1) / cus;
            double cost = (double)rounds * (6.5 + (double)(per * tpb) * tile_us);
            if (segs > 1) cost += 3.0 + (double)segs * outputs * 4.0 / 3.0e6;
            if (cost < best) { best = cost; best_ppw = ppw; best_per = per; }
            if (rounds > 64) break;  // shorter segments only add rounds from here on
        }
    }
    return best;
}

// The form with a build phase, modelled (microseconds): 5 us of start-up, then 2.3 us of table build and 0.44 us of
// look-ups per active wavefront for every k-tile of 64 columns; workgroups in rounds of one per compute unit; the
// second pass reads one partial sum per segment and output.  `ppw` panels of 256 rows per workgroup.
static double phase_form_cost(int64_t panels, int64_t ktiles, int tpb, int col_passes, int64_t cus, int ppw)
{
    const int64_t row_blocks = (panels + ppw - 1) / ppw;
    const int64_t blocks = (ktiles + tpb - 1) / tpb;  // indivisible runs of k-tiles
    const int64_t segs = phase_form_segments(blocks, row_blocks * col_passes, cus);
    const int64_t tiles_per_seg = ((blocks + segs - 1) / segs) * tpb;
    const int64_t wgs = segs * row_blocks * col_passes;
    double us = (double)((wgs + cus - 1) / cus) * (5.0 + (double)tiles_per_seg * (2.3 + 0.44 * ppw));
    if (segs > 1) us += 3.0 + (double)segs * (double)(panels * 256) * col_passes * kBC * 4.0 / 3.0e6;
    return us;
}

// Panels per workgroup of that form.  As many as its wavefronts while that still gives every compute unit a
// workgroup, else half, a quarter, ...; between such a count and the next lower one the model above decides: one
// panel less per workgroup can turn a grid that leaves compute units idle into one that fills them (56 panels:
// 7 row blocks of 8 are 224 workgroups on 256 compute units, 8 of 7 are 256 -- measured 2 % faster).
int batched_phase_form_panels(int64_t panels, int64_t ktiles, int64_t scale_group, int col_passes, int64_t cus)
{
    int ppw = 8;
    while (ppw > 1 && ktiles * col_passes * ((panels + ppw - 1) / ppw) < cus) ppw >>= 1;
    const int tpb = scale_group > 0 ? (int)(scale_group / (2 * kBG)) : 1;
    if (tpb < 1) return ppw;
    int best = ppw;
    double best_us = phase_form_cost(panels, ktiles, tpb, col_passes, cus, ppw);
    for (int c = ppw - 1; c > ppw / 2 && c >= 1; --c) {
        const double us = phase_form_cost(panels, ktiles, tpb, col_passes, cus, c);
        if (us < best_us - 1e-9) { best_us = us; best = c; }
    }
    return best;
}

// Which of the two forms a problem gets: the one the models predict to be faster, the pipelined
// one only when by more than a tenth (the models are good to about that).
bool batched_pipelined_is_faster(int64_t m, int64_t k, int64_t b, int64_t scale_group, int cus)
{
    const int col_passes = (int)((b + kBC - 1) / kBC);
    // pipelined form: 512-row panels, k-tiles of 32 columns
    int ppw;
    int64_t per;
    const double pipe_us = pipe_form_choice((m + 511) / 512, (k / 2 + kPG - 1) / kPG, scale_group > 0 ? (int)(scale_group / (2 * kPG)) : 1,
                                            col_passes, cus, 8, 8, ppw, per);
    // form with a build phase: 256-row panels, k-tiles of 64 columns
    const int64_t panels = (m + 255) / 256, ktiles = (k / 2 + kBG - 1) / kBG;
    const int tpb = scale_group > 0 ? (int)(scale_group / (2 * kBG)) : 1;
    if (tpb < 1) return true;  // scale blocks of 32 columns: only the pipelined form has k-tiles that small
    const int ppw0 = batched_phase_form_panels(panels, ktiles, scale_group, col_passes, cus);
    const double phase_us = phase_form_cost(panels, ktiles, tpb, col_passes, cus, ppw0);
    return pipe_us < 0.9 * phase_us;
}

// The pipelined form with its k-tiles dealt evenly (8 rows per lane): every workgroup has all its wavefronts busy
// (row blocks of `waves` panels) and as many scale blocks as any other, taken from the row-block-major sequence of
// one column pass -- so a workgroup's share may end one row block and begin the next (two runs, a partial sum each),
// and row blocks are cut into different numbers of runs.  Worth it where equal segments cannot fill the device:
// 56 panels x 8 passes are 224 workgroups of 8 wavefronts or 256 of 7 (4 segments, 64 k-tiles each); dealt, 256
// workgroups of 8 run through 56 k-tiles (measured: 245 -> 233 us).  Modelled like the other grids.
// Returns the modelled time (1e300: not possible); `deal_blocks` scale blocks per workgroup, `max_runs` the most
// runs a row block is cut into (the partial sums per output).
static double pipe_form_dealt(int64_t panels, int64_t ktiles, int tpb, int col_passes, int64_t cus, int waves,
                              int64_t max_tiles, int64_t& deal_blocks, int& max_runs)
{
    const int64_t blocks = (ktiles + tpb - 1) / tpb;
    const int64_t row_blocks = (panels + waves - 1) / waves;
    // workgroups per column pass: one round, and no XCD with more workgroups than compute units (the column passes of
    // a share run on one XCD, for the codes they have in common)
    const int64_t chunks = kXcds * ((cus / kXcds) / col_passes);
    if (chunks < 2 || row_blocks * blocks < 2 * chunks) return 1e300;
    const int64_t total = row_blocks * blocks;
    deal_blocks = (total + chunks - 1) / chunks;
    if (deal_blocks > blocks || deal_blocks * tpb > max_tiles) return 1e300;  // (a share spans two row blocks at most)
    max_runs = 0;
    for (int64_t rb = 0; rb < row_blocks; ++rb) {
        const int runs = (int)(((rb + 1) * blocks - 1) / deal_blocks - (rb * blocks) / deal_blocks + 1);
        if (runs > max_runs) max_runs = runs;
    }
    if (max_runs < 2) return 1e300;
    const double outputs = (double)panels * 512 * col_passes * kBC;
    // (a share that crosses a row-block border stores its sums in mid-stream: about 6 us, measured on 20480 x 5120 x 64,
    // where equal segments are as long as the shares)
    return 6.5 + 6.0 + (double)(deal_blocks * tpb) * (2.75 + 0.12 * waves) + 3.0 + (double)max_runs * outputs * 4.0 / 3.0e6;
}

void batched_choose_rows_and_segments(Plan& p, int64_t panels, int& ppw_out)
{
    const int tpb = p.scale_group > 0 ? (int)(p.scale_group / (2 * p.fs.groups)) : 1;
    const int64_t blocks = (p.ktiles + tpb - 1) / tpb;  // indivisible runs of k-tiles
    int best_ppw;
    int64_t best_per;
    const double regular_us =
        pipe_form_choice(panels, p.ktiles, tpb, p.col_passes, p.cus, p.fs.lane_bytes, p.fs.waves, best_ppw, best_per);
    p.deal_blocks = 0;
    // k-tiles dealt evenly: when the model sees 3 % or more in it (option batched_deal: 1 never, 2 whenever possible)
    if (p.fs.lane_bytes == 8 && p.opt.batched_deal != 1 && p.opt.panels_per_workgroup == 0 && p.opt.batched_segments == 0) {
        int64_t deal_blocks = 0;
        int max_runs = 0;
        const int64_t max_tiles = p.x_dtype == MSGEMM_I8 ? 8192 / p.fs.groups : (int64_t)1 << 40;
        const double dealt_us = pipe_form_dealt(panels, p.ktiles, tpb, p.col_passes, p.cus, p.fs.waves, max_tiles, deal_blocks, max_runs);
        if (dealt_us < 1e299 && (p.opt.batched_deal == 2 || dealt_us < 0.97 * regular_us)) {
            ppw_out = p.fs.waves;
            p.deal_blocks = (int)deal_blocks;
            p.tiles_per_segment = (int)(deal_blocks * tpb);
            p.segments = max_runs;
            return;
        }
    }
    const int forced_ppw = p.opt.panels_per_workgroup;
    if (forced_ppw >= 1 && forced_ppw <= p.fs.waves) best_ppw = forced_ppw;
    int64_t segs = (blocks + best_per - 1) / best_per;
    const int forced = p.opt.batched_segments;
    if (forced >= 1 && forced <= blocks) segs = forced;
    const int64_t per = (blocks + segs - 1) / segs;
    ppw_out = best_ppw;
    p.tiles_per_segment = (int)(per * tpb);
    cap_exact_segment(p);
    p.segments = (int)((p.ktiles + p.tiles_per_segment - 1) / p.tiles_per_segment);
}

int launch_repack_scales_batched(const Plan& p, hipStream_t s)
{
    const int64_t panels = p.m_pad / p.fs.panel_rows;
    int64_t blocks = (p.nblocks * panels * 64 * p.fs.lane_bytes + 255) / 256;
    if (blocks > 65536) blocks = 65536;
    if (p.fs.groups == kPG && p.fs.lane_bytes == 8)
        hipLaunchKernelGGL((repack_scales_batched_kernel<1, 8>), dim3((unsigned)blocks), dim3(256), 0, s,
                           (const __half*)p.scales, (__half*)p.scales_ordered, p.m, p.nblocks, panels);
    else if (p.fs.groups == kPG)
        hipLaunchKernelGGL((repack_scales_batched_kernel<1, 4>), dim3((unsigned)blocks), dim3(256), 0, s,
                           (const __half*)p.scales, (__half*)p.scales_ordered, p.m, p.nblocks, panels);
    else if (p.fs.lane_bytes == 8)
        hipLaunchKernelGGL((repack_scales_batched_kernel<2, 8>), dim3((unsigned)blocks), dim3(256), 0, s,
                           (const __half*)p.scales, (__half*)p.scales_ordered, p.m, p.nblocks, panels);
    else
        hipLaunchKernelGGL((repack_scales_batched_kernel<2, 4>), dim3((unsigned)blocks), dim3(256), 0, s,
                           (const __half*)p.scales, (__half*)p.scales_ordered, p.m, p.nblocks, panels);
    MSGEMM_HIP_TRY(hipGetLastError());
    return MSGEMM_OK;
}

// Does this device deal the workgroups of a launch over its XCDs in turn (id % 8 = XCD)?  The XCD-local reduction
// places its workgroups by that rule; it is how these devices are known to dispatch, but no interface promises it, so
// it is looked at once per device: a launch of 2048 small workgroups, each recording the XCD id it finds itself on.
// Called when a plan is made (it allocates and waits), never from a launch.
__global__ void xcd_probe_kernel(unsigned* out)
{
    if (threadIdx.x == 0) out[blockIdx.x] = xcc_id();
}

bool xcd_round_robin(int device, hipStream_t s)
{
    constexpr int kMaxDevices = 64, kProbe = 2048;
    static int known[kMaxDevices];  // 0 not looked at, 1 yes, 2 no
    if (device < 0 || device >= kMaxDevices) return false;
    if (known[device]) return known[device] == 1;
    unsigned* d = nullptr;
    if (hipMalloc((void**)&d, kProbe * sizeof(unsigned)) != hipSuccess) return false;
    bool ok = true;
    unsigned h[kProbe];
    for (int rep = 0; rep < 2 && ok; ++rep) {
        hipLaunchKernelGGL(xcd_probe_kernel, dim3(kProbe), dim3(64), 0, s, d);
        ok = hipMemcpyAsync(h, d, sizeof(h), hipMemcpyDeviceToHost, s) == hipSuccess && hipStreamSynchronize(s) == hipSuccess;
        for (int i = 0; i < kProbe && ok; ++i) ok = h[i] == (unsigned)(i % kXcds);
    }
    (void)hipFree(d);
    known[device] = ok ? 1 : 2;
    return ok;
}

int launch_batched(const Plan& p, const void* X, int64_t ldx, void* Y, int64_t ldy, hipStream_t s)
{
    BatchedArgs a;
    a.tiled = p.codes_tiled;
    a.X = X; a.ldx = ldx; a.Y = Y; a.ldy = ldy;
    for (int i = 0; i < 16; ++i) a.values.v[i] = p.values[i];
    a.values256 = p.values256;
    a.scales = (const __half*)p.scales_ordered;
    a.partials = p.partials;
    a.error = p.error_word;
    {
        // the largest entry is value(c0) x0 + value(c1) x1 (one product for 8-bit weights)
        float vmax = 0.0f;
        for (int i = 0; i < 16; ++i) vmax = fmaxf(vmax, fabsf(p.values[i]));
        if (p.codes8) vmax = 0.5f * p.values256_max;
        a.x_limit = vmax > 0.0f ? 65504.0f / (2.0f * vmax) : 3.0e38f;
    }
    a.m = p.m; a.k = p.k; a.b = p.b; a.m_pad = p.m_pad;
    a.b_pad = (int64_t)p.col_passes * kBC;
    a.ktiles = (int)p.ktiles;
    a.panels_total = (int)(p.m_pad / p.fs.panel_rows);
    a.panels_per_wg = p.fs.panels;
    a.row_blocks = (int)p.row_blocks;
    a.col_passes = p.col_passes;
    a.segments = p.segments;
    a.tiles_per_segment = p.tiles_per_segment;
    a.tiles_per_block = p.scale_group > 0 ? (int)(p.scale_group / (2 * p.fs.groups)) : 1;
    a.units = (int)(p.segments * p.row_blocks);
    a.direct = p.segments == 1;
    a.dealt = p.deal_blocks > 0 ? 1 : 0;
    a.deal_blocks = p.deal_blocks;
    a.blocks_per_rb = (int)((p.ktiles + a.tiles_per_block - 1) / a.tiles_per_block);
    a.deal_total = (int)(p.row_blocks * a.blocks_per_rb);
    if (a.dealt) a.units = (a.deal_total + a.deal_blocks - 1) / a.deal_blocks;  // workgroups per column pass
    a.div_blocks_per_rb = make_fastdiv((uint32_t)a.blocks_per_rb);
    a.div_deal_blocks = make_fastdiv((uint32_t)(a.dealt ? a.deal_blocks : 1));
    a.partial_span = (int64_t)p.segments * a.b_pad * p.m_pad * 4;
    a.div_col_passes = make_fastdiv((uint32_t)a.col_passes);
    a.div_segments = make_fastdiv((uint32_t)a.segments);
    a.div_tiles_per_block = make_fastdiv((uint32_t)a.tiles_per_block);
    int64_t grid = (int64_t)kXcds * a.col_passes * ((a.units + kXcds - 1) / kXcds);
    // On request (reduce_mode 3) the segments are added inside the launch, if every workgroup is resident at once:
    // each needs more than half of a compute unit's LDS, so that is one workgroup per compute unit.  Not the default:
    // the partial sums of a batch are tens of megabytes, and reading them with loads that are coherent across the
    // device inside the launch measured slower than the second launch (config 3a 30.8 against 24.7 us, config 5
    // 263 against 242), unlike the single-column forms whose sums are a megabyte.
    const int threads = (p.fs.groups == kPG) ? (64 / p.fs.lane_bytes) * 64 : (p.fs.lane_bytes == 8 ? 8 : 12) * 64;
    a.resident = (!a.direct && !a.dealt && p.epochs && p.forced_reduce == 3 && grid <= p.cus) ? 1 : 0;
    // The hand-over inside an XCD (resident = 2; reduce_mode 4 asks for it): every (row block, column pass) gets all
    // its segments onto one XCD, which needs the pairs -- or, with the passes of a row block kept together for the
    // codes they share, the row blocks -- to divide evenly over the XCDs, a workgroup per compute unit at most, and a
    // device that deals workgroup ids over its XCDs in turn (probed once, at the first plan).
    a.local_inner = 1;
    a.arrivals = nullptr;
    if (!a.direct && !a.dealt && p.epochs && p.xcd_round_robin && (p.forced_reduce == 4 || (p.forced_reduce == 0 && kLocalByDefault))) {
        const int64_t RB = p.row_blocks, CP = p.col_passes, S = p.segments;
        const int inner = (RB % kXcds == 0) ? (int)CP : 1;
        const int64_t dealt = RB * CP / inner;
        if (dealt % kXcds == 0 && RB * CP * S <= p.cus && p.cus % kXcds == 0 && (dealt / kXcds) * inner * S <= p.cus / kXcds) {
            a.resident = 2;
            a.local_inner = inner;
            a.arrivals = p.epochs + (p.epoch_words - (size_t)(RB * CP));
            grid = RB * CP * S;
        }
    }
    a.div_local_inner = make_fastdiv((uint32_t)a.local_inner);
    a.publish = p.opt.skip_publish ? 0 : 1;
    a.epochs = p.epochs;
    a.poll_limit = p.opt.poll_limit > 0 ? (unsigned)p.opt.poll_limit : kMaxFlagPolls;
    {
        int64_t pieces = a.b_pad * p.m_pad / 4, readers = (int64_t)a.units * a.col_passes;
        if (a.resident == 2) {  // the pieces of one (row block, column pass), over its segments
            pieces = (int64_t)kBC * p.fs.panels * p.fs.panel_rows / 4;
            readers = a.segments;
        }
        a.red_pieces = (int)((pieces + readers - 1) / readers);
        int g = 1;
        while (g < 8 && 2 * g <= a.segments && (int64_t)a.red_pieces * (2 * g) <= threads) g *= 2;
        a.red_groups = g;
    }
    const int lb = p.fs.lane_bytes;
    const dim3 g((unsigned)grid), blk((unsigned)(lb == 8 ? 8 : 12) * 64);
    const bool scaled = p.scales != nullptr;
    const bool pipe = p.fs.groups == kPG;
    if (pipe && lb != 8 && lb != 4) return MSGEMM_ERR_UNSUPPORTED;
    if (pipe && p.codes8 && p.x_dtype == MSGEMM_I8) return MSGEMM_ERR_UNSUPPORTED;
#define MSGEMM_PIPE_LB(XT, YT, AT, SC, C8)                                                           \
    do {                                                                                            \
        if (lb == 8) hipLaunchKernelGGL((batched_pipe_kernel<XT, YT, AT, SC, C8, 8>), g, dim3(pipe_waves<8>() * 64), 0, s, a); \
        else hipLaunchKernelGGL((batched_pipe_kernel<XT, YT, AT, SC, C8, 4>), g, dim3(pipe_waves<4>() * 64), 0, s, a);         \
    } while (0)
#define MSGEMM_BATCHED_PIPE(XD, XT, YT, AT)                                                         \
    if (pipe && p.x_dtype == XD) {                                                                  \
        if constexpr (!std::is_same<AT, int>::value) {                                              \
            if (p.codes8 && scaled) MSGEMM_PIPE_LB(XT, YT, AT, true, true);                         \
            else if (p.codes8) MSGEMM_PIPE_LB(XT, YT, AT, false, true);                             \
        }                                                                                           \
        if (p.codes8) { }                                                                           \
        else if (scaled) MSGEMM_PIPE_LB(XT, YT, AT, true, false);                                   \
        else MSGEMM_PIPE_LB(XT, YT, AT, false, false);                                              \
        MSGEMM_HIP_TRY(hipGetLastError());                                                          \
        if (!a.direct && !a.resident) return launch_reduce_second_pass(p, a.partials, Y, ldy, a.segments, a.partial_span, s); \
        return MSGEMM_OK;                                                                           \
    }
    if (!pipe && p.codes8 && (lb != 8 || p.x_dtype == MSGEMM_I8)) return MSGEMM_ERR_UNSUPPORTED;
#define MSGEMM_BATCHED(XD, XT, YT, AT)                                                              \
    if (p.x_dtype == XD) {                                                                          \
        if constexpr (!std::is_same<AT, int>::value) {                                              \
            if (p.codes8 && scaled) hipLaunchKernelGGL((batched_kernel<XT, YT, AT, true, 8, true>), g, blk, 0, s, a);  \
            else if (p.codes8) hipLaunchKernelGGL((batched_kernel<XT, YT, AT, false, 8, true>), g, blk, 0, s, a);      \
        }                                                                                           \
        if (p.codes8) { }                                                                           \
        else if (scaled && lb == 8) hipLaunchKernelGGL((batched_kernel<XT, YT, AT, true, 8, false>), g, blk, 0, s, a);   \
        else if (scaled) hipLaunchKernelGGL((batched_kernel<XT, YT, AT, true, 4, false>), g, blk, 0, s, a);              \
        else if (lb == 8) hipLaunchKernelGGL((batched_kernel<XT, YT, AT, false, 8, false>), g, blk, 0, s, a);            \
        else hipLaunchKernelGGL((batched_kernel<XT, YT, AT, false, 4, false>), g, blk, 0, s, a);                         \
        MSGEMM_HIP_TRY(hipGetLastError());                                                          \
        if (!a.direct && !a.resident) return launch_reduce_second_pass(p, a.partials, Y, ldy, a.segments, a.partial_span, s); \
        return MSGEMM_OK;                                                                           \
    }
    MSGEMM_BATCHED_PIPE(MSGEMM_F16, __half, __half, float)
    MSGEMM_BATCHED_PIPE(MSGEMM_BF16, bf16_t, bf16_t, float)
    MSGEMM_BATCHED_PIPE(MSGEMM_I8, int8_t, int, int)
#undef MSGEMM_BATCHED_PIPE
#undef MSGEMM_PIPE_LB
    MSGEMM_BATCHED(MSGEMM_F16, __half, __half, float)
    MSGEMM_BATCHED(MSGEMM_BF16, bf16_t, bf16_t, float)
    MSGEMM_BATCHED(MSGEMM_I8, int8_t, int, int)
#undef MSGEMM_BATCHED
    return MSGEMM_ERR_UNSUPPORTED;
}

}  // namespace msgemm
