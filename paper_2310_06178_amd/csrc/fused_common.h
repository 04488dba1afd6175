// Device helpers shared by the fused kernels (single-column and batched).
// Internal to libmsgemm.so.
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>
#include <stdlib.h>

namespace msgemm {

constexpr int kLoadsPerPanel = 16;  // one load per group of a 16-group class
constexpr int kAuxSc1 = 16;         // buffer cache policy bit: coherent at agent scope
constexpr int kXcds = 8;            // L2 slices (XCDs); workgroups are dealt to them round-robin

// n / d for a divisor fixed at launch, without the hardware-less division
// sequence (round-up multiplier of Granlund and Montgomery; exact for every
// 32-bit n): q = (t + ((n - t) >> s1)) >> s2 with t = high word of n * magic.
struct FastDiv { uint32_t magic, s1, s2; };

inline FastDiv make_fastdiv(uint32_t d)
{
    uint32_t l = 0;
    while (l < 32 && ((uint64_t)1 << l) < d) ++l;
    FastDiv f;
    f.magic = (uint32_t)((((uint64_t)1 << 32) * (((uint64_t)1 << l) - d)) / d + 1);
    f.s1 = l < 1 ? l : 1;
    f.s2 = l - f.s1;
    return f;
}

__device__ __forceinline__ uint32_t fast_div(uint32_t n, const FastDiv& f)
{
    const uint32_t t = __umulhi(n, f.magic);
    return (t + ((n - t) >> f.s1)) >> f.s2;
}

typedef unsigned v2u __attribute__((ext_vector_type(2)));
typedef unsigned v4u __attribute__((ext_vector_type(4)));

__device__ __forceinline__ unsigned bits_of(float v) { return __float_as_uint(v); }
__device__ __forceinline__ unsigned bits_of(int v) { return (unsigned)v; }
__device__ __forceinline__ void set_bits(float& d, unsigned u) { d = __uint_as_float(u); }
__device__ __forceinline__ void set_bits(int& d, unsigned u) { d = (int)u; }

// Sum across the wave halves, two registers at a time: afterwards lanes 0..31
// hold the full sum of `a` and lanes 32..63 the full sum of `b`.
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

// A load from the code stream.  Every code byte is used once per column pass, so the loads are marked as
// streaming (non-temporal: the bytes are not kept in the caches); on the 32 MiB GEMV that alone is worth a tenth
// of the launch.  MSGEMM_STREAM_NT=0 builds with plain loads for comparison.
#ifndef MSGEMM_STREAM_NT
#define MSGEMM_STREAM_NT 1
#endif
__device__ __forceinline__ uint4 load_codes(const uint4* p)
{
#if MSGEMM_STREAM_NT
    const v4u v = __builtin_nontemporal_load((const v4u*)p);
    return make_uint4(v.x, v.y, v.z, v.w);
#else
    return *p;
#endif
}
__device__ __forceinline__ uint2 load_codes(const uint2* p)
{
#if MSGEMM_STREAM_NT
    const v2u v = __builtin_nontemporal_load((const v2u*)p);
    return make_uint2(v.x, v.y);
#else
    return *p;
#endif
}
__device__ __forceinline__ uint32_t load_codes(const uint32_t* p)
{
#if MSGEMM_STREAM_NT
    return __builtin_nontemporal_load(p);
#else
    return *p;
#endif
}

// The partial sums of one output come from workgroups that may sit on different
// XCDs, whose L2 slices are not coherent with each other.  When they are reduced
// inside the launch, partials and flags are therefore only touched with
// agent-coherent accesses (they go to the point of coherence) and ordered by
// waiting for the stores to be acknowledged before the flag is raised.  No
// cache-wide write-back / invalidate is needed.
__device__ __forceinline__ void wait_vmem()
{
    asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
}

constexpr unsigned kMaxFlagPolls = 1u << 22;  // default bound of the in-launch reductions' waits (seconds)

// A partial sum and the parity of its launch in one word (the reductions done by the workgroups of the launch that
// wrote the sums): floating point gives up its last mantissa bit, integers move up by one bit.
__device__ __forceinline__ unsigned tag_partial(float v, unsigned parity) { return (__float_as_uint(v) & ~1u) | parity; }
__device__ __forceinline__ unsigned tag_partial(int v, unsigned parity) { return ((unsigned)v << 1) | parity; }
__device__ __forceinline__ void untag_partial(float& d, unsigned u) { d = __uint_as_float(u & ~1u); }
__device__ __forceinline__ void untag_partial(int& d, unsigned u) { d = (int)u >> 1; }

// Which lane's rows the partial sums of slot group l (= slot / sums per lane) of a panel belong to.  The
// single-column kernels store lane by lane (owner = l).  The batched kernels get their sums from the matrix cores
// transposed within quads of lanes -- register i of lane (quad, j) belongs to the rows of lane 4 quad + i -- and
// store them quad-major, slot group 16 i + quad: the 16 quads of one store instruction then write one contiguous
// run per batch column instead of 16-byte pieces 64 bytes apart.
__device__ __forceinline__ int slot_owner(int l, int quad_major) { return quad_major ? 4 * (l & 15) + (l >> 4) : l; }

template <int N, int AUX>
__device__ __forceinline__ void store_partials(__amdgpu_buffer_rsrc_t rsrc, uint32_t off, const unsigned (&v)[N])
{
    if constexpr (N % 4 == 0) {
#pragma unroll
        for (int i = 0; i < N; i += 4) {
            v4u q = {v[i], v[i + 1], v[i + 2], v[i + 3]};
            __builtin_amdgcn_raw_buffer_store_b128(q, rsrc, (int)(off + 4 * i), 0, AUX);
        }
    } else if constexpr (N % 2 == 0) {
#pragma unroll
        for (int i = 0; i < N; i += 2) {
            v2u q = {v[i], v[i + 1]};
            __builtin_amdgcn_raw_buffer_store_b64(q, rsrc, (int)(off + 4 * i), 0, AUX);
        }
    } else {
#pragma unroll
        for (int i = 0; i < N; ++i) __builtin_amdgcn_raw_buffer_store_b32(v[i], rsrc, (int)(off + 4 * i), 0, AUX);
    }
}

template <int N, int AUX>
__device__ __forceinline__ void load_partials(__amdgpu_buffer_rsrc_t rsrc, uint32_t off, unsigned (&v)[N])
{
    if constexpr (N % 4 == 0) {
#pragma unroll
        for (int i = 0; i < N; i += 4) {
            v4u q = __builtin_amdgcn_raw_buffer_load_b128(rsrc, (int)(off + 4 * i), 0, AUX);
            v[i] = q.x; v[i + 1] = q.y; v[i + 2] = q.z; v[i + 3] = q.w;
        }
    } else if constexpr (N % 2 == 0) {
#pragma unroll
        for (int i = 0; i < N; i += 2) {
            v2u q = __builtin_amdgcn_raw_buffer_load_b64(rsrc, (int)(off + 4 * i), 0, AUX);
            v[i] = q.x; v[i + 1] = q.y;
        }
    } else {
#pragma unroll
        for (int i = 0; i < N; ++i) v[i] = __builtin_amdgcn_raw_buffer_load_b32(rsrc, (int)(off + 4 * i), 0, AUX);
    }
}

// Row of a panel that lane (q, j) keeps in accumulator slot s.  Chosen so that
// after the cross-lane fold lane l holds the rows 64*i + l of the panel.
template <int NQ, int LB>
__host__ __device__ __forceinline__ int panel_row(int q, int j, int s)
{
    constexpr int nfinal = LB / NQ;
    const int qr = q / NQ;
    return (s % nfinal) * 64 + (qr * NQ + s / nfinal) * 16 + j;
}

}  // namespace msgemm
