// Internal declarations shared by the translation units of libmsgemm.so.
// Nothing here is part of the public ABI (see include/msgemm.h and include/msgemm_measure.h).
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

#include "msgemm.h"
#include "msgemm_measure.h"

namespace msgemm {

// How the 64 lanes of a wavefront share one streamed panel of codes in the
// fused kernel.  A k-tile holds `groups` tables (d = 2: one per pair of
// k-indices); a panel is `panel_rows` rows by `groups` groups and is read as
// 16 loads of 64 lanes x `lane_bytes` bytes.
struct FusedShape {
    int groups;       // tables resident in LDS per workgroup: 16, 32 or 64
    int lane_bytes;   // bytes (= rows) a lane takes per load: 4, 8 or 16
    int cols;         // batch columns per table entry (one pass over the codes)
    int entry_bytes;  // bytes per table value: 4 (fp32/int32) or 2 (fp16/int16)
    int waves;        // wavefronts per workgroup
    int panels;       // panels per workgroup
    int panel_rows;   // 64 * 16 / groups * lane_bytes
    int tile_rows;    // panels * panel_rows
    size_t lds_bytes; // 256 * groups * cols * entry_bytes
};

struct Plan {
    int64_t m, k, b;
    int x_dtype, y_dtype, lut_dtype;
    int d, scale_group, variant;
    int64_t block;        // columns per scale block (k when there are no scales)
    int64_t nblocks;      // k / block
    int64_t gpb;          // LUT groups per block = ceil(block / d)
    int64_t lut_groups;   // nblocks * gpb
    int device;

    float values[16];     // value of each 4-bit pattern (b(.) of Section 3.1 by default)
    bool custom_values;   // another encoding has been installed with msgemm_plan_set_codebook
    bool codes8;          // 8-bit weights: k counts two per code byte internally, a table group is one real column
    float* values256;     // device, 256 floats: the value of each 8-bit pattern (codes8 plans), else nullptr
    float values256_max;  // largest magnitude among them
    uint8_t* codes;       // device, [m][k/2] row-major, plan-owned: always for the two-launch variant; for the fused ones
                          // made from the streaming order when an entry point that reads rows is first called
    uint16_t* scales;     // device fp16 [m][nblocks] or nullptr
    float* lut_ws;        // device workspace for the two-launch variant
    size_t lut_ws_bytes;
    bool half_table;         // two-launch variant: only the half of each table with the last code's top bit clear
    float half_c;            // value(~i) + value(i) of the plan's value map (half tables)
    uint32_t* codes_words;   // two-launch variant: codes as [64-row tile][word of the row][lane], or nullptr
    float* global_partials;  // two-launch variant: [segment][b][m] fp32 / int32, or nullptr
    int global_segments;     // two-launch variant: runs of k handled by different workgroups

    // fused variant
    FusedShape fs;
    int64_t ktiles;       // k-tiles (split-k factor)
    int64_t row_blocks;   // workgroups along m
    int64_t m_pad;        // row_blocks * tile_rows
    int col_passes;       // ceil(b / cols)
    int cus;              // compute units of the device
    msgemm_plan_options_t opt;  // the caller's requests (all zero: none), fixed when the plan is made
    int xcd_map_allowed;  // !opt.no_xcd_map
    int forced_reduce;    // opt.reduce_mode: 0 none, 1 second pass, 2 in launch (single-column kernels)
    int global_plain;     // two-launch variant with the plain consumer
    int global_chunk_kib; // two-launch variant: table KiB per chunk (default 1024)
    int build_mfma;       // phase 1 alone on the matrix cores (default: from 16 batch columns on)
    int segments;         // batched kernel: k-segments (partial sums per output); 0 otherwise
    int tiles_per_segment; // batched kernel: k-tiles a workgroup runs through
    int deal_blocks;      // batched kernel, pipelined form with its k-tiles dealt evenly: scale blocks per workgroup (0: equal segments)
    uint16_t* scales_ordered;  // device fp16 [nblocks][m_pad], rows in the order the lanes own outputs; nullptr without scales
    uint8_t* codes_tiled; // device, [ktiles][m_pad / panel_rows][16][64][lane_bytes]
    float* partials;      // device, [ktiles or segments][b_pad][m_pad] fp32 / int32
    unsigned* flags;      // device, [panels][col_passes][slices] arrival flags of the trailing-workgroup reduction, zero
                          // between launches; then the error word
    size_t partial_bytes; // size of `partials`
    unsigned* epochs;     // device, wide form: launch count of every workgroup of the grid (resident reduction), or nullptr
    size_t epoch_words;   // (batched kernels: the last row_blocks * col_passes words are the arrival counts of the XCD-local reduction)
    int xcd_round_robin;  // 1: the device was seen to deal workgroup ids over its XCDs in turn (probed at the first batched plan)
    size_t flag_words;    // flags in that buffer
    unsigned* error_word; // device, flags + flag_words: set by a wavefront that gave up waiting (msgemm_plan_check)
    bool d3;              // depth-3 tables in LDS (kernels_depth3.hip): codes_tiled holds its rotated 96-bit runs
    bool d3_half;         // ... with half tables (Section 4.1)
    int d3_sub;           // ... sub-panels of 64 rows per wavefront
    int wide_tables;      // single-column kernel, wide form: tables a workgroup holds (1 or 2); 0 = another form
    size_t workspace_bytes;
};

void set_hip_error(hipError_t e);

#define MSGEMM_HIP_TRY(expr)                         \
    do {                                             \
        hipError_t e__ = (expr);                     \
        if (e__ != hipSuccess) {                     \
            ::msgemm::set_hip_error(e__);            \
            return MSGEMM_ERR_HIP;                   \
        }                                            \
    } while (0)

// kernels_global_lut.hip
int launch_build_lut(const Plan& p, const void* X, int64_t ldx, void* L, hipStream_t s);
int launch_consume_lut(const Plan& p, const void* L, void* Y, int64_t ldy, hipStream_t s);
int global_plan_setup(Plan& p, hipStream_t s);  // transposed codes and partial sums of the tiled consumer

// kernels_fused.hip
int fused_choose_shape(Plan& p, int requested_variant);  // fills p.fs, ktiles, ...; MSGEMM_ERR_UNSUPPORTED if not applicable
int launch_repack(const Plan& p, const void* W_codes, hipStream_t s);  // scales and codes into the kernels' order
int launch_unpack(const Plan& p, uint8_t* row_major, hipStream_t s);   // the codes back to row-major
int launch_fused(const Plan& p, const void* X, int64_t ldx, void* Y, int64_t ldy, hipStream_t s);
// adds `slices` partial-sum slices ([slice][b_pad][m_pad], output order) and writes Y in the plan's output type
int launch_reduce_second_pass(const Plan& p, const float* partials, void* Y, int64_t ldy, int slices,
                              int64_t span, hipStream_t s);

// kernels_depth3.hip (d = 3, tables in LDS, single column)
int depth3_choose_shape(Plan& p);  // fills row_blocks, m_pad, ktiles, segments, fs; MSGEMM_ERR_UNSUPPORTED if not applicable
int launch_repack3(const Plan& p, uint8_t* row_major, bool inverse, hipStream_t s);
int launch_depth3(const Plan& p, const void* X, int64_t ldx, void* Y, int64_t ldy, hipStream_t s);

// kernels_batched.hip (16-bit table entries, 8 batch columns per pass)
void batched_choose_segments(Plan& p);  // needs ktiles, row_blocks, col_passes, cus; fills segments, tiles_per_segment
// pipelined batched kernel: panels per workgroup and segments together (needs fs, ktiles, col_passes, cus)
void batched_choose_rows_and_segments(Plan& p, int64_t panels, int& ppw_out);
// which form of the batched kernel the time models predict to be faster for a problem
bool batched_pipelined_is_faster(int64_t m, int64_t k, int64_t b, int64_t scale_group, int cus);
// panels of 256 rows per workgroup of the batched form with a build phase (8 rows per lane)
int batched_phase_form_panels(int64_t panels, int64_t ktiles, int64_t scale_group, int col_passes, int64_t cus);
int launch_repack_scales_batched(const Plan& p, hipStream_t s);
bool xcd_round_robin(int device, hipStream_t s);
int launch_batched(const Plan& p, const void* X, int64_t ldx, void* Y, int64_t ldy, hipStream_t s);

// calibration.hip
int launch_calib_stream_read(const void* src, size_t bytes, void* sink, hipStream_t s);
int launch_calib_stream_read_shape(const void* src, size_t bytes, void* sink, int waves_per_workgroup,
                                   int workgroups_per_cu, int depth, int non_temporal, hipStream_t s);
int launch_calib_lds_read(int width_bytes, int reads, void* sink, size_t* bytes_out, hipStream_t s);
int launch_calib_lookup_add(int tiles, void* sink, size_t* lookups_out, hipStream_t s);

// kernels_mfma.hip
int launch_dequant_mfma(const Plan& p, const void* X, int64_t ldx, void* Y, int64_t ldy, hipStream_t s);

}  // namespace msgemm
