/*
 * msgemm.h -- C ABI of the msGeMM library for AMD MI355X (gfx950).
 *
 * msGeMM (arxiv 2310.06178) computes the GeMM  M x X = Y  (Section 1, Eq. 1;
 * sizes m x k x b, Section 2) for a 4-bit weight matrix M without multiplying
 * in the inner loop: for every group of d consecutive k-indices and every
 * column of X a table L of all 16^d partial dot products is produced once
 * (phase 1, Section 3.1), and every output row then adds up the table entries
 * addressed by its packed d x 4-bit codes (phase 2, Section 3.2).  Weights
 * that share a scale per block of a row are handled by multiplying the block's
 * partial sum after the table has been consumed (Section 3.3).
 *
 * All pointers named "device" are HIP device pointers on the current device;
 * "stream" is a hipStream_t passed as void* (NULL = the null stream).  Every
 * call only enqueues work on that stream and never synchronises it, except
 * msgemm_plan (which returns after its one-off weight repack has been
 * enqueued; the caller may free W_codes / scales once the stream has been
 * synchronised) and msgemm_destroy (which synchronises the device before it
 * frees).  No exception or abort crosses this boundary: every entry point
 * returns MSGEMM_OK (0) or a negative msgemm_status_t.
 *
 * Storage conventions (the paper fixes none; Section 4 only requires that the
 * d codes of a group are adjacent in a row-major M):
 *   W_codes  uint8 [m][k/2] row-major; byte t of row i holds column 2t in bits
 *            3:0 and column 2t+1 in bits 7:4.  A code is the two's-complement
 *            pattern of its value: b(0000)=0 .. b(0111)=7, b(1000)=-8 ..
 *            b(1111)=-1 (Section 3.1).  k must be even.
 *   scales   fp16 [m][k/scale_group], or NULL when scale_group == 0.
 *   X        column c of the paper's k x b matrix is contiguous:
 *            X(j,c) = X[c*ldx + j], ldx >= k, in x_dtype.
 *   Y        Y(i,c) = Y[c*ldy + i], ldy >= m, in y_dtype.
 *   L        [groups][16^d][b] in the LUT dtype (fp32 for floating-point X,
 *            int32 for int8 X); the entry index of codes (i_0..i_{d-1}) is
 *            sum_r i_r << 4r, so a packed code byte is itself the d = 2 index.
 *            Groups restart at every scale-block boundary; a group cut short
 *            by the end of its block (d does not divide the block length)
 *            ignores the missing positions.
 */
#ifndef MSGEMM_H
#define MSGEMM_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef struct msgemm_plan_s msgemm_plan_t; /* opaque, owned by the library */

typedef enum {
    MSGEMM_F32 = 0,
    MSGEMM_F16 = 1,
    MSGEMM_BF16 = 2,
    MSGEMM_I8 = 3,
    MSGEMM_I32 = 4
} msgemm_dtype_t;

typedef enum {
    MSGEMM_OK = 0,
    MSGEMM_ERR_INVALID_ARG = -1, /* null pointer, bad size, bad d, bad dtype pair */
    MSGEMM_ERR_ALLOC = -2,       /* host or device allocation failed */
    MSGEMM_ERR_HIP = -3,         /* a HIP call failed; see msgemm_last_hip_error */
    MSGEMM_ERR_UNSUPPORTED = -4, /* valid request that the chosen variant cannot serve */
    MSGEMM_ERR_INCOMPLETE = -5,  /* msgemm_plan_check: a reduction inside a launch gave up waiting */
    MSGEMM_ERR_RANGE = -6        /* msgemm_plan_check: an activation too large for 16-bit table entries was seen */
} msgemm_status_t;

/* How phase 1 and phase 2 are scheduled on the GPU. */
typedef enum {
    MSGEMM_VARIANT_AUTO = 0,
    /* Two launches: L is written to device memory once and shared by all rows
     * (the arrangement of Section 4: one L, kept in cache between the phases); any d in 1..4. */
    MSGEMM_VARIANT_GLOBAL_LUT = 1,
    /* One launch, d = 2: each workgroup builds the tables of its k-tiles in LDS
     * (phase 1 and 2 pipelined over the last dimension of L, Section 4), streams
     * its repacked code tiles; partial sums over k-tiles are added inside the
     * launch (b <= 2: by the workgroups that produced them, or by trailing
     * workgroups) or by a small second kernel.
     * Table entries are fp32 (int32 for int8 X).  A scale block must be a whole
     * number of k-tiles: scale_group % 128 == 0, or % 64 == 0 for fp32 X with
     * b > 2; otherwise MSGEMM_ERR_UNSUPPORTED, and AUTO takes GLOBAL_LUT.
     * With d = 3 (on request only, never by AUTO; b <= 2, no scales, the paper's
     * encoding): tables of 16 KiB per group, 8 groups = 24 columns per k-tile --
     * the depth the paper's operation count prefers (Section 5), kept as the
     * measured point beside d = 2; option half_tables_in_lds stores half of each
     * table (Section 4.1) and holds 16 groups per k-tile. */
    MSGEMM_VARIANT_FUSED_LDS = 2,
    /* Same schedule with fp16 table entries, 8 batch columns per entry.  For
     * int8 X the entries are integers of magnitude <= 2048, exact in fp16, and
     * the sums are kept exact (result bit-exact); for fp16 / bf16 X each entry
     * is rounded to fp16, which needs 2 max|value(code)| |x| (16 |x| for the
     * paper's int4) inside the fp16 range.  A larger activation is detected by
     * the kernel: the outputs may then hold infinities, and msgemm_plan_check
     * returns MSGEMM_ERR_RANGE; such callers ask for FUSED_LDS.  Value maps
     * (msgemm_plan_set_codebook, msgemm_plan_codes8) with a value beyond +-65504
     * are refused on such a plan; values that fp16 cannot hold exactly are rounded
     * to nearest.  Accumulation is fp32.  scale_group % 32 == 0.  Not available
     * for fp32 X.  AUTO picks it for b > 2 unless the problem is small (columns
     * times code bytes up to 64 MiB, scale blocks of whole k-tiles): then
     * FUSED_LDS runs one pass per column, which is faster there. */
    MSGEMM_VARIANT_FUSED_LDS16 = 3,
    /* GLOBAL_LUT with half of every table (the optimisation sketched in Section
     * 4.1): only the combinations whose last code has its top bit clear are
     * stored.  With a value map that satisfies value(~i) + value(i) = c for all i
     * (two's complement: c = -1; uint4: c = 15) the other half follows from
     *   L(~i_0, .., ~i_{d-1}, j) = c * S(j) - L(i_0, .., i_{d-1}, j),
     * S(j) = the sum of the group's activations.  L_out of msgemm_build_lut is
     * then [group][16^d / 2][b] followed by S as [group][b] (msgemm_lut_bytes
     * covers both).  msgemm_plan_set_codebook refuses a map without that
     * property on such a plan.  Never chosen by AUTO. */
    MSGEMM_VARIANT_GLOBAL_LUT_HALF = 4
} msgemm_variant_t;

typedef struct {
    int64_t m, k, b;
    int x_dtype, y_dtype, lut_dtype;
    int d;
    int scale_group;
    int variant;         /* the variant actually chosen */
    int64_t lut_groups;  /* last dimension of L */
    int tile_rows;       /* rows per workgroup (fused variant), else 0 */
    int tile_groups;     /* table groups of a k-tile (one table in LDS), else 0 */
    int split_k;         /* partial sums reduced per output: k-tiles, or runs of k-tiles (long k, batches; with the
                            k-tiles of a batched plan dealt evenly: the most any output has) */
    int col_chunk;       /* batch columns handled per pass over the codes */
    int64_t workspace_bytes; /* device memory the plan owns besides the codes in its kernels' order */
} msgemm_plan_info_t;

/*
 * Choices the library otherwise makes itself, for tests and measurements that
 * need a particular kernel form on a problem that would not get it.  A
 * zero-filled structure (with struct_size set) asks for nothing.  Fields that
 * do not apply to the plan's variant are ignored; values out of range fall
 * back to the library's choice.  Nothing here changes what is computed.
 */
typedef struct {
    size_t struct_size;          /* sizeof(msgemm_plan_options_t) as the caller was compiled; required */
    int panels_per_workgroup;    /* fused kernels: panels of rows per workgroup (1..64); 0 = library's choice */
    int k_tiles_per_workgroup;   /* single-column kernels: consecutive k-tiles a workgroup runs through
                                    (1 = one k-tile per workgroup, n > 2 = the long-k form); 0 = library's choice */
    int reduce_mode;             /* sums over k-tiles / k-segments: 0 = library's choice, 1 = a second launch,
                                    2 = trailing workgroups of the same launch (single-column kernels), 3 = the
                                    workgroups that produced them (needs the whole grid resident; else 1 is
                                    taken; the batched kernels do it on request only: it measured slower),
                                    4 = batched kernels: the producing workgroups, with all workgroups of a (row
                                    block, column pass) placed on one XCD and the sums handed over through its L2
                                    (needs the whole grid resident, the pairs to divide evenly over the XCDs and a
                                    device seen to deal workgroup ids over its XCDs in turn; else as 0) */
    int rows_per_lane;           /* single-column kernel: 16 (default) or 8 (its 16-wavefront form);
                                    batched kernel: 8 (default) or 4 */
    int no_xcd_map;              /* 1: workgroup ids in k-tile-major order instead of grouped per L2 */
    int batched_form;            /* batched kernel: 0 = library's choice, 1 = build phase per k-tile, 2 = pipelined */
    int batched_segments;        /* batched kernel: k-segments (partial sums per output); 0 = library's choice */
    int global_plain_consumer;   /* two-launch variant: 1 = the one-thread-per-output consumer */
    int global_chunk_kib;        /* two-launch variant: table KiB per chunk; 0 = 1024 */
    int global_segments;         /* two-launch variant: runs of chunks; 0 = library's choice */
    int build_on_matrix_cores;   /* msgemm_build_lut: 0 = from 16 columns on, 1 = never, 2 = always */
    int half_tables_in_lds;      /* FUSED_LDS at d = 3: keep only the half of each table whose last code has its top
                                    bit clear (Section 4.1): 16 instead of 8 groups per k-tile */
    int poll_limit;              /* in-launch reductions: polls before a waiting wavefront gives up; 0 = 2^22 */
    int skip_publish;            /* test aid: producers never announce their partial sums, so every waiting
                                    wavefront gives up after poll_limit polls (see msgemm_plan_check) */
    int batched_deal;            /* batched kernel, pipelined form: the k-tiles of all row blocks dealt evenly over the
                                    workgroups (a workgroup may end one row block and begin the next); 0 = library's
                                    choice, 1 = never, 2 = whenever the problem allows */
} msgemm_plan_options_t;

/*
 * Validate an m x k x b problem (Section 2), choose the kernel variant and
 * tile shape, and make the plan's own device copies of the weights: the scales
 * and the codes -- row-major for the two-launch variants, reordered into the
 * order the kernels stream them for the fused ones (which keep no row-major
 * copy: see msgemm_consume_lut).  M is a static model weight (Section 1), so
 * this is one-off work outside the hot path.
 *
 *   d            1..4 (Section 5: larger d is never useful), or 0 = library's choice
 *   scale_group  0 = no scales; else the number r of consecutive row elements
 *                sharing a scale; needs r >= d and k % r == 0 (Section 3.3)
 *   W_codes      device, m*k/2 bytes, read during this call's stream work
 *   scales       device, fp16 [m][k/scale_group], or NULL
 *   variant      a msgemm_variant_t
 * Supported (x_dtype, y_dtype): (F32,F32) (F16,F16) (BF16,BF16) (I8,I32);
 * the int8 pair takes no scales.  On failure *out is NULL.
 */
int msgemm_plan(msgemm_plan_t** out, int64_t m, int64_t k, int64_t b,
                int x_dtype, int y_dtype, int d, int scale_group,
                const void* W_codes, const void* scales, int variant, void* stream);

/* The same with options (NULL = none).  MSGEMM_ERR_INVALID_ARG if options->struct_size is not the size this
 * library was built with. */
int msgemm_plan_with_options(msgemm_plan_t** out, int64_t m, int64_t k, int64_t b,
                             int x_dtype, int y_dtype, int d, int scale_group,
                             const void* W_codes, const void* scales, int variant,
                             const msgemm_plan_options_t* options, void* stream);

/*
 * The same for weights of 8 bits (Section 2 names an 8-bit floating-point
 * weight matrix as another datatype the method applies to).  One code byte per
 * element: W_codes8 is device, uint8 [m][k], row-major, copied and repacked
 * like the 4-bit codes.  values256 (host, 256 finite floats) gives the value of
 * each bit pattern -- e.g. the E4M3 or E5M2 values, or a 256-entry codebook;
 * patterns that stand for NaN or infinity in such a format need a finite
 * stand-in and must not occur in W_codes8.  The table of a k-index then holds
 * values256[code] * x(j) for the 256 codes (the paper's look-up table with one
 * element per group and 256 instead of 16 patterns per element), and an output
 * is the sum of one entry per element (Section 3.2).  scale_group (0, or a
 * multiple of 64 that divides k; 32 for fp16 / bf16 activations with b > 2)
 * and scales as in msgemm_plan.  Runs with the tables in LDS, full-width
 * entries for b <= 2 and for fp32 activations, fp16 entries (values256[code] *
 * x rounded to fp16) for wider fp16 / bf16 batches; floating-point activations
 * only (MSGEMM_ERR_UNSUPPORTED for int8).  The plan works with msgemm_run,
 * msgemm_plan_get_info (d reads 1, lut_groups k) and msgemm_destroy; the
 * other entry points refuse it.  options: as for msgemm_plan_with_options, NULL = none.
 */
int msgemm_plan_codes8(msgemm_plan_t** out, int64_t m, int64_t k, int64_t b,
                       int x_dtype, int y_dtype, int scale_group,
                       const void* W_codes8, const void* scales,
                       const float* values256, const msgemm_plan_options_t* options, void* stream);

/*
 * Other encodings of the 4-bit codes.  Section 2 notes that the exact datatype
 * of the weights is irrelevant to the method; b(.) of Section 3.1 is the only
 * place where the encoding enters.  values16 (host, 16 floats, finite) gives the
 * value of each bit pattern 0000..1111 -- e.g. 0..15 for unsigned int4, or a
 * non-uniform 16-entry codebook -- and replaces b(.) in every table this plan
 * builds from now on (msgemm_build_lut, msgemm_run).  NULL restores the
 * paper's two's complement.  Floating-point plans only (MSGEMM_ERR_UNSUPPORTED
 * for int8 activations, whose integer tables keep b(.)); with 16-bit table
 * entries the values are rounded to fp16.  The comparison entry point
 * msgemm_dequant_mfma_run refuses a plan with a custom map.  The map travels
 * in the arguments of each launch: launches already enqueued keep the old one.
 */
int msgemm_plan_set_codebook(msgemm_plan_t* plan, const float* values16);

/* Fill *info with what the plan chose. */
int msgemm_plan_get_info(const msgemm_plan_t* plan, msgemm_plan_info_t* info);

/* Bytes the caller must provide for L_out: lut_groups * 16^d * b * 4. */
size_t msgemm_lut_bytes(const msgemm_plan_t* plan);

/*
 * Phase 1 alone (Section 3.1): L(i_0..i_{d-1}, j, c) = sum_r b(i_r) X(j d + r, c)
 * for every code combination, group j and column c, written to L_out (device,
 * msgemm_lut_bytes bytes, layout above).  X: device, ldx >= k.
 */
int msgemm_build_lut(const msgemm_plan_t* plan, const void* X, int64_t ldx,
                     void* L_out, void* stream);

/*
 * Phase 2 alone (Section 3.2, second line of the y(i) equation, and Section
 * 3.3): Y(i,c) = sum_blocks q(i,block) * sum_{groups j of the block}
 * L(codes of row i at group j, j, c).  L: device, as written by
 * msgemm_build_lut for the same plan.  Y: device, ldy >= m.
 * This kernel reads the codes row by row.  A fused plan keeps them in its
 * streaming order only: the first call on such a plan allocates m*k/2 bytes
 * (MSGEMM_ERR_ALLOC if that fails) and fills them on `stream`; it must not run
 * at the same time as another first call on that plan.
 */
int msgemm_consume_lut(const msgemm_plan_t* plan, const void* L,
                       void* Y, int64_t ldy, void* stream);

/*
 * The whole hot path, Y = M x X, by the plan's variant (both phases).
 * X, Y: device.  Uses the plan's workspace: calls on the same plan must not
 * overlap (use one stream, or one plan per stream).
 */
int msgemm_run(const msgemm_plan_t* plan, const void* X, int64_t ldx,
               void* Y, int64_t ldy, void* stream);

/*
 * msgemm_run for callers that cannot allocate or hold a workspace: code under
 * HIP graph capture, serving loops and harnesses that forbid hipMalloc.  The
 * same Y by the same kernels, but the partial sums over the k-tiles live in a
 * static array in the library's device image (16 MiB on every device the
 * library runs on, held until the process ends) instead of the plan's
 * workspace, and are added by a second launch; the call allocates and frees
 * nothing.  Plans of the fused variants only (MSGEMM_ERR_UNSUPPORTED for
 * GLOBAL_LUT / GLOBAL_LUT_HALF) whose partial sums fit the array
 * (split_k * b * m rounded up to whole panels * 4 bytes <= 16 MiB, else
 * MSGEMM_ERR_UNSUPPORTED); the plan's device must be current
 * (MSGEMM_ERR_INVALID_ARG).  All calls on one device share the array: calls
 * that overlap on a device -- different streams, different plans -- race.
 * Nothing in the array needs a particular value when a call starts.
 */
int msgemm_run_static(const msgemm_plan_t* plan, const void* X, int64_t ldx,
                      void* Y, int64_t ldy, void* stream);

/*
 * The single-column kernels add the partial sums of the k-tiles (the sum over
 * j in Section 3.2, cut into pieces that different workgroups hold) inside the
 * launch: wavefronts wait, for a bounded number of polls, until the partial
 * sums they need have been announced.  A wavefront whose wait runs out cannot
 * make msgemm_run fail (the call has long returned): it sets a sticky word in
 * the plan's device memory, writes no valid output and leaves its flags up.
 * This call waits for `stream`, reads that word and returns MSGEMM_OK if no
 * wavefront has given up since the last check; otherwise it clears the word and
 * the flags, so that the plan works again, and returns MSGEMM_ERR_INCOMPLETE:
 * the outputs of the msgemm_run calls on this plan since the last check are not
 * valid.  With the default poll bound (about a second of polling) a give-up
 * means that the producing workgroups never ran -- which can also happen
 * when kernels of other streams occupy the device so that the workgroups of
 * one launch are not all resident together (the library checks that the grid
 * fits an otherwise idle device, not what else runs); a plan made with option
 * reduce_mode = 1 adds its partial sums in a second launch and waits for
 * nothing inside a launch.  The same word records that
 * a kernel with 16-bit table entries met an activation too large for them
 * (see MSGEMM_VARIANT_FUSED_LDS16): then, and if no reduction gave up, the word
 * is cleared and MSGEMM_ERR_RANGE is returned.  Synchronises the stream.
 */
int msgemm_plan_check(const msgemm_plan_t* plan, void* stream);

/* Synchronise the device, free everything the plan owns.  NULL is allowed. */
void msgemm_destroy(msgemm_plan_t* plan);

/* Static text for a status code. */
const char* msgemm_status_string(int status);

/* hipError_t (as int) of the most recent failing HIP call on this thread, 0 if none. */
int msgemm_last_hip_error(void);

/* Library version, "major.minor". */
const char* msgemm_version(void);

#ifdef __cplusplus
}
#endif
#endif /* MSGEMM_H */
