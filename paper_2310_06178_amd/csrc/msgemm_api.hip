// The C ABI of libmsgemm.so: argument checking, plan ownership, dispatch.
// See include/msgemm.h for the contract of every entry point.
#include <math.h>
#include <new>

#include "msgemm_internal.h"
#include "fused_common.h"

namespace msgemm {

static thread_local int g_last_hip_error = 0;
void set_hip_error(hipError_t e) { g_last_hip_error = (int)e; }

namespace {

bool dtype_pair_ok(int x, int y)
{
    return (x == MSGEMM_F32 && y == MSGEMM_F32) || (x == MSGEMM_F16 && y == MSGEMM_F16) ||
           (x == MSGEMM_BF16 && y == MSGEMM_BF16) || (x == MSGEMM_I8 && y == MSGEMM_I32);
}

void free_plan(Plan* p)
{
    if (!p) return;
    if (p->codes) (void)hipFree(p->codes);
    if (p->scales) (void)hipFree(p->scales);
    if (p->lut_ws) (void)hipFree(p->lut_ws);
    if (p->values256) (void)hipFree(p->values256);
    if (p->codes_words) (void)hipFree(p->codes_words);
    if (p->global_partials) (void)hipFree(p->global_partials);
    if (p->codes_tiled) (void)hipFree(p->codes_tiled);
    if (p->scales_ordered) (void)hipFree(p->scales_ordered);
    if (p->partials) (void)hipFree(p->partials);
    if (p->flags) (void)hipFree(p->flags);
    if (p->epochs) (void)hipFree(p->epochs);
    delete p;
}

size_t lut_bytes_of(const Plan& p)
{
    const size_t entries = (size_t)1 << (4 * p.d);
    if (p.half_table) return (size_t)p.lut_groups * (entries / 2 + 1) * (size_t)p.b * 4u;  // half tables, then the group sums
    return (size_t)p.lut_groups * entries * (size_t)p.b * 4u;
}

}  // namespace
}  // namespace msgemm

using msgemm::Plan;

// The entry points that read the weights row by row (the phase-2-alone consumer on a fused plan, the dense
// comparison kernel) need the row-major codes, which a fused plan does not keep: made here, once, from the
// streaming order.  Allocates on first use; not safe against two first uses of one plan at the same time.
static int ensure_row_major(const Plan& cp, hipStream_t s)
{
    if (cp.codes) return MSGEMM_OK;
    Plan& p = const_cast<Plan&>(cp);
    const size_t code_bytes = (size_t)p.m * (size_t)(p.k / 2);
    uint8_t* buf = nullptr;
    hipError_t e = hipMalloc((void**)&buf, code_bytes);
    if (e != hipSuccess) { msgemm::set_hip_error(e); return MSGEMM_ERR_ALLOC; }
    const int rc = p.d3 ? msgemm::launch_repack3(p, buf, true, s) : msgemm::launch_unpack(p, buf, s);
    if (rc != MSGEMM_OK) { (void)hipFree(buf); return rc; }
    p.codes = buf;
    p.workspace_bytes += code_bytes;
    return MSGEMM_OK;
}

// values256 != nullptr: 8-bit weights.  k and scale_group then count two per code
// byte (the kernels see a code byte as the pair of 4-bit codes it would be for
// int4 weights; only the table build knows better), d is 2, the variant FUSED_LDS.
static int plan_impl(msgemm_plan_t** out, int64_t m, int64_t k, int64_t b, int x_dtype, int y_dtype, int d,
                     int scale_group, const void* W_codes, const void* scales, int variant, void* stream,
                     const float* values256, const msgemm_plan_options_t* options)
{
    if (!out) return MSGEMM_ERR_INVALID_ARG;
    *out = nullptr;
    if (options && options->struct_size != sizeof(msgemm_plan_options_t)) return MSGEMM_ERR_INVALID_ARG;
    if (m <= 0 || k <= 0 || b <= 0 || (k & 1) || !W_codes) return MSGEMM_ERR_INVALID_ARG;
    if (m > ((int64_t)1 << 31) || k > ((int64_t)1 << 31) || b > 65536) return MSGEMM_ERR_INVALID_ARG;
    if (d < 0 || d > 4) return MSGEMM_ERR_INVALID_ARG;  // Section 5: d cannot usefully exceed 4
    if (!msgemm::dtype_pair_ok(x_dtype, y_dtype)) return MSGEMM_ERR_INVALID_ARG;
    if (variant < MSGEMM_VARIANT_AUTO || variant > MSGEMM_VARIANT_GLOBAL_LUT_HALF) return MSGEMM_ERR_INVALID_ARG;
    const bool half_table = variant == MSGEMM_VARIANT_GLOBAL_LUT_HALF;
    if (half_table) variant = MSGEMM_VARIANT_GLOBAL_LUT;
    if (scale_group < 0) return MSGEMM_ERR_INVALID_ARG;
    if (scale_group > 0) {
        if (!scales || x_dtype == MSGEMM_I8) return MSGEMM_ERR_INVALID_ARG;
        if (k % scale_group) return MSGEMM_ERR_INVALID_ARG;
    } else if (scales) {
        return MSGEMM_ERR_INVALID_ARG;
    }
    const int d_eff = d == 0 ? 2 : d;
    // Section 3.3: a scale must be shared by at least d row elements.
    if (scale_group > 0 && scale_group < d_eff) return MSGEMM_ERR_INVALID_ARG;

    Plan* p = new (std::nothrow) Plan();
    if (!p) return MSGEMM_ERR_ALLOC;
    p->m = m; p->k = k; p->b = b;
    if (options) p->opt = *options;  // (a new Plan is zero-filled: no requests)
    p->x_dtype = x_dtype; p->y_dtype = y_dtype;
    p->lut_dtype = (x_dtype == MSGEMM_I8) ? MSGEMM_I32 : MSGEMM_F32;
    p->d = d_eff;
    p->scale_group = scale_group;
    p->block = scale_group > 0 ? scale_group : k;
    p->nblocks = k / p->block;
    p->gpb = (p->block + p->d - 1) / p->d;
    p->lut_groups = p->nblocks * p->gpb;
    p->half_table = half_table;
    p->half_c = -1.0f;  // two's complement: b(~i) = -1 - b(i)
    p->codes8 = values256 != nullptr;

    hipStream_t s = (hipStream_t)stream;
    int rc = MSGEMM_OK;
    auto fail = [&](int code) { msgemm::free_plan(p); return code; };
    auto hip_fail = [&](hipError_t e) { msgemm::set_hip_error(e); return fail(MSGEMM_ERR_HIP); };

    hipError_t e = hipGetDevice(&p->device);
    if (e != hipSuccess) return hip_fail(e);

    // variant
    p->variant = MSGEMM_VARIANT_GLOBAL_LUT;
    if (variant != MSGEMM_VARIANT_GLOBAL_LUT) {
        rc = msgemm::fused_choose_shape(*p, variant);
        if (rc == MSGEMM_OK) {
            p->variant = p->fs.entry_bytes == 2 ? MSGEMM_VARIANT_FUSED_LDS16 : MSGEMM_VARIANT_FUSED_LDS;
        } else if (variant != MSGEMM_VARIANT_AUTO || rc != MSGEMM_ERR_UNSUPPORTED) {
            return fail(rc);
        }
    }

    if (p->codes8) {
        // the kernels that have a table build for it: one column with 16 rows per lane,
        // four fp32 columns, eight fp16 columns with 8 rows per lane
        const bool ok = (p->variant == MSGEMM_VARIANT_FUSED_LDS && p->fs.cols == 1 && p->fs.lane_bytes == 16) ||
                        (p->variant == MSGEMM_VARIANT_FUSED_LDS && p->fs.cols == 4) ||
                        (p->variant == MSGEMM_VARIANT_FUSED_LDS16 && (p->fs.lane_bytes == 8 || p->fs.groups == 16));
        if (!ok) return fail(MSGEMM_ERR_UNSUPPORTED);
        e = hipMalloc((void**)&p->values256, 256 * sizeof(float));
        if (e != hipSuccess) { msgemm::set_hip_error(e); return fail(MSGEMM_ERR_ALLOC); }
        e = hipMemcpy(p->values256, values256, 256 * sizeof(float), hipMemcpyHostToDevice);
        if (e != hipSuccess) return hip_fail(e);
        p->values256_max = 0.0f;
        for (int i = 0; i < 256; ++i) p->values256_max = fmaxf(p->values256_max, fabsf(values256[i]));
        // 16-bit tables hold values256[code] * x in fp16: the values themselves must be inside its range
        if (p->variant == MSGEMM_VARIANT_FUSED_LDS16 && p->values256_max > 65504.0f) return fail(MSGEMM_ERR_UNSUPPORTED);
    }

    // the value of each 4-bit pattern: b(.) of Section 3.1 until the caller installs another map
    for (int i = 0; i < 16; ++i) p->values[i] = (float)(((i ^ 8) & 15) - 8);
    p->custom_values = false;

    // the plan's own copies of the weights: row-major for the two-launch variant; the fused variants keep the
    // codes in their streaming order only (made straight from W_codes below)
    const size_t code_bytes = (size_t)m * (size_t)(k / 2);
    if (p->variant == MSGEMM_VARIANT_GLOBAL_LUT) {
        e = hipMalloc((void**)&p->codes, code_bytes);
        if (e != hipSuccess) { msgemm::set_hip_error(e); return fail(MSGEMM_ERR_ALLOC); }
        e = hipMemcpyAsync(p->codes, W_codes, code_bytes, hipMemcpyDeviceToDevice, s);
        if (e != hipSuccess) return hip_fail(e);
    }
    if (scale_group > 0) {
        const size_t sb = (size_t)m * (size_t)p->nblocks * 2u;
        e = hipMalloc((void**)&p->scales, sb);
        if (e != hipSuccess) { msgemm::set_hip_error(e); return fail(MSGEMM_ERR_ALLOC); }
        e = hipMemcpyAsync(p->scales, scales, sb, hipMemcpyDeviceToDevice, s);
        if (e != hipSuccess) return hip_fail(e);
    }

    p->build_mfma = p->opt.build_on_matrix_cores == 1 ? 0 : p->opt.build_on_matrix_cores == 2 ? 1 : (p->b >= 16 ? 1 : 0);
    if (p->variant == MSGEMM_VARIANT_GLOBAL_LUT) {
        p->lut_ws_bytes = msgemm::lut_bytes_of(*p);
        e = hipMalloc((void**)&p->lut_ws, p->lut_ws_bytes);
        if (e != hipSuccess) { msgemm::set_hip_error(e); return fail(MSGEMM_ERR_ALLOC); }
        p->workspace_bytes = p->lut_ws_bytes;
        rc = msgemm::global_plan_setup(*p, s);
        if (rc != MSGEMM_OK) return fail(rc);
    } else if (p->d3) {
        // depth-3 tables in LDS: the rotated code runs and one partial sum per (segment, column, row)
        const size_t tiled = (size_t)p->ktiles * (size_t)(p->fs.groups / 8) * (size_t)p->m_pad * 12u;
        const size_t part = (size_t)p->segments * (size_t)p->b * (size_t)p->m_pad * 4u;
        e = hipMalloc((void**)&p->codes_tiled, tiled);
        if (e != hipSuccess) { msgemm::set_hip_error(e); return fail(MSGEMM_ERR_ALLOC); }
        e = hipMalloc((void**)&p->partials, part);
        if (e != hipSuccess) { msgemm::set_hip_error(e); return fail(MSGEMM_ERR_ALLOC); }
        p->partial_bytes = part;
        p->workspace_bytes = tiled + part;
        rc = msgemm::launch_repack3(*p, (uint8_t*)W_codes, false, s);  // (read only in this direction)
        if (rc != MSGEMM_OK) return fail(rc);
    } else {
        const size_t tiled = (size_t)p->ktiles * (size_t)p->m_pad * (size_t)(p->fs.groups);
        const size_t b_pad = (size_t)p->col_passes * (size_t)p->fs.cols;
        const size_t slices = p->segments > 0 ? (size_t)p->segments : (size_t)p->ktiles;
        const size_t part = slices * b_pad * (size_t)p->m_pad * 4u;
        // arrival flags per (panel, column pass, slice) for trailing reducers; one more word for give-ups
        const size_t words = (size_t)(p->m_pad / p->fs.panel_rows) * (size_t)p->col_passes * (size_t)p->ktiles;
        p->flag_words = words;
        const size_t cnt = (words + 1) * sizeof(unsigned);
        e = hipMalloc((void**)&p->codes_tiled, tiled);
        if (e != hipSuccess) { msgemm::set_hip_error(e); return fail(MSGEMM_ERR_ALLOC); }
        e = hipMalloc((void**)&p->partials, part);
        if (e != hipSuccess) { msgemm::set_hip_error(e); return fail(MSGEMM_ERR_ALLOC); }
        e = hipMalloc((void**)&p->flags, cnt);
        if (e != hipSuccess) { msgemm::set_hip_error(e); return fail(MSGEMM_ERR_ALLOC); }
        e = hipMemsetAsync(p->flags, 0, cnt, s);
        if (e != hipSuccess) return hip_fail(e);
        p->error_word = p->flags + words;
        p->partial_bytes = part;
        p->workspace_bytes = tiled + part + cnt;
        const bool batched = p->fs.entry_bytes == 2 && p->segments > 1;
        const bool long_form = p->wide_tables == 0 && p->segments > 0 && p->fs.cols == 1 && p->fs.lane_bytes == 16 &&
                               p->fs.entry_bytes == 4;
        if (p->wide_tables > 0 || batched || long_form) {
            // reductions by the workgroups of the launch itself: every partial sum carries the parity of its launch,
            // counted per workgroup; both start at zero
            if (batched) {
                p->epoch_words = (size_t)msgemm::kXcds * (size_t)p->col_passes *
                                 (((size_t)p->segments * (size_t)p->row_blocks + msgemm::kXcds - 1) / msgemm::kXcds);
                p->epoch_words += (size_t)p->row_blocks * (size_t)p->col_passes;  // arrival counts (XCD-local reduction)
                p->xcd_round_robin = msgemm::xcd_round_robin(p->device, s) ? 1 : 0;
            }
            else {
                // one word per workgroup id of the grid, in either order of the ids (row groups or units dealt over the XCDs)
                const size_t by_row_groups = (size_t)slices * msgemm::kXcds * (((size_t)p->row_blocks * p->col_passes + msgemm::kXcds - 1) / msgemm::kXcds);
                const size_t by_units = (size_t)msgemm::kXcds * (size_t)p->col_passes * (((size_t)slices * (size_t)p->row_blocks + msgemm::kXcds - 1) / msgemm::kXcds);
                p->epoch_words = by_row_groups > by_units ? by_row_groups : by_units;
            }
            e = hipMalloc((void**)&p->epochs, p->epoch_words * sizeof(unsigned));
            if (e != hipSuccess) { msgemm::set_hip_error(e); return fail(MSGEMM_ERR_ALLOC); }
            e = hipMemsetAsync(p->epochs, 0, p->epoch_words * sizeof(unsigned), s);
            if (e != hipSuccess) return hip_fail(e);
            e = hipMemsetAsync(p->partials, 0, part, s);
            if (e != hipSuccess) return hip_fail(e);
            p->workspace_bytes += p->epoch_words * sizeof(unsigned);
        }
        if (p->scales) {
            // (the batched kernel keeps one scale per look-up slot: twice the rows)
            const size_t so = (size_t)p->nblocks * (size_t)p->m_pad * (p->fs.entry_bytes == 2 ? 4u : 2u);
            e = hipMalloc((void**)&p->scales_ordered, so);
            if (e != hipSuccess) { msgemm::set_hip_error(e); return fail(MSGEMM_ERR_ALLOC); }
            p->workspace_bytes += so;
        }
        rc = msgemm::launch_repack(*p, W_codes, s);
        if (rc != MSGEMM_OK) return fail(rc);
    }
    *out = reinterpret_cast<msgemm_plan_t*>(p);
    return MSGEMM_OK;
}

extern "C" {

int msgemm_plan(msgemm_plan_t** out, int64_t m, int64_t k, int64_t b, int x_dtype, int y_dtype, int d,
                int scale_group, const void* W_codes, const void* scales, int variant, void* stream)
{
    return plan_impl(out, m, k, b, x_dtype, y_dtype, d, scale_group, W_codes, scales, variant, stream, nullptr, nullptr);
}

int msgemm_plan_with_options(msgemm_plan_t** out, int64_t m, int64_t k, int64_t b, int x_dtype, int y_dtype, int d,
                             int scale_group, const void* W_codes, const void* scales, int variant,
                             const msgemm_plan_options_t* options, void* stream)
{
    return plan_impl(out, m, k, b, x_dtype, y_dtype, d, scale_group, W_codes, scales, variant, stream, nullptr, options);
}

int msgemm_plan_codes8(msgemm_plan_t** out, int64_t m, int64_t k, int64_t b, int x_dtype, int y_dtype,
                       int scale_group, const void* W_codes8, const void* scales, const float* values256,
                       const msgemm_plan_options_t* options, void* stream)
{
    if (!out) return MSGEMM_ERR_INVALID_ARG;
    *out = nullptr;
    if (!values256 || k <= 0 || k > ((int64_t)1 << 30) || scale_group < 0 || scale_group > (1 << 30))
        return MSGEMM_ERR_INVALID_ARG;
    if (x_dtype == MSGEMM_I8) return MSGEMM_ERR_UNSUPPORTED;  // the value map is floating point
    for (int i = 0; i < 256; ++i)
        if (!(values256[i] == values256[i]) || values256[i] > 3.0e38f || values256[i] < -3.0e38f)
            return MSGEMM_ERR_INVALID_ARG;  // NaN / infinity: give such patterns a finite value (they must not occur)
    // full-width tables for one or two columns and for fp32 activations, 16-bit tables for wider batches
    const int variant = (b <= 2 || x_dtype == MSGEMM_F32) ? MSGEMM_VARIANT_FUSED_LDS : MSGEMM_VARIANT_FUSED_LDS16;
    return plan_impl(out, m, 2 * k, b, x_dtype, y_dtype, 2, 2 * scale_group, W_codes8, scales, variant, stream,
                     values256, options);
}

int msgemm_plan_set_codebook(msgemm_plan_t* plan, const float* values16)
{
    if (!plan) return MSGEMM_ERR_INVALID_ARG;
    Plan& p = *reinterpret_cast<Plan*>(plan);
    if (p.codes8) return MSGEMM_ERR_UNSUPPORTED;  // its value map is given when the plan is made
    if (p.d3 && values16) return MSGEMM_ERR_UNSUPPORTED;  // the depth-3 LDS kernel builds its tables from b(.) only
    float v[16];
    for (int i = 0; i < 16; ++i) v[i] = values16 ? values16[i] : (float)(((i ^ 8) & 15) - 8);
    for (int i = 0; i < 16; ++i)
        if (!(v[i] == v[i]) || v[i] > 3.0e38f || v[i] < -3.0e38f) return MSGEMM_ERR_INVALID_ARG;  // NaN / infinity
    // integer tables are built from b(.) itself: the int8 path keeps the paper's encoding
    if (values16 && p.x_dtype == MSGEMM_I8) return MSGEMM_ERR_UNSUPPORTED;
    if (p.half_table) {
        // half tables need value(~i) + value(i) to be one constant
        const float c = v[0] + v[15];
        for (int i = 1; i < 8; ++i)
            if (v[i] + v[15 - i] != c) return MSGEMM_ERR_UNSUPPORTED;
        p.half_c = c;
    }
    // 16-bit tables keep the values in fp16 (rounded to nearest): outside its range they cannot be held at all
    if (p.variant == MSGEMM_VARIANT_FUSED_LDS16)
        for (int i = 0; i < 16; ++i)
            if (v[i] > 65504.0f || v[i] < -65504.0f) return MSGEMM_ERR_UNSUPPORTED;
    for (int i = 0; i < 16; ++i) p.values[i] = v[i];  // travels in the arguments of every later launch
    p.custom_values = values16 != nullptr;
    return MSGEMM_OK;
}

int msgemm_plan_get_info(const msgemm_plan_t* plan, msgemm_plan_info_t* info)
{
    if (!plan || !info) return MSGEMM_ERR_INVALID_ARG;
    const Plan& p = *reinterpret_cast<const Plan*>(plan);
    info->m = p.m; info->k = p.codes8 ? p.k / 2 : p.k; info->b = p.b;
    info->x_dtype = p.x_dtype; info->y_dtype = p.y_dtype; info->lut_dtype = p.lut_dtype;
    info->d = p.codes8 ? 1 : p.d; info->scale_group = p.codes8 ? p.scale_group / 2 : p.scale_group; info->variant = p.half_table ? (int)MSGEMM_VARIANT_GLOBAL_LUT_HALF : p.variant;
    info->lut_groups = p.codes8 ? p.k / 2 : p.lut_groups;
    const bool fused = p.variant != MSGEMM_VARIANT_GLOBAL_LUT;
    info->tile_rows = fused ? p.fs.tile_rows : 0;
    info->tile_groups = fused ? p.fs.groups : 0;
    info->split_k = fused ? (p.segments > 0 ? p.segments : (int)p.ktiles) : 1;
    info->col_chunk = fused ? p.fs.cols : (int)p.b;
    info->workspace_bytes = (int64_t)p.workspace_bytes;
    return MSGEMM_OK;
}

size_t msgemm_lut_bytes(const msgemm_plan_t* plan)
{
    if (!plan || reinterpret_cast<const Plan*>(plan)->codes8) return 0;
    return msgemm::lut_bytes_of(*reinterpret_cast<const Plan*>(plan));
}

int msgemm_build_lut(const msgemm_plan_t* plan, const void* X, int64_t ldx, void* L_out, void* stream)
{
    if (!plan || !X || !L_out) return MSGEMM_ERR_INVALID_ARG;
    const Plan& p = *reinterpret_cast<const Plan*>(plan);
    if (p.codes8) return MSGEMM_ERR_UNSUPPORTED;
    if (ldx < p.k) return MSGEMM_ERR_INVALID_ARG;
    return msgemm::launch_build_lut(p, X, ldx, L_out, (hipStream_t)stream);
}

int msgemm_consume_lut(const msgemm_plan_t* plan, const void* L, void* Y, int64_t ldy, void* stream)
{
    if (!plan || !L || !Y) return MSGEMM_ERR_INVALID_ARG;
    const Plan& p = *reinterpret_cast<const Plan*>(plan);
    if (p.codes8) return MSGEMM_ERR_UNSUPPORTED;
    if (ldy < p.m) return MSGEMM_ERR_INVALID_ARG;
    const int rc = ensure_row_major(p, (hipStream_t)stream);
    if (rc != MSGEMM_OK) return rc;
    return msgemm::launch_consume_lut(p, L, Y, ldy, (hipStream_t)stream);
}

int msgemm_run(const msgemm_plan_t* plan, const void* X, int64_t ldx, void* Y, int64_t ldy, void* stream)
{
    if (!plan || !X || !Y) return MSGEMM_ERR_INVALID_ARG;
    const Plan& p = *reinterpret_cast<const Plan*>(plan);
    if (ldx < (p.codes8 ? p.k / 2 : p.k) || ldy < p.m) return MSGEMM_ERR_INVALID_ARG;
    hipStream_t s = (hipStream_t)stream;
    if (p.variant != MSGEMM_VARIANT_GLOBAL_LUT) return msgemm::launch_fused(p, X, ldx, Y, ldy, s);
    int rc = msgemm::launch_build_lut(p, X, ldx, p.lut_ws, s);
    if (rc != MSGEMM_OK) return rc;
    return msgemm::launch_consume_lut(p, p.lut_ws, Y, ldy, s);
}

// Scratch memory of msgemm_run_static: one array per device for the life of the process.  In host code the
// array's name is only a handle; its device address is looked up once per device (scratch_on_device).
namespace {
constexpr size_t kScratchBytes = (size_t)16 << 20;
static __device__ __align__(256) unsigned char scratch[kScratchBytes];

constexpr int kMaxDevices = 64;
void* g_scratch_ptr[kMaxDevices];   // device address of `scratch` on each device, once looked up
bool g_scratch_known[kMaxDevices];

// Address of this device's copy of `scratch` (the device must be current); nullptr and the HIP error kept on failure.
void* scratch_on_device(int device)
{
    if (device < 0 || device >= kMaxDevices) return nullptr;
    if (!g_scratch_known[device]) {
        void* ptr = nullptr;
        const hipError_t e = hipGetSymbolAddress((void**)&ptr, HIP_SYMBOL(scratch));
        if (e != hipSuccess || !ptr) {
            msgemm::set_hip_error(e);
            return nullptr;
        }
        g_scratch_ptr[device] = ptr;
        g_scratch_known[device] = true;
    }
    return g_scratch_ptr[device];
}
}  // namespace

int msgemm_run_static(const msgemm_plan_t* plan, const void* X, int64_t ldx, void* Y, int64_t ldy, void* stream)
{
    if (!plan || !X || !Y) return MSGEMM_ERR_INVALID_ARG;
    const Plan& p = *reinterpret_cast<const Plan*>(plan);
    if (ldx < (p.codes8 ? p.k / 2 : p.k) || ldy < p.m) return MSGEMM_ERR_INVALID_ARG;
    if (p.variant == MSGEMM_VARIANT_GLOBAL_LUT) return MSGEMM_ERR_UNSUPPORTED;  // its table alone can be gigabytes
    int device = -1;
    MSGEMM_HIP_TRY(hipGetDevice(&device));
    if (device != p.device) return MSGEMM_ERR_INVALID_ARG;
    // the partial sums over the k-tiles (or k-segments) are the only memory the fused kernels need besides the
    // plan's weights, X and Y when those sums are added by a second launch: no flag, count or table outlives a call
    if (p.partial_bytes > kScratchBytes) return MSGEMM_ERR_UNSUPPORTED;
    void* ptr = scratch_on_device(device);
    if (!ptr) return MSGEMM_ERR_HIP;
    Plan q = p;  // (a plain copy of pointers and numbers: nothing is owned twice, nothing is freed)
    q.partials = (float*)ptr;
    q.forced_reduce = 1;   // second launch: every partial sum is written before it is read, nothing needs clearing
    q.flags = nullptr;
    q.epochs = nullptr;
    q.error_word = nullptr;
    return msgemm::launch_fused(q, X, ldx, Y, ldy, (hipStream_t)stream);
}

int msgemm_plan_check(const msgemm_plan_t* plan, void* stream)
{
    if (!plan) return MSGEMM_ERR_INVALID_ARG;
    const Plan& p = *reinterpret_cast<const Plan*>(plan);
    if (!p.flags) return MSGEMM_OK;  // no in-launch reduction in this plan's variant
    hipStream_t s = (hipStream_t)stream;
    unsigned err = 0;
    MSGEMM_HIP_TRY(hipMemcpyAsync(&err, p.error_word, sizeof(err), hipMemcpyDeviceToHost, s));
    MSGEMM_HIP_TRY(hipStreamSynchronize(s));
    if (!err) return MSGEMM_OK;
    if (!(err & 1u)) {
        // only the range bit: an activation was too large for the 16-bit tables; nothing else is out of order
        MSGEMM_HIP_TRY(hipMemsetAsync(p.error_word, 0, sizeof(unsigned), s));
        MSGEMM_HIP_TRY(hipStreamSynchronize(s));
        return MSGEMM_ERR_RANGE;
    }
    // a reducer gave up: flags may be left up, outputs of that call are not the result.  Clear, so that the plan works again.
    MSGEMM_HIP_TRY(hipMemsetAsync(p.flags, 0, (p.flag_words + 1) * sizeof(unsigned), s));
    if (p.epochs) {  // partial sums of the failed launch may be missing: parities and launch counts start over
        MSGEMM_HIP_TRY(hipMemsetAsync(p.partials, 0, p.partial_bytes, s));
        MSGEMM_HIP_TRY(hipMemsetAsync(p.epochs, 0, p.epoch_words * sizeof(unsigned), s));
    }
    MSGEMM_HIP_TRY(hipStreamSynchronize(s));
    return MSGEMM_ERR_INCOMPLETE;
}

int msgemm_dequant_mfma_run(const msgemm_plan_t* plan, const void* X, int64_t ldx, void* Y, int64_t ldy,
                            void* stream)
{
    if (!plan || !X || !Y) return MSGEMM_ERR_INVALID_ARG;
    const Plan& p = *reinterpret_cast<const Plan*>(plan);
    if (ldx < p.k || ldy < p.m) return MSGEMM_ERR_INVALID_ARG;
    if (p.x_dtype == MSGEMM_I8 || p.custom_values || p.codes8) return MSGEMM_ERR_UNSUPPORTED;  // it dequantises with b(.) only
    const int rc = ensure_row_major(p, (hipStream_t)stream);
    if (rc != MSGEMM_OK) return rc;
    return msgemm::launch_dequant_mfma(p, X, ldx, Y, ldy, (hipStream_t)stream);
}

int msgemm_calib_stream_read(const void* src, size_t bytes, void* sink, void* stream)
{
    if (!src || !sink || ((uintptr_t)src & 15)) return MSGEMM_ERR_INVALID_ARG;
    return msgemm::launch_calib_stream_read(src, bytes, sink, (hipStream_t)stream);
}

int msgemm_calib_stream_read_shape(const void* src, size_t bytes, void* sink, int waves_per_workgroup,
                                   int workgroups_per_cu, int depth, int non_temporal, void* stream)
{
    if (!src || !sink || ((uintptr_t)src & 15)) return MSGEMM_ERR_INVALID_ARG;
    return msgemm::launch_calib_stream_read_shape(src, bytes, sink, waves_per_workgroup, workgroups_per_cu, depth,
                                                  non_temporal, (hipStream_t)stream);
}

int msgemm_calib_lookup_add(int tiles, void* sink, size_t* lookups_out, void* stream)
{
    return msgemm::launch_calib_lookup_add(tiles, sink, lookups_out, (hipStream_t)stream);
}

int msgemm_calib_lds_read(int width_bytes, int reads, void* sink, size_t* bytes_out, void* stream)
{
    return msgemm::launch_calib_lds_read(width_bytes, reads, sink, bytes_out, (hipStream_t)stream);
}

void msgemm_destroy(msgemm_plan_t* plan)
{
    if (!plan) return;
    (void)hipDeviceSynchronize();
    msgemm::free_plan(reinterpret_cast<Plan*>(plan));
}

const char* msgemm_status_string(int status)
{
    switch (status) {
    case MSGEMM_OK: return "ok";
    case MSGEMM_ERR_INVALID_ARG: return "invalid argument";
    case MSGEMM_ERR_ALLOC: return "allocation failed";
    case MSGEMM_ERR_HIP: return "HIP runtime error";
    case MSGEMM_ERR_UNSUPPORTED: return "not supported by the requested variant";
    case MSGEMM_ERR_RANGE: return "an activation was too large for 16-bit table entries; the outputs of the calls since the last check may hold infinities (use MSGEMM_VARIANT_FUSED_LDS)";
    case MSGEMM_ERR_INCOMPLETE: return "a reduction inside a launch gave up waiting for partial sums; the outputs of the calls since the last check are not valid";
    default: return "unknown status";
    }
}

int msgemm_last_hip_error(void) { return msgemm::g_last_hip_error; }

const char* msgemm_version(void) { return "0.1"; }

}  // extern "C"
