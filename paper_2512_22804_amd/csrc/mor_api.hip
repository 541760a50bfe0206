// C ABI of the MoR analyse-select-quantize library: argument validation and dispatch only.
// Every step of the path runs in the kernels of mor_kernels.hip.
#include <mutex>

#include "../../include/mor.h"
#include "mor_launch.h"

// Built-in scratch of mor_analyze_quantize_static.  Every GPU the library runs on holds its own copy of this array at
// its own address until the process ends.  In host code the NAME of the array is only a handle for
// hipGetSymbolAddress: it is never passed to a kernel, a copy or a fill (static_scratch() below returns the device
// address that is).
static __device__ __align__(256) unsigned char scratch[MOR_STATIC_SCRATCH_BYTES];

namespace {

// Device address of `scratch` on the current device, looked up once per device.
constexpr int kMaxDevices = 64;
std::mutex g_scratch_mutex;
void* g_scratch_ptr[kMaxDevices] = {};
mor_status static_scratch(void** out) {
    int dev = -1;
    if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= kMaxDevices) return MOR_ERR_HIP;
    std::lock_guard<std::mutex> lock(g_scratch_mutex);
    if (g_scratch_ptr[dev] == nullptr) {
        void* ptr = nullptr;
        if (hipGetSymbolAddress(&ptr, HIP_SYMBOL(scratch)) != hipSuccess || ptr == nullptr) return MOR_ERR_HIP;
        g_scratch_ptr[dev] = ptr;
    }
    *out = g_scratch_ptr[dev];
    return MOR_OK;
}

bool aligned16(const void* p) { return (reinterpret_cast<uintptr_t>(p) & 15u) == 0; }

// Shape rules shared by every entry point.
mor_status check_shape(int32_t gran, int64_t rows, int64_t cols, bool ragged) {
    if (gran < MOR_GRAN_TENSOR || gran > MOR_GRAN_BLOCK_64x64) return MOR_ERR_UNSUPPORTED;
    if (rows <= 0 || cols <= 0) return MOR_ERR_SHAPE;
    if (cols % 8) return MOR_ERR_SHAPE;                            // 16-byte rows
    const mor::StatsGeom g = mor::make_geom(gran, rows, cols);
    if (!ragged && !g.uniform) return MOR_ERR_SHAPE;
    if (gran == MOR_GRAN_CHANNEL_ROW && cols > 65536) return MOR_ERR_SHAPE;   // a row is held in the registers of one workgroup
    return MOR_OK;
}
mor_status check_common(const mor_params* p) {
    if (!p) return MOR_ERR_NULL;
    if (p->flags & ~(uint32_t)(MOR_FLAG_RAGGED | MOR_FLAG_LEAN_FP8)) return MOR_ERR_UNSUPPORTED;
    return check_shape(p->granularity, p->rows, p->cols, (p->flags & MOR_FLAG_RAGGED) != 0);
}
// Rows per group of Algorithm 1 as the kernels see it: 0 = one group.  `*st` receives the argument error, if any.
int64_t group_rows_of(const mor_params* p, mor_status* st) {
    *st = MOR_OK;
    if (p->scaling != MOR_SCALE_GAM || p->gam_group_rows == 0 || (int64_t)p->gam_group_rows >= p->rows) return 0;
    if (p->granularity == MOR_GRAN_TENSOR || p->granularity == MOR_GRAN_CHANNEL_COL) { *st = MOR_ERR_UNSUPPORTED; return 0; }
    const mor::StatsGeom g = mor::make_geom(p->granularity, p->rows, p->cols);
    if (p->gam_group_rows % g.pr) { *st = MOR_ERR_SHAPE; return 0; }      // a band holds whole blocks
    return (int64_t)p->gam_group_rows;
}

}  // namespace

extern "C" {

int64_t mor_num_partitions(int32_t granularity, int64_t rows, int64_t cols) {
    if (check_shape(granularity, rows, cols, false) != MOR_OK) return -1;
    return mor::geom_parts(mor::make_geom(granularity, rows, cols));
}
int64_t mor_params_num_partitions(const mor_params* p) {
    if (check_common(p) != MOR_OK) return -1;
    return mor::geom_parts(mor::make_geom(p->granularity, p->rows, p->cols));
}

// Validates one operand and converts it to the launcher's descriptor.  `fake_y` non-null: fake quantization
// into fake_y (the FP8 payload and the fallback buffer of `out` are then ignored).
static mor_status make_item(const mor_params* p, const uint16_t* x, const mor_outputs* out, mor_stats* stats, uint16_t* fake_y,
                            int64_t ld_fake, mor::BatchItem* item) {
    if (!p || !x || !out) return MOR_ERR_NULL;
    mor_status st = check_common(p);
    if (st != MOR_OK) return st;
    if (p->scope != MOR_SCOPE_PARTITION && p->scope != MOR_SCOPE_TENSOR) return MOR_ERR_UNSUPPORTED;
    if (p->criterion != MOR_CRIT_MEAN_REL_ERR && p->criterion != MOR_CRIT_E4M3_VS_E5M2) return MOR_ERR_UNSUPPORTED;
    if (p->scaling < MOR_SCALE_FP32_AMAX || p->scaling > MOR_SCALE_E8M0) return MOR_ERR_UNSUPPORTED;
    const bool three = p->formats == (MOR_FMT_E4M3 | MOR_FMT_E5M2 | MOR_FMT_BF16);
    if (!three && p->formats != (MOR_FMT_E4M3 | MOR_FMT_BF16)) return MOR_ERR_UNSUPPORTED;
    if (three && p->scope != MOR_SCOPE_PARTITION) return MOR_ERR_UNSUPPORTED;
    if ((!fake_y && !out->fp8) || !out->scale || !out->amax || !out->err_sum || !out->nnz || !out->mask) return MOR_ERR_NULL;
    if (p->criterion == MOR_CRIT_E4M3_VS_E5M2 && !out->err5_sum) return MOR_ERR_NULL;
    if (p->ld < p->cols) return MOR_ERR_SHAPE;
    if (p->ld % 8) return MOR_ERR_ALIGN;
    if (!aligned16(x)) return MOR_ERR_ALIGN;
    bool want_bf16;
    if (fake_y) {
        if (ld_fake < p->cols) return MOR_ERR_SHAPE;
        if (ld_fake % 8 || !aligned16(fake_y)) return MOR_ERR_ALIGN;
        if (fake_y == x) return MOR_ERR_UNSUPPORTED;
        want_bf16 = true;
    } else {
        if (out->ld_fp8 < p->cols) return MOR_ERR_SHAPE;
        want_bf16 = out->bf16 != nullptr && out->bf16 != x;
        if (want_bf16 && out->ld_bf16 < p->cols) return MOR_ERR_SHAPE;
        if (out->ld_fp8 % 8 || (want_bf16 && out->ld_bf16 % 8)) return MOR_ERR_ALIGN;
        if ((reinterpret_cast<uintptr_t>(out->fp8) & 7u) || (want_bf16 && !aligned16(out->bf16))) return MOR_ERR_ALIGN;
    }
    static_assert(MOR_MAX_ROWS_TENSOR_SCOPE == 65535 * 128 + 127, "documented row limit");
    if (p->granularity != MOR_GRAN_TENSOR && p->rows > MOR_MAX_ROWS_TENSOR_SCOPE && p->scope == MOR_SCOPE_TENSOR) return MOR_ERR_SHAPE;
    // kernels whose blocks span several rows address a tile of up to 128 rows with 32-bit byte offsets
    if (p->granularity == MOR_GRAN_BLOCK_128x128 || p->granularity == MOR_GRAN_BLOCK_64x64 || p->granularity == MOR_GRAN_SUB_128x1 ||
        p->granularity == MOR_GRAN_CHANNEL_COL) {
        if (p->ld > MOR_MAX_LD || (fake_y ? ld_fake > MOR_MAX_LD : (out->ld_fp8 > MOR_MAX_LD || (want_bf16 && out->ld_bf16 > MOR_MAX_LD))))
            return MOR_ERR_SHAPE;
    }
    if ((reinterpret_cast<uintptr_t>(out->scale) | reinterpret_cast<uintptr_t>(out->amax) |
         reinterpret_cast<uintptr_t>(out->err_sum) | reinterpret_cast<uintptr_t>(out->nnz) |
         reinterpret_cast<uintptr_t>(out->amin)) & 3u) return MOR_ERR_ALIGN;
    if (stats && (reinterpret_cast<uintptr_t>(stats) & 7u)) return MOR_ERR_ALIGN;
    if (reinterpret_cast<uintptr_t>(out->group_mantissa) & 3u) return MOR_ERR_ALIGN;
    item->group_rows = group_rows_of(p, &st);
    if (st != MOR_OK) return st;
    item->sh = mor::KShape{p->rows, p->cols, p->ld};
    if (fake_y)
        item->o = mor::KOut{nullptr, p->cols, fake_y, ld_fake, out->scale, out->amax, out->err_sum, out->nnz, out->mask,
                            out->err5_sum, out->scale_e8m0, out->group_mantissa, out->amin, fake_y, ld_fake};
    else
        item->o = mor::KOut{out->fp8, out->ld_fp8, want_bf16 ? out->bf16 : nullptr, want_bf16 ? out->ld_bf16 : p->cols,
                            out->scale, out->amax, out->err_sum, out->nnz, out->mask, out->err5_sum,
                            out->scale_e8m0, out->group_mantissa, out->amin, nullptr, 0};
    item->x = x;
    item->gran = p->granularity;
    item->crit = p->criterion;
    item->scaling = p->scaling;
    item->scope = p->granularity == MOR_GRAN_TENSOR ? MOR_SCOPE_PARTITION : p->scope;
    item->three = three ? 1 : 0;
    item->ragged = (p->flags & MOR_FLAG_RAGGED) ? 1 : 0;
    item->lean = ((p->flags & MOR_FLAG_LEAN_FP8) && !fake_y) ? 1 : 0;
    item->th = p->threshold;
    item->stats = stats;
    return MOR_OK;
}

size_t mor_workspace_bytes(const mor_params* p) {
    if (check_common(p) != MOR_OK) return 0;
    mor::BatchItem it{};
    it.sh = mor::KShape{p->rows, p->cols, p->ld};
    it.gran = p->granularity;
    it.scope = p->granularity == MOR_GRAN_TENSOR ? MOR_SCOPE_PARTITION : p->scope;
    it.o.ld_fp8 = p->cols;
    it.scaling = p->scaling;
    it.ragged = (p->flags & MOR_FLAG_RAGGED) ? 1 : 0;
    mor_status st;
    it.group_rows = group_rows_of(p, &st);
    if (st != MOR_OK) return 0;
    return mor::batch_workspace_bytes(&it, 1);
}

static mor_status run_batch(const mor::BatchItem* items, int n, float near_tol, void* workspace, size_t workspace_bytes, void* stream,
                            mor_profile* profile) {
    const size_t need = mor::batch_workspace_bytes(items, n);
    if (need && (!workspace || workspace_bytes < need)) return MOR_ERR_WORKSPACE;
    if (need && !aligned16(workspace)) return MOR_ERR_ALIGN;
    static_assert(sizeof(mor_profile) == sizeof(mor::KProf), "mor_profile layout");
    if (profile) {
        profile->count = 0;
        for (int i = 0; i < profile->capacity && i < mor::kProfMax; ++i)
            if (!profile->start[i] || !profile->stop[i]) return MOR_ERR_NULL;
    }
    hipError_t e = mor::launch_batch(items, n, near_tol, workspace, workspace_bytes, static_cast<hipStream_t>(stream),
                                     reinterpret_cast<mor::KProf*>(profile));
    if (e == hipErrorOutOfMemory) return MOR_ERR_WORKSPACE;      // the launcher's own bound check on the workspace
    return e == hipSuccess ? MOR_OK : MOR_ERR_HIP;
}

mor_status mor_analyze_quantize(const mor_params* p, const uint16_t* x, const mor_outputs* out, void* workspace,
                                size_t workspace_bytes, void* stream) {
    mor::BatchItem it{};
    mor_status st = make_item(p, x, out, nullptr, nullptr, 0, &it);
    if (st != MOR_OK) return st;
    return run_batch(&it, 1, 0.0f, workspace, workspace_bytes, stream, nullptr);
}

mor_status mor_analyze_quantize_static(const mor_params* p, const uint16_t* x, const mor_outputs* out, void* stream) {
    mor::BatchItem it{};
    mor_status st = make_item(p, x, out, nullptr, nullptr, 0, &it);
    if (st != MOR_OK) return st;
    if (mor::batch_workspace_bytes(&it, 1) > (size_t)MOR_STATIC_SCRATCH_BYTES) return MOR_ERR_WORKSPACE;
    void* ws = nullptr;
    st = static_scratch(&ws);
    if (st != MOR_OK) return st;
    // the kernels write every scratch word before they read it, so nothing of the previous call's content has to be cleared
    return run_batch(&it, 1, 0.0f, ws, MOR_STATIC_SCRATCH_BYTES, stream, nullptr);
}

mor_status mor_analyze_quantize_profiled(const mor_params* p, const uint16_t* x, const mor_outputs* out, void* workspace,
                                         size_t workspace_bytes, void* stream, mor_profile* profile) {
    if (!profile) return MOR_ERR_NULL;
    mor::BatchItem it{};
    mor_status st = make_item(p, x, out, nullptr, nullptr, 0, &it);
    if (st != MOR_OK) return st;
    return run_batch(&it, 1, 0.0f, workspace, workspace_bytes, stream, profile);
}

size_t mor_batch_workspace_bytes(const mor_batch_item* items, int32_t n_items) {
    if (!items || n_items <= 0) return 0;
    size_t total = 0;
    for (int32_t i = 0; i < n_items; ++i) {
        mor::BatchItem it{};
        if (make_item(&items[i].params, items[i].x, &items[i].out, items[i].stats, items[i].fake_y, items[i].ld_fake_y, &it) != MOR_OK) return 0;
        total += mor::batch_workspace_bytes(&it, 1);
    }
    return total;
}

mor_status mor_analyze_quantize_batch(const mor_batch_item* items, int32_t n_items, float near_tol, void* workspace,
                                      size_t workspace_bytes, void* stream, mor_profile* profile) {
    if (!items) return MOR_ERR_NULL;
    if (n_items <= 0 || n_items > MOR_BATCH_MAX) return MOR_ERR_SHAPE;
    static_assert(MOR_BATCH_MAX == mor::kBatchMax, "batch limit");
    mor::BatchItem its[MOR_BATCH_MAX];
    for (int32_t i = 0; i < n_items; ++i) {
        mor_status st = make_item(&items[i].params, items[i].x, &items[i].out, items[i].stats, items[i].fake_y, items[i].ld_fake_y, &its[i]);
        if (st != MOR_OK) return st;
    }
    return run_batch(its, n_items, near_tol, workspace, workspace_bytes, stream, profile);
}

mor_status mor_fake_quantize(const mor_params* p, const uint16_t* x, uint16_t* y, int64_t ld_y, const mor_outputs* meta,
                             void* workspace, size_t workspace_bytes, void* stream) {
    if (!y) return MOR_ERR_NULL;
    mor::BatchItem it{};
    mor_status st = make_item(p, x, meta, nullptr, y, ld_y, &it);
    if (st != MOR_OK) return st;
    return run_batch(&it, 1, 0.0f, workspace, workspace_bytes, stream, nullptr);
}

static mor_status check_dequantize(const mor_params* p, const uint8_t* fp8, int64_t ld_fp8, const float* scale,
                                   const uint8_t* e8m0, const uint32_t* gmant, const uint8_t* mask, const uint16_t* bf16,
                                   int64_t ld_bf16, uint16_t* y, int64_t ld_y) {
    if (!p || !fp8 || !mask || !y) return MOR_ERR_NULL;
    if (!scale && !(e8m0 && gmant)) return MOR_ERR_NULL;
    mor_status st = check_common(p);
    if (st != MOR_OK) return st;
    if (ld_fp8 < p->cols || ld_y < p->cols || (bf16 && ld_bf16 < p->cols)) return MOR_ERR_SHAPE;
    if (ld_fp8 % 8 || ld_y % 8 || (bf16 && ld_bf16 % 8)) return MOR_ERR_ALIGN;
    if ((reinterpret_cast<uintptr_t>(fp8) & 7u) || !aligned16(y) || (bf16 && !aligned16(bf16))) return MOR_ERR_ALIGN;
    if ((reinterpret_cast<uintptr_t>(scale) | reinterpret_cast<uintptr_t>(gmant)) & 3u) return MOR_ERR_ALIGN;
    return MOR_OK;
}
static mor_status dequantize_any(const mor_params* p, const uint8_t* fp8, int64_t ld_fp8, const float* scale,
                                 const uint8_t* e8m0, const uint32_t* gmant, const uint8_t* mask, const uint16_t* bf16,
                                 int64_t ld_bf16, uint16_t* y, int64_t ld_y, void* stream) {
    mor_status st = check_dequantize(p, fp8, ld_fp8, scale, e8m0, gmant, mask, bf16, ld_bf16, y, ld_y);
    if (st != MOR_OK) return st;
    mor_status gs;
    const int64_t group_rows = group_rows_of(p, &gs);
    if (e8m0 && gs != MOR_OK) return gs;
    hipError_t e = mor::launch_dequantize(mor::make_geom(p->granularity, p->rows, p->cols), fp8, ld_fp8, scale, mask, bf16, ld_bf16,
                                          y, ld_y, e8m0, gmant, e8m0 ? group_rows : 0, static_cast<hipStream_t>(stream));
    return e == hipSuccess ? MOR_OK : MOR_ERR_HIP;
}

mor_status mor_dequantize_batch(const mor_dequant_item* items, int32_t n_items, void* stream) {
    if (!items) return MOR_ERR_NULL;
    if (n_items <= 0 || n_items > MOR_BATCH_MAX) return MOR_ERR_SHAPE;
    mor::DeqItem its[MOR_BATCH_MAX];
    for (int32_t i = 0; i < n_items; ++i) {
        const mor_dequant_item& d = items[i];
        const bool stored = d.scale == nullptr;
        mor_status st = check_dequantize(&d.params, d.fp8, d.ld_fp8, d.scale, d.scale_e8m0, d.group_mantissa, d.mask, d.bf16, d.ld_bf16,
                                         d.y, d.ld_y);
        if (st != MOR_OK) return st;
        mor_status gs;
        const int64_t group_rows = group_rows_of(&d.params, &gs);
        if (stored && gs != MOR_OK) return gs;
        its[i] = mor::DeqItem{mor::make_geom(d.params.granularity, d.params.rows, d.params.cols), d.fp8, d.ld_fp8, d.scale, d.mask,
                              d.bf16, d.ld_bf16, d.y, d.ld_y, stored ? d.scale_e8m0 : nullptr, stored ? d.group_mantissa : nullptr,
                              stored ? group_rows : 0};
    }
    hipError_t e = mor::launch_dequantize_batch(its, n_items, static_cast<hipStream_t>(stream));
    return e == hipSuccess ? MOR_OK : MOR_ERR_HIP;
}

mor_status mor_dequantize(const mor_params* p, const uint8_t* fp8, int64_t ld_fp8, const float* scale, const uint8_t* mask,
                          const uint16_t* bf16, int64_t ld_bf16, uint16_t* y, int64_t ld_y, void* stream) {
    if (!scale) return MOR_ERR_NULL;
    return dequantize_any(p, fp8, ld_fp8, scale, nullptr, nullptr, mask, bf16, ld_bf16, y, ld_y, stream);
}

mor_status mor_dequantize_e8m0(const mor_params* p, const uint8_t* fp8, int64_t ld_fp8, const uint8_t* scale_e8m0,
                               const uint32_t* group_mantissa, const uint8_t* mask, const uint16_t* bf16, int64_t ld_bf16,
                               uint16_t* y, int64_t ld_y, void* stream) {
    if (!scale_e8m0 || !group_mantissa) return MOR_ERR_NULL;
    return dequantize_any(p, fp8, ld_fp8, nullptr, scale_e8m0, group_mantissa, mask, bf16, ld_bf16, y, ld_y, stream);
}

mor_status mor_select_stats(const mor_params* p, const float* err_sum, const uint32_t* nnz, const uint8_t* mask, float near_tol,
                            mor_stats* out_dev, void* stream) {
    if (!p || !err_sum || !nnz || !mask || !out_dev) return MOR_ERR_NULL;
    mor_status st = check_common(p);
    if (st != MOR_OK) return st;
    if ((reinterpret_cast<uintptr_t>(err_sum) | reinterpret_cast<uintptr_t>(nnz)) & 3u) return MOR_ERR_ALIGN;
    if (reinterpret_cast<uintptr_t>(out_dev) & 7u) return MOR_ERR_ALIGN;
    static_assert(sizeof(mor_stats) == 144, "mor_stats layout");
    hipError_t e = mor::launch_select_stats(mor::make_geom(p->granularity, p->rows, p->cols), err_sum, nnz,
                                            mask, p->threshold, near_tol, out_dev, static_cast<hipStream_t>(stream));
    return e == hipSuccess ? MOR_OK : MOR_ERR_HIP;
}

mor_status mor_histogram_update(uint32_t* hist12_dev, const mor_stats* stats_dev, int64_t step, int64_t reset_interval, void* stream) {
    if (!hist12_dev || !stats_dev) return MOR_ERR_NULL;
    if (step < 0 || reset_interval < 0) return MOR_ERR_SHAPE;
    if ((reinterpret_cast<uintptr_t>(hist12_dev) & 3u) || (reinterpret_cast<uintptr_t>(stats_dev) & 7u)) return MOR_ERR_ALIGN;
    const int clear = (reset_interval > 0 && step % reset_interval == 0) ? 1 : 0;
    hipError_t e = mor::launch_histogram_update(hist12_dev, stats_dev, clear, static_cast<hipStream_t>(stream));
    return e == hipSuccess ? MOR_OK : MOR_ERR_HIP;
}

const char* mor_status_string(mor_status s) {
    switch (s) {
    case MOR_OK: return "ok";
    case MOR_ERR_NULL: return "a required pointer is NULL";
    case MOR_ERR_SHAPE: return "invalid shape or leading dimension for the granularity";
    case MOR_ERR_ALIGN: return "pointer or leading dimension not aligned";
    case MOR_ERR_UNSUPPORTED: return "unsupported enum value or format set";
    case MOR_ERR_WORKSPACE: return "workspace missing or too small";
    case MOR_ERR_HIP: return "HIP launch failed";
    default: return "unknown status";
    }
}

}  // extern "C"
