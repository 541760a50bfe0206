// C ABI of the MoR analyse-select-quantize library: argument validation and dispatch only.
// Every step of the path runs in the kernels of mor_kernels.hip.
#include "../../include/mor.h"
#include "mor_launch.h"

namespace {

bool aligned16(const void* p) { return (reinterpret_cast<uintptr_t>(p) & 15u) == 0; }

mor_status check_common(const mor_params* p) {
    if (!p) return MOR_ERR_NULL;
    if (p->granularity < MOR_GRAN_TENSOR || p->granularity > MOR_GRAN_BLOCK_128x128) return MOR_ERR_UNSUPPORTED;
    if (p->rows <= 0 || p->cols <= 0) return MOR_ERR_SHAPE;
    if (mor_num_partitions(p->granularity, p->rows, p->cols) < 0) return MOR_ERR_SHAPE;
    return MOR_OK;
}

int64_t elems_per_part(const mor_params* p) {
    switch (p->granularity) {
    case MOR_GRAN_SUB_1x128: return 128;
    case MOR_GRAN_BLOCK_128x128: return 128 * 128;
    default: return p->rows * p->cols;
    }
}

}  // namespace

extern "C" {

int64_t mor_num_partitions(int32_t granularity, int64_t rows, int64_t cols) {
    if (rows <= 0 || cols <= 0) return -1;
    switch (granularity) {
    case MOR_GRAN_TENSOR: return (cols % 8) ? -1 : 1;            // 16-byte rows
    case MOR_GRAN_SUB_1x128: return (cols % 128) ? -1 : rows * (cols / 128);
    case MOR_GRAN_BLOCK_128x128: return (rows % 128 || cols % 128) ? -1 : (rows / 128) * (cols / 128);
    default: return -1;
    }
}

size_t mor_workspace_bytes(const mor_params* p) {
    if (check_common(p) != MOR_OK) return 0;
    if (p->granularity == MOR_GRAN_TENSOR) return mor::plan_tensor(p->rows, p->cols).bytes;
    if (p->scope == MOR_SCOPE_TENSOR) return mor::scope_workspace_bytes(mor_num_partitions(p->granularity, p->rows, p->cols));
    return 0;
}

static mor_status analyze_quantize_impl(const mor_params* p, const uint16_t* x, const mor_outputs* out, void* workspace,
                                        size_t workspace_bytes, void* stream, mor::KProf* prof) {
    if (!p || !x || !out) return MOR_ERR_NULL;
    mor_status st = check_common(p);
    if (st != MOR_OK) return st;
    if (p->scope != MOR_SCOPE_PARTITION && p->scope != MOR_SCOPE_TENSOR) return MOR_ERR_UNSUPPORTED;
    if (p->criterion != MOR_CRIT_MEAN_REL_ERR && p->criterion != MOR_CRIT_E4M3_VS_E5M2) return MOR_ERR_UNSUPPORTED;
    if (p->scaling != MOR_SCALE_FP32_AMAX) return MOR_ERR_UNSUPPORTED;
    if (p->formats != (MOR_FMT_E4M3 | MOR_FMT_BF16)) return MOR_ERR_UNSUPPORTED;
    if (!out->fp8 || !out->scale || !out->amax || !out->err_sum || !out->nnz || !out->mask) return MOR_ERR_NULL;
    if (p->criterion == MOR_CRIT_E4M3_VS_E5M2 && !out->err5_sum) return MOR_ERR_NULL;
    if (p->ld < p->cols || out->ld_fp8 < p->cols) return MOR_ERR_SHAPE;
    const bool want_bf16 = out->bf16 != nullptr && out->bf16 != x;
    if (want_bf16 && out->ld_bf16 < p->cols) return MOR_ERR_SHAPE;
    if (p->ld % 8 || out->ld_fp8 % 8 || (want_bf16 && out->ld_bf16 % 8)) return MOR_ERR_ALIGN;
    if (!aligned16(x) || (reinterpret_cast<uintptr_t>(out->fp8) & 7u) || (want_bf16 && !aligned16(out->bf16))) return MOR_ERR_ALIGN;
    if ((reinterpret_cast<uintptr_t>(out->scale) | reinterpret_cast<uintptr_t>(out->amax) |
         reinterpret_cast<uintptr_t>(out->err_sum) | reinterpret_cast<uintptr_t>(out->nnz)) & 3u) return MOR_ERR_ALIGN;
    const size_t need = mor_workspace_bytes(p);
    if (need && (!workspace || workspace_bytes < need)) return MOR_ERR_WORKSPACE;
    if (need && !aligned16(workspace)) return MOR_ERR_ALIGN;

    mor::KShape sh{p->rows, p->cols, p->ld};
    mor::KOut ko{out->fp8, out->ld_fp8, want_bf16 ? out->bf16 : nullptr, want_bf16 ? out->ld_bf16 : p->cols,
                 out->scale, out->amax, out->err_sum, out->nnz, out->mask, out->err5_sum};
    hipStream_t hs = static_cast<hipStream_t>(stream);
    const bool defer = p->scope == MOR_SCOPE_TENSOR;
    hipError_t e;
    switch (p->granularity) {
    case MOR_GRAN_TENSOR:
        e = mor::launch_tensor(x, sh, ko, p->criterion, p->threshold, workspace, hs, prof);
        break;
    case MOR_GRAN_SUB_1x128:
        e = mor::launch_sub1x128(x, sh, ko, p->criterion, defer, p->threshold, hs, prof);
        break;
    default:
        e = mor::launch_block128(x, sh, ko, p->criterion, defer, p->threshold, hs, prof);
        break;
    }
    if (e == hipSuccess && defer && p->granularity != MOR_GRAN_TENSOR)
        e = mor::launch_scope_finalize(x, sh, ko, mor_num_partitions(p->granularity, p->rows, p->cols), p->criterion,
                                       p->threshold, workspace, hs, prof);
    return e == hipSuccess ? MOR_OK : MOR_ERR_HIP;
}

mor_status mor_analyze_quantize(const mor_params* p, const uint16_t* x, const mor_outputs* out, void* workspace,
                                size_t workspace_bytes, void* stream) {
    return analyze_quantize_impl(p, x, out, workspace, workspace_bytes, stream, nullptr);
}

mor_status mor_analyze_quantize_profiled(const mor_params* p, const uint16_t* x, const mor_outputs* out, void* workspace,
                                         size_t workspace_bytes, void* stream, mor_profile* profile) {
    static_assert(sizeof(mor_profile) == sizeof(mor::KProf), "mor_profile layout");
    if (!profile) return MOR_ERR_NULL;
    profile->count = 0;
    for (int i = 0; i < profile->capacity && i < 8; ++i)
        if (!profile->start[i] || !profile->stop[i]) return MOR_ERR_NULL;
    return analyze_quantize_impl(p, x, out, workspace, workspace_bytes, stream, reinterpret_cast<mor::KProf*>(profile));
}

mor_status mor_dequantize(const mor_params* p, const uint8_t* fp8, int64_t ld_fp8, const float* scale, const uint8_t* mask,
                          const uint16_t* bf16, int64_t ld_bf16, uint16_t* y, int64_t ld_y, void* stream) {
    if (!p || !fp8 || !scale || !mask || !y) return MOR_ERR_NULL;
    mor_status st = check_common(p);
    if (st != MOR_OK) return st;
    if (ld_fp8 < p->cols || ld_y < p->cols || (bf16 && ld_bf16 < p->cols)) return MOR_ERR_SHAPE;
    if (ld_fp8 % 8 || ld_y % 8 || (bf16 && ld_bf16 % 8)) return MOR_ERR_ALIGN;
    if ((reinterpret_cast<uintptr_t>(fp8) & 7u) || !aligned16(y) || (bf16 && !aligned16(bf16))) return MOR_ERR_ALIGN;
    if (reinterpret_cast<uintptr_t>(scale) & 3u) return MOR_ERR_ALIGN;
    hipError_t e = mor::launch_dequantize(p->granularity, p->rows, p->cols, fp8, ld_fp8, scale, mask, bf16, ld_bf16, y, ld_y,
                                          static_cast<hipStream_t>(stream));
    return e == hipSuccess ? MOR_OK : MOR_ERR_HIP;
}

mor_status mor_select_stats(const mor_params* p, const float* err_sum, const uint32_t* nnz, const uint8_t* mask, float near_tol,
                            mor_stats* out_dev, void* stream) {
    if (!p || !err_sum || !nnz || !mask || !out_dev) return MOR_ERR_NULL;
    mor_status st = check_common(p);
    if (st != MOR_OK) return st;
    if ((reinterpret_cast<uintptr_t>(err_sum) | reinterpret_cast<uintptr_t>(nnz)) & 3u) return MOR_ERR_ALIGN;
    if (reinterpret_cast<uintptr_t>(out_dev) & 7u) return MOR_ERR_ALIGN;
    static_assert(sizeof(mor_stats) == 128, "mor_stats layout");
    hipError_t e = mor::launch_select_stats(mor_num_partitions(p->granularity, p->rows, p->cols), elems_per_part(p), err_sum, nnz,
                                            mask, p->threshold, near_tol, out_dev, static_cast<hipStream_t>(stream));
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
