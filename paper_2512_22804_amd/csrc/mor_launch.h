// Host-side launch interface between the C ABI (mor_api.hip) and the kernels (mor_kernels.hip).
#pragma once
#include <hip/hip_runtime.h>
#include <stddef.h>
#include <stdint.h>

namespace mor {

// Device pointers of one call, passed to kernels by value.
struct KOut {
    uint8_t*  fp8;      int64_t ld_fp8;
    uint16_t* bf16;     int64_t ld_bf16;     // bf16 == nullptr: no fallback payload is written
    float*    scale;
    float*    amax;
    float*    err_sum;
    uint32_t* nnz;
    uint8_t*  mask;
    float*    err5_sum;
    uint8_t*  e8m0;     // [P] biased exponents of the applied scales (GAM / E8M0 scaling), may be nullptr
    uint32_t* gmant;    // [2] fraction bits of the group mantissas (E4M3, E5M2), may be nullptr
    float*    amin;     // [P] smallest non-zero magnitude of blocks that failed M_1 (three-way recipe), may be nullptr
    uint16_t* fake;     // fake quantization: de-quantized BF16 output instead of the FP8 payload (then bf16 == fake
    int64_t   ld_fake;  //   so that BF16 blocks pass through); nullptr otherwise
};

struct KShape {
    int64_t rows, cols, ld;
};

// Block grid of an operand: nominal block pr x pc, grid gr x gc (edge blocks smaller when ragged).
struct StatsGeom {
    int64_t rows, cols, pr, pc, gc;
    int32_t uniform;        // 1: every block has pr * pc elements
};
enum { kGranTensor = 0, kGranSub = 1, kGranBlock = 2, kGranRow = 3, kGranCol = 4, kGranSubCol = 5, kGranBlock64 = 6 };
inline StatsGeom make_geom(int gran, int64_t rows, int64_t cols) {
    StatsGeom g{rows, cols, rows, cols, 1, 1};
    switch (gran) {
    case kGranSub:     g.pr = 1;   g.pc = 128; break;
    case kGranBlock:   g.pr = 128; g.pc = 128; break;
    case kGranRow:     g.pr = 1;   g.pc = cols; break;
    case kGranCol:     g.pr = rows; g.pc = 1;  break;
    case kGranSubCol:  g.pr = 128; g.pc = 1;   break;
    case kGranBlock64: g.pr = 64;  g.pc = 64;  break;
    default: break;
    }
    g.gc = (cols + g.pc - 1) / g.pc;
    g.uniform = (rows % g.pr == 0 && cols % g.pc == 0) ? 1 : 0;
    return g;
}
inline int64_t geom_parts(const StatsGeom& g) { return ((g.rows + g.pr - 1) / g.pr) * g.gc; }

// Workspace layout for the passes that need one (all offsets 16-byte aligned).
struct TensorPlan {
    int     amax_blocks;     // grid of the amax pass
    int64_t quant_blocks;    // grid of the quantize pass
    size_t  off_amax_part;   // uint32[amax_blocks]
    size_t  off_err_part;    // float[quant_blocks]
    size_t  off_err5_part;   // float[quant_blocks]
    size_t  off_nnz_part;    // uint32[quant_blocks]
    size_t  off_decision;    // uint32[4]: [0] global amax bits
    size_t  off_flush_part;  // uint32[amax_blocks]
    size_t  bytes;
};
TensorPlan plan_tensor(int64_t rows, int64_t cols);
size_t scope_workspace_bytes(int64_t n_part);

constexpr int kProfMax = 16;
// Optional per-kernel timing: when non-null, start[i]/stop[i] are recorded around the i-th kernel.
struct KProf {
    int32_t capacity;
    int32_t count;
    hipEvent_t start[kProfMax];
    hipEvent_t stop[kProfMax];
    int32_t kernel[kProfMax];
};
enum KernelId {
    kKernSub1x128 = 1, kKernBlock128 = 2, kKernTensorAmax = 3, kKernTensorQuant = 4, kKernTensorFinalize = 5,
    kKernFallbackCopy = 6, kKernScopeReduce = 7, kKernScopeDecide = 8, kKernScopeFillMask = 9,
    kKernStatsPartial = 10, kKernStatsFinal = 11, kKernGroupAmax = 12, kKernGroupMantissa = 13,
    kKernTeamBlock = 14, kKernColumnTile = 15, kKernColumnCombine = 16
};

// Records the caller's events around one kernel launch when profiling is requested.
struct ProfScope {
    KProf* prof; hipStream_t st; int slot;
    ProfScope(KProf* p, int kernel_id, hipStream_t s) : prof(p), st(s), slot(-1) {
        if (prof && prof->count < prof->capacity && prof->count < kProfMax) {
            slot = prof->count++;
            prof->kernel[slot] = kernel_id;
            (void)hipEventRecord(prof->start[slot], st);
        }
    }
    ~ProfScope() { if (slot >= 0) (void)hipEventRecord(prof->stop[slot], st); }
};

// Residency caps: bytes of dynamic LDS a launch reserves (and never touches) so that only 3 or 5 workgroups of 256
// lanes fit the 160 KB of a compute unit.  The streaming passes run faster with FEWER workgroups in flight than
// their register use would allow (measured on MI355X: pass B of the per-tensor path 214 us at 3 per unit, 226 us at 4,
// 237 us at 6, 223 us at 2; pass A 79 us at 3 against 81 us uncapped; the 128x128 team kernel 114 us at 4 or 5 against
// 116 us at 7; the quantize pass of the per-channel columns 0.609 ms per twelve-operand pass at 4 against 0.620 ms
// uncapped): fewer concurrent streams keep the accesses of each HBM channel closer together.  Kernels that need many
// waves to hide latency (de-quantization, 128x1 sub-columns) lose with a cap and have none.
constexpr int kResidency3 = 52000;
constexpr int kResidency4 = 39000;
constexpr int kResidency5 = 31000;

constexpr int kBatchMax = 64;     // operands per batch call

// One operand of a batch (validated by the caller).
struct BatchItem {
    KShape sh;
    KOut o;
    const uint16_t* x;
    int gran, crit, scope;
    int scaling;            // 0 FP32 amax, 1 GAM, 2 E8M0 only
    int three;              // 1: type list [E4M3, E5M2, BF16]
    int ragged;             // 1: edge blocks may be smaller
    int lean;               // 1: the FP8 payload of blocks already known to stay in BF16 need not be written
    float th;
    void* stats;            // device mor_stats* or nullptr
    int64_t group_rows;     // GAM: 0 = one group (the whole operand); else the groups of Algorithm 1 are bands of this many rows
};
size_t batch_workspace_bytes(const BatchItem* items, int n);
hipError_t launch_batch(const BatchItem* items, int n, float near_tol, void* ws, size_t ws_bytes, hipStream_t st, KProf* prof);

// mor_partitions.hip: team kernels (64x64, per-channel rows, general 128x128) and column kernels
enum { kCritEq2 = 0, kCritEq3 = 1 };

// That many elements certain to flush (each contributes exactly 1 to the error sum of Eq. 2) prove "mean relative error
// >= th" for a block of `n` elements, whatever the other terms are: the 1 % margin over th * n covers the rounding of the
// binary32 error sums that the decision itself is taken from.  Only used for 0 < th < 0.9.
inline unsigned long long flush_need_of(float th, int64_t n) { return (unsigned long long)(1.01 * (double)th * (double)n) + 1ull; }

// Tensor-level decision (Section 3.1) over GAM-scaled sub-tensor blocks (128 x 128, 64 x 64, per-channel rows, 1 x 128 sub-rows,
// 128 x 1 sub-columns): the amax pre-pass of Algorithm 1 can prove the BF16 decision under Eq. 2 from elements that are certain to
// flush inside their block, so the block kernel writes the BF16 payload from its registers and the operand is not read a third time.
inline bool scope_proof_applies(const BatchItem& it) {
    // (fake quantization: o.bf16 == o.fake, and a proven operand's output is its input)
    if (it.scaling != 1 || it.scope != 1 || it.crit != kCritEq2 || it.three || it.o.bf16 == nullptr || it.group_rows != 0) return false;
    if (!(it.th > 0.0f && it.th < 0.9f)) return false;      // the flush count is compared with 1.01 * th * N + 1
    const bool whole_tiles = it.sh.rows % 128 == 0 && it.sh.cols % 128 == 0;
    if (it.gran == kGranBlock || it.gran == kGranBlock64 || it.gran == kGranSubCol) return whole_tiles;
    if (it.gran == kGranSub)      // the flat 1 x 128 kernel only (dense operand)
        return whole_tiles && it.sh.ld == it.sh.cols && it.o.ld_bf16 == it.sh.cols && (it.o.fake != nullptr ? it.o.ld_fake == it.sh.cols : it.o.ld_fp8 == it.sh.cols);
    return it.gran == kGranRow;
}
// Work units of the pre-pass (16384 elements each) and its per-operand arguments: per workgroup the largest amax and
// the number of certain flushes it saw.
inline int64_t scope_proof_units(const BatchItem& it) {
    if (it.gran == kGranRow) return (it.sh.rows * ((it.sh.cols + 4095) / 4096) + 3) / 4;
    return (it.sh.rows / 128) * (it.sh.cols / 128);
}
enum { kProveKindBlock128 = 0, kProveKindRows = 1, kProveKindBlock64 = 2, kProveKindSubRow = 3, kProveKindSubCol = 4 };
inline int scope_proof_kind(const BatchItem& it) {
    switch (it.gran) {
    case kGranRow: return kProveKindRows;
    case kGranBlock64: return kProveKindBlock64;
    case kGranSub: return kProveKindSubRow;
    case kGranSubCol: return kProveKindSubCol;
    default: return kProveKindBlock128;
    }
}
struct BlockProveItem {
    const uint16_t* x;
    int64_t rows, cols, ld;
    uint32_t* amax_part;     // [n_wg]
    uint32_t* flush_part;    // [n_wg]
    int n_wg;
    int kind;                // kProveKind*
};
hipError_t launch_block_amax_prove(const BlockProveItem* ops, int n, hipStream_t st);

constexpr int kTeamKinds = 5;      // team kinds are numbered 0 .. kTeamKinds - 1 (mor_partitions.hip)
int team_kind_of(const BatchItem& it);
struct TeamRiders;      // mor_sub1x128.h
hipError_t launch_team_items(const BatchItem* items, const int* idx, int cnt, int kind, int crit, const uint32_t* const* gam_of,
                             TeamRiders* riders, hipStream_t st, KProf* prof);
hipError_t launch_subcol_items(const BatchItem* items, const int* idx, int cnt, int crit, const uint32_t* const* gam_of,
                               hipStream_t st, KProf* prof);
size_t column_workspace_bytes(int64_t rows, int64_t cols);
// Per-channel columns with a tensor-level decision: the column-amax pass counts certain flushes per column anyway, and their
// total may prove the operand's BF16 decision (Eq. 2); the quantize pass then writes the fallback and the word below says so.
inline bool column_tensor_proof_applies(const BatchItem& it) {
    return it.gran == kGranCol && it.scope == 1 && it.crit == kCritEq2 && !it.three && it.o.bf16 != nullptr && it.o.fake == nullptr &&
           it.th > 0.0f && it.th < 0.9f;
}
uint32_t* column_tensor_proven_word(char* column_workspace, int64_t rows, int64_t cols);
hipError_t launch_channel_col_items(const BatchItem* items, const int* idx, int cnt, int crit, const uint32_t* const* gam_of,
                                    char* const* ws_of, hipStream_t st, KProf* prof);

hipError_t launch_dequantize(const StatsGeom& geom, const uint8_t* fp8, int64_t ld_fp8, const float* scale,
                             const uint8_t* mask, const uint16_t* bf16, int64_t ld_bf16, uint16_t* y, int64_t ld_y,
                             const uint8_t* e8m0, const uint32_t* gmant, int64_t group_rows, hipStream_t st);
// One operand of a de-quantize batch (validated by the caller).
struct DeqItem {
    StatsGeom geom;
    const uint8_t* fp8; int64_t ld_fp8;
    const float* scale; const uint8_t* mask;
    const uint16_t* bf16; int64_t ld_bf16;
    uint16_t* y; int64_t ld_y;
    const uint8_t* e8m0; const uint32_t* gmant;
    int64_t group_rows;      // stored GAM form: rows per group (0 = one group)
};
hipError_t launch_dequantize_batch(const DeqItem* items, int n, hipStream_t st);
hipError_t launch_select_stats(const StatsGeom& geom, const float* err_sum, const uint32_t* nnz,
                               const uint8_t* mask, float th, float near_tol, void* out_dev, hipStream_t st);
hipError_t launch_histogram_update(uint32_t* hist, const void* stats_dev, int clear, hipStream_t st);

}  // namespace mor
