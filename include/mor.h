/*
 * mor.h -- C ABI of the MI355X (gfx950) MoR analyse-select-quantize library.
 *
 * MoR (Mixture of Representations) takes a BF16 GEMM operand X, a partition B of
 * X into blocks, an ordered list of representation types and acceptance metrics,
 * and returns the quantized tensor X_Q plus per-block metadata D (Algorithm 2).
 * This library implements the recipes with the type lists [E4M3, BF16] and
 * [E4M3, E5M2, BF16]: for every block it computes amax and a scale (Algorithm 1:
 * plain per-block FP32 form, GAM, or E8M0 only), quantizes to FP8 E4M3, evaluates
 * the acceptance metric (Eq. 1-2 or Eq. 3) on the de-quantized values, and keeps
 * the E4M3 payload, (three-way recipe, Eq. 4) an E5M2 payload, or the original
 * BF16 block.
 *
 * Conventions shared by all entry points
 *   - Every data pointer is DEVICE memory owned by the caller.  mor_params and
 *     mor_outputs themselves are HOST structs, read before the call returns.
 *   - `stream` is a hipStream_t passed as void* (NULL = the default stream).
 *     Calls only enqueue work on it; they never allocate, free or synchronize.
 *     Results are valid once the stream has reached the end of the call's work.
 *   - Tensors are row-major; a leading dimension `ld` counts ELEMENTS between
 *     the starts of consecutive rows.
 *   - Blocks are numbered row-major over the block grid: for blocks of pr x pc elements
 *     p = (r/pr) * ceil(cols/pc) + c/pc (1x128 sub-channels: p = r * (cols/128) + c/128;
 *     128x128 blocks: p = (r/128)*(cols/128) + c/128; per-tensor: one block, p = 0).
 *     P = number of blocks.
 *   - mask[p] = 0: block kept as FP8 E4M3;  mask[p] = 1: block kept as BF16;
 *     mask[p] = 2 (three-way recipe only): block kept as FP8 E5M2.
 *   - Argument errors are reported synchronously through the return code and
 *     nothing is launched.  Non-finite data is not an error: a block holding Inf
 *     or NaN gets scale 1, err_sum = +inf and is kept in BF16.
 *   - No call is made into any CPU fallback: without a working HIP device the
 *     entry points return MOR_ERR_HIP.
 */
#ifndef MOR_H_
#define MOR_H_

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

#define MOR_MAX_LD 4194304   /* elements (2^22): largest leading dimension of a call whose blocks span several rows */
#define MOR_MAX_ROWS_TENSOR_SCOPE 8388607   /* MOR_SCOPE_TENSOR over a sub-tensor granularity: rows / 128 <= 65535 */

typedef enum {
    MOR_OK = 0,
    MOR_ERR_NULL = 1,        /* a required pointer is NULL */
    MOR_ERR_SHAPE = 2,       /* rows/cols <= 0, ld < cols, not a multiple of the block shape, a leading dimension
                                above MOR_MAX_LD for a granularity whose blocks span several rows, or more than
                                MOR_MAX_ROWS_TENSOR_SCOPE rows for a tensor-level decision over sub-tensor blocks */
    MOR_ERR_ALIGN = 3,       /* a pointer is not 16-byte aligned or a leading dimension breaks 16-byte rows */
    MOR_ERR_UNSUPPORTED = 4, /* enum value or format set this build does not implement */
    MOR_ERR_WORKSPACE = 5,   /* workspace NULL or smaller than mor_workspace_bytes() */
    MOR_ERR_HIP = 6          /* a HIP launch or runtime call failed */
} mor_status;

/* The partition B of the tensor (Section 3, first paragraph). */
typedef enum {
    MOR_GRAN_TENSOR = 0,        /* one block: the whole tensor */
    MOR_GRAN_SUB_1x128 = 1,     /* sub-channel blocks of 1 x 128 along the columns (sub-rows) */
    MOR_GRAN_BLOCK_128x128 = 2, /* 2-D blocks of 128 x 128 */
    MOR_GRAN_CHANNEL_ROW = 3,   /* per-channel: every row is one block (first GEMM operand, Section 4.1.1);
                                   cols <= 65536 */
    MOR_GRAN_CHANNEL_COL = 4,   /* per-channel: every column is one block (second GEMM operand) */
    MOR_GRAN_SUB_128x1 = 5,     /* sub-channel blocks of 128 x 1 along the rows (sub-columns: the transposed
                                   operands of the backward GEMMs, Section 4) */
    MOR_GRAN_BLOCK_64x64 = 6    /* 2-D blocks of 64 x 64 (block-size ablation of Section 4.1.2) */
} mor_granularity;
/* Unless MOR_FLAG_RAGGED is set, rows and cols must be whole numbers of blocks.  cols % 8 == 0 always
 * (16-byte rows). */

/* Representation types, most to least aggressive (Section 3); `formats` is a bit-or:
 * MOR_FMT_E4M3 | MOR_FMT_BF16 (two types) or MOR_FMT_E4M3 | MOR_FMT_E5M2 | MOR_FMT_BF16 (the three-way
 * recipe of Section 3.2: a block that fails M_1 is kept in E5M2 when its dynamic range fits E5M2's
 * normal range, Eq. (4): max|b| / min|b| < 57344 / 2^-14, the minimum taken over the non-zero elements,
 * a block without non-zero elements passing; otherwise BF16).  Three types need MOR_SCOPE_PARTITION (the
 * recipe decides block by block); every granularity supports them. */
enum { MOR_FMT_E4M3 = 1, MOR_FMT_E5M2 = 2, MOR_FMT_BF16 = 4 };

/* mor_params.flags */
enum {
    MOR_FLAG_RAGGED = 1,        /* rows / cols need not be multiples of the block shape (the paper is silent on
                                   edges): the grid is ceil(rows/pr) x ceil(cols/pc) and edge blocks are smaller */
    MOR_FLAG_LEAN_FP8 = 2       /* Algorithm 2 keeps one representation per block: with this flag the FP8 payload of a
                                   block whose BF16 decision is already known when its codes would be stored is not
                                   written (those bytes of out->fp8 keep their previous content; mask[p] == 1 says so).
                                   Today that is a per-tensor operand whose decision the amax pass has proven (see
                                   MOR_STATS_FLAG_FUSED_FALLBACK): the quantize pass then moves 4 instead of 5 bytes
                                   per element.  All other outputs are unchanged.  Ignored by mor_fake_quantize. */
};

/* Acceptance metric M_1 for E4M3. */
typedef enum {
    MOR_CRIT_MEAN_REL_ERR = 0,  /* Eq. (1)-(2): mean relative error over non-zeros < threshold */
    MOR_CRIT_E4M3_VS_E5M2 = 1   /* Eq. (3), two-way recipe of Section 3.2: total relative error of
                                   E4M3 strictly below that of E5M2; E5M2 itself is never emitted */
} mor_criterion;

/* Where the decision is taken. */
typedef enum {
    MOR_SCOPE_PARTITION = 0,    /* sub-tensor MoR (Section 3.2): one decision per block */
    MOR_SCOPE_TENSOR = 1        /* tensor-level MoR (Section 3.1): block error sums are aggregated,
                                   sum(err_sum)/sum(nnz) (or the two Eq. 3 totals) decides once and
                                   every mask[p] receives that decision.  With a sub-tensor granularity the
                                   operand may have at most MOR_MAX_ROWS_TENSOR_SCOPE rows (MOR_ERR_SHAPE) */
} mor_scope;

/* How the per-block scale is formed. */
typedef enum {
    MOR_SCALE_FP32_AMAX = 0,    /* s = fl32(448 / amax): one binary32 scale per block straight from its amax
                                   (first scaling variant of the ablation in Section 4.1.2).  amax == 0 -> s = 1;
                                   an overflowing quotient -> s = FLT_MAX; non-finite amax -> s = 1. */
    MOR_SCALE_GAM = 1,          /* Group Amax Mantissa scaling (Algorithm 1).  One group = the whole operand unless
                                   mor_params.gam_group_rows says otherwise: s_g = fl32(448 / amax of the group), m_g = its mantissa;
                                   per block s_b as above, e = exponent(s_b), lowered by one when
                                   m_g > mantissa(s_b); applied scale s = m_g * 2^e (s_b/2 < s <= s_b).
                                   Stored form: one 23-bit mantissa + one E8M0 byte per block.  The
                                   operand is read once more for its amax (Section 3.1, Figure 2).
                                   For Eq. (3) the E5M2 side uses its own m_g from 57344 / amax. */
    MOR_SCALE_E8M0 = 2          /* E8M0-only per-block scaling (ablation of Section 4.1.2): the power of
                                   two 2^exponent(s_b), i.e. the above with m_g = 1; no extra read. */
} mor_scaling;

typedef struct mor_params {
    int64_t  rows, cols;  /* operand shape, elements */
    int64_t  ld;          /* leading dimension of x in elements, >= cols, multiple of 8; at most MOR_MAX_LD (as every
                             other leading dimension of the call) when blocks span several rows (128x128, 64x64, 128x1,
                             per-channel columns): their kernels address a tile of rows with 32-bit byte offsets */
    int32_t  granularity; /* mor_granularity */
    int32_t  scope;       /* mor_scope */
    int32_t  criterion;   /* mor_criterion */
    int32_t  scaling;     /* mor_scaling */
    uint32_t formats;     /* MOR_FMT_E4M3 | MOR_FMT_BF16, or MOR_FMT_E4M3 | MOR_FMT_E5M2 | MOR_FMT_BF16 */
    float    threshold;   /* th_E4M3 of Eq. (2), e.g. 0.045f (Section 4.1.1); ignored for Eq. (3) */
    uint32_t flags;       /* MOR_FLAG_* bits */
    uint32_t gam_group_rows; /* MOR_SCALE_GAM only (ignored otherwise): 0 = one group, the whole operand (the configuration of the
                                paper's experiments); else the groups of Algorithm 1 are bands of this many consecutive rows,
                                each with its own mantissa m_g.  A band must hold whole blocks (a multiple of the block
                                height: 128, 64 or 1), so per-tensor granularity and per-channel columns take 0 only
                                (MOR_ERR_UNSUPPORTED); a value >= rows means one group.  n_groups = ceil(rows / gam_group_rows) */
} mor_params;

typedef struct mor_outputs {
    uint8_t*  fp8;      /* [rows x ld_fp8] E4M3 codes, written for EVERY block (also BF16 ones); E5M2 codes in
                           blocks with mask == 2 */
    int64_t   ld_fp8;   /* >= cols, multiple of 8 */
    uint16_t* bf16;     /* [rows x ld_bf16] BF16 fallback: input bits, written ONLY in blocks with
                           mask == 1, other regions untouched.  May be NULL (no payload emitted)
                           and may equal the input pointer (writes are then skipped). */
    int64_t   ld_bf16;  /* >= cols, multiple of 8 (ignored when bf16 is NULL) */
    float*    scale;    /* [P] multiplier s of the payload in fp8: q = E4M3(fl32(x * s)); in blocks with
                           mask == 2 the E5M2 scale (from 57344 / amax): q = E5M2(fl32(x * s)) */
    float*    amax;     /* [P] max |x| of the block (a BF16 value widened to float) */
    float*    err_sum;  /* [P] sum over non-zero x of |y - q| / |y|, y = fl32(x * s); a non-zero x
                           whose q is zero contributes 1 */
    uint32_t* nnz;      /* [P] number of non-zero elements (+-0 excluded) */
    uint8_t*  mask;     /* [P] 0 = E4M3, 1 = BF16 */
    float*    err5_sum; /* [P] the same error sum for E5M2 with s5 = fl32(57344 / amax); required
                           for MOR_CRIT_E4M3_VS_E5M2, otherwise ignored and may be NULL */
    uint8_t*  scale_e8m0;     /* [P] MOR_SCALE_GAM / MOR_SCALE_E8M0: biased exponent (bias 127) of scale[p];
                                 optional (NULL = not written); untouched for MOR_SCALE_FP32_AMAX */
    uint32_t* group_mantissa; /* [2 * n_groups] MOR_SCALE_GAM / MOR_SCALE_E8M0 (n_groups = 1 unless gam_group_rows is set):
                                 [2g] the 23 fraction bits of group g's m_g (0 for E8M0-only), so that for a block p of
                                 group g scale[p] == bits((scale_e8m0[p] << 23) | group_mantissa[2g]);
                                 [2g + 1] the same for the E5M2 scales (used by blocks with mask == 2);
                                 optional; untouched for MOR_SCALE_FP32_AMAX */
    float*    amin;     /* [P] three-way recipe: smallest non-zero |x| of blocks that failed M_1 (0 when the block
                           has no non-zero element, and for blocks kept in E4M3); optional */
} mor_outputs;

/* Selection statistics (Section 4.1.3). Lives in DEVICE memory; 8-byte aligned. */
typedef struct mor_stats {
    uint64_t n_part;            /* P */
    uint64_t n_fp8_part;        /* blocks with mask == 0 (E4M3) */
    uint64_t n_bf16_part;       /* blocks with mask == 1 */
    uint64_t n_elem_fp8;        /* elements inside FP8 blocks */
    uint64_t n_elem_bf16;       /* elements inside BF16 blocks */
    uint64_t nnz_total;         /* sum of nnz */
    uint64_t n_near_threshold;  /* blocks with |metric - th| <= near_tol * th */
    double   err_sum_total;     /* sum of err_sum */
    double   mean_err;          /* err_sum_total / nnz_total (0 when nnz_total == 0) */
    uint32_t hist[12];          /* block metrics err_sum/nnz (binary32) in bins [0,0.5%), [0.5%,1%),
                                   ..., [5%,5.5%), [5.5%, inf] */
    uint32_t flags;             /* MOR_STATS_FLAG_* bits; 0 from mor_select_stats */
    uint32_t reserved;
    uint64_t n_e5m2_part;       /* blocks with mask == 2 (three-way recipe) */
    uint64_t n_elem_e5m2;       /* elements inside E5M2 blocks */
} mor_stats;
/* Set by mor_analyze_quantize_batch for a per-tensor operand whose BF16 decision was already proven
 * by the amax pass (enough elements certain to flush to zero), so that the fallback payload was
 * written by the quantize pass and the separate copy pass was skipped.  Informational only: the
 * outputs do not depend on it. */
#define MOR_STATS_FLAG_FUSED_FALLBACK 1u

/* Number of blocks for a shape made of whole blocks, or -1 if the shape is invalid for the granularity. */
int64_t mor_num_partitions(int32_t granularity, int64_t rows, int64_t cols);
/* The same for a parameter set (honours MOR_FLAG_RAGGED). */
int64_t mor_params_num_partitions(const mor_params* params);

/* Bytes of device scratch mor_analyze_quantize needs for these parameters (0 on invalid
 * parameters).  Contents need no initialisation and are meaningless afterwards. */
size_t mor_workspace_bytes(const mor_params* params);

/*
 * Algorithm 2 with [E4M3, BF16] over one operand.
 *   x          device, [rows x ld] BF16 bit patterns, 16-byte aligned, read-only
 *   out        host struct of device pointers, see mor_outputs
 *   workspace  device scratch of at least mor_workspace_bytes(params) bytes, 16-byte aligned;
 *              may be NULL when that size is 0
 * One fused pass for the granularities whose blocks fit a workgroup; per-tensor granularity and
 * per-channel columns need an amax that spans the operand first and therefore read x twice, and so do
 * sub-tensor blocks under GAM scaling (group amax of Algorithm 1).  Concurrent calls must not share a workspace.
 */
mor_status mor_analyze_quantize(const mor_params* params, const uint16_t* x, const mor_outputs* out,
                                void* workspace, size_t workspace_bytes, void* stream);

/*
 * The same call for callers that cannot allocate device memory or pass a workspace: code under HIP graph
 * capture, tight serving loops, harnesses that forbid hipMalloc.  The scratch is a fixed array of
 * MOR_STATIC_SCRATCH_BYTES inside the library's device image (one copy per GPU, held until the process ends);
 * the call allocates and frees nothing.  Parameters whose mor_workspace_bytes() exceeds MOR_STATIC_SCRATCH_BYTES
 * are refused with MOR_ERR_WORKSPACE and nothing is launched (per-tensor operands and tensor-level decisions of
 * any size fit; per-channel columns up to about 2048 x 4096 elements).  Outputs are identical to
 * mor_analyze_quantize.  Every call on one GPU shares that GPU's array: calls whose work overlaps in time on
 * one GPU (different streams, or threads) race; calls on one stream are ordered and safe.  The first call on a
 * device looks the array's address up (hipGetSymbolAddress, no allocation); make that call outside any capture.
 */
#define MOR_STATIC_SCRATCH_BYTES 1048576   /* 1 MiB */
mor_status mor_analyze_quantize_static(const mor_params* params, const uint16_t* x, const mor_outputs* out,
                                       void* stream);

/*
 * Measurement aid: the same call, with the caller's HIP events recorded on `stream` right before
 * and after each kernel it launches, so a benchmark can time individual kernels inside its own
 * timed loop.  `profile` is a HOST struct: the caller fills `capacity` (<= MOR_PROFILE_MAX) and that many
 * created hipEvent_t handles in start[] / stop[]; on return `count` kernels were bracketed and
 * kernel[i] names the i-th one (mor_kernel_id).  Kernels beyond `capacity` run un-bracketed.
 */
typedef enum {
    MOR_KERNEL_SUB_1x128 = 1, MOR_KERNEL_BLOCK_128x128 = 2, MOR_KERNEL_TENSOR_AMAX = 3,
    MOR_KERNEL_TENSOR_QUANT = 4, MOR_KERNEL_TENSOR_FINALIZE = 5, MOR_KERNEL_FALLBACK_COPY = 6,
    MOR_KERNEL_SCOPE_REDUCE = 7, MOR_KERNEL_SCOPE_DECIDE = 8, MOR_KERNEL_SCOPE_FILL_MASK = 9,
    MOR_KERNEL_STATS_PARTIAL = 10, MOR_KERNEL_STATS_FINAL = 11,
    MOR_KERNEL_GROUP_AMAX = 12,      /* amax of the whole operand for GAM scaling of sub-tensor blocks */
    MOR_KERNEL_GROUP_MANTISSA = 13,
    MOR_KERNEL_TEAM_BLOCK = 14,      /* 128x128 blocks, 64x64 blocks, per-channel rows (id 2 is no longer used) */
    MOR_KERNEL_COLUMN_TILE = 15,     /* 128x1 sub-columns; per-channel columns: amax and quantize passes */
    MOR_KERNEL_COLUMN_COMBINE = 16   /* per-channel columns: scales from the amax partials, final decision */
} mor_kernel_id;
#define MOR_PROFILE_MAX 16
typedef struct mor_profile {
    int32_t capacity;
    int32_t count;
    void*   start[MOR_PROFILE_MAX];   /* hipEvent_t */
    void*   stop[MOR_PROFILE_MAX];    /* hipEvent_t */
    int32_t kernel[MOR_PROFILE_MAX];  /* mor_kernel_id */
} mor_profile;
mor_status mor_analyze_quantize_profiled(const mor_params* params, const uint16_t* x, const mor_outputs* out,
                                         void* workspace, size_t workspace_bytes, void* stream,
                                         mor_profile* profile);

/*
 * Many operands in one call.  MoR is applied to every GEMM operand of the four linear layers of each
 * transformer block (Section 4): dozens of calls per layer, each worth only tens of microseconds of HBM
 * time.  The batch entry point groups dense operands of equal granularity and criterion into single
 * launches (descriptor tables travel in the kernel arguments), so launch overhead is paid per group,
 * not per operand.  Results are identical to calling mor_analyze_quantize (and mor_select_stats when
 * `stats` is set) operand by operand, in order, on the same stream.
 *   items      host array; every pointer inside is device memory as for the single-operand calls;
 *              `stats` (optional, device mor_stats*) receives the operand's selection statistics
 *   near_tol   as for mor_select_stats
 *   workspace  device scratch of mor_batch_workspace_bytes(items, n_items) bytes, 16-byte aligned
 *   profile    optional measurement aid as in mor_analyze_quantize_profiled (NULL for none)
 * An item with fake_y set is fake-quantized into fake_y (leading dimension ld_fake_y) as by
 * mor_fake_quantize; its out.fp8 and out.bf16 are then ignored.
 * n_items must be in [1, MOR_BATCH_MAX].  Operands must not overlap each other's outputs.
 */
#define MOR_BATCH_MAX 64
typedef struct mor_batch_item {
    mor_params      params;
    const uint16_t* x;
    mor_outputs     out;
    mor_stats*      stats;
    uint16_t*       fake_y;      /* NULL: FP8 payload + BF16 fallback; else the fake-quantized tensor */
    int64_t         ld_fake_y;
} mor_batch_item;
size_t     mor_batch_workspace_bytes(const mor_batch_item* items, int32_t n_items);
mor_status mor_analyze_quantize_batch(const mor_batch_item* items, int32_t n_items, float near_tol,
                                      void* workspace, size_t workspace_bytes, void* stream,
                                      mor_profile* profile);

/*
 * Inverse path (the de-quantize / de-scale half of the fake-quantization workflow, Section 4,
 * Figure 4): y = bf16_rne(fl32(E4M3value(fp8) * fl32(1 / scale[p]))) in blocks with mask 0,
 * the same with the E5M2 value of the code in blocks with mask 2,
 * y = bf16 fallback bits in blocks with mask 1.  `bf16` may be NULL; blocks with mask 1 are then
 * left untouched in y.
 * Uses rows, cols, granularity and flags of params; params->ld is ignored.
 */
mor_status mor_dequantize(const mor_params* params, const uint8_t* fp8, int64_t ld_fp8,
                          const float* scale, const uint8_t* mask,
                          const uint16_t* bf16, int64_t ld_bf16,
                          uint16_t* y, int64_t ld_y, void* stream);

/*
 * The same from the stored form of GAM / E8M0 scaling (Algorithm 1 and the paragraph before it: the
 * per-block scale is rebuilt on the fly from the shared 23-bit group mantissa and the block's 8-bit
 * exponent): scale[p] = bits((scale_e8m0[p] << 23) | group_mantissa[2g]) for a block of group g, with
 * group_mantissa[2g + 1] in blocks with mask 2.  scale_e8m0 [P] and group_mantissa [2 * n_groups] are device
 * arrays as written by mor_analyze_quantize with the same params (gam_group_rows included).
 */
mor_status mor_dequantize_e8m0(const mor_params* params, const uint8_t* fp8, int64_t ld_fp8,
                               const uint8_t* scale_e8m0, const uint32_t* group_mantissa, const uint8_t* mask,
                               const uint16_t* bf16, int64_t ld_bf16,
                               uint16_t* y, int64_t ld_y, void* stream);

/*
 * Many operands in one call (e.g. every operand of a layer before a BF16 GEMM): the operands share kernel launches.
 * Each item is de-quantized as by mor_dequantize (scale != NULL) or mor_dequantize_e8m0 (scale == NULL, scale_e8m0 and
 * group_mantissa set).  n_items must be in [1, MOR_BATCH_MAX].
 */
typedef struct mor_dequant_item {
    mor_params      params;          /* rows, cols, granularity, flags are used */
    const uint8_t*  fp8;   int64_t ld_fp8;
    const float*    scale;           /* [P], or NULL for the stored GAM / E8M0 form */
    const uint8_t*  scale_e8m0;      /* [P] when scale == NULL */
    const uint32_t* group_mantissa;  /* [2 * n_groups] when scale == NULL */
    const uint8_t*  mask;            /* [P] */
    const uint16_t* bf16;  int64_t ld_bf16;   /* fallback payload, may be NULL */
    uint16_t*       y;     int64_t ld_y;
} mor_dequant_item;
mor_status mor_dequantize_batch(const mor_dequant_item* items, int32_t n_items, void* stream);

/*
 * Fake quantization (Section 4, Figure 4), the form in which the paper's training runs applied MoR:
 * y = de-quantize(quantize(x)) in one call, BF16 in and BF16 out.  Blocks kept in E4M3 (or E5M2) carry
 * the information loss of that format, y = bf16_rne(fl32(value(code) * fl32(1 / scale[p]))); blocks kept
 * in BF16 are copied unchanged.  The FP8 payload itself is not materialised: meta->fp8 and meta->bf16
 * are ignored (may be NULL); the [P] arrays of `meta` are written as by mor_analyze_quantize.
 *   y          device, [rows x ld_y] BF16 bit patterns, 16-byte aligned, ld_y >= cols, ld_y % 8 == 0;
 *              must not overlap x
 *   workspace  device scratch of at least mor_workspace_bytes(params) bytes
 * Equivalent to mor_analyze_quantize followed by mor_dequantize, with 2 bytes read and 2 written per
 * element (per-tensor granularity: 4 read) instead of 2 + 1 (+ 2) written and 1 (+ 2) + 2 read again.
 */
mor_status mor_fake_quantize(const mor_params* params, const uint16_t* x, uint16_t* y, int64_t ld_y,
                             const mor_outputs* meta, void* workspace, size_t workspace_bytes, void* stream);

/*
 * Selection statistics of one analysed operand (Section 4.1.3): counts of blocks and elements
 * per chosen type, aggregate error, 0.5 %-bin histogram of the block metrics, and the number of
 * blocks within near_tol * threshold of the threshold.  err_sum, nnz, mask are the [P] arrays
 * mor_analyze_quantize wrote; out_dev is a device mor_stats, fully overwritten.
 */
mor_status mor_select_stats(const mor_params* params, const float* err_sum, const uint32_t* nnz,
                            const uint8_t* mask, float near_tol, mor_stats* out_dev, void* stream);

/*
 * Running histogram of one tensor's relative error over training steps (Section 4.1.3, the paragraphs
 * on the heat maps): every mini-batch adds ONE count to the 0.5 %-wide bin (last bin open from 5.5 %)
 * that holds the tensor's error of that step, and the histogram is cleared every reset_interval steps
 * (6000 in the paper) before the step's count is added.
 *   hist12_dev      device uint32[12], updated in place (not atomically: one call at a time per histogram)
 *   stats_dev       device mor_stats of this step's call for the tensor; the tensor's error is
 *                   (float)stats_dev->mean_err = sum(err_sum) / sum(nnz)
 *   step            step counter from 0; step % reset_interval == 0 clears first
 *   reset_interval  > 0, or 0 to never clear
 */
mor_status mor_histogram_update(uint32_t* hist12_dev, const mor_stats* stats_dev, int64_t step,
                                int64_t reset_interval, void* stream);

const char* mor_status_string(mor_status status);

#ifdef __cplusplus
}
#endif
#endif /* MOR_H_ */
