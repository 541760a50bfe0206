/*
 * mor_oracle.c -- TEST INFRASTRUCTURE ONLY.
 *
 * A plain, slow, obviously-correct CPU implementation of what the MoR
 * analyse-select-quantize path computes, written from the paper's definitions.
 * It exists so that the HIP kernels can be checked against something that was
 * not derived from them.  It shares no code, header, table or constant
 * generator with the HIP path, and nothing in the product path may call it.
 * Only tests/, __graft_entry__.smoke() and bench.py's cpu_baseline leg use it.
 *
 * What follows the paper, passage by passage:
 *   - partitioning of X into blocks B (per tensor, 2-D block, sub-channel):
 *     Section 3, first paragraph;
 *   - amax = max(abs(b)) and scale = q_amax / amax: Algorithm 1, the two
 *     assignments at the top of the group loop and of the block loop, used
 *     here in their plain form, one binary32 scale per block straight from
 *     its amax (the first scaling variant of the ablation in Section 4.1.2);
 *   - E4M3 / E5M2 value sets, saturation and underflow: Section 1 (format
 *     widths) and Section 2, first paragraph (ranges 2^-9..448, 2^-16..57344,
 *     clipping large values, flushing small ones to zero);
 *   - mean relative error over non-zero elements, strict "<" against the
 *     threshold: Eq. (1)-(2);
 *   - local errors aggregated into one global error and one tensor-wide
 *     decision: Section 3.1, the paragraph on Figure 2;
 *   - total relative error of E4M3 strictly below that of E5M2, else BF16
 *     (E5M2 is a yardstick only): Eq. (3) and the two-way paragraph of
 *     Section 3.2;
 *   - first accepted type wins, last type unconditional: Algorithm 2;
 *   - BF16 = leave the block in its original precision: Section 3;
 *   - dequantize and de-scale back to the original range: Section 4, the
 *     fake-quantization paragraph (Figure 4);
 *   - 0.5 %-wide histogram bins, last bin open-ended from 5.5 %: Section 4.1.3;
 *   - group amax mantissa scaling, exponent lowered by one when m_g > m_b:
 *     Algorithm 1; global mantissa from the global amax before the blocks are
 *     quantized: Section 3.1, the paragraph on Figure 2.
 *
 * Readings taken where the paper is silent (each is also listed in the design
 * notes of the repository):
 *   R1  amax is the integer maximum of (bits & 0x7FFF) over BF16 bit patterns.
 *   R2  scale s = fl32(q_amax / amax), a multiplier; amax == 0 -> s = 1;
 *       quotient overflowing to +inf -> s = FLT_MAX; non-finite amax -> s = 1.
 *   R3  OCP E4M3 (no infinities, 0x7F/0xFF = NaN, bias 7) and E5M2 (bias 15),
 *       round to nearest, ties to the even code, magnitudes above the largest
 *       finite value clip to it, sign always kept, NaN -> 0x7F | sign.
 *   R4  tensor-wide error = sum of block error sums / sum of block non-zero
 *       counts (Eq. (2) taken over the whole tensor).
 *   R5  Q(x) in Eq. (2) is the de-scaled FP8 value without re-rounding to BF16.
 *   R6  the scaled value is y = fl32(x * s) (one binary32 multiply); the error
 *       term is |y - q| / |y| evaluated in binary64.  The unscaled-domain form
 *       |x - q/s| / |x| is also produced so tests can show the two agree.
 *   R7  a non-zero x whose quantized value is zero contributes exactly 1;
 *       a block without non-zero elements has metric 0.
 *   R8  Eq. (3) is strict: a tie selects BF16.
 *   R9  a block holding Inf or NaN: amax = that pattern, s = 1, codes by R3,
 *       error sums = +inf, selection = BF16.
 *   R10 de-scaling multiplies by s_inv = fl32(1 / s), then rounds to BF16 RNE
 *       (the paper only says the values are de-scaled to their original range;
 *       a division by s would round differently on some elements).
 *   R4b the tensor-wide decision under Eq. (3) compares the two totals,
 *       sum of block err_sum < sum of block err5_sum.  This is an extension:
 *       the paper states Eq. (3) per block (Section 3.2) and the aggregation
 *       of local errors for Eq. (2) only (Section 3.1).
 *   R16 GAM (Algorithm 1) is run with one group = the whole tensor, the
 *       configuration of the paper's experiments (Section 2, the paragraph
 *       after the algorithm's description), or, on request, with the groups
 *       of G taken as bands of `group_rows` consecutive rows (whole blocks
 *       each; the last band may be shorter): Algorithm 1 leaves G open.  mantissa(s) and exponent(s) are
 *       those of the binary32 number s = m * 2^e, 1 <= m < 2.  The scale that
 *       is applied is m_g * 2^e, exact in binary32.  The stored E8M0 code is
 *       e + 127, the stored group mantissa the 23 fraction bits of m_g.
 *   R17 "E8M0 per-block scaling" (Section 4.1.2, third ablation) is the power
 *       of two 2^exponent(s_b), i.e. Algorithm 1 with m_g = 1: the largest
 *       power of two that cannot saturate.
 *   R18 s_g and s_b in Algorithm 1 follow R2 (zero / non-finite amax -> 1,
 *       overflow -> FLT_MAX) before mantissa and exponent are taken.
 *   R19 three-way selection [E4M3, E5M2, BF16] (Section 3.2, first recipe): M_1 is
 *       the chosen criterion (the paper uses Eq. (3)); M_2 is Eq. (4),
 *       max|b| / min|b| < 57344 / 2^-14, with the minimum taken over the NON-ZERO
 *       elements (every metric of the paper excludes zeros; a zero would make the
 *       ratio infinite for any block that holds one).  A block without non-zero
 *       elements passes M_2 (there is no range to cover).  The ratio test is
 *       evaluated exactly as amax < 57344 * 2^14 * amin.  An E5M2 block is
 *       quantized with the E5M2 scale (q_amax = 57344); its scale / E8M0 outputs
 *       are those of that scale.  A block holding Inf or NaN fails M_2 (R9).
 *   R20 further partitions: per-channel rows (1 x cols) and columns (rows x 1)
 *       (Section 3, first paragraph; Section 4.1.1), column sub-channels 128 x 1
 *       (the "sub-columns" of Section 3 / the transposed operands of Section 4),
 *       64 x 64 blocks (Section 4.1.2, first ablation).  Ragged edges, on which
 *       the paper is silent: the grid is ceil(rows/pr) x ceil(cols/pc) and the
 *       last block of a row / column of the grid is simply smaller.
 *   R21 fake quantization (Section 4, Figure 4) is de-quantize(quantize(x)):
 *       BF16 in, BF16 out; blocks kept in BF16 pass through unchanged.
 *
 * parity unpinned: R8 (tie handling), R9 (non-finite policy), R10 (product with
 * the rounded reciprocal rather than a quotient), R4b (Eq. (3) over a whole
 * tensor), R17 (which power of two the E8M0 ablation uses), R19 (zeros in the
 * minimum of Eq. (4)) and R20 (ragged edges) are fixed by these readings only;
 * nothing in the paper pins the CHOICE.  The arithmetic of each reading is
 * pinned by the CPU tests (exact-rational model, hand-worked blocks).
 */
#include <float.h>
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>

#ifdef _OPENMP
#include <omp.h>
#endif

/* ------------------------------------------------------------------ formats */

static float bits_to_f32(uint32_t u) { float f; memcpy(&f, &u, 4); return f; }
static uint32_t f32_to_bits(float f) { uint32_t u; memcpy(&u, &f, 4); return u; }

/* BF16 is the upper half of a binary32: widening is exact. */
static float bf16_to_f32(uint16_t b) { return bits_to_f32((uint32_t)b << 16); }

/* Value of an FP8 code from the format definition.  ebits/mbits = 4/3 (E4M3,
 * bias 7, no infinities, S.1111.111 = NaN) or 5/2 (E5M2, bias 15, IEEE-like
 * infinities and NaNs).  Returns NaN / +-inf as doubles where the code says so. */
static double fp8_value(unsigned code, int ebits, int mbits)
{
    int bias = (1 << (ebits - 1)) - 1;
    unsigned sign = (code >> 7) & 1u;
    unsigned e = (code >> mbits) & ((1u << ebits) - 1u);
    unsigned m = code & ((1u << mbits) - 1u);
    double mag;
    if (ebits == 4) {
        if (e == 15u && m == 7u) return NAN;
    } else {
        if (e == 31u) return m ? NAN : (sign ? -INFINITY : INFINITY);
    }
    if (e == 0u)
        mag = ldexp((double)m, 1 - bias - mbits);              /* subnormal: m * 2^(1-bias-mbits) */
    else
        mag = ldexp(1.0 + ldexp((double)m, -mbits), (int)e - bias);
    return sign ? -mag : mag;
}

static unsigned fp8_max_finite_code(int ebits) { return ebits == 4 ? 0x7Eu : 0x7Bu; }

/* Round-to-nearest, ties-to-even-code, clipping encoder, written as a search
 * over the decoded non-negative finite values (they increase with the code). */
static uint8_t fp8_encode(float y, int ebits, int mbits)
{
    unsigned sign = (f32_to_bits(y) >> 31) << 7;
    unsigned top = fp8_max_finite_code(ebits);
    double a;
    unsigned lo, hi;
    if (isnan(y)) return (uint8_t)(sign | 0x7Fu);
    a = fabs((double)y);
    if (a >= fp8_value(top, ebits, mbits)) return (uint8_t)(sign | top);   /* clip (also Inf) */
    /* largest code lo with value(lo) <= a; value(0) = 0 <= a always */
    lo = 0; hi = top;
    while (hi - lo > 1u) {
        unsigned mid = (lo + hi) / 2u;
        if (fp8_value(mid, ebits, mbits) <= a) lo = mid; else hi = mid;
    }
    {
        double dlo = a - fp8_value(lo, ebits, mbits);
        double dhi = fp8_value(hi, ebits, mbits) - a;
        unsigned pick;
        if (dlo < dhi) pick = lo;
        else if (dhi < dlo) pick = hi;
        else pick = (lo & 1u) ? hi : lo;                       /* tie: even code */
        return (uint8_t)(sign | pick);
    }
}

uint8_t mor_oracle_e4m3_encode(float y) { return fp8_encode(y, 4, 3); }
uint8_t mor_oracle_e5m2_encode(float y) { return fp8_encode(y, 5, 2); }
double  mor_oracle_e4m3_decode(uint8_t c) { return fp8_value(c, 4, 3); }
double  mor_oracle_e5m2_decode(uint8_t c) { return fp8_value(c, 5, 2); }

/* binary32 -> BF16, round to nearest even; NaN -> quiet NaN with the sign kept. */
uint16_t mor_oracle_f32_to_bf16(float f)
{
    uint32_t u = f32_to_bits(f);
    if ((u & 0x7FFFFFFFu) > 0x7F800000u) return (uint16_t)(((u >> 16) & 0x8000u) | 0x7FC0u);
    u += 0x7FFFu + ((u >> 16) & 1u);
    return (uint16_t)(u >> 16);
}

/* R2: the FP32 scale of a block from its amax. */
float mor_oracle_scale(float amax, float q_amax)
{
    volatile float s;
    if (!(amax < INFINITY)) return 1.0f;       /* Inf or NaN */
    if (amax == 0.0f) return 1.0f;
    s = q_amax / amax;                          /* one correctly rounded binary32 division */
    if (isinf(s)) return FLT_MAX;
    return s;
}

/* --------------------------------------------------- Algorithm 1 (GAM, R16-R18) */

enum { SCALING_FP32_AMAX = 0, SCALING_GAM = 1, SCALING_E8M0 = 2 };

/* s = m * 2^e with 1 <= m < 2, for a positive finite s. */
static void mantissa_exponent(float s, double *m, int *e)
{
    int k;
    double f = frexp((double)s, &k);     /* s = f * 2^k, 0.5 <= f < 1 */
    *m = 2.0 * f;
    *e = k - 1;
}

/* m_g of Algorithm 1 for a group whose amax is g_amax (1.0 for E8M0-only scaling, R17). */
double mor_oracle_group_mantissa(float g_amax, float q_amax, int scaling)
{
    double m_g;
    int e_g;
    if (scaling != SCALING_GAM) return 1.0;
    mantissa_exponent(mor_oracle_scale(g_amax, q_amax), &m_g, &e_g);
    return m_g;
}

/* The block loop of Algorithm 1: exponent of s_b, one lower when m_g > m_b.
 * Returns the scale that is applied, m_g * 2^e; *e_out receives e. */
float mor_oracle_gam_block_scale(float b_amax, float q_amax, double m_g, int *e_out)
{
    double m_b;
    int e;
    mantissa_exponent(mor_oracle_scale(b_amax, q_amax), &m_b, &e);
    if (!(m_g <= m_b)) e = e - 1;
    if (e_out) *e_out = e;
    return (float)ldexp(m_g, e);          /* 24 significant bits, normal range: exact */
}

/* ------------------------------------------------------------ partitioning */

enum { GRAN_TENSOR = 0, GRAN_SUB_1x128 = 1, GRAN_BLOCK_128x128 = 2, GRAN_CHANNEL_ROW = 3,
       GRAN_CHANNEL_COL = 4, GRAN_SUB_128x1 = 5, GRAN_BLOCK_64x64 = 6 };
enum { FMT_E4M3 = 1, FMT_E5M2 = 2, FMT_BF16 = 4 };
enum { CRIT_MEAN_REL_ERR = 0, CRIT_E4M3_VS_E5M2 = 1 };
enum { SCOPE_PARTITION = 0, SCOPE_TENSOR = 1 };

/* Nominal block shape pr x pc of a partition (Section 3, first paragraph; R20).  With
 * ragged == 0 the tensor must be a whole number of blocks, otherwise edge blocks are smaller. */
static int part_shape_ex(int gran, int64_t rows, int64_t cols, int ragged, int64_t *pr, int64_t *pc)
{
    switch (gran) {
    case GRAN_TENSOR:        *pr = rows; *pc = cols; break;
    case GRAN_SUB_1x128:     *pr = 1;    *pc = 128;  break;
    case GRAN_BLOCK_128x128: *pr = 128;  *pc = 128;  break;
    case GRAN_CHANNEL_ROW:   *pr = 1;    *pc = cols; break;
    case GRAN_CHANNEL_COL:   *pr = rows; *pc = 1;    break;
    case GRAN_SUB_128x1:     *pr = 128;  *pc = 1;    break;
    case GRAN_BLOCK_64x64:   *pr = 64;   *pc = 64;   break;
    default: return -1;
    }
    if (!ragged && (rows % *pr || cols % *pc)) return -1;
    return 0;
}

int64_t mor_oracle_num_partitions_ex(int gran, int64_t rows, int64_t cols, int ragged)
{
    int64_t pr, pc;
    if (rows <= 0 || cols <= 0 || part_shape_ex(gran, rows, cols, ragged, &pr, &pc)) return -1;
    return ((rows + pr - 1) / pr) * ((cols + pc - 1) / pc);
}
int64_t mor_oracle_num_partitions(int gran, int64_t rows, int64_t cols)
{
    return mor_oracle_num_partitions_ex(gran, rows, cols, 0);
}

/* --------------------------------------------------- one block of the tensor */

typedef struct {
    float  amax, amin, scale, scale5;
    double err_sum, err5_sum, err_sum_unscaled;
    uint32_t nnz;
    int    e8m0, e8m0_5;    /* biased exponents of the E4M3 / E5M2 scales (GAM / E8M0 scaling), else 0 */
    int    nonfinite;
} block_result;

/* Error sums of one block for one FP8 format; optionally writes the codes. */
static double block_error(const uint16_t *x, int64_t ld, int64_t pr, int64_t pc, float s,
                          int ebits, int mbits, int nonfinite,
                          uint8_t *codes, int64_t ld_codes, double *unscaled_out)
{
    double sum = 0.0, sum_u = 0.0;
    /* rows of one large block (per-tensor granularity) are spread over threads; for small
     * blocks the caller already runs one block per thread and this region stays serial */
#pragma omp parallel for reduction(+ : sum, sum_u) schedule(static) if (pr * pc >= 65536)
    for (int64_t r = 0; r < pr; ++r) {
        for (int64_t c = 0; c < pc; ++c) {
            uint16_t b = x[r * ld + c];
            float xf = bf16_to_f32(b);
            volatile float y = xf * s;                     /* R6: one binary32 multiply */
            uint8_t code = fp8_encode(y, ebits, mbits);
            if (codes) codes[r * ld_codes + c] = code;
            if ((b & 0x7FFFu) == 0u) continue;             /* Eq. (1): non-zero elements only */
            if (nonfinite) continue;                        /* R9: sums forced to +inf below */
            {
                double qv = fp8_value(code, ebits, mbits);
                double yd = (double)y;
                if (qv == 0.0) {                            /* R7: flushed */
                    sum += 1.0;
                    sum_u += 1.0;
                } else {
                    sum += fabs(yd - qv) / fabs(yd);
                    sum_u += fabs((double)xf - qv / (double)s) / fabs((double)xf);
                }
            }
        }
    }
    if (nonfinite) { sum = INFINITY; sum_u = INFINITY; }
    if (unscaled_out) *unscaled_out = sum_u;
    return sum;
}

/* amax, smallest non-zero magnitude, non-zero count, the scales of Algorithm 1 for both FP8
 * formats, the E4M3 codes and error sum, and (want5) the E5M2 error sum of one block. */
static void analyze_block(const uint16_t *x, int64_t ld, int64_t pr, int64_t pc, int want5,
                          int scaling, double m_g, double m_g5,
                          uint8_t *codes, int64_t ld_codes, block_result *out)
{
    uint16_t a = 0, lo = 0;
    uint32_t nnz = 0;
    for (int64_t r = 0; r < pr; ++r)
        for (int64_t c = 0; c < pc; ++c) {
            uint16_t m = (uint16_t)(x[r * ld + c] & 0x7FFFu);
            if (m > a) a = m;                               /* R1 */
            if (m) { ++nnz; if (lo == 0 || m < lo) lo = m; }
        }
    out->nonfinite = a >= 0x7F80u;
    out->amax = bf16_to_f32(a);
    out->amin = bf16_to_f32(lo);
    out->nnz = nnz;
    out->e8m0 = 0; out->e8m0_5 = 0;
    if (scaling == SCALING_FP32_AMAX) {
        out->scale = mor_oracle_scale(out->amax, 448.0f);
        out->scale5 = mor_oracle_scale(out->amax, 57344.0f);
    } else {
        int e;
        out->scale = mor_oracle_gam_block_scale(out->amax, 448.0f, m_g, &e);
        out->e8m0 = e + 127;
        out->scale5 = mor_oracle_gam_block_scale(out->amax, 57344.0f, m_g5, &e);
        out->e8m0_5 = e + 127;
    }
    out->err_sum = block_error(x, ld, pr, pc, out->scale, 4, 3, out->nonfinite, codes, ld_codes,
                               &out->err_sum_unscaled);
    out->err5_sum = want5 ? block_error(x, ld, pr, pc, out->scale5, 5, 2, out->nonfinite, NULL, 0, NULL) : 0.0;
}

/* M_1 of Algorithm 2 for E4M3: 1 = accept. */
static int accept_e4m3(int crit, double err_sum, double err5_sum, uint64_t nnz, float threshold)
{
    if (crit == CRIT_E4M3_VS_E5M2) return err_sum < err5_sum;             /* Eq. (3), R8 */
    {
        double metric = nnz ? err_sum / (double)nnz : 0.0;                /* Eq. (1)-(2), R7 */
        return metric < (double)threshold;
    }
}

/* M_2 of the three-way recipe, Eq. (4), R19: the block's dynamic range fits E5M2's normal range. */
static int accept_e5m2(float amax, float amin, uint32_t nnz, int nonfinite)
{
    if (nonfinite) return 0;
    if (nnz == 0) return 1;
    return (double)amax < 57344.0 * 16384.0 * (double)amin;   /* exact: both are BF16 values */
}

/* -------------------------------------------------------------- entry points */

typedef struct {
    int64_t  rows, cols, ld;
    int32_t  gran, scope, crit, scaling;
    uint32_t formats;       /* FMT_E4M3 | FMT_BF16, or FMT_E4M3 | FMT_E5M2 | FMT_BF16 (three-way) */
    int32_t  ragged;        /* 1: edge blocks may be smaller than the nominal block (R20) */
    float    threshold;
    int32_t  group_rows;    /* GAM: 0 = one group (the whole tensor); else the groups of Algorithm 1 are bands of this many rows */
} oracle_params;

typedef struct {
    uint8_t  *fp8;          /* [rows x cols] dense: E4M3 codes; E5M2 codes in blocks with mask == 2 */
    uint16_t *bf16;         /* [rows x cols] dense; written only where mask == 1; may be NULL */
    float    *scale;        /* [P] scale of the payload in fp8 (E5M2 scale where mask == 2) */
    float    *amax;         /* [P] */
    double   *err_sum;      /* [P] */
    uint32_t *nnz;          /* [P] */
    uint8_t  *mask;         /* [P] 0 = E4M3, 1 = BF16, 2 = E5M2 */
    double   *err5_sum;     /* [P] or NULL */
    double   *err_sum_unscaled; /* [P] or NULL */
    uint8_t  *e8m0;         /* [P] or NULL (GAM / E8M0 scaling) */
    uint32_t *group_mantissa;   /* [n_groups][2] or NULL: fraction bits of m_g for E4M3 and for E5M2, group by group */
    float    *amin;         /* [P] or NULL: smallest non-zero magnitude (0 when there is none) */
    uint16_t *fake;         /* [rows x cols] or NULL: fake-quantized tensor (R21) */
} oracle_out;

/*
 * Full analyse-select-quantize of one operand (Algorithm 2; scales by Algorithm 1).
 * Blocks are numbered row-major over the block grid.  Returns 0, or -1 on bad arguments.
 */
int mor_oracle_run(const oracle_params *pp, const uint16_t *x, const oracle_out *o)
{
    const int64_t rows = pp->rows, cols = pp->cols, ld = pp->ld;
    const int three = pp->formats == (FMT_E4M3 | FMT_E5M2 | FMT_BF16);
    const int want5 = pp->crit == CRIT_E4M3_VS_E5M2;
    int64_t pr, pc, gr, gc, P;
    int64_t band, n_groups;
    double *m_g, *m_g5;
    float *scale5;
    uint8_t *e8m0_5;
    if (rows <= 0 || cols <= 0 || ld < cols || part_shape_ex(pp->gran, rows, cols, pp->ragged, &pr, &pc)) return -1;
    /* groups of Algorithm 1: bands of whole blocks (a block never straddles two groups) */
    if (pp->group_rows < 0) return -1;
    band = pp->group_rows > 0 && pp->scaling == SCALING_GAM ? pp->group_rows : rows;
    if (band >= rows) band = rows;                           /* one group */
    else if (band % pr) return -1;
    n_groups = (rows + band - 1) / band;
    if (pp->scaling < SCALING_FP32_AMAX || pp->scaling > SCALING_E8M0) return -1;
    if (!three && pp->formats != (FMT_E4M3 | FMT_BF16)) return -1;
    if (three && pp->scope != SCOPE_PARTITION) return -1;     /* the paper's three-way recipe is per block */
    if (want5 && !o->err5_sum) return -1;
    gr = (rows + pr - 1) / pr; gc = (cols + pc - 1) / pc; P = gr * gc;
    scale5 = (float *)malloc(sizeof(float) * (size_t)P);
    e8m0_5 = (uint8_t *)malloc((size_t)P);
    m_g = (double *)malloc(sizeof(double) * (size_t)n_groups);
    m_g5 = (double *)malloc(sizeof(double) * (size_t)n_groups);
    if (!scale5 || !e8m0_5 || !m_g || !m_g5) { free(scale5); free(e8m0_5); free(m_g); free(m_g5); return -1; }

    for (int64_t gi = 0; gi < n_groups; ++gi) {           /* the group loop of Algorithm 1 */
        m_g[gi] = 1.0; m_g5[gi] = 1.0;
        if (pp->scaling == SCALING_GAM) {
            uint16_t g = 0;
            float g_amax;
            int64_t r_end = (gi + 1) * band < rows ? (gi + 1) * band : rows;
            for (int64_t r = gi * band; r < r_end; ++r)
                for (int64_t c = 0; c < cols; ++c) {
                    uint16_t m = (uint16_t)(x[r * ld + c] & 0x7FFFu);
                    if (m > g) g = m;
                }
            g_amax = bf16_to_f32(g);
            m_g[gi] = mor_oracle_group_mantissa(g_amax, 448.0f, pp->scaling);
            m_g5[gi] = mor_oracle_group_mantissa(g_amax, 57344.0f, pp->scaling);
        }
        if (o->group_mantissa) {
            o->group_mantissa[2 * gi] = (uint32_t)ldexp(m_g[gi] - 1.0, 23);
            o->group_mantissa[2 * gi + 1] = (uint32_t)ldexp(m_g5[gi] - 1.0, 23);
        }
    }

#pragma omp parallel for schedule(dynamic, 16) if (P > 1)
    for (int64_t p = 0; p < P; ++p) {
        int64_t br = p / gc, bc = p % gc;
        int64_t r0 = br * pr, c0 = bc * pc;
        int64_t h = rows - r0 < pr ? rows - r0 : pr, w = cols - c0 < pc ? cols - c0 : pc;
        block_result res;
        analyze_block(x + r0 * ld + c0, ld, h, w, want5, pp->scaling, m_g[r0 / band], m_g5[r0 / band],
                      o->fp8 + r0 * cols + c0, cols, &res);
        if (o->e8m0) o->e8m0[p] = (uint8_t)res.e8m0;
        e8m0_5[p] = (uint8_t)res.e8m0_5; scale5[p] = res.scale5;
        o->scale[p] = res.scale; o->amax[p] = res.amax; o->err_sum[p] = res.err_sum; o->nnz[p] = res.nnz;
        if (o->amin) o->amin[p] = res.amin;
        if (o->err5_sum) o->err5_sum[p] = res.err5_sum;
        if (o->err_sum_unscaled) o->err_sum_unscaled[p] = res.err_sum_unscaled;
        /* Algorithm 2: the first accepted type wins, the last type is unconditional */
        if (accept_e4m3(pp->crit, res.err_sum, res.err5_sum, res.nnz, pp->threshold)) o->mask[p] = 0;
        else if (three && accept_e5m2(res.amax, res.amin, res.nnz, res.nonfinite)) o->mask[p] = 2;
        else o->mask[p] = 1;
    }

    if (pp->scope == SCOPE_TENSOR) {                        /* R4: one decision for the tensor */
        double tot = 0.0, tot5 = 0.0;
        uint64_t n = 0;
        uint8_t m;
        for (int64_t p = 0; p < P; ++p) {
            tot += o->err_sum[p]; n += o->nnz[p];
            if (want5) tot5 += o->err5_sum[p];
        }
        m = accept_e4m3(pp->crit, tot, tot5, n, pp->threshold) ? 0 : 1;
        for (int64_t p = 0; p < P; ++p) o->mask[p] = m;
    }

    /* emit: E5M2 payload and scale where E5M2 was chosen, original bits where BF16 was chosen */
#pragma omp parallel for schedule(dynamic, 16) if (P > 1)
    for (int64_t p = 0; p < P; ++p) {
        int64_t br = p / gc, bc = p % gc;
        int64_t r0 = br * pr, c0 = bc * pc;
        int64_t h = rows - r0 < pr ? rows - r0 : pr, w = cols - c0 < pc ? cols - c0 : pc;
        if (o->mask[p] == 2) {
            (void)block_error(x + r0 * ld + c0, ld, h, w, scale5[p], 5, 2, 0, o->fp8 + r0 * cols + c0, cols, NULL);
            o->scale[p] = scale5[p];
            if (o->e8m0) o->e8m0[p] = e8m0_5[p];
        }
        if (o->mask[p] == 1 && o->bf16)
            for (int64_t r = 0; r < h; ++r)
                memcpy(o->bf16 + (r0 + r) * cols + c0, x + (r0 + r) * ld + c0, (size_t)w * 2);
        if (o->fake) {                                      /* R21, R10 */
            volatile float s_inv = 1.0f / o->scale[p];
            for (int64_t r = 0; r < h; ++r)
                for (int64_t c = 0; c < w; ++c) {
                    int64_t i = (r0 + r) * cols + c0 + c;
                    if (o->mask[p] == 1) { o->fake[i] = x[(r0 + r) * ld + c0 + c]; continue; }
                    {
                        float q = (float)(o->mask[p] == 2 ? fp8_value(o->fp8[i], 5, 2) : fp8_value(o->fp8[i], 4, 3));
                        volatile float v = q * s_inv;
                        o->fake[i] = mor_oracle_f32_to_bf16(v);
                    }
                }
        }
    }
    free(scale5); free(e8m0_5); free(m_g); free(m_g5);
    return 0;
}

/* Two-way recipe with a choice of scaling algorithm: 0 = FP32 amax, 1 = GAM (Algorithm 1, one
 * group), 2 = E8M0 only.  group_mantissa [1] receives the 23 fraction bits of m_g. */
int mor_oracle_analyze_quantize_ex(const uint16_t *x, int64_t rows, int64_t cols, int64_t ld,
                                   int gran, int scope, int crit, int scaling, float threshold,
                                   uint8_t *fp8, uint16_t *bf16,
                                   float *scale, float *amax, double *err_sum, uint32_t *nnz,
                                   uint8_t *mask, double *err5_sum, double *err_sum_unscaled,
                                   uint8_t *e8m0, uint32_t *group_mantissa)
{
    oracle_params pp = { rows, cols, ld, gran, scope, crit, scaling, FMT_E4M3 | FMT_BF16, 0, threshold, 0 };
    uint32_t gm[2] = { 0u, 0u };
    oracle_out o = { fp8, bf16, scale, amax, err_sum, nnz, mask, err5_sum, err_sum_unscaled, e8m0, gm, NULL, NULL };
    int rc = mor_oracle_run(&pp, x, &o);
    if (group_mantissa) *group_mantissa = gm[0];
    return rc;
}

/* FP32 amax scaling (the hot path's default). */
int mor_oracle_analyze_quantize(const uint16_t *x, int64_t rows, int64_t cols, int64_t ld,
                                int gran, int scope, int crit, float threshold,
                                uint8_t *fp8, uint16_t *bf16,
                                float *scale, float *amax, double *err_sum, uint32_t *nnz,
                                uint8_t *mask, double *err5_sum, double *err_sum_unscaled)
{
    return mor_oracle_analyze_quantize_ex(x, rows, cols, ld, gran, scope, crit, SCALING_FP32_AMAX,
                                          threshold, fp8, bf16, scale, amax, err_sum, nnz, mask,
                                          err5_sum, err_sum_unscaled, NULL, NULL);
}

/*
 * De-quantize: E4M3 blocks -> bf16_rne(fl32(q * s_inv)), s_inv = fl32(1 / s) (R10); E5M2 blocks
 * (mask 2) the same with the E5M2 value of the code; BF16 blocks -> the fallback bits verbatim.
 * All arrays dense (leading dimension cols).
 */
int mor_oracle_dequantize_ex(const uint8_t *fp8, const float *scale, const uint8_t *mask,
                             const uint16_t *bf16, int64_t rows, int64_t cols, int gran, int ragged,
                             uint16_t *y)
{
    int64_t pr, pc, gr, gc, P;
    if (rows <= 0 || cols <= 0 || part_shape_ex(gran, rows, cols, ragged, &pr, &pc)) return -1;
    gr = (rows + pr - 1) / pr; gc = (cols + pc - 1) / pc; P = gr * gc;
#pragma omp parallel for schedule(dynamic, 16)
    for (int64_t p = 0; p < P; ++p) {
        int64_t br = p / gc, bc = p % gc;
        int64_t r0 = br * pr, c0 = bc * pc;
        int64_t h = rows - r0 < pr ? rows - r0 : pr, w = cols - c0 < pc ? cols - c0 : pc;
        volatile float s_inv = 1.0f / scale[p];
        for (int64_t r = 0; r < h; ++r)
            for (int64_t c = 0; c < w; ++c) {
                int64_t i = (r0 + r) * cols + c0 + c;
                if (mask[p] == 1) {
                    if (!bf16) continue;
                    y[i] = bf16[i];
                } else {
                    float q = (float)(mask[p] == 2 ? fp8_value(fp8[i], 5, 2) : fp8_value(fp8[i], 4, 3));  /* exact */
                    volatile float v = q * s_inv;
                    y[i] = mor_oracle_f32_to_bf16(v);
                }
            }
    }
    return 0;
}
int mor_oracle_dequantize(const uint8_t *fp8, const float *scale, const uint8_t *mask,
                          const uint16_t *bf16, int64_t rows, int64_t cols, int gran,
                          uint16_t *y)
{
    return mor_oracle_dequantize_ex(fp8, scale, mask, bf16, rows, cols, gran, 0, y);
}

/*
 * Selection statistics over the per-block outputs (Section 4.1.3): block and element counts
 * per chosen type, aggregate error, a 12-bin histogram of block metrics in 0.5 % steps with
 * an open last bin, and the number of blocks whose metric lies within near_tol * threshold
 * of the threshold.  The block metric is taken in binary32, err_sum / nnz (0 when nnz = 0),
 * because it decides integer bin indices and both sides must decide in the same precision.
 */
typedef struct {
    uint64_t n_part, n_fp8_part, n_bf16_part, n_elem_fp8, n_elem_bf16, nnz_total, n_near_threshold;
    double err_sum_total, mean_err;
    uint32_t hist[12];
    uint32_t pad_;
    uint64_t n_e5m2_part, n_elem_e5m2;
} oracle_stats;

int mor_oracle_select_stats_ex(const float *err_sum, const uint32_t *nnz, const uint8_t *mask,
                               int64_t rows, int64_t cols, int gran, int ragged, float threshold, float near_tol,
                               oracle_stats *out)
{
    int64_t pr, pc, gc, P;
    if (rows <= 0 || cols <= 0 || part_shape_ex(gran, rows, cols, ragged, &pr, &pc)) return -1;
    gc = (cols + pc - 1) / pc;
    P = ((rows + pr - 1) / pr) * gc;
    memset(out, 0, sizeof *out);
    out->n_part = (uint64_t)P;
    for (int64_t p = 0; p < P; ++p) {
        int64_t r0 = (p / gc) * pr, c0 = (p % gc) * pc;
        int64_t h = rows - r0 < pr ? rows - r0 : pr, w = cols - c0 < pc ? cols - c0 : pc;
        volatile float metric = nnz[p] ? err_sum[p] / (float)nnz[p] : 0.0f;
        int bin = 0;
        if (mask[p] == 1)      { out->n_bf16_part++; out->n_elem_bf16 += (uint64_t)(h * w); }
        else if (mask[p] == 2) { out->n_e5m2_part++; out->n_elem_e5m2 += (uint64_t)(h * w); }
        else                   { out->n_fp8_part++;  out->n_elem_fp8  += (uint64_t)(h * w); }
        out->err_sum_total += (double)err_sum[p];
        out->nnz_total += nnz[p];
        if (!(metric < INFINITY)) bin = 11;
        else
            for (int k = 1; k <= 11; ++k)
                if (metric >= (float)(0.005 * k)) bin = k;
        out->hist[bin]++;
        if (fabs((double)metric - (double)threshold) <= (double)near_tol * (double)threshold)
            out->n_near_threshold++;
    }
    out->mean_err = out->nnz_total ? out->err_sum_total / (double)out->nnz_total : 0.0;
    return 0;
}
int mor_oracle_select_stats(const float *err_sum, const uint32_t *nnz, const uint8_t *mask,
                            int64_t rows, int64_t cols, int gran, float threshold, float near_tol,
                            oracle_stats *out)
{
    return mor_oracle_select_stats_ex(err_sum, nnz, mask, rows, cols, gran, 0, threshold, near_tol, out);
}

/*
 * Running histogram of one tensor's metric over mini-batches (Section 4.1.3, the paragraphs on
 * Figure "annotation"): every mini-batch adds ONE count, in the bin of the tensor's relative
 * error of that step; the histogram is cleared every `reset_interval` steps (6000 in the paper)
 * before the step's count is added.  `step` counts from 0.  The metric is taken in binary32.
 */
void mor_oracle_histogram_update(uint32_t *hist12, float tensor_metric, int64_t step, int64_t reset_interval)
{
    int bin = 0;
    if (reset_interval > 0 && step % reset_interval == 0) memset(hist12, 0, 12 * sizeof(uint32_t));
    if (!(tensor_metric < INFINITY)) bin = 11;
    else
        for (int k = 1; k <= 11; ++k)
            if (tensor_metric >= (float)(0.005 * k)) bin = k;
    hist12[bin]++;
}

/* Number of OpenMP threads the oracle may use from now on (benchmark's single-thread baseline). */
void mor_oracle_set_threads(int n)
{
#ifdef _OPENMP
    if (n > 0) omp_set_num_threads(n);
#else
    (void)n;
#endif
}

int mor_oracle_threads(void)
{
#ifdef _OPENMP
    return omp_get_max_threads();
#else
    return 1;
#endif
}
