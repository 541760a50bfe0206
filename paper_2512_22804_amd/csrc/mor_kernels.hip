// HIP kernels of the MoR analyse-select-quantize path for gfx950 (MI355X), and their launchers.
//
// One fused HBM pass per operand for sub-tensor granularities: 128-bit BF16 loads, integer amax,
// one IEEE division per block, hardware OCP-E4M3 conversion, relative-error reduction, decision
// (Algorithm 2 with [E4M3, BF16]) and emission, all from registers.  Per-tensor granularity needs
// the global amax before anything can be scaled and therefore reads the operand twice.
// The path is HBM-bound: there is no contraction in it, so no MFMA.
#include <type_traits>

#include "mor_device.h"
#include "mor_launch.h"
#include "mor_sub1x128.h"

namespace mor {


// ======================================================================================
// 1 x 128 sub-channel blocks (Section 3: sub-channel partition; DeepSeek-style activations)
// A 16-lane DPP row owns one block at a time (16 lanes x 8 elements); a wave works on 4 blocks
// per load instruction and keeps 4 loads in flight, so every reduction stays inside a row.
// ======================================================================================
// One block per 16-lane row, 8 elements per lane.  `valid` is false for lanes beyond the last column of a
// ragged tensor (they hold zeros and store nothing).  FAKE: the de-quantized values go to dst_fake instead
// of the codes to dst_fp8.  `three`: the block may end in E5M2 (Section 3.2, three-way recipe).
template <int CRIT, bool DEFER, bool FAKE>
__device__ __forceinline__ void sub_block_body(const u32x4& raw, const uint16_t* __restrict__ src, bool valid, int l, int64_t p,
                                               const KOut& o, uint8_t* __restrict__ dst_fp8, uint16_t* __restrict__ dst_bf16,
                                               uint16_t* __restrict__ dst_fake, float th, uint32_t mode, uint32_t mg, uint32_t mg5,
                                               bool three) {
    Scan8 sc{0u, 0u};
    scan8(raw, sc);
    const uint32_t abits = row_allmax_u32(fold_max16(sc.amax2));
    float s = block_scale(abits, kE4M3Max, mode, mg);
    const float s5 = block_scale(abits, kE5M2Max, mode, mg5);
    const bool fast = abits < fast_amax_limit(mode);
    auto quantize = [&](auto fmt, float sc_, bool emit) -> float {
        constexpr bool E5 = decltype(fmt)::value;
        const float s_inv = FAKE ? 1.0f / sc_ : 0.0f;
        float e0 = 0.0f, e1 = 0.0f;
        if (fast) {
            u32x4 deq;
            const u32x2 codes = quant8_fast_deq<E5, FAKE>(raw, sc_, s_inv, e0, e1, deq);
            if (emit && valid) {
                if constexpr (FAKE) store16(dst_fake, deq);
                else store8(dst_fp8, codes);
            }
        } else if (valid) {
            e0 = quant8_careful_mem<E5>(src, sc_, emit && !FAKE ? dst_fp8 : nullptr, emit && FAKE ? dst_fake : nullptr, s_inv);
        }
        return e0 + e1;
    };
    float err = row_allsum_f32(quantize(std::false_type{}, s, true));
    float err5 = 0.0f;
    if constexpr (CRIT == kCritEq3) err5 = row_allsum_f32(quantize(std::true_type{}, s5, false));
    const uint32_t nnz = 128u - row_allsum_u32(fold_add16(sc.zero2));
    if (abits >= kInfBits) { err = __builtin_inff(); err5 = __builtin_inff(); }
    uint32_t mask = 0u;
    if constexpr (!DEFER) mask = (CRIT == kCritEq3) ? decide_eq3(err, err5) : decide_eq2(err, nnz, th);
    uint32_t amin_bits = 0u;
    if (three) {                                              // uniform over the launch
        const uint32_t mn = ~row_allmax_u32(~fold_min16(min_nonzero_m1(raw, 0xFFFFFFFFu))) & 0xFFFFu;
        if (mask == 1u) {
            amin_bits = nnz ? mn + 1u : 0u;
            if (range_fits_e5m2(abits, amin_bits, nnz)) {
                mask = 2u;
                s = s5;
                (void)quantize(std::true_type{}, s5, true);   // the E5M2 payload replaces the E4M3 one
            }
        }
    }
    if (l == 0) {
        o.scale[p] = s;
        o.amax[p] = __uint_as_float(abits << 16);
        o.err_sum[p] = err;
        o.nnz[p] = nnz;
        if constexpr (CRIT == kCritEq3) o.err5_sum[p] = err5;
        if constexpr (!DEFER) o.mask[p] = (uint8_t)mask;
        if (mode != kScaleFp32 && o.e8m0) o.e8m0[p] = (uint8_t)(__float_as_uint(s) >> 23);
        if (three && o.amin) o.amin[p] = __uint_as_float(amin_bits << 16);
    }
    if constexpr (!DEFER) {
        if (mask == 1u && dst_bf16 && valid) store16(dst_bf16, raw);
    }
}

// General 1 x 128 kernel (padded leading dimensions, ragged last column block, three types, fake
// quantization): grid.x = 128-column block, grid.y strides over groups of 16 rows.
template <int CRIT, bool DEFER, bool FAKE>
__global__ __launch_bounds__(256) void k_sub1x128_strided(const uint16_t* __restrict__ x, KShape sh, KOut o, float th,
                                                          uint32_t mode, const uint32_t* __restrict__ gam, uint32_t three, uint32_t group_rows) {
    const int lane = threadIdx.x & 63, g = lane >> 4, l = lane & 15;
    const int64_t cb = blockIdx.x, cpr = (sh.cols + 127) / 128;
    const int64_t c = cb * 128 + l * 8;
    const bool valid = c < sh.cols;
    for (int64_t r = (int64_t)blockIdx.y * 16 + (threadIdx.x >> 6) * 4 + g; r < sh.rows; r += (int64_t)gridDim.y * 16) {
        const uint16_t* src = x + r * sh.ld + c;
        u32x4 raw; raw.x = 0u; raw.y = 0u; raw.z = 0u; raw.w = 0u;
        if (valid) raw = load16(src);
        uint32_t mg = 0u, mg5 = 0u;
        if (mode) { const uint32_t* gw = gam_words(gam, group_rows, r); mg = gw[0]; mg5 = gw[1]; }
        sub_block_body<CRIT, DEFER, FAKE>(raw, src, valid, l, r * cpr + cb, o, FAKE ? nullptr : o.fp8 + r * o.ld_fp8 + c,
                                          o.bf16 ? o.bf16 + r * o.ld_bf16 + c : nullptr, FAKE ? o.fake + r * o.ld_fake + c : nullptr,
                                          th, mode, mg, mg5, three != 0u);
    }
}

// ======================================================================================
// Per-tensor granularity (Section 4.1.1 "Per-Tensor"): pass A = global amax, pass B = quantize
// with the global scale; the last workgroup of pass B to finish sums the per-workgroup error
// partials in binary64 and takes the decision; then a conditional copy of the BF16 fallback.
// Everything is stream-ordered; the host never waits.
// ======================================================================================
constexpr int kTensorChunksPerThread = 8;                       // 16-byte chunks per thread in pass B
constexpr int kTensorChunksPerBlock = 256 * kTensorChunksPerThread;
constexpr int kMaxAmaxBlocks = 2048;     // pass A of the six gradient operands: 78 us at 2048 workgroups, 86 us at 1024, 84 us at 4096
constexpr int kProveMaxWg = 8192;      // workgroups of one launch (and partial records per operand) of the block-shaped GAM pre-pass

__device__ __forceinline__ uint32_t block_allmax_u32(uint32_t v, uint32_t* sh4) {
    const uint32_t wv = wave_allmax_u32(v);
    if ((threadIdx.x & 63) == 0) sh4[threadIdx.x >> 6] = wv;
    __syncthreads();
    const uint32_t r = max(max(sh4[0], sh4[1]), max(sh4[2], sh4[3]));
    __syncthreads();
    return r;
}
__device__ __forceinline__ uint32_t amax2_of(const u32x4& v, uint32_t a2) {
#pragma unroll
    for (int j = 0; j < 4; ++j) a2 = pk_max_u16(a2, v[j] & 0x7FFF7FFFu);
    return a2;
}

// Pass A, strided: one workgroup strides over rows; lanes stride over the row's chunks.
// A partial word of pass A: low half = amax pattern; high half = (smallest non-zero pattern - 1) when the three-way
// recipe needs it for Eq. (4) (0xFFFF: no non-zero element seen), else 0.
__device__ __forceinline__ uint32_t block_allmin_u16(uint32_t v, uint32_t* sh4) { return 0xFFFFu - block_allmax_u32(0xFFFFu - v, sh4); }
__global__ __launch_bounds__(256) void k_tensor_amax_strided(const uint16_t* __restrict__ x, KShape sh,
                                                             uint32_t* __restrict__ part, uint32_t three) {
    __shared__ uint32_t sh4[4];
    uint32_t a2 = 0u, mn2 = 0xFFFFFFFFu;
    const int64_t cpr = sh.cols / 8;
    for (int64_t r = blockIdx.x; r < sh.rows; r += gridDim.x)
        for (int64_t c = threadIdx.x; c < cpr; c += 256) {
            const u32x4 v = load16(x + r * sh.ld + c * 8);
            a2 = amax2_of(v, a2);
            if (three) mn2 = min_nonzero_m1(v, mn2);
        }
    const uint32_t a = block_allmax_u32(fold_max16(a2), sh4);
    uint32_t mn = 0u;
    if (three) mn = block_allmin_u16(fold_min16(mn2), sh4);
    if (threadIdx.x == 0) part[blockIdx.x] = a | (mn << 16);
}

__device__ __forceinline__ uint32_t global_amax_bits(const uint32_t* __restrict__ part, int n_part_amax, uint32_t* sh4) {
    uint32_t a = 0u;
    for (int i = threadIdx.x; i < n_part_amax; i += 256) a = max(a, part[i] & 0xFFFFu);
    return block_allmax_u32(a, sh4);
}
// Smallest non-zero magnitude pattern of the operand from the partial words (0 when it has no non-zero element).
__device__ __forceinline__ uint32_t global_amin_bits(const uint32_t* __restrict__ part, int n_part_amax, uint32_t* sh4) {
    uint32_t m = 0xFFFFu;
    for (int i = threadIdx.x; i < n_part_amax; i += 256) m = min(m, part[i] >> 16);
    m = block_allmin_u16(m, sh4);
    return m == 0xFFFFu ? 0u : m + 1u;
}
// The E5M2 payload of a whole operand (three-way recipe, per-tensor granularity): one more sweep that overwrites the
// E4M3 codes (or the fake-quantized values) of pass B.  One 8-element chunk:
__device__ __forceinline__ void requant_chunk_e5m2(const uint16_t* __restrict__ src, uint8_t* __restrict__ d8, uint16_t* __restrict__ df,
                                                   float s5, float s_inv, bool fast) {
    if (fast) {
        const u32x4 raw = load16(src);
        float e0 = 0.0f, e1 = 0.0f;
        u32x4 deq;
        if (df) { (void)quant8_fast_deq<true, true>(raw, s5, s_inv, e0, e1, deq); store16(df, deq); }
        else store8(d8, quant8_fast_deq<true, false>(raw, s5, s_inv, e0, e1, deq));
    } else {
        (void)quant8_careful_mem<true>(src, s5, df ? nullptr : d8, df, s_inv);
    }
}

struct TensorPartials {   // one slot per pass-B workgroup (at most kMaxQuantBlocks)
    float* err;
    float* err5;
    uint32_t* zero;        // zero elements seen by the workgroup (padding chunks count as zeros)
    uint32_t* abits;       // [0] = global amax bits, published by workgroup 0 of pass B
};
constexpr int kMaxQuantBlocks = 16384;
constexpr int kSoloAmaxBlocks = 768, kSoloQuantBlocks = 1536;     // launch shape of a per-tensor operand that is alone in its launches

template <typename T>
__device__ __forceinline__ T block_sum_256(T v, T* sh) {
    sh[threadIdx.x] = v;
    __syncthreads();
#pragma unroll
    for (int s = 128; s > 0; s >>= 1) {
        if ((int)threadIdx.x < s) sh[threadIdx.x] += sh[threadIdx.x + s];
        __syncthreads();
    }
    const T r = sh[0];
    __syncthreads();
    return r;
}
// Same result on every thread, two barriers, fixed summation order.
template <typename T>
__device__ __forceinline__ T block_sum_shfl(T v, T* sh4) {
#pragma unroll
    for (int m = 32; m > 0; m >>= 1) v += __shfl_xor(v, m, 64);
    if ((threadIdx.x & 63) == 0) sh4[threadIdx.x >> 6] = v;
    __syncthreads();
    const T r = (sh4[0] + sh4[1]) + (sh4[2] + sh4[3]);
    __syncthreads();
    return r;
}

struct TensorAcc {
    float e0, e1, f0, f1;
    uint32_t zero2;
};
__device__ __forceinline__ uint32_t zero2_of(const u32x4& v, uint32_t z2) {
#pragma unroll
    for (int j = 0; j < 4; ++j) z2 = pk_add_u16(z2, pk_is_zero_u16(v[j] & 0x7FFF7FFFu));
    return z2;
}
template <int CRIT>
__device__ __forceinline__ void tensor_publish(const TensorAcc& a, const TensorPartials& tp, int slot) {
    __shared__ float shf[8];
    __shared__ uint32_t shu[4];
    const float werr = wave_allsum_f32(a.e0 + a.e1);
    const uint32_t wzero = wave_allsum_u32(fold_add16(a.zero2));
    float werr5 = 0.0f;
    if constexpr (CRIT == kCritEq3) werr5 = wave_allsum_f32(a.f0 + a.f1);
    const int w = threadIdx.x >> 6;
    if ((threadIdx.x & 63) == 0) { shf[w] = werr; shf[4 + w] = werr5; shu[w] = wzero; }
    __syncthreads();
    if (threadIdx.x == 0) {
        tp.err[slot] = (shf[0] + shf[1]) + (shf[2] + shf[3]);
        tp.zero[slot] = (shu[0] + shu[1]) + (shu[2] + shu[3]);
        if constexpr (CRIT == kCritEq3) tp.err5[slot] = (shf[4] + shf[5]) + (shf[6] + shf[7]);
    }
}

// Pass B, strided: persistent workgroups stride over 16-row x 128-column tiles, one chunk per thread.
template <int CRIT, bool FAKE>
__global__ __launch_bounds__(256) void k_tensor_quant_strided(const uint16_t* __restrict__ x, KShape sh, uint32_t tiles_x,
                                                              uint32_t n_tiles, KOut o, const uint32_t* __restrict__ amax_part,
                                                              int n_amax_part, TensorPartials tp, uint32_t mode) {
    __shared__ uint32_t sh4[4];
    const uint32_t abits = global_amax_bits(amax_part, n_amax_part, sh4);
    if (blockIdx.x == 0 && threadIdx.x == 0) tp.abits[0] = abits;
    // one block = the group: under GAM the block's own mantissa is the group mantissa, the scale is s_b
    const float s = block_scale(abits, kE4M3Max, mode, group_mantissa_bits(abits, kE4M3Max, mode));
    const float s5 = (CRIT == kCritEq3) ? block_scale(abits, kE5M2Max, mode, group_mantissa_bits(abits, kE5M2Max, mode)) : 0.0f;
    const float s_inv = FAKE ? 1.0f / s : 0.0f;
    TensorAcc acc{0.0f, 0.0f, 0.0f, 0.0f, 0u};
    for (uint32_t tile = blockIdx.x; tile < n_tiles; tile += gridDim.x) {
        const uint32_t ty = tile / tiles_x, tx = tile - ty * tiles_x;
        const int64_t r = (int64_t)ty * 16 + (threadIdx.x >> 4);
        const int64_t c = (int64_t)tx * 128 + (threadIdx.x & 15) * 8;
        const bool live = r < sh.rows && c < sh.cols;
        u32x4 raw; raw.x = 0u; raw.y = 0u; raw.z = 0u; raw.w = 0u;
        if (live) raw = load16(x + r * sh.ld + c);
        acc.zero2 = zero2_of(raw, acc.zero2);
        if (abits < fast_amax_limit(mode)) {
            u32x4 deq;
            const u32x2 codes = quant8_fast_deq<false, FAKE>(raw, s, s_inv, acc.e0, acc.e1, deq);
            if (live) {
                if constexpr (FAKE) store16(o.fake + r * o.ld_fake + c, deq);
                else store8(o.fp8 + r * o.ld_fp8 + c, codes);
            }
            if constexpr (CRIT == kCritEq3) (void)quant8_fast<true>(raw, s5, acc.f0, acc.f1);
        } else if (live) {
            acc.e0 += quant8_careful_mem<false>(x + r * sh.ld + c, s, FAKE ? nullptr : o.fp8 + r * o.ld_fp8 + c,
                                                FAKE ? o.fake + r * o.ld_fake + c : nullptr, s_inv);
            if constexpr (CRIT == kCritEq3) acc.f0 += quant8_careful_mem<true>(x + r * sh.ld + c, s5, nullptr);
        }
    }
    tensor_publish<CRIT>(acc, tp, blockIdx.x);
}

// Pass C: every workgroup re-derives the tensor's decision from the per-workgroup partials
// (binary64 sums in a fixed order, so all workgroups agree), workgroup 0 writes the block outputs
// (P = 1), and if the decision is BF16 the grid copies the operand into the fallback buffer.
// A thread's share of the per-workgroup partial sums of pass B (slots threadIdx.x, threadIdx.x + 256, ... in that order).
// Eight slots' loads are in flight together: the workgroup that does this is on the critical path of the call (one
// dependent load per slot took 11 round trips for the 2731 slots of an operand of the layer sweep).  A slot beyond the
// end adds +0, which leaves the (non-negative) sums as they are, so the result is that of the plain loop bit for bit.
template <int CRIT>
__device__ __forceinline__ void tensor_partial_sums(const float* __restrict__ err, const float* __restrict__ err5,
                                                    const uint32_t* __restrict__ zero, int n_slots, double& se, double& se5,
                                                    unsigned long long& sz) {
    for (int i0 = threadIdx.x; i0 < n_slots; i0 += 8 * 256) {
        float e[8], e5[8];
        uint32_t z[8];
#pragma unroll
        for (int u = 0; u < 8; ++u) {
            const int i = i0 + u * 256;
            const bool ok = i < n_slots;
            const int ic = ok ? i : n_slots - 1;           // always a valid slot: the loads need no branch
            const float ev = err[ic];
            const uint32_t zv = zero[ic];
            e[u] = ok ? ev : 0.0f;
            z[u] = ok ? zv : 0u;
            if constexpr (CRIT == kCritEq3) { const float e5v = err5[ic]; e5[u] = ok ? e5v : 0.0f; } else e5[u] = 0.0f;
        }
#pragma unroll
        for (int u = 0; u < 8; ++u) {
            se += (double)e[u];
            sz += z[u];
            if constexpr (CRIT == kCritEq3) se5 += (double)e5[u];
        }
    }
}
template <int CRIT>
__global__ __launch_bounds__(256) void k_tensor_finish(TensorPartials tp, int n_slots, unsigned long long n_padded, KOut o, float th,
                                                       const uint16_t* __restrict__ x, KShape sh, int flat, uint32_t mode,
                                                       uint32_t three, const uint32_t* __restrict__ amax_part, int n_amax_part) {
    __shared__ double shd[4];
    __shared__ unsigned long long shl[4];
    __shared__ uint32_t sh4[4];
    double se = 0.0, se5 = 0.0;
    unsigned long long sz = 0;
    tensor_partial_sums<CRIT>(tp.err, tp.err5, tp.zero, n_slots, se, se5, sz);
    se = block_sum_shfl<double>(se, shd);
    sz = block_sum_shfl<unsigned long long>(sz, shl);
    if constexpr (CRIT == kCritEq3) se5 = block_sum_shfl<double>(se5, shd);
    const uint32_t abits = tp.abits[0];
    const unsigned long long n = n_padded - sz;
    if (abits >= kInfBits) { se = (double)__builtin_inff(); se5 = se; }
    uint32_t mask;
    if constexpr (CRIT == kCritEq3) mask = (se < se5) ? 0u : 1u;
    else mask = ((n ? se / (double)n : 0.0) < (double)th) ? 0u : 1u;
    const float s5 = block_scale(abits, kE5M2Max, mode, group_mantissa_bits(abits, kE5M2Max, mode));
    uint32_t amin_bits = 0u;
    if (three && mask == 1u) {             // Eq. (4): the operand is kept in E5M2 if its dynamic range fits
        amin_bits = global_amin_bits(amax_part, n_amax_part, sh4);
        if (range_fits_e5m2(abits, amin_bits, n ? 1u : 0u)) mask = 2u;
    }
    if (blockIdx.x == 0 && threadIdx.x == 0) {
        const uint32_t mg = group_mantissa_bits(abits, kE4M3Max, mode);
        const float s = mask == 2u ? s5 : block_scale(abits, kE4M3Max, mode, mg);
        if (three && o.amin) o.amin[0] = __uint_as_float(amin_bits << 16);
        o.scale[0] = s;
        if (mode != kScaleFp32 && o.e8m0) o.e8m0[0] = (uint8_t)(__float_as_uint(s) >> 23);
        if (mode != kScaleFp32 && o.gmant) { o.gmant[0] = mg; o.gmant[1] = group_mantissa_bits(abits, kE5M2Max, mode); }
        o.amax[0] = __uint_as_float(abits << 16);
        o.err_sum[0] = (float)se;
        o.nnz[0] = n > 0xFFFFFFFFull ? 0xFFFFFFFFu : (uint32_t)n;
        if constexpr (CRIT == kCritEq3) o.err5_sum[0] = (float)se5;
        o.mask[0] = (uint8_t)mask;
    }
    if (mask == 2u) {
        const bool fast = abits < fast_amax_limit(mode);
        const float s_inv = o.fake ? 1.0f / s5 : 0.0f;
        const int64_t cpr = sh.cols / 8;
        for (int64_t r = blockIdx.x; r < sh.rows; r += gridDim.x)
            for (int64_t c = threadIdx.x; c < cpr; c += 256)
                requant_chunk_e5m2(x + r * sh.ld + c * 8, o.fake ? nullptr : o.fp8 + r * o.ld_fp8 + c * 8,
                                   o.fake ? o.fake + r * o.ld_fake + c * 8 : nullptr, s5, s_inv, fast);
        return;
    }
    if (mask == 0u || o.bf16 == nullptr) return;
    if (flat) {
        const int64_t n_chunks = sh.rows * sh.cols / 8;
        const int64_t stride = (int64_t)gridDim.x * 256;
        int64_t c = (int64_t)blockIdx.x * 256 + threadIdx.x;
        for (; c + 3 * stride < n_chunks; c += 4 * stride) {
            u32x4 v[4];
#pragma unroll
            for (int u = 0; u < 4; ++u) v[u] = load16(x + (c + u * stride) * 8);
#pragma unroll
            for (int u = 0; u < 4; ++u) store16(o.bf16 + (c + u * stride) * 8, v[u]);
        }
        for (; c < n_chunks; c += stride) store16(o.bf16 + c * 8, load16(x + c * 8));
    } else {
        const int64_t cpr = sh.cols / 8;
        for (int64_t r = blockIdx.x; r < sh.rows; r += gridDim.x)
            for (int64_t c = threadIdx.x; c < cpr; c += 256) store16(o.bf16 + r * o.ld_bf16 + c * 8, load16(x + r * sh.ld + c * 8));
    }
}

// Copies `n_chunks` 16-byte chunks from x to dst with workgroup `b` of `nb`: tiles of 1024 consecutive chunks (16 KB),
// four 16-byte loads in flight per lane.
__device__ __forceinline__ void copy_chunk_tiles(const uint16_t* __restrict__ x, uint16_t* __restrict__ dst, int64_t n_chunks, int b, int nb) {
    const int64_t n_tiles = (n_chunks + 1023) / 1024;
    for (int64_t ct = b; ct < n_tiles; ct += nb) {
        const int64_t c0 = ct * 1024 + threadIdx.x;
        if (c0 + 3 * 256 < n_chunks) {
            u32x4 v[4];
#pragma unroll
            for (int u = 0; u < 4; ++u) v[u] = load16(x + (c0 + u * 256) * 8);
#pragma unroll
            for (int u = 0; u < 4; ++u) store16(dst + (c0 + u * 256) * 8, v[u]);
        } else {
            for (int u = 0; u < 4; ++u)
                if (c0 + u * 256 < n_chunks) store16(dst + (c0 + u * 256) * 8, load16(x + (c0 + u * 256) * 8));
        }
    }
}

// ======================================================================================
// Tensor-level decision over sub-tensor scaling (Section 3.1): the deferred block kernels wrote
// err_sum / nnz per block; aggregate sum(err_sum) / sum(nnz), decide once, broadcast the mask.
// ======================================================================================
// Grouped: every operand with a tensor-level decision shares two launches -- partial sums per workgroup, then the decision
// (re-derived by every workgroup of the operand from the partials in a fixed order, so all agree) with the mask
// broadcast and the conditional copy of the BF16 fallback.
constexpr int kScopeBlocks = 256;       // partial records per operand
constexpr int kMaxGroupScope = 16;
struct ScopeOp {
    const float* err_sum; const float* err5_sum; const uint32_t* nnz; uint8_t* mask;
    int64_t n_part;
    double* part_err; double* part_err5; unsigned long long* part_nnz;     // [kScopeBlocks] each
    uint32_t* decision;                                                    // [1]
    const uint32_t* proven;                                                // non-null and [0] != 0: the block kernel wrote the fallback
    float th;
    int32_t crit;
    int32_t n_red;                                                         // workgroups of the reduce pass (<= kScopeBlocks)
    // fallback copy
    const uint16_t* x; uint16_t* bf16;
    int64_t rows, cols, ld, ld_bf16;
};
struct GroupScope {
    int n;
    int32_t red_end[kMaxGroupScope], copy_end[kMaxGroupScope];
    ScopeOp op[kMaxGroupScope];
};
__global__ __launch_bounds__(256) void k_scope_reduce_group(GroupScope g) {
    __shared__ double shd[4];
    __shared__ unsigned long long shl[4];
    const int op = group_find32(g.red_end, g.n, blockIdx.x);
    const ScopeOp& t = g.op[op];
    const int b = blockIdx.x - (op ? g.red_end[op - 1] : 0);
    double e = 0.0, e5 = 0.0;
    unsigned long long n = 0;
    const int64_t stride = (int64_t)t.n_red * 256;
    for (int64_t p = (int64_t)b * 256 + threadIdx.x; p < t.n_part; p += stride) {
        e += (double)t.err_sum[p];
        n += t.nnz[p];
        if (t.crit == kCritEq3) e5 += (double)t.err5_sum[p];
    }
    e = block_sum_shfl<double>(e, shd);
    n = block_sum_shfl<unsigned long long>(n, shl);
    e5 = block_sum_shfl<double>(e5, shd);
    if (threadIdx.x == 0) { t.part_err[b] = e; t.part_nnz[b] = n; t.part_err5[b] = e5; }
}
// Same decision in every workgroup that calls it (fixed summation order over the operand's partial records).
__device__ __forceinline__ uint32_t scope_decision(const ScopeOp& t, double* shd, unsigned long long* shl) {
    double e = 0.0, e5 = 0.0;
    unsigned long long n = 0;
    if ((int)threadIdx.x < t.n_red) { e = t.part_err[threadIdx.x]; n = t.part_nnz[threadIdx.x]; e5 = t.part_err5[threadIdx.x]; }
    e = block_sum_shfl<double>(e, shd);
    n = block_sum_shfl<unsigned long long>(n, shl);
    e5 = block_sum_shfl<double>(e5, shd);
    if (t.crit == kCritEq3) return (e < e5) ? 0u : 1u;
    return ((n ? e / (double)n : 0.0) < (double)t.th) ? 0u : 1u;
}
// Decision (every workgroup re-derives it from the partial records: the same value everywhere), mask broadcast over the
// operand's workgroups, then the copy of a BF16 tensor that no earlier pass has proven and written.
__global__ __launch_bounds__(256) void k_scope_copy_group(GroupScope g) {
    __shared__ double shd[4];
    __shared__ unsigned long long shl[4];
    const int op = group_find32(g.copy_end, g.n, blockIdx.x);
    const ScopeOp& t = g.op[op];
    const int b = blockIdx.x - (op ? g.copy_end[op - 1] : 0);
    const int nb = g.copy_end[op] - (op ? g.copy_end[op - 1] : 0);
    const uint32_t m = scope_decision(t, shd, shl);
    if (b == 0 && threadIdx.x == 0) t.decision[0] = m;
    for (int64_t p = (int64_t)b * 256 + threadIdx.x; p < t.n_part; p += (int64_t)nb * 256) t.mask[p] = (uint8_t)m;
    if (t.bf16 == nullptr || m == 0u || (t.proven && t.proven[0] != 0u)) return;
    if (t.ld == t.cols && t.ld_bf16 == t.cols) {
        copy_chunk_tiles(t.x, t.bf16, t.rows * t.cols / 8, b, nb);
    } else {
        const int64_t cpr = t.cols / 8;
        for (int64_t r = b; r < t.rows; r += nb)
            for (int64_t c = threadIdx.x; c < cpr; c += 256) store16(t.bf16 + r * t.ld_bf16 + c * 8, load16(t.x + r * t.ld + c * 8));
    }
}

// ======================================================================================
// De-quantize / de-scale (Section 4, Figure 4).  Blocks whose width is a multiple of 8 (or the whole
// row): grid.x = 128-column strip, grid.y strides over groups of 16 rows, one 8-element chunk per
// thread and row.  Blocks one column wide: one workgroup per 128 x 128 tile, so that a thread's 8
// column scales are inverted once per tile.
// ======================================================================================
__device__ __forceinline__ float dequant_scale(const float* __restrict__ scale, const uint8_t* __restrict__ e8m0,
                                               const uint32_t* __restrict__ gmant, int64_t p, uint32_t mk, int64_t band) {
    // stored GAM form (Algorithm 1): the scale is rebuilt from the group's shared mantissa and the block's E8M0 byte
    return e8m0 ? __uint_as_float(((uint32_t)e8m0[p] << 23) | gmant[2 * band + (mk == 2u ? 1 : 0)]) : scale[p];
}
template <bool E5M2>
__device__ __forceinline__ u32x4 dequant8(const u32x2& q, float s_inv) {
    u32x4 out;
#pragma unroll
    for (int j = 0; j < 4; ++j) {
        const int word = (int)(j < 2 ? q.x : q.y);
        const f32x2 v = (j & 1) ? cvt_pk_f32<E5M2>(word, true) : cvt_pk_f32<E5M2>(word, false);
        out[j] = f32_to_bf16_rne(v.x * s_inv) | (f32_to_bf16_rne(v.y * s_inv) << 16);
    }
    return out;
}
__global__ __launch_bounds__(256) void k_dequant(StatsGeom g, int pr_log2, int pc_log2, const uint8_t* __restrict__ fp8, int64_t ld_fp8,
                                                 const float* __restrict__ scale, const uint8_t* __restrict__ mask,
                                                 const uint16_t* __restrict__ bf16, int64_t ld_bf16, uint16_t* __restrict__ y,
                                                 int64_t ld_y, const uint8_t* __restrict__ e8m0, const uint32_t* __restrict__ gmant,
                                                 int64_t group_rows) {
    const int64_t c = (int64_t)blockIdx.x * 128 + (threadIdx.x & 15) * 8;
    if (c >= g.cols) return;
    for (int64_t r = (int64_t)blockIdx.y * 16 + (threadIdx.x >> 4); r < g.rows; r += (int64_t)gridDim.y * 16) {
        const int64_t p = (r >> pr_log2) * g.gc + (c >> pc_log2);
        const uint32_t mk = mask[p];
        if (mk == 1u) {
            if (bf16) store16(y + r * ld_y + c, load16(bf16 + r * ld_bf16 + c));
            continue;
        }
        const float s_inv = 1.0f / dequant_scale(scale, e8m0, gmant, p, mk, group_rows ? r / group_rows : 0);     // correctly rounded IEEE division
        const u32x2 q = *reinterpret_cast<const u32x2*>(fp8 + r * ld_fp8 + c);
        store16(y + r * ld_y + c, mk == 2u ? dequant8<true>(q, s_inv) : dequant8<false>(q, s_inv));
    }
}
// Grouped form for many operands (blocks whose width is a multiple of 8): a workgroup takes 64 rows x 128 columns of
// one operand, four 8-byte payload loads in flight per lane.
constexpr int kMaxGroupDeq = 16;
struct DeqOp {
    StatsGeom g;
    int32_t pr_log2, pc_log2;
    int64_t strips_x;
    const uint8_t* fp8; int64_t ld_fp8;
    const float* scale; const uint8_t* mask;
    const uint16_t* bf16; int64_t ld_bf16;
    uint16_t* y; int64_t ld_y;
    const uint8_t* e8m0; const uint32_t* gmant;
    int64_t group_rows;
};
struct GroupDeq {
    int n;
    int64_t unit_end[kMaxGroupDeq];
    DeqOp op[kMaxGroupDeq];
};
__global__ __launch_bounds__(256) void k_dequant_group(GroupDeq gd) {
    const int op = group_find(gd.unit_end, gd.n, blockIdx.x);
    const DeqOp& t = gd.op[op];
    const int64_t unit = (int64_t)blockIdx.x - (op ? gd.unit_end[op - 1] : 0);
    const int64_t rg = unit / t.strips_x, strip = unit - rg * t.strips_x;
    const int64_t c = strip * 128 + (threadIdx.x & 15) * 8;
    if (c >= t.g.cols) return;
    const int64_t r0 = rg * 64 + (threadIdx.x >> 4);
    u32x2 q[4];
    uint32_t mk[4];
    float s[4];
#pragma unroll
    for (int k = 0; k < 4; ++k) {
        const int64_t r = r0 + 16 * k;
        mk[k] = 1u; s[k] = 1.0f; q[k].x = 0u; q[k].y = 0u;
        if (r < t.g.rows) {
            const int64_t p = (r >> t.pr_log2) * t.g.gc + (c >> t.pc_log2);
            mk[k] = t.mask[p];
            s[k] = dequant_scale(t.scale, t.e8m0, t.gmant, p, mk[k], t.group_rows ? r / t.group_rows : 0);
            if (mk[k] != 1u) q[k] = *reinterpret_cast<const u32x2*>(t.fp8 + r * t.ld_fp8 + c);
        }
    }
#pragma unroll
    for (int k = 0; k < 4; ++k) {
        const int64_t r = r0 + 16 * k;
        if (r >= t.g.rows) continue;
        if (mk[k] == 1u) {
            if (t.bf16) store16(t.y + r * t.ld_y + c, load16(t.bf16 + r * t.ld_bf16 + c));
            continue;
        }
        const float s_inv = 1.0f / s[k];                                   // correctly rounded IEEE division
        store16(t.y + r * t.ld_y + c, mk[k] == 2u ? dequant8<true>(q[k], s_inv) : dequant8<false>(q[k], s_inv));
    }
}
__global__ __launch_bounds__(256) void k_dequant_columns(StatsGeom g, int pr_log2, const uint8_t* __restrict__ fp8, int64_t ld_fp8,
                                                         const float* __restrict__ scale, const uint8_t* __restrict__ mask,
                                                         const uint16_t* __restrict__ bf16, int64_t ld_bf16, uint16_t* __restrict__ y,
                                                         int64_t ld_y, const uint8_t* __restrict__ e8m0, const uint32_t* __restrict__ gmant,
                                                         int64_t group_rows) {
    const int64_t c = (int64_t)blockIdx.x * 128 + (threadIdx.x & 15) * 8;
    if (c >= g.cols) return;
    for (int64_t tr = blockIdx.y; tr * 128 < g.rows; tr += gridDim.y) {
        const int64_t band = group_rows ? tr * 128 / group_rows : 0;        // (a band holds whole 128 x 1 blocks)
        const int64_t p0 = ((tr * 128) >> pr_log2) * g.gc + c;
        float s_inv[8];
        uint32_t mk[8];
        bool any_bf16 = false;
#pragma unroll
        for (int j = 0; j < 8; ++j) {
            mk[j] = mask[p0 + j];
            any_bf16 |= mk[j] == 1u;
            s_inv[j] = 1.0f / dequant_scale(scale, e8m0, gmant, p0 + j, mk[j], band);
        }
#pragma unroll 1
        for (int i = 0; i < 8; ++i) {
            const int64_t r = tr * 128 + (threadIdx.x >> 4) + i * 16;
            if (r >= g.rows) break;
            const u32x2 q = *reinterpret_cast<const u32x2*>(fp8 + r * ld_fp8 + c);
            u32x4 keep; keep.x = 0u; keep.y = 0u; keep.z = 0u; keep.w = 0u;
            if (any_bf16) keep = bf16 ? load16(bf16 + r * ld_bf16 + c) : load16(y + r * ld_y + c);
            u32x4 out;
#pragma unroll
            for (int j = 0; j < 4; ++j) {
                const int word = (int)(j < 2 ? q.x : q.y);
                const f32x2 v4 = (j & 1) ? cvt_pk_f32<false>(word, true) : cvt_pk_f32<false>(word, false);
                const f32x2 v5 = (j & 1) ? cvt_pk_f32<true>(word, true) : cvt_pk_f32<true>(word, false);
                const uint32_t lo = mk[2 * j] == 1u ? (keep[j] & 0xFFFFu) : f32_to_bf16_rne((mk[2 * j] == 2u ? v5.x : v4.x) * s_inv[2 * j]);
                const uint32_t hi = mk[2 * j + 1] == 1u ? (keep[j] >> 16) : f32_to_bf16_rne((mk[2 * j + 1] == 2u ? v5.y : v4.y) * s_inv[2 * j + 1]);
                out[j] = lo | (hi << 16);
            }
            store16(y + r * ld_y + c, out);
        }
    }
}

// ======================================================================================
// Selection statistics (Section 4.1.3)
// ======================================================================================
struct StatsDev {   // must match mor_stats in include/mor.h
    unsigned long long n_part, n_fp8_part, n_bf16_part, n_elem_fp8, n_elem_bf16, nnz_total, n_near_threshold;
    double err_sum_total, mean_err;
    uint32_t hist[12];
    uint32_t reserved;      // flags
    uint32_t reserved2;
    unsigned long long n_e5m2_part, n_elem_e5m2;
};
// Number of elements of block p: blocks at the right / bottom edge of a ragged tensor are smaller.
__device__ __forceinline__ unsigned long long block_elems(const StatsGeom& g, int64_t p) {
    if (g.uniform) return (unsigned long long)(g.pr * g.pc);
    const int64_t br = p / g.gc, bc = p - br * g.gc;
    const int64_t h = g.rows - br * g.pr < g.pr ? g.rows - br * g.pr : g.pr;
    const int64_t w = g.cols - bc * g.pc < g.pc ? g.cols - bc * g.pc : g.pc;
    return (unsigned long long)(h * w);
}
struct StatsAcc {
    double e;
    unsigned long long n, eb, e5;        // non-zeros; elements in BF16 blocks; elements in E5M2 blocks
    uint32_t cnt[kStatCnt];
};
__device__ __forceinline__ void stats_acc_clear(StatsAcc& a) {
    a.e = 0.0; a.n = 0ull; a.eb = 0ull; a.e5 = 0ull;
#pragma unroll
    for (int k = 0; k < kStatCnt; ++k) a.cnt[k] = 0u;
}
__device__ __forceinline__ void stats_accumulate(int64_t p, const float* __restrict__ err_sum, const uint32_t* __restrict__ nnz,
                                                 const uint8_t* __restrict__ mask, float th, float near_tol, const StatsGeom& geom,
                                                 StatsAcc& a) {
    const float es = err_sum[p];
    const uint32_t nz = nnz[p];
    const uint32_t mk = mask[p];
    const float metric = nz ? es / (float)nz : 0.0f;           // binary32, IEEE division
    const int bin = stats_bin(metric);
#pragma unroll
    for (int k = 0; k < 12; ++k) a.cnt[k] += (bin == k) ? 1u : 0u;
    a.e += (double)es;
    a.n += nz;
    a.cnt[12] += mk == 1u ? 1u : 0u;
    a.cnt[13] += (fabs((double)metric - (double)th) <= (double)near_tol * (double)th) ? 1u : 0u;
    a.cnt[14] += mk == 2u ? 1u : 0u;
    if (mk) {
        const unsigned long long ne = block_elems(geom, p);
        if (mk == 1u) a.eb += ne; else a.e5 += ne;
    }
}
__device__ __forceinline__ void stats_finish(StatsDev* st, int64_t n_part, unsigned long long total_elems, double e,
                                             unsigned long long n, unsigned long long n_bf16, unsigned long long n_near,
                                             unsigned long long n_e5, unsigned long long eb, unsigned long long ee5, uint32_t flags) {
    st->n_part = (unsigned long long)n_part;
    st->n_fp8_part = (unsigned long long)n_part - n_bf16 - n_e5;
    st->n_bf16_part = n_bf16;
    st->n_e5m2_part = n_e5;
    st->n_elem_fp8 = total_elems - eb - ee5;
    st->n_elem_bf16 = eb;
    st->n_elem_e5m2 = ee5;
    st->nnz_total = n;
    st->n_near_threshold = n_near;
    st->err_sum_total = e;
    st->mean_err = n ? e / (double)n : 0.0;
    st->reserved = flags;
    st->reserved2 = 0u;
}
// Block-wide sums of the small counters without same-address atomics: DPP wave sums, one LDS row per
// wave, then kStatCnt lanes add the four rows.  Result in sh[0][*].
__device__ __forceinline__ void block_counts(const uint32_t (&v)[kStatCnt], uint32_t (*sh)[kStatCnt]) {
    const int w = threadIdx.x >> 6;
#pragma unroll
    for (int k = 0; k < kStatCnt; ++k) {
        const uint32_t s = wave_allsum_u32(v[k]);
        if ((threadIdx.x & 63) == 0) sh[w][k] = s;
    }
    __syncthreads();
    if (threadIdx.x < kStatCnt) sh[0][threadIdx.x] = (sh[0][threadIdx.x] + sh[1][threadIdx.x]) + (sh[2][threadIdx.x] + sh[3][threadIdx.x]);
    __syncthreads();
}
struct StatsShared {
    uint32_t cnt[4][kStatCnt];
    double d[4];
    unsigned long long l[4];
};
// Reduces an accumulator over the workgroup: counters end in sh.cnt[0][*], the sums are returned in `a` on every thread.
__device__ __forceinline__ void stats_block_reduce(StatsAcc& a, StatsShared& sh) {
    block_counts(a.cnt, sh.cnt);
    a.e = block_sum_shfl<double>(a.e, sh.d);            // fixed order: deterministic
    a.n = block_sum_shfl<unsigned long long>(a.n, sh.l);
    a.eb = block_sum_shfl<unsigned long long>(a.eb, sh.l);
    a.e5 = block_sum_shfl<unsigned long long>(a.e5, sh.l);
}

// Up to a few thousand blocks: one workgroup, no atomics on global memory, deterministic sums.
__global__ __launch_bounds__(256) void k_stats_single(int64_t n_part, StatsGeom geom,
                                                      const float* __restrict__ err_sum, const uint32_t* __restrict__ nnz,
                                                      const uint8_t* __restrict__ mask, float th, float near_tol,
                                                      StatsDev* __restrict__ st) {
    __shared__ StatsShared sh;
    StatsAcc a;
    stats_acc_clear(a);
    for (int64_t p = threadIdx.x; p < n_part; p += 256) stats_accumulate(p, err_sum, nnz, mask, th, near_tol, geom, a);
    stats_block_reduce(a, sh);
    if (threadIdx.x < 12) st->hist[threadIdx.x] = sh.cnt[0][threadIdx.x];
    if (threadIdx.x == 0)
        stats_finish(st, n_part, (unsigned long long)(geom.rows * geom.cols), a.e, a.n, sh.cnt[0][12], sh.cnt[0][13], sh.cnt[0][14], a.eb, a.e5, 0u);
}

// Many blocks: the accumulators live in the output struct, cleared by a tiny kernel first and
// turned into the derived fields by a tiny kernel afterwards (no device-wide fences needed).
__global__ void k_stats_zero(StatsDev* st) {
    if (threadIdx.x < sizeof(StatsDev) / 4) reinterpret_cast<uint32_t*>(st)[threadIdx.x] = 0u;
}
__global__ __launch_bounds__(256) void k_stats_multi(int64_t n_part, StatsGeom geom,
                                                     const float* __restrict__ err_sum, const uint32_t* __restrict__ nnz,
                                                     const uint8_t* __restrict__ mask, float th, float near_tol,
                                                     StatsDev* __restrict__ st) {
    __shared__ StatsShared sh;
    StatsAcc a;
    stats_acc_clear(a);
    const int64_t stride = (int64_t)gridDim.x * 256;
    for (int64_t p = (int64_t)blockIdx.x * 256 + threadIdx.x; p < n_part; p += stride)
        stats_accumulate(p, err_sum, nnz, mask, th, near_tol, geom, a);
    stats_block_reduce(a, sh);
    if (threadIdx.x < 12 && sh.cnt[0][threadIdx.x]) atomicAdd(&st->hist[threadIdx.x], sh.cnt[0][threadIdx.x]);
    if (threadIdx.x == 0) {
        atomicAdd(&st->err_sum_total, a.e);
        atomicAdd(&st->nnz_total, a.n);
        atomicAdd(&st->n_bf16_part, (unsigned long long)sh.cnt[0][12]);
        atomicAdd(&st->n_near_threshold, (unsigned long long)sh.cnt[0][13]);
        atomicAdd(&st->n_e5m2_part, (unsigned long long)sh.cnt[0][14]);
        atomicAdd(&st->n_elem_bf16, a.eb);
        atomicAdd(&st->n_elem_e5m2, a.e5);
    }
}
// Derived fields once every workgroup of k_stats_multi has finished (next kernel on the stream).
__global__ void k_stats_finish(int64_t n_part, unsigned long long total_elems, StatsDev* __restrict__ st) {
    if (threadIdx.x == 0)
        stats_finish(st, n_part, total_elems, st->err_sum_total, st->nnz_total, st->n_bf16_part, st->n_near_threshold,
                     st->n_e5m2_part, st->n_elem_bf16, st->n_elem_e5m2, 0u);
}

// Running histogram of a tensor's error over training steps (Section 4.1.3): one count per step in the
// bin of (float)mean_err, cleared first on every reset step.
__global__ void k_histogram_update(uint32_t* __restrict__ hist, const StatsDev* __restrict__ st, int clear) {
    const int bin = stats_bin((float)st->mean_err);
    if (threadIdx.x < 12) {
        const uint32_t old = clear ? 0u : hist[threadIdx.x];
        hist[threadIdx.x] = old + ((int)threadIdx.x == bin ? 1u : 0u);
    }
}

// ======================================================================================
// Grouped kernels: one launch processes up to kMaxGroup dense operands of the same granularity and
// criterion.  A training step quantizes many operands (four linear layers x {activation, weight,
// gradient} per transformer block, Section 4), each worth only tens of microseconds of HBM time, so
// per-launch overhead is paid once per group instead of once per operand.  The descriptor tables
// travel in the kernel-argument segment: no staging copy, nothing allocated.
// ======================================================================================
constexpr int kMaxGroup = 8;           // per-tensor operands / GAM pre-pass per launch (their table shares the 4 KB
                                       // kernel-argument segment with the statistics riders)

template <int CRIT, bool FAKE>
__global__ __launch_bounds__(256) void k_sub1x128_group(GroupSub g) {
    sub_group_body<CRIT, FAKE>(g, (int64_t)blockIdx.x, (int64_t)gridDim.x);
}

// Statistics of sub-tensor operands of a group: pass 1 writes one partial record per workgroup into
// the workspace, pass 2 (one workgroup per operand) combines them in a fixed order.
struct StatsRec {      // 128 bytes
    double e;
    unsigned long long n, eb, e5;
    uint32_t cnt[kStatCnt];
    uint32_t pad[9];
};
struct StatsOp {
    const float* err_sum; const uint32_t* nnz; const uint8_t* mask;
    int64_t n_part;
    StatsGeom geom;
    float th;
    StatsRec* rec;          // [n_wg]
    StatsDev* out;
};
constexpr int kMaxGroupStats = 12;
struct GroupStats {
    int n;
    int32_t wg_end[kMaxGroupStats];
    float near_tol;
    StatsOp op[kMaxGroupStats];
};
__device__ __forceinline__ void stats_partial_body(const GroupStats& g, int block) {
    __shared__ StatsShared sh;
    const int op = group_find32(g.wg_end, g.n, block);
    const StatsOp& t = g.op[op];
    const int b = block - (op ? g.wg_end[op - 1] : 0);
    const int nb = g.wg_end[op] - (op ? g.wg_end[op - 1] : 0);
    StatsAcc a;
    stats_acc_clear(a);
    for (int64_t p = (int64_t)b * 256 + threadIdx.x; p < t.n_part; p += (int64_t)nb * 256)
        stats_accumulate(p, t.err_sum, t.nnz, t.mask, t.th, g.near_tol, t.geom, a);
    stats_block_reduce(a, sh);
    if (nb == 1) {      // the whole operand in one workgroup: write the result, no second pass needed
        if (threadIdx.x < 12) t.out->hist[threadIdx.x] = sh.cnt[0][threadIdx.x];
        if (threadIdx.x == 0)
            stats_finish(t.out, t.n_part, (unsigned long long)(t.geom.rows * t.geom.cols), a.e, a.n, sh.cnt[0][12], sh.cnt[0][13],
                         sh.cnt[0][14], a.eb, a.e5, 0u);
        return;
    }
    StatsRec* r = t.rec + b;
    if (threadIdx.x < kStatCnt) r->cnt[threadIdx.x] = sh.cnt[0][threadIdx.x];
    if (threadIdx.x == 0) { r->e = a.e; r->n = a.n; r->eb = a.eb; r->e5 = a.e5; }
}
__device__ __forceinline__ void stats_final_body(const GroupStats& g, int op) {
    __shared__ StatsShared sh;
    const StatsOp& t = g.op[op];
    const int nb = g.wg_end[op] - (op ? g.wg_end[op - 1] : 0);       // <= 256: one record per thread
    if (nb == 1) return;                                             // already final
    StatsAcc a;
    stats_acc_clear(a);
    if ((int)threadIdx.x < nb) {
        const StatsRec& r = t.rec[threadIdx.x];
        a.e = r.e; a.n = r.n; a.eb = r.eb; a.e5 = r.e5;
#pragma unroll
        for (int k = 0; k < kStatCnt; ++k) a.cnt[k] = r.cnt[k];      // per-workgroup counts fit 32 bits
    }
    stats_block_reduce(a, sh);
    if (threadIdx.x < 12) t.out->hist[threadIdx.x] = sh.cnt[0][threadIdx.x];
    if (threadIdx.x == 0)
        stats_finish(t.out, t.n_part, (unsigned long long)(t.geom.rows * t.geom.cols), a.e, a.n, sh.cnt[0][12], sh.cnt[0][13],
                     sh.cnt[0][14], a.eb, a.e5, 0u);
}

// ---- statistics launches of their own (operands that found no per-tensor launch to ride on, e.g. a single sub-tensor
//      operand): here the statistics are on the critical path of the call, so the kernels are built for latency --
//      workgroups of 1024 lanes, every lane's loads in flight together, the fifteen small counters packed two per
//      dword, wave sums through DPP, one barrier.  An operand of up to kStatsDirectParts blocks is finished by one
//      workgroup in one launch; larger ones leave one record per workgroup for the combine launch.
constexpr int kStatsFastThreads = 1024;
constexpr int kStatsFastPerLane = 4;                   // blocks per lane of a partial workgroup
constexpr int64_t kStatsDirectParts = 16384;           // one workgroup, 16 blocks per lane at most: packed 16-bit counters cannot overflow
template <int CTRL>
__device__ __forceinline__ unsigned long long dpp_u64(unsigned long long v) {
    return ((unsigned long long)dpp_u32<CTRL>((uint32_t)(v >> 32)) << 32) | dpp_u32<CTRL>((uint32_t)v);
}
__device__ __forceinline__ unsigned long long readlane_u64(unsigned long long v, int lane) {
    return ((unsigned long long)(uint32_t)__builtin_amdgcn_readlane((int)(v >> 32), lane) << 32) | (uint32_t)__builtin_amdgcn_readlane((int)v, lane);
}
__device__ __forceinline__ unsigned long long wave_allsum_u64(unsigned long long v) {
    v += dpp_u64<kDppXor1>(v); v += dpp_u64<kDppXor2>(v); v += dpp_u64<kDppHalfMirror>(v); v += dpp_u64<kDppMirror>(v);
    return (readlane_u64(v, 0) + readlane_u64(v, 16)) + (readlane_u64(v, 32) + readlane_u64(v, 48));
}
__device__ __forceinline__ double wave_allsum_f64(double v) {      // fixed order: deterministic
    auto sh = [](double x, auto ctrl) { return __longlong_as_double((long long)dpp_u64<decltype(ctrl)::value>((unsigned long long)__double_as_longlong(x))); };
    v += sh(v, std::integral_constant<int, kDppXor1>{}); v += sh(v, std::integral_constant<int, kDppXor2>{});
    v += sh(v, std::integral_constant<int, kDppHalfMirror>{}); v += sh(v, std::integral_constant<int, kDppMirror>{});
    auto rl = [&](int lane) { return __longlong_as_double((long long)readlane_u64((unsigned long long)__double_as_longlong(v), lane)); };
    return (rl(0) + rl(16)) + (rl(32) + rl(48));
}
struct StatsPacked {
    double e;
    unsigned long long n, eb, e5;
    uint32_t pk[8];        // counter k of StatsAcc::cnt in half (k & 1) of pk[k >> 1]
};
// Totals of one workgroup: the packed per-lane counters (at most 65535 blocks per lane) are widened before they are summed.
struct StatsTotals {
    double e;
    unsigned long long n, eb, e5;
    uint32_t c[kStatCnt];
};
template <int WAVES>
struct StatsFastShared {
    double e[WAVES];
    unsigned long long n[WAVES], eb[WAVES], e5[WAVES];
    uint32_t c[WAVES][kStatCnt];
};
__device__ __forceinline__ void stats_accumulate_packed(float es, uint32_t nz, uint32_t mk, unsigned long long ne, float th, float near_tol,
                                                        StatsPacked& a) {
    const float metric = nz ? es / (float)nz : 0.0f;           // binary32, IEEE division
    const int bin = stats_bin(metric);
    const uint32_t inc = 1u << ((bin & 1) * 16);
#pragma unroll
    for (int k = 0; k < 6; ++k) a.pk[k] += ((bin >> 1) == k) ? inc : 0u;
    a.e += (double)es;
    a.n += nz;
    a.pk[6] += (mk == 1u ? 1u : 0u) + ((fabs((double)metric - (double)th) <= (double)near_tol * (double)th) ? 0x10000u : 0u);
    a.pk[7] += mk == 2u ? 1u : 0u;
    if (mk == 1u) a.eb += ne;
    if (mk == 2u) a.e5 += ne;
}
__device__ __forceinline__ void stats_wave_sums(StatsTotals& t) {
    t.e = wave_allsum_f64(t.e); t.n = wave_allsum_u64(t.n); t.eb = wave_allsum_u64(t.eb); t.e5 = wave_allsum_u64(t.e5);
#pragma unroll
    for (int k = 0; k < kStatCnt; ++k) t.c[k] = wave_allsum_u32(t.c[k]);
}
// Sums over the workgroup (WAVES <= 64 waves), fixed order; the totals arrive in every lane of wave 0 (the other waves
// return with meaningless values).
template <int WAVES>
__device__ __forceinline__ void stats_fast_reduce(StatsTotals& t, StatsFastShared<WAVES>& sh) {
    const int w = threadIdx.x >> 6, lane = threadIdx.x & 63;
    stats_wave_sums(t);
    if (lane == 0) {
        sh.e[w] = t.e; sh.n[w] = t.n; sh.eb[w] = t.eb; sh.e5[w] = t.e5;
#pragma unroll
        for (int k = 0; k < kStatCnt; ++k) sh.c[w][k] = t.c[k];
    }
    __syncthreads();
    if (w != 0) return;
    const bool live = lane < WAVES;
    const int src = live ? lane : 0;
    t.e = live ? sh.e[src] : 0.0; t.n = live ? sh.n[src] : 0ull; t.eb = live ? sh.eb[src] : 0ull; t.e5 = live ? sh.e5[src] : 0ull;
#pragma unroll
    for (int k = 0; k < kStatCnt; ++k) t.c[k] = live ? sh.c[src][k] : 0u;
    stats_wave_sums(t);
}
// Value k (per lane, 0 .. kStatCnt - 1) of the totals, without indexing registers dynamically.
__device__ __forceinline__ uint32_t stats_pick(const StatsTotals& t, int k) {
    uint32_t v = 0u;
#pragma unroll
    for (int j = 0; j < kStatCnt; ++j) v = k == j ? t.c[j] : v;
    return v;
}
// Wave 0 writes either the operand's final statistics (`final_out`) or this workgroup's record.
__device__ __forceinline__ void stats_emit(const StatsTotals& t, StatsDev* out, int64_t n_part, unsigned long long total_elems, StatsRec* rec) {
    if (threadIdx.x >= 64) return;
    const uint32_t mine = stats_pick(t, (int)threadIdx.x < kStatCnt ? (int)threadIdx.x : 0);
    if (rec == nullptr) {
        if (threadIdx.x < 12) out->hist[threadIdx.x] = mine;
        if (threadIdx.x == 0)
            stats_finish(out, n_part, total_elems, t.e, t.n, t.c[12], t.c[13], t.c[14], t.eb, t.e5, 0u);
        return;
    }
    if (threadIdx.x < kStatCnt) rec->cnt[threadIdx.x] = mine;
    if (threadIdx.x == 0) { rec->e = t.e; rec->n = t.n; rec->eb = t.eb; rec->e5 = t.e5; }
}
__global__ __launch_bounds__(kStatsFastThreads) void k_stats_group_partial(GroupStats g) {
    __shared__ StatsFastShared<kStatsFastThreads / 64> sh;
    const int op = group_find32(g.wg_end, g.n, blockIdx.x);
    const StatsOp& t = g.op[op];
    const int b = blockIdx.x - (op ? g.wg_end[op - 1] : 0);
    const int nb = g.wg_end[op] - (op ? g.wg_end[op - 1] : 0);
    StatsPacked a;
    a.e = 0.0; a.n = 0ull; a.eb = 0ull; a.e5 = 0ull;
#pragma unroll
    for (int k = 0; k < 8; ++k) a.pk[k] = 0u;
    const int64_t stride = (int64_t)nb * kStatsFastThreads;
    for (int64_t p0 = (int64_t)b * kStatsFastThreads + threadIdx.x; p0 < t.n_part; p0 += 4 * stride) {
        float es[4]; uint32_t nz[4], mk[4];
#pragma unroll
        for (int u = 0; u < 4; ++u) {                          // four blocks' loads in flight per lane
            const int64_t p = p0 + u * stride;
            const bool ok = p < t.n_part;
            es[u] = ok ? t.err_sum[p] : 0.0f; nz[u] = ok ? t.nnz[p] : 0u; mk[u] = ok ? (uint32_t)t.mask[p] : 3u;
        }
#pragma unroll
        for (int u = 0; u < 4; ++u)
            if (mk[u] != 3u) stats_accumulate_packed(es[u], nz[u], mk[u], mk[u] ? block_elems(t.geom, p0 + u * stride) : 0ull, t.th, g.near_tol, a);
    }
    StatsTotals tot;
    tot.e = a.e; tot.n = a.n; tot.eb = a.eb; tot.e5 = a.e5;
#pragma unroll
    for (int k = 0; k < kStatCnt; ++k) tot.c[k] = (k & 1) ? a.pk[k >> 1] >> 16 : a.pk[k >> 1] & 0xFFFFu;
    stats_fast_reduce(tot, sh);
    stats_emit(tot, t.out, t.n_part, (unsigned long long)(t.geom.rows * t.geom.cols), nb == 1 ? nullptr : t.rec + b);
}
// Combine launch: one workgroup of 256 lanes per operand, one record per lane.
__global__ __launch_bounds__(256) void k_stats_group_final(GroupStats g) {
    __shared__ StatsFastShared<4> sh;
    const StatsOp& t = g.op[blockIdx.x];
    const int nb = g.wg_end[blockIdx.x] - (blockIdx.x ? g.wg_end[blockIdx.x - 1] : 0);       // <= kStatsMaxWg = 256
    if (nb == 1) return;                                                                       // already final
    StatsTotals tot;
    tot.e = 0.0; tot.n = 0ull; tot.eb = 0ull; tot.e5 = 0ull;
#pragma unroll
    for (int k = 0; k < kStatCnt; ++k) tot.c[k] = 0u;
    if ((int)threadIdx.x < nb) {
        const StatsRec& r = t.rec[threadIdx.x];
        tot.e = r.e; tot.n = r.n; tot.eb = r.eb; tot.e5 = r.e5;
#pragma unroll
        for (int k = 0; k < kStatCnt; ++k) tot.c[k] = r.cnt[k];
    }
    stats_fast_reduce(tot, sh);
    stats_emit(tot, t.out, t.n_part, (unsigned long long)(t.geom.rows * t.geom.cols), nullptr);
}

// ---- a lone dense 1 x 128 operand: the block kernel gathers the statistics of its workgroups itself (one record per
//      workgroup), so that the call needs one small combine launch afterwards instead of two statistics launches that
//      read the per-block outputs again.  (Combining the records inside the block kernel as well -- the workgroup that
//      draws the last of a set of ticket counters reads all records -- was built and measured: device-wide atomics on one
//      address complete about 15 ns apart, a device-wide release fence per workgroup writes back what its XCD still
//      holds of the payload (80 us per call), and with write-through record stores and two levels of counters the chain
//      of dependent device-scope round trips at the end of the kernel took as long as the launch it was to save.)
constexpr int kSoloRecWords = 20;          // dwords of a workgroup's record in use: 15 counters, pad, the sum (2), non-zeros, pad
struct SoloStats {
    StatsRec* rec;         // [gridDim.x]: 128 bytes apart, the first kSoloRecWords dwords used
    StatsDev* out;
    int64_t n_part;
    float near_tol;
    int n_rec;
};
// (Six workgroups per compute unit as for the kernel without statistics: the second launch bound makes the compiler fit
// Eq. 2's variants into 80 registers, which it does without spilling; Eq. 3's variants need more either way.)
template <int CRIT, bool FAKE>
__global__ __launch_bounds__(256, CRIT == kCritEq3 ? 4 : 6) void k_sub1x128_solo_stats(SubRiders g, SoloStats s) {
    __shared__ SubStatsShared ssh;
    const int w = threadIdx.x >> 6, lane = threadIdx.x & 63;
    if (threadIdx.x < 17) reinterpret_cast<uint32_t*>(&ssh)[threadIdx.x] = 0u;      // c[16], n
    ssh.e_lane[threadIdx.x] = 0.0;
    ssh.n_lane[threadIdx.x] = 0u;
    __syncthreads();
    sub_group_body<CRIT, FAKE, true>(g, (int64_t)blockIdx.x, (int64_t)gridDim.x, &ssh, s.near_tol);
    const double e_w = wave_allsum_f64(ssh.e_lane[threadIdx.x]);
    const uint32_t n_w = wave_allsum_u32(ssh.n_lane[threadIdx.x]);
    if (lane == 0) { ssh.e[w] = e_w; atomicAdd(&ssh.n, n_w); }
    __syncthreads();
    if (w != 0) return;
    uint32_t word = 0u;                                   // one dword of the record per lane
    if (lane < kStatCnt) word = ssh.c[lane];
    const double e_wg = (ssh.e[0] + ssh.e[1]) + (ssh.e[2] + ssh.e[3]);
    const unsigned long long e_bits = (unsigned long long)__double_as_longlong(e_wg);
    if (lane == 16) word = (uint32_t)e_bits;
    if (lane == 17) word = (uint32_t)(e_bits >> 32);
    if (lane == 18) word = ssh.n;
    if (lane < kSoloRecWords) reinterpret_cast<uint32_t*>(s.rec + blockIdx.x)[lane] = word;
}
// Combine launch of the above: one workgroup, the records in a fixed order.
constexpr int kSoloFinalThreads = 1024;
__global__ __launch_bounds__(kSoloFinalThreads) void k_solo_stats_final(SoloStats s) {
    __shared__ StatsFastShared<kSoloFinalThreads / 64> fin;
    StatsTotals tot;
    tot.e = 0.0; tot.n = 0ull; tot.eb = 0ull; tot.e5 = 0ull;
#pragma unroll
    for (int k = 0; k < kStatCnt; ++k) tot.c[k] = 0u;
    // a lane's records (lane, lane + 1024; there are at most 2048) are loaded together: one round trip instead of two
    unsigned long long q[2][kSoloRecWords / 2];
#pragma unroll
    for (int j = 0; j < 2; ++j) {
        const int i = (int)threadIdx.x + j * kSoloFinalThreads;
        const unsigned long long* r = reinterpret_cast<const unsigned long long*>(s.rec + (i < s.n_rec ? i : s.n_rec - 1));
#pragma unroll
        for (int k = 0; k < kSoloRecWords / 2; ++k) q[j][k] = r[k];
    }
#pragma unroll
    for (int j = 0; j < 2; ++j) {
        if ((int)threadIdx.x + j * kSoloFinalThreads >= s.n_rec) continue;
#pragma unroll
        for (int k = 0; k < kStatCnt; ++k) tot.c[k] += (uint32_t)(q[j][k >> 1] >> (32 * (k & 1)));
        tot.e += __longlong_as_double((long long)q[j][8]);
        tot.n += (uint32_t)q[j][9];
    }
    tot.eb = 128ull * tot.c[12];          // (per lane; the sums below add the lanes' products)
    stats_fast_reduce(tot, fin);
    stats_emit(tot, s.out, s.n_part, (unsigned long long)s.n_part * 128ull, nullptr);
}

// Per-tensor operands of a group share three launches (amax, quantize, finish + fallback copy).
struct TensorOp {
    const uint16_t* x;
    int64_t n_chunks, n_tiles;
    KOut o;
    float th;
    uint32_t mode;                       // scaling algorithm
    uint32_t three;                      // type list [E4M3, E5M2, BF16]
    uint32_t lean;                       // a proven BF16 operand gets no FP8 payload
    int n_amax, n_slots;                 // workgroups this operand gets in pass A / pass B
    uint32_t* amax_part;                 // [n_amax]
    float* err; float* err5; uint32_t* zero;   // [n_slots] each
    uint32_t* abits;                     // [2]: global amax bits; 1 if pass B wrote the fallback
    uint32_t* flush_part;                // [n_amax] lower bounds on the number of elements certain to flush to zero
    unsigned long long flush_need;       // that many certain flushes prove the BF16 decision (0 = proof not attempted)
    StatsDev* stats;                     // optional
};
struct GroupTensor {
    int n;
    int32_t amax_end[kMaxGroup], slot_end[kMaxGroup], copy_end[kMaxGroup];   // running workgroup totals per pass
    float near_tol;
    TensorOp op[kMaxGroup];
};
// Pass A also gathers a PROOF of the BF16 decision where one exists.  Section 4.1.3 observes that a
// per-tensor scale falls back as soon as ~2.4 % of the values flush to zero; each flushed non-zero
// element contributes exactly 1 to the error sum of Eq. (1)-(2), so "flushed >= th * N" already implies
// "mean relative error >= th".  An element certainly flushes when |x| < amax * 2^-20 (then
// |x * 448/amax| < 2^-11, below half of E4M3's smallest subnormal); with the lane's RUNNING amax in
// place of the final one the test only becomes stricter, so the count is a lower bound.  When the
// bound reaches flush_need, pass B writes the BF16 fallback in the same sweep and the separate copy
// pass (2 more bytes read per element) is skipped.  The outputs are the same either way.
// Workgroups from `stats_first` on do not belong to pass A: they compute the partial statistics records of the batch's
// sub-tensor operands (whose kernels have already run), in the shadow of this bandwidth-bound pass.
__global__ __launch_bounds__(256) void k_tensor_amax_group(GroupTensor g, GroupStats riders, int stats_first) {
    if ((int)blockIdx.x >= stats_first) { stats_partial_body(riders, (int)blockIdx.x - stats_first); return; }
    __shared__ uint32_t sh4[4];
    const int op = group_find32(g.amax_end, g.n, blockIdx.x);
    const TensorOp& t = g.op[op];
    const int b = blockIdx.x - (op ? g.amax_end[op - 1] : 0);
    const bool prove = t.flush_need != 0ull;
    const bool three = t.three != 0u;
    uint32_t a2 = 0u, keep2 = 0u, seen = 0u;      // keep2: per half-word count of elements NOT certain to flush
    uint32_t mn2 = 0xFFFFFFFFu;                   // three-way recipe: smallest non-zero pattern, minus one, per half-word
    for (int64_t tile = b; tile < t.n_tiles; tile += t.n_amax) {
        const int64_t c0 = tile * kTensorChunksPerBlock + threadIdx.x;
        if (c0 + 7 * 256 < t.n_chunks) {
            u32x4 v[8];
#pragma unroll
            for (int u = 0; u < 8; ++u) v[u] = load16(t.x + (c0 + u * 256) * 8);
#pragma unroll
            for (int u = 0; u < 8; ++u) a2 = amax2_of(v[u], a2);
            if (three) {
#pragma unroll
                for (int u = 0; u < 8; ++u) mn2 = min_nonzero_m1(v[u], mn2);
            }
            if (prove) {
                // t = running amax with 20 taken off the exponent (0 if that underflows); 1 <= m < t  <=>  m-1 < t-1
                const uint32_t t2 = pk_sub_sat_u16(a2, 0x0A000A00u);
                const uint32_t tm1 = pk_sub_sat_u16(t2, 0x00010001u);
#pragma unroll
                for (int u = 0; u < 8; ++u)
#pragma unroll
                    for (int j = 0; j < 4; ++j) {
                        const uint32_t mm1 = pk_sub_u16(v[u][j] & 0x7FFF7FFFu, 0x00010001u);     // wraps to 0xFFFF for zeros
                        keep2 = pk_add_u16(keep2, pk_is_zero_u16(pk_sub_sat_u16(tm1, mm1)));
                    }
                seen += 64u;
            }
        } else {
            for (int u = 0; u < 8; ++u)
                if (c0 + u * 256 < t.n_chunks) {
                    const u32x4 v = load16(t.x + (c0 + u * 256) * 8);
                    a2 = amax2_of(v, a2);
                    if (three) mn2 = min_nonzero_m1(v, mn2);
                }
        }
    }
    const uint32_t a = block_allmax_u32(fold_max16(a2), sh4);
    uint32_t mn = 0u;
    if (three) mn = block_allmin_u16(fold_min16(mn2), sh4);
    if (threadIdx.x == 0) t.amax_part[b] = a | (mn << 16);
    if (prove) {
        const uint32_t wf = wave_allsum_u32(seen - fold_add16(keep2));
        __syncthreads();
        if ((threadIdx.x & 63) == 0) sh4[threadIdx.x >> 6] = wf;
        __syncthreads();
        if (threadIdx.x == 0) t.flush_part[b] = (sh4[0] + sh4[1]) + (sh4[2] + sh4[3]);
    }
}
// Sum of the certain-flush lower bounds of an operand; same value in every workgroup that calls it.
__device__ __forceinline__ bool tensor_fallback_proven(const TensorOp& t, unsigned long long* shl) {
    if (t.flush_need == 0ull) return false;
    unsigned long long f = 0;
    for (int i = threadIdx.x; i < t.n_amax; i += 256) f += t.flush_part[i];
    f = block_sum_shfl<unsigned long long>(f, shl);
    return f >= t.flush_need;
}
template <int CRIT, bool FAKE>
__global__ __launch_bounds__(256) void k_tensor_quant_group(GroupTensor g) {
    __shared__ uint32_t sh4[4];
    const int op = group_find32(g.slot_end, g.n, blockIdx.x);
    const TensorOp& t = g.op[op];
    const int b = blockIdx.x - (op ? g.slot_end[op - 1] : 0);
    const uint16_t* __restrict__ x = t.x;
    uint8_t* __restrict__ fp8 = t.o.fp8;
    const int64_t n_chunks = t.n_chunks, n_tiles = t.n_tiles, G = t.n_slots;
    u32x4 bufA[kTensorChunksPerThread];
    auto load_tile = [&](u32x4* raw, int64_t tile) {
        const int64_t c0 = tile * kTensorChunksPerBlock + threadIdx.x;
#pragma unroll
        for (int u = 0; u < kTensorChunksPerThread; ++u) {
            const int64_t c = c0 + u * 256;
            if (c < n_chunks) raw[u] = load16(x + c * 8);
            else { raw[u].x = 0u; raw[u].y = 0u; raw[u].z = 0u; raw[u].w = 0u; }
        }
    };
    int64_t tl = b;
    load_tile(bufA, tl);
    __shared__ unsigned long long shl4[4];
    const uint32_t abits = global_amax_bits(t.amax_part, t.n_amax, sh4);
    const bool proven = tensor_fallback_proven(t, shl4);     // then the BF16 fallback is written in this sweep
    uint16_t* __restrict__ bf16 = t.o.bf16;
    if (b == 0 && threadIdx.x == 0) { t.abits[0] = abits; t.abits[1] = proven ? 1u : 0u; }
    // one block = the group: under GAM the block's own mantissa is the group mantissa and the scale is s_b
    const uint32_t mode = t.mode;
    const float s = block_scale(abits, kE4M3Max, mode, group_mantissa_bits(abits, kE4M3Max, mode));
    const float s5 = (CRIT == kCritEq3) ? block_scale(abits, kE5M2Max, mode, group_mantissa_bits(abits, kE5M2Max, mode)) : 0.0f;
    const bool fast = abits < fast_amax_limit(mode);
    const bool dual = CRIT == kCritEq3 && s5 == 128.0f * s;
    const bool emit = !(proven && t.lean != 0u);             // lean payload: the codes of a proven BF16 operand are not stored
    const float s_inv = FAKE ? 1.0f / s : 0.0f;
    uint16_t* __restrict__ fakep = t.o.fake;     // fake quantization: == bf16, so a proven fallback is already in place
    TensorAcc acc{0.0f, 0.0f, 0.0f, 0.0f, 0u};
    // Stores go through bounds-checked buffer windows over the tile (a tail tile's window is shorter; a payload that
    // is not wanted gets a null window), so the quantization sweep has no branches and stays one basic block: with
    // per-lane or per-operand branches around the stores the compiler defers the error terms of all eight chunks
    // and keeps their scaled values in registers.
    auto process = [&](const u32x4* raw, int64_t tile) {
        const int64_t c_first = tile * kTensorChunksPerBlock;
        const int64_t c0 = c_first + threadIdx.x;
        const int64_t left = n_chunks - c_first;
        const uint32_t valid = (uint32_t)(left < kTensorChunksPerBlock ? left : kTensorChunksPerBlock);      // chunks of this tile
        const BufRsrc r8 = make_buf_window(fp8 + c_first * 8, (FAKE || !emit) ? 0u : valid * 8u);
        const BufRsrc rb = make_buf_window(bf16 + c_first * 8, proven ? valid * 16u : 0u);
        const BufRsrc rf = make_buf_window(fakep + c_first * 8, (FAKE && !proven) ? valid * 16u : 0u);
        const uint32_t off8 = threadIdx.x * 8u, off16 = threadIdx.x * 16u;
#pragma unroll
        for (int u = 0; u < kTensorChunksPerThread; ++u) acc.zero2 = zero2_of(raw[u], acc.zero2);
        asm volatile("" : "+v"(acc.zero2));      // counted here, not sunk below the sweep (which would keep the masked words alive)
#pragma unroll
        for (int u = 0; u < kTensorChunksPerThread; ++u) buf_store16(rb, off16 + u * 4096u, raw[u]);       // proven fallback
        if (fast && FAKE && proven) {
            // fake quantization of an operand already proven to stay in BF16: the output is the input (stored above);
            // only the error sums are still needed
#pragma unroll
            for (int u = 0; u < kTensorChunksPerThread; ++u) {
                (void)quant8_fast<false>(raw[u], s, acc.e0, acc.e1);
                if constexpr (CRIT == kCritEq3) (void)quant8_fast<true>(raw[u], s5, acc.f0, acc.f1);
                __builtin_amdgcn_sched_barrier(0);
            }
        } else if (CRIT == kCritEq3 && fast && dual) {
            // both formats in one sweep with one reciprocal per element (see quant8_dual)
#pragma unroll
            for (int u = 0; u < kTensorChunksPerThread; ++u) {
                u32x4 deq;
                const u32x2 codes = quant8_dual<FAKE>(raw[u], s, s_inv, acc.e0, acc.e1, acc.f0, acc.f1, deq);
                if constexpr (FAKE) buf_store16(rf, off16 + u * 4096u, deq);
                else buf_store8(r8, off8 + u * 2048u, 0u, codes);
                __builtin_amdgcn_sched_barrier(0);
            }
        } else if (fast) {
#pragma unroll
            for (int u = 0; u < kTensorChunksPerThread; ++u) {
                u32x4 deq;
                const u32x2 codes = quant8_fast_deq<false, FAKE>(raw[u], s, s_inv, acc.e0, acc.e1, deq);
                if constexpr (FAKE) buf_store16(rf, off16 + u * 4096u, deq);
                else buf_store8(r8, off8 + u * 2048u, 0u, codes);
                if constexpr (CRIT == kCritEq3) (void)quant8_fast<true>(raw[u], s5, acc.f0, acc.f1);
                __builtin_amdgcn_sched_barrier(0);
            }
        } else {
#pragma clang loop unroll(disable)
            for (int u = 0; u < kTensorChunksPerThread; ++u) {
                const int64_t c = c0 + u * 256;
                if (c < n_chunks) {
                    acc.e0 += quant8_careful_mem<false>(x + c * 8, s, (FAKE || !emit) ? nullptr : fp8 + c * 8,
                                                        (FAKE && !proven) ? fakep + c * 8 : nullptr, s_inv);
                    if constexpr (CRIT == kCritEq3) acc.f0 += quant8_careful_mem<true>(x + c * 8, s5, nullptr);
                }
            }
        }
    };
    for (;;) {
        process(bufA, tl);
        tl += G;
        if (tl >= n_tiles) break;
        load_tile(bufA, tl);
    }
    TensorPartials tp{t.err, t.err5, t.zero, t.abits};
    tensor_publish<CRIT>(acc, tp, b);
}
// Workgroups from `stats_first` on combine the riders' partial statistics records (one workgroup per operand).
template <int CRIT>
__global__ __launch_bounds__(256) void k_tensor_finish_group(GroupTensor g, GroupStats riders, int stats_first) {
    if ((int)blockIdx.x >= stats_first) { stats_final_body(riders, (int)blockIdx.x - stats_first); return; }
    const int op = group_find32(g.copy_end, g.n, blockIdx.x);
    const TensorOp& t = g.op[op];
    const int b = blockIdx.x - (op ? g.copy_end[op - 1] : 0);
    const int nb = g.copy_end[op] - (op ? g.copy_end[op - 1] : 0);
    const bool proven = t.abits[1] != 0u;                     // pass B already wrote the fallback
    if (proven && b != 0) return;                             // only the operand's first workgroup has work left
    __shared__ double shd[4];
    __shared__ unsigned long long shl[4];
    double se = 0.0, se5 = 0.0;
    unsigned long long sz = 0;
    tensor_partial_sums<CRIT>(t.err, t.err5, t.zero, t.n_slots, se, se5, sz);
    se = block_sum_shfl<double>(se, shd);
    sz = block_sum_shfl<unsigned long long>(sz, shl);
    if constexpr (CRIT == kCritEq3) se5 = block_sum_shfl<double>(se5, shd);
    const uint32_t abits = t.abits[0];
    const unsigned long long n_padded = (unsigned long long)t.n_tiles * kTensorChunksPerBlock * 8;
    const unsigned long long n = n_padded - sz;
    if (abits >= kInfBits) { se = (double)__builtin_inff(); se5 = se; }
    uint32_t mask;
    if constexpr (CRIT == kCritEq3) mask = (se < se5) ? 0u : 1u;
    else mask = ((n ? se / (double)n : 0.0) < (double)t.th) ? 0u : 1u;
    const float s5 = block_scale(abits, kE5M2Max, t.mode, group_mantissa_bits(abits, kE5M2Max, t.mode));
    uint32_t amin_bits = 0u;
    if (t.three && mask == 1u) {           // Eq. (4): the operand is kept in E5M2 if its dynamic range fits
        __shared__ uint32_t sh4[4];
        amin_bits = global_amin_bits(t.amax_part, t.n_amax, sh4);
        if (range_fits_e5m2(abits, amin_bits, n ? 1u : 0u)) mask = 2u;
    }
    if (b == 0 && threadIdx.x == 0) {
        const KOut& o = t.o;
        const float err_f = (float)se;
        const uint32_t nnz32 = n > 0xFFFFFFFFull ? 0xFFFFFFFFu : (uint32_t)n;
        const uint32_t mg = group_mantissa_bits(abits, kE4M3Max, t.mode);
        const float s = mask == 2u ? s5 : block_scale(abits, kE4M3Max, t.mode, mg);
        if (t.three && o.amin) o.amin[0] = __uint_as_float(amin_bits << 16);
        o.scale[0] = s;
        if (t.mode != kScaleFp32 && o.e8m0) o.e8m0[0] = (uint8_t)(__float_as_uint(s) >> 23);
        if (t.mode != kScaleFp32 && o.gmant) { o.gmant[0] = mg; o.gmant[1] = group_mantissa_bits(abits, kE5M2Max, t.mode); }
        o.amax[0] = __uint_as_float(abits << 16);
        o.err_sum[0] = err_f;
        o.nnz[0] = nnz32;
        if constexpr (CRIT == kCritEq3) o.err5_sum[0] = (float)se5;
        o.mask[0] = (uint8_t)mask;
        if (t.stats) {     // statistics of a one-block operand, same arithmetic as k_stats_single
            StatsDev* st = t.stats;
            const float metric = nnz32 ? err_f / (float)nnz32 : 0.0f;
#pragma unroll
            for (int k = 0; k < 12; ++k) st->hist[k] = 0u;
            st->hist[stats_bin(metric)] = 1u;
            const bool near = fabs((double)metric - (double)t.th) <= (double)g.near_tol * (double)t.th;
            const unsigned long long total = (unsigned long long)t.n_chunks * 8ull;
            stats_finish(st, 1, total, (double)err_f, nnz32, mask == 1u ? 1ull : 0ull, near ? 1ull : 0ull, mask == 2u ? 1ull : 0ull,
                         mask == 1u ? total : 0ull, mask == 2u ? total : 0ull, proven ? 1u : 0u);
        }
    }
    if (mask == 2u) {
        const bool fast = abits < fast_amax_limit(t.mode);
        uint16_t* __restrict__ fakep = t.o.fake;
        const float s_inv = fakep ? 1.0f / s5 : 0.0f;
        for (int64_t c = (int64_t)b * 256 + threadIdx.x; c < t.n_chunks; c += (int64_t)nb * 256)
            requant_chunk_e5m2(t.x + c * 8, fakep ? nullptr : t.o.fp8 + c * 8, fakep ? fakep + c * 8 : nullptr, s5, s_inv, fast);
        return;
    }
    if (proven || mask == 0u || t.o.bf16 == nullptr) return;
    copy_chunk_tiles(t.x, t.o.bf16, t.n_chunks, b, nb);
}

// Group loop of Algorithm 1 for sub-tensor operands: the operand's amax (partials of pass A) gives the
// group mantissas for E4M3 and E5M2, which the block kernels read; also written to the caller's output.
// E8M0-only operands have no amax pass (n_amax = 0) and a zero mantissa.
struct GamOp {
    const uint32_t* amax_part; int n_amax;
    uint32_t mode;
    uint32_t* gam;         // [4] workspace words read by the block kernels: the two mantissas, then 1 if the pre-pass proved
                           // the tensor-level BF16 decision
    uint32_t* gmant;       // caller's group-mantissa output, may be nullptr
    const uint32_t* flush_part;          // [n_amax] certain flushes counted by the pre-pass, or nullptr
    unsigned long long flush_need;       // that many prove the decision
    uint32_t skip;                       // per-channel columns under GAM: their own combine kernel derives the mantissas
};
struct GroupGam {
    int n;
    GamOp op[kMaxGroup];
};
__global__ __launch_bounds__(256) void k_gam_prepare(GroupGam g) {
    __shared__ uint32_t sh4[4];
    __shared__ unsigned long long shl[4];
    const GamOp& t = g.op[blockIdx.x];
    if (t.skip) return;                  // uniform over the workgroup
    const uint32_t gbits = global_amax_bits(t.amax_part, t.n_amax, sh4);
    unsigned long long fl = 0ull;
    if (t.flush_part)
        for (int i = threadIdx.x; i < t.n_amax; i += 256) fl += t.flush_part[i];
    fl = block_sum_shfl<unsigned long long>(fl, shl);
    if (threadIdx.x == 0) {
        t.gam[2] = (t.flush_part && fl >= t.flush_need) ? 1u : 0u;
        const uint32_t mg = group_mantissa_bits(gbits, kE4M3Max, t.mode);
        t.gam[0] = mg;
        const uint32_t mg5 = group_mantissa_bits(gbits, kE5M2Max, t.mode);
        t.gam[1] = mg5;
        if (t.gmant) { t.gmant[0] = mg; t.gmant[1] = mg5; }
    }
}

// Group loop of Algorithm 1 with bands of rows as groups: workgroup (band, w) scans its share of the band's 16-byte chunks,
// then one lane per band turns the band's amax into its two mantissas (table behind the four header words of `gam`).
__global__ __launch_bounds__(256) void k_band_amax(const uint16_t* __restrict__ x, KShape sh, int64_t group_rows, int wpb,
                                                   uint32_t* __restrict__ part) {
    __shared__ uint32_t sh4[4];
    const int64_t band = blockIdx.x / wpb;
    const int w = blockIdx.x - (int)band * wpb;
    const int64_t r_first = band * group_rows;
    const int64_t n_rows = sh.rows - r_first < group_rows ? sh.rows - r_first : group_rows;
    const int64_t cpr = sh.cols / 8, n_chunks = n_rows * cpr;
    uint32_t a2 = 0u;
    for (int64_t c = (int64_t)w * 256 + threadIdx.x; c < n_chunks; c += (int64_t)wpb * 256) {
        const int64_t r = c / cpr, cc = c - r * cpr;
        a2 = amax2_of(load16(x + (r_first + r) * sh.ld + cc * 8), a2);
    }
    const uint32_t a = block_allmax_u32(fold_max16(a2), sh4);
    if (threadIdx.x == 0) part[blockIdx.x] = a;
}
__global__ __launch_bounds__(256) void k_gam_prepare_bands(const uint32_t* __restrict__ part, int wpb, int64_t n_groups,
                                                           uint32_t* __restrict__ gam, uint32_t* __restrict__ gmant) {
    const int64_t g = (int64_t)blockIdx.x * 256 + threadIdx.x;
    if (blockIdx.x == 0 && threadIdx.x < kGamHeaderWords) gam[threadIdx.x] = 0u;     // no single mantissa, nothing proven
    if (g >= n_groups) return;
    uint32_t a = 0u;
    for (int k = 0; k < wpb; ++k) a = max(a, part[g * wpb + k]);
    const uint32_t mg = group_mantissa_bits(a, kE4M3Max, kScaleGam), mg5 = group_mantissa_bits(a, kE5M2Max, kScaleGam);
    gam[kGamHeaderWords + 2 * g] = mg; gam[kGamHeaderWords + 2 * g + 1] = mg5;
    if (gmant) { gmant[2 * g] = mg; gmant[2 * g + 1] = mg5; }
}

// ======================================================================================
// Launchers
// ======================================================================================
static inline size_t align16(size_t v) { return (v + 15) & ~(size_t)15; }
// Workgroups per band of the band-amax pass: about 2048 in all, at most one per 8 KB of the band.
static int band_wgs(const BatchItem& it) {
    const int64_t n_groups = (it.sh.rows + it.group_rows - 1) / it.group_rows;
    int64_t per = 2048 / n_groups, cap = (it.group_rows * it.sh.cols + 4095) / 4096;
    if (per > cap) per = cap;
    return (int)(per < 1 ? 1 : per);
}


TensorPlan plan_tensor(int64_t, int64_t) {
    TensorPlan pl;
    pl.amax_blocks = kMaxAmaxBlocks;
    pl.quant_blocks = kMaxQuantBlocks;
    size_t off = 0;
    pl.off_amax_part = off; off = align16(off + sizeof(uint32_t) * (size_t)pl.amax_blocks);
    pl.off_err_part = off;  off = align16(off + sizeof(float) * (size_t)pl.quant_blocks);
    pl.off_err5_part = off; off = align16(off + sizeof(float) * (size_t)pl.quant_blocks);
    pl.off_nnz_part = off;  off = align16(off + sizeof(uint32_t) * (size_t)pl.quant_blocks);   // zero counts
    pl.off_decision = off;  off = align16(off + 16);                                           // [0] global amax bits
    pl.off_flush_part = off; off = align16(off + sizeof(uint32_t) * (size_t)pl.amax_blocks);   // certain-flush lower bounds
    pl.bytes = off;
    return pl;
}

size_t scope_workspace_bytes(int64_t) { return align16(3 * sizeof(double) * kScopeBlocks + 16); }

static bool is_flat(const KShape& sh, const KOut& o) {
    return sh.ld == sh.cols && o.ld_fp8 == sh.cols && (o.bf16 == nullptr || o.ld_bf16 == sh.cols) &&
           (o.fake == nullptr || o.ld_fake == sh.cols);
}
constexpr int64_t kSubRiderMaxUnits = 16384;  // 1x128 operands of at most 128 MiB ride on a team launch; larger ones run faster uncapped
constexpr int64_t kSubFlatMaxBlocks = 1536;   // workgroups of 4 waves, each wave strides over 8 KB units: 6 per compute unit is what the kernel's
                                              // registers let be resident, so no workgroup waits for another to end (one 64 MiB operand, cold
                                              // caches: 21.0 us at 1536 against 23.2 us at 2048 (one unit per wave); 112 MiB: 32.1 against 34.5 us;
                                              // 224 MiB: 65 us either way)
static_assert(kSubFlatMaxBlocks <= 2 * kSoloFinalThreads, "k_solo_stats_final takes two records per lane");
static int clamp_grid_y(int64_t v) { return (int)(v < 1 ? 1 : (v > 65535 ? 65535 : v)); }

// The general 1 x 128 kernel: one operand per launch.
template <int CRIT>
static void launch_sub1x128_crit(const dim3& grid, const uint16_t* x, const KShape& sh, const KOut& o, bool defer, float th,
                                 uint32_t mode, const uint32_t* gam, uint32_t three, uint32_t group_rows, hipStream_t st) {
    const bool fake = o.fake != nullptr;
    if (defer) {
        if (fake) k_sub1x128_strided<CRIT, true, true><<<grid, dim3(256), 0, st>>>(x, sh, o, th, mode, gam, three, group_rows);
        else k_sub1x128_strided<CRIT, true, false><<<grid, dim3(256), 0, st>>>(x, sh, o, th, mode, gam, three, group_rows);
    } else {
        if (fake) k_sub1x128_strided<CRIT, false, true><<<grid, dim3(256), 0, st>>>(x, sh, o, th, mode, gam, three, group_rows);
        else k_sub1x128_strided<CRIT, false, false><<<grid, dim3(256), 0, st>>>(x, sh, o, th, mode, gam, three, group_rows);
    }
}
static hipError_t launch_sub1x128(const uint16_t* x, const KShape& sh, const KOut& o, int crit, bool defer, float th, uint32_t mode,
                                  const uint32_t* gam, uint32_t three, uint32_t group_rows, hipStream_t st, KProf* prof) {
    ProfScope ps(prof, kKernSub1x128, st);
    const dim3 grid((unsigned)((sh.cols + 127) / 128), (unsigned)clamp_grid_y((sh.rows + 15) / 16));
    if (crit == kCritEq3) launch_sub1x128_crit<kCritEq3>(grid, x, sh, o, defer, th, mode, gam, three, group_rows, st);
    else launch_sub1x128_crit<kCritEq2>(grid, x, sh, o, defer, th, mode, gam, three, group_rows, st);
    return hipGetLastError();
}

static hipError_t launch_tensor(const uint16_t* x, const KShape& sh, const KOut& o, int crit, float th, uint32_t mode, uint32_t three,
                                void* ws, hipStream_t st, KProf* prof) {
    const TensorPlan pl = plan_tensor(sh.rows, sh.cols);
    char* w = static_cast<char*>(ws);
    uint32_t* amax_part = reinterpret_cast<uint32_t*>(w + pl.off_amax_part);
    TensorPartials tp{reinterpret_cast<float*>(w + pl.off_err_part), reinterpret_cast<float*>(w + pl.off_err5_part),
                      reinterpret_cast<uint32_t*>(w + pl.off_nnz_part), reinterpret_cast<uint32_t*>(w + pl.off_decision)};
    const int n_amax = (int)(sh.rows < kMaxAmaxBlocks ? sh.rows : kMaxAmaxBlocks);
    { ProfScope ps(prof, kKernTensorAmax, st); k_tensor_amax_strided<<<dim3(n_amax), dim3(256), 0, st>>>(x, sh, amax_part, three); }
    const int64_t gx = (sh.cols + 127) / 128, gy = (sh.rows + 15) / 16;
    if (gx * gy > 0x7FFFFFFF) return hipErrorInvalidValue;
    // 16-bit zero counters per lane: at most 8 zeros per tile and lane, so 4096 tiles per workgroup are safe
    const int64_t min_blocks = (gx * gy + 4095) / 4096;
    if (min_blocks > kMaxQuantBlocks) return hipErrorInvalidValue;
    const int n_slots = (int)(gx * gy < kMaxQuantBlocks ? gx * gy : kMaxQuantBlocks);
    const unsigned long long n_padded = (unsigned long long)(gx * gy) * 2048ull;
    {
        ProfScope ps(prof, kKernTensorQuant, st);
        const uint32_t tx = (uint32_t)gx, nt = (uint32_t)(gx * gy);
        if (o.fake) {
            if (crit == kCritEq3) k_tensor_quant_strided<kCritEq3, true><<<dim3(n_slots), dim3(256), 0, st>>>(x, sh, tx, nt, o, amax_part, n_amax, tp, mode);
            else k_tensor_quant_strided<kCritEq2, true><<<dim3(n_slots), dim3(256), 0, st>>>(x, sh, tx, nt, o, amax_part, n_amax, tp, mode);
        } else {
            if (crit == kCritEq3) k_tensor_quant_strided<kCritEq3, false><<<dim3(n_slots), dim3(256), 0, st>>>(x, sh, tx, nt, o, amax_part, n_amax, tp, mode);
            else k_tensor_quant_strided<kCritEq2, false><<<dim3(n_slots), dim3(256), 0, st>>>(x, sh, tx, nt, o, amax_part, n_amax, tp, mode);
        }
    }
    {
        ProfScope ps(prof, kKernFallbackCopy, st);
        const int grid = (o.bf16 || three) ? 2048 : 1;
        const int flat = (sh.ld == sh.cols && o.ld_bf16 == sh.cols) ? 1 : 0;
        if (crit == kCritEq3) k_tensor_finish<kCritEq3><<<dim3(grid), dim3(256), 0, st>>>(tp, n_slots, n_padded, o, th, x, sh, flat, mode, three, amax_part, n_amax);
        else k_tensor_finish<kCritEq2><<<dim3(grid), dim3(256), 0, st>>>(tp, n_slots, n_padded, o, th, x, sh, flat, mode, three, amax_part, n_amax);
    }
    return hipGetLastError();
}

// ---- batches ---------------------------------------------------------------------------------
namespace {
constexpr int kStatsMaxWg = 256;

// Which kernels take an operand.
enum Route {
    kRouteTensorGroup,      // per-tensor, dense: grouped three-pass kernels
    kRouteTensorStrided,    // per-tensor, padded leading dimensions
    kRouteSubFlat,          // 1 x 128, dense, whole blocks, two types, FP8 payload: the persistent grouped kernel
    kRouteSubGeneral,       // 1 x 128, everything else
    kRouteTeam,             // 128 x 128, 64 x 64, per-channel rows: a team of lanes keeps the block in registers
    kRouteSubCol,           // 128 x 1
    kRouteChannelCol        // per-channel columns
};
bool item_is_flat(const BatchItem& it) { return is_flat(it.sh, it.o); }
Route route_of(const BatchItem& it) {
    const bool plain = !it.three;
    switch (it.gran) {
    case kGranTensor: return item_is_flat(it) ? kRouteTensorGroup : kRouteTensorStrided;
    case kGranSub:      // (with bands of rows as GAM groups the flat kernel takes whole 32-block units only: no renumbered tail)
        return (plain && item_is_flat(it) && it.sh.cols % 128 == 0 && (it.group_rows == 0 || (it.sh.rows * (it.sh.cols / 128)) % 32 == 0))
                   ? kRouteSubFlat : kRouteSubGeneral;
    case kGranBlock: case kGranBlock64: case kGranRow: return kRouteTeam;
    case kGranSubCol: return kRouteSubCol;
    default: return kRouteChannelCol;
    }
}
int64_t item_parts(const BatchItem& it) { return geom_parts(make_geom(it.gran, it.sh.rows, it.sh.cols)); }
// A dense 1 x 128 operand of whole 32-block units whose blocks are decided one by one can gather its statistics in its own
// kernel (k_sub1x128_solo_stats) when it is alone in its launch and the batch has no per-tensor launch they could ride on.
bool solo_stats_candidate(const BatchItem& it) {
    return it.stats && it.scope == 0 && route_of(it) == kRouteSubFlat && item_parts(it) % 32 == 0;
}
int stats_wgs(int64_t n_part) {                        // riding in a launch of 256-lane workgroups
    if (n_part <= 4096) return 1;                       // one workgroup writes the result directly
    int64_t w = (n_part + 1023) / 1024;
    return (int)(w > kStatsMaxWg ? kStatsMaxWg : w);
}
int stats_wgs_fast(int64_t n_part) {                   // launch of its own: workgroups of kStatsFastThreads lanes
    if (n_part <= kStatsDirectParts) return 1;
    int64_t w = (n_part + kStatsFastThreads * kStatsFastPerLane - 1) / (kStatsFastThreads * kStatsFastPerLane);
    return (int)(w > kStatsMaxWg ? kStatsMaxWg : w);
}
size_t item_workspace(const BatchItem& it) {
    size_t b = 0;
    if (it.gran == kGranTensor) b += plan_tensor(it.sh.rows, it.sh.cols).bytes;
    else if (it.scope == 1) b += scope_workspace_bytes(item_parts(it));
    if (it.gran == kGranCol) b += column_workspace_bytes(it.sh.rows, it.sh.cols);
    if (it.stats && it.gran != kGranTensor) b += align16(sizeof(StatsRec) * (solo_stats_candidate(it) ? kSubFlatMaxBlocks : kStatsMaxWg));
    if (it.gran != kGranTensor && it.scaling != kScaleFp32) {
        b += 16;                                                                   // group mantissa words
        if (it.scaling == kScaleGam && it.group_rows == 0) b += 2 * align16(sizeof(uint32_t) * kProveMaxWg);   // amax and flush partials of the pre-pass
        if (it.scaling == kScaleGam && it.group_rows != 0) {                       // bands of rows as groups: mantissa table, amax partials
            const size_t n_groups = (size_t)((it.sh.rows + it.group_rows - 1) / it.group_rows);
            b += align16(8 * n_groups) + align16(sizeof(uint32_t) * n_groups * (size_t)band_wgs(it));
        }
    }
    return b;
}
int share(int64_t mine, int64_t total, int budget, int64_t cap) {
    int64_t v = total > 0 ? (mine * budget + total - 1) / total : 1;
    if (v > cap) v = cap;
    if (v > budget) v = budget;
    return (int)(v < 1 ? 1 : v);
}
constexpr int kMaxGroupTensor = 8;
}  // namespace

size_t batch_workspace_bytes(const BatchItem* items, int n) {
    size_t b = 0;
    for (int i = 0; i < n; ++i) b += item_workspace(items[i]);
    return b;
}

namespace {
// One batch call: the launches of every phase, in stream order.  The phases share the workspace cursor, the routes, the
// group-mantissa words of Algorithm 1 and the statistics groups, which is all this object holds.
constexpr int kMaxStatsGroups = (kBatchMax + kMaxGroupStats - 1) / kMaxGroupStats;
struct BatchRun {
    const BatchItem* items;
    int n;
    float near_tol;
    hipStream_t st;
    KProf* prof;
    char* wsp;
    size_t ws_off = 0;
    hipError_t err = hipSuccess;
    Route route[kBatchMax];
    const uint32_t* gam_of[kBatchMax] = {};      // per operand: {mantissa for E4M3, for E5M2, "BF16 proven" flag}
    char* col_ws[kBatchMax] = {};                // per operand with per-channel columns: its column workspace
    GroupStats stats_groups[kMaxStatsGroups];
    int n_stats_groups = 0;
    bool will_ride = false;                      // the batch has grouped per-tensor launches for statistics to ride on
    bool riders_used = false;                    // the first statistics group went along with a per-tensor launch
    bool stats_done[kBatchMax] = {};             // the operand's block kernel has written its statistics already

    size_t ws_bytes = 0;
    // Next `bytes` of the caller's workspace.  The phases below carve exactly what item_workspace() adds up; should the
    // two ever drift apart, the call fails (hipErrorOutOfMemory) instead of writing beyond the workspace: once `err`
    // is set no further kernel is launched, so the pointer returned here is never dereferenced.
    char* carve(size_t bytes) {
        const size_t need = align16(bytes);
        if (err != hipSuccess || need > ws_bytes - ws_off) { if (err == hipSuccess) err = hipErrorOutOfMemory; return wsp; }
        char* p = wsp + ws_off;
        ws_off += need;
        return p;
    }
    void group_mantissas();
    void sub_tensor_operands(int crit);
    void tensor_level_decisions();
    void collect_statistics();
    void per_tensor_operands(int crit);
    void leftover_statistics();
};

// ---- Algorithm 1, group loop: operands with sub-tensor blocks and GAM / E8M0 scaling get their group
//      mantissas first (GAM: one more read of the operand for its amax)
void BatchRun::group_mantissas() {
    int idx[kBatchMax];
    int cnt = 0;
    for (int i = 0; i < n; ++i)
        if (items[i].gran != kGranTensor && items[i].scaling != kScaleFp32 && items[i].group_rows == 0) idx[cnt++] = i;
    // operands whose groups are bands of rows: one mantissa pair per band, in a table behind the four header words
    for (int i = 0; i < n && err == hipSuccess; ++i) {
        const BatchItem& it = items[i];
        if (it.group_rows == 0) continue;
        const int64_t n_groups = (it.sh.rows + it.group_rows - 1) / it.group_rows;
        const int wpb = band_wgs(it);
        if (n_groups * wpb > 0x7FFFFFFF) { err = hipErrorInvalidValue; return; }
        uint32_t* gam = reinterpret_cast<uint32_t*>(carve(16 + align16(8 * (size_t)n_groups)));
        uint32_t* part = reinterpret_cast<uint32_t*>(carve(sizeof(uint32_t) * (size_t)n_groups * (size_t)wpb));
        if (err != hipSuccess) return;
        gam_of[i] = gam;
        { ProfScope ps(prof, kKernGroupAmax, st); k_band_amax<<<dim3((unsigned)(n_groups * wpb)), dim3(256), 0, st>>>(it.x, it.sh, it.group_rows, wpb, part); }
        { ProfScope ps(prof, kKernGroupMantissa, st); k_gam_prepare_bands<<<dim3((unsigned)((n_groups + 255) / 256)), dim3(256), 0, st>>>(part, wpb, n_groups, gam, it.o.gmant); }
    }
    // operands whose tensor-level decision the pre-pass may prove: block-shaped pre-pass (group amax and, per block,
    // the elements that are certain to flush), as many operands per launch as its argument table holds
    uint32_t* pv_part[kBatchMax] = {};
    uint32_t* pv_flush[kBatchMax] = {};
    int pv_wg[kBatchMax] = {};
    {
        constexpr int kProveGroup = 12;
        BlockProveItem pv[kProveGroup];
        int pv_item[kProveGroup];
        int n_pv = 0;
        int64_t pv_units = 0;
        auto flush = [&]() {
            if (n_pv == 0 || err != hipSuccess) { n_pv = 0; pv_units = 0; return; }
            for (int j = 0; j < n_pv; ++j) {
                const int64_t units = scope_proof_units(items[pv_item[j]]);
                // twelve operands, 128x128: 0.577 ms per pass at 2048 workgroups in all, 0.564 ms at 4096 and at 8192
                pv[j].n_wg = share(units, pv_units, kProveMaxWg, units);
                pv_wg[pv_item[j]] = pv[j].n_wg;
            }
            ProfScope ps(prof, kKernGroupAmax, st);
            err = launch_block_amax_prove(pv, n_pv, st);
            n_pv = 0; pv_units = 0;
        };
        for (int k = 0; k < cnt && err == hipSuccess; ++k) {
            const int i = idx[k];
            const BatchItem& it = items[i];
            if (!scope_proof_applies(it)) continue;
            pv_part[i] = reinterpret_cast<uint32_t*>(carve(sizeof(uint32_t) * kProveMaxWg));
            pv_flush[i] = reinterpret_cast<uint32_t*>(carve(sizeof(uint32_t) * kProveMaxWg));
            pv[n_pv] = BlockProveItem{it.x, it.sh.rows, it.sh.cols, it.sh.ld, pv_part[i], pv_flush[i], 0, scope_proof_kind(it)};
            pv_units += scope_proof_units(it);
            pv_item[n_pv] = i;
            if (++n_pv == kProveGroup) flush();
        }
        flush();
    }
    for (int base = 0; base < cnt && err == hipSuccess; base += kMaxGroupTensor) {
        const int m = cnt - base < kMaxGroupTensor ? cnt - base : kMaxGroupTensor;
        GroupGam gg; gg.n = m;
        GroupTensor ga; ga.n = 0; ga.near_tol = near_tol;
        int slot_of[kMaxGroupTensor];
        int64_t total_tiles = 0;
        for (int k = 0; k < m; ++k) {
            const int i = idx[base + k];
            const BatchItem& it = items[i];
            uint32_t* gam = reinterpret_cast<uint32_t*>(carve(16));
            gam_of[i] = gam;
            GamOp& q = gg.op[k];
            q.amax_part = nullptr; q.n_amax = 0; q.mode = (uint32_t)it.scaling; q.gam = gam; q.gmant = it.o.gmant;
            q.flush_part = nullptr; q.flush_need = 0ull; q.skip = 0u;
            slot_of[k] = -1;
            if (it.scaling != kScaleGam) continue;
            if (it.gran == kGranCol) { q.skip = 1u; continue; }      // the group amax comes out of the column-amax pass
            if (pv_part[i]) {
                q.amax_part = pv_part[i]; q.n_amax = pv_wg[i];
                q.flush_part = pv_flush[i];
                q.flush_need = flush_need_of(it.th, it.sh.rows * it.sh.cols);
                continue;
            }
            uint32_t* part = reinterpret_cast<uint32_t*>(carve(2 * sizeof(uint32_t) * kProveMaxWg));
            q.amax_part = part;
            if (it.sh.ld == it.sh.cols) {
                TensorOp& t = ga.op[ga.n];
                t = TensorOp{};
                t.x = it.x;
                t.n_chunks = it.sh.rows * it.sh.cols / 8;
                t.n_tiles = (t.n_chunks + kTensorChunksPerBlock - 1) / kTensorChunksPerBlock;
                t.amax_part = part;
                total_tiles += t.n_tiles;
                slot_of[k] = ga.n++;
            } else if (err == hipSuccess) {
                q.n_amax = (int)(it.sh.rows < kMaxAmaxBlocks ? it.sh.rows : kMaxAmaxBlocks);
                ProfScope ps(prof, kKernGroupAmax, st);
                k_tensor_amax_strided<<<dim3(q.n_amax), dim3(256), 0, st>>>(it.x, it.sh, part, 0u);
            }
        }
        int a_end = 0;
        for (int j = 0; j < ga.n; ++j) {
            TensorOp& t = ga.op[j];
            t.n_amax = share(t.n_tiles, total_tiles, kMaxAmaxBlocks, t.n_tiles);
            a_end += t.n_amax;
            ga.amax_end[j] = a_end;
        }
        for (int k = 0; k < m; ++k)
            if (slot_of[k] >= 0) gg.op[k].n_amax = ga.op[slot_of[k]].n_amax;
        if (err != hipSuccess) return;
        if (ga.n) {
            GroupStats none; none.n = 0; none.near_tol = near_tol;
            ProfScope ps(prof, kKernGroupAmax, st);
            k_tensor_amax_group<<<dim3(a_end), dim3(256), kResidency3, st>>>(ga, none, a_end);
        }
        { ProfScope ps(prof, kKernGroupMantissa, st); k_gam_prepare<<<dim3(m), dim3(256), 0, st>>>(gg); }
    }
}

// ---- operands with sub-tensor blocks of one criterion
void BatchRun::sub_tensor_operands(int crit) {
    // ---- small flat 1x128 operands ride on the first 128x128 team launch of the same criterion and output kind
    // (extra workgroups of that launch) instead of paying the ramp and tail of a launch of their own
    TeamRiders riders;
    riders.table.n = 0; riders.blocks = 0; riders.fake = false; riders.used = false;
    int64_t rider_units = 0;
    bool team_has[2] = {false, false};
    for (int i = 0; i < n; ++i)
        if (route[i] == kRouteTeam && items[i].crit == crit && team_kind_of(items[i]) == 0) team_has[items[i].o.fake ? 1 : 0] = true;
    // ---- 1x128 sub-channel operands, persistent grouped kernel (FP8 payload, then fake quantization)
    for (int fake = 0; fake < 2 && err == hipSuccess; ++fake) {
        GroupSub g; g.n = 0;
        int64_t total = 0;
        int newest = -1;                                  // the item added to the table last
        auto flush = [&]() {
            if (g.n == 0 || err != hipSuccess) { g.n = 0; total = 0; return; }
            int64_t blocks = (total + 3) / 4;
            if (blocks > kSubFlatMaxBlocks) blocks = kSubFlatMaxBlocks;
            if (g.n == 1 && !will_ride && solo_stats_candidate(items[newest])) {
                // a lone operand: its kernel gathers the statistics as well
                SoloStats ss;
                ss.rec = reinterpret_cast<StatsRec*>(carve(sizeof(StatsRec) * (size_t)blocks));
                ss.out = static_cast<StatsDev*>(items[newest].stats);
                ss.n_part = item_parts(items[newest]);
                ss.near_tol = near_tol;
                ss.n_rec = (int)blocks;
                if (err != hipSuccess) { g.n = 0; total = 0; return; }
                SubRiders one; one.n = 1;
                one.unit_end[0] = g.unit_end[0]; one.x[0] = g.x[0]; one.o[0] = g.o[0]; one.th[0] = g.th[0]; one.defer[0] = g.defer[0];
                one.mode[0] = g.mode[0]; one.prove[0] = g.prove[0]; one.gam[0] = g.gam[0]; one.group_rows[0] = g.group_rows[0]; one.bpr[0] = g.bpr[0];
                {
                    ProfScope ps(prof, kKernSub1x128, st);
                    const dim3 grid((unsigned)blocks);
                    if (fake) {
                        if (crit == kCritEq3) k_sub1x128_solo_stats<kCritEq3, true><<<grid, dim3(256), 0, st>>>(one, ss);
                        else k_sub1x128_solo_stats<kCritEq2, true><<<grid, dim3(256), 0, st>>>(one, ss);
                    } else {
                        if (crit == kCritEq3) k_sub1x128_solo_stats<kCritEq3, false><<<grid, dim3(256), 0, st>>>(one, ss);
                        else k_sub1x128_solo_stats<kCritEq2, false><<<grid, dim3(256), 0, st>>>(one, ss);
                    }
                }
                { ProfScope ps2(prof, kKernStatsFinal, st); k_solo_stats_final<<<dim3(1), dim3(kSoloFinalThreads), 0, st>>>(ss); }
                stats_done[newest] = true;
                g.n = 0; total = 0;
                return;
            }
            ProfScope ps(prof, kKernSub1x128, st);
            if (fake) {
                if (crit == kCritEq3) k_sub1x128_group<kCritEq3, true><<<dim3((unsigned)blocks), dim3(256), 0, st>>>(g);
                else k_sub1x128_group<kCritEq2, true><<<dim3((unsigned)blocks), dim3(256), 0, st>>>(g);
            } else {
                if (crit == kCritEq3) k_sub1x128_group<kCritEq3, false><<<dim3((unsigned)blocks), dim3(256), 0, st>>>(g);
                else k_sub1x128_group<kCritEq2, false><<<dim3((unsigned)blocks), dim3(256), 0, st>>>(g);
            }
            g.n = 0; total = 0;
        };
        for (int i = 0; i < n; ++i) {
            const BatchItem& it = items[i];
            if (route[i] != kRouteSubFlat || it.crit != crit || (it.o.fake != nullptr) != (fake != 0)) continue;
            const int64_t n_part = item_parts(it), n_units = n_part / 32, n_full = n_units * 32, n_tail = n_part - n_full;
            if (n_units > 0 && n_units <= kSubRiderMaxUnits && team_has[fake] && riders.table.n < kMaxSubRiders &&
                (riders.table.n == 0 || riders.fake == (fake != 0))) {
                SubRiders& r = riders.table;
                rider_units += n_units;
                r.unit_end[r.n] = rider_units; r.x[r.n] = it.x; r.o[r.n] = it.o; r.th[r.n] = it.th; r.defer[r.n] = it.scope == 1;
                r.mode[r.n] = (uint8_t)it.scaling; r.gam[r.n] = gam_of[i]; r.prove[r.n] = scope_proof_applies(it) ? 1 : 0;
                r.group_rows[r.n] = (uint32_t)it.group_rows; r.bpr[r.n] = (uint32_t)(it.sh.cols / 128);
                ++r.n;
                riders.fake = fake != 0;
                riders.blocks = (rider_units + 3) / 4 < kSubFlatMaxBlocks ? (rider_units + 3) / 4 : kSubFlatMaxBlocks;
            } else if (n_units > 0) {
                total += n_units;
                g.unit_end[g.n] = total; g.x[g.n] = it.x; g.o[g.n] = it.o; g.th[g.n] = it.th; g.defer[g.n] = it.scope == 1;
                g.mode[g.n] = (uint8_t)it.scaling; g.gam[g.n] = gam_of[i]; g.prove[g.n] = scope_proof_applies(it) ? 1 : 0;
                g.group_rows[g.n] = (uint32_t)it.group_rows; g.bpr[g.n] = (uint32_t)(it.sh.cols / 128);
                newest = i;
                if (++g.n == kMaxGroupSub) flush();
            }
            if (n_tail > 0) {     // fewer than 32 blocks left: the general kernel takes them
                KShape ts{n_tail, 128, 128};
                KOut to = it.o;
                if (to.fp8) to.fp8 += n_full * 128;
                to.ld_fp8 = 128;
                if (to.fake) { to.fake += n_full * 128; to.ld_fake = 128; }
                if (to.bf16) to.bf16 += n_full * 128;
                to.ld_bf16 = 128;
                to.scale += n_full; to.amax += n_full; to.err_sum += n_full; to.nnz += n_full; to.mask += n_full;
                if (to.err5_sum) to.err5_sum += n_full;
                if (to.e8m0) to.e8m0 += n_full;
                // (the tail's rows are renumbered from 0; an operand with bands of rows as GAM groups has no tail, see route_of)
                if (err == hipSuccess) err = launch_sub1x128(it.x + n_full * 128, ts, to, crit, it.scope == 1, it.th, (uint32_t)it.scaling, gam_of[i], 0u, 0u, st, nullptr);
            }
        }
        flush();
    }
    // ---- 1x128 sub-channel operands, general kernel
    for (int i = 0; i < n && err == hipSuccess; ++i) {
        const BatchItem& it = items[i];
        if (route[i] != kRouteSubGeneral || it.crit != crit) continue;
        err = launch_sub1x128(it.x, it.sh, it.o, crit, it.scope == 1, it.th, (uint32_t)it.scaling, gam_of[i], (uint32_t)it.three,
                              (uint32_t)it.group_rows, st, prof);
    }
    // ---- team kernels: 128x128 and 64x64 blocks, per-channel rows
    for (int kind = 0; kind < kTeamKinds && err == hipSuccess; ++kind) {
        int idx[kBatchMax];
        int cnt = 0;
        for (int i = 0; i < n; ++i)
            if (route[i] == kRouteTeam && items[i].crit == crit && team_kind_of(items[i]) == kind) idx[cnt++] = i;
        if (cnt) err = launch_team_items(items, idx, cnt, kind, crit, gam_of, &riders, st, prof);
    }
    if (err == hipSuccess && riders.table.n > 0 && !riders.used) {      // no team launch took them: a launch of their own
        GroupSub g; g.n = riders.table.n;
        for (int k = 0; k < g.n; ++k) {
            const SubRiders& r = riders.table;
            g.unit_end[k] = r.unit_end[k]; g.x[k] = r.x[k]; g.o[k] = r.o[k]; g.th[k] = r.th[k]; g.defer[k] = r.defer[k];
            g.mode[k] = r.mode[k]; g.gam[k] = r.gam[k]; g.prove[k] = r.prove[k]; g.group_rows[k] = r.group_rows[k]; g.bpr[k] = r.bpr[k];
        }
        ProfScope ps(prof, kKernSub1x128, st);
        const dim3 grid((unsigned)riders.blocks);
        if (riders.fake) {
            if (crit == kCritEq3) k_sub1x128_group<kCritEq3, true><<<grid, dim3(256), 0, st>>>(g);
            else k_sub1x128_group<kCritEq2, true><<<grid, dim3(256), 0, st>>>(g);
        } else {
            if (crit == kCritEq3) k_sub1x128_group<kCritEq3, false><<<grid, dim3(256), 0, st>>>(g);
            else k_sub1x128_group<kCritEq2, false><<<grid, dim3(256), 0, st>>>(g);
        }
        riders.used = true;
    }
    // ---- 128x1 sub-columns
    if (err == hipSuccess) {
        int idx[kBatchMax];
        int cnt = 0;
        for (int i = 0; i < n; ++i)
            if (route[i] == kRouteSubCol && items[i].crit == crit) idx[cnt++] = i;
        if (cnt) err = launch_subcol_items(items, idx, cnt, crit, gam_of, st, prof);
    }
    // ---- per-channel columns
    if (err == hipSuccess) {
        int idx[kBatchMax];
        char* ws_of[kBatchMax];
        int cnt = 0;
        for (int i = 0; i < n; ++i)
            if (route[i] == kRouteChannelCol && items[i].crit == crit) {
                ws_of[cnt] = carve(column_workspace_bytes(items[i].sh.rows, items[i].sh.cols));
                col_ws[i] = ws_of[cnt];
                idx[cnt++] = i;
            }
        if (cnt && err == hipSuccess) err = launch_channel_col_items(items, idx, cnt, crit, gam_of, ws_of, st, prof);
    }
}

// ---- tensor-level decision (Section 3.1) over the per-block sums the block kernels left behind
void BatchRun::tensor_level_decisions() {
    GroupScope g; g.n = 0;
    int red = 0, copy = 0;
    auto flush = [&]() {
        if (g.n == 0 || err != hipSuccess) { g.n = 0; red = 0; copy = 0; return; }
        { ProfScope ps(prof, kKernScopeReduce, st); k_scope_reduce_group<<<dim3(red), dim3(256), 0, st>>>(g); }
        { ProfScope ps(prof, kKernFallbackCopy, st); k_scope_copy_group<<<dim3(copy), dim3(256), 0, st>>>(g); }
        g.n = 0; red = 0; copy = 0;
    };
    int64_t total_elems = 0;
    for (int i = 0; i < n; ++i)
        if (items[i].gran != kGranTensor && items[i].scope == 1) total_elems += items[i].sh.rows * items[i].sh.cols;
    for (int i = 0; i < n; ++i) {
        const BatchItem& it = items[i];
        if (it.gran == kGranTensor || it.scope != 1) continue;
        ScopeOp& t = g.op[g.n];
        char* w = carve(scope_workspace_bytes(0));
        t.err_sum = it.o.err_sum; t.err5_sum = it.o.err5_sum; t.nnz = it.o.nnz; t.mask = it.o.mask;
        t.n_part = item_parts(it);
        t.part_err = reinterpret_cast<double*>(w); t.part_err5 = t.part_err + kScopeBlocks;
        t.part_nnz = reinterpret_cast<unsigned long long*>(w) + 2 * kScopeBlocks;
        t.decision = reinterpret_cast<uint32_t*>(w + 3 * sizeof(double) * kScopeBlocks);
        t.th = it.th; t.crit = it.crit;
        t.proven = scope_proof_applies(it) ? gam_of[i] + 2 : nullptr;
        if (column_tensor_proof_applies(it)) t.proven = column_tensor_proven_word(col_ws[i], it.sh.rows, it.sh.cols);
        int64_t want = (t.n_part + 1023) / 1024;
        t.n_red = (int)(want < 1 ? 1 : (want > kScopeBlocks ? kScopeBlocks : want));
        t.x = it.x; t.bf16 = it.o.bf16;
        t.rows = it.sh.rows; t.cols = it.sh.cols; t.ld = it.sh.ld; t.ld_bf16 = it.o.ld_bf16;
        red += t.n_red;
        {   // workgroups of the decision / mask / copy launch: enough for the copy, and never fewer than the reduce pass had
            const int c = it.o.bf16 ? share(it.sh.rows * it.sh.cols, total_elems, 4096, 4096) : 1;
            copy += c > t.n_red ? c : t.n_red;
        }
        g.red_end[g.n] = red; g.copy_end[g.n] = copy;
        if (++g.n == kMaxGroupScope) flush();
    }
    flush();
}

// ---- statistics of the operands with sub-tensor blocks: their kernels (and tensor-level decisions) are done, so the
//      first group can ride on the first per-tensor launches: partial records in the shadow of pass A, the combine
//      step next to the finish pass.  Groups that find no such launch run on their own at the end.
void BatchRun::collect_statistics() {
    GroupStats* g = nullptr;
    for (int i = 0; i < n; ++i) {
        const BatchItem& it = items[i];
        if (!it.stats || it.gran == kGranTensor || stats_done[i]) continue;
        if (!g || g->n == kMaxGroupStats) { g = &stats_groups[n_stats_groups++]; g->n = 0; g->near_tol = near_tol; }
        StatsOp& t = g->op[g->n];
        t.err_sum = it.o.err_sum; t.nnz = it.o.nnz; t.mask = it.o.mask;
        t.geom = make_geom(it.gran, it.sh.rows, it.sh.cols);
        t.n_part = geom_parts(t.geom);
        t.th = it.th;
        t.rec = reinterpret_cast<StatsRec*>(carve(sizeof(StatsRec) * kStatsMaxWg));
        t.out = static_cast<StatsDev*>(it.stats);
        // the first group rides on the first grouped per-tensor launches if the batch has any, the others are launched on their own
        const bool rides = n_stats_groups == 1 && will_ride;
        g->wg_end[g->n] = (g->n ? g->wg_end[g->n - 1] : 0) + (rides ? stats_wgs(t.n_part) : stats_wgs_fast(t.n_part));
        ++g->n;
    }
}

void BatchRun::per_tensor_operands(int crit) {
    // ---- per-tensor operands: amax pass, quantize pass, finish (+ fallback copy) pass; FP8 payload and fake
    //      quantization are different kernels
    for (int fake = 0; fake < 2 && err == hipSuccess; ++fake) {
        int idx[kMaxGroupTensor];
        int cnt = 0;
        auto flush = [&]() {
            if (cnt == 0 || err != hipSuccess) { cnt = 0; return; }
            GroupTensor g; g.n = cnt; g.near_tol = near_tol;
            int64_t total_tiles = 0;
            for (int k = 0; k < cnt; ++k) {
                const BatchItem& it = items[idx[k]];
                const int64_t n_chunks = it.sh.rows * it.sh.cols / 8;
                total_tiles += (n_chunks + kTensorChunksPerBlock - 1) / kTensorChunksPerBlock;
            }
            int a_end = 0, s_end = 0, c_end = 0;
            // Launch shape.  Several operands in the launch: one 32 KB tile per workgroup of pass B (up to 16384), at most three
            // workgroups resident per compute unit.  One operand alone does better with persistent workgroups that are all
            // resident from the start (measured with cold caches: 112 MiB, E4M3 kept: 57 us against 77 us per call; 336 MiB:
            // 148 against 195 us; 224 MiB falling back: 146 against 157 us), whereas the six gradients of the layer sweep
            // lose with that shape (333 against 294 us for the three launches).
            const bool solo = cnt == 1 && total_tiles <= 2000ll * kSoloQuantBlocks;
            const int amax_cap = solo ? kSoloAmaxBlocks : kMaxAmaxBlocks, quant_cap = solo ? kSoloQuantBlocks : kMaxQuantBlocks;
            const int pass_lds = solo ? 0 : kResidency3;
            for (int k = 0; k < cnt; ++k) {
                const BatchItem& it = items[idx[k]];
                TensorOp& t = g.op[k];
                t.x = it.x; t.o = it.o; t.th = it.th; t.mode = (uint32_t)it.scaling; t.three = it.three ? 1u : 0u; t.lean = it.lean ? 1u : 0u;
                t.n_chunks = it.sh.rows * it.sh.cols / 8;
                t.n_tiles = (t.n_chunks + kTensorChunksPerBlock - 1) / kTensorChunksPerBlock;
                t.n_amax = share(t.n_tiles, total_tiles, amax_cap, t.n_tiles);
                t.n_slots = share(t.n_tiles, total_tiles, quant_cap, t.n_tiles);
                const TensorPlan pl = plan_tensor(it.sh.rows, it.sh.cols);
                char* w = carve(pl.bytes);
                t.amax_part = reinterpret_cast<uint32_t*>(w + pl.off_amax_part);
                t.err = reinterpret_cast<float*>(w + pl.off_err_part);
                t.err5 = reinterpret_cast<float*>(w + pl.off_err5_part);
                t.zero = reinterpret_cast<uint32_t*>(w + pl.off_nnz_part);
                t.abits = reinterpret_cast<uint32_t*>(w + pl.off_decision);
                t.flush_part = reinterpret_cast<uint32_t*>(w + pl.off_flush_part);
                t.flush_need = 0ull;
                if (crit == kCritEq2 && it.o.bf16 && !it.three && it.th > 0.0f && it.th < 0.9f)
                    t.flush_need = flush_need_of(it.th, it.sh.rows * it.sh.cols);
                t.stats = static_cast<StatsDev*>(it.stats);
                a_end += t.n_amax; s_end += t.n_slots;
                c_end += (it.o.bf16 || it.three) ? share(t.n_tiles, total_tiles, 2048, 2048) : 1;
                g.amax_end[k] = a_end; g.slot_end[k] = s_end; g.copy_end[k] = c_end;
            }
            if (err != hipSuccess) { cnt = 0; return; }      // the workspace ran out while carving
            GroupStats riders; riders.n = 0; riders.near_tol = near_tol;
            int ride_partial = 0, ride_final = 0;
            if (!riders_used && n_stats_groups > 0) {
                riders = stats_groups[0];
                ride_partial = riders.wg_end[riders.n - 1];
                ride_final = ride_partial > riders.n ? riders.n : 0;      // single-workgroup operands are final already
                riders_used = true;
            }
            { ProfScope ps(prof, kKernTensorAmax, st); k_tensor_amax_group<<<dim3(a_end + ride_partial), dim3(256), pass_lds, st>>>(g, riders, a_end); }
            {
                ProfScope ps(prof, kKernTensorQuant, st);
                if (fake) {
                    if (crit == kCritEq3) k_tensor_quant_group<kCritEq3, true><<<dim3(s_end), dim3(256), pass_lds, st>>>(g);
                    else k_tensor_quant_group<kCritEq2, true><<<dim3(s_end), dim3(256), pass_lds, st>>>(g);
                } else {
                    if (crit == kCritEq3) k_tensor_quant_group<kCritEq3, false><<<dim3(s_end), dim3(256), pass_lds, st>>>(g);
                    else k_tensor_quant_group<kCritEq2, false><<<dim3(s_end), dim3(256), pass_lds, st>>>(g);
                }
            }
            {
                ProfScope ps(prof, kKernFallbackCopy, st);
                if (crit == kCritEq3) k_tensor_finish_group<kCritEq3><<<dim3(c_end + ride_final), dim3(256), 0, st>>>(g, riders, c_end);
                else k_tensor_finish_group<kCritEq2><<<dim3(c_end + ride_final), dim3(256), 0, st>>>(g, riders, c_end);
            }
            cnt = 0;
        };
        for (int i = 0; i < n; ++i) {
            const BatchItem& it = items[i];
            if (route[i] != kRouteTensorGroup || it.crit != crit || (it.o.fake != nullptr) != (fake != 0)) continue;
            const int64_t n_tiles = (it.sh.rows * it.sh.cols / 8 + kTensorChunksPerBlock - 1) / kTensorChunksPerBlock;
            if (n_tiles > 2000ll * kMaxQuantBlocks) { err = hipErrorInvalidValue; return; }   // 16-bit per-lane zero counters
            idx[cnt] = i;
            if (++cnt == kMaxGroupTensor) flush();
        }
        flush();
    }
    // ---- per-tensor operands with padded leading dimensions, one at a time
    for (int i = 0; i < n && err == hipSuccess; ++i) {
        const BatchItem& it = items[i];
        if (route[i] != kRouteTensorStrided || it.crit != crit) continue;
        char* w = carve(plan_tensor(it.sh.rows, it.sh.cols).bytes);
        if (err != hipSuccess) return;
        err = launch_tensor(it.x, it.sh, it.o, it.crit, it.th, (uint32_t)it.scaling, it.three ? 1u : 0u, w, st, prof);
        if (err == hipSuccess && it.stats)
            err = launch_select_stats(make_geom(it.gran, it.sh.rows, it.sh.cols), it.o.err_sum, it.o.nnz, it.o.mask, it.th, near_tol, it.stats, st);
    }
}

// ---- statistics of the operands with sub-tensor blocks that found no per-tensor launch to ride on
void BatchRun::leftover_statistics() {
    for (int k = riders_used ? 1 : 0; k < n_stats_groups && err == hipSuccess; ++k) {
        const GroupStats& g = stats_groups[k];
        const int wg_total = g.wg_end[g.n - 1];
        { ProfScope ps(prof, kKernStatsPartial, st); k_stats_group_partial<<<dim3(wg_total), dim3(kStatsFastThreads), 0, st>>>(g); }
        if (wg_total > g.n) { ProfScope ps(prof, kKernStatsFinal, st); k_stats_group_final<<<dim3(g.n), dim3(256), 0, st>>>(g); }
    }
}

}  // namespace

hipError_t launch_batch(const BatchItem* items, int n, float near_tol, void* ws, size_t ws_bytes, hipStream_t st, KProf* prof) {
    static_assert(sizeof(GroupSub) <= 3800 && sizeof(GroupTensor) + sizeof(GroupStats) <= 3800 &&
                  sizeof(GroupGam) <= 3800 && sizeof(GroupScope) <= 3800, "kernel-argument segment is 4 KB");
    static_assert(sizeof(StatsRec) == 128, "StatsRec layout");
    BatchRun run;
    run.items = items; run.n = n; run.near_tol = near_tol; run.st = st; run.prof = prof;
    run.wsp = static_cast<char*>(ws);
    run.ws_bytes = ws_bytes;
    for (int i = 0; i < n; ++i) run.route[i] = route_of(items[i]);
    for (int i = 0; i < n; ++i) run.will_ride |= run.route[i] == kRouteTensorGroup;
    run.group_mantissas();
    for (int crit = 0; crit < 2 && run.err == hipSuccess; ++crit) run.sub_tensor_operands(crit);
    if (run.err == hipSuccess) run.tensor_level_decisions();
    // the statistics of the sub-tensor operands are collected after their kernels (and tensor-level decisions)
    if (run.err == hipSuccess) run.collect_statistics();
    for (int crit = 0; crit < 2 && run.err == hipSuccess; ++crit) run.per_tensor_operands(crit);
    run.leftover_statistics();
    if (run.err != hipSuccess) return run.err;
    return hipGetLastError();
}

static int log2_or_whole(int64_t block, int64_t dim) {
    if (block >= dim) return 62;                 // one block spans the dimension: index >> 62 == 0
    int l = 0;
    while ((1ll << l) < block) ++l;
    return l;
}
hipError_t launch_dequantize_batch(const DeqItem* items, int n, hipStream_t st) {
    static_assert(sizeof(GroupDeq) <= 3800, "kernel-argument segment is 4 KB");
    GroupDeq g; g.n = 0;
    int64_t total = 0;
    auto flush = [&]() {
        if (g.n == 0) return;
        k_dequant_group<<<dim3((unsigned)total), dim3(256), 0, st>>>(g);
        g.n = 0; total = 0;
    };
    for (int i = 0; i < n; ++i) {
        const DeqItem& it = items[i];
        if (it.geom.pc == 1 && it.geom.cols > 1) {       // one column per block: its own kernel
            hipError_t e = launch_dequantize(it.geom, it.fp8, it.ld_fp8, it.scale, it.mask, it.bf16, it.ld_bf16, it.y, it.ld_y, it.e8m0,
                                             it.gmant, it.group_rows, st);
            if (e != hipSuccess) return e;
            continue;
        }
        const int64_t strips_x = (it.geom.cols + 127) / 128, units = strips_x * ((it.geom.rows + 63) / 64);
        if (units > 0x7FFFFFFF) return hipErrorInvalidValue;
        if (total + units > 0x7FFFFFFF) flush();
        DeqOp& t = g.op[g.n];
        t.g = it.geom; t.pr_log2 = log2_or_whole(it.geom.pr, it.geom.rows); t.pc_log2 = log2_or_whole(it.geom.pc, it.geom.cols);
        t.strips_x = strips_x;
        t.fp8 = it.fp8; t.ld_fp8 = it.ld_fp8; t.scale = it.scale; t.mask = it.mask; t.bf16 = it.bf16; t.ld_bf16 = it.ld_bf16;
        t.y = it.y; t.ld_y = it.ld_y; t.e8m0 = it.e8m0; t.gmant = it.gmant; t.group_rows = it.group_rows;
        total += units;
        g.unit_end[g.n] = total;
        if (++g.n == kMaxGroupDeq) flush();
    }
    flush();
    return hipGetLastError();
}

hipError_t launch_dequantize(const StatsGeom& geom, const uint8_t* fp8, int64_t ld_fp8, const float* scale,
                             const uint8_t* mask, const uint16_t* bf16, int64_t ld_bf16, uint16_t* y, int64_t ld_y,
                             const uint8_t* e8m0, const uint32_t* gmant, int64_t group_rows, hipStream_t st) {
    const int prl = log2_or_whole(geom.pr, geom.rows), pcl = log2_or_whole(geom.pc, geom.cols);
    if (geom.pc == 1 && geom.cols > 1) {
        const dim3 grid((unsigned)((geom.cols + 127) / 128), (unsigned)clamp_grid_y((geom.rows + 127) / 128));
        k_dequant_columns<<<grid, dim3(256), 0, st>>>(geom, prl, fp8, ld_fp8, scale, mask, bf16, ld_bf16, y, ld_y, e8m0, gmant, group_rows);
    } else {
        const dim3 grid((unsigned)((geom.cols + 127) / 128), (unsigned)clamp_grid_y((geom.rows + 15) / 16));
        k_dequant<<<grid, dim3(256), 0, st>>>(geom, prl, pcl, fp8, ld_fp8, scale, mask, bf16, ld_bf16, y, ld_y, e8m0, gmant, group_rows);
    }
    return hipGetLastError();
}

hipError_t launch_select_stats(const StatsGeom& geom, const float* err_sum, const uint32_t* nnz,
                               const uint8_t* mask, float th, float near_tol, void* out_dev, hipStream_t st) {
    static_assert(sizeof(StatsDev) == 144, "mor_stats layout");
    StatsDev* sd = static_cast<StatsDev*>(out_dev);
    const int64_t n_part = geom_parts(geom);
    if (n_part <= 8192) {
        k_stats_single<<<dim3(1), dim3(256), 0, st>>>(n_part, geom, err_sum, nnz, mask, th, near_tol, sd);
    } else {
        k_stats_zero<<<dim3(1), dim3(64), 0, st>>>(sd);
        int64_t want = (n_part + 1023) / 1024;
        const int nb = (int)(want > 1024 ? 1024 : want);
        k_stats_multi<<<dim3(nb), dim3(256), 0, st>>>(n_part, geom, err_sum, nnz, mask, th, near_tol, sd);
        k_stats_finish<<<dim3(1), dim3(64), 0, st>>>(n_part, (unsigned long long)(geom.rows * geom.cols), sd);
    }
    return hipGetLastError();
}

hipError_t launch_histogram_update(uint32_t* hist, const void* stats_dev, int clear, hipStream_t st) {
    k_histogram_update<<<dim3(1), dim3(64), 0, st>>>(hist, static_cast<const StatsDev*>(stats_dev), clear);
    return hipGetLastError();
}

}  // namespace mor
