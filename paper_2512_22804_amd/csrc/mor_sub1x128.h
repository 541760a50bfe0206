// The flat 1 x 128 kernel body (dense operands whose blocks are consecutive 256-byte runs), shared by the kernel of
// its own and by the block-team kernel, in whose launch a few 1 x 128 operands can ride in extra workgroups.
#pragma once

#include "mor_device.h"
#include "mor_launch.h"

namespace mor {

// Dense operands (every leading dimension == cols): blocks are consecutive 256-byte runs.
// A wave owns 64 consecutive blocks.  DPP row g (16 lanes x 8 elements) works through blocks
// g*16 .. g*16+15, eight at a time with all eight loads in flight; lane j of the row keeps the
// scalars of block g*16+j, so the per-block work (division, decision, metadata) is done once per
// 16 blocks by 64 lanes in parallel and the metadata stores are contiguous 256-byte runs.
// Batched 16-lane butterflies over N independent values: the N chains interleave, which hides the
// DPP read-after-write wait states.
template <int CTRL, int N>
__device__ __forceinline__ void rows_max_step(uint32_t (&v)[N]) {
#pragma unroll
    for (int i = 0; i < N; ++i) v[i] = max(v[i], dpp_u32<CTRL>(v[i]));
}
template <int CTRL, int N>
__device__ __forceinline__ void rows_add_step(float (&v)[N]) {
#pragma unroll
    for (int i = 0; i < N; ++i) v[i] += dpp_f32<CTRL>(v[i]);
}
template <int N>
__device__ __forceinline__ void rows_allmax(uint32_t (&v)[N]) {
    rows_max_step<kDppXor1, N>(v); rows_max_step<kDppXor2, N>(v); rows_max_step<kDppHalfMirror, N>(v); rows_max_step<kDppMirror, N>(v);
}
template <int N>
__device__ __forceinline__ void rows_allsum(float (&v)[N]) {
    rows_add_step<kDppXor1, N>(v); rows_add_step<kDppXor2, N>(v); rows_add_step<kDppHalfMirror, N>(v); rows_add_step<kDppMirror, N>(v);
}

// Rarely taken: some block of this unit has amax >= 2^25 or is non-finite.  Rolled loop, data re-read
// from memory, every block of the unit goes through the careful element path (valid for any input).
template <int CRIT>
__device__ __forceinline__ void sub_unit_careful(const uint16_t* __restrict__ xl, uint8_t* __restrict__ fl, uint16_t* __restrict__ ff,
                                                 int lane, float my_s, float my_s5, float& my_err, float& my_err5) {
    const int l = lane & 15;
#pragma clang loop unroll(disable)
    for (int k = 0; k < 8; ++k) {
        const int src_lane = (lane & 48) + k;
        const float s_k = __shfl(my_s, src_lane, 64);
        float e = quant8_careful_mem<false>(xl + k * 128, s_k, ff ? nullptr : fl + k * 128, ff ? ff + k * 128 : nullptr, 1.0f / s_k);
        e = row_allsum_f32(e);
        if ((l & 7) == k) my_err = e;
        if constexpr (CRIT == kCritEq3) {
            const float s5_k = __shfl(my_s5, src_lane, 64);
            float e5 = quant8_careful_mem<true>(xl + k * 128, s5_k, nullptr);
            e5 = row_allsum_f32(e5);
            if ((l & 7) == k) my_err5 = e5;
        }
    }
}

// Statistics gathered by the block kernel itself (a lone operand has no later launch to give them to): the small counters
// of a workgroup live in shared memory and take one atomic add per block from the lane that owns the block; the two sums
// stay with the owner lanes until the workgroup's last unit is done.
struct SubStatsShared {
    uint32_t c[16];        // kStatCnt counters of the workgroup (12 histogram bins, BF16 blocks, near-threshold blocks, unused)
    uint32_t n;            // non-zero elements
    uint32_t pad;
    double e[4];           // per wave: sum of the blocks' error sums
    double e_lane[256];    // per lane: running sum of its blocks' error sums (kept here to spare registers)
    uint32_t n_lane[256];  // per lane: non-zero elements of its blocks
};

// One unit = 32 consecutive blocks: DPP row g (16 lanes x 8 elements) owns blocks g*8 .. g*8+7 of the
// unit, all eight already loaded into raw[].  Lane j (and its mirror j+8) of the row keeps the scalars of
// block g*8+j, so the per-block work (division, decision, metadata) runs once per 8 blocks.
template <int CRIT, bool FAKE, bool STATS = false>
__device__ __forceinline__ void sub_unit_process(const u32x4 (&raw)[8], const uint16_t* __restrict__ x, const KOut& o, int64_t unit,
                                                 int lane, float th, bool defer, uint32_t mode, uint32_t mg, uint32_t mg5, bool proven,
                                                 const uint32_t* __restrict__ gam, uint32_t group_rows, uint32_t bpr,
                                                 SubStatsShared* ssh = nullptr, float near_tol = 0.0f) {
    const int g = lane >> 4, l = lane & 15, own = l & 7;
    const int64_t prow = unit * 32 + g * 8;
    if (group_rows) {                                      // the owner lane's block may lie in another band than its neighbours'
        const uint32_t* gw = gam_words(gam, group_rows, (prow + own) / bpr);
        mg = gw[0];
        if constexpr (CRIT == kCritEq3) mg5 = gw[1];
    }
    const int64_t off = prow * 128 + l * 8;
    uint8_t* __restrict__ fl = FAKE ? nullptr : o.fp8 + off;
    uint16_t* __restrict__ ff = FAKE ? o.fake + off : nullptr;       // fake quantization: the de-quantized values go here
    // phase 1: per-block amax (to the owner lane) and zero counts (packed 4 blocks per dword)
    uint32_t ab[8];
    uint32_t zp0 = 0u, zp1 = 0u;
#pragma unroll
    for (int k = 0; k < 8; ++k) {
        Scan8 sc{0u, 0u};
        scan8(raw[k], sc);
        ab[k] = fold_max16(sc.amax2);
        const uint32_t zc = __builtin_amdgcn_sad_u16(sc.zero2, 0u, 0u);       // low + high half-word counts (<= 8)
        if (k < 4) zp0 |= zc << (8 * k); else zp1 |= zc << (8 * (k - 4));
    }
    rows_allmax<8>(ab);
    uint32_t amax_unit = 0u, my_abits = 0u;
#pragma unroll
    for (int k = 0; k < 8; ++k) {
        amax_unit = max(amax_unit, ab[k]);
        if (own == k) my_abits = ab[k];
    }
    zp0 = row_allsum_u32(zp0);        // byte sums <= 128: no carry between bytes
    zp1 = row_allsum_u32(zp1);
    const uint32_t my_zero = (((own & 4) ? zp1 : zp0) >> (8 * (own & 3))) & 0xFFu;
    const float my_s = block_scale(my_abits, kE4M3Max, mode, mg);
    float my_s5 = 0.0f;
    if constexpr (CRIT == kCritEq3) my_s5 = block_scale(my_abits, kE5M2Max, mode, mg5);
    // phase 2: quantize with the owner's scale, reduce the error terms to the owner
    float my_err = 0.0f, my_err5 = 0.0f;
    if (__any(amax_unit >= fast_amax_limit(mode))) {
        sub_unit_careful<CRIT>(x + off, fl, ff, lane, my_s, my_s5, my_err, my_err5);
    } else {
        float e[8], e5[8];
        // Eq. 3: when every E5M2 scale of the wave is 128 times the E4M3 one, both formats share a reciprocal (quant8_dual)
        const bool dual = CRIT == kCritEq3 && __all(my_s5 == 128.0f * my_s);
        const float my_sinv = FAKE ? 1.0f / my_s : 0.0f;
#define MOR_SUB_ONE(K)                                                                     \
        {                                                                                  \
            float e0 = 0.0f, e1 = 0.0f;                                                    \
            const float s_K = row_bcast_f32<K>(my_s);                                      \
            const float sinv_K = FAKE ? row_bcast_f32<K>(my_sinv) : 0.0f;                  \
            u32x4 deq;                                                                     \
            u32x2 codes;                                                                   \
            if (CRIT == kCritEq3 && dual) {                                                \
                float f0 = 0.0f, f1 = 0.0f;                                                \
                codes = quant8_dual<FAKE>(raw[K], s_K, sinv_K, e0, e1, f0, f1, deq);       \
                e5[K] = f0 + f1;                                                           \
            } else {                                                                       \
                codes = quant8_fast_deq<false, FAKE>(raw[K], s_K, sinv_K, e0, e1, deq);    \
                if constexpr (CRIT == kCritEq3) {                                          \
                    float f0 = 0.0f, f1 = 0.0f;                                            \
                    (void)quant8_fast<true>(raw[K], row_bcast_f32<K>(my_s5), f0, f1);      \
                    e5[K] = f0 + f1;                                                       \
                }                                                                          \
            }                                                                              \
            if constexpr (FAKE) store16(ff + K * 128, deq);                                \
            else store8(fl + K * 128, codes);                                              \
            e[K] = e0 + e1;                                                                \
            __builtin_amdgcn_sched_barrier(0);                                             \
        }
        MOR_SUB_ONE(0) MOR_SUB_ONE(1) MOR_SUB_ONE(2) MOR_SUB_ONE(3) MOR_SUB_ONE(4) MOR_SUB_ONE(5) MOR_SUB_ONE(6) MOR_SUB_ONE(7)
#undef MOR_SUB_ONE
        rows_allsum<8>(e);
#pragma unroll
        for (int k = 0; k < 8; ++k)
            if (own == k) my_err = e[k];
        if constexpr (CRIT == kCritEq3) {
            rows_allsum<8>(e5);
#pragma unroll
            for (int k = 0; k < 8; ++k)
                if (own == k) my_err5 = e5[k];
        }
    }
    if (my_abits >= kInfBits) { my_err = __builtin_inff(); my_err5 = my_err; }
    uint32_t my_mask = 0u;
    if (!defer) my_mask = (CRIT == kCritEq3) ? decide_eq3(my_err, my_err5) : decide_eq2(my_err, 128u - my_zero, th);
    if (l < 8) {
        const int64_t p = prow + l;
        o.scale[p] = my_s;
        o.amax[p] = __uint_as_float(my_abits << 16);
        o.err_sum[p] = my_err;
        o.nnz[p] = 128u - my_zero;
        if constexpr (CRIT == kCritEq3) o.err5_sum[p] = my_err5;
        if (!defer) o.mask[p] = (uint8_t)my_mask;
        if (mode != kScaleFp32 && o.e8m0) o.e8m0[p] = (uint8_t)(__float_as_uint(my_s) >> 23);
    }
    if (defer && proven) {
        // tensor-level decision already proven to be BF16 by the pre-pass (uniform over the launch's operand): the fallback
        // payload of every block is stored from the registers (for fake quantization this overwrites the de-quantized values)
        uint16_t* __restrict__ bl = o.bf16 + off;
#pragma unroll
        for (int k = 0; k < 8; ++k) store16(bl + k * 128, raw[k]);
    }
    if (!defer && o.bf16) {
        const unsigned long long want = __ballot(l < 8 && my_mask != 0u);
        if (want) {
            const uint32_t bits = (uint32_t)(want >> (lane & 48)) & 0xFFu;   // my row's eight blocks
            uint16_t* __restrict__ bl = o.bf16 + off;
#pragma unroll
            for (int k = 0; k < 8; ++k)
                if ((bits >> k) & 1u) store16(bl + k * 128, raw[k]);
        }
    }
    if constexpr (STATS) {          // the same arithmetic as the statistics kernels apply to the stored per-block values
        if (l < 8) {
            const uint32_t nz = 128u - my_zero;
            const float metric = nz ? my_err / (float)nz : 0.0f;
            atomicAdd(&ssh->c[stats_bin(metric)], 1u);
            ssh->e_lane[threadIdx.x] += (double)my_err;
            ssh->n_lane[threadIdx.x] += nz;
            if (my_mask == 1u) atomicAdd(&ssh->c[12], 1u);
            if (fabs((double)metric - (double)th) <= (double)near_tol * (double)th) atomicAdd(&ssh->c[13], 1u);
        }
    }
}


// Descriptor table of a flat 1 x 128 launch (N operands); it travels in the kernel-argument segment.
template <int N>
struct GroupSubT {
    int n;
    int64_t unit_end[N];       // running total of 32-block units
    const uint16_t* x[N];
    KOut o[N];
    float th[N];
    uint8_t defer[N];          // 1: tensor-level decision follows, write no mask / fallback here
    uint8_t mode[N];           // scaling algorithm
    uint8_t prove[N];          // 1: gam[2] != 0 says that the tensor-level BF16 decision is already proven (fallback stored here)
    const uint32_t* gam[N];    // mode != 0: {mantissa for E4M3, mantissa for E5M2, proven flag} of the operand's group
    uint32_t group_rows[N];    // GAM with bands of rows as groups (0: one group): the band's mantissas come from the table behind gam
    uint32_t bpr[N];           // blocks per row (cols / 128), to find a block's row
};
constexpr int kMaxGroupSub = 16;       // operands per launch of the kernel of its own
constexpr int kMaxSubRiders = 2;       // operands that can ride on a block-team launch
typedef GroupSubT<kMaxGroupSub> GroupSub;
typedef GroupSubT<kMaxSubRiders> SubRiders;
// Riders offered to the block-team launcher: the table, its workgroup count, the output kind, and whether they went along.
struct TeamRiders {
    SubRiders table;
    int64_t blocks;
    bool fake, used;
};

// Workgroup `block` of `n_blocks` (4 waves each): a wave strides over the 8 KB units of all operands of the table.
template <int CRIT, bool FAKE, bool STATS = false, class G>
__device__ __forceinline__ void sub_group_body(const G& g, int64_t block, int64_t n_blocks, SubStatsShared* ssh = nullptr,
                                               float near_tol = 0.0f) {
    const int lane = threadIdx.x & 63, row = lane >> 4, l = lane & 15;
    const int64_t W = n_blocks * 4, total = g.unit_end[g.n - 1];
    int64_t u = block * 4 + (threadIdx.x >> 6);
    if (u >= total) return;
    const int lane_off = (row * 8) * 128 + l * 8;
    u32x4 bufA[8];
    auto load_unit = [&](u32x4 (&raw)[8], int64_t unit, int& op, int64_t& local) {
        op = group_find(g.unit_end, g.n, unit);
        local = unit - (op ? g.unit_end[op - 1] : 0);
        const uint16_t* __restrict__ src = g.x[op] + local * (32 * 128) + lane_off;
#pragma unroll
        for (int k = 0; k < 8; ++k) raw[k] = load16(src + k * 128);
    };
    auto process = [&](const u32x4 (&raw)[8], int op, int64_t local) {
        const uint32_t mode = g.mode[op];
        uint32_t mg = 0u, mg5 = 0u;
        if (mode) { mg = g.gam[op][0]; if constexpr (CRIT == kCritEq3) mg5 = g.gam[op][1]; }
        const bool proven = g.prove[op] != 0 && g.gam[op][2] != 0u;
        sub_unit_process<CRIT, FAKE, STATS>(raw, g.x[op], g.o[op], local, lane, g.th[op], g.defer[op] != 0, mode, mg, mg5, proven,
                                            g.gam[op], mode == kScaleGam ? g.group_rows[op] : 0u, g.bpr[op], ssh, near_tol);
    };
    int opA;
    int64_t locA;
    load_unit(bufA, u, opA, locA);
    for (;;) {
        process(bufA, opA, locA);
        u += W;
        if (u >= total) break;
        load_unit(bufA, u, opA, locA);
    }
}

}  // namespace mor
