// Kernels for the further partitions of the MoR analyse-select-quantize path on gfx950 (MI355X):
// 64 x 64 blocks, per-channel rows and columns, 128 x 1 sub-columns, ragged edges, the three-way
// recipe [E4M3, E5M2, BF16] (Section 3.2) and the fake-quantization output (Section 4, Figure 4).
//
// "Team" kernels: a team of threads (a wave or a whole workgroup) owns one block and keeps it in
// registers (8 x 16 bytes per lane), so one HBM pass computes amax, scale, codes, error sums and the
// decision.  "Column" kernels: a workgroup owns a 128 x 128 tile whose 128 columns belong to 128
// different blocks; a lane keeps the scalars of its 8 columns.
#include <type_traits>

#include "mor_device.h"
#include "mor_launch.h"
#include "mor_sub1x128.h"

namespace mor {

constexpr int kChunks = 8;     // 16-byte chunks per lane

// ======================================================================================
// Team kernels
// ======================================================================================
enum {
    kTeamWg128 = 0,     // 128 x 128 block, one workgroup
    kTeamHalf64 = 1,    // 64 x 64 blocks, two side by side per wave (32 lanes each, 16 chunks per lane), so that a wave's loads
                        // cover 256-byte row segments; a workgroup takes a tile of 128 rows x 256 columns (eight blocks)
    kTeamWaveRow = 2,   // one row of at most 4096 elements, one wave; four rows per workgroup
    kTeamWgRow = 3,     // one row of at most 16384 elements, one workgroup of 256
    kTeamBigRow = 4     // one row of at most 65536 elements, one workgroup of 1024
};
static_assert(kTeamBigRow + 1 == kTeamKinds, "the batch launcher walks over every team kind");
constexpr int kMaxTeamGroup = 12;
struct TeamOp {
    const uint16_t* x;
    KOut o;
    int64_t ld, rows, cols;
    int64_t units_x;        // 128-column tiles per row of tiles (block kinds)
    float th;
    uint8_t defer, mode, three, prove;      // prove: gam[2] != 0 says the tensor-level BF16 decision is already proven
    uint32_t group_rows;                    // GAM with bands of rows as groups (0: one group)
    const uint32_t* gam;
};
struct GroupTeam {
    int n;
    int64_t unit_end[kMaxTeamGroup];
    TeamOp op[kMaxTeamGroup];
};
struct TeamShared {
    uint32_t u[16];
    float f[32];
};

template <int TEAM> __device__ __forceinline__ constexpr bool team_is_wg() { return TEAM == kTeamWg128 || TEAM == kTeamWgRow || TEAM == kTeamBigRow; }
template <int TEAM> __device__ __forceinline__ constexpr int team_threads() { return TEAM == kTeamBigRow ? 1024 : 256; }
template <int TEAM> __device__ __forceinline__ constexpr int team_waves() { return team_threads<TEAM>() / 64; }
template <int TEAM> __device__ __forceinline__ constexpr int team_chunks() { return TEAM == kTeamHalf64 ? 16 : kChunks; }

// All-reduce over the 32 lanes of a half-wave team: lanes with the same bit 3 (8-lane groups of the four 16-lane rows).
// The lanes of the other half never enter, so the two blocks of a wave may sit in different branches.
__device__ __forceinline__ uint32_t half_allmax_u32(uint32_t v) {
    v = max(v, dpp_u32<kDppXor1>(v));
    v = max(v, dpp_u32<kDppXor2>(v));
    v = max(v, dpp_u32<kDppHalfMirror>(v));
    const auto r = __builtin_amdgcn_permlane16_swap(v, v, false, false);
    v = max(r[0], r[1]);
    const auto q = __builtin_amdgcn_permlane32_swap(v, v, false, false);
    return max(q[0], q[1]);
}
__device__ __forceinline__ uint32_t half_allsum_u32(uint32_t v) {
    v += dpp_u32<kDppXor1>(v);
    v += dpp_u32<kDppXor2>(v);
    v += dpp_u32<kDppHalfMirror>(v);
    const auto r = __builtin_amdgcn_permlane16_swap(v, v, false, false);
    v = r[0] + r[1];
    const auto q = __builtin_amdgcn_permlane32_swap(v, v, false, false);
    return q[0] + q[1];
}
__device__ __forceinline__ float half_allsum_f32(float v) {
    v += dpp_f32<kDppXor1>(v);
    v += dpp_f32<kDppXor2>(v);
    v += dpp_f32<kDppHalfMirror>(v);
    const auto r = __builtin_amdgcn_permlane16_swap(__float_as_uint(v), __float_as_uint(v), false, false);
    v = __uint_as_float(r[0]) + __uint_as_float(r[1]);
    const auto q = __builtin_amdgcn_permlane32_swap(__float_as_uint(v), __float_as_uint(v), false, false);
    return __uint_as_float(q[0]) + __uint_as_float(q[1]);
}

// All-reduce over the team.  Workgroup teams combine the four wave results through LDS (every thread
// of the workgroup must call); wave teams stay inside the wave.
template <int TEAM>
__device__ __forceinline__ uint32_t team_allmax(uint32_t v, TeamShared& sh) {
    if constexpr (TEAM == kTeamHalf64) return half_allmax_u32(v);
    v = wave_allmax_u32(v);
    if constexpr (team_is_wg<TEAM>()) {
        if ((threadIdx.x & 63) == 0) sh.u[threadIdx.x >> 6] = v;
        __syncthreads();
        v = sh.u[0];
#pragma unroll
        for (int k = 1; k < team_waves<TEAM>(); ++k) v = max(v, sh.u[k]);
        __syncthreads();
    }
    return v;
}
// `b` (the E5M2 error sum) is only reduced when WITH_B; otherwise it stays as it is (zero under Eq. 2).
template <int TEAM, bool WITH_B>
__device__ __forceinline__ void team_allsum3(float& a, float& b, uint32_t& z, TeamShared& sh) {
    if constexpr (TEAM == kTeamHalf64) {
        a = half_allsum_f32(a);
        if constexpr (WITH_B) b = half_allsum_f32(b);
        z = half_allsum_u32(z);
        return;
    }
    a = wave_allsum_f32(a);
    if constexpr (WITH_B) b = wave_allsum_f32(b);
    z = wave_allsum_u32(z);
    if constexpr (team_is_wg<TEAM>()) {
        constexpr int NW = team_waves<TEAM>();
        const int w = threadIdx.x >> 6;
        if ((threadIdx.x & 63) == 0) { sh.f[w] = a; if constexpr (WITH_B) sh.f[NW + w] = b; sh.u[w] = z; }
        __syncthreads();
        a = 0.0f; z = 0u;
        if constexpr (WITH_B) b = 0.0f;
#pragma unroll
        for (int k = 0; k < NW; k += 4) {       // fixed order: deterministic
            a += (sh.f[k] + sh.f[k + 1]) + (sh.f[k + 2] + sh.f[k + 3]);
            if constexpr (WITH_B) b += (sh.f[NW + k] + sh.f[NW + k + 1]) + (sh.f[NW + k + 2] + sh.f[NW + k + 3]);
            z += (sh.u[k] + sh.u[k + 1]) + (sh.u[k + 2] + sh.u[k + 3]);
        }
        __syncthreads();
    }
}

// EDGE = false: the operand has no partial blocks (block teams), or its rows are a whole number of the
// team's sweeps (row teams), so chunk validity is uniform over the team and costs no per-lane predicates.
template <int TEAM, int CRIT, bool FAKE, bool EDGE>
__device__ __forceinline__ void team_block(const TeamOp& t, int64_t unit, TeamShared& sh) {
    const int tid = threadIdx.x, lane = tid & 63, w = __builtin_amdgcn_readfirstlane(tid >> 6);
    const KOut& o = t.o;
    // ---- geometry: block index p, origin (r0, c0), valid extent h x wd, this lane's chunk positions
    constexpr int NCH = team_chunks<TEAM>();
    int64_t p, r0, c0;
    int h, wd, trow, tcol, rstep, cstep;
    int bcol = 0;                                          // kTeamHalf64: this lane's column inside its block
    bool active = true, leader;
    if constexpr (TEAM == kTeamWg128) {
        const int64_t tr = unit / t.units_x, tc = unit - tr * t.units_x;
        p = unit; r0 = tr * 128; c0 = tc * 128;
        trow = tid >> 4; tcol = (tid & 15) * 8; rstep = 16; cstep = 0;
        h = (int)(t.rows - r0 < 128 ? t.rows - r0 : 128); wd = (int)(t.cols - c0 < 128 ? t.cols - c0 : 128);
        leader = tid == 0;
    } else if constexpr (TEAM == kTeamHalf64) {
        // wave w: rows (w >> 1) * 64 .., columns (w & 1) * 128 .. of the workgroup's 128 x 256 tile; lanes with bit 3 set
        // own the right one of the wave's two blocks
        const int64_t tr = unit / t.units_x, tc = unit - tr * t.units_x;
        const int64_t gc = (t.cols + 63) / 64;
        const int side = (lane >> 3) & 1;
        r0 = tr * 128 + (w >> 1) * 64; c0 = tc * 256 + (w & 1) * 128;
        if (r0 >= t.rows || c0 >= t.cols) return;          // the whole wave is outside: uniform, and no barrier follows
        p = (r0 >> 6) * gc + (c0 >> 6) + side;
        trow = lane >> 4; tcol = (lane & 15) * 8; rstep = 4; cstep = 0;
        bcol = tcol & 63;
        h = (int)(t.rows - r0 < 64 ? t.rows - r0 : 64);
        const int64_t left = t.cols - (c0 + side * 64);
        wd = (int)(left < 0 ? 0 : (left < 64 ? left : 64));   // 0: this lane's block lies outside the tensor
        leader = (lane & 0x37) == 0 && wd > 0;
    } else if constexpr (TEAM == kTeamWaveRow) {
        p = unit * 4 + w; r0 = p; c0 = 0;
        active = p < t.rows;
        trow = 0; tcol = lane * 8; rstep = 0; cstep = 64 * 8;
        h = 1; wd = (int)t.cols;
        leader = lane == 0;
    } else {
        p = unit; r0 = p; c0 = 0;
        trow = 0; tcol = tid * 8; rstep = 0; cstep = team_threads<TEAM>() * 8;
        h = 1; wd = (int)t.cols;
        leader = tid == 0;
    }
    if (!active) return;                                   // wave teams only: no barrier is skipped
    const uint16_t* __restrict__ src = t.x + (r0 + trow) * t.ld + c0 + tcol;
    const int64_t src_step = (int64_t)rstep * t.ld + cstep;
    // Whole-block operands of the block teams use plain pointers; everything else (ragged edges, rows) goes through
    // bounds-checked buffer accesses relative to the block origin, where a lane outside the block costs no branch.
    constexpr bool BUF = EDGE || TEAM == kTeamWaveRow || TEAM == kTeamWgRow || TEAM == kTeamBigRow;
    auto in_block = [&](int i) -> bool {
        if constexpr (TEAM == kTeamHalf64) return (trow + i * rstep < h) && (bcol < wd);
        else return (trow + i * rstep < h) && (tcol + i * cstep < wd);
    };
    auto is_valid = [&](int i) -> bool {
        if constexpr (BUF) return in_block(i);
        else return true;
    };
    const BufRsrc rx = make_buf(t.x + r0 * t.ld + c0);
    const uint32_t xoff = (uint32_t)((trow * t.ld + tcol) * 2), xstep = (uint32_t)(src_step * 2);
    u32x4 raw[NCH];
#pragma unroll
    for (int i = 0; i < NCH; ++i) {
        if constexpr (BUF) raw[i] = buf_load16(rx, is_valid(i) ? xoff : kBufOutside, i * xstep);
        else raw[i] = load16(src + i * src_step);
    }
    // ---- amax and zero count (chunks outside the tensor count as zeros and change nothing)
    Scan8 sc{0u, 0u};
#pragma unroll
    for (int i = 0; i < NCH; ++i) scan8(raw[i], sc);
    // pin both results here: otherwise the compiler sinks the zero count below the quantization sweep and keeps the
    // 32 masked words of the block alive across it
    asm volatile("" : "+v"(sc.amax2), "+v"(sc.zero2));
    const uint32_t abits = team_allmax<TEAM>(fold_max16(sc.amax2), sh);
    const uint32_t mode = t.mode;
    uint32_t mg = 0u, mg5 = 0u;
    if (mode) { const uint32_t* gw = gam_words(t.gam, t.group_rows, r0); mg = gw[0]; mg5 = gw[1]; }
    float s = block_scale(abits, kE4M3Max, mode, mg);
    float s5 = 0.0f;                                       // only Eq. 3 and the three-way recipe look at E5M2
    if (CRIT == kCritEq3 || t.three) s5 = block_scale(abits, kE5M2Max, mode, mg5);
    // ---- destinations
    uint8_t* __restrict__ dst8 = FAKE ? nullptr : o.fp8 + (r0 + trow) * o.ld_fp8 + c0 + tcol;
    const int64_t dst8_step = (int64_t)rstep * o.ld_fp8 + cstep;
    uint16_t* __restrict__ dstf = FAKE ? o.fake + (r0 + trow) * o.ld_fake + c0 + tcol : nullptr;
    const int64_t dstf_step = (int64_t)rstep * o.ld_fake + cstep;
    const BufRsrc r8 = make_buf(FAKE ? nullptr : o.fp8 + r0 * o.ld_fp8 + c0);
    const uint32_t off8 = (uint32_t)(trow * o.ld_fp8 + tcol), step8 = (uint32_t)dst8_step;
    const BufRsrc rf = make_buf(FAKE ? o.fake + r0 * o.ld_fake + c0 : nullptr);
    const uint32_t offf = (uint32_t)((trow * o.ld_fake + tcol) * 2), stepf = (uint32_t)(dstf_step * 2);
    const bool fast = abits < fast_amax_limit(mode);
    // quantizes the block with scale `sc_` for format E5M2 ? E5M2 : E4M3; returns this lane's error sum
    auto quantize = [&](auto fmt, float sc_, bool emit) -> float {
        constexpr bool E5 = decltype(fmt)::value;
        const float s_inv = FAKE ? 1.0f / sc_ : 0.0f;        // correctly rounded IEEE division
        float e0 = 0.0f, e1 = 0.0f;
        if (fast) {
#pragma unroll
            for (int i = 0; i < NCH; ++i) {
                u32x4 deq;
                const u32x2 codes = quant8_fast_deq<E5, FAKE>(raw[i], sc_, s_inv, e0, e1, deq);
                // (fake quantization always stores through the buffer window: `emit` is a run-time value there, and a
                // branch around the stores would split the sweep into basic blocks and cost > 100 registers)
                if constexpr (BUF || FAKE) {
                    const bool put = emit && is_valid(i);
                    if constexpr (FAKE) buf_store16(rf, put ? offf + i * stepf : kBufOutside, deq);
                    else buf_store8(r8, put ? off8 : kBufOutside, i * step8, codes);
                } else if (emit) {
                    if constexpr (FAKE) store16(dstf + i * dstf_step, deq);
                    else store8(dst8 + i * dst8_step, codes);
                }
                __builtin_amdgcn_sched_barrier(0);            // one chunk at a time keeps the register count down
            }
        } else {
#pragma clang loop unroll(disable)
            for (int i = 0; i < NCH; ++i)
                if (in_block(i))
                    e0 += quant8_careful_mem<E5>(src + i * src_step, sc_, emit && !FAKE ? dst8 + i * dst8_step : nullptr,
                                                 emit && FAKE ? dstf + i * dstf_step : nullptr, s_inv);
        }
        return e0 + e1;
    };
    // tensor-level decision already proven by the pre-pass (uniform): the BF16 payload is stored below; a fake-quantized
    // output of such an operand is its input, so the de-quantized values are not stored at all
    bool proven = false;
    if (t.prove) proven = t.gam[2] != 0u;
    float err, err5 = 0.0f;
    if (CRIT == kCritEq3 && fast && s5 == 128.0f * s) {
        // both formats in one sweep, one reciprocal per element (see quant8_dual)
        const float s_inv = FAKE ? 1.0f / s : 0.0f;
        float e0 = 0.0f, e1 = 0.0f, f0 = 0.0f, f1 = 0.0f;
#pragma unroll
        for (int i = 0; i < NCH; ++i) {
            u32x4 deq;
            const u32x2 codes = quant8_dual<FAKE>(raw[i], s, s_inv, e0, e1, f0, f1, deq);
            if constexpr (BUF) {
                if constexpr (FAKE) buf_store16(rf, is_valid(i) ? offf + i * stepf : kBufOutside, deq);
                else buf_store8(r8, is_valid(i) ? off8 : kBufOutside, i * step8, codes);
            } else {
                if constexpr (FAKE) store16(dstf + i * dstf_step, deq);
                else store8(dst8 + i * dst8_step, codes);
            }
            __builtin_amdgcn_sched_barrier(0);
        }
        err = e0 + e1;
        err5 = f0 + f1;
    } else {
        err = quantize(std::false_type{}, s, !(FAKE && proven));
        if constexpr (CRIT == kCritEq3) err5 = quantize(std::true_type{}, s5, false);
    }
    uint32_t zeros = fold_add16(sc.zero2);
    team_allsum3<TEAM, CRIT == kCritEq3>(err, err5, zeros, sh);
    constexpr uint32_t kTeamElems = (team_is_wg<TEAM>() ? (uint32_t)team_threads<TEAM>() : (TEAM == kTeamHalf64 ? 32u : 64u)) * NCH * 8u;
    const uint32_t nnz = kTeamElems - zeros;
    if (abits >= kInfBits) { err = __builtin_inff(); err5 = __builtin_inff(); }
    const bool defer = t.defer != 0;
    uint32_t mask = defer ? 0u : ((CRIT == kCritEq3) ? decide_eq3(err, err5) : decide_eq2(err, nnz, t.th));
    // ---- three-way recipe: a block that failed M_1 is kept in E5M2 if its dynamic range fits (Eq. 4)
    uint32_t amin_bits = 0u;
    if (t.three && mask == 1u) {                           // uniform over the team
        uint32_t mn2 = 0xFFFFFFFFu;
#pragma unroll
        for (int i = 0; i < NCH; ++i) {
            u32x4 w = raw[i];
            asm volatile("" : "+v"(w.x), "+v"(w.y), "+v"(w.z), "+v"(w.w));      // no reuse of the masked words of the amax sweep
            mn2 = min_nonzero_m1(w, mn2);
        }
        const uint32_t mn = ~team_allmax<TEAM>(~fold_min16(mn2), sh) & 0xFFFFu;
        amin_bits = nnz ? mn + 1u : 0u;
        if (range_fits_e5m2(abits, amin_bits, nnz)) {
            mask = 2u;
            s = s5;
            (void)quantize(std::true_type{}, s5, true);    // the E5M2 payload replaces the E4M3 one
        }
    }
    if (leader) {
        o.scale[p] = s;
        o.amax[p] = __uint_as_float(abits << 16);
        o.err_sum[p] = err;
        o.nnz[p] = nnz;
        if constexpr (CRIT == kCritEq3) o.err5_sum[p] = err5;
        if (!defer) o.mask[p] = (uint8_t)mask;
        if (mode != kScaleFp32 && o.e8m0) o.e8m0[p] = (uint8_t)(__float_as_uint(s) >> 23);
        if (t.three && o.amin) o.amin[p] = __uint_as_float(amin_bits << 16);
    }
    const bool keep = mask == 1u || proven;                // (a deferred decision has mask 0 here)
    if (keep && o.bf16) {                                  // BF16: the block stays as it is
        uint16_t* __restrict__ dbf = o.bf16 + (r0 + trow) * o.ld_bf16 + c0 + tcol;
        const int64_t dbf_step = (int64_t)rstep * o.ld_bf16 + cstep;
        const BufRsrc rb = make_buf(o.bf16 + r0 * o.ld_bf16 + c0);
        const uint32_t offb = (uint32_t)((trow * o.ld_bf16 + tcol) * 2), stepb = (uint32_t)(dbf_step * 2);
#pragma unroll
        for (int i = 0; i < NCH; ++i) {
            if constexpr (BUF) buf_store16(rb, is_valid(i) ? offb + i * stepb : kBufOutside, raw[i]);
            else store16(dbf + i * dbf_step, raw[i]);
        }
    }
}

// Workgroups from `sub_first` on (block teams of 256 lanes only) run the flat 1 x 128 body over the riders: a small
// 1 x 128 operand then shares this launch instead of paying the ramp and tail of a launch of its own.
// RIDE is a template parameter so that launches without riders keep the team body's smaller register allocation.
template <int TEAM, int CRIT, bool FAKE, bool EDGE, bool RIDE>
__global__ __launch_bounds__(TEAM == kTeamBigRow ? 1024 : 256) void k_team_group(GroupTeam g, SubRiders riders, int64_t sub_first) {
    if constexpr (RIDE) {
        if ((int64_t)blockIdx.x >= sub_first) {
            sub_group_body<CRIT, FAKE>(riders, (int64_t)blockIdx.x - sub_first, (int64_t)gridDim.x - sub_first);
            return;
        }
    }
    __shared__ TeamShared sh;
    const int op = group_find(g.unit_end, g.n, blockIdx.x);
    const TeamOp& t = g.op[op];
    const int64_t unit = (int64_t)blockIdx.x - (op ? g.unit_end[op - 1] : 0);
    team_block<TEAM, CRIT, FAKE, EDGE>(t, unit, sh);
}

// Pre-pass of Algorithm 1 (group amax) for operands with 128 x 128 / 64 x 64 blocks or per-channel rows whose decision is taken
// per tensor under Eq. 2: a workgroup walks over tiles, keeps the running maximum and counts the elements that are
// certain to flush -- non-zero and below 2^-20 of a LOWER bound of their own block's amax (the amax of the part of the
// block that the lane's wave holds: 32 rows of a 128 x 128 block, 16 rows of a 64 x 64 block, up to 4096 consecutive elements of a row), so that
// under any scale of Algorithm 1 (never above 448 / amax) they land below half the smallest E4M3 subnormal and contribute
// exactly 1 to the error sum.  The waves of a workgroup never wait for each other inside the loop, and the next tile's
// loads are in flight while the current one is counted.
struct ProveOp {
    const uint16_t* x;
    int64_t ld, cols;
    int64_t units_x;         // blocks: 128-column tiles per row of tiles; rows: pieces of 4096 elements per row
    int64_t n_units;         // blocks: tiles; rows: pieces (one per wave)
    uint32_t* amax_part;
    uint32_t* flush_part;
    int32_t kind;            // kProveBlock128, kProveRows, kProveBlock64
};
enum { kProveBlock128 = kProveKindBlock128, kProveRows = kProveKindRows, kProveBlock64 = kProveKindBlock64,
       kProveSubRow = kProveKindSubRow,       // 1 x 128 sub-rows: the 16 lanes of a DPP row hold one whole block per chunk
       kProveSubCol = kProveKindSubCol };     // 128 x 1 sub-columns: a lane holds 8 rows of 8 column blocks, its wave 32 rows of each
__device__ __forceinline__ uint32_t colgroup_max2(uint32_t v);
struct GroupProve {
    int n;
    int32_t wg_end[kMaxTeamGroup];
    ProveOp op[kMaxTeamGroup];
};
constexpr int kProvePiece = 64 * 8 * kChunks;      // elements of a row that one wave holds at a time
static_assert(kProvePiece == 4096, "scope_proof_units() counts pieces of 4096 elements");
// KIND kProveBlock64: the same 128 x 128 tiles as for kProveBlock128, four blocks each; a lane's first four chunks lie
// in an upper block, the others in a lower one, lanes with bit 3 set in a right-hand one.
template <int KIND>
__device__ __forceinline__ void prove_tiles(const ProveOp& t, int b, int nb, uint32_t& amax_run, uint32_t& flush_run) {
    const int tid = threadIdx.x, lane = tid & 63, w = tid >> 6;
    auto load_tile = [&](u32x4 (&raw)[kChunks], int64_t unit) {
        if constexpr (KIND == kProveRows) {
            // wave w of the workgroup's unit takes piece 4 * unit + w; chunks beyond the row (or beyond the operand) load zeros
            const int64_t piece = unit * 4 + w, row = piece / t.units_x, c0 = (piece - row * t.units_x) * kProvePiece;
            const BufRsrc rx = make_buf(t.x + row * t.ld + c0);
            const bool inside = piece < t.n_units;
#pragma unroll
            for (int i = 0; i < kChunks; ++i)
                raw[i] = buf_load16(rx, (inside && c0 + (i * 64 + lane) * 8 < t.cols) ? (uint32_t)(lane * 16) : kBufOutside, i * 1024);
        } else {
            const int64_t tr = unit / t.units_x, tc = unit - tr * t.units_x;
            const uint16_t* __restrict__ src = t.x + (tr * 128 + (tid >> 4)) * t.ld + tc * 128 + (tid & 15) * 8;
#pragma unroll
            for (int i = 0; i < kChunks; ++i) raw[i] = load16(src + (int64_t)i * 16 * t.ld);
        }
    };
    const int64_t n_wg_units = KIND == kProveRows ? (t.n_units + 3) / 4 : t.n_units;
    u32x4 cur[kChunks], nxt[kChunks];
    int64_t unit = b;
    if (unit < n_wg_units) load_tile(cur, unit);
    while (unit < n_wg_units) {
        const int64_t next = unit + nb;
        if (next < n_wg_units) load_tile(nxt, next);        // uniform over the workgroup
        if constexpr (KIND == kProveSubRow) {
            // every chunk of a DPP row is one block: its exact amax, and the flushes relative to it
            uint32_t ab[kChunks];
#pragma unroll
            for (int i = 0; i < kChunks; ++i) {
                uint32_t a2 = 0u;
#pragma unroll
                for (int j = 0; j < 4; ++j) a2 = pk_max_u16(a2, cur[i][j] & 0x7FFF7FFFu);
                ab[i] = fold_max16(a2);
            }
            rows_allmax<kChunks>(ab);
            uint32_t f2 = 0u;
#pragma unroll
            for (int i = 0; i < kChunks; ++i) {
                amax_run = max(amax_run, ab[i]);
                const uint32_t t1 = ab[i] > 0x0A00u ? ab[i] - 0x0A01u : 0u;
                const uint32_t bound2 = t1 | (t1 << 16);
#pragma unroll
                for (int j = 0; j < 4; ++j) f2 = pk_add_u16(f2, pk_certain_flush(cur[i][j], bound2));
            }
            flush_run += fold_add16(f2);
#pragma unroll
            for (int i = 0; i < kChunks; ++i) cur[i] = nxt[i];
            unit = next;
            continue;
        }
        if constexpr (KIND == kProveSubCol) {
            // word j of every chunk holds two of the lane's eight columns: column maxima over the lane's 8 rows and the wave's
            // four row groups (32 of the block's 128 rows: a lower bound of the block's amax), flushes relative to them
            uint32_t c2[4] = {0u, 0u, 0u, 0u};
#pragma unroll
            for (int i = 0; i < kChunks; ++i)
#pragma unroll
                for (int j = 0; j < 4; ++j) c2[j] = pk_max_u16(c2[j], cur[i][j] & 0x7FFF7FFFu);
            uint32_t f2 = 0u;
#pragma unroll
            for (int j = 0; j < 4; ++j) {
                c2[j] = colgroup_max2(c2[j]);
                amax_run = max(amax_run, fold_max16(c2[j]));
                const uint32_t bound2 = pk_sub_sat_u16(pk_sub_sat_u16(c2[j], 0x0A000A00u), 0x00010001u);
#pragma unroll
                for (int i = 0; i < kChunks; ++i) f2 = pk_add_u16(f2, pk_certain_flush(cur[i][j], bound2));
            }
            flush_run += fold_add16(f2);
#pragma unroll
            for (int i = 0; i < kChunks; ++i) cur[i] = nxt[i];
            unit = next;
            continue;
        }
        // amax of what this wave holds of the lane's block(s): one value, or one for each half of the chunks
        uint32_t a2[2] = {0u, 0u};
#pragma unroll
        for (int i = 0; i < kChunks; ++i)
#pragma unroll
            for (int j = 0; j < 4; ++j) {
                const int h = KIND == kProveBlock64 ? i / (kChunks / 2) : 0;
                a2[h] = pk_max_u16(a2[h], cur[i][j] & 0x7FFF7FFFu);
            }
        uint32_t abits[2];
        if constexpr (KIND == kProveBlock64) {
            abits[0] = half_allmax_u32(fold_max16(a2[0]));
            abits[1] = half_allmax_u32(fold_max16(a2[1]));
        } else {
            abits[0] = abits[1] = wave_allmax_u32(fold_max16(a2[0]));
        }
        amax_run = max(amax_run, max(abits[0], abits[1]));
        // t - 1, with t the amax pattern taken down by 20 binades (0 if that underflows)
        uint32_t bound2[2];
#pragma unroll
        for (int h = 0; h < 2; ++h) {
            const uint32_t t1 = abits[h] > 0x0A00u ? abits[h] - 0x0A01u : 0u;
            bound2[h] = t1 | (t1 << 16);
        }
        uint32_t f2 = 0u;
#pragma unroll
        for (int i = 0; i < kChunks; ++i)
#pragma unroll
            for (int j = 0; j < 4; ++j) f2 = pk_add_u16(f2, pk_certain_flush(cur[i][j], bound2[i / (kChunks / 2)]));
        flush_run += fold_add16(f2);                       // at most 64 per tile and lane
#pragma unroll
        for (int i = 0; i < kChunks; ++i) cur[i] = nxt[i];
        unit = next;
    }
}
__global__ __launch_bounds__(256) void k_block_amax_prove(GroupProve g) {
    __shared__ uint32_t sh[8];
    const int op = group_find32(g.wg_end, g.n, blockIdx.x);
    const ProveOp& t = g.op[op];
    const int first = op ? g.wg_end[op - 1] : 0;
    const int b = blockIdx.x - first, nb = g.wg_end[op] - first;
    const int tid = threadIdx.x;
    uint32_t amax_run = 0u, flush_run = 0u;
    if (t.kind == kProveRows) prove_tiles<kProveRows>(t, b, nb, amax_run, flush_run);
    else if (t.kind == kProveBlock64) prove_tiles<kProveBlock64>(t, b, nb, amax_run, flush_run);
    else if (t.kind == kProveSubRow) prove_tiles<kProveSubRow>(t, b, nb, amax_run, flush_run);
    else if (t.kind == kProveSubCol) prove_tiles<kProveSubCol>(t, b, nb, amax_run, flush_run);
    else prove_tiles<kProveBlock128>(t, b, nb, amax_run, flush_run);
    amax_run = wave_allmax_u32(amax_run);
    flush_run = wave_allsum_u32(flush_run);
    if ((tid & 63) == 0) { sh[tid >> 6] = amax_run; sh[4 + (tid >> 6)] = flush_run; }
    __syncthreads();
    if (tid == 0) {
        t.amax_part[b] = max(max(sh[0], sh[1]), max(sh[2], sh[3]));
        t.flush_part[b] = (sh[4] + sh[5]) + (sh[6] + sh[7]);
    }
}

// ======================================================================================
// Column kernels: 128 x 1 sub-columns (Section 3: "sub-columns"; the transposed operands of the
// backward GEMMs, Section 4) and per-channel columns (Section 4.1.1 "Per-Channel", second operand).
// A workgroup sweeps a strip of 128-row x 128-column tiles; a lane holds 8 rows x 8 columns of a tile
// and keeps per-column scalars.  Per-channel columns span all strips, so they take three passes:
//   kColAmax      column amax of the strip                     -> workspace partials
//   (combine)     column amax, scales                          -> outputs + workspace scales
//   kColExternal  quantize with those scales, strip error sums -> workspace partials
//   (combine)     column error sums, decision, fallback columns
// 128 x 1 sub-columns are complete inside a tile (kColLocal): one pass.
// Proven columns (Eq. 2, two types, fallback buffer present): the amax pass also counts, per column, elements that are
// certain to flush -- non-zero and below 2^-20 of a LOWER bound of the column amax (the column's amax inside the
// strip's first tile), hence below 2^-20 of the final amax: they scale to less than half the smallest E4M3
// subnormal and contribute exactly 1 each.  A count above 1.01 * th * rows + 1 fixes the BF16 decision whatever the
// other terms are; the quantize pass then writes those columns' BF16 payload from its registers and the fallback
// pass skips them.  The decision itself is still taken from the full error sums.
// ======================================================================================
enum { kColLocal = 0, kColAmax = 1, kColExternal = 2 };
struct ColOp {
    const uint16_t* x;
    KOut o;
    int64_t ld, rows, cols;
    int64_t tiles_x;            // 128-column strips
    int32_t tiles_per_strip;    // 128-row tiles a workgroup sweeps (1 for kColLocal)
    float th;
    uint32_t group_rows;        // 128 x 1 blocks under GAM with bands of rows as groups (0: one group)
    uint8_t defer, mode, three, prove;   // prove: count certain flushes in the amax pass (see below)
    uint8_t derive_gam;
    const uint32_t* gam;
    // per-channel columns: workspace, [n_strips x cols_padded] each, cols_padded = tiles_x * 128
    uint16_t* part_amax;
    float* part_err; float* part_err5; uint16_t* part_zero;
    float* col_scale; float* col_scale5;                 // [cols_padded]
    uint16_t* col_amin;                                  // [cols_padded] (smallest non-zero pattern - 1), three-way recipe; its
                                                         // per-strip partials use part_zero, which is free until the quantize pass
    uint8_t* col_proven;                                 // [cols_padded] 1: the column's BF16 decision is proven before the quantize
                                                         // pass; the per-strip flush counts (16 bits) use part_err until then
    uint32_t flush_need;                                 // that many certain flushes in a column prove its BF16 decision
    int32_t n_strips;
    int32_t copy_groups;                                 // workgroups per 128-column strip in the fallback-column pass
    // tensor-level decision (Section 3.1) over per-channel columns: the certain flushes of ALL columns together may prove the
    // BF16 decision of the operand; every column then counts as proven and the quantize pass writes the whole fallback
    uint32_t* wg;                                        // [2 + 2 x n_strips x tiles_x]: word 0 = "BF16 proven for the whole operand" (read by the
                                                         // tensor-level copy pass), then per workgroup of the amax pass its largest column
                                                         // amax and its flush total
    unsigned long long tensor_need;                      // 0: columns are proven one by one (decisions per column)
    // GAM scaling (derive_gam): the group amax is the largest column amax, so the first combine derives the group mantissas
    // itself (no pre-pass over the operand) and leaves them in `gam` and in the caller's output
    uint32_t* gmant;                                     // caller's [2] or nullptr
};
struct GroupCol {
    int n;
    int64_t unit_end[kMaxTeamGroup];
    int32_t comb_end[kMaxTeamGroup];      // running workgroup totals of the combine kernels (256 columns each)
    int32_t copy_end[kMaxTeamGroup];      // running workgroup totals of the fallback-column copy
    ColOp op[kMaxTeamGroup];
};
struct ColShared {
    uint32_t amax[4][16][4];     // packed per-column maxima: wave, lane column group, 4 words (8 columns)
    float scale[128], scale5[128];
    float err[4][128], err5[4][128];
    uint32_t zero[4][16][4];     // packed per-column zero counts
    uint32_t amin[4][16][4];     // packed per-column (smallest non-zero pattern - 1), three-way recipe
    uint16_t abits[128];         // column amax patterns of the tile
    uint8_t mask[128];
    uint32_t wg[8];              // per-wave amax / flush totals of a strip (column-amax pass)
};

// Combines a lane's 8 per-column values with the lanes that hold the same columns in the other row groups
// of the wave (lane ^ 16, lane ^ 32).  gfx950's v_permlane16_swap / v_permlane32_swap, given the same register
// twice, return the values of the even and of the odd 16-lane row of each pair (of the lower and of the upper half
// of the wave): one VALU instruction per step instead of an LDS permute, and every lane combines in the same order.
__device__ __forceinline__ uint32_t colgroup_max2(uint32_t v) {
    const auto r = __builtin_amdgcn_permlane16_swap(v, v, false, false);
    v = pk_max_u16(r[0], r[1]);
    const auto q = __builtin_amdgcn_permlane32_swap(v, v, false, false);
    return pk_max_u16(q[0], q[1]);
}
__device__ __forceinline__ uint32_t colgroup_min2(uint32_t v) {
    const auto r = __builtin_amdgcn_permlane16_swap(v, v, false, false);
    v = pk_min_u16(r[0], r[1]);
    const auto q = __builtin_amdgcn_permlane32_swap(v, v, false, false);
    return pk_min_u16(q[0], q[1]);
}
__device__ __forceinline__ uint32_t colgroup_add2(uint32_t v) {
    const auto r = __builtin_amdgcn_permlane16_swap(v, v, false, false);
    v = pk_add_u16(r[0], r[1]);
    const auto q = __builtin_amdgcn_permlane32_swap(v, v, false, false);
    return pk_add_u16(q[0], q[1]);
}
__device__ __forceinline__ float colgroup_addf(float v) {
    const auto r = __builtin_amdgcn_permlane16_swap(__float_as_uint(v), __float_as_uint(v), false, false);
    v = __uint_as_float(r[0]) + __uint_as_float(r[1]);
    const auto q = __builtin_amdgcn_permlane32_swap(__float_as_uint(v), __float_as_uint(v), false, false);
    return __uint_as_float(q[0]) + __uint_as_float(q[1]);
}

template <int CRIT, int MODE, bool FAKE, bool EDGE>
__device__ __forceinline__ void col_strip(const ColOp& t, int64_t unit, ColShared& sh) {
    const int tid = threadIdx.x, lane = tid & 63, w = tid >> 6, cg = tid & 15;
    const KOut& o = t.o;
    const int64_t strip = unit / t.tiles_x, tc = unit - strip * t.tiles_x;
    const int64_t c0 = tc * 128, col = c0 + cg * 8;
    const bool col_ok = col < t.cols;
    const int64_t cols_padded = t.tiles_x * 128;
    const uint32_t mode = t.mode;
    uint32_t mg = 0u, mg5 = 0u;
    if (mode) {      // (bands of rows as groups only occur with 128 x 1 blocks, where a strip is one tile)
        const uint32_t* gw = gam_words(t.gam, MODE == kColLocal ? t.group_rows : 0u, strip * t.tiles_per_strip * 128);
        mg = gw[0]; mg5 = gw[1];
    }
    // strip-level accumulators (per-channel columns); for kColLocal a strip is one tile
    uint32_t amax2[4] = {0u, 0u, 0u, 0u}, zero2[4] = {0u, 0u, 0u, 0u};
    float err[8], err5[8];
#pragma unroll
    for (int k = 0; k < 8; ++k) { err[k] = 0.0f; err5[k] = 0.0f; }
    float s[8], s5[8], s_inv[8];
    bool strip_fast = true;
    uint32_t mn_strip[4] = {0xFFFFFFFFu, 0xFFFFFFFFu, 0xFFFFFFFFu, 0xFFFFFFFFu};      // kColAmax with three types
    uint32_t bound2[4] = {0u, 0u, 0u, 0u}, flush2[4] = {0u, 0u, 0u, 0u};              // kColAmax with the flush-count proof
    uint64_t pv8 = 0ull;                                                                // kColExternal: proven flags of my 8 columns
    if constexpr (MODE == kColExternal) {
        if (t.prove) pv8 = *reinterpret_cast<const uint64_t*>(t.col_proven + c0 + cg * 8);
    }
    if constexpr (MODE == kColExternal) {
        bool f = true;
#pragma unroll
        for (int k = 0; k < 8; ++k) {
            s[k] = t.col_scale[c0 + cg * 8 + k];
            s5[k] = CRIT == kCritEq3 ? t.col_scale5[c0 + cg * 8 + k] : 0.0f;
            s_inv[k] = FAKE ? 1.0f / s[k] : 0.0f;
            const uint32_t col_abits = col_ok ? __float_as_uint(o.amax[col + k]) >> 16 : 0u;
            f = f && col_abits < fast_amax_limit(mode);
        }
        strip_fast = f;      // per lane: the careful path has no cross-lane step, so no barrier is needed before the loads
    }
    for (int tt = 0; tt < t.tiles_per_strip; ++tt) {
        const int64_t r0 = (strip * t.tiles_per_strip + tt) * 128;
        if (r0 >= t.rows) break;                                       // uniform over the workgroup
        const int64_t row = r0 + (tid >> 4);
        const uint16_t* __restrict__ src = t.x + row * t.ld + col;
        auto is_valid = [&](int i) -> bool {
            if constexpr (EDGE) return col_ok && row + i * 16 < t.rows;
            else return true;                                          // rows and cols are multiples of 128
        };
        // ragged operands: bounds-checked buffer accesses relative to the tile origin (a lane outside loads zeros
        // and stores nothing, without a branch)
        const BufRsrc rx = make_buf(t.x + r0 * t.ld + c0);
        const uint32_t xoff = (uint32_t)(((tid >> 4) * t.ld + cg * 8) * 2), xstep = (uint32_t)(16 * t.ld * 2);
        // (the next tile's loads are not started early: with 32 more registers fewer workgroups fit, and the quantize pass
        // of the per-channel columns took 407 us instead of 396 us)
        u32x4 raw[kChunks];
#pragma unroll
        for (int i = 0; i < kChunks; ++i) {
            if constexpr (EDGE) raw[i] = buf_load16(rx, is_valid(i) ? xoff : kBufOutside, i * xstep);
            else raw[i] = load16(src + (int64_t)i * 16 * t.ld);
        }
        // one sweep over the chunks for everything that reads the magnitudes (column amax, zero counts, smallest
        // non-zero magnitude), so that no masked copy of the tile stays in registers
        uint32_t mn2[4] = {0xFFFFFFFFu, 0xFFFFFFFFu, 0xFFFFFFFFu, 0xFFFFFFFFu};
        const bool want_min = MODE != kColExternal && t.three;
#pragma unroll
        for (int i = 0; i < kChunks; ++i) {
#pragma unroll
            for (int j = 0; j < 4; ++j) {
                const uint32_t m = raw[i][j] & 0x7FFF7FFFu;
                if constexpr (MODE != kColExternal) amax2[j] = pk_max_u16(amax2[j], m);
                if constexpr (MODE != kColAmax) zero2[j] = pk_add_u16(zero2[j], pk_is_zero_u16(m));
                if constexpr (MODE != kColExternal) {
                    if (want_min) mn2[j] = pk_min_u16(mn2[j], pk_sub_u16(m, 0x00010001u));
                }
            }
            __builtin_amdgcn_sched_barrier(0);
        }
        // pin the results here: otherwise the compiler sinks these sweeps below the quantization loop and keeps the 32
        // masked words alive across it
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            if constexpr (MODE != kColAmax) asm volatile("" : "+v"(zero2[j]));
            if constexpr (MODE != kColExternal) asm volatile("" : "+v"(amax2[j]));
        }
        if (want_min) {
#pragma unroll
            for (int j = 0; j < 4; ++j) asm volatile("" : "+v"(mn2[j]));
        }
        if constexpr (MODE == kColAmax) {
            if (t.three) {
#pragma unroll
                for (int j = 0; j < 4; ++j) mn_strip[j] = pk_min_u16(mn_strip[j], mn2[j]);
            }
            if (t.prove) {                                             // uniform over the workgroup
                if (tt == 0) {
                    // lower bound of the column amax: this tile's column amax over the whole workgroup, taken down by
                    // 20 binades (0 if that underflows), minus one for the comparison below
                    uint32_t a[4];
#pragma unroll
                    for (int j = 0; j < 4; ++j) a[j] = colgroup_max2(amax2[j]);
                    if (lane < 16) {
#pragma unroll
                        for (int j = 0; j < 4; ++j) sh.amax[w][cg][j] = a[j];
                    }
                    __syncthreads();
#pragma unroll
                    for (int j = 0; j < 4; ++j) {
                        a[j] = pk_max_u16(pk_max_u16(sh.amax[0][cg][j], sh.amax[1][cg][j]), pk_max_u16(sh.amax[2][cg][j], sh.amax[3][cg][j]));
                        bound2[j] = pk_sub_sat_u16(pk_sub_sat_u16(a[j], 0x0A000A00u), 0x00010001u);
                    }
                    __syncthreads();                                   // sh.amax is written again when the strip is published
                }
#pragma unroll
                for (int i = 0; i < kChunks; ++i)
#pragma unroll
                    for (int j = 0; j < 4; ++j) flush2[j] = pk_add_u16(flush2[j], pk_certain_flush(raw[i][j], bound2[j]));
            }
            continue;
        }
        if constexpr (MODE == kColExternal) {
            if (pv8) {                                                 // per lane: some of my columns are proven to stay in BF16
                if (pv8 == 0x0101010101010101ull) {
                    const BufRsrc rb = make_buf(o.bf16 + r0 * o.ld_bf16 + c0);
                    const uint32_t offb = (uint32_t)(((tid >> 4) * o.ld_bf16 + cg * 8) * 2), stepb = (uint32_t)(16 * o.ld_bf16 * 2);
#pragma unroll
                    for (int i = 0; i < kChunks; ++i) {
                        if constexpr (EDGE) buf_store16(rb, is_valid(i) ? offb + i * stepb : kBufOutside, raw[i]);
                        else store16(o.bf16 + (row + (int64_t)i * 16) * o.ld_bf16 + col, raw[i]);
                    }
                } else {
#pragma clang loop unroll(disable)
                    for (int i = 0; i < kChunks; ++i) {
                        if (!is_valid(i)) continue;
                        const uint16_t* sp = src + (int64_t)i * 16 * t.ld;
                        uint16_t* dp = o.bf16 + (row + (int64_t)i * 16) * o.ld_bf16 + col;
                        for (int k = 0; k < 8; ++k)
                            if ((pv8 >> (8 * k)) & 1ull) dp[k] = sp[k];
                    }
                }
            }
        }
        if constexpr (MODE == kColLocal) {
            // column amax of the tile: row groups of the wave, then the four waves through LDS
#pragma unroll
            for (int j = 0; j < 4; ++j) amax2[j] = colgroup_max2(amax2[j]);
            if (lane < 16) {
#pragma unroll
                for (int j = 0; j < 4; ++j) sh.amax[w][cg][j] = amax2[j];
            }
            __syncthreads();
            bool slow = false;                                         // some column needs the careful element path
            if (tid < 128) {                                           // thread tid owns column tid of the tile
                const int g16 = tid >> 3, k = tid & 7;
                uint32_t a = 0u;
#pragma unroll
                for (int ww = 0; ww < 4; ++ww) a = max(a, (sh.amax[ww][g16][k >> 1] >> ((k & 1) * 16)) & 0xFFFFu);
                sh.scale[tid] = block_scale(a, kE4M3Max, mode, mg);
                if (CRIT == kCritEq3 || t.three) sh.scale5[tid] = block_scale(a, kE5M2Max, mode, mg5);
                sh.abits[tid] = (uint16_t)a;
                slow = a >= fast_amax_limit(mode);
            }
            strip_fast = __syncthreads_or(slow ? 1 : 0) == 0;         // also publishes the scales
#pragma unroll
            for (int k = 0; k < 8; ++k) {
                s[k] = sh.scale[cg * 8 + k];
                s5[k] = CRIT == kCritEq3 ? sh.scale5[cg * 8 + k] : 0.0f;     // Eq. 2: read again by the three-way path only
                s_inv[k] = FAKE ? 1.0f / s[k] : 0.0f;
            }
        }
        // ---- quantize the tile with the per-column scales
        uint8_t* __restrict__ dst8 = FAKE ? nullptr : o.fp8 + row * o.ld_fp8 + col;
        uint16_t* __restrict__ dstf = FAKE ? o.fake + row * o.ld_fake + col : nullptr;
        const BufRsrc r8 = make_buf(FAKE ? nullptr : o.fp8 + r0 * o.ld_fp8 + c0);
        const uint32_t off8 = (uint32_t)((tid >> 4) * o.ld_fp8 + cg * 8), step8 = (uint32_t)(16 * o.ld_fp8);
        const BufRsrc rf = make_buf(FAKE ? o.fake + r0 * o.ld_fake + c0 : nullptr);
        const uint32_t offf = (uint32_t)(((tid >> 4) * o.ld_fake + cg * 8) * 2), stepf = (uint32_t)(16 * o.ld_fake * 2);
        if (strip_fast) {
#pragma unroll
            for (int i = 0; i < kChunks; ++i) {
                u32x4 deq;
                const u32x2 codes = quant8_cols<false, FAKE>(raw[i], s, s_inv, err, deq);
                if constexpr (EDGE) {
                    if constexpr (FAKE) buf_store16(rf, is_valid(i) ? offf + i * stepf : kBufOutside, deq);
                    else buf_store8(r8, is_valid(i) ? off8 : kBufOutside, i * step8, codes);
                } else {
                    if constexpr (FAKE) store16(dstf + (int64_t)i * 16 * o.ld_fake, deq);
                    else store8(dst8 + (int64_t)i * 16 * o.ld_fp8, codes);
                }
                if constexpr (CRIT == kCritEq3) { u32x4 d5; (void)quant8_cols<true, false>(raw[i], s5, s_inv, err5, d5); }
                __builtin_amdgcn_sched_barrier(0);            // one chunk at a time keeps the register count down
            }
        } else {
            // some column of the strip has amax >= 2^24..2^25 or is non-finite: element-wise careful path
#pragma clang loop unroll(disable)
            for (int i = 0; i < kChunks; ++i) {
                if (!is_valid(i)) continue;
                const uint32_t* src32 = reinterpret_cast<const uint32_t*>(src + (int64_t)i * 16 * t.ld);
                uint32_t cw[2] = {0u, 0u};
                uint32_t dq[4];
#pragma unroll
                for (int j = 0; j < 4; ++j) {
                    const uint32_t wv = src32[j];
                    const uint32_t c_lo = quant1_careful<false>(wv & 0xFFFFu, s[2 * j], err[2 * j]);
                    const uint32_t c_hi = quant1_careful<false>(wv >> 16, s[2 * j + 1], err[2 * j + 1]);
                    cw[j >> 1] |= (c_lo | (c_hi << 8)) << ((j & 1) * 16);
                    if constexpr (FAKE) {
                        const f32x2 q = cvt_pk_f32<false>((int)(c_lo | (c_hi << 8)), false);
                        dq[j] = f32_to_bf16_rne(q.x * s_inv[2 * j]) | (f32_to_bf16_rne(q.y * s_inv[2 * j + 1]) << 16);
                    }
                    if constexpr (CRIT == kCritEq3) {
                        (void)quant1_careful<true>(wv & 0xFFFFu, s5[2 * j], err5[2 * j]);
                        (void)quant1_careful<true>(wv >> 16, s5[2 * j + 1], err5[2 * j + 1]);
                    }
                }
                if constexpr (FAKE) { u32x4 d; d.x = dq[0]; d.y = dq[1]; d.z = dq[2]; d.w = dq[3]; store16(dstf + (int64_t)i * 16 * o.ld_fake, d); }
                else { u32x2 c; c.x = cw[0]; c.y = cw[1]; store8(dst8 + (int64_t)i * 16 * o.ld_fp8, c); }
            }
        }
        if constexpr (MODE == kColLocal) {
            // ---- per-column error sums / zero counts of the tile, decision, metadata, fallback columns
#pragma unroll
            for (int k = 0; k < 8; ++k) {
                err[k] = colgroup_addf(err[k]);
                if constexpr (CRIT == kCritEq3) err5[k] = colgroup_addf(err5[k]);
            }
#pragma unroll
            for (int j = 0; j < 4; ++j) zero2[j] = colgroup_add2(zero2[j]);
            if (t.three) {
#pragma unroll
                for (int j = 0; j < 4; ++j) mn2[j] = colgroup_min2(mn2[j]);
            }
            if (lane < 16) {
#pragma unroll
                for (int k = 0; k < 8; ++k) { sh.err[w][cg * 8 + k] = err[k]; if constexpr (CRIT == kCritEq3) sh.err5[w][cg * 8 + k] = err5[k]; }
#pragma unroll
                for (int j = 0; j < 4; ++j) { sh.zero[w][cg][j] = zero2[j]; sh.amin[w][cg][j] = mn2[j]; }
            }
            __syncthreads();
            if (tid < 128) {
                const int g16 = tid >> 3, k = tid & 7;
                const uint32_t a = sh.abits[tid];
                float e = (sh.err[0][tid] + sh.err[1][tid]) + (sh.err[2][tid] + sh.err[3][tid]);
                float e5 = 0.0f;
                if constexpr (CRIT == kCritEq3) e5 = (sh.err5[0][tid] + sh.err5[1][tid]) + (sh.err5[2][tid] + sh.err5[3][tid]);
                uint32_t z = 0u;
#pragma unroll
                for (int ww = 0; ww < 4; ++ww) z += (sh.zero[ww][g16][k >> 1] >> ((k & 1) * 16)) & 0xFFFFu;
                const uint32_t nnz = 128u - z;
                if (a >= kInfBits) { e = __builtin_inff(); e5 = e; }
                const bool defer = t.defer != 0;
                uint32_t mk = defer ? 0u : ((CRIT == kCritEq3) ? decide_eq3(e, e5) : decide_eq2(e, nnz, t.th));
                // three-way recipe: a column that failed M_1 is kept in E5M2 if its dynamic range fits (Eq. 4)
                uint32_t amin_bits = 0u;
                float s_out = sh.scale[tid];
                if (t.three && mk == 1u) {
                    uint32_t mn = 0xFFFFu;
#pragma unroll
                    for (int ww = 0; ww < 4; ++ww) mn = min(mn, (sh.amin[ww][g16][k >> 1] >> ((k & 1) * 16)) & 0xFFFFu);
                    amin_bits = nnz ? ((mn + 1u) & 0xFFFFu) : 0u;
                    if (range_fits_e5m2(a, amin_bits, nnz)) { mk = 2u; s_out = sh.scale5[tid]; }
                }
                // (128 x 1 blocks whose tensor-level BF16 decision the pre-pass has proven: every column's payload is stored below)
                sh.mask[tid] = (uint8_t)((defer && t.prove && t.gam[2] != 0u) ? 1u : mk);
                if (c0 + tid < t.cols) {
                    const int64_t p = (r0 >> 7) * t.cols + c0 + tid;
                    o.scale[p] = s_out;
                    o.amax[p] = __uint_as_float(a << 16);
                    o.err_sum[p] = e;
                    o.nnz[p] = nnz;
                    if constexpr (CRIT == kCritEq3) o.err5_sum[p] = e5;
                    if (!defer) o.mask[p] = (uint8_t)mk;
                    if (mode != kScaleFp32 && o.e8m0) o.e8m0[p] = (uint8_t)(__float_as_uint(s_out) >> 23);
                    if (t.three && o.amin) o.amin[p] = __uint_as_float(amin_bits << 16);
                }
            }
            __syncthreads();
            if (t.three) {
                const uint64_t mk8 = *reinterpret_cast<const uint64_t*>(&sh.mask[cg * 8]);
                const uint64_t sel = (mk8 >> 1) & 0x0101010101010101ull;       // byte k = 1: column k is kept in E5M2
                if (sel) {
                    // the E5M2 payload replaces the E4M3 one in those columns (whole chunks are stored again)
                    if constexpr (CRIT != kCritEq3) {
#pragma unroll
                        for (int k = 0; k < 8; ++k) s5[k] = sh.scale5[cg * 8 + k];
                    }
#pragma clang loop unroll(disable)
                    for (int i = 0; i < kChunks; ++i) {
                        if (!is_valid(i)) continue;
                        const uint32_t* src32 = reinterpret_cast<const uint32_t*>(src + (int64_t)i * 16 * t.ld);
                        uint32_t cw[2] = {0u, 0u};
                        uint32_t dq[4];
#pragma unroll
                        for (int j = 0; j < 4; ++j) {
                            const uint32_t wv = src32[j];
                            const bool lo5 = (sel >> (16 * j)) & 1u, hi5 = (sel >> (16 * j + 8)) & 1u;
                            float dummy = 0.0f;
                            const uint32_t c_lo = lo5 ? quant1_careful<true>(wv & 0xFFFFu, s5[2 * j], dummy)
                                                      : quant1_careful<false>(wv & 0xFFFFu, s[2 * j], dummy);
                            const uint32_t c_hi = hi5 ? quant1_careful<true>(wv >> 16, s5[2 * j + 1], dummy)
                                                      : quant1_careful<false>(wv >> 16, s[2 * j + 1], dummy);
                            cw[j >> 1] |= (c_lo | (c_hi << 8)) << ((j & 1) * 16);
                            if constexpr (FAKE) {
                                const float q_lo = lo5 ? cvt_pk_f32<true>((int)c_lo, false).x : cvt_pk_f32<false>((int)c_lo, false).x;
                                const float q_hi = hi5 ? cvt_pk_f32<true>((int)c_hi, false).x : cvt_pk_f32<false>((int)c_hi, false).x;
                                const float i_lo = 1.0f / (lo5 ? s5[2 * j] : s[2 * j]), i_hi = 1.0f / (hi5 ? s5[2 * j + 1] : s[2 * j + 1]);
                                dq[j] = f32_to_bf16_rne(q_lo * i_lo) | (f32_to_bf16_rne(q_hi * i_hi) << 16);
                            }
                        }
                        if constexpr (FAKE) { u32x4 d; d.x = dq[0]; d.y = dq[1]; d.z = dq[2]; d.w = dq[3]; store16(dstf + (int64_t)i * 16 * o.ld_fake, d); }
                        else { u32x2 c; c.x = cw[0]; c.y = cw[1]; store8(dst8 + (int64_t)i * 16 * o.ld_fp8, c); }
                    }
                }
            }
            if (o.bf16) {
                uint64_t mk8 = *reinterpret_cast<const uint64_t*>(&sh.mask[cg * 8]);
                mk8 &= 0x0101010101010101ull;                          // byte k = 1: column k stays in BF16 (2 = E5M2 does not)
                uint16_t* __restrict__ dbf = o.bf16 + row * o.ld_bf16 + col;
                if (mk8 == 0x0101010101010101ull) {                    // all eight columns of this lane stay in BF16
                    const BufRsrc rb = make_buf(o.bf16 + r0 * o.ld_bf16 + c0);
                    const uint32_t offb = (uint32_t)(((tid >> 4) * o.ld_bf16 + cg * 8) * 2), stepb = (uint32_t)(16 * o.ld_bf16 * 2);
#pragma unroll
                    for (int i = 0; i < kChunks; ++i) {
                        if constexpr (EDGE) buf_store16(rb, is_valid(i) ? offb + i * stepb : kBufOutside, raw[i]);
                        else store16(dbf + (int64_t)i * 16 * o.ld_bf16, raw[i]);
                    }
                } else if (mk8) {                                      // some of them: element by element
#pragma clang loop unroll(disable)
                    for (int i = 0; i < kChunks; ++i) {
                        if (!is_valid(i)) continue;
                        const uint16_t* sp = src + (int64_t)i * 16 * t.ld;
                        uint16_t* dp = dbf + (int64_t)i * 16 * o.ld_bf16;
                        for (int k = 0; k < 8; ++k)
                            if ((mk8 >> (8 * k)) & 0xFFu) dp[k] = sp[k];
                    }
                }
            }
            if (tt + 1 < t.tiles_per_strip) __syncthreads();           // the LDS arrays are written again by the next tile
            // reset the per-tile accumulators (a strip of kColLocal is a single tile anyway)
#pragma unroll
            for (int k = 0; k < 8; ++k) { err[k] = 0.0f; err5[k] = 0.0f; }
#pragma unroll
            for (int j = 0; j < 4; ++j) { amax2[j] = 0u; zero2[j] = 0u; }
        }
    }
    // ---- per-channel columns: publish the strip's partials
    if constexpr (MODE == kColAmax) {
#pragma unroll
        for (int j = 0; j < 4; ++j) amax2[j] = colgroup_max2(amax2[j]);
        if (t.three) {
#pragma unroll
            for (int j = 0; j < 4; ++j) mn_strip[j] = colgroup_min2(mn_strip[j]);
        }
        if (t.prove) {
#pragma unroll
            for (int j = 0; j < 4; ++j) flush2[j] = colgroup_add2(flush2[j]);     // <= 4 x 8 x 16 per half-word
        }
        if (lane < 16) {
#pragma unroll
            for (int j = 0; j < 4; ++j) { sh.amax[w][cg][j] = amax2[j]; sh.amin[w][cg][j] = mn_strip[j]; sh.zero[w][cg][j] = flush2[j]; }
        }
        __syncthreads();
        uint32_t a = 0u, fl = 0u;
        if (tid < 128) {
            const int g16 = tid >> 3, k = tid & 7;
            uint32_t mn = 0xFFFFu;
#pragma unroll
            for (int ww = 0; ww < 4; ++ww) {
                a = max(a, (sh.amax[ww][g16][k >> 1] >> ((k & 1) * 16)) & 0xFFFFu);
                mn = min(mn, (sh.amin[ww][g16][k >> 1] >> ((k & 1) * 16)) & 0xFFFFu);
                fl += (sh.zero[ww][g16][k >> 1] >> ((k & 1) * 16)) & 0xFFFFu;
            }
            t.part_amax[strip * cols_padded + c0 + tid] = (uint16_t)a;
            if (t.three) t.part_zero[strip * cols_padded + c0 + tid] = (uint16_t)mn;
            if (t.prove) reinterpret_cast<uint16_t*>(t.part_err)[strip * cols_padded + c0 + tid] = (uint16_t)fl;
        }
        // the strip's largest column amax and its flush total, for the combine kernel's whole-operand figures
        // (group amax of Algorithm 1, tensor-level proof)
        a = wave_allmax_u32(a);
        fl = wave_allsum_u32(t.prove ? fl : 0u);
        if (lane == 0) { sh.wg[w] = a; sh.wg[4 + w] = fl; }
        __syncthreads();
        if (tid == 0) {
            t.wg[2 + 2 * unit] = max(max(sh.wg[0], sh.wg[1]), max(sh.wg[2], sh.wg[3]));
            t.wg[3 + 2 * unit] = (sh.wg[4] + sh.wg[5]) + (sh.wg[6] + sh.wg[7]);
        }
    }
    if constexpr (MODE == kColExternal) {
#pragma unroll
        for (int k = 0; k < 8; ++k) {
            err[k] = colgroup_addf(err[k]);
            if constexpr (CRIT == kCritEq3) err5[k] = colgroup_addf(err5[k]);
        }
        // per-lane zero counts: at most 8 per tile and column, 16 tiles per strip -> fit 16 bits after the wave sum (<= 512)
#pragma unroll
        for (int j = 0; j < 4; ++j) zero2[j] = colgroup_add2(zero2[j]);
        if (lane < 16) {
#pragma unroll
            for (int k = 0; k < 8; ++k) { sh.err[w][cg * 8 + k] = err[k]; if constexpr (CRIT == kCritEq3) sh.err5[w][cg * 8 + k] = err5[k]; }
#pragma unroll
            for (int j = 0; j < 4; ++j) sh.zero[w][cg][j] = zero2[j];
        }
        __syncthreads();
        if (tid < 128) {
            const int g16 = tid >> 3, k = tid & 7;
            uint32_t z = 0u;
#pragma unroll
            for (int ww = 0; ww < 4; ++ww) z += (sh.zero[ww][g16][k >> 1] >> ((k & 1) * 16)) & 0xFFFFu;
            const int64_t idx = strip * cols_padded + c0 + tid;
            t.part_err[idx] = (sh.err[0][tid] + sh.err[1][tid]) + (sh.err[2][tid] + sh.err[3][tid]);
            if constexpr (CRIT == kCritEq3) t.part_err5[idx] = (sh.err5[0][tid] + sh.err5[1][tid]) + (sh.err5[2][tid] + sh.err5[3][tid]);
            t.part_zero[idx] = (uint16_t)z;
        }
    }
}

template <int CRIT, int MODE, bool FAKE, bool EDGE>
__global__ __launch_bounds__(256) void k_col_group(GroupCol g) {
    __shared__ ColShared sh;
    const int op = group_find(g.unit_end, g.n, blockIdx.x);
    const ColOp& t = g.op[op];
    const int64_t unit = (int64_t)blockIdx.x - (op ? g.unit_end[op - 1] : 0);
    col_strip<CRIT, MODE, FAKE, EDGE>(t, unit, sh);
}

// Per-channel columns, first combine: column amax over the strips -> amax, scale (Algorithm 1), E8M0 byte.
// Under GAM every workgroup first takes the largest column amax of the operand (the group amax of Algorithm 1), and for a tensor-level decision the sum of all columns' certain flushes: the same values in every
// workgroup, from the per-workgroup figures of the amax pass (a handful of loads per thread).
__global__ __launch_bounds__(256) void k_col_scales(GroupCol g) {
    __shared__ uint32_t sh4[4];
    __shared__ unsigned long long shl[4];
    const int op = group_find32(g.comb_end, g.n, blockIdx.x);
    const ColOp& t = g.op[op];
    const int b = blockIdx.x - (op ? g.comb_end[op - 1] : 0);
    const int tid = threadIdx.x;
    const int64_t c = (int64_t)b * 256 + tid;
    const int64_t cols_padded = t.tiles_x * 128;
    const int64_t n_wg = (int64_t)t.n_strips * t.tiles_x;  // workgroups of the amax pass
    uint32_t mg = 0u, mg5 = 0u;
    if (t.derive_gam) {                                    // GAM (uniform over the workgroup)
        uint32_t ga = 0u;
        for (int64_t i = tid; i < n_wg; i += 256) ga = max(ga, t.wg[2 + 2 * i]);
        ga = wave_allmax_u32(ga);
        if ((tid & 63) == 0) sh4[tid >> 6] = ga;
        __syncthreads();
        ga = max(max(sh4[0], sh4[1]), max(sh4[2], sh4[3]));
        mg = group_mantissa_bits(ga, kE4M3Max, t.mode);
        mg5 = group_mantissa_bits(ga, kE5M2Max, t.mode);
        if (b == 0 && tid == 0) {
            uint32_t* gam_out = const_cast<uint32_t*>(t.gam);
            gam_out[0] = mg; gam_out[1] = mg5;
            if (t.gmant) { t.gmant[0] = mg; t.gmant[1] = mg5; }
        }
    } else if (t.mode) {
        mg = t.gam[0]; mg5 = t.gam[1];
    }
    bool all_proven = false;
    if (t.prove && t.tensor_need) {                        // uniform over the workgroup
        unsigned long long f = 0ull;
        for (int64_t i = tid; i < n_wg; i += 256) f += t.wg[3 + 2 * i];
#pragma unroll
        for (int m = 32; m > 0; m >>= 1) f += __shfl_xor(f, m, 64);
        if ((tid & 63) == 0) shl[tid >> 6] = f;
        __syncthreads();
        f = (shl[0] + shl[1]) + (shl[2] + shl[3]);
        all_proven = f >= t.tensor_need;
        if (b == 0 && tid == 0) t.wg[0] = all_proven ? 1u : 0u;
    }
    if (c >= cols_padded) return;
    uint32_t a = 0u;
#pragma unroll 8
    for (int sidx = 0; sidx < t.n_strips; ++sidx) a = max(a, (uint32_t)t.part_amax[sidx * cols_padded + c]);
    if (t.three) {
        uint32_t mn = 0xFFFFu;
#pragma unroll 8
        for (int sidx = 0; sidx < t.n_strips; ++sidx) mn = min(mn, (uint32_t)t.part_zero[sidx * cols_padded + c]);
        t.col_amin[c] = (uint16_t)mn;
    }
    if (t.prove) {
        if (t.tensor_need) {
            t.col_proven[c] = (c < t.cols && all_proven) ? 1 : 0;
        } else {
            const uint16_t* __restrict__ part_flush = reinterpret_cast<const uint16_t*>(t.part_err);
            uint32_t fl = 0u;
#pragma unroll 8
            for (int sidx = 0; sidx < t.n_strips; ++sidx) fl += part_flush[sidx * cols_padded + c];
            t.col_proven[c] = (c < t.cols && fl >= t.flush_need) ? 1 : 0;
        }
    }
    const float s = block_scale(a, kE4M3Max, t.mode, mg);
    t.col_scale[c] = s;
    t.col_scale5[c] = block_scale(a, kE5M2Max, t.mode, mg5);
    if (c < t.cols) {
        t.o.amax[c] = __uint_as_float(a << 16);
        t.o.scale[c] = s;
        if (t.mode != kScaleFp32 && t.o.e8m0) t.o.e8m0[c] = (uint8_t)(__float_as_uint(s) >> 23);
    }
}
// Second combine: column error sums over the strips (binary64, fixed order), non-zero counts, decision.
template <int CRIT>
__global__ __launch_bounds__(256) void k_col_finish(GroupCol g) {
    const int op = group_find32(g.comb_end, g.n, blockIdx.x);
    const ColOp& t = g.op[op];
    const int64_t c = (int64_t)(blockIdx.x - (op ? g.comb_end[op - 1] : 0)) * 256 + threadIdx.x;
    const int64_t cols_padded = t.tiles_x * 128;
    if (c >= t.cols) return;
    double e = 0.0, e5 = 0.0;
    unsigned long long z = 0;
#pragma unroll 8
    for (int sidx = 0; sidx < t.n_strips; ++sidx) {
        e += (double)t.part_err[sidx * cols_padded + c];
        z += t.part_zero[sidx * cols_padded + c];
        if constexpr (CRIT == kCritEq3) e5 += (double)t.part_err5[sidx * cols_padded + c];
    }
    // rows beyond the tensor were loaded as zeros, up to the end of the last 128-row tile
    const unsigned long long padded = (unsigned long long)((t.rows + 127) / 128) * 128ull;
    const unsigned long long n = padded - z;
    const uint32_t abits = __float_as_uint(t.o.amax[c]) >> 16;
    if (abits >= kInfBits) { e = (double)__builtin_inff(); e5 = e; }
    t.o.err_sum[c] = (float)e;
    t.o.nnz[c] = n > 0xFFFFFFFFull ? 0xFFFFFFFFu : (uint32_t)n;
    if constexpr (CRIT == kCritEq3) t.o.err5_sum[c] = (float)e5;
    if (!t.defer) {
        uint32_t mk;
        if constexpr (CRIT == kCritEq3) mk = (e < e5) ? 0u : 1u;
        else mk = ((n ? e / (double)n : 0.0) < (double)t.th) ? 0u : 1u;
        if (t.three) {                     // a column that failed M_1 is kept in E5M2 if its dynamic range fits (Eq. 4)
            uint32_t amin_bits = 0u;
            if (mk == 1u) {
                amin_bits = n ? (((uint32_t)t.col_amin[c] + 1u) & 0xFFFFu) : 0u;
                if (range_fits_e5m2(abits, amin_bits, n ? 1u : 0u)) {
                    mk = 2u;
                    const float s5 = t.col_scale5[c];
                    t.o.scale[c] = s5;
                    if (t.mode != kScaleFp32 && t.o.e8m0) t.o.e8m0[c] = (uint8_t)(__float_as_uint(s5) >> 23);
                }
            }
            if (t.o.amin) t.o.amin[c] = __uint_as_float(amin_bits << 16);
        }
        t.o.mask[c] = (uint8_t)mk;
    }
}
// Columns kept in BF16 are copied: 16 bytes at a time where all eight columns of a chunk are kept, else by element.
// Columns kept in E5M2 (three-way recipe) get their payload here, element by element, over the E4M3 one.
// A workgroup takes one 128-column strip and strides over the rows with the other workgroups of that strip.
constexpr int kColCopyRowGroups = 32;      // at most, per 128-column strip
constexpr int kColCopyBudget = 4096;       // workgroups per launch, about
__global__ __launch_bounds__(256) void k_col_fallback(GroupCol g) {
    const int op = group_find32(g.copy_end, g.n, blockIdx.x);
    const ColOp& t = g.op[op];
    if (t.defer || (t.o.bf16 == nullptr && !t.three)) return;
    const int b = blockIdx.x - (op ? g.copy_end[op - 1] : 0);
    const int64_t strip = b / t.copy_groups, rg = b - strip * t.copy_groups;
    const int64_t c = strip * 128 + (threadIdx.x & 15) * 8;
    if (c >= t.cols) return;
    uint32_t keep = 0u, five = 0u;
#pragma unroll
    for (int k = 0; k < 8; ++k) {
        const uint32_t mk = t.o.mask[c + k];
        const bool done = t.prove && t.col_proven[c + k] != 0;       // written by the quantize pass already
        keep |= ((mk == 1u && !done) ? 1u : 0u) << k;
        five |= (mk == 2u ? 1u : 0u) << k;
    }
    if (t.o.bf16 == nullptr) keep = 0u;
    if (!keep && !five) return;
    uint16_t* __restrict__ fakep = t.o.fake;
    const int64_t rstep = (int64_t)t.copy_groups * 16;
    int64_t r = rg * 16 + (threadIdx.x >> 4);
    if (keep == 0xFFu && !five) {          // whole chunks stay in BF16: four 16-byte loads in flight per lane
        for (; r + 3 * rstep < t.rows; r += 4 * rstep) {
            u32x4 v[4];
#pragma unroll
            for (int u = 0; u < 4; ++u) v[u] = load16(t.x + (r + u * rstep) * t.ld + c);
#pragma unroll
            for (int u = 0; u < 4; ++u) store16(t.o.bf16 + (r + u * rstep) * t.o.ld_bf16 + c, v[u]);
        }
    }
    for (; r < t.rows; r += rstep) {
        const uint16_t* sp = t.x + r * t.ld + c;
        if (keep == 0xFFu) store16(t.o.bf16 + r * t.o.ld_bf16 + c, load16(sp));
        else if (keep) {
            uint16_t* dp = t.o.bf16 + r * t.o.ld_bf16 + c;
            for (int k = 0; k < 8; ++k)
                if ((keep >> k) & 1u) dp[k] = sp[k];
        }
        if (five) {
            for (int k = 0; k < 8; ++k) {
                if (!((five >> k) & 1u)) continue;
                const float s5 = t.col_scale5[c + k];
                float dummy = 0.0f;
                const uint32_t code = quant1_careful<true>((uint32_t)sp[k], s5, dummy);
                if (fakep) fakep[r * t.o.ld_fake + c + k] = (uint16_t)f32_to_bf16_rne(cvt_pk_f32<true>((int)code, false).x * (1.0f / s5));
                else t.o.fp8[r * t.o.ld_fp8 + c + k] = (uint8_t)code;
            }
        }
    }
}

// ======================================================================================
// Launchers
// ======================================================================================
namespace {
size_t align16p(size_t v) { return (v + 15) & ~(size_t)15; }

template <int TEAM, bool FAKE, bool EDGE>
void launch_team_crit(const GroupTeam& g, int64_t total, int crit, const SubRiders& riders, int64_t rider_blocks, hipStream_t st) {
    const dim3 grid((unsigned)(total + rider_blocks)), block(TEAM == kTeamBigRow ? 1024 : 256);
    const int lds = TEAM == kTeamWg128 ? kResidency5 : 0;      // the other kinds show no gain from a cap
    if constexpr (TEAM == kTeamWg128) {
        if (rider_blocks > 0) {
            if (crit == kCritEq3) k_team_group<TEAM, kCritEq3, FAKE, EDGE, true><<<grid, block, lds, st>>>(g, riders, total);
            else k_team_group<TEAM, kCritEq2, FAKE, EDGE, true><<<grid, block, lds, st>>>(g, riders, total);
            return;
        }
    }
    if (crit == kCritEq3) k_team_group<TEAM, kCritEq3, FAKE, EDGE, false><<<grid, block, lds, st>>>(g, riders, total);
    else k_team_group<TEAM, kCritEq2, FAKE, EDGE, false><<<grid, block, lds, st>>>(g, riders, total);
}
template <int TEAM>
void launch_team_kind(const GroupTeam& g, int64_t total, int crit, bool fake, bool edge, const SubRiders& riders, int64_t rider_blocks,
                      hipStream_t st) {
    if (fake) {
        if (edge) launch_team_crit<TEAM, true, true>(g, total, crit, riders, rider_blocks, st);
        else launch_team_crit<TEAM, true, false>(g, total, crit, riders, rider_blocks, st);
    } else {
        if (edge) launch_team_crit<TEAM, false, true>(g, total, crit, riders, rider_blocks, st);
        else launch_team_crit<TEAM, false, false>(g, total, crit, riders, rider_blocks, st);
    }
}
// Does the operand need per-lane validity predicates in the team kernel of this kind?
bool team_needs_edge(const BatchItem& it, int kind) {
    switch (kind) {
    case kTeamWg128: return it.sh.rows % 128 != 0 || it.sh.cols % 128 != 0;
    case kTeamHalf64: return it.sh.rows % 64 != 0 || it.sh.cols % 128 != 0;      // a wave spans 128 columns
    default: return false;      // row teams always use the bounds-checked accesses
    }
}
}  // namespace

int team_kind_of(const BatchItem& it) {
    switch (it.gran) {
    case kGranBlock: return kTeamWg128;
    case kGranBlock64: return kTeamHalf64;
    case kGranRow: return it.sh.cols <= 4096 ? kTeamWaveRow : (it.sh.cols <= 16384 ? kTeamWgRow : kTeamBigRow);
    default: return -1;
    }
}

// All operands of `items` (indices idx[0..cnt)) that share one team kind and criterion, in groups.  `riders`
// (may be null): flat 1 x 128 operands of the same criterion that ride on the first 128 x 128 launch whose output
// kind (FP8 payload or fake quantization) matches theirs; `riders->used` is set when they went along.
hipError_t launch_team_items(const BatchItem* items, const int* idx, int cnt, int kind, int crit, const uint32_t* const* gam_of,
                             TeamRiders* riders, hipStream_t st, KProf* prof) {
    static_assert(sizeof(GroupTeam) + sizeof(SubRiders) <= 3800 && sizeof(GroupCol) <= 3800, "kernel-argument segment is 4 KB");
    SubRiders none; none.n = 0;
    for (int variant = 0; variant < 4; ++variant) {
    const bool fake = (variant & 1) != 0, edge = (variant & 2) != 0;
    GroupTeam g; g.n = 0;
    int64_t total = 0;
    auto flush = [&]() {
        if (g.n == 0) return;
        ProfScope ps(prof, kKernTeamBlock, st);
        const bool ride = kind == kTeamWg128 && riders && !riders->used && riders->table.n > 0 && riders->fake == fake;
        const SubRiders& rt = ride ? riders->table : none;
        const int64_t rb = ride ? riders->blocks : 0;
        if (ride) riders->used = true;
        switch (kind) {
        case kTeamWg128: launch_team_kind<kTeamWg128>(g, total, crit, fake, edge, rt, rb, st); break;
        case kTeamHalf64: launch_team_kind<kTeamHalf64>(g, total, crit, fake, edge, rt, rb, st); break;
        case kTeamWaveRow: launch_team_kind<kTeamWaveRow>(g, total, crit, fake, edge, rt, rb, st); break;
        case kTeamWgRow: launch_team_kind<kTeamWgRow>(g, total, crit, fake, edge, rt, rb, st); break;
        default: launch_team_kind<kTeamBigRow>(g, total, crit, fake, edge, rt, rb, st); break;
        }
        g.n = 0; total = 0;
    };
    for (int k = 0; k < cnt; ++k) {
        const BatchItem& it = items[idx[k]];
        if ((it.o.fake != nullptr) != fake || team_needs_edge(it, kind) != edge) continue;
        int64_t units;
        TeamOp& t = g.op[g.n];
        t.units_x = kind == kTeamHalf64 ? (it.sh.cols + 255) / 256 : (it.sh.cols + 127) / 128;
        if (kind == kTeamWg128 || kind == kTeamHalf64) units = ((it.sh.rows + 127) / 128) * t.units_x;
        else if (kind == kTeamWaveRow) units = (it.sh.rows + 3) / 4;
        else units = it.sh.rows;
        if (units > 0x7FFFFFFF) return hipErrorInvalidValue;
        if (total + units > 0x7FFF0000) { flush(); }       // leaves room for the riders' workgroups
        TeamOp& u = g.op[g.n];
        u.x = it.x; u.o = it.o; u.ld = it.sh.ld; u.rows = it.sh.rows; u.cols = it.sh.cols;
        u.units_x = kind == kTeamHalf64 ? (it.sh.cols + 255) / 256 : (it.sh.cols + 127) / 128;
        u.th = it.th; u.defer = it.scope == 1; u.mode = (uint8_t)it.scaling; u.three = (uint8_t)it.three;
        u.prove = scope_proof_applies(it);
        u.gam = gam_of[idx[k]];
        u.group_rows = (uint32_t)it.group_rows;
        total += units;
        g.unit_end[g.n] = total;
        if (++g.n == kMaxTeamGroup) flush();
    }
    flush();
    }
    return hipGetLastError();
}

hipError_t launch_block_amax_prove(const BlockProveItem* ops, int n, hipStream_t st) {
    static_assert(sizeof(GroupProve) <= 3800, "kernel-argument segment is 4 KB");
    for (int base = 0; base < n; base += kMaxTeamGroup) {
        GroupProve g; g.n = 0;
        int end = 0;
        for (int k = base; k < n && k < base + kMaxTeamGroup; ++k) {
            ProveOp& t = g.op[g.n];
            t.x = ops[k].x; t.ld = ops[k].ld; t.cols = ops[k].cols; t.kind = ops[k].kind;
            if (t.kind == kProveRows) { t.units_x = (ops[k].cols + kProvePiece - 1) / kProvePiece; t.n_units = ops[k].rows * t.units_x; }
            else { t.units_x = ops[k].cols / 128; t.n_units = (ops[k].rows / 128) * t.units_x; }
            t.amax_part = ops[k].amax_part; t.flush_part = ops[k].flush_part;
            end += ops[k].n_wg;
            g.wg_end[g.n++] = end;
        }
        k_block_amax_prove<<<dim3((unsigned)end), dim3(256), 0, st>>>(g);
    }
    return hipGetLastError();
}

// ---- column kinds
namespace {
struct ColPlan {
    int32_t tiles_per_strip;
    int n_strips;
    int64_t cols_padded;
    size_t off_amax, off_err, off_err5, off_zero, off_scale, off_scale5, off_amin, off_proven, off_wg, bytes;
};
ColPlan plan_columns(int64_t rows, int64_t cols) {
    ColPlan pl;
    const int64_t tiles_x = (cols + 127) / 128, tiles_y = (rows + 127) / 128;
    int64_t per = (tiles_x * tiles_y + 1023) / 1024;      // ~1024 workgroups per large operand: the per-workgroup set-up is amortised over several tiles
    if (per < 1) per = 1;
    if (per > 16) per = 16;                               // 16-bit zero counters: 16 tiles x 128 rows
    pl.tiles_per_strip = (int32_t)per;
    pl.n_strips = (int)((tiles_y + per - 1) / per);
    pl.cols_padded = tiles_x * 128;
    const size_t n = (size_t)pl.n_strips * (size_t)pl.cols_padded;
    size_t off = 0;
    pl.off_amax = off; off = align16p(off + 2 * n);
    pl.off_err = off; off = align16p(off + 4 * n);
    pl.off_err5 = off; off = align16p(off + 4 * n);
    pl.off_zero = off; off = align16p(off + 2 * n);
    pl.off_scale = off; off = align16p(off + 4 * (size_t)pl.cols_padded);
    pl.off_scale5 = off; off = align16p(off + 4 * (size_t)pl.cols_padded);
    pl.off_amin = off; off = align16p(off + 2 * (size_t)pl.cols_padded);
    pl.off_proven = off; off = align16p(off + (size_t)pl.cols_padded);
    pl.off_wg = off; off = align16p(off + 4 * (2 + 2 * (size_t)pl.n_strips * (size_t)tiles_x));
    pl.bytes = off;
    return pl;
}
void fill_col_op(ColOp& t, const BatchItem& it, const uint32_t* gam) {
    t = ColOp{};
    t.x = it.x; t.o = it.o; t.ld = it.sh.ld; t.rows = it.sh.rows; t.cols = it.sh.cols;
    t.tiles_x = (it.sh.cols + 127) / 128;
    t.tiles_per_strip = 1;
    t.th = it.th; t.defer = it.scope == 1; t.mode = (uint8_t)it.scaling; t.three = (uint8_t)it.three;
    t.gam = gam;
    t.group_rows = it.gran == kGranSubCol ? (uint32_t)it.group_rows : 0u;
    t.prove = (it.gran == kGranSubCol && scope_proof_applies(it)) ? 1 : 0;     // (per-channel columns set their own meaning afterwards)
}
template <int MODE, bool FAKE, bool EDGE>
void launch_col_crit(const GroupCol& g, int64_t total, int crit, hipStream_t st) {
    const dim3 grid((unsigned)total), block(256);
    const int lds = MODE == kColExternal ? kResidency4 : 0;      // 0.609 ms per twelve-operand pass at 4 per unit, 0.620 uncapped
    if (crit == kCritEq3) k_col_group<kCritEq3, MODE, FAKE, EDGE><<<grid, block, lds, st>>>(g);
    else k_col_group<kCritEq2, MODE, FAKE, EDGE><<<grid, block, lds, st>>>(g);
}
template <int MODE>
void launch_col_kind(const GroupCol& g, int64_t total, int crit, bool fake, bool edge, hipStream_t st) {
    if (fake) { if (edge) launch_col_crit<MODE, true, true>(g, total, crit, st); else launch_col_crit<MODE, true, false>(g, total, crit, st); }
    else      { if (edge) launch_col_crit<MODE, false, true>(g, total, crit, st); else launch_col_crit<MODE, false, false>(g, total, crit, st); }
}
bool col_needs_edge(const BatchItem& it) { return it.sh.rows % 128 != 0 || it.sh.cols % 128 != 0; }
}  // namespace

uint32_t* column_tensor_proven_word(char* ws, int64_t rows, int64_t cols) {
    return reinterpret_cast<uint32_t*>(ws + plan_columns(rows, cols).off_wg);
}
size_t column_workspace_bytes(int64_t rows, int64_t cols) { return plan_columns(rows, cols).bytes; }

// 128 x 1 sub-columns: grouped, one pass.
hipError_t launch_subcol_items(const BatchItem* items, const int* idx, int cnt, int crit, const uint32_t* const* gam_of,
                               hipStream_t st, KProf* prof) {
    for (int variant = 0; variant < 4; ++variant) {
    const bool fake = (variant & 1) != 0, edge = (variant & 2) != 0;
    GroupCol g; g.n = 0;
    int64_t total = 0;
    auto flush = [&]() {
        if (g.n == 0) return;
        ProfScope ps(prof, kKernColumnTile, st);
        launch_col_kind<kColLocal>(g, total, crit, fake, edge, st);
        g.n = 0; total = 0;
    };
    for (int k = 0; k < cnt; ++k) {
        const BatchItem& it = items[idx[k]];
        if ((it.o.fake != nullptr) != fake || col_needs_edge(it) != edge) continue;
        const int64_t units = ((it.sh.rows + 127) / 128) * ((it.sh.cols + 127) / 128);
        if (units > 0x7FFFFFFF) return hipErrorInvalidValue;
        if (total + units > 0x7FFFFFFF) flush();
        fill_col_op(g.op[g.n], it, gam_of[idx[k]]);
        total += units;
        g.unit_end[g.n] = total;
        if (++g.n == kMaxTeamGroup) flush();
    }
    flush();
    }
    return hipGetLastError();
}

// Per-channel columns: all operands of one criterion share five launches per kernel variant (amax, scales, quantize,
// finish, fallback columns).  ws_of[k] is the workspace of operand idx[k] (column_workspace_bytes).
hipError_t launch_channel_col_items(const BatchItem* items, const int* idx, int cnt, int crit, const uint32_t* const* gam_of,
                                    char* const* ws_of, hipStream_t st, KProf* prof) {
    for (int variant = 0; variant < 4; ++variant) {
        const bool fake = (variant & 1) != 0, edge = (variant & 2) != 0;
        GroupCol g; g.n = 0;
        int64_t total = 0;
        int comb = 0, copy = 0;
        auto flush = [&]() {
            if (g.n == 0) return;
            // fallback-column pass: about kColCopyBudget workgroups over all operands of the launch (a workgroup that finds
            // every kept column already written costs a few nanoseconds of dispatch, which adds up over 12 000 of them)
            copy = 0;
            for (int k = 0; k < g.n; ++k) {
                ColOp& t = g.op[k];
                int64_t groups = (kColCopyBudget / g.n + t.tiles_x - 1) / t.tiles_x;
                if (groups < 2) groups = 2;
                if (groups > kColCopyRowGroups) groups = kColCopyRowGroups;
                t.copy_groups = (int32_t)groups;
                copy += (int)(t.tiles_x * groups);
                g.copy_end[k] = copy;
            }
            { ProfScope ps(prof, kKernColumnTile, st); launch_col_kind<kColAmax>(g, total, kCritEq2, false, edge, st); }
            { ProfScope ps(prof, kKernColumnCombine, st); k_col_scales<<<dim3((unsigned)comb), dim3(256), 0, st>>>(g); }
            { ProfScope ps(prof, kKernColumnTile, st); launch_col_kind<kColExternal>(g, total, crit, fake, edge, st); }
            {
                ProfScope ps(prof, kKernColumnCombine, st);
                if (crit == kCritEq3) k_col_finish<kCritEq3><<<dim3((unsigned)comb), dim3(256), 0, st>>>(g);
                else k_col_finish<kCritEq2><<<dim3((unsigned)comb), dim3(256), 0, st>>>(g);
            }
            { ProfScope ps(prof, kKernFallbackCopy, st); k_col_fallback<<<dim3((unsigned)copy), dim3(256), 0, st>>>(g); }
            g.n = 0; total = 0; comb = 0; copy = 0;
        };
        for (int k = 0; k < cnt; ++k) {
            const BatchItem& it = items[idx[k]];
            if ((it.o.fake != nullptr) != fake || col_needs_edge(it) != edge) continue;
            const ColPlan pl = plan_columns(it.sh.rows, it.sh.cols);
            const int64_t tiles_x = (it.sh.cols + 127) / 128;
            const int64_t units = (int64_t)pl.n_strips * tiles_x;
            if (units > 0x3FFFFFFF || tiles_x * kColCopyRowGroups > 0x3FFFFFFF) return hipErrorInvalidValue;
            if (total + units > 0x7FFFFFFF || (int64_t)copy + tiles_x * kColCopyRowGroups > 0x7FFFFFFF) flush();
            ColOp& t = g.op[g.n];
            fill_col_op(t, it, gam_of[idx[k]]);
            char* w = ws_of[k];
            t.tiles_per_strip = pl.tiles_per_strip;
            t.n_strips = pl.n_strips;
            t.part_amax = reinterpret_cast<uint16_t*>(w + pl.off_amax);
            t.part_err = reinterpret_cast<float*>(w + pl.off_err);
            t.part_err5 = reinterpret_cast<float*>(w + pl.off_err5);
            t.part_zero = reinterpret_cast<uint16_t*>(w + pl.off_zero);
            t.col_scale = reinterpret_cast<float*>(w + pl.off_scale);
            t.col_scale5 = reinterpret_cast<float*>(w + pl.off_scale5);
            t.col_amin = reinterpret_cast<uint16_t*>(w + pl.off_amin);
            t.col_proven = reinterpret_cast<uint8_t*>(w + pl.off_proven);
            t.prove = (crit == kCritEq2 && it.o.bf16 && !it.o.fake && !it.three && it.th > 0.0f && it.th < 0.9f) ? 1 : 0;
            t.flush_need = (uint32_t)flush_need_of(it.th, it.sh.rows);
            t.tensor_need = it.scope == 1 ? flush_need_of(it.th, it.sh.rows * it.sh.cols) : 0ull;
            t.wg = reinterpret_cast<uint32_t*>(w + pl.off_wg);
            t.derive_gam = it.scaling == kScaleGam ? 1 : 0;
            t.gmant = it.o.gmant;
            total += units;
            comb += (int)((pl.cols_padded + 255) / 256);
            copy += (int)(tiles_x * kColCopyRowGroups);          // upper bound, for the overflow check above; set in flush()
            g.unit_end[g.n] = total; g.comb_end[g.n] = comb;
            if (++g.n == kMaxTeamGroup) flush();
        }
        flush();
    }
    return hipGetLastError();
}

}  // namespace mor
