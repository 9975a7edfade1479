// Hybrid-sparse product for block-rows of uneven length (plain block pruning over the whole grid,
// CRISP_LAYER_TOPK: the non-uniform baseline that Sec. 3.1 / 3.3 contrast the uniform rows with).
//
// The kernels of spmm_reg.h give every (block-row, column strip) one wave, whatever the row holds:
// a row with 30 kept blocks keeps its wave 30 times as long as a row with one, and an empty row
// still costs a wave.  Here the unit of work is the kept block.  row_ptr is the exclusive prefix
// sum of the rows' block counts, so "the blocks of rows [r0, r1)" is the range
// [row_ptr[r0], row_ptr[r1]) of the block list:
//   * the block-rows are cut into G groups of about nk / G blocks each -- group g starts at the
//     first row whose prefix sum reaches g * nk / G, found by every wave with ballots and
//     population counts over row_ptr (a wave-level search in the prefix sums);
//   * a workgroup owns (column strip, group) and deals the group's blocks evenly to its 4 waves:
//     wave w takes blocks [T0 + cnt*w/4, T0 + cnt*(w+1)/4) wherever the row boundaries fall;
//   * a wave walks its blocks in list order.  A row that lies wholly inside the wave's range is
//     stored straight from the accumulators.  A row cut by the range boundaries is finished by the
//     wave that holds its first block: the waves that hold later parts leave their partial tile in
//     LDS (one per wave at most: only the first row of a range can have begun earlier) and the owner
//     adds them in wave order after one barrier -- a fixed order, so results are reproducible;
//   * rows without any kept block are written as zeros (through the epilogue) by wave (row % 4).
#pragma once
#include "spmm_reg.h"

namespace crisp {

constexpr int BAL_NW = 4;                 // waves per workgroup
constexpr int BAL_MAX_ROWS = 1024;        // block-rows at most (row_ptr is held in LDS; three workgroups share a compute unit)

template <int N, int M, int B, bool SMF>
__global__ __launch_bounds__(64 * BAL_NW) __attribute__((amdgpu_waves_per_eu(2, 3))) void spmm_balanced_kernel(SpmmArgs p, int G) {
    typedef Fmt<N, M, B> F;
    constexpr int RT = F::RT, KS = F::KS, NACC = 2, NW = BAL_NW;
    typedef BlockBody<N, M, B, 1, true, 0, SMF> BodyP;
    typedef BlockBody<N, M, B, 1, false, 0, SMF> BodyL;
    typedef typename BodyP::xvec_t xvec_t;

    __shared__ int rp[BAL_MAX_ROWS + 1];                  // row_ptr
    __shared__ int cnt_lo[NW], cnt_hi[NW];                // per-wave counts of the boundary search
    __shared__ int head_row[NW];                          // block-row of the partial tile a wave left (-1: none)
    __shared__ float part[NW - 1][RT * 16][NACC][64];     // partial tiles of waves 1 .. NW-1 (wave 0 begins at a row boundary)

    // workgroup -> (column strip, group of block-rows); the groups of a strip get neighbouring ids
    // on one XCD (ids are dealt round-robin to the 8 XCDs) so that they share its L2 for X
    const int id = blockIdx.x;
    const int xcd = id & 7, slot = id >> 3;
    const int g = slot % G;
    const int nt = (slot / G) * 8 + xcd;
    if (nt >= p.NT) return;

    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    // selector table of the dense 4:8 expansion (visible after the barrier that follows the row_ptr copy)
    constexpr bool LUT48 = lut48_pattern<N, M, SMF>();
    __shared__ u32x4 lut48[LUT48 ? 256 : 1];
    if constexpr (LUT48) lut48_fill(lut48, tid, 64 * NW);
    const int jj = lane & 31, hh = lane >> 5;
    const int64_t wave_col = (int64_t)nt * 64;
    const int64_t col0 = wave_col + jj * NACC;
    const bool col_ok = col0 < p.Ncol;
    const int64_t col_ld = col_ok ? col0 : 0;             // lanes past the last column read column 0 and never store
    const uint32_t lane_off = (uint32_t)(((int64_t)hh * 8 * p.ldx + col_ld) * 2);
    const uint32_t a_off = (uint32_t)((jj * F::SLOTS + hh * F::FS * (SMF ? 2 : 1)) * 2);
    const uint32_t i_off = (uint32_t)(jj * F::WPR * 4);
    const uint32_t aw_sh = (uint32_t)hh * F::HB * (SMF ? 2 : 1);

    // ---- the group's rows: a search in the prefix sums with ballots -------------------------------
    // first row of group g = number of entries row_ptr[0 .. Sb] below g * nk / G (the entries ascend)
    const int nk = p.row_ptr[p.Sb];
    const int target_lo = (int)((int64_t)g * nk / G), target_hi = (int)((int64_t)(g + 1) * nk / G);
    int below_lo = 0, below_hi = 0;
    for (int base = 0; base <= p.Sb; base += 64 * NW) {
        const int i = base + tid;
        const int v = i <= p.Sb ? p.row_ptr[i] : 0x7FFFFFFF;
        if (i <= p.Sb) rp[i] = v;
        below_lo += __popcll(__ballot(v < target_lo));
        below_hi += __popcll(__ballot(v < target_hi));
    }
    if (lane == 0) { cnt_lo[wave] = below_lo; cnt_hi[wave] = below_hi; head_row[wave] = -1; }
    __syncthreads();
    // (values read back from LDS are the same in every lane; readfirstlane tells the compiler so, which keeps
    // the block walk below in scalar registers)
    auto rpu = [&](int i) __attribute__((always_inline)) { return __builtin_amdgcn_readfirstlane(rp[i]); };
    int r0 = 0, r1 = 0;
#pragma unroll
    for (int w = 0; w < NW; ++w) { r0 += cnt_lo[w]; r1 += cnt_hi[w]; }
    r0 = __builtin_amdgcn_readfirstlane(r0);
    r1 = __builtin_amdgcn_readfirstlane(r1);
    if (g == 0) r0 = 0;
    if (g == G - 1) r1 = p.Sb;                            // trailing rows without blocks belong to the last group
    r0 = min(r0, p.Sb); r1 = min(r1, p.Sb);
    if (r0 >= r1) return;                                 // whole workgroup (uniform), before the second barrier

    const int T0 = rpu(r0), T1 = rpu(r1);
    const int t0 = T0 + (int)((int64_t)(T1 - T0) * wave / NW), t1 = T0 + (int)((int64_t)(T1 - T0) * (wave + 1) / NW);

    f32x16 acc[RT][NACC];
    auto zero_acc = [&]() __attribute__((always_inline)) {
#pragma unroll
        for (int rt = 0; rt < RT; ++rt)
#pragma unroll
            for (int c = 0; c < NACC; ++c)
#pragma unroll
                for (int r = 0; r < 16; ++r) acc[rt][c][r] = 0.0f;
    };
    auto store_acc = [&](int bi) __attribute__((always_inline)) {
        // the lane's row half behind an opaque copy: the row addresses are then computed here, per row, instead
        // of being hoisted out of the loop over the rows and kept in (spilled) registers
        int hh_now = hh;
        asm volatile("" : "+v"(hh_now));
        store_rows<B, 1, RT * 16, 1>(p, bi, hh_now, col0, col_ok, 0, [&](int pr, float (&v)[NACC]) __attribute__((always_inline)) {
#pragma unroll
            for (int c = 0; c < NACC; ++c) v[c] = acc[pr >> 4][c][pr & 15];
        });
    };

    // ---- the group's rows: those that keep nothing are written as zeros by wave (row % NW); of the others a
    // wave takes, in order, those that intersect its block range.  Requests never cross a row boundary (the
    // last block of a row segment requests nothing), so no request is in flight while a row is stored and
    // the registers of the request ring are free for the store's own operands.
    for (int bi = r0; bi < r1; ++bi) {
        if (rpu(bi) == rpu(bi + 1) && (bi & (NW - 1)) == wave) {
            zero_acc();
            store_acc(bi);
        }
    }
    int pending_row = -1;                                 // row begun here that later waves continue
    const ConvPos cp = {0, 0, 0, 0u, 0, 0, 0, lut48};
    for (int bi = r0; bi < r1; ++bi) {
        const int row_begin = rpu(bi), row_end = rpu(bi + 1);
        bool store = false;
        {
            const int seg_begin = max(row_begin, t0), seg_end = min(row_end, t1);
            if (seg_begin >= seg_end) continue;           // (also every row without blocks)
            zero_acc();
            {
                xvec_t xr[KS][8];
                uint32_t av[RT][KS][F::VW], aw[RT][F::WPR];
                XCtx cx = XCtx{lane_off, SEL_LO, SEL_HI, 0u};
                // The segment's part of the block list sits in one register, 64 entries at a time (lane l:
                // entry list_base + l), and is read with a lane index: the kernel stores between segments, so
                // the compiler would not use scalar loads for it, and a vector load per block would have to
                // be waited for before the block's successor could be requested.
                int list_base = seg_begin;
                int list = p.col_idx[min(seg_begin + lane, seg_end - 1)];
                auto block_column = [&](int tt) __attribute__((always_inline)) {
                    if (tt - list_base >= 64) {
                        list_base = tt;
                        list = p.col_idx[min(tt + lane, seg_end - 1)];
                    }
                    return __builtin_amdgcn_readlane(list, tt - list_base);
                };
                const int bj = block_column(seg_begin);
#pragma unroll
                for (int ks = 0; ks < KS; ++ks) BodyL::load_x(xr[ks], p, cp, cx.off, cx.off2, bj, ks);
                BodyL::load_a(av, aw, p, a_off, i_off, seg_begin);
                for (int t = seg_begin; t < seg_end - 1; ++t)
                    BodyP::run(acc, xr, av, aw, cx, p, cp, a_off, i_off, aw_sh, t + 1, block_column(t + 1));
                BodyL::run(acc, xr, av, aw, cx, p, cp, a_off, i_off, aw_sh, 0);
            }
            if (seg_begin > row_begin) {
                // a later part of a row that an earlier wave owns (only the first row of a range can be one)
#pragma unroll
                for (int rt = 0; rt < RT; ++rt)
#pragma unroll
                    for (int r = 0; r < 16; ++r)
#pragma unroll
                        for (int c = 0; c < NACC; ++c) part[wave - 1][rt * 16 + r][c][lane] = acc[rt][c][r];
                if (lane == 0) head_row[wave] = bi;
            } else if (seg_end == row_end) {
                store = true;                             // the whole row lies inside this wave's range
            } else {
                pending_row = bi;                         // its first part; the range ends here, so the loop does too
                break;
            }
        }
        if (store) store_acc(bi);
    }
    __syncthreads();
    if (pending_row >= 0) {
        // later waves' parts of the row, in wave order
        for (int w = wave + 1; w < NW; ++w) {
            if (__builtin_amdgcn_readfirstlane(head_row[w]) == pending_row) {
#pragma unroll
                for (int rt = 0; rt < RT; ++rt)
#pragma unroll
                    for (int r = 0; r < 16; ++r)
#pragma unroll
                        for (int c = 0; c < NACC; ++c) acc[rt][c][r] += part[w - 1][rt * 16 + r][c][lane];
            }
        }
        store_acc(pending_row);
    }
}

// Covered: plain X, B in {32, 64}, K a multiple of 16, Ncol a multiple of 4, at most BAL_MAX_ROWS
// block-rows, row strides of Y and of a residual within 2^23 (checked by the caller).
template <int N, int M, int B, bool SMF>
hipError_t launch_balanced_k(const SpmmArgs& a, hipStream_t st) {
    SpmmArgs p = a;
    p.NT = (int)((a.Ncol + 63) / 64);
    // groups of block-rows per strip: enough workgroups to give every compute unit four, but no more
    // groups than rows
    int G = (int)((1024 + p.NT - 1) / p.NT);
    if (G > a.Sb) G = a.Sb;
    if (G < 1) G = 1;
    const int64_t groups = (int64_t)((p.NT + 7) / 8) * G * 8;
    if (groups > INT32_MAX) return hipErrorInvalidValue;
    const dim3 grd((unsigned)groups), blk(64 * BAL_NW);
    if (a.ev_start || a.ev_stop)
        hipExtLaunchKernelGGL((spmm_balanced_kernel<N, M, B, SMF>), grd, blk, 0, st, a.ev_start, a.ev_stop, 0, p, G);
    else
        spmm_balanced_kernel<N, M, B, SMF><<<grd, blk, 0, st>>>(p, G);
    return hipGetLastError();
}

template <int N, int M>
hipError_t launch_balanced(const SpmmArgs& a, int B, hipStream_t st) {
    if constexpr (smf_pattern<N, M>()) {
        if (a.use_smf) return B == 64 ? launch_balanced_k<N, M, 64, true>(a, st) : launch_balanced_k<N, M, 32, true>(a, st);
    }
    return B == 64 ? launch_balanced_k<N, M, 64, false>(a, st) : launch_balanced_k<N, M, 32, false>(a, st);
}

}  // namespace crisp
