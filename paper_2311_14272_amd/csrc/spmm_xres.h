// Hybrid-sparse product for short K (at most two 64-wide block columns): X stays in registers.
//
// With one or two block columns every block-row that keeps anything needs the same few X rows
// (Sec. 3.5 walks the kept blocks of a block-row; here all block-rows walk the same one or two).
// The kernels of spmm_reg.h give every block-row a wave of its own, so the strip of X is fetched
// once per block-row and each wave lives for one block only: three dependent memory round trips
// (block list, X, store) per 64 x 64 outputs.  Here a wave owns a strip of 64 columns, turns its X
// rows into matrix-core B operands once, and walks a group of block-rows with them: per block-row
// one packed slice is fetched (the next one is requested before the current rows are stored) and
// 64 output rows are stored.  X is read once per group of block-rows instead of once per block-row.
#pragma once
#include "spmm_reg.h"

namespace crisp {

constexpr int XRES_SHAPE = 20;          // launch shape code of this kernel for launch_reg_nm
constexpr int XRES_MAX_GROUP = 32;      // block-rows per wave at most (their block list sits in one register per lane)

// KB: block columns held (1 or 2).  rows_per_group: block-rows a wave walks.
template <int N, int M, bool SMF, int KB>
__global__ __launch_bounds__(256, 2) void spmm_xres_kernel(SpmmArgs p, int rows_per_group, int row_groups) {
    constexpr int B = 64;
    typedef Fmt<N, M, B> F;
    constexpr int RT = F::RT, KS = F::KS, NACC = 2;
    typedef BlockBody<N, M, B, 1, false, 0, SMF> Body;

    // workgroup -> (strip group, group of block-rows); the groups of block-rows of a strip group get
    // neighbouring ids
    const int id = blockIdx.x;
    const int rg = id % row_groups, nt = id / row_groups;
    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int jj = lane & 31, hh = lane >> 5;
    // selector table of the dense 4:8 expansion, built by the whole workgroup before any wave leaves
    constexpr bool LUT48 = lut48_pattern<N, M, SMF>();
    __shared__ u32x4 lut48[LUT48 ? 256 : 1];
    if constexpr (LUT48) {
        lut48_fill(lut48, tid, 256);
        __syncthreads();
    }
    const int64_t wave_col = ((int64_t)nt * 4 + wave) * 64;
    if (wave_col >= p.Ncol) return;                // no further barriers in this kernel
    const int64_t col0 = wave_col + jj * NACC;
    const bool col_ok = col0 < p.Ncol;
    const int64_t col_ld = col_ok ? col0 : 0;     // lanes past the last column read column 0 and never store
    const uint32_t lane_off = (uint32_t)(((int64_t)hh * 8 * p.ldx + col_ld) * 2);
    const uint32_t a_off = (uint32_t)((jj * F::SLOTS + hh * F::FS * (SMF ? 2 : 1)) * 2);
    const uint32_t i_off = (uint32_t)(jj * F::WPR * 4);
    const uint32_t aw_sh = (uint32_t)hh * F::HB * (SMF ? 2 : 1);

    // the group's block list, read before anything is stored: lane l holds row_ptr[bi0 + l] and the
    // block column of the group's l-th block (at most XRES_MAX_GROUP block-rows x KB blocks <= 64)
    const int bi0 = rg * rows_per_group;
    const int bi1 = min(bi0 + rows_per_group, p.Sb);
    const int my_ptr = p.row_ptr[min(bi0 + lane, p.Sb)];
    const int t0 = __builtin_amdgcn_readfirstlane(my_ptr);
    const int t_last = __builtin_amdgcn_readlane(my_ptr, bi1 - bi0) - 1;          // last block of the group
    const int my_bj = p.col_idx[max(min(t0 + lane, t_last), 0)];

    // ---- X rows of the strip -> B operands (8 K-values of one column per register quad) ------------
    u32x4 bop[KB][KS][NACC];
    {
        uint32_t xr[KB][KS][8];
#pragma unroll
        for (int kb = 0; kb < KB; ++kb)
#pragma unroll
            for (int ks = 0; ks < KS; ++ks) {
                // a step past the end of K re-reads the last 16 rows (finite values times stored zeros)
                const int k_first = min(kb * B + ks * 16, p.K - 16);
                const rsrc_t r = make_rsrc(p.X + (int64_t)k_first * p.ldx);
                const uint32_t row_bytes = (uint32_t)p.ldx * 2u;
#pragma unroll
                for (int i = 0; i < 8; ++i) xr[kb][ks][i] = __builtin_amdgcn_raw_buffer_load_b32(r, lane_off, (uint32_t)i * row_bytes, 0);
            }
#pragma unroll
        for (int kb = 0; kb < KB; ++kb)
#pragma unroll
            for (int ks = 0; ks < KS; ++ks)
#pragma unroll
                for (int q = 0; q < 4; ++q) {
                    bop[kb][ks][0][q] = __builtin_amdgcn_perm(xr[kb][ks][2 * q + 1], xr[kb][ks][2 * q], SEL_LO);   // first column of the pair
                    bop[kb][ks][1][q] = __builtin_amdgcn_perm(xr[kb][ks][2 * q + 1], xr[kb][ks][2 * q], SEL_HI);   // second column
                }
    }

    f32x16 acc[RT][NACC];
    auto multiply = [&](const uint32_t (&av)[RT][KS][F::VW], const uint32_t (&aw)[RT][F::WPR], const u32x4 (&bo)[KS][NACC]) __attribute__((always_inline)) {
        uint32_t ws[RT][F::WPR];
        if constexpr (N != M) {
#pragma unroll
            for (int rt = 0; rt < RT; ++rt)
#pragma unroll
                for (int i = 0; i < F::WPR; ++i)
                    ws[rt][i] = __builtin_amdgcn_alignbit(i + 1 < F::WPR ? aw[rt][i + 1] : 0u, aw[rt][i], aw_sh);
        }
        if constexpr (SMF) {
#pragma unroll
            for (int s2 = 0; s2 < KS / 2; ++s2) {
                typedef __attribute__((ext_vector_type(8))) uint32_t u32x8;
#pragma unroll
                for (int rt = 0; rt < RT; ++rt) {
                    u32x4 a4;
                    uint32_t idx;
                    if (s2 == 0) smf_operand<N, M, B, 0>(av[rt], ws[rt], a4, idx);
                    else smf_operand<N, M, B, 1>(av[rt], ws[rt], a4, idx);
                    const bf16x8 afrag = __builtin_bit_cast(bf16x8, a4);
#pragma unroll
                    for (int c = 0; c < NACC; ++c) {
                        const u32x4 lo = bo[2 * s2][c], hi = bo[2 * s2 + 1][c];
                        const u32x8 b8 = {lo[0], lo[1], lo[2], lo[3], hi[0], hi[1], hi[2], hi[3]};
                        acc[rt][c] = __builtin_amdgcn_smfmac_f32_32x32x32_bf16(afrag, __builtin_bit_cast(bf16x16, b8), acc[rt][c],
                                                                               (int)idx, 0, 0);
                    }
                }
            }
        } else {
            auto dense_step = [&](auto ks_c) __attribute__((always_inline)) {
                constexpr int ks = decltype(ks_c)::value;
#pragma unroll
                for (int rt = 0; rt < RT; ++rt) {
                    u32x4 a4;
                    if constexpr (LUT48) a4 = expand_frag_lut48<B, ks>(av[rt][ks], ws[rt], lut48);
                    else a4 = expand_frag<N, M, B, ks>(av[rt][ks], ws[rt]);
                    const bf16x8 afrag = __builtin_bit_cast(bf16x8, a4);
#pragma unroll
                    for (int c = 0; c < NACC; ++c)
                        acc[rt][c] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(afrag, __builtin_bit_cast(bf16x8, bo[ks][c]), acc[rt][c], 0, 0, 0);
                }
            };
            dense_step(std::integral_constant<int, 0>{});
            dense_step(std::integral_constant<int, 1>{});
            dense_step(std::integral_constant<int, 2>{});
            dense_step(std::integral_constant<int, 3>{});
        }
    };

    // ---- the group's block-rows.  One packed slice in flight: the next block's is requested as soon
    // as the current one has been multiplied, i.e. before the block-row's 64 rows are stored ----
    uint32_t av[RT][KS][F::VW], aw[RT][F::WPR];
    int t = t0;
    if (t0 <= t_last) Body::load_a(av, aw, p, a_off, i_off, t0);
    for (int bi = bi0; bi < bi1; ++bi) {
        const int t_end = __builtin_amdgcn_readlane(my_ptr, bi + 1 - bi0);
#pragma unroll
        for (int rt = 0; rt < RT; ++rt)
#pragma unroll
            for (int c = 0; c < NACC; ++c)
#pragma unroll
                for (int r = 0; r < 16; ++r) acc[rt][c][r] = 0.0f;
        for (; t < t_end; ++t) {
            const int bj = __builtin_amdgcn_readlane(my_bj, t - t0);
            if (KB == 1 || bj == 0) multiply(av, aw, bop[0]);
            else multiply(av, aw, bop[KB - 1]);
            Body::load_a(av, aw, p, a_off, i_off, min(t + 1, t_last));   // past the end: the last block again, never used
        }
        // the lane's row half behind an opaque copy: the row addresses are then computed here, per
        // block-row, instead of being kept in (spilled) registers across the whole loop
        int hh_now = hh;
        asm volatile("" : "+v"(hh_now));
        // eight rows at a time: the epilogue's operands of a batch of rows live beside the X operands
#pragma unroll
        for (int r0 = 0; r0 < RT * 16; r0 += 8)
            store_rows<B, 1, 8, 1>(p, bi, hh_now, col0, col_ok, r0, [&](int pr, float (&v)[NACC]) __attribute__((always_inline)) {
#pragma unroll
                for (int c = 0; c < NACC; ++c) v[c] = acc[pr >> 4][c][pr & 15];
            });
    }
}

// Covered: plain X (no lowering), 64 x 64 blocks, K <= 128 and a multiple of 16, Ncol a multiple of 4.
inline bool xres_covers(const SpmmArgs& a, int B) {
    return a.act == nullptr && B == 64 && a.K <= 128 && (a.K % 16) == 0 && (a.Ncol % 4) == 0 && a.ldy <= ((int64_t)1 << 23) &&
           !(a.ep_on && a.ep_res && a.ep_ldr > ((int64_t)1 << 23));
}

template <int N, int M, bool SMF, int KB>
hipError_t launch_xres_k(const SpmmArgs& a, hipStream_t st) {
    const int64_t strips = (a.Ncol + 255) / 256;
    // all block-rows in one group unless that leaves the chip short of workgroups
    int rpg = a.Sb < XRES_MAX_GROUP ? a.Sb : XRES_MAX_GROUP;
    while (rpg > 2 && strips * ((a.Sb + rpg - 1) / rpg) < 1024) rpg = (rpg + 1) / 2;
    const int row_groups = (a.Sb + rpg - 1) / rpg;
    const int64_t wgs = strips * row_groups;
    if (wgs > INT32_MAX) return hipErrorInvalidValue;
    const dim3 grd((unsigned)wgs), blk(256);
    if (a.ev_start || a.ev_stop)
        hipExtLaunchKernelGGL((spmm_xres_kernel<N, M, SMF, KB>), grd, blk, 0, st, a.ev_start, a.ev_stop, 0, a, rpg, row_groups);
    else
        spmm_xres_kernel<N, M, SMF, KB><<<grd, blk, 0, st>>>(a, rpg, row_groups);
    return hipGetLastError();
}

template <int N, int M>
hipError_t launch_xres(const SpmmArgs& a, hipStream_t st) {
    if constexpr (smf_pattern<N, M>() || smf_flagged_pattern<N, M>()) {
        if (smf_wanted<N, M>(a)) return a.K <= 64 ? launch_xres_k<N, M, true, 1>(a, st) : launch_xres_k<N, M, true, 2>(a, st);
    }
    return a.K <= 64 ? launch_xres_k<N, M, false, 1>(a, st) : launch_xres_k<N, M, false, 2>(a, st);
}

}  // namespace crisp
