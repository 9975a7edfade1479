// Hybrid-sparse product for moderate K (at most eight 64-wide block columns) and many block-rows:
// a strip of X is turned into matrix-core operands once and kept in LDS for all block-rows.
//
// The kernels of spmm_reg.h give every (block-row, strip) a wave of its own: a layer with K = 256
// and S = 1024 fetches each strip of X sixteen times (from L2 after the first), and a wave lives for
// the two or three kept blocks of its block-row only: block list, X, store -- three dependent memory
// round trips per 64 x 64 outputs.  spmm_xres.h avoids that for K <= 128 by holding the strip's
// operands in registers.  Here a workgroup of four waves owns a strip of 64 columns:
//   * the waves bring the strip's K rows in (8 rows per request batch and lane half, as everywhere),
//     transpose pairs of rows into B operands with v_perm_b32 and leave them in LDS, operand-major:
//     the operand of lane l for block column kb, 16-deep step ks and column c of the lane's pair sits
//     at (((kb * 4 + ks) * 2 + c) * 64 + l) * 16 bytes -- one conflict-free ds_read_b128;
//   * after one barrier each wave walks every fourth block-row of the workgroup's group of block-rows
//     (Sec. 3.5: only the kept blocks), with the packed slice of the next block requested before
//     the current one is multiplied, and stores 64 output rows per block-row.
// X is read once per group of block-rows, the loop holds no X requests at all, and a wave lives for
// many block-rows.
#pragma once
#include "spmm_reg.h"
#include <atomic>

namespace crisp {

constexpr int XLDS_SHAPE = 22;          // launch shape code of this kernel for launch_reg_nm
constexpr int XLDS_MAX_KB = 8;          // block columns held at most (64 KB of operands)
constexpr int XLDS_MAX_GROUP = 60;      // block-rows per workgroup at most (row_ptr of the group sits in one register per lane)
constexpr int XLDS_LIST = 512;          // block-list entries of a group staged in LDS at most

// CONV == 4: X is the implicit lowering of a 1 x 1 filter with stride 2 (no padding, even W and Wo) over the
// activation [C][batch][H][W]: K-row c is channel c, and the lane's two columns are elements 0 and 2 of one
// 8-byte piece of input row 2 * oh, so the strided gather is done once per strip here instead of once per
// block-row.
template <int N, int M, bool SMF, int CONV>
__global__ __launch_bounds__(256, 4) void spmm_xlds_kernel(SpmmArgs p, int rows_per_group, int row_groups, int Kb) {
    static_assert(CONV == 0 || CONV == 4, "plain X or the strided 1 x 1 lowering");
    constexpr int B = 64;
    typedef Fmt<N, M, B> F;
    constexpr int RT = F::RT, KS = F::KS, NACC = 2;
    typedef BlockBody<N, M, B, 1, false, 0, SMF> Body;
    extern __shared__ __attribute__((aligned(16))) unsigned char xl[];   // Kb * 8 KB of operands, then the block list
    int* lst = reinterpret_cast<int*>(xl + (size_t)Kb * KS * NACC * 1024);
    constexpr bool LUT48 = lut48_pattern<N, M, SMF>();     // dense expansion of 4:8 through the selector table
    __shared__ u32x4 lut48[LUT48 ? 256 : 1];

    const int id = blockIdx.x;
    const int rg = id % row_groups, nt = id / row_groups;
    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int jj = lane & 31, hh = lane >> 5;
    const int64_t col0 = (int64_t)nt * 64 + jj * NACC;
    const bool col_ok = col0 < p.Ncol;
    const int64_t col_ld = col_ok ? col0 : 0;     // lanes past the last column read column 0 and never store
    uint32_t lane_off;
    if constexpr (CONV == 4) {
        // column -> (image, oh, ow); exact division through fp64 reciprocals (col < 2^31)
        const int j = (int)col_ld;
        int t = (int)((double)j * p.inv_Wo);
        t -= (t * p.Wo > j);
        t += ((t + 1) * p.Wo <= j);
        const int ow = j - t * p.Wo;
        int im = (int)((double)t * p.inv_Ho);
        im -= (im * p.Ho > t);
        im += ((im + 1) * p.Ho <= t);
        const int oh = t - im * p.Ho;
        lane_off = (uint32_t)((int64_t)hh * 8 * p.plane * 2) + (uint32_t)((im * p.H + oh * 2) * p.W + ow * 2) * 2u;
    } else {
        lane_off = (uint32_t)(((int64_t)hh * 8 * p.ldx + col_ld) * 2);
    }
    const uint32_t a_off = (uint32_t)((jj * F::SLOTS + hh * F::FS * (SMF ? 2 : 1)) * 2);
    const uint32_t i_off = (uint32_t)(jj * F::WPR * 4);
    const uint32_t aw_sh = (uint32_t)hh * F::HB * (SMF ? 2 : 1);

    // the group's block list: lane l holds row_ptr[bi0 + l]; the block columns go to LDS
    const int bi0 = rg * rows_per_group;
    const int bi1 = min(bi0 + rows_per_group, p.Sb);
    const int my_ptr = p.row_ptr[min(bi0 + lane, p.Sb)];
    const int t0 = __builtin_amdgcn_readfirstlane(my_ptr);
    const int t1 = __builtin_amdgcn_readlane(my_ptr, bi1 - bi0);                  // end of the group's list
    for (int i = tid; i < min(t1 - t0, XLDS_LIST); i += 256) lst[i] = p.col_idx[t0 + i];
    if constexpr (LUT48) lut48_fill(lut48, tid, 256);

    // ---- X rows of the strip -> B operands in LDS.  Unit u = (block column, 16-deep step); a wave takes
    // every fourth unit, four units (32 requests) in flight before the first is transposed ----
    {
        const int units = Kb * KS;
        const uint32_t row_bytes = CONV == 4 ? (uint32_t)p.plane * 2u : (uint32_t)p.ldx * 2u;
        typedef typename XVec<CONV == 4 ? 2 : 1>::type xv_t;
        for (int u0 = wave; u0 < units; u0 += 16) {
            xv_t xr[4][8];
#pragma unroll
            for (int k = 0; k < 4; ++k) {
                const int u = min(u0 + 4 * k, units - 1);
                // a step past the end of K re-reads the last 16 rows (finite values times stored zeros)
                const int k_first = min(u * 16, p.K - 16);
                const rsrc_t r = CONV == 4 ? make_rsrc(p.act + (int64_t)k_first * p.plane) : make_rsrc(p.X + (int64_t)k_first * p.ldx);
#pragma unroll
                for (int i = 0; i < 8; ++i) xr[k][i] = buf_load_x<CONV == 4 ? 2 : 1>(r, lane_off, (uint32_t)i * row_bytes);
            }
#pragma unroll
            for (int k = 0; k < 4; ++k) {
                const int u = u0 + 4 * k;
                if (u < units) {
                    u32x4 lo, hi;
#pragma unroll
                    for (int q = 0; q < 4; ++q) {
                        if constexpr (CONV == 4) {
                            uint32_t r0[2], r1[2];
                            xvec_unpack(xr[k][2 * q], r0);
                            xvec_unpack(xr[k][2 * q + 1], r1);
                            lo[q] = __builtin_amdgcn_perm(r1[0], r0[0], SEL_LO);   // element 0 of the piece: first column
                            hi[q] = __builtin_amdgcn_perm(r1[1], r0[1], SEL_LO);   // element 2: second column
                        } else {
                            uint32_t r0[1], r1[1];
                            xvec_unpack(xr[k][2 * q], r0);
                            xvec_unpack(xr[k][2 * q + 1], r1);
                            lo[q] = __builtin_amdgcn_perm(r1[0], r0[0], SEL_LO);   // first column of the pair
                            hi[q] = __builtin_amdgcn_perm(r1[0], r0[0], SEL_HI);   // second column
                        }
                    }
                    *reinterpret_cast<u32x4*>(xl + ((u * NACC + 0) * 64 + lane) * 16) = lo;
                    *reinterpret_cast<u32x4*>(xl + ((u * NACC + 1) * 64 + lane) * 16) = hi;
                }
            }
        }
    }
    __syncthreads();

    f32x16 acc[RT][NACC];
    const unsigned char* xlane = xl + lane * 16;
    auto multiply = [&](const uint32_t (&av)[RT][KS][F::VW], const uint32_t (&aw)[RT][F::WPR], int bj) __attribute__((always_inline)) {
        const unsigned char* bo = xlane + bj * (KS * NACC * 1024);
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
                u32x8 b8[NACC];
#pragma unroll
                for (int c = 0; c < NACC; ++c) {
                    const u32x4 lo = *reinterpret_cast<const u32x4*>(bo + ((2 * s2) * NACC + c) * 1024);
                    const u32x4 hi = *reinterpret_cast<const u32x4*>(bo + ((2 * s2 + 1) * NACC + c) * 1024);
                    b8[c] = u32x8{lo[0], lo[1], lo[2], lo[3], hi[0], hi[1], hi[2], hi[3]};
                }
#pragma unroll
                for (int rt = 0; rt < RT; ++rt) {
                    u32x4 a4;
                    uint32_t idx;
                    if (s2 == 0) smf_operand<N, M, B, 0>(av[rt], ws[rt], a4, idx);
                    else smf_operand<N, M, B, 1>(av[rt], ws[rt], a4, idx);
                    const bf16x8 afrag = __builtin_bit_cast(bf16x8, a4);
#pragma unroll
                    for (int c = 0; c < NACC; ++c)
                        acc[rt][c] = __builtin_amdgcn_smfmac_f32_32x32x32_bf16(afrag, __builtin_bit_cast(bf16x16, b8[c]), acc[rt][c],
                                                                               (int)idx, 0, 0);
                }
            }
        } else {
            auto dense_step = [&](auto ks_c) __attribute__((always_inline)) {
                constexpr int ks = decltype(ks_c)::value;
                u32x4 b4[NACC];
#pragma unroll
                for (int c = 0; c < NACC; ++c) b4[c] = *reinterpret_cast<const u32x4*>(bo + (ks * NACC + c) * 1024);
#pragma unroll
                for (int rt = 0; rt < RT; ++rt) {
                    u32x4 a4;
                    if constexpr (LUT48) a4 = expand_frag_lut48<B, ks>(av[rt][ks], ws[rt], lut48);
                    else a4 = expand_frag<N, M, B, ks>(av[rt][ks], ws[rt]);
                    const bf16x8 afrag = __builtin_bit_cast(bf16x8, a4);
#pragma unroll
                    for (int c = 0; c < NACC; ++c)
                        acc[rt][c] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(afrag, __builtin_bit_cast(bf16x8, b4[c]), acc[rt][c], 0, 0, 0);
                }
            };
            dense_step(std::integral_constant<int, 0>{});
            dense_step(std::integral_constant<int, 1>{});
            dense_step(std::integral_constant<int, 2>{});
            dense_step(std::integral_constant<int, 3>{});
        }
    };
    // block column of block t of the group (entries past the staged part of the list come from memory)
    auto column_of = [&](int t) __attribute__((always_inline)) {
        const int i = t - t0;
        const int bj = i < XLDS_LIST ? lst[i] : p.col_idx[t];
        return __builtin_amdgcn_readfirstlane(bj);
    };

    // ---- the wave's block-rows: bi0 + wave, + 4, ...  One packed slice in flight: the next block's (of this
    // wave: the first block of its next non-empty block-row when the row ends) is requested as soon as the
    // current one has been handed to the matrix core, i.e. before the block-row's 64 rows are stored ----
    uint32_t av[RT][KS][F::VW], aw[RT][F::WPR];
    // first block of this wave's rows from row `bi` on (t1 if there is none)
    auto next_block_from = [&](int bi) __attribute__((always_inline)) {
        int t = t1;
        for (int b = bi; b < bi1; b += 4) {
            const int tb = __builtin_amdgcn_readlane(my_ptr, b - bi0), te = __builtin_amdgcn_readlane(my_ptr, b + 1 - bi0);
            if (tb < te) { t = tb; break; }
        }
        return t;
    };
    {
        const int tf = next_block_from(bi0 + wave);
        if (tf < t1) Body::load_a(av, aw, p, a_off, i_off, tf);
    }
    for (int bi = bi0 + wave; bi < bi1; bi += 4) {
        const int t_begin = __builtin_amdgcn_readlane(my_ptr, bi - bi0);
        const int t_end = __builtin_amdgcn_readlane(my_ptr, bi + 1 - bi0);
#pragma unroll
        for (int rt = 0; rt < RT; ++rt)
#pragma unroll
            for (int c = 0; c < NACC; ++c)
#pragma unroll
                for (int r = 0; r < 16; ++r) acc[rt][c][r] = 0.0f;
        for (int t = t_begin; t < t_end; ++t) {
            const int bj = column_of(t);
            multiply(av, aw, bj);
            const int tn = t + 1 < t_end ? t + 1 : next_block_from(bi + 4);
            Body::load_a(av, aw, p, a_off, i_off, min(tn, t1 - 1));      // past the end: the last block again, never used
        }
        int hh_now = hh;
        asm volatile("" : "+v"(hh_now));
#pragma unroll
        for (int r0 = 0; r0 < RT * 16; r0 += 8)
            store_rows<B, 1, 8, 1>(p, bi, hh_now, col0, col_ok, r0, [&](int pr, float (&v)[NACC]) __attribute__((always_inline)) {
#pragma unroll
                for (int c = 0; c < NACC; ++c) v[c] = acc[pr >> 4][c][pr & 15];
            });
    }
}

// Covered: 64 x 64 blocks, K <= 512 and a multiple of 16, Ncol a multiple of 4; plain X, or the fused
// lowering of a strided 1 x 1 filter (conv mode 4; channel planes of at most 2^27 elements as for every fused
// lowering).
inline bool xlds_covers(const SpmmArgs& a, int B) {
    const bool x_ok = a.act == nullptr ? a.ldx <= ((int64_t)1 << 23) : a.conv_mode == 4;
    return x_ok && B == 64 && a.K <= XLDS_MAX_KB * 64 && (a.K % 16) == 0 && (a.Ncol % 4) == 0 &&
           a.ldy <= ((int64_t)1 << 23) && !(a.ep_on && a.ep_res && a.ep_ldr > ((int64_t)1 << 23));
}

template <int N, int M, bool SMF, int CONV>
hipError_t launch_xlds_k(const SpmmArgs& a, hipStream_t st) {
    const int Kb = (a.K + 63) / 64;
    const int64_t strips = (a.Ncol + 63) / 64;
    // all block-rows in one group unless that leaves a compute unit without a workgroup (measured on
    // 2048 x 512 x 12544: 392 workgroups of 16 block-rows 20-23 us, 784 of 8 26-30 us, 196 of 32 26-30 us;
    // on 1024 x 256 x 50176: 784 workgroups of 16 block-rows 32 us, 1568 of 8 40 us); a group has at least
    // four block-rows (one per wave)
    int rpg = a.Sb < XLDS_MAX_GROUP ? a.Sb : XLDS_MAX_GROUP;
    while (rpg > 4 && strips * ((a.Sb + rpg - 1) / rpg) < 256) rpg = (rpg + 1) / 2;
    const int row_groups = (a.Sb + rpg - 1) / rpg;
    const int64_t wgs = strips * row_groups;
    if (wgs > INT32_MAX) return hipErrorInvalidValue;
    const size_t lds = (size_t)Kb * 8192 + XLDS_LIST * 4;
    if (lds > 64 * 1024) {
        // more dynamic LDS than a kernel gets by default: raised once per device for this instantiation
        static std::atomic<uint64_t> raised{0};
        int dev = 0;
        if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= 64) return hipErrorInvalidDevice;
        if (!(raised.load() >> dev & 1)) {
            const hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(&spmm_xlds_kernel<N, M, SMF, CONV>),
                                                     hipFuncAttributeMaxDynamicSharedMemorySize, XLDS_MAX_KB * 8192 + XLDS_LIST * 4);
            if (e != hipSuccess) return e;
            raised.fetch_or((uint64_t)1 << dev);
        }
    }
    const dim3 grd((unsigned)wgs), blk(256);
    if (a.ev_start || a.ev_stop)
        hipExtLaunchKernelGGL((spmm_xlds_kernel<N, M, SMF, CONV>), grd, blk, lds, st, a.ev_start, a.ev_stop, 0, a, rpg, row_groups, Kb);
    else
        spmm_xlds_kernel<N, M, SMF, CONV><<<grd, blk, lds, st>>>(a, rpg, row_groups, Kb);
    return hipGetLastError();
}

template <int N, int M>
hipError_t launch_xlds(const SpmmArgs& a, hipStream_t st) {
    const bool strided = a.act != nullptr;
    if constexpr (smf_pattern<N, M>() || smf_flagged_pattern<N, M>()) {
        if (smf_wanted<N, M>(a)) return strided ? launch_xlds_k<N, M, true, 4>(a, st) : launch_xlds_k<N, M, true, 0>(a, st);
    }
    return strided ? launch_xlds_k<N, M, false, 4>(a, st) : launch_xlds_k<N, M, false, 0>(a, st);
}

}  // namespace crisp
