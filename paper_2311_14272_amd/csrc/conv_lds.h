// Hybrid-sparse convolution with the input staged in LDS (C a multiple of 64, 64x64 blocks).
//
// The fused lowering of spmm_reg.h fetches the X rows of every kept block straight from the
// convolution's input: for a kh x kw filter the same input element is then fetched up to kh*kw
// times per block-row that keeps its channel block (Sec. 3.5 walks kept blocks; the K index is
// (tap, channel), so the taps of one channel block are different block columns).  The level-1
// caches carry that inflated traffic and bound the 3x3 layers.  Here a workgroup owns a tile of
// output positions (whole output rows of one image) and up to four block-rows, and brings the
// input patch of one 64-channel block -- with its halo -- into LDS once; all taps and all
// block-rows read their operands from there.
//
// LDS layout: patch[row][col][channel], 64 channels (128 bytes, padded to 144) per position.  The
// matrix core's B operand -- 8 consecutive K values = 8 consecutive channels of one output
// position's tap -- is then one 16-byte LDS read, with no transposition in registers.
//
// Workgroup = 4 waves = RG block-rows x PT sub-tiles of R output rows each (RG * PT = 4).  A wave
// walks the kept blocks of its block-row in (channel block, tap) order; the packed slice of the
// next block is requested while the current one is multiplied.
#pragma once
#include "spmm_reg.h"
#include "spmm_xres.h"
#include "spmm_xlds.h"
#include "conv_patch.h"
#include "spmm_balanced.h"
#include "spmm_k8.h"

namespace crisp {

constexpr int CONV_LDS_POS_BYTES = 144;      // 64 channels x 2 bytes + padding against bank conflicts
constexpr int CONV_LDS_MAX_KB = 128;         // block columns (taps x channel blocks)
constexpr int CONV_LDS_MAX_PATCH = 60 * 1024;
constexpr int CONV_LDS_ORD = CONV_LDS_MAX_KB + 3 * 64;    // entries of a wave's padded block list
constexpr uint32_t CONV_LDS_IDLE = 0x80000000u;

struct ConvLdsSched {
    int RG, PT, R;          // block-rows per workgroup, sub-tiles per workgroup, output rows per sub-tile
    int tiles_per_img;      // workgroup tiles (PT * R output rows) per image
    int row_groups;         // groups of RG block-rows
    int CB, kh, taps;       // channel blocks, filter height, kh * kw
    int PR, PC;             // patch rows and columns
    int row_mul, ih_step;   // patch rows per output row; input rows per patch row (a 1-row filter with a stride
                            // skips the input rows in between: row_mul 1, ih_step = stride; else stride, 1)
    int Kb;
};

template <int N, int M, bool SMF>
__global__ __launch_bounds__(256, 4) void conv_lds_kernel(SpmmArgs p, ConvLdsSched sc) {
    constexpr int B = 64;
    typedef Fmt<N, M, B> F;
    constexpr int RT = F::RT, KS = F::KS, NACC = 2;
    typedef BlockBody<N, M, B, 1, false, 0, SMF> Body;
    constexpr int PB = CONV_LDS_POS_BYTES;
    // packed slices in flight per wave (ring).  The kernel has to fit 128 registers so that four workgroups
    // share a compute unit (at three per compute unit it was 1.2-1.3x slower on the 14x14 layers of ResNet-50,
    // whose 1024 workgroups are exactly four per compute unit): two slices where a slice is ten or twelve
    // registers (at most two stored values per eight columns; 1.0-1.1x over a ring of one, most on 1:8),
    // else one
    constexpr int R = F::FS <= 2 ? 2 : 1;
    extern __shared__ __attribute__((aligned(16))) unsigned char patch[];      // [PR][PC][PB]
    __shared__ uint32_t kept_bits[4][CONV_LDS_MAX_KB / 32];
    // per wave: its kept blocks in (channel block, tap) order, each channel block's run padded with
    // idle entries to a multiple of the ring length R: (block index - t_begin) << 16 | byte offset of
    // the tap inside the patch, bit 31 = idle entry
    __shared__ uint32_t ord[4][CONV_LDS_ORD];
    __shared__ uint16_t cb_cnt[4][CONV_LDS_MAX_KB];    // kept blocks per channel block
    __shared__ uint16_t cb_end[4][CONV_LDS_MAX_KB];    // end of each channel block's padded run

    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int jj = lane & 31, hh = lane >> 5;
    const int rgp = (int)blockIdx.x % sc.row_groups;
    const int tile = (int)blockIdx.x / sc.row_groups;
    const int img = tile / sc.tiles_per_img;
    const int oh_base = (tile - img * sc.tiles_per_img) * sc.PT * sc.R;
    const int bi = rgp * sc.RG + wave % sc.RG;
    const int pt = wave / sc.RG;
    const int oh0 = oh_base + pt * sc.R;
    const int rows_valid = max(0, min(sc.R, p.Ho - oh0));
    const int TP = rows_valid * p.Wo;                 // output positions of this wave (even)
    const bool works = bi < p.Sb && TP > 0;

    // ---- the wave's kept blocks in (channel block, tap) order -------------------------------------
    for (int e = tid; e < 4 * (CONV_LDS_MAX_KB / 32); e += 256) (&kept_bits[0][0])[e] = 0u;
    // selector table of the dense 4:8 expansion (visible after the barriers below)
    constexpr bool LUT48 = lut48_pattern<N, M, SMF>();
    __shared__ u32x4 lut48[LUT48 ? 256 : 1];
    if constexpr (LUT48) lut48_fill(lut48, tid, 256);
    __syncthreads();
    int t_begin = 0, cnt = 0;
    if (works) {
        t_begin = p.row_ptr[bi];
        cnt = p.row_ptr[bi + 1] - t_begin;
        for (int e = lane; e < cnt; e += 64) {
            const int bj = p.col_idx[t_begin + e];
            atomicOr(&kept_bits[wave][bj >> 5], 1u << (bj & 31));
        }
    }
    __syncthreads();
    for (int e = tid; e < 4 * CONV_LDS_ORD; e += 256) (&ord[0][0])[e] = CONV_LDS_IDLE;
    if (works) {
        for (int cb = lane; cb < sc.CB; cb += 64) {
            int c = 0;
            for (int otap = 0; otap < sc.taps; ++otap) {
                const int o = otap * sc.CB + cb;
                c += (int)((kept_bits[wave][o >> 5] >> (o & 31)) & 1u);
            }
            cb_cnt[wave][cb] = (uint16_t)c;
        }
    }
    __syncthreads();
    if (works) {
        // block column bj = tap * CB + cb; its place in the list: the padded runs of the channel
        // blocks before cb, then the kept taps of cb before tap
        for (int bj = lane; bj < sc.Kb; bj += 64) {
            if ((kept_bits[wave][bj >> 5] >> (bj & 31)) & 1u) {
                const int tap = bj / sc.CB, cb = bj - tap * sc.CB;
                int place = 0;
                for (int ocb = 0; ocb < cb; ++ocb) place += (cb_cnt[wave][ocb] + R - 1) / R * R;
                for (int otap = 0; otap < tap; ++otap) {
                    const int o = otap * sc.CB + cb;
                    place += (int)((kept_bits[wave][o >> 5] >> (o & 31)) & 1u);
                }
                int below = 0;                    // kept block columns below bj = place in the packed arrays
                for (int w = 0; w < (bj >> 5); ++w) below += __popc(kept_bits[wave][w]);
                below += __popc(kept_bits[wave][bj >> 5] & ((1u << (bj & 31)) - 1u));
                const int fa = tap / p.kw, fb = tap - fa * p.kw;
                ord[wave][place] = ((uint32_t)below << 16) | (uint32_t)((fa * sc.PC + fb) * PB);
            }
        }
        for (int cb = lane; cb < sc.CB; cb += 64) {
            int upto = 0;
            for (int ocb = 0; ocb <= cb; ++ocb) upto += (cb_cnt[wave][ocb] + R - 1) / R * R;
            cb_end[wave][cb] = (uint16_t)upto;
        }
    }
    __syncthreads();

    // ---- lane constants ------------------------------------------------------------------------------
    // columns 2jj, 2jj+1 of the wave's sub-tile (same output row: Wo is even); lanes past the last
    // position read position 0 and store nothing
    const int n0 = 2 * jj;
    const bool col_ok = n0 < TP;
    const int n_ld = col_ok ? n0 : 0;
    const int r_local = n_ld / p.Wo, ow = n_ld - r_local * p.Wo;
    const uint32_t lane_pos = (uint32_t)(((pt * sc.R + r_local) * sc.row_mul * sc.PC + ow * p.stride) * PB + hh * 16);
    const uint32_t col_step = (uint32_t)(p.stride * PB);       // from a lane's first output column to its second
    const uint32_t a_off = (uint32_t)((jj * F::SLOTS + hh * F::FS * (SMF ? 2 : 1)) * 2);
    const uint32_t i_off = (uint32_t)(jj * F::WPR * 4);
    const uint32_t aw_sh = (uint32_t)hh * F::HB * (SMF ? 2 : 1);

    f32x16 acc[RT][NACC];
#pragma unroll
    for (int rt = 0; rt < RT; ++rt)
#pragma unroll
        for (int c = 0; c < NACC; ++c)
#pragma unroll
            for (int r = 0; r < 16; ++r) acc[rt][c][r] = 0.0f;
    // ring of R packed slices: entry e of the list lives in slot e % R (runs are padded to multiples
    // of R, so the slot of an entry is known at compile time); idle entries request block t_begin
    uint32_t av[R][RT][KS][F::VW], aw[R][RT][F::WPR];
    const bool busy = works && cnt > 0;
    auto block_of = [&](int entry_index) __attribute__((always_inline)) {
        const uint32_t en = ord[wave][min(entry_index, CONV_LDS_ORD - 1)];
        return t_begin + (int)((en >> 16) & 0x7FFFu);
    };
    int e = 0;
    if (busy) {
#pragma unroll
        for (int r = 0; r < R; ++r) {
            Body::load_a(av[r], aw[r], p, a_off, i_off, block_of(r));
            __builtin_amdgcn_sched_barrier(0);
        }
    }

    // one kept block: B operands from the patch (tap window at byte offset tap_off), A from the slice
    auto multiply = [&](const uint32_t (&av)[RT][KS][F::VW], const uint32_t (&aw)[RT][F::WPR], uint32_t tap_off) __attribute__((always_inline)) {
        uint32_t ws[RT][F::WPR];
        if constexpr (N != M) {
#pragma unroll
            for (int rt = 0; rt < RT; ++rt)
#pragma unroll
                for (int i = 0; i < F::WPR; ++i)
                    ws[rt][i] = __builtin_amdgcn_alignbit(i + 1 < F::WPR ? aw[rt][i + 1] : 0u, aw[rt][i], aw_sh);
        }
        const unsigned char* base = patch + lane_pos + tap_off;
        if constexpr (SMF) {
#pragma unroll
            for (int s2 = 0; s2 < KS / 2; ++s2) {
                typedef __attribute__((ext_vector_type(8))) uint32_t u32x8;
                u32x8 b8[NACC];
#pragma unroll
                for (int c = 0; c < NACC; ++c) {
                    const u32x4 lo = *reinterpret_cast<const u32x4*>(base + c * col_step + (2 * s2) * 32);
                    const u32x4 hi = *reinterpret_cast<const u32x4*>(base + c * col_step + (2 * s2 + 1) * 32);
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
                        acc[rt][c] = __builtin_amdgcn_smfmac_f32_32x32x32_bf16(afrag, __builtin_bit_cast(bf16x16, b8[c]),
                                                                               acc[rt][c], (int)idx, 0, 0);
                }
            }
        } else {
            auto dense_step = [&](auto ks_c) __attribute__((always_inline)) {
                constexpr int ks = decltype(ks_c)::value;
                bf16x8 bfrag[NACC];
#pragma unroll
                for (int c = 0; c < NACC; ++c)
                    bfrag[c] = __builtin_bit_cast(bf16x8, *reinterpret_cast<const u32x4*>(base + c * col_step + ks * 32));
#pragma unroll
                for (int rt = 0; rt < RT; ++rt) {
                    u32x4 a4;
                    if constexpr (LUT48) a4 = expand_frag_lut48<B, ks>(av[rt][ks], ws[rt], lut48);
                    else a4 = expand_frag<N, M, B, ks>(av[rt][ks], ws[rt]);
                    const bf16x8 afrag = __builtin_bit_cast(bf16x8, a4);
#pragma unroll
                    for (int c = 0; c < NACC; ++c)
                        acc[rt][c] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(afrag, bfrag[c], acc[rt][c], 0, 0, 0);
                }
            };
            dense_step(std::integral_constant<int, 0>{});
            dense_step(std::integral_constant<int, 1>{});
            dense_step(std::integral_constant<int, 2>{});
            dense_step(std::integral_constant<int, 3>{});
        }
    };

    // Staging: a lane loads one dword (two neighbouring input positions) of one channel; lanes 0..31
    // of a wave walk along a row of an even channel, lanes 32..63 along the same positions of the
    // next channel.  One lane-swap instruction hands every lane both dwords; the lower half then
    // writes the channel pair of the first position and the upper half that of the second as one
    // dword each (patch[pos][channel]).  A lane keeps its place in the row and its channel pair(s)
    // for the whole kernel and walks down the patch rows: the row is the scalar offset of a buffer
    // load, so a load costs no address arithmetic (coalesced loads, one LDS write per load).
    const int segs = p.W >> 1;                                 // dwords of one input row of one channel
    const int segw_log = segs > 16 ? 5 : segs > 8 ? 4 : segs > 4 ? 3 : segs > 2 ? 2 : segs > 1 ? 1 : 0;   // lanes per row: 2^segw_log >= segs
    const int pairs_per_half = 32 >> segw_log;                 // channel pairs a half-wave covers at a time
    const int l32 = lane & 31, upper = lane >> 5;
    const int seg = l32 & ((1 << segw_log) - 1);
    const int q0 = wave * pairs_per_half + (l32 >> segw_log);  // the lane's first channel pair
    const int q_step = 4 * pairs_per_half;                     // from one of its channel pairs to the next
    const int q_turns = q_step >= 32 ? 1 : 32 / q_step;        // (32 is a multiple of a smaller q_step)
    const bool lane_writes = seg < segs && wave * pairs_per_half < 32;
    const uint32_t pair_sel = upper ? SEL_HI : SEL_LO;
    const uint32_t write0 = (uint32_t)((2 * seg + upper + p.pad) * PB + q0 * 4);
    const uint32_t lane_off = ((uint32_t)(2 * min(q0, 31) + upper) * (uint32_t)p.plane + (uint32_t)(2 * min(seg, segs - 1))) * 2u;
    const uint32_t turn_bytes = (uint32_t)(2 * q_step) * (uint32_t)p.plane * 2u;   // from one channel pair of a lane to its next
    const uint32_t pr_inv = (65536u + (uint32_t)sc.PR - 1u) / (uint32_t)sc.PR;     // u / PR = (u * pr_inv) >> 16 for the few hundred units
    {
        // zero columns of the patch left and right of the image: staging never touches them
        const int halo_cols = sc.PC - p.W;
        for (int i = tid; i < sc.PR * halo_cols * 8; i += 256) {
            const int part = i & 7, pos = i >> 3;
            const int pr = pos / halo_cols, hcol = pos - pr * halo_cols;
            const int pc = hcol < p.pad ? hcol : p.W + hcol;   // left halo, then right halo
            *reinterpret_cast<u32x4*>(patch + ((pr * sc.PC + pc) * PB + part * 16)) = u32x4{0u, 0u, 0u, 0u};
        }
    }
    for (int cb = 0; cb < sc.CB; ++cb) {
        __syncthreads();                                       // everybody is done with the previous patch
        const rsrc_t ract = make_rsrc(p.act + (int64_t)cb * 64 * p.plane + (int64_t)img * p.H * p.W);
        // UN loads per lane are requested before the first is used: taken one at a time, every row
        // would wait out a memory round trip.  The lane's (channel pair, patch row) units are numbered
        // u = turn * PR + pr; what depends on the unit is uniform and goes into the scalar offset of
        // the load and one scalar addend of the LDS address.
        constexpr int UN = 12;
        const int units = q_turns * sc.PR;
        for (int u0 = 0; u0 < units; u0 += UN) {
            uint32_t got[UN];
#pragma unroll
            for (int k = 0; k < UN; ++k) {
                const int u = min(u0 + k, units - 1);
                const int turn = (int)(((uint32_t)u * pr_inv) >> 16), pr = u - turn * sc.PR;
                const int ih = (oh_base * sc.row_mul + pr) * sc.ih_step - p.pad;
                const int ihc = min(max(ih, 0), p.H - 1);
                const uint32_t soff = (uint32_t)turn * turn_bytes + (uint32_t)(ihc * p.W * 2);
                const uint32_t mine = __builtin_amdgcn_raw_buffer_load_b32(ract, lane_off, soff, 0);
                got[k] = ((unsigned)ih < (unsigned)p.H) ? mine : 0u;
            }
#pragma unroll
            for (int k = 0; k < UN; ++k) {
                const int u = u0 + k;
                const int turn = (int)(((uint32_t)u * pr_inv) >> 16), pr = u - turn * sc.PR;
                // [0]: the even channel's dword in every lane, [1]: the odd channel's
                const auto both = __builtin_amdgcn_permlane32_swap(got[k], got[k], false, false);
                // lower half: first position, (even.lo, odd.lo); upper half: second position, (even.hi, odd.hi)
                const uint32_t pair = __builtin_amdgcn_perm(both[1], both[0], pair_sel);
                if (lane_writes && u < units)
                    *reinterpret_cast<uint32_t*>(patch + write0 + (uint32_t)(turn * q_step * 4 + pr * sc.PC * PB)) = pair;
            }
        }
        __syncthreads();
        // ---- the wave's kept blocks of this channel block, all taps --------------------------------
        if (busy) {
            const int e_end = cb_end[wave][cb];
            for (; e < e_end; e += R) {
#pragma unroll
                for (int r = 0; r < R; ++r) {
                    const uint32_t en = ord[wave][e + r];
                    // the slice must have arrived whether or not the entry is idle (wait outside the branch)
#pragma unroll
                    for (int rt = 0; rt < RT; ++rt) {
#pragma unroll
                        for (int ks = 0; ks < KS; ++ks)
#pragma unroll
                            for (int x = 0; x < F::VW; ++x) asm volatile("" ::"v"(av[r][rt][ks][x]));
#pragma unroll
                        for (int x = 0; x < F::WPR; ++x) asm volatile("" ::"v"(aw[r][rt][x]));
                    }
                    if (!(__builtin_amdgcn_readfirstlane((int)en) & (int)CONV_LDS_IDLE)) multiply(av[r], aw[r], en & 0xFFFFu);
                    Body::load_a(av[r], aw[r], p, a_off, i_off, block_of(e + r + R));   // past the end: an idle entry
                }
            }
        }
    }
    if (works) {
        const int64_t col0 = (int64_t)img * p.Ho * p.Wo + (int64_t)oh0 * p.Wo + n0;
        store_rows<B, 1, RT * 16, 1>(p, bi, hh, col0, col_ok, 0, [&](int pr, float (&v)[NACC]) __attribute__((always_inline)) {
#pragma unroll
            for (int c = 0; c < NACC; ++c) v[c] = acc[pr >> 4][c][pr & 15];
        });
    }
}

// Geometry of the LDS-staged convolution for this problem; false if it does not apply.
inline bool conv_lds_plan(const SpmmArgs& a, int B, int kh, ConvLdsSched* out) {
    if (a.act == nullptr || B != 64 || a.stride > 4 || a.C % 64 != 0 || (a.Wo & 1) || a.Wo > 64 || (a.W & 1) || a.W > 64)
        return false;    // (32 lanes stage one input row as dwords)
    const int taps = kh * a.kw;
    ConvLdsSched s;
    s.CB = a.C / 64; s.kh = kh; s.taps = taps; s.Kb = taps * s.CB;
    if (taps > 64 || s.CB > 64 || s.Kb > CONV_LDS_MAX_KB || a.K != taps * a.C) return false;
    if (a.plane >= ((int64_t)1 << 25)) return false;    // staging addresses 64 channel planes with 32-bit byte offsets
    s.RG = a.Sb >= 4 ? 4 : a.Sb >= 2 ? 2 : 1;
    s.PT = 4 / s.RG;
    s.R = 64 / a.Wo;
    if (s.R > a.Ho) s.R = a.Ho;
    s.tiles_per_img = (a.Ho + s.PT * s.R - 1) / (s.PT * s.R);
    s.row_groups = (a.Sb + s.RG - 1) / s.RG;
    s.row_mul = kh == 1 ? 1 : a.stride;
    s.ih_step = kh == 1 ? a.stride : 1;
    s.PR = (s.PT * s.R - 1) * s.row_mul + kh;
    s.PC = (a.Wo - 1) * a.stride + a.kw;
    if (s.PC < a.W + a.pad) s.PC = a.W + a.pad;        // every input column has a place in the patch
    if ((int64_t)s.PR * s.PC * CONV_LDS_POS_BYTES > CONV_LDS_MAX_PATCH) return false;
    *out = s;
    return true;
}

template <int N, int M, bool SMF>
hipError_t launch_conv_lds_k(const SpmmArgs& a, const ConvLdsSched& s, int batch, hipStream_t st) {
    const int64_t wgs = (int64_t)batch * s.tiles_per_img * s.row_groups;
    if (wgs > INT32_MAX) return hipErrorInvalidValue;
    const size_t lds = (size_t)s.PR * s.PC * CONV_LDS_POS_BYTES;
    const dim3 grd((unsigned)wgs), blk(256);
    if (a.ev_start || a.ev_stop)
        hipExtLaunchKernelGGL((conv_lds_kernel<N, M, SMF>), grd, blk, lds, st, a.ev_start, a.ev_stop, 0, a, s);
    else
        conv_lds_kernel<N, M, SMF><<<grd, blk, lds, st>>>(a, s);
    return hipGetLastError();
}

template <int N, int M>
hipError_t launch_conv_lds(const SpmmArgs& a, const ConvLdsSched& s, int batch, hipStream_t st) {
    if constexpr (smf_pattern<N, M>()) {
        if (a.use_smf) return launch_conv_lds_k<N, M, true>(a, s, batch, st);
    }
    return launch_conv_lds_k<N, M, false>(a, s, batch, st);
}

// One translation unit per N:M pattern provides these.
template <int N, int M>
hipError_t launch_reg_nm(const SpmmArgs& a, int B, int shape, hipStream_t st);
template <int N, int M>
hipError_t launch_conv_lds_nm(const SpmmArgs& a, const ConvLdsSched& s, int batch, hipStream_t st);
template <int N, int M>
hipError_t launch_conv_patch_nm(const SpmmArgs& a, const ConvPatchSched& s, int batch, hipStream_t st);
template <int N, int M>
hipError_t launch_balanced_nm(const SpmmArgs& a, int B, hipStream_t st);
template <int N, int M>
hipError_t launch_k8_nm(const SpmmArgs& a, int B, hipStream_t st);

#define CRISP_INSTANTIATE_NM(N, M)                                                           \
    template <>                                                                              \
    hipError_t launch_reg_nm<N, M>(const SpmmArgs& a, int B, int shape, hipStream_t st) {    \
        if (shape == XRES_SHAPE) return launch_xres<N, M>(a, st);                            \
        if (shape == XLDS_SHAPE) return launch_xlds<N, M>(a, st);                            \
        return B == 64 ? launch_reg_shape<N, M, 64>(a, shape, st) : launch_reg_shape<N, M, 32>(a, shape, st); \
    }                                                                                        \
    template <>                                                                              \
    hipError_t launch_conv_lds_nm<N, M>(const SpmmArgs& a, const ConvLdsSched& s, int batch, hipStream_t st) { \
        return launch_conv_lds<N, M>(a, s, batch, st);                                      \
    }                                                                                        \
    template <>                                                                              \
    hipError_t launch_conv_patch_nm<N, M>(const SpmmArgs& a, const ConvPatchSched& s, int batch, hipStream_t st) { \
        return launch_conv_patch<N, M>(a, s, batch, st);                                    \
    }                                                                                        \
    template <>                                                                              \
    hipError_t launch_balanced_nm<N, M>(const SpmmArgs& a, int B, hipStream_t st) {          \
        return launch_balanced<N, M>(a, B, st);                                              \
    }                                                                                        \
    template <>                                                                              \
    hipError_t launch_k8_nm<N, M>(const SpmmArgs& a, int B, hipStream_t st) {                \
        return launch_k8<N, M>(a, B, st);                                                    \
    }

}  // namespace crisp
