// Hybrid-sparse convolution for channel counts that are no multiple of the block size (a network's
// first layer): the input patch of a workgroup's output positions sits in LDS in its own layout.
//
// With C % B != 0 a block column of W spans several filter taps, so every K-row k = (a*kw + b)*C + c
// has its own source window (spmm_reg.h, conv mode 3, fetches each element of X with a 2-byte
// request of its own and splits every k into (a, b, c) in vector arithmetic: the 7x7 first layer of
// ResNet-50 is bound by the request rate of the load unit and by that arithmetic).  Here a
// workgroup owns 1024 consecutive output positions of one image (4 waves x 4 strips of 64) and
//   * copies the input rows they touch into LDS as patch[c][row][col], rows and columns outside the
//     image present as zeros, so the product loop needs no border tests (one more, all-zero channel
//     plane stands in for the K-rows past K of the last block column);
//   * tabulates, once, the LDS offset of every K-row (channel plane, filter row, filter column);
//   * builds the matrix core's B operand of a 16-row step from 16 two-byte LDS reads per lane
//     (address = the lane's position + the K-row's offset) and walks the block-rows with it as the
//     other kernels do (Sec. 3.5: only kept blocks are visited).
#pragma once
#include "spmm_reg.h"

namespace crisp {

constexpr int CONV_PATCH_SHAPE = 21;            // launch shape code of this kernel for launch_reg_nm
constexpr int CONV_PATCH_MAX_LDS = 64 * 1024;
constexpr int CONV_PATCH_STRIPS = 4;            // strips of 64 output positions a wave takes in turn
constexpr int CONV_PATCH_TILE = 256 * CONV_PATCH_STRIPS;   // output positions per workgroup

struct ConvPatchSched {
    int kh, taps;
    int PR, PCW;            // patch rows per channel (the most a tile can touch) and columns (W + 2 * pad)
    int tiles_per_img;
    int k_pad;              // K rounded up to whole blocks: entries of the K-row table
    int patch_off;          // byte offset of the patch behind the table
    int zero_off;           // byte offset of the all-zero channel plane (K-rows past K read there)
    int lds_bytes;
};

template <int N, int M, bool SMF>
__global__ __launch_bounds__(256, 3) void conv_patch_kernel(SpmmArgs p, ConvPatchSched sc) {
    constexpr int B = 64;
    typedef Fmt<N, M, B> F;
    constexpr int RT = F::RT, KS = F::KS, NACC = 2;
    typedef BlockBody<N, M, B, 1, false, 0, SMF> Body;
    extern __shared__ __attribute__((aligned(16))) unsigned char lds[];   // [k_pad] uint32 K-row offsets, then the patch

    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int jj = lane & 31, hh = lane >> 5;
    const int img = (int)blockIdx.x / sc.tiles_per_img;
    const int p0 = ((int)blockIdx.x - img * sc.tiles_per_img) * CONV_PATCH_TILE;     // first output position of the tile
    const int HoWo = p.Ho * p.Wo;
    const int oh_first = p0 / p.Wo;
    const int oh_last = min(p0 + CONV_PATCH_TILE - 1, HoWo - 1) / p.Wo;
    const int ih_first = oh_first * p.stride - p.pad;
    const int rows_here = (oh_last - oh_first) * p.stride + sc.kh;                  // <= sc.PR

    // the block list, read before anything is stored (lane l: row_ptr[l], and the l-th block's column;
    // the number of kept blocks is only known on the device: blocks from the 64th on are looked up in
    // memory as they come)
    const int my_ptr = p.row_ptr[min(lane, p.Sb)];
    const int t_last = __builtin_amdgcn_readlane(my_ptr, p.Sb) - 1;
    const int my_bj = p.col_idx[max(min(lane, t_last), 0)];

    // selector table of the dense 4:8 expansion (visible after the barriers below)
    constexpr bool LUT48 = lut48_pattern<N, M, SMF>();
    __shared__ u32x4 lut48[LUT48 ? 256 : 1];
    if constexpr (LUT48) lut48_fill(lut48, tid, 256);
    // ---- K-row table, zeroed patch ------------------------------------------------------------------
    uint32_t* koff = reinterpret_cast<uint32_t*>(lds);
    unsigned char* patch = lds + sc.patch_off;
    for (int k = tid; k < sc.k_pad; k += 256) {
        uint32_t off = (uint32_t)sc.zero_off;
        if (k < p.K) {
            const int tap = k / p.C, c = k - tap * p.C;
            const int a = tap / p.kw, b = tap - a * p.kw;
            off = (uint32_t)(sc.patch_off + ((c * sc.PR + a) * sc.PCW + b) * 2);
        }
        koff[k] = off;
    }
    for (int e = tid; e < (sc.lds_bytes - sc.patch_off) / 16; e += 256)
        reinterpret_cast<u32x4*>(patch)[e] = u32x4{0u, 0u, 0u, 0u};
    __syncthreads();
    // ---- input rows -> patch.  A wave takes every fourth (channel, patch row) pair, its lanes the row's
    // dwords (64 at a time); UN rows are requested before the first is written (one at a time, every row
    // would wait out a memory round trip).  What depends on the row is uniform: the scalar offset of the
    // buffer load and one scalar addend of the LDS address. ----
    {
        const int segs = p.W >> 1;                             // dwords per input row (W is even)
        const int units = p.C * rows_here;
        // u / rows_here by a multiplication (exact: u < 2^12, rows_here < 2^7); one row per channel needs none
        const uint32_t rows_inv = rows_here > 1 ? (uint32_t)((((uint64_t)1 << 32) + rows_here - 1) / rows_here) : 0u;
        const rsrc_t ract = make_rsrc(p.act + (int64_t)img * p.H * p.W);
        constexpr int UN = 8;
        for (int s0 = 0; s0 < segs; s0 += 64) {
            const int sg = s0 + lane;
            const uint32_t lane_off = (uint32_t)min(sg, segs - 1) * 4u;
            for (int u0 = wave; u0 < units; u0 += 4 * UN) {
                uint32_t got[UN];
#pragma unroll
                for (int k = 0; k < UN; ++k) {
                    const int u = min(u0 + 4 * k, units - 1);
                    const int c = rows_here > 1 ? (int)__umulhi((uint32_t)u, rows_inv) : u, pr = u - c * rows_here;
                    const int ihc = min(max(ih_first + pr, 0), p.H - 1);
                    got[k] = __builtin_amdgcn_raw_buffer_load_b32(ract, lane_off, (uint32_t)c * (uint32_t)p.plane * 2u + (uint32_t)(ihc * p.W * 2), 0);
                }
#pragma unroll
                for (int k = 0; k < UN; ++k) {
                    const int u = u0 + 4 * k;
                    const int c = rows_here > 1 ? (int)__umulhi((uint32_t)min(u, units - 1), rows_inv) : min(u, units - 1), pr = min(u, units - 1) - c * rows_here;
                    const bool row_in = (unsigned)(ih_first + pr) < (unsigned)p.H;
                    if (u < units && row_in && sg < segs) {
                        uint16_t* dst = reinterpret_cast<uint16_t*>(patch) + (c * sc.PR + pr) * sc.PCW + p.pad + 2 * sg;
                        dst[0] = (uint16_t)got[k];
                        dst[1] = (uint16_t)(got[k] >> 16);
                    }
                }
            }
        }
    }
    __syncthreads();

    const uint32_t a_off = (uint32_t)((jj * F::SLOTS + hh * F::FS * (SMF ? 2 : 1)) * 2);
    const uint32_t i_off = (uint32_t)(jj * F::WPR * 4);
    const uint32_t aw_sh = (uint32_t)hh * F::HB * (SMF ? 2 : 1);
    uint32_t pos_a = 0, pos_b = 0;                             // the lane's two positions inside the patch (bytes)

    // B operands of step ks of block column bj: 8 K-rows of the lane's half for its two positions
    auto operands = [&](int bj, int ks, u32x4& first, u32x4& second) __attribute__((always_inline)) {
        const u32x4* tab = reinterpret_cast<const u32x4*>(koff + bj * B + ks * 16 + hh * 8);
        const u32x4 o0 = tab[0], o1 = tab[1];
        const uint32_t o[8] = {o0[0], o0[1], o0[2], o0[3], o1[0], o1[1], o1[2], o1[3]};
#pragma unroll
        for (int q = 0; q < 4; ++q) {
            const uint32_t a0 = *reinterpret_cast<const uint16_t*>(lds + o[2 * q] + pos_a);
            const uint32_t a1 = *reinterpret_cast<const uint16_t*>(lds + o[2 * q + 1] + pos_a);
            const uint32_t b0 = *reinterpret_cast<const uint16_t*>(lds + o[2 * q] + pos_b);
            const uint32_t b1 = *reinterpret_cast<const uint16_t*>(lds + o[2 * q + 1] + pos_b);
            first[q] = a0 | (a1 << 16);
            second[q] = b0 | (b1 << 16);
        }
    };

    f32x16 acc[RT][NACC];
    uint32_t av[RT][KS][F::VW], aw[RT][F::WPR];
    if (t_last >= 0) Body::load_a(av, aw, p, a_off, i_off, 0);
    for (int strip = 0; strip < CONV_PATCH_STRIPS; ++strip) {
    // ---- lane constants of this strip ---------------------------------------------------------------
    const int q0 = p0 + (strip * 4 + wave) * 64 + 2 * jj;     // the lane's first output position inside the image
    if (p0 + (strip * 4 + wave) * 64 >= HoWo) break;           // (uniform: the strip lies past the image)
    const bool col_ok = q0 < HoWo;                             // (Ho*Wo is even: then the second one exists too)
    const int qa = col_ok ? q0 : p0, qb = col_ok ? q0 + 1 : p0;
    const int oha = qa / p.Wo, owa = qa - oha * p.Wo;
    const int ohb = qb / p.Wo, owb = qb - ohb * p.Wo;
    pos_a = (uint32_t)((((oha - oh_first) * p.stride) * sc.PCW + owa * p.stride) * 2);
    pos_b = (uint32_t)((((ohb - oh_first) * p.stride) * sc.PCW + owb * p.stride) * 2);
    const int64_t col0 = (int64_t)img * HoWo + q0;
    int t = 0;
    for (int bi = 0; bi < p.Sb; ++bi) {
        const int t_end = __builtin_amdgcn_readlane(my_ptr, bi + 1);
#pragma unroll
        for (int rt = 0; rt < RT; ++rt)
#pragma unroll
            for (int c = 0; c < NACC; ++c)
#pragma unroll
                for (int r = 0; r < 16; ++r) acc[rt][c][r] = 0.0f;
        for (; t < t_end; ++t) {
            const int bj = t < 64 ? __builtin_amdgcn_readlane(my_bj, t) : p.col_idx[t];
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
                    u32x4 lo[NACC], hi[NACC];
                    operands(bj, 2 * s2, lo[0], lo[1]);
                    operands(bj, 2 * s2 + 1, hi[0], hi[1]);
#pragma unroll
                    for (int rt = 0; rt < RT; ++rt) {
                        u32x4 a4;
                        uint32_t idx;
                        if (s2 == 0) smf_operand<N, M, B, 0>(av[rt], ws[rt], a4, idx);
                        else smf_operand<N, M, B, 1>(av[rt], ws[rt], a4, idx);
                        const bf16x8 afrag = __builtin_bit_cast(bf16x8, a4);
#pragma unroll
                        for (int c = 0; c < NACC; ++c) {
                            const u32x8 b8 = {lo[c][0], lo[c][1], lo[c][2], lo[c][3], hi[c][0], hi[c][1], hi[c][2], hi[c][3]};
                            acc[rt][c] = __builtin_amdgcn_smfmac_f32_32x32x32_bf16(afrag, __builtin_bit_cast(bf16x16, b8), acc[rt][c],
                                                                                   (int)idx, 0, 0);
                        }
                    }
                }
            } else {
                auto dense_step = [&](auto ks_c) __attribute__((always_inline)) {
                    constexpr int ks = decltype(ks_c)::value;
                    u32x4 bo[NACC];
                    operands(bj, ks, bo[0], bo[1]);
#pragma unroll
                    for (int rt = 0; rt < RT; ++rt) {
                        u32x4 a4;
                        if constexpr (LUT48) a4 = expand_frag_lut48<B, ks>(av[rt][ks], ws[rt], lut48);
                        else a4 = expand_frag<N, M, B, ks>(av[rt][ks], ws[rt]);
                        const bf16x8 afrag = __builtin_bit_cast(bf16x8, a4);
#pragma unroll
                        for (int c = 0; c < NACC; ++c)
                            acc[rt][c] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(afrag, __builtin_bit_cast(bf16x8, bo[c]), acc[rt][c], 0, 0, 0);
                    }
                };
                dense_step(std::integral_constant<int, 0>{});
                dense_step(std::integral_constant<int, 1>{});
                dense_step(std::integral_constant<int, 2>{});
                dense_step(std::integral_constant<int, 3>{});
            }
            // the next block's slice; after the last block the first one again, for the wave's next strip
            Body::load_a(av, aw, p, a_off, i_off, t + 1 <= t_last ? t + 1 : 0);
        }
        // (row addresses from an opaque copy of the lane's row half: not hoisted out of the loop and spilled)
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
}

// Covered: C % 64 != 0 (conv mode 3), 64 x 64 blocks, even W and Ho * Wo, at most 63 block-rows,
// K-row table and patch within 64 KB of LDS.
inline bool conv_patch_plan(const SpmmArgs& a, int B, int kh, int Kb, ConvPatchSched* out) {
    if (a.act == nullptr || a.conv_mode != 3 || B != 64 || (a.W & 1) || ((a.Ho * a.Wo) & 1) || a.Sb > 63) return false;
    ConvPatchSched s;
    s.kh = kh; s.taps = kh * a.kw;
    if (a.K != s.taps * a.C || (int64_t)a.C * a.plane * 2 >= ((int64_t)1 << 32)) return false;
    const int rows_out = (CONV_PATCH_TILE + a.Wo - 2) / a.Wo + 1;       // output rows a run of 256 positions can touch
    s.PR = (rows_out - 1) * a.stride + kh;
    s.PCW = a.W + 2 * a.pad;
    s.PCW += s.PCW & 1;
    s.tiles_per_img = (a.Ho * a.Wo + CONV_PATCH_TILE - 1) / CONV_PATCH_TILE;
    s.k_pad = Kb * 64;
    s.patch_off = s.k_pad * 4;
    const int64_t plane_bytes = (int64_t)s.PR * s.PCW * 2;
    s.zero_off = (int)(s.patch_off + a.C * plane_bytes);
    const int64_t total = (s.zero_off + plane_bytes + 15) / 16 * 16;
    if (total > CONV_PATCH_MAX_LDS) return false;
    s.lds_bytes = (int)total;
    *out = s;
    return true;
}

template <int N, int M, bool SMF>
hipError_t launch_conv_patch_k(const SpmmArgs& a, const ConvPatchSched& s, int batch, hipStream_t st) {
    const int64_t wgs = (int64_t)batch * s.tiles_per_img;
    if (wgs > INT32_MAX) return hipErrorInvalidValue;
    const dim3 grd((unsigned)wgs), blk(256);
    if (a.ev_start || a.ev_stop)
        hipExtLaunchKernelGGL((conv_patch_kernel<N, M, SMF>), grd, blk, (size_t)s.lds_bytes, st, a.ev_start, a.ev_stop, 0, a, s);
    else
        conv_patch_kernel<N, M, SMF><<<grd, blk, (size_t)s.lds_bytes, st>>>(a, s);
    return hipGetLastError();
}

template <int N, int M>
hipError_t launch_conv_patch(const SpmmArgs& a, const ConvPatchSched& s, int batch, hipStream_t st) {
    if constexpr (smf_pattern<N, M>()) {
        if (a.use_smf) return launch_conv_patch_k<N, M, true>(a, s, batch, st);
    }
    return launch_conv_patch_k<N, M, false>(a, s, batch, st);
}

}  // namespace crisp
