// Hybrid-sparse product over octet-interleaved operands: X is [K/8][ldx][8] (the 8 consecutive
// K-values of one column are 16 contiguous bytes) and Y is written as [S/8][ldy][8].
//
// The matrix core wants, per lane, 8 consecutive K-values of ONE column of X.  With X stored row by
// row (K x Ncol, columns contiguous) a lane has to fetch 8 rows with a request each and transpose
// 16-bit halves in registers: 32 requests of 256 bytes per 64 x 64 block and wave, and the address
// unit's time goes with the number of requests, not with their bytes.  Stored in octets of K, the
// operand is one 16-byte load: 8 requests of 1 KB per block and wave, no transposition.  The
// accumulators hold 4 consecutive rows of one column per register quad, i.e. half an octet of the
// output in the same interleaved form, so a layer's Y is the next layer's X (for a convolution: the
// channel-octet-major activation [C/8][batch][H][W][8]) and every store instruction of a wave writes
// 512 contiguous bytes.
//
// Work split as in spmm_reg.h (narrow strips): one wave per (block-row, strip of 64 columns), four
// neighbouring strips per workgroup, the wave walks the block-row's kept blocks with one block of X
// and one packed slice requested ahead.  Lane (jj = lane % 32, hh = lane / 32) owns columns
// strip*64 + jj and strip*64 + 32 + jj.
#pragma once
#include "spmm_reg.h"

namespace crisp {

// Store of a wave's 64 x 64 (or 32 x 64) tile in octet-interleaved form, optional epilogue.
// acc[rt][c][r]: row rt*32 + 8*(r/4) + 4*hh + r%4 of the block-row, column col[c].
template <int B>
__device__ __forceinline__ void store_tile_k8(const SpmmArgs& p, int bi, int hh, const int64_t (&col)[2], const bool (&ok)[2],
                                              const f32x16 (&acc)[B / 32][2]) {
    constexpr int RT = B / 32;
    const uint32_t esz = p.y_bf16 ? 2u : 4u;
    const uint32_t oct_bytes = (uint32_t)p.ldy * 8u * esz;                  // one octet of rows
    const int octs_here = min(B / 8, (p.S >> 3) - bi * (B / 8));            // octets of this block-row that exist
    const rsrc_t ry = __builtin_amdgcn_make_buffer_rsrc(reinterpret_cast<char*>(p.Y) + (int64_t)bi * (B / 8) * p.ldy * 8 * esz, 0,
                                                        (uint32_t)max(octs_here, 0) * oct_bytes, 0x00020000);
    uint32_t off[2];
#pragma unroll
    for (int c = 0; c < 2; ++c) off[c] = ok[c] ? ((uint32_t)col[c] * 8u + 4u * (uint32_t)hh) * esz : 0x80000000u;
    auto emit = [&](auto with_ep, auto as_bf16) __attribute__((always_inline)) {
        constexpr bool EP = decltype(with_ep)::value, BF16 = decltype(as_bf16)::value;
        rsrc_t rres = ry, rsc = ry, rbs = ry;
        if constexpr (EP) {
            rres = __builtin_amdgcn_make_buffer_rsrc(
                const_cast<char*>(reinterpret_cast<const char*>(p.ep_res)) + (p.ep_res ? (int64_t)bi * (B / 8) * p.ep_ldr * 8 * esz : 0), 0,
                p.ep_res ? (uint32_t)max(octs_here, 0) * (uint32_t)p.ep_ldr * 8u * esz : 0u, 0x00020000);
            rsc = __builtin_amdgcn_make_buffer_rsrc(const_cast<float*>(p.ep_scale), 0, p.ep_scale ? (uint32_t)p.S * 4u : 0u, 0x00020000);
            rbs = __builtin_amdgcn_make_buffer_rsrc(const_cast<float*>(p.ep_bias), 0, p.ep_bias ? (uint32_t)p.S * 4u : 0u, 0x00020000);
        }
        const uint32_t res_oct_bytes = (uint32_t)p.ep_ldr * 8u * esz;
#pragma unroll
        for (int rt = 0; rt < RT; ++rt) {
            // the epilogue's operands of the 4 octets of this row tile, requested together
            uint32_t res[4][2][BF16 ? 2 : 4];
            f32x4e sc[4], bs[4];
            if constexpr (EP) {
#pragma unroll
                for (int q = 0; q < 4; ++q) {
                    const uint32_t o = (uint32_t)(rt * 4 + q);
#pragma unroll
                    for (int c = 0; c < 2; ++c) {
                        const uint32_t roff = ok[c] ? o * res_oct_bytes + ((uint32_t)col[c] * 8u + 4u * (uint32_t)hh) * esz : 0x80000000u;
                        if constexpr (BF16) {
                            const u32x2 t = __builtin_bit_cast(u32x2, __builtin_amdgcn_raw_buffer_load_b64(rres, roff, 0, 0));
                            res[q][c][0] = t[0]; res[q][c][1] = t[1];
                        } else {
                            const u32x4 t = __builtin_bit_cast(u32x4, __builtin_amdgcn_raw_buffer_load_b128(rres, roff, 0, 0));
                            res[q][c][0] = t[0]; res[q][c][1] = t[1]; res[q][c][2] = t[2]; res[q][c][3] = t[3];
                        }
                    }
                    const uint32_t row_bytes = (uint32_t)(bi * B + (int)o * 8 + 4 * hh) * 4u;
                    sc[q] = __builtin_bit_cast(f32x4e, __builtin_amdgcn_raw_buffer_load_b128(rsc, row_bytes, 0, 0));
                    bs[q] = __builtin_bit_cast(f32x4e, __builtin_amdgcn_raw_buffer_load_b128(rbs, row_bytes, 0, 0));
                }
            }
#pragma unroll
            for (int q = 0; q < 4; ++q) {
                const uint32_t o = (uint32_t)(rt * 4 + q);
#pragma unroll
                for (int c = 0; c < 2; ++c) {
                    float v[4];
#pragma unroll
                    for (int i = 0; i < 4; ++i) {
                        float y = acc[rt][c][4 * q + i];
                        if constexpr (EP) {
                            float r;
                            if constexpr (BF16) r = __uint_as_float((i & 1) ? (res[q][c][i / 2] & 0xFFFF0000u) : (res[q][c][i / 2] << 16));
                            else r = __uint_as_float(res[q][c][i]);
                            y = p.ep_scale ? __fmul_rn(y, sc[q][i]) : y;
                            y = p.ep_bias ? __fadd_rn(y, bs[q][i]) : y;
                            y = p.ep_res ? __fadd_rn(y, r) : y;
                            y = p.ep_relu ? fmaxf(y, 0.0f) : y;
                        }
                        v[i] = y;
                    }
                    const uint32_t yoff = off[c] + o * oct_bytes;
                    if constexpr (BF16) {
                        const f32x2 a = {v[0], v[1]}, b = {v[2], v[3]};
                        const u32x2 two = {__builtin_bit_cast(uint32_t, __builtin_convertvector(a, bf16x2)),
                                           __builtin_bit_cast(uint32_t, __builtin_convertvector(b, bf16x2))};
                        __builtin_amdgcn_raw_buffer_store_b64(two, ry, yoff, 0, 0);
                    } else {
                        const u32x4 four = {__float_as_uint(v[0]), __float_as_uint(v[1]), __float_as_uint(v[2]), __float_as_uint(v[3])};
                        __builtin_amdgcn_raw_buffer_store_b128(four, ry, yoff, 0, 0);
                    }
                }
            }
        }
    };
    if (p.ep_on) {
        if (p.y_bf16) emit(std::true_type{}, std::true_type{});
        else emit(std::true_type{}, std::false_type{});
    } else {
        if (p.y_bf16) emit(std::false_type{}, std::true_type{});
        else emit(std::false_type{}, std::false_type{});
    }
}

// PF: blocks requested ahead per wave (ring of PF register slots).
template <int N, int M, int B, bool SMF, int PF>
__global__ __launch_bounds__(256) __attribute__((amdgpu_waves_per_eu(2, PF == 1 ? 3 : 2)))
void spmm_k8_kernel(SpmmArgs p) {
    typedef Fmt<N, M, B> F;
    constexpr int RT = F::RT, KS = F::KS, NACC = 2;
    typedef BlockBody<N, M, B, 1, true, 5, SMF> BodyP;
    typedef BlockBody<N, M, B, 1, false, 5, SMF> BodyL;

    // Workgroup -> (block-row, strip group); ids are dealt round-robin to the 8 XCDs, and all
    // block-rows of a strip group get ids on the same XCD so they share its L2 for X.
    const int id = blockIdx.x;
    const int xcd = id & 7, slot = id >> 3;
    const int bi = slot % p.Sb;
    const int nt = (slot / p.Sb) * 8 + xcd;
    if (nt >= p.NT) return;
    const int tid = threadIdx.x, wave = tid >> 6, lane = tid & 63;
    const int jj = lane & 31, hh = lane >> 5;
    // selector table of the dense 4:8 expansion, built by the whole workgroup before any wave leaves
    constexpr bool LUT48 = lut48_pattern<N, M, SMF>();
    __shared__ u32x4 lut48[LUT48 ? 256 : 1];
    if constexpr (LUT48) {
        lut48_fill(lut48, tid, 256);
        __syncthreads();
    }
    const int64_t wave_col = ((int64_t)nt * 4 + wave) * 64;
    if (wave_col >= p.Ncol) return;                          // no further barriers in this kernel
    const int64_t col[2] = {wave_col + jj, wave_col + 32 + jj};
    const bool ok[2] = {col[0] < p.Ncol, col[1] < p.Ncol};
    // lanes past the last column read the last column instead (in bounds) and never store
    const uint32_t off0 = (uint32_t)(((int64_t)hh * p.ldx + min(col[0], p.Ncol - 1)) * 16);
    const uint32_t off1 = (uint32_t)(((int64_t)hh * p.ldx + min(col[1], p.Ncol - 1)) * 16);
    const uint32_t a_off = (uint32_t)((jj * F::SLOTS + hh * F::FS * (SMF ? 2 : 1)) * 2);
    const uint32_t i_off = (uint32_t)(jj * F::WPR * 4);
    const uint32_t aw_sh = (uint32_t)hh * F::HB * (SMF ? 2 : 1);

    const int t_begin = p.row_ptr[bi], t_end = p.row_ptr[bi + 1];
    const int cnt = t_end - t_begin;
    f32x16 acc[RT][NACC];
#pragma unroll
    for (int rt = 0; rt < RT; ++rt)
#pragma unroll
        for (int c = 0; c < NACC; ++c)
#pragma unroll
            for (int r = 0; r < 16; ++r) acc[rt][c][r] = 0.0f;

    {
        uint32_t xr[PF][KS][8];
        uint32_t av[PF][RT][KS][F::VW], aw[PF][RT][F::WPR];
        XCtx cx[PF];
        const ConvPos cp = {0, 0, 0, 0u, 0, 0, 0, lut48};
        // ---- prologue: up to PF blocks in flight ------------------------------------------------
#pragma unroll
        for (int d = 0; d < PF; ++d) {
            cx[d] = XCtx{off0, SEL_LO, SEL_HI, off1};
            if (d < cnt) {
                const int bj = p.col_idx[t_begin + d];
#pragma unroll
                for (int ks = 0; ks < KS; ++ks) BodyL::load_x(xr[d][ks], p, cp, cx[d].off, cx[d].off2, bj, ks);
                BodyL::load_a(av[d], aw[d], p, a_off, i_off, t_begin + d);
            }
        }
        // ---- steady state: every block of a group of PF has a successor PF blocks later -----------
        int i0 = 0;
        for (; i0 + 2 * PF <= cnt; i0 += PF) {
#pragma unroll
            for (int d = 0; d < PF; ++d)
                BodyP::run(acc, xr[d], av[d], aw[d], cx[d], p, cp, a_off, i_off, aw_sh, t_begin + i0 + d + PF);
        }
        // ---- tail: at most 2*PF-1 blocks; the first PF-1 of them may still have a successor --------
#pragma unroll
        for (int e = 0; e < 2 * PF - 1; ++e) {
            const int i = i0 + e;
            if (i < cnt) {
                if (e < PF - 1 && i + PF < cnt)
                    BodyP::run(acc, xr[e % PF], av[e % PF], aw[e % PF], cx[e % PF], p, cp, a_off, i_off, aw_sh, t_begin + i + PF);
                else
                    BodyL::run(acc, xr[e % PF], av[e % PF], aw[e % PF], cx[e % PF], p, cp, a_off, i_off, aw_sh, 0);
            }
        }
    }
    store_tile_k8<B>(p, bi, hh, col, ok, acc);
}

// Covered: B in {32, 64}, K a multiple of 16, S a multiple of 8, row strides within the 32-bit offsets
// of a block-row (checked by the caller).
template <int N, int M, int B, bool SMF, int PF>
hipError_t launch_k8_k(const SpmmArgs& a, hipStream_t st) {
    SpmmArgs p = a;
    p.NT = (int)((a.Ncol + 255) / 256);
    const int64_t groups = (int64_t)((p.NT + 7) / 8) * p.Sb * 8;
    if (groups > INT32_MAX) return hipErrorInvalidValue;
    const dim3 grd((unsigned)groups), blk(256);
    if (a.ev_start || a.ev_stop)
        hipExtLaunchKernelGGL((spmm_k8_kernel<N, M, B, SMF, PF>), grd, blk, 0, st, a.ev_start, a.ev_stop, 0, p);
    else
        spmm_k8_kernel<N, M, B, SMF, PF><<<grd, blk, 0, st>>>(p);
    return hipGetLastError();
}

// One block requested ahead: a ring of two (more registers, two waves per SIMD instead of three) was measured
// equal or slower on every layer shape tried.
template <int N, int M>
hipError_t launch_k8(const SpmmArgs& a, int B, hipStream_t st) {
    constexpr int PF = 1;
    if constexpr (smf_pattern<N, M>()) {
        if (a.use_smf) return B == 64 ? launch_k8_k<N, M, 64, true, PF>(a, st) : launch_k8_k<N, M, 32, true, PF>(a, st);
    }
    return B == 64 ? launch_k8_k<N, M, 64, false, PF>(a, st) : launch_k8_k<N, M, 32, false, PF>(a, st);
}

}  // namespace crisp
