// Register-resident hybrid-sparse product kernel for gfx950, specialised per N:M pattern.
//
// Sec. 3.5 of the CRISP paper walks a block-row's kept blocks, selects the activations the
// in-group positions point at, and multiply-accumulates.  On CDNA4 the same walk is done by one
// 64-lane wave per (block-row, strip of output columns):
//   * X rows of a kept block are loaded row-wise, coalesced, straight into registers; a lane
//     holds 2*WD consecutive columns of 8 K-rows and transposes the 16-bit halves into 2*WD
//     MFMA B operands (8 K-values of one column each), so the accumulators of a lane are
//     consecutive output columns and Y is written with wide stores;
//   * the lane's slice of the compressed values and log2(m)-bit positions (canonical packed
//     form, read as is) is expanded in registers into the dense 8-value A operand and fed to
//     v_mfma_f32_32x32x16_bf16 -- or, for patterns with at most two kept per group (SMF), handed
//     almost unchanged to the sparse matrix-core instruction v_smfmac_f32_32x32x32_bf16;
//   * accumulation in fp32.
// With CONV != 0 the X rows are not read from a materialised matrix but located inside the
// convolution's input (three modes, see SpmmArgs).
// Nothing goes through LDS in the loop and waves never wait for each other, so every wave keeps
// PF blocks of X in flight.  Two ways to spread work:
//   NWK == 1: the 4 waves of a workgroup own 4 neighbouring column strips (large Ncol);
//   NWK  > 1: the NWK waves of a workgroup share one strip and split the block list between
//             them (small Ncol: more waves, more loads in flight); partial sums are added in a
//             fixed order through LDS at the end, so results stay deterministic.
#pragma once
#include <type_traits>



#include <hip/hip_ext.h>

#include "crisp_internal.h"

namespace crisp {

typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8;
typedef __attribute__((ext_vector_type(16))) __bf16 bf16x16;
typedef __attribute__((ext_vector_type(16))) float f32x16;
typedef __attribute__((ext_vector_type(4))) uint32_t u32x4;

struct SpmmArgs {
    int S, K, n, m, w, slots, wpr;
    int Sb;          // block-rows
    int NT;          // groups of column strips (one per workgroup)
    int64_t Ncol, ldx, ldy;
    const int32_t* row_ptr;
    const int32_t* col_idx;
    const uint16_t* vals;
    const uint32_t* idxw;
    const uint16_t* X;
    void* Y;
    int y_bf16;
    // implicit lowering (conv mode): X is not materialised; its rows are read from the activation
    // [C][batch][H][W], C % B == 0.  conv_mode 1: stride 1 and (even Wo, or padding (k-1)/2 in both
    // directions): the sources of a lane's two output columns are neighbours in memory and come from one dword.  conv_mode 2: any stride and Wo, the two
    // columns are located independently and loaded with one 2-byte load each.  conv_mode 4: 1x1 filter
    // with stride 2 (no padding, even W and Wo): the two columns come from one 8-byte load.  conv_mode 3: any C
    // (a block column may span several filter taps): like 2, and in addition every K-row is split
    // into (tap, channel) on its own; elements outside the image or past K are requested at an
    // offset beyond the activation's buffer range, for which the hardware returns zero.
    const uint16_t* act;
    int conv_mode;
    uint32_t act_bytes;       // size of the activation (conv_mode 3: range of the buffer resource)
    float inv_C;
    int C, H, W, kw, pad, stride, Ho, Wo;
    int64_t plane;            // batch*H*W elements of one channel
    float inv_cpb, inv_kw;    // reciprocals of C/B (block columns per tap) and kw
    double inv_Wo, inv_Ho;
    // optional epilogue on the fp32 sums before the output rounding: y = relu(y * scale[row] +
    // bias[row] + residual[row][col]), every step one fp32 rounding, absent parts skipped
    int ep_on, ep_relu;
    const float* ep_scale;
    const float* ep_bias;
    const void* ep_res;       // S x ep_ldr, same element type as Y
    int64_t ep_ldr;
    int use_smf;              // host side only: sparse-MFMA instantiation wanted (eligible patterns)
    int two_of_four;          // host side only: 4:8 pack with at most two values per aligned four (caller's assertion)
    // host side only: optional events that receive the kernel's own start and stop time stamps
    hipEvent_t ev_start, ev_stop;
};

// Lane-dependent part of the X addressing for one block column, and the byte selectors that turn
// two loaded rows into the two per-column operands.  Explicit X: constant.  Conv mode: depends on
// the block column's filter tap (shifted window, zero padding at the image border).
struct XCtx {
    uint32_t off;
    uint32_t sel_lo, sel_hi;
    uint32_t off2;   // conv mode 2: address part of the lane's second column
};
constexpr uint32_t SEL_LO = 0x05040100u;    // r0.lo | r1.lo << 16
constexpr uint32_t SEL_HI = 0x07060302u;    // r0.hi | r1.hi << 16
constexpr uint32_t SEL_ZERO = 0x0C0C0C0Cu;  // v_perm_b32: selector byte 0x0c yields 0x00

// Output position (image, oh, ow) of a lane's first column in conv mode, fixed for the wave.
struct ConvPos {
    int img, oh, ow;
    uint32_t half_off;   // hh * 8 channel planes, in bytes
    int img1, oh1, ow1;  // conv mode 2: position of the lane's second column
    const u32x4* lut48;  // selector table of the dense 4:8 expansion (LDS; set by the kernels that expand 4:8)
};

__device__ __forceinline__ uint16_t float_to_bf16_rne(float f) {
    uint32_t u = __float_as_uint(f);
    if ((u & 0x7FFFFFFFu) > 0x7F800000u) return (uint16_t)((u >> 16) | 0x40u);  // NaN stays NaN
    u += 0x7FFFu + ((u >> 16) & 1u);
    return (uint16_t)(u >> 16);
}

typedef __attribute__((ext_vector_type(2))) uint32_t u32x2;
typedef __attribute__((ext_vector_type(2))) float f32x2;
typedef __attribute__((ext_vector_type(4))) float f32x4e;
typedef __attribute__((ext_vector_type(2))) __bf16 bf16x2;
template <int WD> struct XVec;
template <> struct XVec<1> { typedef uint32_t type; };
template <> struct XVec<2> { typedef u32x2 type; };
__device__ __forceinline__ void xvec_unpack(const uint32_t& v, uint32_t (&d)[1]) { d[0] = v; }
__device__ __forceinline__ void xvec_unpack(const u32x2& v, uint32_t (&d)[2]) { d[0] = v[0]; d[1] = v[1]; }

// Buffer addressing (MUBUF): a 128-bit resource in SGPRs gives the base, a 32-bit SGPR a
// uniform offset and a 32-bit VGPR the lane's offset, so per-load address arithmetic is scalar.
// Resource words: base[31:0], base[47:32] (stride 0), number of bytes, 0x00020000 (raw 32-bit
// data format on gfx9-family targets).  The range is left at its maximum: every address formed
// below is in bounds by construction.
typedef __amdgpu_buffer_rsrc_t rsrc_t;
__device__ __forceinline__ rsrc_t make_rsrc(const void* base) {
    return __builtin_amdgcn_make_buffer_rsrc(const_cast<void*>(base), 0, 0xFFFFFFFFu, 0x00020000);
}
template <int WD> __device__ __forceinline__ typename XVec<WD>::type buf_load_x(rsrc_t r, uint32_t voff, uint32_t soff);
template <> __device__ __forceinline__ uint32_t buf_load_x<1>(rsrc_t r, uint32_t voff, uint32_t soff) {
    return __builtin_amdgcn_raw_buffer_load_b32(r, voff, soff, 0);
}
template <> __device__ __forceinline__ u32x2 buf_load_x<2>(rsrc_t r, uint32_t voff, uint32_t soff) {
    return __builtin_bit_cast(u32x2, __builtin_amdgcn_raw_buffer_load_b64(r, voff, soff, 0));
}

// Epilogue on NV consecutive outputs (row, col .. col+NV-1) of a lane, all of which exist
// (callers pass ok = false otherwise): per-row scale and bias (folded normalisation), residual
// of the output's element type, ReLU.  fp32 throughout, one rounding per step.
template <int NV>
__device__ __forceinline__ void apply_epilogue(const SpmmArgs& p, int row, int64_t col, bool ok, float (&v)[NV]) {
    if (!p.ep_on || !ok) return;
    float res[NV];
#pragma unroll
    for (int c = 0; c < NV; ++c) res[c] = 0.0f;
    if (p.ep_res) {
        if (p.y_bf16) {
            const uint16_t* r = reinterpret_cast<const uint16_t*>(p.ep_res) + (int64_t)row * p.ep_ldr + col;
            if constexpr (NV == 4) {
                const u32x2 t = *reinterpret_cast<const u32x2*>(r);
                res[0] = __uint_as_float(t[0] << 16); res[1] = __uint_as_float(t[0] & 0xFFFF0000u);
                res[2] = __uint_as_float(t[1] << 16); res[3] = __uint_as_float(t[1] & 0xFFFF0000u);
            } else if constexpr (NV == 2) {
                const uint32_t t = *reinterpret_cast<const uint32_t*>(r);
                res[0] = __uint_as_float(t << 16); res[1] = __uint_as_float(t & 0xFFFF0000u);
            } else {
#pragma unroll
                for (int c = 0; c < NV; ++c) res[c] = __uint_as_float((uint32_t)r[c] << 16);
            }
        } else {
            const float* r = reinterpret_cast<const float*>(p.ep_res) + (int64_t)row * p.ep_ldr + col;
#pragma unroll
            for (int c = 0; c < NV; ++c) res[c] = r[c];
        }
    }
    const float sc = p.ep_scale ? p.ep_scale[row] : 1.0f;
    const float bi = p.ep_bias ? p.ep_bias[row] : 0.0f;
#pragma unroll
    for (int c = 0; c < NV; ++c) {
        float y = v[c];
        if (p.ep_scale) y = __fmul_rn(y, sc);
        if (p.ep_bias) y = __fadd_rn(y, bi);
        if (p.ep_res) y = __fadd_rn(y, res[c]);
        if (p.ep_relu) y = fmaxf(y, 0.0f);
        v[c] = y;
    }
}

// The epilogue's operands for CH output rows of a lane, requested together so that their
// latencies overlap (one at a time, every row would wait out a memory round trip).  All requests
// go through buffer resources whose range is the existing part of the operand -- zero for an
// absent operand -- so they need no branches: out-of-range requests return 0 and are not used.
// RW: dwords of residual per row and lane (bf16: one per column pair, fp32: one per column).
template <int CH, int RW>
struct EpBatch {
    uint32_t res[CH][RW];
    float sc[CH], bs[CH];
};
struct EpSource {
    rsrc_t res, scale, bias;
    uint32_t res_row_bytes;
    uint32_t res_off;       // lane part of the residual address inside the block-row; out of range for lanes that store nothing
    uint32_t row0_bytes;    // (first row of the lane in the block-row) * 4, for scale and bias
};
__device__ __forceinline__ EpSource make_ep_source(const SpmmArgs& p, int bi, int B, int hh, int64_t col0, bool col_ok) {
    const uint32_t esz = p.y_bf16 ? 2u : 4u;
    const int rows_here = min(B, p.S - bi * B);
    EpSource e;
    e.res_row_bytes = (uint32_t)p.ep_ldr * esz;
    e.res = __builtin_amdgcn_make_buffer_rsrc(
        const_cast<char*>(reinterpret_cast<const char*>(p.ep_res)) + (p.ep_res ? (int64_t)bi * B * p.ep_ldr * esz : 0), 0,
        p.ep_res ? (uint32_t)rows_here * e.res_row_bytes : 0u, 0x00020000);
    e.scale = __builtin_amdgcn_make_buffer_rsrc(const_cast<float*>(p.ep_scale), 0, p.ep_scale ? (uint32_t)p.S * 4u : 0u, 0x00020000);
    e.bias = __builtin_amdgcn_make_buffer_rsrc(const_cast<float*>(p.ep_bias), 0, p.ep_bias ? (uint32_t)p.S * 4u : 0u, 0x00020000);
    e.res_off = col_ok ? (uint32_t)(4 * hh) * e.res_row_bytes + (uint32_t)col0 * esz : 0x80000000u;
    e.row0_bytes = (uint32_t)(bi * B + 4 * hh) * 4u;
    return e;
}
template <int RW>
__device__ __forceinline__ void ep_request_residual(const EpSource& e, int tile_row, uint32_t (&dst)[RW]) {
    const uint32_t off = e.res_off + (uint32_t)tile_row * e.res_row_bytes;
    if constexpr (RW == 1) {
        dst[0] = __builtin_amdgcn_raw_buffer_load_b32(e.res, off, 0, 0);
    } else if constexpr (RW == 2) {
        const u32x2 t = __builtin_bit_cast(u32x2, __builtin_amdgcn_raw_buffer_load_b64(e.res, off, 0, 0));
        dst[0] = t[0]; dst[1] = t[1];
    } else {
        static_assert(RW == 4, "two or four columns per lane");
        const u32x4 t = __builtin_bit_cast(u32x4, __builtin_amdgcn_raw_buffer_load_b128(e.res, off, 0, 0));
        dst[0] = t[0]; dst[1] = t[1]; dst[2] = t[2]; dst[3] = t[3];
    }
}
__device__ __forceinline__ void ep_request_row_terms(const EpSource& e, int tile_row, float& sc, float& bs) {
    const uint32_t off = e.row0_bytes + (uint32_t)tile_row * 4u;
    sc = __uint_as_float(__builtin_amdgcn_raw_buffer_load_b32(e.scale, off, 0, 0));
    bs = __uint_as_float(__builtin_amdgcn_raw_buffer_load_b32(e.bias, off, 0, 0));
}
// y = relu(y * scale + bias + residual) on the NV values of one row, every step one fp32 rounding,
// absent parts skipped (same arithmetic as apply_epilogue).
template <int NV, bool BF16>
__device__ __forceinline__ void ep_apply(const SpmmArgs& p, const uint32_t (&res)[BF16 ? NV / 2 : NV], float sc, float bs, float (&v)[NV]) {
#pragma unroll
    for (int c = 0; c < NV; ++c) {
        float r;
        if constexpr (BF16) r = __uint_as_float((c & 1) ? (res[c / 2] & 0xFFFF0000u) : (res[c / 2] << 16));
        else r = __uint_as_float(res[c]);
        float y = v[c];
        y = p.ep_scale ? __fmul_rn(y, sc) : y;
        y = p.ep_bias ? __fadd_rn(y, bs) : y;
        y = p.ep_res ? __fadd_rn(y, r) : y;
        y = p.ep_relu ? fmaxf(y, 0.0f) : y;
        v[c] = y;
    }
}

// Geometry of the canonical packed form as seen by one lane.
template <int N, int M, int B>
struct Fmt {
    static constexpr int WB = (M == 4) ? 2 : 3;             // bits per in-group position
    static constexpr int FS = 8 * N / M;                    // value slots behind 8 columns of one row
    static constexpr int VW = (FS + 1) / 2;                 // dwords that hold them
    static constexpr int HB = FS * WB;                      // position bits behind 8 columns
    static constexpr int SLOTS = B / M * N;                 // slots per block row
    static constexpr int WPR = (SLOTS * WB + 31) / 32;      // position words per block row
    static constexpr int KS = B / 16;                       // MFMA steps per block
    static constexpr int RT = B / 32;                       // 32-row tiles per block
};

template <int FS>
__device__ __forceinline__ void load_vals(rsrc_t r, uint32_t voff, uint32_t soff, uint32_t (&v)[(FS + 1) / 2]) {
    if constexpr (FS == 1) {
        v[0] = __builtin_amdgcn_raw_buffer_load_b16(r, voff, soff, 0);
    } else if constexpr (FS == 2) {
        v[0] = __builtin_amdgcn_raw_buffer_load_b32(r, voff, soff, 0);
    } else if constexpr (FS == 4) {
        const u32x2 t = __builtin_bit_cast(u32x2, __builtin_amdgcn_raw_buffer_load_b64(r, voff, soff, 0));
        v[0] = t[0]; v[1] = t[1];
    } else if constexpr (FS == 8) {
        const u32x4 t = __builtin_bit_cast(u32x4, __builtin_amdgcn_raw_buffer_load_b128(r, voff, soff, 0));
        v[0] = t[0]; v[1] = t[1]; v[2] = t[2]; v[3] = t[3];
    } else if constexpr (FS == 6) {
        // 12 bytes, 4-byte aligned: one request (three dword requests would each touch the lines of all
        // 32 rows again, and the address unit's time per request goes with the lines touched)
        typedef __attribute__((ext_vector_type(3))) uint32_t u32x3;
        const u32x3 t = __builtin_bit_cast(u32x3, __builtin_amdgcn_raw_buffer_load_b96(r, voff, soff, 0));
        v[0] = t[0]; v[1] = t[1]; v[2] = t[2];
    } else {
#pragma unroll
        for (int i = 0; i < (FS + 1) / 2; ++i) v[i] = __builtin_amdgcn_raw_buffer_load_b32(r, voff + 4 * i, soff, 0);
    }
}

// The WPR position words of one block row (consecutive, 4-byte aligned; 8-byte aligned for WPR == 2).
template <int WPR>
__device__ __forceinline__ void load_positions(rsrc_t r, uint32_t voff, uint32_t soff, uint32_t (&w)[WPR]) {
    if constexpr (WPR == 2) {
        const u32x2 t = __builtin_bit_cast(u32x2, __builtin_amdgcn_raw_buffer_load_b64(r, voff, soff, 0));
        w[0] = t[0]; w[1] = t[1];
    } else if constexpr (WPR == 3) {
        typedef __attribute__((ext_vector_type(3))) uint32_t u32x3;
        const u32x3 t = __builtin_bit_cast(u32x3, __builtin_amdgcn_raw_buffer_load_b96(r, voff, soff, 0));
        w[0] = t[0]; w[1] = t[1]; w[2] = t[2];
    } else {
#pragma unroll
        for (int i = 0; i < WPR; ++i) w[i] = __builtin_amdgcn_raw_buffer_load_b32(r, voff + 4 * i, soff, 0);
    }
}

// Dense A operand (8 bf16 = 4 dwords) of one row for MFMA step KSTEP from the lane's compressed
// values `v` and its position stream `ws` (already shifted so that bit 0 is the lane's half).
template <int N, int M, int B, int KSTEP>
__device__ __forceinline__ u32x4 expand_frag(const uint32_t (&v)[Fmt<N, M, B>::VW],
                                             const uint32_t (&ws)[Fmt<N, M, B>::WPR]) {
    typedef Fmt<N, M, B> F;
    u32x4 out = {0u, 0u, 0u, 0u};
    if constexpr (N == M) {
        // every column kept: slot s is column s
#pragma unroll
        for (int x = 0; x < 4; ++x) out[x] = v[x];
    } else if constexpr (M == 4) {
        // the 8 columns are two groups of four; a group's four 16-bit places are one 64-bit word, and a
        // stored value goes to place `pos` by a 64-bit shift of 16 * pos.  The two position bits are moved
        // to bits 4..5 of the shift amount straight from the stream (2-bit fields never straddle words)
        constexpr int P0 = KSTEP * 2 * F::HB;
#pragma unroll
        for (int gi = 0; gi < 2; ++gi) {
            uint64_t places = 0;
#pragma unroll
            for (int j = 0; j < N; ++j) {
                const int s = gi * N + j;
                const int P = P0 + s * F::WB;
                const int wi = P >> 5, sh = P & 31;
                const uint32_t by = (sh >= 4 ? (ws[wi] >> (sh >= 4 ? sh - 4 : 0)) : (ws[wi] << (sh >= 4 ? 0 : 4 - sh))) & 0x30u;
                const uint32_t val = (s & 1) ? (v[s >> 1] >> 16) : (v[s >> 1] & 0xFFFFu);
                places |= (uint64_t)val << by;
            }
            out[2 * gi] = (uint32_t)places;
            out[2 * gi + 1] = (uint32_t)(places >> 32);
        }
    } else {
#pragma unroll
        for (int s = 0; s < F::FS; ++s) {
            constexpr int P0 = KSTEP * 2 * F::HB;
            const int P = P0 + s * F::WB;
            const int wi = P >> 5, sh = P & 31;
            uint32_t field = ws[wi] >> sh;
            if (sh + F::WB > 32 && wi + 1 < F::WPR) field |= ws[(wi + 1 < F::WPR) ? wi + 1 : wi] << ((32 - sh) & 31);
            const uint32_t pos = field & (uint32_t)(M - 1);
            const uint32_t val = (s & 1) ? (v[s >> 1] >> 16) : (v[s >> 1] & 0xFFFFu);
            const uint32_t vv = val << ((pos & 1u) << 4);
            const uint32_t dw = pos >> 1;
#pragma unroll
            for (int x = 0; x < 4; ++x) out[x] |= (dw == (uint32_t)x) ? vv : 0u;
        }
    }
    return out;
}

// 4:8 through a table: the four 3-bit positions of a full group of eight are distinct and ascending, so the
// group's 8-bit occupancy mask names the layout, and the j-th stored value belongs to the j-th set bit.  The
// table (256 entries of four v_perm_b32 selectors, 4 KB of LDS, built once per workgroup) turns the two stored
// dwords straight into the four operand dwords: 4 bit-field extracts, 4 shift-ors, one 16-byte LDS read and 4
// permutes instead of about 76 vector instructions.  Needs whole groups (K a multiple of 8: the specialised
// kernels require 16); groups wholly past K or S hold zeros at positions 0..3, which the same rule covers.
// Entry of mask m, operand dword x: low half from position 2x, high half from 2x + 1; a position that is the
// r-th set bit of m takes bytes 2r, 2r + 1 of the stored pair (v_perm_b32 numbers the second source's bytes
// 0..3 and the first's 4..7), an empty position the selector 0x0c (zero).
__device__ __forceinline__ void lut48_fill(u32x4* lut, int tid, int nthreads) {
    for (int m = tid; m < 256; m += nthreads) {
        u32x4 e;
#pragma unroll
        for (int x = 0; x < 4; ++x) {
            uint32_t sel = 0;
#pragma unroll
            for (int h = 0; h < 2; ++h) {
                const int q = 2 * x + h;
                const uint32_t r = (uint32_t)__builtin_popcount((unsigned)m & ((1u << q) - 1u)) & 3u;
                const uint32_t half = ((unsigned)m >> q) & 1u ? ((2u * r + 1u) << 8 | 2u * r) : 0x0C0Cu;
                sel |= half << (16 * h);
            }
            e[x] = sel;
        }
        lut[m] = e;
    }
}
// patterns whose dense expansion goes through the table
template <int N, int M, bool SMF>
constexpr bool lut48_pattern() { return !SMF && N == 4 && M == 8; }
template <int B, int KSTEP>
__device__ __forceinline__ u32x4 expand_frag_lut48(const uint32_t (&v)[2], const uint32_t (&ws)[Fmt<4, 8, B>::WPR], const u32x4* lut) {
    typedef Fmt<4, 8, B> F;
    constexpr int P0 = KSTEP * 2 * F::HB;          // first position bit of this step in the lane's (shifted) stream
    constexpr int wi = P0 >> 5, sh = P0 & 31;
    const uint32_t field = sh + F::HB > 32 ? __builtin_amdgcn_alignbit(ws[wi + 1 < F::WPR ? wi + 1 : wi], ws[wi], sh) : ws[wi] >> sh;
    const uint32_t m = (1u << (field & 7u)) | (1u << ((field >> 3) & 7u)) | (1u << ((field >> 6) & 7u)) | (1u << ((field >> 9) & 7u));
    const u32x4 sel = lut[m];
    return u32x4{__builtin_amdgcn_perm(v[1], v[0], sel[0]), __builtin_amdgcn_perm(v[1], v[0], sel[1]),
                 __builtin_amdgcn_perm(v[1], v[0], sel[2]), __builtin_amdgcn_perm(v[1], v[0], sel[3])};
}

// A operand and index register of the sparse matrix-core instruction for 32-row tile values `av`
// (the lane's stored values per 16-deep step) and position stream `ws` (shifted so that bit 0 is
// the lane's half), 32-deep step s2.
template <int N, int M, int B, int s2>
__device__ __forceinline__ void smf_operand(const uint32_t (&av)[Fmt<N, M, B>::KS][Fmt<N, M, B>::VW],
                                            const uint32_t (&ws)[Fmt<N, M, B>::WPR], u32x4& a4, uint32_t& idx) {
    typedef Fmt<N, M, B> F;
    constexpr int P = 4 * s2 * F::HB;   // first position bit of this step in the lane's (shifted) stream
    if constexpr (M == 8) {
        // the lane's 16 columns are two groups of 8; position bits of both: 2 * HB bits from P
        uint32_t field = ws[P >> 5] >> (P & 31);
        if constexpr ((P & 31) + 2 * F::HB > 32 && (P >> 5) + 1 < F::WPR) field |= ws[(P >> 5) + 1] << (32 - (P & 31));
        if constexpr (N == 4) {
            // 4:8 with at most two kept values per aligned four (the pack's flag, asserted by the caller): every
            // full group of eight holds exactly two in its lower and two in its upper four, stored in ascending
            // column order, so the stored values are the operand as they are (like 2:4) and a value's position
            // inside its four is the low two bits of its 3-bit position.  (Groups past K or S hold zeros at
            // positions 0..3: two "values" per four as well.)
            a4 = u32x4{av[2 * s2][0], av[2 * s2][1], av[2 * s2 + 1][0], av[2 * s2 + 1][1]};
            idx = 0;
#pragma unroll
            for (int i = 0; i < 8; ++i) idx |= ((field >> (3 * i)) & 3u) << (2 * i);
        } else if constexpr (N == 2) {
            // group g: stored (v0, v1) at positions (p0, p1); the lower 4-group takes those with
            // position < 4, the upper the others, both with in-group positions (p0 & 3, p1 & 3)
            uint32_t d[4];
            idx = 0;
#pragma unroll
            for (int g = 0; g < 2; ++g) {
                const uint32_t w = av[2 * s2 + g][0];
                const uint32_t p0 = (field >> (6 * g)) & 7u, p1 = (field >> (6 * g + 3)) & 7u;
                const uint32_t lowmask = ((p0 & 4u) ? 0u : 0x0000FFFFu) | ((p1 & 4u) ? 0u : 0xFFFF0000u);
                d[2 * g] = w & lowmask;
                d[2 * g + 1] = w & ~lowmask;
                const uint32_t nib = (p0 & 3u) | ((p1 & 3u) << 2);
                idx |= (nib | (nib << 4)) << (8 * g);
            }
            a4 = u32x4{d[0], d[1], d[2], d[3]};
        } else {
            // one stored value per group of 8, paired with a zero at the same position
            const uint32_t va = av[2 * s2][0], vb2 = av[2 * s2 + 1][0];
            const uint32_t pa = field & 7u, pb = (field >> 3) & 7u;
            a4 = u32x4{(pa & 4u) ? 0u : va, (pa & 4u) ? va : 0u, (pb & 4u) ? 0u : vb2, (pb & 4u) ? vb2 : 0u};
            const uint32_t na = (pa & 3u) * 5u, nb = (pb & 3u) * 5u;     // (p, p) as a nibble
            idx = (na | (na << 4)) | ((nb | (nb << 4)) << 8);
        }
    } else if constexpr (N == 2) {
        // 2:4: values and positions as packed
        a4 = u32x4{av[2 * s2][0], av[2 * s2][1], av[2 * s2 + 1][0], av[2 * s2 + 1][1]};
        idx = ws[P >> 5] >> (P & 31);
    } else {
        // 1:4: each stored value gets a zero partner at the same position
        const uint32_t w0 = av[2 * s2][0], w1 = av[2 * s2 + 1][0];
        a4 = u32x4{w0 & 0xFFFFu, w0 >> 16, w1 & 0xFFFFu, w1 >> 16};
        uint32_t y = (ws[P >> 5] >> (P & 31)) & 0xFFu;   // p3 p2 p1 p0, two bits each
        y = (y | (y << 4)) & 0x0F0Fu;
        y = (y | (y << 2)) & 0x3333u;
        idx = y | (y << 2);
    }
}

// One kept block: multiply the block held in ring slot (xr, av, aw) into acc.  With PREFETCH the
// X rows of block column bj_next are requested into the same registers as soon as their
// current contents have been turned into MFMA operands, and block t_next's compressed slice
// after the last step; the body is straight-line code, so the compiler's wait counters stay exact.
// SMF: the A operand goes to the sparse matrix core instruction (v_smfmac_f32_32x32x32_bf16, "at
// most 2 non-zeros in every aligned group of 4" along K) instead of being expanded to dense form.
// Operand layout as measured on gfx950: lane (row l % 32, half h = l / 32) supplies the 8 stored
// values of its row for the 16 dense columns 16h .. 16h+15 of the 32-deep step and, in bits 0..15 of
// the index register, a 2-bit position per stored value; the B operand is the concatenation of the
// two dense 32x32x16 operands of the step's two 16-deep halves (exactly what the X path builds);
// two stored values of a group may name the same position when one of them is zero.  For 2:4 the
// lane's slice of the canonical pack IS the operand: 16 bytes of values and 16 position bits.
// m = 8 with at most two kept per group also qualifies (any two of eight put at most two into each
// aligned four): the 8-group's stored values go to the lower or the upper 4-group by position bit 2.
template <int N, int M>
constexpr bool smf_pattern() { return N <= 2; }
// 4:8 also qualifies when the packed layer holds at most two values per aligned four (the flag crisp_pack
// reports; SpmmArgs::two_of_four carries the caller's assertion).  Only the kernel families for plain X
// are instantiated for it (register kernels, X-resident kernels, LDS-resident sparse operands).
template <int N, int M>
constexpr bool smf_flagged_pattern() { return N == 4 && M == 8; }
// whether the launch of pattern N:M goes to the sparse matrix-core instantiation
template <int N, int M>
inline bool smf_wanted(const SpmmArgs& a) { return a.use_smf && (smf_pattern<N, M>() || a.two_of_four); }

template <int N, int M, int B, int WD, bool PREFETCH, int CONV, bool SMF = false>
struct BlockBody {
    typedef Fmt<N, M, B> F;
    static constexpr int XW = (CONV >= 2 && CONV <= 4) ? 2 : WD;    // registers per loaded X row
    typedef typename XVec<XW>::type xvec_t;
    static constexpr int RT = F::RT, KS = F::KS, NACC = 2 * WD;

    // Conv mode: context of block column bj.  All B K-rows of the block column belong to one
    // filter tap (a, b) because C % B == 0.  The lane's two columns are output positions
    // (oh, ow), (oh, ow+1) of one image; their sources are act[c][img][oh+a-pad][ow+b-pad (+1)].
    // Both inside the image: one (possibly 2-byte-aligned) dword load.  Left border (only the
    // second inside) or right border (only the first): the neighbouring in-row dword is loaded
    // instead and the selectors pick the valid half and a zero.  Row outside: any valid address,
    // selectors yield zeros.
    __device__ static __forceinline__ XCtx conv_ctx(const SpmmArgs& p, const ConvPos& cp, int bj) {
        const int tap = (int)(((float)bj + 0.5f) * p.inv_cpb);
        const int a = (int)(((float)tap + 0.5f) * p.inv_kw);
        const int b = tap - a * p.kw;
        if constexpr (CONV == 3) {
            // nothing depends on the block column: window origins of the two columns
            XCtx c;
            c.off = (uint32_t)((cp.img * p.H + cp.oh * p.stride - p.pad) * p.W + cp.ow * p.stride - p.pad);
            c.off2 = (uint32_t)((cp.img1 * p.H + cp.oh1 * p.stride - p.pad) * p.W + cp.ow1 * p.stride - p.pad);
            c.sel_lo = SEL_LO;
            c.sel_hi = SEL_LO;
            return c;
        }
        if constexpr (CONV == 4) {
            // 1x1 filter, stride 2, no padding, even W and Wo: the lane's two columns are the elements 0
            // and 2 of one 8-byte piece of input row 2*oh (always inside the image)
            XCtx c;
            c.off = cp.half_off + (uint32_t)((cp.img * p.H + cp.oh * 2) * p.W + cp.ow * 2) * 2u;
            c.off2 = 0u;
            c.sel_lo = SEL_LO;
            c.sel_hi = SEL_LO;
            return c;
        }
        if constexpr (CONV == 2) {
            // each column on its own: source act[c][img][oh*stride + a - pad][ow*stride + b - pad]
            // or, outside the image, any valid address and a selector that yields zeros
            const int ih0 = cp.oh * p.stride + a - p.pad, iw0 = cp.ow * p.stride + b - p.pad;
            const int ih1 = cp.oh1 * p.stride + a - p.pad, iw1 = cp.ow1 * p.stride + b - p.pad;
            const bool v0 = (unsigned)ih0 < (unsigned)p.H && (unsigned)iw0 < (unsigned)p.W;
            const bool v1 = (unsigned)ih1 < (unsigned)p.H && (unsigned)iw1 < (unsigned)p.W;
            const int safe = (cp.img * p.H + cp.oh * p.stride) * p.W + cp.ow * p.stride;   // inside the image
            const int s0 = v0 ? (cp.img * p.H + ih0) * p.W + iw0 : safe;
            const int s1 = v1 ? (cp.img1 * p.H + ih1) * p.W + iw1 : safe;
            XCtx c;
            c.off = cp.half_off + (uint32_t)s0 * 2u;
            c.off2 = cp.half_off + (uint32_t)s1 * 2u;
            c.sel_lo = v0 ? SEL_LO : SEL_ZERO;
            c.sel_hi = v1 ? SEL_LO : SEL_ZERO;
            return c;
        }
        // The lane's second column is the next output position, which may lie in the next output row or
        // image (odd Wo).  The host picks this mode only where the two sources are then still neighbours in
        // memory when both are inside the image: always inside one output row, and across rows and images
        // when the padding is (k - 1) / 2 in both directions (then consecutive output positions read
        // consecutive input elements for every tap).
        const int ih = cp.oh + a - p.pad, iw = cp.ow + b - p.pad;
        const int ih1 = cp.oh1 + a - p.pad, iw1 = cp.ow1 + b - p.pad;
        const bool v0 = (unsigned)ih < (unsigned)p.H && (unsigned)iw < (unsigned)p.W;
        const bool v1 = (unsigned)ih1 < (unsigned)p.H && (unsigned)iw1 < (unsigned)p.W;
        const int centre = (cp.img * p.H + cp.oh) * p.W + cp.ow;
        const int src = (cp.img * p.H + ih) * p.W + iw;
        const int src1 = (cp.img1 * p.H + ih1) * p.W + iw1;
        XCtx c;
        int off = centre;
        c.sel_lo = SEL_ZERO;
        c.sel_hi = SEL_ZERO;
        if (v0 && v1) { off = src; c.sel_lo = SEL_LO; c.sel_hi = SEL_HI; }
        else if (v1) {
            // loaded (e0, e1) at the second column's source: column 1 <- e0; at the very end of a channel
            // plane the dword one element earlier is loaded instead and column 1 <- e1
            const bool last = (int64_t)src1 + 1 >= p.plane;
            off = last ? src1 - 1 : src1;
            c.sel_hi = last ? SEL_HI : SEL_LO;
        }
        else if (v0) { off = src - 1; c.sel_lo = SEL_HI; }   // loaded (e[src-1], e[src]): column 0 <- e[src]
        c.off = cp.half_off + (uint32_t)off * 2u;
        c.off2 = 0u;
        return c;
    }

    // X rows of block column bj, MFMA step ks.  K is a multiple of 16 here, so a step lies either
    // wholly inside the matrix or wholly past its end; a step past the end re-reads the last 16
    // rows instead (finite values times the zero padding of the packed block).
    __device__ static __forceinline__ void load_x(xvec_t (&dst)[8], const SpmmArgs& p, const ConvPos& cp,
                                                   uint32_t lane_off, uint32_t lane_off2, int bj, int ks) {
        if constexpr (CONV == 5) {
            // octet-interleaved X, [K/8][ldx][8]: the 8 K-values a lane feeds to the matrix core for one column
            // are 16 consecutive bytes.  dst[0..3] = operand of the lane's first column (offset lane_off),
            // dst[4..7] = of its second (lane_off2); the lane's half hh is part of both offsets.
            static_assert(WD == 1, "two columns per lane");
            const int kb = min(bj * B + ks * 16, p.K - 16);
            const rsrc_t r = make_rsrc(p.X + (int64_t)(kb >> 3) * p.ldx * 8);
            const u32x4 t0 = __builtin_bit_cast(u32x4, __builtin_amdgcn_raw_buffer_load_b128(r, lane_off, 0, 0));
            const u32x4 t1 = __builtin_bit_cast(u32x4, __builtin_amdgcn_raw_buffer_load_b128(r, lane_off2, 0, 0));
#pragma unroll
            for (int i = 0; i < 4; ++i) { dst[i] = t0[i]; dst[4 + i] = t1[i]; }
        } else if constexpr (CONV == 3) {
            // K-row k = tap*C + c with tap = a*kw + b, per row; lane_off / lane_off2 are the element
            // offsets of the two columns' window origins (oh*stride - pad, ow*stride - pad) inside a
            // channel plane, cp.half_off holds hh*8 here (rows, not bytes)
            const rsrc_t r = __builtin_amdgcn_make_buffer_rsrc(const_cast<uint16_t*>(p.act), 0, p.act_bytes, 0x00020000);
            const int ih0 = cp.oh * p.stride - p.pad, iw0 = cp.ow * p.stride - p.pad;
            const int ih1 = cp.oh1 * p.stride - p.pad, iw1 = cp.ow1 * p.stride - p.pad;
#pragma unroll
            for (int i = 0; i < 8; ++i) {
                const int k = bj * B + ks * 16 + (int)cp.half_off + i;
                const int tap = (int)(((float)k + 0.5f) * p.inv_C);
                const int c = k - tap * p.C;
                const int a = (int)(((float)tap + 0.5f) * p.inv_kw);
                const int b = tap - a * p.kw;
                const bool kin = k < p.K;
                const bool v0 = kin && (unsigned)(ih0 + a) < (unsigned)p.H && (unsigned)(iw0 + b) < (unsigned)p.W;
                const bool v1 = kin && (unsigned)(ih1 + a) < (unsigned)p.H && (unsigned)(iw1 + b) < (unsigned)p.W;
                const uint32_t shift = (uint32_t)(c * (int)p.plane + a * p.W + b);
                const uint32_t o0 = v0 ? (lane_off + shift) * 2u : 0xFFFFFFFEu;
                const uint32_t o1 = v1 ? (lane_off2 + shift) * 2u : 0xFFFFFFFEu;
                const uint32_t e0 = __builtin_amdgcn_raw_buffer_load_b16(r, o0, 0, 0);
                const uint32_t e1 = __builtin_amdgcn_raw_buffer_load_b16(r, o1, 0, 0);
                dst[i] = u32x2{e0, e1};
            }
        } else if constexpr (CONV != 0) {
            // K-row = tap*C + c: the 16 rows of the step are 16 consecutive channel planes
            const int tap = (int)(((float)bj + 0.5f) * p.inv_cpb);
            const int c0 = bj * B - tap * p.C + ks * 16;
            const rsrc_t r = make_rsrc(p.act + (int64_t)c0 * p.plane);
            const uint32_t row_bytes = (uint32_t)p.plane * 2u;
            if constexpr (CONV == 4) {
#pragma unroll
                for (int i = 0; i < 8; ++i) dst[i] = buf_load_x<2>(r, lane_off, (uint32_t)i * row_bytes);
            } else if constexpr (CONV == 2) {
#pragma unroll
                for (int i = 0; i < 8; ++i) {
                    const uint32_t e0 = __builtin_amdgcn_raw_buffer_load_b16(r, lane_off, (uint32_t)i * row_bytes, 0);
                    const uint32_t e1 = __builtin_amdgcn_raw_buffer_load_b16(r, lane_off2, (uint32_t)i * row_bytes, 0);
                    dst[i] = u32x2{e0, e1};
                }
            } else {
#pragma unroll
                for (int i = 0; i < 8; ++i) dst[i] = buf_load_x<WD>(r, lane_off, (uint32_t)i * row_bytes);
            }
        } else {
            const int kb = min(bj * B + ks * 16, p.K - 16);
            const rsrc_t r = make_rsrc(p.X + (int64_t)kb * p.ldx);
            const uint32_t row_bytes = (uint32_t)p.ldx * 2u;
#pragma unroll
            for (int i = 0; i < 8; ++i) dst[i] = buf_load_x<WD>(r, lane_off, (uint32_t)i * row_bytes);
        }
    }

    // Requests the lane's slice of block t: values of rows rt*32 + jj, columns ks*16 + hh*8 .. +8,
    // and the whole position stream of those rows (a_off / i_off carry the lane part of the
    // address).  Nothing is consumed here, so no wait is placed next to the requests.
    __device__ static __forceinline__ void load_a(uint32_t (&v)[RT][KS][F::VW], uint32_t (&w)[RT][F::WPR],
                                                   const SpmmArgs& p, uint32_t a_off, uint32_t i_off, int t) {
        const rsrc_t rv = make_rsrc(p.vals);
        const rsrc_t ri = make_rsrc(p.idxw);
        const uint32_t vb = (uint32_t)t * (B * F::SLOTS * 2);
        const uint32_t ib = (uint32_t)t * (B * F::WPR * 4);
#pragma unroll
        for (int rt = 0; rt < RT; ++rt) {
            if constexpr (SMF) {
                // one request per 32-deep step: the 2*FS stored values behind the lane's 16 columns
#pragma unroll
                for (int s2 = 0; s2 < KS / 2; ++s2) {
                    uint32_t t[(2 * F::FS + 1) / 2];
                    load_vals<2 * F::FS>(rv, a_off + (rt * 32 * F::SLOTS + s2 * 4 * F::FS) * 2, vb, t);
                    if constexpr (F::FS == 1) {
                        v[rt][2 * s2][0] = t[0] & 0xFFFFu;       // one stored value per 8 columns
                        v[rt][2 * s2 + 1][0] = t[0] >> 16;
                    } else {
#pragma unroll
                        for (int x = 0; x < F::VW; ++x) { v[rt][2 * s2][x] = t[x]; v[rt][2 * s2 + 1][x] = t[F::VW + x]; }
                    }
                }
            } else {
#pragma unroll
                for (int ks = 0; ks < KS; ++ks)
                    load_vals<F::FS>(rv, a_off + (rt * 32 * F::SLOTS + ks * 2 * F::FS) * 2, vb, v[rt][ks]);
            }
            if constexpr (N != M) load_positions<F::WPR>(ri, i_off + rt * 32 * F::WPR * 4, ib, w[rt]);
        }
    }

    template <int ks>
    __device__ static __forceinline__ void step(f32x16 (&acc)[RT][NACC], xvec_t (&xr)[KS][8],
                                                const uint32_t (&av)[RT][KS][F::VW], const uint32_t (&ws)[RT][F::WPR],
                                                const SpmmArgs& p, const ConvPos& cp, const XCtx& cur, const XCtx& next,
                                                int bj_next) {
        // 8 rows x 2*WD columns of 16-bit halves -> 2*WD operands of 8 K-values each
        uint32_t xd[8][XW];
#pragma unroll
        for (int r = 0; r < 8; ++r) xvec_unpack(xr[ks][r], xd[r]);
        bf16x8 bfrag[NACC];
#pragma unroll
        for (int pd = 0; pd < WD; ++pd) {
            u32x4 lo, hi;
#pragma unroll
            for (int q = 0; q < 4; ++q) {
                // v_perm_b32: result bytes picked from {r1 (bytes 4..7), r0 (bytes 0..3)}
                if constexpr (CONV == 5) {
                    lo[q] = xd[q][0];           // loaded in operand form
                    hi[q] = xd[4 + q][0];
                } else if constexpr (CONV >= 2) {
                    // register 0 of a row holds the first column's element, register 1 the second's
                    lo[q] = __builtin_amdgcn_perm(xd[2 * q + 1][0], xd[2 * q][0], cur.sel_lo);
                    hi[q] = __builtin_amdgcn_perm(xd[2 * q + 1][1], xd[2 * q][1], cur.sel_hi);
                } else {
                    const uint32_t r0 = xd[2 * q][pd], r1 = xd[2 * q + 1][pd];
                    lo[q] = __builtin_amdgcn_perm(r1, r0, CONV ? cur.sel_lo : SEL_LO);  // first column of the pair
                    hi[q] = __builtin_amdgcn_perm(r1, r0, CONV ? cur.sel_hi : SEL_HI);  // second column
                }
            }
            bfrag[2 * pd] = __builtin_bit_cast(bf16x8, lo);
            bfrag[2 * pd + 1] = __builtin_bit_cast(bf16x8, hi);
        }
        if constexpr (PREFETCH) load_x(xr[ks], p, cp, next.off, next.off2, bj_next, ks);
#pragma unroll
        for (int rt = 0; rt < RT; ++rt) {
            u32x4 a4;
            if constexpr (lut48_pattern<N, M, SMF>()) a4 = expand_frag_lut48<B, ks>(av[rt][ks], ws[rt], cp.lut48);
            else a4 = expand_frag<N, M, B, ks>(av[rt][ks], ws[rt]);
            const bf16x8 afrag = __builtin_bit_cast(bf16x8, a4);
#pragma unroll
            for (int c = 0; c < NACC; ++c)
                acc[rt][c] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(afrag, bfrag[c], acc[rt][c], 0, 0, 0);
        }
    }

    // Sparse-MFMA version of two consecutive steps (one 32-deep step of the sparse instruction).
    template <int s2>
    __device__ static __forceinline__ void step_smf(f32x16 (&acc)[RT][NACC], xvec_t (&xr)[KS][8],
                                                    const uint32_t (&av)[RT][KS][F::VW], const uint32_t (&ws)[RT][F::WPR],
                                                    const SpmmArgs& p, const ConvPos& cp, const XCtx& cur, const XCtx& next,
                                                    int bj_next) {
        u32x4 half[2][NACC];
#pragma unroll
        for (int k2 = 0; k2 < 2; ++k2) {
            const int ks = 2 * s2 + k2;
            uint32_t xd[8][XW];
#pragma unroll
            for (int r = 0; r < 8; ++r) xvec_unpack(xr[ks][r], xd[r]);
#pragma unroll
            for (int pd = 0; pd < WD; ++pd) {
                u32x4 lo, hi;
#pragma unroll
                for (int q = 0; q < 4; ++q) {
                    if constexpr (CONV == 5) {
                        lo[q] = xd[q][0];
                        hi[q] = xd[4 + q][0];
                    } else if constexpr (CONV >= 2) {
                        lo[q] = __builtin_amdgcn_perm(xd[2 * q + 1][0], xd[2 * q][0], cur.sel_lo);
                        hi[q] = __builtin_amdgcn_perm(xd[2 * q + 1][1], xd[2 * q][1], cur.sel_hi);
                    } else {
                        const uint32_t r0 = xd[2 * q][pd], r1 = xd[2 * q + 1][pd];
                        lo[q] = __builtin_amdgcn_perm(r1, r0, CONV ? cur.sel_lo : SEL_LO);
                        hi[q] = __builtin_amdgcn_perm(r1, r0, CONV ? cur.sel_hi : SEL_HI);
                    }
                }
                half[k2][2 * pd] = lo;
                half[k2][2 * pd + 1] = hi;
            }
            if constexpr (PREFETCH) load_x(xr[ks], p, cp, next.off, next.off2, bj_next, ks);
        }
#pragma unroll
        for (int rt = 0; rt < RT; ++rt) {
            u32x4 a4;
            uint32_t idx;
            smf_operand<N, M, B, s2>(av[rt], ws[rt], a4, idx);
            const bf16x8 afrag = __builtin_bit_cast(bf16x8, a4);
#pragma unroll
            for (int c = 0; c < NACC; ++c) {
                typedef __attribute__((ext_vector_type(8))) uint32_t u32x8;
                const u32x8 b8 = {half[0][c][0], half[0][c][1], half[0][c][2], half[0][c][3],
                                  half[1][c][0], half[1][c][1], half[1][c][2], half[1][c][3]};
                acc[rt][c] = __builtin_amdgcn_smfmac_f32_32x32x32_bf16(afrag, __builtin_bit_cast(bf16x16, b8), acc[rt][c],
                                                                       (int)idx, 0, 0);
            }
        }
    }

    // cx: context of the block held in this ring slot; replaced by the next block's on prefetch.
    __device__ static __forceinline__ void run(f32x16 (&acc)[RT][NACC], xvec_t (&xr)[KS][8],
                                               uint32_t (&av)[RT][KS][F::VW], uint32_t (&aw)[RT][F::WPR], XCtx& cx,
                                               const SpmmArgs& p, const ConvPos& cp, uint32_t a_off, uint32_t i_off,
                                               uint32_t aw_sh, int t_next, int bj_known = -1) {
        // bj_known: block column of block t_next when the caller already holds it (else it is read here)
        int bj_next = 0;
        XCtx nx = cx;
        if constexpr (PREFETCH) {
            bj_next = bj_known >= 0 ? bj_known : p.col_idx[t_next];
            if constexpr (CONV != 0 && CONV != 5) nx = conv_ctx(p, cp, bj_next);
        }
        // drop the other half-wave's position bits: bit 0 of ws is this lane's first slot
        uint32_t ws[RT][F::WPR];
        if constexpr (N != M) {
#pragma unroll
            for (int rt = 0; rt < RT; ++rt)
#pragma unroll
                for (int i = 0; i < F::WPR; ++i)
                    ws[rt][i] = __builtin_amdgcn_alignbit(i + 1 < F::WPR ? aw[rt][i + 1] : 0u, aw[rt][i], aw_sh);
        }
        if constexpr (SMF) {
            step_smf<0>(acc, xr, av, ws, p, cp, cx, nx, bj_next);
            if constexpr (KS == 4) step_smf<1>(acc, xr, av, ws, p, cp, cx, nx, bj_next);
        } else {
            step<0>(acc, xr, av, ws, p, cp, cx, nx, bj_next);
            step<1>(acc, xr, av, ws, p, cp, cx, nx, bj_next);
            if constexpr (KS == 4) {
                step<2>(acc, xr, av, ws, p, cp, cx, nx, bj_next);
                step<3>(acc, xr, av, ws, p, cp, cx, nx, bj_next);
            }
        }
        if constexpr (PREFETCH) {
            load_a(av, aw, p, a_off, i_off, t_next);
            cx = nx;
        }
    }
};

// Output of one wave: ROWS accumulator rows of a 64*WD-column strip of block-row bi, namely the
// rows with accumulator index pr = row_first + q * ROW_STEP (pr = rt*16 + r; register r of a 32x32
// tile is row 8*(r/4) + 4*hh + r%4 of the tile, column jj; the NACC tiles of a lane are consecutive
// columns).  row_source(pr, v) fills v with the lane's NACC values of that row.  Y is written
// through a buffer resource that spans the block-row's existing rows: rows past S and lanes past
// the last column fall outside its range and the hardware drops them, so the stores need no
// branches.  (Ncol is a multiple of 4 here, so a lane's columns are all inside or all outside.)
// The four (epilogue yes/no) x (bf16/fp32 output) variants of the store loop are separate copies
// chosen once per wave, so the loop itself holds no branches; with an epilogue its operands are
// requested for a batch of rows before the first of them is used.
template <int B, int WD, int ROWS, int ROW_STEP, typename RowSource>
__device__ __forceinline__ void store_rows(const SpmmArgs& p, int bi, int hh, int64_t col0, bool col_ok, int row_first,
                                           RowSource row_source) {
    constexpr int NACC = 2 * WD;
    const uint32_t esz = p.y_bf16 ? 2u : 4u;
    const uint32_t row_bytes = (uint32_t)p.ldy * esz;
    const int rows_here = min(B, p.S - bi * B);
    const rsrc_t ry = __builtin_amdgcn_make_buffer_rsrc(
        reinterpret_cast<char*>(p.Y) + (int64_t)bi * B * p.ldy * esz, 0, (uint32_t)rows_here * row_bytes, 0x00020000);
    const uint32_t y_off = col_ok ? (uint32_t)(4 * hh) * row_bytes + (uint32_t)col0 * esz : 0x80000000u;
    auto tile_row_of = [&](int q) __attribute__((always_inline)) {
        const int pr = row_first + q * ROW_STEP;
        return (pr >> 4) * 32 + 8 * ((pr & 15) >> 2) + (pr & 3);
    };
    auto emit = [&](auto with_ep, auto as_bf16) __attribute__((always_inline)) {
        constexpr bool BF16 = decltype(as_bf16)::value;
        auto store_row = [&](int tile_row, const float (&v)[NACC]) __attribute__((always_inline)) {
            const uint32_t off = y_off + (uint32_t)tile_row * row_bytes;
            if constexpr (BF16) {
                uint32_t pk[WD];
#pragma unroll
                for (int c = 0; c < WD; ++c) {
                    const f32x2 two = {v[2 * c], v[2 * c + 1]};
                    pk[c] = __builtin_bit_cast(uint32_t, __builtin_convertvector(two, bf16x2));  // v_cvt_pk_bf16_f32 (RNE)
                }
                if constexpr (WD == 1) {
                    __builtin_amdgcn_raw_buffer_store_b32(pk[0], ry, off, 0, 0);
                } else {
                    const u32x2 two = {pk[0], pk[WD - 1]};
                    __builtin_amdgcn_raw_buffer_store_b64(two, ry, off, 0, 0);
                }
            } else {
                if constexpr (WD == 1) {
                    const u32x2 two = {__float_as_uint(v[0]), __float_as_uint(v[1])};
                    __builtin_amdgcn_raw_buffer_store_b64(two, ry, off, 0, 0);
                } else {
                    const u32x4 four = {__float_as_uint(v[0]), __float_as_uint(v[1]), __float_as_uint(v[NACC - 2]),
                                        __float_as_uint(v[NACC - 1])};
                    __builtin_amdgcn_raw_buffer_store_b128(four, ry, off, 0, 0);
                }
            }
        };
        if constexpr (decltype(with_ep)::value) {
            constexpr int RW = BF16 ? WD : NACC;
            constexpr int CH = ROWS < 16 ? ROWS : 16;          // rows per batch of requests
            static_assert(ROWS % CH == 0, "whole batches");
            const EpSource src = make_ep_source(p, bi, B, hh, col0, col_ok);
#pragma unroll
            for (int q0 = 0; q0 < ROWS; q0 += CH) {
                EpBatch<CH, RW> eb;
#pragma unroll
                for (int j = 0; j < CH; ++j) {
                    const int tile_row = tile_row_of(q0 + j);
                    ep_request_residual<RW>(src, tile_row, eb.res[j]);
                    ep_request_row_terms(src, tile_row, eb.sc[j], eb.bs[j]);
                }
#pragma unroll
                for (int j = 0; j < CH; ++j) {
                    float v[NACC];
                    row_source(row_first + (q0 + j) * ROW_STEP, v);
                    ep_apply<NACC, BF16>(p, eb.res[j], eb.sc[j], eb.bs[j], v);
                    store_row(tile_row_of(q0 + j), v);
                }
            }
        } else {
#pragma unroll
            for (int q = 0; q < ROWS; ++q) {
                float v[NACC];
                row_source(row_first + q * ROW_STEP, v);
                store_row(tile_row_of(q), v);
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

// Two waves per SIMD (256 registers each) wherever the lane's slice of the packed block is small
// enough to fit beside 128 accumulators and 64 X registers; the wide-strip kernels of the denser
// patterns would spill there and run with one wave per SIMD instead.
template <int N, int M, int B, int WD, bool SMF>
constexpr int waves_per_simd() { return (WD == 2 && B == 64 && Fmt<N, M, B>::FS >= 4 && !SMF) ? 1 : 2; }

// (upper limit: three for the narrow-strip kernels of the sparse matrix-core patterns on plain X, whose
// registers allow it)
template <int N, int M, int B, int WD, int NWK, int CONV, bool SMF>
constexpr int waves_per_simd_max() { return (WD == 1 && SMF && NWK == 1 && CONV == 0 && B == 64) ? 3 : 2; }

template <int N, int M, int B, int WD, int NWK, int PF, int CONV, bool SMF = false>
__global__ __launch_bounds__(NWK > 1 ? 64 * NWK : 256)
__attribute__((amdgpu_waves_per_eu(waves_per_simd_max<N, M, B, WD, NWK, CONV, SMF>() == 3 ? 3 : waves_per_simd<N, M, B, WD, SMF>(),
                                   waves_per_simd_max<N, M, B, WD, NWK, CONV, SMF>())))
void spmm_reg_kernel(SpmmArgs p) {
    static_assert(!CONV || WD == 1, "conv modes work on two output columns per lane");
    typedef Fmt<N, M, B> F;
    constexpr int RT = F::RT, KS = F::KS;
    constexpr int STRIPS = NWK > 1 ? 1 : 4;       // column strips per workgroup
    constexpr int NACC = 2 * WD;                   // accumulator tiles (consecutive columns) per lane
    typedef BlockBody<N, M, B, WD, true, CONV, SMF> BodyP;
    typedef BlockBody<N, M, B, WD, false, CONV, SMF> BodyL;
    typedef typename BodyP::xvec_t xvec_t;

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
        lut48_fill(lut48, tid, NWK > 1 ? 64 * NWK : 256);
        __syncthreads();
    }
    const int64_t wave_col = ((int64_t)nt * STRIPS + (NWK > 1 ? 0 : wave)) * (64 * WD);
    if (NWK == 1 && wave_col >= p.Ncol) return;   // no further barriers in this mode
    const int64_t col0 = wave_col + jj * NACC;
    const bool col_ok = col0 < p.Ncol;
    // lane part of every X address (bytes): its 8-row half and its columns; lanes past the last
    // column read column 0 instead (in bounds) and never store
    const int64_t col_ld = col_ok ? col0 : 0;
    ConvPos cp = {0, 0, 0, 0u, 0, 0, 0, lut48};
    uint32_t lane_off = 0;
    if constexpr (CONV != 0) {
        // column -> (image, oh, ow); exact division through fp64 reciprocals (col < 2^31)
        const int j = (int)col_ld;
        int t = (int)((double)j * p.inv_Wo);
        t -= (t * p.Wo > j);
        t += ((t + 1) * p.Wo <= j);
        cp.ow = j - t * p.Wo;
        int im = (int)((double)t * p.inv_Ho);
        im -= (im * p.Ho > t);
        im += ((im + 1) * p.Ho <= t);
        cp.oh = t - im * p.Ho;
        cp.img = im;
        cp.half_off = CONV == 3 ? (uint32_t)(hh * 8) : (uint32_t)((int64_t)hh * 8 * p.plane * 2);
        // the next column (conv mode 2; Ncol is even, so it exists whenever the first one does)
        cp.ow1 = cp.ow + 1; cp.oh1 = cp.oh; cp.img1 = cp.img;
        if (cp.ow1 == p.Wo) { cp.ow1 = 0; cp.oh1 += 1; }
        if (cp.oh1 == p.Ho) { cp.oh1 = 0; cp.img1 += 1; }
        if (cp.img1 * p.Ho * p.Wo + cp.oh1 * p.Wo + cp.ow1 >= p.Ncol) { cp.img1 = cp.img; cp.oh1 = cp.oh; cp.ow1 = cp.ow; }
    } else {
        lane_off = (uint32_t)(((int64_t)hh * 8 * p.ldx + col_ld) * 2);
    }
    // lane part of the packed block's addresses: its row, and the slots behind its half of a step
    // (8 dense columns of a 16-deep step, 16 of a 32-deep sparse step)
    const uint32_t a_off = (uint32_t)((jj * F::SLOTS + hh * F::FS * (SMF ? 2 : 1)) * 2);
    const uint32_t i_off = (uint32_t)(jj * F::WPR * 4);
    const uint32_t aw_sh = (uint32_t)hh * F::HB * (SMF ? 2 : 1);

    const int t_begin = p.row_ptr[bi], t_end = p.row_ptr[bi + 1];
    const int first = t_begin + (NWK > 1 ? wave : 0);
    const int cnt = first < t_end ? (t_end - first + NWK - 1) / NWK : 0;

    f32x16 acc[RT][NACC];
#pragma unroll
    for (int rt = 0; rt < RT; ++rt)
#pragma unroll
        for (int c = 0; c < NACC; ++c)
#pragma unroll
            for (int r = 0; r < 16; ++r) acc[rt][c][r] = 0.0f;

    xvec_t xr[PF][KS][8];
    uint32_t av[PF][RT][KS][F::VW];
    uint32_t aw[PF][RT][F::WPR];
    XCtx cx[PF];

    // ---- prologue: up to PF blocks in flight -------------------------------------------------
#pragma unroll
    for (int d = 0; d < PF; ++d) {
        if (d < cnt) {
            const int t = first + d * NWK;
            const int bj = p.col_idx[t];
            if constexpr (CONV != 0) cx[d] = BodyL::conv_ctx(p, cp, bj);
            else cx[d] = XCtx{lane_off, SEL_LO, SEL_HI, 0u};
#pragma unroll
            for (int ks = 0; ks < KS; ++ks) BodyL::load_x(xr[d][ks], p, cp, cx[d].off, cx[d].off2, bj, ks);
            BodyL::load_a(av[d], aw[d], p, a_off, i_off, t);
        }
    }

    // ---- steady state: every block of the group of PF has a successor PF blocks later ---------
    int i0 = 0;
    for (; i0 + 2 * PF <= cnt; i0 += PF) {
#pragma unroll
        for (int d = 0; d < PF; ++d)
            BodyP::run(acc, xr[d], av[d], aw[d], cx[d], p, cp, a_off, i_off, aw_sh, first + (i0 + d + PF) * NWK);
    }
    // ---- tail: at most 2*PF-1 blocks; the first PF-1 of them may still have a successor -------
#pragma unroll
    for (int e = 0; e < 2 * PF - 1; ++e) {
        const int i = i0 + e;
        if (i < cnt) {
            if (e < PF - 1 && i + PF < cnt)
                BodyP::run(acc, xr[e % PF], av[e % PF], aw[e % PF], cx[e % PF], p, cp, a_off, i_off, aw_sh,
                           first + (i + PF) * NWK);
            else
                BodyL::run(acc, xr[e % PF], av[e % PF], aw[e % PF], cx[e % PF], p, cp, a_off, i_off, aw_sh, 0);
        }
    }

    // ---- epilogue ---------------------------------------------------------------------------
    if constexpr (NWK == 1) {
        store_rows<B, WD, RT * 16, 1>(p, bi, hh, col0, col_ok, 0, [&](int pr, float (&v)[NACC]) __attribute__((always_inline)) {
#pragma unroll
            for (int c = 0; c < NACC; ++c) v[c] = acc[pr >> 4][c][pr & 15];
        });
    } else {
        // partial sums of the NWK waves -> LDS, then wave w adds up and stores every NWK-th row
        __shared__ float red[NWK][RT * 16][NACC][64];
#pragma unroll
        for (int rt = 0; rt < RT; ++rt)
#pragma unroll
            for (int r = 0; r < 16; ++r)
#pragma unroll
                for (int c = 0; c < NACC; ++c) red[wave][rt * 16 + r][c][lane] = acc[rt][c][r];
        __syncthreads();
        store_rows<B, WD, RT * 16 / NWK, NWK>(p, bi, hh, col0, col_ok, wave, [&](int pr, float (&v)[NACC]) __attribute__((always_inline)) {
#pragma unroll
            for (int c = 0; c < NACC; ++c) {
                float s = red[0][pr][c][lane];
#pragma unroll
                for (int w = 1; w < NWK; ++w) s += red[w][pr][c][lane];
                v[c] = s;
            }
        });
    }
}

template <int N, int M, int B, int WD, int NWK, int PF, int CONV, bool SMF = false>
hipError_t launch_reg_k(const SpmmArgs& a, hipStream_t st) {
    SpmmArgs p = a;
    constexpr int STRIPS = NWK > 1 ? 1 : 4;
    const int64_t span = (int64_t)STRIPS * 64 * WD;
    p.NT = (int)((a.Ncol + span - 1) / span);
    const int64_t groups = (int64_t)((p.NT + 7) / 8) * p.Sb * 8;
    if (groups > INT32_MAX) return hipErrorInvalidValue;
    const dim3 grd((unsigned)groups), blk(NWK > 1 ? 64 * NWK : 256);
    if (a.ev_start || a.ev_stop)
        hipExtLaunchKernelGGL((spmm_reg_kernel<N, M, B, WD, NWK, PF, CONV, SMF>), grd, blk, 0, st, a.ev_start, a.ev_stop, 0, p);
    else
        spmm_reg_kernel<N, M, B, WD, NWK, PF, CONV, SMF><<<grd, blk, 0, st>>>(p);
    return hipGetLastError();
}

template <int N, int M, int B, int WD, int NWK, int PF, int CONV>
hipError_t launch_reg(const SpmmArgs& a, hipStream_t st) {
    if constexpr (smf_pattern<N, M>() || (smf_flagged_pattern<N, M>() && CONV == 0)) {
        if (smf_wanted<N, M>(a)) return launch_reg_k<N, M, B, WD, NWK, PF, CONV, true>(a, st);
    }
    return launch_reg_k<N, M, B, WD, NWK, PF, CONV, false>(a, st);
}

// Launch shape: 0 = wide strips, waves own strips; 1 = narrow strips, waves own strips;
// 2 / 3 = narrow strips, 4 / 8 waves split the block list.  Conv mode has the narrow shapes only.
template <int N, int M, int B>
hipError_t launch_reg_shape(const SpmmArgs& a, int shape, hipStream_t st) {
    if (a.act != nullptr && a.conv_mode == 3) {
        switch (shape) {
            case 0:
            case 1: return launch_reg<N, M, B, 1, 1, 1, 3>(a, st);
            case 2: return launch_reg<N, M, B, 1, 4, 1, 3>(a, st);
            default: return launch_reg<N, M, B, 1, 8, 1, 3>(a, st);
        }
    }
    if (a.act != nullptr && a.conv_mode == 4) {
        switch (shape) {
            case 0:
            case 1: return launch_reg<N, M, B, 1, 1, 1, 4>(a, st);
            case 2: return launch_reg<N, M, B, 1, 4, 1, 4>(a, st);
            default: return launch_reg<N, M, B, 1, 8, 1, 4>(a, st);
        }
    }
    if (a.act != nullptr && a.conv_mode == 2) {
        switch (shape) {
            case 0:
            case 1: return launch_reg<N, M, B, 1, 1, 1, 2>(a, st);
            case 2: return launch_reg<N, M, B, 1, 4, 1, 2>(a, st);
            default: return launch_reg<N, M, B, 1, 8, 1, 2>(a, st);
        }
    }
    if (a.act != nullptr) {
        switch (shape) {
            case 0:
            case 1: return launch_reg<N, M, B, 1, 1, 1, 1>(a, st);
            case 2: return launch_reg<N, M, B, 1, 4, 1, 1>(a, st);
            default: return launch_reg<N, M, B, 1, 8, 1, 1>(a, st);
        }
    }
    switch (shape) {
        case 0: return launch_reg<N, M, B, 2, 1, 1, 0>(a, st);
        case 1: return launch_reg<N, M, B, 1, 1, 1, 0>(a, st);
        case 2: return launch_reg<N, M, B, 1, 4, 1, 0>(a, st);
        default: return launch_reg<N, M, B, 1, 8, 1, 0>(a, st);
    }
}

}  // namespace crisp
