// Convolution lowering: activation [C][batch][H][W] -> X[(a*kw+b)*C + c][(i*Ho+oh)*Wo+ow]
// (Sec. 3 "Notation": the conv becomes a matrix product).  Pure data movement, bound by the X write.
#include "crisp_internal.h"

namespace crisp {

struct Im2colArgs {
    int C, H, W, batch, kh, kw, stride, pad, Ho, Wo;
    int Ncol;
    int TG, CG;               // filter taps and channels handled by one thread
    double inv_Wo, inv_Ho;
    int64_t ldx, plane;       // row stride of X, elements of one channel plane (batch*H*W)
    const uint16_t* act;
    uint16_t* X;
};

// One thread owns two neighbouring columns (output positions) and writes them, one 4-byte store
// per row, for TG filter taps x CG channels: all rows of one tap share the source position, so
// the split of the column number into (image, oh, ow) and the border tests are done once per
// thread and tap, and the loop over channels is loads and stores only.  Neighbouring lanes own
// neighbouring column pairs: a wave reads and writes contiguous runs.
// PAIR: ldx is even, so the two columns of a thread are one aligned 32-bit word of X.
template <bool PAIR>
__global__ __launch_bounds__(256) void im2col_kernel(Im2colArgs p) {
    const int j0 = (blockIdx.x * 256 + threadIdx.x) * 2;
    if (j0 >= p.Ncol) return;
    const bool has1 = j0 + 1 < p.Ncol;
    // exact unsigned division through fp64 reciprocals (operands are below 2^31)
    int t = (int)((double)j0 * p.inv_Wo);
    t -= (t * p.Wo > j0);
    t += ((t + 1) * p.Wo <= j0);
    const int ow0 = j0 - t * p.Wo;
    int i0 = (int)((double)t * p.inv_Ho);
    i0 -= (i0 * p.Ho > t);
    i0 += ((i0 + 1) * p.Ho <= t);
    const int oh0 = t - i0 * p.Ho;
    int ow1 = ow0 + 1, oh1 = oh0, i1 = i0;
    if (ow1 == p.Wo) { ow1 = 0; ++oh1; }
    if (oh1 == p.Ho) { oh1 = 0; ++i1; }
    if (!has1) { ow1 = ow0; oh1 = oh0; i1 = i0; }

    const int tap_end = min(p.kh * p.kw, ((int)blockIdx.y + 1) * p.TG);
    const int c_begin = blockIdx.z * p.CG, c_end = min(p.C, c_begin + p.CG);
    for (int tap = blockIdx.y * p.TG; tap < tap_end; ++tap) {
        const int a = tap / p.kw, b = tap - a * p.kw;
        const int ih0 = oh0 * p.stride + a - p.pad, iw0 = ow0 * p.stride + b - p.pad;
        const int ih1 = oh1 * p.stride + a - p.pad, iw1 = ow1 * p.stride + b - p.pad;
        const bool v0 = (unsigned)ih0 < (unsigned)p.H && (unsigned)iw0 < (unsigned)p.W;
        const bool v1 = has1 && (unsigned)ih1 < (unsigned)p.H && (unsigned)iw1 < (unsigned)p.W;
        // positions outside the image read element 0 of the plane (always there) and are zeroed
        const int off0 = v0 ? (i0 * p.H + ih0) * p.W + iw0 : 0;
        const int off1 = v1 ? (i1 * p.H + ih1) * p.W + iw1 : 0;
        const uint16_t* src = p.act + (int64_t)c_begin * p.plane;
        uint16_t* dst = p.X + ((int64_t)tap * p.C + c_begin) * p.ldx + j0;
        // eight channels at a time: all loads first (X may not alias act, but the compiler cannot
        // know), then the stores, so that the loads are in flight together
        for (int c = c_begin; c < c_end; c += 8) {
            uint32_t e0[8], e1[8];
#pragma unroll
            for (int u = 0; u < 8; ++u) {
                const int64_t po = (int64_t)min(u, c_end - 1 - c) * p.plane;   // channels past the end re-read the last
                e0[u] = src[po + off0];
                e1[u] = src[po + off1];
            }
#pragma unroll
            for (int u = 0; u < 8; ++u) {
                if (c + u < c_end) {
                    const uint32_t a0 = v0 ? e0[u] : 0u, a1 = v1 ? e1[u] : 0u;
                    uint16_t* d = dst + (int64_t)u * p.ldx;
                    if (PAIR && has1) {
                        *reinterpret_cast<uint32_t*>(d) = a0 | (a1 << 16);
                    } else {
                        d[0] = (uint16_t)a0;
                        if (has1) d[1] = (uint16_t)a1;
                    }
                }
            }
            src += 8 * p.plane;
            dst += 8 * p.ldx;
        }
    }
}

hipError_t launch_im2col(const crisp_conv_desc& c, const uint16_t* act, uint16_t* X, int64_t ldx, hipStream_t st) {
    Im2colArgs p;
    p.C = c.C; p.H = c.H; p.W = c.W; p.batch = c.batch; p.kh = c.kh; p.kw = c.kw; p.stride = c.stride; p.pad = c.pad;
    p.Ho = (c.H + 2 * c.pad - c.kh) / c.stride + 1;
    p.Wo = (c.W + 2 * c.pad - c.kw) / c.stride + 1;
    p.Ncol = c.batch * p.Ho * p.Wo;
    p.inv_Wo = 1.0 / p.Wo;
    p.inv_Ho = 1.0 / p.Ho;
    p.ldx = ldx;
    p.plane = (int64_t)c.batch * c.H * c.W;
    p.act = act;
    p.X = X;
    // 16 to 32 rows per thread: whole channel runs of one tap, or for thin inputs (the first
    // layer's 3 channels) a few taps with all their channels
    p.CG = c.C < 16 ? c.C : 16;
    p.TG = c.C < 16 ? (16 + c.C - 1) / c.C : 1;
    const int taps = c.kh * c.kw;
    const int pairs = (p.Ncol + 1) / 2;
    const dim3 grd((pairs + 255) / 256, (taps + p.TG - 1) / p.TG, (c.C + p.CG - 1) / p.CG);
    if (grd.y > 65535 || grd.z > 65535) return hipErrorInvalidValue;
    if ((ldx & 1) == 0)
        im2col_kernel<true><<<grd, 256, 0, st>>>(p);
    else
        im2col_kernel<false><<<grd, 256, 0, st>>>(p);
    return hipGetLastError();
}

}  // namespace crisp

namespace crisp {

// Max pooling over kh x kw windows of a channel-major activation [C][batch][H][W] (the glue between
// the first convolution and the first residual stage of the ResNet workload; not part of the paper's
// method).  Positions outside the image do not take part.  bf16 values are compared as floats; the
// result is one of the inputs, so no rounding occurs.  One thread per output element; a window that
// lies wholly outside (cannot happen for pad < kernel size) would yield -inf.
// KH, KW > 0: window size known at compile time.  Every tap is then loaded from a clamped (always
// valid) position and masked afterwards, so the loop holds no branches and all loads of a thread
// are in flight together; with the bounds tests as branches every tap waits for the one before.
// KH == 0: any window size, taps outside the image skipped.
template <int KH, int KW>
__global__ __launch_bounds__(256) void maxpool_kernel(Im2colArgs p, uint32_t total) {
    const uint32_t e = blockIdx.x * 256u + threadIdx.x;
    if (e >= total) return;
    const uint32_t wo = (uint32_t)p.Wo, ho = (uint32_t)p.Ho;
    const int ow = (int)(e % wo);
    const uint32_t t = e / wo;
    const int oh = (int)(t % ho);
    const uint32_t plane = t / ho;              // c * batch + image
    const uint16_t* src = p.act + (int64_t)plane * p.H * p.W;
    float best = -__builtin_inff();
    uint32_t best_bits = 0xFF80u;               // -inf
    if constexpr (KH > 0) {
        uint32_t bits[KH][KW];
#pragma unroll
        for (int a = 0; a < KH; ++a) {
            const int ih = min(max(oh * p.stride + a - p.pad, 0), p.H - 1);
#pragma unroll
            for (int b = 0; b < KW; ++b) {
                const int iw = min(max(ow * p.stride + b - p.pad, 0), p.W - 1);
                bits[a][b] = src[ih * p.W + iw];
            }
        }
#pragma unroll
        for (int a = 0; a < KH; ++a) {
            const bool row_in = (unsigned)(oh * p.stride + a - p.pad) < (unsigned)p.H;
#pragma unroll
            for (int b = 0; b < KW; ++b) {
                const bool in = row_in && (unsigned)(ow * p.stride + b - p.pad) < (unsigned)p.W;
                const float v = in ? bf16_bits_to_float((uint16_t)bits[a][b]) : -__builtin_inff();
                const bool better = v > best;
                best = better ? v : best;
                best_bits = better ? bits[a][b] : best_bits;
            }
        }
    } else {
        for (int a = 0; a < p.kh; ++a) {
            const int ih = oh * p.stride + a - p.pad;
            if ((unsigned)ih >= (unsigned)p.H) continue;
            for (int b = 0; b < p.kw; ++b) {
                const int iw = ow * p.stride + b - p.pad;
                if ((unsigned)iw >= (unsigned)p.W) continue;
                const uint32_t bits = src[ih * p.W + iw];
                const float v = bf16_bits_to_float((uint16_t)bits);
                if (v > best) { best = v; best_bits = bits; }
            }
        }
    }
    p.X[e] = (uint16_t)best_bits;
}

// 3x3 window, stride 2, padding 1, W a multiple of 8 (the pooling layer of ResNet-like networks):
// a thread produces four neighbouring outputs from, per input row, one 16-byte load (input columns
// 8j .. 8j+7) and one 2-byte load (column 8j-1): 6 loads for 4 outputs instead of 36, which takes
// the kernel from the load units' instruction rate to the memory rate.  Same comparison order as
// maxpool_kernel (rows outer, columns inner, strict >), so the results are the same bits.
__global__ __launch_bounds__(256) void maxpool_3x3s2_kernel(Im2colArgs p, uint32_t quads) {
    typedef __attribute__((ext_vector_type(4))) uint32_t u32x4;
    const uint32_t e = blockIdx.x * 256u + threadIdx.x;
    if (e >= quads) return;
    const uint32_t wq = (uint32_t)p.Wo / 4u, ho = (uint32_t)p.Ho;
    const int j = (int)(e % wq);
    const uint32_t t = e / wq;
    const int oh = (int)(t % ho);
    const uint32_t plane = t / ho;              // c * batch + image
    const uint16_t* src = p.act + (int64_t)plane * p.H * p.W;
    u32x4 main_[3];
    uint32_t left[3];
#pragma unroll
    for (int a = 0; a < 3; ++a) {
        const int ih = min(max(oh * 2 + a - 1, 0), p.H - 1);
        main_[a] = *reinterpret_cast<const u32x4*>(src + ih * p.W + 8 * j);
        left[a] = src[ih * p.W + max(8 * j - 1, 0)];
    }
    float best[4];
    uint32_t best_bits[4];
#pragma unroll
    for (int k = 0; k < 4; ++k) { best[k] = -__builtin_inff(); best_bits[k] = 0xFF80u; }
#pragma unroll
    for (int a = 0; a < 3; ++a) {
        const bool row_in = (unsigned)(oh * 2 + a - 1) < (unsigned)p.H;
        uint32_t el[9];                         // columns 8j-1 .. 8j+7
        el[0] = left[a];
#pragma unroll
        for (int i = 0; i < 4; ++i) { el[1 + 2 * i] = main_[a][i] & 0xFFFFu; el[2 + 2 * i] = main_[a][i] >> 16; }
#pragma unroll
        for (int k = 0; k < 4; ++k) {
#pragma unroll
            for (int b = 0; b < 3; ++b) {
                const bool in = row_in && (k > 0 || b > 0 || j > 0);      // column 8j-1 of the first quad is padding
                const uint32_t bits = el[2 * k + b];
                const float v = in ? bf16_bits_to_float((uint16_t)bits) : -__builtin_inff();
                const bool better = v > best[k];
                best[k] = better ? v : best[k];
                best_bits[k] = better ? bits : best_bits[k];
            }
        }
    }
    typedef __attribute__((ext_vector_type(2))) uint32_t u32x2;
    const u32x2 out = {best_bits[0] | (best_bits[1] << 16), best_bits[2] | (best_bits[3] << 16)};
    *reinterpret_cast<u32x2*>(p.X + (size_t)e * 4u) = out;
}

hipError_t launch_maxpool(const crisp_conv_desc& c, const uint16_t* act, uint16_t* out, hipStream_t st) {
    Im2colArgs p = {};
    p.C = c.C; p.H = c.H; p.W = c.W; p.batch = c.batch; p.kh = c.kh; p.kw = c.kw; p.stride = c.stride; p.pad = c.pad;
    p.Ho = (c.H + 2 * c.pad - c.kh) / c.stride + 1;
    p.Wo = (c.W + 2 * c.pad - c.kw) / c.stride + 1;
    p.act = act;
    p.X = out;
    const int64_t total = (int64_t)c.C * c.batch * p.Ho * p.Wo;
    if (total <= 0 || total > (int64_t)0xFFFFFF00u) return hipErrorInvalidValue;
    if (c.kh == 3 && c.kw == 3 && c.stride == 2 && c.pad == 1 && c.W % 8 == 0 && (reinterpret_cast<uintptr_t>(act) & 15) == 0 &&
        (reinterpret_cast<uintptr_t>(out) & 7) == 0) {
        // (then Wo = W / 2 is a multiple of 4 and every row of act starts 16-byte aligned)
        const int64_t quads = total / 4;
        maxpool_3x3s2_kernel<<<(unsigned)((quads + 255) / 256), 256, 0, st>>>(p, (uint32_t)quads);
        return hipGetLastError();
    }
    const unsigned grid = (unsigned)((total + 255) / 256);
    if (c.kh == 3 && c.kw == 3) maxpool_kernel<3, 3><<<grid, 256, 0, st>>>(p, (uint32_t)total);
    else if (c.kh == 2 && c.kw == 2) maxpool_kernel<2, 2><<<grid, 256, 0, st>>>(p, (uint32_t)total);
    else maxpool_kernel<0, 0><<<grid, 256, 0, st>>>(p, (uint32_t)total);
    return hipGetLastError();
}

}  // namespace crisp
