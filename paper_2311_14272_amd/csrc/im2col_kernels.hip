// Convolution lowering: activation [C][batch][H][W] -> X[(a*kw+b)*C + c][(i*Ho+oh)*Wo+ow]
// (Sec. 3 "Notation": the conv becomes a matrix product).  Pure data movement, bound by the X write.
#include "crisp_internal.h"

namespace crisp {

struct Im2colArgs {
    int C, H, W, batch, kh, kw, stride, pad, Ho, Wo;
    int Ncol;
    int64_t ldx;
    const uint16_t* act;
    uint16_t* X;
};

// One thread produces 8 consecutive columns of one X row (one 16-byte store when aligned).
template <bool VEC>
__global__ __launch_bounds__(256) void im2col_kernel(Im2colArgs p) {
    const int row = blockIdx.y;
    const int64_t j0 = ((int64_t)blockIdx.x * 256 + threadIdx.x) * 8;
    if (j0 >= p.Ncol) return;
    const int c = row % p.C;
    const int tap = row / p.C;
    const int a = tap / p.kw, b = tap % p.kw;
    int ow = (int)(j0 % p.Wo);
    int64_t rest = j0 / p.Wo;
    int oh = (int)(rest % p.Ho);
    int i = (int)(rest / p.Ho);
    const uint16_t* plane = p.act + (size_t)c * p.batch * p.H * p.W;
    uint16_t v[8];
#pragma unroll
    for (int e = 0; e < 8; ++e) {
        const int ih = oh * p.stride + a - p.pad, iw = ow * p.stride + b - p.pad;
        const bool inside = (j0 + e < p.Ncol) && ih >= 0 && ih < p.H && iw >= 0 && iw < p.W;
        v[e] = inside ? plane[((size_t)i * p.H + ih) * p.W + iw] : (uint16_t)0;
        if (++ow == p.Wo) {
            ow = 0;
            if (++oh == p.Ho) { oh = 0; ++i; }
        }
    }
    uint16_t* dst = p.X + (size_t)row * p.ldx + j0;
    if (VEC && j0 + 8 <= p.Ncol) {
        uint4 pk;
        pk.x = v[0] | ((uint32_t)v[1] << 16);
        pk.y = v[2] | ((uint32_t)v[3] << 16);
        pk.z = v[4] | ((uint32_t)v[5] << 16);
        pk.w = v[6] | ((uint32_t)v[7] << 16);
        *reinterpret_cast<uint4*>(dst) = pk;
    } else {
#pragma unroll
        for (int e = 0; e < 8; ++e)
            if (j0 + e < p.Ncol) dst[e] = v[e];
    }
}

hipError_t launch_im2col(const crisp_conv_desc& c, const uint16_t* act, uint16_t* X, int64_t ldx, hipStream_t st) {
    Im2colArgs p;
    p.C = c.C; p.H = c.H; p.W = c.W; p.batch = c.batch; p.kh = c.kh; p.kw = c.kw; p.stride = c.stride; p.pad = c.pad;
    p.Ho = (c.H + 2 * c.pad - c.kh) / c.stride + 1;
    p.Wo = (c.W + 2 * c.pad - c.kw) / c.stride + 1;
    p.Ncol = c.batch * p.Ho * p.Wo;
    p.ldx = ldx;
    p.act = act;
    p.X = X;
    const int K = c.kh * c.kw * c.C;
    const int chunks = (p.Ncol + 7) / 8;
    dim3 grd((chunks + 255) / 256, K);
    if (K > 65535) return hipErrorInvalidValue;
    if ((ldx & 7) == 0)
        im2col_kernel<true><<<grd, 256, 0, st>>>(p);
    else
        im2col_kernel<false><<<grd, 256, 0, st>>>(p);
    return hipGetLastError();
}

}  // namespace crisp
