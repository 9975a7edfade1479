// Convolution lowering: activation [C][batch][H][W] -> X[(a*kw+b)*C + c][(i*Ho+oh)*Wo+ow]
// (Sec. 3 "Notation": the conv becomes a matrix product).  Pure data movement, bound by the X write.
#include "crisp_internal.h"

namespace crisp {

struct Im2colArgs {
    int C, H, W, batch, kh, kw, stride, pad, Ho, Wo;
    int Ncol;
    double inv_Wo, inv_Ho;
    int64_t ldx;
    const uint16_t* act;
    uint16_t* X;
};

// One thread produces 8 consecutive columns of one X row (one 16-byte store when aligned).
// The row's tap (a, b) and channel c are uniform per workgroup; the thread splits its first
// column into (image, oh, ow) once and then walks the 8 columns with incremental updates, all
// in 32-bit arithmetic (a channel plane batch*H*W is below 2^31 elements).
template <bool VEC>
__global__ __launch_bounds__(256) void im2col_kernel(Im2colArgs p) {
    const int row = blockIdx.y;
    const int j0 = (blockIdx.x * 256 + threadIdx.x) * 8;
    if (j0 >= p.Ncol) return;
    const int c = row % p.C;
    const int tap = row / p.C;
    const int a = tap / p.kw, b = tap % p.kw;
    // exact unsigned division through fp64 reciprocals (operands are below 2^31)
    int t = (int)((double)j0 * p.inv_Wo);
    t -= (t * p.Wo > j0);
    t += ((t + 1) * p.Wo <= j0);
    int ow = j0 - t * p.Wo;
    int i = (int)((double)t * p.inv_Ho);
    i -= (i * p.Ho > t);
    i += ((i + 1) * p.Ho <= t);
    int oh = t - i * p.Ho;
    const uint16_t* plane = p.act + (size_t)c * p.batch * p.H * p.W;
    int ih = oh * p.stride + a - p.pad;
    int iw = ow * p.stride + b - p.pad;
    int rowbase = (i * p.H + ih) * p.W;
    // all 8 loads are issued unconditionally (index 0 stands in for positions outside the image)
    // so that they are in flight together; the selection happens after they return
    uint16_t v[8];
    bool in[8];
#pragma unroll
    for (int e = 0; e < 8; ++e) {
        in[e] = (j0 + e < p.Ncol) && ((unsigned)ih < (unsigned)p.H) && ((unsigned)iw < (unsigned)p.W);
        v[e] = plane[in[e] ? rowbase + iw : 0];
        iw += p.stride;
        if (++ow == p.Wo) {
            ow = 0;
            iw = b - p.pad;
            ih += p.stride;
            rowbase += p.stride * p.W;
            if (++oh == p.Ho) {
                oh = 0;
                ++i;
                ih = a - p.pad;
                rowbase = (i * p.H + ih) * p.W;
            }
        }
    }
#pragma unroll
    for (int e = 0; e < 8; ++e) v[e] = in[e] ? v[e] : (uint16_t)0;
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
    p.inv_Wo = 1.0 / p.Wo;
    p.inv_Ho = 1.0 / p.Ho;
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
