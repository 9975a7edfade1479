// Generic hybrid-sparse product kernel (any n:m the format allows) and the launch dispatcher.
//
// The generic kernel expands each kept block in LDS: the compressed values and in-group
// positions are streamed with 16-byte coalesced loads into a staging area and expanded into a
// dense bf16 B x B tile, stored fragment-major so that each lane fetches its MFMA A operand
// with one conflict-free ds_read_b128; the four waves of a workgroup share the tile and each
// multiplies it with its own strip of X (loaded as in spmm_reg.h).  The patterns the paper and
// the benchmark workloads use have register-resident specialisations (spmm_reg.h), which the
// dispatcher prefers.
#include "conv_lds.h"

namespace crisp {

template <int WD>
__device__ __forceinline__ void xvec_unpack_t(const typename XVec<WD>::type& v, uint32_t (&d)[WD]) { xvec_unpack(v, d); }

// B: block edge (32 or 64).  WD: dwords a lane loads per X row (2*WD columns per lane, 64*WD
// columns per wave).  NW: waves per workgroup (workgroup strip = NW*64*WD columns).
template <int B, int WD, int NW>
__global__ __launch_bounds__(64 * NW) void spmm_expand_mfma_kernel(SpmmArgs p) {
    constexpr int RT = B / 32;            // 32-row MFMA tiles per block
    constexpr int KS = B / 16;            // 16-deep MFMA steps per block
    constexpr int NTHR = 64 * NW;
    constexpr int A_BYTES = B * B * 2;    // dense bf16 tile
    constexpr int STAGE_MAX = B * B * 2 + B * 6 * 4;           // values (n == m) + positions (8:8)
    constexpr int NCHUNK = (STAGE_MAX / 16 + NTHR - 1) / NTHR;  // 16-byte chunks per thread
    typedef typename XVec<WD>::type xvec_t;

    __shared__ __attribute__((aligned(16))) unsigned char lds_a[2 * A_BYTES];
    __shared__ __attribute__((aligned(16))) unsigned char lds_stage[STAGE_MAX];

    // Workgroup -> (block-row, column strip).  Consecutive workgroup ids go round-robin over the
    // 8 XCDs; all block-rows of one column strip are given ids that land on the same XCD next to
    // each other, so the X rows they share are served by that XCD's L2.
    const int id = blockIdx.x;
    const int xcd = id & 7;
    const int slot = id >> 3;
    const int bi = slot % p.Sb;
    const int nt = (slot / p.Sb) * 8 + xcd;
    if (nt >= p.NT) return;  // whole workgroup leaves before any barrier

    const int tid = threadIdx.x, wave = tid >> 6, lane = tid & 63;
    const int jj = lane & 31, hh = lane >> 5;
    const int64_t wave_col = ((int64_t)nt * NW + wave) * (64 * WD);
    const bool wave_on = wave_col < p.Ncol;
    const int64_t col0 = wave_col + jj * (2 * WD);
    const bool col_ok = col0 < p.Ncol;
    // Lanes past the last column read column 0 instead (in bounds); their results are never stored.
    const uint16_t* xlane = p.X + (col_ok ? col0 : 0) + (int64_t)hh * 8 * p.ldx;

    const int t_begin = p.row_ptr[bi], t_end = p.row_ptr[bi + 1];
    const int vbytes = B * p.slots * 2;             // compressed values of one block
    const int sbytes = vbytes + B * p.wpr * 4;      // + positions
    const int G = B / p.m;

    f32x16 acc[RT][2 * WD];
#pragma unroll
    for (int rt = 0; rt < RT; ++rt)
#pragma unroll
        for (int c = 0; c < 2 * WD; ++c)
#pragma unroll
            for (int r = 0; r < 16; ++r) acc[rt][c][r] = 0.0f;

    xvec_t xr[KS][8];
    u32x4 raw[NCHUNK];

    // ---- helpers -------------------------------------------------------------------------
    auto load_raw = [&](int t) {
#pragma unroll
        for (int i = 0; i < NCHUNK; ++i) {
            const int off = (tid + i * NTHR) * 16;
            if (off < sbytes) {
                const unsigned char* src = off < vbytes
                    ? reinterpret_cast<const unsigned char*>(p.vals) + (size_t)t * vbytes + off
                    : reinterpret_cast<const unsigned char*>(p.idxw) + (size_t)t * (sbytes - vbytes) + (off - vbytes);
                raw[i] = *reinterpret_cast<const u32x4*>(src);
            }
        }
    };
    auto store_raw = [&]() {
#pragma unroll
        for (int i = 0; i < NCHUNK; ++i) {
            const int off = (tid + i * NTHR) * 16;
            if (off < sbytes) *reinterpret_cast<u32x4*>(lds_stage + off) = raw[i];
        }
    };
    // Staging area -> dense tile in lds_a[buf], fragment-major:
    //   element (row, kl) lives at ((rt*KS + ks)*64 + h*32 + j)*8 + e  with row = rt*32 + j,
    //   kl = ks*16 + h*8 + e, i.e. exactly the 8 bf16 lane (h*32+j) feeds to MFMA step ks.
    auto expand = [&](int buf) {
        const uint16_t* sv = reinterpret_cast<const uint16_t*>(lds_stage);
        const uint32_t* si = reinterpret_cast<const uint32_t*>(lds_stage + vbytes);
        uint16_t* dst = reinterpret_cast<uint16_t*>(lds_a + buf * A_BYTES);
        for (int e = tid; e < B * G; e += NTHR) {
            const int r = e / G, g = e - r * G;
            uint32_t d[4] = {0u, 0u, 0u, 0u};
            for (int s = 0; s < p.n; ++s) {
                const int q = g * p.n + s;
                const int bit = q * p.w;
                const int wi = bit >> 5;
                uint64_t two = si[r * p.wpr + wi];
                if (wi + 1 < p.wpr) two |= (uint64_t)si[r * p.wpr + wi + 1] << 32;
                const uint32_t pos = (uint32_t)(two >> (bit & 31)) & (uint32_t)(p.m - 1);
                const uint32_t v = (uint32_t)sv[r * p.slots + q] << ((pos & 1u) * 16u);
                const uint32_t dw = pos >> 1;
#pragma unroll
                for (int x = 0; x < 4; ++x) d[x] |= (dw == (uint32_t)x) ? v : 0u;
            }
            const int kl = g * p.m;
            const int rt = r >> 5, j = r & 31, ks = kl >> 4, h = (kl >> 3) & 1, e8 = kl & 7;
            uint16_t* o = dst + ((((rt * KS + ks) * 64) + h * 32 + j) * 8 + e8);
            if (p.m == 4) {
                *reinterpret_cast<uint2*>(o) = make_uint2(d[0], d[1]);
            } else {
                u32x4 v4 = {d[0], d[1], d[2], d[3]};
                *reinterpret_cast<u32x4*>(o) = v4;
            }
        }
    };
    // X rows of block column bj, MFMA step ks: lane (hh, jj) takes rows bj*B + ks*16 + hh*8 + i.
    auto load_x = [&](xvec_t (&dst)[8], int bj, int ks) {
        const int kbase = bj * B + ks * 16;
        const uint16_t* src = xlane + (int64_t)kbase * p.ldx;
        if (kbase + 16 <= p.K) {
#pragma unroll
            for (int i = 0; i < 8; ++i) dst[i] = *reinterpret_cast<const xvec_t*>(src + (int64_t)i * p.ldx);
        } else {
            // ragged last block column: rows >= K do not exist; they must read as zero because
            // the matching weights are zero padding and 0 * garbage could be NaN
#pragma unroll
            for (int i = 0; i < 8; ++i) {
                xvec_t z = {};
                if (kbase + hh * 8 + i < p.K) z = *reinterpret_cast<const xvec_t*>(src + (int64_t)i * p.ldx);
                dst[i] = z;
            }
        }
    };

    // ---- prologue ------------------------------------------------------------------------
    if (t_begin < t_end) {
        load_raw(t_begin);
        if (wave_on) {
            const int bj = p.col_idx[t_begin];
#pragma unroll
            for (int ks = 0; ks < KS; ++ks) load_x(xr[ks], bj, ks);
        }
        store_raw();
        __syncthreads();
        expand(0);
        __syncthreads();
    }

    // ---- walk the kept blocks of this block-row -------------------------------------------
    for (int t = t_begin; t < t_end; ++t) {
        const int buf = (t - t_begin) & 1;
        const bool has_next = t + 1 < t_end;
        const int bj_next = has_next ? p.col_idx[t + 1] : 0;
        if (has_next) load_raw(t + 1);
        if (wave_on) {
            const unsigned char* abase = lds_a + buf * A_BYTES + lane * 16;
#pragma unroll
            for (int ks = 0; ks < KS; ++ks) {
                // 8 rows x 2*WD columns of 16-bit halves -> 2*WD operands of 8 K-values each
                uint32_t xd[8][WD];
#pragma unroll
                for (int i = 0; i < 8; ++i) xvec_unpack(xr[ks][i], xd[i]);
                bf16x8 bfrag[2 * WD];
#pragma unroll
                for (int pdw = 0; pdw < WD; ++pdw) {
                    u32x4 lo, hi;
#pragma unroll
                    for (int q = 0; q < 4; ++q) {
                        const uint32_t r0 = xd[2 * q][pdw], r1 = xd[2 * q + 1][pdw];
                        lo[q] = (r0 & 0xFFFFu) | (r1 << 16);
                        hi[q] = (r0 >> 16) | (r1 & 0xFFFF0000u);
                    }
                    bfrag[2 * pdw] = __builtin_bit_cast(bf16x8, lo);
                    bfrag[2 * pdw + 1] = __builtin_bit_cast(bf16x8, hi);
                }
                if (has_next) load_x(xr[ks], bj_next, ks);
#pragma unroll
                for (int rt = 0; rt < RT; ++rt) {
                    const u32x4 av = *reinterpret_cast<const u32x4*>(abase + (rt * KS + ks) * 1024);
                    const bf16x8 afrag = __builtin_bit_cast(bf16x8, av);
#pragma unroll
                    for (int c = 0; c < 2 * WD; ++c)
                        acc[rt][c] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(afrag, bfrag[c], acc[rt][c], 0, 0, 0);
                }
            }
        }
        if (has_next) store_raw();
        __syncthreads();
        if (has_next) expand(buf ^ 1);
        __syncthreads();
    }

    // ---- epilogue: accumulator register r of a 32x32 tile is row 8*(r/4) + 4*hh + r%4,
    //      column jj; the 2*WD accumulators of a lane are consecutive columns ---------------
    if (!wave_on || !col_ok) return;
    const bool full = col0 + 2 * WD <= p.Ncol;
#pragma unroll
    for (int rt = 0; rt < RT; ++rt)
#pragma unroll
        for (int r = 0; r < 16; ++r) {
            const int row = bi * B + rt * 32 + 8 * (r >> 2) + 4 * hh + (r & 3);
            if (row >= p.S) continue;
            float v[2 * WD];
#pragma unroll
            for (int c = 0; c < 2 * WD; ++c) v[c] = acc[rt][c][r];
            if (full) {
                apply_epilogue<2 * WD>(p, row, col0, true, v);
            } else {
#pragma unroll
                for (int c = 0; c < 2 * WD; ++c) {
                    float one[1] = {v[c]};
                    apply_epilogue<1>(p, row, col0 + c, col0 + c < p.Ncol, one);
                    v[c] = one[0];
                }
            }
            if (p.y_bf16) {
                uint16_t* y = reinterpret_cast<uint16_t*>(p.Y) + (int64_t)row * p.ldy + col0;
                if (full) {
                    uint32_t pk[WD];
#pragma unroll
                    for (int c = 0; c < WD; ++c)
                        pk[c] = float_to_bf16_rne(v[2 * c]) | ((uint32_t)float_to_bf16_rne(v[2 * c + 1]) << 16);
                    if (WD == 1) *reinterpret_cast<uint32_t*>(y) = pk[0];
                    else *reinterpret_cast<uint2*>(y) = make_uint2(pk[0], pk[WD - 1]);
                } else {
#pragma unroll
                    for (int c = 0; c < 2 * WD; ++c)
                        if (col0 + c < p.Ncol) y[c] = float_to_bf16_rne(v[c]);
                }
            } else {
                float* y = reinterpret_cast<float*>(p.Y) + (int64_t)row * p.ldy + col0;
                if (full) {
                    if (WD == 1) *reinterpret_cast<float2*>(y) = make_float2(v[0], v[1]);
                    else *reinterpret_cast<float4*>(y) = make_float4(v[0], v[1], v[2 * WD - 2], v[2 * WD - 1]);
                } else {
#pragma unroll
                    for (int c = 0; c < 2 * WD; ++c)
                        if (col0 + c < p.Ncol) y[c] = v[c];
                }
            }
        }
}

template <int B, int WD, int NW>
static hipError_t launch_one(const SpmmArgs& a, hipStream_t st) {
    SpmmArgs p = a;
    const int64_t strip = (int64_t)NW * 64 * WD;
    p.NT = (int)((a.Ncol + strip - 1) / strip);
    const int64_t groups = (int64_t)((p.NT + 7) / 8) * p.Sb * 8;
    if (groups > INT32_MAX) return hipErrorInvalidValue;
    if (a.ev_start || a.ev_stop)
        hipExtLaunchKernelGGL((spmm_expand_mfma_kernel<B, WD, NW>), dim3((unsigned)groups), dim3(64 * NW), 0, st,
                              a.ev_start, a.ev_stop, 0, p);
    else
        spmm_expand_mfma_kernel<B, WD, NW><<<dim3((unsigned)groups), dim3(64 * NW), 0, st>>>(p);
    return hipGetLastError();
}

// 16 x 16 blocks (the paper's smallest block size).  One wave per (block-row, strip of 64 output
// columns); lane (j = lane % 16, q = lane / 16).  v_mfma_f32_16x16x16_bf16: A operand = row j of the
// block, columns 4q..4q+3; B operand = one X column, K-rows 4q..4q+3; result = column j, rows
// 4q..4q+3.  The lane loads 4 consecutive X columns (8 bytes) of each of its 4 K-rows and
// transposes 16-bit halves as in the larger kernels, so its 4 accumulators are 4 consecutive
// output columns.  Any n:m, any K and Ncol (rows past K and columns past Ncol are predicated).
typedef __attribute__((ext_vector_type(4))) short s16x4;
typedef __attribute__((ext_vector_type(4))) float f32x4;

__global__ __launch_bounds__(256) void spmm_b16_kernel(SpmmArgs p) {
    const int id = blockIdx.x;
    const int xcd = id & 7, slot = id >> 3;
    const int bi = slot % p.Sb;
    const int nt = (slot / p.Sb) * 8 + xcd;
    if (nt >= p.NT) return;
    const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
    const int j = lane & 15, q = lane >> 4;
    const int64_t wave_col = ((int64_t)nt * 4 + wave) * 64;
    if (wave_col >= p.Ncol) return;
    const int64_t col0 = wave_col + j * 4;
    const bool col_ok = col0 < p.Ncol;          // chunk starts inside; ldx % 8 == 0 keeps the 8-byte load in the row
    const uint16_t* xcol = p.X + (col_ok ? col0 : 0);
    const int t_begin = p.row_ptr[bi], t_end = p.row_ptr[bi + 1];
    f32x4 acc[4];
#pragma unroll
    for (int c = 0; c < 4; ++c) acc[c] = f32x4{0.f, 0.f, 0.f, 0.f};
    for (int t = t_begin; t < t_end; ++t) {
        const int bj = p.col_idx[t];
        // X: rows bj*16 + 4q + i; rows at or past K read as zero
        uint2 xr[4];
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            const int k = bj * 16 + 4 * q + i;
            const int kc = min(k, p.K - 1);
            const uint2 v = *reinterpret_cast<const uint2*>(xcol + (int64_t)kc * p.ldx);
            xr[i] = (k < p.K) ? v : make_uint2(0u, 0u);
        }
        // A: row j of block t, columns 4q..4q+3, expanded from the packed slots
        const size_t brow = (size_t)t * 16 + j;
        const uint16_t* vrow = p.vals + brow * p.slots;
        const uint32_t* irow = p.idxw + brow * p.wpr;
        uint64_t stream = irow[0];
        if (p.wpr > 1) stream |= (uint64_t)irow[1] << 32;
        const int g = (p.m == 4) ? q : (q >> 1);        // group of this lane's 4 columns
        const uint32_t half_sel = (uint32_t)(q & 1);     // m == 8: which half of the group
        uint32_t a0 = 0u, a1 = 0u;
        for (int s = 0; s < p.n; ++s) {
            const int sl = g * p.n + s;
            const uint32_t pos = (uint32_t)(stream >> (sl * p.w)) & (uint32_t)(p.m - 1);
            const bool mine = (p.m == 4) || ((pos >> 2) == half_sel);
            const uint32_t pl = pos & 3u;
            const uint32_t v = mine ? ((uint32_t)vrow[sl] << ((pl & 1u) * 16u)) : 0u;
            a0 |= (pl < 2u) ? v : 0u;
            a1 |= (pl < 2u) ? 0u : v;
        }
        const uint2 av = make_uint2(a0, a1);
        const s16x4 afrag = __builtin_bit_cast(s16x4, av);
#pragma unroll
        for (int pd = 0; pd < 2; ++pd) {
            const uint32_t r0 = pd ? xr[0].y : xr[0].x, r1 = pd ? xr[1].y : xr[1].x;
            const uint32_t r2 = pd ? xr[2].y : xr[2].x, r3 = pd ? xr[3].y : xr[3].x;
            const uint2 lo = make_uint2(__builtin_amdgcn_perm(r1, r0, SEL_LO), __builtin_amdgcn_perm(r3, r2, SEL_LO));
            const uint2 hi = make_uint2(__builtin_amdgcn_perm(r1, r0, SEL_HI), __builtin_amdgcn_perm(r3, r2, SEL_HI));
            acc[2 * pd] = __builtin_amdgcn_mfma_f32_16x16x16bf16_1k(afrag, __builtin_bit_cast(s16x4, lo), acc[2 * pd], 0, 0, 0);
            acc[2 * pd + 1] = __builtin_amdgcn_mfma_f32_16x16x16bf16_1k(afrag, __builtin_bit_cast(s16x4, hi), acc[2 * pd + 1], 0, 0, 0);
        }
    }
    if (!col_ok) return;
#pragma unroll
    for (int r = 0; r < 4; ++r) {
        const int row = bi * 16 + 4 * q + r;
        if (row >= p.S) continue;
#pragma unroll
        for (int c = 0; c < 4; ++c) {
            if (col0 + c >= p.Ncol) continue;
            float one[1] = {acc[c][r]};
            apply_epilogue<1>(p, row, col0 + c, true, one);
            const float v = one[0];
            if (p.y_bf16) reinterpret_cast<uint16_t*>(p.Y)[(int64_t)row * p.ldy + col0 + c] = float_to_bf16_rne(v);
            else reinterpret_cast<float*>(p.Y)[(int64_t)row * p.ldy + col0 + c] = v;
        }
    }
}

static hipError_t launch_b16(const SpmmArgs& a, hipStream_t st) {
    SpmmArgs p = a;
    p.NT = (int)((a.Ncol + 255) / 256);
    const int64_t groups = (int64_t)((p.NT + 7) / 8) * p.Sb * 8;
    if (groups > INT32_MAX) return hipErrorInvalidValue;
    if (a.ev_start || a.ev_stop)
        hipExtLaunchKernelGGL(spmm_b16_kernel, dim3((unsigned)groups), dim3(256), 0, st, a.ev_start, a.ev_stop, 0, p);
    else
        spmm_b16_kernel<<<dim3((unsigned)groups), dim3(256), 0, st>>>(p);
    return hipGetLastError();
}

int lds_capacity(int B);
hipError_t launch_spmm_lds(const SpmmArgs& a, int B, int max_blocks, bool wide, hipStream_t st);
int lds_smf_capacity();
hipError_t launch_spmm_lds_smf(const SpmmArgs& a, int max_blocks, int variant, hipStream_t st);

template <> hipError_t launch_reg_nm<1, 4>(const SpmmArgs&, int, int, hipStream_t);
template <> hipError_t launch_reg_nm<2, 4>(const SpmmArgs&, int, int, hipStream_t);
template <> hipError_t launch_reg_nm<3, 4>(const SpmmArgs&, int, int, hipStream_t);
template <> hipError_t launch_reg_nm<4, 4>(const SpmmArgs&, int, int, hipStream_t);
template <> hipError_t launch_reg_nm<1, 8>(const SpmmArgs&, int, int, hipStream_t);
template <> hipError_t launch_reg_nm<2, 8>(const SpmmArgs&, int, int, hipStream_t);
template <> hipError_t launch_reg_nm<4, 8>(const SpmmArgs&, int, int, hipStream_t);
template <> hipError_t launch_reg_nm<8, 8>(const SpmmArgs&, int, int, hipStream_t);
template <> hipError_t launch_conv_patch_nm<1, 4>(const SpmmArgs&, const ConvPatchSched&, int, hipStream_t);
template <> hipError_t launch_conv_patch_nm<2, 4>(const SpmmArgs&, const ConvPatchSched&, int, hipStream_t);
template <> hipError_t launch_conv_patch_nm<3, 4>(const SpmmArgs&, const ConvPatchSched&, int, hipStream_t);
template <> hipError_t launch_conv_patch_nm<4, 4>(const SpmmArgs&, const ConvPatchSched&, int, hipStream_t);
template <> hipError_t launch_conv_patch_nm<1, 8>(const SpmmArgs&, const ConvPatchSched&, int, hipStream_t);
template <> hipError_t launch_conv_patch_nm<2, 8>(const SpmmArgs&, const ConvPatchSched&, int, hipStream_t);
template <> hipError_t launch_conv_patch_nm<4, 8>(const SpmmArgs&, const ConvPatchSched&, int, hipStream_t);
template <> hipError_t launch_conv_patch_nm<8, 8>(const SpmmArgs&, const ConvPatchSched&, int, hipStream_t);
template <> hipError_t launch_k8_nm<1, 4>(const SpmmArgs&, int, hipStream_t);
template <> hipError_t launch_k8_nm<2, 4>(const SpmmArgs&, int, hipStream_t);
template <> hipError_t launch_k8_nm<3, 4>(const SpmmArgs&, int, hipStream_t);
template <> hipError_t launch_k8_nm<4, 4>(const SpmmArgs&, int, hipStream_t);
template <> hipError_t launch_k8_nm<1, 8>(const SpmmArgs&, int, hipStream_t);
template <> hipError_t launch_k8_nm<2, 8>(const SpmmArgs&, int, hipStream_t);
template <> hipError_t launch_k8_nm<4, 8>(const SpmmArgs&, int, hipStream_t);
template <> hipError_t launch_k8_nm<8, 8>(const SpmmArgs&, int, hipStream_t);
template <> hipError_t launch_balanced_nm<1, 4>(const SpmmArgs&, int, hipStream_t);
template <> hipError_t launch_balanced_nm<2, 4>(const SpmmArgs&, int, hipStream_t);
template <> hipError_t launch_balanced_nm<3, 4>(const SpmmArgs&, int, hipStream_t);
template <> hipError_t launch_balanced_nm<4, 4>(const SpmmArgs&, int, hipStream_t);
template <> hipError_t launch_balanced_nm<1, 8>(const SpmmArgs&, int, hipStream_t);
template <> hipError_t launch_balanced_nm<2, 8>(const SpmmArgs&, int, hipStream_t);
template <> hipError_t launch_balanced_nm<4, 8>(const SpmmArgs&, int, hipStream_t);
template <> hipError_t launch_balanced_nm<8, 8>(const SpmmArgs&, int, hipStream_t);
template <> hipError_t launch_conv_lds_nm<1, 4>(const SpmmArgs&, const ConvLdsSched&, int, hipStream_t);
template <> hipError_t launch_conv_lds_nm<2, 4>(const SpmmArgs&, const ConvLdsSched&, int, hipStream_t);
template <> hipError_t launch_conv_lds_nm<3, 4>(const SpmmArgs&, const ConvLdsSched&, int, hipStream_t);
template <> hipError_t launch_conv_lds_nm<4, 4>(const SpmmArgs&, const ConvLdsSched&, int, hipStream_t);
template <> hipError_t launch_conv_lds_nm<1, 8>(const SpmmArgs&, const ConvLdsSched&, int, hipStream_t);
template <> hipError_t launch_conv_lds_nm<2, 8>(const SpmmArgs&, const ConvLdsSched&, int, hipStream_t);
template <> hipError_t launch_conv_lds_nm<4, 8>(const SpmmArgs&, const ConvLdsSched&, int, hipStream_t);
template <> hipError_t launch_conv_lds_nm<8, 8>(const SpmmArgs&, const ConvLdsSched&, int, hipStream_t);

// Launch shape of the register-expansion kernels from the problem size (thresholds from sweeps
// over the layer shapes of ResNet-50 at batch 256 and the small single-layer workloads):
// wide strips once they give every SIMD work or the block-rows are long (the expansion of A is
// shared by twice the columns); otherwise narrow strips; and when even those are few, 4 or 8
// waves split each block-row's list so that enough loads are in flight to cover the latency.
static int pick_shape(const Geometry& g, int64_t Ncol, int blocks_per_row, bool smf);

// Whether the LDS-staged convolution is the faster choice (measured on 3x3 layers of the ResNet-50
// shapes, all patterns, block densities 0.25 .. 1): with at least half of the blocks kept the patch
// is reused often enough in every shape (1.1-1.4x over the register kernels); below that only where
// a staged patch still serves about six kept blocks, the tiles are small (output width <= 28) and
// one group of block-rows covers the layer (1.1-1.7x there, 0.7-0.9x elsewhere), and the grid
// gives every compute unit a workgroup.
static bool conv_lds_pays(const ConvLdsSched& s, int Sb, double density, int batch, int Wo) {
    if (s.taps <= 1 || Sb < 2 || !(density <= 1.0)) return false;
    if (density >= 0.5) return true;
    const double blocks_per_patch = s.RG * density * s.taps;
    const int64_t wgs = (int64_t)batch * s.tiles_per_img * s.row_groups;
    return blocks_per_patch >= 6.0 && Sb <= 4 && Wo <= 28 && wgs >= 256;
}

static int pick_shape(const Geometry& g, int64_t Ncol, int blocks_per_row, bool smf) {
    const int64_t wide = (int64_t)g.Sb * ((Ncol + 127) / 128);
    const int64_t narrow = (int64_t)g.Sb * ((Ncol + 63) / 64);
    if (smf) {
        // sparse matrix-core instantiations: no (or little) expansion work to share between
        // columns, so narrow strips (more waves) win more often, most clearly for 2:4
        const bool heavy = 8 * g.n / g.m >= 4;   // 2:4
        if (blocks_per_row <= 2) return wide >= 2048 ? 0 : 1;
        if (narrow >= 1024) return ((!heavy && blocks_per_row >= 7) || blocks_per_row >= 20) ? 0 : 1;
        // few tiles and long rows: four waves split a tile's block list (32x32 blocks only when the tiles
        // are very few: c1 with 392 tiles 9.5 vs 11.7 us, c4a with 490 tiles 14.7 vs 12.2 us)
        return (blocks_per_row >= 8 && (g.B == 64 || narrow < 448)) ? 2 : 1;
    }
    // 4:8 expands through a selector table (a handful of instructions per operand): as with the sparse
    // instruction there is little to share between columns, and narrow strips win from two blocks per row on
    // (five 1x1 layers of ResNet-50 at batch 256: 44-86 us against 52-94 us; equal or slower for single blocks)
    if (g.n == 4 && g.m == 8 && blocks_per_row >= 2 && narrow >= 1024) return 1;
    if (wide >= 4096) return 0;
    if (blocks_per_row >= 8 && wide >= 512) return 0;
    if (narrow >= 3072 || blocks_per_row < 3) return 1;
    if (wide >= 512) return 0;
    // the 8-way split keeps 8 partial tiles in LDS (128 KB for 64-row blocks: one workgroup per
    // CU), so it only pays when all workgroups are resident at once
    const int64_t resident8 = g.B == 64 ? 256 : 512;
    if (blocks_per_row >= 8 && narrow <= resident8) return 3;
    return 2;
}

// Whether the LDS-resident kernels are expected to beat the register-expansion ones: the rows
// must fit, there must be several strips per wave to amortise the expansion, and the per-block
// expansion in registers must be expensive (4 packed slots per operand: 2:4, 4:8, ...) or
// repeated often (long block-rows).
static bool prefer_lds(const Geometry& g, int64_t Ncol, int blocks_per_row) {
    if (g.B != 64 || blocks_per_row > lds_capacity(g.B)) return false;
    // patterns that feed the sparse matrix core need no (or little) expansion: the register kernels, or
    // residency in that operand form (prefer_lds_smf), are faster
    if (g.n <= 2 || g.two_of_four) return false;
    const int64_t narrow = (int64_t)g.Sb * ((Ncol + 63) / 64);
    const int slots_per_operand = (8 / g.m) * g.n;
    // (4:8 in registers goes through the selector table: residency only pays on long rows there -- 12 blocks:
    // 54 against 57 us, 9 blocks: 49 against 47 us, 3 blocks: 48-95 against 44-86 us)
    // (single blocks: the wide LDS-resident kernel, 76 against 81 us)
    if (g.n == 4 && g.m == 8) return narrow >= 2048 && (blocks_per_row >= 10 || blocks_per_row <= 1);
    return narrow >= 2048 && (slots_per_operand >= 4 || blocks_per_row >= 6);
}

// Block-rows resident in LDS as sparse matrix-core operands: a wave's loop then holds no requests for packed
// slices at all.  Measured on the 1x1 layers of ResNet-50 at batch 256 and on the 512 x 4608 x 50176 2:8 layer
// against the register kernels: 1.03-1.12x from six blocks per block-row on (1.15x on the latter, 18 blocks:
// 117 vs 132-138 us), 0.85-1.0x for rows of one to three blocks (the expansion is not amortised); always the
// 30-tile instantiation (one workgroup of eight waves per compute unit), which beat the 15-tile one (two
// workgroups of four) on every layer with six or more blocks.
static bool prefer_lds_smf(const Geometry& g, int64_t Ncol, int blocks_per_row) {
    if (g.B != 64 || !(g.n <= 2 || g.two_of_four) || blocks_per_row < 6 || blocks_per_row > lds_smf_capacity()) return false;
    const int64_t narrow = (int64_t)g.Sb * ((Ncol + 63) / 64);
    return narrow >= 2048;
}

// Geometry of an implicitly lowered convolution as the product kernels want it (everything but the
// activation pointer).
static void fill_conv_args(SpmmArgs& a, const Geometry& g, const crisp_conv_desc& conv) {
    a.C = conv.C; a.H = conv.H; a.W = conv.W; a.kw = conv.kw; a.pad = conv.pad; a.stride = conv.stride;
    a.Ho = (conv.H + 2 * conv.pad - conv.kh) / conv.stride + 1;
    a.Wo = (conv.W + 2 * conv.pad - conv.kw) / conv.stride + 1;
    // a lane's two columns from one dword when their sources are neighbours in memory (stride 1 and either an
    // even output width, so that a pair never leaves its output row, or padding (k - 1) / 2 in both directions,
    // so that consecutive output positions read consecutive input elements even across rows and images), else
    // column by column
    const bool same_pad = conv.kh == 2 * conv.pad + 1 && conv.kw == 2 * conv.pad + 1;
    a.conv_mode = (conv.stride == 1 && ((a.Wo & 1) == 0 || same_pad) && conv.W >= 2 && a.Wo >= 2) ? 1 : 2;
    if (conv.kh == 1 && conv.kw == 1 && conv.stride == 2 && conv.pad == 0 && (conv.W & 1) == 0 && (a.Wo & 1) == 0)
        a.conv_mode = 4;                       // strided 1x1: both columns from one 8-byte piece of the input row
    if (conv.C % g.B != 0) a.conv_mode = 3;   // block columns span filter taps: every K-row on its own
    a.plane = (int64_t)conv.batch * conv.H * conv.W;
    a.act_bytes = a.conv_mode == 3 ? (uint32_t)((int64_t)conv.C * a.plane * 2) : 0u;
    a.inv_C = 1.0f / (float)conv.C;
    a.inv_cpb = conv.C >= g.B ? 1.0f / (float)(conv.C / g.B) : 1.0f;
    a.inv_kw = 1.0f / (float)conv.kw;
    a.inv_Wo = 1.0 / a.Wo;
    a.inv_Ho = 1.0 / a.Ho;
}

// Where the kernel that keeps a strip of X in LDS for all block-rows is the automatic choice (patterns with
// n <= 2; the caller checks that and xlds_covers).
static bool xlds_pays(int Sb, int Kb, int64_t Ncol, bool strided_1x1) {
    return Kb >= 2 && Sb >= (strided_1x1 ? 8 : 16) && Ncol >= 8192;
}

// Whether launch_spmm, left to its own choice, runs this strided 1 x 1 convolution in that kernel (asked by the
// callers that choose between the fused lowering and a materialised X).
bool xlds_conv_would_run(const Geometry& g, const crisp_conv_desc& conv, int64_t Ncol) {
    const int64_t Wo = ((int64_t)conv.W + 2 * conv.pad - conv.kw) / conv.stride + 1;
    const bool strided_1x1 = conv.kh == 1 && conv.kw == 1 && conv.stride == 2 && conv.pad == 0 && (conv.W & 1) == 0 &&
                             (Wo & 1) == 0 && conv.C % 64 == 0;
    const bool sparse_ok = g.n <= 2 || g.two_of_four, dense48 = g.n == 4 && g.m == 8;
    return strided_1x1 && g.B == 64 && g.K <= XLDS_MAX_KB * 64 && (Ncol % 4) == 0 &&
           ((sparse_ok && xlds_pays(g.Sb, g.Kb, Ncol, true)) || (dense48 && xlds_pays(g.Sb, g.Kb, Ncol, false)));
}

// Whether launch_spmm, left to its own choice, runs this convolution in the kernel that stages the
// input patch in LDS (the callers that choose between the fused lowering and a materialised X ask).
bool conv_lds_would_run(const Geometry& g, double density_hint, const crisp_conv_desc& conv, int64_t Ncol) {
    if (g.B == 16) return false;
    SpmmArgs a = {};
    a.S = g.S; a.K = g.K; a.Sb = g.Sb; a.Ncol = Ncol;
    a.act = reinterpret_cast<const uint16_t*>(&a);      // any non-null value: never dereferenced on the host
    fill_conv_args(a, g, conv);
    ConvLdsSched cs;
    return (Ncol % 4) == 0 && conv_lds_plan(a, g.B, conv.kh, &cs) && conv_lds_pays(cs, g.Sb, density_hint, conv.batch, a.Wo);
}

hipError_t launch_spmm(const Geometry& g, double density_hint, bool uniform_rows, int force_shape, const int32_t* row_ptr,
                       const int32_t* col_idx, const uint16_t* vals, const uint32_t* idxw, const uint16_t* X,
                       const crisp_conv_desc* conv, int64_t Ncol, int64_t ldx, void* Y, int64_t ldy, int y_dtype,
                       const crisp_epilogue* ep, hipEvent_t ev_start, hipEvent_t ev_stop, hipStream_t st, int32_t* kernel_code,
                       int x_layout) {
    // what ran, for callers that ask: family | shape << 8 | conv_mode << 16 | sparse << 24
    auto report = [&](int family, int shape, int conv_mode, int sparse) {
        if (kernel_code) *kernel_code = family | (shape << 8) | (conv_mode << 16) | (sparse << 24);
    };
    SpmmArgs a = {};
    a.ev_start = ev_start; a.ev_stop = ev_stop;
    a.S = g.S; a.K = g.K; a.n = g.n; a.m = g.m; a.w = g.w; a.slots = g.slots; a.wpr = g.wpr;
    a.Sb = g.Sb; a.NT = 0; a.Ncol = Ncol; a.ldx = ldx; a.ldy = ldy;
    a.row_ptr = row_ptr; a.col_idx = col_idx; a.vals = vals; a.idxw = idxw; a.X = X; a.Y = Y;
    a.y_bf16 = (y_dtype == CRISP_Y_BF16);
    // patterns that may go to the sparse matrix-core instruction: at most two kept per group, or 4:8 whose pack
    // the caller asserts to hold at most two values per aligned four (kernel families for plain X only)
    const bool smf_ok = g.n <= 2 || g.two_of_four;
    a.two_of_four = g.two_of_four;
    if (ep && (ep->scale || ep->bias || ep->residual || ep->relu)) {
        a.ep_on = 1; a.ep_relu = ep->relu ? 1 : 0;
        a.ep_scale = ep->scale; a.ep_bias = ep->bias; a.ep_res = ep->residual; a.ep_ldr = ep->ldr;
    }
    // the specialised kernels address a block-row of Y, and of the residual, with 32-bit byte offsets:
    // both row strides must stay within 2^23 elements there (beyond that the generic kernel runs)
    const int64_t ld_wide = (a.ep_on && a.ep_res && a.ep_ldr > ldy) ? a.ep_ldr : ldy;
    a.act = nullptr;
    if (conv) {
        // implicit lowering: X is the activation itself
        a.act = X;
        a.X = nullptr;
        fill_conv_args(a, g, *conv);
    }
    if (x_layout == CRISP_X_K8) {
        // octet-interleaved operands: one kernel family (the caller has checked what it covers)
        a.use_smf = 1;
        report(CRISP_KERNEL_K8, 1, 0, g.n <= 2);
        switch (g.n * 16 + g.m) {
            case 1 * 16 + 4: return launch_k8_nm<1, 4>(a, g.B, st);
            case 2 * 16 + 4: return launch_k8_nm<2, 4>(a, g.B, st);
            case 3 * 16 + 4: return launch_k8_nm<3, 4>(a, g.B, st);
            case 4 * 16 + 4: return launch_k8_nm<4, 4>(a, g.B, st);
            case 1 * 16 + 8: return launch_k8_nm<1, 8>(a, g.B, st);
            case 2 * 16 + 8: return launch_k8_nm<2, 8>(a, g.B, st);
            case 4 * 16 + 8: return launch_k8_nm<4, 8>(a, g.B, st);
            case 8 * 16 + 8: return launch_k8_nm<8, 8>(a, g.B, st);
            default: return hipErrorInvalidValue;
        }
    }
    if (g.B == 16) { report(CRISP_KERNEL_B16, 0, 0, 0); return launch_b16(a, st); }
    // convolution with the input patch staged in LDS (forced shape 12)
    ConvLdsSched cs;
    const bool conv_lds_wanted = force_shape == 12 || force_shape < 0;
    if (conv && conv_lds_wanted && (Ncol % 4) == 0 && ld_wide <= ((int64_t)1 << 23) && conv_lds_plan(a, g.B, conv->kh, &cs) &&
        (force_shape == 12 || conv_lds_pays(cs, g.Sb, density_hint, conv->batch, a.Wo))) {
        a.use_smf = 1;
        report(CRISP_KERNEL_CONV_LDS, 0, a.conv_mode, g.n <= 2);
        switch (g.n * 16 + g.m) {
            case 1 * 16 + 4: return launch_conv_lds_nm<1, 4>(a, cs, conv->batch, st);
            case 2 * 16 + 4: return launch_conv_lds_nm<2, 4>(a, cs, conv->batch, st);
            case 3 * 16 + 4: return launch_conv_lds_nm<3, 4>(a, cs, conv->batch, st);
            case 4 * 16 + 4: return launch_conv_lds_nm<4, 4>(a, cs, conv->batch, st);
            case 1 * 16 + 8: return launch_conv_lds_nm<1, 8>(a, cs, conv->batch, st);
            case 2 * 16 + 8: return launch_conv_lds_nm<2, 8>(a, cs, conv->batch, st);
            case 4 * 16 + 8: return launch_conv_lds_nm<4, 8>(a, cs, conv->batch, st);
            case 8 * 16 + 8: return launch_conv_lds_nm<8, 8>(a, cs, conv->batch, st);
            default: break;
        }
    }
    // channel counts that are no multiple of the block size (first layers): input patch in LDS in its
    // own layout (forced shape 14)
    ConvPatchSched ps;
    if (conv && (force_shape == 14 || force_shape < 0) && ld_wide <= ((int64_t)1 << 23) &&
        conv_patch_plan(a, g.B, conv->kh, g.Kb, &ps)) {
        a.use_smf = 1;
        report(CRISP_KERNEL_CONV_PATCH, 0, a.conv_mode, g.n <= 2);
        switch (g.n * 16 + g.m) {
            case 1 * 16 + 4: return launch_conv_patch_nm<1, 4>(a, ps, conv->batch, st);
            case 2 * 16 + 4: return launch_conv_patch_nm<2, 4>(a, ps, conv->batch, st);
            case 3 * 16 + 4: return launch_conv_patch_nm<3, 4>(a, ps, conv->batch, st);
            case 4 * 16 + 4: return launch_conv_patch_nm<4, 4>(a, ps, conv->batch, st);
            case 1 * 16 + 8: return launch_conv_patch_nm<1, 8>(a, ps, conv->batch, st);
            case 2 * 16 + 8: return launch_conv_patch_nm<2, 8>(a, ps, conv->batch, st);
            case 4 * 16 + 8: return launch_conv_patch_nm<4, 8>(a, ps, conv->batch, st);
            case 8 * 16 + 8: return launch_conv_patch_nm<8, 8>(a, ps, conv->batch, st);
            default: break;
        }
    }
    // LDS-resident block-rows (forced shapes 5 = narrow strips, 6 = wide strips)
    // kept blocks per block-row as the descriptor states them (a hint: only speed depends on it)
    const bool hint = density_hint > 0.0 && density_hint <= 1.0;
    int bpr = hint ? (int)(density_hint * g.Kb + 0.5) : (g.Kb + 1) / 2;
    if (bpr < 1) bpr = 1;
    // LDS-resident block-rows (forced shapes 5 = narrow strips, 6 = wide strips)
    const bool lds_ok = !conv && (g.K % 16) == 0 && (Ncol % 4) == 0 && ld_wide <= ((int64_t)1 << 23);
    // (reported shape of this family: bit 0 = wide strips, bit 1 = the instantiation with the larger tile capacity
    // where the block size has two; the kernels are not specialised by pattern)
    auto lds_variant = [&](bool wide) { return (wide ? 1 : 0) | ((g.B == 64 ? (wide && bpr > 9) : bpr > 36) ? 2 : 0); };
    if (lds_ok && (force_shape == 5 || force_shape == 6)) {
        report(CRISP_KERNEL_LDS, lds_variant(force_shape == 6), 0, 0);
        return launch_spmm_lds(a, g.B, bpr, force_shape == 6, st);
    }
    // the same with the blocks resident as sparse matrix-core operands (forced shapes 16 and 17, the latter
    // always the 30-tile instantiation): 64 x 64 blocks, at most two kept values per group
    const bool lds_smf_ok = lds_ok && g.B == 64 && smf_ok;
    if (lds_smf_ok && (force_shape == CRISP_SHAPE_LDS_SMF || force_shape == CRISP_SHAPE_LDS_SMF_30)) {
        const int variant = force_shape == CRISP_SHAPE_LDS_SMF ? 0 : 2;
        report(CRISP_KERNEL_LDS, (variant == 2 || bpr > 14) ? 2 : 0, 0, 1);
        return launch_spmm_lds_smf(a, bpr, variant, st);
    }
    // the kernels that keep X on chip for all block-rows come first where their rules (further down) apply
    const bool x_dense48 = g.n == 4 && g.m == 8;           // dense expansion through the selector table
    const bool xres_auto = !conv && g.Kb == 1 && g.Sb >= 2 && (smf_ok || x_dense48) && Ncol >= ((int64_t)1 << 18);
    const bool xlds_auto = (smf_ok && xlds_pays(g.Sb, g.Kb, Ncol, conv != nullptr)) ||
                           (x_dense48 && xlds_pays(g.Sb, g.Kb, Ncol, false));
    const bool x_on_chip = force_shape < 0 && g.B == 64 && (g.K % 16) == 0 && (Ncol % 4) == 0 && (xres_auto || xlds_auto);
    if (lds_smf_ok && force_shape < 0 && hint && uniform_rows && !x_on_chip && prefer_lds_smf(g, Ncol, bpr)) {
        report(CRISP_KERNEL_LDS, 2, 0, 1);
        return launch_spmm_lds_smf(a, bpr, 2, st);
    }
    if (lds_ok && force_shape < 0 && hint && uniform_rows && !x_on_chip && prefer_lds(g, Ncol, bpr)) {
        report(CRISP_KERNEL_LDS, lds_variant(bpr <= 1), 0, 0);
        return launch_spmm_lds(a, g.B, bpr, bpr <= 1, st);
    }
    // Block-rows of uneven length (forced shape 15; chosen for plain block pruning over the whole grid): the
    // block list is dealt evenly to the waves
    const bool bal_ok = !conv && (g.K % 16) == 0 && (Ncol % 4) == 0 && ld_wide <= ((int64_t)1 << 23) && g.Sb <= BAL_MAX_ROWS;
    if (bal_ok && (force_shape == CRISP_SHAPE_BALANCED || (force_shape < 0 && !uniform_rows && g.Sb >= 2))) {
        a.use_smf = 1;
        const int key = g.n * 16 + g.m;
        report(CRISP_KERNEL_BALANCED, 0, 0, g.n <= 2);
        switch (key) {
            case 1 * 16 + 4: return launch_balanced_nm<1, 4>(a, g.B, st);
            case 2 * 16 + 4: return launch_balanced_nm<2, 4>(a, g.B, st);
            case 3 * 16 + 4: return launch_balanced_nm<3, 4>(a, g.B, st);
            case 4 * 16 + 4: return launch_balanced_nm<4, 4>(a, g.B, st);
            case 1 * 16 + 8: return launch_balanced_nm<1, 8>(a, g.B, st);
            case 2 * 16 + 8: return launch_balanced_nm<2, 8>(a, g.B, st);
            case 4 * 16 + 8: return launch_balanced_nm<4, 8>(a, g.B, st);
            case 8 * 16 + 8: return launch_balanced_nm<8, 8>(a, g.B, st);
            default: break;
        }
    }
    // forced shapes 7..10: shapes 0..3 of the register kernels with the sparse matrix-core instruction
    // (the automatic choice always takes it where the pattern is eligible: it was faster for every
    // measured layer; shapes 0..3 force the dense-expansion instantiations)
    a.use_smf = (force_shape < 0 || force_shape == 13 || force_shape == CRISP_SHAPE_XLDS || (force_shape >= 7 && force_shape <= 10)) ? 1 : 0;
    // X-resident kernel for short K (forced shape 13).  Chosen for one block column, several
    // block-rows, patterns that go to the sparse matrix-core instruction and long X rows: 1.12x on the
    // 64 -> 256 channel layers of ResNet-50 at batch 256 (107 vs 120 us for 103 MB read and 411 MB
    // written; a plain fill of 411 MB takes 61 us, a copy of 257 + 257 MB 97 us), 1.19x for 4:8 expanded
    // through the selector table (117 vs 140 us in the LDS-resident kernel); equal within 6 % either way for
    // two block columns or the other dense-expansion patterns
    const bool xres = xres_covers(a, g.B) &&
        (force_shape == 13 || (force_shape < 0 && xres_auto));
    // X strip resident in LDS as operands for all block-rows (forced shape 18)
    // Chosen for patterns that go to the sparse matrix-core instruction when at least 16 block-rows share
    // two to eight block columns and there are enough columns for a workgroup per compute unit: 1.2-1.45x on
    // the 256 -> 1024 and 512 -> 2048 channel layers of ResNet-50 at batch 256 (rows of one to three blocks:
    // 29-37 us against 37-52 us, 20-23 us against 23-28 us); 0.75-1.0x with 8 block-rows or fewer, with one
    // block column (the register-resident kernel above is for those).  4:8 expanded through the selector table
    // gains as well from 16 block-rows on (1024 x 256 x 50176: 39.5 against 49.4 us in the LDS-resident kernel,
    // 2048 x 512 x 12544: 39.7 against 48.7 us; stage-3 shortcut of ResNet-50 with the strided lowering fused in:
    // 112 us against 123 us through a materialised X); the other dense-expansion patterns do not.
    // With the lowering of a strided 1 x 1 filter fused in, the strided gather is done once per strip instead of
    // once per block-row: chosen from 8 block-rows on (512 x 256 x 200704 1:8: 134 against 165 us; the input
    // alone is 411 MB there, of which every line is touched).
    const bool xlds = !xres && xlds_covers(a, g.B) &&
        (force_shape == CRISP_SHAPE_XLDS ||
         (force_shape < 0 && xlds_auto));
    const int shape = xres ? XRES_SHAPE : xlds ? XLDS_SHAPE
                    : (force_shape >= 0 && force_shape <= 3) ? force_shape
                    : (force_shape >= 7 && force_shape <= 10) ? force_shape - 7
                    : pick_shape(g, Ncol, bpr, a.use_smf && smf_ok);
    // the specialised kernels assume whole 16-row MFMA steps of X (K % 16 == 0) and whole groups
    // of four output columns per lane (Ncol % 4 == 0)
    if (conv || (force_shape != 4 && (g.K % 16) == 0 && (Ncol % 4) == 0 && ld_wide <= ((int64_t)1 << 23))) {
        const int key = g.n * 16 + g.m;
        const bool known = key == 0x14 || key == 0x24 || key == 0x34 || key == 0x44 || key == 0x18 || key == 0x28 ||
                           key == 0x48 || key == 0x88;
        // (the fused lowering has the narrow shapes only)
        const int shape_run = (xres || xlds) ? 0 : (conv && shape == 0) ? 1 : shape;
        if (known) report(xres ? CRISP_KERNEL_XRES : xlds ? CRISP_KERNEL_XLDS : CRISP_KERNEL_REG, shape_run, conv ? a.conv_mode : 0,
                          a.use_smf && (g.n <= 2 || (g.two_of_four && (!conv || xlds))));
        switch (key) {
            case 1 * 16 + 4: return launch_reg_nm<1, 4>(a, g.B, shape, st);
            case 2 * 16 + 4: return launch_reg_nm<2, 4>(a, g.B, shape, st);
            case 3 * 16 + 4: return launch_reg_nm<3, 4>(a, g.B, shape, st);
            case 4 * 16 + 4: return launch_reg_nm<4, 4>(a, g.B, shape, st);
            case 1 * 16 + 8: return launch_reg_nm<1, 8>(a, g.B, shape, st);
            case 2 * 16 + 8: return launch_reg_nm<2, 8>(a, g.B, shape, st);
            case 4 * 16 + 8: return launch_reg_nm<4, 8>(a, g.B, shape, st);
            case 8 * 16 + 8: return launch_reg_nm<8, 8>(a, g.B, shape, st);
            default: break;
        }
        if (conv) return hipErrorInvalidValue;  // callers check the pattern first
    }
    // any other n:m (or forced): the generic LDS-expansion kernel
    const bool wide = (int64_t)g.Sb * ((Ncol + 511) / 512) >= 512;
    report(CRISP_KERNEL_GENERIC, wide, 0, 0);
    if (g.B == 64) return wide ? launch_one<64, 2, 4>(a, st) : launch_one<64, 1, 4>(a, st);
    return wide ? launch_one<32, 2, 4>(a, st) : launch_one<32, 1, 4>(a, st);
}

}  // namespace crisp
