// Hybrid-sparse product for large Ncol: the block-row's kept blocks are expanded ONCE per
// workgroup into dense bf16 tiles that stay in LDS (160 KB per CU holds 19 tiles of 64 x 64),
// and the workgroup's waves then stream strip after strip of X against them.  Compared with the
// register-expansion kernels (spmm_reg.h) the per-tile work of a wave shrinks to: row-wise X loads,
// two v_perm_b32 per pair of rows, one ds_read_b128 per A operand, MFMA -- for any n:m pattern,
// because the expansion is generic code that runs once.
//
// Sec. 3.5 of the CRISP paper keeps the compressed weights next to the MACs and selects
// activations per weight group; here the compressed block is what travels from HBM/L2 (a few KB
// per block, once per workgroup) and the selection is undone on chip, next to the matrix cores.
//
// Work split: workgroup (bi, g) owns block-row bi and, in iteration it, the strips
// (it*G + g)*NW + wave.  All waves of all workgroups run the same number of iterations, chosen on
// the host so that the strips divide as evenly as possible.
// If a block-row holds more blocks than fit (CAP), it is processed in chunks and every iteration
// re-expands each chunk (correct for any input, only slower); the host only picks this kernel when
// the layer descriptor says the rows fit.
#include "spmm_reg.h"
#include <type_traits>

namespace crisp {

struct LdsSched {
    int G;       // workgroups per block-row
    int iters;   // strips per wave
    int NS;      // strips in total
    int SW;      // columns per strip: a multiple of 4, at most 64 * WD (lanes past it stay idle)
};

// SN:SM != 0:0 -- the resident form of a block is the operand of the sparse matrix-core instruction
// (patterns with at most two kept values per aligned four, 64 x 64 blocks): per lane, 32-row tile and
// 32-deep step 16 bytes of stored values and one index word, 5 KB per block instead of 8, so that 30
// blocks fit, each step reads 20 bytes per lane from LDS instead of 32 and issues half the matrix-core
// instructions.  The kernel is then specialised by pattern, because the operand is built by the same
// code as in the register kernels (smf_operand).
template <int B, int WD, int NW, int CAP, int PF, int WPS, int SN = 0, int SM = 0>
__global__ __launch_bounds__(64 * NW) __attribute__((amdgpu_waves_per_eu(WPS, WPS)))
void spmm_lds_kernel(SpmmArgs p, LdsSched sch) {
    constexpr int RT = B / 32, KS = B / 16, NACC = 2 * WD;
    constexpr bool SMF = SN > 0;
    static_assert(!SMF || B == 64, "sparse-operand tiles are laid out for 64 x 64 blocks");
    constexpr int SMF_IDX = RT * (KS / 2) * 1024;            // index words behind the value operands
    constexpr int A_BYTES = SMF ? SMF_IDX + RT * (KS / 2) * 256 : B * B * 2;
    typedef typename XVec<WD>::type xvec_t;
    __shared__ __attribute__((aligned(16))) unsigned char lds_a[CAP * A_BYTES];
    // block columns of the resident tiles.  Read back through LDS rather than from global memory:
    // once the kernel has stored to Y the compiler no longer uses scalar loads for the list, and a
    // vector load would sit in the same in-order counter as the X requests and drain them.
    __shared__ int lds_bj[CAP];
    // per-row terms of the optional epilogue for this block-row (0 where absent or past S)
    __shared__ float lds_sc[B], lds_bs[B];

    // workgroup -> (block-row, column group); all block-rows of a column group get ids on the same
    // XCD so that the X strips they share are served by that XCD's L2
    const int id = blockIdx.x;
    const int xcd = id & 7, slot = id >> 3;
    const int bi = slot % p.Sb;
    const int g = (slot / p.Sb) * 8 + xcd;
    if (g >= sch.G) return;

    // (the wave index is made provably uniform so that everything derived from it -- strip numbers,
    // block-list indices -- stays in scalar registers and scalar loads)
    const int tid = threadIdx.x, wave = __builtin_amdgcn_readfirstlane(tid >> 6), lane = tid & 63;
    const int jj = lane & 31, hh = lane >> 5;
    if (p.ep_on && tid < B) {          // visible after the first barrier of the expansion
        const int row = bi * B + tid;
        lds_sc[tid] = (p.ep_scale && row < p.S) ? p.ep_scale[row] : 0.0f;
        lds_bs[tid] = (p.ep_bias && row < p.S) ? p.ep_bias[row] : 0.0f;
    }
    const int t_begin = p.row_ptr[bi], t_end = p.row_ptr[bi + 1];
    const int cnt = t_end - t_begin;
    const int nchunks = (cnt + CAP - 1) / CAP;
    const int cnt_pad = (cnt + PF - 1) / PF * PF;   // fast path: groups of PF blocks, padded with zero tiles

    // ---- expansion of blocks [c_begin, c_end) of this block-row into lds_a ----------------------
    // Wave w expands blocks c_begin + w, + NW, ... on its own, no barriers in between.  Each lane
    // builds, for every (row tile rt, MFMA step ks), exactly the 8 bf16 it will later feed to the
    // matrix core: row rt*32 + jj of the block, columns ks*16 + hh*8 .. +7, which are 8/m whole
    // groups = (8/m)*n packed slots and their position codes (at most 24 bits).  The tile is stored
    // fragment-major: the operand of lane l for (rt, ks) lives at ((rt*KS + ks)*64 + l)*16 bytes,
    // one conflict-free ds_read_b128.
    //   n == m: the operand is 8 consecutive stored values, one 16-byte load.
    //   n <  m: the block's packed values (at most 7/8 of a tile) are first copied with coalesced
    //           16-byte loads into the tile's own LDS space, the lanes pick their slots from there,
    //           and only when every lane holds its operands are they written over the copy (the
    //           LDS executes one wave's instructions in order).  Position words come straight
    //           from global memory.  Padding slots carry value 0, so OR-ing them in is harmless.
    auto expand_chunk = [&](int c_begin, int c_end, auto lean) __attribute__((always_inline)) {
        __syncthreads();                           // every wave is done with the previous chunk
        if (tid < c_end - c_begin) lds_bj[tid] = p.col_idx[c_begin + tid];
        const int nq = (8 / p.m) * p.n;            // slots behind one operand
        const int vbytes = B * p.slots * 2;
        const uint32_t pmask = (uint32_t)p.m - 1u;
        if constexpr (SMF) {
            constexpr int EN = SMF ? SN : 1, EM = SMF ? SM : 4;   // (the dense instantiation never gets here)
            typedef Fmt<EN, EM, B> F;
            typedef BlockBody<EN, EM, B, 1, false, 0, true> Body;
            const uint32_t a_off = (uint32_t)((jj * F::SLOTS + hh * F::FS * 2) * 2);
            const uint32_t i_off = (uint32_t)(jj * F::WPR * 4);
            const uint32_t aw_sh = (uint32_t)hh * F::HB * 2;
            for (int t = c_begin + wave; t < c_end; t += NW) {
                unsigned char* tile = lds_a + (t - c_begin) * A_BYTES;
                uint32_t av[RT][KS][F::VW], aw[RT][F::WPR], ws[RT][F::WPR];
                Body::load_a(av, aw, p, a_off, i_off, t);
#pragma unroll
                for (int rt = 0; rt < RT; ++rt) {
#pragma unroll
                    for (int i = 0; i < F::WPR; ++i)
                        ws[rt][i] = __builtin_amdgcn_alignbit(i + 1 < F::WPR ? aw[rt][i + 1] : 0u, aw[rt][i], aw_sh);
                    u32x4 a4[2];
                    uint32_t idx[2];
                    smf_operand<EN, EM, B, 0>(av[rt], ws[rt], a4[0], idx[0]);
                    smf_operand<EN, EM, B, 1>(av[rt], ws[rt], a4[1], idx[1]);
#pragma unroll
                    for (int s2 = 0; s2 < 2; ++s2) {
                        *reinterpret_cast<u32x4*>(tile + ((rt * 2 + s2) * 64 + lane) * 16) = a4[s2];
                        *reinterpret_cast<uint32_t*>(tile + SMF_IDX + ((rt * 2 + s2) * 64 + lane) * 4) = idx[s2];
                    }
                }
            }
            if constexpr (!decltype(lean)::value) {
                for (int t = c_end + wave; t < c_begin + cnt_pad; t += NW) {
                    unsigned char* tile = lds_a + (t - c_begin) * A_BYTES;
#pragma unroll
                    for (int q = 0; q < RT * 2; ++q) {
                        *reinterpret_cast<u32x4*>(tile + (q * 64 + lane) * 16) = u32x4{0u, 0u, 0u, 0u};
                        *reinterpret_cast<uint32_t*>(tile + SMF_IDX + (q * 64 + lane) * 4) = 0u;
                    }
                }
            }
            __syncthreads();
            return;
        }
        for (int t = c_begin + wave; t < c_end; t += NW) {
            unsigned char* tile = lds_a + (t - c_begin) * A_BYTES;
            u32x4 frag[RT * KS];
            if (p.n == p.m) {
#pragma unroll
                for (int q = 0; q < RT * KS; ++q) {
                    const int rt = q / KS, ks = q % KS;
                    frag[q] = *reinterpret_cast<const u32x4*>(p.vals + ((size_t)t * B + rt * 32 + jj) * B + ks * 16 + hh * 8);
                }
            } else {
                constexpr int NCH = A_BYTES / 1024;
                const unsigned char* src = reinterpret_cast<const unsigned char*>(p.vals) + (size_t)t * vbytes;
                u32x4 raw[NCH];
#pragma unroll
                for (int i = 0; i < NCH; ++i) {
                    const int off = (lane + i * 64) * 16;
                    raw[i] = *reinterpret_cast<const u32x4*>(src + min(off, vbytes - 16));
                }
                uint64_t pos_words[RT * KS];
#pragma unroll
                for (int q = 0; q < RT * KS; ++q) {
                    const int rt = q / KS, ks = q % KS;
                    const uint32_t* irow = p.idxw + ((size_t)t * B + rt * 32 + jj) * p.wpr;
                    const int wi = (((ks * 16 + hh * 8) / p.m) * p.n * p.w) >> 5;
                    pos_words[q] = (uint64_t)irow[wi] | ((uint64_t)irow[min(wi + 1, p.wpr - 1)] << 32);
                }
#pragma unroll
                for (int i = 0; i < NCH; ++i) {
                    const int off = (lane + i * 64) * 16;
                    if (off < vbytes) *reinterpret_cast<u32x4*>(tile + off) = raw[i];
                }
                const uint16_t* sv = reinterpret_cast<const uint16_t*>(tile);
#pragma unroll
                for (int q = 0; q < RT * KS; ++q) {
                    const int rt = q / KS, ks = q % KS;
                    const int q0 = ((ks * 16 + hh * 8) / p.m) * p.n;
                    const uint32_t stream = (uint32_t)(pos_words[q] >> ((q0 * p.w) & 31));
                    const uint16_t* vrow = sv + (rt * 32 + jj) * p.slots + q0;
                    uint32_t d[4] = {0u, 0u, 0u, 0u};
#pragma unroll
                    for (int sl = 0; sl < 8; ++sl) {
                        // slots past nq re-read the last one and contribute nothing
                        const uint32_t v16 = vrow[min(sl, nq - 1)];
                        const uint32_t pos = (stream >> (sl * p.w)) & pmask;
                        const uint32_t kk = pos + ((p.m == 4 && sl >= p.n) ? 4u : 0u);
                        const uint32_t v = sl < nq ? v16 << ((kk & 1u) * 16u) : 0u;
#pragma unroll
                        for (int x = 0; x < 4; ++x) d[x] |= ((kk >> 1) == (uint32_t)x) ? v : 0u;
                    }
                    frag[q] = u32x4{d[0], d[1], d[2], d[3]};
                    __builtin_amdgcn_sched_barrier(0);   // one operand's LDS reads at a time: few live registers
                }
            }
#pragma unroll
            for (int q = 0; q < RT * KS; ++q) *reinterpret_cast<u32x4*>(tile + q * 1024 + lane * 16) = frag[q];
        }
        if constexpr (!decltype(lean)::value) {
            // all-zero tiles that pad the block count to a multiple of PF
            for (int t = c_end + wave; t < c_begin + cnt_pad; t += NW) {
                const u32x4 z = {0u, 0u, 0u, 0u};
#pragma unroll
                for (int q = 0; q < RT * KS; ++q)
                    *reinterpret_cast<u32x4*>(lds_a + (t - c_begin) * A_BYTES + lane * 16 + q * 1024) = z;
            }
        }
        __syncthreads();                           // tiles visible to every wave
    };

    // X rows of block column bj, MFMA step ks (K % 16 == 0: a step past the end re-reads the last
    // 16 rows, finite values times the zero padding of the packed block)
    auto load_x = [&](xvec_t (&dst)[8], uint32_t lane_off, int bj, int ks) __attribute__((always_inline)) {
        const int kb = min(bj * B + ks * 16, p.K - 16);
        const rsrc_t r = make_rsrc(p.X + (int64_t)kb * p.ldx);
        const uint32_t row_bytes = (uint32_t)p.ldx * 2u;
#pragma unroll
        for (int i = 0; i < 8; ++i) dst[i] = buf_load_x<WD>(r, lane_off, (uint32_t)i * row_bytes);
    };

    const uint32_t esz = p.y_bf16 ? 2u : 4u;
    const uint32_t yrow_bytes = (uint32_t)p.ldy * esz;
    const int rows_here = min(B, p.S - bi * B);
    const rsrc_t ry = __builtin_amdgcn_make_buffer_rsrc(
        reinterpret_cast<char*>(p.Y) + (int64_t)bi * B * p.ldy * esz, 0, (uint32_t)rows_here * yrow_bytes, 0x00020000);

    // one kept block: 16-bit transposes of the X rows in registers, request of the rows that take
    // their place (block column bj_next at lane offset off_next), A operands from LDS, MFMA
    auto mma_block = [&](f32x16 (&acc)[RT][NACC], xvec_t (&xr)[KS][8], const unsigned char* abase,
                         uint32_t off_next, int bj_next) __attribute__((always_inline)) {
        if constexpr (SMF) {
            // abase: the tile + lane * 16; the lane's index words sit at a quarter of that offset behind the values
            const unsigned char* ibase = abase + SMF_IDX - (lane * 16) + lane * 4;
#pragma unroll
            for (int s2 = 0; s2 < KS / 2; ++s2) {
                u32x4 half[2][NACC];
#pragma unroll
                for (int k2 = 0; k2 < 2; ++k2) {
                    const int ks = 2 * s2 + k2;
                    uint32_t xd[8][WD];
#pragma unroll
                    for (int r = 0; r < 8; ++r) xvec_unpack(xr[ks][r], xd[r]);
#pragma unroll
                    for (int pd = 0; pd < WD; ++pd) {
#pragma unroll
                        for (int q = 0; q < 4; ++q) {
                            half[k2][2 * pd][q] = __builtin_amdgcn_perm(xd[2 * q + 1][pd], xd[2 * q][pd], SEL_LO);
                            half[k2][2 * pd + 1][q] = __builtin_amdgcn_perm(xd[2 * q + 1][pd], xd[2 * q][pd], SEL_HI);
                        }
                    }
                    load_x(xr[ks], off_next, bj_next, ks);
                }
                __builtin_amdgcn_sched_barrier(0);
#pragma unroll
                for (int rt = 0; rt < RT; ++rt) {
                    const u32x4 a4 = *reinterpret_cast<const u32x4*>(abase + (rt * 2 + s2) * 1024);
                    const uint32_t idx = *reinterpret_cast<const uint32_t*>(ibase + (rt * 2 + s2) * 256);
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
            return;
        }
#pragma unroll
        for (int ks = 0; ks < KS; ++ks) {
            uint32_t xd[8][WD];
#pragma unroll
            for (int r = 0; r < 8; ++r) xvec_unpack(xr[ks][r], xd[r]);
            bf16x8 bfrag[NACC];
#pragma unroll
            for (int pd = 0; pd < WD; ++pd) {
                u32x4 lo, hi;
#pragma unroll
                for (int q = 0; q < 4; ++q) {
                    lo[q] = __builtin_amdgcn_perm(xd[2 * q + 1][pd], xd[2 * q][pd], SEL_LO);
                    hi[q] = __builtin_amdgcn_perm(xd[2 * q + 1][pd], xd[2 * q][pd], SEL_HI);
                }
                bfrag[2 * pd] = __builtin_bit_cast(bf16x8, lo);
                bfrag[2 * pd + 1] = __builtin_bit_cast(bf16x8, hi);
            }
            load_x(xr[ks], off_next, bj_next, ks);
            // keep the requests where they are written: the scheduler otherwise sinks them to the
            // end of the loop body, which shortens the distance between request and use
            __builtin_amdgcn_sched_barrier(0);
#pragma unroll
            for (int rt = 0; rt < RT; ++rt) {
                const u32x4 a4 = *reinterpret_cast<const u32x4*>(abase + (rt * KS + ks) * 1024);
                const bf16x8 afrag = __builtin_bit_cast(bf16x8, a4);
#pragma unroll
                for (int c = 0; c < NACC; ++c)
                    acc[rt][c] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(afrag, bfrag[c], acc[rt][c], 0, 0, 0);
            }
        }
    };
    // accumulator register r of a 32x32 tile is row 8*(r/4) + 4*hh + r%4, column jj; rows past S
    // and lanes past the last column fall outside the store resource's range and are dropped
    // With an epilogue the residual values of a batch of rows are requested together before the
    // first of them is used (the requests share the in-order counter with the X rows in flight for
    // the next strip, so every wait for them also waits for those: one wait per batch, not per row);
    // scale and bias come from LDS.
    auto store_strip_t = [&](const f32x16 (&acc)[RT][NACC], bool col_ok, int64_t col0, auto as_bf16, auto with_ep) __attribute__((always_inline)) {
        constexpr bool BF16 = decltype(as_bf16)::value;
        const uint32_t y_off = col_ok ? (uint32_t)(4 * hh) * yrow_bytes + (uint32_t)col0 * esz : 0x80000000u;
        auto store_row = [&](int tile_row, const float (&v)[NACC]) __attribute__((always_inline)) {
            const uint32_t off = y_off + (uint32_t)tile_row * yrow_bytes;
            if constexpr (BF16) {
                uint32_t pk[WD];
#pragma unroll
                for (int c = 0; c < WD; ++c) {
                    const f32x2 two = {v[2 * c], v[2 * c + 1]};
                    pk[c] = __builtin_bit_cast(uint32_t, __builtin_convertvector(two, bf16x2));
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
                    const u32x4 four = {__float_as_uint(v[0]), __float_as_uint(v[1]),
                                        __float_as_uint(v[NACC - 2]), __float_as_uint(v[NACC - 1])};
                    __builtin_amdgcn_raw_buffer_store_b128(four, ry, off, 0, 0);
                }
            }
        };
        if constexpr (decltype(with_ep)::value) {
            constexpr int RW = BF16 ? WD : NACC;
            constexpr int CH = 16 / WD;
            const EpSource src = make_ep_source(p, bi, B, hh, col0, col_ok);
#pragma unroll
            for (int q0 = 0; q0 < RT * 16; q0 += CH) {
                EpBatch<CH, RW> eb;
#pragma unroll
                for (int j = 0; j < CH; ++j) {
                    const int rt = (q0 + j) >> 4, r = (q0 + j) & 15;
                    const int tile_row = rt * 32 + 8 * (r >> 2) + (r & 3);
                    ep_request_residual<RW>(src, tile_row, eb.res[j]);
                    eb.sc[j] = lds_sc[tile_row + 4 * hh];
                    eb.bs[j] = lds_bs[tile_row + 4 * hh];
                }
#pragma unroll
                for (int j = 0; j < CH; ++j) {
                    const int rt = (q0 + j) >> 4, r = (q0 + j) & 15;
                    float v[NACC];
#pragma unroll
                    for (int c = 0; c < NACC; ++c) v[c] = acc[rt][c][r];
                    ep_apply<NACC, BF16>(p, eb.res[j], eb.sc[j], eb.bs[j], v);
                    store_row(rt * 32 + 8 * (r >> 2) + (r & 3), v);
                }
            }
        } else {
#pragma unroll
            for (int rt = 0; rt < RT; ++rt)
#pragma unroll
                for (int r = 0; r < 16; ++r) {
                    float v[NACC];
#pragma unroll
                    for (int c = 0; c < NACC; ++c) v[c] = acc[rt][c][r];
                    store_row(rt * 32 + 8 * (r >> 2) + (r & 3), v);
                }
        }
    };
    auto store_strip = [&](const f32x16 (&acc)[RT][NACC], bool col_ok, int64_t col0) __attribute__((always_inline)) {
        if (p.ep_on) {
            if (p.y_bf16) store_strip_t(acc, col_ok, col0, std::true_type{}, std::true_type{});
            else store_strip_t(acc, col_ok, col0, std::false_type{}, std::true_type{});
        } else {
            if (p.y_bf16) store_strip_t(acc, col_ok, col0, std::true_type{}, std::false_type{});
            else store_strip_t(acc, col_ok, col0, std::false_type{}, std::false_type{});
        }
    };
    // lane part of the X addresses of a strip (bytes); lanes past the last column read column 0
    auto lane_offset = [&](int strip, bool& col_ok, int64_t& col0) __attribute__((always_inline)) {
        col0 = (int64_t)strip * sch.SW + jj * NACC;
        col_ok = strip < sch.NS && jj * NACC < sch.SW && col0 < p.Ncol;
        return (uint32_t)(((int64_t)hh * 8 * p.ldx + (col_ok ? col0 : 0)) * 2);
    };
    const int strip_step = sch.G * NW;

    auto zero_acc = [&](f32x16 (&acc)[RT][NACC]) __attribute__((always_inline)) {
#pragma unroll
        for (int rt = 0; rt < RT; ++rt)
#pragma unroll
            for (int c = 0; c < NACC; ++c)
#pragma unroll
                for (int r = 0; r < 16; ++r) acc[rt][c][r] = 0.0f;
    };

    // The fast path walks each strip's blocks in groups of PF (one ring slot per member, constant
    // register indices); a block count that is not a multiple of PF is padded with all-zero tiles.
    if (cnt_pad <= CAP) {
        // ---- the block-row fits: expand once, then the waves run free --------------------------
        expand_chunk(t_begin, t_end, std::false_type{});
        const int first = g * NW + wave;
        if (first >= sch.NS) return;
        f32x16 acc[RT][NACC];
        zero_acc(acc);
        // X rows are requested PF steps ahead, across strip boundaries; requests past the last
        // strip go to strips that do not exist, where every lane reads column 0 (cached lines).
        // The loop bodies hold no branches, so the compiler can count outstanding loads exactly.
        int l_t = 0, l_strip = first;
        bool ok_unused; int64_t c0_unused;
        uint32_t l_off = lane_offset(l_strip, ok_unused, c0_unused);
        auto advance_requests = [&]() __attribute__((always_inline)) {
            const bool wrap = l_t + 1 >= cnt_pad;
            l_t = wrap ? 0 : l_t + 1;
            l_strip += wrap ? strip_step : 0;
            l_off = lane_offset(l_strip, ok_unused, c0_unused);
        };
        auto requested_bj = [&]() __attribute__((always_inline)) {
            return __builtin_amdgcn_readfirstlane(lds_bj[max(min(l_t, cnt - 1), 0)]);   // padding re-requests the last block
        };
        xvec_t xr[PF][KS][8];
        auto first_request = [&](xvec_t (&slot)[KS][8]) __attribute__((always_inline)) {
            const int bj = requested_bj();
#pragma unroll
            for (int ks = 0; ks < KS; ++ks) load_x(slot[ks], l_off, bj, ks);
            advance_requests();
        };
        auto one_step = [&](xvec_t (&slot)[KS][8], int tl) __attribute__((always_inline)) {
            mma_block(acc, slot, lds_a + tl * A_BYTES + lane * 16, l_off, requested_bj());
            advance_requests();
        };
        if (cnt > 0) {
            // (spelled out per slot: the ring must stay in registers, which needs constant indices)
            first_request(xr[0]);
            if constexpr (PF > 1) first_request(xr[1]);
            if constexpr (PF > 2) first_request(xr[2]);
            if constexpr (PF > 3) first_request(xr[3]);
        }
        for (int strip = first; strip < sch.NS; strip += strip_step) {
#pragma unroll 1
            for (int tl = 0; tl < cnt_pad; tl += PF) {
                one_step(xr[0], tl);
                if constexpr (PF > 1) one_step(xr[1], tl + 1);
                if constexpr (PF > 2) one_step(xr[2], tl + 2);
                if constexpr (PF > 3) one_step(xr[3], tl + 3);
            }
            bool ok; int64_t c0;
            lane_offset(strip, ok, c0);
            store_strip(acc, ok, c0);
            zero_acc(acc);
        }
        return;
    }

    // ---- more blocks than LDS holds: chunks, re-expanded for every iteration (lock-step) --------
    for (int it = 0; it < sch.iters; ++it) {
        const int strip = (it * sch.G + g) * NW + wave;
        const bool active = strip < sch.NS;
        bool col_ok; int64_t col0;
        const uint32_t lane_off = lane_offset(strip, col_ok, col0);
        f32x16 acc[RT][NACC];
        zero_acc(acc);
        for (int ch = 0; ch < nchunks; ++ch) {
            const int c_begin = t_begin + ch * CAP, c_end = min(t_end, c_begin + CAP);
            expand_chunk(c_begin, c_end, std::true_type{});   // uniform over the workgroup
            if (!active) continue;
            xvec_t xr[KS][8];
            {
                const int bj = __builtin_amdgcn_readfirstlane(lds_bj[0]);
#pragma unroll
                for (int ks = 0; ks < KS; ++ks) load_x(xr[ks], lane_off, bj, ks);
            }
            for (int t = c_begin; t < c_end; ++t)
                mma_block(acc, xr, lds_a + (t - c_begin) * A_BYTES + lane * 16, lane_off,
                          __builtin_amdgcn_readfirstlane(lds_bj[min(t + 1, c_end - 1) - c_begin]));
        }
        if (active) store_strip(acc, col_ok, col0);
    }
}

template <int B, int WD, int NW, int CAP, int PF, int SN = 0, int SM = 0>
static hipError_t launch_lds(const SpmmArgs& a, int wgs_per_cu, hipStream_t st) {
    constexpr int TILE = SN > 0 ? 5 * 1024 : B * B * 2;
    constexpr int WPS = NW / 4 * (CAP * TILE > 80 * 1024 ? 1 : 2);   // waves per SIMD
    // With W waves per block-row resident at once the columns take
    // iters = ceil(strips / W) strips per wave.  (Shrinking the strips so that the last round is
    // as full as the others was measured to be slower: the time per block step does not shrink
    // with the strip.)
    LdsSched s;
    const int slots = 256 * wgs_per_cu;
    const int gmax = a.Sb >= slots ? 1 : slots / a.Sb;
    s.SW = 64 * WD;
    s.NS = (int)((a.Ncol + s.SW - 1) / s.SW);
    const int64_t waves_max = (int64_t)gmax * NW;
    s.iters = (int)((s.NS + waves_max - 1) / waves_max);
    s.G = (int)((s.NS + (int64_t)NW * s.iters - 1) / ((int64_t)NW * s.iters));
    const int64_t groups = (int64_t)((s.G + 7) / 8) * a.Sb * 8;
    const dim3 grd((unsigned)groups), blk(64 * NW);
    if (a.ev_start || a.ev_stop)
        hipExtLaunchKernelGGL((spmm_lds_kernel<B, WD, NW, CAP, PF, WPS, SN, SM>), grd, blk, 0, st, a.ev_start, a.ev_stop, 0, a, s);
    else
        spmm_lds_kernel<B, WD, NW, CAP, PF, WPS, SN, SM><<<grd, blk, 0, st>>>(a, s);
    return hipGetLastError();
}

// max_blocks: kept blocks per block-row according to the layer descriptor.  Rows with more
// blocks than the chosen variant holds (9 or 19 tiles of 64 x 64, 36 or 76 of 32 x 32) are still
// computed correctly, chunk by chunk, only slowly: callers decide whether the family pays.
// Narrow strips (64 columns per wave) run with a two-block request ring, wide strips (128 columns)
// with one block ahead: both keep the wave near the limit of 63 outstanding vector loads.
int lds_capacity(int B) { return B == 64 ? 19 : 76; }

// Blocks in the sparse-operand form (64 x 64 blocks, n <= 2): narrow strips, 15 tiles with two
// workgroups of four waves per compute unit or 30 tiles with one workgroup of eight waves (the block count
// is padded to a multiple of the request ring's two slots: 14 and 30 blocks are what fits).
int lds_smf_capacity() { return 30; }

template <int N, int M>
static hipError_t launch_lds_smf_nm(const SpmmArgs& a, int max_blocks, int variant, hipStream_t st) {
    const bool small = variant == 1 || (variant == 0 && max_blocks <= 14);
    return small ? launch_lds<64, 1, 4, 15, 2, N, M>(a, 2, st) : launch_lds<64, 1, 8, 30, 2, N, M>(a, 1, st);
}

// variant: 0 = by max_blocks, 1 = the 15-tile instantiation, 2 = the 30-tile one (rows that do not fit are
// computed chunk by chunk)
hipError_t launch_spmm_lds_smf(const SpmmArgs& a, int max_blocks, int variant, hipStream_t st) {
    switch (a.n * 16 + a.m) {
        case 1 * 16 + 4: return launch_lds_smf_nm<1, 4>(a, max_blocks, variant, st);
        case 2 * 16 + 4: return launch_lds_smf_nm<2, 4>(a, max_blocks, variant, st);
        case 1 * 16 + 8: return launch_lds_smf_nm<1, 8>(a, max_blocks, variant, st);
        case 2 * 16 + 8: return launch_lds_smf_nm<2, 8>(a, max_blocks, variant, st);
        case 4 * 16 + 8: return a.two_of_four ? launch_lds_smf_nm<4, 8>(a, max_blocks, variant, st) : hipErrorInvalidValue;
        default: return hipErrorInvalidValue;
    }
}

hipError_t launch_spmm_lds(const SpmmArgs& a, int B, int max_blocks, bool wide, hipStream_t st) {
    if (B == 64) {
        if (!wide) return launch_lds<64, 1, 8, 19, 2>(a, 1, st);
        return max_blocks <= 9 ? launch_lds<64, 2, 4, 9, 1>(a, 2, st) : launch_lds<64, 2, 8, 19, 1>(a, 1, st);
    }
    if (B == 32) {
        if (max_blocks <= 36) return wide ? launch_lds<32, 2, 4, 36, 2>(a, 2, st) : launch_lds<32, 1, 4, 36, 4>(a, 2, st);
        return wide ? launch_lds<32, 2, 8, 76, 2>(a, 1, st) : launch_lds<32, 1, 8, 76, 4>(a, 1, st);
    }
    return hipErrorInvalidValue;
}

}  // namespace crisp
