// Packing kernels: kept blocks -> compressed values + in-group positions (Sec. 3.1, Sec. 3.5).
#include "crisp_internal.h"

namespace crisp {

__global__ void pack_init_flags_kernel(int32_t* flags) {
    if (threadIdx.x == 0) { flags[0] = 1; flags[1] = 0; flags[2] = 0; flags[3] = 0; }
}

// Block-row that owns kept block t: the last bi with row_ptr[bi] <= t (rows may be empty).
__device__ __forceinline__ int owner_row(const int32_t* __restrict__ row_ptr, int Sb, int t) {
    int lo = 0, hi = Sb;
    while (hi - lo > 1) {
        const int mid = (lo + hi) >> 1;
        if (row_ptr[mid] <= t) lo = mid; else hi = mid;
    }
    return lo;
}

// Position stored in slot j of a group: the j-th kept column of the group (0-based inside the
// group), 0 when the group holds fewer kept elements (short last group), j when the group lies
// wholly outside the matrix.
__device__ __forceinline__ uint32_t slot_position(uint32_t bits, int j, bool outside) {
    if (outside) return (uint32_t)j;
    for (int i = 0; i < j; ++i) bits &= bits - 1u;  // drop the j lowest set bits
    return bits ? (uint32_t)(__ffs(bits) - 1) : 0u;
}

// The N:M keep bits of row s for the B columns of block column bj, as one 64-bit value
// (bit c = column bj*B + c; bits of columns past K are zero because the mask never sets them).
template <int B>
__device__ __forceinline__ uint64_t block_row_bits(const uint32_t* __restrict__ nm_mask, int mwpr, int s, int bj) {
    const uint32_t* row = nm_mask + (size_t)s * mwpr;
    if (B == 64) {
        const int w0 = bj * 2;
        const uint64_t lo = row[w0];
        const uint64_t hi = (w0 + 1 < mwpr) ? row[w0 + 1] : 0u;
        return lo | (hi << 32);
    }
    if (B == 32) return row[bj];
    return (row[bj >> 1] >> ((bj & 1) * 16)) & 0xFFFFu;
}

// One workgroup per kept block.  Phase 1: one thread per (block row, group) gathers the kept
// values in ascending column order.  Phase 2: one thread per (block row, index word) assembles
// the little-endian stream of log2(m)-bit positions.  B and M are compile-time so that the
// item loops unroll and all loads of a phase are issued before the first one is consumed.
// uniform_k_row > 0: every block-row holds exactly that many blocks, so the owner of block t is
// t / uniform_k_row and no search is needed.  flag_mode: 0 = flags[0] was preset to 1 and is
// cleared when an aligned group of four holds more than two kept elements; 1 = the pattern can
// never do that (n <= 2), workgroup 0 writes the constant.
// VEC: K % m == 0, so a group's m weights are one aligned 8- or 16-byte load.
template <int B, int M, bool VEC>
__global__ __launch_bounds__(256) void pack_block_kernel(int S, int K, int n, int Sb, int w, int slots, int wpr,
                                                         int mwpr, int uniform_k_row, int flag_mode,
                                                         const uint16_t* __restrict__ W,
                                                         const uint32_t* __restrict__ nm_mask,
                                                         const int32_t* __restrict__ row_ptr,
                                                         const int32_t* __restrict__ col_idx,
                                                         uint16_t* __restrict__ vals, uint32_t* __restrict__ idxw,
                                                         int32_t* __restrict__ flags) {
    constexpr int G = B / M;                         // groups per block row
    constexpr int ITEMS = (B * G + 255) / 256;       // (row, group) items per thread: 1..4
    constexpr int WMAX = (B * 3 + 31) / 32;          // upper bound of index words per block row
    constexpr int WITEMS = (B * WMAX + 255) / 256;   // (row, word) items per thread: 1..2
    const int t = blockIdx.x;
    const int bi = uniform_k_row > 0 ? t / uniform_k_row : owner_row(row_ptr, Sb, t);
    const int bj = col_idx[t];
    if (flag_mode == 1 && t == 0 && threadIdx.x == 0) { flags[0] = 1; flags[1] = 0; flags[2] = 0; flags[3] = 0; }

    // ---- phase 1 -----------------------------------------------------------------------------
    uint64_t rbits[ITEMS];
    uint16_t wv[ITEMS][M];
    bool live[ITEMS];
#pragma unroll
    for (int it = 0; it < ITEMS; ++it) {
        const int e = threadIdx.x + it * 256;
        const int r = e / G, g = e % G;
        const int s = bi * B + r, k0 = bj * B + g * M;
        live[it] = (e < B * G) && (s < S) && (k0 < K);
        rbits[it] = 0;
#pragma unroll
        for (int o = 0; o < M; ++o) wv[it][o] = 0;
        if (live[it]) {
            rbits[it] = block_row_bits<B>(nm_mask, mwpr, s, bj);
            const uint16_t* src = W + (size_t)s * K + k0;
            if (VEC) {
                if (M == 4) {
                    const uint2 q = *reinterpret_cast<const uint2*>(src);
                    wv[it][0] = q.x & 0xFFFFu; wv[it][1] = q.x >> 16; wv[it][2] = q.y & 0xFFFFu; wv[it][3] = q.y >> 16;
                } else {
                    const uint4 q = *reinterpret_cast<const uint4*>(src);
                    wv[it][0] = q.x & 0xFFFFu; wv[it][1] = q.x >> 16; wv[it][2] = q.y & 0xFFFFu; wv[it][3] = q.y >> 16;
                    wv[it][M - 4] = q.z & 0xFFFFu; wv[it][M - 3] = q.z >> 16; wv[it][M - 2] = q.w & 0xFFFFu; wv[it][M - 1] = q.w >> 16;
                }
            } else {
#pragma unroll
                for (int o = 0; o < M; ++o)
                    if (k0 + o < K) wv[it][o] = src[o];
            }
        }
    }
    bool violates = false;
#pragma unroll
    for (int it = 0; it < ITEMS; ++it) {
        const int e = threadIdx.x + it * 256;
        if (e < B * G) {
            const int r = e / G, g = e % G;
            const uint32_t bits = (uint32_t)(rbits[it] >> (g * M)) & ((1u << M) - 1u);
            uint16_t v[M];
#pragma unroll
            for (int q = 0; q < M; ++q) v[q] = 0;
            int filled = 0;
#pragma unroll
            for (int o = 0; o < M; ++o) {
                const bool on = (bits >> o) & 1u;
#pragma unroll
                for (int q = 0; q < M; ++q)
                    if (on && filled == q) v[q] = wv[it][o];
                filled += on;
            }
            if (__popc(bits & 0xFu) > 2 || __popc(bits >> 4) > 2) violates = true;
            uint16_t* out = vals + ((size_t)t * B + r) * slots + g * n;
#pragma unroll
            for (int q = 0; q < M; ++q)
                if (q < n) out[q] = v[q];
        }
    }
    // one atomic per wave at most, and none once the flag is already cleared
    if (flag_mode == 0 && __any(violates) && (threadIdx.x & 63) == 0 && flags[0] != 0) atomicAnd(flags, 0);

    // ---- phase 2 -----------------------------------------------------------------------------
    uint64_t rb2[WITEMS];
#pragma unroll
    for (int it = 0; it < WITEMS; ++it) {
        const int e = threadIdx.x + it * 256;
        const int r = e / wpr;
        const int s = bi * B + r;
        rb2[it] = (e < B * wpr && s < S) ? block_row_bits<B>(nm_mask, mwpr, s, bj) : 0ull;
    }
#pragma unroll
    for (int it = 0; it < WITEMS; ++it) {
        const int e = threadIdx.x + it * 256;
        if (e < B * wpr) {
            const int r = e / wpr, x = e % wpr;
            const bool row_outside = bi * B + r >= S;
            const int q_begin = (32 * x) / w;                         // first slot touching this word
            const int q_end = min(slots, (32 * x + 31) / w + 1);      // one past the last
            uint32_t word = 0;
            for (int q = q_begin; q < q_end; ++q) {
                const int g = q / n, j = q % n;
                const bool outside = row_outside || (bj * B + g * M >= K);
                const uint32_t bits = (uint32_t)(rb2[it] >> (g * M)) & ((1u << M) - 1u);
                const uint32_t pos = slot_position(bits, j, outside);
                const int bit = q * w - 32 * x;                       // may be negative: field began in the previous word
                word |= bit >= 0 ? (pos << bit) : (pos >> (-bit));
            }
            idxw[((size_t)t * B + r) * wpr + x] = word;
        }
    }
}

template <int B, int M>
static void launch_pack_bm(const Geometry& g, int ukr, int flag_mode, const uint16_t* W, const uint32_t* nm_mask,
                           const int32_t* row_ptr, const int32_t* col_idx, uint16_t* vals, uint32_t* idxw,
                           int32_t* flags, hipStream_t st) {
    if (g.K % M == 0)
        pack_block_kernel<B, M, true><<<g.nk, 256, 0, st>>>(g.S, g.K, g.n, g.Sb, g.w, g.slots, g.wpr, g.mwpr, ukr,
                                                            flag_mode, W, nm_mask, row_ptr, col_idx, vals, idxw, flags);
    else
        pack_block_kernel<B, M, false><<<g.nk, 256, 0, st>>>(g.S, g.K, g.n, g.Sb, g.w, g.slots, g.wpr, g.mwpr, ukr,
                                                             flag_mode, W, nm_mask, row_ptr, col_idx, vals, idxw, flags);
}

hipError_t launch_pack(const Geometry& g, int select_mode, const uint16_t* W, const uint32_t* nm_mask,
                       const int32_t* row_ptr, const int32_t* col_idx, uint16_t* vals, uint32_t* idxw,
                       int32_t* flags, hipStream_t st) {
    // n <= 2 can never put three kept elements into an aligned group of four
    const int flag_mode = (g.n <= 2 && g.nk > 0) ? 1 : 0;
    if (flag_mode == 0) pack_init_flags_kernel<<<1, 64, 0, st>>>(flags);
    const int ukr = select_mode == CRISP_ROW_UNIFORM ? g.k_row : 0;
    if (g.nk > 0) {
        switch (g.B * 16 + g.m) {
            case 64 * 16 + 4: launch_pack_bm<64, 4>(g, ukr, flag_mode, W, nm_mask, row_ptr, col_idx, vals, idxw, flags, st); break;
            case 64 * 16 + 8: launch_pack_bm<64, 8>(g, ukr, flag_mode, W, nm_mask, row_ptr, col_idx, vals, idxw, flags, st); break;
            case 32 * 16 + 4: launch_pack_bm<32, 4>(g, ukr, flag_mode, W, nm_mask, row_ptr, col_idx, vals, idxw, flags, st); break;
            case 32 * 16 + 8: launch_pack_bm<32, 8>(g, ukr, flag_mode, W, nm_mask, row_ptr, col_idx, vals, idxw, flags, st); break;
            case 16 * 16 + 4: launch_pack_bm<16, 4>(g, ukr, flag_mode, W, nm_mask, row_ptr, col_idx, vals, idxw, flags, st); break;
            default: launch_pack_bm<16, 8>(g, ukr, flag_mode, W, nm_mask, row_ptr, col_idx, vals, idxw, flags, st); break;
        }
    }
    return hipGetLastError();
}

}  // namespace crisp
