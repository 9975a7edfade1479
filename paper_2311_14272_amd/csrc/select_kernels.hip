// Mask selection kernels: saliency -> N:M choice -> block scores -> block choice.
// Alg. 1 lines 2, 4-6 and 10 of the CRISP paper; every ordering decision below is a total
// order so that the result is unique and reproducible bit for bit.
#include "crisp_internal.h"

namespace crisp {

// Saliency of one element (Sec. 3.4, Eq. 1): one fp32 multiply, then the absolute value.
template <int KIND>
__device__ __forceinline__ float saliency_at(const uint16_t* __restrict__ W, const float* __restrict__ TG, size_t e) {
    if (KIND == CRISP_SAL_GIVEN) return TG[e];
    if (KIND == CRISP_SAL_GRAD) return fabsf(__fmul_rn(bf16_bits_to_float(W[e]), TG[e]));
    return fabsf(bf16_bits_to_float(W[e]));
}

// One thread per aligned group of M columns.  The M keep bits of the 32/M groups that share a
// mask word are OR-combined across neighbouring lanes with xor-shuffles; one lane stores the word.
// grid.x covers ceil(K/32)*(32/M) groups in units of 64 lanes, grid.y covers rows in units of 4.
template <int M, int KIND>
__global__ __launch_bounds__(256) void nm_select_kernel(int S, int K, int n, int mwpr,
                                                        const uint16_t* __restrict__ W,
                                                        const float* __restrict__ TG,
                                                        uint32_t* __restrict__ nm_mask) {
    constexpr int GPW = 32 / M;  // groups per mask word
    const int gx = blockIdx.x * 64 + threadIdx.x;
    const int s = blockIdx.y * 4 + threadIdx.y;
    const int word = gx / GPW;
    const bool live = (s < S) && (word < mwpr);
    uint32_t bits = 0;
    if (live) {
        const int k0 = gx * M;
        const int len = min(M, K - k0);  // may be <= 0 in the last word of a ragged row
        float t[M];
#pragma unroll
        for (int i = 0; i < M; ++i) t[i] = (i < len) ? saliency_at<KIND>(W, TG, (size_t)s * K + k0 + i) : -1.0f;
#pragma unroll
        for (int i = 0; i < M; ++i) {
            int before = 0;
#pragma unroll
            for (int j = 0; j < M; ++j) before += (j < len) && (t[j] > t[i] || (t[j] == t[i] && j < i));
            if (i < len && before < n) bits |= 1u << i;
        }
        bits <<= (gx % GPW) * M;
    }
    // all 64 lanes of the wave take part in the shuffles; GPW consecutive lanes form one word
#pragma unroll
    for (int d = 1; d < GPW; d <<= 1) bits |= __shfl_xor(bits, d, 64);
    if (live && (gx % GPW) == 0) nm_mask[(size_t)s * mwpr + word] = bits;
}

// One workgroup (one wave) per block.  Lane r walks row r of the block left to right and adds
// the kept saliencies in fp64; lane 0 then adds the row sums top to bottom.  This order is part
// of the definition of the score (a tree reduction would round differently).
template <int KIND>
__global__ __launch_bounds__(64) void block_score_kernel(int S, int K, int B, int Kb, int mwpr,
                                                         const uint16_t* __restrict__ W,
                                                         const float* __restrict__ TG,
                                                         const uint32_t* __restrict__ nm_mask,
                                                         double* __restrict__ score) {
    __shared__ double rowsum[64];
    const int bj = blockIdx.x, bi = blockIdx.y, r = threadIdx.x;
    const int s = bi * B + r;
    double acc = 0.0;
    if (r < B && s < S) {
        const int k_begin = bj * B, k_end = min(K, k_begin + B);
        for (int k = k_begin; k < k_end; ++k) {
            const uint32_t wbits = nm_mask[(size_t)s * mwpr + (k >> 5)];
            if ((wbits >> (k & 31)) & 1u) acc = __dadd_rn(acc, (double)saliency_at<KIND>(W, TG, (size_t)s * K + k));
        }
    }
    rowsum[r] = acc;
    __syncthreads();
    if (r == 0) {
        double total = 0.0;
        for (int i = 0; i < B; ++i) total = __dadd_rn(total, rowsum[i]);
        score[(size_t)bi * Kb + bj] = total;
    }
}

// Compaction of a keep-flag array into ascending indices by one wave: ballot + popcount prefix.
__device__ __forceinline__ int wave_compact(const uint8_t* flags, int count, int32_t* out, int lane) {
    int written = 0;
    for (int base = 0; base < count; base += 64) {
        const int j = base + lane;
        const bool f = (j < count) && flags[j];
        const unsigned long long ballot = __ballot(f);
        const int pos = __popcll(ballot & ((1ull << lane) - 1ull));
        if (f) out[written + pos] = j;
        written += __popcll(ballot);
    }
    return written;
}

// Uniform block pruning: one workgroup per block-row keeps the k_row blocks that come first
// under (score descending, column ascending) and writes their columns in ascending order.
__global__ __launch_bounds__(256) void block_topk_rows_kernel(int Sb, int Kb, int k_row,
                                                              const double* __restrict__ score,
                                                              int32_t* __restrict__ row_ptr,
                                                              int32_t* __restrict__ col_idx) {
    __shared__ double sc[4096];
    __shared__ uint8_t kept[4096];
    const int bi = blockIdx.x, tid = threadIdx.x;
    for (int j = tid; j < Kb; j += 256) sc[j] = score[(size_t)bi * Kb + j];
    __syncthreads();
    for (int j = tid; j < Kb; j += 256) {
        const double mine = sc[j];
        int before = 0;
        for (int o = 0; o < Kb; ++o) before += (sc[o] > mine) || (sc[o] == mine && o < j);
        kept[j] = before < k_row;
    }
    __syncthreads();
    if (tid < 64) wave_compact(kept, Kb, col_idx + (size_t)bi * k_row, tid);
    if (tid == 0) {
        row_ptr[bi] = bi * k_row;
        if (bi == Sb - 1) row_ptr[Sb] = Sb * k_row;
    }
}

// Plain block pruning over the whole grid (the non-uniform baseline): keep the `budget` blocks
// that come first under (score descending, block-row ascending, column ascending).  One
// workgroup; rows may come out uneven or empty.
__global__ __launch_bounds__(1024) void block_topk_layer_kernel(int Sb, int Kb, int budget,
                                                                const double* __restrict__ score,
                                                                int32_t* __restrict__ row_ptr,
                                                                int32_t* __restrict__ col_idx) {
    __shared__ double sc[8192];
    __shared__ uint8_t kept[8192];
    __shared__ int rowcnt[1024];
    const int total = Sb * Kb, tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    for (int a = tid; a < total; a += 1024) sc[a] = score[a];
    __syncthreads();
    for (int a = tid; a < total; a += 1024) {
        const double mine = sc[a];
        int before = 0;
        for (int o = 0; o < total; ++o) before += (sc[o] > mine) || (sc[o] == mine && o < a);
        kept[a] = before < budget;
    }
    __syncthreads();
    for (int bi = wave; bi < Sb; bi += 16) {
        int c = 0;
        for (int base = 0; base < Kb; base += 64) {
            const int j = base + lane;
            c += __popcll(__ballot((j < Kb) && kept[bi * Kb + j]));
        }
        if (lane == 0) rowcnt[bi] = c;
    }
    __syncthreads();
    if (tid == 0) {
        int pos = 0;
        for (int bi = 0; bi < Sb; ++bi) {
            const int c = rowcnt[bi];
            row_ptr[bi] = pos;
            rowcnt[bi] = pos;
            pos += c;
        }
        row_ptr[Sb] = pos;
    }
    __syncthreads();
    for (int bi = wave; bi < Sb; bi += 16) wave_compact(kept + bi * Kb, Kb, col_idx + rowcnt[bi], lane);
}

template <int KIND>
static hipError_t launch_select_kind(const Geometry& g, int select_mode, const uint16_t* W, const float* TG,
                                     uint32_t* nm_mask, int32_t* row_ptr, int32_t* col_idx, double* score,
                                     hipStream_t st) {
    const int gpw = 32 / g.m;
    dim3 blk(64, 4);
    dim3 grd((g.mwpr * gpw + 63) / 64, (g.S + 3) / 4);
    if (g.m == 4)
        nm_select_kernel<4, KIND><<<grd, blk, 0, st>>>(g.S, g.K, g.n, g.mwpr, W, TG, nm_mask);
    else
        nm_select_kernel<8, KIND><<<grd, blk, 0, st>>>(g.S, g.K, g.n, g.mwpr, W, TG, nm_mask);
    block_score_kernel<KIND><<<dim3(g.Kb, g.Sb), 64, 0, st>>>(g.S, g.K, g.B, g.Kb, g.mwpr, W, TG, nm_mask, score);
    if (select_mode == CRISP_ROW_UNIFORM)
        block_topk_rows_kernel<<<g.Sb, 256, 0, st>>>(g.Sb, g.Kb, g.k_row, score, row_ptr, col_idx);
    else
        block_topk_layer_kernel<<<1, 1024, 0, st>>>(g.Sb, g.Kb, g.Sb * g.k_row, score, row_ptr, col_idx);
    return hipGetLastError();
}

hipError_t launch_select(const Geometry& g, int sal_kind, int select_mode, const uint16_t* W, const float* TG,
                         uint32_t* nm_mask, int32_t* row_ptr, int32_t* col_idx, double* score_out, double* score,
                         hipStream_t st) {
    (void)score_out;
    if (sal_kind == CRISP_SAL_GIVEN)
        return launch_select_kind<CRISP_SAL_GIVEN>(g, select_mode, W, TG, nm_mask, row_ptr, col_idx, score, st);
    if (sal_kind == CRISP_SAL_GRAD)
        return launch_select_kind<CRISP_SAL_GRAD>(g, select_mode, W, TG, nm_mask, row_ptr, col_idx, score, st);
    return launch_select_kind<CRISP_SAL_MAG>(g, select_mode, W, TG, nm_mask, row_ptr, col_idx, score, st);
}

}  // namespace crisp
