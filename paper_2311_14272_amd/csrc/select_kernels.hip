// Mask selection kernels: saliency -> N:M choice -> block scores -> block choice.
// Alg. 1 lines 2, 4-6 and 10 of the CRISP paper; every ordering decision below is a total
// order so that the result is unique and reproducible bit for bit.
#include "crisp_internal.h"

namespace crisp {

typedef __attribute__((ext_vector_type(4))) uint32_t u32x4;
typedef __attribute__((ext_vector_type(4))) float f32x4;

// Saliency of one element (Sec. 3.4, Eq. 1): one fp32 multiply, then the absolute value.
template <int KIND>
__device__ __forceinline__ float saliency_of(uint16_t w, float tg) {
    if (KIND == CRISP_SAL_GIVEN) return tg;
    if (KIND == CRISP_SAL_GRAD) return fabsf(__fmul_rn(bf16_bits_to_float(w), tg));
    return fabsf(bf16_bits_to_float(w));
}

// One workgroup per B x B block, Q lanes per block row (Q * CPT = B columns, CPT = 16 or 8).
// Each lane loads its CPT weights (and gradient / saliency values) with 16-byte loads, ranks
// every aligned group of M columns (keep the n first under: larger saliency first, on a tie the
// smaller column first), and leaves "saliency if kept else +0" in LDS.  The Q lanes of a row
// OR their mask bits together with xor-shuffles.  Then lane r of the first wave adds row r's B
// values left to right in fp64 and lane 0 adds the row sums top to bottom: that summation order
// is part of the definition of the block score (a tree reduction would round differently;
// adding +0.0 for a pruned element leaves the non-negative running sum unchanged bit for bit).
// VEC: row segments are 16-byte aligned and lie wholly inside the matrix (K % B == 0).
template <int B, int M, int KIND, bool VEC>
__global__ __launch_bounds__(B * (B / 16)) void score_select_kernel(int S, int K, int n, int Kb, int mwpr,
                                                                   const uint16_t* __restrict__ W,
                                                                   const float* __restrict__ TG,
                                                                   uint32_t* __restrict__ nm_mask,
                                                                   double* __restrict__ score) {
    constexpr int CPT = 16;          // columns per lane
    constexpr int Q = B / CPT;       // lanes per block row (1, 2 or 4)
    constexpr int LDT = B + 4;       // padded LDS row stride in floats (keeps 16-byte alignment)
    __shared__ __attribute__((aligned(16))) float tkept[B * LDT];
    __shared__ double rowsum[B];
    const int bj = blockIdx.x, bi = blockIdx.y;
    const int r = threadIdx.x / Q, q = threadIdx.x % Q;
    const int s = bi * B + r;
    const int c0 = q * CPT;                      // first column of this lane inside the block
    const int k0 = bj * B + c0;
    uint32_t bits = 0;
    {
        uint16_t w[CPT];
        float tg[CPT];
        const int len = (s < S) ? min(CPT, K - k0) : 0;   // columns of this lane that exist (may be <= 0)
        const size_t e0 = (size_t)s * K + k0;
        if (VEC && s < S) {
            if (KIND != CRISP_SAL_GIVEN) {
#pragma unroll
                for (int i = 0; i < CPT / 8; ++i) {
                    const u32x4 v = *reinterpret_cast<const u32x4*>(W + e0 + 8 * i);
#pragma unroll
                    for (int x = 0; x < 4; ++x) {
                        w[8 * i + 2 * x] = (uint16_t)(v[x] & 0xFFFFu);
                        w[8 * i + 2 * x + 1] = (uint16_t)(v[x] >> 16);
                    }
                }
            }
            if (KIND != CRISP_SAL_MAG) {
#pragma unroll
                for (int i = 0; i < CPT / 4; ++i) {
                    const f32x4 v = *reinterpret_cast<const f32x4*>(TG + e0 + 4 * i);
#pragma unroll
                    for (int x = 0; x < 4; ++x) tg[4 * i + x] = v[x];
                }
            }
        } else {
#pragma unroll
            for (int i = 0; i < CPT; ++i) {
                w[i] = (KIND != CRISP_SAL_GIVEN && i < len) ? W[e0 + i] : (uint16_t)0;
                tg[i] = (KIND != CRISP_SAL_MAG && i < len) ? TG[e0 + i] : 0.0f;
            }
        }
        float kept_t[CPT];
#pragma unroll
        for (int g = 0; g < CPT / M; ++g) {
            float t[M];
#pragma unroll
            for (int i = 0; i < M; ++i) t[i] = saliency_of<KIND>(w[g * M + i], tg[g * M + i]);
            const int glen = len - g * M;
#pragma unroll
            for (int i = 0; i < M; ++i) {
                int before = 0;
#pragma unroll
                for (int j = 0; j < M; ++j) before += (j < glen) && (t[j] > t[i] || (t[j] == t[i] && j < i));
                const bool kept = (i < glen) && (before < n);
                bits |= (kept ? 1u : 0u) << (g * M + i);
                kept_t[g * M + i] = kept ? t[i] : 0.0f;
            }
        }
#pragma unroll
        for (int i = 0; i < CPT / 4; ++i) {
            const f32x4 v = {kept_t[4 * i], kept_t[4 * i + 1], kept_t[4 * i + 2], kept_t[4 * i + 3]};
            *reinterpret_cast<f32x4*>(&tkept[r * LDT + c0 + 4 * i]) = v;
        }
    }
    // mask: the Q lanes of a row hold 16 bits each; pairs of lanes form one 32-bit word
    if (Q >= 2) {
        uint32_t word = bits << ((q & 1) * 16);
        word |= __shfl_xor(word, 1, 64);
        const int widx = (bj * B + c0) >> 5;
        if ((q & 1) == 0 && s < S && widx < mwpr) nm_mask[(size_t)s * mwpr + widx] = word;
    } else if (s < S) {
        // B == 16: two blocks share a mask word; each writes its own half
        uint16_t* half = reinterpret_cast<uint16_t*>(nm_mask) + ((size_t)s * mwpr) * 2;
        const int h = (bj * B) >> 4;
        half[h] = (uint16_t)bits;
        // an odd number of block columns leaves the upper half of the last word to nobody
        if (bj == Kb - 1 && (h & 1) == 0) half[h + 1] = 0;
    }
    __syncthreads();
    if (threadIdx.x < B) {
        const int row = threadIdx.x;
        double acc = 0.0;
#pragma unroll
        for (int i = 0; i < B / 4; ++i) {
            const f32x4 v = *reinterpret_cast<const f32x4*>(&tkept[row * LDT + 4 * i]);
            acc = __dadd_rn(acc, (double)v[0]);
            acc = __dadd_rn(acc, (double)v[1]);
            acc = __dadd_rn(acc, (double)v[2]);
            acc = __dadd_rn(acc, (double)v[3]);
        }
        rowsum[row] = acc;
    }
    __syncthreads();
    if (threadIdx.x == 0) {
        double part[B];
#pragma unroll
        for (int i = 0; i < B; ++i) part[i] = rowsum[i];
        double total = 0.0;
#pragma unroll
        for (int i = 0; i < B; ++i) total = __dadd_rn(total, part[i]);
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

template <int B, int M, int KIND>
static void launch_score_select(const Geometry& g, const uint16_t* W, const float* TG, uint32_t* nm_mask,
                                double* score, hipStream_t st) {
    const dim3 grd(g.Kb, g.Sb);
    if (g.K % B == 0)
        score_select_kernel<B, M, KIND, true><<<grd, B * (B / 16), 0, st>>>(g.S, g.K, g.n, g.Kb, g.mwpr, W, TG, nm_mask, score);
    else
        score_select_kernel<B, M, KIND, false><<<grd, B * (B / 16), 0, st>>>(g.S, g.K, g.n, g.Kb, g.mwpr, W, TG, nm_mask, score);
}

template <int KIND>
static hipError_t launch_select_kind(const Geometry& g, int select_mode, const uint16_t* W, const float* TG,
                                     uint32_t* nm_mask, int32_t* row_ptr, int32_t* col_idx, double* score,
                                     hipStream_t st) {
    const int key = g.B * 16 + g.m;
    switch (key) {
        case 64 * 16 + 4: launch_score_select<64, 4, KIND>(g, W, TG, nm_mask, score, st); break;
        case 64 * 16 + 8: launch_score_select<64, 8, KIND>(g, W, TG, nm_mask, score, st); break;
        case 32 * 16 + 4: launch_score_select<32, 4, KIND>(g, W, TG, nm_mask, score, st); break;
        case 32 * 16 + 8: launch_score_select<32, 8, KIND>(g, W, TG, nm_mask, score, st); break;
        case 16 * 16 + 4: launch_score_select<16, 4, KIND>(g, W, TG, nm_mask, score, st); break;
        default: launch_score_select<16, 8, KIND>(g, W, TG, nm_mask, score, st); break;
    }
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
