// What one lane does with its 16 consecutive columns of one weight row inside a B x B block:
// load, saliency, N:M choice, and the packed form of its groups.  Shared by the selection kernels
// (Alg. 1 lines 2 and 4-5; storage format of Sec. 3.1 / 3.5).
#pragma once
#include "crisp_internal.h"

namespace crisp {

typedef __attribute__((ext_vector_type(4))) uint32_t u32x4;
typedef __attribute__((ext_vector_type(4))) float f32x4;

#define SEL_BATCH CRISP_SELECT_BATCH
// One layer of a batched selection launch.
struct SelLayer {
    int S, K, n, Kb, Sb, mwpr, k_row, clear_flag;
    int wbits, slots, wpr, pad_;  // bits per position, packed slots and position words per block row
    const uint16_t* W;
    const float* TG;
    uint32_t* nm_mask;
    double* score;
    uint16_t* st_vals;            // staging [Sb*Kb][B][slots]
    uint32_t* st_idxw;            // staging [Sb*Kb][B][wpr]
    int32_t* st_viol;             // staging [Sb*Kb]: an aligned group of four holds more than two kept
    int32_t* flags;               // the layer's flags
    int32_t* row_ptr;
    int32_t* col_idx;
    uint16_t* vals;
    uint32_t* idxw;
};
struct SelBatch {
    int n;
    int first[SEL_BATCH + 1];     // first workgroup of each layer in the scoring launch
    int firstk[SEL_BATCH + 1];    // first workgroup of each layer in the gather launch (kept blocks)
    SelLayer L[SEL_BATCH];
};

constexpr int LANE_COLS = 16;     // columns per lane

// Saliency of one element (Sec. 3.4, Eq. 1): one fp32 multiply, then the absolute value.
template <int KIND>
__device__ __forceinline__ float saliency_of(uint16_t w, float tg) {
    if (KIND == CRISP_SAL_GIVEN) return tg;
    if (KIND == CRISP_SAL_GRAD) return fabsf(__fmul_rn(bf16_bits_to_float(w), tg));
    return fabsf(bf16_bits_to_float(w));
}

// The lane's columns as they come from memory (kept in this form until used, so that the loads
// can stay in flight).
struct LaneRaw {
    u32x4 w[LANE_COLS / 8];
    f32x4 tg[LANE_COLS / 4];
};

// row_base: element offset of the start of a row that exists; k0: first column of the lane.
// VEC: the segment is 16-byte aligned and lies wholly inside the row.  Otherwise element loads;
// a column at or past K re-reads column K - 1 (the caller zeroes it afterwards), so every address
// is valid and the instruction stream has no branch.
template <int KIND, bool VEC, bool NEEDW>
__device__ __forceinline__ void lane_load(LaneRaw& d, const uint16_t* __restrict__ W, const float* __restrict__ TG,
                                          size_t row_base, int k0, int K) {
    if (VEC) {
        if (NEEDW) {
#pragma unroll
            for (int i = 0; i < LANE_COLS / 8; ++i) d.w[i] = *reinterpret_cast<const u32x4*>(W + row_base + k0 + 8 * i);
        }
        if (KIND != CRISP_SAL_MAG) {
#pragma unroll
            for (int i = 0; i < LANE_COLS / 4; ++i) d.tg[i] = *reinterpret_cast<const f32x4*>(TG + row_base + k0 + 4 * i);
        }
    } else {
#pragma unroll
        for (int i = 0; i < LANE_COLS; ++i) {
            const size_t e = row_base + (size_t)min(k0 + i, K - 1);
            if (NEEDW) {
                const uint32_t v = W[e];
                if (i & 1) d.w[i / 8][(i % 8) / 2] |= v << 16;
                else d.w[i / 8][(i % 8) / 2] = v;
            }
            if (KIND != CRISP_SAL_MAG) d.tg[i / 4][i % 4] = TG[e];
        }
    }
}

// The lane's weights as values; those at or past `len` (<= 0 for a lane outside the matrix) are zero.
__device__ __forceinline__ void lane_weights(const LaneRaw& d, int len, uint16_t (&w)[LANE_COLS]) {
#pragma unroll
    for (int i = 0; i < LANE_COLS; ++i) {
        const uint32_t pair = d.w[i / 8][(i % 8) / 2];
        w[i] = (i < len) ? (uint16_t)((i & 1) ? (pair >> 16) : (pair & 0xFFFFu)) : (uint16_t)0;
    }
}

// N:M choice in every aligned group of M columns: keep the n first under (larger saliency first,
// on a tie the smaller column first); columns at or past `len` do not exist.  Returns the keep
// bits; STORE: also leaves "saliency if kept else +0" of the 16 columns at kept_dst (LDS, 16-byte
// aligned), group by group, so that only one group's values are live at a time.
// Every pair of columns is compared once: column i (< j) comes before j when t[i] >= t[j];
// a column is kept when it comes before at least M - n others.  Columns that do not exist carry
// -inf and, having the larger numbers, lose every comparison against one that exists.
template <int M, int KIND, bool NEEDW, bool STORE>
__device__ __forceinline__ uint32_t lane_select(const LaneRaw& d, int n, int len, float* kept_dst) {
    uint32_t bits = 0;
#pragma unroll
    for (int g = 0; g < LANE_COLS / M; ++g) {
        float t[M], kept_t[M];
        int wins[M];
#pragma unroll
        for (int i = 0; i < M; ++i) {
            const int c = g * M + i;
            const uint32_t pair = NEEDW ? d.w[c / 8][(c % 8) / 2] : 0u;
            const uint16_t w = (uint16_t)((c & 1) ? (pair >> 16) : (pair & 0xFFFFu));
            const float tg = (KIND != CRISP_SAL_MAG) ? d.tg[c / 4][c % 4] : 0.0f;
            t[i] = (c < len) ? saliency_of<KIND>(w, tg) : -__builtin_inff();
            wins[i] = 0;
        }
#pragma unroll
        for (int i = 0; i < M; ++i) {
#pragma unroll
            for (int j = i + 1; j < M; ++j) {
                const int first = t[i] >= t[j] ? 1 : 0;
                wins[i] += first;
                wins[j] += 1 - first;
            }
        }
#pragma unroll
        for (int i = 0; i < M; ++i) {
            const bool kept = (g * M + i < len) & (wins[i] >= M - n);
            bits |= (kept ? 1u : 0u) << (g * M + i);
            kept_t[i] = kept ? t[i] : 0.0f;
        }
        if (STORE) {
#pragma unroll
            for (int i = 0; i < M / 4; ++i) {
                const f32x4 v = {kept_t[4 * i], kept_t[4 * i + 1], kept_t[4 * i + 2], kept_t[4 * i + 3]};
                *reinterpret_cast<f32x4*>(kept_dst + g * M + 4 * i) = v;
            }
        }
    }
    return bits;
}

__device__ __forceinline__ uint32_t slot_position_of(uint32_t bits, int j, bool outside) {
    // j-th kept column of the group; 0 when the group holds fewer; j for a group outside the matrix
    if (outside) return (uint32_t)j;
    for (int i = 0; i < j; ++i) bits &= bits - 1u;
    return bits ? (uint32_t)(__ffs(bits) - 1) : 0u;
}

// Packed form of the lane's LANE_COLS / M groups: n slots each, kept values in ascending column
// order, then zeros, stored at sv; positions per the canonical rules, OR-ed into the block row's
// position words in LDS (prow, zeroed beforehand, `wmax` words).  slot0: first slot of the lane in
// its block row; row_outside: the weight row does not exist; k0: first column of the lane.
// Returns whether an aligned group of four columns holds more than two kept elements.
template <int M>
__device__ __forceinline__ bool lane_pack(const uint16_t (&w)[LANE_COLS], uint32_t bits, int n, int wbits, bool row_outside,
                                          int k0, int K, uint16_t* sv, uint32_t* prow, int slot0, int wmax) {
    uint64_t stream = 0;                 // at most 16 slots x 3 bits
    int nb = 0;
    bool violates = false;
#pragma unroll
    for (int g = 0; g < LANE_COLS / M; ++g) {
        const uint32_t gb = (bits >> (g * M)) & ((1u << M) - 1u);
        const bool outside = row_outside || (k0 + g * M >= K);
        uint16_t v[M];
#pragma unroll
        for (int x = 0; x < M; ++x) v[x] = 0;
        int filled = 0;
#pragma unroll
        for (int o = 0; o < M; ++o) {
            const bool on = (gb >> o) & 1u;
#pragma unroll
            for (int x = 0; x < M; ++x)
                if (on && filled == x) v[x] = w[g * M + o];
            filled += on;
        }
#pragma unroll
        for (int x = 0; x < M; ++x) {
            if (x < n) {
                sv[g * n + x] = v[x];
                stream |= (uint64_t)slot_position_of(gb, x, outside) << nb;
                nb += wbits;
            }
        }
        violates = violates || __popc(gb & 0xFu) > 2 || __popc(gb >> 4) > 2;
    }
    const int bit0 = slot0 * wbits, wi = bit0 >> 5, sh = bit0 & 31;
    const uint32_t p0 = (uint32_t)(stream << sh);
    const uint32_t p1 = (uint32_t)(sh ? (stream >> (32 - sh)) : (stream >> 32));
    const uint32_t p2 = (uint32_t)(sh ? (stream >> (64 - sh)) : 0u);
    if (p0) atomicOr(prow + wi, p0);
    if (p1 && wi + 1 < wmax) atomicOr(prow + wi + 1, p1);
    if (p2 && wi + 2 < wmax) atomicOr(prow + wi + 2, p2);
    return violates;
}

}  // namespace crisp
