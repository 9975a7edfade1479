// Mask selection kernels: saliency -> N:M choice -> block scores -> block choice.
// Alg. 1 lines 2, 4-6 and 10 of the CRISP paper; every ordering decision below is a total
// order so that the result is unique and reproducible bit for bit.
#include "select_lane.h"

namespace crisp {

// One workgroup per B x B block, Q lanes per block row (Q * CPT = B columns, CPT = 16).
// Each lane loads its CPT weights (and gradient / saliency values) with 16-byte loads, ranks
// every aligned group of M columns (keep the n first under: larger saliency first, on a tie the
// smaller column first), and leaves "saliency if kept else +0" in LDS.  The Q lanes of a row
// OR their mask bits together with xor-shuffles.  Then lane r of the first wave adds row r's B
// values left to right in fp64 and lane 0 adds the row sums top to bottom: that summation order
// is part of the definition of the block score (a tree reduction would round differently;
// adding +0.0 for a pruned element leaves the non-negative running sum unchanged bit for bit).
// VEC: row segments are 16-byte aligned and lie wholly inside the matrix (K % B == 0).
// PACK: while the block's weights and keep bits are in registers, its packed form (compressed
// values, position stream, 2-of-4 violation) is also written, to a staging area indexed by the
// block's place in the grid; whether the block is kept is only known after the block choice,
// which then just copies the kept blocks' packed forms to their final place (topk_gather_kernel).
// Up to SEL_BATCH layers of equal (B, m, saliency kind, alignment class) share one launch: a
// model's layers have block grids of a few dozen to a few hundred workgroups each, far too few to
// fill 256 compute units one layer at a time.  Workgroup ids are mapped to (layer, block) through
// the prefix sums in `first`.
template <int B, int M, int KIND, bool VEC, bool PACK>
__global__ __launch_bounds__(B * (B / 16)) void score_select_kernel(SelBatch bt) {
    int li = 0;
#pragma unroll
    for (int i = 1; i < SEL_BATCH; ++i) li += (i < bt.n && (int)blockIdx.x >= bt.first[i]);
    const SelLayer& sa = bt.L[li];
    const int S = sa.S, K = sa.K, n = sa.n, Kb = sa.Kb, mwpr = sa.mwpr;
    const uint16_t* __restrict__ W = sa.W;
    const float* __restrict__ TG = sa.TG;
    uint32_t* __restrict__ nm_mask = sa.nm_mask;
    double* __restrict__ score = sa.score;
    constexpr int CPT = LANE_COLS;   // columns per lane
    constexpr int Q = B / CPT;       // lanes per block row (1, 2 or 4)
    constexpr int LDT = B + 4;       // padded LDS row stride in floats (keeps 16-byte alignment)
    constexpr int WMAX = (B * 3 + 31) / 32;   // upper bound of position words per block row
    constexpr int NTHR = B * (B / 16);
    __shared__ __attribute__((aligned(16))) float tkept[B * LDT];
    __shared__ double rowsum[B];
    __shared__ uint32_t pos_lds[PACK ? B * WMAX : 1];
    __shared__ int viol_lds;
    const int local = (int)blockIdx.x - bt.first[li];
    const int bi = local / Kb, bj = local - bi * Kb;
    const int r = threadIdx.x / Q, q = threadIdx.x % Q;
    const int s = bi * B + r;
    const int c0 = q * CPT;                      // first column of this lane inside the block
    const int k0 = bj * B + c0;
    if constexpr (PACK) {
        for (int e = threadIdx.x; e < B * WMAX; e += NTHR) pos_lds[e] = 0u;
        if (threadIdx.x == 0) {
            viol_lds = 0;
            if (bi == 0 && bj == 0) { sa.flags[0] = 1; sa.flags[1] = 0; sa.flags[2] = 0; sa.flags[3] = 0; }
        }
        __syncthreads();
    }
    uint32_t bits;
    {
        constexpr bool NEEDW = PACK || KIND != CRISP_SAL_GIVEN;
        const int len = (s < S) ? min(CPT, K - k0) : 0;   // columns of this lane that exist (may be <= 0)
        LaneRaw raw;
        lane_load<KIND, VEC, NEEDW>(raw, W, TG, (size_t)min(s, S - 1) * K, k0, K);
        bits = lane_select<M, KIND, NEEDW, true>(raw, n, len, &tkept[r * LDT + c0]);
        if constexpr (PACK) {
            // packed form of the lane's groups, to the staging area of block (bi, bj)
            const size_t blk = (size_t)bi * Kb + bj;
            const int slot0 = (c0 / M) * n;
            uint16_t* sv = sa.st_vals + (blk * B + r) * sa.slots + slot0;
            uint16_t w[CPT];
            lane_weights(raw, len, w);
            if (lane_pack<M>(w, bits, n, sa.wbits, s >= S, k0, K, sv, pos_lds + r * WMAX, slot0, WMAX)) viol_lds = 1;
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
        if constexpr (PACK) sa.st_viol[(size_t)bi * Kb + bj] = viol_lds;
    }
    if constexpr (PACK) {
        uint32_t* dst = sa.st_idxw + ((size_t)bi * Kb + bj) * B * sa.wpr;
        for (int e = threadIdx.x; e < B * sa.wpr; e += NTHR) dst[e] = pos_lds[(e / sa.wpr) * WMAX + e % sa.wpr];
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

// One launch of the scoring kernel for a batch whose layers share (B, m, kind, vec).
template <int KIND, bool PACK>
static void launch_score_batch(int B, int m, bool vec, const SelBatch& bt, hipStream_t st) {
    const unsigned grid = (unsigned)bt.first[bt.n];
    if (grid == 0) return;
#define CRISP_SCORE_CASE(BB, MM)                                                                       \
    if (vec) score_select_kernel<BB, MM, KIND, true, PACK><<<grid, BB * (BB / 16), 0, st>>>(bt);          \
    else score_select_kernel<BB, MM, KIND, false, PACK><<<grid, BB * (BB / 16), 0, st>>>(bt);
    switch (B * 16 + m) {
        case 64 * 16 + 4: CRISP_SCORE_CASE(64, 4) break;
        case 64 * 16 + 8: CRISP_SCORE_CASE(64, 8) break;
        case 32 * 16 + 4: CRISP_SCORE_CASE(32, 4) break;
        case 32 * 16 + 8: CRISP_SCORE_CASE(32, 8) break;
        case 16 * 16 + 4: CRISP_SCORE_CASE(16, 4) break;
        default: CRISP_SCORE_CASE(16, 8) break;
    }
#undef CRISP_SCORE_CASE
}

template <bool PACK>
static void launch_score_kind(int sal_kind, int B, int m, bool vec, const SelBatch& bt, hipStream_t st) {
    if (sal_kind == CRISP_SAL_GIVEN) launch_score_batch<CRISP_SAL_GIVEN, PACK>(B, m, vec, bt, st);
    else if (sal_kind == CRISP_SAL_GRAD) launch_score_batch<CRISP_SAL_GRAD, PACK>(B, m, vec, bt, st);
    else launch_score_batch<CRISP_SAL_MAG, PACK>(B, m, vec, bt, st);
}

static SelLayer sel_layer_of(const Geometry& g, const uint16_t* W, const float* TG, uint32_t* nm_mask, double* score) {
    SelLayer L = {};
    L.S = g.S; L.K = g.K; L.n = g.n; L.Kb = g.Kb; L.Sb = g.Sb; L.mwpr = g.mwpr; L.k_row = g.k_row;
    L.wbits = g.w; L.slots = g.slots; L.wpr = g.wpr;
    L.W = W; L.TG = TG; L.nm_mask = nm_mask; L.score = score;
    return L;
}

hipError_t launch_select(const Geometry& g, int sal_kind, int select_mode, const uint16_t* W, const float* TG,
                         uint32_t* nm_mask, int32_t* row_ptr, int32_t* col_idx, double* score, hipStream_t st) {
    SelBatch bt = {};
    bt.n = 1;
    bt.L[0] = sel_layer_of(g, W, TG, nm_mask, score);
    bt.first[1] = g.Sb * g.Kb;
    launch_score_kind<false>(sal_kind, g.B, g.m, g.K % g.B == 0, bt, st);
    if (select_mode == CRISP_ROW_UNIFORM)
        block_topk_rows_kernel<<<g.Sb, 256, 0, st>>>(g.Sb, g.Kb, g.k_row, score, row_ptr, col_idx);
    else
        block_topk_layer_kernel<<<1, 1024, 0, st>>>(g.Sb, g.Kb, g.Sb * g.k_row, score, row_ptr, col_idx);
    return hipGetLastError();
}

// Second half of the fused select + pack (uniform rows): the workgroup of kept block (bi, t)
// works out the block choice of block-row bi on its own (k_row blocks first under score
// descending, column ascending; the Kb scores are few, so doing this once per kept block costs
// less than a launch), takes the t-th kept column in ascending order and copies that block's
// packed form from the staging area to its final place.  Results are identical to
// crisp_select_mask followed by crisp_pack.
__global__ __launch_bounds__(256) void topk_gather_kernel(SelBatch bt, int B) {
    __shared__ double sc[512];
    __shared__ uint8_t kept[512];
    __shared__ int sel;
    int li = 0;
#pragma unroll
    for (int i = 1; i < SEL_BATCH; ++i) li += (i < bt.n && (int)blockIdx.x >= bt.firstk[i]);
    const SelLayer& L = bt.L[li];
    const int local = (int)blockIdx.x - bt.firstk[li];
    const int Kb = L.Kb, k_row = L.k_row, Sb = L.Sb;
    const int bi = local / k_row, t = local - bi * k_row, tid = threadIdx.x;
    const int vbytes = B * L.slots * 2, ibytes = B * L.wpr * 4;
    for (int j = tid; j < Kb; j += 256) sc[j] = L.score[(size_t)bi * Kb + j];
    __syncthreads();
    for (int j = tid; j < Kb; j += 256) {
        const double mine = sc[j];
        int before = 0;
        for (int o = 0; o < Kb; ++o) before += (sc[o] > mine) || (sc[o] == mine && o < j);
        kept[j] = before < k_row;
    }
    __syncthreads();
    for (int j = tid; j < Kb; j += 256) {
        if (kept[j]) {
            int pos = 0;
            for (int o = 0; o < j; ++o) pos += kept[o];
            if (pos == t) sel = j;
        }
    }
    __syncthreads();
    const int bj = sel;
    const size_t src = (size_t)bi * Kb + bj, dst = (size_t)bi * k_row + t;
    const u32x4* sv = reinterpret_cast<const u32x4*>(reinterpret_cast<const unsigned char*>(L.st_vals) + src * vbytes);
    u32x4* dv = reinterpret_cast<u32x4*>(reinterpret_cast<unsigned char*>(L.vals) + dst * vbytes);
    for (int e = tid; e < vbytes / 16; e += 256) dv[e] = sv[e];
    const u32x4* si = reinterpret_cast<const u32x4*>(reinterpret_cast<const unsigned char*>(L.st_idxw) + src * ibytes);
    u32x4* di = reinterpret_cast<u32x4*>(reinterpret_cast<unsigned char*>(L.idxw) + dst * ibytes);
    for (int e = tid; e < ibytes / 16; e += 256) di[e] = si[e];
    if (tid == 0) {
        L.col_idx[dst] = bj;
        if (t == 0) {
            L.row_ptr[bi] = bi * k_row;
            if (bi == Sb - 1) L.row_ptr[Sb] = Sb * k_row;
        }
        if (L.clear_flag && L.st_viol[src] && L.flags[0] != 0) atomicAnd(L.flags, 0);
    }
}

bool select_pack_fusable(const Geometry& g, int select_mode) {
    return select_mode == CRISP_ROW_UNIFORM && g.Kb <= 512 && g.nk > 0;
}

size_t select_pack_stage_bytes(const Geometry& g) {
    const size_t blocks = (size_t)g.Sb * g.Kb;
    const size_t viol = (blocks * sizeof(int32_t) + 15) / 16 * 16;
    return viol + blocks * g.B * g.slots * 2 + blocks * g.B * g.wpr * 4;
}

// Fused selection + packing of up to SEL_BATCH layers that share (B, m, saliency kind, alignment
// class) in two launches.  stage[i]: select_pack_stage_bytes(g[i]) bytes, 16-byte aligned.
hipError_t launch_select_pack_batch(int n, const Geometry* g, int sal_kind, const SelPackPtrs* pp, hipStream_t st) {
    SelBatch bt = {};
    bt.n = n;
    for (int i = 0; i < n; ++i) {
        const size_t blocks = (size_t)g[i].Sb * g[i].Kb;
        unsigned char* base = static_cast<unsigned char*>(pp[i].stage);
        SelLayer L = sel_layer_of(g[i], pp[i].W, pp[i].TG, pp[i].nm_mask, pp[i].score);
        L.st_viol = reinterpret_cast<int32_t*>(base);
        base += (blocks * sizeof(int32_t) + 15) / 16 * 16;
        L.st_vals = reinterpret_cast<uint16_t*>(base);
        base += blocks * g[i].B * g[i].slots * 2;
        L.st_idxw = reinterpret_cast<uint32_t*>(base);
        L.flags = pp[i].flags; L.row_ptr = pp[i].row_ptr; L.col_idx = pp[i].col_idx; L.vals = pp[i].vals; L.idxw = pp[i].idxw;
        // n <= 2 can never put three kept elements into an aligned group of four
        L.clear_flag = g[i].n > 2;
        bt.L[i] = L;
        bt.first[i + 1] = bt.first[i] + g[i].Sb * g[i].Kb;
        bt.firstk[i + 1] = bt.firstk[i] + g[i].nk;
    }
    launch_score_kind<true>(sal_kind, g[0].B, g[0].m, g[0].K % g[0].B == 0, bt, st);
    if (bt.firstk[n] > 0) topk_gather_kernel<<<(unsigned)bt.firstk[n], 256, 0, st>>>(bt, g[0].B);
    return hipGetLastError();
}

}  // namespace crisp
