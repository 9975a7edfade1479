// Global block budget across layers (Alg. 1 lines 6-9, Sec. 3.3): per-row ascending order of
// the block scores, rank-column sums, one global ascending order over all layers, pruning of
// rank columns until the target sparsity is reached.  The outcome per layer is the number of
// kept blocks per block-row.  Everything is tiny (a few thousand numbers), so one workgroup does
// it; the arithmetic and every tie rule are fixed so that the result is reproducible bit for bit.
#include "crisp_internal.h"

namespace crisp {

__global__ __launch_bounds__(1024) void global_budget_kernel(BudgetArgs a, double* __restrict__ sorted_ws,
                                                             int32_t* __restrict__ k_row_out,
                                                             double* __restrict__ achieved) {
    __shared__ double c[CRISP_BUDGET_MAX_COLS];      // rank-column sums
    __shared__ double w[CRISP_BUDGET_MAX_COLS];      // kept weights a rank column holds
    __shared__ uint16_t lay[CRISP_BUDGET_MAX_COLS];  // layer of a rank column
    __shared__ uint16_t order[CRISP_BUDGET_MAX_COLS];
    __shared__ int k_row[CRISP_BUDGET_MAX_LAYERS];
    __shared__ int col0[CRISP_BUDGET_MAX_LAYERS + 1];
    const int tid = threadIdx.x;
    if (tid == 0) {
        int pos = 0;
        for (int l = 0; l < a.L; ++l) { col0[l] = pos; pos += a.Kb[l]; k_row[l] = a.Kb[l]; }
        col0[a.L] = pos;
    }
    __syncthreads();
    const int ncols = col0[a.L];
    for (int x = tid; x < ncols; x += 1024) { c[x] = 0.0; w[x] = 0.0; }
    // 1. ascending position of every block inside its block-row (exact reverse of the keep order:
    //    score ascending, on a tie the larger column first); scores re-ordered into the workspace
    size_t ws0 = 0;
    for (int l = 0; l < a.L; ++l) {
        const int Sb = a.Sb[l], Kb = a.Kb[l];
        const double* sc = a.score[l];
        for (int e = tid; e < Sb * Kb; e += 1024) {
            const int bi = e / Kb, j = e - bi * Kb;
            const double mine = sc[e];
            int before = 0;
            for (int o = 0; o < Kb; ++o) {
                const double other = sc[bi * Kb + o];
                before += (other < mine) || (other == mine && o > j);
            }
            sorted_ws[ws0 + (size_t)bi * Kb + before] = mine;
            // kept weights of this block: in-range rows x in-range columns x n/m (a dyadic
            // rational, so the fp64 sums below are exact in any order)
            const int rows = min(a.B[l], a.S[l] - bi * a.B[l]);
            const int cols = min(a.B[l], a.K[l] - j * a.B[l]);
            atomicAdd(&w[col0[l] + before], (double)rows * (double)cols * (double)a.n[l] / (double)a.m[l]);
        }
        ws0 += (size_t)Sb * Kb;
    }
    __threadfence_block();
    __syncthreads();
    // 2. rank-column sums, block-rows ascending, fp64
    ws0 = 0;
    for (int l = 0; l < a.L; ++l) {
        const int Sb = a.Sb[l], Kb = a.Kb[l];
        for (int o = tid; o < Kb; o += 1024) {
            double s = 0.0;
            for (int bi = 0; bi < Sb; ++bi) s = __dadd_rn(s, sorted_ws[ws0 + (size_t)bi * Kb + o]);
            c[col0[l] + o] = s;
            lay[col0[l] + o] = (uint16_t)l;
        }
        ws0 += (size_t)Sb * Kb;
    }
    __syncthreads();
    // 3. one ascending order over all rank columns: (sum, layer, rank) -- the flat index already
    //    runs layer-major, rank-minor
    for (int x = tid; x < ncols; x += 1024) {
        const double mine = c[x];
        int before = 0;
        for (int o = 0; o < ncols; ++o) before += (c[o] < mine) || (c[o] == mine && o < x);
        order[before] = (uint16_t)x;
    }
    __syncthreads();
    // 4. prune in that order until the target is reached; never a layer's last rank column
    if (tid == 0) {
        double total = 0.0, kept = 0.0;
        for (int l = 0; l < a.L; ++l) {
            total += (double)a.S[l] * (double)a.K[l];
            kept += (double)a.S[l] * (double)a.K[l] * (double)a.n[l] / (double)a.m[l];
        }
        for (int r = 0; r < ncols && 1.0 - kept / total < a.target; ++r) {
            const int x = order[r];
            const int l = lay[x];
            if (k_row[l] <= 1) continue;
            kept -= w[x];
            k_row[l] -= 1;
        }
        for (int l = 0; l < a.L; ++l) k_row_out[l] = k_row[l];
        if (achieved) achieved[0] = 1.0 - kept / total;
    }
}

hipError_t launch_global_budget(const BudgetArgs& a, double* ws, int32_t* k_row, double* achieved, hipStream_t st) {
    global_budget_kernel<<<1, 1024, 0, st>>>(a, ws, k_row, achieved);
    return hipGetLastError();
}

}  // namespace crisp
