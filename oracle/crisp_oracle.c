/*
 * CRISP hybrid-sparsity oracle -- TEST INFRASTRUCTURE, NOT A PRODUCT PATH.
 *
 * A plain, slow, obviously-correct CPU statement of what the hybrid-sparse
 * (block AND N:M) inference path of CRISP (arXiv 2311.14272) computes.  Only
 * the test-suite, the smoke check and the benchmark's cpu_baseline leg may
 * call it.  It shares no code with the HIP library: nothing here is included
 * by, linked into or generated for the GPU path, and nothing of the GPU path
 * is used here.
 *
 * All floating point is fp64 except the saliency product, which the method
 * takes in fp32 (one multiply, one rounding) because the selection that
 * follows compares those fp32 numbers.
 *
 * Orientation (Sec. 3 "Notation" together with Sec. 3.1): the reshaped weight
 * has S rows (output channels) and K = kh*kw*C columns (reduction dimension).
 * N:M groups run along K inside one row; blocks are B x B tiles of that S x K
 * matrix; the uniform count of pruned blocks per row that Sec. 3.1 requires is
 * taken per row of the block grid.
 *
 * Every function returns 0 on success and a negative number on bad arguments.
 *
 * Parity pins: every function below is pinned by tests/test_oracle_*.py
 * (brute force, invariants, closed forms of Sec. 3.1, library fp64 matmul,
 * exact rational sums, the worked index example of Sec. 3.5).
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>

static float bf16_to_f32(uint16_t h)
{
    uint32_t u = (uint32_t)h << 16;
    float f;
    memcpy(&f, &u, sizeof f);
    return f;
}

static int ceil_div(int a, int b) { return (a + b - 1) / b; }

static int log2_exact(int m)
{
    int w = 0;
    while ((1 << w) < m) ++w;
    return w;
}

/* ------------------------------------------------------------------------
 * Saliency (Sec. 3.4, Eq. 1).  T = |grad * W|; the 1/H averaging factor is a
 * positive constant that cannot change any ranking and is left out.
 * kind 0: T is given (copied); kind 1: T = |W*G| in fp32; kind 2: T = |W|.
 * ---------------------------------------------------------------------- */
int oracle_saliency(int S, int K, int kind, const uint16_t *W, const float *G_or_T, float *T)
{
    if (S < 1 || K < 1 || !T) return -1;
    if (kind != 2 && !G_or_T) return -1;
    if (kind != 0 && !W) return -1;
    for (long i = 0; i < (long)S * K; ++i) {
        if (kind == 0) {
            T[i] = G_or_T[i];
        } else if (kind == 1) {
            volatile float p = bf16_to_f32(W[i]) * G_or_T[i]; /* one fp32 rounding */
            T[i] = fabsf(p);
        } else if (kind == 2) {
            T[i] = fabsf(bf16_to_f32(W[i]));
        } else {
            return -1;
        }
    }
    return 0;
}

/* ------------------------------------------------------------------------
 * Fine-grained N:M pruning (Alg. 1 line 2; Sec. 3.1: at most N non-zeros in
 * every M consecutive elements).  In every aligned group of m consecutive
 * columns of a row the n most salient positions are kept.  Total order used:
 * larger T first, on equal T the smaller column first.  A short last group
 * (K not a multiple of m) keeps min(n, length) positions.
 * keep[s*K+k] is 1 for kept, 0 for pruned.
 * ---------------------------------------------------------------------- */
int oracle_nm_select(int S, int K, int n, int m, const float *T, uint8_t *keep)
{
    if (S < 1 || K < 1 || m < 1 || n < 1 || n > m || !T || !keep) return -1;
    for (int s = 0; s < S; ++s) {
        const float *t = T + (long)s * K;
        uint8_t *kp = keep + (long)s * K;
        for (int g0 = 0; g0 < K; g0 += m) {
            int len = (K - g0 < m) ? K - g0 : m;
            for (int i = 0; i < len; ++i) {
                int before = 0; /* how many group members precede i in the order */
                for (int j = 0; j < len; ++j) {
                    if (t[g0 + j] > t[g0 + i] || (t[g0 + j] == t[g0 + i] && j < i)) ++before;
                }
                kp[g0 + i] = (uint8_t)(before < n);
            }
        }
    }
    return 0;
}

/* Bit-packed form of the N:M keep map: S rows of ceil(K/32) words, bit (k%32)
 * of word k/32 set when column k of that row is kept. */
int oracle_keep_to_bits(int S, int K, const uint8_t *keep, uint32_t *bits)
{
    if (S < 1 || K < 1 || !keep || !bits) return -1;
    int wpr = ceil_div(K, 32);
    memset(bits, 0, (size_t)S * wpr * sizeof(uint32_t));
    for (int s = 0; s < S; ++s)
        for (int k = 0; k < K; ++k)
            if (keep[(long)s * K + k]) bits[(long)s * wpr + k / 32] |= (uint32_t)1 << (k % 32);
    return 0;
}

/* ------------------------------------------------------------------------
 * Block score (Alg. 1 lines 4-5): s_j = sum of |T| over the elements of block
 * j.  The saliency is evaluated after the N:M step and T = |g*w| vanishes on a
 * zeroed weight, so only N:M-kept elements contribute.  Summation order is
 * part of the definition: for each row of the block, columns ascending, in
 * fp64; then the row sums, rows ascending, in fp64.  Edge blocks sum the
 * in-range elements only.
 * ---------------------------------------------------------------------- */
int oracle_block_score(int S, int K, int B, const float *T, const uint8_t *keep, double *score)
{
    if (S < 1 || K < 1 || B < 1 || !T || !keep || !score) return -1;
    int Sb = ceil_div(S, B), Kb = ceil_div(K, B);
    for (int bi = 0; bi < Sb; ++bi) {
        for (int bj = 0; bj < Kb; ++bj) {
            double total = 0.0;
            for (int r = 0; r < B; ++r) {
                int s = bi * B + r;
                if (s >= S) break;
                double rowsum = 0.0;
                for (int c = 0; c < B; ++c) {
                    int k = bj * B + c;
                    if (k >= K) break;
                    if (keep[(long)s * K + k]) rowsum += (double)T[(long)s * K + k];
                }
                total += rowsum;
            }
            score[(long)bi * Kb + bj] = total;
        }
    }
    return 0;
}

/* Kept blocks per block-row for a target block density (the per-layer outcome
 * of Alg. 1 lines 7-9: a prefix of the ascending per-row ranks is dropped, the
 * same count in every row).  Never less than one block, so a layer cannot
 * collapse (Sec. 3.3, last paragraph). */
int oracle_k_row(double density, int Kb)
{
    if (!(density > 0.0) || density > 1.0 || Kb < 1) return -1;
    double v = floor(density * (double)Kb + 0.5);
    int k = (int)v;
    if (k < 1) k = 1;
    if (k > Kb) k = Kb;
    return k;
}

/* ------------------------------------------------------------------------
 * Uniform block pruning (Alg. 1 lines 6 and 10; Sec. 3.1 and 3.3: the same
 * number of pruned blocks in every row of the block grid).
 * mode 0: in each block-row keep the k_row blocks that come first under
 *         (score descending, column ascending).
 * mode 1: plain (non-uniform) block pruning, the baseline the paper contrasts
 *         with: keep the Sb*k_row best blocks of the whole grid under (score
 *         descending, block-row ascending, column ascending); rows may end up
 *         uneven or empty.
 * Output is Blocked-ELL / block-CSR (Sec. 3.1): row_ptr[Sb+1] and the kept
 * block columns of each row in ascending order ("row-major").
 * ---------------------------------------------------------------------- */
int oracle_block_select(int Sb, int Kb, int k_row, int mode, const double *score,
                        int32_t *row_ptr, int32_t *col_idx)
{
    if (Sb < 1 || Kb < 1 || k_row < 1 || k_row > Kb || !score || !row_ptr || !col_idx) return -1;
    long total = (long)Sb * Kb;
    uint8_t *kept = (uint8_t *)calloc((size_t)total, 1);
    if (!kept) return -2;
    if (mode == 0) {
        for (int bi = 0; bi < Sb; ++bi) {
            const double *sc = score + (long)bi * Kb;
            for (int j = 0; j < Kb; ++j) {
                int before = 0;
                for (int o = 0; o < Kb; ++o)
                    if (sc[o] > sc[j] || (sc[o] == sc[j] && o < j)) ++before;
                kept[(long)bi * Kb + j] = (uint8_t)(before < k_row);
            }
        }
    } else if (mode == 1) {
        long budget = (long)Sb * k_row;
        for (long a = 0; a < total; ++a) {
            long before = 0;
            for (long o = 0; o < total; ++o)
                if (score[o] > score[a] || (score[o] == score[a] && o < a)) ++before;
            kept[a] = (uint8_t)(before < budget);
        }
    } else {
        free(kept);
        return -1;
    }
    int32_t pos = 0;
    for (int bi = 0; bi < Sb; ++bi) {
        row_ptr[bi] = pos;
        for (int j = 0; j < Kb; ++j)
            if (kept[(long)bi * Kb + j]) col_idx[pos++] = j;
    }
    row_ptr[Sb] = pos;
    free(kept);
    return 0;
}

/* Final binary mask M_l (Sec. 3 "Notation"; Alg. 1 line 10, f <- f (.) r):
 * N:M keep map AND membership in a kept block. */
int oracle_dense_mask(int S, int K, int B, const uint8_t *keep, const int32_t *row_ptr,
                      const int32_t *col_idx, uint8_t *mask)
{
    if (S < 1 || K < 1 || B < 1 || !keep || !row_ptr || !col_idx || !mask) return -1;
    int Sb = ceil_div(S, B);
    memset(mask, 0, (size_t)S * K);
    for (int bi = 0; bi < Sb; ++bi)
        for (int t = row_ptr[bi]; t < row_ptr[bi + 1]; ++t) {
            int bj = col_idx[t];
            for (int r = 0; r < B && bi * B + r < S; ++r)
                for (int c = 0; c < B && bj * B + c < K; ++c) {
                    long e = (long)(bi * B + r) * K + bj * B + c;
                    mask[e] = keep[e];
                }
        }
    return 0;
}

/* ------------------------------------------------------------------------
 * Canonical packed form (Sec. 3.1 metadata paragraph; Sec. 3.5 second step).
 * For kept block t (in row_ptr/col_idx order), block row r, group g of m
 * columns: n slots.  Kept elements of the group fill the slots in ascending
 * column order; a slot stores the bf16 value and the 0-based position of the
 * value inside its group of m (log2 m bits; Sec. 3.5: the second place of a group is position 1).
 * Padding: a short group (K not a multiple of m) fills its unused slots with
 * value 0 and position 0; a group wholly outside the matrix (row >= S or
 * first column >= K) holds value 0 with positions 0..n-1.
 * vals  : [nk][B][B*n/m] bf16
 * idxw  : per block row a little-endian bit stream, slot q at bits
 *         [q*w, q*w+w), padded to whole 32-bit words; [nk][B][wpr] words.
 * flags : flags[0] = 1 when no aligned group of 4 columns inside any kept
 *         block holds more than 2 kept elements (the 2-of-4 hardware form).
 * ---------------------------------------------------------------------- */
int oracle_pack(int S, int K, int n, int m, int B, const uint16_t *W, const uint8_t *keep,
                const int32_t *row_ptr, const int32_t *col_idx, uint16_t *vals, uint32_t *idxw,
                int32_t *flags)
{
    if (S < 1 || K < 1 || n < 1 || n > m || (m != 4 && m != 8) || B % m != 0) return -1;
    if (!W || !keep || !row_ptr || !col_idx || !vals || !idxw || !flags) return -1;
    int Sb = ceil_div(S, B);
    int w = log2_exact(m);
    int slots = B / m * n;
    int wpr = ceil_div(slots * w, 32);
    int ok24 = 1;
    for (int bi = 0; bi < Sb; ++bi) {
        for (int t = row_ptr[bi]; t < row_ptr[bi + 1]; ++t) {
            int bj = col_idx[t];
            for (int r = 0; r < B; ++r) {
                int s = bi * B + r;
                uint16_t *vrow = vals + ((long)t * B + r) * slots;
                uint32_t *irow = idxw + ((long)t * B + r) * wpr;
                for (int x = 0; x < wpr; ++x) irow[x] = 0;
                for (int g = 0; g < B / m; ++g) {
                    int k0 = bj * B + g * m;
                    int q = g * n;
                    if (s >= S || k0 >= K) {
                        for (int j = 0; j < n; ++j) {
                            vrow[q + j] = 0;
                            long bit = (long)(q + j) * w;
                            irow[bit / 32] |= (uint32_t)j << (bit % 32);
                            if (bit % 32 + w > 32) irow[bit / 32 + 1] |= (uint32_t)j >> (32 - bit % 32);
                        }
                        continue;
                    }
                    int filled = 0;
                    for (int o = 0; o < m && k0 + o < K; ++o) {
                        if (!keep[(long)s * K + k0 + o]) continue;
                        if (filled >= n) return -3; /* keep map is not n:m */
                        vrow[q + filled] = W[(long)s * K + k0 + o];
                        long bit = (long)(q + filled) * w;
                        irow[bit / 32] |= (uint32_t)o << (bit % 32);
                        if (bit % 32 + w > 32) irow[bit / 32 + 1] |= (uint32_t)o >> (32 - bit % 32);
                        ++filled;
                    }
                    for (; filled < n; ++filled) vrow[q + filled] = 0; /* position bits stay 0 */
                    for (int h = 0; h < m; h += 4) {
                        int cnt = 0;
                        for (int o = h; o < h + 4 && k0 + o < K; ++o) cnt += keep[(long)s * K + k0 + o];
                        if (cnt > 2) ok24 = 0;
                    }
                }
            }
        }
    }
    flags[0] = ok24;
    return 0;
}

/* Inverse of oracle_pack: scatter the slots back to a dense S x K bf16 matrix
 * (zeros elsewhere).  A kept block sits where it sat in W (Sec. 3.3). */
int oracle_unpack(int S, int K, int n, int m, int B, const int32_t *row_ptr, const int32_t *col_idx,
                  const uint16_t *vals, const uint32_t *idxw, uint16_t *Wd)
{
    if (S < 1 || K < 1 || n < 1 || n > m || (m != 4 && m != 8) || B % m != 0) return -1;
    int Sb = ceil_div(S, B);
    int w = log2_exact(m);
    int slots = B / m * n;
    int wpr = ceil_div(slots * w, 32);
    memset(Wd, 0, (size_t)S * K * sizeof(uint16_t));
    for (int bi = 0; bi < Sb; ++bi)
        for (int t = row_ptr[bi]; t < row_ptr[bi + 1]; ++t) {
            int bj = col_idx[t];
            for (int r = 0; r < B && bi * B + r < S; ++r) {
                const uint16_t *vrow = vals + ((long)t * B + r) * slots;
                const uint32_t *irow = idxw + ((long)t * B + r) * wpr;
                for (int q = 0; q < slots; ++q) {
                    long bit = (long)q * w;
                    uint64_t two = irow[bit / 32];
                    if (bit / 32 + 1 < wpr) two |= (uint64_t)irow[bit / 32 + 1] << 32;
                    int off = (int)((two >> (bit % 32)) & (uint64_t)(m - 1));
                    int k = bj * B + (q / n) * m + off;
                    if (k < K && vrow[q] != 0) Wd[(long)(bi * B + r) * K + k] = vrow[q];
                }
            }
        }
    return 0;
}

/* ------------------------------------------------------------------------
 * The product itself, by its plain definition: Y* = (W (.) mask) X, fp64,
 * a triple loop over the dense masked weight, terms added in ascending k.
 * Also A* = |W (.) mask| |X| (the scale of the element-wise error bound).
 * X is K x ldx bf16 row-major; columns [c0, c0+nc) are computed and written
 * to Y/A as S x nc row-major.  OpenMP splits the columns only; every output
 * element is still one sequential sum.
 * ---------------------------------------------------------------------- */
int oracle_gemm_masked(int S, int K, const uint16_t *W, const uint8_t *mask, const uint16_t *X,
                       long ldx, long c0, long nc, double *Y, double *A)
{
    if (S < 1 || K < 1 || nc < 0 || !W || !mask || !X || !Y) return -1;
#pragma omp parallel for schedule(static)
    for (long j = 0; j < nc; ++j) {
        for (int s = 0; s < S; ++s) {
            double acc = 0.0, aacc = 0.0;
            for (int k = 0; k < K; ++k) {
                double wv = mask[(long)s * K + k] ? (double)bf16_to_f32(W[(long)s * K + k]) : 0.0;
                double xv = (double)bf16_to_f32(X[(long)k * ldx + c0 + j]);
                acc += wv * xv;
                aacc += fabs(wv) * fabs(xv);
            }
            Y[(long)s * nc + j] = acc;
            if (A) A[(long)s * nc + j] = aacc;
        }
    }
    return 0;
}

/* Same product computed from the packed structure (Sec. 3.5: block indices
 * pick the activation rows, in-group positions pick the activation inside
 * each group, then multiply-accumulate).  Kept blocks of a row ascending,
 * slots ascending: the same ascending-k order as the dense loop with the zero
 * terms left out. */
int oracle_spmm_packed(int S, int K, int n, int m, int B, const int32_t *row_ptr,
                       const int32_t *col_idx, const uint16_t *vals, const uint32_t *idxw,
                       const uint16_t *X, long ldx, long c0, long nc, double *Y)
{
    if (S < 1 || K < 1 || n < 1 || n > m || (m != 4 && m != 8) || B % m != 0) return -1;
    int w = log2_exact(m);
    int slots = B / m * n;
    int wpr = ceil_div(slots * w, 32);
    for (int s = 0; s < S; ++s) {
        int bi = s / B, r = s % B;
        for (long j = 0; j < nc; ++j) {
            double acc = 0.0;
            for (int t = row_ptr[bi]; t < row_ptr[bi + 1]; ++t) {
                const uint16_t *vrow = vals + ((long)t * B + r) * slots;
                const uint32_t *irow = idxw + ((long)t * B + r) * wpr;
                for (int q = 0; q < slots; ++q) {
                    long bit = (long)q * w;
                    uint64_t two = irow[bit / 32];
                    if (bit / 32 + 1 < wpr) two |= (uint64_t)irow[bit / 32 + 1] << 32;
                    int off = (int)((two >> (bit % 32)) & (uint64_t)(m - 1));
                    int k = col_idx[t] * B + (q / n) * m + off;
                    if (k >= K) continue; /* padding slot outside the matrix */
                    acc += (double)bf16_to_f32(vrow[q]) * (double)bf16_to_f32(X[(long)k * ldx + c0 + j]);
                }
            }
            Y[(long)s * nc + j] = acc;
        }
    }
    return 0;
}

/* ------------------------------------------------------------------------
 * Convolution lowering (Sec. 3 "Notation": the kernel is reshaped so that the
 * conv becomes a matrix product).  Activation is channel-major
 * act[c][b][h][w]; X[(kh*KW + kw)*C + c][(b*Ho + oh)*Wo + ow] =
 * act[c][b][oh*stride + kh - pad][ow*stride + kw - pad], zero outside.
 * ---------------------------------------------------------------------- */
int oracle_im2col(int C, int H, int Wd, int batch, int kh, int kw, int stride, int pad,
                  const uint16_t *act, uint16_t *X, long ldx)
{
    if (C < 1 || H < 1 || Wd < 1 || batch < 1 || kh < 1 || kw < 1 || stride < 1 || pad < 0) return -1;
    int Ho = (H + 2 * pad - kh) / stride + 1, Wo = (Wd + 2 * pad - kw) / stride + 1;
    if (Ho < 1 || Wo < 1 || !act || !X) return -1;
    for (int a = 0; a < kh; ++a)
        for (int b2 = 0; b2 < kw; ++b2)
            for (int c = 0; c < C; ++c) {
                long row = ((long)a * kw + b2) * C + c;
                for (int b = 0; b < batch; ++b)
                    for (int oh = 0; oh < Ho; ++oh)
                        for (int ow = 0; ow < Wo; ++ow) {
                            int ih = oh * stride + a - pad, iw = ow * stride + b2 - pad;
                            uint16_t v = 0;
                            if (ih >= 0 && ih < H && iw >= 0 && iw < Wd)
                                v = act[(((long)c * batch + b) * H + ih) * Wd + iw];
                            X[row * ldx + ((long)b * Ho + oh) * Wo + ow] = v;
                        }
            }
    return 0;
}

/* Metadata size closed forms of Sec. 3.1 (bits), for S x K' kept columns:
 * out[0] block indices with the paper's floor(log2(K'/B)) field width,
 * out[1] block indices with the width actually needed, ceil(log2(K/B)),
 * out[2] in-group positions, S*K'*(n/m)*log2(m). */
int oracle_metadata_bits(int S, int K, int Kp, int n, int m, int B, double *out)
{
    if (S < 1 || K < 1 || Kp < B || B < 1 || n < 1 || n > m || !out) return -1;
    double blocks = (double)S * (double)Kp / ((double)B * (double)B);
    out[0] = blocks * floor(log2((double)Kp / (double)B));
    int Kb = ceil_div(K, B), wb = 0;
    while ((1 << wb) < Kb) ++wb;
    out[1] = blocks * (double)wb;
    out[2] = (double)S * (double)Kp * ((double)n / (double)m) * (double)log2_exact(m);
    return 0;
}

/* Threads the OpenMP loops above will use (for reporting next to timings). */
#ifdef _OPENMP
#include <omp.h>
int oracle_num_threads(void) { return omp_get_max_threads(); }
#else
int oracle_num_threads(void) { return 1; }
#endif

/* ------------------------------------------------------------------------
 * Global block budget across layers (Alg. 1 lines 6-9; Sec. 3.3).
 * For every layer: each block-row's scores are ordered ascending (the block
 * that uniform pruning would drop first comes first; this is the exact reverse
 * of the keep order of oracle_block_select: score ascending, on a tie the
 * larger column first), and the scores at the same rank position o are added
 * over the block-rows, rows ascending, in fp64: c_l[o].  All c_l[o] of all
 * layers are then ordered ascending (ties: layer ascending, rank ascending)
 * and rank columns are pruned in that order until the overall sparsity
 * 1 - kept/total reaches `target`; one rank column of layer l removes that
 * rank's block from every block-row of layer l, so rows stay uniform.  Within
 * a layer c_l[o] is non-decreasing in o, hence a layer always loses a prefix of
 * its ranks.  The last rank column of a layer is never pruned (no layer
 * collapse, Sec. 3.3).  Weight counts: total = sum S*K; a block contributes
 * its in-range elements times n/m (exact for full groups; the count is only
 * used to decide when to stop).
 * Inputs per layer l: S, K, n, m, B and score (Sb x Kb, fp64).
 * Output: k_row[l] = kept blocks per block-row; achieved[0] = reached sparsity.
 * ---------------------------------------------------------------------- */
int oracle_global_budget(int L, const int *S, const int *K, const int *n, const int *m, const int *B,
                         const double *const *score, double target, int *k_row, double *achieved)
{
    if (L < 1 || !S || !K || !n || !m || !B || !score || !k_row || !(target >= 0.0) || target > 1.0) return -1;
    long ncols = 0;
    double total = 0.0, kept = 0.0;
    for (int l = 0; l < L; ++l) {
        int Kb = ceil_div(K[l], B[l]);
        ncols += Kb;
        total += (double)S[l] * (double)K[l];
        kept += (double)S[l] * (double)K[l] * (double)n[l] / (double)m[l];
        k_row[l] = Kb;
    }
    double *c = (double *)malloc((size_t)ncols * sizeof(double));
    double *w = (double *)malloc((size_t)ncols * sizeof(double)); /* kept weights a rank column holds */
    int *lay = (int *)malloc((size_t)ncols * sizeof(int));
    int *rk = (int *)malloc((size_t)ncols * sizeof(int));
    if (!c || !w || !lay || !rk) return -2;
    long pos = 0;
    for (int l = 0; l < L; ++l) {
        int Sb = ceil_div(S[l], B[l]), Kb = ceil_div(K[l], B[l]);
        for (int o = 0; o < Kb; ++o) { c[pos + o] = 0.0; w[pos + o] = 0.0; lay[pos + o] = l; rk[pos + o] = o; }
        for (int bi = 0; bi < Sb; ++bi) {
            const double *sc = score[l] + (long)bi * Kb;
            int rows = (S[l] - bi * B[l] < B[l]) ? S[l] - bi * B[l] : B[l];
            for (int j = 0; j < Kb; ++j) {
                /* ascending position of block j in its row: how many come before it */
                int before = 0;
                for (int o = 0; o < Kb; ++o)
                    if (sc[o] < sc[j] || (sc[o] == sc[j] && o > j)) ++before;
                int cols = (K[l] - j * B[l] < B[l]) ? K[l] - j * B[l] : B[l];
                c[pos + before] += sc[j]; /* rows ascending: bi is the outer loop */
                w[pos + before] += (double)rows * (double)cols * (double)n[l] / (double)m[l];
            }
        }
        pos += Kb;
    }
    /* repeatedly take the smallest remaining column under (c, layer, rank) */
    uint8_t *gone = (uint8_t *)calloc((size_t)ncols, 1);
    if (!gone) return -2;
    while (1.0 - kept / total < target) {
        long best = -1;
        for (long a = 0; a < ncols; ++a) {
            if (gone[a]) continue;
            if (k_row[lay[a]] <= 1) continue; /* keep the last rank column of every layer */
            if (best < 0 || c[a] < c[best]) best = a; /* ascending scan keeps (layer, rank) order on ties */
        }
        if (best < 0) break;
        gone[best] = 1;
        kept -= w[best];
        k_row[lay[best]] -= 1;
    }
    if (achieved) achieved[0] = 1.0 - kept / total;
    free(c); free(w); free(lay); free(rk); free(gone);
    return 0;
}
