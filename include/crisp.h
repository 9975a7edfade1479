/*
 * libcrisp -- hybrid-sparse (block AND N:M) GEMM for AMD MI355X (gfx950).
 *
 * C ABI of the inference hot path of CRISP (arXiv 2311.14272): a pruned
 * convolution is lowered to Y = W_hybrid * X, where W_hybrid (S x K, S output
 * channels, K = kh*kw*C) has whole B x B blocks dropped, the same number in
 * every row of the block grid, and at most n non-zeros in every m consecutive
 * columns inside the blocks that remain (Sec. 3.1).
 *
 * Conventions that hold for every entry point
 *   - Returns a crisp_status; CRISP_OK is 0.  No exceptions, no errno, no
 *     global state; calls on different streams may run concurrently.
 *   - All arguments are validated on the host before any device call, so bad
 *     arguments are reported even on a machine without a GPU.
 *   - "device" pointers are HIP device memory owned by the caller, 16-byte
 *     aligned.  The library does not allocate, free or synchronise; work is
 *     enqueued on `stream` (a hipStream_t passed as void*, NULL = default
 *     stream) and the buffers must stay alive until that work has finished.
 *   - bf16 values travel as raw uint16_t bit patterns.
 *   - Matrices are row-major.  W is S x K.  X is K x ldx (K rows of Ncol
 *     used columns); Y is S x ldy.
 */
#ifndef CRISP_H
#define CRISP_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

#define CRISP_API __attribute__((visibility("default")))

typedef int32_t crisp_status;
enum {
    CRISP_OK = 0,
    CRISP_EINVAL = 1,       /* null pointer, n/m/B/density/kind out of range       */
    CRISP_ESHAPE = 2,       /* S, K, Ncol, ld*, conv geometry inconsistent         */
    CRISP_EBUFSIZE = 3,     /* workspace or scratch smaller than crisp_pack_sizes /
                               crisp_conv_plan report                              */
    CRISP_EALIGN = 4,       /* pointer or leading dimension alignment              */
    CRISP_EUNSUPPORTED = 5, /* valid request this build has no kernel for          */
    CRISP_EDEVICE = 6       /* a HIP launch reported an error                      */
};

/* saliency kinds (Sec. 3.4, Eq. 1) */
enum {
    CRISP_SAL_GIVEN = 0, /* T_or_G is the saliency T itself (fp32, S x K)                 */
    CRISP_SAL_GRAD = 1,  /* T = |W * G| with G = T_or_G, one fp32 multiply (Eq. 1; the     */
                         /* 1/H averaging factor is positive and cannot change a ranking)  */
    CRISP_SAL_MAG = 2    /* T = |W|, T_or_G unused (magnitude pruning, the 2:4 prior art)  */
};

/* block selection modes */
enum {
    CRISP_ROW_UNIFORM = 0, /* same number of kept blocks in every block-row (Sec. 3.1, 3.3) */
    CRISP_LAYER_TOPK = 1   /* plain block pruning over the whole grid; rows may be uneven   */
};

enum {
    CRISP_X_KN = 0,   /* X is K x ldx, columns contiguous; Y is S x ldy                                       */
    CRISP_X_K8 = 1    /* octet-interleaved: X is [K/8][ldx][8] (X8[k/8][j][k%8] = X[k][j]) and Y is written
                         the same way, [S/8][ldy][8], so that a layer's output is the next layer's operand   */
};
enum { CRISP_Y_F32 = 0, CRISP_Y_BF16 = 1 };
enum { CRISP_ACT_CBHW = 0 };           /* activation layout: [C][batch][H][W], W contiguous */

typedef struct {
    double block_density;  /* (0,1]; kept blocks per block-row k_row = clamp(floor(d*Kb+0.5),1,Kb) */
    int32_t S, K;          /* weight rows (output channels) and reduction length, >= 1; the packed
                              values of the whole block grid, Sb*Kb*B*(B*n/m)*2 bytes, must stay
                              below 4 GiB (ESHAPE otherwise)                                       */
    int32_t n, m;          /* 1 <= n <= m, m in {4,8}; n == m switches the fine-grained part off   */
    int32_t B;             /* block edge, 16 | 32 | 64, B % m == 0                                 */
    int32_t sal_kind;      /* CRISP_SAL_*                                                          */
    int32_t select_mode;   /* CRISP_ROW_UNIFORM | CRISP_LAYER_TOPK                                 */
    int32_t hints;         /* CRISP_HINT_* bits, read by the product calls only; other bits must be 0 */
} crisp_layer_desc;

/*
 * CRISP_HINT_TWO_OF_FOUR: the caller has read flags[0] == 1 from the crisp_pack / crisp_select_pack call
 * that produced the vals / idx_words it passes to the product: no aligned group of four columns holds more
 * than two kept values.  A 4:8 layer may then go to the sparse matrix-core instruction like a 2:4 layer
 * (Sec. 3.5 keeps the weights compressed next to the multipliers).  The flag lives on the device and the
 * kernel is chosen on the host, hence a hint; unlike block_density it is an assertion: with the bit set
 * for a pack whose flag is 0 the product is wrong.  Ignored for every pattern other than 4:8.
 */
enum { CRISP_HINT_TWO_OF_FOUR = 1 };

typedef struct {
    int32_t Sb, Kb;            /* block grid: ceil(S/B) x ceil(K/B)                              */
    int32_t k_row;             /* kept blocks per block-row                                      */
    int32_t nk;                /* kept blocks in total = Sb * k_row (both selection modes)       */
    int32_t slots_per_row;     /* B*n/m value slots per block row                                */
    int32_t idx_bits;          /* log2(m) bits per slot                                          */
    int32_t idx_words_per_row; /* ceil(slots_per_row*idx_bits/32)                                */
    int32_t mask_words_per_row;/* ceil(K/32)                                                     */
    int64_t mask_words;        /* S * mask_words_per_row  (uint32)                               */
    int64_t row_ptr_elems;     /* Sb + 1                  (int32)                                */
    int64_t col_idx_elems;     /* nk                      (int32)                                */
    int64_t score_elems;       /* Sb * Kb                 (double)                               */
    int64_t vals_elems;        /* nk * B * slots_per_row  (uint16 bf16)                          */
    int64_t idx_words;         /* nk * B * idx_words_per_row (uint32)                            */
    int64_t flags_elems;       /* 4                       (int32)                                */
    size_t select_ws_bytes;    /* workspace of crisp_select_mask                                 */
    size_t pack_ws_bytes;      /* workspace of crisp_pack                                        */
    size_t spmm_ws_bytes;      /* workspace of crisp_spmm                                        */
    size_t select_pack_ws_bytes; /* workspace of crisp_select_pack                               */
} crisp_sizes;

typedef struct {
    int32_t C, H, W, batch;    /* input channels, height, width, batch                           */
    int32_t kh, kw, stride, pad;
    int32_t act_layout;        /* CRISP_ACT_CBHW                                                 */
    int32_t x_layout;          /* CRISP_X_KN                                                     */
} crisp_conv_desc;

/*
 * Optional epilogue of the product entry points (the usual tail of a convolution layer once batch
 * normalisation is folded into a per-channel scale and bias; not part of the paper's method):
 *   y = sum;  y = y * scale[s]  (if scale);  y = y + bias[s]  (if bias);
 *   y = y + residual[s][j]  (if residual);  y = max(y, 0)  (if relu);  Y[s][j] = round(y)
 * in fp32 with one rounding per step, before the rounding to y_dtype.
 */
typedef struct {
    const float *scale;        /* S values (device) or NULL                                      */
    const float *bias;         /* S values (device) or NULL                                      */
    const void *residual;      /* S x ldr elements of the output's type (device) or NULL         */
    int64_t ldr;               /* >= Ncol, multiple of 8, <= 2^27 (only read when residual != NULL);
                                  above 2^23 the generic kernel runs (fused lowering: EUNSUPPORTED)  */
    int32_t relu;              /* 0 or 1                                                         */
    int32_t reserved;          /* 0                                                              */
} crisp_epilogue;

/* Text for a status code (static storage, never NULL). */
CRISP_API const char *crisp_status_str(crisp_status st);

/*
 * Buffer sizes for a layer.  Host only, pure function of the descriptor.
 * Derived from the storage format of Sec. 3.1: block column indices in
 * Blocked-ELL / block-CSR order, one log2(m)-bit in-group position per kept
 * value.  Errors: CRISP_EINVAL for a bad descriptor or null pointer.
 */
CRISP_API crisp_status crisp_pack_sizes(const crisp_layer_desc *desc, crisp_sizes *out);

/*
 * Mask selection for one layer (Alg. 1 lines 2, 4-6 and 10; Sec. 3.3).
 *   1. saliency T (Eq. 1) per desc->sal_kind, fp32;
 *   2. N:M: in each aligned group of m consecutive columns of a row keep the n
 *      positions that come first under (T descending, column ascending); a short
 *      last group keeps min(n, length);
 *   3. block score = sum of T over the N:M-kept, in-range elements of the block,
 *      in fp64, columns ascending inside a row, then rows ascending;
 *   4. ROW_UNIFORM: per block-row keep the k_row blocks first under (score
 *      descending, column ascending).  LAYER_TOPK: keep the Sb*k_row blocks first
 *      under (score descending, block-row ascending, column ascending).
 * Inputs (device):  W  S x K bf16;  T_or_G  S x K fp32 (may be NULL for SAL_MAG).
 * Outputs (device): nm_mask  S x ceil(K/32) uint32, bit k%32 of word k/32 set when
 *                   column k is kept by step 2 (the block choice is NOT folded in);
 *                   row_ptr  Sb+1 int32;  col_idx  nk int32, ascending inside a row;
 *                   block_score  Sb x Kb fp64, optional (NULL to skip).
 * ws: device workspace of select_ws_bytes (may be NULL when that is 0).
 * NaN saliency is outside the contract (order undefined).
 * Errors: EINVAL, EALIGN, EBUFSIZE, EUNSUPPORTED (block grid beyond 8192 blocks
 * in LAYER_TOPK mode, Kb > 4096), EDEVICE.
 */
CRISP_API crisp_status crisp_select_mask(const crisp_layer_desc *desc, const uint16_t *W, const float *T_or_G,
                               uint32_t *nm_mask, int32_t *row_ptr, int32_t *col_idx,
                               double *block_score, void *ws, size_t ws_bytes, void *stream);

/*
 * Packing (Sec. 3.1 metadata paragraph; Sec. 3.5, second step).  For kept block t
 * (row_ptr/col_idx order), block row r, group g of m columns there are n slots;
 * kept elements fill them in ascending column order.
 *   vals       [nk][B][B*n/m] bf16
 *   idx_words  [nk][B][idx_words_per_row] uint32: per block row a little-endian bit
 *              stream, slot q at bits [q*w, q*w+w), w = log2 m, 0-based position of
 *              the value inside its group (Sec. 3.5: a value in the second place of its
 *              group is stored with position 1).
 *   Padding: unused slots of a short group hold value 0, position 0; groups wholly
 *   outside the matrix (row >= S or first column >= K) hold value 0, positions 0..n-1.
 *   flags[0] = 1 when no aligned group of 4 columns in a kept block holds more
 *   than 2 kept elements (eligible for the 2-of-4 sparse matrix instruction).
 * All pointers device.  Errors as above.
 */
CRISP_API crisp_status crisp_pack(const crisp_layer_desc *desc, const uint16_t *W, const uint32_t *nm_mask,
                        const int32_t *row_ptr, const int32_t *col_idx, uint16_t *vals,
                        uint32_t *idx_words, int32_t *flags, void *ws, size_t ws_bytes, void *stream);

/*
 * crisp_select_mask followed by crisp_pack for the same layer, in fewer launches
 * (Alg. 1 lines 2, 4-6, 10 and the storage format of Sec. 3.1 / 3.5): while a block's
 * weights and keep bits are in registers for scoring, its packed form is written to
 * the workspace; once the block choice is known the kept blocks are copied to their
 * place.  Arguments, outputs and their contents are exactly those of the two calls
 * (nm_mask, row_ptr, col_idx, optional block_score; vals, idx_words, flags); W is
 * required for every sal_kind.
 * ws: device workspace of select_pack_ws_bytes (scores + packed form of all Sb*Kb
 * blocks), 16-byte aligned; contents on entry and exit are unspecified.
 * LAYER_TOPK and grids wider than 512 block columns run the two steps one after the
 * other internally.  Errors: as crisp_select_mask and crisp_pack.
 */
CRISP_API crisp_status crisp_select_pack(const crisp_layer_desc *desc, const uint16_t *W, const float *T_or_G,
                               uint32_t *nm_mask, int32_t *row_ptr, int32_t *col_idx,
                               double *block_score, uint16_t *vals, uint32_t *idx_words,
                               int32_t *flags, void *ws, size_t ws_bytes, void *stream);

/*
 * crisp_select_pack for callers that cannot allocate device memory (code under HIP graph capture,
 * tight serving loops, harnesses that forbid hipMalloc): same arguments, outputs and results, but
 * the workspace is a device array of CRISP_STATIC_SCRATCH_BYTES built into the library (each GPU the
 * library runs on holds one until the process ends).  The call allocates nothing, on the host or on
 * the device; the first call on a device looks the array's address up.  Layers whose
 * select_pack_ws_bytes exceed CRISP_STATIC_SCRATCH_BYTES are rejected with CRISP_EBUFSIZE (nothing
 * is enqueued).  All calls on one GPU share the array: calls that may run at the same time there
 * (different streams, threads) race; calls ordered on one stream are fine.  Nothing in the array
 * needs clearing between calls: every part that is read has been written by the same call.
 * Errors: as crisp_select_pack; EDEVICE when the array's address cannot be obtained.
 */
#define CRISP_STATIC_SCRATCH_BYTES (8u << 20)
CRISP_API crisp_status crisp_select_pack_noalloc(const crisp_layer_desc *desc, const uint16_t *W, const float *T_or_G,
                                       uint32_t *nm_mask, int32_t *row_ptr, int32_t *col_idx,
                                       double *block_score, uint16_t *vals, uint32_t *idx_words,
                                       int32_t *flags, void *stream);

/* The buffers of one layer for crisp_select_pack_batch: the arguments of crisp_select_pack. */
typedef struct {
    const uint16_t *W;
    const float *T_or_G;
    uint32_t *nm_mask;
    int32_t *row_ptr;
    int32_t *col_idx;
    double *block_score;       /* optional */
    uint16_t *vals;
    uint32_t *idx_words;
    int32_t *flags;
    void *ws;                  /* select_pack_ws_bytes of this layer */
    size_t ws_bytes;
} crisp_layer_buffers;

/*
 * crisp_select_pack for n_layers layers at once (Alg. 1 prunes all layers of a model in one
 * shot): layers that use the same kernel instantiation (block size, m, saliency kind, K a
 * multiple of B or not) share launches, up to 24 layers per launch pair, so that the small block
 * grids of single layers together fill the GPU.  Results per layer are exactly those of
 * crisp_select_pack.  descs and bufs are host arrays of n_layers elements (1 <= n_layers <=
 * 4096); the layers' buffers must not overlap.  All arguments are checked before anything is
 * enqueued.  Errors: as crisp_select_pack (the first failing layer's status).
 */
CRISP_API crisp_status crisp_select_pack_batch(int32_t n_layers, const crisp_layer_desc *descs,
                                     const crisp_layer_buffers *bufs, void *stream);

/*
 * Convolution lowering (Sec. 3 "Notation": the kernel tensor is reshaped so that
 * the convolution becomes a matrix product).  act is [C][batch][H][W] bf16;
 *   X[(a*kw + b)*C + c][(i*Ho + oh)*Wo + ow] = act[c][i][oh*stride + a - pad][ow*stride + b - pad]
 * and zero outside the image.  X is K x ldx with K = kh*kw*C, Ncol = batch*Ho*Wo
 * columns written, ldx >= Ncol.  For kh = kw = stride = 1, pad = 0 the result equals
 * act viewed as C x (batch*H*W); callers may skip the call and pass act as X.
 * Limits: kh, kw <= 255, stride, pad <= 65535, C < 2^20 - 16, batch*H*W < 2^31 (EUNSUPPORTED beyond),
 * Ncol < 2^31 - 1024 (ESHAPE beyond).
 * All pointers device.  Errors: EINVAL, ESHAPE, EUNSUPPORTED (layouts, limits), EDEVICE.
 */
CRISP_API crisp_status crisp_im2col(const crisp_conv_desc *conv, const uint16_t *act, uint16_t *X, int64_t ldx,
                          void *stream);

/*
 * The product (Sec. 3.5): Y[s][j] = sum over kept blocks (bi = s/B, bj) of the
 * block-row, over the block's slots, of value * X[bj*B + g*m + position][j];
 * bf16 x bf16 products accumulated in fp32.  Blocks that were dropped are never
 * touched, neither their weights nor the X rows only they would need.
 *   row_ptr/col_idx/vals/idx_words: output of crisp_pack (device).
 *   X: K x ldx bf16 (device), Ncol used columns, ldx >= Ncol, ldx % 8 == 0; the
 *      allocation must cover K*ldx elements.  x_layout = CRISP_X_KN, or CRISP_X_K8 for
 *      operands interleaved in octets of rows: X as [K/8][ldx][8], Y (and an epilogue's
 *      residual) as [S/8][ld][8], which makes every matrix-core operand one 16-byte load
 *      and every store of a wave 512 contiguous bytes.  CRISP_X_K8 needs K % 16 == 0,
 *      S % 8 == 0, B in {32, 64}, n:m in {1..4}:4 or {1,2,4,8}:8, ldx <= 2^26, ldy and a
 *      residual's stride <= 2^23 (EUNSUPPORTED otherwise: there is no other kernel for it).
 *   Y: S x ldy, fp32 or bf16 per y_dtype (device), ldy >= Ncol, ldy % 8 == 0.
 *      Every element Y[0..S)[0..Ncol) is written (rows of empty block-rows get 0).
 *   Ncol, ldx and ldy may be up to 2^27 (ESHAPE beyond); with ldy above 2^23 the
 *   generic kernel runs whatever the pattern.
 *   desc->sal_kind is not used here.  desc->block_density and select_mode only
 *   steer the choice of kernel (how many blocks a block-row holds, whether all
 *   rows hold the same number); a wrong or out-of-range density costs speed, never
 *   correctness.
 *   ws, ws_bytes: reserved (spmm_ws_bytes is 0); both are ignored.  Results of the launch
 *   shapes the library may choose agree within the summation-order tolerance.
 * Errors: EINVAL, ESHAPE, EALIGN, EUNSUPPORTED (x_layout and what it covers), EDEVICE.
 */
CRISP_API crisp_status crisp_spmm(const crisp_layer_desc *desc, const int32_t *row_ptr, const int32_t *col_idx,
                        const uint16_t *vals, const uint32_t *idx_words, const uint16_t *X,
                        int64_t Ncol, int64_t ldx, int32_t x_layout, void *Y, int64_t ldy,
                        int32_t y_dtype, void *ws, size_t ws_bytes, void *stream);

/*
 * Product with implicit lowering: Y = W_hybrid * im2col(act) without materialising X
 * (Sec. 3.5, first step: only the activations that kept blocks need are fetched, here straight
 * from the convolution's input).  Same result as crisp_im2col followed by crisp_spmm up to
 * the fp32 summation order (bit for bit when both are forced into the same launch shape of the
 * register kernels).  act is [C][batch][H][W] bf16 (device); desc->K must equal kh*kw*C; Y is
 * S x ldy with Ncol = batch*Ho*Wo columns written.
 * Covered: Ncol even, B in {32, 64}, n:m in {1..4}:4 or {1,2,4,8}:8, kw <= 16,
 * kh*kw <= 64, stride <= 16, batch*H*W <= 2^27, ldy <= 2^23.  With C % B == 0 every block
 * column belongs to one filter tap: for stride 1 and either an even Wo or padding (k-1)/2
 * in both directions a lane's two output columns come from one 4-byte load, for a 1x1 filter
 * with stride 2, no padding and even W and Wo from one 8-byte load, otherwise each column is
 * located and loaded on its own.  Other channel counts (the first layer of a network):
 * every K-row is split into (tap, channel) on its own; needs K <= 65535 and an activation
 * below 4 GiB.  For stride <= 4, C % 64 == 0, 64x64 blocks, even W <= 64 and even Wo there is also
 * a kernel that stages the input patch of a tile of output rows in LDS once for all filter
 * taps and up to four block-rows (chosen for dense multi-row layers).  Channel counts that are
 * no multiple of 64 with 64x64 blocks, even W and even Ho*Wo run in a kernel that keeps the input
 * patch of 1024 output positions in LDS.  ws, ws_bytes: reserved, ignored.
 * Anything else returns CRISP_EUNSUPPORTED (use crisp_im2col + crisp_spmm).
 * Errors: EINVAL, ESHAPE, EALIGN, EUNSUPPORTED, EDEVICE.
 */
CRISP_API crisp_status crisp_conv_spmm(const crisp_layer_desc *desc, const crisp_conv_desc *conv,
                                       const int32_t *row_ptr, const int32_t *col_idx, const uint16_t *vals,
                                       const uint32_t *idx_words, const uint16_t *act, void *Y, int64_t ldy,
                                       int32_t y_dtype, void *ws, size_t ws_bytes, void *stream);

/*
 * Max pooling of a channel-major activation (glue of the ResNet workload between the first
 * convolution and the first residual stage; not part of the paper's method):
 *   out[c][i][oh][ow] = max over a < kh, b < kw of act[c][i][oh*stride + a - pad][ow*stride + b - pad],
 * positions outside the image excluded; Ho, Wo as for a convolution; pad < kh, kw.  The result is
 * one of the inputs (no rounding).  act and out device, bf16, out holds C*batch*Ho*Wo elements
 * (fewer than 2^32); kh, kw <= 255, stride <= 65535.
 * Errors: EINVAL, ESHAPE, EUNSUPPORTED (layout, size), EDEVICE.
 */
CRISP_API crisp_status crisp_maxpool(const crisp_conv_desc *pool, const uint16_t *act, uint16_t *out, void *stream);

/*
 * crisp_spmm / crisp_conv_spmm with an epilogue (see crisp_epilogue; ep == NULL: none).  The
 * residual may not overlap Y.  Errors: those of the plain entry points, plus EALIGN / ESHAPE /
 * EINVAL for a bad epilogue.
 */
CRISP_API crisp_status crisp_spmm_ep(const crisp_layer_desc *desc, const int32_t *row_ptr, const int32_t *col_idx,
                           const uint16_t *vals, const uint32_t *idx_words, const uint16_t *X,
                           int64_t Ncol, int64_t ldx, int32_t x_layout, void *Y, int64_t ldy,
                           int32_t y_dtype, const crisp_epilogue *ep, void *ws, size_t ws_bytes,
                           void *stream);
CRISP_API crisp_status crisp_conv_spmm_ep(const crisp_layer_desc *desc, const crisp_conv_desc *conv,
                                const int32_t *row_ptr, const int32_t *col_idx, const uint16_t *vals,
                                const uint32_t *idx_words, const uint16_t *act, void *Y, int64_t ldy,
                                int32_t y_dtype, const crisp_epilogue *ep, void *ws, size_t ws_bytes,
                                void *stream);

/*
 * For tests and tuning sweeps only (callers that cannot allocate or that want the library's own
 * choice use the entry points above): crisp_spmm_ep / crisp_conv_spmm_ep with the launch shape
 * chosen by the caller, and a report of the kernel that ran.
 *   shape: CRISP_SHAPE_AUTO, or one of the shapes below; a shape that does not apply to the problem
 *          (pattern, block size, K or Ncol alignment, geometry) falls back to the automatic choice.
 *   kernel_code (optional, host): receives family | shape << 8 | conv_mode << 16 | sparse << 24 of
 *          the kernel that was launched (family: CRISP_KERNEL_*; shape: the register kernels' launch
 *          shape 0..3; for the LDS-resident family bit 0 = wide strips, bit 1 = the instantiation with
 *          the larger tile capacity; else 0; conv_mode: 0 plain X, 1..4 the fused-lowering modes;
 *          sparse: 1 when the sparse matrix-core instruction is used).  Together with (n, m, B) --
 *          B alone for the generic and 16 x 16 families and for the LDS-resident family with sparse = 0,
 *          which are not specialised by pattern -- the code names one compiled kernel.
 * Results agree across shapes within the summation-order tolerance.  Errors as for the plain calls.
 */
enum {
    CRISP_SHAPE_AUTO = -1,
    CRISP_SHAPE_REG_WIDE = 0,    /* register expansion, waves own strips of 128 columns          */
    CRISP_SHAPE_REG_NARROW = 1,  /* ... strips of 64 columns                                      */
    CRISP_SHAPE_REG_SPLIT4 = 2,  /* ... 4 waves split the block list of one tile                  */
    CRISP_SHAPE_REG_SPLIT8 = 3,  /* ... 8 waves                                                   */
    CRISP_SHAPE_GENERIC = 4,     /* generic LDS-expansion kernel (any K, Ncol, pattern)           */
    CRISP_SHAPE_LDS_NARROW = 5,  /* block-row resident in LDS, strips of 64 columns               */
    CRISP_SHAPE_LDS_WIDE = 6,    /* ... strips of 128 columns                                     */
    CRISP_SHAPE_SMF_WIDE = 7,    /* shapes 0..3 with the sparse matrix-core instruction where the */
    CRISP_SHAPE_SMF_NARROW = 8,  /* pattern allows it                                             */
    CRISP_SHAPE_SMF_SPLIT4 = 9,
    CRISP_SHAPE_SMF_SPLIT8 = 10,
    CRISP_SHAPE_CONV_LDS = 12,   /* fused lowering with the input patch staged in LDS             */
    CRISP_SHAPE_XRES = 13,       /* K <= 128: X operands resident in registers                    */
    CRISP_SHAPE_CONV_PATCH = 14, /* fused lowering for channel counts that are no multiple of 64  */
    CRISP_SHAPE_BALANCED = 15,   /* block list dealt evenly to the waves (uneven block-rows)      */
    CRISP_SHAPE_LDS_SMF = 16,    /* block-row resident in LDS as sparse matrix-core operands      */
    CRISP_SHAPE_LDS_SMF_30 = 17, /* ... always the instantiation that holds 30 blocks             */
    CRISP_SHAPE_XLDS = 18        /* K <= 512: a strip of X resident in LDS for all block-rows     */
};
enum {
    CRISP_KERNEL_REG = 1, CRISP_KERNEL_GENERIC = 2, CRISP_KERNEL_LDS = 3, CRISP_KERNEL_XRES = 4,
    CRISP_KERNEL_CONV_LDS = 5, CRISP_KERNEL_CONV_PATCH = 6, CRISP_KERNEL_B16 = 7, CRISP_KERNEL_BALANCED = 8,
    CRISP_KERNEL_K8 = 9, CRISP_KERNEL_XLDS = 10
};
CRISP_API crisp_status crisp_spmm_forced(const crisp_layer_desc *desc, const int32_t *row_ptr, const int32_t *col_idx,
                               const uint16_t *vals, const uint32_t *idx_words, const uint16_t *X,
                               int64_t Ncol, int64_t ldx, int32_t x_layout, void *Y, int64_t ldy,
                               int32_t y_dtype, const crisp_epilogue *ep, int32_t shape,
                               int32_t *kernel_code, void *stream);
CRISP_API crisp_status crisp_conv_spmm_forced(const crisp_layer_desc *desc, const crisp_conv_desc *conv,
                                    const int32_t *row_ptr, const int32_t *col_idx, const uint16_t *vals,
                                    const uint32_t *idx_words, const uint16_t *act, void *Y, int64_t ldy,
                                    int32_t y_dtype, const crisp_epilogue *ep, int32_t shape,
                                    int32_t *kernel_code, void *stream);

/*
 * A whole convolution layer (Sec. 3 "Notation" + Sec. 3.5): the product of a packed layer with the
 * lowering of act [C][batch][H][W], by whichever of three ways is fastest for the geometry:
 *   CRISP_CONV_DIRECT  1x1 filter, stride 1, no padding, batch*H*W a multiple of 8: act is X as it stands;
 *   CRISP_CONV_FUSED   crisp_conv_spmm_ep (X never materialised);
 *   CRISP_CONV_IM2COL  crisp_im2col into x_scratch, K x round_up(Ncol, 8) bf16, then crisp_spmm_ep.
 * The fused kernels that locate strided or odd-width columns one by one repeat that for every kept block;
 * they are chosen where desc->block_density (used here, unlike in the product calls: it must be the
 * layer's) says the kept blocks of all block-rows are not many more than X has block columns, where the
 * kernel that stages the input in LDS applies, or where column pairs come from one aligned piece of
 * an input row; everything the fused entry point does not cover is materialised.
 * crisp_conv_plan (host only, pure) reports the way and the scratch bytes it needs (0 unless IM2COL).
 * crisp_conv_forward enqueues it; x_scratch may be NULL when no scratch is needed; with Y or residual
 * row strides above 2^23 a FUSED plan is run as IM2COL (then scratch of K x round_up(Ncol, 8) is needed
 * after all); *path_taken (optional, host) receives the way taken.
 * Errors: those of the entry points named above; EBUFSIZE when the scratch is missing or too small.
 */
enum { CRISP_CONV_DIRECT = 0, CRISP_CONV_FUSED = 1, CRISP_CONV_IM2COL = 2 };
CRISP_API crisp_status crisp_conv_plan(const crisp_layer_desc *desc, const crisp_conv_desc *conv, int32_t *path,
                             size_t *scratch_bytes);
CRISP_API crisp_status crisp_conv_forward(const crisp_layer_desc *desc, const crisp_conv_desc *conv,
                                const int32_t *row_ptr, const int32_t *col_idx, const uint16_t *vals,
                                const uint32_t *idx_words, const uint16_t *act, void *Y, int64_t ldy,
                                int32_t y_dtype, const crisp_epilogue *ep, uint16_t *x_scratch,
                                size_t scratch_bytes, int32_t *path_taken, void *stream);

/*
 * Global block budget across layers (Alg. 1 lines 6-9; Sec. 3.3): turns one overall target
 * sparsity into kept blocks per block-row for every layer.
 *   Per layer, each block-row's scores (output block_score of crisp_select_mask) are ordered
 *   ascending (score ascending, on a tie the larger column first: the reverse of the keep order),
 *   scores of equal rank position are added over the block-rows (rows ascending, fp64), all rank
 *   columns of all layers are ordered ascending (ties: layer, then rank) and pruned in that order
 *   until 1 - kept/total >= target_sparsity, where total = sum S*K and a block counts its in-range
 *   elements times n/m.  A layer never loses its last rank column (no layer collapse).
 *   descs, block_scores: HOST arrays of n_layers entries; block_scores[l] is a DEVICE pointer to
 *   Sb x Kb fp64.  desc fields used: S, K, n, m, B.
 *   k_row: DEVICE, n_layers int32 (kept blocks per block-row; a density k_row/Kb reproduces it in
 *   crisp_select_mask).  achieved: DEVICE, 1 double, optional.  ws: DEVICE, sum Sb*Kb doubles.
 * Limits: n_layers <= 64, sum of Kb <= 4096 (EUNSUPPORTED beyond).
 * Errors: EINVAL, EALIGN, EBUFSIZE, EUNSUPPORTED, EDEVICE.
 */
CRISP_API crisp_status crisp_global_budget(int32_t n_layers, const crisp_layer_desc *descs,
                                           const double *const *block_scores, double target_sparsity,
                                           int32_t *k_row, double *achieved, void *ws, size_t ws_bytes,
                                           void *stream);

/*
 * The same product as crisp_spmm (conv == NULL, X_or_act = X) or crisp_conv_spmm (conv != NULL,
 * X_or_act = act; Ncol and ldx ignored), with two optional hipEvent_t (created by the caller with
 * timing enabled, passed as void*) that receive the time stamps of the product kernel's own start
 * and end on `stream`.  For measurement: an event pair recorded around a launch also times the
 * gaps around it; these two do not.  Errors as for the two calls above.
 */
CRISP_API crisp_status crisp_spmm_timed(const crisp_layer_desc *desc, const crisp_conv_desc *conv,
                                        const int32_t *row_ptr, const int32_t *col_idx, const uint16_t *vals,
                                        const uint32_t *idx_words, const uint16_t *X_or_act, int64_t Ncol,
                                        int64_t ldx, void *Y, int64_t ldy, int32_t y_dtype, void *start_event,
                                        void *stop_event, void *stream);

#ifdef __cplusplus
}
#endif
#endif /* CRISP_H */
