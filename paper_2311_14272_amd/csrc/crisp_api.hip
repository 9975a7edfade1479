// C ABI of libcrisp: argument validation on the host, size queries, dispatch to the launchers.
#include <mutex>
#include <vector>

#include "crisp_internal.h"

#include <cmath>

namespace crisp {

static int ceil_div(int a, int b) { return (a + b - 1) / b; }

crisp_status make_geometry(const crisp_layer_desc* d, bool need_density, Geometry* g) {
    if (!d || !g) return CRISP_EINVAL;
    if (d->S < 1 || d->K < 1) return CRISP_ESHAPE;
    if (d->m != 4 && d->m != 8) return CRISP_EINVAL;
    if (d->n < 1 || d->n > d->m) return CRISP_EINVAL;
    if (d->B != 16 && d->B != 32 && d->B != 64) return CRISP_EINVAL;
    if (d->B % d->m != 0) return CRISP_EINVAL;
    if (d->sal_kind < CRISP_SAL_GIVEN || d->sal_kind > CRISP_SAL_MAG) return CRISP_EINVAL;
    if (d->select_mode != CRISP_ROW_UNIFORM && d->select_mode != CRISP_LAYER_TOPK) return CRISP_EINVAL;
    if (d->hints & ~CRISP_HINT_TWO_OF_FOUR) return CRISP_EINVAL;
    g->S = d->S; g->K = d->K; g->n = d->n; g->m = d->m; g->B = d->B;
    g->two_of_four = (d->hints & CRISP_HINT_TWO_OF_FOUR) && d->n == 4 && d->m == 8;
    g->Sb = ceil_div(d->S, d->B);
    g->Kb = ceil_div(d->K, d->B);
    g->w = d->m == 4 ? 2 : 3;
    g->slots = d->B / d->m * d->n;
    g->wpr = ceil_div(g->slots * g->w, 32);
    g->mwpr = ceil_div(d->K, 32);
    g->k_row = 0;
    g->nk = 0;
    // the kernels address a layer's packed values with 32-bit byte offsets: even with every block kept
    // they must stay below 4 GiB
    if ((int64_t)g->Sb * g->Kb * g->B * g->slots * 2 >= ((int64_t)1 << 32)) return CRISP_ESHAPE;
    if (need_density) {
        // Kept blocks per block-row for the layer's block density; at least one so that a
        // layer cannot collapse (Sec. 3.3, last paragraph).
        if (!(d->block_density > 0.0) || d->block_density > 1.0) return CRISP_EINVAL;
        double v = std::floor(d->block_density * (double)g->Kb + 0.5);
        int k = (int)v;
        if (k < 1) k = 1;
        if (k > g->Kb) k = g->Kb;
        g->k_row = k;
        if ((int64_t)g->Sb * k > INT32_MAX) return CRISP_ESHAPE;
        g->nk = g->Sb * k;
    }
    return CRISP_OK;
}

static bool misaligned(const void* p, size_t a) { return ((uintptr_t)p & (a - 1)) != 0; }

}  // namespace crisp

using namespace crisp;

extern "C" {

const char* crisp_status_str(crisp_status st) {
    switch (st) {
        case CRISP_OK: return "ok";
        case CRISP_EINVAL: return "invalid argument";
        case CRISP_ESHAPE: return "inconsistent shape";
        case CRISP_EBUFSIZE: return "workspace too small";
        case CRISP_EALIGN: return "misaligned pointer or leading dimension";
        case CRISP_EUNSUPPORTED: return "unsupported configuration";
        case CRISP_EDEVICE: return "device error";
        default: return "unknown status";
    }
}

crisp_status crisp_pack_sizes(const crisp_layer_desc* desc, crisp_sizes* out) {
    if (!out) return CRISP_EINVAL;
    Geometry g;
    crisp_status st = make_geometry(desc, true, &g);
    if (st != CRISP_OK) return st;
    out->Sb = g.Sb; out->Kb = g.Kb; out->k_row = g.k_row; out->nk = g.nk;
    out->slots_per_row = g.slots;
    out->idx_bits = g.w;
    out->idx_words_per_row = g.wpr;
    out->mask_words_per_row = g.mwpr;
    out->mask_words = (int64_t)g.S * g.mwpr;
    out->row_ptr_elems = (int64_t)g.Sb + 1;
    out->col_idx_elems = g.nk;
    out->score_elems = (int64_t)g.Sb * g.Kb;
    out->vals_elems = (int64_t)g.nk * g.B * g.slots;
    out->idx_words = (int64_t)g.nk * g.B * g.wpr;
    out->flags_elems = 4;
    // block scores live in the workspace when the caller does not ask for them
    out->select_ws_bytes = (size_t)g.Sb * g.Kb * sizeof(double);
    out->pack_ws_bytes = 0;
    out->spmm_ws_bytes = 0;
    // fused selection + packing: scores, then the packed form of every block of the grid
    out->select_pack_ws_bytes = ((size_t)g.Sb * g.Kb * sizeof(double) + 15) / 16 * 16 + select_pack_stage_bytes(g);
    return CRISP_OK;
}

crisp_status crisp_select_mask(const crisp_layer_desc* desc, const uint16_t* W, const float* T_or_G,
                               uint32_t* nm_mask, int32_t* row_ptr, int32_t* col_idx, double* block_score,
                               void* ws, size_t ws_bytes, void* stream) {
    Geometry g;
    crisp_status st = make_geometry(desc, true, &g);
    if (st != CRISP_OK) return st;
    if (!nm_mask || !row_ptr || !col_idx) return CRISP_EINVAL;
    if (desc->sal_kind != CRISP_SAL_GIVEN && !W) return CRISP_EINVAL;
    if (desc->sal_kind != CRISP_SAL_MAG && !T_or_G) return CRISP_EINVAL;
    if (misaligned(W, 16) || misaligned(T_or_G, 16) || misaligned(nm_mask, 16) || misaligned(row_ptr, 4) ||
        misaligned(col_idx, 4) || misaligned(block_score, 8) || misaligned(ws, 16))
        return CRISP_EALIGN;
    double* score = block_score;
    if (!score) {
        size_t need = (size_t)g.Sb * g.Kb * sizeof(double);
        if (!ws || ws_bytes < need) return CRISP_EBUFSIZE;
        score = (double*)ws;
    }
    if (g.Kb > 4096) return CRISP_EUNSUPPORTED;
    if (desc->select_mode == CRISP_LAYER_TOPK && ((int64_t)g.Sb * g.Kb > 8192 || g.Sb > 1024)) return CRISP_EUNSUPPORTED;
    hipError_t e = launch_select(g, desc->sal_kind, desc->select_mode, W, T_or_G, nm_mask, row_ptr, col_idx,
                                 score, (hipStream_t)stream);
    return e == hipSuccess ? CRISP_OK : CRISP_EDEVICE;
}

crisp_status crisp_pack(const crisp_layer_desc* desc, const uint16_t* W, const uint32_t* nm_mask,
                        const int32_t* row_ptr, const int32_t* col_idx, uint16_t* vals, uint32_t* idx_words,
                        int32_t* flags, void* ws, size_t ws_bytes, void* stream) {
    (void)ws; (void)ws_bytes;
    Geometry g;
    crisp_status st = make_geometry(desc, true, &g);
    if (st != CRISP_OK) return st;
    if (!W || !nm_mask || !row_ptr || !col_idx || !vals || !idx_words || !flags) return CRISP_EINVAL;
    if (misaligned(W, 16) || misaligned(nm_mask, 16) || misaligned(row_ptr, 4) || misaligned(col_idx, 4) ||
        misaligned(vals, 16) || misaligned(idx_words, 16) || misaligned(flags, 4))
        return CRISP_EALIGN;
    hipError_t e = launch_pack(g, desc->select_mode, W, nm_mask, row_ptr, col_idx, vals, idx_words, flags,
                               (hipStream_t)stream);
    return e == hipSuccess ? CRISP_OK : CRISP_EDEVICE;
}

// Argument checks of one layer of crisp_select_pack / crisp_select_pack_batch (host only).
static crisp_status check_select_pack(const crisp_layer_desc* desc, const crisp_layer_buffers* b, Geometry* g) {
    crisp_status st = make_geometry(desc, true, g);
    if (st != CRISP_OK) return st;
    if (!b->W || !b->nm_mask || !b->row_ptr || !b->col_idx || !b->vals || !b->idx_words || !b->flags) return CRISP_EINVAL;
    if (desc->sal_kind != CRISP_SAL_MAG && !b->T_or_G) return CRISP_EINVAL;
    if (misaligned(b->W, 16) || misaligned(b->T_or_G, 16) || misaligned(b->nm_mask, 16) || misaligned(b->row_ptr, 4) ||
        misaligned(b->col_idx, 4) || misaligned(b->block_score, 8) || misaligned(b->vals, 16) ||
        misaligned(b->idx_words, 16) || misaligned(b->flags, 4) || misaligned(b->ws, 16))
        return CRISP_EALIGN;
    const size_t score_bytes = ((size_t)g->Sb * g->Kb * sizeof(double) + 15) / 16 * 16;
    if (!b->ws || b->ws_bytes < score_bytes + select_pack_stage_bytes(*g)) return CRISP_EBUFSIZE;
    if (g->Kb > 4096) return CRISP_EUNSUPPORTED;
    if (desc->select_mode == CRISP_LAYER_TOPK && ((int64_t)g->Sb * g->Kb > 8192 || g->Sb > 1024)) return CRISP_EUNSUPPORTED;
    return CRISP_OK;
}

// Enqueues the fused selection + packing of layers whose arguments have been checked (geo[i] filled by
// check_select_pack); done: n_layers bytes of scratch.
static crisp_status select_pack_run(int32_t n_layers, const crisp_layer_desc* descs, const crisp_layer_buffers* bufs,
                                    const Geometry* geo, char* done, void* stream) {
    for (int i = 0; i < n_layers; ++i) done[i] = 0;
    hipError_t e = hipSuccess;
    for (int i = 0; i < n_layers && e == hipSuccess; ++i) {
        if (done[i]) continue;
        const Geometry& g = geo[i];
        double* score = bufs[i].block_score ? bufs[i].block_score : (double*)bufs[i].ws;
        if (!select_pack_fusable(g, descs[i].select_mode)) {
            // uneven rows or very wide grids: the two steps one after the other
            done[i] = 1;
            e = launch_select(g, descs[i].sal_kind, descs[i].select_mode, bufs[i].W, bufs[i].T_or_G, bufs[i].nm_mask,
                              bufs[i].row_ptr, bufs[i].col_idx, score, (hipStream_t)stream);
            if (e == hipSuccess)
                e = launch_pack(g, descs[i].select_mode, bufs[i].W, bufs[i].nm_mask, bufs[i].row_ptr, bufs[i].col_idx,
                                bufs[i].vals, bufs[i].idx_words, bufs[i].flags, (hipStream_t)stream);
            continue;
        }
        // this layer and the later ones of the same kernel instantiation, CRISP_SELECT_BATCH per launch pair
        Geometry gg[CRISP_SELECT_BATCH];
        SelPackPtrs pp[CRISP_SELECT_BATCH];
        int cnt = 0;
        int64_t blocks = 0;
        for (int j = i; j < n_layers && cnt < CRISP_SELECT_BATCH; ++j) {
            const Geometry& h = geo[j];
            if (done[j] || !select_pack_fusable(h, descs[j].select_mode)) continue;
            if (h.B != g.B || h.m != g.m || descs[j].sal_kind != descs[i].sal_kind || (h.K % h.B == 0) != (g.K % g.B == 0))
                continue;
            if (blocks + (int64_t)h.Sb * h.Kb > (1 << 30)) break;
            blocks += (int64_t)h.Sb * h.Kb;
            const size_t sb = ((size_t)h.Sb * h.Kb * sizeof(double) + 15) / 16 * 16;
            gg[cnt] = h;
            pp[cnt] = SelPackPtrs{bufs[j].W, bufs[j].T_or_G, bufs[j].nm_mask, bufs[j].row_ptr, bufs[j].col_idx,
                                  bufs[j].block_score ? bufs[j].block_score : (double*)bufs[j].ws, bufs[j].vals,
                                  bufs[j].idx_words, bufs[j].flags, (unsigned char*)bufs[j].ws + sb};
            done[j] = 1;
            ++cnt;
        }
        e = launch_select_pack_batch(cnt, gg, descs[i].sal_kind, pp, (hipStream_t)stream);
    }
    return e == hipSuccess ? CRISP_OK : CRISP_EDEVICE;
}

crisp_status crisp_select_pack_batch(int32_t n_layers, const crisp_layer_desc* descs, const crisp_layer_buffers* bufs,
                                     void* stream) {
    if (n_layers < 1 || n_layers > 4096 || !descs || !bufs) return CRISP_EINVAL;
    std::vector<Geometry> geo((size_t)n_layers);
    for (int i = 0; i < n_layers; ++i) {       // everything is checked before anything is enqueued
        crisp_status st = check_select_pack(&descs[i], &bufs[i], &geo[i]);
        if (st != CRISP_OK) return st;
    }
    std::vector<char> done((size_t)n_layers, 0);
    return select_pack_run(n_layers, descs, bufs, geo.data(), done.data(), stream);
}

crisp_status crisp_select_pack(const crisp_layer_desc* desc, const uint16_t* W, const float* T_or_G,
                               uint32_t* nm_mask, int32_t* row_ptr, int32_t* col_idx, double* block_score,
                               uint16_t* vals, uint32_t* idx_words, int32_t* flags, void* ws, size_t ws_bytes,
                               void* stream) {
    if (!desc) return CRISP_EINVAL;
    const crisp_layer_buffers b = {W, T_or_G, nm_mask, row_ptr, col_idx, block_score, vals, idx_words, flags, ws, ws_bytes};
    Geometry geo;
    crisp_status st = check_select_pack(desc, &b, &geo);
    if (st != CRISP_OK) return st;
    char done = 0;
    return select_pack_run(1, desc, &b, &geo, &done, stream);
}

// ---- crisp_select_pack for callers that cannot allocate ------------------------------------------
// The workspace of crisp_select_pack (block scores + packed form of every block of the grid) lives in
// a file-scope device array.  In host code the array's name is only a stand-in: its device address is
// looked up once per device with hipGetSymbolAddress (each GPU holds its own copy of the array at its
// own address) and that pointer is what the kernels are given.
static __device__ __align__(256) unsigned char scratch[CRISP_STATIC_SCRATCH_BYTES];

static const int MAX_DEVICES = 64;
static std::mutex scratch_mutex;
static void* scratch_ptr[MAX_DEVICES];     // per device, filled on the first call there

static crisp_status static_scratch(void** out) {
    int dev = -1;
    if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= MAX_DEVICES) return CRISP_EDEVICE;
    std::lock_guard<std::mutex> lock(scratch_mutex);
    if (!scratch_ptr[dev]) {
        void* p = nullptr;
        if (hipGetSymbolAddress(&p, HIP_SYMBOL(scratch)) != hipSuccess || !p) return CRISP_EDEVICE;
        scratch_ptr[dev] = p;
    }
    *out = scratch_ptr[dev];
    return CRISP_OK;
}

crisp_status crisp_select_pack_noalloc(const crisp_layer_desc* desc, const uint16_t* W, const float* T_or_G,
                                       uint32_t* nm_mask, int32_t* row_ptr, int32_t* col_idx, double* block_score,
                                       uint16_t* vals, uint32_t* idx_words, int32_t* flags, void* stream) {
    if (!desc) return CRISP_EINVAL;
    // every argument is checked first, with a stand-in for the workspace (aligned, never dereferenced)
    crisp_layer_buffers b = {W, T_or_G, nm_mask, row_ptr, col_idx, block_score, vals, idx_words, flags,
                             reinterpret_cast<void*>(uintptr_t(256)), ~size_t(0)};
    Geometry geo;
    crisp_status st = check_select_pack(desc, &b, &geo);
    if (st != CRISP_OK) return st;
    const size_t need = ((size_t)geo.Sb * geo.Kb * sizeof(double) + 15) / 16 * 16 + select_pack_stage_bytes(geo);
    if (need > (size_t)CRISP_STATIC_SCRATCH_BYTES) return CRISP_EBUFSIZE;   // the layer does not fit the built-in scratch
    void* ws = nullptr;
    st = static_scratch(&ws);
    if (st != CRISP_OK) return st;
    b.ws = ws;
    b.ws_bytes = CRISP_STATIC_SCRATCH_BYTES;
    char done = 0;
    return select_pack_run(1, desc, &b, &geo, &done, stream);
}

crisp_status crisp_im2col(const crisp_conv_desc* c, const uint16_t* act, uint16_t* X, int64_t ldx, void* stream) {
    if (!c || !act || !X) return CRISP_EINVAL;
    if (c->C < 1 || c->H < 1 || c->W < 1 || c->batch < 1 || c->kh < 1 || c->kw < 1 || c->stride < 1 || c->pad < 0)
        return CRISP_ESHAPE;
    if (c->act_layout != CRISP_ACT_CBHW || c->x_layout != CRISP_X_KN) return CRISP_EUNSUPPORTED;
    // (filter and step sizes far beyond any layer; they keep the 32-bit index arithmetic below exact)
    if (c->kh > 255 || c->kw > 255 || c->stride > 65535 || c->pad > 65535) return CRISP_EUNSUPPORTED;
    int64_t Ho = ((int64_t)c->H + 2 * c->pad - c->kh) / c->stride + 1;
    int64_t Wo = ((int64_t)c->W + 2 * c->pad - c->kw) / c->stride + 1;
    if (c->H + 2 * c->pad < c->kh || c->W + 2 * c->pad < c->kw || Ho < 1 || Wo < 1) return CRISP_ESHAPE;
    int64_t Ncol = (int64_t)c->batch * Ho * Wo;
    int64_t K = (int64_t)c->kh * c->kw * c->C;
    if (ldx < Ncol || Ncol > INT32_MAX - 1024 || K > INT32_MAX) return CRISP_ESHAPE;   // (column index of a thread: int)
    // (one grid slice per 16 channels: at most 65535 of them)
    if ((int64_t)c->batch * c->H * c->W >= ((int64_t)1 << 31) || c->C > (1 << 20) - 16) return CRISP_EUNSUPPORTED;
    if (misaligned(act, 16) || misaligned(X, 16)) return CRISP_EALIGN;
    hipError_t e = launch_im2col(*c, act, X, ldx, (hipStream_t)stream);
    return e == hipSuccess ? CRISP_OK : CRISP_EDEVICE;
}

crisp_status crisp_maxpool(const crisp_conv_desc* c, const uint16_t* act, uint16_t* out, void* stream) {
    if (!c || !act || !out) return CRISP_EINVAL;
    if (c->C < 1 || c->H < 1 || c->W < 1 || c->batch < 1 || c->kh < 1 || c->kw < 1 || c->stride < 1 || c->pad < 0)
        return CRISP_ESHAPE;
    if (c->kh > 255 || c->kw > 255 || c->stride > 65535) return CRISP_EUNSUPPORTED;
    if (c->pad >= c->kh || c->pad >= c->kw) return CRISP_ESHAPE;      // every window must touch the image
    if (c->H + 2 * c->pad < c->kh || c->W + 2 * c->pad < c->kw) return CRISP_ESHAPE;
    if (c->act_layout != CRISP_ACT_CBHW) return CRISP_EUNSUPPORTED;
    if ((int64_t)c->H * c->W >= ((int64_t)1 << 31)) return CRISP_EUNSUPPORTED;
    {
        const int64_t Ho = (c->H + 2 * c->pad - c->kh) / c->stride + 1, Wo = (c->W + 2 * c->pad - c->kw) / c->stride + 1;
        if ((int64_t)c->C * c->batch * Ho * Wo >= ((int64_t)1 << 32) - 256) return CRISP_EUNSUPPORTED;   // 32-bit output index
    }
    if (misaligned(act, 2) || misaligned(out, 2)) return CRISP_EALIGN;
    hipError_t e = launch_maxpool(*c, act, out, (hipStream_t)stream);
    return e == hipSuccess ? CRISP_OK : CRISP_EDEVICE;
}

static crisp_status check_epilogue(const crisp_epilogue* ep, int64_t Ncol) {
    if (!ep) return CRISP_OK;
    if (misaligned(ep->scale, 4) || misaligned(ep->bias, 4) || misaligned(ep->residual, 16)) return CRISP_EALIGN;
    if (ep->residual && (ep->ldr < Ncol || ep->ldr > ((int64_t)1 << 27))) return CRISP_ESHAPE;
    if (ep->residual && (ep->ldr & 7)) return CRISP_EALIGN;
    if (ep->relu != 0 && ep->relu != 1) return CRISP_EINVAL;
    return CRISP_OK;
}

static crisp_status spmm_impl(const crisp_layer_desc* desc, const int32_t* row_ptr, const int32_t* col_idx,
                              const uint16_t* vals, const uint32_t* idx_words, const uint16_t* X, int64_t Ncol,
                              int64_t ldx, int32_t x_layout, void* Y, int64_t ldy, int32_t y_dtype, int force_shape,
                              int32_t* kernel_code, void* stream, void* ev_start, void* ev_stop,
                              const crisp_epilogue* ep = nullptr) {
    Geometry g;
    crisp_status st = make_geometry(desc, false, &g);
    if (st != CRISP_OK) return st;
    if (!row_ptr || !col_idx || !vals || !idx_words || !X || !Y) return CRISP_EINVAL;
    if (y_dtype != CRISP_Y_F32 && y_dtype != CRISP_Y_BF16) return CRISP_EINVAL;
    if (Ncol < 1 || ldx < Ncol || ldy < Ncol) return CRISP_ESHAPE;
    if (Ncol > ((int64_t)1 << 27) || ldx > ((int64_t)1 << 27) || ldy > ((int64_t)1 << 27)) return CRISP_ESHAPE;
    if ((ldx & 7) || (ldy & 7)) return CRISP_EALIGN;
    if (misaligned(row_ptr, 4) || misaligned(col_idx, 4) || misaligned(vals, 16) || misaligned(idx_words, 16) ||
        misaligned(X, 16) || misaligned(Y, 16))
        return CRISP_EALIGN;
    if (x_layout != CRISP_X_KN && x_layout != CRISP_X_K8) return CRISP_EUNSUPPORTED;
    { crisp_status es = check_epilogue(ep, Ncol); if (es != CRISP_OK) return es; }
    if (x_layout == CRISP_X_K8) {
        // what the octet-interleaved kernels cover (there is no other path for this layout)
        const bool pattern_ok = (g.m == 4 && g.n <= 4) || (g.m == 8 && (g.n == 1 || g.n == 2 || g.n == 4 || g.n == 8));
        if (g.B == 16 || (g.K % 16) != 0 || (g.S % 8) != 0 || !pattern_ok || ldx > ((int64_t)1 << 26) || ldy > ((int64_t)1 << 23) ||
            (ep && ep->residual && ep->ldr > ((int64_t)1 << 23)))
            return CRISP_EUNSUPPORTED;
    }
    // shapes of the plain product that may be forced (anything else: the automatic choice)
    if (!((force_shape >= 0 && force_shape <= 10) || force_shape == CRISP_SHAPE_XRES ||
          (force_shape >= CRISP_SHAPE_BALANCED && force_shape <= CRISP_SHAPE_XLDS)))
        force_shape = -1;
    hipError_t e = launch_spmm(g, desc->block_density, desc->select_mode == CRISP_ROW_UNIFORM, force_shape, row_ptr, col_idx, vals,
                               idx_words, X, nullptr, Ncol,
                               ldx, Y, ldy, y_dtype, ep, (hipEvent_t)ev_start, (hipEvent_t)ev_stop, (hipStream_t)stream,
                               kernel_code, x_layout);
    return e == hipSuccess ? CRISP_OK : CRISP_EDEVICE;
}

// The geometries the fused lowering covers (row strides of Y and of a residual are checked by the caller).
static bool fused_lowering_covers(const Geometry& g, const crisp_conv_desc& conv, int64_t Ncol, int64_t plane) {
    const bool pattern_ok = (g.m == 4 && g.n <= 4) || (g.m == 8 && (g.n == 1 || g.n == 2 || g.n == 4 || g.n == 8));
    if (g.B == 16 || (Ncol & 1) || conv.kw > 16 || conv.kh * conv.kw > 64 || conv.stride > 16 ||
        plane > ((int64_t)1 << 27) || !pattern_ok)
        return false;
    // channel counts that are no multiple of B: rows are located one by one inside one buffer range
    if (conv.C % g.B != 0 && ((int64_t)conv.C * plane * 2 >= ((int64_t)1 << 32) - 16 || g.K > 65535)) return false;
    return true;
}

static crisp_status conv_spmm_impl(const crisp_layer_desc* desc, const crisp_conv_desc* conv, const int32_t* row_ptr,
                                   const int32_t* col_idx, const uint16_t* vals, const uint32_t* idx_words,
                                   const uint16_t* act, void* Y, int64_t ldy, int32_t y_dtype, int force_shape,
                                   int32_t* kernel_code, void* stream, void* ev_start, void* ev_stop,
                                   const crisp_epilogue* ep = nullptr) {
    Geometry g;
    crisp_status st = make_geometry(desc, false, &g);
    if (st != CRISP_OK) return st;
    if (!conv || !row_ptr || !col_idx || !vals || !idx_words || !act || !Y) return CRISP_EINVAL;
    if (y_dtype != CRISP_Y_F32 && y_dtype != CRISP_Y_BF16) return CRISP_EINVAL;
    if (conv->C < 1 || conv->H < 1 || conv->W < 1 || conv->batch < 1 || conv->kh < 1 || conv->kw < 1 ||
        conv->stride < 1 || conv->pad < 0)
        return CRISP_ESHAPE;
    if (conv->act_layout != CRISP_ACT_CBHW) return CRISP_EUNSUPPORTED;
    if ((int64_t)conv->kh * conv->kw * conv->C != g.K) return CRISP_ESHAPE;
    if (conv->H + 2 * conv->pad < conv->kh || conv->W + 2 * conv->pad < conv->kw) return CRISP_ESHAPE;
    const int64_t Ho = ((int64_t)conv->H + 2 * conv->pad - conv->kh) / conv->stride + 1;
    const int64_t Wo = ((int64_t)conv->W + 2 * conv->pad - conv->kw) / conv->stride + 1;
    if (Ho < 1 || Wo < 1) return CRISP_ESHAPE;
    const int64_t Ncol = (int64_t)conv->batch * Ho * Wo;
    const int64_t plane = (int64_t)conv->batch * conv->H * conv->W;
    if (ldy < Ncol || Ncol > ((int64_t)1 << 27)) return CRISP_ESHAPE;
    if ((ldy & 7) || misaligned(act, 16) || misaligned(Y, 16) || misaligned(vals, 16) || misaligned(idx_words, 16))
        return CRISP_EALIGN;
    { crisp_status es = check_epilogue(ep, Ncol); if (es != CRISP_OK) return es; }
    // what the fused kernels cover; everything else goes through crisp_im2col + crisp_spmm
    if (!fused_lowering_covers(g, *conv, Ncol, plane) || ldy > ((int64_t)1 << 23) ||
        (ep && ep->residual && ep->ldr > ((int64_t)1 << 23)))
        return CRISP_EUNSUPPORTED;
    // shapes of the fused lowering that may be forced (anything else: the automatic choice)
    if (!((force_shape >= 0 && force_shape <= 3) || (force_shape >= 7 && force_shape <= 10) ||
          force_shape == CRISP_SHAPE_CONV_LDS || force_shape == CRISP_SHAPE_CONV_PATCH || force_shape == CRISP_SHAPE_XLDS))
        force_shape = -1;
    hipError_t e = launch_spmm(g, desc->block_density, desc->select_mode == CRISP_ROW_UNIFORM, force_shape, row_ptr, col_idx, vals,
                               idx_words, act, conv,
                               Ncol, Ncol, Y, ldy, y_dtype, ep, (hipEvent_t)ev_start, (hipEvent_t)ev_stop, (hipStream_t)stream,
                               kernel_code);
    return e == hipSuccess ? CRISP_OK : CRISP_EDEVICE;
}

crisp_status crisp_spmm(const crisp_layer_desc* desc, const int32_t* row_ptr, const int32_t* col_idx,
                        const uint16_t* vals, const uint32_t* idx_words, const uint16_t* X, int64_t Ncol,
                        int64_t ldx, int32_t x_layout, void* Y, int64_t ldy, int32_t y_dtype, void* ws,
                        size_t ws_bytes, void* stream) {
    (void)ws; (void)ws_bytes;
    return spmm_impl(desc, row_ptr, col_idx, vals, idx_words, X, Ncol, ldx, x_layout, Y, ldy, y_dtype, -1, nullptr,
                     stream, nullptr, nullptr);
}

crisp_status crisp_conv_spmm(const crisp_layer_desc* desc, const crisp_conv_desc* conv, const int32_t* row_ptr,
                             const int32_t* col_idx, const uint16_t* vals, const uint32_t* idx_words,
                             const uint16_t* act, void* Y, int64_t ldy, int32_t y_dtype, void* ws, size_t ws_bytes,
                             void* stream) {
    (void)ws; (void)ws_bytes;
    return conv_spmm_impl(desc, conv, row_ptr, col_idx, vals, idx_words, act, Y, ldy, y_dtype, -1, nullptr, stream,
                          nullptr, nullptr);
}

crisp_status crisp_spmm_ep(const crisp_layer_desc* desc, const int32_t* row_ptr, const int32_t* col_idx,
                           const uint16_t* vals, const uint32_t* idx_words, const uint16_t* X, int64_t Ncol,
                           int64_t ldx, int32_t x_layout, void* Y, int64_t ldy, int32_t y_dtype,
                           const crisp_epilogue* ep, void* ws, size_t ws_bytes, void* stream) {
    (void)ws; (void)ws_bytes;
    return spmm_impl(desc, row_ptr, col_idx, vals, idx_words, X, Ncol, ldx, x_layout, Y, ldy, y_dtype, -1, nullptr,
                     stream, nullptr, nullptr, ep);
}

crisp_status crisp_conv_spmm_ep(const crisp_layer_desc* desc, const crisp_conv_desc* conv, const int32_t* row_ptr,
                                const int32_t* col_idx, const uint16_t* vals, const uint32_t* idx_words,
                                const uint16_t* act, void* Y, int64_t ldy, int32_t y_dtype, const crisp_epilogue* ep,
                                void* ws, size_t ws_bytes, void* stream) {
    (void)ws; (void)ws_bytes;
    return conv_spmm_impl(desc, conv, row_ptr, col_idx, vals, idx_words, act, Y, ldy, y_dtype, -1, nullptr, stream,
                          nullptr, nullptr, ep);
}

crisp_status crisp_spmm_forced(const crisp_layer_desc* desc, const int32_t* row_ptr, const int32_t* col_idx,
                               const uint16_t* vals, const uint32_t* idx_words, const uint16_t* X, int64_t Ncol,
                               int64_t ldx, int32_t x_layout, void* Y, int64_t ldy, int32_t y_dtype,
                               const crisp_epilogue* ep, int32_t shape, int32_t* kernel_code, void* stream) {
    return spmm_impl(desc, row_ptr, col_idx, vals, idx_words, X, Ncol, ldx, x_layout, Y, ldy, y_dtype, shape, kernel_code,
                     stream, nullptr, nullptr, ep);
}

crisp_status crisp_conv_spmm_forced(const crisp_layer_desc* desc, const crisp_conv_desc* conv, const int32_t* row_ptr,
                                    const int32_t* col_idx, const uint16_t* vals, const uint32_t* idx_words,
                                    const uint16_t* act, void* Y, int64_t ldy, int32_t y_dtype, const crisp_epilogue* ep,
                                    int32_t shape, int32_t* kernel_code, void* stream) {
    return conv_spmm_impl(desc, conv, row_ptr, col_idx, vals, idx_words, act, Y, ldy, y_dtype, shape, kernel_code, stream,
                          nullptr, nullptr, ep);
}

// Thresholds of crisp_conv_plan, measured on the ResNet-50 shapes at batch 256.  A kept block gathered
// with 2-byte loads costs about 0.8 of a block column of X written and read back once, the product over a
// materialised X about 0.2 per kept block: the fused register kernels pay while block-rows x density (kept
// blocks per block column of X) stays below 1.6.  For a strided 1x1 filter (8-byte pieces, X not inflated)
// the break-even is near 6 (the stride-2 shortcuts: 161 vs 186 us with 4 gathers per block column, 148 vs
// 115 us with 11).
static const double FUSED_GENERAL_MAX_GATHER = 1.6;
static const double STRIDED_1X1_MAX_GATHER = 6.0;

static crisp_status conv_plan_impl(const crisp_layer_desc* desc, const crisp_conv_desc* conv, Geometry* g, int32_t* path,
                                   int64_t* Ncol_out, int64_t* scratch_elems) {
    crisp_status st = make_geometry(desc, true, g);
    if (st != CRISP_OK) return st;
    if (conv->C < 1 || conv->H < 1 || conv->W < 1 || conv->batch < 1 || conv->kh < 1 || conv->kw < 1 ||
        conv->stride < 1 || conv->pad < 0)
        return CRISP_ESHAPE;
    if (conv->act_layout != CRISP_ACT_CBHW || conv->x_layout != CRISP_X_KN) return CRISP_EUNSUPPORTED;
    if (conv->kh > 255 || conv->kw > 255 || conv->stride > 65535 || conv->pad > 65535) return CRISP_EUNSUPPORTED;
    if ((int64_t)conv->kh * conv->kw * conv->C != g->K) return CRISP_ESHAPE;
    if (conv->H + 2 * conv->pad < conv->kh || conv->W + 2 * conv->pad < conv->kw) return CRISP_ESHAPE;
    const int64_t Ho = ((int64_t)conv->H + 2 * conv->pad - conv->kh) / conv->stride + 1;
    const int64_t Wo = ((int64_t)conv->W + 2 * conv->pad - conv->kw) / conv->stride + 1;
    const int64_t Ncol = (int64_t)conv->batch * Ho * Wo;
    const int64_t plane = (int64_t)conv->batch * conv->H * conv->W;
    if (Ncol > ((int64_t)1 << 27)) return CRISP_ESHAPE;
    *Ncol_out = Ncol;
    *scratch_elems = 0;
    const bool pointwise = conv->kh == 1 && conv->kw == 1 && conv->stride == 1 && conv->pad == 0;
    if (pointwise && (Ncol & 7) == 0) { *path = CRISP_CONV_DIRECT; return CRISP_OK; }
    if (!pointwise && fused_lowering_covers(*g, *conv, Ncol, plane)) {
        const double gathers = (double)g->Sb * desc->block_density;   // kept blocks per block column of X
        const bool aligned = conv->C % g->B == 0;
        const bool same_pad = conv->kh == 2 * conv->pad + 1 && conv->kw == 2 * conv->pad + 1;
        const bool paired = conv->stride == 1 && ((Wo & 1) == 0 || same_pad) && conv->W >= 2 && Wo >= 2 && aligned;
        const bool strided_1x1 = conv->kh == 1 && conv->kw == 1 && conv->stride == 2 && conv->pad == 0 && (conv->W & 1) == 0 &&
                                 (Wo & 1) == 0 && aligned;
        if ((strided_1x1 && gathers <= STRIDED_1X1_MAX_GATHER) || paired || xlds_conv_would_run(*g, *conv, Ncol) ||
            conv_lds_would_run(*g, desc->block_density, *conv, Ncol) ||
            (conv->kh * conv->kw > 1 && gathers <= FUSED_GENERAL_MAX_GATHER)) {
            *path = CRISP_CONV_FUSED;
            return CRISP_OK;
        }
    }
    *path = CRISP_CONV_IM2COL;
    *scratch_elems = (int64_t)g->K * ((Ncol + 7) / 8 * 8);
    return CRISP_OK;
}

crisp_status crisp_conv_plan(const crisp_layer_desc* desc, const crisp_conv_desc* conv, int32_t* path, size_t* scratch_bytes) {
    if (!desc || !conv || !path) return CRISP_EINVAL;
    Geometry g;
    int64_t Ncol = 0, elems = 0;
    crisp_status st = conv_plan_impl(desc, conv, &g, path, &Ncol, &elems);
    if (st == CRISP_OK && scratch_bytes) *scratch_bytes = (size_t)elems * 2;
    return st;
}

crisp_status crisp_conv_forward(const crisp_layer_desc* desc, const crisp_conv_desc* conv, const int32_t* row_ptr,
                                const int32_t* col_idx, const uint16_t* vals, const uint32_t* idx_words,
                                const uint16_t* act, void* Y, int64_t ldy, int32_t y_dtype, const crisp_epilogue* ep,
                                uint16_t* x_scratch, size_t scratch_bytes, int32_t* path_taken, void* stream) {
    if (!desc || !conv) return CRISP_EINVAL;
    Geometry g;
    int32_t path = 0;
    int64_t Ncol = 0, elems = 0;
    crisp_status st = conv_plan_impl(desc, conv, &g, &path, &Ncol, &elems);
    if (st != CRISP_OK) return st;
    // the fused kernels address a block-row of Y and of the residual with 32-bit offsets: wider row strides
    // go through a materialised X and the generic product kernel
    if (path == CRISP_CONV_FUSED && (ldy > ((int64_t)1 << 23) || (ep && ep->residual && ep->ldr > ((int64_t)1 << 23)))) {
        path = CRISP_CONV_IM2COL;
        elems = (int64_t)g.K * ((Ncol + 7) / 8 * 8);
    }
    if (path_taken) *path_taken = path;
    if (path == CRISP_CONV_DIRECT)
        return spmm_impl(desc, row_ptr, col_idx, vals, idx_words, act, Ncol, Ncol, CRISP_X_KN, Y, ldy, y_dtype, -1, nullptr, stream,
                         nullptr, nullptr, ep);
    if (path == CRISP_CONV_FUSED)
        return conv_spmm_impl(desc, conv, row_ptr, col_idx, vals, idx_words, act, Y, ldy, y_dtype, -1, nullptr, stream, nullptr,
                              nullptr, ep);
    if (!x_scratch || scratch_bytes < (size_t)elems * 2) return CRISP_EBUFSIZE;
    const int64_t ldx = (Ncol + 7) / 8 * 8;
    st = crisp_im2col(conv, act, x_scratch, ldx, stream);
    if (st != CRISP_OK) return st;
    return spmm_impl(desc, row_ptr, col_idx, vals, idx_words, x_scratch, Ncol, ldx, CRISP_X_KN, Y, ldy, y_dtype, -1, nullptr,
                     stream, nullptr, nullptr, ep);
}

crisp_status crisp_global_budget(int32_t n_layers, const crisp_layer_desc* descs, const double* const* block_scores,
                                 double target_sparsity, int32_t* k_row, double* achieved, void* ws, size_t ws_bytes,
                                 void* stream) {
    if (!descs || !block_scores || !k_row) return CRISP_EINVAL;
    if (n_layers < 1 || !(target_sparsity >= 0.0) || target_sparsity > 1.0) return CRISP_EINVAL;
    if (n_layers > CRISP_BUDGET_MAX_LAYERS) return CRISP_EUNSUPPORTED;
    BudgetArgs a;
    a.L = n_layers;
    a.target = target_sparsity;
    int64_t cols = 0;
    size_t need = 0;
    for (int l = 0; l < n_layers; ++l) {
        Geometry g;
        crisp_status st = make_geometry(&descs[l], false, &g);
        if (st != CRISP_OK) return st;
        if (!block_scores[l]) return CRISP_EINVAL;
        if (misaligned(block_scores[l], 8)) return CRISP_EALIGN;
        a.score[l] = block_scores[l];
        a.S[l] = g.S; a.K[l] = g.K; a.n[l] = g.n; a.m[l] = g.m; a.B[l] = g.B; a.Sb[l] = g.Sb; a.Kb[l] = g.Kb;
        cols += g.Kb;
        need += (size_t)g.Sb * g.Kb * sizeof(double);
    }
    if (cols > CRISP_BUDGET_MAX_COLS) return CRISP_EUNSUPPORTED;
    if (!ws || ws_bytes < need) return CRISP_EBUFSIZE;
    if (misaligned(ws, 16) || misaligned(k_row, 4) || misaligned(achieved, 8)) return CRISP_EALIGN;
    hipError_t e = launch_global_budget(a, (double*)ws, k_row, achieved, (hipStream_t)stream);
    return e == hipSuccess ? CRISP_OK : CRISP_EDEVICE;
}

crisp_status crisp_spmm_timed(const crisp_layer_desc* desc, const crisp_conv_desc* conv, const int32_t* row_ptr,
                              const int32_t* col_idx, const uint16_t* vals, const uint32_t* idx_words,
                              const uint16_t* X_or_act, int64_t Ncol, int64_t ldx, void* Y, int64_t ldy,
                              int32_t y_dtype, void* start_event, void* stop_event, void* stream) {
    if (conv)
        return conv_spmm_impl(desc, conv, row_ptr, col_idx, vals, idx_words, X_or_act, Y, ldy, y_dtype, -1, nullptr,
                              stream, start_event, stop_event);
    return spmm_impl(desc, row_ptr, col_idx, vals, idx_words, X_or_act, Ncol, ldx, CRISP_X_KN, Y, ldy, y_dtype, -1,
                     nullptr, stream, start_event, stop_event);
}

}  // extern "C"
