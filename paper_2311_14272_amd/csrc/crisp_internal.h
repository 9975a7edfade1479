// Internal declarations shared by the libcrisp translation units (not installed).
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "crisp.h"

namespace crisp {

struct Geometry {
    int S, K, n, m, B;
    int Sb, Kb, k_row, nk;
    int w;      // bits per in-group position
    int slots;  // value slots per block row
    int wpr;    // index words per block row
    int mwpr;   // mask words per weight row
    int two_of_four;   // 4:8 whose pack the caller asserts to hold at most two values per aligned four (products only)
};

// Host-side validation + derived sizes; no device calls.
crisp_status make_geometry(const crisp_layer_desc* d, bool need_density, Geometry* g);

// Launchers (enqueue only).  Each returns hipGetLastError() of its launches.
hipError_t launch_select(const Geometry& g, int sal_kind, int select_mode, const uint16_t* W, const float* TG,
                         uint32_t* nm_mask, int32_t* row_ptr, int32_t* col_idx, double* score, hipStream_t st);
bool select_pack_fusable(const Geometry& g, int select_mode);
size_t select_pack_stage_bytes(const Geometry& g);
struct SelPackPtrs {
    const uint16_t* W; const float* TG; uint32_t* nm_mask; int32_t* row_ptr; int32_t* col_idx; double* score;
    uint16_t* vals; uint32_t* idxw; int32_t* flags; void* stage;
};
#define CRISP_SELECT_BATCH 24  // layers per launch pair of launch_select_pack_batch (the batch travels in the kernel arguments: 3.7 of 4 KB)
hipError_t launch_select_pack_batch(int n, const Geometry* g, int sal_kind, const SelPackPtrs* pp, hipStream_t st);
hipError_t launch_pack(const Geometry& g, int select_mode, const uint16_t* W, const uint32_t* nm_mask,
                       const int32_t* row_ptr, const int32_t* col_idx, uint16_t* vals, uint32_t* idxw,
                       int32_t* flags, hipStream_t st);
hipError_t launch_im2col(const crisp_conv_desc& c, const uint16_t* act, uint16_t* X, int64_t ldx, hipStream_t st);
hipError_t launch_maxpool(const crisp_conv_desc& c, const uint16_t* act, uint16_t* out, hipStream_t st);
// density_hint and uniform_rows (every block-row keeps the same number of blocks) only steer the
// choice of kernel; force_shape < 0 lets the library choose (0..3 = shapes of the specialised
// kernels, 4 = generic LDS-expansion kernel, 5 / 6 = LDS-resident block-rows, narrow / wide).
hipError_t launch_spmm(const Geometry& g, double density_hint, bool uniform_rows, int force_shape, const int32_t* row_ptr,
                       const int32_t* col_idx, const uint16_t* vals, const uint32_t* idxw, const uint16_t* X,
                       const crisp_conv_desc* conv, int64_t Ncol, int64_t ldx, void* Y, int64_t ldy, int y_dtype,
                       const crisp_epilogue* ep,
                       hipEvent_t ev_start, hipEvent_t ev_stop, hipStream_t st, int32_t* kernel_code = nullptr,
                       int x_layout = CRISP_X_KN);

// Whether launch_spmm would run this convolution with the input patch staged in LDS (host only).
bool conv_lds_would_run(const Geometry& g, double density_hint, const crisp_conv_desc& conv, int64_t Ncol);
bool xlds_conv_would_run(const Geometry& g, const crisp_conv_desc& conv, int64_t Ncol);

#define CRISP_BUDGET_MAX_LAYERS 64
#define CRISP_BUDGET_MAX_COLS 4096
struct BudgetArgs {
    int L;
    double target;
    const double* score[CRISP_BUDGET_MAX_LAYERS];
    int S[CRISP_BUDGET_MAX_LAYERS], K[CRISP_BUDGET_MAX_LAYERS], n[CRISP_BUDGET_MAX_LAYERS], m[CRISP_BUDGET_MAX_LAYERS],
        B[CRISP_BUDGET_MAX_LAYERS], Sb[CRISP_BUDGET_MAX_LAYERS], Kb[CRISP_BUDGET_MAX_LAYERS];
};
hipError_t launch_global_budget(const BudgetArgs& a, double* ws, int32_t* k_row, double* achieved, hipStream_t st);

__device__ __forceinline__ float bf16_bits_to_float(uint16_t b) { return __uint_as_float(((uint32_t)b) << 16); }

}  // namespace crisp
