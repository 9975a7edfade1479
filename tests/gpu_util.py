"""Helpers for the GPU tests: numpy <-> device memory, and one run of the HIP path per layer."""
import numpy as np
import torch

from paper_2311_14272_amd import crisp


def dev(a: np.ndarray):
    """Upload a numpy array; 16/32-bit unsigned patterns travel as signed torch dtypes."""
    a = np.ascontiguousarray(a)
    if a.dtype == np.uint16:
        a = a.view(np.int16)
    elif a.dtype == np.uint32:
        a = a.view(np.int32)
    return torch.from_numpy(a).cuda()


def host(t, dtype):
    a = t.cpu().numpy()
    return a.view(dtype) if a.dtype != dtype else a


def desc_of(L):
    return crisp.layer_desc(L.S, L.K, L.n, L.m, L.B, L.density, L.sal_kind, L.select_mode)


def run_select_pack(L, W, G, fused=True, desc=None):
    """Selection + packing on the device (crisp_select_pack, or crisp_select_mask + crisp_pack when
    fused is False); returns the DeviceLayer and host copies.  Outputs are poisoned first so that
    anything the library leaves unwritten shows up."""
    layer = crisp.alloc_layer(desc if desc is not None else desc_of(L))
    for t in (layer.nm_mask, layer.row_ptr, layer.col_idx, layer.vals, layer.idx_words, layer.flags):
        t.fill_(-1)
    layer.score.fill_(float("nan"))
    dW = dev(W)
    dG = dev(G) if G is not None else None
    crisp.prune_and_pack(layer, dW, dG, fused=fused)
    torch.cuda.synchronize()
    sz = layer.sizes
    out = dict(
        nm_bits=host(layer.nm_mask, np.uint32)[: sz.mask_words].reshape(L.S, sz.mask_words_per_row),
        row_ptr=host(layer.row_ptr, np.int32),
        col_idx=host(layer.col_idx, np.int32)[: sz.nk],
        score=host(layer.score, np.float64).reshape(sz.Sb, sz.Kb),
        vals=host(layer.vals, np.uint16)[: sz.vals_elems].reshape(sz.nk, L.B, sz.slots_per_row),
        idxw=host(layer.idx_words, np.uint32)[: sz.idx_words].reshape(sz.nk, L.B, sz.idx_words_per_row),
        flags=host(layer.flags, np.int32))
    return layer, out


def spmm(desc, row_ptr, col_idx, vals, idx_words, X, Ncol, ldx, Y, ldy, y_dtype, shape=None):
    """The product through crisp_spmm (shape None: the library's own choice, the production call) or
    through crisp_spmm_forced with launch shape `shape` (returns the code of the kernel that ran)."""
    if shape is None:
        crisp.crisp_spmm(desc, row_ptr, col_idx, vals, idx_words, X, Ncol, ldx, Y, ldy, y_dtype)
        return None
    return crisp.crisp_spmm_forced(desc, row_ptr, col_idx, vals, idx_words, X, Ncol, ldx, Y, ldy, y_dtype, None, shape)


def spmm_ep(desc, row_ptr, col_idx, vals, idx_words, X, Ncol, ldx, Y, ldy, y_dtype, ep, shape=None):
    if shape is None:
        crisp.crisp_spmm_ep(desc, row_ptr, col_idx, vals, idx_words, X, Ncol, ldx, Y, ldy, y_dtype, ep)
    else:
        crisp.crisp_spmm_forced(desc, row_ptr, col_idx, vals, idx_words, X, Ncol, ldx, Y, ldy, y_dtype, ep, shape)


def conv_spmm(desc, conv, row_ptr, col_idx, vals, idx_words, act, Y, ldy, y_dtype, shape=None):
    if shape is None:
        crisp.crisp_conv_spmm(desc, conv, row_ptr, col_idx, vals, idx_words, act, Y, ldy, y_dtype)
    else:
        crisp.crisp_conv_spmm_forced(desc, conv, row_ptr, col_idx, vals, idx_words, act, Y, ldy, y_dtype, None, shape)


def conv_spmm_ep(desc, conv, row_ptr, col_idx, vals, idx_words, act, Y, ldy, y_dtype, ep, shape=None):
    if shape is None:
        crisp.crisp_conv_spmm_ep(desc, conv, row_ptr, col_idx, vals, idx_words, act, Y, ldy, y_dtype, ep)
    else:
        crisp.crisp_conv_spmm_forced(desc, conv, row_ptr, col_idx, vals, idx_words, act, Y, ldy, y_dtype, ep, shape)


def run_spmm(layer, dX, Ncol, ldx, y_dtype, S, ldy=None, fill=None, shape=None, with_code=False):
    """crisp_spmm into a fresh Y with a guard band of columns (ldy > Ncol) that must stay untouched."""
    if ldy is None:
        ldy = (Ncol + 7) // 8 * 8 + 8
    tdt = torch.float32 if y_dtype == crisp.Y_F32 else torch.bfloat16
    Y = torch.full((S + 1, ldy), float("nan") if fill is None else fill, dtype=tdt, device="cuda")
    # shape: None = the library's own choice (crisp_spmm); otherwise crisp_spmm_forced with that launch shape
    code = spmm(layer.desc, layer.row_ptr, layer.col_idx, layer.vals, layer.idx_words, dX, Ncol, ldx, Y, ldy, y_dtype, shape=shape)
    torch.cuda.synchronize()
    Yh = Y.float().cpu().numpy().astype(np.float64)
    assert np.isnan(Yh[:S, Ncol:]).all(), "columns beyond Ncol were written"
    assert np.isnan(Yh[S]).all(), "row beyond S was written"
    return (Yh[:S, :Ncol], code) if with_code else Yh[:S, :Ncol]


def check_product(Y, Yref, Aref, y_dtype, what=""):
    """Tolerance of the product: relative Frobenius error <= 2e-3 and |err| <= 1e-2 * (|W||X|)
    element-wise (bf16 inputs, fp32 accumulation).  With fp32 output the only error source is
    the summation order, so a much tighter tripwire of 1e-5 applies as well."""
    assert np.isfinite(Y).all(), what
    err = np.abs(Y - Yref)
    fro = np.linalg.norm(Y - Yref) / max(np.linalg.norm(Yref), 1e-300)
    assert fro <= 2e-3, (what, fro)
    assert (err <= 1e-2 * Aref + 1e-30).all(), (what, float((err - 1e-2 * Aref).max()))
    if y_dtype == crisp.Y_F32:
        assert fro <= 1e-5, (what, fro)
    return fro


def check_bf16_is_rounded_f32(Y16, Y32, what=""):
    """A bf16 output must be exactly the round-to-nearest-even of the fp32 output of the same launch
    shape (same fp32 arithmetic, one more rounding).  Used where the outputs are too few for the
    Frobenius bound to be a statistic of that rounding."""
    from paper_2311_14272_amd import synth
    a = synth.f32_to_bf16_bits(np.asarray(Y16, dtype=np.float32))
    b = synth.f32_to_bf16_bits(np.asarray(Y32, dtype=np.float32))
    assert (a == b).all(), (what, int((a != b).sum()))


def lowering_gather_index(C, H, W, batch, kh, kw, stride, pad, cols):
    """Flat indices into act[C][batch][H][W] of the X entries of the given output columns
    (rows ordered (kh, kw, c), c fastest) and a mask of entries that fall into the zero padding.
    Checked against the oracle's full lowering in a CPU test."""
    Ho = (H + 2 * pad - kh) // stride + 1
    Wo = (W + 2 * pad - kw) // stride + 1
    cols = np.asarray(cols, dtype=np.int64)
    img, rem = np.divmod(cols, Ho * Wo)
    oh, ow = np.divmod(rem, Wo)
    a = np.repeat(np.arange(kh), kw * C)[:, None]
    b = np.tile(np.repeat(np.arange(kw), C), kh)[:, None]
    c = np.tile(np.arange(C), kh * kw)[:, None]
    ih = oh[None, :] * stride + a - pad
    iw = ow[None, :] * stride + b - pad
    inside = (ih >= 0) & (ih < H) & (iw >= 0) & (iw < W)
    idx = ((c * batch + img[None, :]) * H + np.clip(ih, 0, H - 1)) * W + np.clip(iw, 0, W - 1)
    return idx, inside
