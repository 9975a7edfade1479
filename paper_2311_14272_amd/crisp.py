"""Thin binding of libcrisp.so: argument marshalling only, every step runs in the HIP kernels.

Function names mirror the C ABI (include/crisp.h).  Device buffers are torch tensors used as
plain memory; the current torch stream is passed as the HIP stream.
"""
from __future__ import annotations

import ctypes as C
import os
from dataclasses import dataclass
from typing import Optional

HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(HERE, "libcrisp.so")

OK, EINVAL, ESHAPE, EBUFSIZE, EALIGN, EUNSUPPORTED, EDEVICE = range(7)
SAL_GIVEN, SAL_GRAD, SAL_MAG = 0, 1, 2
ROW_UNIFORM, LAYER_TOPK = 0, 1
X_KN, X_K8 = 0, 1
HINT_TWO_OF_FOUR = 1
Y_F32, Y_BF16 = 0, 1
ACT_CBHW = 0


class LayerDesc(C.Structure):
    _fields_ = [("block_density", C.c_double), ("S", C.c_int32), ("K", C.c_int32), ("n", C.c_int32),
                ("m", C.c_int32), ("B", C.c_int32), ("sal_kind", C.c_int32), ("select_mode", C.c_int32),
                ("hints", C.c_int32)]


class Sizes(C.Structure):
    _fields_ = [("Sb", C.c_int32), ("Kb", C.c_int32), ("k_row", C.c_int32), ("nk", C.c_int32),
                ("slots_per_row", C.c_int32), ("idx_bits", C.c_int32), ("idx_words_per_row", C.c_int32),
                ("mask_words_per_row", C.c_int32), ("mask_words", C.c_int64), ("row_ptr_elems", C.c_int64),
                ("col_idx_elems", C.c_int64), ("score_elems", C.c_int64), ("vals_elems", C.c_int64),
                ("idx_words", C.c_int64), ("flags_elems", C.c_int64), ("select_ws_bytes", C.c_size_t),
                ("pack_ws_bytes", C.c_size_t), ("spmm_ws_bytes", C.c_size_t), ("select_pack_ws_bytes", C.c_size_t)]


class ConvDesc(C.Structure):
    _fields_ = [("C", C.c_int32), ("H", C.c_int32), ("W", C.c_int32), ("batch", C.c_int32), ("kh", C.c_int32),
                ("kw", C.c_int32), ("stride", C.c_int32), ("pad", C.c_int32), ("act_layout", C.c_int32),
                ("x_layout", C.c_int32)]


class LayerBuffers(C.Structure):
    _fields_ = [("W", C.c_void_p), ("T_or_G", C.c_void_p), ("nm_mask", C.c_void_p), ("row_ptr", C.c_void_p),
                ("col_idx", C.c_void_p), ("block_score", C.c_void_p), ("vals", C.c_void_p), ("idx_words", C.c_void_p),
                ("flags", C.c_void_p), ("ws", C.c_void_p), ("ws_bytes", C.c_size_t)]


class Epilogue(C.Structure):
    _fields_ = [("scale", C.c_void_p), ("bias", C.c_void_p), ("residual", C.c_void_p), ("ldr", C.c_int64),
                ("relu", C.c_int32), ("reserved", C.c_int32)]


def epilogue(scale=None, bias=None, residual=None, ldr=0, relu=False) -> Epilogue:
    """Epilogue descriptor from device tensors (kept alive by the caller)."""
    return Epilogue(_ptr(scale), _ptr(bias), _ptr(residual), int(ldr), 1 if relu else 0, 0)


class CrispError(RuntimeError):
    def __init__(self, fn: str, status: int):
        self.status = status
        super().__init__("%s: %s (status %d)" % (fn, status_str(status), status))


_lib = None


def lib():
    """Load libcrisp.so; there is no fallback path when it is missing."""
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise RuntimeError("libcrisp.so is not built (run `python -m paper_2311_14272_amd.build`); "
                               "there is no CPU fallback")
        L = C.CDLL(LIB_PATH)
        vp = C.c_void_p
        L.crisp_status_str.restype = C.c_char_p
        L.crisp_status_str.argtypes = [C.c_int32]
        L.crisp_pack_sizes.argtypes = [C.POINTER(LayerDesc), C.POINTER(Sizes)]
        L.crisp_select_mask.argtypes = [C.POINTER(LayerDesc), vp, vp, vp, vp, vp, vp, vp, C.c_size_t, vp]
        L.crisp_pack.argtypes = [C.POINTER(LayerDesc), vp, vp, vp, vp, vp, vp, vp, vp, C.c_size_t, vp]
        L.crisp_select_pack.argtypes = [C.POINTER(LayerDesc), vp, vp, vp, vp, vp, vp, vp, vp, vp, vp, C.c_size_t, vp]
        L.crisp_select_pack_noalloc.argtypes = [C.POINTER(LayerDesc), vp, vp, vp, vp, vp, vp, vp, vp, vp, vp]
        L.crisp_select_pack_batch.argtypes = [C.c_int32, C.POINTER(LayerDesc), C.POINTER(LayerBuffers), vp]
        L.crisp_im2col.argtypes = [C.POINTER(ConvDesc), vp, vp, C.c_int64, vp]
        L.crisp_spmm.argtypes = [C.POINTER(LayerDesc), vp, vp, vp, vp, vp, C.c_int64, C.c_int64, C.c_int32, vp,
                                 C.c_int64, C.c_int32, vp, C.c_size_t, vp]
        L.crisp_conv_spmm.argtypes = [C.POINTER(LayerDesc), C.POINTER(ConvDesc), vp, vp, vp, vp, vp, vp, C.c_int64,
                                      C.c_int32, vp, C.c_size_t, vp]
        L.crisp_maxpool.argtypes = [C.POINTER(ConvDesc), vp, vp, vp]
        L.crisp_maxpool.restype = C.c_int32
        L.crisp_spmm_ep.argtypes = [C.POINTER(LayerDesc), vp, vp, vp, vp, vp, C.c_int64, C.c_int64, C.c_int32, vp,
                                    C.c_int64, C.c_int32, C.POINTER(Epilogue), vp, C.c_size_t, vp]
        L.crisp_conv_spmm_ep.argtypes = [C.POINTER(LayerDesc), C.POINTER(ConvDesc), vp, vp, vp, vp, vp, vp, C.c_int64,
                                         C.c_int32, C.POINTER(Epilogue), vp, C.c_size_t, vp]
        L.crisp_spmm_forced.argtypes = [C.POINTER(LayerDesc), vp, vp, vp, vp, vp, C.c_int64, C.c_int64, C.c_int32, vp,
                                        C.c_int64, C.c_int32, C.POINTER(Epilogue), C.c_int32, C.POINTER(C.c_int32), vp]
        L.crisp_conv_spmm_forced.argtypes = [C.POINTER(LayerDesc), C.POINTER(ConvDesc), vp, vp, vp, vp, vp, vp, C.c_int64,
                                             C.c_int32, C.POINTER(Epilogue), C.c_int32, C.POINTER(C.c_int32), vp]
        L.crisp_spmm_timed.argtypes = [C.POINTER(LayerDesc), C.POINTER(ConvDesc), vp, vp, vp, vp, vp, C.c_int64,
                                       C.c_int64, vp, C.c_int64, C.c_int32, vp, vp, vp]
        L.crisp_global_budget.argtypes = [C.c_int32, vp, vp, C.c_double, vp, vp, vp, C.c_size_t, vp]
        L.crisp_conv_plan.argtypes = [C.POINTER(LayerDesc), C.POINTER(ConvDesc), C.POINTER(C.c_int32), C.POINTER(C.c_size_t)]
        L.crisp_conv_forward.argtypes = [C.POINTER(LayerDesc), C.POINTER(ConvDesc), vp, vp, vp, vp, vp, vp, C.c_int64, C.c_int32,
                                         C.POINTER(Epilogue), vp, C.c_size_t, C.POINTER(C.c_int32), vp]
        for f in (L.crisp_pack_sizes, L.crisp_select_mask, L.crisp_pack, L.crisp_select_pack, L.crisp_select_pack_batch,
                  L.crisp_select_pack_noalloc,
                  L.crisp_im2col, L.crisp_spmm, L.crisp_spmm_ep, L.crisp_conv_spmm_ep,
                  L.crisp_conv_spmm, L.crisp_spmm_timed, L.crisp_spmm_forced, L.crisp_conv_spmm_forced, L.crisp_global_budget, L.crisp_conv_plan, L.crisp_conv_forward):
            f.restype = C.c_int32
        _lib = L
    return _lib


def status_str(st: int) -> str:
    return lib().crisp_status_str(st).decode()


def _ptr(t) -> Optional[int]:
    if t is None:
        return None
    if isinstance(t, int):
        return t
    return t.data_ptr()


def _stream() -> Optional[int]:
    import torch
    return torch.cuda.current_stream().cuda_stream or None


def layer_desc(S, K, n, m, B, block_density=1.0, sal_kind=SAL_MAG, select_mode=ROW_UNIFORM, hints=0) -> LayerDesc:
    return LayerDesc(float(block_density), S, K, n, m, B, sal_kind, select_mode, hints)


def crisp_pack_sizes(desc: LayerDesc) -> Sizes:
    out = Sizes()
    st = lib().crisp_pack_sizes(C.byref(desc), C.byref(out))
    if st != OK:
        raise CrispError("crisp_pack_sizes", st)
    return out


def crisp_select_mask(desc, W, T_or_G, nm_mask, row_ptr, col_idx, block_score=None, ws=None, ws_bytes=0, stream=-1):
    st = lib().crisp_select_mask(C.byref(desc), _ptr(W), _ptr(T_or_G), _ptr(nm_mask), _ptr(row_ptr), _ptr(col_idx),
                                 _ptr(block_score), _ptr(ws), ws_bytes, _stream() if stream == -1 else stream)
    if st != OK:
        raise CrispError("crisp_select_mask", st)


def crisp_pack(desc, W, nm_mask, row_ptr, col_idx, vals, idx_words, flags, ws=None, ws_bytes=0, stream=-1):
    st = lib().crisp_pack(C.byref(desc), _ptr(W), _ptr(nm_mask), _ptr(row_ptr), _ptr(col_idx), _ptr(vals),
                          _ptr(idx_words), _ptr(flags), _ptr(ws), ws_bytes, _stream() if stream == -1 else stream)
    if st != OK:
        raise CrispError("crisp_pack", st)


def crisp_select_pack(desc, W, T_or_G, nm_mask, row_ptr, col_idx, vals, idx_words, flags, ws, ws_bytes, block_score=None,
                      stream=-1):
    st = lib().crisp_select_pack(C.byref(desc), _ptr(W), _ptr(T_or_G), _ptr(nm_mask), _ptr(row_ptr), _ptr(col_idx),
                                 _ptr(block_score), _ptr(vals), _ptr(idx_words), _ptr(flags), _ptr(ws), ws_bytes,
                                 _stream() if stream == -1 else stream)
    if st != OK:
        raise CrispError("crisp_select_pack", st)


STATIC_SCRATCH_BYTES = 8 << 20


def crisp_select_pack_noalloc(desc, W, T_or_G, nm_mask, row_ptr, col_idx, vals, idx_words, flags, block_score=None, stream=-1):
    st = lib().crisp_select_pack_noalloc(C.byref(desc), _ptr(W), _ptr(T_or_G), _ptr(nm_mask), _ptr(row_ptr), _ptr(col_idx),
                                         _ptr(block_score), _ptr(vals), _ptr(idx_words), _ptr(flags),
                                         _stream() if stream == -1 else stream)
    if st != OK:
        raise CrispError("crisp_select_pack_noalloc", st)


def crisp_select_pack_batch(descs, buffers, stream=-1):
    """descs: ctypes array of LayerDesc, buffers: ctypes array of LayerBuffers (see make_batch)."""
    st = lib().crisp_select_pack_batch(len(descs), descs, buffers, _stream() if stream == -1 else stream)
    if st != OK:
        raise CrispError("crisp_select_pack_batch", st)


def crisp_im2col(conv: ConvDesc, act, X, ldx, stream=-1):
    st = lib().crisp_im2col(C.byref(conv), _ptr(act), _ptr(X), ldx, _stream() if stream == -1 else stream)
    if st != OK:
        raise CrispError("crisp_im2col", st)


def crisp_spmm(desc, row_ptr, col_idx, vals, idx_words, X, Ncol, ldx, Y, ldy, y_dtype=Y_F32, x_layout=X_KN,
               ws=None, ws_bytes=0, stream=-1):
    st = lib().crisp_spmm(C.byref(desc), _ptr(row_ptr), _ptr(col_idx), _ptr(vals), _ptr(idx_words), _ptr(X), Ncol,
                          ldx, x_layout, _ptr(Y), ldy, y_dtype, _ptr(ws), ws_bytes,
                          _stream() if stream == -1 else stream)
    if st != OK:
        raise CrispError("crisp_spmm", st)


def crisp_conv_spmm(desc, conv: ConvDesc, row_ptr, col_idx, vals, idx_words, act, Y, ldy, y_dtype=Y_F32, ws=None,
                    ws_bytes=0, stream=-1):
    st = lib().crisp_conv_spmm(C.byref(desc), C.byref(conv), _ptr(row_ptr), _ptr(col_idx), _ptr(vals),
                               _ptr(idx_words), _ptr(act), _ptr(Y), ldy, y_dtype, _ptr(ws), ws_bytes,
                               _stream() if stream == -1 else stream)
    if st != OK:
        raise CrispError("crisp_conv_spmm", st)


def crisp_maxpool(pool: ConvDesc, act, out, stream=-1):
    st = lib().crisp_maxpool(C.byref(pool), _ptr(act), _ptr(out), _stream() if stream == -1 else stream)
    if st != OK:
        raise CrispError("crisp_maxpool", st)


def crisp_spmm_ep(desc, row_ptr, col_idx, vals, idx_words, X, Ncol, ldx, Y, ldy, y_dtype, ep: Epilogue, x_layout=X_KN,
                  ws=None, ws_bytes=0, stream=-1):
    st = lib().crisp_spmm_ep(C.byref(desc), _ptr(row_ptr), _ptr(col_idx), _ptr(vals), _ptr(idx_words), _ptr(X), Ncol,
                             ldx, x_layout, _ptr(Y), ldy, y_dtype, C.byref(ep) if ep is not None else None, _ptr(ws),
                             ws_bytes, _stream() if stream == -1 else stream)
    if st != OK:
        raise CrispError("crisp_spmm_ep", st)


def crisp_conv_spmm_ep(desc, conv: ConvDesc, row_ptr, col_idx, vals, idx_words, act, Y, ldy, y_dtype, ep: Epilogue,
                       ws=None, ws_bytes=0, stream=-1):
    st = lib().crisp_conv_spmm_ep(C.byref(desc), C.byref(conv), _ptr(row_ptr), _ptr(col_idx), _ptr(vals),
                                  _ptr(idx_words), _ptr(act), _ptr(Y), ldy, y_dtype,
                                  C.byref(ep) if ep is not None else None, _ptr(ws), ws_bytes,
                                  _stream() if stream == -1 else stream)
    if st != OK:
        raise CrispError("crisp_conv_spmm_ep", st)


SHAPE_AUTO = -1
KERNEL_FAMILIES = {1: "reg", 2: "generic", 3: "lds", 4: "xres", 5: "conv_lds", 6: "conv_patch", 7: "b16", 8: "balanced", 9: "k8", 10: "xlds"}


def crisp_spmm_forced(desc, row_ptr, col_idx, vals, idx_words, X, Ncol, ldx, Y, ldy, y_dtype, ep=None, shape=SHAPE_AUTO,
                      x_layout=X_KN, stream=-1) -> int:
    """crisp_spmm_forced (tests, tuning): returns the kernel code of the launch."""
    code = C.c_int32(0)
    st = lib().crisp_spmm_forced(C.byref(desc), _ptr(row_ptr), _ptr(col_idx), _ptr(vals), _ptr(idx_words), _ptr(X), Ncol,
                                 ldx, x_layout, _ptr(Y), ldy, y_dtype, C.byref(ep) if ep is not None else None, shape,
                                 C.byref(code), _stream() if stream == -1 else stream)
    if st != OK:
        raise CrispError("crisp_spmm_forced", st)
    return code.value


def crisp_conv_spmm_forced(desc, conv: ConvDesc, row_ptr, col_idx, vals, idx_words, act, Y, ldy, y_dtype, ep=None,
                           shape=SHAPE_AUTO, stream=-1) -> int:
    """crisp_conv_spmm_forced (tests, tuning): returns the kernel code of the launch."""
    code = C.c_int32(0)
    st = lib().crisp_conv_spmm_forced(C.byref(desc), C.byref(conv), _ptr(row_ptr), _ptr(col_idx), _ptr(vals),
                                      _ptr(idx_words), _ptr(act), _ptr(Y), ldy, y_dtype,
                                      C.byref(ep) if ep is not None else None, shape, C.byref(code),
                                      _stream() if stream == -1 else stream)
    if st != OK:
        raise CrispError("crisp_conv_spmm_forced", st)
    return code.value


def kernel_code_fields(code: int) -> dict:
    """The fields of a kernel code as crisp_spmm_forced reports it."""
    return {"family": KERNEL_FAMILIES.get(code & 0xFF, "?"), "shape": (code >> 8) & 0xFF, "conv_mode": (code >> 16) & 0xFF,
            "sparse_mfma": (code >> 24) & 1}


def crisp_spmm_timed(desc, conv, row_ptr, col_idx, vals, idx_words, X_or_act, Ncol, ldx, Y, ldy, y_dtype,
                     start_event, stop_event, stream=-1):
    """start_event / stop_event: raw hipEvent_t handles (see HipEvents)."""
    st = lib().crisp_spmm_timed(C.byref(desc), C.byref(conv) if conv is not None else None, _ptr(row_ptr),
                                _ptr(col_idx), _ptr(vals), _ptr(idx_words), _ptr(X_or_act), Ncol, ldx, _ptr(Y), ldy,
                                y_dtype, start_event, stop_event, _stream() if stream == -1 else stream)
    if st != OK:
        raise CrispError("crisp_spmm_timed", st)


def crisp_global_budget(descs, score_tensors, target_sparsity, k_row, achieved=None, ws=None, ws_bytes=0, stream=-1):
    """descs: list of LayerDesc; score_tensors: list of device tensors (Sb x Kb fp64)."""
    n = len(descs)
    darr = (LayerDesc * n)(*descs)
    parr = (C.c_void_p * n)(*[_ptr(t) for t in score_tensors])
    st = lib().crisp_global_budget(n, darr, parr, float(target_sparsity), _ptr(k_row), _ptr(achieved), _ptr(ws),
                                   ws_bytes, _stream() if stream == -1 else stream)
    if st != OK:
        raise CrispError("crisp_global_budget", st)


class HipEvents:
    """A pool of raw hipEvent_t pairs (timing enabled) from the HIP runtime torch already loaded."""

    def __init__(self, pairs: int):
        self.hip = C.CDLL("libamdhip64.so")
        self.hip.hipEventElapsedTime.argtypes = [C.POINTER(C.c_float), C.c_void_p, C.c_void_p]
        self.pairs = []
        for _ in range(pairs):
            a, b = C.c_void_p(), C.c_void_p()
            if self.hip.hipEventCreate(C.byref(a)) != 0 or self.hip.hipEventCreate(C.byref(b)) != 0:
                raise RuntimeError("hipEventCreate failed")
            self.pairs.append((a, b))

    def elapsed_ms(self, i: int) -> float:
        a, b = self.pairs[i]
        out = C.c_float()
        rc = self.hip.hipEventElapsedTime(C.byref(out), a, b)
        if rc != 0:
            raise RuntimeError("hipEventElapsedTime failed (%d)" % rc)
        return out.value

    def __del__(self):
        for a, b in self.pairs:
            self.hip.hipEventDestroy(a)
            self.hip.hipEventDestroy(b)


@dataclass
class DeviceLayer:
    """Device buffers of one pruned layer (plain torch tensors used as memory)."""
    desc: LayerDesc
    sizes: Sizes
    nm_mask: object
    row_ptr: object
    col_idx: object
    score: object
    vals: object
    idx_words: object
    flags: object
    ws: object = None          # workspace of crisp_select_pack (allocated on first use)


def alloc_layer(desc: LayerDesc, device="cuda") -> DeviceLayer:
    """Allocate the outputs of crisp_select_mask and crisp_pack for a layer."""
    import torch
    sz = crisp_pack_sizes(desc)
    i32, dev = torch.int32, device
    return DeviceLayer(
        desc, sz,
        torch.empty(max(1, sz.mask_words), dtype=i32, device=dev),
        torch.empty(sz.row_ptr_elems, dtype=i32, device=dev),
        torch.empty(max(1, sz.col_idx_elems), dtype=i32, device=dev),
        torch.empty(sz.score_elems, dtype=torch.float64, device=dev),
        torch.empty(max(1, sz.vals_elems), dtype=torch.int16, device=dev),
        torch.empty(max(1, sz.idx_words), dtype=i32, device=dev),
        torch.empty(4, dtype=i32, device=dev))


def prune_and_pack(layer: DeviceLayer, W, T_or_G=None, fused=True):
    """Selection and packing on the current stream: crisp_select_pack, or (fused=False)
    crisp_select_mask followed by crisp_pack.  Both leave the same bytes in the layer's buffers."""
    if fused:
        if layer.ws is None:
            import torch
            layer.ws = torch.empty(max(16, layer.sizes.select_pack_ws_bytes), dtype=torch.uint8, device=W.device)
        crisp_select_pack(layer.desc, W, T_or_G, layer.nm_mask, layer.row_ptr, layer.col_idx, layer.vals, layer.idx_words,
                          layer.flags, layer.ws, layer.ws.numel(), block_score=layer.score)
        return
    crisp_select_mask(layer.desc, W, T_or_G, layer.nm_mask, layer.row_ptr, layer.col_idx, layer.score)
    crisp_pack(layer.desc, W, layer.nm_mask, layer.row_ptr, layer.col_idx, layer.vals, layer.idx_words, layer.flags)


def make_batch(layers, Ws, TGs):
    """Argument arrays of crisp_select_pack_batch for DeviceLayers and their weight / saliency tensors
    (built once; the arrays hold raw device pointers, so the tensors must stay alive)."""
    import torch
    n = len(layers)
    descs = (LayerDesc * n)()
    bufs = (LayerBuffers * n)()
    for i, (layer, W, TG) in enumerate(zip(layers, Ws, TGs)):
        if layer.ws is None:
            layer.ws = torch.empty(max(16, layer.sizes.select_pack_ws_bytes), dtype=torch.uint8, device=W.device)
        descs[i] = layer.desc
        bufs[i] = LayerBuffers(_ptr(W), _ptr(TG), _ptr(layer.nm_mask), _ptr(layer.row_ptr), _ptr(layer.col_idx),
                               _ptr(layer.score), _ptr(layer.vals), _ptr(layer.idx_words), _ptr(layer.flags),
                               _ptr(layer.ws), layer.ws.numel())
    return descs, bufs


def conv_desc_of(cv) -> ConvDesc:
    """ConvDesc from a synth.ConvShape-like object (C, H, W, batch, kh, kw, stride, pad)."""
    return ConvDesc(cv.C, cv.H, cv.W, cv.batch, cv.kh, cv.kw, cv.stride, cv.pad, ACT_CBHW, X_KN)


CONV_PATHS = ("none", "fused", "im2col")     # CRISP_CONV_DIRECT, CRISP_CONV_FUSED, CRISP_CONV_IM2COL


def conv_plan(desc: LayerDesc, cv):
    """crisp_conv_plan: (path, scratch bytes) for a layer descriptor and a ConvShape-like geometry."""
    path = C.c_int32(-1)
    nbytes = C.c_size_t(0)
    conv = conv_desc_of(cv)
    st = lib().crisp_conv_plan(C.byref(desc), C.byref(conv), C.byref(path), C.byref(nbytes))
    if st != OK:
        raise CrispError("crisp_conv_plan", st)
    return CONV_PATHS[path.value], nbytes.value


def lowering_path(cv, B: int, n: int, m: int, S: int, density: float) -> str:
    """How the library runs this convolution: "none" (act is X), "fused" (crisp_conv_spmm) or "im2col"
    (crisp_im2col into a scratch X, then crisp_spmm); the rule itself lives in crisp_conv_plan."""
    return conv_plan(layer_desc(S, cv.kh * cv.kw * cv.C, n, m, B, density), cv)[0]


def conv_needs_scratch(cv, B: int, n: int, m: int, S: int, density: float) -> bool:
    """Whether conv_forward needs an X scratch buffer (K x round_up(Ncol, 8) bf16) for this layer."""
    return lowering_path(cv, B, n, m, S, density) == "im2col"


def conv_forward(layer: DeviceLayer, cv, act, Y, ldy, y_dtype=Y_F32, X_scratch=None, ep=None, stream=-1):
    """crisp_conv_forward on the current stream: the product of a packed layer with a convolution input
    act [C][batch][H][W].  X_scratch (K x round_up(Ncol, 8) bf16, allocated by the caller) is needed where
    crisp_conv_plan says so.  Returns the path taken."""
    taken = C.c_int32(-1)
    conv = conv_desc_of(cv)
    nbytes = 0 if X_scratch is None else X_scratch.numel() * X_scratch.element_size()
    st = lib().crisp_conv_forward(C.byref(layer.desc), C.byref(conv), _ptr(layer.row_ptr), _ptr(layer.col_idx), _ptr(layer.vals),
                                  _ptr(layer.idx_words), _ptr(act), _ptr(Y), ldy, y_dtype,
                                  C.byref(ep) if ep is not None else None, _ptr(X_scratch), nbytes, C.byref(taken),
                                  _stream() if stream == -1 else stream)
    if st == EBUFSIZE and X_scratch is None:
        raise ValueError("this convolution needs an X scratch buffer of K x round_up(Ncol, 8) bf16")
    if st != OK:
        raise CrispError("crisp_conv_forward", st)
    return CONV_PATHS[taken.value]


