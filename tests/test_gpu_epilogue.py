"""Product with the optional epilogue (per-row scale and bias, residual, ReLU) against the oracle."""
import numpy as np
import pytest
import torch

import oracle
from paper_2311_14272_amd import crisp, synth

from gpu_util import dev, run_select_pack, spmm_ep, conv_spmm_ep

pytestmark = pytest.mark.gpu

CASES = [synth.small_cases()[i] for i in (0, 1, 2, 5, 7, 9, 13)] + synth.b16_cases()[:2] + [
    # short K: the kernel that keeps X in registers (forced shape 13) stores block-row by block-row
    synth.LayerSpec("ep_k128_2:8", 200, 128, 520, 2, 8, 64, 0.5, synth.SAL_MAG, 0.05),
    synth.LayerSpec("ep_k64_4:8", 256, 64, 264, 4, 8, 64, 1.0, synth.SAL_MAG, 0.05)]


def _check(Y, Yref, Aref, bf16, what):
    """The product's stated tolerance (relative Frobenius error 2e-3, |err| <= 1e-2 |W|.|X| element-wise)
    carried through the epilogue: the oracle scales |W|.|X| like the sum, the added terms are exact inputs,
    the fp32 steps round at 2^-24.  A bf16 output adds one rounding of the final value, unit roundoff
    2^-8, to an fp32 result that is itself within 1e-2 |W|.|X| of the reference: element-wise
    |err| <= 1e-2 A + 2^-8 (|Y*| + 1e-2 A); in the Frobenius norm that rounding is about 1.5e-3 (uniform
    rounding error, values spread over a binade) and stays under the stated 2e-3."""
    assert np.isfinite(Y).all(), what
    err = np.abs(Y - Yref)
    fro = np.linalg.norm(Y - Yref) / max(np.linalg.norm(Yref), 1e-300)
    assert fro <= (2e-3 if bf16 else 1e-5), (what, fro)
    u = 2.0 ** -8 if bf16 else 2.0 ** -20
    bound = 1e-2 * Aref + u * (np.abs(Yref) + 1e-2 * Aref) + 1e-30
    assert (err <= bound).all(), (what, float((err - bound).max()))


def _draw_ep(rng, S, Ncol, ldr, bf16):
    scale = rng.uniform(0.5, 2.0, size=S).astype(np.float32) * rng.choice([-1.0, 1.0], size=S).astype(np.float32)
    bias = rng.normal(0.0, 0.5, size=S).astype(np.float32)
    res = rng.normal(0.0, 1.0, size=(S, Ncol)).astype(np.float32)
    if bf16:
        res_bits = synth.f32_to_bf16_bits(res)
        res = synth.bf16_bits_to_f32(res_bits)
        pad = np.zeros((S, ldr), dtype=np.uint16)
        pad[:, :Ncol] = res_bits
    else:
        pad = np.zeros((S, ldr), dtype=np.float32)
        pad[:, :Ncol] = res
    return scale, bias, res, pad


@pytest.mark.parametrize("L", CASES, ids=lambda L: L.name)
def test_spmm_epilogue(L):
    W, G, X = synth.draw_small(L, 71)
    sel = oracle.select(W, G, L.n, L.m, L.B, L.density, L.sal_kind, L.select_mode)
    layer, _ = run_select_pack(L, W, G)
    Y0, A0 = oracle.gemm_masked(W, sel.mask, X)
    ldx = (L.Ncol + 7) // 8 * 8
    Xp = np.zeros((L.K, ldx), dtype=np.uint16)
    Xp[:, : L.Ncol] = X
    dX = dev(Xp)
    ldy = ldx + 8
    ldr = ldx
    rng = np.random.default_rng(L.S * 131 + L.K)
    combos = [dict(scale=True, bias=True, res=True, relu=True), dict(scale=False, bias=True, res=False, relu=False),
              dict(scale=True, bias=False, res=False, relu=True), dict(scale=False, bias=False, res=True, relu=False),
              dict(scale=False, bias=False, res=False, relu=True)]
    for bf16 in (False, True):
        yd = crisp.Y_BF16 if bf16 else crisp.Y_F32
        tdt = torch.bfloat16 if bf16 else torch.float32
        scale, bias, res, respad = _draw_ep(rng, L.S, L.Ncol, ldr, bf16)
        dscale, dbias, dres = dev(scale), dev(bias), dev(respad)
        for cb in combos:
            Yref, Aref = oracle.epilogue(Y0, A0, scale if cb["scale"] else None, bias if cb["bias"] else None,
                                         res if cb["res"] else None, cb["relu"])
            ep = crisp.epilogue(dscale if cb["scale"] else None, dbias if cb["bias"] else None,
                                dres if cb["res"] else None, ldr, cb["relu"])
            for shape in (None, 0, 1, 2, 4, 5, 6, 8, 13, 15, 16, 17, 18):
                Y = torch.full((L.S + 1, ldy), float("nan"), dtype=tdt, device="cuda")
                spmm_ep(layer.desc, layer.row_ptr, layer.col_idx, layer.vals, layer.idx_words, dX, L.Ncol, ldx,
                                    Y, ldy, yd, ep, shape=shape)
                torch.cuda.synchronize()
                Yh = Y.float().cpu().numpy().astype(np.float64)
                assert np.isnan(Yh[: L.S, L.Ncol:]).all() and np.isnan(Yh[L.S]).all()
                _check(Yh[: L.S, : L.Ncol], Yref, Aref, bf16, "%s %s shape %s bf16=%s" % (L.name, cb, shape, bf16))


def test_residual_with_a_very_wide_row_stride():
    """A residual whose row stride exceeds 2^23 elements (a view into a much wider tensor) while Y is
    narrow: the kernels that address a block-row with 32-bit offsets must not be used for it."""
    L = synth.LayerSpec("ep_wide_ldr", 96, 128, 264, 2, 4, 32, 0.5, synth.SAL_MAG, 0.05)
    W, G, X = synth.draw_small(L, 73)
    sel = oracle.select(W, G, L.n, L.m, L.B, L.density, L.sal_kind, L.select_mode)
    layer, _ = run_select_pack(L, W, G)
    Y0, A0 = oracle.gemm_masked(W, sel.mask, X)
    ldx = (L.Ncol + 7) // 8 * 8
    Xp = np.zeros((L.K, ldx), dtype=np.uint16)
    Xp[:, : L.Ncol] = X
    dX = dev(Xp)
    ldr = (1 << 23) + 8
    rng = np.random.default_rng(5)
    res = synth.bf16_bits_to_f32(synth.f32_to_bf16_bits(rng.normal(0.0, 1.0, size=(L.S, L.Ncol)).astype(np.float32)))
    dres = torch.zeros((L.S, ldr), dtype=torch.bfloat16, device="cuda")
    dres[:, : L.Ncol] = torch.from_numpy(res).cuda().to(torch.bfloat16)
    Yref, Aref = oracle.epilogue(Y0, A0, None, None, res, True)
    ep = crisp.epilogue(None, None, dres.view(torch.int16), ldr, True)
    for shape in (None, 1, 8):
        Y = torch.full((L.S, ldx), float("nan"), dtype=torch.bfloat16, device="cuda")
        spmm_ep(layer.desc, layer.row_ptr, layer.col_idx, layer.vals, layer.idx_words, dX, L.Ncol, ldx, Y, ldx,
                            crisp.Y_BF16, ep, shape=shape)
        torch.cuda.synchronize()
        _check(Y.float().cpu().numpy().astype(np.float64)[:, : L.Ncol], Yref, Aref, True, "wide ldr shape %s" % shape)
    # the fused lowering has no generic kernel to hand over to
    conv = crisp.ConvDesc(128, 12, 22, 1, 1, 1, 1, 0, crisp.ACT_CBHW, crisp.X_KN)
    with pytest.raises(crisp.CrispError) as e:
        crisp.crisp_conv_spmm_ep(layer.desc, conv, layer.row_ptr, layer.col_idx, layer.vals, layer.idx_words, dX, Y, ldx,
                                 crisp.Y_BF16, ep)
    assert e.value.status == crisp.EUNSUPPORTED


def test_epilogue_none_equals_plain_product():
    """ep == NULL and an epilogue with nothing switched on give the plain product, bit for bit."""
    L = synth.small_cases()[0]
    W, G, X = synth.draw_small(L, 72)
    layer, _ = run_select_pack(L, W, G)
    ldx = (L.Ncol + 7) // 8 * 8
    Xp = np.zeros((L.K, ldx), dtype=np.uint16)
    Xp[:, : L.Ncol] = X
    dX = dev(Xp)
    outs = []
    for ep in ("plain", None, crisp.epilogue()):
        Y = torch.zeros((L.S, ldx), dtype=torch.float32, device="cuda")
        if ep == "plain":
            crisp.crisp_spmm(layer.desc, layer.row_ptr, layer.col_idx, layer.vals, layer.idx_words, dX, L.Ncol, ldx, Y, ldx)
        else:
            crisp.crisp_spmm_ep(layer.desc, layer.row_ptr, layer.col_idx, layer.vals, layer.idx_words, dX, L.Ncol, ldx, Y,
                                ldx, crisp.Y_F32, ep)
        torch.cuda.synchronize()
        outs.append(Y.cpu().numpy())
    assert (outs[0] == outs[1]).all() and (outs[0] == outs[2]).all()


def test_conv_spmm_epilogue():
    """Fused lowering + epilogue (the tail of a residual block: scale, bias, shortcut, ReLU)."""
    # the last three run in the kernel that stages the input patch in LDS (also forced: shape 12): stride 1
    # and 2, with the sparse matrix-core instruction and with dense expansion, ragged S
    for (C_, H, Wd, b, k, pad, stride, S, n, m, B) in ((64, 8, 8, 2, 3, 1, 1, 64, 2, 4, 64), (32, 9, 7, 2, 3, 1, 2, 32, 4, 8, 32),
                                                       (3, 12, 12, 2, 3, 1, 1, 32, 2, 4, 32), (128, 14, 14, 2, 3, 1, 1, 256, 2, 8, 64),
                                                       (64, 28, 28, 1, 3, 1, 2, 200, 4, 8, 64), (64, 12, 12, 2, 3, 1, 1, 128, 1, 4, 64),
                                                       # few channels, 64x64 blocks: the kernel with the patch in its own layout (shape 14)
                                                       (3, 16, 16, 2, 3, 1, 1, 100, 2, 4, 64), (12, 20, 20, 1, 5, 2, 2, 64, 4, 8, 64)):
        cv = synth.ConvShape(C_, H, Wd, b, k, k, stride, pad)
        L = synth.LayerSpec("convep", S, cv.K, cv.Ncol, n, m, B, 0.6, synth.SAL_MAG, 0.05, conv=cv)
        rng = np.random.default_rng(C_ + H)
        W = synth.draw_weight(rng, L)
        act = synth.draw_relu_normal(rng, (C_, b, H, Wd))
        sel = oracle.select(W, None, n, m, B, L.density, L.sal_kind, L.select_mode)
        layer, _ = run_select_pack(L, W, None)
        Y0, A0 = oracle.gemm_masked(W, sel.mask, oracle.im2col(act, k, k, stride, pad))
        Ncol = cv.Ncol
        ld = (Ncol + 7) // 8 * 8
        for bf16 in (False, True):
            scale, bias, res, respad = _draw_ep(rng, S, Ncol, ld, bf16)
            Yref, Aref = oracle.epilogue(Y0, A0, scale, bias, res, True)
            dscale, dbias, dres = dev(scale), dev(bias), dev(respad)     # the descriptor holds raw pointers
            ep = crisp.epilogue(dscale, dbias, dres, ld, True)
            for shape in (None, 12, 14):
                Y = torch.full((S, ld), float("nan"), dtype=torch.bfloat16 if bf16 else torch.float32, device="cuda")
                conv_spmm_ep(layer.desc, crisp.conv_desc_of(cv), layer.row_ptr, layer.col_idx, layer.vals,
                                         layer.idx_words, dev(act), Y, ld, crisp.Y_BF16 if bf16 else crisp.Y_F32, ep, shape=shape)
                torch.cuda.synchronize()
                Yh = Y.float().cpu().numpy().astype(np.float64)
                _check(Yh[:, :Ncol], Yref, Aref, bf16, "conv epilogue C=%d bf16=%s shape %s" % (C_, bf16, shape))
