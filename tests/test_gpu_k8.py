"""Product over octet-interleaved operands (x_layout = CRISP_X_K8: X as [K/8][ldx][8], Y written as
[S/8][ldy][8]) against the oracle.  The layout change is made on the host (a pure permutation of the
same bf16 bits); selection and packing are the usual device calls."""
import numpy as np
import pytest
import torch

import oracle
from paper_2311_14272_amd import crisp, synth

from gpu_util import check_bf16_is_rounded_f32, check_product, dev, run_select_pack
from test_gpu_epilogue import _check as check_epilogue_product

pytestmark = pytest.mark.gpu


def to_k8(X, ld, fill=0x7FC0):
    """K x Ncol bits -> [K/8][ld][8] with NaN in the padding columns."""
    K, N = X.shape
    out = np.full((K // 8, ld, 8), fill, dtype=X.dtype)
    out[:, :N, :] = X.reshape(K // 8, 8, N).transpose(0, 2, 1)
    return out


def from_k8(Y8, S, N):
    return Y8.reshape(S // 8, -1, 8).transpose(0, 2, 1).reshape(S, -1)[:, :N]


mk = synth.LayerSpec
CASES = [
    mk("k8_2:4_b64", 128, 320, 328, 2, 4, 64, 0.5, synth.SAL_GRAD, 0.05),
    mk("k8_1:4_b32", 96, 160, 203, 1, 4, 32, 0.5, synth.SAL_MAG, 0.05),          # Ncol not a multiple of 4
    mk("k8_2:8_b64_ragged", 72, 144, 520, 2, 8, 64, 0.67, synth.SAL_MAG, 0.05),  # S and K no multiples of B
    mk("k8_1:8_b64", 64, 192, 72, 1, 8, 64, 0.67, synth.SAL_MAG, 0.05),
    mk("k8_3:4_b32", 64, 96, 264, 3, 4, 32, 0.67, synth.SAL_MAG, 0.05),
    mk("k8_4:8_b64", 192, 256, 136, 4, 8, 64, 0.5, synth.SAL_GRAD, 0.05),
    mk("k8_4:4_b32", 64, 128, 96, 4, 4, 32, 0.5, synth.SAL_MAG, 0.05),
    mk("k8_8:8_b64", 64, 128, 160, 8, 8, 64, 0.5, synth.SAL_MAG, 0.05),
    mk("k8_uneven", 256, 512, 264, 2, 4, 64, 0.3, synth.SAL_GRAD, 0.05, None, synth.LAYER_TOPK),   # empty block-rows
    mk("k8_many_strips", 128, 256, 4100, 1, 4, 64, 0.5, synth.SAL_MAG, 0.05),
]


@pytest.mark.parametrize("L", CASES, ids=lambda L: L.name)
def test_k8_product(L):
    W, G, X = synth.draw_small(L, 61)
    sel = oracle.select(W, G, L.n, L.m, L.B, L.density, L.sal_kind, L.select_mode)
    layer, out = run_select_pack(L, W, G)
    assert (out["row_ptr"] == sel.row_ptr).all() and (out["col_idx"] == sel.col_idx).all()
    Yref, Aref = oracle.gemm_masked(W, sel.mask, X)
    S, K, N = L.S, L.K, L.Ncol
    ldx = (N + 7) // 8 * 8 + 8
    ldy = (N + 7) // 8 * 8 + 16
    dX8 = dev(to_k8(X, ldx))
    Y32 = None
    for yd, tdt in ((crisp.Y_F32, torch.float32), (crisp.Y_BF16, torch.bfloat16)):
        Y8 = torch.full((S // 8 + 1, ldy, 8), float("nan"), dtype=tdt, device="cuda")
        code = crisp.crisp_spmm_forced(layer.desc, layer.row_ptr, layer.col_idx, layer.vals, layer.idx_words, dX8, N, ldx, Y8, ldy, yd,
                                       None, crisp.SHAPE_AUTO, x_layout=crisp.X_K8)
        torch.cuda.synchronize()
        assert crisp.kernel_code_fields(code)["family"] == "k8"
        Yh = Y8.float().cpu().numpy().astype(np.float64)
        assert np.isnan(Yh[S // 8]).all(), "octet beyond S was written"
        assert np.isnan(Yh[: S // 8, N:, :]).all(), "columns beyond Ncol were written"
        Y = from_k8(Yh[: S // 8], S, N)
        check_product(Y, Yref, Aref, yd, "%s y_dtype %d" % (L.name, yd))
        if yd == crisp.Y_F32:
            Y32 = Y
        else:
            check_bf16_is_rounded_f32(Y, Y32, L.name)
    # the plain entry point takes the layout too
    Y8 = torch.full((S // 8, ldy, 8), float("nan"), dtype=torch.float32, device="cuda")
    crisp.crisp_spmm(layer.desc, layer.row_ptr, layer.col_idx, layer.vals, layer.idx_words, dX8, N, ldx, Y8, ldy, crisp.Y_F32,
                     x_layout=crisp.X_K8)
    torch.cuda.synchronize()
    assert (from_k8(Y8.cpu().numpy().astype(np.float64), S, N) == Y32).all()


@pytest.mark.parametrize("L", [CASES[0], CASES[2], CASES[5], CASES[8]], ids=lambda L: L.name)
def test_k8_epilogue(L):
    """Scale, bias, residual (in the output's interleaved layout) and ReLU."""
    W, G, X = synth.draw_small(L, 62)
    sel = oracle.select(W, G, L.n, L.m, L.B, L.density, L.sal_kind, L.select_mode)
    layer, _ = run_select_pack(L, W, G)
    Y0, A0 = oracle.gemm_masked(W, sel.mask, X)
    S, K, N = L.S, L.K, L.Ncol
    ld = (N + 7) // 8 * 8 + 8
    rng = np.random.default_rng(5)
    scale = rng.uniform(0.5, 2.0, size=S).astype(np.float32) * rng.choice([-1.0, 1.0], size=S).astype(np.float32)
    bias = rng.normal(0.0, 0.5, size=S).astype(np.float32)
    dX8 = dev(to_k8(X, ld))
    for bf16 in (False, True):
        res = rng.normal(0.0, 1.0, size=(S, N)).astype(np.float32)
        if bf16:
            bits = synth.f32_to_bf16_bits(res)
            res = synth.bf16_bits_to_f32(bits)
            res8 = to_k8(bits, ld, fill=0)
        else:
            res8 = to_k8(res, ld, fill=0)
        dscale, dbias, dres = dev(scale), dev(bias), dev(res8)
        for cb in (dict(scale=True, bias=True, res=True, relu=True), dict(scale=False, bias=True, res=False, relu=False),
                   dict(scale=True, bias=False, res=True, relu=False)):
            Yref, Aref = oracle.epilogue(Y0, A0, scale if cb["scale"] else None, bias if cb["bias"] else None,
                                         res if cb["res"] else None, cb["relu"])
            ep = crisp.epilogue(dscale if cb["scale"] else None, dbias if cb["bias"] else None, dres if cb["res"] else None, ld, cb["relu"])
            Y8 = torch.full((S // 8, ld, 8), float("nan"), dtype=torch.bfloat16 if bf16 else torch.float32, device="cuda")
            crisp.crisp_spmm_ep(layer.desc, layer.row_ptr, layer.col_idx, layer.vals, layer.idx_words, dX8, N, ld, Y8, ld,
                                crisp.Y_BF16 if bf16 else crisp.Y_F32, ep, x_layout=crisp.X_K8)
            torch.cuda.synchronize()
            Y = from_k8(Y8.float().cpu().numpy().astype(np.float64), S, N)
            check_epilogue_product(Y, Yref, Aref, bf16, "%s %s bf16=%s" % (L.name, cb, bf16))


def test_k8_rejects_what_it_does_not_cover():
    L = mk("k8_bad", 60, 128, 64, 2, 4, 32, 0.5, synth.SAL_MAG, 0.05)        # S not a multiple of 8
    W, G, X = synth.draw_small(L, 63)
    layer, _ = run_select_pack(L, W, G)
    Y = torch.empty((8, 64, 8), dtype=torch.float32, device="cuda")
    with pytest.raises(crisp.CrispError) as e:
        crisp.crisp_spmm(layer.desc, layer.row_ptr, layer.col_idx, layer.vals, layer.idx_words, dev(to_k8(X, 64)), 64, 64, Y, 64,
                         crisp.Y_F32, x_layout=crisp.X_K8)
    assert e.value.status == crisp.EUNSUPPORTED
