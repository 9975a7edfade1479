"""4:8 layers whose kept values fall two per aligned four (flags[0] == 1 from the pack) and the hint that lets the
product treat them like 2:4 on the sparse matrix-core instruction: every kernel family that consumes the hint,
against the oracle, with and without the hint."""
import numpy as np
import pytest

import oracle
from paper_2311_14272_amd import crisp, synth

from gpu_util import check_bf16_is_rounded_f32, check_product, dev, run_select_pack, run_spmm

pytestmark = pytest.mark.gpu


CASES = [
    # S, K, Ncol, B, density, select mode, forced shapes that must report the sparse instruction with the hint
    (200, 512, 520, 64, 0.5, synth.ROW_UNIFORM, (7, 8, 9, 10, 16, 17, 18, None)),
    (1024, 256, 8200, 64, 0.5, synth.ROW_UNIFORM, (8, 18, None)),            # the library's choice: X strip in LDS
    (320, 128, 264, 64, 1.0, synth.ROW_UNIFORM, (8, 13, 18)),                # X operands in registers
    (128, 1024, 4100, 64, 0.75, synth.ROW_UNIFORM, (8, 16, 17)),             # 12 blocks per row resident as sparse operands
    (96, 160, 200, 32, 0.6, synth.ROW_UNIFORM, (7, 8, 9, 10, None)),         # 32 x 32 blocks
    (200, 208, 136, 64, 0.75, synth.ROW_UNIFORM, (8, 16, 18)),               # last block column partly past K
    (256, 512, 264, 64, 0.3, synth.LAYER_TOPK, (8, 16, 18)),                 # uneven rows, some empty
]


@pytest.mark.parametrize("case", CASES, ids=lambda c: "S%d_K%d_B%d" % (c[0], c[1], c[3]))
def test_hint_sends_4_of_8_to_the_sparse_instruction(case):
    S, K, Ncol, B, dens, mode, sparse_shapes = case
    L = synth.LayerSpec("two_of_four", S, K, Ncol, 4, 8, B, dens, synth.SAL_MAG, 1.0, None, mode)
    rng = np.random.default_rng(S * 13 + K)
    W = synth.draw_two_per_quad_weight(rng, S, K)
    X = synth.draw_relu_normal(rng, (K, Ncol))
    sel = oracle.select(W, None, 4, 8, B, dens, synth.SAL_MAG, mode)
    layer, out = run_select_pack(L, W, None)
    assert int(out["flags"][0]) == 1
    Yref, Aref = oracle.gemm_masked(W, sel.mask, X)
    ldx = (Ncol + 7) // 8 * 8
    Xp = np.zeros((K, ldx), dtype=np.uint16)
    Xp[:, :Ncol] = X
    dX = dev(Xp)
    plain = layer.desc
    hinted = crisp.layer_desc(S, K, 4, 8, B, dens, synth.SAL_MAG, mode, hints=crisp.HINT_TWO_OF_FOUR)
    forced_sparse = [s for s in sparse_shapes if s is not None]
    for desc, with_hint in ((hinted, True), (plain, False)):
        layer.desc = desc
        for shape in sorted(set(forced_sparse) | {0, 1, 5, 15}) + [crisp.SHAPE_AUTO]:
            print("S", S, "K", K, "hint", with_hint, "shape", shape, flush=True)
            Y32, code = run_spmm(layer, dX, Ncol, ldx, crisp.Y_F32, S, shape=shape, with_code=True)
            sparse = crisp.kernel_code_fields(code)["sparse_mfma"]
            if shape == crisp.SHAPE_AUTO:
                if not with_hint:
                    assert sparse == 0
                elif None in sparse_shapes:
                    assert sparse == 1, crisp.kernel_code_fields(code)
            else:
                assert sparse == int(with_hint and shape in forced_sparse), (shape, with_hint, crisp.kernel_code_fields(code))
            check_product(Y32, Yref, Aref, crisp.Y_F32, "shape %s hint %s" % (shape, with_hint))
            Y16 = run_spmm(layer, dX, Ncol, ldx, crisp.Y_BF16, S, shape=shape)
            check_product(Y16, Yref, Aref, crisp.Y_BF16, "shape %s hint %s bf16" % (shape, with_hint))
            check_bf16_is_rounded_f32(Y16, Y32, "shape %s hint %s" % (shape, with_hint))
    layer.desc = plain


def test_hint_is_ignored_for_other_patterns():
    """The hint on a 2:4 layer (always eligible) and on a 3:4 layer (never): same kernels, same bits as without."""
    for (n, m) in ((2, 4), (3, 4)):
        L = synth.LayerSpec("hint_%d_%d" % (n, m), 128, 256, 264, n, m, 64, 0.5, synth.SAL_MAG, 0.05)
        W, G, X = synth.draw_small(L, 37)
        layer, _ = run_select_pack(L, W, G)
        dX = dev(np.ascontiguousarray(X))
        plain = layer.desc
        outs = []
        for hints in (0, crisp.HINT_TWO_OF_FOUR):
            layer.desc = crisp.layer_desc(L.S, L.K, n, m, 64, 0.5, synth.SAL_MAG, synth.ROW_UNIFORM, hints=hints)
            outs.append(run_spmm(layer, dX, L.Ncol, L.Ncol, crisp.Y_F32, L.S, shape=8, with_code=True))
        assert outs[0][1] == outs[1][1] and np.array_equal(outs[0][0], outs[1][0])
        layer.desc = plain


@pytest.mark.parametrize("geom", [
    # C, H, W, batch, k, stride, pad, S: strided 1x1 (the X-strip kernel gathers it; sparse instruction with the hint),
    # 3x3 (the fused-lowering kernels do not take the hint: dense expansion, same results)
    (128, 12, 12, 3, 1, 2, 0, 1100), (256, 8, 8, 4, 1, 2, 0, 192), (64, 10, 10, 2, 3, 1, 1, 128), (64, 14, 14, 2, 3, 2, 1, 256)],
    ids=lambda g: "C%d_k%d_s%d_S%d" % (g[0], g[4], g[5], g[7]))
def test_hint_with_fused_lowering(geom):
    from gpu_util import conv_spmm
    import torch
    C_, H, Wd, b, k, stride, pad, S = geom
    cv = synth.ConvShape(C_, H, Wd, b, k, k, stride, pad)
    L = synth.LayerSpec("two_of_four_conv", S, cv.K, cv.Ncol, 4, 8, 64, 0.6, synth.SAL_MAG, 1.0, conv=cv)
    rng = np.random.default_rng(C_ + S)
    W = synth.draw_two_per_quad_weight(rng, S, cv.K)
    act = synth.draw_relu_normal(rng, (C_, b, H, Wd))
    sel = oracle.select(W, None, 4, 8, 64, L.density, synth.SAL_MAG, synth.ROW_UNIFORM)
    layer, out = run_select_pack(L, W, None)
    assert int(out["flags"][0]) == 1
    Yref, Aref = oracle.gemm_masked(W, sel.mask, oracle.im2col(act, k, k, stride, pad))
    conv = crisp.conv_desc_of(cv)
    hinted = crisp.layer_desc(S, cv.K, 4, 8, 64, L.density, synth.SAL_MAG, synth.ROW_UNIFORM, hints=crisp.HINT_TWO_OF_FOUR)
    Ncol = cv.Ncol
    ld = (Ncol + 7) // 8 * 8
    dact = dev(act)
    for desc in (hinted, layer.desc):
        for shape in (None, 1, 18):
            for yd, tdt in ((crisp.Y_F32, torch.float32), (crisp.Y_BF16, torch.bfloat16)):
                Y = torch.full((S, ld), float("nan"), dtype=tdt, device="cuda")
                conv_spmm(desc, conv, layer.row_ptr, layer.col_idx, layer.vals, layer.idx_words, dact, Y, ld, yd, shape=shape)
                torch.cuda.synchronize()
                check_product(Y.float().cpu().numpy().astype(np.float64)[:, :Ncol], Yref, Aref, yd,
                              "conv %s hints %d shape %s" % (geom, desc.hints, shape))
