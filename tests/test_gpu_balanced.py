"""Product over block-rows of very uneven length (plain block pruning over the whole grid): the kernel
that deals the block list evenly to the waves (forced launch shape 15, and the library's own choice for
CRISP_LAYER_TOPK layers) against the oracle.  The skew comes from the saliency handed in
(CRISP_SAL_GIVEN): block-rows are scaled so that the whole-grid block choice concentrates the kept
blocks in a few rows and leaves others empty; selection and packing run on the device as usual and
are compared bit for bit first."""
import numpy as np
import pytest
import torch

import oracle
from paper_2311_14272_amd import crisp, synth

from gpu_util import check_bf16_is_rounded_f32, check_product, dev, run_select_pack, run_spmm, spmm

pytestmark = pytest.mark.gpu

BALANCED = 15


def _skewed_layer(name, S, K, Ncol, n, m, B, density, row_scale, seed):
    """Weights N(0, 0.05), saliency |W| times a per-block-row factor."""
    L = synth.LayerSpec(name, S, K, Ncol, n, m, B, density, synth.SAL_GIVEN, 0.05, None, synth.LAYER_TOPK)
    rng = np.random.Generator(np.random.PCG64([synth.SEED_BASE, seed]))
    W = synth.draw_weight(rng, L)
    X = synth.draw_relu_normal(rng, (K, Ncol))
    Sb = (S + B - 1) // B
    scale = np.asarray([row_scale(bi, Sb) for bi in range(Sb)], dtype=np.float32)
    T = (np.abs(synth.bf16_bits_to_f32(W)) * np.repeat(scale, B)[:S, None]).astype(np.float32)
    return L, W, T, X


CASES = [
    # two rows take everything, six stay empty
    ("two_heavy", 512, 1024, 712, 2, 4, 64, 0.25, lambda bi, Sb: 1000.0 if bi in (1, 6) else 1.0),
    # geometric decay over 20 rows of 32: a long tail of one-block and empty rows
    ("geometric_b32", 640, 640, 456, 1, 4, 32, 0.3, lambda bi, Sb: 0.96 ** bi),
    # first row alone holds all kept blocks; dense-expansion pattern
    ("one_row_4:8", 256, 1024, 200, 4, 8, 64, 0.25, lambda bi, Sb: 1e6 if bi == 0 else 1.0),
    # last row heavy, empty rows in front of it (trailing group boundary)
    ("last_heavy_2:8", 384, 512, 328, 2, 8, 64, 0.17, lambda bi, Sb: 1e6 if bi == Sb - 1 else 1.0),
    # fewer kept blocks than waves in a group
    ("tiny_3:4", 64, 128, 72, 3, 4, 32, 0.25, lambda bi, Sb: 1.0 + bi),
    # more than 64 block-rows (several rounds of the ballot search)
    ("many_rows", 32 * 150, 128, 136, 2, 4, 32, 0.3, lambda bi, Sb: 1.0 + (bi % 7 == 0) * 50.0),
]


@pytest.mark.parametrize("case", CASES, ids=lambda c: c[0])
def test_skewed_rows(case):
    name, S, K, Ncol, n, m, B, dens, row_scale = case
    L, W, T, X = _skewed_layer(name, S, K, Ncol, n, m, B, dens, row_scale, 400 + len(name))
    sel = oracle.select(W, T, n, m, B, dens, synth.SAL_GIVEN, synth.LAYER_TOPK)
    vals, idxw, flags = oracle.pack(W, sel.keep, n, m, B, sel.row_ptr, sel.col_idx)
    counts = np.diff(sel.row_ptr)
    assert counts.max() >= 4 * max(1, int(np.median(counts))) or (counts == 0).any(), "the case is meant to be skewed"
    layer, out = run_select_pack(L, W, T)
    assert (out["row_ptr"] == sel.row_ptr).all() and (out["col_idx"] == sel.col_idx).all()
    assert (out["vals"] == vals).all() and (out["idxw"] == idxw).all()
    Yref, Aref = oracle.gemm_masked(W, sel.mask, X)
    ldx = (Ncol + 7) // 8 * 8
    Xp = np.full((K, ldx), 0x7FC0, dtype=np.uint16)        # NaN in the padding columns: must not leak
    Xp[:, :Ncol] = X
    dX = dev(Xp)
    for shape in (BALANCED, None):
        print("skewed", name, "rows", counts.tolist()[:24], "shape", shape, flush=True)
        Y32 = run_spmm(layer, dX, Ncol, ldx, crisp.Y_F32, S, shape=shape)
        check_product(Y32, Yref, Aref, crisp.Y_F32, "%s shape %s" % (name, shape))
        Y16 = run_spmm(layer, dX, Ncol, ldx, crisp.Y_BF16, S, shape=shape)
        check_bf16_is_rounded_f32(Y16, Y32, name)
        check_product(Y16, Yref, Aref, crisp.Y_BF16, "%s shape %s bf16" % (name, shape))
    # the kernel report: a whole-grid layer is dealt block by block when the library chooses
    Y = torch.empty((S, ldx), dtype=torch.float32, device="cuda")
    code = crisp.crisp_spmm_forced(layer.desc, layer.row_ptr, layer.col_idx, layer.vals, layer.idx_words, dX, Ncol, ldx, Y, ldx,
                                   crisp.Y_F32, None, crisp.SHAPE_AUTO)
    if K % 16 == 0 and Ncol % 4 == 0 and S > B:
        assert crisp.kernel_code_fields(code)["family"] == "balanced"


def test_skewed_rows_epilogue():
    """Empty rows and rows finished from partial tiles go through the epilogue like any other row."""
    name, S, K, Ncol, n, m, B, dens, row_scale = CASES[0]
    L, W, T, X = _skewed_layer(name, S, K, Ncol, n, m, B, dens, row_scale, 431)
    sel = oracle.select(W, T, n, m, B, dens, synth.SAL_GIVEN, synth.LAYER_TOPK)
    layer, _ = run_select_pack(L, W, T)
    Y0, A0 = oracle.gemm_masked(W, sel.mask, X)
    rng = np.random.default_rng(7)
    scale = rng.uniform(0.5, 2.0, size=S).astype(np.float32)
    bias = rng.normal(0.0, 0.5, size=S).astype(np.float32)
    ld = (Ncol + 7) // 8 * 8
    res = np.zeros((S, ld), dtype=np.float32)
    res[:, :Ncol] = rng.normal(0.0, 1.0, size=(S, Ncol)).astype(np.float32)
    Yref, Aref = oracle.epilogue(Y0, A0, scale, bias, res[:, :Ncol], True)
    dscale, dbias, dres = dev(scale), dev(bias), dev(res)
    ep = crisp.epilogue(dscale, dbias, dres, ld, True)
    Xp = np.zeros((K, ld), dtype=np.uint16)
    Xp[:, :Ncol] = X
    Y = torch.full((S, ld), float("nan"), dtype=torch.float32, device="cuda")
    crisp.crisp_spmm_forced(layer.desc, layer.row_ptr, layer.col_idx, layer.vals, layer.idx_words, dev(Xp), Ncol, ld, Y, ld,
                            crisp.Y_F32, ep, BALANCED)
    torch.cuda.synchronize()
    Yh = Y.cpu().numpy().astype(np.float64)[:, :Ncol]
    err = np.abs(Yh - Yref)
    assert np.linalg.norm(Yh - Yref) / np.linalg.norm(Yref) <= 1e-5
    assert (err <= 1e-2 * Aref + 2.0 ** -20 * (np.abs(Yref) + 1e-2 * Aref) + 1e-30).all()


def test_skewed_rows_many_strips():
    """More than 1024 column strips: one group holds all block-rows and four waves share the whole block
    list; sampled column windows against the oracle."""
    S, K, Ncol, n, m, B, dens = 256, 512, 66000, 2, 4, 64, 0.3
    L, W, T, X = _skewed_layer("many_strips", S, K, Ncol, n, m, B, dens, lambda bi, Sb: (1e6, 1.0, 50.0, 1.0)[bi], 477)
    sel = oracle.select(W, T, n, m, B, dens, synth.SAL_GIVEN, synth.LAYER_TOPK)
    layer, out = run_select_pack(L, W, T)
    assert (out["row_ptr"] == sel.row_ptr).all() and (out["col_idx"] == sel.col_idx).all()
    dX = dev(X)
    Y = torch.full((S + 1, Ncol), float("nan"), dtype=torch.float32, device="cuda")
    spmm(layer.desc, layer.row_ptr, layer.col_idx, layer.vals, layer.idx_words, dX, Ncol, Ncol, Y, Ncol, crisp.Y_F32, shape=BALANCED)
    torch.cuda.synchronize()
    assert bool(torch.isnan(Y[S]).all()) and bool(torch.isfinite(Y[:S]).all())
    for c0, nc in ((0, 256), (33001, 300), (Ncol - 200, 200)):
        Yref, Aref = oracle.gemm_masked(W, sel.mask, X, c0, nc)
        check_product(Y[:S, c0:c0 + nc].cpu().numpy().astype(np.float64), Yref, Aref, crisp.Y_F32, "many strips %d" % c0)
