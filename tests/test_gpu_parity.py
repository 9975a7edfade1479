"""Parity of the HIP path (through the C ABI) against the CPU oracle on the same seeded inputs:
masks, block scores, block lists and packing bit-exact; products within the stated tolerance."""
import numpy as np
import pytest
import torch

import oracle
from paper_2311_14272_amd import crisp, synth

from gpu_util import check_product, desc_of, dev, host, lowering_gather_index, run_select_pack, run_spmm, spmm, conv_spmm

pytestmark = pytest.mark.gpu


def oracle_all(L, W, G):
    sel = oracle.select(W, G, L.n, L.m, L.B, L.density, L.sal_kind, L.select_mode)
    vals, idxw, flags = oracle.pack(W, sel.keep, L.n, L.m, L.B, sel.row_ptr, sel.col_idx)
    return sel, vals, idxw, flags


def assert_select_pack_equal(L, out, sel, vals, idxw, flags):
    assert (out["nm_bits"] == sel.nm_bits).all(), "n:m mask"
    assert (out["score"].view(np.uint64) == sel.score.view(np.uint64)).all(), "block scores (bit pattern)"
    assert (out["row_ptr"] == sel.row_ptr).all(), "row_ptr"
    assert (out["col_idx"] == sel.col_idx).all(), "col_idx"
    assert (out["vals"] == vals).all(), "packed values"
    assert (out["idxw"] == idxw).all(), "packed positions"
    assert out["flags"][0] == flags[0], "2-of-4 flag"


@pytest.mark.parametrize("L", synth.small_cases(), ids=lambda L: L.name)
def test_small_cases_end_to_end(L):
    print("case", L.name, flush=True)
    W, G, X = synth.draw_small(L, 21)
    sel, vals, idxw, flags = oracle_all(L, W, G)
    layer, out = run_select_pack(L, W, G)
    assert_select_pack_equal(L, out, sel, vals, idxw, flags)
    Yref, Aref = oracle.gemm_masked(W, sel.mask, X)
    ldx = (L.Ncol + 7) // 8 * 8
    Xp = np.zeros((L.K, ldx), dtype=np.uint16)
    Xp[:, : L.Ncol] = X
    # poison the padding columns: they must not leak into valid outputs
    Xp[:, L.Ncol:] = 0x7FC0
    dX = dev(Xp)
    for yd in (crisp.Y_F32, crisp.Y_BF16):
        Y = run_spmm(layer, dX, L.Ncol, ldx, yd, L.S)
        check_product(Y, Yref, Aref, yd, L.name)


@pytest.mark.parametrize("L", synth.small_cases() + synth.b16_cases(), ids=lambda L: L.name)
def test_select_then_pack_as_two_calls(L):
    """crisp_select_mask followed by crisp_pack (the other tests go through crisp_select_pack):
    the same bytes, bit for bit."""
    W, G, X = synth.draw_small(L, 21)
    sel, vals, idxw, flags = oracle_all(L, W, G)
    layer, out = run_select_pack(L, W, G, fused=False)
    assert_select_pack_equal(L, out, sel, vals, idxw, flags)


FUSED_EXTRA = [
    # patterns that can break the 2-of-4 flag, given saliency, ragged edges, wide grids
    synth.LayerSpec("sp_3:4_b64", 128, 320, 8, 3, 4, 64, 0.6, synth.SAL_MAG, 0.05),
    synth.LayerSpec("sp_4:8_b32", 96, 224, 8, 4, 8, 32, 0.5, synth.SAL_GRAD, 0.05),
    synth.LayerSpec("sp_8:8_b64", 64, 192, 8, 8, 8, 64, 0.67, synth.SAL_MAG, 0.05),
    synth.LayerSpec("sp_4:4_b16", 48, 80, 8, 4, 4, 16, 0.5, synth.SAL_MAG, 0.05),
    synth.LayerSpec("sp_ragged_4:8", 70, 147, 8, 4, 8, 64, 0.67, synth.SAL_GRAD, 0.1),
    synth.LayerSpec("sp_ragged_3:4_b32", 40, 150, 8, 3, 4, 32, 0.5, synth.SAL_GRAD, 0.1),
    synth.LayerSpec("sp_wide_grid", 64, 4096, 8, 1, 8, 16, 0.1, synth.SAL_MAG, 0.05),
    synth.LayerSpec("sp_1:8_b16", 40, 90, 8, 1, 8, 16, 0.5, synth.SAL_MAG, 0.05),
    # more than 512 block columns: crisp_select_pack runs the two steps one after the other
    synth.LayerSpec("sp_very_wide_grid", 16, 9600, 8, 2, 4, 16, 0.05, synth.SAL_MAG, 0.05),
    synth.LayerSpec("sp_uneven_rows", 256, 512, 8, 3, 4, 64, 0.3, synth.SAL_GRAD, 0.05, None, synth.LAYER_TOPK),
]


@pytest.mark.parametrize("L", FUSED_EXTRA, ids=lambda L: L.name)
def test_select_pack_extra_patterns(L):
    """crisp_select_pack on the patterns the small cases do not reach, against the oracle and
    against the two separate calls; also with the saliency handed in directly."""
    W, G, X = synth.draw_small(L, 29)
    sel, vals, idxw, flags = oracle_all(L, W, G)
    for fused in (True, False):
        layer, out = run_select_pack(L, W, G, fused=fused)
        assert_select_pack_equal(L, out, sel, vals, idxw, flags)
    # SAL_GIVEN: hand the oracle's saliency in; masks and packing must not change
    T = np.abs(synth.bf16_bits_to_f32(W) * G).astype(np.float32) if G is not None else np.abs(synth.bf16_bits_to_f32(W))
    d = crisp.layer_desc(L.S, L.K, L.n, L.m, L.B, L.density, crisp.SAL_GIVEN, L.select_mode)
    layer, out = run_select_pack(L, W, T.astype(np.float32), fused=True, desc=d)
    assert_select_pack_equal(L, out, sel, vals, idxw, flags)


def test_select_pack_batch_matches_single_calls():
    """crisp_select_pack_batch over a mixed bag of layers (several kernel instantiations, more than
    eight layers of one kind, uneven-row and very wide layers that fall back to separate steps):
    every layer's outputs equal the oracle's, bit for bit."""
    cases = synth.small_cases() + synth.b16_cases() + FUSED_EXTRA + synth.small_cases()[:5]
    layers, Ws, TGs, keep, expect = [], [], [], [], []
    for i, L in enumerate(cases):
        W, G, _ = synth.draw_small(L, 60 + i)
        expect.append(oracle_all(L, W, G))
        layer = crisp.alloc_layer(desc_of(L))
        for t in (layer.nm_mask, layer.row_ptr, layer.col_idx, layer.vals, layer.idx_words, layer.flags):
            t.fill_(-1)
        layers.append(layer)
        Ws.append(dev(W))
        TGs.append(dev(G) if G is not None else None)
    descs, bufs = crisp.make_batch(layers, Ws, TGs)
    crisp.crisp_select_pack_batch(descs, bufs)
    torch.cuda.synchronize()
    for L, layer, (sel, vals, idxw, flags) in zip(cases, layers, expect):
        sz = layer.sizes
        out = dict(
            nm_bits=host(layer.nm_mask, np.uint32)[: sz.mask_words].reshape(L.S, sz.mask_words_per_row),
            row_ptr=host(layer.row_ptr, np.int32), col_idx=host(layer.col_idx, np.int32)[: sz.nk],
            score=host(layer.score, np.float64).reshape(sz.Sb, sz.Kb),
            vals=host(layer.vals, np.uint16)[: sz.vals_elems].reshape(sz.nk, L.B, sz.slots_per_row),
            idxw=host(layer.idx_words, np.uint32)[: sz.idx_words].reshape(sz.nk, L.B, sz.idx_words_per_row),
            flags=host(layer.flags, np.int32))
        assert_select_pack_equal(L, out, sel, vals, idxw, flags)


@pytest.mark.parametrize("L", synth.small_cases()[:6], ids=lambda L: L.name)
def test_spmm_from_oracle_pack(L):
    """The product kernel alone, fed with the oracle's packed structure."""
    print("case", L.name, flush=True)
    W, G, X = synth.draw_small(L, 22)
    sel, vals, idxw, flags = oracle_all(L, W, G)
    layer = crisp.alloc_layer(desc_of(L))
    layer.row_ptr.copy_(dev(sel.row_ptr))
    layer.col_idx[: sel.col_idx.size].copy_(dev(sel.col_idx))
    layer.vals[: vals.size].copy_(dev(vals.reshape(-1)))
    layer.idx_words[: idxw.size].copy_(dev(idxw.reshape(-1)))
    ldx = (L.Ncol + 7) // 8 * 8
    Xp = np.zeros((L.K, ldx), dtype=np.uint16)
    Xp[:, : L.Ncol] = X
    Yref, Aref = oracle.gemm_masked(W, sel.mask, X)
    Y = run_spmm(layer, dev(Xp), L.Ncol, ldx, crisp.Y_F32, L.S)
    check_product(Y, Yref, Aref, crisp.Y_F32, L.name)


@pytest.mark.parametrize("shape", [0, 1, 2, 3, 4, 5, 6, 7, 8, 9, 10, 15, 16, 17, 18])
@pytest.mark.parametrize("L", synth.small_cases(), ids=lambda L: L.name)
def test_every_launch_shape(L, shape):
    """Each launch shape of the product (wide / narrow strips, 4- and 8-way split of the block
    list, generic LDS-expansion kernel, LDS-resident block-rows with narrow / wide strips, shapes 0-3 again
    with the sparse matrix-core instruction where the pattern allows it, the uneven-row kernel, block-rows
    resident as sparse matrix-core operands) must give the same result within tolerance."""
    print("case", L.name, "shape", shape, flush=True)
    W, G, X = synth.draw_small(L, 23)
    sel, vals, idxw, flags = oracle_all(L, W, G)
    layer, out = run_select_pack(L, W, G)
    ldx = (L.Ncol + 7) // 8 * 8
    Xp = np.zeros((L.K, ldx), dtype=np.uint16)
    Xp[:, : L.Ncol] = X
    Yref, Aref = oracle.gemm_masked(W, sel.mask, X)
    for yd in (crisp.Y_F32, crisp.Y_BF16):
        Y = run_spmm(layer, dev(Xp), L.Ncol, ldx, yd, L.S, shape=shape)
        check_product(Y, Yref, Aref, yd, "%s shape %d" % (L.name, shape))


LDS_CASES = [
    # spec, density hint given to crisp_spmm (None = the layer's own)
    # several strips per wave (the strip loop and its cross-strip prefetch)
    (synth.LayerSpec("lds_iters_b64", 1024, 256, 20000, 2, 4, 64, 0.5, synth.SAL_MAG, 0.05), None),
    (synth.LayerSpec("lds_iters_b32", 512, 128, 9000, 1, 4, 32, 0.5, synth.SAL_MAG, 0.05), None),
    # 19-tile variant (more than 9 blocks per block-row), ragged S
    (synth.LayerSpec("lds_big_b64", 100, 1024, 1032, 2, 8, 64, 0.75, synth.SAL_MAG, 0.05), None),
    # block-rows longer than the variant the hint selects: chunked re-expansion
    (synth.LayerSpec("lds_chunk_b64", 128, 768, 3000, 3, 4, 64, 1.0, synth.SAL_MAG, 0.05), 0.25),
    (synth.LayerSpec("lds_chunk_b32", 64, 1280, 520, 2, 4, 32, 1.0, synth.SAL_MAG, 0.05), 0.1),
    # more blocks per row than the largest variant holds (20 > 19)
    (synth.LayerSpec("lds_chunk_big", 64, 1280, 2000, 1, 4, 64, 1.0, synth.SAL_MAG, 0.05), None),
    # uneven rows, some empty or longer than the hint says
    (synth.LayerSpec("lds_uneven", 256, 1024, 1200, 2, 4, 64, 0.3, synth.SAL_MAG, 0.05, None, synth.LAYER_TOPK), None),
]


LDS_SMF_CASES = [
    # all four patterns the sparse matrix-core instruction takes, several strips per wave, ragged S and Ncol
    (synth.LayerSpec("ldss_1:4", 200, 512, 20004, 1, 4, 64, 0.5, synth.SAL_MAG, 0.05), None),
    (synth.LayerSpec("ldss_2:4", 1024, 256, 20000, 2, 4, 64, 0.5, synth.SAL_MAG, 0.05), None),
    (synth.LayerSpec("ldss_1:8", 128, 448, 9000, 1, 8, 64, 0.6, synth.SAL_MAG, 0.05), None),
    (synth.LayerSpec("ldss_2:8", 100, 320, 5128, 2, 8, 64, 0.8, synth.SAL_GRAD, 0.05), None),
    # more than 15 blocks per block-row: the 30-tile instantiation
    (synth.LayerSpec("ldss_big", 100, 1536, 1032, 2, 8, 64, 0.75, synth.SAL_MAG, 0.05), None),
    # block-rows longer than the variant the hint selects (24 > 15) and than the largest holds (32 > 30)
    (synth.LayerSpec("ldss_chunk15", 128, 1536, 3000, 2, 4, 64, 1.0, synth.SAL_MAG, 0.05), 0.25),
    (synth.LayerSpec("ldss_chunk30", 64, 2048, 2000, 1, 4, 64, 1.0, synth.SAL_MAG, 0.05), None),
    # uneven rows, some empty or longer than the hint says
    (synth.LayerSpec("ldss_uneven", 256, 1024, 1200, 2, 4, 64, 0.3, synth.SAL_MAG, 0.05, None, synth.LAYER_TOPK), None),
    # a single block per row and an odd block count (the padding tile of the two-block request ring)
    (synth.LayerSpec("ldss_one", 192, 64, 4100, 2, 8, 64, 1.0, synth.SAL_MAG, 0.05), None),
    (synth.LayerSpec("ldss_three", 64, 256, 4100, 1, 8, 64, 0.75, synth.SAL_MAG, 0.05), None),
]


@pytest.mark.parametrize("case", LDS_SMF_CASES, ids=lambda c: c[0].name)
def test_lds_resident_sparse_operands(case):
    """Block-rows resident in LDS in the operand form of the sparse matrix-core instruction (forced shapes 16:
    capacity by the descriptor's density, 17: always the 30-tile instantiation)."""
    L, hint = case
    print("case", L.name, flush=True)
    W, G, X = synth.draw_small(L, 29)
    sel, vals, idxw, flags = oracle_all(L, W, G)
    layer, out = run_select_pack(L, W, G)
    assert_select_pack_equal(L, out, sel, vals, idxw, flags)
    if hint is not None:
        layer.desc = crisp.layer_desc(L.S, L.K, L.n, L.m, L.B, hint, L.sal_kind, L.select_mode)
    ldx = (L.Ncol + 7) // 8 * 8
    Xp = np.zeros((L.K, ldx), dtype=np.uint16)
    Xp[:, : L.Ncol] = X
    dX = dev(Xp)
    Yref, Aref = oracle.gemm_masked(W, sel.mask, X)
    for shape in (16, 17):
        for yd in (crisp.Y_F32, crisp.Y_BF16):
            Y, code = run_spmm(layer, dX, L.Ncol, ldx, yd, L.S, shape=shape, with_code=True)
            f = crisp.kernel_code_fields(code)
            assert f["family"] == "lds" and f["sparse_mfma"] == 1, (L.name, shape, f)
            check_product(Y, Yref, Aref, yd, "%s shape %d" % (L.name, shape))


def test_lds_sparse_operands_are_the_choice_for_long_rows():
    """Six or more kept blocks per block-row, 64 x 64 blocks, n <= 2, many columns: the library's own choice is
    the kernel with the block-row resident as sparse matrix-core operands, and its result is within tolerance."""
    L = synth.LayerSpec("ldss_auto", 128, 512, 65544, 2, 8, 64, 0.75, synth.SAL_MAG, 0.05)
    W, G, X = synth.draw_small(L, 31)
    sel, vals, idxw, flags = oracle_all(L, W, G)
    layer, out = run_select_pack(L, W, G)
    dX = dev(X)
    Yref, Aref = oracle.gemm_masked(W, sel.mask, X)
    for yd in (crisp.Y_F32, crisp.Y_BF16):
        Y, code = run_spmm(layer, dX, L.Ncol, L.Ncol, yd, L.S, shape=crisp.SHAPE_AUTO, with_code=True)
        f = crisp.kernel_code_fields(code)
        assert f["family"] == "lds" and f["sparse_mfma"] == 1, f
        check_product(Y, Yref, Aref, yd, L.name)
        Yp = run_spmm(layer, dX, L.Ncol, L.Ncol, yd, L.S)          # crisp_spmm itself: the same launch
        assert np.array_equal(Y, Yp)


@pytest.mark.parametrize("case", LDS_CASES, ids=lambda c: c[0].name)
def test_lds_resident_block_rows(case):
    """The kernels that keep a block-row's expanded tiles in LDS: strip loop, both tile capacities,
    and the chunked fallback for block-rows that do not fit."""
    L, hint = case
    print("case", L.name, flush=True)
    W, G, X = synth.draw_small(L, 27)
    sel, vals, idxw, flags = oracle_all(L, W, G)
    layer, out = run_select_pack(L, W, G)
    assert_select_pack_equal(L, out, sel, vals, idxw, flags)
    if hint is not None:
        layer.desc = crisp.layer_desc(L.S, L.K, L.n, L.m, L.B, hint, L.sal_kind, L.select_mode)
    ldx = (L.Ncol + 7) // 8 * 8
    Xp = np.zeros((L.K, ldx), dtype=np.uint16)
    Xp[:, : L.Ncol] = X
    dX = dev(Xp)
    Yref, Aref = oracle.gemm_masked(W, sel.mask, X)
    for shape in (5, 6):
        for yd in (crisp.Y_F32, crisp.Y_BF16):
            Y = run_spmm(layer, dX, L.Ncol, ldx, yd, L.S, shape=shape)
            check_product(Y, Yref, Aref, yd, "%s shape %d" % (L.name, shape))


XLDS_CASES = [
    # K of up to eight 64-wide block columns: the kernel that keeps a strip of X in LDS as operands for all
    # block-rows.  Full and partial last block column, ragged S, more block-rows than a group holds (> 60),
    # fewer block-rows than waves, patterns with and without the sparse matrix-core instruction, uneven rows
    # with empty ones, a block list longer than the part staged in LDS (> 512 entries), the largest K
    synth.LayerSpec("xlds_k256_2:4", 1024, 256, 1000, 2, 4, 64, 0.5, synth.SAL_MAG, 0.05),
    synth.LayerSpec("xlds_k512_1:8", 520, 512, 264, 1, 8, 64, 0.4, synth.SAL_GRAD, 0.05),
    synth.LayerSpec("xlds_k208_4:8", 300, 208, 520, 4, 8, 64, 0.75, synth.SAL_MAG, 0.05),
    synth.LayerSpec("xlds_k320_3:4", 128, 320, 72, 3, 4, 64, 0.6, synth.SAL_MAG, 0.05),
    synth.LayerSpec("xlds_k192_2:8_rows70", 4480, 192, 68, 2, 8, 64, 0.67, synth.SAL_MAG, 0.05),
    synth.LayerSpec("xlds_k512_1:4_rows60", 3840, 512, 132, 1, 4, 64, 1.0, synth.SAL_MAG, 0.05),
    synth.LayerSpec("xlds_one_group", 1280, 128, 32776, 2, 8, 64, 0.5, synth.SAL_MAG, 0.05),
    synth.LayerSpec("xlds_k384_2:4_uneven", 640, 384, 300, 2, 4, 64, 0.3, synth.SAL_MAG, 0.05, None, synth.LAYER_TOPK),
    synth.LayerSpec("xlds_k128_8:8", 192, 128, 260, 8, 8, 64, 1.0, synth.SAL_MAG, 0.05),
    synth.LayerSpec("xlds_k64_4:4", 64, 64, 64, 4, 4, 64, 1.0, synth.SAL_MAG, 0.05),
]


@pytest.mark.parametrize("L", XLDS_CASES, ids=lambda L: L.name)
def test_x_strip_resident_in_lds(L):
    """Forced shape 18: the strip's operands staged once per workgroup in LDS, waves walk the block-rows."""
    print("case", L.name, flush=True)
    W, G, X = synth.draw_small(L, 33)
    sel, vals, idxw, flags = oracle_all(L, W, G)
    layer, out = run_select_pack(L, W, G)
    assert_select_pack_equal(L, out, sel, vals, idxw, flags)
    ldx = (L.Ncol + 7) // 8 * 8
    Xp = np.zeros((L.K, ldx), dtype=np.uint16)
    Xp[:, : L.Ncol] = X
    dX = dev(Xp)
    Yref, Aref = oracle.gemm_masked(W, sel.mask, X)
    for yd in (crisp.Y_F32, crisp.Y_BF16):
        Y, code = run_spmm(layer, dX, L.Ncol, ldx, yd, L.S, shape=18, with_code=True)
        assert crisp.kernel_code_fields(code)["family"] == "xlds", (L.name, crisp.kernel_code_fields(code))
        check_product(Y, Yref, Aref, yd, "%s shape 18" % L.name)


def test_x_strip_in_lds_is_the_choice_for_many_short_block_rows():
    """16 or more block-rows over two to eight block columns, n <= 2, enough columns: the library's own choice is
    the kernel with the strip of X resident in LDS."""
    L = synth.LayerSpec("xlds_auto", 1024, 256, 8200, 2, 4, 64, 0.5, synth.SAL_MAG, 0.05)
    W, G, X = synth.draw_small(L, 35)
    sel, vals, idxw, flags = oracle_all(L, W, G)
    layer, out = run_select_pack(L, W, G)
    dX = dev(X)
    Yref, Aref = oracle.gemm_masked(W, sel.mask, X)
    for yd in (crisp.Y_F32, crisp.Y_BF16):
        Y, code = run_spmm(layer, dX, L.Ncol, L.Ncol, yd, L.S, shape=crisp.SHAPE_AUTO, with_code=True)
        f = crisp.kernel_code_fields(code)
        assert f["family"] == "xlds" and f["sparse_mfma"] == 1, f
        check_product(Y, Yref, Aref, yd, L.name)
        Yp = run_spmm(layer, dX, L.Ncol, L.Ncol, yd, L.S)          # crisp_spmm itself: the same launch
        assert np.array_equal(Y, Yp)


XRES_CASES = [
    # short K (one or two 64-wide block columns): the kernel that keeps the strip of X in registers.
    # One and two block columns, ragged S, a last strip group with idle waves, more block-rows than
    # one group holds, patterns with and without the sparse matrix-core instruction, uneven rows
    synth.LayerSpec("xres_k64_2:8", 256, 64, 1000, 2, 8, 64, 1.0, synth.SAL_MAG, 0.05),
    synth.LayerSpec("xres_k128_1:4", 200, 128, 520, 1, 4, 64, 0.5, synth.SAL_MAG, 0.05),
    synth.LayerSpec("xres_k128_2:4_full", 512, 128, 264, 2, 4, 64, 1.0, synth.SAL_GRAD, 0.05),
    synth.LayerSpec("xres_k96_4:8", 320, 96, 136, 4, 8, 64, 0.5, synth.SAL_MAG, 0.05),
    synth.LayerSpec("xres_k48_3:4", 64, 48, 72, 3, 4, 64, 1.0, synth.SAL_MAG, 0.05),
    synth.LayerSpec("xres_k128_1:8_rows40", 2560, 128, 68, 1, 8, 64, 0.5, synth.SAL_MAG, 0.05),
    synth.LayerSpec("xres_k128_4:4_uneven", 384, 128, 300, 4, 4, 64, 0.4, synth.SAL_MAG, 0.05, None, synth.LAYER_TOPK),
    synth.LayerSpec("xres_k64_8:8", 128, 64, 260, 8, 8, 64, 1.0, synth.SAL_MAG, 0.05),
]


@pytest.mark.parametrize("L", XRES_CASES, ids=lambda L: L.name)
def test_x_resident_short_k(L):
    """The short-K product kernel (forced, and whatever the library picks) against the oracle."""
    print("case", L.name, flush=True)
    W, G, X = synth.draw_small(L, 29)
    sel, vals, idxw, flags = oracle_all(L, W, G)
    layer, out = run_select_pack(L, W, G)
    assert_select_pack_equal(L, out, sel, vals, idxw, flags)
    ldx = (L.Ncol + 7) // 8 * 8
    Xp = np.zeros((L.K, ldx), dtype=np.uint16)
    Xp[:, : L.Ncol] = X
    dX = dev(Xp)
    Yref, Aref = oracle.gemm_masked(W, sel.mask, X)
    for shape in (13, None):
        for yd in (crisp.Y_F32, crisp.Y_BF16):
            Y = run_spmm(layer, dX, L.Ncol, ldx, yd, L.S, shape=shape)
            check_product(Y, Yref, Aref, yd, "%s shape %s" % (L.name, shape))


TINY_CASES = [
    # degenerate sizes: one row, one group, one column, fewer rows than a block, K below one block
    synth.LayerSpec("tiny_1x4x1", 1, 4, 1, 1, 4, 16, 1.0, synth.SAL_MAG, 0.5),
    synth.LayerSpec("tiny_1x8x3", 1, 8, 3, 2, 8, 32, 1.0, synth.SAL_MAG, 0.5),
    synth.LayerSpec("tiny_3x5x2", 3, 5, 2, 1, 4, 64, 1.0, synth.SAL_MAG, 0.5),
    synth.LayerSpec("tiny_2x16x4", 2, 16, 4, 2, 4, 16, 0.5, synth.SAL_GRAD, 0.5),
    synth.LayerSpec("tiny_7x9x5", 7, 9, 5, 3, 4, 32, 0.5, synth.SAL_GRAD, 0.5),
    synth.LayerSpec("tiny_1row_wide", 1, 256, 130, 2, 4, 64, 0.5, synth.SAL_MAG, 0.5),
    synth.LayerSpec("tiny_1col", 200, 128, 1, 4, 8, 64, 0.5, synth.SAL_MAG, 0.5),
    synth.LayerSpec("tiny_ncol4", 64, 64, 4, 2, 4, 64, 1.0, synth.SAL_MAG, 0.5),
    synth.LayerSpec("tiny_all_kept_8:8", 32, 32, 8, 8, 8, 32, 1.0, synth.SAL_MAG, 0.5),
]


@pytest.mark.parametrize("L", TINY_CASES, ids=lambda L: L.name)
def test_degenerate_sizes(L):
    """The smallest shapes the interface admits, through both selection paths and every product kernel
    family the shape can reach."""
    W, G, X = synth.draw_small(L, 31)
    sel, vals, idxw, flags = oracle_all(L, W, G)
    for fused in (True, False):
        layer, out = run_select_pack(L, W, G, fused=fused)
        assert_select_pack_equal(L, out, sel, vals, idxw, flags)
    Yref, Aref = oracle.gemm_masked(W, sel.mask, X)
    ldx = (L.Ncol + 7) // 8 * 8
    Xp = np.zeros((L.K, ldx), dtype=np.uint16)
    Xp[:, : L.Ncol] = X
    dX = dev(Xp)
    for shape in (None, 1, 4, 5, 8):
        Y = run_spmm(layer, dX, L.Ncol, ldx, crisp.Y_F32, L.S, shape=shape)
        check_product(Y, Yref, Aref, crisp.Y_F32, "%s shape %s" % (L.name, shape))
        # with a handful of outputs the Frobenius bound is no statistic of bf16 rounding any more:
        # the bf16 result must be exactly the rounded fp32 result instead
        Y16 = run_spmm(layer, dX, L.Ncol, ldx, crisp.Y_BF16, L.S, shape=shape)
        assert (synth.f32_to_bf16_bits(Y16.astype(np.float32)) == synth.f32_to_bf16_bits(Y.astype(np.float32))).all()


def test_zero_weights_and_zero_activations():
    """All-zero W keeps exactly n per group by the tie rule and gives Y = 0; all-zero X gives Y = 0."""
    L = synth.LayerSpec("zeros", 96, 160, 72, 2, 4, 32, 0.5, synth.SAL_MAG, 0.05)
    W, G, X = synth.draw_small(L, 32)
    Wz = np.zeros_like(W)
    sel, vals, idxw, flags = oracle_all(L, Wz, None)
    layer, out = run_select_pack(L, Wz, None)
    assert_select_pack_equal(L, out, sel, vals, idxw, flags)
    assert sel.nm_bits.any(), "the tie rule keeps the first n columns of every group"
    ldx = (L.Ncol + 7) // 8 * 8
    Xp = np.zeros((L.K, ldx), dtype=np.uint16)
    Xp[:, : L.Ncol] = X
    assert (run_spmm(layer, dev(Xp), L.Ncol, ldx, crisp.Y_F32, L.S) == 0).all()
    layer, out = run_select_pack(L, W, None)
    assert (run_spmm(layer, dev(np.zeros_like(Xp)), L.Ncol, ldx, crisp.Y_BF16, L.S) == 0).all()


@pytest.mark.parametrize("L", synth.b16_cases(), ids=lambda L: L.name)
def test_block16_end_to_end(L):
    """16 x 16 blocks (the paper's smallest): selection and packing bit-exact, product in tolerance."""
    W, G, X = synth.draw_small(L, 24)
    sel, vals, idxw, flags = oracle_all(L, W, G)
    layer, out = run_select_pack(L, W, G)
    assert_select_pack_equal(L, out, sel, vals, idxw, flags)
    Yref, Aref = oracle.gemm_masked(W, sel.mask, X)
    ldx = (L.Ncol + 7) // 8 * 8
    Xp = np.zeros((L.K, ldx), dtype=np.uint16)
    Xp[:, : L.Ncol] = X
    for yd in (crisp.Y_F32, crisp.Y_BF16):
        Y = run_spmm(layer, dev(Xp), L.Ncol, ldx, yd, L.S)
        check_product(Y, Yref, Aref, yd, L.name)


def test_bf16_output_is_rounded_fp32_output():
    """bf16 Y must be the round-to-nearest-even of the fp32 Y the same launch shape produces."""
    for L in synth.small_cases()[:4]:
        W, G, X = synth.draw_small(L, 25)
        layer, _ = run_select_pack(L, W, G)
        ldx = (L.Ncol + 7) // 8 * 8
        Xp = np.zeros((L.K, ldx), dtype=np.uint16)
        Xp[:, : L.Ncol] = X
        dX = dev(Xp)
        for shape in (0, 1, 2, 4, 7, 9, 15, 16, 18):
            y32 = run_spmm(layer, dX, L.Ncol, ldx, crisp.Y_F32, L.S, shape=shape).astype(np.float32)
            y16 = run_spmm(layer, dX, L.Ncol, ldx, crisp.Y_BF16, L.S, shape=shape).astype(np.float32)
            assert (synth.f32_to_bf16_bits(y16) == synth.f32_to_bf16_bits(y32)).all(), (L.name, shape)


CONV_CASES = [
    # C, H, W, batch, kh, kw, pad, S, n, m, B, density
    (64, 8, 8, 2, 3, 3, 1, 64, 2, 4, 64, 0.5),
    (32, 6, 10, 3, 3, 3, 1, 96, 1, 4, 32, 0.5),
    (64, 6, 6, 2, 5, 5, 2, 64, 2, 8, 64, 0.4),
    (128, 14, 14, 2, 3, 3, 1, 128, 1, 4, 64, 0.3),
    (64, 7, 10, 2, 1, 1, 0, 64, 4, 8, 32, 0.5),
    (64, 9, 10, 1, 3, 3, 0, 32, 3, 4, 32, 0.6),
    (64, 5, 4, 5, 3, 3, 1, 64, 4, 4, 64, 0.5),
    (32, 12, 2, 2, 3, 3, 1, 32, 2, 4, 32, 1.0),
    # shapes of the LDS-staged convolution: several channel blocks, 1 / 2 / 4+ block-rows per workgroup,
    # tiles that end inside the image, patterns with and without the sparse matrix-core instruction
    (128, 14, 14, 3, 3, 3, 1, 256, 2, 8, 64, 0.6),
    (64, 28, 28, 2, 3, 3, 1, 128, 2, 4, 64, 0.7),
    (64, 56, 56, 1, 3, 3, 1, 64, 1, 8, 64, 0.5),
    (256, 14, 14, 2, 3, 3, 1, 320, 4, 8, 64, 0.5),
    (64, 10, 12, 2, 3, 3, 1, 192, 3, 4, 64, 0.5),
    (128, 9, 16, 2, 3, 5, 2, 64, 1, 4, 64, 0.4),
    # with a 13th element: stride.  Strided, odd output width, strided 1x1: columns located one by one
    (64, 8, 8, 2, 3, 3, 1, 64, 2, 4, 64, 0.5, 2),
    (64, 8, 8, 2, 1, 1, 0, 64, 1, 4, 64, 0.5, 2),
    (64, 7, 7, 2, 3, 3, 1, 64, 2, 8, 64, 0.5, 1),
    (32, 9, 7, 2, 3, 3, 1, 32, 4, 8, 32, 0.6, 2),
    (32, 11, 10, 2, 5, 5, 2, 64, 3, 4, 32, 0.5, 3),
    (128, 14, 14, 4, 3, 3, 1, 128, 2, 4, 64, 0.4, 2),
    (64, 14, 14, 6, 1, 1, 0, 128, 1, 8, 64, 0.5, 2),
    # stride 1, odd output width, padding (k-1)/2: a lane's column pair may straddle output rows and images, yet
    # its two sources stay neighbours in memory (one dword); all-border images, 5x5 and 1x1 filters, last pair at
    # the very end of the channel plane
    (128, 7, 7, 4, 3, 3, 1, 128, 2, 4, 64, 0.5, 1),
    (64, 3, 3, 6, 3, 3, 1, 64, 4, 8, 64, 1.0, 1),
    (64, 5, 5, 2, 5, 5, 2, 64, 1, 4, 64, 0.6, 1),
    (64, 7, 9, 2, 1, 1, 0, 128, 2, 4, 64, 0.7, 1),
    (32, 5, 7, 2, 3, 3, 1, 64, 3, 4, 32, 0.6, 1),
    (512, 7, 7, 8, 3, 3, 1, 128, 1, 4, 64, 0.3, 1),
    # stride 1, odd output width, other paddings: the pair's sources are not neighbours across rows
    (64, 9, 9, 2, 3, 3, 0, 64, 2, 4, 64, 0.6, 1),
    (64, 7, 7, 2, 3, 3, 2, 64, 2, 8, 64, 0.6, 1),
    # strided 1x1 with even W and Wo: both columns of a lane from one 8-byte piece of the input row
    (128, 12, 12, 3, 1, 1, 0, 192, 2, 8, 64, 0.5, 2),
    (64, 8, 16, 2, 1, 1, 0, 96, 4, 8, 32, 0.6, 2),
    # the same with many block-rows (forced shape 18: the gathered strip staged once in LDS for all of them),
    # sparse and dense matrix-core patterns, the largest channel count that kernel takes
    (256, 8, 12, 3, 1, 1, 0, 1100, 1, 8, 64, 0.5, 2),
    (512, 4, 8, 5, 1, 1, 0, 320, 4, 8, 64, 0.6, 2),
    (128, 28, 28, 2, 1, 1, 0, 512, 2, 4, 64, 0.5, 2),
    # strided shapes of the LDS-staged convolution (3x3, 5x5, 1x1 that skips input rows, stride 3)
    (128, 28, 28, 2, 3, 3, 1, 256, 2, 4, 64, 0.6, 2),
    (256, 28, 28, 2, 1, 1, 0, 256, 2, 4, 64, 0.6, 2),
    (64, 56, 56, 1, 1, 1, 0, 128, 1, 4, 64, 0.7, 2),
    (64, 12, 16, 2, 3, 3, 1, 128, 2, 8, 64, 0.5, 3),
    (64, 20, 20, 1, 5, 5, 2, 64, 1, 4, 64, 0.5, 2),
    # input rows wider than the LDS-staged kernel takes (64): it must hand over to the register kernels
    (64, 3, 66, 1, 3, 3, 0, 128, 2, 4, 64, 0.6, 1),
    (64, 5, 128, 1, 3, 3, 1, 128, 2, 4, 64, 0.6, 2),
    # channel counts that are no multiple of B (first layers): every K-row located on its own
    (3, 20, 20, 2, 7, 7, 3, 64, 1, 8, 64, 0.7, 2),
    (3, 12, 12, 2, 3, 3, 1, 32, 2, 4, 32, 0.6, 1),
    (24, 9, 8, 2, 3, 3, 1, 64, 2, 4, 64, 0.5, 1),
    (48, 7, 7, 2, 3, 3, 1, 96, 1, 4, 32, 0.5, 2),
    (5, 8, 8, 4, 5, 5, 2, 32, 4, 8, 32, 1.0, 1),
    # the same with 64x64 blocks and even W and Ho*Wo: the kernel that keeps the input patch in LDS in its own
    # layout (exactly one tile, a ragged second tile, two block-rows, ragged S, ragged last block column)
    (3, 32, 32, 2, 7, 7, 3, 64, 1, 8, 64, 0.7, 2),
    (3, 40, 40, 1, 7, 7, 3, 128, 2, 4, 64, 0.7, 2),
    (16, 12, 12, 2, 3, 3, 1, 64, 4, 8, 64, 0.67, 1),
    (3, 18, 14, 2, 5, 5, 2, 96, 3, 4, 64, 1.0, 1),
    (40, 10, 10, 3, 3, 3, 1, 200, 2, 8, 64, 0.5, 1),
    # more than 64 kept blocks in all (the kernel holds the first 64 block columns in a register)
    (16, 13, 48, 1, 7, 7, 3, 320, 2, 4, 64, 1.0, 1),
    (16, 8, 12, 2, 5, 5, 2, 448, 1, 8, 64, 0.8, 1),
]


@pytest.mark.parametrize("case", CONV_CASES, ids=lambda c: "C%d_%dx%d_b%d_k%dx%d_p%d_%d:%d_B%d_s%d" % (c[0], c[1], c[2], c[3], c[4], c[5], c[6], c[8], c[9], c[10], c[12] if len(c) > 12 else 1))
def test_conv_spmm_implicit_lowering(case):
    """crisp_conv_spmm (no X in memory) against the oracle's im2col + masked product, and bit for
    bit against crisp_im2col + crisp_spmm in the same launch shape."""
    C_, H, Wd, b, kh, kw, pad, S, n, m, B, dens = case[:12]
    stride = case[12] if len(case) > 12 else 1
    print("conv case", case, flush=True)
    cv = synth.ConvShape(C_, H, Wd, b, kh, kw, stride, pad)
    L = synth.LayerSpec("conv", S, cv.K, cv.Ncol, n, m, B, dens, synth.SAL_MAG, 0.05, conv=cv)
    rng = np.random.default_rng(C_ * 7 + H)
    W = synth.draw_weight(rng, L)
    act = synth.draw_relu_normal(rng, (C_, b, H, Wd))
    act[:, :, 0, 0] = synth.f32_to_bf16_bits(np.full((C_, b), 3.0, dtype=np.float32))   # make the borders matter
    act[:, :, -1, -1] = synth.f32_to_bf16_bits(np.full((C_, b), 5.0, dtype=np.float32))
    sel, vals, idxw, flags = oracle_all(L, W, None)
    layer, out = run_select_pack(L, W, None)
    Xref = oracle.im2col(act, kh, kw, stride, pad)
    Yref, Aref = oracle.gemm_masked(W, sel.mask, Xref)
    conv = crisp.ConvDesc(C_, H, Wd, b, kh, kw, stride, pad, crisp.ACT_CBHW, crisp.X_KN)
    dact = dev(act)
    Ncol = cv.Ncol
    ldy = (Ncol + 7) // 8 * 8 + 8
    ldx = (Ncol + 7) // 8 * 8
    dX = torch.zeros((L.K, ldx), dtype=torch.int16, device="cuda")
    crisp.crisp_im2col(conv, dact, dX, ldx)
    for yd, tdt in ((crisp.Y_F32, torch.float32), (crisp.Y_BF16, torch.bfloat16)):
        for shape in (None, 1, 2, 3, 8, 9, 10, 12, 14, 18):    # 12 / 14 / 18: input staged in LDS (where they apply)
            Y = torch.full((S + 1, ldy), float("nan"), dtype=tdt, device="cuda")
            conv_spmm(layer.desc, conv, layer.row_ptr, layer.col_idx, layer.vals, layer.idx_words, dact, Y,
                                  ldy, yd, shape=shape)
            torch.cuda.synchronize()
            Yh = Y.float().cpu().numpy().astype(np.float64)
            assert np.isnan(Yh[:S, Ncol:]).all() and np.isnan(Yh[S]).all()
            check_product(Yh[:S, :Ncol], Yref, Aref, yd, "conv %s shape %s" % (case, shape))
            if shape is not None and shape not in (12, 14, 18) and Ncol % 4 == 0 and L.K % 16 == 0:
                # (other K or Ncol: the explicit path runs the generic kernel, a different summation order)
                Ye = run_spmm(layer, dX, Ncol, ldx, yd, S, ldy=ldy, shape=shape)
                assert (Ye == Yh[:S, :Ncol]).all(), "implicit and explicit lowering differ"


@pytest.mark.parametrize("case", [
    # uneven block-rows (whole-grid block choice: some rows long, some empty) through the kernels that keep
    # the input in LDS: staged patch (shape 12) and few-channel patch (shape 14), and the library's own choice
    (64, 14, 14, 2, 3, 3, 1, 256, 2, 4, 64, 0.35, 1, 12),
    (128, 12, 12, 2, 3, 3, 1, 320, 1, 8, 64, 0.3, 2, 12),
    (3, 24, 24, 2, 7, 7, 3, 192, 2, 8, 64, 0.4, 2, 14),
    (20, 12, 12, 2, 3, 3, 1, 256, 4, 8, 64, 0.3, 1, 14),
], ids=lambda c: "C%d_S%d_shape%d" % (c[0], c[7], c[13]))
def test_conv_spmm_uneven_block_rows(case):
    C_, H, Wd, b, kh, kw, pad, S, n, m, B, dens, stride, forced = case
    cv = synth.ConvShape(C_, H, Wd, b, kh, kw, stride, pad)
    L = synth.LayerSpec("conv_uneven", S, cv.K, cv.Ncol, n, m, B, dens, synth.SAL_MAG, 0.05, conv=cv, select_mode=synth.LAYER_TOPK)
    rng = np.random.default_rng(C_ * 11 + S)
    W = synth.draw_weight(rng, L)
    # make the block scores very uneven so that the whole-grid choice empties some block-rows
    Wf = synth.bf16_bits_to_f32(W).reshape(S, cv.K)
    Wf[: B] *= 8.0
    if S > 2 * B:
        Wf[2 * B: 3 * B] *= 0.01
    W = synth.f32_to_bf16_bits(Wf.astype(np.float32))
    act = synth.draw_relu_normal(rng, (C_, b, H, Wd))
    sel, vals, idxw, flags = oracle_all(L, W, None)
    counts = np.diff(sel.row_ptr)
    assert counts.min() == 0 or counts.max() > counts.min(), "the case is meant to have uneven rows"
    layer, out = run_select_pack(L, W, None)
    assert_select_pack_equal(L, out, sel, vals, idxw, flags)
    Yref, Aref = oracle.gemm_masked(W, sel.mask, oracle.im2col(act, kh, kw, stride, pad))
    conv = crisp.ConvDesc(C_, H, Wd, b, kh, kw, stride, pad, crisp.ACT_CBHW, crisp.X_KN)
    Ncol = cv.Ncol
    ldy = (Ncol + 7) // 8 * 8
    for shape in (forced, None):
        for yd, tdt in ((crisp.Y_F32, torch.float32), (crisp.Y_BF16, torch.bfloat16)):
            Y = torch.full((S, ldy), float("nan"), dtype=tdt, device="cuda")
            conv_spmm(layer.desc, conv, layer.row_ptr, layer.col_idx, layer.vals, layer.idx_words, dev(act), Y, ldy, yd, shape=shape)
            torch.cuda.synchronize()
            Yh = Y.float().cpu().numpy().astype(np.float64)
            check_product(Yh[:, :Ncol], Yref, Aref, yd, "uneven %s shape %s" % (case, shape))


def test_conv_forward_takes_each_of_its_three_ways():
    """crisp_conv_forward: the activation as X, the fused lowering, a materialised X (also when a fused plan
    meets a Y row stride beyond the fused kernels' range), and the error for a missing scratch buffer."""
    for (cvt, S, dens, expect, ldy_extra) in (((64, 6, 8, 2, 1, 1, 1, 0), 128, 0.5, "none", 0),
                                              ((64, 8, 8, 2, 3, 3, 1, 1), 128, 0.5, "fused", 0),
                                              ((64, 9, 7, 2, 3, 3, 2, 1), 256, 1.0, "im2col", 0),
                                              ((64, 8, 8, 2, 3, 3, 1, 1), 64, 0.5, "im2col", (1 << 23) + 8)):
        cv = synth.ConvShape(*cvt)
        L = synth.LayerSpec("fw", S, cv.K, cv.Ncol, 2, 4, 64, dens, synth.SAL_MAG, 0.05, conv=cv)
        rng = np.random.default_rng(S + cv.H)
        W = synth.draw_weight(rng, L)
        act = synth.draw_relu_normal(rng, (cv.C, cv.batch, cv.H, cv.W))
        sel = oracle.select(W, None, L.n, L.m, L.B, dens, synth.SAL_MAG)
        layer, _ = run_select_pack(L, W, None)
        Yref, Aref = oracle.gemm_masked(W, sel.mask, oracle.im2col(act, cv.kh, cv.kw, cv.stride, cv.pad))
        planned, nbytes = crisp.conv_plan(layer.desc, cv)
        assert planned == (expect if not ldy_extra else "fused")
        ld = (cv.Ncol + 7) // 8 * 8
        ldy = ldy_extra or ld
        Y = torch.full((S, ldy), float("nan"), dtype=torch.float32, device="cuda")
        if expect == "im2col":
            with pytest.raises(ValueError):
                crisp.conv_forward(layer, cv, dev(act), Y, ldy, crisp.Y_F32, None)
        Xs = torch.empty((cv.K, ld), dtype=torch.int16, device="cuda") if expect == "im2col" else None
        assert crisp.conv_forward(layer, cv, dev(act), Y, ldy, crisp.Y_F32, Xs) == expect
        torch.cuda.synchronize()
        check_product(Y[:, : cv.Ncol].cpu().numpy().astype(np.float64), Yref, Aref, crisp.Y_F32, "forward %s" % (cvt,))
        assert bool(torch.isnan(Y[:, cv.Ncol:]).all())


def test_conv_spmm_rejects_what_it_does_not_cover():
    d = crisp.layer_desc(64, 9 * 64, 2, 4, 64, 0.5)
    z = torch.zeros(1 << 16, dtype=torch.int16, device="cuda")
    zi = torch.zeros(1 << 12, dtype=torch.int32, device="cuda")
    y = torch.zeros(1 << 16, dtype=torch.float32, device="cuda")
    for cvt, status in (((64, 7, 7, 1, 3, 3, 1, 1), crisp.EUNSUPPORTED),      # odd number of output columns
                        ((64, 8, 8, 1, 3, 3, 17, 1), crisp.EUNSUPPORTED),     # stride beyond the covered range
                        ((32, 8, 8, 1, 3, 3, 1, 1), crisp.ESHAPE)):           # K mismatch
        conv = crisp.ConvDesc(*cvt, crisp.ACT_CBHW, crisp.X_KN)
        with pytest.raises(crisp.CrispError) as e:
            crisp.crisp_conv_spmm(d, conv, zi, zi, z, zi, z, y, 64)
        assert e.value.status == status


def test_global_budget_matches_oracle():
    """crisp_global_budget on device block scores: kept blocks per row and reached sparsity equal
    the oracle's, bit for bit, for several targets; feeding k_row/Kb back as the density reproduces
    the oracle's block lists."""
    cases = synth.small_cases()[:6] + synth.b16_cases()[:2]
    descs, score_t, score_h, layers, Ws = [], [], [], [], []
    for i, L in enumerate(cases):
        W, G, _ = synth.draw_small(L, 40 + i)
        L1 = synth.LayerSpec(L.name, L.S, L.K, L.Ncol, L.n, L.m, L.B, 1.0, L.sal_kind, L.w_sigma)
        layer, out = run_select_pack(L1, W, G)
        sel = oracle.select(W, G, L.n, L.m, L.B, 1.0, L.sal_kind)
        assert (out["score"].view(np.uint64) == sel.score.view(np.uint64)).all()
        descs.append(layer.desc)
        score_t.append(layer.score)
        score_h.append(sel.score)
        layers.append((L.S, L.K, L.n, L.m, L.B))
        Ws.append((L, W, G))
    ws = torch.empty(sum(s.size for s in score_h), dtype=torch.float64, device="cuda")
    k_dev = torch.zeros(len(cases), dtype=torch.int32, device="cuda")
    ach = torch.zeros(1, dtype=torch.float64, device="cuda")
    for target in (0.0, 0.55, 0.7, 0.8, 0.9, 0.97):
        crisp.crisp_global_budget(descs, score_t, target, k_dev, ach, ws, ws.numel() * 8)
        torch.cuda.synchronize()
        k_ref, a_ref = oracle.global_budget(layers, score_h, target)
        assert k_dev.cpu().tolist() == k_ref, target
        assert ach.cpu().numpy().view(np.uint64)[0] == np.array([a_ref]).view(np.uint64)[0], target
    # close the loop for the last target: density = k_row / Kb gives the same block lists
    for (L, W, G), kr in zip(Ws, k_ref):
        Kb = -(-L.K // L.B)
        L2 = synth.LayerSpec(L.name, L.S, L.K, L.Ncol, L.n, L.m, L.B, kr / Kb, L.sal_kind, L.w_sigma)
        _, out = run_select_pack(L2, W, G)
        sel = oracle.select(W, G, L.n, L.m, L.B, kr / Kb, L.sal_kind)
        assert sel.k_row == kr and (out["col_idx"] == sel.col_idx).all()


def test_ties_and_zero_weights():
    """Constant saliency (every comparison is a tie) and weights with exact zeros / negative zeros."""
    L = synth.LayerSpec("ties", 64, 128, 64, 2, 4, 32, 0.5, synth.SAL_GIVEN, 1.0)
    rng = np.random.default_rng(3)
    Wf = rng.standard_normal((L.S, L.K)).astype(np.float32)
    Wf[rng.random((L.S, L.K)) < 0.3] = 0.0
    Wf[rng.random((L.S, L.K)) < 0.1] = -0.0
    W = synth.f32_to_bf16_bits(Wf)
    for T in (np.ones((L.S, L.K), dtype=np.float32),
              rng.integers(0, 3, (L.S, L.K)).astype(np.float32)):
        sel, vals, idxw, flags = oracle_all(L, W, T)
        layer, out = run_select_pack(L, W, T)
        assert_select_pack_equal(L, out, sel, vals, idxw, flags)


@pytest.mark.parametrize("B", [16, 32, 64])
def test_two_of_four_flag_on_4_of_8(B):
    """4:8 patterns whose kept values fall two per aligned quad set the 2-of-4 flag; one row with three
    in a quad clears it.  Random 4:8 layers practically never hit the first case."""
    L = synth.LayerSpec("quads_B%d" % B, 2 * B, 3 * B, 64, 4, 8, B, 1.0, synth.SAL_MAG, 1.0)
    rng = np.random.default_rng(41 + B)
    mag = np.tile(np.array([2.0, 0.5, 0.5, 2.0, 0.5, 2.0, 2.0, 0.5], dtype=np.float32), (L.S, L.K // 8))
    Wf = (mag * rng.uniform(1.0, 1.5, mag.shape) * rng.choice([-1.0, 1.0], mag.shape)).astype(np.float32)
    seen = []
    for skew in (False, True):
        if skew:
            Wf[:, :8] = np.abs(Wf[:, :8])
            Wf[B + 3, :8] = [3.0, 3.0, 3.0, 0.1, 0.1, 0.1, 0.1, 3.0]
        W = synth.f32_to_bf16_bits(Wf)
        sel, vals, idxw, flags = oracle_all(L, W, None)
        layer, out = run_select_pack(L, W, None)
        assert_select_pack_equal(L, out, sel, vals, idxw, flags)
        seen.append(int(out["flags"][0]))
    assert seen == [1, 0]


def test_im2col_matches_oracle():
    rng = np.random.default_rng(5)
    for (C_, H, Wd, b, kh, kw, st, pad) in [(3, 9, 8, 2, 3, 3, 1, 1), (4, 8, 8, 1, 1, 1, 2, 0), (2, 11, 11, 2, 7, 7, 2, 3),
                                            (16, 14, 14, 3, 3, 3, 1, 1), (8, 15, 13, 2, 3, 3, 2, 1), (5, 6, 7, 3, 1, 1, 1, 0)]:
        print("im2col", C_, H, Wd, b, kh, kw, st, pad, flush=True)
        act = synth.f32_to_bf16_bits(rng.standard_normal((C_, b, H, Wd)).astype(np.float32))
        Xref = oracle.im2col(act, kh, kw, st, pad)
        K, Ncol = Xref.shape
        for ldx in ((Ncol + 7) // 8 * 8, Ncol + 3):
            X = torch.full((K, ldx), -1, dtype=torch.int16, device="cuda")
            cv = crisp.ConvDesc(C_, H, Wd, b, kh, kw, st, pad, crisp.ACT_CBHW, crisp.X_KN)
            crisp.crisp_im2col(cv, dev(act), X, ldx)
            torch.cuda.synchronize()
            Xh = host(X, np.uint16)
            assert (Xh[:, :Ncol] == Xref).all()
            assert (Xh[:, Ncol:] == 0xFFFF).all()


@pytest.mark.parametrize("shape", [(3, 2, 9, 7, 3, 3, 2, 1), (4, 1, 8, 8, 2, 2, 2, 0), (2, 3, 5, 6, 3, 3, 1, 1), (64, 2, 112, 112, 3, 3, 2, 1),
                                   (2, 2, 7, 9, 5, 3, 2, 2), (1, 1, 4, 4, 1, 1, 1, 0), (3, 1, 6, 5, 3, 3, 3, 2),
                                   # 3x3 / 2 / 1 with W % 8 == 0: four outputs per thread (one quad per row, odd H, several quads)
                                   (3, 2, 7, 8, 3, 3, 2, 1), (2, 1, 10, 24, 3, 3, 2, 1), (5, 3, 16, 16, 3, 3, 2, 1)])
def test_maxpool_matches_oracle(shape):
    C_, b, H, Wd, kh, kw, stride, pad = shape
    rng = np.random.default_rng(C_ * 100 + H)
    act = synth.f32_to_bf16_bits(rng.standard_normal((C_, b, H, Wd), dtype=np.float32))
    ref = oracle.maxpool(act, kh, kw, stride, pad)
    out = torch.full(ref.shape, -1, dtype=torch.int16, device="cuda")
    crisp.crisp_maxpool(crisp.ConvDesc(C_, H, Wd, b, kh, kw, stride, pad, crisp.ACT_CBHW, crisp.X_KN), dev(act), out)
    torch.cuda.synchronize()
    assert (synth.bf16_bits_to_f32(host(out, np.uint16)) == synth.bf16_bits_to_f32(ref)).all()


def _sample_columns(Ncol, count, rng):
    """First strip, last (ragged) strip and random columns."""
    cols = set(range(min(Ncol, 96))) | set(range(max(0, Ncol - 96), Ncol))
    cols |= set(int(c) for c in rng.integers(0, Ncol, count))
    return np.array(sorted(cols), dtype=np.int64)


@pytest.mark.parametrize("cid", [1, 2, 3, 4])
def test_config_full_size(cid):
    """The benchmark workloads at full size, in the launch configuration bench.py times.
    Selection and packing are compared in full; the product on all columns when the oracle
    finishes in seconds, otherwise on sampled columns (each output column is an independent sum)."""
    wl = synth.config(cid)
    for li, L in enumerate(wl.layers):
        print("config", wl.name, L.name, flush=True)
        t = synth.draw_layer(wl, li)
        W, G = t["W"], t["G"]
        sel, vals, idxw, flags = oracle_all(L, W, G)
        layer, out = run_select_pack(L, W, G)
        assert_select_pack_equal(L, out, sel, vals, idxw, flags)
        if t["X"] is None:
            cv = L.conv
            dact = dev(t["act"])
            dX = torch.empty((L.K, L.Ncol), dtype=torch.int16, device="cuda")
            crisp.crisp_im2col(crisp.ConvDesc(cv.C, cv.H, cv.W, cv.batch, cv.kh, cv.kw, cv.stride, cv.pad, 0, 0),
                               dact, dX, L.Ncol)
            torch.cuda.synchronize()
            X = host(dX, np.uint16)
            assert (X == oracle.im2col(t["act"], cv.kh, cv.kw, cv.stride, cv.pad)).all()
        else:
            X = t["X"]
            dX = dev(X)
        rng = np.random.default_rng(cid * 10 + li)
        full = L.S * L.K * L.Ncol <= 4e9
        cols = np.arange(L.Ncol) if full else _sample_columns(L.Ncol, 1500, rng)
        Xs = np.ascontiguousarray(X[:, cols])
        Yref, Aref = oracle.gemm_masked(W, sel.mask, Xs)
        for yd in (crisp.Y_F32, crisp.Y_BF16):
            Y = run_spmm(layer, dX, L.Ncol, L.Ncol, yd, L.S, ldy=L.Ncol)
            check_product(Y[:, cols], Yref, Aref, yd, L.name)
            if not full:
                # properties that hold at any size: rows of all-zero weight rows are zero, output finite
                assert np.isfinite(Y).all()
                dead = ~sel.mask.any(axis=1)
                assert (Y[dead] == 0).all()
            if t["X"] is None:
                # the path bench.py times for convolution layers: lowering fused into the product
                tdt = torch.float32 if yd == crisp.Y_F32 else torch.bfloat16
                Yc = torch.full((L.S, L.Ncol), float("nan"), dtype=tdt, device="cuda")
                path = crisp.conv_forward(layer, L.conv, dact, Yc, L.Ncol, yd, X_scratch=dX)
                torch.cuda.synchronize()
                assert path == "fused", path
                Yh = Yc.float().cpu().numpy().astype(np.float64)
                check_product(Yh[:, cols], Yref, Aref, yd, L.name + " fused lowering")
        del dX
        torch.cuda.empty_cache()


def _device_relu_normal_bits(shape, seed):
    """ReLU(N(0,1)) rounded to bf16, drawn on the device (too large to draw on the host in reasonable time)."""
    gen = torch.Generator(device="cuda")
    gen.manual_seed(seed)
    out = torch.empty(shape, dtype=torch.bfloat16, device="cuda")
    rows = max(1, (1 << 26) // shape[-1])
    flat = out.view(-1, shape[-1])
    for r0 in range(0, flat.shape[0], rows):
        part = flat[r0:r0 + rows]
        part.copy_(torch.randn(part.shape, generator=gen, device="cuda").clamp_(min=0).to(torch.bfloat16))
    return out.view(torch.int16)


@pytest.mark.parametrize("case", [
    # S, K, n, m, B, density, Ncol (= ldx = ldy), forced shapes
    # the widest Y the specialised kernels take (ldy = 2^23): X-resident kernel (the library's own choice
    # here), narrow and wide strips of the register kernels
    (128, 64, 2, 4, 64, 1.0, 1 << 23, (None, 1, 7)),
    # one step beyond: handed to the generic kernel
    (64, 64, 1, 4, 32, 0.5, (1 << 23) + 8, (None,)),
    # the largest column count the entry point accepts (2^27)
    (32, 32, 2, 8, 32, 1.0, 1 << 27, (None,)),
], ids=lambda c: "S%d_K%d_N%d" % (c[0], c[1], c[6]))
def test_maximum_column_counts(case):
    """Products at the documented column limits, bf16 output, checked on sampled columns (first and last
    strips plus random ones) against the oracle; untouched guard rows below Y."""
    S, K, n, m, B, dens, Ncol, shapes = case
    L = synth.LayerSpec("wide", S, K, Ncol, n, m, B, dens, synth.SAL_MAG, 0.05)
    rng = np.random.default_rng(S + K)
    W = synth.draw_weight(rng, L)
    sel = oracle.select(W, None, n, m, B, dens, synth.SAL_MAG)
    layer, _ = run_select_pack(L, W, None)
    dX = _device_relu_normal_bits((K, Ncol), 77)
    cols = _sample_columns(Ncol, 2000, rng)
    tcols = torch.from_numpy(cols).cuda()
    Xs = np.ascontiguousarray(host(dX[:, tcols], np.uint16))
    Yref, Aref = oracle.gemm_masked(W, sel.mask, Xs)
    for shape in shapes:
        print("wide case", case[:7], "shape", shape, flush=True)
        Y = torch.full((S + 1, Ncol), float("nan"), dtype=torch.bfloat16, device="cuda")
        spmm(layer.desc, layer.row_ptr, layer.col_idx, layer.vals, layer.idx_words, dX, Ncol, Ncol, Y, Ncol,
                         crisp.Y_BF16, shape=shape)
        torch.cuda.synchronize()
        assert bool(torch.isnan(Y[S]).all()), "row beyond S was written"
        assert bool(torch.isfinite(Y[:S]).all())
        Yh = Y[:S][:, tcols].float().cpu().numpy().astype(np.float64)
        check_product(Yh, Yref, Aref, crisp.Y_BF16, "wide %s shape %s" % (case[:7], shape))
        del Y
        torch.cuda.empty_cache()


def test_maximum_row_stride_of_x():
    """X handed over as the first columns of a tensor with the largest accepted row stride (2^27)."""
    L = synth.LayerSpec("wide_ldx", 128, 128, 520, 2, 4, 64, 1.0, synth.SAL_MAG, 0.05)
    W, G, X = synth.draw_small(L, 31)
    sel = oracle.select(W, G, L.n, L.m, L.B, L.density, L.sal_kind)
    layer, _ = run_select_pack(L, W, G)
    Yref, Aref = oracle.gemm_masked(W, sel.mask, X)
    ldx = 1 << 27
    dX = torch.zeros((L.K, ldx), dtype=torch.int16, device="cuda")
    dX[:, : L.Ncol] = dev(X)
    for shape in (None, 0, 1, 2, 4, 5, 6, 8, 13, 15, 16):
        print("wide ldx shape", shape, flush=True)
        for yd in (crisp.Y_F32, crisp.Y_BF16):
            Y = run_spmm(layer, dX, L.Ncol, ldx, yd, L.S, shape=shape)
            check_product(Y, Yref, Aref, yd, "wide ldx shape %s" % shape)


def test_maximum_convolution_plane():
    """Fused lowering with 2^23 output columns (the widest Y the fused kernels take): the kernel that
    stages the input in LDS (the library's own choice) and the register kernels, sampled columns."""
    C_, H, Wd, b, k, pad, S, n, m, B, dens = 64, 64, 64, 2048, 3, 1, 128, 2, 4, 64, 0.5
    cv = synth.ConvShape(C_, H, Wd, b, k, k, 1, pad)
    assert cv.Ncol == 1 << 23
    L = synth.LayerSpec("wide_conv", S, cv.K, cv.Ncol, n, m, B, dens, synth.SAL_MAG, 0.05, conv=cv)
    rng = np.random.default_rng(5)
    W = synth.draw_weight(rng, L)
    sel = oracle.select(W, None, n, m, B, dens, synth.SAL_MAG)
    layer, _ = run_select_pack(L, W, None)
    dact = _device_relu_normal_bits((C_, b, H, Wd), 78)
    cols = _sample_columns(cv.Ncol, 1500, rng)
    idx, inside = lowering_gather_index(C_, H, Wd, b, k, k, 1, pad, cols)
    g = torch.take(dact.view(-1), torch.from_numpy(idx).cuda()).cpu().numpy().view(np.uint16)
    Xs = np.ascontiguousarray(np.where(inside, g, np.uint16(0)))
    Yref, Aref = oracle.gemm_masked(W, sel.mask, Xs)
    tcols = torch.from_numpy(cols).cuda()
    conv = crisp.conv_desc_of(cv)
    for shape in (None, 12, 1, 8):
        print("wide conv shape", shape, flush=True)
        Y = torch.full((S + 1, cv.Ncol), float("nan"), dtype=torch.bfloat16, device="cuda")
        conv_spmm(layer.desc, conv, layer.row_ptr, layer.col_idx, layer.vals, layer.idx_words, dact, Y, cv.Ncol,
                              crisp.Y_BF16, shape=shape)
        torch.cuda.synchronize()
        assert bool(torch.isnan(Y[S]).all()) and bool(torch.isfinite(Y[:S]).all())
        Yh = Y[:S][:, tcols].float().cpu().numpy().astype(np.float64)
        check_product(Yh, Yref, Aref, crisp.Y_BF16, "wide conv shape %s" % shape)
        del Y
        torch.cuda.empty_cache()


@pytest.mark.parametrize("L", [synth.small_cases()[0], synth.small_cases()[13], synth.b16_cases()[2]], ids=lambda L: L.name)
def test_block_scores_are_an_optional_output(L):
    """Without a block_score buffer the scores live in the caller's workspace; masks, block lists and packing
    stay the same bytes (separate calls and the fused call)."""
    W, G, _ = synth.draw_small(L, 95)
    sel, vals, idxw, flags = oracle_all(L, W, G)
    layer = crisp.alloc_layer(desc_of(L))
    sz = layer.sizes
    dW, dG = dev(W), dev(G) if G is not None else None
    for fused in (False, True):
        for t in (layer.nm_mask, layer.row_ptr, layer.col_idx, layer.vals, layer.idx_words, layer.flags):
            t.fill_(-1)
        if fused:
            ws = torch.empty(max(16, sz.select_pack_ws_bytes), dtype=torch.uint8, device="cuda")
            crisp.crisp_select_pack(layer.desc, dW, dG, layer.nm_mask, layer.row_ptr, layer.col_idx, layer.vals, layer.idx_words,
                                    layer.flags, ws, ws.numel(), block_score=None)
        else:
            ws = torch.empty(max(16, sz.select_ws_bytes), dtype=torch.uint8, device="cuda")
            crisp.crisp_select_mask(layer.desc, dW, dG, layer.nm_mask, layer.row_ptr, layer.col_idx, None, ws, ws.numel())
            crisp.crisp_pack(layer.desc, dW, layer.nm_mask, layer.row_ptr, layer.col_idx, layer.vals, layer.idx_words, layer.flags)
        torch.cuda.synchronize()
        assert (host(layer.nm_mask, np.uint32)[: sz.mask_words].reshape(L.S, sz.mask_words_per_row) == sel.nm_bits).all()
        assert (host(layer.row_ptr, np.int32) == sel.row_ptr).all()
        assert (host(layer.col_idx, np.int32)[: int(sel.row_ptr[-1])] == sel.col_idx).all()
        assert (host(layer.vals, np.uint16)[: vals.size] == vals.reshape(-1)).all()
        assert (host(layer.idx_words, np.uint32)[: idxw.size] == idxw.reshape(-1)).all()
        assert host(layer.flags, np.int32)[0] == flags[0]


def test_calls_on_two_streams_do_not_disturb_each_other():
    """The library keeps no state between calls: selection, packing and products of two layers enqueued
    alternately on two streams give the bytes each layer gives on its own."""
    cases = [synth.small_cases()[1], synth.small_cases()[3]]
    work = []
    for i, L in enumerate(cases):
        W, G, X = synth.draw_small(L, 90 + i)
        ldx = (L.Ncol + 7) // 8 * 8
        Xp = np.zeros((L.K, ldx), dtype=np.uint16)
        Xp[:, : L.Ncol] = X
        layer, out = run_select_pack(L, W, G)
        Yalone = run_spmm(layer, dev(Xp), L.Ncol, ldx, crisp.Y_F32, L.S, ldy=ldx)
        fresh = crisp.alloc_layer(desc_of(L))
        work.append(dict(L=L, W=dev(W), G=dev(G) if G is not None else None, X=dev(Xp), ldx=ldx, layer=fresh, alone=(out, Yalone),
                         Y=torch.zeros((L.S, ldx), dtype=torch.float32, device="cuda"), stream=torch.cuda.Stream()))
    torch.cuda.synchronize()
    for it in range(10):
        for w in work:
            with torch.cuda.stream(w["stream"]):
                for t in (w["layer"].vals, w["layer"].idx_words, w["layer"].col_idx):
                    t.fill_(-1)
                crisp.prune_and_pack(w["layer"], w["W"], w["G"])
                crisp.crisp_spmm(w["layer"].desc, w["layer"].row_ptr, w["layer"].col_idx, w["layer"].vals, w["layer"].idx_words,
                                 w["X"], w["L"].Ncol, w["ldx"], w["Y"], w["ldx"])
    torch.cuda.synchronize()
    for w in work:
        out, Yalone = w["alone"]
        sz = w["layer"].sizes
        assert (host(w["layer"].col_idx, np.int32)[: sz.nk] == out["col_idx"]).all()
        assert (host(w["layer"].vals, np.uint16)[: sz.vals_elems] == out["vals"].reshape(-1)).all()
        assert (host(w["layer"].idx_words, np.uint32)[: sz.idx_words] == out["idxw"].reshape(-1)).all()
        assert (w["Y"].cpu().numpy().astype(np.float64)[:, : w["L"].Ncol] == Yalone).all()


def test_determinism():
    L = synth.small_cases()[1]
    W, G, X = synth.draw_small(L, 30)
    layer, _ = run_select_pack(L, W, G)
    ldx = (L.Ncol + 7) // 8 * 8
    Xp = np.zeros((L.K, ldx), dtype=np.uint16)
    Xp[:, : L.Ncol] = X
    dX = dev(Xp)
    a = run_spmm(layer, dX, L.Ncol, ldx, crisp.Y_F32, L.S)
    b = run_spmm(layer, dX, L.Ncol, ldx, crisp.Y_F32, L.S)
    assert (a == b).all()
