"""Host-side checks of the C ABI that need no GPU: the library loads, exports every entry
point the header declares, and rejects bad arguments before touching a device."""
import ctypes as C
import os
import re
import subprocess

import pytest

from paper_2311_14272_amd import crisp

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
HEADER = os.path.join(ROOT, "include", "crisp.h")


def declared_functions():
    text = open(HEADER).read()
    return sorted(set(re.findall(r"CRISP_API[^;(]*?\b(crisp_\w+)\s*\(", text)))


def test_library_exports_every_declared_symbol():
    names = declared_functions()
    assert names == ["crisp_conv_forward", "crisp_conv_plan", "crisp_conv_spmm", "crisp_conv_spmm_ep", "crisp_conv_spmm_forced",
                     "crisp_global_budget", "crisp_im2col", "crisp_maxpool", "crisp_pack", "crisp_pack_sizes", "crisp_select_mask",
                     "crisp_select_pack", "crisp_select_pack_batch", "crisp_select_pack_noalloc", "crisp_spmm", "crisp_spmm_ep", "crisp_spmm_forced",
                     "crisp_spmm_timed", "crisp_status_str"]
    L = crisp.lib()
    for n in names:
        assert getattr(L, n) is not None
    out = subprocess.run(["nm", "-D", "--defined-only", crisp.LIB_PATH], capture_output=True, text=True).stdout
    exported = {l.split()[-1] for l in out.splitlines() if " T " in l}
    assert set(names) <= exported
    assert all(e.startswith("crisp_") or e.startswith("_") for e in exported)


def test_header_compiles_as_c():
    r = subprocess.run(["gcc", "-std=c99", "-Wall", "-Werror", "-fsyntax-only", "-x", "c", HEADER],
                       capture_output=True, text=True)
    assert r.returncode == 0, r.stderr


def test_struct_layout_matches_header():
    src = r'''
    #include <stdio.h>
    #include <stddef.h>
    #include "crisp.h"
    int main(void) {
      printf("%zu %zu %zu %zu %zu %zu\n", sizeof(crisp_layer_desc), offsetof(crisp_layer_desc, S),
             sizeof(crisp_sizes), offsetof(crisp_sizes, mask_words), offsetof(crisp_sizes, select_ws_bytes),
             sizeof(crisp_conv_desc));
      return 0; }'''
    exe = "/tmp/crisp_layout_check"
    r = subprocess.run(["gcc", "-std=c99", "-I", os.path.join(ROOT, "include"), "-x", "c", "-", "-o", exe],
                       input=src, capture_output=True, text=True)
    assert r.returncode == 0, r.stderr
    got = [int(x) for x in subprocess.run([exe], capture_output=True, text=True).stdout.split()]
    assert got == [C.sizeof(crisp.LayerDesc), crisp.LayerDesc.S.offset, C.sizeof(crisp.Sizes),
                   crisp.Sizes.mask_words.offset, crisp.Sizes.select_ws_bytes.offset, C.sizeof(crisp.ConvDesc)]


def test_pack_sizes_values():
    sz = crisp.crisp_pack_sizes(crisp.layer_desc(256, 1152, 2, 4, 32, 0.5))
    assert (sz.Sb, sz.Kb, sz.k_row, sz.nk) == (8, 36, 18, 144)
    assert (sz.slots_per_row, sz.idx_bits, sz.idx_words_per_row) == (16, 2, 1)
    assert sz.vals_elems == 144 * 32 * 16 and sz.idx_words == 144 * 32
    assert sz.mask_words == 256 * 36 and sz.row_ptr_elems == 9 and sz.score_elems == 8 * 36
    # scores + violation flags + packed values and positions of all 8 x 36 blocks
    assert sz.select_pack_ws_bytes == 8 * 36 * 8 + 8 * 36 * 4 + 8 * 36 * 32 * (16 * 2 + 4)
    sz = crisp.crisp_pack_sizes(crisp.layer_desc(24, 144, 2, 4, 32, 0.6))
    assert (sz.Sb, sz.Kb, sz.k_row, sz.nk) == (1, 5, 3, 3)
    sz = crisp.crisp_pack_sizes(crisp.layer_desc(64, 147, 4, 8, 64, 0.5))
    assert (sz.Sb, sz.Kb, sz.k_row) == (1, 3, 2) and sz.idx_words_per_row == 3 and sz.mask_words_per_row == 5
    for cfg, kr in (((256, 1024, 1, 4, 64, 0.3), 5), ((256, 2304, 1, 4, 64, 0.3), 11), ((1024, 256, 1, 4, 64, 0.3), 1),
                    ((512, 4608, 2, 8, 64, 0.25), 18), ((160, 960, 2, 4, 32, 0.6), 18)):
        assert crisp.crisp_pack_sizes(crisp.layer_desc(*cfg)).k_row == kr


@pytest.mark.parametrize("kw,status", [
    (dict(m=5), crisp.EINVAL), (dict(n=0), crisp.EINVAL), (dict(n=5), crisp.EINVAL), (dict(B=48), crisp.EINVAL),
    (dict(B=16, m=8, n=2), None), (dict(block_density=0.0), crisp.EINVAL), (dict(block_density=1.5), crisp.EINVAL),
    (dict(block_density=float("nan")), crisp.EINVAL), (dict(S=0), crisp.ESHAPE), (dict(K=-3), crisp.ESHAPE),
    (dict(sal_kind=7), crisp.EINVAL), (dict(select_mode=2), crisp.EINVAL),
    # hints: the one defined bit is accepted for any pattern (it only means something for 4:8), unknown bits are refused
    (dict(hints=1), None), (dict(hints=1, n=4, m=8), None), (dict(hints=2), crisp.EINVAL), (dict(hints=-1), crisp.EINVAL),
    # packed values of the whole grid: 4 GiB and one block column less
    (dict(S=32768, K=65536, n=4, m=4, B=64), crisp.ESHAPE), (dict(S=32768, K=65536 - 64, n=4, m=4, B=64), None)])
def test_descriptor_validation(kw, status):
    base = dict(S=64, K=128, n=2, m=4, B=32, block_density=0.5)
    base.update(kw)
    d = crisp.layer_desc(**base)
    if status is None:
        crisp.crisp_pack_sizes(d)
        return
    with pytest.raises(crisp.CrispError) as e:
        crisp.crisp_pack_sizes(d)
    assert e.value.status == status


def test_entry_points_reject_bad_arguments_without_a_device():
    L = crisp.lib()
    d = crisp.layer_desc(64, 128, 2, 4, 32, 0.5)
    fake = 0x1000  # never dereferenced: every call below must fail validation first
    assert L.crisp_select_mask(C.byref(d), None, None, None, None, None, None, None, 0, None) == crisp.EINVAL
    assert L.crisp_select_mask(C.byref(d), fake, None, fake, fake, fake, None, None, 0, None) == crisp.EBUFSIZE
    assert L.crisp_select_mask(C.byref(d), fake + 2, None, fake, fake, fake, fake, None, 0, None) == crisp.EALIGN
    dg = crisp.layer_desc(64, 128, 2, 4, 32, 0.5, sal_kind=crisp.SAL_GRAD)
    assert L.crisp_select_mask(C.byref(dg), fake, None, fake, fake, fake, fake, None, 0, None) == crisp.EINVAL
    sp = lambda **k: L.crisp_select_pack(C.byref(k.get("d", d)), k.get("W", fake), k.get("T", None), fake, fake, fake, None,
                                         k.get("vals", fake), fake, fake, k.get("ws", fake), k.get("wsb", 1 << 30), None)
    assert sp(W=None) == crisp.EINVAL
    assert sp(d=dg) == crisp.EINVAL            # gradient saliency without a gradient tensor
    assert sp(vals=fake + 2) == crisp.EALIGN
    assert sp(ws=None) == crisp.EBUFSIZE
    assert sp(wsb=crisp.crisp_pack_sizes(d).select_pack_ws_bytes - 1) == crisp.EBUFSIZE
    # the variant with the built-in workspace: same checks, and a layer beyond the built-in array is refused
    na = lambda **k: L.crisp_select_pack_noalloc(C.byref(k.get("d", d)), k.get("W", fake), None, fake, fake, fake, None,
                                                 k.get("vals", fake), fake, fake, None)
    assert na(W=None) == crisp.EINVAL and na(vals=fake + 2) == crisp.EALIGN and na(d=dg) == crisp.EINVAL
    big = crisp.layer_desc(4096, 4096, 4, 4, 64, 0.5)
    assert crisp.crisp_pack_sizes(big).select_pack_ws_bytes > crisp.STATIC_SCRATCH_BYTES and na(d=big) == crisp.EBUFSIZE
    # batch: every layer is checked before anything is enqueued
    good = crisp.LayerBuffers(fake, None, fake, fake, fake, None, fake, fake, fake, fake, 1 << 30)
    bad = crisp.LayerBuffers(fake, None, fake, fake, fake, None, None, fake, fake, fake, 1 << 30)
    descs = (crisp.LayerDesc * 2)(d, d)
    assert L.crisp_select_pack_batch(2, descs, (crisp.LayerBuffers * 2)(good, bad), None) == crisp.EINVAL
    assert L.crisp_select_pack_batch(0, descs, (crisp.LayerBuffers * 2)(good, good), None) == crisp.EINVAL
    assert L.crisp_select_pack_batch(2, None, (crisp.LayerBuffers * 2)(good, good), None) == crisp.EINVAL
    assert L.crisp_pack(C.byref(d), fake, fake, fake, fake, None, fake, fake, None, 0, None) == crisp.EINVAL
    assert L.crisp_pack(C.byref(d), fake, fake, fake, fake, fake + 8, fake, fake, None, 0, None) == crisp.EALIGN
    spmm = lambda **k: L.crisp_spmm(C.byref(k.get("d", d)), fake, fake, fake, fake, k.get("X", fake), k.get("N", 64),
                                    k.get("ldx", 64), k.get("xl", 0), k.get("Y", fake), k.get("ldy", 64),
                                    k.get("yd", 0), None, 0, None)
    assert spmm(X=None) == crisp.EINVAL
    assert spmm(N=0) == crisp.ESHAPE
    assert spmm(ldx=56) == crisp.ESHAPE
    assert spmm(N=60, ldx=60, ldy=64) == crisp.EALIGN
    assert spmm(ldy=100, N=64) == crisp.EALIGN
    assert spmm(yd=3) == crisp.EINVAL
    assert spmm(xl=2) == crisp.EUNSUPPORTED
    # octet-interleaved operands: S must be a multiple of 8, K of 16, no 16 x 16 blocks
    assert spmm(xl=1, d=crisp.layer_desc(60, 128, 2, 4, 32, 0.5)) == crisp.EUNSUPPORTED
    assert spmm(xl=1, d=crisp.layer_desc(64, 136, 2, 4, 32, 0.5)) == crisp.EUNSUPPORTED
    assert spmm(xl=1, d=crisp.layer_desc(64, 128, 2, 4, 16, 0.5)) == crisp.EUNSUPPORTED
    assert spmm(Y=fake + 4) == crisp.EALIGN
    # the reserved workspace arguments select nothing: a stale size with ws == NULL is validated like any other call
    assert L.crisp_spmm(C.byref(d), fake, fake, fake, fake, None, 64, 64, 0, fake, 64, 0, None, 5, None) == crisp.EINVAL
    code = C.c_int32(-7)
    forced = lambda shape, **k: L.crisp_spmm_forced(C.byref(d), fake, fake, fake, fake, k.get("X", fake), 64, 64, 0, fake,
                                                    k.get("ldy", 64), 0, None, shape, C.byref(code), None)
    assert forced(1, X=None) == crisp.EINVAL and forced(99, ldy=100) == crisp.EALIGN and code.value == -7
    spmm_ep = lambda ep: L.crisp_spmm_ep(C.byref(d), fake, fake, fake, fake, fake, 64, 64, 0, fake, 64, 0, C.byref(ep), None, 0, None)
    assert spmm_ep(crisp.Epilogue(fake + 2, None, None, 0, 0, 0)) == crisp.EALIGN
    assert spmm_ep(crisp.Epilogue(None, None, fake, 56, 0, 0)) == crisp.ESHAPE
    assert spmm_ep(crisp.Epilogue(None, None, fake, 68, 0, 0)) == crisp.EALIGN
    assert spmm_ep(crisp.Epilogue(None, None, None, 0, 2, 0)) == crisp.EINVAL
    cv = crisp.ConvDesc(3, 8, 8, 1, 3, 3, 1, 1, 0, 0)
    assert L.crisp_im2col(C.byref(cv), None, fake, 64, None) == crisp.EINVAL
    assert L.crisp_im2col(C.byref(cv), fake, fake, 8, None) == crisp.ESHAPE
    cv2 = crisp.ConvDesc(3, 2, 2, 1, 5, 5, 1, 0, 0, 0)
    assert L.crisp_im2col(C.byref(cv2), fake, fake, 64, None) == crisp.ESHAPE
    cv3 = crisp.ConvDesc(3, 8, 8, 1, 3, 3, 1, 1, 1, 0)
    assert L.crisp_im2col(C.byref(cv3), fake, fake, 64, None) == crisp.EUNSUPPORTED
    # sizes beyond the stated limits: a filter edge of 256, a million channels, 2^31 - 1024 columns
    assert L.crisp_im2col(C.byref(crisp.ConvDesc(3, 300, 300, 1, 256, 3, 1, 0, 0, 0)), fake, fake, 1 << 20, None) == crisp.EUNSUPPORTED
    assert L.crisp_im2col(C.byref(crisp.ConvDesc(1 << 20, 2, 2, 1, 1, 1, 1, 0, 0, 0)), fake, fake, 64, None) == crisp.EUNSUPPORTED
    assert L.crisp_im2col(C.byref(crisp.ConvDesc(1, 1, (1 << 31) - 512, 1, 1, 1, 1, 0, 0, 0)), fake, fake, 1 << 31, None) == crisp.ESHAPE
    assert L.crisp_maxpool(C.byref(crisp.ConvDesc(3, 600, 600, 1, 256, 256, 1, 0, 0, 0)), fake, fake, None) == crisp.EUNSUPPORTED
    assert crisp.status_str(crisp.EALIGN).startswith("misaligned")


def test_missing_library_fails_loudly(monkeypatch):
    monkeypatch.setattr(crisp, "_lib", None)
    monkeypatch.setattr(crisp, "LIB_PATH", "/nonexistent/libcrisp.so")
    with pytest.raises(RuntimeError, match="no CPU fallback"):
        crisp.lib()


def test_lowering_choice_on_resnet50_shapes():
    """The helper that picks how a convolution is lowered (host logic only)."""
    from paper_2311_14272_amd import synth
    cs = synth.ConvShape
    pick = lambda cv, S, d: crisp.lowering_path(cv, 64, 2, 4, S, d)
    assert pick(cs(256, 14, 14, 8, 1, 1, 1, 0), 1024, 0.5) == "none"          # 1x1 stride 1: the activation is X
    assert pick(cs(256, 14, 14, 8, 3, 3, 1, 1), 256, 0.9) == "fused"          # stride 1, even width: paired loads
    assert pick(cs(128, 56, 56, 8, 3, 3, 2, 1), 128, 0.25) == "fused"         # strided, few gathers per block column
    assert pick(cs(256, 28, 28, 8, 3, 3, 2, 1), 256, 0.70) == "fused"         # strided, dense block-rows: staged in LDS
    assert pick(cs(512, 14, 14, 8, 3, 3, 2, 1), 512, 0.70) == "im2col"        # strided, odd output width, many gathers per block column
    assert pick(cs(512, 7, 7, 8, 3, 3, 1, 1), 512, 0.70) == "fused"           # stride 1, odd width, padding (k-1)/2: paired loads
    assert pick(cs(512, 9, 9, 8, 3, 3, 1, 0), 512, 0.70) == "im2col"          # stride 1, odd width, no padding: column by column
    assert pick(cs(256, 56, 56, 8, 1, 1, 2, 0), 512, 0.5) == "fused"          # 1x1 stride 2, few gathers per block column
    assert pick(cs(512, 28, 28, 8, 1, 1, 2, 0), 1024, 0.66) == "im2col"       # 1x1 stride 2, many: nothing inflated to save
    assert pick(cs(3, 224, 224, 8, 7, 7, 2, 3), 64, 0.5) == "fused"           # first layer: one block-row
    # 1x1 stride 2, many gathers, but at most 512 channels, 8 or more block-rows, n <= 2 and many columns: the strided
    # gather is staged once per strip in LDS for all block-rows
    assert pick(cs(256, 56, 56, 64, 1, 1, 2, 0), 512, 0.9) == "fused"
    assert crisp.lowering_path(cs(256, 56, 56, 64, 1, 1, 2, 0), 64, 4, 8, 512, 0.9) == "im2col"    # dense-expansion pattern
    assert pick(cs(1024, 14, 14, 64, 1, 1, 2, 0), 2048, 0.9) == "im2col"      # more channels than that kernel holds
    assert crisp.conv_needs_scratch(cs(512, 14, 14, 8, 3, 3, 2, 1), 64, 2, 4, 512, 0.70)
    assert not crisp.conv_needs_scratch(cs(256, 14, 14, 8, 3, 3, 1, 1), 64, 2, 4, 256, 0.9)
    # scratch size of the materialised path: K x round_up(Ncol, 8) bf16; argument checks on the host
    cv = cs(512, 14, 14, 3, 3, 3, 2, 1)
    path, nbytes = crisp.conv_plan(crisp.layer_desc(512, 9 * 512, 2, 4, 64, 0.7), cv)
    assert path == "im2col" and nbytes == 9 * 512 * ((3 * 49 + 7) // 8 * 8) * 2
    assert crisp.conv_plan(crisp.layer_desc(256, 9 * 256, 2, 4, 64, 0.9), cs(256, 14, 14, 8, 3, 3, 1, 1)) == ("fused", 0)
    with pytest.raises(crisp.CrispError) as e:
        crisp.conv_plan(crisp.layer_desc(256, 9 * 128, 2, 4, 64, 0.9), cs(256, 14, 14, 8, 3, 3, 1, 1))   # K mismatch
    assert e.value.status == crisp.ESHAPE
    L = crisp.lib()
    d = crisp.layer_desc(512, 9 * 512, 2, 4, 64, 0.7)
    conv = crisp.conv_desc_of(cv)
    fake = 0x1000
    fwd = lambda scratch, nb: L.crisp_conv_forward(C.byref(d), C.byref(conv), fake, fake, fake, fake, fake, fake, 152, 0, None,
                                                   scratch, nb, None, None)
    assert fwd(None, 0) == crisp.EBUFSIZE and fwd(fake, nbytes - 2) == crisp.EBUFSIZE
