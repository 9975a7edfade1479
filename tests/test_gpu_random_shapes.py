"""Seeded random shapes through every entry point, checked against the oracle like the hand-picked cases:
masks, packing, lowering and pooling bit-exact, products within the stated tolerance.  The draws stay
inside the documented limits; what an entry point rejects (odd column counts in the fused lowering, ...)
must be rejected with a status, never computed wrongly.  Every case is printed before it runs."""
import numpy as np
import pytest
import torch

import oracle
from paper_2311_14272_amd import crisp, synth

from gpu_util import check_bf16_is_rounded_f32, check_product, desc_of, dev, host, run_select_pack, run_spmm, spmm_ep, conv_spmm_ep, conv_spmm
from test_gpu_epilogue import _check as check_epilogue_product, _draw_ep

pytestmark = pytest.mark.gpu

PATTERNS = [(1, 4), (2, 4), (3, 4), (4, 4), (1, 8), (2, 8), (4, 8), (8, 8)]


def _report(fails):
    assert not fails, "%d failing cases, first: %s" % (len(fails), fails[:5])


def _draw_conv(rng, max_work):
    """A convolution layer inside the limits of crisp_conv_spmm's argument checks (not necessarily covered)."""
    while True:
        C_ = int(rng.choice([3, 5, 8, 16, 24, 40, 64, 64, 128, 128, 192]))
        kh = int(rng.choice([1, 3, 3, 3, 5, 7]))
        kw = kh if rng.random() < 0.8 else int(rng.choice([1, 3, 5]))
        stride = int(rng.choice([1, 1, 1, 2, 2, 3, 4]))
        pad = int(rng.choice([0, kh // 2, kh // 2]))
        H = int(rng.integers(max(kh - 2 * pad, 1), 30))
        Wd = int(rng.integers(max(kw - 2 * pad, 1), 68))
        if rng.random() < 0.7:
            Wd += Wd & 1
        b = int(rng.integers(1, 5))
        B = int(rng.choice([16, 32, 64, 64, 64]))
        n, m = PATTERNS[int(rng.integers(0, len(PATTERNS)))]
        S = int(rng.choice([32, 64, 96, 128, 200, 256, 320]))
        dens = float(rng.choice([0.2, 0.35, 0.5, 0.7, 1.0]))
        mode = synth.LAYER_TOPK if rng.random() < 0.2 else 0
        cv = synth.ConvShape(C_, H, Wd, b, kh, kw, stride, pad)
        if cv.Ho < 1 or cv.Wo < 1 or S * cv.K * cv.Ncol > max_work:
            continue
        return cv, synth.LayerSpec("rc", S, cv.K, cv.Ncol, n, m, B, dens, synth.SAL_MAG, 0.05, conv=cv, select_mode=mode)


@pytest.mark.parametrize("seed", [101, 102])
def test_random_convolutions(seed):
    """crisp_conv_spmm: the library's own choice of kernel and the forced ones (12 input staged in LDS, 14
    few-channel patch, 1 / 8 register kernels dense / sparse matrix core)."""
    rng = np.random.default_rng(seed)
    fails, computed = [], 0
    for case in range(150):
        cv, L = _draw_conv(rng, 4e8)
        print("conv case", case, cv, (L.S, L.n, L.m, L.B, L.density, L.select_mode), flush=True)
        W = synth.draw_weight(rng, L)
        act = synth.draw_relu_normal(rng, (cv.C, cv.batch, cv.H, cv.W))
        sel = oracle.select(W, None, L.n, L.m, L.B, L.density, synth.SAL_MAG, L.select_mode)
        layer, out = run_select_pack(L, W, None)
        assert (out["col_idx"] == sel.col_idx).all() and (out["row_ptr"] == sel.row_ptr).all()
        Yref, Aref = oracle.gemm_masked(W, sel.mask, oracle.im2col(act, cv.kh, cv.kw, cv.stride, cv.pad))
        conv = crisp.conv_desc_of(cv)
        dact = dev(act)
        S, Ncol = L.S, cv.Ncol
        ldy = (Ncol + 7) // 8 * 8 + 8
        for shape in (None, 12, 14, 1, 8):
            for yd, tdt in ((crisp.Y_F32, torch.float32), (crisp.Y_BF16, torch.bfloat16)):
                Y = torch.full((S + 1, ldy), float("nan"), dtype=tdt, device="cuda")
                try:
                    conv_spmm(layer.desc, conv, layer.row_ptr, layer.col_idx, layer.vals, layer.idx_words, dact, Y,
                                          ldy, yd, shape=shape)
                except crisp.CrispError as e:
                    assert e.status == crisp.EUNSUPPORTED and ((Ncol & 1) or L.B == 16), (cv, e.status)
                    continue
                torch.cuda.synchronize()
                Yh = Y.float().cpu().numpy().astype(np.float64)
                computed += 1
                try:
                    assert np.isnan(Yh[:S, Ncol:]).all() and np.isnan(Yh[S]).all(), "guard band written"
                    if yd == crisp.Y_F32:
                        Y32 = Yh[:S, :Ncol]
                    else:
                        check_bf16_is_rounded_f32(Yh[:S, :Ncol], Y32, "random conv")
                    if yd == crisp.Y_F32 or S * Ncol >= 2000:
                        check_product(Yh[:S, :Ncol], Yref, Aref, yd, "random conv")
                except AssertionError as e:
                    fails.append((cv, (L.S, L.n, L.m, L.B, L.density, L.select_mode), shape, yd, str(e)[:80]))
        # the whole-convolution entry point takes any geometry (odd column counts, 16 x 16 blocks, ...)
        Xs = torch.empty((cv.K, (Ncol + 7) // 8 * 8), dtype=torch.int16, device="cuda")
        for yd, tdt in ((crisp.Y_F32, torch.float32), (crisp.Y_BF16, torch.bfloat16)):
            Y = torch.full((S + 1, ldy), float("nan"), dtype=tdt, device="cuda")
            path = crisp.conv_forward(layer, cv, dact, Y, ldy, yd, Xs)
            torch.cuda.synchronize()
            Yh = Y.float().cpu().numpy().astype(np.float64)
            try:
                assert np.isnan(Yh[:S, Ncol:]).all() and np.isnan(Yh[S]).all(), "guard band written"
                if yd == crisp.Y_F32:
                    Y32 = Yh[:S, :Ncol]
                else:
                    check_bf16_is_rounded_f32(Yh[:S, :Ncol], Y32, "random conv forward")
                if yd == crisp.Y_F32 or S * Ncol >= 2000:
                    check_product(Yh[:S, :Ncol], Yref, Aref, yd, "random conv forward")
            except AssertionError as e:
                fails.append((cv, (L.S, L.n, L.m, L.B, L.density, L.select_mode), "forward " + path, yd, str(e)[:80]))
    assert computed > 900
    _report(fails)


@pytest.mark.parametrize("seed", [111])
def test_random_products(seed):
    """crisp_select_pack / crisp_select_mask + crisp_pack, then crisp_spmm in every launch shape."""
    rng = np.random.default_rng(seed)
    fails = []
    case = 0
    while case < 150:
        B = int(rng.choice([16, 32, 64, 64]))
        n, m = PATTERNS[int(rng.integers(0, len(PATTERNS)))]
        S = int(rng.integers(1, 6 * B + 1)) if rng.random() < 0.5 else int(rng.integers(1, 9)) * B
        kind = rng.random()
        K = int(rng.integers(1, 25)) * B if kind < 0.4 else int(rng.integers(1, 60)) * 16 if kind < 0.7 else int(rng.integers(m, 900))
        Ncol = int(rng.choice([int(rng.integers(1, 300)), int(rng.integers(1, 80)) * 4, int(rng.integers(1, 40)) * 64,
                               int(rng.integers(300, 5000))]))
        if S * K * Ncol > 2.5e8:
            continue
        dens = float(rng.choice([0.1, 0.25, 0.4, 0.5, 0.75, 1.0]))
        mode = synth.LAYER_TOPK if rng.random() < 0.2 else 0
        salk = synth.SAL_GRAD if rng.random() < 0.5 else synth.SAL_MAG
        L = synth.LayerSpec("rp", S, K, Ncol, n, m, B, dens, salk, 0.05, None, mode)
        what = (S, K, Ncol, n, m, B, dens, mode, salk)
        print("product case", case, what, flush=True)
        case += 1
        W, G, X = synth.draw_small(L, int(rng.integers(1, 1 << 30)))
        sel = oracle.select(W, G, n, m, B, dens, salk, mode)
        vals, idxw, flags = oracle.pack(W, sel.keep, n, m, B, sel.row_ptr, sel.col_idx)
        layer, out = run_select_pack(L, W, G, fused=bool(rng.random() < 0.7))
        same = ((out["nm_bits"] == sel.nm_bits).all() and (out["score"].view(np.uint64) == sel.score.view(np.uint64)).all()
                and (out["row_ptr"] == sel.row_ptr).all() and (out["col_idx"] == sel.col_idx).all()
                and (out["vals"] == vals).all() and (out["idxw"] == idxw).all() and out["flags"][0] == flags[0])
        if not same:
            fails.append((what, "select/pack"))
            continue
        Yref, Aref = oracle.gemm_masked(W, sel.mask, X)
        ldx = (Ncol + 7) // 8 * 8 + (8 if rng.random() < 0.3 else 0)
        Xp = np.full((K, ldx), 0x7FC0, dtype=np.uint16)     # NaN in the padding columns: must not leak
        Xp[:, :Ncol] = X
        dX = dev(Xp)
        for shape in (None, 0, 1, 2, 3, 4, 5, 6, 7, 8, 9, 10, 13, 15, 16, 17, 18):
            for yd in (crisp.Y_F32, crisp.Y_BF16):
                try:
                    Y = run_spmm(layer, dX, Ncol, ldx, yd, S, shape=shape)
                    if yd == crisp.Y_F32:
                        Y32 = Y
                    else:
                        check_bf16_is_rounded_f32(Y, Y32, "random product")
                    if yd == crisp.Y_F32 or S * Ncol >= 2000:
                        check_product(Y, Yref, Aref, yd, "random product")
                except AssertionError as e:
                    fails.append((what, shape, yd, str(e)[:80]))
    _report(fails)


@pytest.mark.parametrize("seed", [121])
def test_random_epilogues(seed):
    """crisp_spmm_ep and crisp_conv_spmm_ep with random combinations of scale, bias, residual and ReLU."""
    rng = np.random.default_rng(seed)
    fails = []
    case = 0
    while case < 60:
        n, m = PATTERNS[int(rng.integers(0, len(PATTERNS)))]
        dens = float(rng.choice([0.2, 0.4, 0.6, 1.0]))
        mode = synth.LAYER_TOPK if rng.random() < 0.2 else 0
        is_conv = rng.random() < 0.5
        if is_conv:
            cv, L0 = _draw_conv(rng, 2e8)
            if (cv.Ncol & 1) or L0.B == 16:       # not covered by the fused entry point
                continue
            L = synth.LayerSpec("re", L0.S, cv.K, cv.Ncol, n, m, L0.B, dens, synth.SAL_MAG, 0.05, conv=cv, select_mode=mode)
            W, G = synth.draw_weight(rng, L), None
            act = synth.draw_relu_normal(rng, (cv.C, cv.batch, cv.H, cv.W))
            X = oracle.im2col(act, cv.kh, cv.kw, cv.stride, cv.pad)
            shapes = (None, 12, 14, 1, 2, 8, 9)
        else:
            B = int(rng.choice([16, 32, 64, 64]))
            S = int(rng.integers(1, 6 * B + 1))
            K = int(rng.integers(1, 40)) * 16 if rng.random() < 0.7 else int(rng.integers(m, 700))
            Ncol = int(rng.choice([int(rng.integers(1, 300)), int(rng.integers(1, 80)) * 4, int(rng.integers(300, 3000))]))
            if S * K * Ncol > 2e8:
                continue
            L = synth.LayerSpec("re", S, K, Ncol, n, m, B, dens, synth.SAL_MAG, 0.05, None, mode)
            W, G, X = synth.draw_small(L, int(rng.integers(1, 1 << 30)))
            shapes = (None, 0, 1, 2, 3, 4, 5, 6, 7, 8, 9, 10, 13, 15, 16, 17, 18)
        what = ("conv", cv) if is_conv else "plain", (L.S, L.K, L.Ncol, n, m, L.B, dens, mode)
        print("epilogue case", case, what, flush=True)
        case += 1
        sel = oracle.select(W, G, n, m, L.B, dens, L.sal_kind, mode)
        layer, _ = run_select_pack(L, W, G)
        Y0, A0 = oracle.gemm_masked(W, sel.mask, X)
        S, Ncol = L.S, L.Ncol
        ld = (Ncol + 7) // 8 * 8
        if is_conv:
            dsrc = dev(act)
        else:
            Xp = np.zeros((L.K, ld), dtype=np.uint16)
            Xp[:, :Ncol] = X
            dsrc = dev(Xp)
        ldy = ld + (8 if rng.random() < 0.5 else 0)
        for bf16 in (False, True):
            yd, tdt = (crisp.Y_BF16, torch.bfloat16) if bf16 else (crisp.Y_F32, torch.float32)
            scale, bias, res, respad = _draw_ep(rng, S, Ncol, ld, bf16)
            dscale, dbias, dres = dev(scale), dev(bias), dev(respad)
            for _ in range(2):
                cb = dict(scale=rng.random() < 0.6, bias=rng.random() < 0.6, res=rng.random() < 0.6, relu=rng.random() < 0.5)
                Yref, Aref = oracle.epilogue(Y0, A0, scale if cb["scale"] else None, bias if cb["bias"] else None,
                                             res if cb["res"] else None, cb["relu"])
                ep = crisp.epilogue(dscale if cb["scale"] else None, dbias if cb["bias"] else None,
                                    dres if cb["res"] else None, ld, cb["relu"])
                for shape in shapes:
                    Y = torch.full((S + 1, ldy), float("nan"), dtype=tdt, device="cuda")
                    if is_conv:
                        conv_spmm_ep(layer.desc, crisp.conv_desc_of(cv), layer.row_ptr, layer.col_idx, layer.vals,
                                                 layer.idx_words, dsrc, Y, ldy, yd, ep, shape=shape)
                    else:
                        spmm_ep(layer.desc, layer.row_ptr, layer.col_idx, layer.vals, layer.idx_words, dsrc, Ncol, ld,
                                            Y, ldy, yd, ep, shape=shape)
                    torch.cuda.synchronize()
                    Yh = Y.float().cpu().numpy().astype(np.float64)
                    try:
                        assert np.isnan(Yh[:S, Ncol:]).all() and np.isnan(Yh[S]).all(), "guard band written"
                        if not bf16 or S * Ncol >= 2000:
                            check_epilogue_product(Yh[:S, :Ncol], Yref, Aref, bf16, "random epilogue")
                        else:
                            # too few outputs for the Frobenius statistic of the bf16 rounding: the same launch with
                            # fp32 output and the same (bf16-representable) residual values, rounded, must give the
                            # same bits, and that fp32 result is held to the fp32 bounds
                            pad32 = np.zeros((S, ld), dtype=np.float32)
                            pad32[:, :Ncol] = res
                            dres32 = dev(pad32)
                            ep32 = crisp.epilogue(dscale if cb["scale"] else None, dbias if cb["bias"] else None,
                                                  dres32 if cb["res"] else None, ld, cb["relu"])
                            Yf = torch.full((S + 1, ldy), float("nan"), dtype=torch.float32, device="cuda")
                            if is_conv:
                                conv_spmm_ep(layer.desc, crisp.conv_desc_of(cv), layer.row_ptr, layer.col_idx, layer.vals,
                                             layer.idx_words, dsrc, Yf, ldy, crisp.Y_F32, ep32, shape=shape)
                            else:
                                spmm_ep(layer.desc, layer.row_ptr, layer.col_idx, layer.vals, layer.idx_words, dsrc, Ncol, ld,
                                        Yf, ldy, crisp.Y_F32, ep32, shape=shape)
                            torch.cuda.synchronize()
                            Y32 = Yf.cpu().numpy().astype(np.float64)[:S, :Ncol]
                            check_epilogue_product(Y32, Yref, Aref, False, "random epilogue, fp32 twin")
                            check_bf16_is_rounded_f32(Yh[:S, :Ncol], Y32, "random epilogue")
                    except AssertionError as e:
                        fails.append((what, cb, shape, bf16, str(e)[:80]))
    _report(fails)


@pytest.mark.parametrize("seed", [131])
def test_random_lowering_and_pooling(seed):
    """crisp_im2col (padded and odd row strides of X) and crisp_maxpool, bit for bit."""
    rng = np.random.default_rng(seed)
    fails = []
    case = 0
    while case < 200:
        C_, b = int(rng.integers(1, 70)), int(rng.integers(1, 6))
        kh = int(rng.choice([1, 2, 3, 3, 5, 7]))
        kw = kh if rng.random() < 0.7 else int(rng.choice([1, 2, 3, 5]))
        stride = int(rng.choice([1, 1, 2, 2, 3, 4]))
        pad = int(rng.choice([0, kh // 2, min(kh, kw) // 2]))
        H = int(rng.integers(max(kh - 2 * pad, 1), 40))
        Wd = int(rng.integers(max(kw - 2 * pad, 1), 70))
        if rng.random() < 0.4:
            Wd = (Wd + 7) // 8 * 8
        Ho, Wo = (H + 2 * pad - kh) // stride + 1, (Wd + 2 * pad - kw) // stride + 1
        if Ho < 1 or Wo < 1 or C_ * kh * kw * b * Ho * Wo > 3e7:
            continue
        what = (C_, b, H, Wd, kh, kw, stride, pad)
        print("lowering case", case, what, flush=True)
        case += 1
        act = synth.f32_to_bf16_bits(rng.standard_normal((C_, b, H, Wd)).astype(np.float32))
        cv = crisp.ConvDesc(C_, H, Wd, b, kh, kw, stride, pad, crisp.ACT_CBHW, crisp.X_KN)
        dact = dev(act)
        Xref = oracle.im2col(act, kh, kw, stride, pad)
        K, Ncol = Xref.shape
        for ldx in ((Ncol + 7) // 8 * 8, Ncol + int(rng.integers(0, 9))):
            X = torch.full((K, ldx), -1, dtype=torch.int16, device="cuda")
            crisp.crisp_im2col(cv, dact, X, ldx)
            torch.cuda.synchronize()
            Xh = host(X, np.uint16)
            if not ((Xh[:, :Ncol] == Xref).all() and (Xh[:, Ncol:] == 0xFFFF).all()):
                fails.append(("im2col", what, ldx))
        if pad < kh and pad < kw:
            ref = oracle.maxpool(act, kh, kw, stride, pad)
            out = torch.full(ref.shape, -1, dtype=torch.int16, device="cuda")
            crisp.crisp_maxpool(cv, dact, out)
            torch.cuda.synchronize()
            if not (synth.bf16_bits_to_f32(host(out, np.uint16)) == synth.bf16_bits_to_f32(ref)).all():
                fails.append(("maxpool", what))
    _report(fails)


def _draw_bag_layer(rng, i, common):
    while True:
        B = int(rng.choice([16, 32, 64, 64]))
        n, m = PATTERNS[int(rng.integers(0, len(PATTERNS)))]
        salk = int(rng.choice([synth.SAL_GRAD, synth.SAL_MAG, synth.SAL_GIVEN]))
        if rng.random() < 0.7:                 # most layers of a bag share block size, m and saliency kind: one launch group
            B, m2, salk = common
            if m2 != m:
                n, m = (min(n, m2), m2) if (min(n, m2), m2) in PATTERNS else (1, m2)
        S = int(rng.integers(1, 5 * B + 1)) if rng.random() < 0.5 else int(rng.integers(1, 7)) * B
        K = int(rng.integers(1, 30)) * B if rng.random() < 0.6 else int(rng.integers(m, 1500))
        if S * K > 600000:
            continue
        dens = float(rng.choice([0.05, 0.2, 0.35, 0.5, 0.75, 1.0]))
        mode = synth.LAYER_TOPK if rng.random() < 0.15 else 0
        return synth.LayerSpec("L%d" % i, S, K, 8, n, m, B, dens, salk, 0.05, None, mode)


@pytest.mark.parametrize("seed", [141])
def test_random_layer_bags(seed):
    """crisp_select_pack_batch over random bags of layers (several launch groups, uneven-row layers, given
    saliencies full of ties), then crisp_global_budget on the bag's block scores: all bit for bit."""
    rng = np.random.default_rng(seed)
    fails = []
    for bag in range(30):
        common = (int(rng.choice([32, 64])), int(rng.choice([4, 8])), int(rng.choice([synth.SAL_GRAD, synth.SAL_MAG])))
        cases = [_draw_bag_layer(rng, i, common) for i in range(int(rng.integers(1, 24)))]
        print("bag", bag, [(L.S, L.K, L.n, L.m, L.B, L.density, L.sal_kind, L.select_mode) for L in cases], flush=True)
        layers, Ws, TGs, expect = [], [], [], []
        for L in cases:
            r = np.random.default_rng(int(rng.integers(1, 1 << 30)))
            W, G = synth.draw_weight(r, L), None
            if L.sal_kind == synth.SAL_GRAD:
                G = synth.draw_grad(r, L)
            elif L.sal_kind == synth.SAL_GIVEN:
                G = np.abs(r.standard_normal((L.S, L.K))).astype(np.float32)
                if r.random() < 0.3:
                    G = (np.round(G * 2) / 2).astype(np.float32)       # many equal saliencies
            sel = oracle.select(W, G, L.n, L.m, L.B, L.density, L.sal_kind, L.select_mode)
            expect.append((sel,) + tuple(oracle.pack(W, sel.keep, L.n, L.m, L.B, sel.row_ptr, sel.col_idx)))
            layer = crisp.alloc_layer(desc_of(L))
            for t in (layer.nm_mask, layer.row_ptr, layer.col_idx, layer.vals, layer.idx_words, layer.flags):
                t.fill_(-1)
            layers.append(layer)
            Ws.append(dev(W))
            TGs.append(dev(G) if G is not None else None)
        crisp.crisp_select_pack_batch(*crisp.make_batch(layers, Ws, TGs))
        torch.cuda.synchronize()
        for L, layer, (sel, vals, idxw, flags) in zip(cases, layers, expect):
            sz = layer.sizes
            same = ((host(layer.nm_mask, np.uint32)[: sz.mask_words].reshape(L.S, sz.mask_words_per_row) == sel.nm_bits).all()
                    and (host(layer.score, np.float64).reshape(sz.Sb, sz.Kb).view(np.uint64) == sel.score.view(np.uint64)).all()
                    and (host(layer.row_ptr, np.int32) == sel.row_ptr).all()
                    and (host(layer.col_idx, np.int32)[: int(sel.row_ptr[-1])] == sel.col_idx).all()
                    and (host(layer.vals, np.uint16)[: vals.size] == vals.reshape(-1)).all()
                    and (host(layer.idx_words, np.uint32)[: idxw.size] == idxw.reshape(-1)).all()
                    and host(layer.flags, np.int32)[0] == flags[0])
            if not same:
                fails.append(("batch", bag, L.name))
        descs = [crisp.layer_desc(L.S, L.K, L.n, L.m, L.B, 1.0, L.sal_kind) for L in cases]
        scores_h = [e[0].score for e in expect]
        scores_d = [dev(s) for s in scores_h]
        shapes = [(L.S, L.K, L.n, L.m, L.B) for L in cases]
        ws = torch.empty(sum(s.size for s in scores_h), dtype=torch.float64, device="cuda")
        k_dev = torch.zeros(len(cases), dtype=torch.int32, device="cuda")
        ach = torch.zeros(1, dtype=torch.float64, device="cuda")
        for target in (0.0, float(rng.uniform(0.3, 0.99)), float(rng.uniform(0.5, 0.95)), 1.0):
            crisp.crisp_global_budget(descs, scores_d, target, k_dev, ach, ws, ws.numel() * 8)
            torch.cuda.synchronize()
            k_ref, a_ref = oracle.global_budget(shapes, scores_h, target)
            if k_dev.cpu().tolist() != k_ref or ach.cpu().numpy().view(np.uint64)[0] != np.array([a_ref]).view(np.uint64)[0]:
                fails.append(("budget", bag, target))
    _report(fails)
