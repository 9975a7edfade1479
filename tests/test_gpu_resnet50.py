"""Config 5: all 53 ResNet-50 convolutions as hybrid-sparse GEMMs with on-device select+pack.
Layer-wise mode: every layer gets a fresh ReLU(N(0,1)) input of its true shape (drawn on the
device), and the oracle is fed exactly that input (teacher forcing), so errors do not compound.
Batch 2: every output column is checked.  Batch 256: masks and packing in full, the product on
sampled columns (each output column is an independent sum over K)."""
import numpy as np
import pytest
import torch

import oracle
from paper_2311_14272_amd import crisp, synth

from gpu_util import check_product, desc_of, dev, host, lowering_gather_index, run_select_pack

pytestmark = pytest.mark.gpu


def _device_activation(shape, gen):
    a = torch.randn(shape, generator=gen, device="cuda", dtype=torch.float32).clamp_(min=0).to(torch.bfloat16)
    return a.view(torch.int16)


def _run_layers(batch, sample_cols):
    wl = synth.config(5, batch=batch)
    assert len(wl.layers) == 53
    gen = torch.Generator(device="cuda")
    gen.manual_seed(wl.seed)
    paths = {"none": 0, "fused": 0, "im2col": 0}
    for li, L in enumerate(wl.layers):
        cv = L.conv
        t = synth.draw_layer(wl, li, with_x=False)
        W, G = t["W"], t["G"]
        sel = oracle.select(W, G, L.n, L.m, L.B, L.density, L.sal_kind, L.select_mode)
        vals, idxw, flags = oracle.pack(W, sel.keep, L.n, L.m, L.B, sel.row_ptr, sel.col_idx)
        layer, out = run_select_pack(L, W, G)
        assert (out["nm_bits"] == sel.nm_bits).all() and (out["col_idx"] == sel.col_idx).all(), L.name
        assert (out["score"].view(np.uint64) == sel.score.view(np.uint64)).all(), L.name
        assert (out["vals"] == vals).all() and (out["idxw"] == idxw).all() and out["flags"][0] == flags[0], L.name
        dact = _device_activation((cv.C, cv.batch, cv.H, cv.W), gen)
        Ncol = L.Ncol
        ld = (Ncol + 7) // 8 * 8
        Y = torch.empty((L.S, ld), dtype=torch.float32, device="cuda")
        need_x = crisp.conv_needs_scratch(cv, L.B, L.n, L.m, L.S, L.density)
        Xs = torch.zeros((L.K, ld), dtype=torch.int16, device="cuda") if need_x else None
        path = crisp.conv_forward(layer, cv, dact, Y, ld, crisp.Y_F32, Xs)
        torch.cuda.synchronize()
        paths[path] += 1
        rng = np.random.default_rng(1000 + li)
        if sample_cols is None or Ncol <= sample_cols:
            cols = np.arange(Ncol)
        else:
            cols = np.unique(np.concatenate([np.arange(64), np.arange(Ncol - 64, Ncol),
                                             rng.integers(0, Ncol, sample_cols)]))
        idx, inside = lowering_gather_index(cv.C, cv.H, cv.W, cv.batch, cv.kh, cv.kw, cv.stride, cv.pad, cols)
        g = torch.take(dact.view(-1), torch.from_numpy(idx).cuda()).cpu().numpy().view(np.uint16)
        Xs_host = np.ascontiguousarray(np.where(inside, g, np.uint16(0)))
        Yref, Aref = oracle.gemm_masked(W, sel.mask, Xs_host)
        Yg = Y[:, torch.from_numpy(cols).cuda()].cpu().numpy().astype(np.float64)
        check_product(Yg, Yref, Aref, crisp.Y_F32, "%s (%s)" % (L.name, path))
        del dact, Y, Xs, layer
        torch.cuda.empty_cache()
        print("layer %2d %-8s %4dx%4dx%7d %d:%d d=%.2f path=%s ok" % (li, L.name, L.S, L.K, Ncol, L.n, L.m, L.density, path),
              flush=True)
    return paths


def test_resnet50_batch2_all_columns():
    paths = _run_layers(2, None)
    assert paths["fused"] >= 10 and sum(paths.values()) == 53


def test_resnet50_batch256_sampled_columns():
    paths = _run_layers(256, 384)
    assert sum(paths.values()) == 53


def _bf16_check(Y, Yref, Aref, what):
    """bf16 outputs with added terms: the stated 2e-3 in the Frobenius norm; element-wise the product's
    1e-2 |W|.|X| (scaled) plus the final rounding, unit roundoff 2^-8, of a value within that of Y*."""
    assert np.isfinite(Y).all(), what
    err = np.abs(Y - Yref)
    fro = np.linalg.norm(Y - Yref) / max(np.linalg.norm(Yref), 1e-300)
    assert fro <= 2e-3, (what, fro)
    bound = 1e-2 * Aref + 2.0 ** -8 * (np.abs(Yref) + 1e-2 * Aref) + 1e-30
    assert (err <= bound).all(), (what, float((err - bound).max()))


def test_resnet50_chained_forward_batch8():
    """The chained bf16 forward (epilogues fused, max-pool, shortcuts) with teacher forcing: every
    layer's actual device input (and shortcut) is handed to the oracle, which must reproduce that
    layer's device output; all columns for small layers, sampled columns for the large ones."""
    from paper_2311_14272_amd import resnet
    wl = synth.config(5, batch=8)
    layers, Ws, Gs, sels = [], [], [], []
    for li, L in enumerate(wl.layers):
        t = synth.draw_layer(wl, li, with_x=False)
        sels.append((t["W"], oracle.select(t["W"], t["G"], L.n, L.m, L.B, L.density, L.sal_kind, L.select_mode)))
        layers.append(crisp.alloc_layer(desc_of(L)))
        Ws.append(dev(t["W"]))
        Gs.append(dev(t["G"]))
    crisp.crisp_select_pack_batch(*crisp.make_batch(layers, Ws, Gs))
    scales = resnet.layer_scales(wl, layers)
    need = max([L.K * L.Ncol for L in wl.layers if crisp.conv_needs_scratch(L.conv, L.B, L.n, L.m, L.S, L.density)] + [1])
    xs = torch.empty(need, dtype=torch.int16, device="cuda")
    gen = torch.Generator(device="cuda")
    gen.manual_seed(wl.seed)
    x = torch.randn((3, 8, 224, 224), generator=gen, device="cuda").to(torch.bfloat16).view(torch.int16)
    seen = []

    def record(name, L, inp, residual, out):
        torch.cuda.synchronize()
        if name == "maxpool":
            got = host(out, np.uint16).reshape(L.C, L.batch, 56, 56)
            ref = oracle.maxpool(host(inp, np.uint16).reshape(L.C, L.batch, L.H, L.W), 3, 3, 2, 1)
            assert (synth.bf16_bits_to_f32(got) == synth.bf16_bits_to_f32(ref)).all(), "maxpool"
            seen.append(name)
            return
        li = [l.name for l in wl.layers].index(name)
        W, sel = sels[li]
        cv = L.conv
        rng = np.random.default_rng(2000 + li)
        cols = np.arange(L.Ncol) if L.S * L.K * L.Ncol <= 3e9 else np.unique(rng.integers(0, L.Ncol, 512))
        idx, inside = lowering_gather_index(cv.C, cv.H, cv.W, cv.batch, cv.kh, cv.kw, cv.stride, cv.pad, cols)
        g = torch.take(inp.view(-1), torch.from_numpy(idx).cuda()).cpu().numpy().view(np.uint16)
        X = np.ascontiguousarray(np.where(inside, g, np.uint16(0)))
        Y0, A0 = oracle.gemm_masked(W, sel.mask, X)
        tcols = torch.from_numpy(cols).cuda()
        res = None
        if residual is not None:
            res = synth.bf16_bits_to_f32(residual.view(L.S, L.Ncol)[:, tcols].cpu().numpy().view(np.uint16)).astype(np.float64)
        scale = scales[li].cpu().numpy()
        relu = not name.endswith(".ds")
        Yref, Aref = oracle.epilogue(Y0, A0, scale, None, res, relu)
        Yg = synth.bf16_bits_to_f32(out.view(L.S, L.Ncol)[:, tcols].cpu().numpy().view(np.uint16)).astype(np.float64)
        _bf16_check(Yg, Yref, Aref, name)
        seen.append(name)
        print("chained %-8s ok (%d columns)" % (name, len(cols)), flush=True)

    out = resnet.forward(wl, layers, x, scales, xs, record)
    torch.cuda.synchronize()
    assert len(seen) == 54 and out.shape == (2048, 8 * 7 * 7)
    final = synth.bf16_bits_to_f32(host(out, np.uint16))
    assert np.isfinite(final).all() and (final >= 0).all() and final.max() > 0


def test_resnet50_global_budget():
    """One overall sparsity target for the whole network (Alg. 1 lines 6-9): block scores of all 53 layers
    from the device, kept blocks per row and reached sparsity equal to the oracle's, bit for bit."""
    wl = synth.config(5, batch=8)
    layers, Ws, Gs, shapes, scores_h = [], [], [], [], []
    for li, L in enumerate(wl.layers):
        t = synth.draw_layer(wl, li, with_x=False)
        sel = oracle.select(t["W"], t["G"], L.n, L.m, L.B, 1.0, L.sal_kind)
        scores_h.append(sel.score)
        shapes.append((L.S, L.K, L.n, L.m, L.B))
        layers.append(crisp.alloc_layer(crisp.layer_desc(L.S, L.K, L.n, L.m, L.B, 1.0, L.sal_kind)))
        Ws.append(dev(t["W"]))
        Gs.append(dev(t["G"]))
    crisp.crisp_select_pack_batch(*crisp.make_batch(layers, Ws, Gs))
    torch.cuda.synchronize()
    for layer, sc in zip(layers, scores_h):
        assert (host(layer.score, np.float64).reshape(sc.shape).view(np.uint64) == sc.view(np.uint64)).all()
    ws = torch.empty(sum(s.size for s in scores_h), dtype=torch.float64, device="cuda")
    k_dev = torch.zeros(len(layers), dtype=torch.int32, device="cuda")
    ach = torch.zeros(1, dtype=torch.float64, device="cuda")
    for target in (0.75, 0.9, 0.95):
        crisp.crisp_global_budget([l.desc for l in layers], [l.score for l in layers], target, k_dev, ach, ws, ws.numel() * 8)
        torch.cuda.synchronize()
        k_ref, a_ref = oracle.global_budget(shapes, scores_h, target)
        assert k_dev.cpu().tolist() == k_ref, target
        assert ach.cpu().numpy().view(np.uint64)[0] == np.array([a_ref]).view(np.uint64)[0], target
        assert a_ref >= target and min(k_ref) >= 1
        print("target %.2f: reached %.4f, kept blocks per row %s ..." % (target, a_ref, k_ref[:8]), flush=True)
