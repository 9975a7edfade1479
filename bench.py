#!/usr/bin/env python3
"""Benchmark of the CRISP hybrid-sparse hot path on one MI355X.

A step is one pass of the whole path over one batch of synthetic input: selection and packing of
every layer of the workload on the device (saliency, N:M choice, block scores, block choice,
packing), then for every layer the lowering (fused, none, or crisp_im2col) and the product.  Inputs
are resident in HBM before the timed region.

Default workload: config 5, the 53 convolutions of ResNet-50 at batch 256 (the largest
configuration; one layer's inputs and outputs alone exceed the last-level cache, and a pass touches
17 GB, so every launch finds its inputs in HBM).  The one JSON line carries
  value / ms_per_step   useful (non-zero weight) TFLOP/s of the whole step, timed over --steps passes;
  roofline              the product kernel with the largest share of the step: algorithmic bytes per
                        launch / its average launch duration from HIP event pairs recorded around
                        its launches inside the timed steps;
  cpu_baseline          the CPU oracle timed on the host cores on a bounded sample of the workload;
  layers                per-layer time, useful TFLOP/s, fraction of the HBM / MFMA bound;
  configs               one row per benchmark configuration 1..5 (1..4 measured after the timed
                        region by short runs of their own; --no-config-table skips them).
`--config 1..4` makes one of the small configurations the workload of the line instead.
"""
from __future__ import annotations

import argparse
import hashlib
import json
import os
import sys
import time

import numpy as np

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0           # MI355X HBM3E
MFMA_BF16_PEAK_TFLOPS = 2500.0  # MI355X dense bf16
METRIC = "effective TFLOP/s (nonzero FLOPs) of hybrid-sparse GEMM + % roofline"


def parse():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=0, help="timed steps (default: 30 for config 5, 200 for 1..4)")
    ap.add_argument("--warmup", type=int, default=0, help="untimed steps before (default: 3 for config 5, 20 for 1..4)")
    ap.add_argument("--config", type=int, default=5,
                    help="workload 1..5 (default 5: all 53 ResNet-50 convs at batch 256, the largest configuration)")
    ap.add_argument("--sets", type=int, default=0, help="configs 1..4: independent input sets to rotate through (0 = enough for 600 MB)")
    ap.add_argument("--y-dtype", choices=["bf16", "f32"], default="bf16")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-config-table", action="store_true", help="skip the short runs of the other configurations")
    ap.add_argument("--spmm-only", action="store_true", help="configs 1..4: time only the products (selection and packing done once)")
    ap.add_argument("--chained", action="store_true",
                    help="config 5: time the chained bf16 forward (epilogues fused, max-pool) instead of layer-wise products")
    ap.add_argument("--per-layer-prune", action="store_true",
                    help="select+pack layer by layer (crisp_select_pack) instead of one crisp_select_pack_batch call")
    ap.add_argument("--explicit-im2col", action="store_true",
                    help="configs 1..4: materialise X with crisp_im2col for conv layers instead of the fused crisp_conv_spmm")
    ap.add_argument("--sweep", action="store_true",
                    help="block size x N:M sweep of the paper (B in 16/32/64, N in 1/2/3 of 4) on the layers of "
                         "the chosen workload: product time per setting, one JSON line")
    ap.add_argument("--layer", default=None,
                    help="only the product of this layer of the chosen workload (e.g. --config 5 --layer s4b0.a), launched "
                         "--steps times over rotating inputs that do not fit the last-level cache: isolated cold launches "
                         "for profiler counters")
    ap.add_argument("--topk", action="store_true",
                    help="--layer mode: plain block pruning over the whole grid (CRISP_LAYER_TOPK) instead of uniform rows")
    ap.add_argument("--row-skew", type=float, default=0.0,
                    help="--layer mode: saliency |W| scaled per block-row by skew^(-row), handed in as CRISP_SAL_GIVEN, so that "
                         "whole-grid block pruning leaves block-rows of very different length (e.g. 1.6)")
    ap.add_argument("--shape", type=int, default=None,
                    help="--layer mode, plain products: force this launch shape (crisp_spmm_forced) instead of the library's choice")
    ap.add_argument("--two-of-four", action="store_true",
                    help="--layer mode, 4:8 layers: weights whose kept values fall two per aligned four (magnitude saliency), and the "
                         "product told so (CRISP_HINT_TWO_OF_FOUR) once the pack's flag has been read back as 1")
    ap.add_argument("--copy-calibration", action="store_true",
                    help="also run a plain 512 MiB device copy a few times (known traffic, for scaling profiler counters)")
    return ap.parse_args()


# HBM bytes per launch of dominant kernels from rocprofv3 --pmc runs (FETCH_SIZE and WRITE_SIZE, each scaled by what the
# same counter reads for an elementwise pass of known size): key = (workload, kernel id as this script prints it),
# value = (bytes per launch, file under profiles/ that holds the counter rows).  A kernel without an entry reports null.
TRAFFIC = {
    # (the two kernels whose shares of the step are within a few percent of each other; whichever the warm-up passes find)
    ("c5", "reg 4:8 B64 shape1 conv0 dense-mfma"): (187773965, "profiles/bench_c5_kernels.txt"),
    ("c5", "reg 2:8 B64 shape0 conv0 sparse-mfma"): (int((2.0 * 57488.4 + 122931.2) * 1024), "profiles/bench_c5_kernels.txt"),
    # configs 1-4 as the workload of the line: bytes = (2.0 * FETCH_SIZE + 1.0 * WRITE_SIZE) KiB of the dominant layer's kernel
    ("c1", "reg 2:4 B32 shape2 conv0 sparse-mfma"): (int((2.0 * 4231.0 + 1568.0) * 1024), "profiles/bench_c1_kernels.txt"),
    ("c2", "reg 1:4 B64 shape1 conv0 sparse-mfma"): (int((2.0 * 1762.6 + 12544.0) * 1024), "profiles/bench_c2_kernels.txt"),
    ("c3", "lds 2:8 B64 shape2 conv0 sparse-mfma"): (int((2.0 * 215499.0 + 50176.0) * 1024), "profiles/bench_c3_kernels.txt"),
    ("c4", "reg 2:4 B32 shape1 conv0 sparse-mfma"): (int((2.0 * 37684.9 + 18816.0) * 1024), "profiles/bench_c4_kernels.txt"),
}


# ------------------------------------------------------------------------------------------------
# bookkeeping shared by all workloads
# ------------------------------------------------------------------------------------------------
def kernel_id(code: int, L) -> str:
    """Readable name of the kernel instantiation a product launch ran (from the library's report)."""
    from paper_2311_14272_amd import crisp
    f = crisp.kernel_code_fields(code)
    # (the LDS-resident family with dense tiles, the generic and the 16 x 16 families are one compiled kernel for
    # every pattern)
    one_for_all = f["family"] in ("generic", "b16") or (f["family"] == "lds" and not f["sparse_mfma"])
    pattern = "any n:m" if one_for_all else "%d:%d" % (L.n, L.m)
    return "%s %s B%d shape%d conv%d %s" % (f["family"], pattern, L.B, f["shape"], f["conv_mode"],
                                             "sparse-mfma" if f["sparse_mfma"] else "dense-mfma")


def mask_stats(L, dl):
    """Kept weights, block columns in use and packed bytes of a pruned layer, from the device output."""
    sz = dl.sizes
    row_ptr = dl.row_ptr.cpu().numpy()
    col_idx = dl.col_idx.cpu().numpy()[: sz.nk]
    if L.S % L.B == 0 and L.K % L.B == 0 and L.K % L.m == 0:
        ones = sz.nk * L.B * sz.slots_per_row
    else:                                   # ragged layer: count from the device mask
        bits = dl.nm_mask.cpu().numpy().view(np.uint32)[: sz.mask_words].reshape(L.S, sz.mask_words_per_row)
        keep = np.unpackbits(bits.view(np.uint8), axis=1, bitorder="little")[:, : L.K]
        ones = sum(int(keep[bi * L.B:(bi + 1) * L.B, bj * L.B:(bj + 1) * L.B].sum())
                   for bi in range(sz.Sb) for bj in col_idx[row_ptr[bi]:row_ptr[bi + 1]])
    used_cols = np.unique(col_idx)
    kept_vals = sz.nk * L.B * sz.slots_per_row
    w_bytes = kept_vals * 2 + sz.idx_words * 4 + sz.nk * 4 + (sz.Sb + 1) * 4
    return ones, used_cols, w_bytes, kept_vals


def algorithmic_bytes(L, used_cols, w_bytes, ybytes):
    """Bytes a launch has to move: the activations the kept blocks need (rows of X of block columns kept by
    at least one block-row; for a real convolution the input elements those rows come from, each once),
    the output, the packed weights."""
    cv = L.conv
    lowered = cv is not None and (cv.kh > 1 or cv.kw > 1 or cv.stride > 1)
    if lowered:
        chans = set()
        for bj in used_cols:
            for k in range(int(bj) * L.B, min(L.K, (int(bj) + 1) * L.B)):
                chans.add(k % cv.C)
        rows = cv.H if cv.kh >= cv.stride else min(cv.H, cv.Ho * cv.kh)
        cols = cv.W if cv.kw >= cv.stride else min(cv.W, cv.Wo * cv.kw)
        x_bytes = 2 * len(chans) * cv.batch * rows * cols
    else:
        k_used = int(sum(min(L.K, (int(bj) + 1) * L.B) - int(bj) * L.B for bj in used_cols))
        x_bytes = 2 * k_used * L.Ncol
    return x_bytes + ybytes * L.S * L.Ncol + w_bytes


def useful_ceiling(L) -> float:
    """Upper limit of useful / dense-peak matrix-core throughput of the execution path: the sparse
    matrix-core instruction (patterns with at most two kept per group) skips half of the zeros, dense
    expansion multiplies all of them."""
    return min(1.0, (2.0 if L.n <= 2 else 1.0) * L.n / L.m)


def bound_ms(alg_bytes, useful_flop, L):
    t_hbm = alg_bytes / (HBM_PEAK_GBS * 1e9) * 1e3
    t_mfma = useful_flop / (useful_ceiling(L) * MFMA_BF16_PEAK_TFLOPS * 1e12) * 1e3
    return t_hbm, t_mfma


def layer_row(L, st, ms, ybytes):
    t_hbm, t_mfma = bound_ms(st["alg_bytes"], st["useful_flop"], L)
    return dict(st, forward_ms=round(ms, 5), useful_tflops_forward=round(st["useful_flop"] / (ms * 1e-3) / 1e12, 2),
                hbm_frac=round(t_hbm / ms, 4), mfma_frac_useful=round(st["useful_flop"] / (ms * 1e-3) / 1e12 / MFMA_BF16_PEAK_TFLOPS, 4),
                bound="hbm" if t_hbm >= t_mfma else "mfma", bound_frac=round(max(t_hbm, t_mfma) / ms, 4))


# ------------------------------------------------------------------------------------------------
# config 5: ResNet-50, all 53 convolutions, batch 256
# ------------------------------------------------------------------------------------------------
def run_resnet50(args):
    import torch
    from paper_2311_14272_amd import crisp, synth
    dev = "cuda"
    steps = args.steps or 30
    warmup = args.warmup or 3
    wl = synth.config(5)
    y_dtype = crisp.Y_BF16 if args.y_dtype == "bf16" else crisp.Y_F32
    ybytes = 2 if y_dtype == crisp.Y_BF16 else 4
    ytorch = torch.bfloat16 if y_dtype == crisp.Y_BF16 else torch.float32
    gen = torch.Generator(device=dev)
    gen.manual_seed(wl.seed)
    nl = len(wl.layers)

    # weights, gradients and pack buffers of all 53 layers stay resident; the model is pruned in one
    # crisp_select_pack_batch call per step, as Alg. 1 prunes all layers in one shot
    Wd, Gd, dls, digests = [], [], [], {}
    for li, L in enumerate(wl.layers):
        t = synth.draw_layer(wl, li, with_x=False)
        for key in ("W", "G"):
            digests["%s.%s" % (L.name, key)] = hashlib.sha256(np.ascontiguousarray(t[key]).view(np.uint8)).hexdigest()[:16]
        Wd.append(torch.from_numpy(t["W"].view(np.int16)).to(dev))
        Gd.append(torch.from_numpy(t["G"]).to(dev))
        dls.append(crisp.alloc_layer(crisp.layer_desc(L.S, L.K, L.n, L.m, L.B, L.density, L.sal_kind, L.select_mode), dev))
    batch = crisp.make_batch(dls, Wd, Gd)

    def prune_all():
        if args.per_layer_prune:
            for i in range(nl):
                crisp.prune_and_pack(dls[i], Wd[i], Gd[i])
        else:
            crisp.crisp_select_pack_batch(*batch)

    if args.chained:
        return run_resnet50_chained(args, wl, dls, prune_all, gen, steps, warmup)

    # every layer's own input (ReLU(N(0,1)) of its true shape) and output stay resident: 17 GB per pass,
    # so a layer's input is long gone from the 256 MB last-level cache when the next step reads it again
    acts, Ys = [], []
    need_x = 1
    for L in wl.layers:
        cv = L.conv
        acts.append(torch.randn((cv.C, cv.batch, cv.H, cv.W), generator=gen, device=dev).clamp_(min=0).to(torch.bfloat16).view(torch.int16))
        Ys.append(torch.empty((L.S, L.Ncol), dtype=ytorch, device=dev))
        if crisp.conv_needs_scratch(cv, L.B, L.n, L.m, L.S, L.density):
            need_x = max(need_x, L.K * ((L.Ncol + 7) // 8 * 8))
    Xs = torch.empty(need_x, dtype=torch.int16, device=dev)
    convs = [crisp.conv_desc_of(L.conv) for L in wl.layers]

    def forward(i):
        return crisp.conv_forward(dls[i], wl.layers[i].conv, acts[i], Ys[i], wl.layers[i].Ncol, y_dtype, Xs)

    def forward_timed(i, ev_start, ev_stop):
        """The launches of crisp_conv_forward for layer i, the product through crisp_spmm_timed: the two events
        receive the product kernel's own start and stop (an event pair recorded around the call would also
        hold the dispatch gaps next to the launch, about 3 us here)."""
        L, d = wl.layers[i], dls[i]
        if paths[i] == "fused":
            crisp.crisp_spmm_timed(d.desc, convs[i], d.row_ptr, d.col_idx, d.vals, d.idx_words, acts[i], L.Ncol, L.Ncol, Ys[i], L.Ncol,
                                   y_dtype, ev_start, ev_stop)
            return
        X, ldx = acts[i], L.Ncol
        if paths[i] == "im2col":
            ldx = (L.Ncol + 7) // 8 * 8
            crisp.crisp_im2col(convs[i], acts[i], Xs, ldx)
            X = Xs
        crisp.crisp_spmm_timed(d.desc, None, d.row_ptr, d.col_idx, d.vals, d.idx_words, X, L.Ncol, ldx, Ys[i], L.Ncol, y_dtype,
                               ev_start, ev_stop)

    def step(pairs=None, kernel_events=None):
        prune_all()
        for i in range(nl):
            if kernel_events is not None and i in kernel_events:
                forward_timed(i, *kernel_events[i])
            elif pairs is not None and i in pairs:
                pairs[i][0].record()
                forward(i)
                pairs[i][1].record()
            else:
                forward(i)

    # ---- one untimed pass: masks (for the FLOP and byte counts) and which kernel each layer runs ----
    prune_all()
    torch.cuda.synchronize()
    stats, kids, paths = [], [], []
    for i, L in enumerate(wl.layers):
        ones, used_cols, w_bytes, _ = mask_stats(L, dls[i])
        uf = 2.0 * ones * L.Ncol
        stats.append(dict(name=L.name, S=L.S, K=L.K, Ncol=L.Ncol, nm="%d:%d" % (L.n, L.m), B=L.B, density=round(L.density, 3),
                          k_row=dls[i].sizes.k_row, useful_flop=uf, dense_flop=2.0 * L.S * L.K * L.Ncol,
                          alg_bytes=algorithmic_bytes(L, used_cols, w_bytes, ybytes)))
        path = crisp.conv_plan(dls[i].desc, L.conv)[0]
        d = dls[i]
        if path == "fused":
            code = crisp.crisp_conv_spmm_forced(d.desc, convs[i], d.row_ptr, d.col_idx, d.vals, d.idx_words, acts[i], Ys[i], L.Ncol, y_dtype)
        else:
            X, ldx = acts[i], L.Ncol
            if path == "im2col":
                ldx = (L.Ncol + 7) // 8 * 8
                crisp.crisp_im2col(convs[i], acts[i], Xs, ldx)
                X = Xs
            code = crisp.crisp_spmm_forced(d.desc, d.row_ptr, d.col_idx, d.vals, d.idx_words, X, L.Ncol, ldx, Ys[i], L.Ncol, y_dtype)
        kids.append(kernel_id(code, L))
        paths.append(path)
    torch.cuda.synchronize()
    useful = sum(s["useful_flop"] for s in stats)
    dense = sum(s["dense_flop"] for s in stats)
    if args.copy_calibration:
        copy_calibration()

    def event_pairs(idx):
        return {i: (torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)) for i in idx}

    # ---- warm-up with every layer bracketed: finds the kernel with the largest share of the step ----
    wsum = np.zeros(nl)
    for _ in range(warmup):
        pairs = event_pairs(range(nl))
        step(pairs)
        torch.cuda.synchronize()
        wsum += np.array([pairs[i][0].elapsed_time(pairs[i][1]) for i in range(nl)])
    share = {}
    for i in range(nl):
        # (a bracket around a materialised layer also holds the lowering pass: its share is scaled by the product's part)
        w = wsum[i] * (0.55 if paths[i] == "im2col" else 1.0)
        share[kids[i]] = share.get(kids[i], 0.0) + w
    dom_kid = max(share, key=share.get)
    dom_layers = [i for i in range(nl) if kids[i] == dom_kid]

    # ---- timed region: exactly `steps` passes; the dominant kernel's launches carry HIP events that receive
    # the kernel's own start and stop on the launch stream -------------------------------------------------
    hev = crisp.HipEvents(steps * len(dom_layers))
    kev = [{i: hev.pairs[k * len(dom_layers) + j] for j, i in enumerate(dom_layers)} for k in range(steps)]
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for k in range(steps):
        step(None, kev[k])
    torch.cuda.synchronize()
    ms_per_step = (time.perf_counter() - t0) * 1e3 / steps
    dom_ms = np.array([[hev.elapsed_ms(k * len(dom_layers) + j) for j in range(len(dom_layers))] for k in range(steps)])   # steps x launches
    dom_avg_ms = float(dom_ms.mean())
    dom_bytes = float(np.mean([stats[i]["alg_bytes"] for i in dom_layers]))
    achieved = dom_bytes / (dom_avg_ms * 1e-3) / 1e9

    # ---- breakdown (untimed extras): a few more passes with every launch bracketed --------------------
    reps = max(1, min(steps, 5))
    fsum, isum, psum = np.zeros(nl), np.zeros(nl), 0.0
    for _ in range(reps):
        pa, pb = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        pa.record()
        prune_all()
        pb.record()
        pairs, ipairs = event_pairs(range(nl)), event_pairs([i for i in range(nl) if paths[i] == "im2col"])
        for i, L in enumerate(wl.layers):
            if paths[i] == "im2col":          # the two launches crisp_conv_forward makes, bracketed one by one
                ldx = (L.Ncol + 7) // 8 * 8
                d = dls[i]
                ipairs[i][0].record()
                crisp.crisp_im2col(convs[i], acts[i], Xs, ldx)
                ipairs[i][1].record()
                pairs[i][0].record()
                crisp.crisp_spmm(d.desc, d.row_ptr, d.col_idx, d.vals, d.idx_words, Xs, L.Ncol, ldx, Ys[i], L.Ncol, y_dtype)
                pairs[i][1].record()
            else:
                pairs[i][0].record()
                forward(i)
                pairs[i][1].record()
        torch.cuda.synchronize()
        psum += pa.elapsed_time(pb)
        fsum += np.array([pairs[i][0].elapsed_time(pairs[i][1]) for i in range(nl)])
        for i in ipairs:
            isum[i] += ipairs[i][0].elapsed_time(ipairs[i][1])
    rows = []
    for i, L in enumerate(wl.layers):
        r = layer_row(L, stats[i], (fsum[i] + isum[i]) / reps, ybytes)
        r.update(lowering=paths[i], kernel=kids[i], im2col_ms=round(isum[i] / reps, 5))
        rows.append(r)
    t_fwd = float((fsum.sum() + isum.sum()) / reps)
    t_bound = sum(max(bound_ms(s["alg_bytes"], s["useful_flop"], L)) for s, L in zip(stats, wl.layers))
    t_hbm_all = sum(s["alg_bytes"] for s in stats) / (HBM_PEAK_GBS * 1e9) * 1e3
    traffic = TRAFFIC.get(("c5", dom_kid))
    out = {"metric": METRIC, "value": round(useful / (ms_per_step * 1e-3) / 1e12, 3), "unit": "TFLOP/s", "n_gpus": 1,
           "steps": steps, "warmup": warmup, "ms_per_step": round(ms_per_step, 4), "higher_is_better": True, "scaling": "weak",
           "vs_baseline": None, "dtype": "bf16", "data": "synthetic",
           "config": {"workload": "c5: ResNet-50, 53 convs as GEMMs, batch 256, 224x224, layer-wise inputs (every layer reads its own "
                                  "ReLU(N(0,1)) input of its true shape), B=64, per-layer n:m and block density drawn from the workload seed",
                      "step": ("select+pack layer by layer (crisp_select_pack)" if args.per_layer_prune else
                               "select+pack of all layers in one crisp_select_pack_batch call") +
                              "; then per layer crisp_conv_forward: lowering (fused, im2col or none) and product",
                      "y_dtype": args.y_dtype, "x_layout": "KN", "resident_input_sets": 1,
                      "bytes_touched_per_step": int(sum(s["alg_bytes"] for s in stats))},
           "dense_equivalent_tflops": round(dense / (ms_per_step * 1e-3) / 1e12, 1),
           "roofline": {"bound": "hbm", "achieved": round(achieved, 1), "peak": HBM_PEAK_GBS, "unit": "GB/s",
                        "frac": round(achieved / HBM_PEAK_GBS, 4), "traffic": traffic[0] if traffic else None,
                        "traffic_source": traffic[1] if traffic else None,
                        "kernel": dom_kid, "launches_per_step": len(dom_layers), "layers": [wl.layers[i].name for i in dom_layers],
                        "share_of_step": round(float(dom_ms.sum(axis=1).mean()) / ms_per_step, 4),
                        "avg_launch_ms": round(dom_avg_ms, 5), "median_launch_ms": round(float(np.median(dom_ms)), 5),
                        "algorithmic_bytes_per_launch": int(dom_bytes),
                        "timing": "HIP events on the launch stream that receive the kernel's own start and stop "
                                  "(hipExtLaunchKernelGGL), every launch of this kernel in every timed step; nothing subtracted",
                        "mfma_frac_useful": round(sum(stats[i]["useful_flop"] for i in dom_layers) / len(dom_layers) /
                                                  (dom_avg_ms * 1e-3) / 1e12 / MFMA_BF16_PEAK_TFLOPS, 4)},
           "roofline_all_layers": {"hbm_frac_forward": round(t_hbm_all / t_fwd, 4), "bound_frac_forward": round(t_bound / t_fwd, 4),
                                   "note": "sum over layers of max(algorithmic bytes / 8 TB/s, useful FLOP / (path ceiling x 2.5 PFLOP/s)) "
                                           "over the summed bracketed launch times of the breakdown passes"},
           "select_pack_ms": round(psum / reps, 4), "forward_ms": round(t_fwd, 4), "im2col_ms": round(float(isum.sum() / reps), 4),
           "useful_tflops_forward_only": round(useful / (t_fwd * 1e-3) / 1e12, 2),
           "dense_equivalent_tflops_forward_only": round(dense / (t_fwd * 1e-3) / 1e12, 1),
           "layers": rows,
           "inputs": {"generator": "numpy %s PCG64, seed %d (weights, gradients); torch.Generator(cuda) seed %d (activations)"
                                   % (np.__version__, wl.seed, wl.seed), "sha256_prefix": digests}}
    del acts, Ys, Xs
    torch.cuda.empty_cache()
    return out, useful


def run_resnet50_chained(args, wl, dls, prune_all, gen, steps, warmup):
    """The network as a chain: every layer's bf16 output is the next layer's input, layer tails (folded-
    normalisation scale, shortcut, ReLU) fused into the products, one max-pool kernel."""
    import torch
    from paper_2311_14272_amd import crisp, resnet
    dev = "cuda"
    prune_all()
    scales = resnet.layer_scales(wl, dls)
    need = max([L.K * L.Ncol for L in wl.layers if crisp.conv_needs_scratch(L.conv, L.B, L.n, L.m, L.S, L.density)] + [1])
    xs = torch.empty(need, dtype=torch.int16, device=dev)
    cv1 = wl.layers[0].conv
    x = torch.randn((3, cv1.batch, 224, 224), generator=gen, device=dev).to(torch.bfloat16).view(torch.int16)
    for _ in range(warmup):
        prune_all()
        resnet.forward(wl, dls, x, scales, xs)
    torch.cuda.synchronize()
    a, b, c = (torch.cuda.Event(enable_timing=True) for _ in range(3))
    t_prune = t_chain = 0.0
    t0 = time.perf_counter()
    for _ in range(steps):
        a.record()
        prune_all()
        b.record()
        resnet.forward(wl, dls, x, scales, xs)
        c.record()
        torch.cuda.synchronize()
        t_prune += a.elapsed_time(b)
        t_chain += b.elapsed_time(c)
    total = (time.perf_counter() - t0) * 1e3 / steps
    t_prune /= steps
    t_chain /= steps
    useful = dense = 0.0
    for L, dl in zip(wl.layers, dls):
        useful += 2.0 * mask_stats(L, dl)[0] * L.Ncol
        dense += 2.0 * L.S * L.K * L.Ncol
    out = {"metric": METRIC, "value": round(useful / (total * 1e-3) / 1e12, 3), "unit": "TFLOP/s", "n_gpus": 1, "steps": steps,
           "warmup": warmup, "ms_per_step": round(total, 3), "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
           "dtype": "bf16", "data": "synthetic",
           "config": {"workload": "c5: ResNet-50, 53 convs as GEMMs, batch 256, 224x224, chained bf16 forward "
                                  "(scale / shortcut / ReLU epilogues, max-pool), B=64, per-layer n:m and block "
                                  "density drawn from the workload seed",
                      "step": "select+pack of all layers, then the chained forward (one synchronisation per step)", "y_dtype": "bf16"},
           "select_pack_ms": round(t_prune, 3), "forward_ms": round(t_chain, 3),
           "dense_equivalent_tflops_forward_only": round(dense / (t_chain * 1e-3) / 1e12, 1), "roofline": None}
    return out, useful


def cpu_baseline_resnet50(useful_flop_full):
    """The CPU oracle as it stands on a bounded sample of config 5: selection and packing of all 53 layers at
    full size, lowering and the dense masked fp64 product at a small batch (1/256 .. 32/256 of the columns of
    every layer), the product part scaled to batch 256."""
    import oracle
    from paper_2311_14272_amd import synth
    full = synth.config(5)
    sels, t_sel = [], 0.0
    for li, L in enumerate(full.layers):
        t = synth.draw_layer(full, li, with_x=False)
        t0 = time.perf_counter()
        sel = oracle.select(t["W"], t["G"], L.n, L.m, L.B, L.density, L.sal_kind, L.select_mode)
        oracle.pack(t["W"], sel.keep, L.n, L.m, L.B, sel.row_ptr, sel.col_idx)
        t_sel += time.perf_counter() - t0
        sels.append((t["W"], sel.mask))

    def products(b):
        wl = synth.config(5, batch=b)
        dt = 0.0
        for li, L in enumerate(wl.layers):
            cv = L.conv
            act = synth.draw_relu_normal(synth.layer_rng(wl, li), (cv.C, cv.batch, cv.H, cv.W))
            t0 = time.perf_counter()
            X = oracle.im2col(act, cv.kh, cv.kw, cv.stride, cv.pad)
            oracle.gemm_masked(sels[li][0], sels[li][1], X, want_abs=False)
            dt += time.perf_counter() - t0
        return dt

    t1 = products(1)
    b = int(max(1, min(32, 12.0 // max(t1, 1e-3))))
    tb = products(b) if b > 1 else t1
    dt = t_sel + tb * 256.0 / b
    return {"value": round(useful_flop_full / dt / 1e12, 6), "unit": "TFLOP/s", "cores": oracle.num_threads(), "kind": "oracle",
            "seconds_scaled_to_full_workload": round(dt, 1), "cpu_seconds_spent": round(t_sel + t1 + (tb if b > 1 else 0.0), 1),
            "sample": "select+pack of all 53 layers at full size (%.2f s) + lowering and dense masked fp64 product of every "
                      "layer at batch %d (%.2f s), the product part scaled by 256/%d" % (t_sel, b, tb, b)}


# ------------------------------------------------------------------------------------------------
# configs 1..4: single layers and the three-layer bottleneck
# ------------------------------------------------------------------------------------------------
class LayerState:
    pass


def run_small(cid, args, steps, warmup, want_cpu):
    import torch
    from paper_2311_14272_amd import crisp, synth
    dev = "cuda"
    wl = synth.config(cid)
    y_dtype = crisp.Y_BF16 if args.y_dtype == "bf16" else crisp.Y_F32
    ybytes = 2 if y_dtype == crisp.Y_BF16 else 4
    ytorch = torch.bfloat16 if y_dtype == crisp.Y_BF16 else torch.float32

    def to_dev(a):
        a = np.ascontiguousarray(a)
        if a.dtype == np.uint16:
            a = a.view(np.int16)
        return torch.from_numpy(a).to(dev)

    host_inputs = [synth.draw_layer(wl, i) for i in range(len(wl.layers))]
    per_set = 0
    for L in wl.layers:
        is_conv = L.conv is not None and (L.conv.kh > 1 or L.conv.kw > 1 or L.conv.stride > 1)
        per_set += ybytes * L.S * L.Ncol
        if is_conv:
            per_set += 2 * L.conv.C * L.conv.batch * L.conv.H * L.conv.W
        if not is_conv or args.explicit_im2col:
            per_set += 2 * L.K * L.Ncol
    # enough independent input sets that a rotation exceeds the 256 MB last-level cache more than twice
    nsets = args.sets if args.sets > 0 else max(2, min(80, int(600e6 // per_set) + 1))
    gen = torch.Generator(device=dev)
    gen.manual_seed(wl.seed)
    layers = []
    for i, L in enumerate(wl.layers):
        st = LayerState()
        st.L = L
        st.desc = crisp.layer_desc(L.S, L.K, L.n, L.m, L.B, L.density, L.sal_kind, L.select_mode)
        st.dl = crisp.alloc_layer(st.desc, dev)
        st.W = to_dev(host_inputs[i]["W"])
        st.G = to_dev(host_inputs[i]["G"]) if host_inputs[i]["G"] is not None else None
        cv = L.conv
        st.is_conv = cv is not None and (cv.kh > 1 or cv.kw > 1 or cv.stride > 1)
        st.conv = crisp.conv_desc_of(cv) if st.is_conv else None
        st.fused = False
        if st.is_conv and not args.explicit_im2col:
            Wo = cv.W + 2 * cv.pad - cv.kw + 1
            st.fused = (cv.stride == 1 and cv.C % L.B == 0 and Wo % 2 == 0 and L.B in (32, 64))
        st.act, st.X, st.Y = [], [], []
        for s in range(nsets):
            if st.is_conv:
                a = to_dev(host_inputs[i]["act"]) if s == 0 else \
                    torch.randn((cv.C, cv.batch, cv.H, cv.W), generator=gen, device=dev).clamp_(min=0).to(torch.bfloat16).view(torch.int16)
                st.act.append(a)
                st.X.append(None if st.fused else torch.empty((L.K, L.Ncol), dtype=torch.int16, device=dev))
            else:
                x = to_dev(host_inputs[i]["X"]) if s == 0 else \
                    torch.randn((L.K, L.Ncol), generator=gen, device=dev).clamp_(min=0).to(torch.bfloat16).view(torch.int16)
                st.X.append(x)
            st.Y.append(torch.empty((L.S, L.Ncol), dtype=ytorch, device=dev))
        layers.append(st)

    def prune(st):
        crisp.prune_and_pack(st.dl, st.W, st.G)

    def product(st, s, want_code=False):
        L, d = st.L, st.dl
        if want_code:
            if st.fused:
                return crisp.crisp_conv_spmm_forced(st.desc, st.conv, d.row_ptr, d.col_idx, d.vals, d.idx_words, st.act[s], st.Y[s], L.Ncol, y_dtype)
            return crisp.crisp_spmm_forced(st.desc, d.row_ptr, d.col_idx, d.vals, d.idx_words, st.X[s], L.Ncol, L.Ncol, st.Y[s], L.Ncol, y_dtype)
        if st.fused:
            crisp.crisp_conv_spmm(st.desc, st.conv, d.row_ptr, d.col_idx, d.vals, d.idx_words, st.act[s], st.Y[s], L.Ncol, y_dtype)
        else:
            crisp.crisp_spmm(st.desc, d.row_ptr, d.col_idx, d.vals, d.idx_words, st.X[s], L.Ncol, L.Ncol, st.Y[s], L.Ncol, y_dtype)

    def forward(st, s, events=None):
        if st.is_conv and not st.fused:
            crisp.crisp_im2col(st.conv, st.act[s], st.X[s], st.L.Ncol)
        if events is not None:
            events[0].record()
        product(st, s)
        if events is not None:
            events[1].record()

    batch = crisp.make_batch([st.dl for st in layers], [st.W for st in layers], [st.G for st in layers])

    def step(k, dom=None, events=None):
        s = k % nsets
        # all layers are pruned in one call (the method prunes a model in one shot), then the products
        if not args.spmm_only and not args.per_layer_prune:
            crisp.crisp_select_pack_batch(*batch)
        for i, st in enumerate(layers):
            if not args.spmm_only and args.per_layer_prune:
                prune(st)
            forward(st, s, events if i == dom else None)

    # ---- one untimed pass to learn the mask statistics (metric bookkeeping, from device output) ----
    for st in layers:
        prune(st)
    torch.cuda.synchronize()
    info = []
    for st in layers:
        L, sz = st.L, st.dl.sizes
        ones, used_cols, w_bytes, kept_vals = mask_stats(L, st.dl)
        if st.is_conv and not st.fused:     # materialised X is what the product reads
            k_used = int(sum(min(L.K, (int(bj) + 1) * L.B) - int(bj) * L.B for bj in used_cols))
            alg_bytes = 2 * k_used * L.Ncol + ybytes * L.S * L.Ncol + w_bytes
        else:
            alg_bytes = algorithmic_bytes(L, used_cols, w_bytes, ybytes)
        # metadata of the packed form next to the closed forms of Sec. 3.1 (K' = k_row*B kept columns per row)
        Kp = sz.k_row * L.B
        meta = dict(paper_block_bits=L.S * Kp * int(np.floor(np.log2(max(Kp / L.B, 1)))) // (L.B * L.B),
                    paper_nm_bits=L.S * Kp * L.n * sz.idx_bits // L.m,
                    stored_block_bytes=int(sz.nk * 4 + (sz.Sb + 1) * 4), stored_nm_bytes=int(sz.idx_words * 4),
                    packed_value_bytes=int(kept_vals * 2), dense_bytes=int(L.S * L.K * 2))
        code = product(st, 0, want_code=True)
        info.append(dict(name=L.name, S=L.S, K=L.K, Ncol=L.Ncol, metadata=meta, nm="%d:%d" % (L.n, L.m), B=L.B, k_row=sz.k_row,
                         ones=ones, useful_flop=2.0 * ones * L.Ncol, dense_flop=2.0 * L.S * L.K * L.Ncol,
                         alg_bytes=alg_bytes, smfmac_ok=int(st.dl.flags.cpu()[0]), kernel=kernel_id(code, L),
                         lowering=("fused" if st.fused else ("im2col" if st.is_conv else "none"))))
    useful = sum(x["useful_flop"] for x in info)
    dense_eq = sum(x["dense_flop"] for x in info)
    dom = int(np.argmax([x["alg_bytes"] for x in info]))   # dominant kernel: the product with the most traffic

    if args.copy_calibration:
        copy_calibration()

    # ---- warm-up, then the timed region ----------------------------------------------------
    for k in range(warmup):
        step(k)
    torch.cuda.synchronize()
    ev = [(torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)) for _ in range(steps)]
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for k in range(steps):
        step(warmup + k, dom, ev[k])
    torch.cuda.synchronize()
    ms_per_step = (time.perf_counter() - t0) * 1e3 / steps
    # the bracket as the events give it: it also holds the dispatch gaps next to the launch (about 3 us
    # on this machine against the kernel trace), which matters for kernels of a few microseconds
    dom_raw = [a.elapsed_time(b) for a, b in ev]
    dom_ms = float(np.mean(dom_raw))

    # ---- per-phase breakdown (untimed extras): back-to-back launches over the rotating input sets ----
    def timed(fn, reps=50):
        torch.cuda.synchronize()
        a, b = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        a.record()
        for r in range(reps):
            fn(r)
        b.record()
        torch.cuda.synchronize()
        return a.elapsed_time(b) / reps

    for i, st in enumerate(layers):
        info[i]["prune_pack_ms"] = round(timed(lambda r, st=st: prune(st)), 5)
        ms = timed(lambda r, st=st: forward(st, r % nsets))
        info[i] = layer_row(st.L, info[i], ms, ybytes)

    achieved = info[dom]["alg_bytes"] / (dom_ms * 1e-3) / 1e9
    traffic = TRAFFIC.get((wl.name, info[dom]["kernel"]))
    out = {
        "metric": METRIC, "value": round(useful / (ms_per_step * 1e-3) / 1e12, 4), "unit": "TFLOP/s", "n_gpus": 1,
        "steps": steps, "warmup": warmup, "ms_per_step": round(ms_per_step, 5), "higher_is_better": True, "scaling": "weak",
        "vs_baseline": None, "dtype": "bf16", "data": "synthetic",
        "config": {"workload": "%s: %s" % (wl.name, ", ".join("%s %dx%dx%d %s B%d k_row %d" % (
            x["name"], x["S"], x["K"], x["Ncol"], x["nm"], x["B"], x["k_row"]) for x in info)),
                   "step": (("select+pack of all layers (crisp_select_pack_batch), then " if not args.per_layer_prune else "select+pack (crisp_select_pack)+") if not args.spmm_only else "") + ("im2col+spmm" if args.explicit_im2col else "spmm with the 3x3 layer's lowering fused (crisp_conv_spmm)") + " per layer",
                   "y_dtype": args.y_dtype, "x_layout": "KN", "input_sets": nsets},
        "dense_equivalent_tflops": round(dense_eq / (ms_per_step * 1e-3) / 1e12, 3),
        "roofline": {"bound": "hbm", "achieved": round(achieved, 2), "peak": HBM_PEAK_GBS, "unit": "GB/s",
                     "frac": round(achieved / HBM_PEAK_GBS, 4), "traffic": traffic[0] if traffic else None,
                     "traffic_source": traffic[1] if traffic else None,
                     "kernel": "%s (layer %s)" % (info[dom]["kernel"], info[dom]["name"]),
                     "avg_launch_ms": round(dom_ms, 5), "median_launch_ms": round(float(np.median(dom_raw)), 5),
                     "timing": "HIP event pair around the launch in every timed step (raw bracket, nothing subtracted)",
                     "algorithmic_bytes": info[dom]["alg_bytes"],
                     "forward_ms_back_to_back": info[dom]["forward_ms"]},
        "layers": info,
    }
    digests = {}
    for h, x in zip(host_inputs, info):
        for key in ("W", "G", "X", "act"):
            if h.get(key) is not None:
                digests["%s.%s" % (x["name"], key)] = hashlib.sha256(np.ascontiguousarray(h[key]).view(np.uint8)).hexdigest()[:16]
    out["inputs"] = {"generator": "numpy %s PCG64, seed %d" % (np.__version__, wl.seed), "sha256_prefix": digests}
    if want_cpu:
        out["cpu_baseline"] = cpu_baseline_small(wl, host_inputs, useful, 10.0 if want_cpu == "full" else 2.5)
    del layers, host_inputs
    torch.cuda.empty_cache()
    return out


def cpu_baseline_small(wl, host_inputs, useful_flop, budget_s):
    """The CPU oracle as it stands, timed on the host cores on the same workload: whole passes are
    repeated until about budget_s seconds of CPU work have been spent, and the mean pass is reported."""
    import oracle

    def one_pass():
        t0 = time.perf_counter()
        for i, L in enumerate(wl.layers):
            h = host_inputs[i]
            sel = oracle.select(h["W"], h["G"], L.n, L.m, L.B, L.density, L.sal_kind, L.select_mode)
            oracle.pack(h["W"], sel.keep, L.n, L.m, L.B, sel.row_ptr, sel.col_idx)
            X = h["X"]
            if X is None:
                cv = L.conv
                X = oracle.im2col(h["act"], cv.kh, cv.kw, cv.stride, cv.pad)
            frac = 1.0
            ncols = X.shape[1]
            budget = 2e9 * budget_s / 10.0    # multiply-adds per layer that keep one pass within the budget
            if L.S * L.K * ncols > budget:
                ncols = max(64, int(budget // (L.S * L.K)))
                frac = ncols / X.shape[1]
            tg = time.perf_counter()
            oracle.gemm_masked(h["W"], sel.mask, X, 0, ncols, want_abs=False)
            tg = time.perf_counter() - tg
            t0 -= tg * (1.0 / frac - 1.0)    # scale the sampled columns to the full width
        return time.perf_counter() - t0

    wall0 = time.perf_counter()
    passes = [one_pass()]
    while time.perf_counter() - wall0 < budget_s and len(passes) < 64:
        passes.append(one_pass())
    dt = sum(passes) / len(passes)
    return {"value": round(useful_flop / dt / 1e12, 6), "unit": "TFLOP/s", "cores": oracle.num_threads(), "kind": "oracle",
            "seconds": round(dt, 3), "passes": len(passes), "cpu_seconds_spent": round(time.perf_counter() - wall0, 1),
            "sample": "mean of %d passes of the full workload (select, pack, im2col, dense masked fp64 product); "
                      "products above %.1e multiply-adds are timed on their first columns and scaled" % (len(passes), 2e9 * budget_s / 10.0)}


def copy_calibration():
    """A plain elementwise pass of known traffic (reads 512 MiB, writes 512 MiB) whose profiler counters
    give the scale of FETCH_SIZE / WRITE_SIZE on this machine."""
    import torch
    a = torch.ones(128 << 20, dtype=torch.float32, device="cuda")
    b = torch.empty_like(a)
    for _ in range(5):
        torch.add(a, 1.0, out=b)
    torch.cuda.synchronize()
    del a, b


def run_layer(args):
    """One layer of a workload on its own: select+pack once, then only its product (with its lowering), --steps
    launches back to back over rotating inputs (more than 600 MB in total), for profiler counters on cold launches."""
    import torch
    from paper_2311_14272_amd import crisp, synth
    dev = "cuda"
    wl = synth.config(args.config)
    names = [L.name for L in wl.layers]
    if args.layer not in names:
        print("bench.py: workload c%d has no layer %r (layers: %s)" % (args.config, args.layer, " ".join(names)), file=sys.stderr)
        sys.exit(2)
    li = names.index(args.layer)
    L = wl.layers[li]
    y_dtype = crisp.Y_BF16 if args.y_dtype == "bf16" else crisp.Y_F32
    ybytes = 2 if y_dtype == crisp.Y_BF16 else 4
    ytorch = torch.bfloat16 if y_dtype == crisp.Y_BF16 else torch.float32
    steps = args.steps or 40
    t = synth.draw_layer(wl, li, with_x=False)
    sal_kind, TG = L.sal_kind, t["G"]
    if args.row_skew > 0.0:
        # input generation only: a saliency tensor whose block-rows differ in scale
        Sb = (L.S + L.B - 1) // L.B
        scale = np.repeat(np.float32(args.row_skew) ** -np.arange(Sb, dtype=np.float32), L.B)[: L.S, None]
        TG = (np.abs(synth.bf16_bits_to_f32(t["W"])) * scale).astype(np.float32)
        sal_kind = crisp.SAL_GIVEN
    if args.two_of_four:
        if (L.n, L.m) != (4, 8) or args.row_skew > 0.0:
            print("bench.py: --two-of-four applies to 4:8 layers (without --row-skew)", file=sys.stderr)
            sys.exit(2)
        t["W"] = synth.draw_two_per_quad_weight(np.random.Generator(np.random.PCG64([wl.seed, li])), L.S, L.K)
        sal_kind, TG = crisp.SAL_MAG, None
    desc = crisp.layer_desc(L.S, L.K, L.n, L.m, L.B, L.density, sal_kind, crisp.LAYER_TOPK if args.topk else L.select_mode)
    dl = crisp.alloc_layer(desc, dev)
    W = torch.from_numpy(t["W"].view(np.int16)).to(dev)
    G = torch.from_numpy(TG).to(dev) if TG is not None else None
    crisp.prune_and_pack(dl, W, G)
    if args.two_of_four:
        if int(dl.flags.cpu()[0]) != 1:
            print("bench.py: the pack did not report the 2-of-4 property", file=sys.stderr)
            sys.exit(1)
        desc = crisp.layer_desc(L.S, L.K, L.n, L.m, L.B, L.density, sal_kind, crisp.LAYER_TOPK if args.topk else L.select_mode,
                                hints=crisp.HINT_TWO_OF_FOUR)
        dl.desc = desc
    cv = L.conv if L.conv is not None else synth.ConvShape(L.K, 1, L.Ncol, 1, 1, 1, 1, 0)    # a plain product as a 1x1 layer
    in_elems = cv.C * cv.batch * cv.H * cv.W
    nbuf = max(2, min(16, int(600e6 // (2 * in_elems + ybytes * L.S * L.Ncol)) + 1))
    gen = torch.Generator(device=dev)
    gen.manual_seed(wl.seed)
    acts = [torch.randn((cv.C, cv.batch, cv.H, cv.W), generator=gen, device=dev).clamp_(min=0).to(torch.bfloat16).view(torch.int16)
            for _ in range(nbuf)]
    Ys = [torch.empty((L.S, L.Ncol), dtype=ytorch, device=dev) for _ in range(nbuf)]
    Xs = torch.empty(L.K * ((L.Ncol + 7) // 8 * 8), dtype=torch.int16, device=dev) \
        if crisp.conv_needs_scratch(cv, L.B, L.n, L.m, L.S, L.density) else None
    if args.copy_calibration:
        copy_calibration()
    ones, used_cols, w_bytes, _ = mask_stats(L, dl)
    code = [0]

    def launch(r):
        if args.shape is None:
            return crisp.conv_forward(dl, cv, acts[r % nbuf], Ys[r % nbuf], L.Ncol, y_dtype, Xs)
        code[0] = crisp.crisp_spmm_forced(desc, dl.row_ptr, dl.col_idx, dl.vals, dl.idx_words, acts[r % nbuf], L.Ncol, L.Ncol,
                                          Ys[r % nbuf], L.Ncol, y_dtype, None, args.shape)
        return "none"
    if args.shape is not None and (cv.kh > 1 or cv.kw > 1 or cv.stride > 1):
        print("bench.py: --shape applies to plain products (1x1, stride 1) only", file=sys.stderr)
        sys.exit(2)
    for r in range(3):
        path = launch(r)
    torch.cuda.synchronize()
    a, b = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    a.record()
    for r in range(steps):
        launch(r)
    b.record()
    torch.cuda.synchronize()
    ms = a.elapsed_time(b) / steps
    st = dict(name=L.name, S=L.S, K=L.K, Ncol=L.Ncol, nm="%d:%d" % (L.n, L.m), B=L.B, k_row=dl.sizes.k_row,
              useful_flop=2.0 * ones * L.Ncol, dense_flop=2.0 * L.S * L.K * L.Ncol,
              alg_bytes=algorithmic_bytes(L, used_cols, w_bytes, ybytes), lowering=path, launches=steps, input_sets=nbuf,
              blocks_per_row=np.diff(dl.row_ptr.cpu().numpy()).tolist()[:64],
              kernel=kernel_id(code[0], L) if args.shape is not None else None)
    print(json.dumps({"layer_only": layer_row(L, st, ms, ybytes), "workload": wl.name,
                      "timing": "launches back to back between one event pair, rotating inputs"}))


def config_row(cid, out):
    """One row of the per-configuration table from a run's output."""
    hb = out.get("roofline") or {}
    row = {"config": "c%d" % cid, "ms_per_step": out["ms_per_step"], "useful_tflops": out["value"],
           "dense_equivalent_tflops": out["dense_equivalent_tflops"],
           "useful_tflops_forward_only": out.get("useful_tflops_forward_only"),
           "hbm_frac_dominant_kernel": hb.get("frac"), "dominant_kernel": hb.get("kernel"),
           "layers": [{k: r.get(k) for k in ("name", "kernel", "forward_ms", "useful_tflops_forward", "hbm_frac", "mfma_frac_useful",
                                             "bound", "bound_frac")} for r in out.get("layers", [])]}
    if cid != 5:
        fw = sum(r["forward_ms"] for r in out["layers"])
        row["useful_tflops_forward_only"] = round(sum(r["useful_flop"] for r in out["layers"]) / (fw * 1e-3) / 1e12, 2)
    cb = out.get("cpu_baseline")
    if cb:
        row["oracle_seconds"] = cb.get("seconds", cb.get("seconds_scaled_to_full_workload"))
        row["oracle_cores"] = cb["cores"]
        row["oracle_tflops"] = cb["value"]
    return row


def block_sweep(args):
    """The paper's hardware sweep (Sec. 4.2: N in {1,2,3} of 4, block sizes 16/32/64) on the
    shapes of the chosen workload at equal block density: time of the product alone."""
    import torch
    from paper_2311_14272_amd import crisp, synth
    dev = "cuda"
    wl = synth.config(args.config)
    y_dtype = crisp.Y_BF16 if args.y_dtype == "bf16" else crisp.Y_F32
    ytorch = torch.bfloat16 if y_dtype == crisp.Y_BF16 else torch.float32
    gen = torch.Generator(device=dev)
    gen.manual_seed(wl.seed)
    rows = []
    for li, L in enumerate(wl.layers):
        t = synth.draw_layer(wl, li, with_x=False)
        W = torch.from_numpy(t["W"].view(np.int16)).to(dev)
        nsets = max(2, min(8, int(600e6 // (2 * L.K * L.Ncol + 2 * L.S * L.Ncol)) + 1))
        Xs = [torch.randn((L.K, L.Ncol), generator=gen, device=dev).clamp_(min=0).to(torch.bfloat16).view(torch.int16)
              for _ in range(nsets)]
        Ys = [torch.empty((L.S, L.Ncol), dtype=ytorch, device=dev) for _ in range(nsets)]
        for B in (16, 32, 64):
            for n in (1, 2, 3):
                desc = crisp.layer_desc(L.S, L.K, n, 4, B, L.density, crisp.SAL_MAG)
                dl = crisp.alloc_layer(desc, dev)
                crisp.prune_and_pack(dl, W, None)

                def run(r):
                    crisp.crisp_spmm(desc, dl.row_ptr, dl.col_idx, dl.vals, dl.idx_words, Xs[r % nsets], L.Ncol, L.Ncol,
                                     Ys[r % nsets], L.Ncol, y_dtype)
                for r in range(3):
                    run(r)
                torch.cuda.synchronize()
                a, b = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
                reps = 30
                a.record()
                for r in range(reps):
                    run(r)
                b.record()
                torch.cuda.synchronize()
                us = a.elapsed_time(b) * 1e3 / reps
                sz = dl.sizes
                kept = sz.nk * B * sz.slots_per_row
                rows.append(dict(layer=L.name, B=B, nm="%d:4" % n, k_row=sz.k_row, us=round(us, 2),
                                 useful_tflops=round(2.0 * kept * L.Ncol / us / 1e6, 2),
                                 metadata_bytes=int(sz.idx_words * 4 + sz.nk * 4 + (sz.Sb + 1) * 4),
                                 value_bytes=int(kept * 2)))
        del Xs, Ys
        torch.cuda.empty_cache()
    print(json.dumps({"sweep": "block size x N:M at the workload's block density, product only (back-to-back launches, "
                               "rotating input sets)", "workload": wl.name, "y_dtype": args.y_dtype, "rows": rows}))


def main():
    args = parse()
    if args.gpus != 1:
        print("bench.py: this build runs on one GPU only (no collectives, no sharding); use --gpus 1", file=sys.stderr)
        sys.exit(2)
    import torch
    from paper_2311_14272_amd import crisp

    if not torch.cuda.is_available():
        print("bench.py: no GPU visible; the HIP path has no CPU fallback", file=sys.stderr)
        sys.exit(2)
    crisp.lib()
    if args.sweep:
        block_sweep(args)
        return
    if args.layer:
        run_layer(args)
        return
    want_cpu = not args.no_cpu_baseline
    if args.config != 5:
        out = run_small(args.config, args, args.steps or 200, args.warmup or 20, "full" if want_cpu else None)
        print(json.dumps(out))
        return
    out, useful = run_resnet50(args)
    if want_cpu and not args.chained:
        out["cpu_baseline"] = cpu_baseline_resnet50(useful)
    if not args.no_config_table and not args.chained:
        # the other configurations, by short runs of their own after the timed region (same process)
        table = []
        for cid in (1, 2, 3, 4):
            table.append(config_row(cid, run_small(cid, args, 100, 10, "short" if want_cpu else None)))
        table.append(config_row(5, out))
        out["configs"] = table
    print(json.dumps(out))


if __name__ == "__main__":
    main()
