"""Chained bf16 forward of the ResNet-50 workload (config 5): the 53 hybrid-sparse convolutions in
network order, each layer's output being the next layer's input, with the layer tails (folded
normalisation scale, shortcut, ReLU) fused into the products' epilogues and one max-pool kernel.
Call sequencing only: every arithmetic step runs in libcrisp's kernels.

Activations are channel-major [C][batch][H][W] bf16, so a product's output S x Ncol is the next
layer's activation as it stands; this needs batch*Ho*Wo to be a multiple of 8 in every layer
(batch a multiple of 8)."""
import math

from . import crisp


def layer_scales(wl, layers, device="cuda"):
    """Per-layer folded-normalisation scale (one constant per layer, as a vector of S floats):
    1/sqrt(kept fraction) keeps the activation variance of a He-initialised layer after pruning;
    the last convolution of a bottleneck gets half of that because its output is added to the
    shortcut."""
    import torch
    out = []
    for L, dl in zip(wl.layers, layers):
        rho = (L.n / L.m) * (dl.sizes.k_row / dl.sizes.Kb)
        s = 1.0 / math.sqrt(rho)
        if L.name.endswith(".c"):
            s *= 0.5
        out.append(torch.full((L.S,), s, dtype=torch.float32, device=device))
    return out


def forward(wl, layers, x, scales, x_scratch=None, record=None):
    """Runs the network on input x ([3][batch][224][224] bf16 as int16).  layers: DeviceLayers
    (already pruned and packed) in wl.layers order; scales: layer_scales(...); x_scratch: int16
    tensor large enough for the largest materialised X (crisp.conv_needs_scratch layers).
    record(name, L, inp, residual, out): called after each convolution was enqueued (tests).
    Returns the final activation [2048][batch][7][7]."""
    import torch
    idx = {L.name: i for i, L in enumerate(wl.layers)}
    dev = x.device

    def conv(name, inp, relu, residual=None):
        i = idx[name]
        L, dl, cv = wl.layers[i], layers[i], wl.layers[i].conv
        assert L.Ncol % 8 == 0, "chained forward needs batch*Ho*Wo % 8 == 0"
        out = torch.empty((L.S, L.Ncol), dtype=torch.int16, device=dev)
        ep = crisp.epilogue(scales[i], None, residual, L.Ncol, relu)
        crisp.conv_forward(dl, cv, inp, out, L.Ncol, crisp.Y_BF16, x_scratch, ep)
        if record is not None:
            record(name, L, inp, residual, out)
        return out

    y = conv("conv1", x, True)
    cv1 = wl.layers[idx["conv1"]].conv
    ho = (cv1.H + 2 * cv1.pad - cv1.kh) // cv1.stride + 1
    pool = crisp.ConvDesc(64, ho, ho, cv1.batch, 3, 3, 2, 1, crisp.ACT_CBHW, crisp.X_KN)
    hp = (ho + 2 - 3) // 2 + 1
    cur = torch.empty((64, cv1.batch * hp * hp), dtype=torch.int16, device=dev)
    crisp.crisp_maxpool(pool, y, cur)
    if record is not None:
        record("maxpool", pool, y, None, cur)
    for si, blocks in enumerate((3, 4, 6, 3)):
        for bi in range(blocks):
            pre = "s%db%d" % (si + 1, bi)
            a = conv(pre + ".a", cur, True)
            b = conv(pre + ".b", a, True)
            shortcut = conv(pre + ".ds", cur, False) if bi == 0 else cur
            cur = conv(pre + ".c", b, True, residual=shortcut)
    return cur
