"""The entry points under HIP graph capture: they only enqueue kernels (no allocation, no
synchronisation, no memory-clearing calls), so a captured step must replay to the same bytes as the
eager step, also on later replays with other work in between."""
import numpy as np
import pytest
import torch

from paper_2311_14272_amd import crisp, synth

from gpu_util import desc_of, dev

pytestmark = pytest.mark.gpu

CASES = [synth.small_cases()[i] for i in (0, 2, 7)]


@pytest.mark.parametrize("L", CASES, ids=lambda L: L.name)
def test_captured_step_replays_like_eager(L):
    print("case", L.name, flush=True)
    W, G, X = synth.draw_small(L, 31)
    ldx = (L.Ncol + 7) // 8 * 8
    Xp = np.zeros((L.K, ldx), dtype=np.uint16)
    Xp[:, : L.Ncol] = X
    dW, dX = dev(W), dev(Xp)
    dG = dev(G) if G is not None else None
    layer = crisp.alloc_layer(desc_of(L))
    Y = torch.zeros((L.S, ldx), dtype=torch.float32, device="cuda")
    outputs = (layer.nm_mask, layer.row_ptr, layer.col_idx, layer.vals, layer.idx_words, layer.flags, Y)

    def step():
        crisp.prune_and_pack(layer, dW, dG)
        crisp.crisp_spmm(layer.desc, layer.row_ptr, layer.col_idx, layer.vals, layer.idx_words, dX, L.Ncol, ldx, Y, ldx,
                         crisp.Y_F32)

    step()
    torch.cuda.synchronize()
    eager = [t.clone() for t in outputs]
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph):
        step()
    other = torch.randn(1 << 16, device="cuda")
    for replay in range(4):
        for t in outputs:
            t.fill_(-1)                       # a replay must rewrite everything it owns
        graph.replay()
        torch.cuda.synchronize()
        for name, t, e in zip(("nm_mask", "row_ptr", "col_idx", "vals", "idx_words", "flags", "Y"), outputs, eager):
            sz = layer.sizes
            n = {"nm_mask": sz.mask_words, "col_idx": sz.nk, "vals": sz.vals_elems, "idx_words": sz.idx_words}.get(name)
            a, b = (t.view(-1)[:n], e.view(-1)[:n]) if n is not None else (t, e)
            if name == "Y":
                a, b = t[:, : L.Ncol], e[:, : L.Ncol]
            if name == "flags":
                a, b = t[:1], e[:1]
            assert torch.equal(a, b), (name, replay)
        other = other * 1.0001 + 1.0          # eager work and a synchronisation between the replays
        step()
        torch.cuda.synchronize()
