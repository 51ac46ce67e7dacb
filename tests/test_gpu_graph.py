"""A whole layer-set step captured in a HIP graph: the library's calls enqueue kernels only (no allocation once the
workspace has its size, no memset, no synchronisation), so a step can be recorded once on the context's stream and
replayed.  Every replay is compared bit for bit with the same calls issued eagerly, with eager work and
synchronisations between the replays."""
import numpy as np
import pytest
import torch

from paper_2601_17261_amd import binding, synth

pytestmark = pytest.mark.gpu

EPS = float(np.float32(1e-3))
LR = float(np.float32(1e-3))


def layer_set(n_tokens, shapes, seed):
    inputs, out = {}, []
    for i, (name, d_in, d_out) in enumerate(shapes):
        key = (d_in, name in ("q", "k", "v"), name in ("gate", "up"))
        if key not in inputs:
            x = torch.randn(n_tokens, d_in, device="cuda", generator=torch.Generator(device="cuda").manual_seed(seed + i))
            inputs[key] = (x / x.pow(2).mean(dim=1, keepdim=True).sqrt()).to(torch.bfloat16)
        X = inputs[key]
        W, T = synth.device_weights_and_target(seed + 100 + i, X, d_out)
        out.append((W, X, T))
    return out


def test_captured_step_replays_bit_identically():
    r, K = 8, 3
    stream = torch.cuda.Stream()
    ctx = binding.Context(stream=stream)
    layers = layer_set(512, synth.QWEN3_0P6B_LAYER, 5)
    descs = [(binding.make_layer(W, X, r), W, X, binding.make_loss(T)) for W, X, T in layers]
    bases = [torch.empty(W.shape[1], r, dtype=torch.float32, device="cuda") for W, _, _ in layers]
    out = torch.zeros(len(layers), 4, dtype=torch.float64, device="cuda")

    def step():
        for li, (L, W, X, loss) in enumerate(descs):
            ctx.step_no_update(L, W, X, loss, K, EPS, 40 + li, 0, out[li], bases[li])
        ctx.update_many([(W, bases[li], 40 + li, LR, out[li, 3:4]) for li, (_, W, _, _) in enumerate(descs)])

    W0 = [W.clone() for W, _, _ in layers]
    torch.cuda.synchronize()
    # eager reference: three steps in a row (the seed is part of the recorded arguments, so every replay repeats it)
    ref = []
    with torch.cuda.stream(stream):
        for _ in range(3):
            step()
            stream.synchronize()
            ref.append(([W.clone() for W, _, _ in layers], out.clone()))
        ctx.check()
        for (W, _, _), w0 in zip(layers, W0):
            W.copy_(w0)
        stream.synchronize()
        graph = torch.cuda.CUDAGraph()
        with torch.cuda.graph(graph, stream=stream):
            step()
    torch.cuda.synchronize()
    for (W, _, _), w0 in zip(layers, W0):
        assert torch.equal(W, w0)                      # recording runs nothing
    for k in range(3):
        graph.replay()
        torch.cuda.synchronize()
        Wk, outk = ref[k]
        assert torch.equal(out, outk), k
        for (W, _, _), w in zip(layers, Wk):
            assert torch.equal(W, w), k
        # eager work of the program's own between the replays
        scratch = torch.empty(1 << 20, device="cuda").normal_()
        assert torch.isfinite(scratch.sum()).item()
        torch.cuda.synchronize()
    with torch.cuda.stream(stream):
        ctx.check()
    ctx.close()
