"""The hot call inside a captured HIP graph: zm_decode_experts allocates nothing and passes everything as kernel
arguments, so a serving loop may record a model's layer calls once and replay them.  Every replay is compared
with the eager result and with the original tensors, with the program's own eager work between the replays."""
import numpy as np
import pytest

from oracle import oracle as zo
from paper_2601_21198_amd import synth, zipmoe as zm

pytestmark = pytest.mark.gpu


@pytest.mark.parametrize("stores", [zm.STORES_AUTO, zm.STORES_STREAMING])
def test_layer_calls_replayed_from_a_graph(stores):
    import torch
    wl = synth.CFG2
    n_experts, top_k, n_layers = 4, 2, 3
    # small experts of the config-2 kind: three matrices each, lengths that are no multiple of a stream
    originals, layers = [], []
    for layer_no in range(n_layers):
        tensors = [[m.ravel()[: 150_000 + 4099 * (layer_no + e) + 7 * i].copy()
                    for i, m in enumerate(synth.expert_tensors(wl, layer_no, e))] for e in range(n_experts)]
        blobs = [[zm.compress(w, wl.chunk_values, 4096)[0] for w in ts] for ts in tensors]
        originals.append(tensors)
        layers.append(zm.ExpertLayer(blobs))
    routed = [[(layer_no + 1) % n_experts, (layer_no + 3) % n_experts] for layer_no in range(n_layers)]
    assert all(len(set(r)) == top_k for r in routed)

    side = torch.cuda.Stream()
    outs, calls = [], []
    for layer_no, layer in enumerate(layers):
        # every expert of these layers has its own lengths: one buffer set per routed expert
        bufs, starts_of = [], []
        for e in routed[layer_no]:
            b, starts, _ = layer.alloc_outputs(1, expert=e)
            bufs.append(b[0])
            starts_of.append(starts)
        outs.append((bufs, starts_of))
        # one call per routed expert: the per-expert starts differ
        for j, e in enumerate(routed[layer_no]):
            calls.append(layer.make_call([e], [bufs[j]], starts_of[j], stores))

    def clear():
        for bufs, _ in outs:
            for b in bufs:
                b.zero_()

    def check(what):
        for layer_no in range(n_layers):
            bufs, starts_of = outs[layer_no]
            for j, e in enumerate(routed[layer_no]):
                got = bufs[j].cpu().numpy().view(np.uint16)
                for i, w in enumerate(originals[layer_no][e]):
                    s = starts_of[j][i]
                    assert np.array_equal(got[s: s + w.size], w), f"{what}: layer {layer_no} expert {e} tensor {i}"

    # eager, on the side stream
    with torch.cuda.stream(side):
        clear()
        for c in calls:
            c(side.cuda_stream)
    torch.cuda.synchronize()
    check("eager")
    # one expert against the reference decoder as well
    e0 = routed[0][0]
    ref = zo.decode(zm.compress(originals[0][e0][1], wl.chunk_values, 4096)[0])
    assert np.array_equal(ref, originals[0][e0][1])

    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph, stream=side):
        for c in calls:
            c(torch.cuda.current_stream().cuda_stream)
    torch.cuda.synchronize()
    for replay in range(4):
        clear()                                    # eager work between the replays
        torch.cuda.synchronize()
        check_zero = all(int(b.abs().max()) == 0 for bufs, _ in outs for b in bufs)
        assert check_zero
        graph.replay()
        torch.cuda.synchronize()
        check(f"replay {replay}")
