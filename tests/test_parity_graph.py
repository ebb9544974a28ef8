"""The hot calls allocate nothing, never synchronise and record no memset, so a
caller may capture a whole layer step into a HIP graph.  Captured and replayed
several times (with eager work and synchronisations in between), the step must
give bit-for-bit what the eager calls give."""
import numpy as np
import pytest
import torch

from paper_2502_06643_amd import synth
from paper_2502_06643_amd.layer import MoELayer, to_device

pytestmark = pytest.mark.gpu


@pytest.mark.parametrize("T,d,f,E,k,G,local", [(64, 256, 512, 8, 2, 1, -1),      # decode-sized: streaming FFN kernels, fused index kernel
                                               (1500, 256, 320, 8, 2, 4, 1)])    # tiled GEMMs, tile height chosen on the device, split tail
def test_layer_step_replays_from_a_graph(lib, T, d, f, E, k, G, local):
    rng = np.random.default_rng(T)
    x = to_device(synth.normal(T, 0, (T, d), 1.0, "bf16"))
    lg = torch.from_numpy(rng.standard_normal((T, E)).astype(np.float32)).cuda()
    w1 = synth.normal(T, 2, (E, d, f), d ** -0.5, "bf16")
    w3 = synth.normal(T, 3, (E, d, f), d ** -0.5, "bf16")
    w2 = synth.normal(T, 4, (E, f, d), f ** -0.5, "bf16")
    L = MoELayer(T, d, f, E, k, G, local, "bf16")
    L.set_placement(rng.integers(0, G, E).astype(np.int32) if G > 1 else np.zeros(E, dtype=np.int32))
    L.set_weights(w1, w3, w2)
    prev = torch.from_numpy(synth.random_topk_idx(T + 1, T, E, k)).cuda()
    R = torch.zeros((E, E), dtype=torch.int64, device="cuda")

    def step():
        L.forward(x, lg)
        lib.moe_transition_counts(prev, L.topk_idx, T, k, k, E, E, R)

    outputs = lambda: [t.clone() for t in (L.topk_idx, L.topk_w, L.perm, L.inv_perm, L.expert_counts, L.expert_start,
                                           L.gpu_counts, L.gpu_offsets, L.send_buf, L.y)]
    step()                                   # eager: also the one-time kernel attribute set-up, which must not fall into the capture
    torch.cuda.synchronize()
    want, R1 = outputs(), R.clone()

    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.stream(side):
        step()                               # warm-up on the capture stream
        torch.cuda.synchronize()
        with torch.cuda.graph(graph, stream=side):
            step()
    torch.cuda.synchronize()
    R.zero_()
    for rep in range(1, 4):
        for t in (L.topk_idx, L.perm, L.inv_perm, L.expert_counts, L.send_buf, L.y):
            t.fill_(0)                       # eager work between the replays
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        for a, b in zip(outputs(), want):
            assert torch.equal(a.view(torch.uint8), b.view(torch.uint8))
        assert torch.equal(R, R1 * rep)
