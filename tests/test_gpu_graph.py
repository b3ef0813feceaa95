"""The forward launches only kernels on the caller's stream (no allocation, no host synchronisation, no memset
nodes), so it can be captured into a HIP graph once N' is known; replays must reproduce the eager result."""
import numpy as np
import pytest
import torch

from paper_2601_15013_amd import binding, harness, synth
from tests.test_gpu_forward import SMALL_BF16

pytestmark = pytest.mark.gpu


@pytest.mark.parametrize("fused", [False, True])
def test_forward_replays_from_a_captured_graph(fused):
    w = synth.SynthWeights(SMALL_BF16, 61)
    b = synth.multilevel_batch(9, 10, 60, 2, 20, 1, 120, SMALL_BF16.vocab)
    model = harness.upload_model(w)
    run = harness.Runner(model, b.N, b.B)
    tok, cu = harness.upload_batch(b)
    I_s, I_g, n_dev, n_c = run.build_index(tok, cu)
    out = torch.empty((b.N, SMALL_BF16.d), dtype=torch.float32, device="cuda")

    def forward():
        binding.radix_prefill_forward(model, tok, None, cu, b.max_seqlen, I_s, I_g, n_c, run.ws, out=out,
                                      force_dedup=True, fused_attention=fused)

    forward()                                   # eager: reference, and first-call set-up outside the capture
    torch.cuda.synchronize()
    want = out.clone()
    side = torch.cuda.Stream()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.stream(side):
        side.wait_stream(torch.cuda.current_stream())
        with torch.cuda.graph(graph, stream=side):
            forward()
    for i in range(3):
        out.fill_(float(i))                     # eager work between replays
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        assert run.status() == 0
        assert torch.equal(out, want), f"replay {i} differs from the eager forward"
    model.close()
