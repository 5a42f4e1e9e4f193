"""The compression and decompression calls recorded into a HIP graph and replayed: every replay must give
what the oracle gives for that step.  A call can be captured once its layer list has been seen by the
context (the first call with a new list allocates and uploads descriptor tables); everything that changes
from step to step (residual, velocity, threshold hints, per-layer state machine) lives in device memory,
so a replay continues where the previous step ended.  Between the replays the test does ordinary eager
work on the same stream (new gradients copied in, results copied out)."""
import numpy as np
import pytest

from rgc_testutil import GpuLayers, assert_layers_equal, oracle_step, u32

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def rgc():
    torch = pytest.importorskip("torch")
    if not torch.cuda.is_available():
        pytest.skip("needs a GPU")
    import paper_1808_04357_amd as pkg
    pkg.load_library()
    return pkg


def test_compress_and_decompress_replayed_from_a_graph(rgc, oracle):
    import torch
    g = np.random.default_rng(2718)
    sizes = [300_000, 70_013, 5_000, 64]
    ks = [rgc.rgc_k_for_density(n) for n in sizes]
    V0 = [(g.standard_normal(n) * 5e-3).astype(np.float32) for n in sizes]
    U0 = [(g.standard_normal(n) * 1e-3).astype(np.float32) for n in sizes]
    steps = 7
    Gs = [[(g.standard_normal(n) * 1e-3).astype(np.float32) for n in sizes] for _ in range(steps)]
    m, scale = 0.9, 0.5
    dev = GpuLayers(rgc, V0, ks, U0)
    cuda = torch.device("cuda:0")
    dense = [torch.full((n,), float("nan"), dtype=torch.float32, device=cuda) for n in sizes]
    msgs = rgc.MessageList([dev.out_idx], [dev.out_val], dense)
    ctx = rgc.Context(sum(sizes), len(sizes))
    Vh = [v.copy() for v in V0]
    Uh = [u.copy() for u in U0]
    s = torch.cuda.Stream()
    torch.cuda.synchronize()                          # the buffers were filled on the default stream

    def check(t, tag):
        ref = oracle_step(oracle, Gs[t], Vh, ks, U=Uh, m=m)
        got = dev.results()
        assert_layers_equal("%s step %d" % (tag, t), ks, got, ref, Vh, Uh)
        for l, n in enumerate(sizes):
            want = oracle.decompress([ref[l][0]], [ref[l][1]], n, scale)
            assert np.array_equal(u32(dense[l].cpu().numpy()), u32(want)), "%s step %d layer %d: dense" % (tag, t, l)

    with torch.cuda.stream(s):
        # step 0 eagerly: the context sees the layer list and the message list (tables allocated and uploaded)
        dev.set_grads(Gs[0])
        rgc.rgc_compress_layers(ctx, dev.layers, m, 0, s)
        rgc.rgc_decompress_accumulate(ctx, msgs, scale, rgc.RGC_OVERWRITE, s)
        s.synchronize()
        check(0, "eager")
        graph = torch.cuda.CUDAGraph()
        with torch.cuda.graph(graph, stream=s):
            rgc.rgc_compress_layers(ctx, dev.layers, m, 0, s)
            rgc.rgc_decompress_accumulate(ctx, msgs, scale, rgc.RGC_OVERWRITE, s)
        for t in range(1, steps):
            print("  replay for step %d" % t, flush=True)
            dev.set_grads(Gs[t])
            for d in dense:
                d.fill_(float("nan"))
            graph.replay()
            s.synchronize()
            check(t, "graph")
    assert ctx.last_paths(len(sizes), s)[0] == 0      # the large layer reached the hinted one-pass path
    ctx.close()
