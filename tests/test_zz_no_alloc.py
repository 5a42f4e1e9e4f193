"""GPU test of rgc_message_means_noalloc, the entry point for callers that cannot allocate: its output
must equal rgc_message_means' bit for bit (same kernels), on two calls in a row that share the
library's static scratch array, the second with a smaller input, and both must agree with the CPU
oracle's average bit for bit as well (the sum behind it is the exactly rounded one on both sides).
Collected last on purpose."""
import ctypes

import numpy as np
import pytest

from rgc_testutil import GpuLayers, u32

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def rgc():
    torch = pytest.importorskip("torch")
    if not torch.cuda.is_available():
        pytest.skip("needs a GPU")
    import paper_1808_04357_amd as pkg
    pkg.load_library()
    return pkg


def ulps(a, b):
    return abs(int(np.array(a, np.float32).view(np.int32)) - int(np.array(b, np.float32).view(np.int32)))


def messages(rgc, seed, sizes, density_ppm):
    """One compression step on the GPU: messages (device) of the given layers and the values on the host."""
    g = np.random.default_rng(seed)
    V = [(g.standard_normal(n) * 5e-3).astype(np.float32) for n in sizes]
    G = [(g.standard_normal(n) * 1e-3).astype(np.float32) for n in sizes]
    ks = [rgc.rgc_k_for_density(n, density_ppm) for n in sizes]
    dev = GpuLayers(rgc, V, ks)
    ctx = rgc.Context(sum(sizes), len(sizes))
    dev.set_grads(G)
    dev.step(ctx, 0.0, rgc.RGC_SELECT_LARGEST)
    return dev, ctx, ks


def check_call(rgc, oracle_mean_of, dev, ctx, ks, tag):
    import torch
    stream = torch.cuda.current_stream()
    L = len(ks)
    cuda = torch.device("cuda:0")
    want = torch.full((L,), float("nan"), dtype=torch.float32, device=cuda)
    got = torch.full((L,), float("nan"), dtype=torch.float32, device=cuda)
    rgc.rgc_message_means(ctx, dev.layers, want, stream)
    print("  %s: rgc_message_means_noalloc, %d layers, longest message %d" % (tag, L, max(ks)), flush=True)
    rgc.rgc_message_means_noalloc(dev.out_val, dev.out_count, ks, got, stream)
    torch.cuda.synchronize()
    w, g_ = want.cpu().numpy(), got.cpu().numpy()
    assert np.array_equal(u32(g_), u32(w)), "%s: %r vs %r" % (tag, g_, w)
    _, val, cnt, _, _ = dev.results()
    for l in range(L):
        assert int(cnt[l]) == ks[l]
        assert ulps(g_[l], oracle_mean_of(val[l])) == 0, "%s layer %d" % (tag, l)
    return g_


def test_no_alloc_means_equal_the_context_call_twice_in_a_row(rgc, oracle):
    def oracle_mean_of(values):
        # the oracle's average of a message: a layer made of exactly these values, all of them selected
        v = np.ascontiguousarray(values, dtype=np.float32)
        _, mean, _ = oracle.compress_layer_asq(v.copy(), np.zeros(v.size, np.float32), v.size, +1)
        return mean

    # first call: several parts per message (longest 30,000 values), ragged small layers beside it
    dev1, ctx1, ks1 = messages(rgc, 901, [3_000_000, 200_000, 4099, 300, 7], 10_000)
    first = check_call(rgc, oracle_mean_of, dev1, ctx1, ks1, "first call")
    # second call, smaller: fewer layers, shorter messages; the scratch still holds the first call's sums
    dev2, ctx2, ks2 = messages(rgc, 902, [50_000, 2049], 1_000)
    check_call(rgc, oracle_mean_of, dev2, ctx2, ks2, "second call (smaller)")
    # and the first input once more: nothing of the smaller call may leak into it
    again = check_call(rgc, oracle_mean_of, dev1, ctx1, ks1, "first input again")
    assert np.array_equal(u32(first), u32(again))
    ctx1.close()
    ctx2.close()


def test_no_alloc_limits_and_arguments(rgc):
    import torch
    cuda = torch.device("cuda:0")
    lib = rgc.load_library()
    n = rgc.RGC_NOALLOC_MAX_LAYERS + 1
    vals = [torch.zeros(4, dtype=torch.float32, device=cuda) for _ in range(n)]
    counts = torch.full((n,), 4, dtype=torch.int32, device=cuda)
    means = torch.zeros(n, dtype=torch.float32, device=cuda)
    with pytest.raises(rgc.RgcError) as e:
        rgc.rgc_message_means_noalloc(vals, counts, [4] * n, means)
    assert e.value.status == -2                       # RGC_ENOMEM: more layers than the static scratch holds
    with pytest.raises(rgc.RgcError) as e:
        rgc.rgc_message_means_noalloc(vals[:2], counts, [4, 0], means)
    assert e.value.status == -1
    assert lib.rgc_message_means_noalloc(None, None, None, 1, None, None) == -1
    # the limit itself is accepted; a length word above the capacity is read as the capacity
    L = rgc.RGC_NOALLOC_MAX_LAYERS
    counts[:] = 9
    vals = [torch.full((4,), float(l + 1), dtype=torch.float32, device=cuda) for l in range(L)]
    rgc.rgc_message_means_noalloc(vals, counts, [4] * L, means)
    torch.cuda.synchronize()
    assert means[:L].cpu().numpy().tolist() == [float(l + 1) for l in range(L)]
    counts[:] = 0                                      # an empty message has the average 0
    rgc.rgc_message_means_noalloc(vals[:3], counts, [4] * 3, means)
    torch.cuda.synchronize()
    assert means[:3].cpu().numpy().tolist() == [0.0, 0.0, 0.0]
