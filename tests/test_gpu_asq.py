"""GPU parity of the Alternating Signs Quantization pieces (Section 2.2) against the CPU oracle:
selection of the k largest / k smallest elements (indices, residual and velocity bit for bit),
the one value of each message (the average of the exactly rounded sum: bit for bit, whatever the order
the kernels add in), and decompression of one-value messages (bit for bit)."""
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


def same_f32(a, b):
    a, b = np.float32(a), np.float32(b)
    return (np.isnan(a) and np.isnan(b)) or a.view(np.uint32) == b.view(np.uint32)


def run_asq(rgc, oracle, V0, G_list, ks, U0=None, m=0.0, tag="", extra_flags=0):
    import torch
    dev = GpuLayers(rgc, V0, ks, U0)
    ctx = rgc.Context(sum(v.size for v in V0), len(V0))
    means = torch.full((len(V0),), float("nan"), dtype=torch.float32, device=torch.device("cuda:0"))
    Vh = [v.copy() for v in V0]
    Uh = [u.copy() for u in U0] if U0 is not None else None
    paths = []
    for t, G in enumerate(G_list):
        sign = +1 if t % 2 == 0 else -1
        flags = (rgc.RGC_SELECT_LARGEST if sign > 0 else rgc.RGC_SELECT_SMALLEST) | extra_flags
        print("  %s step %d sign %+d" % (tag, t, sign), flush=True)
        dev.set_grads(G)
        a_ref = [Vh[l] + G[l] for l in range(len(V0))] if U0 is None else None
        dev.step(ctx, m, flags)
        rgc.rgc_message_means(ctx, dev.layers, means, torch.cuda.current_stream())
        idx, val, cnt, V, U = dev.results()
        got_means = means.cpu().numpy()
        for l, k in enumerate(ks):
            oi, omean, oc = oracle.compress_layer_asq(G[l], Vh[l], k, sign, momentum=Uh[l] if Uh is not None else None, m=m)
            where = "%s step %d layer %d (n=%d, k=%d)" % (tag, t, l, V0[l].size, k)
            assert int(cnt[l]) == oc == k, where + ": count"
            assert np.array_equal(idx[l], oi), where + ": indices"
            assert np.array_equal(u32(V[l]), u32(Vh[l])), where + ": residual"
            if Uh is not None:
                assert np.array_equal(u32(U[l]), u32(Uh[l])), where + ": velocity"
            if a_ref is not None:
                assert np.array_equal(u32(val[l]), u32(a_ref[l][oi])), where + ": values"
            assert same_f32(got_means[l], omean), where + ": mean %r vs %r" % (got_means[l], omean)
        paths.append(ctx.last_paths(len(V0)))
    ctx.close()
    return paths


def test_selection_of_largest_and_smallest_alternating(rgc, oracle):
    g = np.random.default_rng(81)
    sizes = [200_000, 50_001, 4096, 300, 7]
    V = [(g.standard_normal(n) * 5e-3).astype(np.float32) for n in sizes]
    Gs = [[(g.standard_normal(n) * 1e-3).astype(np.float32) for n in sizes] for _ in range(8)]
    ks = [rgc.rgc_k_for_density(n) for n in sizes]
    paths = run_asq(rgc, oracle, V, Gs, ks, tag="asq plain")
    # the hints of the two signs are kept apart: both directions reach the one-pass path on the large layers
    assert paths[-1][0] == 0 and paths[-2][0] == 0, paths


def test_selection_with_momentum_correction(rgc, oracle):
    g = np.random.default_rng(82)
    sizes = [150_000, 9_999]
    V = [(g.standard_normal(n) * 5e-3).astype(np.float32) for n in sizes]
    U = [(g.standard_normal(n) * 1e-3).astype(np.float32) for n in sizes]
    Gs = [[(g.standard_normal(n) * 1e-3).astype(np.float32) for n in sizes] for _ in range(5)]
    ks = [rgc.rgc_k_for_density(n) for n in sizes]
    run_asq(rgc, oracle, V, Gs, ks, U0=U, m=0.9, tag="asq momentum")


def test_layers_short_of_one_sign(rgc, oracle):
    """All-positive, all-negative, all-zero and nearly-all-zero layers: the set goes on by value (zeros, then
    the elements of the other sign closest to zero), the same on both sides."""
    g = np.random.default_rng(83)
    n = 30_000
    V = [np.abs(g.standard_normal(n)).astype(np.float32),
         -np.abs(g.standard_normal(n)).astype(np.float32),
         np.zeros(n, np.float32),
         np.where(np.arange(n) % 5000 == 17, 1.0, 0.0).astype(np.float32),
         np.where(np.arange(n) % 2 == 0, 0.0, -0.0).astype(np.float32)]
    ks = [30, 30, 30, 30, 30]
    zero = [np.zeros(n, np.float32) for _ in V]
    run_asq(rgc, oracle, V, [zero, zero, zero], ks, tag="asq short of a sign")


def test_mean_of_a_long_message(rgc, oracle):
    """1 % density on 2.5 M elements: the message's values span several parts of the device sum and a ragged tail."""
    g = np.random.default_rng(85)
    sizes = [2_500_003, 1_000]
    V = [(g.standard_normal(n) * 5e-3).astype(np.float32) for n in sizes]
    Gs = [[(g.standard_normal(n) * 1e-3).astype(np.float32) for n in sizes] for _ in range(2)]
    ks = [rgc.rgc_k_for_density(n, 10_000) for n in sizes]
    assert ks[0] > 10 * 2048
    run_asq(rgc, oracle, V, Gs, ks, tag="asq long message")


@pytest.mark.parametrize("law", ["cancelling", "wide", "subnormal", "nonfinite"])
def test_means_of_hard_sums(rgc, oracle, law):
    """The mean is that of the exactly rounded sum: values that cancel, values 250 binary orders apart,
    subnormal values, infinities and NaNs among them, in messages that span several workgroups and in tiny ones."""
    import torch
    g = np.random.default_rng({"cancelling": 1, "wide": 2, "subnormal": 3, "nonfinite": 4}[law])
    sizes = [70_001, 5_000, 257, 3]
    V = []
    for n in sizes:
        if law == "cancelling":
            h = (g.standard_normal(n // 2) * np.exp2(g.integers(-30, 90, n // 2))).astype(np.float32)
            v = np.concatenate([h, -h, np.full(n - 2 * (n // 2), 1e-30, np.float32)])
            g.shuffle(v)
        elif law == "wide":
            v = (g.standard_normal(n) * np.exp2(g.integers(-125, 125, n).astype(np.float64))).astype(np.float32)
        elif law == "subnormal":
            v = (g.integers(-2 ** 20, 2 ** 20, n).astype(np.float64) * 2.0 ** -149).astype(np.float32)
            v[::3] = np.float32(g.standard_normal())
        else:
            v = g.standard_normal(n).astype(np.float32)
            v[g.integers(0, n)] = np.inf
        V.append(v.astype(np.float32))
    if law == "nonfinite":
        V[1][7] = -np.inf           # infinities of both signs: NaN
        V[1][9] = np.inf
        V[2][100] = np.nan          # a NaN beside an infinity: NaN
        V[3][:] = [-np.inf, 1.0, -np.inf]
    # the messages are written by hand: rgc_message_means reads the value buffers and the counts of the list
    dev = GpuLayers(rgc, [np.zeros(n, np.float32) for n in sizes], sizes)
    for l, n in enumerate(sizes):
        dev.out_val[l].copy_(torch.from_numpy(V[l]))
    dev.out_count.copy_(torch.tensor(sizes, dtype=torch.int32))
    ctx = rgc.Context(sum(sizes), len(sizes))
    means = torch.full((len(sizes),), 7.0, dtype=torch.float32, device=torch.device("cuda:0"))
    print("  hard sums: %s" % law, flush=True)
    rgc.rgc_message_means(ctx, dev.layers, means, torch.cuda.current_stream())
    got = means.cpu().numpy()
    naive_differs = 0
    for l, n in enumerate(sizes):
        # the oracle's mean of these values: a layer made of them, every element sent (k = n)
        _, omean, oc = oracle.compress_layer_asq(np.zeros(n, np.float32), V[l].copy(), n, +1)
        assert oc == n
        assert same_f32(got[l], omean), "%s layer %d: %r vs %r" % (law, l, got[l], omean)
        with np.errstate(all="ignore"):
            naive_differs += not same_f32(np.float32(np.cumsum(V[l].astype(np.float64))[-1] / n), omean)
    if law == "cancelling":
        assert naive_differs > 0, "the inputs do not tell an ordered fp64 sum from the exact one"
    ctx.close()


@pytest.mark.parametrize("ppm", [250_000, 62_500])
def test_alternating_selection_at_warmup_densities(rgc, oracle, ppm):
    """The densities of a warm-up period (Section 2.5) with the alternating selection: the large layers take the
    hinted path of the dense layers once their hints exist, with the signed key; gradients larger than the residual
    keep the k-th value steady, so the hints hit."""
    g = np.random.default_rng(86)
    sizes = [600_000, 200_003, 9_000]
    V = [(g.standard_normal(n) * 1e-3).astype(np.float32) for n in sizes]
    U = [(g.standard_normal(n) * 1e-3).astype(np.float32) for n in sizes]
    Gs = [[(g.standard_normal(n) * 5e-3).astype(np.float32) for n in sizes] for _ in range(10)]
    ks = [rgc.rgc_k_for_density(n, ppm) for n in sizes]
    paths = run_asq(rgc, oracle, V, Gs, ks, U0=U, m=0.5, tag="asq %d ppm" % ppm)
    assert paths[-1][0] == 0 and paths[-2][0] == 0, paths      # both signs' hints lead the largest layer along its hinted path


def test_no_hints_gives_the_same(rgc, oracle):
    g = np.random.default_rng(84)
    sizes = [120_000, 5_000]
    V = [(g.standard_normal(n) * 5e-3).astype(np.float32) for n in sizes]
    Gs = [[(g.standard_normal(n) * 1e-3).astype(np.float32) for n in sizes] for _ in range(3)]
    ks = [rgc.rgc_k_for_density(n) for n in sizes]
    run_asq(rgc, oracle, V, Gs, ks, tag="asq no hints", extra_flags=rgc.RGC_NO_HINTS)


def test_full_size_lstm_set_alternating(rgc, oracle):
    """The LSTM-shaped layer set at full size (66.0 M elements, row-sparse embedding gradient): two hint-free
    and two hinted calls, largest and smallest in turn."""
    from paper_1808_04357_amd import synth
    cfg = synth.config_lstm(num_grads=4)
    ks = [rgc.rgc_k_for_density(v.size) for v in cfg["V"]]
    assert sum(ks) == 66_024
    run_asq(rgc, oracle, cfg["V"], cfg["G"], ks, tag="asq C4")


def test_full_size_vgg16_set_alternating_with_momentum(rgc, oracle):
    """The VGG16-shaped set at full size with the momentum correction, as the benchmark's alternating-signs
    block runs it: the k largest, then the k smallest (both calls on the multi-pass path)."""
    from paper_1808_04357_amd import synth
    cfg = synth.config_vgg16(num_grads=2)
    ks = [rgc.rgc_k_for_density(v.size) for v in cfg["V"]]
    assert sum(ks) == 138_351
    run_asq(rgc, oracle, cfg["V"], cfg["G"], ks, U0=cfg["U"], m=cfg["momentum"], tag="asq C3")


def test_both_selection_flags_are_rejected(rgc):
    import torch
    dev = torch.device("cuda:0")
    V = torch.zeros(100, device=dev)
    G = torch.zeros(100, device=dev)
    oi = torch.zeros(1, dtype=torch.int32, device=dev)
    ov = torch.zeros(1, device=dev)
    oc = torch.zeros(1, dtype=torch.int32, device=dev)
    layers = rgc.LayerList([G], [V], [1], [oi], [ov], oc)
    ctx = rgc.Context(100, 1)
    with pytest.raises(rgc.RgcError):
        rgc.rgc_compress_layers(ctx, layers, 0.0, rgc.RGC_SELECT_LARGEST | rgc.RGC_SELECT_SMALLEST, torch.cuda.current_stream())
    ctx.close()


@pytest.mark.parametrize("N", [1, 3, 128, 200])
def test_decompression_of_one_value_messages(rgc, oracle, N):
    import torch
    g = np.random.default_rng(90 + N)
    sizes = [5000, 3 * 4096 + 11, 1]
    counts = [40, 300, 1]
    dev = torch.device("cuda:0")
    idx = [[np.sort(g.choice(n, size=min(c, n), replace=False)).astype(np.int32) for n, c in zip(sizes, counts)] for _ in range(N)]
    one = [[np.float32(x) for x in g.standard_normal(len(sizes))] for _ in range(N)]
    d_idx = [[torch.from_numpy(idx[w][l]).to(dev) for l in range(len(sizes))] for w in range(N)]
    d_one = [[torch.full((1,), float(one[w][l]), dtype=torch.float32, device=dev) for l in range(len(sizes))] for w in range(N)]
    ctx = rgc.Context(1024, 1)
    for add in (False, True):
        init = [g.standard_normal(n).astype(np.float32) for n in sizes] if add else None
        dense = [torch.from_numpy(init[l]).to(dev) if add else torch.full((n,), float("nan"), dtype=torch.float32, device=dev)
                 for l, n in enumerate(sizes)]
        msgs = rgc.MessageList(d_idx, d_one, dense)
        # the binding counts a message's entries by its index tensor; its value tensor has one element
        flags = (rgc.RGC_ADD_TO_DST if add else rgc.RGC_OVERWRITE) | rgc.RGC_ONE_VALUE | rgc.RGC_VALIDATE
        rgc.rgc_decompress_accumulate(ctx, msgs, 0.5, flags, torch.cuda.current_stream())
        assert ctx.decompress_status(torch.cuda.current_stream()) == 0
        for l, n in enumerate(sizes):
            ref = oracle.decompress_scalar([idx[w][l] for w in range(N)], [one[w][l] for w in range(N)], n, 0.5,
                                           dense=init[l].copy() if add else None)
            got = dense[l].cpu().numpy()
            assert np.array_equal(u32(got), u32(ref)), "N=%d layer %d add=%s" % (N, l, add)
    ctx.close()
