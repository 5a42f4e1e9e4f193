"""GPU parity of the compression step with threshold binary search selection (Section 2.1,
Algorithm 3, and its sampled variant that reuses a threshold) against the CPU oracle: thresholds,
counts, indices, values, residual and velocity bit for bit."""
from fractions import Fraction

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


class Runner:
    def __init__(self, rgc, oracle, V0, ks, U0=None, m=0.0, misalign=0, tag=""):
        import torch
        self.torch, self.rgc, self.oracle, self.tag = torch, rgc, oracle, tag
        self.dev = GpuLayers(rgc, V0, ks, U0, misalign=misalign, out_factor=2)
        self.ks, self.m = list(ks), m
        self.ctx = rgc.Context(sum(v.size for v in V0), len(V0))
        d = torch.device("cuda:0")
        self.thr = torch.full((len(V0),), float("nan"), dtype=torch.float32, device=d)
        self.nnz = torch.full((len(V0),), -7, dtype=torch.int32, device=d)
        self.Vh = [v.copy() for v in V0]
        self.Uh = [u.copy() for u in U0] if U0 is not None else None
        self.thr_h = [0.0] * len(V0)
        self.t = 0

    def step(self, G, search, nesterov=False, grad_scale=None):
        rgc, torch = self.rgc, self.torch
        print("  %s step %d %s" % (self.tag, self.t, "search" if search else "reuse"), flush=True)
        self.dev.set_grads(G)
        flags = (rgc.RGC_THRESHOLD_SEARCH if search else 0) | (rgc.RGC_NESTEROV if nesterov else 0)
        d_scale = None
        if grad_scale is not None:
            d_scale = torch.full((1,), float(grad_scale), dtype=torch.float32, device=self.thr.device)
        rgc.rgc_compress_layers_threshold(self.ctx, self.dev.layers, self.m, self.thr, self.nnz, flags,
                                          torch.cuda.current_stream(), grad_scale=d_scale)
        idx, val, cnt, V, U = self.dev.results()
        thr = self.thr.cpu().numpy()
        nnz = self.nnz.cpu().numpy()
        out = []
        for l, k in enumerate(self.ks):
            oi, ov, onnz, othr, trace = self.oracle.compress_layer_threshold(
                G[l], self.Vh[l], k, search=search, threshold=float(self.thr_h[l]),
                momentum=self.Uh[l] if self.Uh is not None else None, m=self.m, nesterov=nesterov,
                grad_scale=grad_scale)
            self.thr_h[l] = othr
            where = "%s step %d layer %d (n=%d, k=%d)" % (self.tag, self.t, l, self.Vh[l].size, k)
            assert u32(np.array([thr[l]], np.float32))[0] == u32(np.array([othr], np.float32))[0], \
                where + ": threshold %r vs %r" % (thr[l], othr)
            assert int(nnz[l]) == onnz, where + ": nnz %d vs %d" % (nnz[l], onnz)
            c = min(onnz, 2 * k)
            assert int(cnt[l]) == c == oi.size, where + ": count"
            assert np.array_equal(idx[l][:c], oi), where + ": indices"
            assert np.array_equal(u32(val[l][:c]), u32(ov)), where + ": values"
            assert np.all(idx[l][c:] == -1), where + ": wrote beyond the count"
            assert np.array_equal(u32(V[l]), u32(self.Vh[l])), where + ": residual"
            if self.Uh is not None:
                assert np.array_equal(u32(U[l]), u32(self.Uh[l])), where + ": velocity"
            out.append((onnz, othr, trace))
            # the buffers are reused: restore the fill the checks above rely on
        for t_ in self.dev.out_idx:
            t_.fill_(-1)
        self.t += 1
        return out

    def close(self):
        self.ctx.close()


def test_search_then_reuse_on_ragged_layers(rgc, oracle):
    g = np.random.default_rng(401)
    sizes = [300_000, 70_001, 8192, 4099, 257, 5, 1]
    V = [(g.standard_normal(n) * 5e-3).astype(np.float32) for n in sizes]
    ks = [rgc.rgc_k_for_density(n) for n in sizes]
    r = Runner(rgc, oracle, V, ks, tag="threshold plain")
    accepted = 0
    for t in range(7):                                   # the paper's schedule: search every fifth iteration
        G = [(g.standard_normal(n) * 1e-3).astype(np.float32) for n in sizes]
        out = r.step(G, search=(t % 5 == 0))
        if t % 5 == 0:
            accepted += sum(1 for (nnz, _, _), k in zip(out, ks) if k < nnz < 2 * k)
    assert accepted >= 4                                 # the large layers do stop between k and 2k
    r.close()


def test_search_with_momentum_and_nesterov_unaligned(rgc, oracle):
    g = np.random.default_rng(402)
    sizes = [120_003, 9_000, 513]
    V = [(g.laplace(0, 5e-3, n)).astype(np.float32) for n in sizes]
    U = [(g.laplace(0, 1e-3, n)).astype(np.float32) for n in sizes]
    ks = [rgc.rgc_k_for_density(n) for n in sizes]
    for nesterov, misalign in ((False, 0), (True, 1)):
        r = Runner(rgc, oracle, [v.copy() for v in V], ks, U0=[u.copy() for u in U], m=0.9, misalign=misalign,
                   tag="threshold momentum nesterov=%s misalign=%d" % (nesterov, misalign))
        for t in range(3):
            G = [(g.laplace(0, 1e-3, n)).astype(np.float32) for n in sizes]
            r.step(G, search=(t != 1), nesterov=nesterov, grad_scale=None if t == 0 else 0.37)
        r.close()


def test_hand_traced_search_on_a_uniform_grid(rgc, oracle):
    """|a| = i/4096: mean, max and every threshold are exact, the expected values are derived by hand
    (see the oracle's pins): k = 100 stops at the fourth count with 128 elements."""
    n = 4096
    g = np.random.default_rng(5)
    a = (((g.permutation(n) + 1) / n).astype(np.float32) * np.where(g.random(n) < 0.5, -1.0, 1.0).astype(np.float32))
    for k, nnz, thr in ((600, 1024, Fraction(12289, 16384)), (100, 128, Fraction(15872125, 16384000)),
                        (3000, 2046, Fraction(8194 * 1024 + 8190, 16384 * 1024))):
        r = Runner(rgc, oracle, [np.zeros(n, np.float32)], [k], tag="threshold grid k=%d" % k)
        out = r.step([a], search=True)
        assert out[0][0] == nnz and Fraction(float(out[0][1])) == thr
        r.close()


def test_degenerate_layers_and_full_buffers(rgc, oracle):
    """Constant magnitudes (max = mean: nothing passes), a count that jumps over [k, 2k] (the search takes its
    ten counts and keeps the last threshold), zeros, and a reused threshold that lets more than 2k elements
    pass (the first 2k in index order are sent, the others stay)."""
    n = 20_000
    const = np.full(n, -3.0, np.float32)
    jump = np.full(n, 0.25, np.float32)
    jump[::1000] = -4.0                                  # 20 large ones, k = 40 wants more than 40
    zeros = np.zeros(n, np.float32)
    g = np.random.default_rng(403)
    rnd = (g.standard_normal(n) * 1e-2).astype(np.float32)
    V = [const, jump, zeros, rnd]
    ks = [20, 40, 20, 20]
    r = Runner(rgc, oracle, V, ks, tag="threshold degenerate")
    Z = [np.zeros(n, np.float32) for _ in V]
    out = r.step(Z, search=True)
    assert out[0][0] == 0 and out[2][0] == 0
    assert out[1][0] in (20, n) and out[1][2][2] == 10
    r.close()
    # reuse of a low threshold: 0.5 sigma lets about 60 % of the elements pass
    r = Runner(rgc, oracle, [rnd.copy()], [20], tag="threshold overflow")
    r.thr_h[0] = np.float32(5e-3)
    r.thr.fill_(5e-3)
    out = r.step([np.zeros(n, np.float32)], search=False)
    assert out[0][0] > 2 * 20
    r.close()


def test_exact_selection_after_a_threshold_call_on_the_same_context(rgc, oracle):
    """Both entry points share the context's scratch (the histogram among it)."""
    import torch
    g = np.random.default_rng(404)
    sizes = [200_000, 3_000]
    V = [(g.standard_normal(n) * 5e-3).astype(np.float32) for n in sizes]
    ks = [rgc.rgc_k_for_density(n) for n in sizes]
    r = Runner(rgc, oracle, V, ks, tag="threshold then exact")
    r.step([(g.standard_normal(n) * 1e-3).astype(np.float32) for n in sizes], search=True)
    for t in range(3):
        G = [(g.standard_normal(n) * 1e-3).astype(np.float32) for n in sizes]
        r.dev.set_grads(G)
        rgc.rgc_compress_layers(r.ctx, r.dev.layers, 0.0, 0, torch.cuda.current_stream())
        idx, val, cnt, Vd, _ = r.dev.results()
        for l, k in enumerate(ks):
            oi, ov, oc = oracle.compress_layer(G[l], r.Vh[l], k)
            assert int(cnt[l]) == k and np.array_equal(idx[l][:k], oi) and np.array_equal(u32(val[l][:k]), u32(ov))
            assert np.array_equal(u32(Vd[l]), u32(r.Vh[l]))
        for t_ in r.dev.out_idx:
            t_.fill_(-1)
        r.step([(g.standard_normal(n) * 1e-3).astype(np.float32) for n in sizes], search=(t == 1))
    r.close()


def test_argument_errors(rgc):
    import torch
    dev = torch.device("cuda:0")
    V = torch.zeros(100, device=dev)
    G = torch.zeros(100, device=dev)
    oi = torch.zeros(2, dtype=torch.int32, device=dev)
    ov = torch.zeros(2, device=dev)
    oc = torch.zeros(1, dtype=torch.int32, device=dev)
    thr = torch.zeros(1, device=dev)
    layers = rgc.LayerList([G], [V], [1], [oi], [ov], oc)
    ctx = rgc.Context(100, 1)
    with pytest.raises(rgc.RgcError):
        rgc.rgc_compress_layers_threshold(ctx, layers, 0.0, None, None, 0, torch.cuda.current_stream())
    with pytest.raises(rgc.RgcError):
        rgc.rgc_compress_layers_threshold(ctx, layers, 0.0, thr, None, rgc.RGC_NO_HINTS, torch.cuda.current_stream())
    ctx.close()


def test_full_size_vgg16_search_and_reuse(rgc, oracle):
    """The configuration the benchmark times: the 16 VGG16-shaped tensors with momentum correction."""
    from paper_1808_04357_amd import synth
    cfg = synth.config_vgg16(num_grads=2)
    ks = [rgc.rgc_k_for_density(int(v.size)) for v in cfg["V"]]
    r = Runner(rgc, oracle, cfg["V"], ks, U0=cfg["U"], m=float(cfg["momentum"]), tag="threshold vgg16")
    out = r.step(cfg["G"][0], search=True)
    big = int(np.argmax([v.size for v in cfg["V"]]))
    assert ks[big] < out[big][0] < 2 * ks[big]
    r.step(cfg["G"][1], search=False)
    r.close()


def test_variable_length_messages_feed_decompression(rgc, oracle):
    """Sections 2.1 + 2.3 together: three workers select by threshold search (message lengths differ from worker to
    worker and from step to step), the length elements are read back, and the messages are decompressed; the dense
    result must equal the oracle's decompression of the oracle's messages bit for bit, every step, although the
    message descriptors change with every call."""
    import torch
    g = np.random.default_rng(91)
    sizes = [120_000, 33_333, 4_097]
    ks = [rgc.rgc_k_for_density(n) for n in sizes]
    N = 3
    workers = [Runner(rgc, oracle, [(g.standard_normal(n) * 5e-3).astype(np.float32) for n in sizes], ks,
                      tag="flow worker %d" % w) for w in range(N)]
    dev = torch.device("cuda:0")
    dense = [torch.full((n,), float("nan"), dtype=torch.float32, device=dev) for n in sizes]
    dctx = rgc.Context(sum(sizes), len(sizes))
    for step in range(4):
        Vh_before = [[v.copy() for v in w.Vh] for w in workers]
        Gs = [[(g.standard_normal(n) * 1e-3).astype(np.float32) for n in sizes] for _ in range(N)]
        ref_msgs = []
        for w in range(N):
            # the oracle's messages of this step, from a copy of the state the runner's own oracle call will also use
            row = []
            for l, k in enumerate(ks):
                oi, ov, _, _, _ = oracle.compress_layer_threshold(Gs[w][l], Vh_before[w][l], k, search=(step % 2 == 0),
                                                                  threshold=float(workers[w].thr_h[l]))
                row.append((oi, ov))
            ref_msgs.append(row)
        d_idx, d_val = [], []
        for w in range(N):
            wk = workers[w]
            wk.dev.set_grads(Gs[w])
            rgc.rgc_compress_layers_threshold(wk.ctx, wk.dev.layers, 0.0, wk.thr, wk.nnz,
                                              rgc.RGC_THRESHOLD_SEARCH if step % 2 == 0 else 0, torch.cuda.current_stream())
            counts = wk.dev.out_count.cpu().numpy()                       # the host round trip of the flow
            d_idx.append([wk.dev.out_idx[l][:int(counts[l])] for l in range(len(sizes))])
            d_val.append([wk.dev.out_val[l][:int(counts[l])] for l in range(len(sizes))])
            for l in range(len(sizes)):
                assert int(counts[l]) == ref_msgs[w][l][0].size, "step %d worker %d layer %d: length" % (step, w, l)
        rgc.rgc_decompress_accumulate(dctx, rgc.MessageList(d_idx, d_val, dense), 1.0 / N, rgc.RGC_OVERWRITE,
                                      torch.cuda.current_stream())
        torch.cuda.synchronize()
        for l, n in enumerate(sizes):
            want = oracle.decompress([ref_msgs[w][l][0] for w in range(N)], [ref_msgs[w][l][1] for w in range(N)], n, 1.0 / N)
            assert np.array_equal(u32(dense[l].cpu().numpy()), u32(want)), "step %d layer %d: dense" % (step, l)
        # keep the runners' host state in step with the device (thresholds and residuals)
        for w in range(N):
            thr = workers[w].thr.cpu().numpy()
            for l in range(len(sizes)):
                workers[w].Vh[l] = Vh_before[w][l]
                workers[w].thr_h[l] = float(thr[l])
    dctx.close()
    for w in workers:
        w.ctx.close()
