"""Randomised GPU parity: random layer sets (sizes around the tile and wave-chunk boundaries), densities
from 0.01 % to 10 %, value laws (normal, Laplace, heavy ties, 90 % zeros), unaligned tensors, with and
without momentum correction / its Nesterov form, through the exact selection (with and without hints),
Alternating Signs Quantization and the threshold binary search selection, four calls each, everything
compared with the oracle bit for bit (the average of a quantized message included)."""
import os

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


def test_random_configurations(rgc, oracle):
    import torch
    iters = int(os.environ.get("RGC_RANDOM_ITERS", "80"))      # a longer sweep: RGC_RANDOM_ITERS=2500 pytest -s ...
    for it in range(iters):
        if it % 100 == 99:
            print("  configuration %d of %d" % (it + 1, iters), flush=True)
        g = np.random.default_rng(770_000 + it)
        L = int(g.integers(1, 7))
        sizes = [int(g.choice([1, 3, 63, 64, 255, 256, 257, 1000, 4095, 4096, 8191, 8193, 33000, 100_003, 400_000, 1_500_000])) for _ in range(L)]
        ppm = int(g.choice([100, 1000, 1000, 10_000, 100_000, 250_000]))
        ks = [rgc.rgc_k_for_density(n, ppm) for n in sizes]
        mom = bool(g.integers(0, 2)); nest = mom and bool(g.integers(0, 2))
        mode = int(g.integers(0, 4))      # 0 plain,1 asq alternating, 2 threshold, 3 plain no hints
        mis = int(g.choice([0, 0, 1, 3]))
        dist = int(g.integers(0, 4))
        def draw(n, s):
            if dist == 0: return (g.standard_normal(n) * s).astype(np.float32)
            if dist == 1: return g.laplace(0, s, n).astype(np.float32)
            if dist == 2: return (np.round(g.standard_normal(n) * 3) * s).astype(np.float32)   # heavy ties
            x = (g.standard_normal(n) * s).astype(np.float32); x[g.random(n) < 0.9] = 0; return x  # sparse
        V = [draw(n, 5e-3) for n in sizes]
        U = [draw(n, 1e-3) for n in sizes] if mom else None
        m = 0.9 if mom else 0.0
        dev = GpuLayers(rgc, V, ks, U, misalign=mis, out_factor=2 if mode == 2 else 1)
        ctx = rgc.Context(sum(sizes), L)
        Vh = [v.copy() for v in V]; Uh = [u.copy() for u in U] if mom else None
        thr = torch.zeros(L, device="cuda:0"); nnz = torch.zeros(L, dtype=torch.int32, device="cuda:0"); thr_h = [0.0] * L
        means = torch.zeros(L, device="cuda:0")
        desc = "it %d sizes %s ppm %d mom %s nest %s mode %d mis %d dist %d" % (it, sizes, ppm, mom, nest, mode, mis, dist)
        print(desc, flush=True)
        for step in range(4):
            G = [draw(n, 1e-3) for n in sizes]
            dev.set_grads(G)
            st = torch.cuda.current_stream()
            if mode in (0, 3):
                fl = (rgc.RGC_NESTEROV if nest else 0) | (rgc.RGC_NO_HINTS if mode == 3 else 0)
                dev.step(ctx, m, fl)
                idx, val, cnt, Vd, Ud = dev.results()
                for l, k in enumerate(ks):
                    oi, ov, oc = oracle.compress_layer(G[l], Vh[l], k, momentum=Uh[l] if mom else None, m=m, nesterov=nest)
                    assert int(cnt[l]) == k and np.array_equal(idx[l], oi) and np.array_equal(u32(val[l]), u32(ov)), desc + " step %d layer %d" % (step, l)
                    assert np.array_equal(u32(Vd[l]), u32(Vh[l])), desc
                    if mom: assert np.array_equal(u32(Ud[l]), u32(Uh[l])), desc
            elif mode == 1:
                sign = 1 if step % 2 == 0 else -1
                dev.step(ctx, m, rgc.RGC_SELECT_LARGEST if sign > 0 else rgc.RGC_SELECT_SMALLEST)
                rgc.rgc_message_means(ctx, dev.layers, means, st)
                idx, val, cnt, Vd, Ud = dev.results()
                gm = means.cpu().numpy()
                for l, k in enumerate(ks):
                    oi, om, oc = oracle.compress_layer_asq(G[l], Vh[l], k, sign, momentum=Uh[l] if mom else None, m=m)
                    assert int(cnt[l]) == k and np.array_equal(idx[l], oi), desc + " step %d layer %d" % (step, l)
                    assert np.array_equal(u32(Vd[l]), u32(Vh[l])), desc
                    if mom: assert np.array_equal(u32(Ud[l]), u32(Uh[l])), desc
                    assert np.float32(gm[l]).view(np.uint32) == np.float32(om).view(np.uint32), desc + " mean %r %r" % (gm[l], om)
            else:
                search = step % 2 == 0
                rgc.rgc_compress_layers_threshold(ctx, dev.layers, m, thr, nnz, (rgc.RGC_THRESHOLD_SEARCH if search else 0) | (rgc.RGC_NESTEROV if nest else 0), st)
                idx, val, cnt, Vd, Ud = dev.results()
                th = thr.cpu().numpy(); nz = nnz.cpu().numpy()
                for l, k in enumerate(ks):
                    oi, ov, onnz, othr, tr = oracle.compress_layer_threshold(G[l], Vh[l], k, search=search, threshold=float(thr_h[l]), momentum=Uh[l] if mom else None, m=m, nesterov=nest)
                    thr_h[l] = othr
                    assert np.float32(th[l]).view(np.uint32) == np.float32(othr).view(np.uint32), desc + " step %d layer %d thr %r %r" % (step, l, th[l], othr)
                    c = min(onnz, 2 * k)
                    assert int(nz[l]) == onnz and int(cnt[l]) == c and np.array_equal(idx[l][:c], oi) and np.array_equal(u32(val[l][:c]), u32(ov)), desc + " step %d layer %d" % (step, l)
                    assert np.array_equal(u32(Vd[l]), u32(Vh[l])), desc
                    if mom: assert np.array_equal(u32(Ud[l]), u32(Uh[l])), desc
        ctx.close()


def test_random_decompressions(rgc, oracle):
    """Random worker counts (both kernel families: up to 128 workers per batch and more), layer sizes around
    the tile size, message lengths from empty to dense, hot positions shared by many workers, both destination
    modes, full and one-value messages; bit for bit against the oracle's worker-order sums."""
    import torch
    dev = torch.device("cuda:0")
    ctx = rgc.Context(1024, 1)
    iters = int(os.environ.get("RGC_RANDOM_ITERS", "80")) * 3 // 4
    for it in range(iters):
        if it % 100 == 99:
            print("  decompression %d of %d" % (it + 1, iters), flush=True)
        g = np.random.default_rng(880_000 + it)
        N = int(g.choice([0, 1, 2, 7, 64, 128, 129, 260]))
        L = int(g.integers(1, 5))
        sizes = [int(g.choice([1, 5, 4095, 4096, 4097, 12_289, 50_000, 300_001])) for _ in range(L)]
        add = bool(g.integers(0, 2))
        one_value = bool(g.integers(0, 2))
        scale = float(g.choice([1.0, 0.5, 1.0 / 3.0, 1.0 / max(N, 1)]))
        hot = [g.choice(n, size=max(1, min(n, 64)), replace=False) for n in sizes]
        idx, val = [], []
        for w in range(N):
            ri, rv = [], []
            for l, n in enumerate(sizes):
                c = int(g.choice([0, 1, min(n, 17), min(n, max(1, n // 100)), min(n, max(1, n // 3))]))
                pick = g.choice(n, size=c, replace=False) if c else np.empty(0, np.int64)
                if c and g.random() < 0.7:                 # many workers hit the same positions
                    pick = np.union1d(pick[: c // 2], hot[l][: max(1, c - c // 2)])
                ii = np.unique(pick).astype(np.int32)
                ri.append(ii)
                rv.append(np.float32(g.standard_normal()) * np.ones(1, np.float32) if one_value
                          else g.standard_normal(ii.size).astype(np.float32))
            idx.append(ri)
            val.append(rv)
        print("  decompress it %d N %d sizes %s add %s one_value %s" % (it, N, sizes, add, one_value), flush=True)
        d_idx = [[torch.from_numpy(a).to(dev) for a in row] for row in idx]
        d_val = [[torch.from_numpy(a).to(dev) for a in row] for row in val]
        init = [g.standard_normal(n).astype(np.float32) for n in sizes]
        dense = [torch.from_numpy(a.copy()).to(dev) if add else torch.full((a.size,), float("nan"), device=dev) for a in init]
        msgs = rgc.MessageList(d_idx, d_val, dense)
        flags = (rgc.RGC_ADD_TO_DST if add else rgc.RGC_OVERWRITE) | (rgc.RGC_ONE_VALUE if one_value else 0) | rgc.RGC_VALIDATE
        rgc.rgc_decompress_accumulate(ctx, msgs, scale, flags, torch.cuda.current_stream())
        assert ctx.decompress_status(torch.cuda.current_stream()) == 0
        for l, n in enumerate(sizes):
            ii = [idx[w][l] for w in range(N)]
            if one_value:
                ref = oracle.decompress_scalar(ii, [val[w][l][0] for w in range(N)], n, scale,
                                               dense=init[l].copy() if add else None)
            else:
                ref = oracle.decompress(ii, [val[w][l] for w in range(N)], n, scale, dense=init[l].copy() if add else None)
            got = dense[l].cpu().numpy()
            assert np.array_equal(u32(got), u32(ref)), "it %d layer %d" % (it, l)
    ctx.close()
