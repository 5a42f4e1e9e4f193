"""Helpers shared by the GPU parity tests: run the HIP path on numpy inputs, run the oracle on the
same inputs, compare bit for bit."""
from __future__ import annotations

from typing import List, Optional, Sequence

import numpy as np


def u32(a: np.ndarray) -> np.ndarray:
    return np.ascontiguousarray(a).view(np.uint32)


class GpuLayers:
    """Device copies of a layer set plus output buffers, and the rgc_layer list over them."""

    def __init__(self, rgc, V: Sequence[np.ndarray], ks: Sequence[int], U: Optional[Sequence[np.ndarray]] = None,
                 misalign: int = 0, out_factor: int = 1):
        import torch
        self.torch = torch
        self.rgc = rgc
        dev = torch.device("cuda:0")
        self.L = len(V)
        self.ks = [int(k) for k in ks]
        self.mis = misalign

        def up(a):
            if misalign:
                buf = torch.empty(a.size + misalign, dtype=torch.float32, device=dev)
                view = buf[misalign:]
                view.copy_(torch.from_numpy(a))
                return view
            return torch.from_numpy(a).to(dev)

        self._up = up
        self.V = [up(v) for v in V]
        self.U = [up(u) for u in U] if U is not None else None
        self.G = [torch.empty_like(v) for v in self.V]
        self.out_idx = [torch.full((out_factor * k,), -1, dtype=torch.int32, device=dev) for k in self.ks]
        self.out_val = [torch.full((out_factor * k,), float("nan"), dtype=torch.float32, device=dev) for k in self.ks]
        self.out_count = torch.full((self.L,), -1, dtype=torch.int32, device=dev)
        self.layers = rgc.LayerList(self.G, self.V, self.ks, self.out_idx, self.out_val, self.out_count, self.U)

    def set_grads(self, G: Sequence[np.ndarray]) -> None:
        for l in range(self.L):
            self.G[l].copy_(self.torch.from_numpy(G[l]))

    def step(self, ctx, m: float = 0.0, flags: int = 0, grad_scale=None) -> None:
        if grad_scale is None:
            self.rgc.rgc_compress_layers(ctx, self.layers, m, flags, self.torch.cuda.current_stream())
        else:
            self.rgc.rgc_compress_layers_scaled(ctx, self.layers, m, grad_scale, flags,
                                                self.torch.cuda.current_stream())

    def results(self):
        self.torch.cuda.synchronize()
        idx = [t.cpu().numpy() for t in self.out_idx]
        val = [t.cpu().numpy() for t in self.out_val]
        cnt = self.out_count.cpu().numpy()
        V = [t.cpu().numpy() for t in self.V]
        U = [t.cpu().numpy() for t in self.U] if self.U is not None else None
        return idx, val, cnt, V, U


def assert_layers_equal(tag, ks, got, oracle_msgs, V_ref, U_ref=None):
    idx, val, cnt, V, U = got
    for l, k in enumerate(ks):
        oi, ov, oc = oracle_msgs[l]
        where = "%s layer %d (n=%d, k=%d)" % (tag, l, V_ref[l].size, k)
        assert int(cnt[l]) == oc == k, where + ": count"
        if not np.array_equal(idx[l], oi):
            bad = np.nonzero(idx[l] != oi)[0]
            raise AssertionError("%s: %d index mismatches, first at %d: got %d want %d"
                                 % (where, bad.size, bad[0], idx[l][bad[0]], oi[bad[0]]))
        assert np.array_equal(u32(val[l]), u32(ov)), where + ": values"
        assert np.array_equal(u32(V[l]), u32(V_ref[l])), where + ": residual"
        if U_ref is not None:
            assert np.array_equal(u32(U[l]), u32(U_ref[l])), where + ": momentum"


def oracle_step(oracle, G, V, ks, U=None, m=0.0, mask_momentum=True, threads=1, nesterov=False, grad_scale=None):
    """Runs the oracle in place on host copies V (and U); returns the messages."""
    return oracle.compress_layers(G, V, ks, momenta=U, m=m, mask_momentum=mask_momentum, threads=threads,
                                  nesterov=nesterov, grad_scale=grad_scale)


def check_properties(a: np.ndarray, k: int, idx: np.ndarray, val: np.ndarray, cnt: int, v_new: np.ndarray):
    """Properties that pin the result at any size without sorting (see test_oracle_pins)."""
    n = a.size
    assert cnt == k
    assert np.all(idx[1:] > idx[:-1]) and idx[0] >= 0 and idx[-1] < n
    assert np.array_equal(u32(val), u32(a[idx]))
    sel = np.zeros(n, dtype=bool)
    sel[idx] = True
    vb = u32(v_new)
    assert np.all(vb[sel] == 0)
    assert np.array_equal(vb[~sel], u32(a)[~sel])
    ka = u32(a) & np.uint32(0x7FFFFFFF)
    if k < n:
        kmin = ka[sel].min()
        assert ka[~sel].max() <= kmin
        tie_uns = np.nonzero(~sel & (ka == kmin))[0]
        if tie_uns.size:
            tie_sel = np.nonzero(sel & (ka == kmin))[0]
            assert tie_sel.max() < tie_uns.min()
