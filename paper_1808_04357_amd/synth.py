"""Seeded synthetic inputs for the RGC hot path.

Holds tensor SHAPES of the model families the RedSync paper trains (Table 1:
ResNet-50 and VGG16 on ImageNet, the 2-layer 1500-unit LSTM language model of
its Setups section) and seeded value generators.  It contains none of the
method's arithmetic (no accumulate, no selection, no packing) so that both the
HIP path and the CPU oracle can be fed from it.

All random numbers come from numpy's counter-based Philox generator keyed by
(master seed, stream ordinal); the same call gives the same bits on every host.
"""
from __future__ import annotations

from typing import Dict, List, Sequence, Tuple

import numpy as np

MASTER_SEED = 0x5EED0000


def rng(config_id: int, ordinal: int) -> np.random.Generator:
    return np.random.Generator(np.random.Philox(key=[MASTER_SEED + int(config_id), int(ordinal)]))


# --------------------------------------------------------------------------- shapes

def resnet50_shapes() -> List[Tuple[str, Tuple[int, ...]]]:
    """The 161 weight/bias tensors of the standard bottleneck ResNet-50."""
    out: List[Tuple[str, Tuple[int, ...]]] = []

    def conv_bn(name: str, cout: int, cin: int, ksz: int) -> None:
        out.append((name + ".conv.weight", (cout, cin, ksz, ksz)))
        out.append((name + ".bn.weight", (cout,)))
        out.append((name + ".bn.bias", (cout,)))

    conv_bn("stem", 64, 3, 7)
    inplanes = 64
    for stage, (planes, blocks) in enumerate(zip((64, 128, 256, 512), (3, 4, 6, 3))):
        for b in range(blocks):
            p = "layer%d.%d" % (stage + 1, b)
            conv_bn(p + ".a", planes, inplanes, 1)
            conv_bn(p + ".b", planes, planes, 3)
            conv_bn(p + ".c", planes * 4, planes, 1)
            if b == 0:
                conv_bn(p + ".down", planes * 4, inplanes, 1)
            inplanes = planes * 4
    out.append(("fc.weight", (1000, 2048)))
    out.append(("fc.bias", (1000,)))
    return out


def vgg16_shapes() -> List[Tuple[str, Tuple[int, ...]]]:
    """The 13 conv + 3 FC weight tensors of VGG16 (ImageNet, 224x224 input)."""
    cfg = [(64, 3), (64, 64), (128, 64), (128, 128), (256, 128), (256, 256), (256, 256),
           (512, 256), (512, 512), (512, 512), (512, 512), (512, 512), (512, 512)]
    out = [("conv%d.weight" % (i + 1), (co, ci, 3, 3)) for i, (co, ci) in enumerate(cfg)]
    out.append(("fc6.weight", (4096, 25088)))
    out.append(("fc7.weight", (4096, 4096)))
    out.append(("fc8.weight", (1000, 4096)))
    return out


def lstm_shapes() -> List[Tuple[str, Tuple[int, ...]]]:
    """2-layer LSTM language model, 1500 hidden units, 10000-word vocabulary."""
    out = [("embedding.weight", (10000, 1500)), ("softmax.weight", (10000, 1500))]
    for l in range(2):
        out.append(("lstm%d.w_ih" % l, (6000, 1500)))
        out.append(("lstm%d.w_hh" % l, (6000, 1500)))
        out.append(("lstm%d.b_ih" % l, (6000,)))
        out.append(("lstm%d.b_hh" % l, (6000,)))
    return out


def numel(shape: Sequence[int]) -> int:
    n = 1
    for s in shape:
        n *= int(s)
    return n


# --------------------------------------------------------------------------- value laws

def normal(g: np.random.Generator, n: int, sigma: float) -> np.ndarray:
    a = g.standard_normal(n, dtype=np.float32)
    a *= np.float32(sigma)
    return a


def laplace(g: np.random.Generator, n: int, b: float) -> np.ndarray:
    """Laplace(0, b) by inverse transform of a float32 uniform, generated in blocks."""
    out = np.empty(n, dtype=np.float32)
    step = 1 << 24
    for s in range(0, n, step):
        e = min(n, s + step)
        u = g.random(e - s, dtype=np.float32)          # [0, 1)
        sign = np.where(u < 0.5, np.float32(-1.0), np.float32(1.0))
        t = np.where(u < 0.5, u, np.float32(1.0) - u)  # distance to the nearer end, (0, 0.5]
        t = np.maximum(t, np.float32(1e-30))
        out[s:e] = sign * (np.float32(-b) * np.log(np.float32(2.0) * t))
    return out


# --------------------------------------------------------------------------- configs

def config_single(n: int = 1 << 20, num_grads: int = 1) -> Dict:
    """Single fp32 layer: V ~ N(0, 1e-2), G ~ N(0, 1e-3)."""
    V = normal(rng(1, 0), n, 1e-2)
    G = [normal(rng(1, 1 + t), n, 1e-3) for t in range(num_grads)]
    return {"name": "single", "names": ["layer"], "V": [V], "G": [[g] for g in G], "U": None,
            "momentum": 0.0}


def config_resnet50(num_grads: int = 1) -> Dict:
    """161 tensors; sigma_l = 10**U(-4,-2) per tensor; G ~ N(0, sigma_l), V ~ N(0, 5 sigma_l)."""
    shapes = resnet50_shapes()
    gs = rng(2, 0)
    sig = 10.0 ** gs.uniform(-4.0, -2.0, size=len(shapes))
    V = [normal(rng(2, 1000 + l), numel(s), 5.0 * sig[l]) for l, (_, s) in enumerate(shapes)]
    G = [[normal(rng(2, 2000 + 1000 * t + l), numel(s), sig[l]) for l, (_, s) in enumerate(shapes)]
         for t in range(num_grads)]
    return {"name": "resnet50", "names": [nm for nm, _ in shapes], "V": V, "G": G, "U": None,
            "momentum": 0.0}


def config_vgg16(num_grads: int = 1, shapes=None) -> Dict:
    """16 tensors; G ~ Laplace(0, 1e-3), V ~ Laplace(0, 5e-3), u ~ Laplace(0, 1e-3); m = 0.9."""
    shapes = shapes or vgg16_shapes()
    V = [laplace(rng(3, 1000 + l), numel(s), 5e-3) for l, (_, s) in enumerate(shapes)]
    U = [laplace(rng(3, 500 + l), numel(s), 1e-3) for l, (_, s) in enumerate(shapes)]
    G = [[laplace(rng(3, 2000 + 1000 * t + l), numel(s), 1e-3) for l, (_, s) in enumerate(shapes)]
         for t in range(num_grads)]
    return {"name": "vgg16", "names": [nm for nm, _ in shapes], "V": V, "G": G, "U": U,
            "momentum": 0.9}


def _row_sparse(g: np.random.Generator, rows: int, cols: int, row_ids: np.ndarray,
                sigma: float) -> np.ndarray:
    a = np.zeros((rows, cols), dtype=np.float32)
    a[row_ids] = normal(g, row_ids.size * cols, sigma).reshape(row_ids.size, cols)
    return a.reshape(-1)


def config_lstm(num_grads: int = 1, shapes=None) -> Dict:
    """10 tensors.  Embedding gradient: 5 % of rows nonzero N(0, 1e-2), rest exactly 0;
    other gradients N(0, 1e-3).  Residuals: N(0, 5e-3); embedding residual has 25 % of its
    rows nonzero N(0, 1e-2) (a superset of every gradient's rows)."""
    shapes = shapes or lstm_shapes()
    rows, cols = shapes[0][1]
    gsel = rng(4, 0)
    perm = gsel.permutation(rows)
    v_rows = np.sort(perm[: rows // 4])
    V: List[np.ndarray] = []
    for l, (_, s) in enumerate(shapes):
        if l == 0:
            V.append(_row_sparse(rng(4, 1000), rows, cols, v_rows, 1e-2))
        else:
            V.append(normal(rng(4, 1000 + l), numel(s), 5e-3))
    G: List[List[np.ndarray]] = []
    for t in range(num_grads):
        gt = rng(4, 100 + t)
        g_rows = np.sort(gt.choice(v_rows, size=rows // 20, replace=False))
        layer_g = []
        for l, (_, s) in enumerate(shapes):
            if l == 0:
                layer_g.append(_row_sparse(rng(4, 2000 + 1000 * t), rows, cols, g_rows, 1e-2))
            else:
                layer_g.append(normal(rng(4, 2000 + 1000 * t + l), numel(s), 1e-3))
        G.append(layer_g)
    return {"name": "lstm", "names": [nm for nm, _ in shapes], "V": V, "G": G, "U": None,
            "momentum": 0.0}


def config_uniform(n: int, num_grads: int = 1) -> Dict:
    """The value law of the paper's selection benchmark (Figure 2): standard uniform."""
    V = rng(6, 0).random(n, dtype=np.float32)
    G = [[rng(6, 1 + t).random(n, dtype=np.float32) * np.float32(0.1)] for t in range(num_grads)]
    return {"name": "uniform", "names": ["layer"], "V": [V], "G": G, "U": None, "momentum": 0.0}


def decompress_messages(layer_sizes: Sequence[int], num_workers: int = 128,
                        density_ppm: int = 1000, hot_set: int = 200_000, hot_frac: float = 0.8,
                        sigma: float = 1e-2, config_id: int = 5
                        ) -> Tuple[List[List[np.ndarray]], List[List[np.ndarray]]]:
    """Messages of N virtual workers over a flat buffer split at tensor boundaries.

    Each worker sends ceil(M*ppm/1e6) distinct flat positions: ``hot_frac`` of them drawn
    without replacement from a shared hot set of ``hot_set`` positions (uniform over [0, M)),
    the rest uniform from the remaining positions; sorted ascending; values N(0, sigma).
    Returns (idx[w][l] int32 layer-local ascending, val[w][l] float32).
    """
    sizes = np.asarray(layer_sizes, dtype=np.int64)
    M = int(sizes.sum())
    bounds = np.concatenate([[0], np.cumsum(sizes)])
    per_worker = max(1, -(-M * density_ppm // 1_000_000))
    per_worker = min(per_worker, M)
    H = min(hot_set, M)
    hot = np.sort(rng(config_id, 0).choice(M, size=H, replace=False)) if H > 0 else np.empty(0, np.int64)
    n_hot = min(int(round(per_worker * hot_frac)), H)
    idx_out: List[List[np.ndarray]] = []
    val_out: List[List[np.ndarray]] = []
    for w in range(num_workers):
        g = rng(config_id, 1 + w)
        chosen = g.choice(hot, size=n_hot, replace=False) if n_hot > 0 else np.empty(0, np.int64)
        need = per_worker - n_hot
        # uniform positions outside the already chosen ones (rejection, a few rounds at most)
        picked = np.unique(chosen)
        while picked.size < per_worker:
            extra = g.integers(0, M, size=2 * need + 16)
            picked = np.unique(np.concatenate([picked, extra]))
            if picked.size > per_worker:
                # drop surplus among the newly added uniform ones, keep all hot ones
                is_hot = np.isin(picked, chosen)
                cold = picked[~is_hot]
                cold = g.permutation(cold)[: per_worker - int(is_hot.sum())]
                picked = np.sort(np.concatenate([picked[is_hot], cold]))
        flat = picked.astype(np.int64)
        vals = normal(g, flat.size, sigma)
        cut = np.searchsorted(flat, bounds)
        idx_out.append([(flat[cut[l]:cut[l + 1]] - bounds[l]).astype(np.int32)
                        for l in range(len(sizes))])
        val_out.append([np.ascontiguousarray(vals[cut[l]:cut[l + 1]]) for l in range(len(sizes))])
    return idx_out, val_out
