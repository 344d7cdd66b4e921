"""Seeded synthetic checkpoints (inputs only; none of the method's arithmetic lives here).

The paper evaluates on checkpoints of real training runs (its Tables 3-4 list the models and
datasets); those are not available, so tensors with the same shapes and plausible value
distributions stand in for them.  Every generator is deterministic in its seed.  Small cases are
drawn with numpy on the host (identical bytes for the CPU oracle and the GPU path); the 7B-shaped
case is drawn on the device with torch and copied back only for the tensors the oracle samples.
"""
from __future__ import annotations

import math
from typing import Iterator, List, Sequence, Tuple

import numpy as np

Shape = Tuple[int, ...]

# ----------------------------------------------------------------------------------------------
# configuration grids: (bits, prune_ppm, outlier_ppm), bits-major then prune then outlier
# ----------------------------------------------------------------------------------------------


def make_grid(bits: Sequence[int], prune: Sequence[float], outlier: Sequence[float]):
    return [(int(b), int(round(p * 1e6)), int(round(o * 1e6)))
            for b in bits for p in prune for o in outlier]


def grid_paper(prune=(0.0, 0.1, 0.2, 0.3, 0.4, 0.5), protect=(0.0005, 0.005, 0.01),
               bins=(4, 6, 8, 12, 16, 32)):
    """The search space of the paper's Sec. 5 (magnitude metric): numbers of bins x pruning fractions x
    protection fractions, as (0, prune_ppm, protect_ppm, bins).  All of it has 18 (prune, protect)
    pairs; one call of the library takes 15."""
    return [(0, int(round(p * 1e6)), int(round(o * 1e6)), int(k)) for k in bins for p in prune for o in protect]


def grid_small():
    """24 configurations: bits {2,3,4,8} x prune {0,.1,.3} x protect {0,.001}."""
    return make_grid([2, 3, 4, 8], [0.0, 0.1, 0.3], [0.0, 0.001])


def grid_full():
    """105 configurations: bits 2..8 x prune {0,.05,.1,.2,.4} x protect {0,1e-4,1e-3}."""
    return make_grid(range(2, 9), [0.0, 0.05, 0.1, 0.2, 0.4], [0.0, 1e-4, 1e-3])


EPS_DEFAULT = 1e-2  # relative squared error allowed by the search in tests and bench

# ----------------------------------------------------------------------------------------------
# model shapes
# ----------------------------------------------------------------------------------------------


def resnet50_shapes() -> List[Tuple[str, Shape]]:
    out: List[Tuple[str, Shape]] = []

    def conv(name, cout, cin, k):
        out.append((name + ".weight", (cout, cin, k, k)))

    def bn(name, c):
        out.append((name + ".weight", (c,)))
        out.append((name + ".bias", (c,)))

    conv("conv1", 64, 3, 7)
    bn("bn1", 64)
    inplanes = 64
    for li, (planes, blocks) in enumerate(zip([64, 128, 256, 512], [3, 4, 6, 3]), start=1):
        for b in range(blocks):
            p = f"layer{li}.{b}"
            conv(p + ".conv1", planes, inplanes, 1)
            bn(p + ".bn1", planes)
            conv(p + ".conv2", planes, planes, 3)
            bn(p + ".bn2", planes)
            conv(p + ".conv3", planes * 4, planes, 1)
            bn(p + ".bn3", planes * 4)
            if b == 0:
                conv(p + ".downsample.0", planes * 4, inplanes, 1)
                bn(p + ".downsample.1", planes * 4)
            inplanes = planes * 4
    out.append(("fc.weight", (1000, 2048)))
    out.append(("fc.bias", (1000,)))
    return out


def bert_base_shapes() -> List[Tuple[str, Shape]]:
    h, ff, v = 768, 3072, 30522
    out: List[Tuple[str, Shape]] = [
        ("embeddings.word", (v, h)), ("embeddings.position", (512, h)),
        ("embeddings.token_type", (2, h)), ("embeddings.ln.weight", (h,)),
        ("embeddings.ln.bias", (h,))]
    for l in range(12):
        p = f"layer{l}"
        for nm in ("q", "k", "v", "o"):
            out.append((f"{p}.attn.{nm}.weight", (h, h)))
            out.append((f"{p}.attn.{nm}.bias", (h,)))
        out.append((f"{p}.attn.ln.weight", (h,)))
        out.append((f"{p}.attn.ln.bias", (h,)))
        out.append((f"{p}.ffn.in.weight", (ff, h)))
        out.append((f"{p}.ffn.in.bias", (ff,)))
        out.append((f"{p}.ffn.out.weight", (h, ff)))
        out.append((f"{p}.ffn.out.bias", (h,)))
        out.append((f"{p}.ffn.ln.weight", (h,)))
        out.append((f"{p}.ffn.ln.bias", (h,)))
    out.append(("pooler.weight", (h, h)))
    out.append(("pooler.bias", (h,)))
    return out


def gpt2_medium_shapes() -> List[Tuple[str, Shape]]:
    d, v = 1024, 50257
    out: List[Tuple[str, Shape]] = [("wte", (v, d)), ("wpe", (1024, d))]
    for l in range(24):
        p = f"h{l}"
        out += [(p + ".ln1.weight", (d,)), (p + ".ln1.bias", (d,)),
                (p + ".attn.c_attn.weight", (d, 3 * d)), (p + ".attn.c_attn.bias", (3 * d,)),
                (p + ".attn.c_proj.weight", (d, d)), (p + ".attn.c_proj.bias", (d,)),
                (p + ".ln2.weight", (d,)), (p + ".ln2.bias", (d,)),
                (p + ".mlp.c_fc.weight", (d, 4 * d)), (p + ".mlp.c_fc.bias", (4 * d,)),
                (p + ".mlp.c_proj.weight", (4 * d, d)), (p + ".mlp.c_proj.bias", (d,))]
    out += [("ln_f.weight", (d,)), ("ln_f.bias", (d,))]
    return out


def llama7b_shapes(n_layers: int = 32) -> List[Tuple[str, Shape]]:
    d, ff, v = 4096, 11008, 32000
    out: List[Tuple[str, Shape]] = [("embed_tokens", (v, d))]
    for l in range(n_layers):
        p = f"layers.{l}"
        out += [(p + ".attn.q", (d, d)), (p + ".attn.k", (d, d)), (p + ".attn.v", (d, d)),
                (p + ".attn.o", (d, d)), (p + ".mlp.gate", (ff, d)), (p + ".mlp.up", (ff, d)),
                (p + ".mlp.down", (d, ff)), (p + ".input_norm", (d,)), (p + ".post_norm", (d,))]
    out += [("norm", (d,)), ("lm_head", (v, d))]
    return out


def numel(shape: Shape) -> int:
    n = 1
    for s in shape:
        n *= int(s)
    return n


# ----------------------------------------------------------------------------------------------
# host (numpy) generators
# ----------------------------------------------------------------------------------------------


def config0(seed: int = 0, n: int = 1 << 20):
    """One tensor of n weights ~ 0.9 N(0,0.02) + 0.1 Laplace(0,0.08); next = prev + N(0,1e-4)."""
    rng = np.random.default_rng(seed)
    pick = rng.random(n) < 0.9
    x = np.where(pick, rng.normal(0.0, 0.02, n), rng.laplace(0.0, 0.08, n)).astype(np.float32)
    nxt = (x.astype(np.float64) + rng.normal(0.0, 1e-4, n)).astype(np.float32)
    return x, nxt


def _fan_in(shape: Shape) -> int:
    if len(shape) == 4:
        return shape[1] * shape[2] * shape[3]
    if len(shape) == 2:
        return shape[1]
    return shape[0]


def adam_step(w, m, v, rng, lr=1e-3, g_std=1e-3, mask=None):
    """One Adam-like step: returns (w', m', v').  mask (bool, same shape) limits which entries move."""
    g = rng.normal(0.0, g_std, w.shape).astype(np.float32)
    upd = (lr * m / (np.sqrt(v) + 1e-8)).astype(np.float32)
    m2 = (0.9 * m + 0.1 * g).astype(np.float32)
    v2 = (0.999 * v + 0.001 * g * g).astype(np.float32)
    w2 = (w - upd).astype(np.float32)
    if mask is not None:
        w2 = np.where(mask, w2, w)
        m2 = np.where(mask, m2, m)
        v2 = np.where(mask, v2, v)
    return w2, m2, v2


def resnet50_checkpoint(seed: int = 1000, scale: float = 1.0) -> Iterator[Tuple[str, np.ndarray, np.ndarray]]:
    """Yields (name, prev, cur) flat fp32 arrays for weights, Adam m and Adam v of every tensor.

    scale < 1 shrinks every tensor's leading dimension (for quick tests)."""
    for ti, (name, shape) in enumerate(resnet50_shapes()):
        if scale != 1.0:
            shape = (max(1, int(shape[0] * scale)),) + tuple(shape[1:])
        rng = np.random.default_rng(seed + ti)
        n = numel(shape)
        w = rng.normal(0.0, math.sqrt(2.0 / _fan_in(shape)), n).astype(np.float32)
        heavy = rng.random(n) < 0.01
        w = np.where(heavy, w * np.float32(1.5), w).astype(np.float32)
        m = rng.normal(0.0, 1e-3, n).astype(np.float32)
        v = np.abs(rng.normal(0.0, 1e-6, n)).astype(np.float32)
        w2, m2, v2 = adam_step(w, m, v, rng)
        yield name, w, w2
        yield name + ".adam_m", m, m2
        yield name + ".adam_v", v, v2


def bert_base_checkpoint(seed: int = 2000, scale: float = 1.0) -> Iterator[Tuple[str, np.ndarray, np.ndarray]]:
    """BERT-base-shaped weights N(0,0.02) with Adam state; the word embedding only moves on a
    Zipf-drawn 5 % of its rows, and its untouched rows have zero m."""
    for ti, (name, shape) in enumerate(bert_base_shapes()):
        if scale != 1.0:
            shape = (max(1, int(shape[0] * scale)),) + tuple(shape[1:])
        rng = np.random.default_rng(seed + ti)
        n = numel(shape)
        w = rng.normal(0.0, 0.02, n).astype(np.float32)
        m = rng.normal(0.0, 1e-3, n).astype(np.float32)
        v = np.abs(rng.normal(0.0, 1e-6, n)).astype(np.float32)
        mask = None
        if name == "embeddings.word":
            rows, cols = shape
            pz = 1.0 / np.arange(1, rows + 1)
            pz /= pz.sum()
            hot = rng.choice(rows, size=max(1, rows // 20), replace=False, p=pz)
            rowmask = np.zeros(rows, bool)
            rowmask[hot] = True
            mask = np.repeat(rowmask, cols)
            m = np.where(mask, m, np.float32(0.0)).astype(np.float32)
        w2, m2, v2 = adam_step(w, m, v, rng, mask=mask)
        yield name, w, w2
        yield name + ".adam_m", m, m2
        yield name + ".adam_v", v, v2


def gpt2_medium_steps(seed: int = 3000, scale: float = 1.0, n_steps: int = 5):
    """Yields (name, [step0, ..., step4]) for weights 0.02*Student-t(4) with Adam state and
    learning rate 1e-3 * 0.5^t."""
    for ti, (name, shape) in enumerate(gpt2_medium_shapes()):
        if scale != 1.0:
            shape = (max(1, int(shape[0] * scale)),) + tuple(shape[1:])
        rng = np.random.default_rng(seed + ti)
        n = numel(shape)
        w = (0.02 * rng.standard_t(4, n)).astype(np.float32)
        m = rng.normal(0.0, 1e-3, n).astype(np.float32)
        v = np.abs(rng.normal(0.0, 1e-6, n)).astype(np.float32)
        ws, ms, vs = [w], [m], [v]
        for t in range(n_steps - 1):
            w, m, v = adam_step(w, m, v, rng, lr=1e-3 * 0.5 ** t)
            ws.append(w)
            ms.append(m)
            vs.append(v)
        yield name, ws
        yield name + ".adam_m", ms
        yield name + ".adam_v", vs


def llama_like_tensor(shape: Shape, seed: int):
    """Host version of one 7B-shaped tensor pair: 0.015*Student-t(3), 0.1 % of the columns of a
    2-D weight x20; next step = prev + N(0,1e-4)."""
    rng = np.random.default_rng(seed)
    n = numel(shape)
    w = (0.015 * rng.standard_t(3, n)).astype(np.float32)
    if len(shape) == 2:
        rows, cols = shape
        k = max(1, cols // 1000)
        hot = rng.choice(cols, size=k, replace=False)
        w = w.reshape(rows, cols)
        w[:, hot] *= np.float32(20.0)
        w = w.reshape(-1)
    nxt = (w.astype(np.float64) + rng.normal(0.0, 1e-4, n)).astype(np.float32)
    return w, nxt


# ----------------------------------------------------------------------------------------------
# device (torch) generator for the 7B-shaped checkpoint
# ----------------------------------------------------------------------------------------------


def llama7b_device_checkpoint(device, seed: int = 4000, n_layers: int = 32):
    """Returns (names, prev, cur): lists of flat fp32 device tensors, drawn on the device.

    Student-t(3) is drawn as z / sqrt(chi2_3 / 3) from four normals.  Only input generation:
    the bytes the GPU path and the oracle see are these same buffers."""
    import torch

    gen = torch.Generator(device=device)
    names, prev, cur = [], [], []
    for ti, (name, shape) in enumerate(llama7b_shapes(n_layers)):
        gen.manual_seed(seed + ti)
        n = numel(shape)
        w = torch.empty(n, dtype=torch.float32, device=device)
        step = 1 << 26
        for s in range(0, n, step):
            e = min(n, s + step)
            z = torch.randn(4, e - s, dtype=torch.float32, device=device, generator=gen)
            chi = (z[1] * z[1] + z[2] * z[2] + z[3] * z[3]) / 3.0
            w[s:e] = 0.015 * z[0] / torch.sqrt(chi)
            del z, chi
        if len(shape) == 2:
            rows, cols = shape
            k = max(1, cols // 1000)
            hot = torch.randperm(cols, device=device, generator=gen)[:k]
            w.view(rows, cols)[:, hot] *= 20.0
        nxt = torch.empty_like(w)
        for s in range(0, n, step):
            e = min(n, s + step)
            nxt[s:e] = w[s:e] + 1e-4 * torch.randn(e - s, dtype=torch.float32, device=device,
                                                   generator=gen)
        names.append(name)
        prev.append(w)
        cur.append(nxt)
    return names, prev, cur
