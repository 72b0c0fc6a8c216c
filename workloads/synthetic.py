"""Synthetic LVLM-layer tensors shaped like the workloads the compression step
is measured on (vision hidden states, the layer's K/V rows, text-side queries).

Everything is drawn from one ``numpy.random.default_rng(seed)`` and then cast
(round-to-nearest-even) to the I/O dtype.  bf16 tensors are carried as
``uint16`` bit patterns so that numpy, the oracle and the device all see the
very same stored values.

Recipes (per sequence):
  * mixture hiddens: centres C[n_c, d] ~ N(0,1); token i carries a label c_i and
    X_i = C[c_i] + 0.1 * e_i;  K_i = CK[c_i] + 0.1*N(0,1),  V_i likewise with
    independent centre tables CK, CV.
  * "iid" structure (tiny config): labels uniform, e ~ N(0,1).
  * "grid" structure: labels are a coarse (grid/4 x grid/4) map of uniform
    integers upsampled x4, each token re-drawn uniformly with probability 0.1;
    e is z plus a 3x3 box blur of z over the image grid, rescaled to unit
    variance (spatially correlated noise).
  * multi-tile images: every tile has its own local centres; a token uses one
    of the shared global centres with probability p_global.
  * text queries Q ~ N(0,1), token-major [T, H*d_h].
  * ``pos`` = 0..N-1 : tile-major, row-major inside a tile (the token's cell in
    the original image grid).
"""
from __future__ import annotations

from dataclasses import dataclass, field
from typing import List, Optional, Sequence

import numpy as np
from scipy import ndimage

SEED_BASE = 78900


# --------------------------------------------------------------------------
# storage casts (no method arithmetic here: only dtype conversion)
# --------------------------------------------------------------------------
def f32_to_bf16_bits(x: np.ndarray) -> np.ndarray:
    """Round-to-nearest-even cast of float32 values to bf16 bit patterns."""
    u = np.ascontiguousarray(x, dtype=np.float32).view(np.uint32)
    rounded = u + np.uint32(0x7FFF) + ((u >> np.uint32(16)) & np.uint32(1))
    return (rounded >> np.uint32(16)).astype(np.uint16)


def bf16_bits_to_f32(b: np.ndarray) -> np.ndarray:
    return (b.astype(np.uint32) << np.uint32(16)).view(np.float32)


def _store(x64: np.ndarray, dtype: str) -> np.ndarray:
    if dtype == "f32":
        return np.ascontiguousarray(x64, dtype=np.float32)
    if dtype == "bf16":
        return f32_to_bf16_bits(x64.astype(np.float32))
    raise ValueError(dtype)


# --------------------------------------------------------------------------
@dataclass
class Workload:
    name: str
    dtype: str                     # "f32" | "bf16"
    batch: int
    d: int
    heads: int
    head_dim: int
    tiles: int                     # image tiles per sequence
    grid_h: int                    # token grid of one tile
    grid_w: int
    cu_vis: np.ndarray             # int32 [batch+1] offsets of vision tokens
    cu_txt: np.ndarray             # int32 [batch+1] offsets of text tokens
    X: np.ndarray                  # [sumN, d]        hidden states
    K: np.ndarray                  # [sumN, H*d_h]    key rows (token-major)
    V: np.ndarray                  # [sumN, H*d_h]
    Q: np.ndarray                  # [sumT, H*d_h]    text-side queries
    pos: np.ndarray                # int32 [sumN] original grid cell of a token
    windows_per_axis: List[int]    # w per stage
    targets: List[int]             # vision tokens kept per sequence after each stage
    seed: int = 0
    notes: str = ""
    extra: dict = field(default_factory=dict)

    @property
    def n_per_seq(self) -> int:
        return self.tiles * self.grid_h * self.grid_w

    @property
    def stages(self) -> int:
        return len(self.windows_per_axis)


def stage_targets(n: int, n_final: int, stages: int) -> List[int]:
    """Geometric interpolation of the per-stage token counts between n and
    n_final (the last one is n_final exactly)."""
    out = []
    for k in range(1, stages + 1):
        out.append(int(round(n * (n_final / n) ** (k / stages))))
    out[-1] = n_final
    return out


# --------------------------------------------------------------------------
def _labels_iid(rng, n_tok, n_c):
    return rng.integers(0, n_c, size=n_tok)


def _labels_grid(rng, gh, gw, n_c, redraw=0.1):
    ch, cw = max(gh // 4, 1), max(gw // 4, 1)
    coarse = rng.integers(0, n_c, size=(ch, cw))
    up = np.repeat(np.repeat(coarse, -(-gh // ch), axis=0), -(-gw // cw), axis=1)[:gh, :gw]
    flat = up.reshape(-1).copy()
    flip = rng.random(flat.shape[0]) < redraw
    flat[flip] = rng.integers(0, n_c, size=int(flip.sum()))
    return flat


def _noise_grid(rng, gh, gw, d):
    z = rng.standard_normal((gh, gw, d))
    e = z + ndimage.uniform_filter(z, size=(3, 3, 1), mode="nearest")
    e /= e.std()
    return e.reshape(gh * gw, d)


def _sequence(rng, *, tiles, gh, gw, d, n_c, structure, n_global=0, p_global=0.0):
    """Returns float64 X, K, V of one sequence ([tiles*gh*gw, d] each)."""
    n_tile = gh * gw
    X = np.empty((tiles * n_tile, d))
    K = np.empty_like(X)
    V = np.empty_like(X)
    if n_global:
        G = [rng.standard_normal((n_global, d)) for _ in range(3)]
    for t in range(tiles):
        C = [rng.standard_normal((n_c, d)) for _ in range(3)]
        if structure == "iid":
            lab = _labels_iid(rng, n_tile, n_c)
            e = rng.standard_normal((n_tile, d))
        else:
            lab = _labels_grid(rng, gh, gw, n_c)
            e = _noise_grid(rng, gh, gw, d)
        base = [c[lab] for c in C]
        if n_global:
            use_g = rng.random(n_tile) < p_global
            glab = rng.integers(0, n_global, size=n_tile)
            for j in range(3):
                base[j][use_g] = G[j][glab[use_g]]
        sl = slice(t * n_tile, (t + 1) * n_tile)
        X[sl] = base[0] + 0.1 * e
        K[sl] = base[1] + 0.1 * rng.standard_normal((n_tile, d))
        V[sl] = base[2] + 0.1 * rng.standard_normal((n_tile, d))
    return X, K, V


def make_custom(*, name="custom", seed=0, dtype="bf16", batch=1, tiles=1, grid_h=8, grid_w=8,
                text_lens: Sequence[int] = (16,), d=128, heads=4, head_dim=32, n_c=8,
                structure="iid", n_global=0, p_global=0.0, windows_per_axis=(2,),
                n_final: Optional[int] = None, targets: Optional[Sequence[int]] = None,
                k_outlier_frac=0.0, k_outlier_scale=4.0, per_seq_seed=False, notes="") -> Workload:
    assert heads * head_dim == d, "K/V rows are token-major with H*d_h == d"
    assert len(text_lens) == batch
    n_seq = tiles * grid_h * grid_w
    rng = np.random.default_rng(seed)
    Xs, Ks, Vs, Qs = [], [], [], []
    for b in range(batch):
        r = np.random.default_rng(seed + b) if per_seq_seed else rng
        X, K, V = _sequence(r, tiles=tiles, gh=grid_h, gw=grid_w, d=d, n_c=n_c, structure=structure,
                            n_global=n_global, p_global=p_global)
        if k_outlier_frac > 0:
            n_out = int(round(k_outlier_frac * n_seq))
            idx = r.choice(n_seq, size=n_out, replace=False)
            K[idx] *= k_outlier_scale
        Q = r.standard_normal((int(text_lens[b]), d))
        Xs.append(_store(X, dtype)); Ks.append(_store(K, dtype)); Vs.append(_store(V, dtype))
        Qs.append(_store(Q, dtype))
    cu_vis = np.arange(batch + 1, dtype=np.int32) * n_seq
    cu_txt = np.concatenate([[0], np.cumsum(np.asarray(text_lens, dtype=np.int64))]).astype(np.int32)
    pos = np.tile(np.arange(n_seq, dtype=np.int32), batch)
    stages = len(windows_per_axis)
    if targets is None:
        assert n_final is not None
        targets = stage_targets(n_seq, n_final, stages)
    return Workload(name=name, dtype=dtype, batch=batch, d=d, heads=heads, head_dim=head_dim,
                    tiles=tiles, grid_h=grid_h, grid_w=grid_w, cu_vis=cu_vis, cu_txt=cu_txt,
                    X=np.concatenate(Xs), K=np.concatenate(Ks), V=np.concatenate(Vs),
                    Q=np.concatenate(Qs), pos=pos, windows_per_axis=list(windows_per_axis),
                    targets=list(targets), seed=seed, notes=notes)


# --------------------------------------------------------------------------
# The five measured configurations (+ the paper-style halving schedule)
# --------------------------------------------------------------------------
CONFIGS = {
    1: "tiny_f32",
    2: "llava15_7b",
    3: "llava_next",
    4: "llava15_13b_heavytail",
    5: "batched_prefill",
    "halving": "llava15_7b_halving",
    "global": "llava_next_global",
}


def make_workload(cfg) -> Workload:
    """cfg in {1,2,3,4,5,"halving","global"}."""
    if cfg == 1:
        return make_custom(name=CONFIGS[1], seed=SEED_BASE + 1, dtype="f32", batch=1, grid_h=8, grid_w=8,
                           text_lens=(16,), d=128, heads=4, head_dim=32, n_c=8, structure="iid",
                           windows_per_axis=(2,), n_final=36,
                           notes="N=64, T=16, d=128, 4x32 heads, fp32; 8-centre mixture; 64->36 in one stage")
    if cfg == 2:
        return make_custom(name=CONFIGS[2], seed=SEED_BASE + 2, dtype="bf16", batch=1, grid_h=24, grid_w=24,
                           text_lens=(64,), d=4096, heads=32, head_dim=128, n_c=64, structure="grid",
                           windows_per_axis=(4, 2, 1), n_final=317,
                           notes="LLaVA-1.5-7B-shaped: N=576, T=64, d=4096; 576->472->387->317")
    if cfg == "halving":
        return make_custom(name=CONFIGS["halving"], seed=SEED_BASE + 2, dtype="bf16", batch=1, grid_h=24,
                           grid_w=24, text_lens=(64,), d=4096, heads=32, head_dim=128, n_c=64,
                           structure="grid", windows_per_axis=(4, 2, 1), targets=(288, 144, 72),
                           notes="config-2 tensors, each stage removes half: 576->288->144->72")
    if cfg == 3:
        return make_custom(name=CONFIGS[3], seed=SEED_BASE + 3, dtype="bf16", batch=1, tiles=5, grid_h=24,
                           grid_w=24, text_lens=(128,), d=4096, heads=32, head_dim=128, n_c=64,
                           structure="grid", n_global=16, p_global=0.25, windows_per_axis=(6, 4, 2),
                           n_final=1584,
                           notes="LLaVA-NeXT-shaped: N=2880 (5 tiles x 576), T=128; 2880->2360->1933->1584")
    if cfg == "global":
        wl = make_custom(name=CONFIGS["global"], seed=SEED_BASE + 3, dtype="bf16", batch=1, tiles=5,
                         grid_h=24, grid_w=24, text_lens=(128,), d=4096, heads=32, head_dim=128, n_c=64,
                         structure="grid", n_global=16, p_global=0.25, windows_per_axis=(0,),
                         targets=(2360,),
                         notes="config-3 tensors, one stage, a single window over the whole sequence "
                               "(|A|=|B|=1440): the dense-contraction case")
        return wl
    if cfg == 4:
        return make_custom(name=CONFIGS[4], seed=SEED_BASE + 4, dtype="bf16", batch=1, grid_h=24, grid_w=24,
                           text_lens=(256,), d=5120, heads=40, head_dim=128, n_c=64, structure="grid",
                           windows_per_axis=(4,), n_final=317, k_outlier_frac=0.05, k_outlier_scale=4.0,
                           notes="13B-shaped: N=576, T=256, d=5120, 40x128; 5% of vision K rows x4; 576->317")
    if cfg == 5:
        rng = np.random.default_rng(SEED_BASE + 5)
        lens = rng.integers(32, 257, size=16)
        return make_custom(name=CONFIGS[5], seed=SEED_BASE + 5, dtype="bf16", batch=16, grid_h=24, grid_w=24,
                           text_lens=tuple(int(t) for t in lens), d=4096, heads=32, head_dim=128, n_c=64,
                           structure="grid", windows_per_axis=(4, 2, 1), n_final=317, per_seq_seed=True,
                           notes="batched prefill: 16 x (N=576, T~U[32,256]), ragged text; 3 stages to 317 each")
    raise KeyError(cfg)
