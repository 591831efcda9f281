"""Seeded synthetic inputs for the sparse 3D attention path.

This module only *produces inputs*: named geometries (frames, tokens per frame,
text tokens, head dimension, window half-widths, tile sizes), bf16 q/k/v tensors
with a planted per-frame or per-position component, and the sampled query rows.
It holds none of the method's arithmetic (no masks, no attention, no layout, no
tile lists), so both the CPU oracle's tests and the HIP path's tests may feed
from it without sharing any logic.

Geometry keys (plain dicts, so neither side depends on a class defined here):
  B, H      batch, heads
  F, P, T   frames, tokens per frame, text tokens;  N = F*P + T
  D         head dimension
  text_first  1: text tokens occupy [0,T) ; 0: text tokens occupy [F*P, N)
  w_s       spatial half-window in frames  (keep |f_i - f_j| <= w_s)
  w_t       temporal half-window in positions (keep |p_i - p_j| <= w_t)
  sink_first_frame  0/1, also keep keys of frame 0 in both patterns
  block_m, block_n  query-tile rows, key-tile columns
  t         number of sampled query rows used for profiling
  sigma     std-dev of the i.i.d. Gaussian part of q, k, v
  spatial_heads  callable-free description: list of head indices planted spatial
"""
from __future__ import annotations

import math

import numpy as np
import torch


def _cfg(name, B, H, F, P, T, D, text_first, w_s, w_t, bm, bn, t, sigma, spatial_heads, seed):
    N = F * P + T
    return dict(name=name, B=B, H=H, F=F, P=P, T=T, D=D, N=N, text_first=text_first,
                w_s=w_s, w_t=w_t, sink_first_frame=0, block_m=bm, block_n=bn,
                t=t if t is not None else -(-N // 100), sigma=sigma,
                spatial_heads=list(spatial_heads), seed=seed)


def _alternating(H):
    return [h for h in range(H) if h % 2 == 0]


# The five shapes the benchmark names, plus two extra window settings at the
# 120k-token shape (the kept-tile fraction sweep) and two small shapes that span
# several tiles with ragged tails for element-by-element parity.
CONFIGS = {
    # heads 0-1 spatial, 2-3 temporal; text placement is not stated for this
    # shape, prefix is used.
    "tiny": _cfg("tiny", 1, 4, 4, 64, 16, 64, 1, 1, 4, 32, 32, 16, 0.5, [0, 1], 1000),
    "cogvideox_v1": _cfg("cogvideox_v1", 1, 48, 13, 1350, 226, 64, 1, 1, 22, 128, 64, None, 1.0,
                         _alternating(48), 1001),
    "wan21_14b": _cfg("wan21_14b", 1, 40, 21, 1560, 0, 128, 1, 2, 26, 128, 64, None, 1.0,
                      [h for h in range(40) if h % 5 < 3], 1002),
    "cogvideox_v15": _cfg("cogvideox_v15", 1, 48, 11, 4080, 224, 64, 1, 1, 42, 128, 64, None, 1.0,
                          _alternating(48), 1003),
    "hunyuan": _cfg("hunyuan", 1, 24, 33, 3600, 256, 128, 0, 1, 40, 128, 64, None, 1.0,
                    _alternating(24), 1004),
    # same shape, windows chosen so that ~85% of the tiles are skipped
    "hunyuan_skip85": _cfg("hunyuan_skip85", 1, 24, 33, 3600, 256, 128, 0, 2, 272, 128, 64, None, 1.0,
                           _alternating(24), 1004),
    # same shape, ~31% of tiles kept (c_s ~ 10 frames, c_t ~ 1200 tokens)
    "hunyuan_keep31": _cfg("hunyuan_keep31", 1, 24, 33, 3600, 256, 128, 0, 5, 600, 128, 64, None, 1.0,
                           _alternating(24), 1004),
    # small shapes for full element-by-element parity: several tiles, ragged tails,
    # frame boundaries not tile aligned, text prefix / suffix, both head dims
    "mid64": _cfg("mid64", 2, 4, 5, 150, 37, 64, 1, 1, 9, 128, 64, 24, 1.0, [0, 2], 2001),
    "mid128": _cfg("mid128", 1, 6, 7, 130, 50, 128, 0, 1, 11, 128, 64, 24, 1.0, [0, 2, 4], 2002),
}


def get_config(name: str, **overrides) -> dict:
    cfg = dict(CONFIGS[name])
    cfg.update(overrides)
    cfg["N"] = cfg["F"] * cfg["P"] + cfg["T"]
    return cfg


def planted_labels(cfg) -> np.ndarray:
    """uint8 [B*H]: 0 where a per-frame component was planted, 1 where a per-position one."""
    lab = np.ones(cfg["B"] * cfg["H"], dtype=np.uint8)
    for b in range(cfg["B"]):
        for h in cfg["spatial_heads"]:
            lab[b * cfg["H"] + h] = 0
    return lab


def _unit_rows(gen, n, D):
    x = torch.randn(n, D, generator=gen, dtype=torch.float32, device=gen.device)
    return x / x.norm(dim=1, keepdim=True)


def make_qkv(cfg, boost_nats: float | None = 12.0, amplitude: float | None = None,
             seed: int | None = None, device: str = "cpu"):
    """bf16 tensors q, k, v of shape [B,H,N,D] on `device` (the random stream, and so
    the values, depend on the device the generator lives on).

    Every entry is sigma * N(0,1).  In heads listed in cfg['spatial_heads'] a unit
    vector chosen per frame is added to q and k of all video tokens of that frame;
    in the other heads a unit vector chosen per spatial position is added instead.
    The added vector is scaled by `amplitude`; if that is None it is
    sqrt(boost_nats * sqrt(D)), which makes the q.k/sqrt(D) logit of two tokens of
    the same group about `boost_nats` larger than that of unrelated tokens.
    """
    B, H, F, P, T, D, N = (cfg[k] for k in ("B", "H", "F", "P", "T", "D", "N"))
    if amplitude is None:
        amplitude = math.sqrt(boost_nats * math.sqrt(D))
    gen = torch.Generator(device=device).manual_seed(cfg["seed"] if seed is None else seed)
    off = T if cfg["text_first"] else 0
    q = torch.empty(B, H, N, D, dtype=torch.bfloat16, device=device)
    k = torch.empty_like(q)
    v = torch.empty_like(q)
    spatial = set(cfg["spatial_heads"])
    for b in range(B):
        for h in range(H):
            if h in spatial:
                e = _unit_rows(gen, F, D)                       # one per frame
                add = e[:, None, :].expand(F, P, D).reshape(F * P, D)
            else:
                e = _unit_rows(gen, P, D)                       # one per position
                add = e[None, :, :].expand(F, P, D).reshape(F * P, D)
            for dst, planted in ((q, True), (k, True), (v, False)):
                x = torch.randn(N, D, generator=gen, dtype=torch.float32, device=device) * cfg["sigma"]
                if planted:
                    x[off:off + F * P] += amplitude * add
                dst[b, h] = x.to(torch.bfloat16)
    return q, k, v


def make_plain_qkv(B, H, N, D, seed, sigma=1.0):
    """bf16 CPU tensors of i.i.d. sigma*N(0,1) entries, no planted component."""
    gen = torch.Generator().manual_seed(seed)
    return tuple((torch.randn(B, H, N, D, generator=gen, dtype=torch.float32) * sigma).to(torch.bfloat16)
                 for _ in range(3))


def sample_rows(cfg, seed: int | None = None, t: int | None = None) -> np.ndarray:
    """t distinct query-row indices in [0,N), uniform without replacement, sorted, int32."""
    t = cfg["t"] if t is None else t
    rng = np.random.default_rng((cfg["seed"] if seed is None else seed) + 7919)
    return np.sort(rng.choice(cfg["N"], size=t, replace=False)).astype(np.int32)
