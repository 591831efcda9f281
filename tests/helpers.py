"""Shared plumbing for the GPU parity tests: upload, run the library, download."""
import numpy as np
import torch

import paper_2502_01776_amd as S
from oracle import svg_oracle as O

MAX_ABS = 2e-2     # attention outputs, bf16 result vs fp64 oracle
MEAN_ABS = 2e-3


def f64(x: torch.Tensor) -> np.ndarray:
    return x.detach().cpu().to(torch.float64).numpy()


def bits(x: torch.Tensor) -> np.ndarray:
    return x.detach().cpu().view(torch.int16).numpy().view(np.uint16)


def dev_i32(a) -> torch.Tensor:
    return torch.from_numpy(np.ascontiguousarray(a, dtype=np.int32)).cuda()


def device_tile_lists(shape):
    out = []
    for pat in (S.SVG_HEAD_SPATIAL, S.SVG_HEAD_TEMPORAL):
        rp, ci = S.svg_tile_list_build(shape, pat)
        out += [dev_i32(rp), dev_i32(ci if len(ci) else np.zeros(1, np.int32))]
    return out


def gpu_profile(shape, q, k, v, rows):
    BH = shape.B * shape.H
    t = len(rows)
    nbytes = S.svg_workspace_bytes(shape, t)
    ws = torch.empty(nbytes, dtype=torch.uint8, device="cuda")
    labels = torch.full((BH,), 255, dtype=torch.uint8, device="cuda")
    mse = torch.full((BH, 2), -1.0, dtype=torch.float32, device="cuda")
    S.svg_profile_heads(shape, q, k, v, dev_i32(rows), t, labels, mse, ws, nbytes)
    torch.cuda.synchronize()
    return labels, mse


def gpu_layer(shape, q, k, v, labels, lists=None):
    """layout fwd (q,k,v) -> block-sparse attention -> layout inv; returns o (original order)."""
    lists = lists or device_tile_lists(shape)
    qp, kp, vp, op, o = (torch.empty_like(q) for _ in range(5))
    S.svg_layout_fwd(shape, q, qp, labels)
    S.svg_layout_fwd(shape, k, kp, labels)
    S.svg_layout_fwd(shape, v, vp, labels)
    S.svg_sparse_attn_fwd(shape, qp, kp, vp, op, labels, *lists)
    S.svg_layout_inv(shape, op, o, labels)
    torch.cuda.synchronize()
    return o


def gpu_layer_token_order(shape, q, k, v, labels, lists=None):
    """layout fwd (k,v only) -> block-sparse attention reading q and writing o in token order."""
    lists = lists or device_tile_lists(shape)
    kp, vp, o = (torch.empty_like(q) for _ in range(3))
    S.svg_layout_fwd(shape, k, kp, labels)
    S.svg_layout_fwd(shape, v, vp, labels)
    S.svg_sparse_attn_fwd_ex(shape, q, kp, vp, o, labels, *lists, flags=S.SVG_ATTN_QO_TOKEN_ORDER)
    torch.cuda.synchronize()
    return o


def assert_attn_close(got: torch.Tensor, ref: np.ndarray, what=""):
    g = f64(got)
    assert np.isfinite(g).all(), f"{what}: non-finite output"
    err = np.abs(g - ref)
    assert err.max() <= MAX_ABS, f"{what}: max-abs {err.max():.4g}"
    assert err.mean() <= MEAN_ABS, f"{what}: mean-abs {err.mean():.4g}"


def labels_match(gpu_labels, oracle_mse, oracle_labels, rel=1e-3):
    """Labels must agree except where the oracle's two errors are within rel of each other."""
    gl = gpu_labels.cpu().numpy().reshape(oracle_labels.shape)
    hi = np.maximum(oracle_mse[..., 0], oracle_mse[..., 1])
    gap = np.abs(oracle_mse[..., 0] - oracle_mse[..., 1]) / np.where(hi > 0, hi, 1.0)
    return bool(((gl == oracle_labels) | (gap < rel)).all())
