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


def gpu_layer_kv2(shape, q, k, v, labels, lists=None, flags=0, fill=None):
    """k, v of the temporal heads only -> P-outer copies (one launch) -> block-sparse attention that
    reads the originals for spatial heads; q and o in token order.  Returns (o, k_t, v_t)."""
    lists = lists or device_tile_lists(shape)
    kt, vt, o = (torch.empty_like(q) for _ in range(3))
    if fill is not None:
        kt.view(torch.int16).fill_(fill)
        vt.view(torch.int16).fill_(fill)
    S.svg_layout_kv_temporal(shape, k, v, kt, vt, labels)
    S.svg_sparse_attn_fwd_kv2(shape, q, k, v, kt, vt, o, labels, *lists, flags=flags)
    torch.cuda.synchronize()
    return o, kt, vt


def gpu_layer_in_place(shape, q, k, v, labels, lists=None, canary=64):
    """The sparse pass with no layout pass at all: q, k, v, o of every head in token order, the rows of
    a temporal head's tiles gathered by the kernel.  The workspace (the row table) is given at its
    exact size with guard bytes behind it.  Returns (o, guard bytes intact)."""
    lists = lists or device_tile_lists(shape)
    nq, nk = S.svg_tile_counts(shape)
    need = 8 * nk * shape.block_n
    ws = torch.full((need + canary,), 0x5A, dtype=torch.uint8, device="cuda")
    o = torch.empty_like(q)
    S.svg_sparse_attn_fwd_ex(shape, q, k, v, o, labels, *lists,
                             flags=S.SVG_ATTN_QO_TOKEN_ORDER | S.SVG_ATTN_KV_TOKEN_ORDER,
                             workspace=ws, workspace_bytes=need)
    torch.cuda.synchronize()
    return o, bool((ws[need:] == 0x5A).all())


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


# ----------------------------------------------------------------------------- FP8
def gpu_fp8_quantize(shape, q, k, v, labels):
    """Runs svg_fp8_quantize; returns (q8, k8, v8t, scales) device tensors."""
    BH = shape.B * shape.H
    nq, nk = S.svg_tile_counts(shape)
    q8 = torch.empty(S.svg_fp8_buffer_bytes(shape, S.SVG_FP8_Q), dtype=torch.uint8, device="cuda")
    k8 = torch.full((S.svg_fp8_buffer_bytes(shape, S.SVG_FP8_K),), 0xAA, dtype=torch.uint8, device="cuda")
    v8t = torch.full((S.svg_fp8_buffer_bytes(shape, S.SVG_FP8_VT),), 0xAA, dtype=torch.uint8, device="cuda")
    scales = torch.zeros(S.svg_fp8_buffer_bytes(shape, S.SVG_FP8_SCALES) // 4, dtype=torch.float32, device="cuda")
    S.svg_fp8_quantize(shape, q, k, v, labels, q8, k8, v8t, scales)
    torch.cuda.synchronize()
    return q8, k8, v8t, scales


def gpu_layer_fp8(shape, q, k, v, labels, lists=None):
    """quantise (+ layout of k, v) -> FP8 block-sparse attention; returns o (token order)."""
    lists = lists or device_tile_lists(shape)
    q8, k8, v8t, scales = gpu_fp8_quantize(shape, q, k, v, labels)
    o = torch.empty_like(q)
    S.svg_sparse_attn_fp8_fwd(shape, q8, k8, v8t, scales, o, labels, *lists)
    torch.cuda.synchronize()
    return o


def v8t_rows(v8t: np.ndarray, nk: int) -> np.ndarray:
    """Undoes the tile-image arrangement of v8t for one head: uint8 [nk*8192] -> codes
    [nk*64, 128].  An image is [half-wave g][channel d][32 key slots]; slot 4 j + c of g is
    key 32 (j // 4) + 8 (j % 4) + 4 g + c of the tile; the two 16-byte halves of a channel
    are swapped when bit 3 of d is set."""
    img = v8t.reshape(nk, 2, 128, 2, 16)
    d = np.arange(128)
    sw = (d >> 3) & 1
    slots = np.empty((nk, 2, 128, 32), np.uint8)
    for h in (0, 1):
        slots[:, :, d, 16 * h:16 * h + 16] = img[:, :, d, h ^ sw, :]
    rows = np.empty((nk, 64, 128), np.uint8)
    for g in (0, 1):
        for i in range(32):
            j, c = i >> 2, i & 3
            rows[:, 32 * (j >> 2) + 8 * (j & 3) + 4 * g + c, :] = slots[:, g, :, i]
    return rows.reshape(nk * 64, 128)


FP8_REL_RMS = 0.03      # FP8 attention vs the oracle over the same quantised q, k, v (measured 1.2-2.1 %)


def assert_fp8_attn_close(got: torch.Tensor, ref: np.ndarray, v_absmax: float, what=""):
    """The kernel rounds every attention weight to E4M3 (3 mantissa bits, relative error at
    most 2^-4, about 3.6 % rms) before the second product and normalises by the sum of the
    rounded weights, so the output is a weighted mean of v rows with perturbed weights:
    its error is at most 2 * 2^-4 / (1 - 2^-4) of the spread of v in the worst case and a
    small fraction of that when the errors of many keys average out."""
    g = f64(got)
    assert np.isfinite(g).all(), f"{what}: non-finite output"
    err = np.abs(g - ref)
    assert err.max() <= 2.0 ** -4 * v_absmax + 1e-2, f"{what}: max-abs {err.max():.4g}"
    rel = np.linalg.norm(g - ref) / max(np.linalg.norm(ref), 1e-30)
    assert rel <= FP8_REL_RMS, f"{what}: relative rms error {rel:.4g}"
