"""CPU oracle for the sparse 3D attention path of Sparse VideoGen (arXiv 2502.01776).

TEST INFRASTRUCTURE ONLY.  This file is the slow, plain definition that the HIP
kernels are checked against.  It shares no code with the product library and must
not be imported by it; only tests, the smoke check and the benchmark's CPU
baseline leg may call it.  All floating point is numpy float64.

Notation (the paper's symbols in brackets): F frames [N], P tokens per frame [L],
T text tokens, N = F*P + T tokens in total [S], D head dimension [H], t sampled
rows.  The original token order puts the frame index outermost ("F-outer"):
a video token sits at n = off + f*P + p, with off = T when the text tokens come
first and 0 when they come last.  The transformed order ("P-outer") puts the
position index outermost: n' = off + p*F + f.

Readings taken where the paper is silent (each listed in the design notes):
  * nearby frames / nearby positions are symmetric clipped windows
    |f_i - f_j| <= w_s and |p_i - p_j| <= w_t (Sec. 3.1, Sec. 3.3);
  * text keys are kept by both patterns and text queries attend to everything
    (Sec. 3.1, last paragraph); the first-frame keys are kept only when the
    geometry's sink flag is set, and then the transformed order of a temporal head
    keeps frame 0 as one block (see layout_perm);
  * the per-head error is the mean over (sampled row, channel) of the squared
    difference, and a head is spatial iff MSE_s < MSE_t strictly (Alg. 1);
  * the block-sparse pass keeps a (query tile, key tile) pair iff at least one of
    its elements is kept by the element mask, and then every element of a kept
    tile takes part (Fig. 4, Sec. 4.3).

Pins: every function here is checked in tests/test_oracle_pins.py against a
brute-force loop, a closed form, a library routine, a hand-worked example or an
invariant; no function is left "parity unpinned".
"""
from __future__ import annotations

from dataclasses import dataclass

import numpy as np

SPATIAL = 0   # Alg. 1: best_mask_config is true for the spatial pattern
TEMPORAL = 1
TEMPORAL_FRAME_MAJOR = 2   # tile lists only: the temporal mask for a head left in F-outer order (Sec. 5.5 comparison)


@dataclass(frozen=True)
class Geometry:
    B: int
    H: int
    F: int
    P: int
    T: int
    D: int
    text_first: int = 1
    w_s: int = 1
    w_t: int = 0
    sink_first_frame: int = 0
    block_m: int = 128
    block_n: int = 64
    softmax_scale: float = 0.0   # <= 0 means 1/sqrt(D)

    @property
    def N(self) -> int:
        return self.F * self.P + self.T

    @property
    def off(self) -> int:
        return self.T if self.text_first else 0

    @property
    def scale(self) -> float:
        return self.softmax_scale if self.softmax_scale > 0 else 1.0 / np.sqrt(self.D)

    @staticmethod
    def from_config(cfg: dict) -> "Geometry":
        keys = ("B", "H", "F", "P", "T", "D", "text_first", "w_s", "w_t",
                "sink_first_frame", "block_m", "block_n")
        return Geometry(**{k: int(cfg[k]) for k in keys})


# ----------------------------------------------------------------------------
# token coordinates (Sec. 3.1: tokens of one frame are contiguous; the same
# position in consecutive frames is P tokens apart)
# ----------------------------------------------------------------------------
def token_coords(g: Geometry):
    """Per token of the ORIGINAL order: (is_text bool[N], frame int[N], pos int[N]).
    frame and pos are -1 for text tokens."""
    n = np.arange(g.N)
    v = n - g.off
    is_text = (v < 0) | (v >= g.F * g.P)
    frame = np.where(is_text, -1, v // g.P)
    pos = np.where(is_text, -1, v % g.P)
    return is_text, frame, pos


def _element_mask(g: Geometry, rows, pattern: int) -> np.ndarray:
    is_text, frame, pos = token_coords(g)
    rows = np.arange(g.N) if rows is None else np.asarray(rows)
    coord = frame if pattern == SPATIAL else pos
    width = g.w_s if pattern == SPATIAL else g.w_t
    near = np.abs(coord[rows][:, None] - coord[None, :]) <= width
    keep = near | is_text[rows][:, None] | is_text[None, :]
    if g.sink_first_frame:
        keep = keep | (frame == 0)[None, :]
    return keep


def spatial_mask(g: Geometry, rows=None) -> np.ndarray:
    """bool [len(rows), N] in the original order: key j is kept for query i iff
    either is a text token, or their frames differ by at most w_s (Sec. 3.1
    "same frame and its adjacent frames"; Sec. 3.3 c_s nearby frames)."""
    return _element_mask(g, rows, SPATIAL)


def temporal_mask(g: Geometry, rows=None) -> np.ndarray:
    """bool [len(rows), N] in the original order: key j is kept for query i iff
    either is a text token, or their in-frame positions differ by at most w_t, in
    every frame (Sec. 3.1 "same spatial position across frames"; Sec. 3.3 c_t
    tokens across all frames)."""
    return _element_mask(g, rows, TEMPORAL)


# ----------------------------------------------------------------------------
# masked attention (Alg. 1 mask_attention)
# ----------------------------------------------------------------------------
def attention_weights(q: np.ndarray, k: np.ndarray, mask, scale: float, weight_round=None) -> np.ndarray:
    """Row-stochastic weights softmax(scale * q k^T) restricted to mask.  q [t,D],
    k [N,D], mask bool [t,N] or None (= everything kept).  weight_round (FP8 form only):
    applied to the exponentials relative to the row maximum before they are normalised."""
    s = scale * (q @ k.T)
    if mask is not None:
        s = np.where(mask, s, -np.inf)
    s = s - s.max(axis=1, keepdims=True)
    e = np.exp(s)
    if weight_round is not None:
        e = weight_round(e)
    return e / e.sum(axis=1, keepdims=True)


def masked_attention(q, k, v, mask, scale: float, weight_round=None) -> np.ndarray:
    """O = softmax_mask(scale * q k^T) v for one head.  q [t,D]; k, v [N,D]."""
    return attention_weights(q, k, mask, scale, weight_round) @ v


# ----------------------------------------------------------------------------
# layout transformation (Sec. 4.2, Fig. 4)
# ----------------------------------------------------------------------------
def layout_perm(g: Geometry) -> np.ndarray:
    """pi[n] = index in the transformed (P-outer) order of the token at index n in the
    F-outer order.  Text tokens stay where they are.  With the first-frame sink on
    (Sec. 3.1: the first frame is attended by every query of both head types) the
    transformed order keeps the P tokens of frame 0 together, in position order, in front of
    the video part, and runs the position-outer order over the other F - 1 frames only:
    every query keeps all of frame 0, and as one contiguous run it costs ceil(P / block_n)
    key tiles instead of touching every tile (its tokens would otherwise sit F rows apart)."""
    is_text, frame, pos = token_coords(g)
    n = np.arange(g.N)
    if g.sink_first_frame:
        video = np.where(frame == 0, pos, g.P + pos * (g.F - 1) + (frame - 1))
    else:
        video = pos * g.F + frame
    return np.where(is_text, n, g.off + video)


def layout_fwd(x: np.ndarray, g: Geometry) -> np.ndarray:
    """x [..., N, D] in F-outer order -> P-outer order: out[pi[n]] = x[n]."""
    out = np.empty_like(x)
    out[..., layout_perm(g), :] = x
    return out


def layout_inv(y: np.ndarray, g: Geometry) -> np.ndarray:
    """Inverse of layout_fwd: out[n] = y[pi[n]]."""
    return y[..., layout_perm(g), :]


# ----------------------------------------------------------------------------
# kept-tile lists (the block-sparse format the attention pass consumes)
# ----------------------------------------------------------------------------
def n_tiles(g: Geometry):
    return -(-g.N // g.block_m), -(-g.N // g.block_n)


def kept_tiles_of_row(g: Geometry, pattern: int, a: int) -> np.ndarray:
    """Ascending key-tile indices kept for query tile a of one pattern, in the order
    that pattern's heads are processed in: F-outer for spatial, P-outer for
    temporal.  A tile is kept iff any of its in-range elements is kept by the
    element mask."""
    _, nk = n_tiles(g)
    r = np.arange(a * g.block_m, min(g.N, (a + 1) * g.block_m))
    if pattern == SPATIAL:
        m = spatial_mask(g, r)
    elif pattern == TEMPORAL_FRAME_MAJOR:
        m = temporal_mask(g, r)                    # rows and columns stay in F-outer order
    else:
        inv = np.empty(g.N, dtype=np.int64)
        inv[layout_perm(g)] = np.arange(g.N)       # inv[n'] = original index
        m = temporal_mask(g, inv[r])[:, inv]       # rows and columns in P-outer order
    pad = nk * g.block_n - g.N
    if pad:
        m = np.concatenate([m, np.zeros((m.shape[0], pad), dtype=bool)], axis=1)
    kept = m.reshape(m.shape[0], nk, g.block_n).any(axis=(0, 2))
    return np.nonzero(kept)[0].astype(np.int32)


def tile_list(g: Geometry, pattern: int):
    """CSR (row_ptr int32[nq+1], col_idx int32[nnz]) of the kept tiles of one
    pattern: row a holds kept_tiles_of_row(g, pattern, a)."""
    nq, _ = n_tiles(g)
    row_ptr = np.zeros(nq + 1, dtype=np.int32)
    cols = []
    for a in range(nq):
        c = kept_tiles_of_row(g, pattern, a)
        cols.append(c)
        row_ptr[a + 1] = row_ptr[a] + len(c)
    return row_ptr, (np.concatenate(cols) if cols else np.zeros(0, np.int32))


def full_tile_list(g: Geometry):
    nq, nk = n_tiles(g)
    row_ptr = (np.arange(nq + 1) * nk).astype(np.int32)
    return row_ptr, np.tile(np.arange(nk, dtype=np.int32), nq)


def block_mask(g: Geometry, row_ptr, col_idx) -> np.ndarray:
    """Element expansion bool [N,N] of a tile list (small N only)."""
    m = np.zeros((g.N, g.N), dtype=bool)
    for a in range(len(row_ptr) - 1):
        for b in col_idx[row_ptr[a]:row_ptr[a + 1]]:
            m[a * g.block_m:(a + 1) * g.block_m, b * g.block_n:(b + 1) * g.block_n] = True
    return m


# ----------------------------------------------------------------------------
# block-sparse attention (Sec. 4.3) and dense attention
# ----------------------------------------------------------------------------
def sparse_attention_head(q, k, v, row_ptr, col_idx, g: Geometry, q_tiles=None, weight_round=None) -> np.ndarray:
    """One head, tensors [N,D] already in the order the tile list refers to.
    Each query tile attends to all in-range keys of its kept key tiles.
    q_tiles: optional iterable of query-tile indices; rows of other tiles are left
    NaN (used to check sampled tiles of large shapes)."""
    out = np.full((g.N, g.D), np.nan)
    tiles = range(len(row_ptr) - 1) if q_tiles is None else q_tiles
    for a in tiles:
        r0, r1 = a * g.block_m, min(g.N, (a + 1) * g.block_m)
        kept = col_idx[row_ptr[a]:row_ptr[a + 1]]
        cols = np.concatenate([np.arange(b * g.block_n, min(g.N, (b + 1) * g.block_n)) for b in kept])
        out[r0:r1] = masked_attention(q[r0:r1], k[cols], v[cols], None, g.scale, weight_round)
    return out


def dense_attention_head(q, k, v, g: Geometry, rows=None) -> np.ndarray:
    """softmax(scale q k^T) v for one head; rows selects query rows."""
    qq = q if rows is None else q[rows]
    return masked_attention(qq, k, v, None, g.scale)


# ----------------------------------------------------------------------------
# online profiling (Alg. 1) and the whole layer
# ----------------------------------------------------------------------------
def profile_heads(q, k, v, rows, g: Geometry):
    """q, k, v float64 [B,H,N,D] in the original order; rows int[t].
    Returns (mse float64 [B,H,2] with [...,0]=MSE_s and [...,1]=MSE_t,
             labels uint8 [B,H], SPATIAL iff MSE_s < MSE_t)."""
    rows = np.asarray(rows)
    ms = spatial_mask(g, rows)
    mt = temporal_mask(g, rows)
    mse = np.zeros((g.B, g.H, 2))
    for b in range(g.B):
        for h in range(g.H):
            qi = q[b, h][rows]
            o_full = masked_attention(qi, k[b, h], v[b, h], None, g.scale)
            o_s = masked_attention(qi, k[b, h], v[b, h], ms, g.scale)
            o_t = masked_attention(qi, k[b, h], v[b, h], mt, g.scale)
            mse[b, h, 0] = np.mean((o_full - o_s) ** 2)
            mse[b, h, 1] = np.mean((o_full - o_t) ** 2)
    labels = np.where(mse[..., 0] < mse[..., 1], SPATIAL, TEMPORAL).astype(np.uint8)
    return mse, labels


def svg_attention_layer(q, k, v, labels, g: Geometry, weight_round=None):
    """The sparse pass of one layer given the head labels: spatial heads run the
    block-sparse pass on the original order; temporal heads are permuted to the
    P-outer order, run the block-sparse pass with the temporal tile list, and the
    result is permuted back (Sec. 4.2).  Returns O [B,H,N,D] in the original order."""
    lists = {SPATIAL: tile_list(g, SPATIAL), TEMPORAL: tile_list(g, TEMPORAL)}
    out = np.empty_like(q)
    for b in range(g.B):
        for h in range(g.H):
            lab = int(labels[b, h])
            rp, ci = lists[lab]
            if lab == SPATIAL:
                out[b, h] = sparse_attention_head(q[b, h], k[b, h], v[b, h], rp, ci, g, weight_round=weight_round)
            else:
                o = sparse_attention_head(layout_fwd(q[b, h], g), layout_fwd(k[b, h], g),
                                          layout_fwd(v[b, h], g), rp, ci, g, weight_round=weight_round)
                out[b, h] = layout_inv(o, g)
    return out


# ----------------------------------------------------------------------------
# FP8 attention (Sec. 4.3 "Quantization", Sec. 5.2): the block-sparse pass on q, k, v
# quantised to 8-bit floating point.
#
# Reading (the paper only says that FP8 quantisation is applied to the sparse attention and
# names no format or scaling): the OCP 8-bit format E4M3 (1 sign, 4 exponent bits with bias 7,
# 3 mantissa bits, subnormals, largest finite value 448, no infinities) with one scale per
# head and tensor.  The scale is an output of the quantiser (the attention pass multiplies by
# it), so it is a float32 number: the float32 nearest to max|x| / 448.  The code of an element
# is the E4M3 value nearest to the EXACT quotient x / scale, ties to the even mantissa; a
# quotient beyond 448 (possible by one rounding of the scale) takes 448, the nearest value
# the format has.  Everything after the codes is float64.  The result is defined as exact
# attention over the DEQUANTISED tensors; an optional second form also represents the attention
# weights in E4M3 (fp8_round_weights), the way a second product on 8-bit matrix units has to.
# ----------------------------------------------------------------------------
E4M3_MAX = 448.0


def e4m3_decode(codes) -> np.ndarray:
    """Value of each E4M3 code (uint8) by the format's definition; 0x7f / 0xff are NaN."""
    c = np.asarray(codes, dtype=np.uint8).astype(np.int64)
    sign = np.where(c & 0x80, -1.0, 1.0)
    e = (c >> 3) & 15
    m = (c & 7).astype(np.float64)
    val = np.where(e == 0, m * 2.0 ** -9, (1.0 + m / 8.0) * np.exp2((e - 7).astype(np.float64)))
    val = np.where((e == 15) & ((c & 7) == 7), np.nan, val)
    return sign * val


def e4m3_encode(y) -> np.ndarray:
    """Nearest E4M3 code of each value, ties to the even mantissa; magnitudes above 448 take
    448 (the format has no larger value and no infinity)."""
    y = np.asarray(y, dtype=np.float64)
    a = np.minimum(np.abs(y), E4M3_MAX)
    code = np.zeros(a.shape, dtype=np.int64)
    sub = a < 2.0 ** -6
    code[sub] = np.rint(a[sub] * 512.0).astype(np.int64)          # multiples of 2^-9; 8 is the first normal
    an = a[~sub]
    _, ex = np.frexp(an)                                           # an = mant * 2^ex, mant in [0.5, 1)
    e = ex.astype(np.int64) - 1
    m = np.rint(an / np.exp2((e - 3).astype(np.float64))).astype(np.int64)   # 8 .. 16
    carry = m == 16
    e = e + carry
    m = np.where(carry, 8, m)
    code[~sub] = ((e + 7) << 3) | (m - 8)
    code |= np.where(np.signbit(y), 0x80, 0)
    return code.astype(np.uint8)


def fp8_quantize_head(x):
    """x [N,D] float64 -> (codes uint8 [N,D], scale float32) with x ~ decode(codes) * scale:
    scale = float32(max|x| / 448) (1 if x is all zero), code = E4M3 value nearest to the exact
    quotient x / scale (the float64 division of a 16-bit by a 24-bit significand is far below
    any rounding boundary's resolution that matters here: boundaries are 5-bit numbers)."""
    x = np.asarray(x, dtype=np.float64)
    amax = float(np.max(np.abs(x))) if x.size else 0.0
    scale = np.float32(amax / E4M3_MAX) if amax > 0 else np.float32(1)
    return e4m3_encode(x / np.float64(scale)), scale


def fp8_dequantize(codes, scale) -> np.ndarray:
    return e4m3_decode(codes) * np.float64(scale)


FP8_WEIGHT_GAIN = 256.0   # weights are stored as 2^8 w, w in (0, 1]: non-zero down to 2^-18 of the row's largest


def fp8_round_weights(e: np.ndarray) -> np.ndarray:
    """Unnormalised attention weights e = exp(s - max s) in [0, 1] as an 8-bit second product
    sees them: the E4M3 value nearest to 2^8 e (the power of two only moves the format's
    range down so that small weights survive; it cancels when the row is normalised)."""
    return e4m3_decode(e4m3_encode(FP8_WEIGHT_GAIN * e)) / FP8_WEIGHT_GAIN


def svg_attention_layer_fp8(q, k, v, labels, g: Geometry, round_weights: bool = False):
    """The sparse pass of one layer with q, k, v of every head quantised to E4M3 first
    (per head and tensor); otherwise svg_attention_layer.  The quantisation is elementwise
    with one scale per head, so it commutes with the layout transformation.  round_weights
    additionally rounds every row's weights with fp8_round_weights before they are
    normalised and applied to v."""
    dq = np.empty_like(q)
    dk = np.empty_like(k)
    dv = np.empty_like(v)
    for b in range(g.B):
        for h in range(g.H):
            for src, dst in ((q, dq), (k, dk), (v, dv)):
                codes, scale = fp8_quantize_head(src[b, h])
                dst[b, h] = fp8_dequantize(codes, scale)
    return svg_attention_layer(dq, dk, dv, labels, g, weight_round=fp8_round_weights if round_weights else None)


# ----------------------------------------------------------------------------
# QK-norm and rotary position embedding (Sec. 4.3 "Efficient kernel customization", Table 2):
# the two small per-token operations on q and k in front of the attention.
#
# Reading (the paper names the operations and gives no formula; these are the textbook
# definitions the models it evaluates use):
#   QK-norm  normalisation of every token's head vector x in R^D with a learned weight,
#            RMS form      y = x / sqrt(mean(x^2) + eps) * w           (HunyuanVideo)
#            LayerNorm     y = (x - mean(x)) / sqrt(var(x) + eps) * w + b, biased variance
#                                                                       (CogVideoX)
#   RoPE     every channel pair (a, b) of a VIDEO token is rotated by the angle the model's
#            tables give for that token and pair: (a cos - b sin, b cos + a sin).  The tables
#            cos, sin [F*P, D/2] are inputs (how a model fills them from its 3D positions is
#            its own business).  Pairs are (x[2i], x[2i+1]) ("interleaved") or
#            (x[i], x[i+D/2]) ("half").  Text tokens are not rotated.
# QK-norm comes first, then RoPE.
# ----------------------------------------------------------------------------
NORM_NONE, NORM_RMS, NORM_LAYER = 0, 1, 2
ROPE_INTERLEAVED, ROPE_HALF = 0, 1


def qk_norm(x, kind: int, weight=None, bias=None, eps: float = 1e-6) -> np.ndarray:
    """x [..., D] float64."""
    x = np.asarray(x, dtype=np.float64)
    if kind == NORM_NONE:
        return x.copy()
    if kind == NORM_RMS:
        y = x / np.sqrt(np.mean(x * x, axis=-1, keepdims=True) + eps)
    elif kind == NORM_LAYER:
        mu = np.mean(x, axis=-1, keepdims=True)
        var = np.mean((x - mu) ** 2, axis=-1, keepdims=True)
        y = (x - mu) / np.sqrt(var + eps)
    else:
        raise ValueError(kind)
    if weight is not None:
        y = y * np.asarray(weight, dtype=np.float64)
    if bias is not None and kind == NORM_LAYER:
        y = y + np.asarray(bias, dtype=np.float64)
    return y


def rope(x, cos, sin, g: Geometry, pairing: int = ROPE_INTERLEAVED) -> np.ndarray:
    """x [N, D] float64 of one head in the original token order; cos, sin [F*P, D/2]."""
    x = np.asarray(x, dtype=np.float64)
    out = x.copy()
    D = x.shape[-1]
    vid = slice(g.off, g.off + g.F * g.P)
    xv = x[vid]
    if pairing == ROPE_INTERLEAVED:
        a, b = xv[:, 0::2], xv[:, 1::2]
    else:
        a, b = xv[:, :D // 2], xv[:, D // 2:]
    ra = a * cos - b * sin
    rb = b * cos + a * sin
    yv = np.empty_like(xv)
    if pairing == ROPE_INTERLEAVED:
        yv[:, 0::2], yv[:, 1::2] = ra, rb
    else:
        yv[:, :D // 2], yv[:, D // 2:] = ra, rb
    out[vid] = yv
    return out


def qk_norm_rope(x, g: Geometry, kind=NORM_NONE, weight=None, bias=None, eps=1e-6, cos=None, sin=None,
                 pairing=ROPE_INTERLEAVED) -> np.ndarray:
    """x [B,H,N,D] float64: QK-norm of every token, then RoPE of the video tokens (skipped when
    no tables are given)."""
    y = qk_norm(x, kind, weight, bias, eps)
    if cos is not None:
        for b in range(y.shape[0]):
            for h in range(y.shape[1]):
                y[b, h] = rope(y[b, h], cos, sin, g, pairing)
    return y
