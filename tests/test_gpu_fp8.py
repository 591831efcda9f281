"""GPU parity of the FP8 path (Sec. 4.3 "Quantization"): the quantiser bit for bit against the
oracle's codes and scales, the FP8 block-sparse attention against the oracle's attention over
the same quantised tensors."""
import numpy as np
import pytest
import torch

import paper_2502_01776_amd as S
from oracle import svg_oracle as O
from workloads import get_config, make_qkv, make_plain_qkv, planted_labels
from helpers import (f64, device_tile_lists, gpu_fp8_quantize, gpu_layer_fp8, gpu_layer_token_order, v8t_rows,
                     assert_fp8_attn_close)

pytestmark = pytest.mark.gpu


def setup(name, **ov):
    cfg = get_config(name, **ov)
    return cfg, S.shape_from_config(cfg), O.Geometry.from_config(cfg)


FP32_TWO_ROUNDINGS = 1.01 * 2.0 ** -23     # relative error of a float32 evaluation of x * (1 / scale)
_E4M3_TABLE = np.sort(O.e4m3_decode(np.arange(0, 0x7f, dtype=np.uint8)))


def count_boundary_cases(x, scale, got, want, what):
    """The oracle's code is the E4M3 value nearest to the exact quotient x / scale.  A kernel
    that forms the quotient in float32 may land on the other side of a rounding boundary when
    the exact quotient lies within that arithmetic's error of the boundary, and only then:
    a differing code must be the oracle's neighbour in the format's table, with the midpoint of
    the two no further from the exact quotient than two float32 roundings.  Returns how many
    elements used that allowance."""
    diff = got != want
    n = int(diff.sum())
    if n:
        quo = x[diff] / float(scale)
        a, b = O.e4m3_decode(got[diff]), O.e4m3_decode(want[diff])
        assert np.isfinite(a).all() and (np.sign(a) * np.sign(b) >= 0).all(), what
        ia, ib = np.searchsorted(_E4M3_TABLE, np.abs(a)), np.searchsorted(_E4M3_TABLE, np.abs(b))
        assert (np.abs(ia - ib) == 1).all(), f"{what}: a code is not the oracle's neighbour"
        mid = (np.abs(a) + np.abs(b)) / 2
        assert (np.abs(np.abs(quo) - mid) <= FP32_TWO_ROUNDINGS * np.abs(quo)).all(), \
            f"{what}: a differing code is not explained by float32 rounding at a boundary"
    return n


@pytest.mark.parametrize("with_labels", [False, True])
def test_quantiser_codes_and_scales(with_labels):
    """Scales equal to the oracle's bit for bit; codes equal to the oracle's except at
    rounding boundaries the float32 arithmetic cannot resolve (counted and printed)."""
    cfg, sh, g = setup("mid128")
    q, k, v = make_qkv(cfg)
    # Head 0 of q carries elements whose exact quotient sits on a rounding boundary up to the
    # rounding of the scale: the head's largest magnitude becomes 65/32 and x = 195/128 * 2^-j
    # gives x / (amax / 448) = 336 * 2^-j, midway between two E4M3 values.
    q[0, 0] = q[0, 0].clamp(-2.0, 2.0)
    q[0, 0, 0, 0] = 65.0 / 32.0
    for j in range(7):
        q[0, 0, 1 + j, 3] = 195.0 / 128.0 * 2.0 ** -j
    lab_np = planted_labels(cfg)
    labels = torch.from_numpy(lab_np).cuda() if with_labels else None
    q8, k8, v8t, scales = gpu_fp8_quantize(sh, q.cuda(), k.cuda(), v.cuda(), labels)
    BH = g.B * g.H
    nq, nk = O.n_tiles(g)
    q8 = q8.cpu().numpy().reshape(BH, g.N, g.D)
    k8 = k8.cpu().numpy().reshape(BH, nk * 64, g.D)
    v8t = v8t.cpu().numpy().reshape(BH, nk * 8192)
    sc = scales.cpu().numpy()
    qd, kd, vd = f64(q).reshape(BH, g.N, g.D), f64(k).reshape(BH, g.N, g.D), f64(v).reshape(BH, g.N, g.D)
    boundary = 0
    for bh in range(BH):
        permuted = with_labels and lab_np[bh] == O.TEMPORAL
        cq, sq = O.fp8_quantize_head(qd[bh])
        ck, sk = O.fp8_quantize_head(kd[bh])
        cv, sv = O.fp8_quantize_head(vd[bh])
        xk, xv = kd[bh], vd[bh]
        if permuted:
            ck, cv, xk, xv = O.layout_fwd(ck, g), O.layout_fwd(cv, g), O.layout_fwd(xk, g), O.layout_fwd(xv, g)
        assert sc[bh] == sq and sc[BH + bh] == sk and sc[2 * BH + bh] == sv
        boundary += count_boundary_cases(qd[bh], sq, q8[bh], cq, f"q head {bh}")
        boundary += count_boundary_cases(xk, sk, k8[bh][:g.N], ck, f"k head {bh}")
        assert not k8[bh][g.N:].any()
        rows = v8t_rows(v8t[bh], nk)
        boundary += count_boundary_cases(xv, sv, rows[:g.N], cv, f"v head {bh}")
        assert not rows[g.N:].any()
    total = 3 * BH * g.N * g.D
    print(f"fp8 quantiser: {boundary} of {total} codes differ from the oracle's, all at float32-unresolvable boundaries")
    # (ties are not rare here: a head whose largest magnitude has a significand divisible by 7 puts
    # every x = amax * m / 7 * 2^-n exactly on a boundary of the unrounded quotient)
    assert boundary <= total // 200


@pytest.mark.parametrize("sink", [0, 1])
def test_fp8_layer_against_the_oracle(sink):
    cfg, sh, g = setup("mid128", sink_first_frame=sink)
    q, k, v = make_qkv(cfg)
    lab_np = planted_labels(cfg)
    labels = torch.from_numpy(lab_np).cuda()
    o = gpu_layer_fp8(sh, q.cuda(), k.cuda(), v.cuda(), labels)
    ref = O.svg_attention_layer_fp8(f64(q), f64(k), f64(v), lab_np.reshape(g.B, g.H), g)
    vmax = float(np.abs(f64(v)).max())
    for b in range(g.B):
        for h in range(g.H):
            assert_fp8_attn_close(o[b, h], ref[b, h], vmax, f"fp8 layer b{b} h{h}")
    # and it stays close to the bf16 path (the quantisation error of q, k, v itself)
    o16 = gpu_layer_token_order(sh, q.cuda(), k.cuda(), v.cuda(), labels)
    rel = np.linalg.norm(f64(o) - f64(o16)) / np.linalg.norm(f64(o16))
    assert rel < 0.15


@pytest.mark.parametrize("heads", [5, 64, 67, 258])
def test_fp8_every_head_is_computed_for_any_head_count(heads):
    """Same dispatch order as the bf16 kernel: random labels, more heads than the 64 a label ballot
    covers; every output row finite, two heads against the oracle."""
    cfg, sh, g = setup("mid128", H=heads, spatial_heads=[])
    q, k, v = make_qkv(cfg)
    rng = np.random.default_rng(heads)
    lab_np = rng.integers(0, 2, size=heads).astype(np.uint8)
    labels = torch.from_numpy(lab_np).cuda()
    o = gpu_layer_fp8(sh, q.cuda(), k.cuda(), v.cuda(), labels)
    assert torch.isfinite(o.float()).all()
    vmax = float(np.abs(f64(v)).max())
    g1 = O.Geometry(**{**g.__dict__, "H": 1})
    for h in (0, heads - 1):
        ref = O.svg_attention_layer_fp8(f64(q[:, h:h + 1]), f64(k[:, h:h + 1]), f64(v[:, h:h + 1]),
                                        lab_np[h:h + 1].reshape(1, 1), g1)
        assert_fp8_attn_close(o[0, h], ref[0, 0], vmax, f"fp8 H={heads} head {h}")


def test_fp8_without_labels_uses_the_spatial_list_in_token_order():
    cfg, sh, g = setup("mid128")
    q, k, v = make_qkv(cfg)
    o = gpu_layer_fp8(sh, q.cuda(), k.cuda(), v.cuda(), None)
    ref = O.svg_attention_layer_fp8(f64(q), f64(k), f64(v), np.zeros((g.B, g.H), np.uint8), g)
    vmax = float(np.abs(f64(v)).max())
    for h in range(g.H):
        assert_fp8_attn_close(o[0, h], ref[0, h], vmax, f"fp8 no labels h{h}")


@pytest.mark.parametrize("geo", [
    dict(F=1, P=200, T=0),                  # one frame, no text
    dict(F=9, P=1, T=3),                    # one token per frame
    dict(F=2, P=5, T=0),                    # N = 10, smaller than any tile
    dict(F=3, P=64, T=64, text_first=0),    # tile-aligned everything
    dict(F=4, P=33, T=1, text_first=0, sink_first_frame=1),
    dict(F=5, P=77, T=130, text_first=1, w_t=5),
])
def test_fp8_degenerate_geometries(geo):
    base = dict(get_config("mid128"), B=1, H=2, w_s=1, w_t=2, text_first=1, sink_first_frame=0, spatial_heads=[0])
    base.update(geo)
    base["N"] = base["F"] * base["P"] + base["T"]
    sh, g = S.shape_from_config(base), O.Geometry.from_config(base)
    q, k, v = make_plain_qkv(1, 2, g.N, g.D, seed=31)
    lab = torch.tensor([0, 1], dtype=torch.uint8, device="cuda")
    o = gpu_layer_fp8(sh, q.cuda(), k.cuda(), v.cuda(), lab)
    ref = O.svg_attention_layer_fp8(f64(q), f64(k), f64(v), np.array([[0, 1]]), g)
    vmax = float(np.abs(f64(v)).max())
    for h in range(2):
        assert_fp8_attn_close(o[0, h], ref[0, h], vmax, f"{geo} head {h}")


def test_fp8_large_logits_and_zero_head():
    """Sharp rows (|logit| ~ 60) stay finite; an all-zero v head gives zeros (scale 1).
    With rows this sharp nearly all weight sits on one key and a single differing code can
    change which key that is, so the comparison is only meaningful when the codes are not in
    question: q and k are snapped to E4M3 values times 2^-4 with the largest magnitude 28 =
    448 * 2^-4, which both sides quantise without any rounding."""
    cfg, sh, g = setup("mid128")
    q, k, v = make_plain_qkv(g.B, g.H, g.N, g.D, seed=5)

    def snap(x):
        y = O.e4m3_decode(O.e4m3_encode(np.clip(f64(x) * 6.0, -28.0, 28.0) * 16.0)) / 16.0
        y[:, :, 0, 0] = 28.0
        return torch.from_numpy(y).to(torch.bfloat16)

    q, k = snap(q), snap(k)
    for x in (q, k):        # lossless by construction: the oracle's quantiser reproduces them
        codes, scale = O.fp8_quantize_head(f64(x)[0, 0])
        assert scale == 2.0 ** -4 and np.array_equal(O.fp8_dequantize(codes, scale), f64(x)[0, 0])
    v[0, 1] = 0
    lab_np = planted_labels(cfg)
    labels = torch.from_numpy(lab_np).cuda()
    o = gpu_layer_fp8(sh, q.cuda(), k.cuda(), v.cuda(), labels)
    assert torch.isfinite(o.float()).all() and not o[0, 1].any()
    ref = O.svg_attention_layer_fp8(f64(q), f64(k), f64(v), lab_np.reshape(g.B, g.H), g)
    # sharp rows put nearly all weight on one key, whose weight is exactly 256 * 1.0: the
    # result is close to the oracle again
    vmax = float(np.abs(f64(v)).max())
    for h in (0, 2, 3):
        assert_fp8_attn_close(o[0, h], ref[0, h], vmax, f"sharp rows head {h}")


def test_fp8_rejects_other_shapes():
    sh = S.shape_from_config(get_config("mid64"))
    assert S.svg_fp8_buffer_bytes(sh, S.SVG_FP8_Q) == 0
    x = torch.zeros(64, dtype=torch.uint8, device="cuda")
    with pytest.raises(S.SvgError):
        S.svg_fp8_quantize(sh, x, x, x, None, x, x, x, x)
    sh = S.shape_from_config(get_config("tiny"))
    with pytest.raises(S.SvgError):
        S.svg_sparse_attn_fp8_fwd(sh, x, x, x, x, x, None, x, x, None, None)


def test_fp8_full_size_sampled_tiles():
    """HunyuanVideo shape, the launch configuration bench.py times: sampled query tiles of a
    spatial and a temporal head against the oracle over the quantised head."""
    cfg = get_config("hunyuan_skip85")
    g = O.Geometry.from_config(cfg)
    sh = S.shape_from_config(cfg)
    q, k, v = make_qkv(cfg, device="cuda")
    lab_np = planted_labels(cfg)
    labels = torch.from_numpy(lab_np).cuda()
    o = gpu_layer_fp8(sh, q, k, v, labels)
    nq, nk = O.n_tiles(g)
    tiles = sorted({0, (g.off + g.P) // g.block_m, nq // 2, nq - 2, nq - 1})
    perm = O.layout_perm(g)
    for h in (0, 1):
        pat = int(lab_np[h])
        d = []
        for x in (q, k, v):
            codes, scale = O.fp8_quantize_head(f64(x[0, h]))
            d.append(O.fp8_dequantize(codes, scale))
        qh, kh, vh = d
        if pat == O.TEMPORAL:
            qh, kh, vh = O.layout_fwd(qh, g), O.layout_fwd(kh, g), O.layout_fwd(vh, g)
        rp = np.zeros(nq + 1, dtype=np.int64)
        cols = []
        for a in range(nq):
            c = O.kept_tiles_of_row(g, pat, a) if a in tiles else np.zeros(0, np.int32)
            cols.append(c)
            rp[a + 1] = rp[a] + len(c)
        ref = O.sparse_attention_head(qh, kh, vh, rp, np.concatenate(cols), g, q_tiles=tiles)
        got = f64(o[0, h])
        if pat == O.TEMPORAL:
            got = O.layout_fwd(got, g)         # compare in the order the tile list refers to
        vmax = float(np.abs(vh).max())
        for a in tiles:
            r0, r1 = a * g.block_m, min(g.N, (a + 1) * g.block_m)
            assert_fp8_attn_close(torch.from_numpy(got[r0:r1]), ref[r0:r1], vmax, f"fp8 full size head {h} tile {a}")


def test_fp8_batch_of_two_and_empty_list_rows():
    """B = 2 (head index runs over batch and head), and a query tile whose list row is empty."""
    cfg = dict(get_config("mid128"), B=2, H=3, spatial_heads=[0, 2])
    cfg["N"] = cfg["F"] * cfg["P"] + cfg["T"]
    sh, g = S.shape_from_config(cfg), O.Geometry.from_config(cfg)
    q, k, v = make_plain_qkv(g.B, g.H, g.N, g.D, seed=77)
    lab_np = planted_labels(cfg)
    labels = torch.from_numpy(lab_np).cuda()
    o = gpu_layer_fp8(sh, q.cuda(), k.cuda(), v.cuda(), labels)
    ref = O.svg_attention_layer_fp8(f64(q), f64(k), f64(v), lab_np.reshape(g.B, g.H), g)
    vmax = float(np.abs(f64(v)).max())
    for b in range(g.B):
        for h in range(g.H):
            assert_fp8_attn_close(o[b, h], ref[b, h], vmax, f"fp8 batch b{b} h{h}")
    # spatial list with the row of query tile 1 emptied, every head spatial
    rp, ci = O.tile_list(g, 0)
    rp2 = rp.copy()
    rp2[2:] -= rp[2] - rp[1]
    ci2 = np.concatenate([ci[:rp[1]], ci[rp[2]:]])
    q8, k8, v8t, scales = gpu_fp8_quantize(sh, q.cuda(), k.cuda(), v.cuda(), None)
    o2 = torch.full_like(o, 7.0)
    S.svg_sparse_attn_fp8_fwd(sh, q8, k8, v8t, scales, o2, None, torch.from_numpy(rp2).cuda(),
                              torch.from_numpy(ci2).cuda(), None, None)
    torch.cuda.synchronize()
    assert (o2[:, :, 128:256] == 0).all() and torch.isfinite(o2.float()).all()
    full = gpu_layer_fp8(sh, q.cuda(), k.cuda(), v.cuda(), None)
    assert torch.equal(o2[:, :, :128], full[:, :, :128]) and torch.equal(o2[:, :, 256:], full[:, :, 256:])
