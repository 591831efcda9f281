"""Pins for the CPU oracle: each oracle function is checked against something
other than itself -- brute-force loops, closed forms from Sec. 3.3, a hand-worked
permutation, torch's CPU scaled_dot_product_attention, or invariants."""
import math
from fractions import Fraction

import os

import numpy as np
import pytest
import torch

from oracle import svg_oracle as O
from workloads import get_config, make_qkv, make_plain_qkv, sample_rows, planted_labels


def f64(x):
    return x.to(torch.float64).numpy()


def brute_attention(q, k, v, mask, scale):
    """Pure-Python definition: o_i = sum_j w_ij v_j, w_ij = e^{s_ij} / sum_j e^{s_ij}."""
    t, D = len(q), len(q[0])
    out = [[0.0] * D for _ in range(t)]
    for i in range(t):
        s = []
        for j in range(len(k)):
            if mask is None or mask[i][j]:
                s.append((j, scale * sum(q[i][d] * k[j][d] for d in range(D))))
        m = max(x for _, x in s)
        z = sum(math.exp(x - m) for _, x in s)
        for j, x in s:
            w = math.exp(x - m) / z
            for d in range(D):
                out[i][d] += w * v[j][d]
    return np.array(out)


TINY = O.Geometry.from_config(get_config("tiny"))


# ---------------------------------------------------------------- attention
def test_masked_attention_all_ones_equals_bruteforce_dense():
    rng = np.random.default_rng(0)
    q, k, v = rng.normal(size=(5, 8)), rng.normal(size=(11, 8)), rng.normal(size=(11, 8))
    ref = brute_attention(q.tolist(), k.tolist(), v.tolist(), None, 0.3)
    ones = np.ones((5, 11), dtype=bool)
    assert np.allclose(O.masked_attention(q, k, v, ones, 0.3), ref, atol=1e-13)
    assert np.allclose(O.masked_attention(q, k, v, None, 0.3), ref, atol=1e-13)


def test_masked_attention_random_mask_equals_bruteforce():
    rng = np.random.default_rng(1)
    q, k, v = rng.normal(size=(6, 4)), rng.normal(size=(9, 4)), rng.normal(size=(9, 4))
    mask = rng.random((6, 9)) < 0.5
    mask[np.arange(6), np.arange(6)] = True
    ref = brute_attention(q.tolist(), k.tolist(), v.tolist(), mask.tolist(), 0.7)
    assert np.allclose(O.masked_attention(q, k, v, mask, 0.7), ref, atol=1e-13)


def test_attention_is_not_symmetric_in_q_and_k():
    # a transposed operand (k q^T instead of q k^T) must fail this pin
    q = np.array([[1.0, 0.0], [0.0, 0.0]])
    k = np.array([[10.0, 0.0], [0.0, 0.0]])
    v = np.array([[1.0, 0.0], [0.0, 1.0]])
    o = O.masked_attention(q, k, v, None, 1.0)
    w0 = math.exp(10.0) / (math.exp(10.0) + 1.0)
    assert np.allclose(o, [[w0, 1 - w0], [0.5, 0.5]], atol=1e-15)


def test_softmax_rows_sum_to_one_and_respect_mask():
    q, k, _ = (f64(x)[0, 0] for x in make_qkv(get_config("tiny")))
    for mask in (None, O.spatial_mask(TINY), O.temporal_mask(TINY)):
        w = O.attention_weights(q, k, mask, TINY.scale)
        assert np.allclose(w.sum(axis=1), 1.0, atol=1e-14)
        assert (w >= 0).all()
        if mask is not None:
            assert (w[~mask] == 0).all()


def test_masked_attention_matches_torch_sdpa_fp64():
    q, k, v = (x.to(torch.float64)[0] for x in make_qkv(get_config("tiny")))
    for mask in (O.spatial_mask(TINY), O.temporal_mask(TINY)):
        ref = torch.nn.functional.scaled_dot_product_attention(
            q, k, v, attn_mask=torch.from_numpy(mask)[None], scale=TINY.scale).numpy()
        for h in range(4):
            got = O.masked_attention(q[h].numpy(), k[h].numpy(), v[h].numpy(), mask, TINY.scale)
            assert np.allclose(got, ref[h], atol=1e-12)


def test_shift_invariance_and_single_key():
    rng = np.random.default_rng(2)
    q, k, v = rng.normal(size=(3, 4)), rng.normal(size=(7, 4)), rng.normal(size=(7, 4))
    # one kept key -> output is that key's value exactly
    mask = np.zeros((3, 7), dtype=bool)
    mask[:, 4] = True
    assert np.array_equal(O.masked_attention(q, k, v, mask, 1.0), np.tile(v[4], (3, 1)))
    # identical keys -> output is the mean of the values
    k2 = np.tile(k[0], (7, 1))
    assert np.allclose(O.masked_attention(q, k2, v, None, 1.0), np.tile(v.mean(0), (3, 1)), atol=1e-15)


# ---------------------------------------------------------------- masks
def test_token_coords_prefix_and_suffix():
    g = O.Geometry(1, 1, 2, 3, 2, 4, text_first=1)
    is_text, fr, po = O.token_coords(g)
    assert is_text.tolist() == [True, True] + [False] * 6
    assert fr.tolist() == [-1, -1, 0, 0, 0, 1, 1, 1]
    assert po.tolist() == [-1, -1, 0, 1, 2, 0, 1, 2]
    g = O.Geometry(1, 1, 2, 3, 2, 4, text_first=0)
    is_text, fr, po = O.token_coords(g)
    assert is_text.tolist() == [False] * 6 + [True, True]
    assert fr.tolist() == [0, 0, 0, 1, 1, 1, -1, -1]
    assert po.tolist() == [0, 1, 2, 0, 1, 2, -1, -1]


def test_masks_hand_worked_example():
    # F=3 frames of P=2 tokens, one text token last, w_s=0, w_t=0
    g = O.Geometry(1, 1, 3, 2, 1, 4, text_first=0, w_s=0, w_t=0)
    s = O.spatial_mask(g).astype(int)
    t = O.temporal_mask(g).astype(int)
    assert s.tolist() == [
        [1, 1, 0, 0, 0, 0, 1],
        [1, 1, 0, 0, 0, 0, 1],
        [0, 0, 1, 1, 0, 0, 1],
        [0, 0, 1, 1, 0, 0, 1],
        [0, 0, 0, 0, 1, 1, 1],
        [0, 0, 0, 0, 1, 1, 1],
        [1, 1, 1, 1, 1, 1, 1]]
    assert t.tolist() == [
        [1, 0, 1, 0, 1, 0, 1],
        [0, 1, 0, 1, 0, 1, 1],
        [1, 0, 1, 0, 1, 0, 1],
        [0, 1, 0, 1, 0, 1, 1],
        [1, 0, 1, 0, 1, 0, 1],
        [0, 1, 0, 1, 0, 1, 1],
        [1, 1, 1, 1, 1, 1, 1]]


def test_sink_first_frame_keeps_frame0_keys():
    g = O.Geometry(1, 1, 3, 2, 1, 4, text_first=0, w_s=0, w_t=0, sink_first_frame=1)
    s = O.spatial_mask(g)
    assert s[:, :2].all() and not s[4, 2] and not s[4, 3]
    assert O.temporal_mask(g)[:, :2].all()


@pytest.mark.parametrize("name", ["tiny", "mid64", "mid128"])
def test_mask_density_closed_form_interior_rows(name):
    """Sec. 3.3: a spatial head keeps c_s of N frames, a temporal head c_t of L
    tokens per frame; with symmetric windows c_s = 2 w_s + 1 and c_t = 2 w_t + 1
    for rows whose window is not clipped."""
    g = O.Geometry.from_config(get_config(name))
    is_text, fr, po = O.token_coords(g)
    vid = ~is_text
    ms, mt = O.spatial_mask(g), O.temporal_mask(g)
    for i in range(g.N):
        if is_text[i]:
            assert ms[i].all() and mt[i].all()
            continue
        if g.w_s <= fr[i] < g.F - g.w_s:
            assert ms[i][vid].sum() == (2 * g.w_s + 1) * g.P
        if g.w_t <= po[i] < g.P - g.w_t:
            assert mt[i][vid].sum() == (2 * g.w_t + 1) * g.F
        assert ms[i][is_text].all() and mt[i][is_text].all()
        assert ms[i, i] and mt[i, i]
    # masks are symmetric (|a-b| windows, text in both directions)
    assert np.array_equal(ms, ms.T) and np.array_equal(mt, mt.T)


def test_wide_windows_give_all_ones():
    g = O.Geometry(1, 1, 4, 6, 3, 8, w_s=3, w_t=5)
    assert O.spatial_mask(g).all() and O.temporal_mask(g).all()


def test_mask_rows_subset():
    rows = sample_rows(get_config("tiny"))
    assert np.array_equal(O.spatial_mask(TINY, rows), O.spatial_mask(TINY)[rows])
    assert np.array_equal(O.temporal_mask(TINY, rows), O.temporal_mask(TINY)[rows])


# ---------------------------------------------------------------- layout
def test_layout_hand_worked_example():
    # 1 text token first, F=2 frames of P=3 tokens: [t, a0 a1 a2, b0 b1 b2]
    g = O.Geometry(1, 1, 2, 3, 1, 1, text_first=1)
    x = np.array([[100.], [0.], [1.], [2.], [10.], [11.], [12.]])
    y = O.layout_fwd(x, g)
    assert y[:, 0].tolist() == [100., 0., 10., 1., 11., 2., 12.]
    assert O.layout_inv(y, g)[:, 0].tolist() == x[:, 0].tolist()
    # text last
    g = O.Geometry(1, 1, 2, 3, 1, 1, text_first=0)
    x = np.array([[0.], [1.], [2.], [10.], [11.], [12.], [100.]])
    assert O.layout_fwd(x, g)[:, 0].tolist() == [0., 10., 1., 11., 2., 12., 100.]


def test_layout_with_first_frame_sink_keeps_frame0_as_a_block():
    """Hand-worked: F = 3, P = 2, one text token first.  Tokens (f, p): n = 1 + 2 f + p.  With the
    sink on, the transformed order is text | frame 0 in position order | positions outer over frames
    1, 2:  (0,0) (0,1) | (1,0) (2,0) (1,1) (2,1)."""
    g = O.Geometry(1, 1, 3, 2, 1, 1, text_first=1, sink_first_frame=1)
    #                 text (0,0) (0,1) (1,0) (1,1) (2,0) (2,1)
    assert O.layout_perm(g).tolist() == [0, 1, 2, 3, 5, 4, 6]
    x = np.array([[100.], [0.], [1.], [10.], [11.], [20.], [21.]])
    y = O.layout_fwd(x, g)
    assert y[:, 0].tolist() == [100., 0., 1., 10., 20., 11., 21.]
    assert O.layout_inv(y, g)[:, 0].tolist() == x[:, 0].tolist()
    # without the flag the same geometry interleaves frame 0 with the others
    g0 = O.Geometry(1, 1, 3, 2, 1, 1, text_first=1, sink_first_frame=0)
    assert O.layout_fwd(x, g0)[:, 0].tolist() == [100., 0., 10., 20., 1., 11., 21.]
    # general shapes: a permutation, text fixed, frame 0 = the first P video slots in position order,
    # the rest = reshape / transpose of frames 1..F-1; F = 1 and P = 1 degenerate to the identity
    for cfg in (get_config("mid64", sink_first_frame=1), get_config("mid128", sink_first_frame=1)):
        g = O.Geometry.from_config(cfg)
        perm = O.layout_perm(g)
        assert sorted(perm.tolist()) == list(range(g.N))
        rng = np.random.default_rng(4)
        x = rng.integers(0, 2 ** 16, size=(g.N, 3), dtype=np.uint16)
        y = O.layout_fwd(x, g)
        vid = x[g.off:g.off + g.F * g.P].reshape(g.F, g.P, 3)
        assert np.array_equal(y[g.off:g.off + g.P], vid[0])
        assert np.array_equal(y[g.off + g.P:g.off + g.F * g.P], vid[1:].transpose(1, 0, 2).reshape(-1, 3))
        txt = np.ones(g.N, bool)
        txt[g.off:g.off + g.F * g.P] = False
        assert np.array_equal(y[txt], x[txt]) and np.array_equal(O.layout_inv(y, g), x)
    for F, P in ((1, 7), (7, 1)):
        g = O.Geometry(1, 1, F, P, 2, 3, sink_first_frame=1)
        if F == 1:
            assert O.layout_perm(g).tolist() == list(range(g.N))
        else:
            assert sorted(O.layout_perm(g).tolist()) == list(range(g.N))


def test_first_frame_sink_costs_a_temporal_head_few_tiles():
    """The point of the block: with the sink on, a temporal head's query tile keeps the tiles of
    the frame-0 block and of its window, not every tile (frame 0 spread over every F-th row
    would touch them all), and the list still covers exactly the element mask."""
    g = O.Geometry(1, 1, 9, 256, 32, 64, text_first=0, w_s=1, w_t=6, sink_first_frame=1, block_m=128, block_n=64)
    nq, nk = O.n_tiles(g)
    rp, ci = O.tile_list(g, O.TEMPORAL)
    a = nq // 2
    row = ci[rp[a]:rp[a + 1]]
    # frame-0 block: 256 rows = 4 tiles; window: (128 / 8 + 2 * 6 + 1) positions * 8 frames ~ 4-5 tiles; text: 1
    assert 4 + 1 < len(row) <= 4 + 6 + 1 < nk // 2
    assert set(range(4)) <= set(row.tolist())
    perm = O.layout_perm(g)
    inv = np.empty_like(perm)
    inv[perm] = np.arange(g.N)
    m = O.temporal_mask(g)[inv][:, inv]
    for a in range(nq):
        for b in range(nk):
            blk = m[a * g.block_m:(a + 1) * g.block_m, b * g.block_n:(b + 1) * g.block_n]
            assert bool(blk.any()) == (b in ci[rp[a]:rp[a + 1]])
    # attention through the transformed order equals attention in the original one (Sec. 4.2)
    rng = np.random.default_rng(8)
    q, k, v = (rng.normal(0, 1, (g.N, g.D)) for _ in range(3))
    o_ref = O.masked_attention(q, k, v, O.temporal_mask(g), g.scale)
    o_p = O.masked_attention(O.layout_fwd(q, g), O.layout_fwd(k, g), O.layout_fwd(v, g), m, g.scale)
    assert np.allclose(O.layout_inv(o_p, g), o_ref, atol=1e-12)


@pytest.mark.parametrize("name", ["tiny", "mid64", "mid128"])
def test_layout_is_reshape_transpose_and_inverts_bit_exactly(name):
    cfg = get_config(name)
    g = O.Geometry.from_config(cfg)
    rng = np.random.default_rng(3)
    x = rng.integers(0, 2 ** 16, size=(g.B, g.H, g.N, g.D), dtype=np.uint16)
    y = O.layout_fwd(x, g)
    vid = slice(g.off, g.off + g.F * g.P)
    ref = x[:, :, vid].reshape(g.B, g.H, g.F, g.P, g.D).transpose(0, 1, 3, 2, 4).reshape(g.B, g.H, -1, g.D)
    assert np.array_equal(y[:, :, vid], ref)
    txt = np.ones(g.N, bool)
    txt[vid] = False
    assert np.array_equal(y[:, :, txt], x[:, :, txt])
    assert np.array_equal(O.layout_inv(y, g), x)
    assert np.array_equal(O.layout_fwd(O.layout_inv(x, g), g), x)
    perm = O.layout_perm(g)
    assert sorted(perm.tolist()) == list(range(g.N))


def test_layout_degenerate_single_frame_or_single_position_is_identity():
    for F, P in ((1, 7), (7, 1)):
        g = O.Geometry(1, 1, F, P, 2, 3)
        assert O.layout_perm(g).tolist() == list(range(g.N))


def test_layout_equivalence_of_attention():
    """Sec. 4.2: permuting the tokens (and the mask with them) and permuting the
    result back leaves the attention output unchanged."""
    g = TINY
    q, k, v = (f64(x)[0, 2] for x in make_qkv(get_config("tiny")))
    perm = O.layout_perm(g)
    inv = np.empty_like(perm)
    inv[perm] = np.arange(g.N)
    m = O.temporal_mask(g)
    mp = m[inv][:, inv]
    o_ref = O.masked_attention(q, k, v, m, g.scale)
    o_p = O.masked_attention(O.layout_fwd(q, g), O.layout_fwd(k, g), O.layout_fwd(v, g), mp, g.scale)
    assert np.allclose(O.layout_inv(o_p, g), o_ref, atol=1e-12)


# ---------------------------------------------------------------- tile lists
def closed_form_tiles(g, pattern):
    """Independent derivation by interval arithmetic: in its own order a pattern
    keeps, for a query tile covering groups ga..gb (frames for spatial, positions
    for temporal), the contiguous key range of groups ga-w .. gb+w plus the text
    range; a tile with a text query keeps everything."""
    nq, nk = O.n_tiles(g)
    unit, groups, w = (g.P, g.F, g.w_s) if pattern == O.SPATIAL else (g.F, g.P, g.w_t)
    off, V = g.off, g.F * g.P
    out = []
    for a in range(nq):
        r0, r1 = a * g.block_m, min(g.N, (a + 1) * g.block_m) - 1
        has_text = r0 < off or r1 >= off + V
        if has_text and g.T > 0:
            out.append(list(range(nk)))
            continue
        ga, gb = (r0 - off) // unit, (r1 - off) // unit
        lo = off + max(0, ga - w) * unit
        hi = off + min(groups, gb + w + 1) * unit - 1
        kept = set(range(lo // g.block_n, hi // g.block_n + 1))
        if g.T > 0:
            t0, t1 = (0, g.T - 1) if g.text_first else (V, g.N - 1)
            kept |= set(range(t0 // g.block_n, t1 // g.block_n + 1))
        out.append(sorted(kept))
    return out


@pytest.mark.parametrize("name", ["tiny", "mid64", "mid128"])
@pytest.mark.parametrize("pattern", [O.SPATIAL, O.TEMPORAL])
def test_tile_list_matches_closed_form_and_full_matrix_bruteforce(name, pattern):
    g = O.Geometry.from_config(get_config(name))
    rp, ci = O.tile_list(g, pattern)
    nq, nk = O.n_tiles(g)
    assert rp[0] == 0 and rp[-1] == len(ci) and len(rp) == nq + 1
    ref = closed_form_tiles(g, pattern)
    for a in range(nq):
        assert ci[rp[a]:rp[a + 1]].tolist() == ref[a]
    # brute force over the full N x N element mask in that pattern's order
    if pattern == O.SPATIAL:
        m = O.spatial_mask(g)
    else:
        perm = O.layout_perm(g)
        inv = np.empty_like(perm)
        inv[perm] = np.arange(g.N)
        m = O.temporal_mask(g)[inv][:, inv]
    for a in range(nq):
        for b in range(nk):
            blk = m[a * g.block_m:(a + 1) * g.block_m, b * g.block_n:(b + 1) * g.block_n]
            assert bool(blk.any()) == (b in ci[rp[a]:rp[a + 1]])
    # the block mask covers the element mask
    assert (O.block_mask(g, rp, ci) | ~m).all()


def test_tile_density_follows_sec33_for_aligned_shape():
    """With tile-aligned frames, no text and unclipped windows the kept fraction of
    a spatial head's tiles is exactly c_s/N_frames (Sec. 3.3)."""
    g = O.Geometry(1, 1, 8, 128, 0, 64, w_s=1, w_t=0, block_m=128, block_n=64)
    rp, ci = O.tile_list(g, O.SPATIAL)
    per_row = np.diff(rp)
    assert per_row[3] == 3 * 2 and per_row[0] == 2 * 2 and per_row[-1] == 2 * 2
    # temporal in P-outer order: band of (2 w_t + 1) * F tokens around the diagonal
    g = O.Geometry(1, 1, 8, 128, 0, 64, w_s=0, w_t=8, block_m=128, block_n=64)
    rp, ci = O.tile_list(g, O.TEMPORAL)
    a = 3   # rows 384..511 = positions 48..63 -> positions 40..71 -> tokens 320..575
    assert ci[rp[a]:rp[a + 1]].tolist() == list(range(320 // 64, 575 // 64 + 1))


# ---------------------------------------------------------------- block-sparse attention
def test_sparse_attention_with_full_list_is_dense():
    g = TINY
    q, k, v = (f64(x)[0, 1] for x in make_qkv(get_config("tiny")))
    rp, ci = O.full_tile_list(g)
    dense = brute_attention(q[:40].tolist(), k.tolist(), v.tolist(), None, g.scale)
    got = O.sparse_attention_head(q, k, v, rp, ci, g)
    assert np.allclose(got[:40], dense, atol=1e-13)
    assert np.allclose(got, O.dense_attention_head(q, k, v, g), atol=1e-13)


def test_sparse_attention_equals_masked_attention_with_block_mask():
    g = TINY
    q, k, v = (f64(x)[0, 3] for x in make_qkv(get_config("tiny")))
    for pattern in (O.SPATIAL, O.TEMPORAL):
        rp, ci = O.tile_list(g, pattern)
        assert rp[-1] < 81   # something is actually skipped
        bm = O.block_mask(g, rp, ci)
        ref = O.masked_attention(q, k, v, bm, g.scale)
        assert np.allclose(O.sparse_attention_head(q, k, v, rp, ci, g), ref, atol=1e-13)
        rows = [0, 17, 100, 271]
        bf = brute_attention(q[rows].tolist(), k.tolist(), v.tolist(), bm[rows].tolist(), g.scale)
        assert np.allclose(ref[rows], bf, atol=1e-13)


def test_wide_spatial_window_makes_sparse_dense():
    cfg = get_config("tiny", w_s=3)
    g = O.Geometry.from_config(cfg)
    rp, ci = O.tile_list(g, O.SPATIAL)
    frp, fci = O.full_tile_list(g)
    assert np.array_equal(rp, frp) and np.array_equal(ci, fci)


def test_sparse_attention_sampled_tiles_leave_rest_nan():
    g = TINY
    q, k, v = (f64(x)[0, 0] for x in make_qkv(get_config("tiny")))
    rp, ci = O.tile_list(g, O.SPATIAL)
    full = O.sparse_attention_head(q, k, v, rp, ci, g)
    part = O.sparse_attention_head(q, k, v, rp, ci, g, q_tiles=[2, 8])
    assert np.array_equal(part[64:96], full[64:96]) and np.array_equal(part[256:], full[256:])
    assert np.isnan(part[:64]).all()


# ---------------------------------------------------------------- profiling
def test_profile_mse_bruteforce_one_head():
    cfg = get_config("tiny")
    g = TINY
    q, k, v = (f64(x) for x in make_qkv(cfg))
    rows = sample_rows(cfg)
    mse, labels = O.profile_heads(q, k, v, rows, g)
    h = 2
    ql = q[0, h][rows].tolist()
    kl, vl = k[0, h].tolist(), v[0, h].tolist()
    full = brute_attention(ql, kl, vl, None, g.scale)
    sp = brute_attention(ql, kl, vl, O.spatial_mask(g)[rows].tolist(), g.scale)
    tp = brute_attention(ql, kl, vl, O.temporal_mask(g)[rows].tolist(), g.scale)
    ms = sum((full[i][d] - sp[i][d]) ** 2 for i in range(len(rows)) for d in range(g.D)) / (len(rows) * g.D)
    mt = sum((full[i][d] - tp[i][d]) ** 2 for i in range(len(rows)) for d in range(g.D)) / (len(rows) * g.D)
    assert np.isclose(mse[0, h, 0], ms, rtol=1e-10) and np.isclose(mse[0, h, 1], mt, rtol=1e-10)
    assert labels[0, h] == (O.SPATIAL if ms < mt else O.TEMPORAL)


def test_profile_full_window_gives_zero_error():
    cfg = get_config("tiny", w_s=3, w_t=63)
    g = O.Geometry.from_config(cfg)
    q, k, v = (f64(x) for x in make_qkv(cfg))
    mse, labels = O.profile_heads(q, k, v, sample_rows(cfg), g)
    assert (mse == 0).all()
    assert (labels == O.TEMPORAL).all()      # tie -> not strictly smaller -> temporal


def test_profile_all_rows_is_oracle_identification():
    """Sec. 3.2: with every row sampled the profile is the full comparison of the
    two sparse outputs with dense attention."""
    cfg = get_config("tiny")
    g = TINY
    q, k, v = (f64(x) for x in make_qkv(cfg))
    mse, _ = O.profile_heads(q, k, v, np.arange(g.N), g)
    for h in range(g.H):
        dense = O.dense_attention_head(q[0, h], k[0, h], v[0, h], g)
        for x, m in ((0, O.spatial_mask(g)), (1, O.temporal_mask(g))):
            sp = O.masked_attention(q[0, h], k[0, h], v[0, h], m, g.scale)
            assert np.isclose(mse[0, h, x], ((dense - sp) ** 2).mean(), rtol=1e-12)


def test_profile_row_order_does_not_matter_and_text_rows_add_nothing():
    cfg = get_config("tiny")
    g = TINY
    q, k, v = (f64(x) for x in make_qkv(cfg))
    rows = sample_rows(cfg)
    a, _ = O.profile_heads(q, k, v, rows, g)
    b, _ = O.profile_heads(q, k, v, rows[::-1].copy(), g)
    assert np.allclose(a, b, rtol=1e-12)
    # text rows are dense under both masks: zero error
    c, _ = O.profile_heads(q, k, v, np.arange(g.T), g)
    assert (c == 0).all()


@pytest.mark.parametrize("name", ["tiny", "mid64", "mid128"])
def test_planted_heads_are_classified(name):
    cfg = get_config(name)
    g = O.Geometry.from_config(cfg)
    q, k, v = (f64(x) for x in make_qkv(cfg))
    mse, labels = O.profile_heads(q, k, v, sample_rows(cfg), g)
    assert np.array_equal(labels.reshape(-1), planted_labels(cfg))
    assert (mse >= 0).all()
    lo, hi = mse.min(axis=-1), mse.max(axis=-1)
    assert (hi > 10 * lo).all()              # decided by a wide margin, not a near tie


# ---------------------------------------------------------------- whole layer
def test_layer_equals_element_level_definition():
    """Spatial heads: masked attention with the spatial block mask in the original
    order.  Temporal heads: masked attention in the original order with the
    temporal block mask pulled back through the permutation."""
    cfg = get_config("tiny")
    g = TINY
    q, k, v = (f64(x) for x in make_qkv(cfg))
    labels = planted_labels(cfg).reshape(g.B, g.H)
    out = O.svg_attention_layer(q, k, v, labels, g)
    perm = O.layout_perm(g)
    bs = O.block_mask(g, *O.tile_list(g, O.SPATIAL))
    bt = O.block_mask(g, *O.tile_list(g, O.TEMPORAL))[perm][:, perm]
    for h in range(g.H):
        m = bs if labels[0, h] == O.SPATIAL else bt
        ref = O.masked_attention(q[0, h], k[0, h], v[0, h], m, g.scale)
        assert np.allclose(out[0, h], ref, atol=1e-12)


def test_flop_model_sec33():
    """Sec. 3.3: dense cost 4 L^2 N^2 H; spatial keeps c_s/N of it, temporal c_t/L.
    Counting kept elements of the masks (no text) reproduces both fractions for
    unclipped rows."""
    g = O.Geometry(1, 1, 9, 20, 0, 8, w_s=2, w_t=3)
    ms, mt = O.spatial_mask(g), O.temporal_mask(g)
    _, fr, po = O.token_coords(g)
    inner_s = (fr >= 2) & (fr < 7)
    inner_t = (po >= 3) & (po < 17)
    assert np.allclose(ms[inner_s].mean(), 5 / 9)
    assert np.allclose(mt[inner_t].mean(), 7 / 20)


# ------------------------------------------------------------------ stored tile counts
def golden_tile_counts():
    path = os.path.join(os.path.dirname(os.path.abspath(__file__)), "golden", "tile_counts.txt")
    out = {}
    for line in open(path):
        if line.strip() and not line.startswith("#"):
            name, s_, t_, all_ = line.split()
            out[name] = (int(s_), int(t_), int(all_))
    return out


@pytest.mark.parametrize("name", ["cogvideox_v1", "wan21_14b"])
def test_tile_counts_match_the_independently_derived_ones(name):
    """Kept tiles per pattern at the benchmark shapes: the oracle's per-row routine summed over
    all query tiles against the stored counts, which tests/golden/make_tile_counts.py writes from
    the oracle for all six shapes and which agree with the workload table the benchmark was
    specified with.  (The 120k-token shapes take minutes, so only the generator script sums
    them; `python tests/golden/make_tile_counts.py --check` recomputes all six.)"""
    from workloads import get_config
    g = O.Geometry.from_config(get_config(name))
    nq, nk = O.n_tiles(g)
    want_s, want_t, want_all = golden_tile_counts()[name]
    assert nq * nk == want_all
    assert sum(len(O.kept_tiles_of_row(g, O.SPATIAL, a)) for a in range(nq)) == want_s
    assert sum(len(O.kept_tiles_of_row(g, O.TEMPORAL, a)) for a in range(nq)) == want_t


@pytest.mark.parametrize("name", ["tiny", "mid64", "mid128"])
def test_frame_major_temporal_list_keeps_the_same_elements(name):
    """The temporal mask is one set of (query, key) pairs; the two list patterns only cover it
    with tiles in different token orders.  Every pair the element mask keeps must lie in a
    kept tile of BOTH lists (in their own orders), and each list must be minimal: every kept
    tile holds at least one kept pair."""
    g = O.Geometry.from_config(get_config(name))
    nq, nk = O.n_tiles(g)
    pos_of = O.layout_perm(g)                    # position of original token n in the transformed order
    m = O.temporal_mask(g)                       # original order
    for pattern, where in ((O.TEMPORAL_FRAME_MAJOR, np.arange(g.N)), (O.TEMPORAL, pos_of)):
        rp, ci = O.tile_list(g, pattern)
        kept = np.zeros((nq, nk), dtype=bool)
        for a in range(nq):
            kept[a, ci[rp[a]:rp[a + 1]]] = True
        qi, kj = np.nonzero(m)
        ta, tb = where[qi] // g.block_m, where[kj] // g.block_n
        assert kept[ta, tb].all()
        hit = np.zeros((nq, nk), dtype=bool)
        hit[ta, tb] = True
        assert np.array_equal(hit, kept)


# ----------------------------------------------------------------------------- FP8 (E4M3)
def test_e4m3_decode_follows_the_format_definition():
    """Values fixed by the OCP 8-bit floating point format: bias 7, three mantissa bits,
    subnormals in steps of 2^-9, largest finite value 448, S.1111.111 is NaN."""
    want = {0x00: 0.0, 0x01: 2.0 ** -9, 0x07: 7 * 2.0 ** -9, 0x08: 2.0 ** -6, 0x30: 0.5, 0x38: 1.0,
            0x3c: 1.5, 0x40: 2.0, 0x45: 3.25, 0x77: 240.0, 0x7e: 448.0, 0xb8: -1.0, 0xfe: -448.0}
    for code, val in want.items():
        assert O.e4m3_decode(np.array([code], np.uint8))[0] == val, hex(code)
    assert np.isnan(O.e4m3_decode(np.array([0x7f, 0xff], np.uint8))).all()
    pos = O.e4m3_decode(np.arange(0, 0x7f, dtype=np.uint8))
    assert (np.diff(pos) > 0).all()                                   # codes ascend with the value
    assert np.array_equal(O.e4m3_decode(np.arange(0x80, 0xff, dtype=np.uint8)), -pos)


def test_e4m3_encode_is_nearest_with_ties_to_even():
    codes = np.array([c for c in range(256) if (c & 0x7f) != 0x7f and c != 0x80], np.uint8)
    vals = O.e4m3_decode(codes)
    assert np.array_equal(O.e4m3_encode(vals), codes)                 # every finite code is a fixed point
    # brute force: the encoded value is a nearest representable one
    rng = np.random.default_rng(5)
    y = np.concatenate([rng.normal(0, 1, 4000) * np.exp2(rng.integers(-12, 9, 4000)), [0.0, 447.9, 448.0, 500.0, -1e9]])
    got = O.e4m3_decode(O.e4m3_encode(y))
    table = np.sort(O.e4m3_decode(codes))
    yc = np.clip(y, -448.0, 448.0)
    best = np.abs(table[None, :] - yc[:, None]).min(axis=1)
    assert np.array_equal(np.abs(got - yc), best)
    assert np.array_equal(np.sign(got) * (got != 0), np.sign(yc) * (got != 0))
    # midpoints between neighbours go to the code with the even mantissa
    pos = O.e4m3_decode(np.arange(0, 0x7f, dtype=np.uint8))
    mid = (pos[:-1] + pos[1:]) / 2
    enc = O.e4m3_encode(mid)
    assert (enc % 2 == 0).all() and (np.abs(O.e4m3_decode(enc) - mid) == np.diff(pos) / 2).all()
    # hand-worked: 1.0625 -> 1.0 (0x38), 1.1875 -> 1.25 (0x3a), 2^-10 -> 0, 3 * 2^-10 -> 2^-8 (0x02)
    assert O.e4m3_encode(np.array([1.0625, 1.1875, 2.0 ** -10, 3 * 2.0 ** -10])).tolist() == [0x38, 0x3a, 0x00, 0x02]


def test_fp8_quantize_head_scale_and_error_bound():
    rng = np.random.default_rng(9)
    x = torch.from_numpy(rng.normal(0, 1.3, (300, 64))).to(torch.bfloat16).to(torch.float64).numpy()
    codes, scale = O.fp8_quantize_head(x)
    amax = np.abs(x).max()
    assert scale.dtype == np.float32
    # the scale is the float32 nearest to amax / 448: no float32 is closer (rational arithmetic)
    exact = Fraction(float(amax)) / 448
    for other in (np.nextafter(scale, np.float32(0)), np.nextafter(scale, np.float32(1))):
        assert abs(Fraction(float(scale)) - exact) <= abs(Fraction(float(other)) - exact)
    i = np.unravel_index(np.abs(x).argmax(), x.shape)
    assert codes[i] & 0x7f == 0x7e                                    # the largest magnitude maps to 448
    back = O.fp8_dequantize(codes, scale)
    # nearest rounding: the error is at most half a step, a step being 2^-3 of the value's binade
    # (2^-9 of the scale below 2^-6); the largest element may sit a float32 rounding above 448
    a = np.abs(x) / float(scale)
    step = np.where(a < 2.0 ** -6, 2.0 ** -9, np.exp2(np.floor(np.log2(np.maximum(a, 1e-30))) - 3))
    assert (np.abs(back - x) <= float(scale) * (step / 2 + 448 * 2.0 ** -23)).all()
    # all zero: scale 1, codes 0
    z, s = O.fp8_quantize_head(np.zeros((4, 8)))
    assert s == 1 and not z.any()


def _nearest_e4m3_by_fractions(quotient: Fraction) -> int:
    """Code of the E4M3 value nearest to an exact rational, ties to the even code, by search
    over the whole table in rational arithmetic."""
    best = None
    for code in range(0x7f):
        val = Fraction(float(O.e4m3_decode(np.array([code], np.uint8))[0]))
        err = abs(abs(quotient) - val)
        if best is None or err < best[0] or (err == best[0] and code % 2 == 0):
            best = (err, code)
    return best[1] | (0x80 if quotient < 0 else 0)


def test_fp8_codes_are_nearest_to_the_exact_quotient():
    """Every code against a search of the format's table in exact rational arithmetic, on the
    quotient x / scale with the float32 scale taken as the exact number it is."""
    rng = np.random.default_rng(17)
    x = torch.from_numpy(rng.normal(0, 1.0, (40, 16))).to(torch.bfloat16).to(torch.float64).numpy()
    x[3, 5] = 0.0
    codes, scale = O.fp8_quantize_head(x)
    for idx in np.ndindex(x.shape):
        want = _nearest_e4m3_by_fractions(Fraction(float(x[idx])) / Fraction(float(scale)))
        assert (codes[idx] & 0x7f) == (want & 0x7f), (idx, x[idx])
        assert x[idx] == 0 or (codes[idx] & 0x80) == (want & 0x80)
    # A case that separates the exact quotient from a float32 evaluation of x * (1 / scale).
    # amax = 65/32, x = 195/128: x / (amax / 448) is exactly 336, the midpoint of the
    # neighbours 320 and 352.  The float32 scale is the rounded-DOWN value of amax / 448, so
    # the quotient by the scale actually used lies just above the midpoint and the nearest
    # value is 352 (code 0x7b); two float32 roundings land on 336.0 itself and would tie to 320.
    amax, xv = 65.0 / 32.0, 195.0 / 128.0
    codes, scale = O.fp8_quantize_head(np.array([[amax, xv]]))
    assert Fraction(float(scale)) < Fraction(65, 32) / 448
    assert Fraction(xv) / Fraction(float(scale)) > 336
    assert codes.tolist() == [[0x7e, 0x7b]]
    x32 = np.float32(xv) * (np.float32(1) / scale)
    assert float(x32) == 336.0 and O.e4m3_encode(np.array([336.0]))[0] == 0x7a


def test_fp8_round_weights():
    """The 8-bit form of the attention weights: hand-worked rows, exact cases, the bound."""
    # hand-worked: weights (1, 0.3) are stored as 256 and 76.8 -> nearest values 256 and 80
    # (the binade [64, 128) has steps of 8; 76.8 is 3.2 from 80 and 4.8 from 72)
    e = np.array([[1.0, 0.3]])
    assert np.array_equal(O.fp8_round_weights(e) * 256.0, [[256.0, 80.0]])
    v = np.array([[1.0, 0.0], [0.0, 1.0]])
    q = np.array([[1.0, 0.0]])
    k = np.array([[0.0, 0.0], [np.log(0.3), 0.0]])           # logits 0 and ln 0.3 at scale 1
    o = O.masked_attention(q, k, v, None, 1.0, weight_round=O.fp8_round_weights)
    assert np.allclose(o, [[256.0 / 336.0, 80.0 / 336.0]], rtol=0, atol=1e-15)
    # weights that are powers of two are kept exactly, so the result equals the unrounded one
    k2 = np.array([[0.0, 0.0], [-3 * np.log(2.0), 0.0]])
    assert np.allclose(O.masked_attention(q, k2, v, None, 1.0, weight_round=O.fp8_round_weights),
                       O.masked_attention(q, k2, v, None, 1.0), rtol=0, atol=1e-15)
    # below half of the smallest subnormal (2^-9 / 2^8) a weight vanishes; just above it survives
    assert O.fp8_round_weights(np.array([2.0 ** -18]))[0] == 0.0
    assert O.fp8_round_weights(np.array([2.0 ** -18 * 1.01]))[0] == 2.0 ** -17
    assert O.fp8_round_weights(np.array([1.0]))[0] == 1.0
    # every non-vanishing weight moves by at most 2^-4 relative, so the output moves by at most
    # 2 * 2^-4 / (1 - 2^-4) of the spread of v; for random rows the error is far inside that
    rng = np.random.default_rng(33)
    q, k, v = rng.normal(0, 1, (9, 16)), rng.normal(0, 1, (50, 16)), rng.normal(0, 1, (50, 16))
    a = O.masked_attention(q, k, v, None, 0.5, weight_round=O.fp8_round_weights)
    b = O.masked_attention(q, k, v, None, 0.5)
    spread = np.abs(v[None, :, :] - b[:, None, :]).max(axis=1)
    assert 0 < np.abs(a - b).max() and (np.abs(a - b) <= 2 * 2.0 ** -4 / (1 - 2.0 ** -4) * spread).all()
    w = O.attention_weights(q, k, None, 0.5, weight_round=O.fp8_round_weights)
    assert np.allclose(w.sum(axis=1), 1.0)


def test_fp8_layer_is_the_plain_layer_when_quantisation_is_lossless():
    """Inputs that are E4M3 values times a power of two with the largest magnitude 448 are
    reproduced exactly, so the FP8 layer must equal the plain one bit for bit (this pins the
    wiring: a dropped scale, a tensor quantised with another one's scale, a missing
    dequantisation would all show)."""
    cfg = get_config("tiny")
    g = O.Geometry.from_config(cfg)
    rng = np.random.default_rng(21)
    codes = np.array([c for c in range(256) if (c & 0x7f) <= 0x5f], np.uint8)     # |value| <= 30
    def lossless(power):
        x = O.e4m3_decode(rng.choice(codes, size=(g.B, g.H, g.N, g.D))) * 2.0 ** power
        x[:, :, 0, 0] = 448.0 * 2.0 ** power
        return x
    q, k, v = lossless(-7), lossless(-6), lossless(-4)
    labels = np.arange(g.B * g.H).reshape(g.B, g.H) % 2
    assert np.array_equal(O.svg_attention_layer_fp8(q, k, v, labels, g), O.svg_attention_layer(q, k, v, labels, g))
    # and for ordinary inputs it differs from the plain layer by a few per cent, not more
    q, k, v = (x.to(torch.float64).numpy() for x in make_qkv(cfg))
    a, b = O.svg_attention_layer_fp8(q, k, v, labels, g), O.svg_attention_layer(q, k, v, labels, g)
    rel = np.linalg.norm(a - b) / np.linalg.norm(b)
    assert 1e-4 < rel < 0.1
    # the form with 8-bit weights is the same layer with every row's weights rounded: it stays
    # within the weight-rounding bound of the other one, head by head, and is not identical
    c = O.svg_attention_layer_fp8(q, k, v, labels, g, round_weights=True)
    assert not np.array_equal(c, a)
    assert np.linalg.norm(c - a) / np.linalg.norm(a) < 0.03


# ----------------------------------------------------------------------------- QK-norm, RoPE
def test_qk_norm_against_library_and_closed_forms():
    rng = np.random.default_rng(3)
    x = rng.normal(0.3, 1.7, (5, 7, 64))
    w, b = rng.normal(1, 0.2, 64), rng.normal(0, 0.2, 64)
    ref = torch.nn.functional.layer_norm(torch.from_numpy(x), (64,), torch.from_numpy(w), torch.from_numpy(b), eps=1e-6)
    assert np.allclose(O.qk_norm(x, O.NORM_LAYER, w, b, 1e-6), ref.numpy(), rtol=1e-12, atol=1e-12)
    # RMS form: hand-worked (3, 4) -> rms = sqrt(12.5); unit rms output; invariant to the input's scale
    assert np.allclose(O.qk_norm(np.array([3.0, 4.0]), O.NORM_RMS, None, None, 0.0), np.array([3.0, 4.0]) / math.sqrt(12.5))
    y = O.qk_norm(x, O.NORM_RMS, None, None, 0.0)
    assert np.allclose(np.sqrt((y * y).mean(-1)), 1.0)
    assert np.allclose(O.qk_norm(7.5 * x, O.NORM_RMS, w, None, 0.0), O.qk_norm(x, O.NORM_RMS, w, None, 0.0))
    assert np.allclose(O.qk_norm(x, O.NORM_RMS, w, None, 0.0), y * w)
    # eps enters under the root: a zero vector stays zero instead of dividing by zero
    assert not O.qk_norm(np.zeros(8), O.NORM_RMS, None, None, 1e-6).any()
    # the RMS form does not centre, LayerNorm does
    assert abs(O.qk_norm(x, O.NORM_LAYER, None, None, 0.0).mean(-1)).max() < 1e-12 < abs(y.mean(-1)).max()
    assert np.array_equal(O.qk_norm(x, O.NORM_NONE), x)


def test_rope_is_a_complex_rotation_of_the_video_tokens():
    cfg = get_config("tiny")
    g = O.Geometry.from_config(cfg)
    rng = np.random.default_rng(8)
    x = rng.normal(0, 1, (g.N, g.D))
    theta = rng.uniform(-3, 3, (g.F * g.P, g.D // 2))
    y = O.rope(x, np.cos(theta), np.sin(theta), g, O.ROPE_INTERLEAVED)
    vid = slice(g.off, g.off + g.F * g.P)
    z = (x[vid, 0::2] + 1j * x[vid, 1::2]) * np.exp(1j * theta)       # the same thing in complex arithmetic
    assert np.allclose(y[vid, 0::2], z.real) and np.allclose(y[vid, 1::2], z.imag)
    text = np.ones(g.N, bool)
    text[vid] = False
    assert text.any() and np.array_equal(y[text], x[text])              # text tokens are not rotated
    assert np.allclose((y ** 2).sum(-1), (x ** 2).sum(-1))              # rotations keep the norm
    # rotating by a then b is rotating by a + b; rotating back restores x
    t2 = rng.uniform(-3, 3, theta.shape)
    y2 = O.rope(y, np.cos(t2), np.sin(t2), g)
    assert np.allclose(y2, O.rope(x, np.cos(theta + t2), np.sin(theta + t2), g))
    assert np.allclose(O.rope(y, np.cos(-theta), np.sin(-theta), g), x)
    # hand-worked: a quarter turn maps (a, b) to (-b, a)
    q = O.rope(x, np.zeros_like(theta), np.ones_like(theta), g)
    assert np.allclose(q[vid, 0::2], -x[vid, 1::2]) and np.allclose(q[vid, 1::2], x[vid, 0::2])
    # the "half" pairing is the interleaved one on a vector whose halves are interleaved
    inter = np.empty_like(x)
    inter[:, 0::2], inter[:, 1::2] = x[:, :g.D // 2], x[:, g.D // 2:]
    yi = O.rope(inter, np.cos(theta), np.sin(theta), g, O.ROPE_INTERLEAVED)
    yh = O.rope(x, np.cos(theta), np.sin(theta), g, O.ROPE_HALF)
    assert np.allclose(yh[:, :g.D // 2], yi[:, 0::2]) and np.allclose(yh[:, g.D // 2:], yi[:, 1::2])


def test_rope_scores_depend_on_relative_position_only():
    """With angles proportional to a 1-D position the rotated dot product depends only on the
    distance of the two tokens: the property the embedding exists for."""
    g = O.Geometry(B=1, H=1, F=1, P=40, T=0, D=16)
    rng = np.random.default_rng(12)
    qv, kv = rng.normal(0, 1, 16), rng.normal(0, 1, 16)
    freq = 1.0 / 100.0 ** (np.arange(8) / 8.0)
    theta = np.arange(40)[:, None] * freq[None, :]
    rq = O.rope(np.tile(qv, (40, 1)), np.cos(theta), np.sin(theta), g)
    rk = O.rope(np.tile(kv, (40, 1)), np.cos(theta), np.sin(theta), g)
    s = rq @ rk.T
    for d in (0, 1, 5, 17):
        diag = np.array([s[m, m + d] for m in range(40 - d)])
        assert np.allclose(diag, diag[0])
    assert not np.allclose(s[0, 1], s[0, 2])


def test_qk_norm_rope_composition_order():
    cfg = get_config("tiny")
    g = O.Geometry.from_config(cfg)
    rng = np.random.default_rng(14)
    x = rng.normal(0, 1, (g.B, g.H, g.N, g.D))
    w, b = rng.normal(1, 0.3, g.D), rng.normal(0, 0.3, g.D)
    theta = rng.uniform(-3, 3, (g.F * g.P, g.D // 2))
    y = O.qk_norm_rope(x, g, O.NORM_LAYER, w, b, 1e-6, np.cos(theta), np.sin(theta))
    want = O.rope(O.qk_norm(x[0, 1], O.NORM_LAYER, w, b, 1e-6), np.cos(theta), np.sin(theta), g)
    assert np.allclose(y[0, 1], want)
    # the weight makes the two steps not commute, so the order is observable
    other = O.qk_norm(O.rope(x[0, 1], np.cos(theta), np.sin(theta), g), O.NORM_LAYER, w, b, 1e-6)
    assert not np.allclose(want, other)
    assert np.allclose(O.qk_norm_rope(x, g, O.NORM_RMS, w), O.qk_norm(x, O.NORM_RMS, w))
