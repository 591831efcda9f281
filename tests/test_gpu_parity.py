"""GPU parity: every entry point of the library against the CPU oracle, element by
element on seeded inputs that span several tiles and ragged tails."""
import numpy as np
import pytest
import torch

import paper_2502_01776_amd as S
from oracle import svg_oracle as O
from workloads import get_config, make_qkv, make_plain_qkv, sample_rows, planted_labels
from helpers import (f64, bits, dev_i32, device_tile_lists, gpu_profile, gpu_layer, gpu_layer_token_order,
                     gpu_layer_kv2, gpu_layer_in_place, assert_attn_close,
                     labels_match)

pytestmark = pytest.mark.gpu

SMALL = ["tiny", "mid64", "mid128"]


def setup(name, **ov):
    cfg = get_config(name, **ov)
    return cfg, S.shape_from_config(cfg), O.Geometry.from_config(cfg)


# ------------------------------------------------------------------ layout
@pytest.mark.parametrize("name", SMALL)
@pytest.mark.parametrize("with_labels", [False, True])
def test_layout_bit_exact(name, with_labels):
    cfg, sh, g = setup(name)
    q, _, _ = make_qkv(cfg)
    x = q.cuda()
    lab_np = planted_labels(cfg)
    lab = torch.from_numpy(lab_np).cuda() if with_labels else None
    y = torch.zeros_like(x)
    S.svg_layout_fwd(sh, x, y, lab)
    back = torch.zeros_like(x)
    S.svg_layout_inv(sh, y, back, lab)
    torch.cuda.synchronize()
    xb = bits(x)
    ref = O.layout_fwd(xb, g)
    if with_labels:
        sp = (lab_np.reshape(g.B, g.H) == 0)
        ref[sp] = xb[sp]
    assert np.array_equal(bits(y), ref)
    assert np.array_equal(bits(back), xb)


# ------------------------------------------------------------------ dense
@pytest.mark.parametrize("name", SMALL)
def test_dense_attention(name):
    cfg, sh, g = setup(name)
    q, k, v = make_qkv(cfg)
    o = torch.zeros_like(q).cuda()
    S.svg_dense_attn_fwd(sh, q.cuda(), k.cuda(), v.cuda(), o)
    torch.cuda.synchronize()
    qd, kd, vd = f64(q), f64(k), f64(v)
    for b in range(g.B):
        for h in range(g.H):
            ref = O.dense_attention_head(qd[b, h], kd[b, h], vd[b, h], g)
            assert_attn_close(o[b, h], ref, f"{name} dense b{b} h{h}")


# ------------------------------------------------------------------ block-sparse
@pytest.mark.parametrize("name", SMALL)
def test_sparse_attention_per_pattern(name):
    """Both tile lists applied to every head in the order given (no layout step)."""
    cfg, sh, g = setup(name)
    q, k, v = make_qkv(cfg)
    qd, kd, vd = f64(q), f64(k), f64(v)
    lists = device_tile_lists(sh)
    for pat in (0, 1):
        lab = torch.full((g.B * g.H,), pat, dtype=torch.uint8, device="cuda")
        o = torch.zeros_like(q).cuda()
        S.svg_sparse_attn_fwd(sh, q.cuda(), k.cuda(), v.cuda(), o, lab, *lists)
        torch.cuda.synchronize()
        rp, ci = O.tile_list(g, pat)
        for b in range(g.B):
            for h in range(g.H):
                ref = O.sparse_attention_head(qd[b, h], kd[b, h], vd[b, h], rp, ci, g)
                assert_attn_close(o[b, h], ref, f"{name} pattern {pat} b{b} h{h}")


def test_sparse_with_full_list_equals_dense_kernel_bitwise():
    cfg, sh, g = setup("mid128")
    q, k, v = (x.cuda() for x in make_qkv(cfg))
    rp, ci = O.full_tile_list(g)
    o1, o2 = torch.zeros_like(q), torch.zeros_like(q)
    S.svg_sparse_attn_fwd(sh, q, k, v, o1, None, dev_i32(rp), dev_i32(ci), None, None)
    S.svg_dense_attn_fwd(sh, q, k, v, o2)
    torch.cuda.synchronize()
    assert torch.equal(o1.view(torch.int16), o2.view(torch.int16))


def test_empty_tile_rows_give_zeros():
    cfg, sh, g = setup("mid64")
    q, k, v = (x.cuda() for x in make_qkv(cfg))
    rp, ci = O.tile_list(g, 0)
    rp2 = rp.copy()
    n1 = rp[2] - rp[1]
    rp2[2:] -= n1                      # query tile 1 keeps nothing
    ci2 = np.concatenate([ci[:rp[1]], ci[rp[2]:]])
    o = torch.full_like(q, 7.0)
    S.svg_sparse_attn_fwd(sh, q, k, v, o, None, dev_i32(rp2), dev_i32(ci2), None, None)
    torch.cuda.synchronize()
    assert (o[:, :, 128:256] == 0).all()
    ref = O.sparse_attention_head(f64(q)[0, 0], f64(k)[0, 0], f64(v)[0, 0], rp, ci, g)
    assert_attn_close(o[0, 0, :128], ref[:128])
    assert_attn_close(o[0, 0, 256:], ref[256:])


@pytest.mark.parametrize("name", ["mid64", "mid128"])
def test_sparse_attention_arbitrary_tile_lists(name):
    """Lists that follow no window structure: random subsets of the key tiles per query tile
    (lone 64-key halves, gaps, an empty row), different for the two patterns."""
    cfg, sh, g = setup(name)
    q, k, v = make_qkv(cfg)
    nq, nk = O.n_tiles(g)
    rng = np.random.default_rng(77)
    lists = []
    for pat in (0, 1):
        rp = np.zeros(nq + 1, dtype=np.int32)
        cols = []
        for a in range(nq):
            keep = rng.random(nk) < (0.5 if pat == 0 else 0.25)
            if a == 1 and pat == 1:
                keep[:] = False               # an empty row: output zeros
            elif not keep.any():
                keep[rng.integers(nk)] = True
            c = np.nonzero(keep)[0].astype(np.int32)
            cols.append(c)
            rp[a + 1] = rp[a] + len(c)
        lists.append((rp, np.concatenate(cols)))
    labels = torch.tensor([h & 1 for h in range(g.B * g.H)], dtype=torch.uint8, device="cuda")
    o = torch.empty_like(q).cuda()
    S.svg_sparse_attn_fwd(sh, q.cuda(), k.cuda(), v.cuda(), o, labels, dev_i32(lists[0][0]), dev_i32(lists[0][1]),
                          dev_i32(lists[1][0]), dev_i32(lists[1][1]))
    torch.cuda.synchronize()
    for b in range(g.B):
        for h in range(g.H):
            rp, ci = lists[(b * g.H + h) & 1]
            filled = [a for a in range(nq) if rp[a + 1] > rp[a]]
            ref = O.sparse_attention_head(f64(q)[b, h], f64(k)[b, h], f64(v)[b, h], rp, ci, g, q_tiles=filled)
            ok = ~np.isnan(ref[:, 0])
            assert_attn_close(o[b, h][torch.from_numpy(ok).cuda()], ref[ok], f"{name} b{b} h{h}")
    flat = o.reshape(g.B * g.H, g.N, g.D)
    assert (flat[1::2, g.block_m:2 * g.block_m] == 0).all()


def test_sparse_attention_without_layout_transformation():
    """Temporal heads left in frame-major order with the frame-major temporal list (the
    comparison arm of Sec. 5.5): same kernel, unpermuted inputs, more tiles."""
    cfg, sh, g = setup("mid128")
    q, k, v = make_qkv(cfg)
    rp, ci = S.svg_tile_list_build(sh, S.SVG_LIST_TEMPORAL_FRAME_MAJOR)
    orp, oci = O.tile_list(g, O.TEMPORAL_FRAME_MAJOR)
    assert np.array_equal(rp, orp) and np.array_equal(ci, oci)
    assert len(ci) > len(S.svg_tile_list_build(sh, S.SVG_HEAD_TEMPORAL)[1])
    o = torch.empty_like(q).cuda()
    S.svg_sparse_attn_fwd(sh, q.cuda(), k.cuda(), v.cuda(), o, None, dev_i32(rp), dev_i32(ci), None, None)
    torch.cuda.synchronize()
    for h in (1, g.H - 1):
        ref = O.sparse_attention_head(f64(q)[0, h], f64(k)[0, h], f64(v)[0, h], orp, oci, g)
        assert_attn_close(o[0, h], ref, f"frame-major temporal head {h}")


def test_sparse_attention_with_first_frame_sink():
    """Sink flag (Sec. 3.1: the first frame is kept by both patterns): lists from the host builder,
    both patterns, against the oracle's block-sparse attention over its own lists."""
    cfg, sh, g = setup("mid128", sink_first_frame=1)
    q, k, v = make_qkv(cfg)
    for pat in (O.SPATIAL, O.TEMPORAL):
        rp, ci = S.svg_tile_list_build(sh, pat)
        orp, oci = O.tile_list(g, pat)
        assert np.array_equal(rp, orp) and np.array_equal(ci, oci)
        o = torch.empty_like(q).cuda()
        labels = torch.full((g.B * g.H,), pat, dtype=torch.uint8, device="cuda")
        lists = device_tile_lists(sh)
        S.svg_sparse_attn_fwd(sh, q.cuda(), k.cuda(), v.cuda(), o, labels, *lists)
        torch.cuda.synchronize()
        for h in (0, g.H - 1):
            ref = O.sparse_attention_head(f64(q)[0, h], f64(k)[0, h], f64(v)[0, h], orp, oci, g)
            assert_attn_close(o[0, h], ref, f"sink pattern {pat} head {h}")


# ------------------------------------------------------------------ profiling
@pytest.mark.parametrize("name", SMALL)
def test_profile_heads(name):
    cfg, sh, g = setup(name)
    q, k, v = make_qkv(cfg)
    rows = sample_rows(cfg)
    labels, mse = gpu_profile(sh, q.cuda(), k.cuda(), v.cuda(), rows)
    omse, olab = O.profile_heads(f64(q), f64(k), f64(v), rows, g)
    assert labels_match(labels, omse, olab)
    assert np.array_equal(labels.cpu().numpy(), planted_labels(cfg))
    got = mse.cpu().numpy().astype(np.float64).reshape(g.B, g.H, 2)
    # bf16 rounding of the weights puts a noise floor under the measured errors
    assert np.allclose(got, omse, rtol=0.05, atol=2e-5), (got, omse)


@pytest.mark.parametrize("name", ["tiny", "mid64"])
def test_profile_on_every_row(name):
    """t = N: the sampled estimate becomes the full comparison of Sec. 3.2."""
    cfg, sh, g = setup(name)
    q, k, v = make_qkv(cfg)
    rows = np.arange(g.N, dtype=np.int32)
    labels, mse = gpu_profile(sh, q.cuda(), k.cuda(), v.cuda(), rows)
    omse, olab = O.profile_heads(f64(q), f64(k), f64(v), rows, g)
    assert labels_match(labels, omse, olab)
    assert np.allclose(mse.cpu().numpy().reshape(omse.shape), omse, rtol=0.05, atol=2e-5)


def test_profile_row_set_spanning_several_query_tiles():
    cfg, sh, g = setup("mid128")
    q, k, v = make_qkv(cfg)
    rows = sample_rows(cfg, t=300)          # 3 query tiles of 128, ragged
    labels, mse = gpu_profile(sh, q.cuda(), k.cuda(), v.cuda(), rows)
    omse, olab = O.profile_heads(f64(q), f64(k), f64(v), rows, g)
    assert labels_match(labels, omse, olab)
    assert np.allclose(mse.cpu().numpy().reshape(omse.shape), omse, rtol=0.05, atol=2e-5)


def test_profile_with_sink_and_unstructured_heads():
    cfg, sh, g = setup("mid64", sink_first_frame=1)
    q, k, v = make_plain_qkv(cfg["B"], cfg["H"], cfg["N"], cfg["D"], seed=5)
    rows = sample_rows(cfg, t=40)
    labels, mse = gpu_profile(sh, q.cuda(), k.cuda(), v.cuda(), rows)
    omse, olab = O.profile_heads(f64(q), f64(k), f64(v), rows, g)
    assert labels_match(labels, omse, olab)        # (measured: the two errors of these heads differ by 63-73 %)
    assert np.allclose(mse.cpu().numpy().reshape(omse.shape), omse, rtol=0.05, atol=2e-5)


# ------------------------------------------------------------------ whole layer
@pytest.mark.parametrize("name", SMALL)
def test_whole_layer(name):
    cfg, sh, g = setup(name)
    q, k, v = make_qkv(cfg)
    rows = sample_rows(cfg)
    qc, kc, vc = q.cuda(), k.cuda(), v.cuda()
    labels, _ = gpu_profile(sh, qc, kc, vc, rows)
    o = gpu_layer(sh, qc, kc, vc, labels)
    omse, olab = O.profile_heads(f64(q), f64(k), f64(v), rows, g)
    assert np.array_equal(labels.cpu().numpy().reshape(g.B, g.H), olab)
    ref = O.svg_attention_layer(f64(q), f64(k), f64(v), olab, g)
    for b in range(g.B):
        for h in range(g.H):
            assert_attn_close(o[b, h], ref[b, h], f"{name} layer b{b} h{h}")


@pytest.mark.parametrize("name", SMALL)
@pytest.mark.parametrize("sink", [0, 1])
def test_layer_with_q_and_o_in_token_order(name, sink):
    """The attention kernel gathering q rows and scattering o rows itself (two of the four layout
    passes folded in): against the oracle, and bit-identical to the four-pass pipeline."""
    cfg, sh, g = setup(name, sink_first_frame=sink)
    q, k, v = make_qkv(cfg)
    qc, kc, vc = q.cuda(), k.cuda(), v.cuda()
    lab_np = planted_labels(cfg)
    labels = torch.from_numpy(lab_np).cuda()
    o = gpu_layer_token_order(sh, qc, kc, vc, labels)
    ref = O.svg_attention_layer(f64(q), f64(k), f64(v), lab_np.reshape(g.B, g.H), g)
    for b in range(g.B):
        for h in range(g.H):
            assert_attn_close(o[b, h], ref[b, h], f"{name} token-order layer b{b} h{h}")
    o4 = gpu_layer(sh, qc, kc, vc, labels)
    assert torch.equal(o.view(torch.int16), o4.view(torch.int16))
    # every head temporal, no label array semantics: labels == all ones
    ones = torch.ones_like(labels)
    assert torch.equal(gpu_layer_token_order(sh, qc, kc, vc, ones).view(torch.int16),
                       gpu_layer(sh, qc, kc, vc, ones).view(torch.int16))


@pytest.mark.parametrize("name", SMALL)
@pytest.mark.parametrize("sink", [0, 1])
def test_layer_with_only_temporal_kv_moved(name, sink):
    """svg_layout_kv_temporal + svg_sparse_attn_fwd_kv2: k and v of spatial heads are read in place and
    never copied; against the oracle, bit-identical to the four-pass pipeline, and the slots of
    spatial heads in the copies are neither written nor (NaN filled) read."""
    cfg, sh, g = setup(name, sink_first_frame=sink)
    q, k, v = make_qkv(cfg)
    qc, kc, vc = q.cuda(), k.cuda(), v.cuda()
    lab_np = planted_labels(cfg)
    labels = torch.from_numpy(lab_np).cuda()
    NAN = 0x7FC1                   # a bf16 NaN pattern, as int16
    o, kt, vt = gpu_layer_kv2(sh, qc, kc, vc, labels, fill=NAN)
    assert torch.isfinite(o.float()).all()
    ref = O.svg_attention_layer(f64(q), f64(k), f64(v), lab_np.reshape(g.B, g.H), g)
    for b in range(g.B):
        for h in range(g.H):
            assert_attn_close(o[b, h], ref[b, h], f"{name} kv2 layer b{b} h{h}")
            slot_k, slot_v = kt[b, h].view(torch.int16), vt[b, h].view(torch.int16)
            if lab_np[b * g.H + h] == O.SPATIAL:
                assert (slot_k == NAN).all() and (slot_v == NAN).all()
            else:
                assert np.array_equal(bits(kt[b, h]), O.layout_fwd(bits(kc[b, h]), g))
                assert np.array_equal(bits(vt[b, h]), O.layout_fwd(bits(vc[b, h]), g))
    o4 = gpu_layer(sh, qc, kc, vc, labels)
    assert torch.equal(o.view(torch.int16), o4.view(torch.int16))
    # with the element mask on it equals the flag on the extended entry point
    oe, _, _ = gpu_layer_kv2(sh, qc, kc, vc, labels, flags=S.SVG_ATTN_ELEMENT_MASK)
    kp, vp, oe2 = (torch.empty_like(qc) for _ in range(3))
    S.svg_layout_fwd(sh, kc, kp, labels)
    S.svg_layout_fwd(sh, vc, vp, labels)
    S.svg_sparse_attn_fwd_ex(sh, qc, kp, vp, oe2, labels, *device_tile_lists(sh),
                             flags=S.SVG_ATTN_QO_TOKEN_ORDER | S.SVG_ATTN_ELEMENT_MASK)
    torch.cuda.synchronize()
    assert torch.equal(oe.view(torch.int16), oe2.view(torch.int16))
    with pytest.raises(S.SvgError):
        S.svg_sparse_attn_fwd_kv2(sh, qc, kc, vc, kt, vt, o, labels, *device_tile_lists(sh), flags=1)
    with pytest.raises(S.SvgError):
        S.svg_layout_kv_temporal(sh, kc, vc, kt, kt, labels)           # the two copies overlap


@pytest.mark.parametrize("name", ["mid128", "mid64"])
@pytest.mark.parametrize("sink", [0, 1])
def test_layer_without_any_layout_pass(name, sink):
    """SVG_ATTN_QO_TOKEN_ORDER | SVG_ATTN_KV_TOKEN_ORDER: every tensor stays in token order and the
    kernel gathers the rows of a temporal head's key tiles itself (Sec. 4.3: the transformation fused
    into the kernel).  Against the oracle, bit-identical to the pipeline with the layout passes, and
    nothing written past the row table."""
    cfg, sh, g = setup(name, sink_first_frame=sink)
    q, k, v = make_qkv(cfg)
    qc, kc, vc = q.cuda(), k.cuda(), v.cuda()
    lab_np = planted_labels(cfg)
    labels = torch.from_numpy(lab_np).cuda()
    o, guard_ok = gpu_layer_in_place(sh, qc, kc, vc, labels)
    assert guard_ok
    ref = O.svg_attention_layer(f64(q), f64(k), f64(v), lab_np.reshape(g.B, g.H), g)
    for b in range(g.B):
        for h in range(g.H):
            assert_attn_close(o[b, h], ref[b, h], f"{name} in-place layer b{b} h{h}")
    assert torch.equal(o.view(torch.int16), gpu_layer(sh, qc, kc, vc, labels).view(torch.int16))
    # all heads temporal, all heads spatial
    for lab in (np.ones_like(lab_np), np.zeros_like(lab_np)):
        lt = torch.from_numpy(lab).cuda()
        o1, _ = gpu_layer_in_place(sh, qc, kc, vc, lt)
        assert torch.equal(o1.view(torch.int16), gpu_layer(sh, qc, kc, vc, lt).view(torch.int16))
    # workspace too small / missing, and the combinations that do not exist
    lists = device_tile_lists(sh)
    nq, nk = S.svg_tile_counts(sh)
    ws = torch.empty(8 * nk * sh.block_n, dtype=torch.uint8, device="cuda")
    both = S.SVG_ATTN_QO_TOKEN_ORDER | S.SVG_ATTN_KV_TOKEN_ORDER
    for kwargs in (dict(flags=both), dict(flags=both, workspace=ws, workspace_bytes=ws.numel() - 4),
                   dict(flags=both | S.SVG_ATTN_ELEMENT_MASK, workspace=ws, workspace_bytes=ws.numel())):
        with pytest.raises(S.SvgError):
            S.svg_sparse_attn_fwd_ex(sh, qc, kc, vc, o, labels, *lists, **kwargs)


@pytest.mark.parametrize("heads, label_kind", [(1, "mixed"), (3, "temporal"), (7, "mixed"), (64, "mixed"), (64, "spatial"),
                                                (65, "mixed"), (70, "temporal"), (130, "mixed"), (256, "mixed"), (260, "mixed")])
def test_every_head_and_query_tile_is_computed_for_any_head_count_and_label_mix(heads, label_kind):
    """The dispatch order of the sparse passes (text-row query tiles first, then an eighth of each
    label's tile sequence per XCD; label classes taken from a 64-lane ballot, more than 64 heads in head
    order) must hand out every (head, query tile) exactly once whatever the head count and the labels
    are: the output buffer starts as NaN and every row of every head is compared with the oracle for
    four heads and must be finite and equal to the token-order form for all."""
    cfg, sh, g = setup("mid128", H=heads, spatial_heads=[])
    q, k, v = make_plain_qkv(1, heads, g.N, g.D, seed=77 + heads)
    qc, kc, vc = q.cuda(), k.cuda(), v.cuda()
    rng = np.random.default_rng(heads)
    lab_np = {"mixed": rng.integers(0, 2, size=heads), "temporal": np.ones(heads), "spatial": np.zeros(heads)}[label_kind].astype(np.uint8)
    labels = torch.from_numpy(lab_np).cuda()
    lists = device_tile_lists(sh)
    kp, vp = torch.empty_like(kc), torch.empty_like(vc)
    S.svg_layout_fwd(sh, kc, kp, labels)
    S.svg_layout_fwd(sh, vc, vp, labels)
    o = torch.full_like(qc, float("nan"))
    S.svg_sparse_attn_fwd_ex(sh, qc, kp, vp, o, labels, *lists, flags=S.SVG_ATTN_QO_TOKEN_ORDER)
    torch.cuda.synchronize()
    assert torch.isfinite(o.float()).all(), "some (head, query tile) was never written"
    for h in sorted({0, heads // 2, heads - 1, int(rng.integers(heads))}):
        ref = O.svg_attention_layer(f64(q[:, h:h + 1]), f64(k[:, h:h + 1]), f64(v[:, h:h + 1]),
                                    lab_np[h:h + 1].reshape(1, 1), O.Geometry(**{**g.__dict__, "H": 1}))
        assert_attn_close(o[0, h], ref[0, 0], f"H={heads} {label_kind} head {h}")
    # the other forms hand out the same work
    og, guard_ok = gpu_layer_in_place(sh, qc, kc, vc, labels, lists)
    assert guard_ok and torch.isfinite(og.float()).all()
    assert torch.equal(og.view(torch.int16), o.view(torch.int16))
    o4 = gpu_layer(sh, qc, kc, vc, labels, lists)
    assert torch.equal(o4.view(torch.int16), o.view(torch.int16))


def test_extended_entry_point_rejects_unknown_flags():
    cfg, sh, g = setup("mid64")
    q, k, v = (x.cuda() for x in make_qkv(cfg))
    o = torch.empty_like(q)
    lists = device_tile_lists(sh)
    with pytest.raises(S.SvgError):
        S.svg_sparse_attn_fwd_ex(sh, q, k, v, o, None, *lists, flags=4)
    # flags == 0 is the plain entry point
    o0 = torch.empty_like(q)
    S.svg_sparse_attn_fwd_ex(sh, q, k, v, o, None, *lists, flags=0)
    S.svg_sparse_attn_fwd(sh, q, k, v, o0, None, *lists)
    torch.cuda.synchronize()
    assert torch.equal(o.view(torch.int16), o0.view(torch.int16))


def test_results_are_deterministic():
    cfg, sh, g = setup("mid128")
    q, k, v = (x.cuda() for x in make_qkv(cfg))
    rows = sample_rows(cfg)
    l1, m1 = gpu_profile(sh, q, k, v, rows)
    l2, m2 = gpu_profile(sh, q, k, v, rows)
    assert torch.equal(l1, l2) and torch.equal(m1, m2)
    o1 = gpu_layer(sh, q, k, v, l1)
    o2 = gpu_layer(sh, q, k, v, l1)
    assert torch.equal(o1.view(torch.int16), o2.view(torch.int16))
    # many sampled rows at the same in-frame position (they share a bin of the row grouping of
    # the temporal pass), with unrelated work in between so that the timing differs
    rows = sample_rows(cfg, t=600)
    l1, m1 = gpu_profile(sh, q, k, v, rows)
    for _ in range(3):
        gpu_layer(sh, q, k, v, l1)
        l2, m2 = gpu_profile(sh, q, k, v, rows)
        assert torch.equal(l1, l2) and torch.equal(m1, m2)


# ------------------------------------------------------------------ degenerate geometries
@pytest.mark.parametrize("geo", [
    dict(F=1, P=200, T=0, D=64),            # one frame, no text
    dict(F=9, P=1, T=3, D=128),             # one token per frame
    dict(F=2, P=5, T=0, D=64),              # N = 10, smaller than any tile
    dict(F=3, P=64, T=64, D=128, text_first=0),   # tile-aligned everything
    dict(F=4, P=33, T=1, D=64, text_first=0, sink_first_frame=1),
])
@pytest.mark.parametrize("blocks", [(128, 64), (32, 32)])
def test_degenerate_geometries(geo, blocks):
    base = dict(get_config("mid64"), B=1, H=2, w_s=1, w_t=2, text_first=1, sink_first_frame=0,
                block_m=blocks[0], block_n=blocks[1], spatial_heads=[0])
    base.update(geo)
    base["N"] = base["F"] * base["P"] + base["T"]
    cfg = base
    sh, g = S.shape_from_config(cfg), O.Geometry.from_config(cfg)
    q, k, v = make_plain_qkv(1, 2, g.N, g.D, seed=11)
    qc, kc, vc = q.cuda(), k.cuda(), v.cuda()
    # tile lists bit-exact
    for pat in (0, 1):
        rp, ci = S.svg_tile_list_build(sh, pat)
        orp, oci = O.tile_list(g, pat)
        assert np.array_equal(rp, orp) and np.array_equal(ci, oci)
    rows = np.arange(0, g.N, max(1, g.N // 7), dtype=np.int32)
    labels, mse = gpu_profile(sh, qc, kc, vc, rows)
    omse, olab = O.profile_heads(f64(q), f64(k), f64(v), rows, g)
    assert np.allclose(mse.cpu().numpy().reshape(omse.shape), omse, rtol=0.05, atol=2e-5)
    lab = torch.tensor([0, 1], dtype=torch.uint8, device="cuda")
    o = gpu_layer(sh, qc, kc, vc, lab)
    ref = O.svg_attention_layer(f64(q), f64(k), f64(v), np.array([[0, 1]]), g)
    for h in range(2):
        assert_attn_close(o[0, h], ref[0, h], f"{geo} head {h}")
    od = torch.zeros_like(qc)
    S.svg_dense_attn_fwd(sh, qc, kc, vc, od)
    torch.cuda.synchronize()
    assert_attn_close(od[0, 0], O.dense_attention_head(f64(q)[0, 0], f64(k)[0, 0], f64(v)[0, 0], g))


def test_random_geometries_whole_layer():
    """Seeded random geometries (frames, positions, text length and side, windows, sink, head
    dimension, tile shape): profiling, both layouts, block-sparse attention and the dense pass
    against the oracle."""
    rng = np.random.default_rng(4242)
    for case in range(12):
        F, P = int(rng.integers(1, 8)), int(rng.integers(1, 260))
        T = int(rng.choice([0, 1, 17, 64, 130]))
        bm, bn = ((128, 64), (32, 32))[int(rng.integers(2))]
        cfg = dict(get_config("mid64"), B=1, H=2, F=F, P=P, T=T, D=int(rng.choice([64, 128])),
                   text_first=int(rng.integers(2)), w_s=int(rng.integers(0, F + 1)), w_t=int(rng.integers(0, P + 1)),
                   sink_first_frame=int(rng.integers(2)), block_m=bm, block_n=bn, spatial_heads=[0])
        cfg["N"] = F * P + T
        sh, g = S.shape_from_config(cfg), O.Geometry.from_config(cfg)
        q, k, v = make_plain_qkv(1, 2, g.N, g.D, seed=100 + case)
        qc, kc, vc = q.cuda(), k.cuda(), v.cuda()
        rows = np.unique(rng.integers(0, g.N, size=min(g.N, 40))).astype(np.int32)
        labels, mse = gpu_profile(sh, qc, kc, vc, rows)
        omse, olab = O.profile_heads(f64(q), f64(k), f64(v), rows, g)
        assert np.allclose(mse.cpu().numpy().reshape(omse.shape), omse, rtol=0.05, atol=2e-5), (cfg, case)
        lab = torch.tensor([0, 1], dtype=torch.uint8, device="cuda")
        o = gpu_layer(sh, qc, kc, vc, lab)
        ref = O.svg_attention_layer(f64(q), f64(k), f64(v), np.array([[0, 1]]), g)
        for h in range(2):
            assert_attn_close(o[0, h], ref[0, h], f"case {case} {cfg} head {h}")
        if bm == 128:        # the form that gathers k and v rows in the kernel gives the same bits
            og, guard_ok = gpu_layer_in_place(sh, qc, kc, vc, lab)
            assert guard_ok and torch.equal(og.view(torch.int16), o.view(torch.int16)), (cfg, case)
        od = torch.zeros_like(qc)
        S.svg_dense_attn_fwd(sh, qc, kc, vc, od)
        torch.cuda.synchronize()
        assert_attn_close(od[0, 1], O.dense_attention_head(f64(q)[0, 1], f64(k)[0, 1], f64(v)[0, 1], g))


def test_nothing_is_written_outside_the_outputs():
    """Guard bytes in front of and behind o, labels, mse and the permuted tensors stay untouched
    by profiling, the layout passes, both sparse pipelines and the dense pass (ragged last
    query tile, ragged last key tile, head count that is no multiple of anything)."""
    cfg, sh, g = setup("mid128", H=5, spatial_heads=[0, 3])
    q, k, v = (x.cuda() for x in make_qkv(cfg))
    BH, n = g.B * g.H, g.B * g.H * g.N * g.D
    PAD = 4096          # bytes on each side; keeps the 16-byte alignment of the tensors

    def guarded(nbytes, dtype):
        buf = torch.full((PAD + nbytes + PAD,), 0xA5, dtype=torch.uint8, device="cuda")
        return buf, buf[PAD:PAD + nbytes].view(dtype)

    def intact(buf, nbytes):
        return bool((buf[:PAD] == 0xA5).all()) and bool((buf[PAD + nbytes:] == 0xA5).all())

    rows = sample_rows(cfg)
    t = len(rows)
    lab_buf, labels = guarded(BH, torch.uint8)
    mse_buf, mse = guarded(BH * 2 * 4, torch.float32)
    ws_bytes = S.svg_workspace_bytes(sh, t)
    ws_buf, ws = guarded(ws_bytes, torch.uint8)
    S.svg_profile_heads(sh, q, k, v, dev_i32(rows), t, labels, mse, ws, ws_bytes)
    torch.cuda.synchronize()
    assert intact(lab_buf, BH) and intact(mse_buf, BH * 8) and intact(ws_buf, ws_bytes)
    assert np.array_equal(labels.cpu().numpy(), planted_labels(cfg))

    bufs = {name: guarded(n * 2, torch.bfloat16) for name in ("qp", "kp", "vp", "op", "o", "o2", "od")}
    view = {name: b[1].view(q.shape) for name, b in bufs.items()}
    lists = device_tile_lists(sh)
    S.svg_layout_fwd(sh, q, view["qp"], labels)
    S.svg_layout_fwd(sh, k, view["kp"], labels)
    S.svg_layout_fwd(sh, v, view["vp"], labels)
    S.svg_sparse_attn_fwd(sh, view["qp"], view["kp"], view["vp"], view["op"], labels, *lists)
    S.svg_layout_inv(sh, view["op"], view["o"], labels)
    S.svg_sparse_attn_fwd_ex(sh, q, view["kp"], view["vp"], view["o2"], labels, *lists,
                             flags=S.SVG_ATTN_QO_TOKEN_ORDER | S.SVG_ATTN_ELEMENT_MASK)
    S.svg_dense_attn_fwd(sh, q, k, v, view["od"])
    torch.cuda.synchronize()
    for name, (buf, _) in bufs.items():
        assert intact(buf, n * 2), name
    assert torch.isfinite(view["o"].float()).all() and torch.isfinite(view["od"].float()).all()


def test_large_logits_do_not_overflow():
    """Row maxima far from zero (|logit| ~ 60): the online softmax must stay finite."""
    cfg, sh, g = setup("mid64")
    q, k, v = make_qkv(cfg, boost_nats=60.0)
    o = torch.zeros_like(q).cuda()
    S.svg_dense_attn_fwd(sh, q.cuda(), k.cuda(), v.cuda(), o)
    torch.cuda.synchronize()
    ref = O.dense_attention_head(f64(q)[0, 1], f64(k)[0, 1], f64(v)[0, 1], g)
    assert_attn_close(o[0, 1], ref, "boost 60")


# ------------------------------------------------------------------ exact element mask
@pytest.mark.parametrize("name", SMALL)
@pytest.mark.parametrize("sink", [0, 1])
def test_sparse_attention_with_element_mask(name, sink):
    """SVG_ATTN_ELEMENT_MASK: attention under the exact masks of Sec. 3.1 (not their block cover),
    against the oracle's masked attention in the original token order."""
    cfg, sh, g = setup(name, sink_first_frame=sink)
    q, k, v = make_qkv(cfg)
    qc, kc, vc = q.cuda(), k.cuda(), v.cuda()
    lab_np = planted_labels(cfg)
    labels = torch.from_numpy(lab_np).cuda()
    lists = device_tile_lists(sh)
    kp, vp, o = (torch.empty_like(qc) for _ in range(3))
    S.svg_layout_fwd(sh, kc, kp, labels)
    S.svg_layout_fwd(sh, vc, vp, labels)
    S.svg_sparse_attn_fwd_ex(sh, qc, kp, vp, o, labels, *lists,
                             flags=S.SVG_ATTN_QO_TOKEN_ORDER | S.SVG_ATTN_ELEMENT_MASK)
    torch.cuda.synchronize()
    masks = {O.SPATIAL: O.spatial_mask(g), O.TEMPORAL: O.temporal_mask(g)}
    qd, kd, vd = f64(q), f64(k), f64(v)
    differs = False
    block = gpu_layer_token_order(sh, qc, kc, vc, labels, lists)
    for b in range(g.B):
        for h in range(g.H):
            ref = O.masked_attention(qd[b, h], kd[b, h], vd[b, h], masks[int(lab_np[b * g.H + h])], g.scale)
            assert_attn_close(o[b, h], ref, f"{name} exact mask b{b} h{h}")
            differs |= not torch.equal(o[b, h], block[b, h])
    assert differs        # the block cover keeps more than the element mask on these shapes
    # the four-pass pipeline with the flag gives the same bits
    qp, op, o4 = (torch.empty_like(qc) for _ in range(3))
    S.svg_layout_fwd(sh, qc, qp, labels)
    S.svg_sparse_attn_fwd_ex(sh, qp, kp, vp, op, labels, *lists, flags=S.SVG_ATTN_ELEMENT_MASK)
    S.svg_layout_inv(sh, op, o4, labels)
    torch.cuda.synchronize()
    assert torch.equal(o.view(torch.int16), o4.view(torch.int16))


def test_element_mask_random_geometries():
    rng = np.random.default_rng(777)
    for case in range(10):
        F, P = int(rng.integers(1, 8)), int(rng.integers(1, 260))
        T = int(rng.choice([0, 1, 17, 64, 130]))
        bm, bn = ((128, 64), (32, 32))[int(rng.integers(2))]
        cfg = dict(get_config("mid64"), B=1, H=2, F=F, P=P, T=T, D=int(rng.choice([64, 128])),
                   text_first=int(rng.integers(2)), w_s=int(rng.integers(0, F + 1)), w_t=int(rng.integers(0, P + 1)),
                   sink_first_frame=int(rng.integers(2)), block_m=bm, block_n=bn, spatial_heads=[0])
        cfg["N"] = F * P + T
        sh, g = S.shape_from_config(cfg), O.Geometry.from_config(cfg)
        q, k, v = make_plain_qkv(1, 2, g.N, g.D, seed=300 + case)
        qc, kc, vc = q.cuda(), k.cuda(), v.cuda()
        lab = torch.tensor([0, 1], dtype=torch.uint8, device="cuda")
        kp, vp, o = (torch.empty_like(qc) for _ in range(3))
        S.svg_layout_fwd(sh, kc, kp, lab)
        S.svg_layout_fwd(sh, vc, vp, lab)
        S.svg_sparse_attn_fwd_ex(sh, qc, kp, vp, o, lab, *device_tile_lists(sh),
                                 flags=S.SVG_ATTN_QO_TOKEN_ORDER | S.SVG_ATTN_ELEMENT_MASK)
        torch.cuda.synchronize()
        for h, mask in ((0, O.spatial_mask(g)), (1, O.temporal_mask(g))):
            ref = O.masked_attention(f64(q)[0, h], f64(k)[0, h], f64(v)[0, h], mask, g.scale)
            assert_attn_close(o[0, h], ref, f"case {case} {cfg} head {h}")
