"""CPU-side checks of the C-ABI library: it loads, exports every symbol the header
declares, validates arguments before touching the GPU, and its host tile-list
builder matches the oracle bit-exactly."""
import ctypes as C
import os
import re

import numpy as np
import pytest

import paper_2502_01776_amd as S
from paper_2502_01776_amd import binding
from oracle import svg_oracle as O
from workloads import get_config

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def header_functions():
    text = open(os.path.join(ROOT, "include", "svg.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(svg_[a-z0-9_]+)\s*\(", text)))


def test_library_exports_every_declared_symbol():
    names = header_functions()
    assert "svg_profile_heads" in names and "svg_sparse_attn_fwd" in names and len(names) >= 10
    lib = S.lib()
    for n in names:
        assert hasattr(lib, n), n
    assert sorted(binding.EXPORTS) == names


def test_binding_has_same_names_as_header():
    for n in header_functions():
        assert hasattr(S, n) or n == "svg_last_hip_error", n


def test_shape_struct_matches_header_layout():
    assert C.sizeof(S.SvgShape) == 13 * 4
    assert [f[0] for f in S.SvgShape._fields_] == [
        "B", "H", "F", "P", "T", "D", "text_first", "w_s", "w_t", "sink_first_frame",
        "block_m", "block_n", "softmax_scale"]


def test_strerror_and_version():
    assert S.svg_strerror(0) == "ok"
    for code in (-1, -2, -3, -4, -5, -99):
        assert isinstance(S.svg_strerror(code), str) and S.svg_strerror(code)
    assert re.match(r"^\d+\.\d+$", S.svg_version())


CASES = ["tiny", "mid64", "mid128", "cogvideox_v1"]


@pytest.mark.parametrize("name", CASES)
@pytest.mark.parametrize("pattern", [0, 1, 2])
@pytest.mark.parametrize("sink", [0, 1])
def test_host_tile_list_is_bit_exact(name, pattern, sink):
    if name == "cogvideox_v1" and sink:
        pytest.skip("covered by the smaller shapes")
    cfg = get_config(name, sink_first_frame=sink)
    rp, ci = S.svg_tile_list_build(S.shape_from_config(cfg), pattern)
    g = O.Geometry.from_config(cfg)
    orp, oci = O.tile_list(g, pattern)
    assert rp.dtype == np.int32 and ci.dtype == np.int32
    assert np.array_equal(rp, orp) and np.array_equal(ci, oci)


@pytest.mark.parametrize("name", ["wan21_14b", "cogvideox_v15", "hunyuan", "hunyuan_skip85", "hunyuan_keep31"])
def test_host_tile_list_sampled_rows_at_full_size(name):
    cfg = get_config(name)
    sh, g = S.shape_from_config(cfg), O.Geometry.from_config(cfg)
    nq, nk = S.svg_tile_counts(sh)
    assert (nq, nk) == O.n_tiles(g)
    for pattern in (0, 1, 2):
        rp, ci = S.svg_tile_list_build(sh, pattern)
        assert rp[0] == 0 and rp[-1] == len(ci) and (np.diff(rp) > 0).all()
        for a in (0, 1, nq // 3, nq // 2, nq - 2, nq - 1):
            assert np.array_equal(ci[rp[a]:rp[a + 1]], O.kept_tiles_of_row(g, pattern, a)), (pattern, a)


def test_host_tile_list_with_first_frame_sink_at_full_size():
    """Sink on at the 119k-token shape: sampled list rows against the oracle's brute force (incl. the
    query tile in which the frame-0 block of the transformed order ends), and the kept fraction of a
    temporal head stays far below the dense count it had with frame 0 spread over every F-th row."""
    cfg = get_config("hunyuan_skip85", sink_first_frame=1)
    sh, g = S.shape_from_config(cfg), O.Geometry.from_config(cfg)
    nq, nk = S.svg_tile_counts(sh)
    for pattern in (0, 1, 2):
        rp, ci = S.svg_tile_list_build(sh, pattern)
        for a in (0, g.P // g.block_m, nq // 2, nq - 1):
            assert np.array_equal(ci[rp[a]:rp[a + 1]], O.kept_tiles_of_row(g, pattern, a)), (pattern, a)
        if pattern != 2:
            assert len(ci) < 0.2 * nq * nk


def test_host_tile_counts_match_the_stored_ones():
    """All six benchmark shapes against tests/golden/tile_counts.txt (written from the oracle by
    tests/golden/make_tile_counts.py)."""
    path = os.path.join(ROOT, "tests", "golden", "tile_counts.txt")
    seen = 0
    for line in open(path):
        if not line.strip() or line.startswith("#"):
            continue
        name, want_s, want_t, want_all = line.split()
        cfg = get_config(name)
        sh = S.shape_from_config(cfg)
        nq, nk = S.svg_tile_counts(sh)
        assert nq * nk == int(want_all), name
        assert len(S.svg_tile_list_build(sh, 0)[1]) == int(want_s), name
        assert len(S.svg_tile_list_build(sh, 1)[1]) == int(want_t), name
        seen += 1
    assert seen == 6


def test_tile_list_geometry_variants():
    base = dict(get_config("mid64"), B=1, H=1)
    for F, P, T, tf, ws, wt, bm, bn in [(1, 200, 0, 1, 0, 3, 128, 64), (9, 1, 3, 0, 2, 0, 32, 32),
                                        (2, 5, 0, 1, 1, 1, 128, 64), (3, 64, 64, 0, 0, 0, 32, 32),
                                        (6, 70, 9, 1, 5, 69, 128, 64), (5, 100, 130, 0, 1, 7, 32, 32)]:
        for sink in (0, 1):
            cfg = dict(base, F=F, P=P, T=T, text_first=tf, w_s=ws, w_t=wt, block_m=bm, block_n=bn,
                       sink_first_frame=sink)
            sh, g = S.shape_from_config(cfg), O.Geometry.from_config(cfg)
            for pattern in (0, 1, 2):
                rp, ci = S.svg_tile_list_build(sh, pattern)
                orp, oci = O.tile_list(g, pattern)
                assert np.array_equal(rp, orp) and np.array_equal(ci, oci), (cfg, pattern)


def test_tile_list_random_geometries():
    """Seeded random small geometries (frames, positions, text length and side, windows, sink,
    both tile shapes), all three list patterns, host builder against the oracle's brute force."""
    rng = np.random.default_rng(2025)
    base = dict(get_config("mid64"), B=1, H=1)
    for _ in range(60):
        F, P = int(rng.integers(1, 9)), int(rng.integers(1, 150))
        T = int(rng.choice([0, 0, 1, 17, 64, 130]))
        bm, bn = ((128, 64), (32, 32))[int(rng.integers(2))]
        cfg = dict(base, F=F, P=P, T=T, text_first=int(rng.integers(2)), w_s=int(rng.integers(0, F + 1)),
                   w_t=int(rng.integers(0, P + 1)), block_m=bm, block_n=bn, sink_first_frame=int(rng.integers(2)))
        sh, g = S.shape_from_config(cfg), O.Geometry.from_config(cfg)
        for pattern in (0, 1, 2):
            rp, ci = S.svg_tile_list_build(sh, pattern)
            orp, oci = O.tile_list(g, pattern)
            assert np.array_equal(rp, orp) and np.array_equal(ci, oci), (cfg, pattern)


def test_tile_list_capacity_and_size_query():
    sh = S.shape_from_config(get_config("mid64"))
    nq, _ = S.svg_tile_counts(sh)
    rp = np.zeros(nq + 1, np.int32)
    nnz = C.c_int64()
    lib = S.lib()
    assert lib.svg_tile_list_build(C.byref(sh), 0, rp.ctypes.data, None, 0, C.byref(nnz)) == 0
    assert nnz.value == rp[-1] > 0
    small = np.zeros(3, np.int32)
    assert lib.svg_tile_list_build(C.byref(sh), 0, rp.ctypes.data, small.ctypes.data, 3, C.byref(nnz)) == -1
    assert nnz.value == rp[-1]
    assert lib.svg_tile_list_build(C.byref(sh), 3, rp.ctypes.data, None, 0, C.byref(nnz)) == -1
    assert lib.svg_tile_list_build(C.byref(sh), 0, None, None, 0, C.byref(nnz)) == -1


def _bad_shapes():
    good = get_config("mid64")
    yield dict(good, D=96), -2
    yield dict(good, block_m=64, block_n=64), -2
    yield dict(good, B=0), -1
    yield dict(good, F=0), -1
    yield dict(good, T=-1), -1
    yield dict(good, w_s=-1), -1
    yield dict(good, text_first=2), -1
    yield dict(good, F=4096, P=4096), -2       # N beyond the supported range


def test_invalid_shapes_are_rejected_before_any_launch():
    lib = S.lib()
    a = 0x1000   # never dereferenced: the shape is checked first
    for cfg, code in _bad_shapes():
        sh = S.shape_from_config(cfg)
        assert S.svg_workspace_bytes(sh, 16) == 0
        assert lib.svg_layout_fwd(C.byref(sh), a, a + 0x100000000, None, None) == code
        assert lib.svg_dense_attn_fwd(C.byref(sh), a, a, a, a, None, 0, None) == code
        assert lib.svg_profile_heads(C.byref(sh), a, a, a, a, 4, a, None, a, 1 << 40, None) == code
        with pytest.raises(S.SvgError):
            S.svg_tile_counts(sh)


def test_pointer_checks_without_gpu():
    lib = S.lib()
    sh = S.shape_from_config(get_config("mid64"))
    nbytes = sh.B * sh.H * sh.N * sh.D * 2
    a, b = 0x10000000, 0x10000000 + 4 * nbytes
    # NULL and misaligned tensors
    assert lib.svg_layout_fwd(C.byref(sh), None, b, None, None) == -1
    assert lib.svg_layout_fwd(C.byref(sh), a + 2, b, None, None) == -1
    assert lib.svg_dense_attn_fwd(C.byref(sh), a, a, None, b, None, 0, None) == -1
    assert lib.svg_sparse_attn_fwd(C.byref(sh), a, a, a, b, None, None, None, None, None, None, 0, None) == -1
    assert lib.svg_sparse_attn_fwd(C.byref(sh), a, a, a, b, a, a, a, None, None, None, 0, None) == -1
    # aliasing
    assert lib.svg_layout_fwd(C.byref(sh), a, a, None, None) == -4
    assert lib.svg_layout_inv(C.byref(sh), a, a + nbytes - 16, None, None) == -4
    assert lib.svg_dense_attn_fwd(C.byref(sh), a, a, a, a, None, 0, None) == -4
    # the two-source sparse pass and the temporal-only layout of k and v
    far = [a + i * (1 << 32) for i in range(8)]          # q k v k_t v_t o: far apart
    q_, k_, v_, kt_, vt_, o_ = far[:6]
    kv2 = lambda *args: lib.svg_sparse_attn_fwd_kv2(C.byref(sh), *args)
    assert kv2(q_, k_, v_, None, vt_, o_, a, a, a, a, a, 0, None) == -1
    assert kv2(q_, k_, v_, kt_, vt_, o_, None, a, a, a, a, 0, None) == -1          # labels are required
    assert kv2(q_, k_, v_, kt_, vt_, o_, a, a, a, None, a, 0, None) == -1
    assert kv2(q_, k_, v_, kt_, vt_, o_, a, a, a, a, a, 1, None) == -1             # token order is implied, not a flag
    assert kv2(q_, k_, v_, kt_, vt_, kt_ + 32, a, a, a, a, a, 0, None) == -4
    assert kv2(q_, k_, v_, kt_, vt_, q_, a, a, a, a, a, 2, None) == -4
    # k and v left in token order (rows gathered by the kernel): needs the row table's workspace
    ex = lambda *args: lib.svg_sparse_attn_fwd_ex(C.byref(sh), *args)
    need = 8 * sh.block_n * (-(-(sh.F * sh.P + sh.T) // sh.block_n))
    ws_ = far[6]
    assert ex(q_, k_, v_, o_, a, a, a, a, a, 5, None, 0, None) == -3
    assert ex(q_, k_, v_, o_, a, a, a, a, a, 5, ws_, need - 1, None) == -3
    assert ex(q_, k_, v_, o_, a, a, a, a, a, 5, o_ + 64, need, None) == -4          # table inside o
    assert ex(q_, k_, v_, o_, a, a, a, a, a, 7, ws_, need, None) == -2              # no exact-mask form of it
    assert ex(q_, k_, v_, o_, a, a, a, a, a, 8, ws_, need, None) == -1              # unknown flag
    lkv = lambda *args: lib.svg_layout_kv_temporal(C.byref(sh), *args)
    assert lkv(k_, v_, kt_, None, a, None) == -1
    assert lkv(k_, v_, kt_, vt_, None, None) == -1
    assert lkv(k_, v_, kt_ + 4, vt_, a, None) == -1
    assert lkv(k_, v_, k_, vt_, a, None) == -4
    assert lkv(k_, v_, kt_, kt_ + nbytes - 16, a, None) == -4
    assert lkv(k_, v_, v_ + 16, vt_, a, None) == -4
    # workspace
    need = S.svg_workspace_bytes(sh, 24)
    # s output slots (the parts the three passes are cut into: at least one each) with one set of row
    # statistics each, + partial error sums of 2 row blocks per head + row order
    per_slot = sh.B * sh.H * 24 * (sh.D * 4 + 8)
    slots, rest = divmod(need - (sh.B * sh.H * 2 * 8 + 96), per_slot)
    assert rest == 0 and 3 <= slots <= 14
    assert lib.svg_profile_heads(C.byref(sh), a, a, a, a, 24, a, None, None, 0, None) == -3
    assert lib.svg_profile_heads(C.byref(sh), a, a, a, a, 24, a, None, b, need - 1, None) == -3
    assert lib.svg_profile_heads(C.byref(sh), a, a, a, a, 0, a, None, b, need, None) == -1
    assert lib.svg_profile_heads(C.byref(sh), a, a, a, None, 24, a, None, b, need, None) == -1
    # more heads than one grid dimension holds
    many = S.shape_from_config(dict(get_config("mid64"), B=1024, H=64))
    assert lib.svg_profile_heads(C.byref(many), a, a, a, a, 24, a, None, b, 1 << 60, None) == -2


def test_profile_plan_is_well_formed_for_every_workload():
    """The parts the profiling passes are cut into: bounds ascend from 0 to nk, the part counts stay
    within what the header states, the workspace covers every part, the plan is the same on every
    call, and bad arguments are refused."""
    lib = S.lib()
    for name in ["tiny", "mid64", "mid128", "cogvideox_v1", "wan21_14b", "cogvideox_v15", "hunyuan", "hunyuan_skip85"]:
        cfg = get_config(name)
        sh = S.shape_from_config(cfg)
        nq, nk = S.svg_tile_counts(sh)
        for t in (1, cfg["t"], 5 * cfg["t"], cfg["N"]):
            nf, nm, bound = S.svg_profile_plan(sh, t)
            assert 1 <= nf <= 6 and 1 <= nm <= 4, (name, t, nf, nm)
            assert bound[0] == 0 and bound[-1] == nk and all(a <= b for a, b in zip(bound, bound[1:])), (name, t, bound)
            assert (nf, nm, bound) == S.svg_profile_plan(sh, t)
            BH = cfg["B"] * cfg["H"]
            want = (nf + 2 * nm) * BH * t * (cfg["D"] * 4 + 8) + BH * (-(-t // 16)) * 8 + ((4 * t + 15) & ~15)
            assert S.svg_workspace_bytes(sh, t) == max(want, 8 * nk * sh.block_n), (name, t)
    sh = S.shape_from_config(get_config("mid64"))
    nf, nm = C.c_int32(), C.c_int32()
    assert lib.svg_profile_plan(C.byref(sh), 0, C.byref(nf), C.byref(nm), None) == -1
    assert lib.svg_profile_plan(C.byref(sh), 8, None, C.byref(nm), None) == -1
    assert lib.svg_profile_plan(C.byref(sh), 8, C.byref(nf), C.byref(nm), None) == 0


def test_fp8_buffer_sizes_and_argument_checks_without_gpu():
    lib = S.lib()
    cfg = get_config("mid128")
    sh = S.shape_from_config(cfg)
    nq, nk = S.svg_tile_counts(sh)
    bh = sh.B * sh.H
    assert S.svg_fp8_buffer_bytes(sh, S.SVG_FP8_Q) == bh * cfg["N"] * 128
    assert S.svg_fp8_buffer_bytes(sh, S.SVG_FP8_K) == S.svg_fp8_buffer_bytes(sh, S.SVG_FP8_VT) == bh * nk * 64 * 128
    assert S.svg_fp8_buffer_bytes(sh, S.SVG_FP8_SCALES) == 6 * bh * 4
    assert S.svg_fp8_buffer_bytes(sh, 7) == 0
    a = 0x10000000
    # head dimension 64 and the small tile shape are not supported by the FP8 path
    for name in ("mid64", "tiny"):
        bad = S.shape_from_config(get_config(name))
        assert S.svg_fp8_buffer_bytes(bad, S.SVG_FP8_Q) == 0
        assert lib.svg_fp8_quantize(C.byref(bad), a, a, a, None, a, a, a, a, None) == -2
        assert lib.svg_sparse_attn_fp8_fwd(C.byref(bad), a, a, a, a, a, None, a, a, None, None, None) == -2
    # NULL / misaligned pointers are rejected before any launch
    assert lib.svg_fp8_quantize(C.byref(sh), a, a, None, None, a, a, a, a, None) == -1
    assert lib.svg_fp8_quantize(C.byref(sh), a, a, a, None, a, a + 4, a, a, None) == -1
    assert lib.svg_fp8_quantize(C.byref(sh), a, a, a, None, a, a, a, None, None) == -1
    assert lib.svg_sparse_attn_fp8_fwd(C.byref(sh), a, a, a, None, a, None, a, a, None, None, None) == -1
    assert lib.svg_sparse_attn_fp8_fwd(C.byref(sh), a, a, a, a, a, None, None, a, None, None, None) == -1
    assert lib.svg_sparse_attn_fp8_fwd(C.byref(sh), a, a, a, a, a, a, a, a, None, None, None) == -1
    # overlapping buffers (sizes differ per buffer): the output of the attention pass against each of its
    # inputs, the quantiser's outputs against each other and against its inputs
    big = 1 << 32
    p = [a + i * big for i in range(8)]          # q8, k8, v8t, scales, o, q, k, v: far apart
    nq8 = S.svg_fp8_buffer_bytes(sh, S.SVG_FP8_Q)
    nk8 = S.svg_fp8_buffer_bytes(sh, S.SVG_FP8_K)
    for bad_o in (p[0] + nq8 - 16, p[1] + nk8 - 16, p[2], p[3]):
        assert lib.svg_sparse_attn_fp8_fwd(C.byref(sh), p[0], p[1], p[2], p[3], bad_o, None, a, a, None, None, None) == -4
    assert lib.svg_sparse_attn_fp8_fwd(C.byref(sh), p[0], p[1], p[2], p[3], p[1] - 2 * nq8 + 16, None, a, a, None, None,
                                       None) == -4          # the END of o reaches into k8
    assert lib.svg_fp8_quantize(C.byref(sh), p[5], p[6], p[7], None, p[0], p[0] + nq8 - 16, p[2], p[3], None) == -4
    assert lib.svg_fp8_quantize(C.byref(sh), p[5], p[6], p[7], None, p[0], p[1], p[7] + 16, p[3], None) == -4
    assert lib.svg_fp8_quantize(C.byref(sh), p[5], p[6], p[7], None, p[5], p[1], p[2], p[3], None) == -4
    assert lib.svg_fp8_quantize(C.byref(sh), p[5], p[6], p[7], None, p[0], p[1], p[2], p[2] + 16, None) == -4


def test_rate_probe_argument_checks_without_gpu():
    lib = S.lib()
    a = 0x10000000
    flop = C.c_double()
    assert lib.svg_probe_mfma_bf16(3, 8, 1, a, a, C.byref(flop), None) == -1        # unknown form
    assert lib.svg_probe_mfma_bf16(0, 0, 1, a, a, C.byref(flop), None) == -1
    assert lib.svg_probe_mfma_bf16(0, 8, 0, a, a, C.byref(flop), None) == -1
    assert lib.svg_probe_mfma_bf16(0, 8, 1, None, a, C.byref(flop), None) == -1
    assert lib.svg_probe_mfma_bf16(1, 8, 1, a + 2, a, C.byref(flop), None) == -1
    need = 16 * 8 + 1024 * 4
    assert lib.svg_probe_lds(4, 8, 1, a, need, None) == -1                           # unknown form
    assert lib.svg_probe_lds(0, 0, 1, a, need, None) == -1
    assert lib.svg_probe_lds(0, 17, 1, a, need, None) == -1                          # a workgroup holds 16 wavefronts
    assert lib.svg_probe_lds(0, 8, 0, a, need, None) == -1
    assert lib.svg_probe_lds(0, 8, 1, None, need, None) == -1
    assert lib.svg_probe_lds(0, 8, 1, a + 8, need, None) == -1
    assert lib.svg_probe_lds(0, 8, 1, a, need - 1, None) == -3                       # scratch too small


def test_qk_norm_rope_argument_checks_without_gpu():
    lib = S.lib()
    sh = S.shape_from_config(get_config("mid64"))
    nbytes = sh.B * sh.H * sh.N * sh.D * 2
    a, b, t = 0x10000000, 0x10000000 + 4 * nbytes, 0x70000000
    f = C.c_float(1e-6)
    call = lambda *args: lib.svg_qk_norm_rope(C.byref(sh), *args)
    assert call(None, b, 1, None, None, f, None, None, 0, None) == -1
    assert call(a, b + 2, 1, None, None, f, None, None, 0, None) == -1
    assert call(a, b, 3, None, None, f, None, None, 0, None) == -1            # unknown norm
    assert call(a, b, 1, None, None, f, t, t, 2, None) == -1                  # unknown pairing
    assert call(a, b, 1, None, None, f, t, None, 0, None) == -1               # cos without sin
    assert call(a, b, 1, None, None, f, t + 4, t, 0, None) == -1              # misaligned table
    assert call(a, b, 1, None, None, C.c_float(-1.0), None, None, 0, None) == -1
    assert call(a, a + 16, 1, None, None, f, None, None, 0, None) == -4       # partial overlap
    bad = S.shape_from_config(dict(get_config("mid64"), D=96))
    assert lib.svg_qk_norm_rope(C.byref(bad), a, b, 1, None, None, f, None, None, 0, None) == -2


def test_product_package_does_not_import_the_oracle():
    pkg = os.path.join(ROOT, "paper_2502_01776_amd")
    for dirpath, _, files in os.walk(pkg):
        for f in files:
            if f.endswith((".py", ".cpp", ".hip", ".h")):
                text = open(os.path.join(dirpath, f)).read()
                assert "oracle" not in text, f
    otext = open(os.path.join(ROOT, "oracle", "svg_oracle.py")).read()
    assert "paper_2502_01776_amd" not in otext and "workloads" not in otext
