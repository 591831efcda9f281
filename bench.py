#!/usr/bin/env python3
"""Benchmark of the sparse 3D attention layer on one MI355X.

A step is one pass of the whole hot path over one synthetic layer input that is
already resident in HBM: online profiling (three masked attentions over the
sampled rows + MSE + label), layout transform of k and v of the heads labelled
temporal (one launch; spatial heads are read in place), block-sparse attention
over the kept tiles with the layout transform of q and the inverse transform of o
folded into the kernel (--four-layout-passes: as four separate passes over q, k, v
and o of all heads).  The in-library dense attention is timed beside it, the
matrix cores' sustained rate is measured by a product-only loop, and the CPU oracle
is timed on a bounded sample (in full for the two small workloads).

Prints ONE JSON line on stdout.
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

PEAK_BF16_TFLOPS = 2500.0     # MI355X dense bf16 MFMA peak
PEAK_FP8_TFLOPS = 5000.0      # MI355X dense fp8 MFMA peak
PEAK_HBM_GBS = 8000.0


def parse():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=10)
    ap.add_argument("--warmup", type=int, default=2)
    ap.add_argument("--workload", default="hunyuan_skip85")
    ap.add_argument("--dense-reps", type=int, default=3)
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-dense", action="store_true")
    ap.add_argument("--profile-percent", type=float, default=None,
                    help="percentage of the query rows that online profiling samples (default: the workload's "
                         "1 %%; the paper's ablation uses 0.1, 1, 5 and 100)")
    ap.add_argument("--profile-sweep", action="store_true",
                    help="also time the profiling stage alone at 0.1, 1, 5 and 100 %% of the query rows (the paper's "
                         "Table 3 ratios) and report it as 'profile_ratio_sweep' beside the dense time")
    ap.add_argument("--without-layout-transform", action="store_true",
                    help="also time the comparison arm of Sec. 5.5: temporal heads left in frame-major order "
                         "with the frame-major temporal tile list (no layout kernels)")
    ap.add_argument("--kv-in-kernel", action="store_true",
                    help="no layout pass at all: k and v stay in token order and the sparse kernel gathers the "
                         "rows of a temporal head's key tiles itself (SVG_ATTN_KV_TOKEN_ORDER)")
    ap.add_argument("--four-layout-passes", action="store_true",
                    help="time the pipeline with q, k, v and o all going through the layout kernels, instead of "
                         "the default where the attention kernel gathers q rows and scatters o rows itself")
    ap.add_argument("--no-fp8", action="store_true",
                    help="skip the FP8 variant of the sparse pass (Sec. 4.3 Quantization; head dimension 128 only), "
                         "which is otherwise timed beside the bf16 pipeline and reported in the 'fp8' object")
    ap.add_argument("--no-qk-norm-rope", action="store_true",
                    help="skip the timing of the fused QK-norm + rotary embedding pass on q and k (Table 2), "
                         "otherwise reported in the 'qk_norm_rope' object beside a plain PyTorch version")
    ap.add_argument("--no-hip-graph", action="store_true",
                    help="skip the timing of the same layer captured once as a HIP graph and replayed")
    ap.add_argument("--no-measured-peak", action="store_true",
                    help="skip the two product loops that measure what the matrix cores sustain on this box")
    ap.add_argument("--only", default="", help="time a single stage only (profile|layout|sparse|dense); "
                    "used for per-kernel rocprofv3 runs")
    return ap.parse_args()


def ev():
    import torch
    return torch.cuda.Event(enable_timing=True)


def blas_threads():
    """Threads of the BLAS pool numpy's matrix products run on (the oracle's only parallel part)."""
    try:
        from threadpoolctl import threadpool_info
        n = [i.get("num_threads", 1) for i in threadpool_info() if i.get("user_api") == "blas"]
        return max(n) if n else 1
    except Exception:
        return 1


def rel_rms(a, b):
    import numpy as np
    return float(np.linalg.norm(a - b) / max(np.linalg.norm(b), 1e-30))


def cpu_baseline(cfg, q, k, v, rows, labels_np, nnz_total, o_bf16=None, o_fp8=None):
    """The oracle as it stands, timed on the host cores of this machine.  The two small workloads
    are timed in full; for the others a bounded sample of independent units is timed
    (profiling of one head of each label on a subset of the sampled rows, the block-sparse pass
    of a few query tiles of one spatial and one temporal head) and scaled linearly to a layer."""
    import numpy as np
    import torch
    from oracle import svg_oracle as O
    g = O.Geometry.from_config(cfg)
    nq, nk = O.n_tiles(g)
    host_cpus = len(os.sched_getaffinity(0))
    f64 = lambda x: x.cpu().to(torch.float64).numpy()
    dense_flops = 4.0 * g.N * g.N * g.D * g.H * g.B
    if cfg["name"] in ("tiny", "cogvideox_v1"):
        qd, kd, vd = f64(q), f64(k), f64(v)
        t0 = time.perf_counter()
        _, olab = O.profile_heads(qd, kd, vd, rows, g)
        t_prof = time.perf_counter() - t0
        t0 = time.perf_counter()
        O.svg_attention_layer(qd, kd, vd, olab, g)
        t_attn = time.perf_counter() - t0
        layer_s = t_prof + t_attn
        return {"value": dense_flops / layer_s / 1e12, "unit": "TFLOP/s (effective)", "cores": blas_threads(),
                "host_cpus": host_cpus, "kind": "oracle", "extrapolated": False, "ms_per_layer": layer_s * 1e3,
                "sample": (f"fp64 numpy oracle, the whole layer: profiling of all {g.B * g.H} heads on all "
                           f"{len(rows)} sampled rows ({t_prof:.1f} s) + tile lists, layout and block-sparse pass "
                           f"of all heads ({t_attn:.1f} s)")}
    h_s = int(np.argmax(labels_np == 0)) if (labels_np == 0).any() else 0
    h_t = int(np.argmax(labels_np == 1)) if (labels_np == 1).any() else 0
    budget_rows = max(8, min(len(rows), int(2.0e8 // g.N)))      # bounds the t x N score matrices
    sub = rows[:: max(1, len(rows) // budget_rows)][:budget_rows]
    g1 = O.Geometry(**{**g.__dict__, "B": 1, "H": 1})
    t_prof, n_prof_heads = 0.0, 0
    for h in (h_s, h_t):                                          # one head of each label
        qh, kh, vh = (f64(x[0, h])[None, None] for x in (q, k, v))
        t0 = time.perf_counter()
        O.profile_heads(qh, kh, vh, sub, g1)
        t_prof += time.perf_counter() - t0
        n_prof_heads += 1
    prof_layer_s = t_prof / (n_prof_heads * len(sub)) * len(rows) * g.B * g.H

    tiles_done, t_attn = 0, 0.0
    n_sample = 64
    fp8_split = None
    for pat, h in ((O.SPATIAL, h_s), (O.TEMPORAL, h_t)):
        qh, kh, vh = f64(q[0, h]), f64(k[0, h]), f64(v[0, h])
        pick = sorted(set(int(x) for x in np.linspace(0, nq - 1, n_sample + 2)[1:-1]))
        t0 = time.perf_counter()
        if pat == O.TEMPORAL:
            qh, kh, vh = O.layout_fwd(qh, g), O.layout_fwd(kh, g), O.layout_fwd(vh, g)
        rp = np.zeros(nq + 1, dtype=np.int64)
        cols = []
        for a in range(nq):
            c = O.kept_tiles_of_row(g, pat, a) if a in pick else np.zeros(0, np.int32)
            cols.append(c)
            rp[a + 1] = rp[a] + len(c)
            tiles_done += len(c)
        ref16 = O.sparse_attention_head(qh, kh, vh, rp, np.concatenate(cols), g, q_tiles=pick)
        t_attn += time.perf_counter() - t0
        if o_fp8 is not None and o_bf16 is not None:
            # Where the FP8 layer's difference to the bf16 layer comes from (not timed): the
            # quantisation of q, k, v (oracle over the dequantised tensors against the oracle over
            # the originals), the 8-bit attention weights (oracle with rounded weights against the
            # one without), and the kernel against each; on a few of the sampled query tiles.
            few = pick[:: max(1, len(pick) // 6)]
            dq, dk, dv = (O.fp8_dequantize(*O.fp8_quantize_head(x)) for x in (qh, kh, vh))   # elementwise: any order
            keep = np.concatenate([np.arange(a * g.block_m, min(g.N, (a + 1) * g.block_m)) for a in few])
            rp2 = np.zeros(nq + 1, dtype=np.int64)
            cols2 = []
            for a in range(nq):
                c = cols[a] if a in few else np.zeros(0, np.int32)
                cols2.append(c)
                rp2[a + 1] = rp2[a] + len(c)
            ci2 = np.concatenate(cols2)
            ref8 = O.sparse_attention_head(dq, dk, dv, rp2, ci2, g, q_tiles=few)[keep]
            ref8r = O.sparse_attention_head(dq, dk, dv, rp2, ci2, g, q_tiles=few, weight_round=O.fp8_round_weights)[keep]
            got8, got16 = f64(o_fp8[0, h]), f64(o_bf16[0, h])
            if pat == O.TEMPORAL:
                got8, got16 = O.layout_fwd(got8, g), O.layout_fwd(got16, g)
            part = {"input_quantisation (oracle fp8 vs oracle bf16)": rel_rms(ref8, ref16[keep]),
                    "weight_rounding (oracle 8-bit weights vs oracle fp8)": rel_rms(ref8r, ref8),
                    "kernel_fp8_vs_oracle_fp8": rel_rms(got8[keep], ref8),
                    "kernel_fp8_vs_oracle_fp8_with_8bit_weights": rel_rms(got8[keep], ref8r),
                    "kernel_bf16_vs_oracle_bf16": rel_rms(got16[keep], ref16[keep]),
                    "kernel_fp8_vs_kernel_bf16": rel_rms(got8[keep], got16[keep])}
            fp8_split = fp8_split or {"relative_rms_on": f"{len(few)} query tiles of one head per label"}
            fp8_split["spatial_head" if pat == O.SPATIAL else "temporal_head"] = part
    attn_layer_s = t_attn / max(tiles_done, 1) * nnz_total
    layer_s = prof_layer_s + attn_layer_s
    out = {
        "value": dense_flops / layer_s / 1e12, "unit": "TFLOP/s (effective)", "cores": blas_threads(),
        "host_cpus": host_cpus, "kind": "oracle", "extrapolated": True, "ms_per_layer": layer_s * 1e3,
        "sample": (f"fp64 numpy oracle: profiling of {n_prof_heads} heads on {len(sub)} of {len(rows)} sampled rows "
                   f"({t_prof:.1f} s) + block-sparse pass of {n_sample} query tiles of one spatial and "
                   f"one temporal head incl. tile-list rows and layout ({t_attn:.1f} s, {tiles_done} "
                   f"tiles); scaled linearly to {g.B * g.H} heads, {len(rows)} rows, {nnz_total} tiles"),
    }
    if fp8_split:
        out["fp8_error_split"] = fp8_split
    return out


def measured_matrix_peak(S, torch, head_dim, ms_target=12.0):
    """Sustained rate of the bf16 matrix cores on this machine: a loop of products only (form 0) and
    the same loop with the per-product LDS read and softmax instructions of the attention kernel
    of this head dimension (form 1: D = 128, form 2: D = 64, twice the softmax instructions per
    product and three workgroups per CU), on normally distributed operands, each timed over >= 10 ms; and the
    product-only loop on all-zero operands, which shows how much of the published peak is lost to
    the power the data toggling draws (the clock drops under real data, not under zeros)."""
    gen = torch.Generator(device="cuda").manual_seed(11)
    operands = torch.randn(1 << 19, generator=gen, device="cuda").to(torch.bfloat16)      # 1 MiB
    wgs = 3072         # a multiple of the 512 and of the 768 workgroups the chip holds in forms 0/1 and 2
    sink = torch.empty(wgs * 256, dtype=torch.float32, device="cuda")
    out = {}
    zeros = torch.zeros_like(operands)
    for form, key, ops in ((0, "products_only", operands),
                           (1 if head_dim == 128 else 2, "with_lds_operand_reads_and_softmax_instructions", operands),
                           (0, "products_only_constant_operands", zeros)):
        iters = 500
        for attempt in range(3):
            S.svg_probe_mfma_bf16(form, wgs, iters, ops, sink)          # warm-up / calibration
            torch.cuda.synchronize()
            e0, e1 = ev(), ev()
            e0.record()
            flop = S.svg_probe_mfma_bf16(form, wgs, iters, ops, sink)
            e1.record()
            torch.cuda.synchronize()
            ms = e0.elapsed_time(e1)
            if ms >= ms_target * 0.8:
                break
            iters = int(iters * ms_target / max(ms, 1e-3)) + 1
        out[key] = {"tflops": flop / (ms * 1e-3) / 1e12, "ms": ms}
    return out


def measured_lds_rates(S, torch, waves=8, iters=4000):
    """Bytes per clock the LDS of one compute unit delivers for the operand reads and staging
    writes of the D = 128 attention kernels, with two wavefronts per SIMD as those kernels run
    (svg_probe_lds: one workgroup, shader clocks per wavefront from the kernel's own clock reads)."""
    scratch = torch.zeros(16 + 512, dtype=torch.int64, device="cuda")
    out = {}
    for form, key in ((0, "k_operand_ds_read_b128"), (1, "vt_operand_ds_read_b64_tr_b16_swizzled_rows"),
                      (2, "vt_operand_ds_read_b64_tr_b16_plain_rows"), (3, "staging_ds_write_b128")):
        S.svg_probe_lds(form, waves, 200, scratch)
        nbytes = S.svg_probe_lds(form, waves, iters, scratch)
        torch.cuda.synchronize()
        clocks = float(scratch[:waves].max().item())
        out[key] = {"bytes_per_clock_per_cu": waves * iters * 16 * nbytes / clocks,
                    "cu_clocks_per_wave_instruction": clocks / (iters * 16) / waves}
    out["wavefronts_per_cu"] = waves
    return out


def main():
    args = parse()
    if args.gpus != 1:
        print("bench.py: this build runs on ONE GPU only (heads would shard across GPUs without any "
              "exchange inside the path, but no multi-GPU run is part of it); use --gpus 1",
              file=sys.stderr)
        sys.exit(2)
    import numpy as np
    import torch
    import paper_2502_01776_amd as S
    from workloads import get_config, make_qkv, sample_rows

    S.lib()                                   # fail loudly if the HIP library is not built
    if not torch.cuda.is_available():
        raise SystemExit("bench.py needs a GPU (no CPU fallback exists)")
    cfg = get_config(args.workload)
    sh = S.shape_from_config(cfg)
    B, H, N, D = cfg["B"], cfg["H"], cfg["N"], cfg["D"]
    BH = B * H

    q, k, v = make_qkv(cfg, device="cuda")
    rows_np = sample_rows(cfg) if args.profile_percent is None else \
        sample_rows(cfg, t=max(1, min(cfg["N"], int(np.ceil(cfg["N"] * args.profile_percent / 100.0)))))
    t = len(rows_np)
    rows = torch.from_numpy(rows_np).cuda()
    lists_np = [S.svg_tile_list_build(sh, p) for p in (0, 1)]
    lists = []
    for rp, ci in lists_np:
        lists += [torch.from_numpy(rp).cuda(), torch.from_numpy(ci).cuda()]
    nq, nk = S.svg_tile_counts(sh)
    ws_bytes = S.svg_workspace_bytes(sh, t)
    ws = torch.empty(ws_bytes, dtype=torch.uint8, device="cuda")
    labels = torch.zeros(BH, dtype=torch.uint8, device="cuda")
    mse = torch.zeros(BH, 2, dtype=torch.float32, device="cuda")
    qp, kp, vp, op, o = (torch.empty_like(q) for _ in range(5))

    def stage_profile():
        S.svg_profile_heads(sh, q, k, v, rows, t, labels, mse, ws, ws_bytes)

    folded = not args.four_layout_passes

    in_kernel = args.kv_in_kernel and folded

    def stage_layout_fwd():
        if in_kernel:
            return
        if folded:
            S.svg_layout_kv_temporal(sh, k, v, kp, vp, labels)
        else:
            S.svg_layout_fwd(sh, q, qp, labels)
            S.svg_layout_fwd(sh, k, kp, labels)
            S.svg_layout_fwd(sh, v, vp, labels)

    def stage_sparse():
        if in_kernel:
            S.svg_sparse_attn_fwd_ex(sh, q, k, v, o, labels, *lists,
                                     flags=S.SVG_ATTN_QO_TOKEN_ORDER | S.SVG_ATTN_KV_TOKEN_ORDER,
                                     workspace=ws, workspace_bytes=ws_bytes)
        elif folded:
            S.svg_sparse_attn_fwd_kv2(sh, q, k, v, kp, vp, o, labels, *lists)
        else:
            S.svg_sparse_attn_fwd(sh, qp, kp, vp, op, labels, *lists)

    def stage_layout_inv():
        S.svg_layout_inv(sh, op, o, labels)

    stages = [("profile", stage_profile), ("layout_fwd", stage_layout_fwd), ("sparse_attn", stage_sparse)]
    if not folded:
        stages.append(("layout_inv", stage_layout_inv))

    def step(marks=None):
        for name, fn in stages:
            if marks is not None:
                e0, e1 = ev(), ev()
                e0.record()
                fn()
                e1.record()
                marks.setdefault(name, []).append((e0, e1))
            else:
                fn()

    if args.only:
        # single-stage mode for per-kernel profiling
        step()
        torch.cuda.synchronize()
        fn = {"profile": stage_profile,
              "layout": lambda: (stage_layout_fwd(), None if folded else stage_layout_inv()),
              "sparse": stage_sparse,
              "dense": lambda: S.svg_dense_attn_fwd(sh, q, k, v, o)}[args.only]
        for _ in range(args.warmup):
            fn()
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for _ in range(args.steps):
            fn()
        torch.cuda.synchronize()
        print(json.dumps({"only": args.only, "workload": args.workload,
                          "ms": (time.perf_counter() - t0) * 1e3 / args.steps}))
        return

    for _ in range(args.warmup):
        step()
    torch.cuda.synchronize()
    marks = {}
    t0 = time.perf_counter()
    for _ in range(args.steps):
        step(marks)
    torch.cuda.synchronize()
    wall_ms = (time.perf_counter() - t0) * 1e3 / args.steps
    breakdown = {name: float(np.median([a.elapsed_time(b) for a, b in lst])) for name, lst in marks.items()}

    # The same layer captured once as a HIP graph and replayed (no entry point allocates, synchronises
    # or records a memset): what a caller gains who removes the launch gaps of the layer's six kernels.
    graph_ms, graph_error = None, None
    if not args.no_hip_graph:
        try:
            side = torch.cuda.Stream()
            side.wait_stream(torch.cuda.current_stream())
            with torch.cuda.stream(side):
                step()
            torch.cuda.current_stream().wait_stream(side)
            torch.cuda.synchronize()
            graph = torch.cuda.CUDAGraph()
            with torch.cuda.graph(graph, stream=side):
                step()
            graph.replay()
            torch.cuda.synchronize()
            t1 = time.perf_counter()
            for _ in range(args.steps):
                graph.replay()
            torch.cuda.synchronize()
            graph_ms = (time.perf_counter() - t1) * 1e3 / args.steps
            del graph
        except Exception as e:      # an add-on measurement: the bench line is printed without it
            graph_error = f"{type(e).__name__}: {e}"
            torch.cuda.synchronize()

    labels_np = labels.cpu().numpy()
    n_temporal = int(labels_np.sum())
    nnz = [int(rp[-1]) for rp, _ in lists_np]
    nnz_total = (BH - n_temporal) * nnz[0] + n_temporal * nnz[1]
    kept_fraction = nnz_total / (BH * nq * nk)

    dense_ms = None
    if not args.no_dense:
        od = op        # reuse a buffer
        S.svg_dense_attn_fwd(sh, q, k, v, od)
        torch.cuda.synchronize()
        dense_times = []
        for _ in range(args.dense_reps):
            e0, e1 = ev(), ev()
            e0.record()
            S.svg_dense_attn_fwd(sh, q, k, v, od)
            e1.record()
            torch.cuda.synchronize()
            dense_times.append(e0.elapsed_time(e1))
        dense_ms = float(np.median(dense_times))

    dense_flops = 4.0 * N * N * D * BH
    tile_flops = 4.0 * cfg["block_m"] * cfg["block_n"] * D
    sparse_ms = breakdown["sparse_attn"]
    achieved = tile_flops * nnz_total / (sparse_ms * 1e-3) / 1e12
    # figures that need hardware counters come from the committed rocprofv3 summary of this
    # same command (not measured live): bytes past L2 per launch, and the fraction of shader
    # cycles with the MFMA unit busy together with the shader clock those cycles ran at
    traffic = counters = None
    prof = {}
    tpath = os.path.join(ROOT, "profiles", f"hbm_traffic_{args.workload}.json")
    if os.path.exists(tpath):
        with open(tpath) as f:
            prof = json.load(f)
        traffic = prof.get("sparse_attn_bytes_per_launch")
        if "sparse_attn_mfma_busy_fraction_of_cycles" in prof:
            counters = {"live": False, "measured_on": prof.get("measured_on", "another box of the pool, see source"),
                        "mfma_busy_fraction_of_cycles": prof["sparse_attn_mfma_busy_fraction_of_cycles"],
                        "shader_clock_ghz": prof["sparse_attn_shader_clock_ghz"], "source": prof.get("source")}
    # algorithmic bytes of the layout stage: one read and one write of every tensor row that has to move
    # (temporal heads only); the four-pass form also copies the spatial heads, which is not counted
    layout_bytes = 2.0 * n_temporal * N * D * 2
    peak_live = None if args.no_measured_peak else measured_matrix_peak(S, torch, D)
    out = {
        "metric": "effective TFLOP/s of one sparse attention layer at %dk tokens "
                  "(4*N^2*D*H / ms per layer; profile + layout + block-sparse attention + inverse layout%s)"
                  % (round(N / 1000), ", the layout of q and o folded into the attention kernel" if folded else ""),
        "value": dense_flops / (wall_ms * 1e-3) / 1e12,
        "unit": "TFLOP/s",
        "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": wall_ms, "higher_is_better": True, "scaling": "weak",
        "vs_baseline": None, "dtype": "bf16", "data": "synthetic",
        "config": {"workload": args.workload, "B": B, "H": H, "F": cfg["F"], "P": cfg["P"], "T": cfg["T"],
                   "N": N, "D": D, "w_s": cfg["w_s"], "w_t": cfg["w_t"], "tile": [cfg["block_m"], cfg["block_n"]],
                   "profiled_rows": t, "temporal_heads": n_temporal, "kept_tile_fraction": kept_fraction},
        "ms_per_layer": wall_ms,
        "hip_graph": ({"error": graph_error} if graph_error else None) if graph_ms is None else
                     {"ms_per_layer_replayed": graph_ms, "ms_per_layer_eager": wall_ms,
                      "what": "the layer's launches captured once and replayed"},
        "breakdown_ms": breakdown,
        "dense_ms": dense_ms,
        "dense_tflops": None if dense_ms is None else dense_flops / (dense_ms * 1e-3) / 1e12,
        "speedup_vs_dense": None if dense_ms is None else dense_ms / wall_ms,
        "layout_passes": "k and v of temporal heads in one launch (q and o inside the attention kernel, spatial heads "
                         "read in place)" if folded else "q k v o, all heads",
        "layout_gbs": {"fwd": None if in_kernel else
                       (2 if folded else 3) * layout_bytes / (breakdown["layout_fwd"] * 1e-3) / 1e9,
                       "counts": "rows of temporal heads only, read + write",
                       "inv_o": None if folded else layout_bytes / (breakdown["layout_inv"] * 1e-3) / 1e9},
        # the three masked passes of Alg. 1 counted in full (3 x 4 t N D per head), although the
        # kernel skips the key tiles no sampled row of a workgroup keeps
        "profile_nominal_tflops": 3 * 4.0 * t * N * D * BH / (breakdown["profile"] * 1e-3) / 1e12,
        # algorithmic bytes of profiling: K and V of every head once (the sampled Q rows and the
        # outputs are small); far from the 8 TB/s HBM roof, the stage is MFMA-bound at 1 % of the rows
        "profile_kv_gbs": 2.0 * BH * N * D * 2 / (breakdown["profile"] * 1e-3) / 1e9,
        "roofline": {"kernel": "attn_kernel<128,4,64,sparse>" if D == 128 else "attn_kernel<64,4,64,sparse>",
                     "bound": "mfma", "achieved": achieved, "peak": PEAK_BF16_TFLOPS, "unit": "TFLOP/s",
                     "frac": achieved / PEAK_BF16_TFLOPS, "traffic": traffic,
                     "traffic_live": False if traffic is not None else None, "counters": counters},
    }
    if peak_live:
        # what the matrix cores sustain on THIS box at the clock a matrix load runs at (live, HIP events)
        mp = peak_live["products_only"]["tflops"]
        mix = peak_live["with_lds_operand_reads_and_softmax_instructions"]["tflops"]
        out["roofline"]["measured_peak"] = mp
        out["roofline"]["frac_of_measured_peak"] = achieved / mp
        out["roofline"]["measured_peak_with_kernel_instruction_mix"] = mix
        out["roofline"]["frac_of_instruction_mix_bound"] = achieved / mix
        out["roofline"]["measured_peak_constant_operands"] = peak_live["products_only_constant_operands"]["tflops"]
        out["roofline"]["measured_peak_detail"] = peak_live
        # what the LDS of a compute unit delivers for this kernel's operand reads and staging writes (live)
        try:
            out["roofline"]["lds_rates"] = measured_lds_rates(S, torch)
        except Exception as e:      # an add-on measurement: the bench line is printed without it
            out["roofline"]["lds_rates"] = {"error": f"{type(e).__name__}: {e}"}
    o8_keep = None
    if not args.no_fp8 and S.svg_fp8_buffer_bytes(sh, S.SVG_FP8_Q) > 0:
        # the same layer with the sparse pass in FP8: profiling as above (bf16), one quantisation pass
        # (per-head maxima, conversion, layout of k and v of temporal heads), FP8 attention
        f8 = [torch.empty(S.svg_fp8_buffer_bytes(sh, w), dtype=torch.uint8, device="cuda") for w in range(3)]
        f8s = torch.zeros(S.svg_fp8_buffer_bytes(sh, S.SVG_FP8_SCALES) // 4, dtype=torch.float32, device="cuda")
        o8 = torch.empty_like(q)

        def fp8_quantize():
            S.svg_fp8_quantize(sh, q, k, v, labels, *f8, f8s)

        def fp8_attn():
            S.svg_sparse_attn_fp8_fwd(sh, *f8, f8s, o8, labels, *lists)

        times = {}
        for name, fn in (("quantize", fp8_quantize), ("sparse_attn", fp8_attn)):
            for _ in range(max(1, args.warmup)):
                fn()
            torch.cuda.synchronize()
            e0, e1 = ev(), ev()
            e0.record()
            for _ in range(args.steps):
                fn()
            e1.record()
            torch.cuda.synchronize()
            times[name] = e0.elapsed_time(e1) / args.steps
        if folded:
            diff = (o8.float() - o.float()).norm().item() / max(o.float().norm().item(), 1e-30)
        else:
            diff = None
        o8_keep = o8
        layer8 = breakdown["profile"] + times["quantize"] + times["sparse_attn"]
        tf8 = tile_flops * nnz_total / (times["sparse_attn"] * 1e-3) / 1e12
        out["fp8"] = {
            "format": "E4M3, one scale per head and tensor; attention weights E4M3; fp32 accumulation",
            "breakdown_ms": {"profile": breakdown["profile"], "quantize_and_layout": times["quantize"],
                             "sparse_attn": times["sparse_attn"]},
            "ms_per_layer": layer8,
            "effective_tflops": dense_flops / (layer8 * 1e-3) / 1e12,
            "speedup_vs_bf16_layer": wall_ms / layer8,
            "speedup_vs_bf16_sparse_kernel": sparse_ms / times["sparse_attn"],
            "speedup_vs_dense": None if dense_ms is None else dense_ms / layer8,
            "roofline": {"kernel": "attn_fp8_kernel", "bound": "mfma", "achieved": tf8, "peak": PEAK_FP8_TFLOPS,
                         "unit": "TFLOP/s", "frac": tf8 / PEAK_FP8_TFLOPS,
                         "traffic": prof.get("fp8_attn_bytes_per_launch"),
                         "traffic_live": False if prof.get("fp8_attn_bytes_per_launch") is not None else None,
                         "counters": None if "fp8_attn_mfma_busy_fraction_of_cycles" not in prof else {
                             "live": False,
                             "mfma_busy_fraction_of_cycles": prof["fp8_attn_mfma_busy_fraction_of_cycles"],
                             "shader_clock_ghz": prof["fp8_attn_shader_clock_ghz"], "source": prof.get("source")}},
            # bytes of the quantisation pass: q, k, v read twice (maxima, conversion), written once as bytes
            "quantize_gbs": (2 * 3 * 2 + 3) * BH * N * D / (times["quantize"] * 1e-3) / 1e9,
            "relative_difference_to_bf16_output": diff,
        }
    if not args.no_qk_norm_rope:
        # the two small per-token operations in front of the attention (Sec. 4.3, Table 2), fused into one
        # pass per tensor: RMS form for the D = 128 models, LayerNorm form for the D = 64 ones
        norm = S.SVG_NORM_RMS if D == 128 else S.SVG_NORM_LAYER
        gen = torch.Generator(device="cuda").manual_seed(7)
        wgt = 1.0 + 0.1 * torch.randn(D, generator=gen, device="cuda")
        bia = 0.1 * torch.randn(D, generator=gen, device="cuda")
        nv = cfg["F"] * cfg["P"]
        freq = 1.0 / 10000.0 ** (torch.arange(D // 2, device="cuda", dtype=torch.float32) / (D // 2))
        theta = torch.arange(nv, device="cuda", dtype=torch.float32)[:, None] * freq[None, :]
        cos_t, sin_t = torch.cos(theta).contiguous(), torch.sin(theta).contiguous()
        yq = qp        # scratch outputs: qp and op (kp and vp still hold the copies later comparisons read)

        def fused():
            S.svg_qk_norm_rope(sh, q, yq, norm, wgt, bia, 1e-6, cos_t, sin_t, S.SVG_ROPE_INTERLEAVED)
            S.svg_qk_norm_rope(sh, k, op, norm, wgt, bia, 1e-6, cos_t, sin_t, S.SVG_ROPE_INTERLEAVED)

        off = cfg["T"] if cfg["text_first"] else 0

        def plain_torch(x):
            xf = x.float()
            if norm == S.SVG_NORM_RMS:
                xf = xf * torch.rsqrt(xf.pow(2).mean(-1, keepdim=True) + 1e-6) * wgt
            else:
                xf = torch.nn.functional.layer_norm(xf, (D,), wgt, bia, 1e-6)
            v = xf[:, :, off:off + nv].unflatten(-1, (D // 2, 2))
            a_, b_ = v[..., 0], v[..., 1]
            rot = torch.stack((a_ * cos_t - b_ * sin_t, b_ * cos_t + a_ * sin_t), dim=-1).flatten(-2)
            xf[:, :, off:off + nv] = rot
            return xf.to(torch.bfloat16)

        def timed(fn, reps):
            fn()
            torch.cuda.synchronize()
            e0, e1 = ev(), ev()
            e0.record()
            for _ in range(reps):
                fn()
            e1.record()
            torch.cuda.synchronize()
            return e0.elapsed_time(e1) / reps

        ms_fused = timed(fused, args.steps)
        ms_torch = timed(lambda: (plain_torch(q), plain_torch(k)), 3)
        same = bool(((plain_torch(q).float() - yq.float()).abs() <= 2.0 ** -7 * yq.float().abs() + 1e-3).all())
        moved = 2 * 2.0 * BH * N * D * 2 + 2 * nv * (D // 2) * 4        # q and k read + written, tables once
        out["qk_norm_rope"] = {
            "what": "%s QK-norm + interleaved RoPE of q and k, one fused pass per tensor" %
                    ("RMS" if norm == S.SVG_NORM_RMS else "LayerNorm"),
            "ms_q_and_k": ms_fused, "plain_pytorch_ms": ms_torch, "speedup_vs_plain_pytorch": ms_torch / ms_fused,
            "matches_plain_pytorch": same,
            "roofline": {"kernel": "norm_rope_kernel<%d>" % D, "bound": "hbm", "achieved": moved / (ms_fused * 1e-3) / 1e9,
                         "peak": PEAK_HBM_GBS, "unit": "GB/s", "frac": moved / (ms_fused * 1e-3) / 1e9 / PEAK_HBM_GBS},
        }
    if args.profile_sweep:
        # the stage alone, at the sampling ratios of the paper's ablation; labels must not depend on the ratio
        # for planted heads, so they are reported too
        sweep = []
        for pct in (0.1, 1.0, 5.0, 100.0):
            rows_p = sample_rows(cfg, t=max(1, min(N, int(np.ceil(N * pct / 100.0)))))
            tp = len(rows_p)
            rows_d = torch.from_numpy(rows_p).cuda()
            nb = S.svg_workspace_bytes(sh, tp)
            wsp = torch.empty(nb, dtype=torch.uint8, device="cuda")
            lab_p = torch.zeros(BH, dtype=torch.uint8, device="cuda")
            reps = 2 if pct > 50 else max(3, args.steps)
            S.svg_profile_heads(sh, q, k, v, rows_d, tp, lab_p, mse, wsp, nb)
            torch.cuda.synchronize()
            times = []
            for _ in range(reps):
                e0, e1 = ev(), ev()
                e0.record()
                S.svg_profile_heads(sh, q, k, v, rows_d, tp, lab_p, mse, wsp, nb)
                e1.record()
                torch.cuda.synchronize()
                times.append(e0.elapsed_time(e1))
            ms_p = float(np.median(times))
            sweep.append({"percent_of_rows": pct, "rows": tp, "profile_ms": ms_p,
                          "fraction_of_dense_attention": None if dense_ms is None else ms_p / dense_ms,
                          "labels_equal_to_the_1_percent_run": bool((lab_p.cpu().numpy() == labels_np).all()),
                          "workspace_mb": nb / 1e6})
            del wsp
        out["profile_ratio_sweep"] = sweep
    if folded and not in_kernel and cfg["block_m"] == 128:
        # the same layer with no layout pass and no second copy of k, v: the sparse kernel gathers the
        # rows of a temporal head's key tiles itself (same labels, bit-identical output)
        o_g = torch.empty_like(o)
        both = S.SVG_ATTN_QO_TOKEN_ORDER | S.SVG_ATTN_KV_TOKEN_ORDER
        for _ in range(2):
            S.svg_sparse_attn_fwd_ex(sh, q, k, v, o_g, labels, *lists, flags=both, workspace=ws, workspace_bytes=ws_bytes)
        torch.cuda.synchronize()
        times = []
        for _ in range(args.steps):
            e0, e1 = ev(), ev()
            e0.record()
            S.svg_sparse_attn_fwd_ex(sh, q, k, v, o_g, labels, *lists, flags=both, workspace=ws, workspace_bytes=ws_bytes)
            e1.record()
            torch.cuda.synchronize()
            times.append(e0.elapsed_time(e1))
        ms_g = float(np.median(times))
        out["kv_gathered_in_kernel"] = {
            "sparse_attn_ms": ms_g, "ms_per_layer": breakdown["profile"] + ms_g,
            "against_layout_pass_plus_kernel_ms": breakdown["layout_fwd"] + breakdown["sparse_attn"],
            "output_equal_bit_for_bit": bool(torch.equal(o_g.view(torch.int16), o.view(torch.int16))),
            "extra_device_memory_bytes": 8 * nk * cfg["block_n"],
            "extra_device_memory_bytes_with_layout_pass": 2 * q.numel() * 2}
        del o_g
    if folded and not in_kernel:
        # the same pass under the exact element masks of Sec. 3.1 instead of their block cover
        o_e = torch.empty_like(o)
        for _ in range(2):
            S.svg_sparse_attn_fwd_kv2(sh, q, k, v, kp, vp, o_e, labels, *lists, flags=S.SVG_ATTN_ELEMENT_MASK)
        torch.cuda.synchronize()
        times = []
        for _ in range(args.steps):
            e0, e1 = ev(), ev()
            e0.record()
            S.svg_sparse_attn_fwd_kv2(sh, q, k, v, kp, vp, o_e, labels, *lists, flags=S.SVG_ATTN_ELEMENT_MASK)
            e1.record()
            torch.cuda.synchronize()
            times.append(e0.elapsed_time(e1))
        out["exact_element_mask"] = {
            "sparse_attn_ms": float(np.median(times)), "block_form_ms": breakdown["sparse_attn"],
            "relative_rms_difference_to_block_form": float((o_e.float() - o.float()).norm() / o.float().norm())}
        del o_e
    if args.without_layout_transform:
        # same labels, same kernel, unpermuted q, k, v: the temporal slot gets the list of the
        # temporal mask in frame-major order
        rp2, ci2 = S.svg_tile_list_build(sh, S.SVG_LIST_TEMPORAL_FRAME_MAJOR)
        lists2 = lists[:2] + [torch.from_numpy(rp2).cuda(), torch.from_numpy(ci2).cuda()]
        for _ in range(2):
            S.svg_sparse_attn_fwd(sh, q, k, v, op, labels, *lists2)
        torch.cuda.synchronize()
        e0, e1 = ev(), ev()
        e0.record()
        for _ in range(args.steps):
            S.svg_sparse_attn_fwd(sh, q, k, v, op, labels, *lists2)
        e1.record()
        torch.cuda.synchronize()
        ms2 = e0.elapsed_time(e1) / args.steps
        nnz2 = (BH - n_temporal) * nnz[0] + n_temporal * int(rp2[-1])
        out["without_layout_transform"] = {
            "temporal_tiles_per_head": int(rp2[-1]), "temporal_tiles_per_head_transformed": nnz[1],
            "kept_tile_fraction": nnz2 / (BH * nq * nk), "sparse_attn_ms": ms2,
            "ms_per_layer": breakdown["profile"] + ms2,
            "with_transform_ms_per_layer": wall_ms,
            "speedup_from_transform": (breakdown["profile"] + ms2) / wall_ms}
    if not args.no_cpu_baseline:
        out["cpu_baseline"] = cpu_baseline(cfg, q, k, v, rows_np, labels_np, nnz_total,
                                           o_bf16=o if folded else None, o_fp8=o8_keep)
    print(json.dumps(out))


if __name__ == "__main__":
    main()
